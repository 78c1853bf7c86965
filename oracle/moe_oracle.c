/*
 * CPU oracle for one Mixture-of-Experts layer.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain statement of what the layer computes.  It is
 * used by the tests, by the smoke check and by the benchmark's CPU-baseline
 * leg, never by the product path, and it shares no code with the HIP library.
 *
 * What is computed (paper section 2.1: a gating function selects a subset of
 * k of the n_e expert feed-forward networks for every input token and only
 * those experts run; notation table of section 4.2: h1 = model hidden size,
 * h2 = expert intermediate size, n_e experts, top-k, data type dt; section 3.3:
 * the micro-batch mu is the number of tokens one kernel execution sees).  The
 * paper does not spell out the gate or the expert MLP; the forms used here are
 * the ones of the models it evaluates (Mixtral, DBRX): a linear router, top-k
 * selection, softmax over the selected logits, and SwiGLU experts
 *     o = W2 ( silu(W1 x) * (W3 x) ),  silu(z) = z / (1 + exp(-z)).
 *
 * Conventions
 *   T tokens (= mu), H = h1, F = h2, E = n_e, k, R = T*k routed rows.
 *   Dense weights, out-features major: Wr[E][H], W1[E][F][H], W3[E][F][H],
 *   W2[E][H][F].  dtype 0: arrays hold IEEE float; dtype 1: arrays hold
 *   bfloat16 bit patterns (uint16).  All arithmetic is done in double; the only
 *   rounding that belongs to the function itself is that the SwiGLU product h
 *   is an operand of the second matrix product and therefore has the storage
 *   type dt: for dtype 1 it is rounded to bfloat16 (round-to-nearest-even),
 *   for dtype 0 to float.
 *   Ties between equal logits go to the lower expert index; the k selected
 *   experts of a token are listed by descending logit.
 *   Rows are grouped by expert, and inside an expert ordered by ascending
 *   token index (a stable counting sort of the flat index t*k + s).
 *
 * The oracle knows nothing about weight pages: the paper's paged weights
 * (appendix A.1) change where bytes live, not what is computed.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- storage-type helpers (the oracle's own; nothing shared with the GPU side) ---- */

static double bf16_bits_to_double(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double load_elem(const void* p, int dtype, size_t i) {
    if (dtype == 1) return bf16_bits_to_double(((const uint16_t*)p)[i]);
    return (double)((const float*)p)[i];
}

/* Round a double to the nearest bfloat16 value (ties to even), returned as a
 * double.  bfloat16 has 8 significant bits, a minimum normal exponent of -126
 * and a subnormal spacing of 2^-133. */
double oracle_round_bf16(double v) {
    if (v == 0.0 || isnan(v) || isinf(v)) return v;
    int e;
    (void)frexp(fabs(v), &e);           /* |v| = m * 2^e, m in [0.5, 1) */
    int q = e - 8;                      /* spacing 2^q keeps 8 significant bits */
    if (q < -133) q = -133;
    double r = nearbyint(ldexp(fabs(v), -q));   /* default mode: ties to even */
    double out = ldexp(r, q);
    if (out > 3.3895313892515355e38) out = INFINITY;   /* above bf16 max */
    return v < 0 ? -out : out;
}

static double round_to_dtype(double v, int dtype) {
    if (dtype == 1) return oracle_round_bf16(v);
    return (double)(float)v;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- a1: router --------------------------------------------------------- */
/*
 * logits[t][e] = sum_h x[t][h] * Wr[e][h] (+ bias[e]);
 * ids[t][0..k) = the k largest logits by descending value, ties to the lower
 * expert index; w[t][s] = exp(l_s - l_0) / sum_s' exp(l_s' - l_0) over the k
 * selected logits (identical to a softmax over all E followed by division by
 * the selected mass).
 * gap_next[t]  = logit of the k-th choice minus the best logit left out
 *                (+inf when k == E): small values mark tokens whose SET of
 *                experts is decided by rounding.
 * gap_inner[t] = smallest difference between consecutive selected logits
 *                (+inf when k == 1): small values mark tokens whose ORDER of
 *                experts is decided by rounding.
 */
void oracle_route(int T, int H, int E, int k, int dtype,
                  const void* x, const void* Wr, const double* bias,
                  int32_t* ids, double* w, double* logits,
                  double* gap_next, double* gap_inner) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        double* lg = logits + (size_t)t * E;
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int h = 0; h < H; ++h)
                acc += load_elem(x, dtype, (size_t)t * H + h) * load_elem(Wr, dtype, (size_t)e * H + h);
            lg[e] = acc + (bias ? bias[e] : 0.0);
        }
        unsigned char taken[1024];
        memset(taken, 0, sizeof taken);
        for (int s = 0; s < k; ++s) {
            int best = -1;
            for (int e = 0; e < E; ++e)
                if (!taken[e] && (best < 0 || lg[e] > lg[best])) best = e;   /* strict >: lower index wins ties */
            taken[best] = 1;
            ids[(size_t)t * k + s] = best;
        }
        double m = lg[ids[(size_t)t * k]];
        double den = 0.0;
        for (int s = 0; s < k; ++s) den += exp(lg[ids[(size_t)t * k + s]] - m);
        for (int s = 0; s < k; ++s) w[(size_t)t * k + s] = exp(lg[ids[(size_t)t * k + s]] - m) / den;

        double gn = INFINITY, gi = INFINITY;
        double kth = lg[ids[(size_t)t * k + k - 1]];
        for (int e = 0; e < E; ++e)
            if (!taken[e] && kth - lg[e] < gn) gn = kth - lg[e];
        for (int s = 0; s + 1 < k; ++s) {
            double d = lg[ids[(size_t)t * k + s]] - lg[ids[(size_t)t * k + s + 1]];
            if (d < gi) gi = d;
        }
        if (gap_next) gap_next[t] = gn;
        if (gap_inner) gap_inner[t] = gi;
    }
}

/* ---- a2: permutation of routed rows by expert --------------------------- */
/*
 * counts[e]   = number of (t, s) with ids[t][s] == e          (sum = T*k)
 * offsets     = exclusive prefix sum of counts, offsets[E] = T*k
 * row of flat index i = t*k + s with expert e:
 *     row_of[i] = offsets[e] + #{ i' < i : ids[i'] == e }
 * row_src[row_of[i]] = i.
 */
void oracle_permute(int T, int k, int E, const int32_t* ids,
                    int32_t* counts, int32_t* offsets, int32_t* row_src, int32_t* row_of) {
    int R = T * k;
    for (int e = 0; e < E; ++e) counts[e] = 0;
    for (int i = 0; i < R; ++i) counts[ids[i]] += 1;
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + counts[e];
    int32_t* next = (int32_t*)malloc(sizeof(int32_t) * (size_t)(E > 0 ? E : 1));
    for (int e = 0; e < E; ++e) next[e] = offsets[e];
    for (int i = 0; i < R; ++i) {
        int r = next[ids[i]]++;
        row_of[i] = r;
        row_src[r] = i;
    }
    free(next);
}

/* x_perm[r][:] = x[row_src[r] / k][:]  (a copy in the storage type) */
void oracle_gather_rows(int R, int H, int k, int dtype, const void* x,
                        const int32_t* row_src, void* x_perm) {
    size_t esz = dtype == 1 ? 2 : 4;
    for (int r = 0; r < R; ++r) {
        int t = row_src[r] / k;
        memcpy((char*)x_perm + (size_t)r * H * esz, (const char*)x + (size_t)t * H * esz, (size_t)H * esz);
    }
}

/* ---- a3: SwiGLU expert FFN on permuted rows ----------------------------- */
/*
 * For each selected row r (expert e = the segment of offsets that holds r):
 *   g[f] = sum_h xp[r][h] W1[e][f][h];   u[f] = sum_h xp[r][h] W3[e][f][h]
 *   hh[f] = round_dt( g[f] / (1 + exp(-g[f])) * u[f] )
 *   o[d]  = sum_f hh[f] W2[e][d][f]      (times row_w[r] when row_w is given)
 * sel == NULL means rows 0..n_sel-1.  h_out / o_out are [n_sel][F] / [n_sel][H]
 * doubles (either may be NULL).
 */
void oracle_expert_ffn(int R, int H, int F, int E, int dtype,
                       const void* x_perm, const int32_t* offsets,
                       const void* W1, const void* W3, const void* W2,
                       const double* row_w,
                       int n_sel, const int32_t* sel,
                       double* h_out, double* o_out) {
    (void)R;
    for (int j = 0; j < n_sel; ++j) {
        int r = sel ? sel[j] : j;
        int e = 0;
        while (e < E && !(offsets[e] <= r && r < offsets[e + 1])) ++e;
        if (e >= E) continue;                       /* row outside every segment: left untouched */
        double* xr = (double*)malloc(sizeof(double) * (size_t)H);
        double* hh = (double*)malloc(sizeof(double) * (size_t)F);
        for (int h = 0; h < H; ++h) xr[h] = load_elem(x_perm, dtype, (size_t)r * H + h);
#pragma omp parallel for schedule(static)
        for (int f = 0; f < F; ++f) {
            size_t base = ((size_t)e * F + f) * H;
            double g = 0.0, u = 0.0;
            for (int h = 0; h < H; ++h) {
                g += xr[h] * load_elem(W1, dtype, base + h);
                u += xr[h] * load_elem(W3, dtype, base + h);
            }
            double silu = g / (1.0 + exp(-g));
            hh[f] = round_to_dtype(silu * u, dtype);
        }
        if (h_out) memcpy(h_out + (size_t)j * F, hh, sizeof(double) * (size_t)F);
        if (o_out) {
#pragma omp parallel for schedule(static)
            for (int d = 0; d < H; ++d) {
                size_t base = ((size_t)e * H + d) * F;
                double acc = 0.0;
                for (int f = 0; f < F; ++f) acc += hh[f] * load_elem(W2, dtype, base + f);
                o_out[(size_t)j * H + d] = row_w ? acc * row_w[r] : acc;
            }
        }
        free(xr);
        free(hh);
    }
}

/* ---- a4: gate-weighted un-permute and combine --------------------------- */
/*
 * y[t][d] = sum_{s<k} w[t][s] * o[row_of[t*k+s]][d]; with w == NULL the rows
 * are summed unweighted (the weight was already applied to o).
 */
void oracle_combine(int T, int H, int k, const double* o, const int32_t* row_of,
                    const double* w, double* y) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int d = 0; d < H; ++d) {
            double acc = 0.0;
            for (int s = 0; s < k; ++s) {
                double v = o[(size_t)row_of[(size_t)t * k + s] * H + d];
                acc += w ? w[(size_t)t * k + s] * v : v;
            }
            y[(size_t)t * H + d] = acc;
        }
}
