// a1. Router: logits = x Wr^T (+bias), top-k by descending logit (ties to the
// lower expert index), softmax over the k selected logits.
//
// The product is a tall-skinny contraction (E <= 64 outputs per token), bound
// by reading x from HBM once.
//
// bf16 (route_mfma_kernel): a block of 16 wavefronts (8 beyond 32 experts) owns 16 tokens.  The
// reduction over H is cut into units of 64 elements (one 128-byte line per
// token), dealt round robin to the wavefronts; for a unit, lane (r = lane % 16,
// g = lane / 16) loads bytes g*16 .. g*16+15 of both halves of token r's line and
// of expert row r's line (zero for rows >= E), and two 16x16x32 MFMAs add the
// unit to a 16 x 16 f32 tile per 16 experts.  Which element of the line meets
// which k index of the MFMA does not matter as long as x and Wr use the same
// mapping.  Several units' loads are issued before their MFMAs to cover the
// HBM latency; with 16 wavefronts a row of 4096 elements is a single such batch
// per wavefront.  The wavefronts' tiles are added through LDS.
//
// f32 (route_kernel): on the vector ALUs.  A block of four wavefronts owns
// TPB = 64 / EP tokens (EP = experts padded to 8, 16, 32 or 64) and splits the
// reduction over its 256 lanes: every lane takes 8 consecutive elements per
// step and keeps TPB * EP = 64 float partial sums, folded over the lanes of a
// wavefront with a halving butterfly (63 cross-lane moves: lane j ends up with
// the sum of value j) and over the four wavefronts through LDS.
//
// In both, the selection and the softmax are done by one lane per token.
#include "moe_internal.h"

namespace moe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void load8(const float* base, size_t elem, float (&v)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(base + elem);
    const float4 b = *reinterpret_cast<const float4*>(base + elem + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

// Top-k of lg[0..E) by descending value (strict >: the lower index keeps a tie) and the softmax
// over the selected values, for token tok.
__device__ __forceinline__ void select_top_k(const float* lg, int E, int k, int tok, int32_t* __restrict__ ids,
                                             float* __restrict__ w) {
    uint64_t taken = 0;
    float first = 0.f, den = 0.f;
    for (int s = 0; s < k; ++s) {
        int best = -1;
        float bv = 0.f;
        for (int e = 0; e < E; ++e) {
            const bool free_e = !((taken >> e) & 1ull);
            const float v = lg[e];
            if (free_e && (best < 0 || v > bv)) {
                best = e;
                bv = v;
            }
        }
        taken |= 1ull << best;
        if (s == 0) first = bv;
        const float p = __expf(bv - first);
        den += p;
        ids[(size_t)tok * k + s] = best;
        w[(size_t)tok * k + s] = p;                           // normalised below
    }
    const float inv = 1.0f / den;
    for (int s = 0; s < k; ++s) w[(size_t)tok * k + s] *= inv;
}

// NE: 16-expert tiles (experts padded to 16, 32 or 64); NW: wavefronts of a block.
template <int NE, int NW>
__global__ __launch_bounds__(NW * 64) void route_mfma_kernel(const char* __restrict__ x, const char* __restrict__ Wr,
                                                         const float* __restrict__ bias, int32_t* __restrict__ ids,
                                                         float* __restrict__ w, float* __restrict__ logits,
                                                         int T, int H, int E, int k) {
    constexpr int EP = NE * 16;
    constexpr int UB = NE <= 2 ? 4 : 2;                      // units whose loads are in flight together
    __shared__ float s_part[NW][16][EP];
    __shared__ float s_logit[16][EP];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int t0 = blockIdx.x * 16;
    const int r = lane & 15, g = lane >> 4;
    const size_t row_bytes = (size_t)H * 2;
    const char* xa = x + (size_t)min(t0 + r, T - 1) * row_bytes + g * 16;      // rows past the end repeat the last token
    const char* wb[NE];
    bool wv[NE];
#pragma unroll
    for (int n = 0; n < NE; ++n) {
        const int e = n * 16 + r;
        wv[n] = e < E;
        wb[n] = Wr + (size_t)min(e, E - 1) * row_bytes + g * 16;
    }
    f32x4 acc[NE];
#pragma unroll
    for (int n = 0; n < NE; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};
    const bf16x8 zero = {};
    const int units = H >> 6;
    for (int ub = wave; ub < units; ub += NW * UB) {
        bf16x8 a[UB][2], b[NE][UB][2];
#pragma unroll
        for (int j = 0; j < UB; ++j) {
            const int u = ub + NW * j;
            const bool ok = u < units;                         // the same for the whole wavefront
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const size_t off = (size_t)u * 128 + h * 64;
                a[j][h] = ok ? *reinterpret_cast<const bf16x8*>(xa + off) : zero;
#pragma unroll
                for (int n = 0; n < NE; ++n) b[n][j][h] = (ok && wv[n]) ? *reinterpret_cast<const bf16x8*>(wb[n] + off) : zero;
            }
        }
#pragma unroll
        for (int j = 0; j < UB; ++j)
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int n = 0; n < NE; ++n) acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j][h], b[n][j][h], acc[n], 0, 0, 0);
    }
    // lane (r, g) holds tokens g*4 .. g*4+3 of expert n*16 + r
#pragma unroll
    for (int n = 0; n < NE; ++n)
#pragma unroll
        for (int i = 0; i < 4; ++i) s_part[wave][g * 4 + i][n * 16 + r] = acc[n][i];
    __syncthreads();
    for (int v = threadIdx.x; v < 16 * EP; v += NW * 64) {
        const int t = v / EP, e = v % EP;
        float sum = 0.f;
#pragma unroll
        for (int q = 0; q < NW; ++q) sum += s_part[q][t][e];
        if (bias != nullptr && e < E) sum += bias[e];
        s_logit[t][e] = sum;
        if (logits && e < E && t0 + t < T) logits[(size_t)(t0 + t) * E + e] = sum;
    }
    __syncthreads();
    if (threadIdx.x < 16 && t0 + threadIdx.x < T) select_top_k(s_logit[threadIdx.x], E, k, t0 + threadIdx.x, ids, w);
}

// EP: experts padded to a compile-time bound (a power of two, 8..64).
template <int EP>
__global__ __launch_bounds__(256) void route_kernel(const float* __restrict__ x, const float* __restrict__ Wr,
                                                    const float* __restrict__ bias, int32_t* __restrict__ ids,
                                                    float* __restrict__ w, float* __restrict__ logits,
                                                    int T, int H, int E, int k) {
    constexpr int TPB = 64 / EP;                      // tokens per block
    __shared__ float s_part[4][64];
    __shared__ float s_logit[64];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int t0 = blockIdx.x * TPB;

    float acc[64];                                    // value v = t * EP + e
#pragma unroll
    for (int v = 0; v < 64; ++v) acc[v] = 0.f;

    const int chunks = H >> 3;
    for (int c = threadIdx.x; c < chunks; c += 256) {
        float xv[TPB][8];
#pragma unroll
        for (int t = 0; t < TPB; ++t) {
            const int tt = min(t0 + t, T - 1);           // rows past the end repeat the last token
            load8(x, (size_t)tt * H + (size_t)c * 8, xv[t]);
        }
#pragma unroll
        for (int e = 0; e < EP; ++e) {
            if (e < E) {
                float wv[8];
                load8(Wr, (size_t)e * H + (size_t)c * 8, wv);
#pragma unroll
                for (int t = 0; t < TPB; ++t)
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc[t * EP + e] = fmaf(xv[t][i], wv[i], acc[t * EP + e]);
            }
        }
    }
    // halving butterfly over the lanes: in the step with mask m a lane keeps the half of its
    // values that its bit m selects and receives the partner's sums for that half
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        const bool upper = (lane & m) != 0;
#pragma unroll
        for (int i = 0; i < m; ++i) {
            const float keep = upper ? acc[i + m] : acc[i];
            const float give = upper ? acc[i] : acc[i + m];
            acc[i] = keep + __shfl_xor(give, m, 64);
        }
    }
    s_part[wave][lane] = acc[0];                      // lane j: value j summed over this wavefront's part of H
    __syncthreads();
    if (threadIdx.x < 64) {
        const int v = threadIdx.x, t = v / EP, e = v % EP;
        float sum = (s_part[0][v] + s_part[1][v]) + (s_part[2][v] + s_part[3][v]);
        if (bias != nullptr && e < E) sum += bias[e];
        s_logit[v] = sum;
        if (logits && e < E && t0 + t < T) logits[(size_t)(t0 + t) * E + e] = sum;
    }
    __syncthreads();
    if (threadIdx.x < TPB && t0 + threadIdx.x < T) select_top_k(s_logit + threadIdx.x * EP, E, k, t0 + threadIdx.x, ids, w);
}

template <int EP>
int launch_f32(const moe_shape& s, const void* x, const void* Wr, const float* bias, int32_t* ids, float* w,
               float* logits, hipStream_t st) {
    constexpr int tokens_per_block = 64 / EP;
    const dim3 grid((s.T + tokens_per_block - 1) / tokens_per_block), block(256);
    hipLaunchKernelGGL((route_kernel<EP>), grid, block, 0, st, (const float*)x, (const float*)Wr, bias, ids, w, logits, s.T,
                       s.H, s.E, s.k);
    MOE_HIP_TRY(hipGetLastError());
    return MOE_OK;
}

template <int NE, int NW>
int launch_bf16(const moe_shape& s, const void* x, const void* Wr, const float* bias, int32_t* ids, float* w,
                float* logits, hipStream_t st) {
    const dim3 grid((s.T + 15) / 16), block(NW * 64);
    hipLaunchKernelGGL((route_mfma_kernel<NE, NW>), grid, block, 0, st, (const char*)x, (const char*)Wr, bias, ids, w, logits,
                       s.T, s.H, s.E, s.k);
    MOE_HIP_TRY(hipGetLastError());
    return MOE_OK;
}

}  // namespace

int launch_route(const moe_shape& s, const void* x, const void* Wr, const float* bias, int32_t* ids, float* w,
                 float* logits, hipStream_t st) {
    if (s.T == 0) return MOE_OK;
    if (s.dtype == MOE_DTYPE_BF16) {
        if (s.E <= 16) return launch_bf16<1, 16>(s, x, Wr, bias, ids, w, logits, st);
        if (s.E <= 32) return launch_bf16<2, 16>(s, x, Wr, bias, ids, w, logits, st);
        return launch_bf16<4, 8>(s, x, Wr, bias, ids, w, logits, st);
    }
    if (s.E <= 8) return launch_f32<8>(s, x, Wr, bias, ids, w, logits, st);
    if (s.E <= 16) return launch_f32<16>(s, x, Wr, bias, ids, w, logits, st);
    if (s.E <= 32) return launch_f32<32>(s, x, Wr, bias, ids, w, logits, st);
    return launch_f32<64>(s, x, Wr, bias, ids, w, logits, st);
}

}  // namespace moe
