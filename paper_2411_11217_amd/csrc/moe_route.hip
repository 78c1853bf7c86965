// a1. Router: logits = x Wr^T (+bias), top-k by descending logit (ties to the
// lower expert index), softmax over the k selected logits.
//
// The product is a tall-skinny contraction (E <= 64 outputs per token), bound
// by reading x from HBM once, so it runs on the vector ALUs.  A block of four
// wavefronts owns TPB = 64 / EP tokens (EP = experts padded to 8, 16, 32 or 64)
// and splits the reduction over its 256 lanes: every lane takes 8 consecutive
// elements per step (one 16-byte load per token for bf16), so one step of the
// block reads 4 KiB of every token row, and keeps TPB * EP = 64 float partial
// sums.  Many small blocks keep enough loads in flight to cover the HBM latency;
// Wr is read once per block (from L2).  The 64 sums are folded over the lanes
// of a wavefront with a halving butterfly (63 cross-lane moves: lane j ends up
// with the sum of value j), over the four wavefronts through LDS, and the
// selection and the softmax are done by one lane per token.
#include "moe_internal.h"

namespace moe {
namespace {

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

template <bool BF16>
__device__ __forceinline__ void load8(const void* base, size_t elem, float (&v)[8]) {
    if constexpr (BF16) {
        const uint4 q = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(base) + elem);
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = bf16_bits_to_f32(w[i] & 0xffffu);
            v[2 * i + 1] = bf16_bits_to_f32(w[i] >> 16);
        }
    } else {
        const float4 a = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + elem);
        const float4 b = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + elem + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
}

// EP: experts padded to a compile-time bound (a power of two, 8..64).
template <int EP, bool BF16>
__global__ __launch_bounds__(256) void route_kernel(const void* __restrict__ x, const void* __restrict__ Wr,
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
            load8<BF16>(x, (size_t)tt * H + (size_t)c * 8, xv[t]);
        }
#pragma unroll
        for (int e = 0; e < EP; ++e) {
            if (e < E) {
                float wv[8];
                load8<BF16>(Wr, (size_t)e * H + (size_t)c * 8, wv);
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
    if (threadIdx.x < TPB && t0 + threadIdx.x < T) {
        const int tok = t0 + threadIdx.x;
        const float* lg = s_logit + threadIdx.x * EP;
        uint64_t taken = 0;
        float first = 0.f, den = 0.f;
        for (int s = 0; s < k; ++s) {
            int best = -1;
            float bv = 0.f;
            for (int e = 0; e < E; ++e) {
                const bool free_e = !((taken >> e) & 1ull);
                const float v = lg[e];
                if (free_e && (best < 0 || v > bv)) {             // strict >: the lower index keeps a tie
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
}

template <int EP>
int launch_t(const moe_shape& s, const void* x, const void* Wr, const float* bias, int32_t* ids, float* w,
             float* logits, hipStream_t st) {
    constexpr int tokens_per_block = 64 / EP;
    const dim3 grid((s.T + tokens_per_block - 1) / tokens_per_block), block(256);
    if (s.dtype == MOE_DTYPE_BF16)
        hipLaunchKernelGGL((route_kernel<EP, true>), grid, block, 0, st, x, Wr, bias, ids, w, logits, s.T, s.H, s.E, s.k);
    else
        hipLaunchKernelGGL((route_kernel<EP, false>), grid, block, 0, st, x, Wr, bias, ids, w, logits, s.T, s.H, s.E, s.k);
    MOE_HIP_TRY(hipGetLastError());
    return MOE_OK;
}

}  // namespace

int launch_route(const moe_shape& s, const void* x, const void* Wr, const float* bias, int32_t* ids, float* w,
                 float* logits, hipStream_t st) {
    if (s.T == 0) return MOE_OK;
    if (s.E <= 8) return launch_t<8>(s, x, Wr, bias, ids, w, logits, st);
    if (s.E <= 16) return launch_t<16>(s, x, Wr, bias, ids, w, logits, st);
    if (s.E <= 32) return launch_t<32>(s, x, Wr, bias, ids, w, logits, st);
    return launch_t<64>(s, x, Wr, bias, ids, w, logits, st);
}

}  // namespace moe
