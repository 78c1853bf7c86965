// a1. Router: logits = x Wr^T (+bias), top-k by descending logit (ties to the
// lower expert index), softmax over the k selected logits.
//
// The product is a tall-skinny contraction (E <= 64 outputs per token), bound
// by reading x from HBM once, so it runs on the vector ALUs: one wavefront
// owns TPW tokens, every lane takes 8 consecutive reduction elements per step
// (one 16-byte load per token for bf16), keeps TPW*EP float partial sums in
// registers and the wavefront folds them with a butterfly of cross-lane adds.
// Selection and the softmax are then done by one lane per token.
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

// EP: experts padded to a compile-time bound; TPW: tokens per wavefront.
template <int EP, int TPW, bool BF16>
__global__ __launch_bounds__(256) void route_kernel(const void* __restrict__ x, const void* __restrict__ Wr,
                                                    const float* __restrict__ bias, int32_t* __restrict__ ids,
                                                    float* __restrict__ w, float* __restrict__ logits,
                                                    int T, int H, int E, int k) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int t0 = (blockIdx.x * 4 + wave) * TPW;
    if (t0 >= T) return;

    float acc[TPW][EP];
#pragma unroll
    for (int t = 0; t < TPW; ++t)
#pragma unroll
        for (int e = 0; e < EP; ++e) acc[t][e] = 0.f;

    const int chunks = H >> 3;
    for (int c = lane; c < chunks; c += 64) {
        float xv[TPW][8];
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            const int tt = min(t0 + t, T - 1);           // rows past the end repeat the last token
            load8<BF16>(x, (size_t)tt * H + (size_t)c * 8, xv[t]);
        }
#pragma unroll
        for (int e = 0; e < EP; ++e) {
            if (e < E) {
                float wv[8];
                load8<BF16>(Wr, (size_t)e * H + (size_t)c * 8, wv);
#pragma unroll
                for (int t = 0; t < TPW; ++t)
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc[t][e] = fmaf(xv[t][i], wv[i], acc[t][e]);
            }
        }
    }
    // butterfly: afterwards every lane holds every sum
#pragma unroll
    for (int t = 0; t < TPW; ++t)
#pragma unroll
        for (int e = 0; e < EP; ++e) {
            float v = acc[t][e];
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
            acc[t][e] = v + ((bias != nullptr && e < E) ? bias[e] : 0.f);
        }

#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        if (lane != t || t0 + t >= T) continue;
        const int tok = t0 + t;
        if (logits) {
#pragma unroll
            for (int e = 0; e < EP; ++e)
                if (e < E) logits[(size_t)tok * E + e] = acc[t][e];
        }
        uint64_t taken = 0;
        float first = 0.f, den = 0.f;
        for (int s = 0; s < k; ++s) {
            int best = -1;
            float bv = 0.f;
#pragma unroll
            for (int e = 0; e < EP; ++e) {
                const bool free_e = e < E && !((taken >> e) & 1ull);
                if (free_e && (best < 0 || acc[t][e] > bv)) {     // strict >: the lower index keeps a tie
                    best = e;
                    bv = acc[t][e];
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

template <int EP, int TPW>
int launch_t(const moe_shape& s, const void* x, const void* Wr, const float* bias, int32_t* ids, float* w,
             float* logits, hipStream_t st) {
    const int tokens_per_block = 4 * TPW;
    const dim3 grid((s.T + tokens_per_block - 1) / tokens_per_block), block(256);
    if (s.dtype == MOE_DTYPE_BF16)
        hipLaunchKernelGGL((route_kernel<EP, TPW, true>), grid, block, 0, st, x, Wr, bias, ids, w, logits, s.T, s.H, s.E, s.k);
    else
        hipLaunchKernelGGL((route_kernel<EP, TPW, false>), grid, block, 0, st, x, Wr, bias, ids, w, logits, s.T, s.H, s.E, s.k);
    MOE_HIP_TRY(hipGetLastError());
    return MOE_OK;
}

}  // namespace

int launch_route(const moe_shape& s, const void* x, const void* Wr, const float* bias, int32_t* ids, float* w,
                 float* logits, hipStream_t st) {
    if (s.E <= 8) return launch_t<8, 4>(s, x, Wr, bias, ids, w, logits, st);
    if (s.E <= 16) return launch_t<16, 4>(s, x, Wr, bias, ids, w, logits, st);
    if (s.E <= 32) return launch_t<32, 2>(s, x, Wr, bias, ids, w, logits, st);
    return launch_t<64, 1>(s, x, Wr, bias, ids, w, logits, st);
}

}  // namespace moe
