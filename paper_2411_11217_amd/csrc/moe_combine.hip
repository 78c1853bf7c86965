// a4. Un-permute and combine: y[t] = sum_slot w[t][slot] * out[row_of[t*k+slot]].
// Pure HBM traffic (read R*H floats, write T*H floats): one block per token,
// 16-byte loads along the row, the k rows of a token summed in slot order so the
// result does not depend on scheduling.
#include "moe_internal.h"

namespace moe {
namespace {

__global__ __launch_bounds__(256) void combine_kernel(const float4* __restrict__ out, const int32_t* __restrict__ row_of,
                                                      const float* __restrict__ topk_w, int k, int R, int row_vec,
                                                      float4* __restrict__ y) {
    const int t = blockIdx.x;
    __shared__ int32_t rows[MOE_MAX_EXPERTS];
    __shared__ float wts[MOE_MAX_EXPERTS];
    if (threadIdx.x < k) {
        const int r = row_of[(size_t)t * k + threadIdx.x];
        rows[threadIdx.x] = min(max(r, 0), R - 1);          // never leaves the buffer
        wts[threadIdx.x] = topk_w ? topk_w[(size_t)t * k + threadIdx.x] : 1.0f;
    }
    __syncthreads();
    for (int c = threadIdx.x; c < row_vec; c += 256) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int s = 0; s < k; ++s) {
            const float4 v = out[(size_t)rows[s] * row_vec + c];
            const float ws = wts[s];
            acc.x = fmaf(ws, v.x, acc.x);
            acc.y = fmaf(ws, v.y, acc.y);
            acc.z = fmaf(ws, v.z, acc.z);
            acc.w = fmaf(ws, v.w, acc.w);
        }
        y[(size_t)t * row_vec + c] = acc;
    }
}

}  // namespace

int launch_combine(const moe_shape& s, const float* out, const int32_t* row_of, const float* topk_w, float* y,
                   hipStream_t st) {
    hipLaunchKernelGGL(combine_kernel, dim3(s.T), dim3(256), 0, st, (const float4*)out, row_of, topk_w, s.k,
                       s.T * s.k, s.H / 4, (float4*)y);
    MOE_HIP_TRY(hipGetLastError());
    return MOE_OK;
}

}  // namespace moe
