// The dense neighbours of the MoE FFN inside the paper's GPU tasks (its section 4.1): the
// post-attention task is the O projection followed by the MoE FFN, the pre-attention task a
// normalisation followed by the QKV projection.  Their weights are paged like the experts':
//
//   moe_linear       y = x W^T over paged W, on the matrix cores (the down-projection kernel of
//                    the expert FFN with a single row segment)
//   moe_add_rmsnorm  s = hidden + delta (the residual stream, f32);  x = bf16(s / rms(s) * gamma)
//   moe_cast_bf16    f32 -> bf16, round to nearest even
//   moe_post_attention / moe_pre_attention   the two tasks as sequences of the above and moe_layer
#include <algorithm>
#include <cstring>
#include <vector>

#include "moe_internal.h"

using namespace moe;

namespace {

__global__ void set_bounds_kernel(int32_t* offsets, int32_t T) {
    if (threadIdx.x == 0) {
        offsets[0] = 0;
        offsets[1] = T;
    }
}

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;      // NaN stays NaN
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;                        // round to nearest, ties to even
}

// One block per row.  s = hidden + delta is written as f32 and kept in registers for the second
// pass (H <= 256 * 4 * kMaxVec elements), so the row is read once.
constexpr int kNormThreads = 256;
constexpr int kMaxVec = 8;     // float4 per thread: H <= 8192

__global__ __launch_bounds__(kNormThreads) void add_rmsnorm_kernel(const float4* __restrict__ hidden, const float4* __restrict__ delta,
                                                                   const float4* __restrict__ gamma, float eps, int row_vec,
                                                                   float4* __restrict__ hidden_out, uint2* __restrict__ x_out) {
    __shared__ float part[kNormThreads / 64];
    const size_t row = (size_t)blockIdx.x * row_vec;
    float4 v[kMaxVec];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < kMaxVec; ++i) {
        const int c = threadIdx.x + i * kNormThreads;
        if (c < row_vec) {
            float4 a = delta[row + c];
            if (hidden) {
                const float4 h = hidden[row + c];
                a.x += h.x; a.y += h.y; a.z += h.z; a.w += h.w;
            }
            v[i] = a;
            if (hidden_out) hidden_out[row + c] = a;
            ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
        }
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) ss += __shfl_xor(ss, m, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float total = (part[0] + part[1]) + (part[2] + part[3]);
    const float scale = rsqrtf(total / (float)(row_vec * 4) + eps);
#pragma unroll
    for (int i = 0; i < kMaxVec; ++i) {
        const int c = threadIdx.x + i * kNormThreads;
        if (c < row_vec) {
            const float4 g = gamma[c];
            const float4 a = v[i];
            uint2 o;
            o.x = f32_to_bf16_bits(a.x * scale * g.x) | (f32_to_bf16_bits(a.y * scale * g.y) << 16);
            o.y = f32_to_bf16_bits(a.z * scale * g.z) | (f32_to_bf16_bits(a.w * scale * g.w) << 16);
            x_out[row + c] = o;
        }
    }
}

__global__ __launch_bounds__(256) void cast_bf16_kernel(const float4* __restrict__ in, uint2* __restrict__ out, int64_t n_vec) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += (int64_t)gridDim.x * 256) {
        const float4 a = in[i];
        uint2 o;
        o.x = f32_to_bf16_bits(a.x) | (f32_to_bf16_bits(a.y) << 16);
        o.y = f32_to_bf16_bits(a.z) | (f32_to_bf16_bits(a.w) << 16);
        out[i] = o;
    }
}

int enqueue_linear(const moe_linear_shape& s, const void* x, const int32_t* table, const void* pool, int64_t pool_pages,
                   float* out, void* workspace, int32_t* status, hipStream_t st) {
    int32_t* bounds = (int32_t*)workspace;
    hipLaunchKernelGGL(set_bounds_kernel, dim3(1), dim3(64), 0, st, bounds, s.T);
    MOE_HIP_TRY(hipGetLastError());
    LinearArgs a{x, s.T, s.K, s.N, bounds, table, (const char*)pool, pool_pages, s.page_bytes, linear_pages(s), out, status};
    return launch_linear_bf16(a, st);
}

int enqueue_add_rmsnorm(int32_t T, int32_t H, const float* hidden, const float* delta, const float* gamma, float eps,
                        float* hidden_out, void* x_out, hipStream_t st) {
    hipLaunchKernelGGL(add_rmsnorm_kernel, dim3(T), dim3(kNormThreads), 0, st, (const float4*)hidden, (const float4*)delta,
                       (const float4*)gamma, eps, H / 4, (float4*)hidden_out, (uint2*)x_out);
    MOE_HIP_TRY(hipGetLastError());
    return MOE_OK;
}

}  // namespace

extern "C" {

int moe_linear(const moe_linear_shape* s, const void* x, const int32_t* page_table, const void* page_pool,
               int64_t pool_pages, float* out, void* workspace, size_t workspace_bytes, int32_t* status, void* stream) {
    int rc = validate_linear(s);
    if (rc != MOE_OK) return rc;
    if (s->T == 0) return MOE_OK;
    if (!x || !page_table || !page_pool || !out || !workspace || pool_pages <= 0) return MOE_ERR_INVALID_ARG;
    if (workspace_bytes < MOE_LINEAR_WORKSPACE_BYTES) return MOE_ERR_WORKSPACE_TOO_SMALL;
    return enqueue_linear(*s, x, page_table, page_pool, pool_pages, out, workspace, status, (hipStream_t)stream);
}

int moe_add_rmsnorm(int32_t T, int32_t H, const float* hidden, const float* delta, const float* gamma, float eps,
                    float* hidden_out, void* x_out, void* stream) {
    if (T < 0 || H <= 0 || H % 4 != 0 || H > 4 * kNormThreads * kMaxVec || !(eps >= 0.f)) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    if (!delta || !gamma || !x_out) return MOE_ERR_INVALID_ARG;
    return enqueue_add_rmsnorm(T, H, hidden, delta, gamma, eps, hidden_out, x_out, (hipStream_t)stream);
}

int moe_cast_bf16(int64_t n, const float* in, void* out, void* stream) {
    if (n < 0 || n % 4 != 0) return MOE_ERR_INVALID_ARG;
    if (n == 0) return MOE_OK;
    if (!in || !out) return MOE_ERR_INVALID_ARG;
    const int64_t n_vec = n / 4;
    const int grid = (int)std::min<int64_t>((n_vec + 255) / 256, 65536);
    hipLaunchKernelGGL(cast_bf16_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const float4*)in, (uint2*)out, n_vec);
    MOE_HIP_TRY(hipGetLastError());
    return MOE_OK;
}

int moe_post_attention(const moe_shape* s, const moe_linear_shape* o_proj, const void* attn, const float* hidden,
                       const int32_t* o_table, const float* norm_gamma, float eps, const void* Wr, const float* bias,
                       const int32_t* page_table, const void* page_pool, int64_t pool_pages,
                       float* hidden_mid, void* x_moe, float* y, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = validate_shape(s);
    if (rc != MOE_OK) return rc;
    rc = validate_linear(o_proj);
    if (rc != MOE_OK) return rc;
    if (s->dtype != MOE_DTYPE_BF16) return MOE_ERR_UNSUPPORTED_DTYPE;
    if (o_proj->T != s->T || o_proj->N != s->H || o_proj->page_bytes != s->page_bytes || s->H > 4 * kNormThreads * kMaxVec)
        return MOE_ERR_INVALID_ARG;
    if (s->T == 0) return MOE_OK;
    if (!attn || !hidden || !o_table || !norm_gamma || !Wr || !page_table || !page_pool || !hidden_mid || !x_moe || !y ||
        !workspace || pool_pages <= 0 || !(eps >= 0.f))
        return MOE_ERR_INVALID_ARG;
    // workspace: [the MoE layer's workspace][bounds of the linear][O-projection output f32 [T][H]]
    const size_t layer_bytes = (layer_workspace_bytes(*s) + 255) / 256 * 256;
    const size_t need = layer_bytes + 256 + (size_t)s->T * s->H * 4;
    if (workspace_bytes < need) return MOE_ERR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)workspace & 255) != 0) return MOE_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    char* ws = (char*)workspace;
    float* o = (float*)(ws + layer_bytes + 256);
    rc = enqueue_linear(*o_proj, attn, o_table, page_pool, pool_pages, o, ws + layer_bytes, nullptr, st);
    if (rc != MOE_OK) return rc;
    rc = enqueue_add_rmsnorm(s->T, s->H, hidden, o, norm_gamma, eps, hidden_mid, x_moe, st);
    if (rc != MOE_OK) return rc;
    return layer_resident(*s, x_moe, Wr, bias, page_table, (const char*)page_pool, pool_pages, y, ws, st);
}

int moe_pre_attention(const moe_linear_shape* qkv_proj, const float* hidden, const float* delta, const float* norm_gamma,
                      float eps, const int32_t* qkv_table, const void* page_pool, int64_t pool_pages,
                      float* hidden_out, void* x_norm, float* qkv, void* qkv_bf16, void* workspace, size_t workspace_bytes,
                      void* stream) {
    int rc = validate_linear(qkv_proj);
    if (rc != MOE_OK) return rc;
    if (qkv_proj->K > 4 * kNormThreads * kMaxVec) return MOE_ERR_INVALID_ARG;
    if (qkv_proj->T == 0) return MOE_OK;
    if (!delta || !norm_gamma || !qkv_table || !page_pool || !hidden_out || !x_norm || !qkv || !workspace || pool_pages <= 0 ||
        !(eps >= 0.f))
        return MOE_ERR_INVALID_ARG;
    if (workspace_bytes < MOE_LINEAR_WORKSPACE_BYTES) return MOE_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)stream;
    rc = enqueue_add_rmsnorm(qkv_proj->T, qkv_proj->K, hidden, delta, norm_gamma, eps, hidden_out, x_norm, st);
    if (rc != MOE_OK) return rc;
    rc = enqueue_linear(*qkv_proj, x_norm, qkv_table, page_pool, pool_pages, qkv, workspace, nullptr, st);
    if (rc != MOE_OK) return rc;
    if (qkv_bf16) return moe_cast_bf16((int64_t)qkv_proj->T * qkv_proj->N, qkv, qkv_bf16, stream);
    return MOE_OK;
}

int moe_post_attention_workspace_bytes(const moe_shape* s, size_t* bytes) {
    int rc = validate_shape(s);
    if (rc != MOE_OK) return rc;
    if (!bytes) return MOE_ERR_INVALID_ARG;
    *bytes = (layer_workspace_bytes(*s) + 255) / 256 * 256 + 256 + (size_t)s->T * s->H * 4;
    return MOE_OK;
}

}  // extern "C"
