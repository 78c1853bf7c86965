// a3 for float32 storage (the small correctness workload): the same grouped
// SwiGLU FFN over the same page format, on v_mfma_f32_32x32x2_f32.
//
// A block (256 threads, 4 wavefronts) owns 64 rows x two page tiles (256 raw
// columns).  Per 64-wide k-step the two 32 KiB weight tiles are copied linearly
// from their pages into LDS (they are stored as the LDS image) and the 64 x 64
// activation block goes to LDS row-major with a padded stride; one stage,
// barrier before and after the MFMAs.  Sized for clarity, not speed: float32
// only serves the tiny workload.
#include <mutex>

#include "moe_ffn_common.h"

namespace moe {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 64;
constexpr int kThreads = 256;
constexpr int kAStride = 68;                         // floats per LDS row of A (64 + pad, 16-byte aligned)
constexpr int kABytes = BM * kAStride * 4;           // 17408
constexpr int kTileBytes = 128 * 64 * 4;             // 32768
constexpr int kLdsBytes = kABytes + 2 * kTileBytes;  // 82944

// float offset of element (n, k) inside a page tile: 16-byte chunk c = k/4 sits at
// chunk position (c & 8) | ((c & 7) ^ ((n >> 1) & 7))
__device__ __forceinline__ int b_elem(int n, int k) {
    const int c = k >> 2;
    return n * 64 + ((((c & 8) | ((c & 7) ^ ((n >> 1) & 7)))) << 2) + (k & 3);
}

template <int MODE>
__global__ __launch_bounds__(kThreads) void ffn_gemm_f32(const GemmParams p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    float* sA = (float*)smem;
    float* sB = (float*)(smem + kABytes);
    const int tid = threadIdx.x, lane = tid & 63, wn = tid >> 6;

    const TileCoord tc = locate_tile<BM>(p);
    if (!tc.valid) return;
    const int e = tc.e, nt = tc.nt, row0 = tc.row0, rows_here = tc.rows_here;
    const int32_t* trow = p.table + (size_t)(p.table_row_mod ? e % p.table_row_mod : e) * p.ppe + p.group_base;
    const int pt0 = nt * 2;
    const int pt1 = (pt0 + 1 < p.n_page_tiles) ? pt0 + 1 : pt0;
    int bad = 0;

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int bn0 = (MODE == 0) ? wn * 32 + (lane & 31) : wn * 64 + (lane & 31);
    const int bn1 = (MODE == 0) ? 128 + wn * 32 + (lane & 31) : wn * 64 + 32 + (lane & 31);

    for (int kt = 0; kt < p.KT; ++kt) {
        const float4* b0 = (const float4*)tile_address(p, trow, (int64_t)pt0 * p.KT + kt, &bad);
        const float4* b1 = (const float4*)tile_address(p, trow, (int64_t)pt1 * p.KT + kt, &bad);
        for (int i = tid; i < 2048; i += kThreads) {
            ((float4*)sB)[i] = b0[i];
            ((float4*)sB)[2048 + i] = b1[i];
        }
        for (int i = tid; i < BM * 16; i += kThreads) {
            const int r = min(i >> 4, rows_here - 1), c4 = i & 15;
            const float4 v = *(const float4*)(p.A + (int64_t)(row0 + r) * p.lda_bytes + ((int64_t)kt * 64 + c4 * 4) * 4);
            *(float4*)(sA + (i >> 4) * kAStride + c4 * 4) = v;
        }
        __syncthreads();
#pragma unroll 4
        for (int kk = 0; kk < 32; ++kk) {
            const int k = 2 * kk + (lane >> 5);
            const float a0 = sA[(lane & 31) * kAStride + k];
            const float a1 = sA[(32 + (lane & 31)) * kAStride + k];
            const float v0 = sB[b_elem(bn0, k)];
            const float v1 = sB[b_elem(bn1, k)];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, v0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, v1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, v0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, v1, acc[1][1], 0, 0, 0);
        }
        __syncthreads();
    }

    const int col_l = lane & 31;
#pragma unroll
    for (int ms = 0; ms < 2; ++ms)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = ms * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
            if (row >= rows_here) continue;
            if (MODE == 0) {
                const float g = acc[ms][0][r], u = acc[ms][1][r];
                ((float*)p.out)[(int64_t)(row0 + row) * p.ldo + nt * 128 + wn * 32 + col_l] = g / (1.0f + expf(-g)) * u;
            } else {
                const float wgt = p.row_w ? p.row_w[row0 + row] : 1.0f;
#pragma unroll
                for (int ns = 0; ns < 2; ++ns) {
                    const int d = nt * 256 + wn * 64 + ns * 32 + col_l;
                    if (d < p.n_cols) ((float*)p.out)[(int64_t)(row0 + row) * p.ldo + d] = acc[ms][ns][r] * wgt;
                }
            }
        }
    if (bad && tid == 0 && p.status) atomicOr(p.status, 1);
}

template <int MODE>
int launch_mode(const GemmParams& p, int grid, hipStream_t st) {
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute((const void*)ffn_gemm_f32<MODE>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    });
    MOE_HIP_TRY(attr_err);
    hipLaunchKernelGGL((ffn_gemm_f32<MODE>), dim3(grid), dim3(kThreads), kLdsBytes, st, p);
    MOE_HIP_TRY(hipGetLastError());
    return MOE_OK;
}

}  // namespace

int launch_expert_ffn_f32(const moe_shape& s, const Geom& g, const FfnArgs& a, hipStream_t st) {
    const int R = s.T * s.k;
    GemmParams p{};
    fill_common(p, s, g, a);
    fill_gate_up(p, s, g, a);
    int rc = launch_mode<0>(p, gemm_grid(p.NT, R, BM, a.e_end - a.e_begin, p.chunked), st);
    if (rc != MOE_OK) return rc;
    if (a.mid_event) MOE_HIP_TRY(hipEventRecord(a.mid_event, st));
    fill_down(p, s, g, a);
    return launch_mode<1>(p, gemm_grid(p.NT, R, BM, a.e_end - a.e_begin, p.chunked), st);
}

int launch_expert_ffn(const moe_shape& s, const FfnArgs& a, hipStream_t st) {
    const Geom g = geometry(s);
    if (s.dtype == MOE_DTYPE_BF16) return launch_expert_ffn_bf16(s, g, a, st);
    return launch_expert_ffn_f32(s, g, a, st);
}

}  // namespace moe
