// a3. Grouped SwiGLU expert FFN, bf16 operands, fp32 accumulation, on the CDNA4
// matrix cores (v_mfma_f32_32x32x16_bf16), weights read through the page table.
//
// Two launches of one kernel template:
//   MODE 0 (gate/up):  [g | u] = x_perm . [W1_e ; W3_e]^T,  h = bf16(silu(g) * u)
//   MODE 1 (down):     out     = h . W2_e^T  (* row weight)
//
// Work decomposition.  A block owns a 256-row x 256-column piece of one expert's
// output.  Its columns are two page tiles (128 output features each): for MODE 0
// the W1 tile and the W3 tile of the same 128 features, so gate and up value of
// an element meet in the same lane and the SwiGLU product is formed in
// registers; for MODE 1 two neighbouring tiles of W2.  Row tiles never cross an
// expert boundary; the block finds (expert, row tile, column tile) from the
// offsets array alone, so the host needs no knowledge of the routing result.
// Consecutive tile numbers run over the row tiles of one column tile first (they
// share the weight tiles) and are dealt to the 8 XCDs in contiguous chunks, since
// each XCD has a private L2 and blocks go to XCDs round-robin.
//
// Data movement.  512 threads = 8 wavefronts (2 per SIMD).  Per 64-wide k-step a
// stage of 64 KiB is filled: 256 rows x 128 bytes of activations and two 16 KiB
// weight tiles.  All of it goes global -> LDS directly (global_load_lds, 16 bytes
// per lane), no registers in between.  Weight tiles are stored in the pages as
// the exact LDS image (16-byte chunks XOR-swizzled by row & 7), so their copy is
// linear; activation rows are row-major in HBM and the swizzle is applied by
// choosing which chunk each lane fetches.  With that layout every ds_read_b128
// of an MFMA operand is conflict free.  Two stages are double buffered: the
// loads of step kt+1 are in flight while the MFMAs of step kt run, with one
// barrier per step.
//
// Wavefront w computes rows (w / 4) * 128 .. +127 and, of the 256 columns, for
// MODE 0 columns (w % 4) * 32 .. +31 of both tiles, for MODE 1 columns
// (w % 4) * 64 .. +63: 4 x 2 MFMA tiles of 32 x 32, 128 accumulator registers.
#include <mutex>

#include "moe_ffn_common.h"

namespace moe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

constexpr int BM = 256;
constexpr int kThreads = 512;
constexpr int kStageA = 32768;               // 256 rows x 128 B
constexpr int kStageBytes = 65536;           // + two 16 KiB weight tiles
constexpr int kLdsBytes = 2 * kStageBytes;

__device__ __forceinline__ float silu_mul(float g, float u) {
    return g * __frcp_rn(1.0f + __expf(-g)) * u;
}

template <int MODE>
__global__ __launch_bounds__(kThreads) void ffn_gemm_bf16(const GemmParams p) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;

    // ---- which tile is mine -------------------------------------------------
    const TileCoord tc = locate_tile<BM>(p);
    if (!tc.valid) return;
    const int e = tc.e, nt = tc.nt, row0 = tc.row0, rows_here = tc.rows_here;

    // ---- weight tiles through the page table -------------------------------------
    const int32_t* trow = p.table + (size_t)(p.table_row_mod ? e % p.table_row_mod : e) * p.ppe + p.group_base;
    const int pt0 = nt * 2;
    const int pt1 = (pt0 + 1 < p.n_page_tiles) ? pt0 + 1 : pt0;   // odd tile count: the second half is masked
    int bad = 0;
    auto tile_addr = [&](int64_t ti) -> const char* { return tile_address(p, trow, ti, &bad); };

    // ---- per-lane sources of the activation rows ------------------------------------
    // load instruction q = i*8 + wave fills LDS rows q*8 .. q*8+7 (1 KiB); lane j holds
    // row q*8 + j/8 at chunk position j%8, i.e. global chunk (j%8) ^ (row & 7)
    const char* a_src[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = min((i * 8 + wave) * 8 + (lane >> 3), rows_here - 1);   // rows past the tail repeat the last row
        const int c = (lane & 7) ^ (lane >> 3);
        a_src[i] = p.A + (int64_t)(row0 + r) * p.lda_bytes + c * 16;
    }

    auto issue = [&](int stage, int kt) {
        char* sA = smem + stage * kStageBytes;
        char* sB = sA + kStageA;
        const char* b0 = tile_addr((int64_t)pt0 * p.KT + kt);
        const char* b1 = tile_addr((int64_t)pt1 * p.KT + kt);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int q = i * 8 + wave;
            __builtin_amdgcn_global_load_lds((gptr_t)(a_src[i] + (int64_t)kt * 128), (lptr_t)(sA + q * 1024), 16, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int q = i * 8 + wave;                     // q / 16 = i / 2: first two fill tile 0, last two tile 1
            const char* src = (i < 2 ? b0 : b1) + (q & 15) * 1024 + lane * 16;
            __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)(sB + q * 1024), 16, 0, 0);
        }
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int c0 = (lane >> 5) ^ (lane & 7);
    const int a_row_base = wm * 128;
    const int b_row0 = (MODE == 0) ? wn * 32 : wn * 64;
    const int b_row1 = (MODE == 0) ? 128 + wn * 32 : wn * 64 + 32;

    auto compute = [&](int stage) {
        const char* sA = smem + stage * kStageBytes;
        const char* sB = sA + kStageA;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int off = (lane & 31) * 128 + ((c0 ^ (2 * ks)) << 4);
            bf16x8 a[4], b[2];
#pragma unroll
            for (int ms = 0; ms < 4; ++ms) a[ms] = *(const bf16x8*)(sA + off + (a_row_base + ms * 32) * 128);
            b[0] = *(const bf16x8*)(sB + off + b_row0 * 128);
            b[1] = *(const bf16x8*)(sB + off + b_row1 * 128);
#pragma unroll
            for (int ms = 0; ms < 4; ++ms)
#pragma unroll
                for (int ns = 0; ns < 2; ++ns)
                    acc[ms][ns] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ms], b[ns], acc[ms][ns], 0, 0, 0);
        }
    };

    if (p.variant == 0) {
        // plain schedule: load a stage, wait, compute, and only then load the next
        for (int kt = 0; kt < p.KT; ++kt) {
            issue(0, kt);
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): my direct-to-LDS loads have landed
            __syncthreads();
            compute(0);
            __syncthreads();
        }
    } else {
        issue(0, 0);
        for (int kt = 0; kt < p.KT; ++kt) {
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
            __syncthreads();                      // stage kt complete for everyone; stage kt-1 no longer read
            if (kt + 1 < p.KT) issue((kt + 1) & 1, kt + 1);
            compute(kt & 1);
        }
    }

    // ---- epilogue ---------------------------------------------------------------------
    // accumulator register r of lane l in MFMA tile (ms, ns) is the element at
    // row ms*32 + (r/4)*8 + (l/32)*4 + r%4, column l%32 of that 32 x 32 tile
    const int col_l = lane & 31;
    if (MODE == 0) {
        __bf16* h = (__bf16*)p.out;
        const int f = nt * 128 + wn * 32 + col_l;
#pragma unroll
        for (int ms = 0; ms < 4; ++ms)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = a_row_base + ms * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                if (row < rows_here)
                    h[(int64_t)(row0 + row) * p.ldo + f] = (__bf16)silu_mul(acc[ms][0][r], acc[ms][1][r]);
            }
    } else {
        float* o = (float*)p.out;
#pragma unroll
        for (int ms = 0; ms < 4; ++ms)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = a_row_base + ms * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                if (row < rows_here) {
                    const float wgt = p.row_w ? p.row_w[row0 + row] : 1.0f;
#pragma unroll
                    for (int ns = 0; ns < 2; ++ns) {
                        const int d = nt * 256 + wn * 64 + ns * 32 + col_l;
                        if (d < p.n_cols) o[(int64_t)(row0 + row) * p.ldo + d] = acc[ms][ns][r] * wgt;
                    }
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
        attr_err = hipFuncSetAttribute((const void*)ffn_gemm_bf16<MODE>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    });
    MOE_HIP_TRY(attr_err);
    hipLaunchKernelGGL((ffn_gemm_bf16<MODE>), dim3(grid), dim3(kThreads), kLdsBytes, st, p);
    MOE_HIP_TRY(hipGetLastError());
    return MOE_OK;
}

}  // namespace

int launch_expert_ffn_bf16(const moe_shape& s, const Geom& g, const FfnArgs& a, hipStream_t st) {
    const int R = s.T * s.k;
    GemmParams p{};
    fill_common(p, s, g, a);
    fill_gate_up(p, s, g, a);
    int rc = launch_mode<0>(p, gemm_grid(p.NT, R, BM, a.e_end - a.e_begin), st);
    if (rc != MOE_OK) return rc;
    if (a.mid_event) MOE_HIP_TRY(hipEventRecord(a.mid_event, st));
    fill_down(p, s, g, a);
    return launch_mode<1>(p, gemm_grid(p.NT, R, BM, a.e_end - a.e_begin), st);
}

}  // namespace moe
