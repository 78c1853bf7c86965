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
//
// Data movement.  512 threads = 8 wavefronts (2 per SIMD).  The reduction runs in
// HALF-STEPS of 32 elements.  One half-step needs a STAGE of 32 KiB in LDS: 256
// activation rows x 64 bytes and two weight half-tiles of 128 rows x 64 bytes.  A
// ring of kStages stages is kept; the stage of half-step k + kStages - 1 is loaded
// global -> LDS directly (global_load_lds, 16 bytes per lane, no registers in
// between) while half-step k is computed, so a load has kStages - 2 half-steps to
// land before anybody waits for it (weights come from HBM, activations from L2).
// Weight half-tiles are stored in the pages as the exact LDS image, so their copy is
// linear; activation rows are row-major in HBM and the lane -> chunk choice applies
// the swizzle.  In LDS the 16-byte chunk c of row r sits at chunk position
// c ^ ((r >> 2) & 3): 64 banks hold four 64-byte rows, and this makes every 16-lane
// phase of a ds_read_b128 of an MFMA operand (one row per lane, same chunk) touch
// each bank once.
//
// Schedule.  Measured on this chip: when all wavefronts issue their loads, then
// their LDS fetches, then their MFMAs in blocks after each barrier, the matrix
// cores idle while every wavefront queues at the memory pipeline (about 63 %
// utilisation).  The loop is therefore (a) rotated: the MFMAs of the second
// sub-step of half-step k-1 are issued AFTER the barrier that opens half-step k,
// so the matrix cores have work while the wavefronts synchronise, and (b)
// interleaved: between two MFMAs at most two LDS fetches or one global load are
// issued.  Scheduling fences pin that order.
//
// Wavefront w computes rows (w / 4) * 128 .. +127 and, of the 256 columns, for
// MODE 0 columns (w % 4) * 32 .. +31 of both tiles, for MODE 1 columns
// (w % 4) * 64 .. +63: 4 x 2 MFMA tiles of 32 x 32, 128 accumulator registers.
#include <mutex>
#include <type_traits>

#include "moe_ffn_common.h"

namespace moe {
namespace {

#define MOE_FENCE() __builtin_amdgcn_sched_barrier(0)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

constexpr int BM = 256;
constexpr int kThreads = 512;
constexpr int kRowB = 64;                    // bytes of one row in a stage (32 bf16)
constexpr int kStageA = 256 * kRowB;         // activation part of a stage
constexpr int kStageBytes = 2 * kStageA;     // + two weight half-tiles of 8 KiB
constexpr int kHalfTile = 128 * kRowB;       // one weight half-tile
constexpr int kLoadsPerStage = 4;            // global_load_lds instructions per wavefront per stage

__device__ __forceinline__ float silu_mul(float g, float u) {
    return g * __frcp_rn(1.0f + __expf(-g)) * u;
}

// wait until at most N of my vector-memory loads are outstanding and all my LDS fetches are back
template <int N>
__device__ __forceinline__ void wait_loads_and_lds() {
    __builtin_amdgcn_s_waitcnt(0x0070 | (N & 15) | ((N >> 4) << 14));
}

template <int MODE, int S>
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
    auto page_addr = [&](int page) -> const char* {
        int slot = __builtin_amdgcn_readfirstlane(trow[page]);
        if ((unsigned)slot >= (unsigned)p.pool_pages) {   // never follow an entry outside the pool
            bad = 1;
            slot = 0;
        }
        return p.pool + (int64_t)slot * p.page_bytes;
    };
    // Tile numbers of a column tile are consecutive along k, so the address only needs a new
    // page-table lookup when the walk crosses a page boundary (once per tiles-per-page k-tiles).
    struct TileWalk {
        int page, within;
        const char* base;     // address of the current page
    };
    auto walk_start = [&](int first_tile) {
        TileWalk w;
        w.page = first_tile / p.tpp;
        w.within = first_tile - w.page * p.tpp;
        w.base = page_addr(w.page);
        return w;
    };
    auto walk_next = [&](TileWalk& w) {
        if (++w.within == p.tpp) {
            w.within = 0;
            w.base = page_addr(++w.page);
        }
    };
    TileWalk w0 = walk_start(pt0 * p.KT), w1 = walk_start(pt1 * p.KT);

    // ---- per-lane sources of the activation rows ------------------------------------
    // load instruction q = i*8 + wave (i = 0, 1) fills LDS rows q*16 .. q*16+15 (1 KiB); lane j
    // holds row q*16 + j/4 at chunk position j%4, i.e. global chunk (j%4) ^ ((row >> 2) & 3)
    const char* a_src[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int lrow = (i * 8 + wave) * 16 + (lane >> 2);
        const int r = min(lrow, rows_here - 1);                               // rows past the tail repeat the last row
        const int c = (lane & 3) ^ ((lrow >> 2) & 3);
        a_src[i] = p.A + (int64_t)(row0 + r) * p.lda_bytes + c * 16;
    }
    const int b_lane_off = wave * 1024 + lane * 16;

    // Load instruction i (0, 1: activation rows; 2, 3: weight half-tile 0, 1) of half-step kn
    // into ring slot `slot`.  After the last instruction of an odd half-step the tile walk moves on.
    const int KH = 2 * p.KT;
    auto load_part = [&](int slot, int kn, int i) {
        char* st = smem + slot * kStageBytes;
        if (i < 2) {
            __builtin_amdgcn_global_load_lds((gptr_t)(a_src[i] + (int64_t)kn * kRowB), (lptr_t)(st + (i * 8 + wave) * 1024), 16, 0, 0);
        } else {
            const TileWalk& w = i == 2 ? w0 : w1;
            const char* b = w.base + (int64_t)w.within * 16384 + (kn & 1) * kHalfTile + b_lane_off;
            __builtin_amdgcn_global_load_lds((gptr_t)b, (lptr_t)(st + kStageA + (i - 2) * kHalfTile + wave * 1024), 16, 0, 0);
            if (i == 3 && (kn & 1) && kn + 1 < KH) {
                walk_next(w0);
                walk_next(w1);
            }
        }
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // LDS byte offset of this lane's operand chunk for sub-step ks (0, 1), relative to the first
    // row of a 32-row MFMA tile: row lane%32, chunk 2*ks + lane/32, swizzled
    const int c0 = (lane >> 5) ^ ((lane >> 2) & 3);
    const int lane_row = (lane & 31) * kRowB;
    const int frag_off[2] = {lane_row + (c0 << 4), lane_row + ((c0 ^ 2) << 4)};
    const int a_base = wm * 128 * kRowB;
    const int b_base[2] = {kStageA + ((MODE == 0) ? wn * 32 : wn * 64) * kRowB,
                           kStageA + ((MODE == 0) ? 128 + wn * 32 : wn * 64 + 32) * kRowB};
    // 32-row MFMA tiles of this wavefront that hold at least one valid row
    const int n_ms = max(0, min(4, (rows_here - wm * 128 + 31) >> 5));

    // operand registers: two sets (one per sub-step), each 4 A fragments and 2 B fragments
    bf16x8 fr[2][6];
#pragma unroll
    for (int i = 0; i < 6; ++i)
#pragma unroll
        for (int x = 0; x < 8; ++x) fr[1][i][x] = (__bf16)0.f;    // the first rotated MFMA group adds 0 * 0

    auto fetch = [&](const char* st, int ks, int i) {          // i = 0..3: A fragment, 4..5: B fragment
        const int base = i < 4 ? a_base + i * 32 * kRowB : b_base[i - 4];
        fr[ks][i] = *(const bf16x8*)(st + base + frag_off[ks]);
    };
    auto mfma = [&](int ks, int j, auto full) {                 // j = 0..7: MFMA tile (j / 2, j % 2)
        if (decltype(full)::value || (j >> 1) < n_ms)
            acc[j >> 1][j & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[ks][j >> 1], fr[ks][4 + (j & 1)], acc[j >> 1][j & 1], 0, 0, 0);
    };

    // One half-step.  LOADS: the stage of half-step k + S - 1 is loaded into the slot that
    // half-step k - 1 used.  WAITN: my loads that may still be in flight when the stage of
    // half-step k must be complete (the younger stages).
    int slot = 0;
    auto half_step = [&](int k, auto full, auto loads_c, auto waitn_c) {
        constexpr bool LOADS = decltype(loads_c)::value;
        wait_loads_and_lds<decltype(waitn_c)::value>();
        __builtin_amdgcn_s_barrier();      // stage k is complete for everyone; nobody reads stage k-1 any more
        asm volatile("" ::: "memory");
        const char* st = smem + slot * kStageBytes;
        int nslot = slot + S - 1;
        if (nslot >= S) nslot -= S;
        const int kn = k + S - 1;
        MOE_FENCE();
        // group A: MFMAs of (k-1, sub-step 1); fetch (k, sub-step 0); activation-row loads
        mfma(1, 0, full); MOE_FENCE(); fetch(st, 0, 4); fetch(st, 0, 5); MOE_FENCE();
        mfma(1, 1, full); MOE_FENCE(); fetch(st, 0, 0); fetch(st, 0, 1); MOE_FENCE();
        mfma(1, 2, full); MOE_FENCE(); fetch(st, 0, 2); fetch(st, 0, 3); MOE_FENCE();
        mfma(1, 3, full); MOE_FENCE(); if (LOADS) load_part(nslot, kn, 0); MOE_FENCE();
        mfma(1, 4, full); MOE_FENCE();
        mfma(1, 5, full); MOE_FENCE(); if (LOADS) load_part(nslot, kn, 1); MOE_FENCE();
        mfma(1, 6, full); MOE_FENCE();
        mfma(1, 7, full); MOE_FENCE();
        // group B: MFMAs of (k, sub-step 0); fetch (k, sub-step 1); weight loads
        mfma(0, 0, full); MOE_FENCE(); fetch(st, 1, 4); fetch(st, 1, 5); MOE_FENCE();
        mfma(0, 1, full); MOE_FENCE(); fetch(st, 1, 0); fetch(st, 1, 1); MOE_FENCE();
        mfma(0, 2, full); MOE_FENCE(); fetch(st, 1, 2); fetch(st, 1, 3); MOE_FENCE();
        mfma(0, 3, full); MOE_FENCE(); if (LOADS) load_part(nslot, kn, 2); MOE_FENCE();
        mfma(0, 4, full); MOE_FENCE();
        mfma(0, 5, full); MOE_FENCE(); if (LOADS) load_part(nslot, kn, 3); MOE_FENCE();
        mfma(0, 6, full); MOE_FENCE();
        mfma(0, 7, full); MOE_FENCE();
        if (++slot == S) slot = 0;
    };

    auto main_loop = [&](auto full) {
        // prologue: stages 0 .. S-2 in flight (KH >= 4 >= S - 1 always)
#pragma unroll
        for (int s = 0; s < S - 1; ++s)
#pragma unroll
            for (int i = 0; i < kLoadsPerStage; ++i) load_part(s, s, i);
        constexpr int kYounger = kLoadsPerStage * (S - 2);
        const int k_steady = KH - (S - 1);
        for (int k = 0; k < k_steady; ++k)
            half_step(k, full, std::true_type{}, std::integral_constant<int, kYounger>{});
        // drain: no new loads; one stage fewer is in flight in every half-step
        if (S >= 2) half_step(k_steady, full, std::false_type{}, std::integral_constant<int, kYounger>{});
        if (S >= 3) half_step(k_steady + 1, full, std::false_type{}, std::integral_constant<int, (S >= 3 ? kLoadsPerStage * (S - 3) : 0)>{});
        if (S >= 4) half_step(k_steady + 2, full, std::false_type{}, std::integral_constant<int, (S >= 4 ? kLoadsPerStage * (S - 4) : 0)>{});
        if (S >= 5) half_step(k_steady + 3, full, std::false_type{}, std::integral_constant<int, (S >= 5 ? kLoadsPerStage * (S - 5) : 0)>{});
        // the MFMAs of the last sub-step
        __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0)
#pragma unroll
        for (int j = 0; j < 8; ++j) mfma(1, j, full);
    };
    // a row tile whose last rows are missing skips the MFMA tiles that hold no valid row
    if (n_ms == 4) main_loop(std::true_type{});
    else main_loop(std::false_type{});

    // ---- epilogue ---------------------------------------------------------------------
    // accumulator register r of lane l in MFMA tile (ms, ns) is the element at
    // row ms*32 + (r/4)*8 + (l/32)*4 + r%4, column l%32 of that 32 x 32 tile
    const int col_l = lane & 31;
    const int a_row_base = wm * 128;
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

template <int MODE, int S>
int launch_mode(const GemmParams& p, int grid, hipStream_t st) {
    constexpr int lds = S * kStageBytes;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute((const void*)ffn_gemm_bf16<MODE, S>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    });
    MOE_HIP_TRY(attr_err);
    hipLaunchKernelGGL((ffn_gemm_bf16<MODE, S>), dim3(grid), dim3(kThreads), lds, st, p);
    MOE_HIP_TRY(hipGetLastError());
    return MOE_OK;
}

template <int MODE>
int launch_stages(const GemmParams& p, int grid, hipStream_t st) {
    switch (get_opt(OPT_FFN_STAGES)) {
        case 3: return launch_mode<MODE, 3>(p, grid, st);
        case 5: return launch_mode<MODE, 5>(p, grid, st);
        default: return launch_mode<MODE, 4>(p, grid, st);
    }
}

}  // namespace

int launch_expert_ffn_bf16(const moe_shape& s, const Geom& g, const FfnArgs& a, hipStream_t st) {
    const int R = s.T * s.k;
    GemmParams p{};
    fill_common(p, s, g, a);
    fill_gate_up(p, s, g, a);
    int rc = launch_stages<0>(p, gemm_grid(p.NT, R, BM, a.e_end - a.e_begin), st);
    if (rc != MOE_OK) return rc;
    if (a.mid_event) MOE_HIP_TRY(hipEventRecord(a.mid_event, st));
    fill_down(p, s, g, a);
    return launch_stages<1>(p, gemm_grid(p.NT, R, BM, a.e_end - a.e_begin), st);
}

}  // namespace moe
