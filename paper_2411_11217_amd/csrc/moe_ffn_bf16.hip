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
// the exact LDS image (16-byte chunks XOR-swizzled by (row / 2) & 7), so their copy is
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
#include <type_traits>

#include "moe_ffn_common.h"

namespace moe {
namespace {

// MOE_FFN_PIN = 1 pins the order "LDS fetch of sub-step ks+1, then MFMAs of sub-step ks"
#ifndef MOE_FFN_PIN
#define MOE_FFN_PIN 1
#endif
#if MOE_FFN_PIN
#define MOE_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)
#else
#define MOE_SCHED_FENCE() ((void)0)
#endif

// MOE_FFN_ISSUE_SPLIT: where the next stage's global -> LDS loads are issued inside a k-step.
// 0: all 8 at its start; 1: activation rows after the first LDS fetch, weight tiles after the
// first MFMA group; 2: two per sub-step.
#ifndef MOE_FFN_ISSUE_SPLIT
#define MOE_FFN_ISSUE_SPLIT 1
#endif

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

#ifdef MOE_FFN_TIMELINE   // experiment builds only: per-block time stamps behind the status words
    long long* tl = (long long*)(p.status + 4) + ((size_t)blockIdx.x + MODE * 6144) * 8;
    const long long t_entry = clock64();
#define MOE_TL(i) do { if (tid == 0) tl[i] = clock64() - t_entry; } while (0)
#else
#define MOE_TL(i) ((void)0)
#endif
    // ---- which tile is mine -------------------------------------------------
    const TileCoord tc = locate_tile<BM>(p);
    if (!tc.valid) return;
#ifdef MOE_FFN_TIMELINE
    if (tid == 0) { tl[0] = t_entry; tl[5] = wall_clock64(); tl[7] = 1; }
#endif
    MOE_TL(1);
    const int e = tc.e, nt = tc.nt, row0 = tc.row0, rows_here = tc.rows_here;

    // ---- weight tiles through the page table -------------------------------------
    const int32_t* trow = p.table + (size_t)(p.table_row_mod ? e % p.table_row_mod : e) * p.ppe + p.group_base;
    const int pt0 = p.debug_same_tile ? 0 : nt * 2;
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

    // ---- per-lane sources of the activation rows ------------------------------------
    // load instruction q = i*8 + wave fills LDS rows q*8 .. q*8+7 (1 KiB); lane j holds
    // row q*8 + j/8 at chunk position j%8, i.e. global chunk (j%8) ^ ((row / 2) & 7)
    const char* a_src[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int lrow = (i * 8 + wave) * 8 + (lane >> 3);
        const int r = min(lrow, rows_here - 1);                               // rows past the tail repeat the last row
        const int c = (lane & 7) ^ ((lrow >> 1) & 7);
        a_src[i] = p.A + (int64_t)(p.debug_same_tile ? r : row0 + r) * p.lda_bytes + c * 16;
    }

    // Tile numbers of a column tile are consecutive along k, so the address only needs a new
    // page-table lookup when the walk crosses a page boundary (once per tiles-per-page steps).
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

    // The 8 load instructions of a wavefront for one stage, in 4 parts of 2 (parts 0,1:
    // activation rows; parts 2,3: weight tiles), so that they can be spread over a k-step.
    auto issue_part = [&](int stage, int kt, int part) {
        char* sA = smem + stage * kStageBytes;
        char* sB = sA + kStageA;
        if (part < 2) {
#pragma unroll
            for (int i = 2 * part; i < 2 * part + 2; ++i) {
                const int q = i * 8 + wave;
                __builtin_amdgcn_global_load_lds((gptr_t)(a_src[i] + (int64_t)kt * 128), (lptr_t)(sA + q * 1024), 16, 0, 0);
            }
        } else {
            const TileWalk& w = part == 2 ? w0 : w1;          // part 2 fills tile 0, part 3 tile 1
            const char* b = w.base + (int64_t)w.within * 16384;
#pragma unroll
            for (int i = 2 * part - 4; i < 2 * part - 2; ++i) {
                const int q = i * 8 + wave;
                __builtin_amdgcn_global_load_lds((gptr_t)(b + (q & 15) * 1024 + lane * 16), (lptr_t)(sB + q * 1024), 16, 0, 0);
            }
        }
    };
    auto issue = [&](int stage, int kt) {
#pragma unroll
        for (int part = 0; part < 4; ++part) issue_part(stage, kt, part);
    };
    // called after issue(kt) when a step kt+1 exists; at a page crossing this waits for the
    // table entry (and with it for the loads just issued), which happens once per page
    auto advance = [&]() {
        walk_next(w0);
        walk_next(w1);
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // LDS byte offset of this lane's operand chunk for k-sub-step ks, relative to the first
    // row of a 32-row MFMA tile: row lane%32, chunk 2*ks + lane/32, swizzled
    const int c0 = (lane >> 5) ^ ((lane >> 1) & 7);
    const int lane_row = (lane & 31) * 128;
    const int a_row_base = wm * 128;
    const int b_row0 = (MODE == 0) ? wn * 32 : wn * 64;
    const int b_row1 = (MODE == 0) ? 128 + wn * 32 : wn * 64 + 32;
    // 32-row MFMA tiles of this wavefront that hold at least one valid row
    const int n_ms = max(0, min(4, (rows_here - a_row_base + 31) >> 5));

    auto load_frags = [&](const char* sA, const char* sB, int ks, bf16x8 (&a)[4], bf16x8 (&b)[2], auto full) {
        const int off = lane_row + ((c0 ^ (2 * ks)) << 4);
#pragma unroll
        for (int ms = 0; ms < 4; ++ms)
            if (decltype(full)::value || ms < n_ms) a[ms] = *(const bf16x8*)(sA + off + (a_row_base + ms * 32) * 128);
        b[0] = *(const bf16x8*)(sB + off + b_row0 * 128);
        b[1] = *(const bf16x8*)(sB + off + b_row1 * 128);
    };
    auto mfma_frags = [&](const bf16x8 (&a)[4], const bf16x8 (&b)[2], auto full) {
#pragma unroll
        for (int ms = 0; ms < 4; ++ms)
            if (decltype(full)::value || ms < n_ms) {
#pragma unroll
                for (int ns = 0; ns < 2; ++ns)
                    acc[ms][ns] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ms], b[ns], acc[ms][ns], 0, 0, 0);
            }
    };
    // one 64-wide k-step: the operands of sub-step ks+1 are fetched from LDS while the MFMAs
    // of sub-step ks run
    // One 64-wide k-step on stage `stage`.  The operands of sub-step ks+1 are fetched from LDS
    // while the MFMAs of sub-step ks run, and (when nxt) the global -> LDS loads of the next
    // stage are issued in between, spread over the step so that the texture path, the LDS and
    // the matrix cores are busy at the same time.  The scheduling fences pin that order.
    auto compute = [&](int stage, auto full, bool nxt, int nstage, int nkt) {
        const char* sA = smem + stage * kStageBytes;
        const char* sB = sA + kStageA;
        bf16x8 a0[4], b0[2], a1[4], b1[2];
        auto loads = [&](int first, int last) {
            if (nxt)
                for (int part = first; part <= last; ++part) issue_part(nstage, nkt, part);
        };
        if (MOE_FFN_ISSUE_SPLIT == 0) loads(0, 3);
        load_frags(sA, sB, 0, a0, b0, full);
        MOE_SCHED_FENCE();
        if (MOE_FFN_ISSUE_SPLIT == 1) loads(0, 1);
        if (MOE_FFN_ISSUE_SPLIT == 2) loads(0, 0);
        load_frags(sA, sB, 1, a1, b1, full);
        MOE_SCHED_FENCE();
        mfma_frags(a0, b0, full);
        MOE_SCHED_FENCE();
        if (MOE_FFN_ISSUE_SPLIT == 1) loads(2, 3);
        if (MOE_FFN_ISSUE_SPLIT == 2) loads(1, 1);
        load_frags(sA, sB, 2, a0, b0, full);
        MOE_SCHED_FENCE();
        mfma_frags(a1, b1, full);
        MOE_SCHED_FENCE();
        if (MOE_FFN_ISSUE_SPLIT == 2) loads(2, 2);
        load_frags(sA, sB, 3, a1, b1, full);
        MOE_SCHED_FENCE();
        mfma_frags(a0, b0, full);
        MOE_SCHED_FENCE();
        if (MOE_FFN_ISSUE_SPLIT == 2) loads(3, 3);
        mfma_frags(a1, b1, full);
    };

    // raw workgroup barrier: no implied wait for outstanding loads (the waits are explicit)
    auto barrier = [&]() {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    auto main_loop = [&](auto full) {
        if (p.variant == 0) {
            // plain schedule: load a stage, wait, compute, and only then load the next
            for (int kt = 0; kt < p.KT; ++kt) {
                issue(0, kt);
                if (kt + 1 < p.KT) advance();
                __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): my direct-to-LDS loads have landed
                __syncthreads();
                compute(0, full, false, 0, 0);
                __syncthreads();
            }
        } else if (p.variant == 1) {
            issue(0, 0);
            if (p.KT > 1) advance();
            for (int kt = 0; kt < p.KT; ++kt) {
                __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
                __syncthreads();                      // stage kt complete for everyone; stage kt-1 no longer read
                compute(kt & 1, full, kt + 1 < p.KT, (kt + 1) & 1, kt + 1);
                if (kt + 2 < p.KT) advance();
            }
        } else {
            // Ping-pong.  The two wavefronts of a SIMD (w and w+4; group = w / 4) alternate between
            // a FETCH phase (all MFMA operands of one k-step from LDS into registers) and a COMPUTE
            // phase (its 32 MFMAs), half a k-step apart, so each SIMD's matrix core always has one
            // wavefront with its operands ready while the other one waits on LDS.  Phases are
            // separated by workgroup barriers; barrier number b ends phase b-1:
            //   group 0: FETCH(kt) in phase 2kt,   COMPUTE(kt) in phase 2kt+1
            //   group 1: FETCH(kt) in phase 2kt+1, COMPUTE(kt) in phase 2kt+2
            // Stage kt+1 is loaded global -> LDS by every wavefront during phase 2kt (its buffer was
            // last read in phase 2kt-1) and waited for before the barrier that ends phase 2kt+1.
            bf16x8 fa[4][4], fb[4][2];
            auto fetch = [&](int stage) {
                const char* sA = smem + stage * kStageBytes;
                const char* sB = sA + kStageA;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) load_frags(sA, sB, ks, fa[ks], fb[ks], full);
            };
            auto mfmas = [&]() {
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) mfma_frags(fa[ks], fb[ks], full);
            };
            issue(0, 0);
            if (p.KT > 1) advance();
            __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0)
            barrier();                                // stage 0 is complete
            if (wm == 0) {
                for (int kt = 0; kt < p.KT; ++kt) {
                    if (kt + 1 < p.KT) {
                        issue((kt + 1) & 1, kt + 1);
                        if (kt + 2 < p.KT) advance();
                    }
                    fetch(kt & 1);
                    MOE_SCHED_FENCE();
                    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): operands are in registers
                    barrier();
                    mfmas();
                    MOE_SCHED_FENCE();
                    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): my part of stage kt+1 has landed
                    barrier();
                }
            } else {
                if (p.KT > 1) {
                    issue(1, 1);
                    if (p.KT > 2) advance();
                }
                barrier();
                for (int kt = 0; kt < p.KT; ++kt) {
                    fetch(kt & 1);
                    MOE_SCHED_FENCE();
                    __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0)
                    barrier();
                    if (kt + 2 < p.KT) {
                        issue(kt & 1, kt + 2);
                        if (kt + 3 < p.KT) advance();
                    }
                    mfmas();
                    MOE_SCHED_FENCE();
                    if (kt + 1 < p.KT) barrier();
                }
            }
        }
    };
    MOE_TL(2);
    // a row tile whose last rows are missing skips the MFMA tiles that hold no valid row
    if (n_ms == 4) main_loop(std::true_type{});
    else main_loop(std::false_type{});
    MOE_TL(3);

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
    MOE_TL(4);
#ifdef MOE_FFN_TIMELINE
    if (tid == 0) tl[6] = wall_clock64() - tl[5];
#endif
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
