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
// Data movement.  256 threads = 4 wavefronts, one per SIMD, each with the full
// register file (256 accumulator + 256 vector registers).  The reduction runs in
// HALF-STEPS of 32 elements; two of them are a K-STEP (64 elements = one page tile
// along k).  Operands reach LDS directly (global_load_lds, 16 bytes per lane, no
// registers in between) through two rings that fill all 160 KiB of the compute unit:
//   weights:     four stages of 16 KiB, one per half-step: two half-tiles of 128 rows x
//                64 bytes.  The pages hold the exact LDS image, so the copy is linear.
//                The stage of half-step k + 3 is loaded while half-step k is computed.
//   activations: three stages of 32 KiB, one per k-step: 256 rows x 128 bytes, i.e.
//                one whole cache line per row and load.  Measured: the vector memory
//                path handles about one cache line per two clocks whether a lane
//                group uses all 128 bytes of it or only 64, so fetching a row's line
//                in two halves (a 64-byte stage per half-step, as for the weights)
//                doubles the time of the activation loads (30 instead of 58 bytes per
//                clock and compute unit) and made the load path, not the matrix
//                cores, the longest chain of the loop.  Rows are row-major in HBM; the
//                lane -> chunk choice of the load applies the swizzle.  The stage of
//                k-step K + 2 is loaded during the two half-steps of k-step K.
// Swizzles: in a 64-byte-row stage the 16-byte chunk c of row r sits at position
// c ^ ((r >> 2) & 3), in a 128-byte-row stage at c ^ ((r >> 1) & 7): 64 banks hold
// four (two) rows, and this makes every 16-lane phase of a ds_read_b128 of an MFMA
// operand (one row per lane, same chunk) touch each bank once.
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
// Wavefront w computes rows (w / 2) * 128 .. +127 and, of the 256 columns, for
// MODE 0 columns (w % 2) * 64 .. +63 of both tiles, for MODE 1 columns
// (w % 2) * 128 .. +127: 4 x 4 MFMA tiles of 32 x 32, 256 accumulator registers.
// Measured against 8 wavefronts of 128 x 64 each: a 128 x 128 wavefront tile needs
// 8 LDS fetches per 16 MFMAs instead of 12, a third less LDS traffic; the chip is
// power limited under this load, the clock rises and the loop runs ~10 % faster.
#include <algorithm>
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
constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kComputeUnits = 256;           // MI355X
constexpr int kRowB = 64;                    // bytes of one weight row in a stage (32 bf16: one half-step)
constexpr int kHalfTile = 128 * kRowB;       // one weight half-tile
constexpr int kStageB = 2 * kHalfTile;       // weight stage of one half-step: two half-tiles
constexpr int kStages = 4;                   // depth of the weight ring: the loop below is unrolled over it
constexpr int kARowB = 128;                  // bytes of one activation row in a stage (64 bf16: one k-step = two half-steps)
constexpr int kStageA = 256 * kARowB;        // activation stage of one k-step
constexpr int kStagesA = 3;                  // depth of the activation ring
constexpr int kRingA = kStages * kStageB;    // LDS offset of the activation ring (the weight ring sits at 0)
constexpr int kLdsBytes = kRingA + kStagesA * kStageA;   // 160 KiB: all of a compute unit's LDS

// silu(g) * u with the hardware exp2 and reciprocal (1 ulp each): far below the resolution of
// the bf16 result; an IEEE division would cost a dozen instructions per element
__device__ __forceinline__ float silu_mul(float g, float u) {
    const float e = __builtin_amdgcn_exp2f(g * -1.44269504088896340736f);
    return g * __builtin_amdgcn_rcpf(1.0f + e) * u;
}

// wait until at most N of my vector-memory loads are outstanding and all my LDS fetches are back
template <int N>
__device__ __forceinline__ void wait_loads_and_lds() {
    __builtin_amdgcn_s_waitcnt(0x0070 | (N & 15) | ((N >> 4) << 14));
}

#ifdef MOE_FFN_TIMELINE
__device__ __forceinline__ long long rows_here_tl(int rows) { return (long long)rows << 8; }
#endif

// NB: page tiles per block along the columns.  2: the 256-column block described above.  1 (MODE 1
// only): 256 rows x 128 columns, wavefront tile 128 x 64, for launches with too few 256-wide tiles
// to occupy the chip (few rows per expert: the launch is bound by streaming the weights, and more
// blocks stream more).
template <int MODE, int NB>
__global__ __launch_bounds__(kThreads) void ffn_gemm_bf16(const GemmParams p) {
    constexpr int S = kStages;
    static_assert(NB == 2 || (NB == 1 && MODE == 1), "gate/up needs the W1 and the W3 tile");
    constexpr int NS = 2 * NB;                   // 32-column MFMA tiles (B fragments) per wavefront
    constexpr int NMF = 4 * NS;                  // MFMAs per wavefront per 16-wide sub-step
    constexpr int kLoadsPerStage = 4 + 2 * NB;   // global_load_lds instructions per wavefront per stage
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

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
    if (tid == 0) { tl[0] = t_entry; tl[5] = wall_clock64(); tl[7] = 1 + rows_here_tl(tc.rows_here) + ((long long)(__builtin_amdgcn_s_getreg(6164) & 15) << 32); }
#endif
    MOE_TL(1);
    const int e = tc.e, nt = tc.nt, row0 = tc.row0, rows_here = tc.rows_here;

    // ---- weight tiles through the page table -------------------------------------
    const int32_t* trow = p.table + (size_t)(p.table_row_mod ? e % p.table_row_mod : e) * p.ppe + p.group_base;
    const int pt0 = nt * NB;
    const int pt1 = (pt0 + 1 < p.n_page_tiles) ? pt0 + 1 : pt0;   // odd tile count: the second half is masked (NB = 2)
    int bad = 0;
    auto page_addr = [&](int page) __attribute__((always_inline)) -> const char* {
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
        const char* tile;     // address of the current tile
    };
    auto walk_start = [&](int first_tile) __attribute__((always_inline)) {
        TileWalk w;
        w.page = first_tile / p.tpp;
        w.within = first_tile - w.page * p.tpp;
        w.tile = page_addr(w.page) + (int64_t)w.within * 16384;
        return w;
    };
    auto walk_next = [&](TileWalk& w) __attribute__((always_inline)) {
        w.tile += 16384;
        if (++w.within == p.tpp) {
            w.within = 0;
            w.tile = page_addr(++w.page);
        }
    };
    TileWalk w0 = walk_start(pt0 * p.KT), w1 = walk_start(pt1 * p.KT);

    // ---- sources of the global -> LDS loads: a wave-uniform base that moves along k plus a 32-bit
    // offset per lane that never changes, so a half-step costs a few scalar additions ----------------
    // Activation rows are loaded a k-step (128 bytes = one cache line per row) at a time: load
    // instruction q = i*4 + wave (i = 0..7) fills LDS rows q*8 .. q*8+7 (1 KiB); lane j holds row
    // q*8 + j/8 at chunk position j%8, i.e. global chunk (j%8) ^ ((row >> 1) & 7).  Rows past the
    // tail repeat the last row.
    uint32_t a_off[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int lrow = (i * kWaves + wave) * 8 + (lane >> 3);
        const int r = min(lrow, rows_here - 1);
        const int c = (lane & 7) ^ ((lrow >> 1) & 7);
        a_off[i] = (uint32_t)r * (uint32_t)p.lda_bytes + c * 16;
    }
    const char* a_ptr = p.A + (int64_t)row0 * p.lda_bytes;    // + 128 bytes per k-step
    int a_wr = kRingA;                                         // LDS offset of the activation stage being filled
    const uint32_t b_off = wave * 1024 + lane * 16;            // weight half-tiles are copied linearly

    // The loads issued during half-step h: activation instructions (h & 1) * 4 + i (i = 0..3) of the
    // k-step two ahead, and the weight stage of half-step h + 3 (instructions 4, 5: half-tile 0; 6, 7:
    // half-tile 1) into weight slot `slot`.  After the last instruction of a kind the sources move on.
    const int KH = 2 * p.KT;
    auto load_a = [&](int part, int i) __attribute__((always_inline)) {
        const int ia = part * 4 + i;
#ifndef MOE_FFN_NO_LOADS
        __builtin_amdgcn_global_load_lds((gptr_t)(a_ptr + a_off[ia]), (lptr_t)(smem + a_wr + (ia * kWaves + wave) * 1024), 16, 0, 0);
#endif
        if (ia == 7) {
            a_ptr += kARowB;
            a_wr = (a_wr == kRingA + (kStagesA - 1) * kStageA) ? kRingA : a_wr + kStageA;
        }
    };
    auto load_b = [&](int slot, int kn, int odd, int i) __attribute__((always_inline)) {     // odd = kn & 1, known at compile time by the callers
        char* st = smem + slot * kStageB;
        const TileWalk& w = i < 2 ? w0 : w1;
        const int part = (i & 1) * (kWaves * 1024);                       // first or second 4 KiB of the half-tile
        const char* b = w.tile + odd * kHalfTile + part;
#ifndef MOE_FFN_NO_LOADS
        __builtin_amdgcn_global_load_lds((gptr_t)(b + b_off), (lptr_t)(st + (i >= 2 ? kHalfTile : 0) + part + wave * 1024), 16, 0, 0);
#endif
        if (i == 2 * NB - 1 && odd && kn + 1 < KH) {
            walk_next(w0);
            if (NB == 2) walk_next(w1);
        }
    };

    f32x16 acc[4][NS];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < NS; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // LDS byte offsets of this lane's operand chunks.  Weights (64-byte rows, one half-step per stage):
    // sub-step ks (0, 1) reads row lane%32, chunk 2*ks + lane/32, swizzled.  Activations (128-byte rows,
    // two half-steps per stage): half-step parity hp and sub-step ks read chunk 4*hp + 2*ks + lane/32.
    const int c0 = (lane >> 5) ^ ((lane >> 2) & 3);
    const int lane_row = (lane & 31) * kRowB;
    const int frag_off[2] = {lane_row + (c0 << 4), lane_row + ((c0 ^ 2) << 4)};
    int a_frag[2][2];                 // includes the activation stage being read: moves on after every odd half-step
#pragma unroll
    for (int hp = 0; hp < 2; ++hp)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
            a_frag[hp][ks] = kRingA + wm * 128 * kARowB + (lane & 31) * kARowB + (((4 * hp + 2 * ks + (lane >> 5)) ^ ((lane >> 1) & 7)) << 4);
    int a_rd = 0;                     // activation stage being read
    // B fragment ns: MODE 0: gate rows wn*64 + {0, 32} of tile 0, then the same up rows of tile 1;
    //                MODE 1: rows wn*(32*NS) + ns*32 of the 128*NB rows of the block's tiles
    int b_base[NS];
#pragma unroll
    for (int ns = 0; ns < NS; ++ns)
        b_base[ns] = ((MODE == 0) ? (ns >> 1) * 128 + wn * 64 + (ns & 1) * 32 : wn * (32 * NS) + ns * 32) * kRowB;
    // 32-row MFMA tiles of this wavefront that hold at least one valid row
    const int n_ms = max(0, min(4, (rows_here - wm * 128 + 31) >> 5));

    // operand registers: two sets (one per sub-step), each 4 A fragments and NS B fragments
    bf16x8 fr[2][4 + NS];
#pragma unroll
    for (int i = 0; i < 4 + NS; ++i)
#pragma unroll
        for (int x = 0; x < 8; ++x) fr[1][i][x] = (__bf16)0.f;    // the first rotated MFMA group adds 0 * 0

    auto fetch = [&](const char* st, int hp, int ks, int i) __attribute__((always_inline)) {  // i = 0..3: A fragment, 4..: B fragment; st: weight stage
        if (i < 4) fr[ks][i] = *(const bf16x8*)(smem + a_frag[hp][ks] + i * 32 * kARowB);
        else fr[ks][i] = *(const bf16x8*)(st + b_base[i - 4] + frag_off[ks]);
    };
    auto mfma = [&](int ks, int j, auto full) __attribute__((always_inline)) {                 // j = 0..NMF-1: MFMA tile (j / NS, j % NS)
#ifdef MOE_FFN_NO_MFMA     // experiment builds only
        {
            typedef int i32x4_t __attribute__((ext_vector_type(4)));
            const bf16x8 fa = fr[ks][j / NS], fb = fr[ks][4 + (j % NS)];
            i32x4_t ia, ib;
            __builtin_memcpy(&ia, &fa, 16);
            __builtin_memcpy(&ib, &fb, 16);
            asm volatile("" ::"v"(ia), "v"(ib));
        }
#else
        if (decltype(full)::value || (j / NS) < n_ms)
            acc[j / NS][j % NS] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[ks][j / NS], fr[ks][4 + (j % NS)], acc[j / NS][j % NS], 0, 0, 0);
#endif
    };
    // One group: the NMF MFMAs of operand set `ms_set`, with the LDS fetches of set `fs_ks` (weights
    // from stage `st`) behind the first few of them, two at a time, in the order the next group
    // consumes them, and then global loads, one behind an MFMA (NB = 2: behind every second one):
    // KIND 1 the four activation loads of `part`, KIND 2 the 2 * NB weight loads, KIND 0 none.
    auto group = [&](int ms_set, const char* st, int hp, int fs_ks, auto kind_c, int part, int nslot, int kn, auto full) __attribute__((always_inline)) {
        constexpr int KIND = decltype(kind_c)::value;
        constexpr int order2[8] = {4, 0, 5, 6, 7, 1, 2, 3};
        constexpr int order1[6] = {4, 0, 5, 1, 2, 3};
        constexpr int NR2 = (4 + NS) / 2;        // MFMAs that have fetches behind them
        constexpr int n_loads = KIND == 1 ? 4 : 2 * NB;
#pragma unroll
        for (int j = 0; j < NMF; ++j) {
            mfma(ms_set, j, full);
            MOE_FENCE();
            if (j < NR2) {
                fetch(st, hp, fs_ks, NB == 2 ? order2[2 * j] : order1[2 * j]);
                fetch(st, hp, fs_ks, NB == 2 ? order2[2 * j + 1] : order1[2 * j + 1]);
                MOE_FENCE();
            } else if (KIND != 0) {
                const int li = NB == 2 ? (((j - NR2) & 1) ? (j - NR2 - 1) / 2 : -1) : j - NR2;
                if (li >= 0 && li < n_loads) {
                    if (KIND == 1) load_a(part, li);
                    else load_b(nslot, kn, nslot & 1, li);
                    MOE_FENCE();
                }
            }
        }
    };

    // One half-step on weight-ring slot U (a compile-time constant: every weight address in LDS is an
    // immediate; the activation stage moves through per-lane offsets).  LA / LB: issue the activation /
    // weight loads of this half-step.  WAITN: my loads that may still be in flight when the stages of
    // half-step k must be complete (those issued during the two half-steps before).  Operand set U & 1
    // holds sub-step 0: S is even, so the parity of k is static too.
    auto half_step = [&](int k, auto u_c, auto full, auto la_c, auto lb_c, auto waitn_c) __attribute__((always_inline)) {
        using std::integral_constant;
        constexpr int U = decltype(u_c)::value;
        constexpr int HP = U & 1;
        wait_loads_and_lds<decltype(waitn_c)::value>();
        __builtin_amdgcn_s_barrier();      // the stages of k are complete for everyone; nobody reads those of k-1 any more
        asm volatile("" ::: "memory");
        const char* st = smem + U * kStageB;
        constexpr int nslot = (U + S - 1) % S;
        const int kn = k + S - 1;
        MOE_FENCE();
        // group A: MFMAs of (k-1, sub-step 1); fetch (k, sub-step 0); activation-row loads
        group(1, st, HP, 0, integral_constant<int, decltype(la_c)::value ? 1 : 0>{}, HP, nslot, kn, full);
        // group B: MFMAs of (k, sub-step 0); fetch (k, sub-step 1); weight loads
        group(0, st, HP, 1, integral_constant<int, decltype(lb_c)::value ? 2 : 0>{}, HP, nslot, kn, full);
        if (HP) {                          // the next half-step reads the next activation stage
            const int d = (a_rd == kStagesA - 1) ? -(kStagesA - 1) * kStageA : kStageA;
            a_rd = (a_rd == kStagesA - 1) ? 0 : a_rd + 1;
#pragma unroll
            for (int x = 0; x < 4; ++x) a_frag[x >> 1][x & 1] += d;
        }
    };

    auto main_loop = [&](auto full) __attribute__((always_inline)) {
        using std::integral_constant;
        constexpr int kL = kLoadsPerStage;
        const std::true_type L{};
        const std::false_type N{};
        // prologue, in the order the half-steps -4 .. -1 would have issued them: activation k-steps
        // 0 and 1, weight half-steps 0 .. 2 (KH is a multiple of 4 and at least 4)
#pragma unroll
        for (int i = 0; i < 4; ++i) load_a(0, i);
#pragma unroll
        for (int s = 0; s < S - 1; ++s) {
#pragma unroll
            for (int i = 0; i < 4; ++i) load_a((s + 1) & 1, i);
#pragma unroll
            for (int i = 0; i < 2 * NB; ++i) load_b(s, s, s & 1, i);
        }
        int k = 0;
        for (; k + S < KH; k += S) {
            half_step(k, integral_constant<int, 0>{}, full, L, L, integral_constant<int, 2 * kL>{});
            half_step(k + 1, integral_constant<int, 1>{}, full, L, L, integral_constant<int, 2 * kL>{});
            half_step(k + 2, integral_constant<int, 2>{}, full, L, L, integral_constant<int, 2 * kL>{});
            half_step(k + 3, integral_constant<int, 3>{}, full, L, L, integral_constant<int, 2 * kL>{});
        }
        // last four half-steps: one more weight stage to load, then the rings drain
        half_step(k, integral_constant<int, 0>{}, full, N, L, integral_constant<int, 2 * kL>{});
        half_step(k + 1, integral_constant<int, 1>{}, full, N, N, integral_constant<int, kL + 2 * NB>{});
        half_step(k + 2, integral_constant<int, 2>{}, full, N, N, integral_constant<int, 2 * NB>{});
        half_step(k + 3, integral_constant<int, 3>{}, full, N, N, integral_constant<int, 0>{});
        // the MFMAs of the last sub-step
        __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0)
#pragma unroll
        for (int j = 0; j < NMF; ++j) mfma(1, j, full);
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
    const int a_row_base = wm * 128;
    const bool full_rows = rows_here == BM;
    if (MODE == 0) {
        __bf16* h = (__bf16*)p.out + (int64_t)row0 * p.ldo + nt * 128 + wn * 64 + col_l;
        auto store_rows = [&](auto full) __attribute__((always_inline)) {
#pragma unroll
            for (int ms = 0; ms < 4; ++ms)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = a_row_base + ms * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                    if (decltype(full)::value || row < rows_here) {
#pragma unroll
                        for (int ns = 0; ns < 2; ++ns)
                            h[(int64_t)row * p.ldo + ns * 32] = (__bf16)silu_mul(acc[ms][ns][r], acc[ms][ns + 2][r]);
                    }
                }
        };
        if (full_rows) store_rows(std::true_type{});
        else store_rows(std::false_type{});
    } else {
        // the 256 row weights of the tile go through LDS (free now): one load per thread instead of
        // one dependent global load per accumulator row
        float* sw = (float*)smem;
        __syncthreads();                       // every wavefront has left the main loop
        sw[tid] = (p.row_w && tid < rows_here) ? p.row_w[row0 + tid] : 1.0f;
        __syncthreads();
        const int d0 = nt * (128 * NB) + wn * (32 * NS);   // n_cols is a multiple of 128: with NB = 2 a wavefront's columns are all valid or all not
        if (d0 < p.n_cols) {
            float* o = (float*)p.out + (int64_t)row0 * p.ldo + d0 + col_l;
            auto store_rows = [&](auto full) __attribute__((always_inline)) {
#pragma unroll
                for (int ms = 0; ms < 4; ++ms)
#pragma unroll
                    for (int rq = 0; rq < 4; ++rq) {
                        const int rowq = a_row_base + ms * 32 + rq * 8 + (lane >> 5) * 4;      // 4 consecutive rows
                        const float4 wq = *(const float4*)(sw + rowq);
                        const float w4[4] = {wq.x, wq.y, wq.z, wq.w};
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int row = rowq + i;
                            if (decltype(full)::value || row < rows_here) {
#pragma unroll
                                for (int ns = 0; ns < NS; ++ns)
                                    o[(int64_t)row * p.ldo + ns * 32] = acc[ms][ns][rq * 4 + i] * w4[i];
                            }
                        }
                    }
            };
            if (full_rows) store_rows(std::true_type{});
            else store_rows(std::false_type{});
        }
    }
    MOE_TL(4);
#ifdef MOE_FFN_TIMELINE
    if (tid == 0) tl[6] = wall_clock64() - tl[5];
#endif
    if (bad && tid == 0 && p.status) atomicOr(p.status, 1);
}

template <int MODE, int NB>
int launch_stages(const GemmParams& p, int grid, hipStream_t st) {
    constexpr int lds = kLdsBytes;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute((const void*)ffn_gemm_bf16<MODE, NB>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    });
    MOE_HIP_TRY(attr_err);
    hipLaunchKernelGGL((ffn_gemm_bf16<MODE, NB>), dim3(grid), dim3(kThreads), lds, st, p);
    MOE_HIP_TRY(hipGetLastError());
    return MOE_OK;
}

}  // namespace

int launch_expert_ffn_bf16(const moe_shape& s, const Geom& g, const FfnArgs& a, hipStream_t st) {
    const int R = s.T * s.k;
    const int n_exp = a.e_end - a.e_begin;
    GemmParams p{};
    fill_common(p, s, g, a);
    fill_gate_up(p, s, g, a);
    int rc = launch_stages<0, 2>(p, gemm_grid(p.NT, R, BM, n_exp), st);
    if (rc != MOE_OK) return rc;
    if (a.mid_event) MOE_HIP_TRY(hipEventRecord(a.mid_event, st));
    fill_down(p, s, g, a);
    // Down projection with few row tiles: 256-wide column tiles would leave compute units without a
    // block (the routing result is not known here, R / BM + experts bounds the row tiles), so the
    // columns are cut into 128-wide tiles instead.  down_cols: 0 = this rule, 1 / 2 = force NB.
    const int opt = get_opt(OPT_DOWN_COLS);
    const bool narrow = opt == 1 || (opt == 0 && (int64_t)(R / BM + n_exp) * p.NT < 2 * kComputeUnits);
    if (narrow) {
        p.NT = (int32_t)g.dt;
        return launch_stages<1, 1>(p, gemm_grid(p.NT, R, BM, n_exp), st);
    }
    return launch_stages<1, 2>(p, gemm_grid(p.NT, R, BM, n_exp), st);
}

// y = x W^T for a dense weight matrix held as pages: the down-projection kernel with one "expert"
// that owns all T rows (offsets = {0, T}) and no row weight.
int launch_linear_bf16(const LinearArgs& a, hipStream_t st) {
    GemmParams p{};
    p.A = (const char*)a.x;
    p.lda_bytes = (int64_t)a.K * 2;
    p.offsets = a.offsets;
    p.table = a.page_table;
    p.pool = a.pool;
    p.page_bytes = a.page_bytes;
    p.tile_bytes = (int64_t)kTileN * kTileK * 2;
    p.pool_pages = (int32_t)std::min<int64_t>(a.pool_pages, 0x7fffffff);
    p.tpp = (int32_t)(a.page_bytes / p.tile_bytes);
    p.ppe = (int32_t)a.pages;
    p.group_base = 0;
    p.KT = a.K / kTileK;
    p.n_page_tiles = a.N / kTileN;
    p.e_begin = 0;
    p.e_end = 1;
    p.table_row_mod = 0;
    p.out = a.out;
    p.ldo = a.N;
    p.n_cols = a.N;
    p.row_w = nullptr;
    p.status = a.status;
    p.xcd_remap = get_opt(OPT_XCD_REMAP);
    p.tile_order = get_opt(OPT_TILE_ORDER);
    const int wide_tiles = (p.n_page_tiles + 1) / 2;
    if ((int64_t)(a.T / BM + 1) * wide_tiles < 2 * kComputeUnits) {       // too few 256-wide tiles to fill the chip
        p.NT = p.n_page_tiles;
        return launch_stages<1, 1>(p, gemm_grid(p.NT, a.T, BM, 1), st);
    }
    p.NT = wide_tiles;
    return launch_stages<1, 2>(p, gemm_grid(p.NT, a.T, BM, 1), st);
}


}  // namespace moe
