// a3. Grouped SwiGLU expert FFN, bf16 operands, fp32 accumulation, on the CDNA4
// matrix cores (v_mfma_f32_16x16x32_bf16), weights read through the page table.
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
// Swizzles.  An MFMA operand fetch is a ds_read_b128 with one row per lane (row lane % 16, 16-byte
// chunk lane / 16).  The 64 banks hold 256 consecutive bytes and the 64 lanes are served in four
// phases of 16 lanes - but not 16 consecutive lanes: measured with the bank-conflict counter on ten
// layouts, rows r and r + 8 of two neighbouring chunks meet in a phase.  In a 64-byte-row stage the
// chunk c of row r therefore sits at position c ^ (2 * ((r >> 3) & 1)) (rows r and r + 8 share a bank
// row), in a 128-byte-row stage at c ^ ((r >> 1) & 7): both measured free of conflicts, 4 cycles per
// fetch.  (With c ^ ((r >> 2) & 3), which is right for 16 consecutive lanes and for the lane layout
// of the 32x32 MFMA, every weight fetch of this kernel took 8 cycles.)
//
// Schedule.  Measured on this chip: when all wavefronts issue their loads, then
// their LDS fetches, then their MFMAs in blocks after each barrier, the matrix
// cores idle while every wavefront queues at the memory pipeline (about 63 %
// utilisation).  The loop is therefore (a) rotated: half of the MFMAs of half-step
// k-1 are issued AFTER the barrier that opens half-step k, so the matrix cores have
// work while the wavefronts synchronise and the first operands of k are fetched,
// and (b) interleaved: between two MFMAs of a full tile at most one LDS fetch or one
// global load is issued.  Scheduling fences pin that order.
//
// Wavefront w computes rows (w / 2) * 128 .. +127 and, of the 256 columns, for
// MODE 0 columns (w % 2) * 64 .. +63 of both tiles, for MODE 1 columns
// (w % 2) * 128 .. +127: 8 x 8 MFMA tiles of 16 x 16, 256 accumulator registers.
// Measured against 8 wavefronts of 128 x 64 each: a 128 x 128 wavefront tile needs
// a third less LDS traffic per MFMA; the chip is power limited under this load, the
// clock rises and the loop runs ~10 % faster.  Measured for the MFMA shape (a loop
// of nothing but MFMAs on random bf16 operands, all compute units): 16x16x32 sustains
// 2.08 PFLOP/s at 2.05 GHz, 32x32x16 1.82 PFLOP/s at 1.76 GHz - the same arithmetic,
// but half the accumulator traffic per multiply-add, and the power limit, not the
// issue rate, sets the speed.
#include <algorithm>
#include <mutex>
#include <type_traits>
#include <utility>

#include "moe_ffn_common.h"

namespace moe {
namespace {

#define MOE_FENCE() __builtin_amdgcn_sched_barrier(0)

typedef int i32x4 __attribute__((ext_vector_type(4)));        // an MFMA operand: 8 bf16 in four registers
typedef float f32x4 __attribute__((ext_vector_type(4)));
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

// D = A * B + D on a 16 x 16 tile over 32 k (v_mfma_f32_16x16x32_bf16): lane l holds row l % 16 of A
// and column l % 16 of B, each the 8 elements k = (l / 16) * 8 .. + 7, and D[(l / 16) * 4 + r][l % 16] in
// register r of the tile's four.
//
// The accumulators are the accumulator registers a0 .. a255 (a0 .. a127 for the narrow block) NAMED in
// inline assembly, tile t in a[4t : 4t + 3]; the compiler never sees them as values.  With the
// builtin, or with "+a" operands, the register allocator copies accumulator tiles between registers
// inside or next to the loop; it does not know that the asm is an MFMA whose result lands passes
// later, and such a copy reads or overwrites a register an MFMA in flight still writes.  So:
// acc_declare() makes the registers part of the kernel's register count, acc_zero / acc_read are the
// only other accesses, and acc_read may only run after mfma_drain().
template <int NREGS>
__device__ __forceinline__ void acc_declare() {
#ifdef __HIP_DEVICE_COMPILE__        // the host pass of the compiler does not know these registers
    if (NREGS == 256) asm volatile("" ::: "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", "a10", "a11", "a12", "a13", "a14", "a15", "a16", "a17", "a18", "a19", "a20", "a21", "a22", "a23", "a24", "a25", "a26", "a27", "a28", "a29", "a30", "a31", "a32", "a33", "a34", "a35", "a36", "a37", "a38", "a39", "a40", "a41", "a42", "a43", "a44", "a45", "a46", "a47", "a48", "a49", "a50", "a51", "a52", "a53", "a54", "a55", "a56", "a57", "a58", "a59", "a60", "a61", "a62", "a63", "a64", "a65", "a66", "a67", "a68", "a69", "a70", "a71", "a72", "a73", "a74", "a75", "a76", "a77", "a78", "a79", "a80", "a81", "a82", "a83", "a84", "a85", "a86", "a87", "a88", "a89", "a90", "a91", "a92", "a93", "a94", "a95", "a96", "a97", "a98", "a99", "a100", "a101", "a102", "a103", "a104", "a105", "a106", "a107", "a108", "a109", "a110", "a111", "a112", "a113", "a114", "a115", "a116", "a117", "a118", "a119", "a120", "a121", "a122", "a123", "a124", "a125", "a126", "a127", "a128", "a129", "a130", "a131", "a132", "a133", "a134", "a135", "a136", "a137", "a138", "a139", "a140", "a141", "a142", "a143", "a144", "a145", "a146", "a147", "a148", "a149", "a150", "a151", "a152", "a153", "a154", "a155", "a156", "a157", "a158", "a159", "a160", "a161", "a162", "a163", "a164", "a165", "a166", "a167", "a168", "a169", "a170", "a171", "a172", "a173", "a174", "a175", "a176", "a177", "a178", "a179", "a180", "a181", "a182", "a183", "a184", "a185", "a186", "a187", "a188", "a189", "a190", "a191", "a192", "a193", "a194", "a195", "a196", "a197", "a198", "a199", "a200", "a201", "a202", "a203", "a204", "a205", "a206", "a207", "a208", "a209", "a210", "a211", "a212", "a213", "a214", "a215", "a216", "a217", "a218", "a219", "a220", "a221", "a222", "a223", "a224", "a225", "a226", "a227", "a228", "a229", "a230", "a231", "a232", "a233", "a234", "a235", "a236", "a237", "a238", "a239", "a240", "a241", "a242", "a243", "a244", "a245", "a246", "a247", "a248", "a249", "a250", "a251", "a252", "a253", "a254", "a255");
    else asm volatile("" ::: "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", "a10", "a11", "a12", "a13", "a14", "a15", "a16", "a17", "a18", "a19", "a20", "a21", "a22", "a23", "a24", "a25", "a26", "a27", "a28", "a29", "a30", "a31", "a32", "a33", "a34", "a35", "a36", "a37", "a38", "a39", "a40", "a41", "a42", "a43", "a44", "a45", "a46", "a47", "a48", "a49", "a50", "a51", "a52", "a53", "a54", "a55", "a56", "a57", "a58", "a59", "a60", "a61", "a62", "a63", "a64", "a65", "a66", "a67", "a68", "a69", "a70", "a71", "a72", "a73", "a74", "a75", "a76", "a77", "a78", "a79", "a80", "a81", "a82", "a83", "a84", "a85", "a86", "a87", "a88", "a89", "a90", "a91", "a92", "a93", "a94", "a95", "a96", "a97", "a98", "a99", "a100", "a101", "a102", "a103", "a104", "a105", "a106", "a107", "a108", "a109", "a110", "a111", "a112", "a113", "a114", "a115", "a116", "a117", "a118", "a119", "a120", "a121", "a122", "a123", "a124", "a125", "a126", "a127");
#endif
}
template <int R>
__device__ __forceinline__ void mfma_16x16x32(const i32x4& a, const i32x4& b) {     // tile in a[R : R + 3]
#ifdef __HIP_DEVICE_COMPILE__
    asm volatile("v_mfma_f32_16x16x32_bf16 a[%2:%3], %0, %1, a[%2:%3]" ::"v"(a), "v"(b), "n"(R), "n"(R + 3));
#endif
}
// The same MFMA with one global -> LDS load of 16 bytes per lane behind it: LDS address
// lds_base + LDS_IMM + lane * 16 (through M0, written before the MFMA so that the MFMA fills the
// wait state the load needs after it), global address base + offset[lane].  One statement, so nothing
// can come between the write of M0 and the load; the scalar base + 32-bit lane offset form of the load
// needs no 64-bit vector addition (the builtin's flat-pointer form costs one per load).
// (The compiler puts an s_nop in front of every such statement that follows another within a few instructions, because
// M0 is on the clobber list: six per half-step.  They issue in the shadow of an MFMA: a build without the clobber,
// and so without them, was not faster.)
template <int R, int LDS_IMM>
__device__ __forceinline__ void mfma_16x16x32_then_load(const i32x4& a, const i32x4& b, const char* base, uint32_t offset, uint32_t lds_base) {
#ifdef __HIP_DEVICE_COMPILE__
    asm volatile("s_add_i32 m0, %4, %5\n\tv_mfma_f32_16x16x32_bf16 a[%6:%7], %0, %1, a[%6:%7]\n\tglobal_load_lds_dwordx4 %2, %3"
                 ::"v"(a), "v"(b), "v"(offset), "s"(base), "s"(lds_base), "n"(LDS_IMM), "n"(R), "n"(R + 3)
                 : "memory", "m0");
#endif
}
// The same MFMA with its accumulator tile in vector registers the compiler allocates, and a plain 16-byte load
// into vector registers: the tall tiles' extra row tile.  The load is not known to the compiler's wait counting;
// its result is used only behind a wait that covers it.
__device__ __forceinline__ void mfma_16x16x32_v(f32x4& acc, const i32x4& a, const i32x4& b) {
#ifdef __HIP_DEVICE_COMPILE__
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
#endif
}
// The MFMAs of a tall tile's extra row tile, all in ONE statement: acc[j] += a * b[j] for the column fragments that
// `which` selects - 0: all of them; 1 / 2: the first / second half of a split (see the kernel), i.e. with GATE_UP the
// gate fragments 0, 1 (2, 3) and their up fragments 4, 5 (6, 7), else fragments 0 .. NJ/2-1 (NJ/2 .. NJ-1).  The choice
// is a branch INSIDE the statement: the compiler sees one unconditional read-modify-write of all accumulator tiles and
// has no control flow to merge them across (with a branch in the source it copied the tiles next to the MFMAs that
// were still writing them).
template <bool GATE_UP>
__device__ __forceinline__ void mfma_extra_tile_8(f32x4 (&acc)[8], const i32x4& a, const i32x4 (&b)[8], int which) {
#ifdef __HIP_DEVICE_COMPILE__
#define MOE_XM(J) "v_mfma_f32_16x16x32_bf16 %" #J ", %8, %" MOE_XB_##J ", %" #J "\n\t"
#define MOE_XB_0 "9"
#define MOE_XB_1 "10"
#define MOE_XB_2 "11"
#define MOE_XB_3 "12"
#define MOE_XB_4 "13"
#define MOE_XB_5 "14"
#define MOE_XB_6 "15"
#define MOE_XB_7 "16"
    if constexpr (GATE_UP) {
        asm volatile("s_cmp_lg_u32 %17, 0\n\ts_cbranch_scc1 1f\n\t"
                     MOE_XM(0) MOE_XM(1) MOE_XM(2) MOE_XM(3) MOE_XM(4) MOE_XM(5) MOE_XM(6) MOE_XM(7)
                     "s_branch 3f\n1:\n\ts_cmp_lg_u32 %17, 1\n\ts_cbranch_scc1 2f\n\t"
                     MOE_XM(0) MOE_XM(1) MOE_XM(4) MOE_XM(5)
                     "s_branch 3f\n2:\n\t"
                     MOE_XM(2) MOE_XM(3) MOE_XM(6) MOE_XM(7)
                     "3:\n\t"
                     : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "+v"(acc[4]), "+v"(acc[5]), "+v"(acc[6]), "+v"(acc[7])
                     : "v"(a), "v"(b[0]), "v"(b[1]), "v"(b[2]), "v"(b[3]), "v"(b[4]), "v"(b[5]), "v"(b[6]), "v"(b[7]), "s"(which)
                     : "scc");
    } else {
        asm volatile("s_cmp_lg_u32 %17, 0\n\ts_cbranch_scc1 1f\n\t"
                     MOE_XM(0) MOE_XM(1) MOE_XM(2) MOE_XM(3) MOE_XM(4) MOE_XM(5) MOE_XM(6) MOE_XM(7)
                     "s_branch 3f\n1:\n\ts_cmp_lg_u32 %17, 1\n\ts_cbranch_scc1 2f\n\t"
                     MOE_XM(0) MOE_XM(1) MOE_XM(2) MOE_XM(3)
                     "s_branch 3f\n2:\n\t"
                     MOE_XM(4) MOE_XM(5) MOE_XM(6) MOE_XM(7)
                     "3:\n\t"
                     : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "+v"(acc[4]), "+v"(acc[5]), "+v"(acc[6]), "+v"(acc[7])
                     : "v"(a), "v"(b[0]), "v"(b[1]), "v"(b[2]), "v"(b[3]), "v"(b[4]), "v"(b[5]), "v"(b[6]), "v"(b[7]), "s"(which)
                     : "scc");
    }
#endif
}
// the same for the narrow block's four column fragments (down projection only): halves 0, 1 and 2, 3
__device__ __forceinline__ void mfma_extra_tile_4(f32x4 (&acc)[4], const i32x4& a, const i32x4 (&b)[4], int which) {
#ifdef __HIP_DEVICE_COMPILE__
#define MOE_YM(J, B) "v_mfma_f32_16x16x32_bf16 %" #J ", %4, %" #B ", %" #J "\n\t"
    asm volatile("s_cmp_lg_u32 %9, 0\n\ts_cbranch_scc1 1f\n\t"
                 MOE_YM(0, 5) MOE_YM(1, 6) MOE_YM(2, 7) MOE_YM(3, 8)
                 "s_branch 3f\n1:\n\ts_cmp_lg_u32 %9, 1\n\ts_cbranch_scc1 2f\n\t"
                 MOE_YM(0, 5) MOE_YM(1, 6)
                 "s_branch 3f\n2:\n\t"
                 MOE_YM(2, 7) MOE_YM(3, 8)
                 "3:\n\t"
                 : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3])
                 : "v"(a), "v"(b[0]), "v"(b[1]), "v"(b[2]), "v"(b[3]), "s"(which)
                 : "scc");
#endif
}
__device__ __forceinline__ void load_vgpr_16(i32x4& dst, const char* ptr) {
#ifdef __HIP_DEVICE_COMPILE__
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(ptr) : "memory");
#endif
}
template <int R>
__device__ __forceinline__ void acc_zero() {
#ifdef __HIP_DEVICE_COMPILE__
    asm volatile("v_accvgpr_write_b32 a[%0], 0" ::"n"(R));
#endif
}
template <int R>
__device__ __forceinline__ float acc_read() {
    float v = 0.f;
#ifdef __HIP_DEVICE_COMPILE__
    asm volatile("v_accvgpr_read_b32 %0, a[%1]" : "=v"(v) : "n"(R));
#endif
    return v;
}
__device__ __forceinline__ void mfma_drain() {      // more wait states than the longest MFMA pipeline needs
#ifdef __HIP_DEVICE_COMPILE__
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
#endif
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}


// NB: page tiles per block along the columns.  2: the 256-column block described above.  1 (MODE 1
// only): 256 rows x 128 columns, wavefront tile 128 x 64, for launches with too few 256-wide tiles
// to occupy the chip (few rows per expert: the launch is bound by streaming the weights, and more
// blocks stream more).
template <int MODE, int NB>
__global__ __launch_bounds__(kThreads) void ffn_gemm_bf16(const GemmParams p) {
    constexpr int S = kStages;
    // GU1: the gate/up block with half the columns: 64 features, i.e. the 64 rows of the W1 tile and of the W3 tile that
    // belong to them (rows sel*64 .. of both page tiles; a page tile's LDS image is linear in its rows, so half of it is
    // one 4 KiB piece).  In LDS the stage looks like the one page tile of the narrow down block: rows 0..63 gate, 64..127 up.
    constexpr bool GU1 = MODE == 0 && NB == 1;
    constexpr bool TWO_WALKS = NB == 2 || GU1;   // two page tiles are walked along k
    constexpr int NJ = 4 * NB;                   // 16-column MFMA tiles (B fragments) per wavefront
    constexpr int NMF = 4 * NJ;                  // MFMAs of a group: four 16-row tiles x NJ
    constexpr int kLoadsPerStage = 4 + 2 * NB;   // global_load_lds instructions per wavefront per stage
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    // ---- which tile is mine -------------------------------------------------
    const TileCoord tc = locate_tile<BM>(p);
    if (!tc.valid) return;
    // diagnostic: some blocks report the shader clock they saw (cycle counter against the 100 MHz
    // constant counter over the whole tile); the chip is power limited under this kernel
    const bool clock_probe = p.status && (blockIdx.x & 511) == 256 && tid == 0;
    long long probe_c = 0, probe_w = 0;
    if (clock_probe) {
        probe_c = clock64();
        probe_w = wall_clock64();
    }
    const int e = tc.e, nt = tc.nt, row0 = tc.row0, rows_here = tc.rows_here;
    // With a_gather the activation rows come from the matrix at A through an index: lane L of the wavefront
    // looks up the source of the wavefront's row (L / 8 * 4 + wave) * 8 + L % 8 here (one division per lane,
    // the load under way during the page-table lookups).
    uint32_t gathered = 0;
    if (p.a_gather) {
        const int r = min(((lane >> 3) * kWaves + wave) * 8 + (lane & 7), rows_here - 1);     // row0 + r is a row of this expert
        gathered = (uint32_t)min(max(p.a_gather[row0 + r] / p.a_div, 0), p.a_rows - 1);      // clamped into the matrix at A
    }

    // ---- weight tiles through the page table -------------------------------------
    const int32_t* trow = p.table + (size_t)(p.table_row_mod ? e % p.table_row_mod : e) * p.ppe + p.group_base;
    const int pt0 = GU1 ? (nt >> 1) * 2 : nt * NB;
    const int pt1 = (pt0 + 1 < p.n_page_tiles) ? pt0 + 1 : pt0;   // odd tile count: the second half is masked (NB = 2)
    const int sel = GU1 ? (nt & 1) : 0;                           // GU1: which half of the two page tiles' rows
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
    TileWalk w0 = walk_start(pt0 * p.KT), w1 = walk_start(pt1 * p.KT);
    // Both walks one tile on.  ONE test for the rare page boundary, marked unlikely so that the look-up sits out of line
    // and the common path falls through: with one wavefront per SIMD every taken branch is some 30 cycles without an
    // MFMA, and a test per walk that jumps over its look-up cost two of them per k-step (2.4 % of the loop).
    auto walk_next_both = [&]() __attribute__((always_inline)) {
        w0.tile += 16384;
        ++w0.within;
        if (TWO_WALKS) {
            w1.tile += 16384;
            ++w1.within;
        }
        if (__builtin_expect((w0.within == p.tpp) | (TWO_WALKS && w1.within == p.tpp), 0)) {
            if (w0.within == p.tpp) {
                w0.within = 0;
                w0.tile = page_addr(++w0.page);
            }
            if (TWO_WALKS && w1.within == p.tpp) {
                w1.within = 0;
                w1.tile = page_addr(++w1.page);
            }
        }
    };

    // ---- sources of the global -> LDS loads: a wave-uniform base that moves along k plus a 32-bit
    // offset per lane that never changes, so a half-step costs a few scalar additions ----------------
    // Activation rows are loaded a k-step (128 bytes = one cache line per row) at a time: load
    // instruction q = i*4 + wave (i = 0..7) fills LDS rows q*8 .. q*8+7 (1 KiB); lane j holds row
    // q*8 + j/8 at chunk position j%8, i.e. global chunk (j%8) ^ ((row >> 1) & 7).  Rows past the
    // tail repeat the last row.
    // With a_gather the lanes pick the eight sources they load from the ones looked up above.
    uint32_t a_off[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int lrow = (i * kWaves + wave) * 8 + (lane >> 3);
        const int r = min(lrow, rows_here - 1);
        const int c = (lane & 7) ^ ((lrow >> 1) & 7);
        const uint32_t src = p.a_gather ? (uint32_t)__shfl((int)gathered, i * 8 + (lane >> 3)) : (uint32_t)r;
        a_off[i] = src * (uint32_t)p.lda_bytes + c * 16;
    }
    const char* a_ptr = p.a_gather ? p.A : p.A + (int64_t)row0 * p.lda_bytes;    // + 128 bytes per k-step
    int a_wr = kRingA;                                         // LDS offset of the activation stage being filled
    // A tall tile (up to 32 rows more than BM: its share of the remainder of its expert's rows): wavefront row wm also
    // computes the 16 rows BM + wm*16 .. against its column fragments, which are in registers anyway.  The
    // activation fragment of those rows comes straight from memory (16 bytes per lane and half-step, four
    // half-steps ahead), the eight accumulator tiles live in vector registers.
    // These accumulators and the loaded fragment are values the compiler allocates, and it knows neither that the
    // asm statements that write them are an MFMA (result lands passes later) nor a load (result lands much later):
    // it must never have a reason to copy them.  Any control flow around their uses makes it merge values with
    // register copies next to the asm statements, which then read registers still being written (seen as wrong
    // extra rows when the MFMAs of this block were put under a branch on the number of extra rows).  So: one
    // unconditional sequence per half-step under the single test of `extra`; what varies with the number of extra
    // rows is decided inside the asm statement (mfma_extra_tile_8 / _4).
    const int extra = rows_here > BM ? rows_here - BM : 0;
    // (The 64-feature gate/up block does not split: the halves of its four column fragments are not gate/up pairs.)
    // At most 16 extra rows: ONE extra 16-row MFMA tile, rows BM .. BM + 15, and the two wavefront rows - which hold the
    // same column fragments - take half of the column fragments each (half the extra MFMAs per wavefront).  extra_which:
    // 0 = every fragment (more than 16 extra rows: wavefront row wm has the rows BM + 16 wm ..), 1 / 2 = this
    // wavefront row's half.
    const bool split_extra = !GU1 && extra > 0 && extra <= 16;
    const int extra_which = __builtin_amdgcn_readfirstlane(split_extra ? 1 + wm : 0);
    const char* ae_ptr = p.A;
    i32x4 AE[4];
    f32x4 accE[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) accE[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 4; ++u) AE[u] = i32x4{0, 0, 0, 0};
    if (extra) {
        const int er = min(BM + (split_extra ? 0 : wm * 16) + (lane & 15), rows_here - 1);
        const int64_t src = p.a_gather ? (int64_t)min(max(p.a_gather[row0 + er] / p.a_div, 0), p.a_rows - 1) : (int64_t)row0 + er;
        ae_ptr = p.A + src * p.lda_bytes + (lane >> 4) * 16;      // + 64 bytes per half-step
    }
    const uint32_t b_off = wave * 1024 + lane * 16;            // weight half-tiles are copied linearly

    // The loads issued during half-step h: activation instructions (h & 1) * 4 + i (i = 0..3) of the
    // k-step two ahead, and the weight stage of half-step h + 3 (instructions 4, 5: half-tile 0; 6, 7:
    // half-tile 1) into weight slot `slot`.  After the last instruction of a kind the sources move on.
    const int KH = 2 * p.KT;
    const uint32_t lds_wave = (uint32_t)(uintptr_t)(lptr_t)smem + wave * 1024;      // LDS address of this wavefront's 1 KiB inside a 4 KiB load group
    uint32_t a_wr_w = lds_wave + kRingA;                       // the same inside the activation stage being filled
    const uint32_t a_wr_last = lds_wave + kRingA + (kStagesA - 1) * kStageA;
    uint32_t b_voff[2][2];                                      // [odd half-step][first or second 4 KiB of the half-tile]
#pragma unroll
    for (int o = 0; o < 2; ++o)
#pragma unroll
        for (int h = 0; h < 2; ++h) b_voff[o][h] = o * kHalfTile + (GU1 ? sel : h) * (kWaves * 1024) + b_off;     // GU1: both loads read piece `sel` of their tile
    auto advance_a = [&](int ia) __attribute__((always_inline)) {
        if (ia == 7) {
            a_ptr += kARowB;
            a_wr = (a_wr == kRingA + (kStagesA - 1) * kStageA) ? kRingA : a_wr + kStageA;
            a_wr_w = (a_wr_w == a_wr_last) ? lds_wave + kRingA : a_wr_w + kStageA;
        }
    };
    auto advance_b = [&](int kn, int odd, int i) __attribute__((always_inline)) {
        if (i == 2 * NB - 1 && odd && kn + 1 < KH) walk_next_both();
    };
    // the loads of the prologue (no MFMA to pair them with)
    auto load_a = [&](int part, int i) __attribute__((always_inline)) {
        const int ia = part * 4 + i;
        __builtin_amdgcn_global_load_lds((gptr_t)(a_ptr + a_off[ia]), (lptr_t)(smem + a_wr + (ia * kWaves + wave) * 1024), 16, 0, 0);
        advance_a(ia);
    };
    auto load_b = [&](int slot, int kn, int odd, int i) __attribute__((always_inline)) {     // odd = kn & 1, known at compile time by the callers
        char* st = smem + slot * kStageB;
        const TileWalk& w = (GU1 ? i < 1 : i < 2) ? w0 : w1;
        const int part = (i & 1) * (kWaves * 1024);                       // first or second 4 KiB of the half-tile in LDS
        const char* b = w.tile + odd * kHalfTile + (GU1 ? sel * (kWaves * 1024) : part);
        __builtin_amdgcn_global_load_lds((gptr_t)(b + b_off), (lptr_t)(st + (i >= 2 ? kHalfTile : 0) + part + wave * 1024), 16, 0, 0);
        advance_b(kn, odd, i);
    };

    // accumulator tile (i, j), rows wm*128 + i*16, columns by B fragment j: registers a[(i*NJ + j)*4 ..+3]
    // (zeroed in the main loop, behind the first loads)
    acc_declare<32 * NJ>();

    // LDS byte offsets of this lane's operand chunks: row lane%16 of a 16-row MFMA tile, chunk lane/16
    // of the four a half-step has.  Weights (64-byte rows, one half-step per stage): chunk lane/16;
    // activations (128-byte rows, two half-steps per stage): chunk 4*hp + lane/16 in half-step parity hp.
    const int b_frag0 = (lane & 15) * kRowB + (((lane >> 4) ^ ((lane >> 2) & 2)) << 4);
    // B fragment j: MODE 0: gate rows wn*64 + (j%4)*16 of tile 0 (j < 4), the same up rows of tile 1 (j >= 4);
    //               GU1:    gate rows wn*32 + (j%2)*16 of the stage's rows 0..63 (j < 2), the same up rows of its rows 64..127;
    //               MODE 1: rows wn*(16*NJ) + j*16 of the 128*NB rows of the block's tiles
    int b_base[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j)
        b_base[j] = (GU1 ? (j >> 1) * 64 + wn * 32 + (j & 1) * 16
                         : (MODE == 0) ? (j >> 2) * 128 + wn * 64 + (j & 3) * 16 : wn * (16 * NJ) + j * 16) * kRowB;

    // operand registers: two sets of four activation fragments, two sets of weight fragments
    i32x4 AX[4], AY[4], BF[2][NJ];
#pragma unroll
    for (int i = 0; i < 4; ++i) AX[i] = AY[i] = i32x4{0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < NJ; ++j) BF[0][j] = BF[1][j] = i32x4{0, 0, 0, 0};   // the first rotated MFMA group adds 0 * 0

    auto fetch_b = [&](const char* st, int set, int j) __attribute__((always_inline)) {     // st: weight stage
        BF[set][j] = *(const i32x4*)(st + b_base[j] + b_frag0);
    };
    // accumulator tile (I, J) += a * b, alone or with a load behind it
    auto mfma = [&](auto i_c, auto j_c, const i32x4& a, const i32x4& b) __attribute__((always_inline)) {
        mfma_16x16x32<(decltype(i_c)::value * NJ + decltype(j_c)::value) * 4>(a, b);
    };
    auto mfma_load_a = [&](auto i_c, auto j_c, const i32x4& a, const i32x4& b, auto ia_c) __attribute__((always_inline)) {   // + activation load instruction IA
        constexpr int IA = decltype(ia_c)::value;
        mfma_16x16x32_then_load<(decltype(i_c)::value * NJ + decltype(j_c)::value) * 4, IA * kWaves * 1024>(a, b, a_ptr, a_off[IA], a_wr_w);
        advance_a(IA);
    };
    auto mfma_load_b = [&](auto i_c, auto j_c, const i32x4& a, const i32x4& b, auto slot_c, auto l_c, int kn) __attribute__((always_inline)) {   // + weight load instruction L of half-step kn into slot SLOT
        constexpr int SLOT = decltype(slot_c)::value, I = decltype(l_c)::value;
        constexpr int odd = SLOT & 1;               // S is even: the parity of the half-step is that of its slot
        mfma_16x16x32_then_load<(decltype(i_c)::value * NJ + decltype(j_c)::value) * 4, SLOT * kStageB + (I >= 2 ? kHalfTile : 0) + (I & 1) * (kWaves * 1024)>(
            a, b, ((GU1 ? I < 1 : I < 2) ? w0 : w1).tile, b_voff[odd][I & 1], lds_wave);
        advance_b(kn, odd, I);
    };

    // The main loop for a tile of 256 rows (HALF = false) or of at most 128 rows (HALF = true).
    //
    // 256 rows: wavefront (wm, wn) owns rows wm*128 .. +127: row tiles 0..3 through the fragment set AX,
    // 4..7 through AY.  A half-step on weight-ring slot U (a compile-time constant: every weight address
    // in LDS is an immediate; the activation stage moves through per-lane offsets) is two groups of
    // MFMAs with the other instructions spread between them, at most one behind an MFMA:
    //   group 1: row tiles 4..7 of half-step k-1 (operands fetched during k-1); fetches the weight
    //            fragments of k and the activation fragments of row tiles 0..3; issues the activation loads;
    //   group 2: row tiles 0..3 of half-step k; fetches the activation fragments of row tiles 4..7;
    //            issues the weight loads.
    // Short tiles.  At most 128 rows: wavefront (wm, wn) owns rows wm*64 .. +63, four row tiles; the two
    // fragment sets alternate between half-steps, and the groups split the columns instead:
    //   group 1: the second half of the column fragments of half-step k-1; fetches all fragments of k;
    //            issues the activation loads (even half-steps only: rows 128..255 are not loaded at all);
    //   group 2: the first half of the column fragments of half-step k; issues the weight loads.
    // At most 64 rows: the same with the wavefronts wm = 1 taking part in the loads only; at most 32
    // rows: two row tiles instead of four.  Measured in cycles of a full tile: 0.6 for the first, and
    // the launches of the Mixtral-8x7B-shaped workload (whose short tiles have 4 to 31 rows) got 2-3 %
    // shorter with the other two: under the power limit every MFMA on repeated rows costs time.
    // LA / LB: issue the activation / weight loads of this half-step.  WAITN: my loads that may still
    // be in flight when the stages of half-step k must be complete (those issued during the two
    // half-steps before).  Weight fragment set U & 1 belongs to half-step k: S is even, so the parity of
    // k is static too.
    // TALL: the loop of a tall tile (full loop only).  A copy of the loop of its own rather than a test of `extra` in
    // every half-step: with one wavefront per SIMD a taken branch costs some 30 cycles of an idle matrix core, and the
    // test cost two of them (to the block and back) plus the branch around its load: measured per half-step about as
    // much as the eight extra MFMAs themselves (a tall tile took 15 % longer than a full one for 12.5 % more MFMAs with
    // the extra tile's loads taken out, and still 15 % longer with half the extra MFMAs).
    auto main_loop = [&](auto half_tile_c, auto rt_c, auto na_c, auto tall_c) __attribute__((always_inline)) {
        using std::integral_constant;
        constexpr bool HALF = decltype(half_tile_c)::value;
        constexpr bool TALL = decltype(tall_c)::value;
        static_assert(!(HALF && TALL), "tall tiles run the full loop");
        constexpr int RT = decltype(rt_c)::value;       // short tiles: row tiles a wavefront computes (4, 2)
        constexpr int NA = decltype(na_c)::value;       // short tiles: activation load instructions per k-step (4, 2, 1: 32 rows each)
        constexpr int WROWS = HALF ? 64 : 128;          // rows of a wavefront
        const bool wact = !HALF || wm == 0 || rows_here > 64;    // a short tile with at most 64 rows is the upper wavefronts' alone
        int a_frag[2];                    // includes the activation stage being read: moves on after every odd half-step
#pragma unroll
        for (int hp = 0; hp < 2; ++hp)
            a_frag[hp] = kRingA + wm * WROWS * kARowB + (lane & 15) * kARowB + (((4 * hp + (lane >> 4)) ^ ((lane >> 1) & 7)) << 4);
        int a_rd = 0;                     // activation stage being read
        auto fetch_a = [&](int hp, int i, i32x4& dst) __attribute__((always_inline)) {      // row tile i of this wavefront in the activation stage being read
            dst = *(const i32x4*)(smem + a_frag[hp] + i * 16 * kARowB);
        };

        auto half_step = [&](int k, auto u_c, auto la_c, auto lb_c, auto waitn_c) __attribute__((always_inline)) {
            constexpr int U = decltype(u_c)::value;
            constexpr int HP = U & 1;
            constexpr bool LA = decltype(la_c)::value, LB = decltype(lb_c)::value;
            wait_loads_and_lds<decltype(waitn_c)::value>();
            __builtin_amdgcn_s_barrier();      // the stages of k are complete for everyone; nobody reads those of k-1 any more
            asm volatile("" ::: "memory");
            const char* st = smem + U * kStageB;
            constexpr int nslot = (U + S - 1) % S;
            const int kn = k + S - 1;
            MOE_FENCE();
            if constexpr (!HALF) {
                constexpr int NF1 = NJ + 4;                         // fetches of group 1: B0, A0, B1 .. B(NJ-1), A1, A2, A3
                constexpr int LA0 = NF1 + (NB == 2 ? 2 : 1), LAS = NB == 2 ? 4 : 2;     // MFMAs with an activation load behind them
                static_for<NMF>([&](auto mc) __attribute__((always_inline)) {
                    constexpr int m = decltype(mc)::value;
                    constexpr int r = m / NJ, j = (r & 1) ? NJ - 1 - m % NJ : m % NJ;   // back and forth: one operand stays at each row change
                    constexpr bool ld = LA && m >= LA0 && (m - LA0) % LAS == 0 && (m - LA0) / LAS < 4;
                    if constexpr (ld) mfma_load_a(integral_constant<int, 4 + r>{}, integral_constant<int, j>{}, AY[r], BF[HP ^ 1][j], integral_constant<int, HP * 4 + (m - LA0) / LAS>{});
                    else mfma(integral_constant<int, 4 + r>{}, integral_constant<int, j>{}, AY[r], BF[HP ^ 1][j]);
                    MOE_FENCE();
                    if (m < NF1) {
                        if (m == 1) fetch_a(HP, 0, AX[0]);
                        else if (m > NJ) fetch_a(HP, m - NJ, AX[m - NJ]);
                        else fetch_b(st, HP, m == 0 ? 0 : m - 1);
                        MOE_FENCE();
                    }
                });
                // Every fragment fetched above is in its registers by now (the last fetch is NMF - NF1 MFMAs old).  Said
                // with ONE full wait: left to itself the compiler either does the same or, when it can count the
                // outstanding fetches exactly (seen when a wait instruction stood in front of the loop), puts a counted
                // wait in front of every MFMA that uses a fragment for the first time - ten more instructions per
                // half-step for the one wavefront of the SIMD to issue.
                __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0)
                MOE_FENCE();
                constexpr int LB0 = NB == 2 ? 8 : 6, LBS = NB == 2 ? 6 : 5;             // MFMAs with a weight load behind them
                static_for<NMF>([&](auto mc) __attribute__((always_inline)) {
                    constexpr int m = decltype(mc)::value;
                    constexpr int r = m / NJ, j = (r & 1) ? NJ - 1 - m % NJ : m % NJ;   // back and forth: one operand stays at each row change
                    constexpr bool ld = LB && m >= LB0 && (m - LB0) % LBS == 0 && (m - LB0) / LBS < 2 * NB;
                    if constexpr (ld) mfma_load_b(integral_constant<int, r>{}, integral_constant<int, j>{}, AX[r], BF[HP][j], integral_constant<int, nslot>{}, integral_constant<int, (m - LB0) / LBS>{}, kn);
                    else mfma(integral_constant<int, r>{}, integral_constant<int, j>{}, AX[r], BF[HP][j]);
                    MOE_FENCE();
                    if (m < 4) {
                        fetch_a(HP, 4 + m, AY[m]);
                        MOE_FENCE();
                    }
                });
                if constexpr (TALL) {                        // tall tile: the extra row tile against the column fragments of k
                    if constexpr (NJ == 8) mfma_extra_tile_8<MODE == 0>(accE, AE[U], BF[HP], extra_which);
                    else mfma_extra_tile_4(accE, AE[U], BF[HP], extra_which);
                    MOE_FENCE();
                    // the fragment of half-step k + 4: there is one exactly while the activation loads go on (the last four
                    // half-steps run without LA), so no test of k is needed
                    if constexpr (LA) load_vgpr_16(AE[U], ae_ptr + (int64_t)(k + 4) * 64);
                    MOE_FENCE();
                }
            } else if (wact) {
                constexpr int NH = NJ / 2, NG = RT * NH;            // column fragments and MFMAs of a group
                constexpr int NF1 = NJ + RT;                        // fetches of group 1: B0, A0, B1 .. B(NJ-1), A1 .. A(RT-1)
                static_for<NG>([&](auto mc) __attribute__((always_inline)) {
                    constexpr int m = decltype(mc)::value;
                    constexpr int r = m / NH, j = NH + ((r & 1) ? NH - 1 - m % NH : m % NH);
                    constexpr bool ld = LA && HP == 0 && m >= NG - NA;              // the last NA MFMAs have an activation load behind them
                    const i32x4& a_prev = HP ? AX[r] : AY[r];       // half-step k-1 used the other set
                    if constexpr (ld) mfma_load_a(integral_constant<int, r>{}, integral_constant<int, j>{}, a_prev, BF[HP ^ 1][j], integral_constant<int, ld ? m - (NG - NA) : 0>{});
                    else mfma(integral_constant<int, r>{}, integral_constant<int, j>{}, a_prev, BF[HP ^ 1][j]);
                    MOE_FENCE();
                    static_for<NF1>([&](auto fc) __attribute__((always_inline)) {    // the fetches, spread evenly behind the MFMAs
                        constexpr int f = decltype(fc)::value;
                        if constexpr (f * NG / NF1 == m) {
                            if (f == 1) fetch_a(HP, 0, HP ? AY[0] : AX[0]);
                            else if (f > NJ) fetch_a(HP, f - NJ, HP ? AY[f - NJ] : AX[f - NJ]);
                            else fetch_b(st, HP, f == 0 ? 0 : f - 1);
                            MOE_FENCE();
                        }
                    });
                });
                __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0): as in the full loop
                MOE_FENCE();
                constexpr int LBS = NG / (2 * NB);                  // every LBS-th MFMA has a weight load behind it
                static_for<NG>([&](auto mc) __attribute__((always_inline)) {
                    constexpr int m = decltype(mc)::value;
                    constexpr int r = m / NH, j = (r & 1) ? NH - 1 - m % NH : m % NH;
                    constexpr bool ld = LB && m % LBS == 0 && m / LBS < 2 * NB;
                    const i32x4& a_cur = HP ? AY[r] : AX[r];
                    if constexpr (ld) mfma_load_b(integral_constant<int, r>{}, integral_constant<int, j>{}, a_cur, BF[HP][j], integral_constant<int, nslot>{}, integral_constant<int, ld ? m / LBS : 0>{}, kn);
                    else mfma(integral_constant<int, r>{}, integral_constant<int, j>{}, a_cur, BF[HP][j]);
                    MOE_FENCE();
                });
            } else {                           // a wavefront without rows only takes its part in the loads
                if (LA && HP == 0) {
#pragma unroll
                    for (int i = 0; i < NA; ++i) load_a(0, i);
                }
                if (LB) {
#pragma unroll
                    for (int i = 0; i < 2 * NB; ++i) load_b(nslot, kn, nslot & 1, i);
                }
            }
            if (HALF && LA && HP) {            // a short tile has no second load part: the sources of the k-step two ahead move on here
                a_ptr += kARowB;
                a_wr = (a_wr == kRingA + (kStagesA - 1) * kStageA) ? kRingA : a_wr + kStageA;
                a_wr_w = (a_wr_w == a_wr_last) ? lds_wave + kRingA : a_wr_w + kStageA;
            }
            if (HP) {                          // the next half-step reads the next activation stage
                const int d = (a_rd == kStagesA - 1) ? -(kStagesA - 1) * kStageA : kStageA;
                a_rd = (a_rd == kStagesA - 1) ? 0 : a_rd + 1;
                a_frag[0] += d;
                a_frag[1] += d;
            }
        };

        constexpr int kLB = 2 * NB;                       // weight loads of a half-step
        constexpr int kL2 = HALF ? NA + 2 * kLB : 2 * (4 + kLB);   // loads of two consecutive half-steps
        const std::true_type L{};
        const std::false_type N{};
        // prologue, in the order the half-steps -4 .. -1 would have issued them: activation k-steps
        // 0 and 1, weight half-steps 0 .. 2 (KH is a multiple of 4 and at least 4)
        if constexpr (TALL) {             // the oldest loads of the tile: complete at the first wait
#pragma unroll
            for (int u = 0; u < 4; ++u) load_vgpr_16(AE[u], ae_ptr + u * 64);
        }
#pragma unroll
        for (int i = 0; i < (HALF ? NA : 4); ++i) load_a(0, i);
#pragma unroll
        for (int s = 0; s < S - 1; ++s) {
            if (!HALF || ((s + 1) & 1) == 0) {
#pragma unroll
                for (int i = 0; i < (HALF ? NA : 4); ++i) load_a((s + 1) & 1, i);
            } else {
                advance_a(7);
            }
#pragma unroll
            for (int i = 0; i < kLB; ++i) load_b(s, s, s & 1, i);
        }
        // the accumulators are cleared while the first stages are on their way
        static_for<32 * NJ>([&](auto rc) __attribute__((always_inline)) { acc_zero<decltype(rc)::value>(); });
        int k = 0;
        for (; k + S < KH; k += S) {
            half_step(k, integral_constant<int, 0>{}, L, L, integral_constant<int, kL2>{});
            half_step(k + 1, integral_constant<int, 1>{}, L, L, integral_constant<int, kL2>{});
            half_step(k + 2, integral_constant<int, 2>{}, L, L, integral_constant<int, kL2>{});
            half_step(k + 3, integral_constant<int, 3>{}, L, L, integral_constant<int, kL2>{});
        }
        // last four half-steps: one more weight stage to load, then the rings drain
        half_step(k, integral_constant<int, 0>{}, N, L, integral_constant<int, kL2>{});
        half_step(k + 1, integral_constant<int, 1>{}, N, N, integral_constant<int, (HALF ? 0 : 4) + 2 * kLB>{});
        half_step(k + 2, integral_constant<int, 2>{}, N, N, integral_constant<int, kLB>{});
        half_step(k + 3, integral_constant<int, 3>{}, N, N, integral_constant<int, 0>{});
        // the rotated group of the last half-step (weight fragment set 1: KH is even)
        __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0)
        if constexpr (!HALF) {
            static_for<NMF>([&](auto mc) __attribute__((always_inline)) {
                constexpr int m = decltype(mc)::value;
                mfma(integral_constant<int, 4 + m / NJ>{}, integral_constant<int, m % NJ>{}, AY[m / NJ], BF[1][m % NJ]);
            });
        } else if (wact) {
            static_for<RT * (NJ / 2)>([&](auto mc) __attribute__((always_inline)) {
                constexpr int m = decltype(mc)::value;
                constexpr int NH = NJ / 2;
                mfma(integral_constant<int, m / NH>{}, integral_constant<int, NH + m % NH>{}, AY[m / NH], BF[1][NH + m % NH]);
            });
        }
        mfma_drain();
#pragma unroll
        for (int j = 0; j < NJ; ++j) asm volatile("" : "+v"(accE[j]));      // read only behind the drain
    };
    // A row tile with at most 128 rows takes the half-height loop; any other whose last rows are missing
    // runs the full loop on repeated rows (skipping single MFMAs would take a branch each: a wavefront
    // issues about one instruction in four clocks, and the branches cost more than the MFMAs they skip).
    // Short tiles: at most 128 rows: both wavefront rows, 64 rows each; at most 64: the upper wavefront row
    // alone (the other wavefronts only load); at most 32: two row tiles instead of four.
    const bool half_tile = p.half_tiles && rows_here <= 128;
    using std::integral_constant;
    if (!half_tile && extra) main_loop(std::false_type{}, integral_constant<int, 4>{}, integral_constant<int, 4>{}, std::true_type{});
    else if (!half_tile) main_loop(std::false_type{}, integral_constant<int, 4>{}, integral_constant<int, 4>{}, std::false_type{});
    else if (rows_here > 64) main_loop(std::true_type{}, integral_constant<int, 4>{}, integral_constant<int, 4>{}, std::false_type{});
    else if (rows_here > 32) main_loop(std::true_type{}, integral_constant<int, 4>{}, integral_constant<int, 2>{}, std::false_type{});
    else main_loop(std::true_type{}, integral_constant<int, 2>{}, integral_constant<int, 1>{}, std::false_type{});
    const bool wact = !half_tile || wm == 0 || rows_here > 64;        // this wavefront has rows
    const int row_tiles = !half_tile ? 8 : (rows_here > 32 ? 4 : 2);   // and this many row tiles

    // ---- epilogue ---------------------------------------------------------------------
    // accumulator register r of lane l in MFMA tile (i, j) is the element at row i*16 + (l/16)*4 + r,
    // column l%16 of that 16 x 16 tile
    const int col_l = lane & 15;
    const int a_row_base = wm * (half_tile ? 64 : 128) + (lane >> 4) * 4;
    const bool full_rows = rows_here >= BM;
    // store(i, v): the 4 x NJ x 16 values of row tile i of this wavefront
    auto for_row_tiles = [&](auto n_c, auto&& store) __attribute__((always_inline)) {
        static_for<decltype(n_c)::value>([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value;
            float v[NJ][4];
            static_for<NJ * 4>([&](auto c) __attribute__((always_inline)) {
                constexpr int q = decltype(c)::value;
                v[q >> 2][q & 3] = acc_read<i * NJ * 4 + q>();
            });
            store(i, v);
        });
    };
    if (MODE == 0) {
        constexpr int NP = NJ / 2;             // gate/up pairs of a wavefront: fragments j and j + NP
        __bf16* h = (__bf16*)p.out + (int64_t)row0 * p.ldo + nt * (32 * NP) + wn * (16 * NP) + col_l;
        auto store_rows = [&](auto full, auto n_c) __attribute__((always_inline)) {
            for_row_tiles(n_c, [&](int i, float (&v)[NJ][4]) __attribute__((always_inline)) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = a_row_base + i * 16 + r;
                    if (decltype(full)::value || row < rows_here) {
#pragma unroll
                        for (int j = 0; j < NP; ++j)
                            h[(int64_t)row * p.ldo + j * 16] = (__bf16)silu_mul(v[j][r], v[j + NP][r]);
                    }
                }
            });
        };
        if (full_rows) store_rows(std::true_type{}, std::integral_constant<int, 8>{});
        else if (!wact) {
        } else if (row_tiles == 2) store_rows(std::false_type{}, std::integral_constant<int, 2>{});
        else if (row_tiles == 4) store_rows(std::false_type{}, std::integral_constant<int, 4>{});
        else store_rows(std::false_type{}, std::integral_constant<int, 8>{});
        if (extra) {                           // the extra row tile of a tall tile
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = BM + (split_extra ? 0 : wm * 16) + (lane >> 4) * 4 + r;
                if (row < rows_here) {
#pragma unroll
                    for (int j = 0; j < NP; ++j)
                        if (!split_extra || (j >> 1) == wm)          // split: this wavefront row's gate fragments only
                            h[(int64_t)row * p.ldo + j * 16] = (__bf16)silu_mul(accE[j][r], accE[j + NP][r]);
                }
            }
        }
    } else {
        // the 256 row weights of the tile go through LDS (free now): one load per thread instead of
        // one dependent global load per accumulator row
        float* sw = (float*)smem;
        __syncthreads();                       // every wavefront has left the main loop
        sw[tid] = (p.row_w && tid < rows_here) ? p.row_w[row0 + tid] : 1.0f;
        if (tid < 32) sw[BM + tid] = (p.row_w && BM + tid < rows_here) ? p.row_w[row0 + BM + tid] : 1.0f;     // a tall tile's extra rows
        __syncthreads();
        const int d0 = nt * (128 * NB) + wn * (16 * NJ);   // n_cols is a multiple of 128: with NB = 2 a wavefront's columns are all valid or all not
        if (d0 < p.n_cols) {
            float* o = (float*)p.out + (int64_t)row0 * p.ldo + d0 + col_l;
            auto store_rows = [&](auto full, auto n_c) __attribute__((always_inline)) {
                for_row_tiles(n_c, [&](int i, float (&v)[NJ][4]) __attribute__((always_inline)) {
                    const int rowq = a_row_base + i * 16;      // 4 consecutive rows
                    const float4 wq = *(const float4*)(sw + rowq);
                    const float w4[4] = {wq.x, wq.y, wq.z, wq.w};
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int row = rowq + r;
                        if (decltype(full)::value || row < rows_here) {
#pragma unroll
                            for (int j = 0; j < NJ; ++j)
                                o[(int64_t)row * p.ldo + j * 16] = v[j][r] * w4[r];
                        }
                    }
                });
            };
            if (full_rows) store_rows(std::true_type{}, std::integral_constant<int, 8>{});
            else if (!wact) {
            } else if (row_tiles == 2) store_rows(std::false_type{}, std::integral_constant<int, 2>{});
            else if (row_tiles == 4) store_rows(std::false_type{}, std::integral_constant<int, 4>{});
            else store_rows(std::false_type{}, std::integral_constant<int, 8>{});
            if (extra) {                       // the extra row tile of a tall tile
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = BM + (split_extra ? 0 : wm * 16) + (lane >> 4) * 4 + r;
                    if (row < rows_here) {
                        const float wr = sw[row];
#pragma unroll
                        for (int j = 0; j < NJ; ++j)
                            if (!split_extra || j / (NJ / 2) == wm) o[(int64_t)row * p.ldo + j * 16] = accE[j][r] * wr;      // split: this wavefront row's half
                    }
                }
            }
        }
    }
    if (clock_probe) {
        const long long dc = clock64() - probe_c, dw = wall_clock64() - probe_w;
        if (dw > 0) p.status[2 + MODE] = (int32_t)(dc * 100 / dw);       // MHz
    }
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
    const int64_t rows_each = R / s.E;
    const int64_t row_tiles_each = std::max<int64_t>(1, (rows_each - p.tall_rows + BM - 1) / BM);
    // Gate/up with at most 64 rows per expert on average (the launch streams the weights once): 64-feature column tiles,
    // twice as many blocks of half the work.  Measured on the Mixtral-8x7B shape, narrow against wide, ms for the layer: 32
    // tokens 0.502 / 0.505, 128: 0.506 / 0.514, 256: 0.519 / 0.526, 384: 0.551 / 0.549, 512: 0.623 / 0.592, 1024: 0.83 / 0.77
    // (with more rows a block of half the columns loads the activation rows for half the MFMAs).
    // gate_cols: 0 = this rule, 1 / 2 = force narrow / wide.
    const int gopt = get_opt(OPT_GATE_COLS);
    const bool narrow_gu = gopt == 1 || (gopt == 0 && rows_each <= 64 && n_exp * row_tiles_each * p.NT < 4 * kComputeUnits);
    int rc;
    if (narrow_gu) {
        p.NT = (int32_t)(2 * g.ft);
        rc = launch_stages<0, 1>(p, gemm_grid(p.NT, R, BM, n_exp, p.chunked), st);
    } else {
        rc = launch_stages<0, 2>(p, gemm_grid(p.NT, R, BM, n_exp, p.chunked), st);
    }
    if (rc != MOE_OK) return rc;
    if (a.mid_event) MOE_HIP_TRY(hipEventRecord(a.mid_event, st));
    fill_down(p, s, g, a);
    // Down projection with few row tiles: 256-wide column tiles would leave compute units without a block,
    // so the columns are cut into 128-wide tiles instead.  The routing result is not known here; the choice
    // goes by the row tiles an even split of the rows over the experts would give (the grid is sized by the
    // upper bound as ever).  Measured on the Mixtral-8x7B shape, narrow against wide: 768 tokens 0.23 / 0.29
    // ms, 1024 tokens 0.26 / 0.32, 1280 tokens 0.45 / 0.38, 2048 tokens 0.48 / 0.38.
    // down_cols: 0 = this rule, 1 / 2 = force NB.
    const int opt = get_opt(OPT_DOWN_COLS);
    const bool narrow = opt == 1 || (opt == 0 && n_exp * row_tiles_each * p.NT < kComputeUnits);
    if (narrow) {
        p.NT = (int32_t)g.dt;
        return launch_stages<1, 1>(p, gemm_grid(p.NT, R, BM, n_exp, p.chunked), st);
    }
    return launch_stages<1, 2>(p, gemm_grid(p.NT, R, BM, n_exp, p.chunked), st);
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
    p.half_tiles = get_opt(OPT_HALF_TILES);
    p.tall_rows = get_opt(OPT_TALL_TILES) ? 32 : 0;
    p.tall_first = get_opt(OPT_TALL_FIRST);
    p.balance = get_opt(OPT_BALANCE);
    p.chunked = std::min(std::max(get_opt(OPT_CHUNKED), 0), 32);
    const int wide_tiles = (p.n_page_tiles + 1) / 2;
    if ((int64_t)(a.T / BM + 1) * wide_tiles < 2 * kComputeUnits) {       // too few 256-wide tiles to fill the chip
        p.NT = p.n_page_tiles;
        return launch_stages<1, 1>(p, gemm_grid(p.NT, a.T, BM, 1, p.chunked), st);
    }
    p.NT = wide_tiles;
    return launch_stages<1, 2>(p, gemm_grid(p.NT, a.T, BM, 1, p.chunked), st);
}


}  // namespace moe
