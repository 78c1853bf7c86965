// Pieces shared by the expert-FFN GEMM kernels (bf16 and f32): the launch
// parameter block, the block -> (expert, row tile, column tile) map and the
// page-table lookup of a weight tile.
#pragma once

#include "moe_internal.h"

namespace moe {

struct GemmParams {
    const char* A;            // activations, dtype [R][K] row-major
    int64_t lda_bytes;
    const int32_t* offsets;   // [E+1]
    const int32_t* table;     // page table
    const char* pool;
    int64_t page_bytes;
    int64_t tile_bytes;
    int32_t pool_pages;
    int32_t tpp;              // tiles per page
    int32_t ppe;              // page-table row length
    int32_t group_base;       // first logical page of the weight group (GU: 0, D: pages_gu)
    int32_t KT;               // K / 64
    int32_t NT;               // column tiles of a block grid row (each = two page tiles)
    int32_t n_page_tiles;     // page tiles along N in this group
    int32_t e_begin, e_end;   // experts covered by the launch
    int32_t table_row_mod;    // 0: table row = e; n > 0: table row = e % n
    void* out;
    int32_t ldo;              // elements
    int32_t n_cols;           // valid output columns
    const float* row_w;
    int32_t* status;
    int32_t xcd_remap;
    int32_t half_tiles;       // bf16 kernel: row tiles with at most 128 rows run the half-height loop
    const int32_t* a_gather;  // bf16 kernel, or null: row r of A is row a_gather[r] / a_div of the matrix at A (a_rows rows)
    int32_t a_div, a_rows;
    int32_t tall_rows;        // bf16 kernel: a row tile may be up to this many rows higher than BM (0 or 32), see locate_tile
    int32_t stagger_ticks;    // bf16 kernel: start delay unit of a compute unit's first block, in ticks of the 100 MHz counter
    int32_t stagger_mode;
};

struct TileCoord {
    int e, mt, nt, row0, rows_here;
    bool valid;
};

// Tile order.  The row tiles of one column tile of one expert form a GROUP (they share
// the weight tiles); groups are numbered expert by expert, column tile by column tile.
// With xcd_remap the groups are dealt round robin to the 8 XCDs (block b runs on XCD
// b % 8, each with its own L2): XCD x works through the groups x, x + 8, x + 16, ...
// row tile by row tile, so the blocks an XCD runs at the same time are the row tiles of a
// few column tiles of one expert, and every XCD gets the same mix of experts, hence of
// full and partial row tiles (contiguous chunks of the numbering gave one XCD 22 % more
// full tiles than another on the Mixtral-8x7B-shaped workload).  Without it block b takes
// tile b of the plain numbering.  The tile counts come from offsets[], so the grid is only
// an upper bound and surplus blocks leave at once.
//
// Every wavefront does the search on its own, one expert per lane (at most 64
// experts): one load of the segment bounds, prefix sums of the tile counts over
// the lanes, a ballot to find the expert that holds the tile number.  The result
// is the same in all lanes.
__device__ __forceinline__ int lane_prefix_sum(int v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int u = __shfl_up(v, d, 64);
        if (lane >= d) v += u;
    }
    return v;
}

template <int BM>
__device__ __forceinline__ TileCoord locate_tile(const GemmParams& p) {
    TileCoord t{};
    t.valid = false;
    const int lane = threadIdx.x & 63;
    const int e_l = p.e_begin + lane;
    int seg0 = 0, cnt = 0;
    if (e_l < p.e_end) {
        seg0 = p.offsets[e_l];
        cnt = p.offsets[e_l + 1] - seg0;
    }
    const int stride = p.xcd_remap ? 8 : 1;
    const int x = p.xcd_remap ? (int)(blockIdx.x & 7) : 0;           // my groups: x, x + stride, ...
    const int idx = p.xcd_remap ? (int)(blockIdx.x >> 3) : (int)blockIdx.x;    // my position among their row tiles
    // groups of mine below group number n: ceil((n - x) / stride) for n >= 0 (0 <= x < stride)
    const int g_lo = lane * p.NT, g_hi = g_lo + p.NT;              // group numbers of my lane's expert
    const int c_lo = (g_lo - x + stride - 1) / stride, c_hi = (g_hi - x + stride - 1) / stride;
    // row tiles of my lane's expert.  q full tiles and a remainder r: when r <= tall_rows * q the remainder is
    // spread over the last ceil(r / tall_rows) of the q tiles (each at most BM + tall_rows rows high: as few
    // tall tiles as possible, every one costs an extra 16-row MFMA tile per wavefront), otherwise it is a tile
    // of its own
    const int q_l = cnt / BM, r_l = cnt - q_l * BM;
    const int mtiles_l = (q_l >= 1 && r_l <= p.tall_rows * q_l) ? q_l : q_l + (r_l > 0);
    const int tiles_l = (c_hi - c_lo) * mtiles_l;
    const int incl = lane_prefix_sum(tiles_l, lane);
    if (idx >= __builtin_amdgcn_readlane(incl, 63)) return t;
    const unsigned long long holds = __ballot(idx < incl);           // lanes of this and later experts
    const int src = __builtin_amdgcn_readfirstlane(__ffsll((long long)holds) - 1);
    const int mtiles = __builtin_amdgcn_readfirstlane(__shfl(mtiles_l, src, 64));
    const int before = __builtin_amdgcn_readfirstlane(__shfl(incl - tiles_l, src, 64));
    const int first = __builtin_amdgcn_readfirstlane(__shfl(c_lo, src, 64));       // my groups before this expert
    const int seg = __builtin_amdgcn_readfirstlane(__shfl(seg0, src, 64));
    const int rows = __builtin_amdgcn_readfirstlane(__shfl(cnt, src, 64));
    const int rem = idx - before;
    const int j = rem / mtiles;                                        // my j-th group inside this expert
    t.e = p.e_begin + src;
    t.nt = x + (first + j) * stride - src * p.NT;
    t.mt = rem - j * mtiles;
    const int q = rows / BM, r = rows - q * BM;
    if (r > 0 && q >= 1 && r <= p.tall_rows * q) {
        // the last m tiles are BM + r / m rows high, the first r % m of them one row more
        const int m = (r + p.tall_rows - 1) / p.tall_rows, plain = q - m;
        const int i = t.mt - plain;
        if (i < 0) {
            t.row0 = seg + t.mt * BM;
            t.rows_here = BM;
        } else {
            const int base = BM + r / m, more = r - (r / m) * m;
            t.row0 = seg + plain * BM + i * base + min(i, more);
            t.rows_here = base + (i < more);
        }
    } else {
        t.row0 = seg + t.mt * BM;
        t.rows_here = min(BM, rows - t.mt * BM);
    }
    t.valid = t.rows_here > 0;
    return t;
}

// Address of tile number ti of the group; a page-table entry outside the pool is
// never followed: slot 0 is read instead and *bad is raised.
__device__ __forceinline__ const char* tile_address(const GemmParams& p, const int32_t* trow, int64_t ti, int* bad) {
    const int page = (int)(ti / p.tpp);
    const int within = (int)(ti - (int64_t)page * p.tpp);
    int slot = trow[page];
    if ((unsigned)slot >= (unsigned)p.pool_pages) {
        *bad = 1;
        slot = 0;
    }
    return p.pool + (int64_t)slot * p.page_bytes + (int64_t)within * p.tile_bytes;
}

// grid size that covers every tile for any routing result: an XCD gets at most ceil(NT / 8) of an
// expert's NT groups, each with that expert's row tiles
inline int gemm_grid(int NT, int R, int BM, int n_experts) {
    const int m_tiles_max = R / BM + n_experts;   // >= sum over experts of ceil(rows / BM)
    return 8 * ((NT + 7) / 8) * m_tiles_max;
}

inline void fill_common(GemmParams& p, const moe_shape& s, const Geom& g, const FfnArgs& a) {
    p.offsets = a.offsets;
    p.table = a.page_table;
    p.pool = a.pool;
    p.page_bytes = s.page_bytes;
    p.tile_bytes = g.tile_bytes;
    p.pool_pages = (int32_t)std::min<int64_t>(a.pool_pages, 0x7fffffff);
    p.tpp = (int32_t)g.tpp;
    p.ppe = (int32_t)g.ppe;
    p.e_begin = a.e_begin;
    p.e_end = a.e_end;
    p.table_row_mod = a.table_row_mod;
    p.status = a.status;
    p.xcd_remap = get_opt(OPT_XCD_REMAP);
    p.half_tiles = get_opt(OPT_HALF_TILES);
    p.tall_rows = (s.dtype == MOE_DTYPE_BF16 && get_opt(OPT_TALL_TILES)) ? 32 : 0;
    p.stagger_ticks = get_opt(OPT_STAGGER_NS) / 10;
    p.stagger_mode = get_opt(OPT_STAGGER_MODE);
}

// parameters of the gate/up launch (K = H, output h[R][F]) and of the down launch
// (K = F, output out[R][H])
inline void fill_gate_up(GemmParams& p, const moe_shape& s, const Geom& g, const FfnArgs& a) {
    p.A = (const char*)a.x_perm;
    p.lda_bytes = (int64_t)s.H * g.esize;
    p.group_base = 0;
    p.KT = (int32_t)g.kt_gu;
    p.NT = (int32_t)g.ft;
    p.n_page_tiles = (int32_t)(2 * g.ft);
    p.out = a.h;
    p.ldo = s.F;
    p.n_cols = s.F;
    p.row_w = nullptr;
    p.a_gather = a.gather_src;
    p.a_div = s.k;
    p.a_rows = s.T;
}

inline void fill_down(GemmParams& p, const moe_shape& s, const Geom& g, const FfnArgs& a) {
    p.A = (const char*)a.h;
    p.lda_bytes = (int64_t)s.F * g.esize;
    p.group_base = (int32_t)g.pages_gu;
    p.KT = (int32_t)g.kt_d;
    p.NT = (int32_t)((g.dt + 1) / 2);
    p.n_page_tiles = (int32_t)g.dt;
    p.out = a.out;
    p.ldo = s.H;
    p.n_cols = s.H;
    p.row_w = a.row_w;
    p.a_gather = nullptr;
}

}  // namespace moe
