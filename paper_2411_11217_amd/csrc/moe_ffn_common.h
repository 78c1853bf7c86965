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
    int32_t chunked;          // tile numbering: groups dealt to the XCDs in chunks of about this many tiles (0: single groups), see locate_tile
    int32_t tall_first;       // bf16 kernel: tile numbering with the tall tiles of a chunk of groups first, see locate_tile
    int32_t stagger_ticks;    // bf16 kernel: start delay unit of a compute unit's first block, in ticks of the 100 MHz counter
    int32_t stagger_mode;
};

struct TileCoord {
    int e, mt, nt, row0, rows_here;
    bool valid;
};

// Tile order.  The row tiles of one column tile of one expert form a GROUP (they share
// the weight tiles); the groups of an expert are taken in CHUNKS of G consecutive column
// tiles, G = max(1, 32 / row tiles of the expert): about as many tiles as an XCD has compute
// units.  With xcd_remap the chunks, numbered expert by expert, are dealt round robin to the
// 8 XCDs (block b runs on XCD b % 8, each with its own L2): the blocks an XCD runs at the
// same time are then the row tiles of G column tiles of ONE expert, so an activation row tile
// is fetched into that L2 once for G blocks and a weight tile once for all its row tiles
// (dealing single groups round robin left only NT / 8 groups of an expert on an XCD: two in
// the down projection of the Mixtral-8x7B shape, where every activation row tile then crossed
// the fabric once per pair of blocks).  Without xcd_remap all chunks belong to one sequence.
// The tile counts come from offsets[], so the grid is only an upper bound and surplus blocks
// leave at once.
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

// Tall tiles that take a remainder of r rows along with q full tiles (0 < r <= tall_rows * q).  A tall tile with at
// most 16 extra rows costs half as many extra MFMAs as one with 17 .. 32 (bf16 kernel), so the remainder goes to
// ceil(r / 16) tiles when there are that many, else to as few tiles as possible (ceil(r / tall_rows)).
__device__ __forceinline__ int tall_tiles_of(int r, int q, int tall_rows) {
    const int m16 = (r + 15) / 16;
    return m16 <= q ? m16 : (r + tall_rows - 1) / tall_rows;
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
    const int x = p.xcd_remap ? (int)(blockIdx.x & 7) : 0;           // my chunks: those whose number is x modulo stride
    const int idx = p.xcd_remap ? (int)(blockIdx.x >> 3) : (int)blockIdx.x;    // my position among their tiles
    // row tiles of my lane's expert.  q full tiles and a remainder r: when r <= tall_rows * q the remainder is
    // spread over the last tall_tiles_of(r, q) of the q tiles (each at most BM + tall_rows rows high), otherwise it is
    // a tile of its own
    const int q_l = cnt / BM, r_l = cnt - q_l * BM;
    const bool rides_l = q_l >= 1 && r_l > 0 && r_l <= p.tall_rows * q_l;
    const int mtiles_l = rides_l ? q_l : q_l + (r_l > 0);
    const int tall_l = rides_l ? tall_tiles_of(r_l, q_l, p.tall_rows) : 0;
    // chunks of my lane's expert: nch_l = ceil(NT / G) of them, of Gc_l or Gc_l + 1 groups each (the first big_l ones are
    // the bigger: equal sizes keep the XCDs' shares equal when the groups do not divide); an expert without rows has none
    const int G_l = (p.chunked && cnt > BM / 2) ? min(max(1, p.chunked / max(mtiles_l, 1)), 8) : 1;      // p.chunked: tiles a chunk aims at (32); at most 8 groups
    const int nch_l = mtiles_l > 0 ? (p.NT + G_l - 1) / G_l : 0;
    const int Gc_l = p.NT / max(nch_l, 1), big_l = p.NT - Gc_l * nch_l;
    const int cb_l = lane_prefix_sum(nch_l, lane) - nch_l;          // chunks of the experts before mine
    int c0_l = (x - cb_l) % stride;                                  // my first chunk in this expert
    if (c0_l < 0) c0_l += stride;
    const int mine_l = c0_l < nch_l ? (nch_l - 1 - c0_l) / stride + 1 : 0;
    const int bigmine_l = c0_l < big_l ? (big_l - 1 - c0_l) / stride + 1 : 0;      // my chunks among the bigger ones: my first ones
    const int groups_l = mine_l * Gc_l + bigmine_l;
    const int tiles_l = groups_l * mtiles_l;
    const int incl = lane_prefix_sum(tiles_l, lane);
    if (idx >= __builtin_amdgcn_readlane(incl, 63)) return t;
    const unsigned long long holds = __ballot(idx < incl);           // lanes of this and later experts
    const int src = __builtin_amdgcn_readfirstlane(__ffsll((long long)holds) - 1);
    const int mtiles = __builtin_amdgcn_readfirstlane(__shfl(mtiles_l, src, 64));
    const int tall = __builtin_amdgcn_readfirstlane(__shfl(tall_l, src, 64));
    const int Gc = __builtin_amdgcn_readfirstlane(__shfl(Gc_l, src, 64));
    const int big = __builtin_amdgcn_readfirstlane(__shfl(big_l, src, 64));
    const int bigmine = __builtin_amdgcn_readfirstlane(__shfl(bigmine_l, src, 64));
    const int c0 = __builtin_amdgcn_readfirstlane(__shfl(c0_l, src, 64));
    const int before = __builtin_amdgcn_readfirstlane(__shfl(incl - tiles_l, src, 64));
    const int seg = __builtin_amdgcn_readfirstlane(__shfl(seg0, src, 64));
    const int rows = __builtin_amdgcn_readfirstlane(__shfl(cnt, src, 64));
    const int rem = idx - before;
    // my chunks in their order: bigmine of Gc + 1 groups, then the others of Gc groups
    const int in_big = bigmine * (Gc + 1) * mtiles;
    const int ci = rem < in_big ? rem / ((Gc + 1) * mtiles) : bigmine + (rem - in_big) / (Gc * mtiles);
    const int c = c0 + ci * stride;                                  // chunk number inside the expert
    const int g_c = Gc + (c < big);                                  // its groups
    const int r2 = rem - (ci <= bigmine ? ci * (Gc + 1) : in_big / mtiles + (ci - bigmine) * Gc) * mtiles;      // my tile inside the chunk
    const int G0 = c * Gc + min(c, big);                             // its first group
    // Order inside a chunk.  Blocks are handed to compute units first come, first served, and a tall tile
    // takes longer than the others.  The tall tiles of all groups of the chunk come first, then the other
    // tiles group by group: the compute units that arrive first get the long tiles, those that arrive late
    // (they had a long tile the last time) get ordinary ones, and the blocks that run at the same time keep
    // reading the same stretch of the operands they share.  Numbered with the tall tile last in its group,
    // the late compute units would meet the next tall tile again and fall further behind with every round.
    int jj, mt;
    if (p.tall_first && tall > 0 && r2 < g_c * tall) {
        jj = r2 / tall;
        mt = (mtiles - tall) + (r2 - jj * tall);
    } else if (p.tall_first && tall > 0) {
        const int r3 = r2 - g_c * tall, plain = mtiles - tall;       // plain >= 1: tiles remain behind the tall ones
        jj = r3 / plain;
        mt = r3 - jj * plain;
    } else {
        jj = r2 / mtiles;
        mt = r2 - jj * mtiles;
    }
    t.nt = G0 + jj;
    t.mt = mt;
    t.e = p.e_begin + src;
    const int q = rows / BM, r = rows - q * BM;
    if (r > 0 && q >= 1 && r <= p.tall_rows * q) {
        // the last m tiles are BM + r / m rows high, the first r % m of them one row more
        const int m = tall_tiles_of(r, q, p.tall_rows), plain = q - m;
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

// Grid size that covers every tile for any routing result.  M = R / BM + n_experts bounds the sum of the experts'
// row tiles.  Dealing single groups round robin, an XCD gets at most ceil(NT / 8) groups of an expert: ceil(NT / 8) * M
// tiles.  Dealt in chunks, an expert with m row tiles (G = min(8, max(1, chunk_tiles / m)) groups per chunk, nch =
// ceil(NT / G) chunks of Gc = NT / nch groups, NT - Gc * nch of them one group more) gives an XCD at most
// ceil(nch / 8) chunks, of which at most ceil(big / 8) are the bigger ones; the most that exceeds ceil(NT / 8) * m
// for any m is added once per expert.  (Blocks beyond the tiles leave at once, but each still costs about a
// microsecond of a compute unit: the bound is kept tight.)
inline int gemm_grid(int NT, int R, int BM, int n_experts, int chunk_tiles = 32) {
    const int64_t M = R / BM + n_experts;
    const int64_t plain_groups = (NT + 7) / 8;
    int64_t slack = 0;
    for (int m = 1; m <= chunk_tiles; ++m) {
        const int G = std::min(std::max(1, chunk_tiles / m), 8);
        if (G == 1) continue;                                         // single groups: no more than ceil(NT / 8) * m
        const int nch = (NT + G - 1) / G, Gc = NT / nch, big = NT - Gc * nch;
        const int64_t mine = (nch + 7) / 8, bigmine = std::min<int64_t>((big + 7) / 8, mine);
        slack = std::max(slack, (mine * Gc + bigmine) * m - plain_groups * m);
    }
    return (int)(8 * (plain_groups * M + slack * n_experts));
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
    p.tall_first = get_opt(OPT_TALL_FIRST);
    // chunks only when the experts have more than half a row tile of rows on average: below that the launch streams
    // the weights, single groups spread over the XCDs are the better order, and the grid needs no slack for chunks
    const int64_t rows_each = (int64_t)s.T * s.k / std::max(1, a.e_end - a.e_begin);
    p.chunked = rows_each > 128 ? std::min(std::max(get_opt(OPT_CHUNKED), 0), 32) : 0;
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
