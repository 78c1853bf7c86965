// Pieces shared by the expert-FFN GEMM kernels (bf16 and f32): the launch
// parameter block, the block -> (expert, row tile, column tile) map and the
// page-table lookup of a weight tile.
#pragma once

#include "moe_internal.h"
#include "moe_tile_order.h"

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
    int32_t balance;          // 1: no XCD runs more than an eighth of the launch's tiles, see stolen_tile
};

struct TileCoord {
    int e, mt, nt, row0, rows_here;
    bool valid;
};

// Block -> tile.  The order of the tiles is that of moe_tile_order.h (chunks of about 32 tiles of one expert, dealt
// round robin to the 8 XCDs: block b runs on XCD b % 8, each with its own L2; without xcd_remap all chunks belong
// to one sequence).  The tile counts come from offsets[], so the host never needs the routing result; the grid is
// only an upper bound and surplus blocks leave at once.
//
// Every wavefront does the search on its own, one expert per lane (at most 64
// experts): one load of the segment bounds, prefix sums of the chunk and tile counts over
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

__device__ __forceinline__ int uniform_of(int v_l, int src) { return __builtin_amdgcn_readfirstlane(__shfl(v_l, src, 64)); }

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
    int x = p.xcd_remap ? (int)(blockIdx.x & 7) : 0;                 // my chunks: those whose number is x modulo stride
    int idx = p.xcd_remap ? (int)(blockIdx.x >> 3) : (int)blockIdx.x;          // my position among their tiles
    // (both change below when the block takes a tile of another XCD)
    // my lane's expert: its row tiles, its chunks, and what my XCD gets of each of its row blocks
    const RowTiles rt_l = row_tiles_of(cnt, BM, p.tall_rows);
    const ChunkPlan c_l = plan_chunks(rt_l.mtiles, cnt <= BM / 2, p.NT, p.chunked);
    const int chunks_l = c_l.nb * c_l.nch;
    const int cb_l = lane_prefix_sum(chunks_l, lane) - chunks_l;    // chunks of the experts before mine
    auto share_of = [&](int xx) __attribute__((always_inline)) {     // what XCD xx gets of my lane's expert
        int n = 0;
        for (int b = 0; b < c_l.nb; ++b) n += share_of_block(c_l, b, xx - cb_l, stride).tiles;
        return n;
    };
    int tiles_l = share_of(x);
    int incl = lane_prefix_sum(tiles_l, lane);
    const int mine = __builtin_amdgcn_readlane(incl, 63);            // tiles of my XCD
    if (p.balance && stride == 8) {
        // no XCD runs more than its even share of the launch's tiles (see stolen_tile)
        const int total = __builtin_amdgcn_readlane(lane_prefix_sum(rt_l.mtiles * p.NT, lane), 63);
        const int A = (total + 7) >> 3;
        if (idx >= min(mine, A)) {
            if (idx >= A || mine >= A) return t;                     // given away, or beyond every tile
            int T[8];
#pragma unroll
            for (int xx = 0; xx < 8; ++xx) T[xx] = __builtin_amdgcn_readlane(lane_prefix_sum(share_of(xx), lane), 63);
            const StolenTile st = stolen_tile(T, A, x, idx - mine);
            if (st.idx < 0) return t;
            x = st.x;
            idx = st.idx;
            tiles_l = share_of(x);
            incl = lane_prefix_sum(tiles_l, lane);
        }
    } else if (idx >= mine) {
        return t;
    }
    const unsigned long long holds = __ballot(idx < incl);           // lanes of this and later experts
    const int src = __builtin_amdgcn_readfirstlane(__ffsll((long long)holds) - 1);
    const int mtiles = uniform_of(rt_l.mtiles, src), tall = uniform_of(rt_l.tall, src);
    ChunkPlan c;
    c.nb = uniform_of(c_l.nb, src);
    c.rb = uniform_of(c_l.rb, src);
    c.rbig = uniform_of(c_l.rbig, src);
    c.nch = uniform_of(c_l.nch, src);
    c.Gc = uniform_of(c_l.Gc, src);
    c.big = uniform_of(c_l.big, src);
    const int xrel = x - uniform_of(cb_l, src);
    const int seg = uniform_of(seg0, src), rows = uniform_of(cnt, src);
    int rem = idx - uniform_of(incl - tiles_l, src);                 // my tile among my XCD's tiles of this expert
    int b = 0;
    BlockShare s = share_of_block(c, 0, xrel, stride);
    while (b + 1 < c.nb && rem >= s.tiles) {                         // the row block that holds it
        rem -= s.tiles;
        ++b;
        s = share_of_block(c, b, xrel, stride);
    }
    const TileInExpert te = tile_in_block(c, b, s, rem, stride, mtiles, tall, p.tall_first != 0);
    const RowSpan rs = rows_of_tile(seg, rows, te.mt, BM, p.tall_rows);
    t.nt = te.nt;
    t.mt = te.mt;
    t.e = p.e_begin + src;
    t.row0 = rs.row0;
    t.rows_here = rs.rows_here;
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
    p.balance = get_opt(OPT_BALANCE);
    // chunks only when the experts have more than half a row tile of rows on average: below that the launch streams
    // the weights, single groups spread over the XCDs are the better order, and the grid needs no slack for chunks
    const int64_t rows_each = (int64_t)s.T * s.k / std::max(1, a.e_end - a.e_begin);
    p.chunked = rows_each > 128 ? std::min(std::max(get_opt(OPT_CHUNKED), 0), 32) : 0;
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
