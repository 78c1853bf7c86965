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
    int32_t tile_order;
};

struct TileCoord {
    int e, mt, nt, row0, rows_here;
    bool valid;
};

// Tile order.  Numbers run over the row tiles of one column tile first (they share the
// weight tiles), then over the column tiles, then over the experts, and with xcd_remap
// they are dealt to the 8 XCDs (block b runs on XCD b % 8, each with its own L2) in
// contiguous chunks, so that the blocks an XCD runs at the same time are a few row tiles
// times a few column tiles of one expert.  The at most one PARTIAL row tile at the end
// of an expert's segment is cheaper than a full one (MFMA tiles without valid rows are
// skipped).  tile_order 1 (default) numbers it right after the full row tiles of its
// column tile, so that it finds the weight tiles in L2; tile_order 0 numbers all partial
// tiles after all full ones (longest first), which fills the end of the launch better but
// was measured to read every weight tile from memory a second time (+26 % L2 misses,
// +5 % time on the Mixtral-8x7B-shaped workload).  The tile counts come from offsets[],
// so the grid is only an upper bound and surplus blocks leave at once.
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
    // tile_order 0: partial row tiles form a class of their own; 1: one class, the partial
    // row tile of an expert is numbered right after its full row tiles
    const int full_l = p.tile_order ? (cnt + BM - 1) / BM : cnt / BM;   // row tiles of my expert in the first class
    const int part_l = p.tile_order ? 0 : (cnt % BM) != 0;              // 0 or 1 partial row tile
    const int full_incl = lane_prefix_sum(full_l, lane);
    const int part_incl = lane_prefix_sum(part_l, lane);
    const int total_full = __builtin_amdgcn_readlane(full_incl, 63) * p.NT;
    const int total_part = __builtin_amdgcn_readlane(part_incl, 63) * p.NT;
    // position in the launch order -> (class, number inside the class)
    int L = blockIdx.x;
    bool partial;
    if (p.xcd_remap) {
        const int chunk_f = (total_full + 7) >> 3, chunk_p = (total_part + 7) >> 3;
        const int xcd = blockIdx.x & 7;
        int idx = blockIdx.x >> 3;
        partial = idx >= chunk_f;
        if (partial) {
            idx -= chunk_f;
            if (idx >= chunk_p) return t;
            L = xcd * chunk_p + idx;
        } else {
            L = xcd * chunk_f + idx;
        }
    } else {
        partial = L >= total_full;
        if (partial) L -= total_full;
    }
    if (L >= (partial ? total_part : total_full)) return t;
    const int incl = partial ? part_incl : full_incl;
    const int mine = partial ? part_l : full_l;
    const unsigned long long holds = __ballot(L < incl * p.NT);      // lanes of this and later experts
    const int src = __builtin_amdgcn_readfirstlane(__ffsll((long long)holds) - 1);
    const int mtiles = __builtin_amdgcn_readfirstlane(__shfl(mine, src, 64));
    const int before = __builtin_amdgcn_readfirstlane(__shfl(incl - mine, src, 64));
    const int seg = __builtin_amdgcn_readfirstlane(__shfl(seg0, src, 64));
    const int rows = __builtin_amdgcn_readfirstlane(__shfl(cnt, src, 64));
    L -= before * p.NT;
    t.e = p.e_begin + src;
    t.nt = L / mtiles;
    t.mt = partial ? rows / BM : L - t.nt * mtiles;
    t.row0 = seg + t.mt * BM;
    t.rows_here = min(BM, rows - t.mt * BM);
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

// grid size that covers every tile for any routing result
inline int gemm_grid(int NT, int R, int BM, int n_experts) {
    const int m_tiles_max = R / BM + n_experts;   // >= sum over experts of ceil(rows / BM)
    return ((NT * m_tiles_max + 7) / 8 + 2) * 8;   // each of the two tile classes is rounded up to a multiple of 8
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
    p.tile_order = get_opt(OPT_TILE_ORDER);
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
}

}  // namespace moe
