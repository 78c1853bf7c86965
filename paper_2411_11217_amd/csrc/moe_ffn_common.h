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
    int32_t variant;
};

struct TileCoord {
    int e, mt, nt, row0, rows_here;
    bool valid;
};

// Tile numbers run over the row tiles of a column tile first, then over the
// column tiles, then over the experts.  With xcd_remap the numbers are dealt to
// the 8 XCDs (block b runs on XCD b % 8) in contiguous chunks.  The row-tile
// count of every expert comes from offsets[], so the grid is only an upper bound
// and surplus blocks leave at once.
template <int BM>
__device__ __forceinline__ TileCoord locate_tile(const GemmParams& p) {
    TileCoord t{};
    t.valid = false;
    int total_m = 0;
    for (int e = p.e_begin; e < p.e_end; ++e) total_m += (p.offsets[e + 1] - p.offsets[e] + BM - 1) / BM;
    const int total = total_m * p.NT;
    int L = blockIdx.x;
    if (p.xcd_remap) {
        const int chunk = (total + 7) >> 3;
        const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
        if (idx >= chunk) return t;
        L = xcd * chunk + idx;
    }
    if (L >= total) return t;
    int e = p.e_begin, mtiles = 1;
    for (; e < p.e_end; ++e) {
        mtiles = (p.offsets[e + 1] - p.offsets[e] + BM - 1) / BM;
        const int tiles_e = mtiles * p.NT;
        if (L < tiles_e) break;
        L -= tiles_e;
    }
    if (e >= p.e_end) return t;   // not reachable when offsets are consistent
    t.e = e;
    t.nt = L / mtiles;
    t.mt = L - t.nt * mtiles;
    t.row0 = p.offsets[e] + t.mt * BM;
    t.rows_here = min(BM, p.offsets[e + 1] - t.row0);
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
    return ((NT * m_tiles_max + 7) / 8 + 1) * 8;
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
    p.variant = get_opt(OPT_FFN_VARIANT);
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
