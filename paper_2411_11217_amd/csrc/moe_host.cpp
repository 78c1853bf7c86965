// Host-only part of the C ABI: shape checks, page geometry, the weight packer and the page-table checks.
// Plain C++ with no GPU call, so that it can also be built and tested on its own (with the host
// compiler's sanitizers, for instance).
#include <algorithm>
#include <cstring>
#include <thread>
#include <vector>

#include "moe_host.h"

namespace moe {

int validate_shape(const moe_shape* s) {
    if (!s) return MOE_ERR_INVALID_ARG;
    if (s->dtype != MOE_DTYPE_F32 && s->dtype != MOE_DTYPE_BF16) return MOE_ERR_UNSUPPORTED_DTYPE;
    if (s->T < 0 || s->H <= 0 || s->F <= 0 || s->E < 1 || s->E > MOE_MAX_EXPERTS) return MOE_ERR_INVALID_ARG;
    if (s->k < 1 || s->k > s->E) return MOE_ERR_INVALID_ARG;
    if (s->H % kTileN != 0 || s->F % kTileN != 0) return MOE_ERR_INVALID_ARG;
    if ((int64_t)s->T * s->k > (int64_t)0x3fffffff) return MOE_ERR_INVALID_ARG;
    const int64_t tile = (int64_t)kTileN * kTileK * (s->dtype == MOE_DTYPE_BF16 ? 2 : 4);
    if (s->page_bytes <= 0 || s->page_bytes % tile != 0) return MOE_ERR_INVALID_ARG;
    return MOE_OK;
}

Geom geometry(const moe_shape& s) {
    Geom g;
    g.esize = s.dtype == MOE_DTYPE_BF16 ? 2 : 4;
    g.tile_bytes = (int64_t)kTileN * kTileK * g.esize;
    g.tpp = s.page_bytes / g.tile_bytes;
    g.kt_gu = s.H / kTileK;
    g.ft = s.F / kTileN;
    g.tiles_gu = 2 * g.ft * g.kt_gu;
    g.kt_d = s.F / kTileK;
    g.dt = s.H / kTileN;
    g.tiles_d = g.dt * g.kt_d;
    g.pages_gu = (g.tiles_gu + g.tpp - 1) / g.tpp;
    g.pages_d = (g.tiles_d + g.tpp - 1) / g.tpp;
    g.ppe = g.pages_gu + g.pages_d;
    return g;
}

// ---- packer -------------------------------------------------------------------
// Byte offset inside a page tile of the 16-byte chunk c of row n (the page format of moe.h).
// bf16: two half-tiles of 128 rows x 64 bytes, chunk c & 3 of half c >> 2 at position
// (c & 3) ^ ((n >> 2) & 2).  f32: 128 rows x 256 bytes, chunk c at position
// (c & 8) | ((c & 7) ^ ((n >> 1) & 7)).
static inline int64_t tile_chunk_offset(int esize, int n, int c) {
    if (esize == 2) return (int64_t)(c >> 2) * (kTileN * 64) + n * 64 + (((c & 3) ^ ((n >> 2) & 2)) << 4);
    return (int64_t)n * (kTileK * 4) + (((c & 8) | ((c & 7) ^ ((n >> 1) & 7))) << 4);
}

// Copies one 128 x 64 tile between a dense row-major matrix (leading dimension
// ld elements) and its page image.  to_page: dense -> page, else page -> dense.
void copy_tile(char* page_tile, char* dense, int64_t ld, int esize, bool to_page) {
    const int chunks = kTileK * esize / 16;
    for (int n = 0; n < kTileN; ++n) {
        char* drow = dense + (int64_t)n * ld * esize;
        for (int c = 0; c < chunks; ++c) {
            char* pc = page_tile + tile_chunk_offset(esize, n, c);
            if (to_page) std::memcpy(pc, drow + c * 16, 16);
            else std::memcpy(drow + c * 16, pc, 16);
        }
    }
}

int check_table_host(const moe_shape& s, const Geom& g, const int32_t* table, int64_t pool_pages,
                     bool need_distinct) {
    std::vector<char> seen;
    if (need_distinct) seen.assign((size_t)pool_pages, 0);
    for (int64_t i = 0; i < (int64_t)s.E * g.ppe; ++i) {
        const int32_t v = table[i];
        if (v < 0 || v >= pool_pages) return MOE_ERR_PAGE_NOT_RESIDENT;
        if (need_distinct) {
            if (seen[(size_t)v]) return MOE_ERR_INVALID_ARG;
            seen[(size_t)v] = 1;
        }
    }
    return MOE_OK;
}

static int pack_or_unpack(const moe_shape* s, char* W1, char* W3, char* W2, const int32_t* table,
                          int64_t pool_pages, char* pages, bool to_page) {
    int rc = validate_shape(s);
    if (rc != MOE_OK) return rc;
    if (!W1 || !W3 || !W2 || !table || !pages || pool_pages <= 0) return MOE_ERR_INVALID_ARG;
    const Geom g = geometry(*s);
    rc = check_table_host(*s, g, table, pool_pages, true);
    if (rc != MOE_OK) return rc;
    const int64_t H = s->H, F = s->F;
    auto work = [&](int e) {
        const int32_t* row = table + (int64_t)e * g.ppe;
        auto tile_ptr = [&](int64_t group_base, int64_t ti) {
            return pages + (int64_t)row[group_base + ti / g.tpp] * s->page_bytes + (ti % g.tpp) * g.tile_bytes;
        };
        if (to_page) {   // zero the padding of the last page of each group
            const int64_t pad_gu = g.pages_gu * g.tpp - g.tiles_gu, pad_d = g.pages_d * g.tpp - g.tiles_d;
            for (int64_t i = 0; i < pad_gu; ++i) std::memset(tile_ptr(0, g.tiles_gu + i), 0, (size_t)g.tile_bytes);
            for (int64_t i = 0; i < pad_d; ++i) std::memset(tile_ptr(g.pages_gu, g.tiles_d + i), 0, (size_t)g.tile_bytes);
        }
        for (int64_t f = 0; f < g.ft; ++f)
            for (int w = 0; w < 2; ++w)
                for (int64_t kt = 0; kt < g.kt_gu; ++kt) {
                    char* dense = (w == 0 ? W1 : W3) + (((int64_t)e * F + f * kTileN) * H + kt * kTileK) * g.esize;
                    copy_tile(tile_ptr(0, (f * 2 + w) * g.kt_gu + kt), dense, H, g.esize, to_page);
                }
        for (int64_t d = 0; d < g.dt; ++d)
            for (int64_t kt = 0; kt < g.kt_d; ++kt) {
                char* dense = W2 + (((int64_t)e * H + d * kTileN) * F + kt * kTileK) * g.esize;
                copy_tile(tile_ptr(g.pages_gu, d * g.kt_d + kt), dense, F, g.esize, to_page);
            }
    };
    const int nthr = std::max(1, std::min<int>(s->E, (int)std::min(16u, std::max(1u, std::thread::hardware_concurrency()))));
    std::vector<std::thread> pool;
    for (int t = 0; t < nthr; ++t)
        pool.emplace_back([&, t]() { for (int e = t; e < s->E; e += nthr) work(e); });
    for (auto& th : pool) th.join();
    return MOE_OK;
}

int validate_linear(const moe_linear_shape* s) {
    if (!s) return MOE_ERR_INVALID_ARG;
    if (s->dtype != MOE_DTYPE_BF16) return MOE_ERR_UNSUPPORTED_DTYPE;
    if (s->T < 0 || s->K < 128 || s->N < 128 || s->K % 128 != 0 || s->N % kTileN != 0) return MOE_ERR_INVALID_ARG;
    if ((int64_t)s->T > 0x3fffffff) return MOE_ERR_INVALID_ARG;
    const int64_t tile = (int64_t)kTileN * kTileK * 2;
    if (s->page_bytes <= 0 || s->page_bytes % tile != 0) return MOE_ERR_INVALID_ARG;
    return MOE_OK;
}

int64_t linear_pages(const moe_linear_shape& s) {
    const int64_t tiles = (int64_t)(s.N / kTileN) * (s.K / kTileK);
    const int64_t tpp = s.page_bytes / ((int64_t)kTileN * kTileK * 2);
    return (tiles + tpp - 1) / tpp;
}

}  // namespace moe

using namespace moe;

extern "C" {

const char* moe_status_string(int status) {
    switch (status) {
        case MOE_OK: return "ok";
        case MOE_ERR_INVALID_ARG: return "invalid argument";
        case MOE_ERR_UNSUPPORTED_DTYPE: return "unsupported dtype";
        case MOE_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case MOE_ERR_PAGE_NOT_RESIDENT: return "page not resident";
        case MOE_ERR_HIP: return "HIP error";
        default: return "unknown status";
    }
}

int moe_validate_shape(const moe_shape* s) { return validate_shape(s); }

int moe_tile_bytes(const moe_shape* s, int64_t* tile_bytes) {
    int rc = validate_shape(s);
    if (rc != MOE_OK) return rc;
    if (!tile_bytes) return MOE_ERR_INVALID_ARG;
    *tile_bytes = geometry(*s).tile_bytes;
    return MOE_OK;
}

int moe_pages_required(const moe_shape* s, int64_t* pages_gu, int64_t* pages_d) {
    int rc = validate_shape(s);
    if (rc != MOE_OK) return rc;
    if (!pages_gu || !pages_d) return MOE_ERR_INVALID_ARG;
    const Geom g = geometry(*s);
    *pages_gu = g.pages_gu;
    *pages_d = g.pages_d;
    return MOE_OK;
}

int moe_pack_weights(const moe_shape* s, const void* W1, const void* W3, const void* W2,
                     const int32_t* page_table, int64_t pool_pages, void* pages_out) {
    return pack_or_unpack(s, (char*)W1, (char*)W3, (char*)W2, page_table, pool_pages, (char*)pages_out, true);
}

int moe_unpack_weights(const moe_shape* s, const void* pages, const int32_t* page_table,
                       int64_t pool_pages, void* W1, void* W3, void* W2) {
    return pack_or_unpack(s, (char*)W1, (char*)W3, (char*)W2, page_table, pool_pages, (char*)pages, false);
}

int moe_page_table_validate(const moe_shape* s, const int32_t* page_table_host, int64_t pool_pages) {
    int rc = validate_shape(s);
    if (rc != MOE_OK) return rc;
    if (!page_table_host || pool_pages <= 0) return MOE_ERR_INVALID_ARG;
    return check_table_host(*s, geometry(*s), page_table_host, pool_pages, false);
}

int moe_linear_pages_required(const moe_linear_shape* s, int64_t* pages) {
    int rc = validate_linear(s);
    if (rc != MOE_OK) return rc;
    if (!pages) return MOE_ERR_INVALID_ARG;
    *pages = linear_pages(*s);
    return MOE_OK;
}

int moe_linear_pack(const moe_linear_shape* s, const void* W, const int32_t* page_table, int64_t pool_pages,
                    void* pages_out) {
    int rc = validate_linear(s);
    if (rc != MOE_OK) return rc;
    if (!W || !page_table || !pages_out || pool_pages <= 0) return MOE_ERR_INVALID_ARG;
    const int64_t n_pages = linear_pages(*s), tile_bytes = (int64_t)kTileN * kTileK * 2, tpp = s->page_bytes / tile_bytes;
    std::vector<char> seen((size_t)pool_pages, 0);
    for (int64_t p = 0; p < n_pages; ++p) {
        const int32_t v = page_table[p];
        if (v < 0 || v >= pool_pages) return MOE_ERR_PAGE_NOT_RESIDENT;
        if (seen[(size_t)v]) return MOE_ERR_INVALID_ARG;
        seen[(size_t)v] = 1;
    }
    const int64_t kt_n = s->K / kTileK, nt_n = s->N / kTileN, tiles = kt_n * nt_n;
    auto tile_ptr = [&](int64_t ti) {
        return (char*)pages_out + (int64_t)page_table[ti / tpp] * s->page_bytes + (ti % tpp) * tile_bytes;
    };
    for (int64_t ti = tiles; ti < n_pages * tpp; ++ti) std::memset(tile_ptr(ti), 0, (size_t)tile_bytes);   // padding of the last page
    for (int64_t nt = 0; nt < nt_n; ++nt)
        for (int64_t kt = 0; kt < kt_n; ++kt)
            copy_tile(tile_ptr(nt * kt_n + kt), (char*)W + ((nt * kTileN) * (int64_t)s->K + kt * kTileK) * 2, s->K, 2, true);
    return MOE_OK;
}

}  // extern "C"
