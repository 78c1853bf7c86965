// Declarations of the host-only part of the library (shape checks, page geometry, the weight packer): no GPU
// types, so plain C++ translation units can include it.  Nothing here is part of the C ABI (that is include/moe.h).
#pragma once

#include <stdint.h>

#include "moe.h"

namespace moe {

// Weight tile: 128 output features x 64 reduction elements (see the page
// format in moe.h).  A bf16 tile is stored as two half-tiles of 32 reduction
// elements each.
constexpr int kTileN = 128;
constexpr int kTileK = 64;

struct Geom {
    int esize;            // bytes per element of dtype
    int64_t tile_bytes;   // kTileN * kTileK * esize
    int64_t tpp;          // tiles per page
    int64_t kt_gu;        // H / 64  : k-tiles of the gate/up product
    int64_t ft;           // F / 128 : f-tiles (each has a W1 and a W3 tile row)
    int64_t tiles_gu;     // 2 * ft * kt_gu
    int64_t kt_d;         // F / 64  : k-tiles of the down product
    int64_t dt;           // H / 128 : d-tiles
    int64_t tiles_d;      // dt * kt_d
    int64_t pages_gu, pages_d, ppe;   // pages per expert: GU group, D group, both
};

int validate_shape(const moe_shape* s);          // MOE_OK or error
Geom geometry(const moe_shape& s);               // shape must be valid

// MOE_OK, MOE_ERR_PAGE_NOT_RESIDENT (an entry outside [0, pool_pages)) or, with need_distinct,
// MOE_ERR_INVALID_ARG when two entries name the same slot.  table: host int32[E][ppe].
int check_table_host(const moe_shape& s, const Geom& g, const int32_t* table, int64_t pool_pages, bool need_distinct);

// Copies one 128 x 64 weight tile between a dense row-major matrix (leading dimension ld elements)
// and its page image.
void copy_tile(char* page_tile, char* dense, int64_t ld, int esize, bool to_page);

// Dense paged matrices (moe_linear): MOE_OK or an error; pages of one matrix (shape must be valid).
int validate_linear(const moe_linear_shape* s);
int64_t linear_pages(const moe_linear_shape& s);

}  // namespace moe
