// Host-only checks meant to run under the host compiler's address and undefined-behaviour sanitizers
// (tests/test_host.py builds this file together with csrc/moe_host.cpp and oracle/moe_oracle.c and runs it).
// Every buffer is a heap allocation of exactly the documented size, so an access one element outside
// any of them stops the program.  No GPU call is made and none is linked.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <numeric>
#include <random>
#include <vector>

#include "moe.h"
#include "moe_tile_order.h"

extern "C" {
void oracle_route(int T, int H, int E, int k, int dtype, const void* x, const void* Wr, const double* bias, int32_t* ids,
                  double* w, double* logits, double* gap_next, double* gap_inner);
void oracle_permute(int T, int k, int E, const int32_t* ids, int32_t* counts, int32_t* offsets, int32_t* row_src, int32_t* row_of);
void oracle_gather_rows(int R, int H, int k, int dtype, const void* x, const int32_t* row_src, void* x_perm);
void oracle_expert_ffn(int R, int H, int F, int E, int dtype, const void* x_perm, const int32_t* offsets, const void* W1,
                       const void* W3, const void* W2, const double* row_w, int n_sel, const int32_t* sel, double* h_out,
                       double* o_out);
void oracle_combine(int T, int H, int k, const double* o, const int32_t* row_of, const double* w, double* y);
}

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            std::exit(1);                                                  \
        }                                                                  \
    } while (0)

static std::mt19937 g_rng(1234);

// exact-size heap buffer of random bytes that are valid numbers in either storage type
static std::vector<char>* random_elems(size_t n, int dtype) {
    auto* v = new std::vector<char>(n * (dtype == MOE_DTYPE_BF16 ? 2 : 4));
    std::normal_distribution<float> d(0.f, 0.5f);
    for (size_t i = 0; i < n; ++i) {
        float f = d(g_rng);
        uint32_t u;
        std::memcpy(&u, &f, 4);
        if (dtype == MOE_DTYPE_BF16) {
            uint16_t b = (uint16_t)(u >> 16);
            std::memcpy(v->data() + 2 * i, &b, 2);
        } else {
            std::memcpy(v->data() + 4 * i, &u, 4);
        }
    }
    return v;
}

static void packer_round_trip(int dtype, int H, int F, int E, int64_t page_bytes) {
    moe_shape s{};
    s.T = 7; s.H = H; s.F = F; s.E = E; s.k = 1; s.dtype = dtype; s.page_bytes = page_bytes;
    CHECK(moe_validate_shape(&s) == MOE_OK);
    int64_t pg = 0, pd = 0, tile = 0;
    CHECK(moe_pages_required(&s, &pg, &pd) == MOE_OK);
    CHECK(moe_tile_bytes(&s, &tile) == MOE_OK && tile == 128 * 64 * (dtype == MOE_DTYPE_BF16 ? 2 : 4));
    const int64_t ppe = pg + pd, pool_pages = ppe * E + 3;                      // three slots stay unused
    std::vector<int32_t> slots((size_t)pool_pages);
    std::iota(slots.begin(), slots.end(), 0);
    std::shuffle(slots.begin(), slots.end(), g_rng);
    std::vector<int32_t>* table = new std::vector<int32_t>(slots.begin(), slots.begin() + ppe * E);
    CHECK(moe_page_table_validate(&s, table->data(), pool_pages) == MOE_OK);
    const size_t n1 = (size_t)E * F * H;
    auto *W1 = random_elems(n1, dtype), *W3 = random_elems(n1, dtype), *W2 = random_elems(n1, dtype);
    auto* pages = new std::vector<char>((size_t)(pool_pages * page_bytes), (char)0x5a);
    CHECK(moe_pack_weights(&s, W1->data(), W3->data(), W2->data(), table->data(), pool_pages, pages->data()) == MOE_OK);
    for (int64_t p = ppe * E; p < pool_pages; ++p)                              // unused slots untouched
        for (int64_t i = 0; i < page_bytes; ++i) CHECK((*pages)[(size_t)(slots[(size_t)p] * page_bytes + i)] == (char)0x5a);
    auto *U1 = new std::vector<char>(W1->size()), *U3 = new std::vector<char>(W3->size()), *U2 = new std::vector<char>(W2->size());
    CHECK(moe_unpack_weights(&s, pages->data(), table->data(), pool_pages, U1->data(), U3->data(), U2->data()) == MOE_OK);
    CHECK(*U1 == *W1 && *U3 == *W3 && *U2 == *W2);
    // error paths: an entry outside the pool, a slot named twice, a missing pointer
    std::vector<int32_t> bad(*table);
    bad[1] = (int32_t)pool_pages;
    CHECK(moe_page_table_validate(&s, bad.data(), pool_pages) == MOE_ERR_PAGE_NOT_RESIDENT);
    CHECK(moe_pack_weights(&s, W1->data(), W3->data(), W2->data(), bad.data(), pool_pages, pages->data()) == MOE_ERR_PAGE_NOT_RESIDENT);
    bad[1] = bad[0];
    CHECK(moe_pack_weights(&s, W1->data(), W3->data(), W2->data(), bad.data(), pool_pages, pages->data()) == MOE_ERR_INVALID_ARG);
    CHECK(moe_pack_weights(&s, nullptr, W3->data(), W2->data(), table->data(), pool_pages, pages->data()) == MOE_ERR_INVALID_ARG);
    delete W1; delete W3; delete W2; delete U1; delete U3; delete U2; delete pages; delete table;
    std::printf("packer dtype=%d H=%d F=%d E=%d page=%lld: ok\n", dtype, H, F, E, (long long)page_bytes);
}

static void linear_packer(int K, int N, int64_t page_bytes) {
    moe_linear_shape s{};
    s.T = 5; s.K = K; s.N = N; s.dtype = MOE_DTYPE_BF16; s.page_bytes = page_bytes;
    int64_t pages = 0;
    CHECK(moe_linear_pages_required(&s, &pages) == MOE_OK && pages > 0);
    auto* W = random_elems((size_t)K * N, MOE_DTYPE_BF16);
    auto* table = new std::vector<int32_t>((size_t)pages);
    for (int64_t p = 0; p < pages; ++p) (*table)[(size_t)p] = (int32_t)(pages - 1 - p);
    auto* pool = new std::vector<char>((size_t)(pages * page_bytes));
    CHECK(moe_linear_pack(&s, W->data(), table->data(), pages, pool->data()) == MOE_OK);
    (*table)[0] = -1;
    CHECK(moe_linear_pack(&s, W->data(), table->data(), pages, pool->data()) == MOE_ERR_PAGE_NOT_RESIDENT);
    delete W; delete table; delete pool;
    std::printf("linear packer K=%d N=%d: ok\n", K, N);
}

static void oracle_layer(int dtype, int T, int H, int F, int E, int k, bool with_bias) {
    const int R = T * k;
    auto *x = random_elems((size_t)T * H, dtype), *Wr = random_elems((size_t)E * H, dtype);
    const size_t n1 = (size_t)E * F * H;
    auto *W1 = random_elems(n1, dtype), *W3 = random_elems(n1, dtype), *W2 = random_elems(n1, dtype);
    auto* bias = new std::vector<double>((size_t)E, 0.0);
    if (with_bias) (*bias)[0] = 50.0;                                            // every token takes expert 0, others may stay empty
    auto* ids = new std::vector<int32_t>((size_t)R);
    auto *w = new std::vector<double>((size_t)R), *logits = new std::vector<double>((size_t)T * E);
    auto *gn = new std::vector<double>((size_t)T), *gi = new std::vector<double>((size_t)T);
    oracle_route(T, H, E, k, dtype, x->data(), Wr->data(), with_bias ? bias->data() : nullptr, ids->data(), w->data(),
                 logits->data(), gn->data(), gi->data());
    for (int t = 0; t < T; ++t) {
        double sum = 0;
        for (int s = 0; s < k; ++s) {
            CHECK((*ids)[(size_t)t * k + s] >= 0 && (*ids)[(size_t)t * k + s] < E);
            sum += (*w)[(size_t)t * k + s];
        }
        CHECK(std::fabs(sum - 1.0) < 1e-12);
        if (with_bias) CHECK((*ids)[(size_t)t * k] == 0);
    }
    auto *counts = new std::vector<int32_t>((size_t)E), *offsets = new std::vector<int32_t>((size_t)E + 1);
    auto *row_src = new std::vector<int32_t>((size_t)R), *row_of = new std::vector<int32_t>((size_t)R);
    oracle_permute(T, k, E, ids->data(), counts->data(), offsets->data(), row_src->data(), row_of->data());
    CHECK((*offsets)[(size_t)E] == R);
    for (int i = 0; i < R; ++i) CHECK((*row_src)[(size_t)(*row_of)[(size_t)i]] == i);
    auto* xp = new std::vector<char>((size_t)R * H * (dtype == MOE_DTYPE_BF16 ? 2 : 4));
    oracle_gather_rows(R, H, k, dtype, x->data(), row_src->data(), xp->data());
    // all rows, then a selection (last row, first row)
    auto *h = new std::vector<double>((size_t)R * F), *o = new std::vector<double>((size_t)R * H);
    oracle_expert_ffn(R, H, F, E, dtype, xp->data(), offsets->data(), W1->data(), W3->data(), W2->data(), nullptr, R, nullptr,
                      h->data(), o->data());
    if (R > 0) {
        const int32_t sel[2] = {R - 1, 0};
        auto *h2 = new std::vector<double>((size_t)2 * F), *o2 = new std::vector<double>((size_t)2 * H);
        oracle_expert_ffn(R, H, F, E, dtype, xp->data(), offsets->data(), W1->data(), W3->data(), W2->data(), nullptr, 2, sel,
                          h2->data(), o2->data());
        CHECK(std::memcmp(h2->data(), h->data() + (size_t)(R - 1) * F, sizeof(double) * F) == 0);
        CHECK(std::memcmp(o2->data() + H, o->data(), sizeof(double) * H) == 0);
        oracle_expert_ffn(R, H, F, E, dtype, xp->data(), offsets->data(), W1->data(), W3->data(), W2->data(), nullptr, 2, sel,
                          nullptr, o2->data());
        delete h2; delete o2;
    }
    auto* y = new std::vector<double>((size_t)T * H);
    oracle_combine(T, H, k, o->data(), row_of->data(), w->data(), y->data());
    oracle_combine(T, H, k, o->data(), row_of->data(), nullptr, y->data());
    for (double v : *y) CHECK(std::isfinite(v));
    delete x; delete Wr; delete W1; delete W3; delete W2; delete bias; delete ids; delete w; delete logits; delete gn; delete gi;
    delete counts; delete offsets; delete row_src; delete row_of; delete xp; delete h; delete o; delete y;
    std::printf("oracle dtype=%d T=%d H=%d F=%d E=%d k=%d bias=%d: ok\n", dtype, T, H, F, E, k, (int)with_bias);
}

// The tile order of the expert GEMMs, evaluated the way the kernels do (per expert: row tiles, chunk plan, the share of
// every XCD; per block: the expert by cumulative tile counts, the row block, the tile): every tile of every expert is
// taken by exactly one block (also when the XCDs even out their shares), the row tiles partition the segments, and no XCD
// has more tiles than the grid gives it.
static void tile_order(const std::vector<int>& counts, int NT, int BM, int tall_rows, int chunked, int stride, bool tall_first, bool balance = true) {
    using namespace moe;
    const int E = (int)counts.size();
    int R = 0;
    for (int c : counts) R += c;
    const int grid = gemm_grid(NT, R, BM, E, chunked);
    CHECK(grid % 8 == 0);
    std::vector<RowTiles> rt((size_t)E);
    std::vector<ChunkPlan> plan((size_t)E);
    std::vector<int> cb((size_t)E), seg((size_t)E);
    int chunks = 0, rows0 = 0;
    size_t total = 0;
    for (int e = 0; e < E; ++e) {
        rt[(size_t)e] = row_tiles_of(counts[(size_t)e], BM, tall_rows);
        plan[(size_t)e] = plan_chunks(rt[(size_t)e].mtiles, counts[(size_t)e] <= BM / 2, NT, chunked);
        cb[(size_t)e] = chunks;
        seg[(size_t)e] = rows0;
        chunks += plan[(size_t)e].nb * plan[(size_t)e].nch;
        rows0 += counts[(size_t)e];
        total += (size_t)rt[(size_t)e].mtiles * NT;
        // the row tiles partition the segment, none higher than BM + tall_rows, tall ones last
        int next = seg[(size_t)e];
        for (int mt = 0; mt < rt[(size_t)e].mtiles; ++mt) {
            const RowSpan rs = rows_of_tile(seg[(size_t)e], counts[(size_t)e], mt, BM, tall_rows);
            CHECK(rs.row0 == next && rs.rows_here > 0 && rs.rows_here <= BM + tall_rows);
            CHECK((rs.rows_here > BM) == (mt >= rt[(size_t)e].mtiles - rt[(size_t)e].tall));
            next += rs.rows_here;
        }
        CHECK(next == seg[(size_t)e] + counts[(size_t)e]);
    }
    std::vector<std::vector<char>> seen((size_t)E);
    for (int e = 0; e < E; ++e) seen[(size_t)e].assign((size_t)rt[(size_t)e].mtiles * NT, 0);
    size_t taken = 0;
    // what every XCD was dealt, and - with the balancing - the even share A that none exceeds
    auto share = [&](int x, int e) {
        int n = 0;
        for (int b = 0; b < plan[(size_t)e].nb; ++b) n += share_of_block(plan[(size_t)e], b, x - cb[(size_t)e], stride).tiles;
        return n;
    };
    int T[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int x = 0; x < stride; ++x)
        for (int e = 0; e < E; ++e) T[x] += share(x, e);
    const int A = (int)((total + 7) / 8);
    for (int xb = 0; xb < stride; ++xb) {
        CHECK(T[xb] <= (stride == 8 ? grid / 8 : grid));                  // the grid reaches every tile of this XCD
        // the blocks of XCD xb in their order; with the balancing those beyond min(T, A) take tiles of other XCDs or leave
        const int blocks = balance && stride == 8 ? std::max(T[xb], A) : T[xb];
        int ran = 0;
        for (int blk = 0; blk < blocks; ++blk) {
            int x = xb, idx = blk;
            if (balance && stride == 8 && blk >= std::min(T[xb], A)) {
                if (blk >= A || T[xb] >= A) continue;                      // given away, or beyond every tile
                const StolenTile st = stolen_tile(T, A, xb, blk - T[xb]);
                if (st.idx < 0) continue;
                CHECK(st.x != xb && T[st.x] > A && st.idx >= A && st.idx < T[st.x]);
                x = st.x;
                idx = st.idx;
            }
            ++ran;
            std::vector<int> tiles((size_t)E, 0);
            for (int e = 0; e < E; ++e) tiles[(size_t)e] = share(x, e);
            int e = 0, before = 0;
            while (idx >= before + tiles[(size_t)e]) before += tiles[(size_t)e++];
            const ChunkPlan& c = plan[(size_t)e];
            int rem = idx - before, b = 0;
            BlockShare s = share_of_block(c, 0, x - cb[(size_t)e], stride);
            while (b + 1 < c.nb && rem >= s.tiles) {
                rem -= s.tiles;
                ++b;
                s = share_of_block(c, b, x - cb[(size_t)e], stride);
            }
            CHECK(rem < s.tiles);
            const TileInExpert te = tile_in_block(c, b, s, rem, stride, rt[(size_t)e].mtiles, rt[(size_t)e].tall, tall_first);
            CHECK(te.mt >= 0 && te.mt < rt[(size_t)e].mtiles && te.nt >= 0 && te.nt < NT);
            char& flag = seen[(size_t)e][(size_t)te.mt * NT + te.nt];
            CHECK(flag == 0);
            flag = 1;
            ++taken;
        }
        if (balance && stride == 8) CHECK(ran <= A);                      // no XCD runs more than the even share
    }
    CHECK(taken == total);
}

static void tile_orders() {
    std::uniform_int_distribution<int> small(0, 700), large(0, 20000), pick(0, 9);
    int cases = 0;
    for (int NT : {1, 2, 7, 16, 24, 56, 112}) {
        for (int chunked : {0, 32}) {
            for (int stride : {8, 1}) {
                for (int tall_rows : {0, 32}) {
                    for (int rep = 0; rep < 6; ++rep) {
                        const int E = 1 + (int)(g_rng() % 17);
                        std::vector<int> counts((size_t)E);
                        for (int& c : counts) {
                            const int kind = pick(g_rng);
                            c = kind == 0 ? 0 : kind < 6 ? small(g_rng) : kind < 9 ? 256 * (1 + (int)(g_rng() % 40)) + (int)(g_rng() % 64) : large(g_rng);
                        }
                        tile_order(counts, NT, 256, tall_rows, chunked, stride, rep % 2 == 0, rep % 3 != 0);
                        ++cases;
                    }
                }
            }
        }
    }
    // one expert beyond the row-block limit, the headline routing, a skewed one, exact multiples
    tile_order({256 * 300 + 5, 10, 0, 4000}, 56, 256, 32, 32, 8, true);
    tile_order({1027, 1061, 1029, 995, 1046, 1010, 1014, 1010}, 112, 256, 32, 32, 8, true);
    tile_order({6500, 3000, 2500, 1800, 1200, 800, 400, 184}, 128, 256, 32, 32, 8, true);
    tile_order({1024, 1024, 1024, 1024}, 16, 256, 32, 32, 8, true);
    tile_order({4096}, 24, 256, 32, 32, 8, true);
    tile_order({300, 200, 100}, 4, 64, 0, 32, 8, false);                 // the f32 kernel's row tile
    std::printf("tile order: %d random cases and 6 fixed ones ok\n", cases);
}

int main() {
    tile_orders();
    // packer: tiles that fill their pages exactly, pages with padding at the end of a group, one tile per page
    packer_round_trip(MOE_DTYPE_F32, 128, 256, 3, 2 * 32768);
    packer_round_trip(MOE_DTYPE_F32, 256, 128, 2, 5 * 32768);
    packer_round_trip(MOE_DTYPE_BF16, 256, 384, 4, 65536);
    packer_round_trip(MOE_DTYPE_BF16, 128, 128, 1, 16384);
    packer_round_trip(MOE_DTYPE_BF16, 384, 256, 2, 7 * 16384);
    linear_packer(256, 384, 3 * 16384);
    linear_packer(128, 128, 16384);
    // shapes the GPU library refuses are refused here too, without touching memory
    moe_shape bad{};
    bad.T = 1; bad.H = 100; bad.F = 128; bad.E = 2; bad.k = 1; bad.dtype = MOE_DTYPE_F32; bad.page_bytes = 32768;
    CHECK(moe_validate_shape(&bad) == MOE_ERR_INVALID_ARG);
    CHECK(moe_validate_shape(nullptr) == MOE_ERR_INVALID_ARG);
    // oracle: both storage types, k = E, k = 1, one token, no token, an expert left empty by the bias
    oracle_layer(MOE_DTYPE_F32, 9, 24, 40, 5, 2, false);
    oracle_layer(MOE_DTYPE_BF16, 13, 32, 16, 4, 4, false);
    oracle_layer(MOE_DTYPE_BF16, 6, 16, 24, 3, 1, true);
    oracle_layer(MOE_DTYPE_F32, 1, 8, 8, 1, 1, false);
    oracle_layer(MOE_DTYPE_F32, 0, 8, 8, 2, 1, false);
    std::printf("sanitize driver: all ok\n");
    return 0;
}
