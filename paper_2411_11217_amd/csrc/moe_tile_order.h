// The order in which the blocks of an expert-GEMM launch take the tiles of one expert: plain integer
// arithmetic shared by the kernels (which evaluate it per lane and per block) and by the host (which
// sizes the grid with it, and can be tested with it without a GPU).
//
// An expert with `mtiles` row tiles and NT column tiles has mtiles x NT tiles.  The row tiles of one
// column tile form a GROUP: they read the same weight tiles.  Blocks that run at the same time on one
// XCD (32 compute units, one L2) should read few distinct operand tiles, so the tiles are dealt to the
// XCDs in CHUNKS of about `chunked` (32) tiles, as square as possible:
//   * up to 8 row tiles: a chunk is all row tiles of G = clamp(32 / mtiles, 1, 8) consecutive groups;
//   * 9 .. 256 row tiles: the row tiles are cut into nb ROW BLOCKS of at most max(8, ceil(mtiles / 16))
//     row tiles (equal sizes, the first `rbig` blocks one tile more), and a chunk is the row tiles of one
//     row block in G consecutive groups, G from the row-block height as above;
//   * more row tiles, or an expert with at most half a row tile of rows: single groups (G = 1).
// The NT groups are cut into nch = ceil(NT / G) chunks of Gc = NT / nch groups, the first `big` ones a
// group more (equal sizes keep the XCDs' shares equal when G does not divide NT).  The chunks of an expert
// are numbered row block by row block, the numbering continues from expert to expert, and chunk number n
// belongs to XCD n % stride (stride = 8; 1 when the launch does not deal to XCDs).
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define MOE_HD __host__ __device__ __forceinline__
#else
#define MOE_HD inline
#endif

namespace moe {

// Tall tiles that take a remainder of r rows along with q full tiles (0 < r <= tall_rows * q).  A tall tile with at
// most 16 extra rows costs half as many extra MFMAs as one with 17 .. 32 (bf16 kernel), so the remainder goes to
// ceil(r / 16) tiles when there are that many, else to as few tiles as possible (ceil(r / tall_rows)).
MOE_HD int tall_tiles_of(int r, int q, int tall_rows) {
    const int m16 = (r + 15) / 16;
    return m16 <= q ? m16 : (r + tall_rows - 1) / tall_rows;
}

// Row tiles of a segment of cnt rows: q full tiles of BM rows and a remainder r; when 0 < r <= tall_rows * q the
// remainder rides along with the last `tall` of the q tiles, otherwise it is a tile of its own.
struct RowTiles {
    int mtiles, tall;
};
MOE_HD RowTiles row_tiles_of(int cnt, int BM, int tall_rows) {
    const int q = cnt / BM, r = cnt - q * BM;
    const bool rides = q >= 1 && r > 0 && r <= tall_rows * q;
    RowTiles t;
    t.mtiles = rides ? q : q + (r > 0);
    t.tall = rides ? tall_tiles_of(r, q, tall_rows) : 0;
    return t;
}

constexpr int kMaxRowBlockedTiles = 256;      // experts with more row tiles than this are not cut into row blocks

struct ChunkPlan {
    int nb, rb, rbig;          // row blocks; row tiles of a block (the first rbig blocks have rb + 1)
    int nch, Gc, big;          // chunks per row block; groups of a chunk (the first big chunks have Gc + 1)
};
MOE_HD ChunkPlan plan_chunks(int mtiles, bool few_rows, int NT, int chunked) {
    ChunkPlan c;
    int cap = (mtiles + 15) / 16;
    if (cap < 8) cap = 8;
    c.nb = (chunked > 0 && mtiles > 8 && mtiles <= kMaxRowBlockedTiles) ? (mtiles + cap - 1) / cap : 1;
    c.rb = mtiles / c.nb;
    c.rbig = mtiles - c.rb * c.nb;
    int G = 1;
    if (chunked > 0 && !few_rows && mtiles > 0) {
        G = chunked / (c.rb + (c.rbig > 0));
        G = G < 1 ? 1 : (G > 8 ? 8 : G);
    }
    c.nch = mtiles > 0 ? (NT + G - 1) / G : 0;
    c.Gc = c.nch > 0 ? NT / c.nch : 0;
    c.big = NT - c.Gc * c.nch;
    return c;
}

// What one XCD gets of row block b.  xrel = the XCD's number minus the number of chunks before this expert (any
// integer); its chunks in the row block are c0, c0 + stride, ...: `mine` of them, the first `bigmine` of the bigger kind.
struct BlockShare {
    int c0, mine, bigmine, tiles;
};
MOE_HD BlockShare share_of_block(const ChunkPlan& c, int b, int xrel, int stride) {
    BlockShare s;
    s.c0 = (xrel - b * c.nch) % stride;
    if (s.c0 < 0) s.c0 += stride;
    s.mine = s.c0 < c.nch ? (c.nch - 1 - s.c0) / stride + 1 : 0;
    s.bigmine = s.c0 < c.big ? (c.big - 1 - s.c0) / stride + 1 : 0;
    s.tiles = (s.mine * c.Gc + s.bigmine) * (c.rb + (b < c.rbig));
    return s;
}

// Tile number `rem` (0 <= rem < s.tiles) of the XCD's share of row block b -> row tile mt and column tile (group) nt
// of the expert.  Order inside a chunk: blocks are handed to compute units first come, first served, and a tall tile
// takes longer than the others.  With tall_first the tall tiles of all groups of the chunk come first, then the other
// tiles group by group: the compute units that arrive first get the long tiles, those that arrive late (they had a
// long tile the last time) get ordinary ones, and the blocks that run at the same time keep reading the same stretch
// of the operands they share.  Numbered with the tall tile last in its group, the late compute units would meet the
// next tall tile again and fall further behind with every round.
struct TileInExpert {
    int mt, nt;
};
MOE_HD TileInExpert tile_in_block(const ChunkPlan& c, int b, const BlockShare& s, int rem, int stride, int mtiles, int tall,
                                  bool tall_first) {
    const int rbs = c.rb + (b < c.rbig);                              // row tiles of this row block
    const int m0 = b * c.rb + (b < c.rbig ? b : c.rbig);              // its first row tile
    // the XCD's chunks in their order: bigmine of Gc + 1 groups, then the others of Gc groups
    const int in_big = s.bigmine * (c.Gc + 1) * rbs;
    const int ci = rem < in_big ? rem / ((c.Gc + 1) * rbs) : s.bigmine + (rem - in_big) / (c.Gc * rbs);
    const int ch = s.c0 + ci * stride;                                // chunk number inside the row block
    const int g_c = c.Gc + (ch < c.big);                              // its groups
    const int r2 = rem - (ci <= s.bigmine ? ci * (c.Gc + 1) : s.bigmine * (c.Gc + 1) + (ci - s.bigmine) * c.Gc) * rbs;
    const int G0 = ch * c.Gc + (ch < c.big ? ch : c.big);             // its first group
    int tall_c = m0 + rbs - (mtiles - tall);                          // tall row tiles of this row block: its last ones
    tall_c = tall_c < 0 ? 0 : (tall_c > rbs ? rbs : tall_c);
    TileInExpert t;
    int jj;
    if (tall_first && tall_c > 0 && r2 < g_c * tall_c) {
        jj = r2 / tall_c;
        t.mt = m0 + (rbs - tall_c) + (r2 - jj * tall_c);
    } else if (tall_first && tall_c > 0) {
        const int r3 = r2 - g_c * tall_c, plain = rbs - tall_c;       // plain >= 1 here: tiles remain behind the tall ones
        jj = r3 / plain;
        t.mt = m0 + r3 - jj * plain;
    } else {
        jj = r2 / rbs;
        t.mt = m0 + r2 - jj * rbs;
    }
    t.nt = G0 + jj;
    return t;
}

// Evening out the XCDs.  Dealt in whole chunks, the XCDs' shares T[0..7] of a launch differ by up to a chunk per expert
// (experts of different heights have chunks of different sizes and numbers), and the launch lasts as long as the
// largest share.  So no XCD runs more than A = ceil(all tiles / 8) tiles: an XCD with more gives its tiles number
// A .. T[x] - 1 away, and on an XCD with fewer the blocks number T[x] .. A - 1 take them, in the order of the XCDs on
// both sides.  -> sequence and tile number that block number T[x] + j of XCD x runs instead (idx < 0: none is left).
// The tiles given away are the last ones of their XCD's order, so all but a few blocks still run next to their
// chunk's other tiles.
struct StolenTile {
    int x, idx;
};
MOE_HD StolenTile stolen_tile(const int* T, int A, int x, int j) {
    int d = j, surplus = 0;                                           // d: my number among all takers
    for (int i = 0; i < 8; ++i) {
        if (i < x && T[i] < A) d += A - T[i];
        if (T[i] > A) surplus += T[i] - A;
    }
    StolenTile t;
    t.x = 0;
    t.idx = -1;
    if (d >= surplus) return t;
    for (int i = 0; i < 8; ++i) {
        const int sur = T[i] > A ? T[i] - A : 0;
        if (d < sur) {
            t.x = i;
            t.idx = A + d;
            return t;
        }
        d -= sur;
    }
    return t;
}

// First row and height of row tile mt of a segment of `rows` rows that starts at row seg.
struct RowSpan {
    int row0, rows_here;
};
MOE_HD RowSpan rows_of_tile(int seg, int rows, int mt, int BM, int tall_rows) {
    RowSpan t;
    const int q = rows / BM, r = rows - q * BM;
    if (r > 0 && q >= 1 && r <= tall_rows * q) {
        // the last m tiles are BM + r / m rows high, the first r % m of them one row more
        const int m = tall_tiles_of(r, q, tall_rows), plain = q - m;
        const int i = mt - plain;
        if (i < 0) {
            t.row0 = seg + mt * BM;
            t.rows_here = BM;
        } else {
            const int base = BM + r / m, more = r - (r / m) * m;
            t.row0 = seg + plain * BM + i * base + (i < more ? i : more);
            t.rows_here = base + (i < more);
        }
    } else {
        t.row0 = seg + mt * BM;
        const int left = rows - mt * BM;
        t.rows_here = left < BM ? left : BM;
    }
    return t;
}

// Grid size that covers every tile for any routing result.  M = R / BM + n_experts bounds the sum of the experts'
// row tiles.  Dealing single groups round robin, an XCD gets at most ceil(NT / 8) groups of an expert, i.e.
// ceil(NT / 8) * m tiles of an expert with m row tiles; dealt in chunks it may get more, and the most that any m
// (and any position of the expert's first chunk) exceeds that by is added once per expert.  Found by evaluating the
// kernels' own share arithmetic for every m that uses chunks.  (Blocks beyond the tiles leave at once, but each still
// costs about a microsecond of a compute unit: the bound is kept tight.)
inline int gemm_grid(int NT, int R, int BM, int n_experts, int chunked) {
    const int64_t M = R / BM + n_experts;
    const int64_t plain_groups = (NT + 7) / 8;
    int64_t slack = 0;
    if (chunked > 0) {
        for (int m = 1; m <= kMaxRowBlockedTiles; ++m) {
            const ChunkPlan c = plan_chunks(m, false, NT, chunked);
            for (int xrel = 0; xrel < 8; ++xrel) {
                int64_t tiles = 0;
                for (int b = 0; b < c.nb; ++b) tiles += share_of_block(c, b, xrel, 8).tiles;
                if (tiles - plain_groups * m > slack) slack = tiles - plain_groups * m;
            }
        }
    }
    return (int)(8 * (plain_groups * M + slack * n_experts));
}

}  // namespace moe
