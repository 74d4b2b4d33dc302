// The order in which the grouped GEMMs walk the output tiles of a launch.  Plain integer code for
// host and device: the host side serves sida_tile_order(), with which the order is checked to be
// a bijection without a GPU.
#pragma once

#if defined(__HIPCC__)
#define SIDA_HD __host__ __device__ __forceinline__
#else
#define SIDA_HD inline
#endif

namespace sida {

// Output tile t of a launch -> (token tile, weight-row tile).
//
// What decides the speed is the number of bytes that miss the L2: every XCD has its own 4 MiB L2,
// and whatever misses it (HBM or Infinity Cache alike) arrives at ~6.5 TB/s over all XCDs, a
// third of the L2-hit rate.  Workgroup b runs on XCD b % 8 (round-robin dispatch) and a persistent
// workgroup takes tiles b, b+G, b+2G, ... with G a multiple of 8, so tile t is computed on XCD
// t % 8, and the compute units of an XCD work on consecutive tiles of that XCD's sequence at any
// time.  The sequence is built from groups of gm consecutive token tiles (the list is sorted by
// expert, most tokens first), dealt round-robin to the XCDs:
//  * a group inside one many-token expert is walked as gm x nw blocks (gm token tiles x nw weight-row
//    tiles, at most the 64 workgroups an XCD runs at a time): the concurrent tiles share gm token
//    tiles and nw weight tiles, so the expert's weights enter this L2 once per group instead of
//    once per token tile, and a token tile once per block instead of once per weight-row tile;
//  * any other group (few-token experts, all with different weights) is walked token tile by token
//    tile, so a token tile is fetched once and used by all its weight-row tiles at the same time.
// Groups that do not fill a complete round of 8, and the last (< gm) token tiles, follow in plain
// order.  m_tall: the leading token tiles that belong to experts with more than one tile;
// gm is 4, 8 or 16 (tile_group_height); nw divides n_tiles_n (tile_block_width).  The mapping is a
// bijection on [0, m_tiles * n_tiles_n).
SIDA_HD void map_tile(int t, int m_tiles, int m_tall, int n_tiles_n, int gm, int nw, int *mt, int *nt)
{
    const int per_group = gm * n_tiles_n;
    const int rounds = (m_tiles / gm) / 8;                    // complete rounds of 8 groups
    const int sym = rounds * 8 * per_group;
    if (t >= sym) {
        const int rest = t - sym;
        *mt = rounds * 8 * gm + rest / n_tiles_n;
        *nt = rest % n_tiles_n;
        return;
    }
    const int xcd = t & 7, local = t >> 3;                    // position in the XCD's sequence
    // An XCD's many-token groups are rounds 0 .. n_many-1 (their tiles hit in L2), its few-token
    // groups the other rounds (their weights come from HBM).  With at least two rounds of either
    // kind, blocks of the one alternate with equally long runs of the other, and odd XCDs start
    // with the other kind - so that at any time about half of the compute units stream weights
    // from HBM while the other half works out of L2, instead of the whole chip doing first one and
    // then the other.  On smaller launches the plain order measured faster.
    const int n_many = (m_tall / gm) / 8, n_few = rounds - n_many;
    const int shorter = n_many < n_few ? n_many : n_few;
    int round, r;
    if (shorter < 2) {
        round = local / per_group;
        r = local % per_group;
    } else {
        const int chunk = gm * nw;                            // one block of a many-token group; divides per_group
        const int pairs = shorter * (per_group / chunk);      // chunks of the shorter kind
        const int ci = local / chunk;
        int pos;                                              // position in the XCD's list of one kind
        bool few;
        if (ci < 2 * pairs) {
            few = (ci + xcd) & 1;
            pos = (ci >> 1) * chunk + local % chunk;
        } else {                                              // what is left of the longer kind
            few = n_many <= n_few;
            pos = local - pairs * chunk;
        }
        round = (few ? n_many : 0) + pos / per_group;
        r = pos % per_group;
    }
    const int first = (round * 8 + xcd) * gm;
    if (first + gm <= m_tall) {                               // inside many-token experts: gm x nw blocks
        const int rr = r % (gm * nw);
        *mt = first + rr / nw;
        *nt = (r / (gm * nw)) * nw + rr % nw;
    } else {
        *mt = first + r / n_tiles_n;
        *nt = r % n_tiles_n;
    }
}

// Token tiles per group.  Taller groups re-read a many-token expert's weights less often, but only
// complete rounds of 8 groups get the block order: the tallest of 16, 8, 4 that still covers (nearly)
// as many many-token tiles as groups of 4 do and leaves no more tiles to the plain order at the end.
// long_rows (weight rows longer than the matrix is tall, K > N: the second GEMM of an expert): at
// least 8 when both kinds of tiles still fill two rounds of such groups, i.e. when the XCDs keep
// alternating between them - a pass over 8 token tiles' rows of K values keeps a block's workgroups
// together for long, the expert's weights are fetched half as often (measured at the Switch-large
// shape: 388 -> 373 us; at Switch-base-128, where groups of 8 leave one round of many-token tiles
// and the alternation stops, groups of 4 are faster, 159 against 165 us; for the first GEMM, K < N,
// the coarser alternation costs more than the saved fetches at either shape).
SIDA_HD int tile_group_height(int m_tiles, int m_tall, bool long_rows)
{
    const int covered4 = (m_tall / 32) * 32, left4 = m_tiles - (m_tiles / 32) * 32;
    const int slack = m_tiles / 16 > left4 ? m_tiles / 16 : left4;
    int gm = 4;
    for (int h = 8; h <= 16; h *= 2) {
        const int covered = (m_tall / (8 * h)) * 8 * h, left = m_tiles - (m_tiles / (8 * h)) * 8 * h;
        if (covered > 0 && covered * 10 >= covered4 * 9 && left <= slack) gm = h;
    }
    if (long_rows && gm < 8) {
        const int many8 = (m_tall / 8) / 8, few8 = (m_tiles / 8) / 8 - many8;
        if (many8 >= 2 && few8 >= 2) gm = 8;
    }
    return gm;
}

// Weight-row tiles per block of a many-token group: the largest divisor of n_tiles_n up to 8 that
// keeps a block within the 64 workgroups of an XCD.
SIDA_HD int tile_block_width(int n_tiles_n, int gm)
{
    const int cap = 64 / gm < 8 ? 64 / gm : 8;
    int nw = n_tiles_n < cap ? n_tiles_n : cap;
    while (n_tiles_n % nw) --nw;
    return nw;
}

}  // namespace sida
