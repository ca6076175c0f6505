// The stream-K split of the left-over tiles (kern_igemm.h, kern_wgrad.h): which block computes which units, and
// which pieces a shared tile consists of.  Plain integer arithmetic; the header also compiles as C++ on the host,
// where tests/streamk_check.cpp compares the piece lists with a simulation of the blocks' walk over their ranges.
#pragma once
#include "fastdiv.h"

namespace mcn {

// Blocks on consecutive hardware ids land on different XCDs; give each XCD a contiguous
// share of the work so that neighbouring tiles (shared halo, same weights) meet in one L2.
MCN_HOST_DEVICE inline int sk_virtual_block(int b, int nblocks) {
    return (nblocks % 8 == 0) ? (b % 8) * (nblocks / 8) + b / 8 : b;
}
MCN_HOST_DEVICE inline long long sk_begin(long long total, int nblocks, int vb) {
    return total * vb / nblocks;
}
// The same value for many vb at the price of one 64-bit division (which takes a GPU thread some hundred
// instructions): with total = q * nblocks + r,  total * vb / nblocks = q * vb + r * vb / nblocks, and r * vb stays
// below nblocks^2 (nblocks <= 65535), a 32-bit division.
struct SkSplit {
    long long q;
    unsigned r, n;
};
MCN_HOST_DEVICE inline SkSplit sk_split(long long total, int nblocks) {
    SkSplit s;
    s.q = total / nblocks;
    s.r = (unsigned)(total - s.q * nblocks);
    s.n = (unsigned)nblocks;
    return s;
}
MCN_HOST_DEVICE inline long long sk_begin(const SkSplit &s, int vb) {
    return s.q * vb + (long long)(s.r * (unsigned)vb / s.n);
}
// Rank of virtual block vb among the nshare sharing blocks (in virtual order), or -1; and its inverse.  With
// nshare < nblocks (both multiples of 8) the sharing blocks are hardware ids 0 .. nshare-1, i.e. the first
// nshare/8 virtual blocks of each XCD's run of nblocks/8.
MCN_HOST_DEVICE inline int sk_share_rank(int nblocks, int nshare, int vb) {
    if (nshare == nblocks) return vb;
    const int G = nblocks / 8, S = nshare / 8;
    const int x = vb / G, i = vb - x * G;
    return i < S ? x * S + i : -1;
}
MCN_HOST_DEVICE inline int sk_share_block(int nblocks, int nshare, int r) {
    if (nshare == nblocks) return r;
    const int G = nblocks / 8, S = nshare / 8;
    return (r / S) * G + r % S;
}

// The pieces of left-over tile ts (units [ts*NU, (ts+1)*NU) of `total`), in the order in which the fix-up pass adds
// them: workspace slots 2*block + segment.  The sharing block of rank r holds the units [total*r/nshare,
// total*(r+1)/nshare); the first rank with units of this tile follows from one division (and a step of correction);
// its piece is its first segment if its range starts in this tile, else its second; the pieces of the following
// ranks are first segments.  Returns the number of pieces, 0 when one block computed the whole tile (it stored the
// tile itself), at most max_pieces.
MCN_HOST_DEVICE inline int sk_tile_pieces(long long total, int NU, int nblocks, int nshare, int ts, int *slots, int max_pieces) {
    const long long t_lo = (long long)ts * NU, t_hi = t_lo + NU;
    const SkSplit split = sk_split(total, nshare);
    int first = (int)(t_lo * nshare / total);
    while (first + 1 < nshare && sk_begin(split, first + 1) <= t_lo) ++first;
    while (first > 0 && sk_begin(split, first) > t_lo) --first;
    int n = 0;
    for (int b = first; b < nshare && n < max_pieces; ++b) {
        const long long bb = sk_begin(split, b);
        if (bb >= t_hi) break;
        const long long be = sk_begin(split, b + 1);
        if (be == bb || be <= t_lo) continue;                        // a block without units of this tile wrote nothing
        if (bb <= t_lo && be >= t_hi) return 0;                      // one block computed the whole tile
        slots[n++] = 2 * sk_share_block(nblocks, nshare, b) + (bb >= t_lo ? 0 : 1);
    }
    return n;
}

// Dealt unit order of a tile cut into nchunks chunks, one per block (kern_wgrad.h, WgradParams::deal).  Chunk c
// holds the q or q + 1 units [NU*c/nchunks, NU*(c+1)/nchunks) by count; the chunks c0 .. c0 + n - 1 of the blocks on
// one XCD cover one contiguous range between them, and their blocks take its units in turn: in round k < q block i
// takes unit base + n*k + i, and in the last, partial round the blocks with q + 1 units take the rest in block order.
struct DealSplit {
    int n, q, i, base, n_long;      // chunks on the XCD, units per short chunk, this chunk's place among them,
                                    // first unit of the XCD's range, chunks before this one with q + 1 units
};
MCN_HOST_DEVICE inline DealSplit make_deal(int NU, int nchunks, int n, int chunk) {
    DealSplit d;
    const int q = NU / nchunks, rem = NU - q * nchunks;          // rem * chunk < nchunks^2: 32 bits for nchunks <= 32768
    const int c0 = (chunk / n) * n;
    d.n = n; d.q = q; d.i = chunk - c0;
    d.base = q * c0 + rem * c0 / nchunks;
    d.n_long = rem * chunk / nchunks - rem * c0 / nchunks;
    return d;
}
MCN_HOST_DEVICE inline int dealt_unit(const DealSplit &d, int k) { return d.base + d.n * k + (k < d.q ? d.i : d.n_long); }

}  // namespace mcn
