// Host check of csrc/streamk.h: the piece list of every left-over tile (sk_tile_pieces, what the fix-up pass adds)
// against a simulation of the blocks' walk over their ranges of units (what the main kernel writes: the first
// segment of a block's range goes to slot 2*block, any later partial one to slot 2*block + 1, whole tiles are
// stored by the block itself).
#include <stdio.h>
#include <stdlib.h>
#include <initializer_list>
#include <vector>
#include "streamk.h"
using namespace mcn;

static unsigned long long rng_state = 88172645463325252ull;
static unsigned rnd() { rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17; return (unsigned)(rng_state >> 11); }

static int check(int tiles, int NU, int nblocks, int nshare) {
    const long long total = (long long)tiles * NU;
    std::vector<std::vector<int>> want(tiles);
    std::vector<char> whole(tiles, 0);
    for (int r = 0; r < nshare; ++r) {
        const long long ub = sk_begin(total, nshare, r), ue = sk_begin(total, nshare, r + 1);
        const int block = sk_share_block(nblocks, nshare, r);
        if (sk_share_rank(nblocks, nshare, block) != r) { printf("rank/block mismatch\n"); return 1; }
        bool first = true;
        long long u = ub;
        while (u < ue) {
            const int t = (int)(u / NU);
            const long long t_lo = (long long)t * NU, t_hi = t_lo + NU;
            const long long seg_end = ue < t_hi ? ue : t_hi;
            if (u == t_lo && seg_end == t_hi) whole[t] = 1;
            else want[t].push_back(2 * block + (first ? 0 : 1));
            first = false;
            u = seg_end;
        }
    }
    std::vector<int> slots(4096);
    for (int t = 0; t < tiles; ++t) {
        const int n = sk_tile_pieces(total, NU, nblocks, nshare, t, slots.data(), 4096);
        if (whole[t]) {
            if (n != 0 || !want[t].empty()) { printf("tile %d whole but %d pieces (tiles %d NU %d nblocks %d nshare %d)\n", t, n, tiles, NU, nblocks, nshare); return 1; }
            continue;
        }
        if (n != (int)want[t].size()) { printf("tile %d: %d pieces, want %zu (tiles %d NU %d nblocks %d nshare %d)\n", t, n, want[t].size(), tiles, NU, nblocks, nshare); return 1; }
        for (int i = 0; i < n; ++i)
            if (slots[i] != want[t][i]) { printf("tile %d piece %d: slot %d, want %d (tiles %d NU %d nblocks %d nshare %d)\n", t, i, slots[i], want[t][i], tiles, NU, nblocks, nshare); return 1; }
    }
    return 0;
}

int main() {
    long long cases = 0;
    // the exact split agrees with the one-division form
    for (int i = 0; i < 200000; ++i) {
        const int n = 1 + rnd() % 2048;
        const long long total = 1 + (long long)(rnd() % 4000000) * (1 + rnd() % 64);
        const SkSplit s = sk_split(total, n);
        const int vb = rnd() % (n + 1);
        if (sk_begin(s, vb) != sk_begin(total, n, vb)) { printf("sk_begin differs: total %lld n %d vb %d\n", total, n, vb); return 1; }
    }
    // small cases exhaustively, then random ones; nshare = nblocks, or half of it with both multiples of 16
    for (int nblocks : {1, 2, 3, 5, 8, 16, 31, 32, 256, 512})
        for (int tiles = 1; tiles <= 40; ++tiles)
            for (int NU : {1, 2, 3, 8, 16, 33}) {
                if (tiles >= nblocks && nblocks > 1 && tiles % nblocks == 0) continue;    // no left-over tiles: no fix-up pass
                if (check(tiles, NU, nblocks, nblocks)) return 1;
                ++cases;
                if (nblocks % 16 == 0) { if (check(tiles, NU, nblocks, nblocks / 2)) return 1; ++cases; }
            }
    for (int i = 0; i < 3000; ++i) {
        const int nblocks = 16 * (1 + rnd() % 32);
        const int tiles = 1 + rnd() % (nblocks - 1);
        const int NU = 1 + rnd() % 200;
        if (check(tiles, NU, nblocks, (rnd() & 1) ? nblocks : nblocks / 2)) return 1;
        ++cases;
    }
    // dealt unit order: every unit of the tile exactly once, each XCD's blocks inside their common range, and the
    // units of one round adjacent
    for (int i = 0; i < 4000; ++i) {
        const int n = 2 + rnd() % 64;                   // chunks per XCD
        const int nchunks = 8 * n;
        const int NU = nchunks + rnd() % (i < 2000 ? 4 * nchunks : 100000);
        std::vector<int> seen(NU, 0);
        for (int c = 0; c < nchunks; ++c) {
            const long long ub = sk_begin((long long)NU, nchunks, c), ue = sk_begin((long long)NU, nchunks, c + 1);
            const DealSplit d = make_deal(NU, nchunks, n, c);
            const int c0 = (c / n) * n;
            const long long lo = sk_begin((long long)NU, nchunks, c0), hi = sk_begin((long long)NU, nchunks, c0 + n);
            for (int k = 0; k < (int)(ue - ub); ++k) {
                const int u = dealt_unit(d, k);
                if (u < lo || u >= hi) { printf("dealt unit %d outside [%lld, %lld): NU %d nchunks %d chunk %d k %d\n", u, lo, hi, NU, nchunks, c, k); return 1; }
                if (k < d.q && u != lo + (long long)n * k + (c - c0)) { printf("round %d not adjacent: NU %d nchunks %d chunk %d\n", k, NU, nchunks, c); return 1; }
                ++seen[u];
            }
        }
        for (int u = 0; u < NU; ++u)
            if (seen[u] != 1) { printf("unit %d taken %d times: NU %d nchunks %d\n", u, seen[u], NU, nchunks); return 1; }
        ++cases;
    }
    printf("OK %lld cases\n", cases);
    return 0;
}
