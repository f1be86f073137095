// Host-side check of the dK/dV kernel's tile walk (paper_2603_17484_amd/csrc/dkdv_walk.hpp, the very
// header the kernel compiles): for one problem shape it replays, for every key block and every
// split, the order in which the loads visit the row tiles (the cursor) and the order in which the
// arithmetic expects them (the segments), and compares both with what the masks demand, computed
// here by brute force over (row, key) pairs from the layer's definition:
//   a row at position pos sees key j iff j <= pos (and pos - j <= W in the Local branch), j < T.
// Built with g++ by tests/test_dkdv_walk.py; no GPU code.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../paper_2603_17484_amd/csrc/dkdv_walk.hpp"

using namespace l2a::walk;

namespace {

struct SetDesc {
    int kind;                      // RowKind
    std::vector<int> pos;          // position of every row of the set, ascending
    std::vector<int> first;        // list sets: kblk_first_row, ceil(T/64)+1 entries
};

// per (tile, key block): does any (row, key) pair count, and do all 32 x 128 of them count?
struct Need {
    bool any, all;
};

Need brute(const SetDesc& s, int tile, int k0, int T, int W) {
    Need n{false, true};
    for (int r = tile * kRT; r < (tile + 1) * kRT; ++r) {
        const bool row_ok = r < (int)s.pos.size();
        for (int j = k0; j < k0 + kKeysPerWg; ++j) {
            bool ok = row_ok && j < T && j <= s.pos[row_ok ? r : 0];
            if (ok && s.kind == kLocalRows) ok = s.pos[r] - j <= W;
            n.any = n.any || ok;
            n.all = n.all && ok;
        }
    }
    return n;
}

int fail(char* msg, int len, const char* fmt, int a = 0, int b = 0, int c = 0, int d = 0, int e = 0) {
    snprintf(msg, len, fmt, a, b, c, d, e);
    return 1;
}

}  // namespace

extern "C" {

// The host's choice of launch shape, for the test to sweep the real combinations too.
void walk_launch_shape(int T, long long bh, int* out4) {
    const LaunchShape s = launch_shape(T, bh);
    out4[0] = s.nblk, out4[1] = s.chunk, out4[2] = s.nsplit, out4[3] = s.grid_x;
}

// kinds[i] in {0 Local, 1 dense, 2 list}; for a list set rows_pos/nrows give the routed rows' positions
// (ascending) -- at most one list set per call.  Returns 0 if everything holds, else 1 with a message.
// stats[0] = tiles visited, stats[1] = tiles masked without need (allowed: only costs time).
int walk_check(int T, int G, int W, int chunk, int nsplit, int nsets, const int* kinds, const int* rows_pos, int nrows,
               long long* stats, char* msg, int msglen) {
    msg[0] = 0;
    if (nsets < 1 || nsets > 2) return fail(msg, msglen, "nsets %d", nsets);
    const int Wc = W < T ? W : T;  // the library clamps the window to the sequence
    const int nkb = (T + 63) / 64;
    SetDesc sets[2];
    for (int s = 0; s < nsets; ++s) {
        sets[s].kind = kinds[s];
        if (kinds[s] == kListRows) {
            sets[s].pos.assign(rows_pos, rows_pos + nrows);
            sets[s].first.assign(nkb + 1, 0);
            for (int k = 0; k <= nkb; ++k) {
                int c = 0;
                for (int r = 0; r < nrows; ++r) c += rows_pos[r] < 64 * k;
                sets[s].first[k] = c;
            }
        } else {
            sets[s].pos.resize((size_t)T * G);
            for (int r = 0; r < T * G; ++r) sets[s].pos[r] = r / G;
        }
    }
    const int nblk = (T + kKeysPerWg - 1) / kKeysPerWg;
    const int per = 8 * chunk, grid_x = (nblk + per - 1) / per * per;

    // the block index -> key block map is a bijection on the grid
    std::vector<int> seen(grid_x, 0);
    for (int bx = 0; bx < grid_x; ++bx) {
        const int kb = key_block(bx, chunk);
        if (kb < 0 || kb >= grid_x) return fail(msg, msglen, "key_block(%d, chunk %d) = %d outside the grid %d", bx, chunk, kb, grid_x);
        if (seen[kb]++) return fail(msg, msglen, "key block %d handed out twice (chunk %d)", kb, chunk);
    }

    long long visited = 0, overmasked = 0;
    for (int kblk = 0; kblk < nblk; ++kblk) {
        const int k0 = kblk * kKeysPerWg;
        // visits[s][tile] over all splits
        std::vector<int> visits[2];
        for (int s = 0; s < nsets; ++s) visits[s].assign((sets[s].pos.size() + kRT - 1) / kRT + 1, 0);
        for (int z = 0; z < nsplit; ++z) {
            Runs r[2] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
            for (int s = 0; s < nsets; ++s) {
                int f_lo = 0, f_hi = 0, rows = T * G;
                if (sets[s].kind == kListRows) {
                    rows = (int)sets[s].pos.size();
                    f_lo = sets[s].first[k0 >> 6];
                    const int e = (k0 + kKeysPerWg) >> 6;
                    f_hi = sets[s].first[e < nkb ? e : nkb];
                }
                r[s] = tile_runs(sets[s].kind, k0, T, G, Wc, f_lo, f_hi, rows, nsplit, z);
                if (!(r[s].tb <= r[s].th && r[s].th <= r[s].tt && r[s].tt <= r[s].te))
                    return fail(msg, msglen, "key block %d set %d: runs not ordered: tb %d th %d tt %d", kblk, s, r[s].tb, r[s].th, r[s].tt);
            }
            const Plan plan = make_plan(nsets, r[0], sets[0].kind == kLocalRows, r[1], nsets > 1 && sets[1].kind == kLocalRows,
                                        kblk, chunk, T, G, 1);
            // the arithmetic's sequence of (set, masked)
            std::vector<int> seg_set, seg_masked;
            for_each_segment(plan, [&](int s, bool masked, int count) {
                for (int i = 0; i < count; ++i) seg_set.push_back(s), seg_masked.push_back(masked);
            });
            if ((int)seg_set.size() != plan.total)
                return fail(msg, msglen, "key block %d split %d: segments cover %d steps, the plan has %d", kblk, z, (int)seg_set.size(), plan.total);
            // the loads' sequence of (set, tile)
            Cursor c = cursor_begin(plan);
            for (int i = 0; i < plan.total; ++i) {
                const int s = (int)c.set;
                if (c.i != i) return fail(msg, msglen, "key block %d: cursor index %d at step %d", kblk, c.i, i);
                if (s != seg_set[i])
                    return fail(msg, msglen, "key block %d step %d: loads are in set %d, arithmetic in set %d", kblk, i, s, seg_set[i]);
                if (c.t < r[s].tb || c.t >= r[s].te)
                    return fail(msg, msglen, "key block %d step %d: tile %d outside [%d, %d)", kblk, i, c.t, r[s].tb, r[s].te);
                ++visits[s][c.t];
                ++visited;
                const Need need = brute(sets[s], c.t, k0, T, Wc);
                if (!need.all && !seg_masked[i])
                    return fail(msg, msglen, "key block %d step %d: tile %d of set %d needs a mask but runs unmasked (split %d)", kblk, i, c.t, s, z);
                if (need.all && seg_masked[i]) ++overmasked;
                cursor_advance(c, plan);
            }
            // past the last tile the cursor stays where it is (the kernel keeps issuing loads)
            if (plan.total > 0) {
                const Cursor last = c;
                for (int i = 0; i < 9; ++i) cursor_advance(c, plan);
                if (c.t != last.t || c.set != last.set || c.i != last.i)
                    return fail(msg, msglen, "key block %d: the cursor moves past the last tile (tile %d -> %d)", kblk, last.t, c.t);
                const int s = (int)c.set;
                if (c.t < r[s].tb || c.t >= r[s].te) return fail(msg, msglen, "key block %d: parked outside its range", kblk);
            }
        }
        // every tile some pair of which counts is visited exactly once over the splits; none twice
        for (int s = 0; s < nsets; ++s)
            for (int t = 0; t < (int)visits[s].size(); ++t) {
                const Need need = brute(sets[s], t, k0, T, Wc);
                if (visits[s][t] > 1) return fail(msg, msglen, "key block %d: tile %d of set %d visited %d times", kblk, t, s, visits[s][t]);
                if (need.any && visits[s][t] != 1)
                    return fail(msg, msglen, "key block %d: tile %d of set %d has pairs that count but is never visited", kblk, t, s);
            }
    }
    if (stats) stats[0] = visited, stats[1] = overmasked;
    return 0;
}

}  // extern "C"
