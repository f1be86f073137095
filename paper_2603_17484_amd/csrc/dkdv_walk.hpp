// Index arithmetic of the dK/dV backward kernel's walk over row tiles: which key block a workgroup
// owns, which 32-row tiles of each row set can see it and which of them need a mask, in which order
// the loads visit them (the cursor) and in which order the arithmetic does (the segments).  The two
// orders never name a tile to each other -- the arithmetic only counts steps and trusts that step i
// finds the tile the cursor loaded i-th -- so they are kept here, in one place, in plain integer code
// that compiles for the host as well: the CPU test builds this header with g++ and checks, over
// sweeps of shapes, that every tile is visited exactly once, in the same order by both, with the
// mask class its rows need.  Nothing here touches memory.
#pragma once

#ifdef __HIPCC__
#define L2A_WALK_FN __host__ __device__ inline __attribute__((always_inline))
#else
#define L2A_WALK_FN inline
#endif

namespace l2a {
namespace walk {

constexpr int kKeysPerWg = 128;  // keys owned by one workgroup
constexpr int kRT = 32;          // rows per tile

L2A_WALK_FN int imin(int a, int b) { return a < b ? a : b; }
L2A_WALK_FN int imax(int a, int b) { return a > b ? a : b; }

// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Key blocks are handed out
// in chunks of `chunk` adjacent blocks per XCD, so that the workgroups resident on one XCD stream
// nearly the same rows at the same time; successive rounds of chunks visit the XCDs in snake order,
// which evens out the causal triangle's work between them.  The grid's x size is a multiple of
// 8 chunk, and the map is a bijection on it.
L2A_WALK_FN int key_block(int block_x, int chunk) {
    const int x = block_x & 7, j = block_x >> 3;
    const int round = j / chunk, w = j % chunk;
    const int xx = (round & 1) ? 7 - x : x;
    return (round * 8 + xx) * chunk + w;
}

// Launch shape chosen on the host.  chunk: key blocks handed to one XCD at a time.  nsplit: workgroups
// per key block -- short sequences have too few key blocks to fill the chip (one workgroup per
// compute unit); their row tiles are then shared out until there are two per compute unit; with a
// workgroup per compute unit splitting gains nothing (measured).  grid_x: a multiple of 8 chunk.
struct LaunchShape {
    int nblk, chunk, nsplit, grid_x;
};
inline LaunchShape launch_shape(int T, long long batch_x_kv_heads) {
    LaunchShape s;
    s.nblk = (T + kKeysPerWg - 1) / kKeysPerWg;
    s.chunk = imax(1, imin(32, s.nblk / 32));
    s.nsplit = 1;
    if ((long long)s.nblk * batch_x_kv_heads < 256)
        while (s.nsplit < 8 && (long long)s.nblk * batch_x_kv_heads * s.nsplit < 512) s.nsplit *= 2;
    const int per = 8 * s.chunk;
    s.grid_x = (s.nblk + per - 1) / per * per;
    return s;
}

// Row sets as the walk sees them.
enum RowKind { kLocalRows = 0, kDenseRows = 1, kListRows = 2 };

// The tiles [tb, te) of one set that can see the key block starting at key k0, in three runs:
// [tb, th) may hold rows that lie before some key of the block (causal mask), [th, tt) need no mask,
// [tt, te) hold rows whose window has moved past some key, or the ragged end of the set.
struct Runs {
    int tb, th, tt, te;
};

//   kind        kLocalRows: rows r = pos G + g of every position, band mask 0 <= pos - key <= W
//               kDenseRows: the same rows, causal mask only
//               kListRows : compacted rows; first_k0 / first_kend = number of rows with a position
//                           below k0 / below min(k0 + 128, ceil64(T)) (entries of kblk_first_row)
//   rows        rows of the set (identity sets: T G)
//   nsplit, z   the set's tiles are shared between nsplit workgroups; this is workgroup z
L2A_WALK_FN Runs tile_runs(int kind, int k0, int T, int G, int W, int first_k0, int first_kend, int rows, int nsplit,
                           int z) {
    Runs r{0, 0, 0, 0};
    int rb, re, r_mid;
    const int kend = k0 + kKeysPerWg;  // rows at positions >= kend see every key of the block
    if (kind == kLocalRows) {
        rb = k0 * G;
        re = imin(T, kend + W) * G;
        r_mid = kend * G;
    } else if (kind == kDenseRows) {
        rb = k0 * G;
        re = T * G;
        r_mid = kend * G;
    } else {
        re = rows;
        rb = imin(imax(first_k0, 0), re);
        r_mid = imin(imax(first_kend, rb), re);
    }
    if (kend > T) r_mid = re;  // keys past the end of the sequence: mask everywhere
    if (re <= rb) return r;
    r.tb = rb / kRT;
    r.te = (re + kRT - 1) / kRT;
    r.th = imin(r.te, imax(r.tb, (r_mid + kRT - 1) / kRT));
    int tl = (re % kRT) ? r.te - 1 : r.te;
    if (kind == kLocalRows) {
        const long long r_suf = (long long)(k0 + W + 1) * G;  // first row whose window starts after k0
        if (r_suf < re) tl = imin(tl, (int)(r_suf / kRT));
    }
    r.tt = imax(tl, r.th);
    if (nsplit > 1) {  // this workgroup's share of the tiles
        const int nt = r.te - r.tb;
        const int b2 = r.tb + (int)((long long)nt * z / nsplit), e2 = r.tb + (int)((long long)nt * (z + 1) / nsplit);
        r.tb = b2, r.te = e2;
        r.th = imin(imax(r.th, r.tb), r.te);
        r.tt = imin(imax(r.tt, r.th), r.te);
    }
    return r;
}

// A Local set is walked upwards, but every key block of an XCD's chunk starts at the first tile of
// the chunk's *last* key block and wraps around to its own first tiles at the end: the ranges of
// neighbouring key blocks are shifted copies of each other, and this rotation makes them meet on
// the same tile at the same step.  n = te - tb tiles; returns the offset of the first tile walked.
L2A_WALK_FN int rotation(bool local, int n, int tb, int kblk, int chunk, int T, int G) {
    if (!local || n <= 0) return 0;
    const int nblk = (T + kKeysPerWg - 1) / kKeysPerWg;
    const int last = imin((kblk / chunk) * chunk + chunk - 1, nblk - 1);
    const int r = (int)(((long long)last * kKeysPerWg * G) / kRT) - tb;
    return (r >= 0 && r < n) ? r : 0;  // ranges that do not overlap share nothing
}

// Everything the walk of one workgroup needs: up to two sets (set 0 first), each with its runs,
// direction and rotation.  A Global set is walked downwards from its last tile, so that all key
// blocks of a head read the same tile at the same step (they only stop at different tiles).
struct Plan {
    Runs r0, r1;          // scalar members, selected with s ? x1 : x0: indexing arrays with the set's number
    int n0, n1;           // made the compiler move this (wave-uniform) arithmetic to the vector unit
    int rot0, rot1;
    bool rev0, rev1;      // walked downwards
    int nsets, total, t_set1;  // t_set1: first tile walked of set 1
    long long set_stride;      // what Cursor::set advances by when the walk moves on to set 1
};

L2A_WALK_FN Plan make_plan(int nsets, const Runs& r0, bool local0, const Runs& r1, bool local1, int kblk, int chunk, int T,
                           int G, long long set_stride) {
    Plan p;
    p.nsets = nsets;
    p.set_stride = set_stride;
    p.r0 = r0, p.r1 = r1;
    p.n0 = r0.te - r0.tb, p.n1 = r1.te - r1.tb;
    p.total = p.n0 + p.n1;
    p.rev0 = !local0, p.rev1 = nsets > 1 && !local1;
    p.rot0 = nsets > 0 ? rotation(local0, p.n0, r0.tb, kblk, chunk, T, G) : 0;
    p.rot1 = nsets > 1 ? rotation(local1, p.n1, r1.tb, kblk, chunk, T, G) : 0;
    p.t_set1 = p.rev1 ? r1.te - 1 : r1.tb + p.rot1;
    return p;
}

// Loads walk the tiles with a cursor that is advanced once per step: tile te - 1 - j for a reversed
// set, tb + (j + rot) mod n otherwise; after the last tile of set 0 it moves on to set 1.  Past the
// very last tile it stays there: the steps near the end re-load that tile into buffers nobody reads
// any more, so that every step issues the same number of loads.
struct Cursor {
    int t, left, tb, te, i;  // tile; tiles left in the set; the set's range (for the wrap); flat index
    bool rev;
    long long set;           // 0 in set 0, Plan::set_stride in set 1 (the kernel: byte offset of the set's arrays)
};

L2A_WALK_FN Cursor cursor_begin(const Plan& p) {
    Cursor c;
    c.i = 0;
    if (p.n0 > 0) {
        c.left = p.n0, c.tb = p.r0.tb, c.te = p.r0.te, c.rev = p.rev0, c.set = 0;
        c.t = p.rev0 ? p.r0.te - 1 : p.r0.tb + p.rot0;
    } else {
        c.left = p.n1, c.tb = p.r1.tb, c.te = p.r1.te, c.rev = p.rev1, c.set = p.set_stride;
        c.t = p.t_set1;
    }
    return c;
}

// Branch-free: the kernel runs it between matrix instructions.
L2A_WALK_FN void cursor_advance(Cursor& c, const Plan& p) {
    const bool more = c.i + 1 < p.total;
    const bool sw = more && c.left == 1;  // only set 0 can end before the last tile
    int t1 = c.rev ? c.t - 1 : c.t + 1;
    t1 = (!c.rev && t1 == c.te) ? c.tb : t1;
    c.t = sw ? p.t_set1 : (more ? t1 : c.t);
    c.left = sw ? p.n1 : (more ? c.left - 1 : c.left);
    c.tb = sw ? p.r1.tb : c.tb;
    c.te = sw ? p.r1.te : c.te;
    c.rev = sw ? p.rev1 : c.rev;
    c.set = sw ? p.set_stride : c.set;
    c.i = more ? c.i + 1 : c.i;
}

// The arithmetic's order: per set, the tiles from the rotation point to the end, then (rotated sets)
// the ones before it; each stretch split into its runs, in walking direction.  f(set, masked, count)
// is called once per non-empty segment, in order; inside a segment the mask flag is constant.
template <class F>
L2A_WALK_FN void for_each_segment_of(const Plan& p, int s, int b, int e, F&& f) {  // tiles [b, e) of set s
    const int sth = s ? p.r1.th : p.r0.th, stt = s ? p.r1.tt : p.r0.tt;
    const bool rev = s ? p.rev1 : p.rev0;
#pragma unroll
    for (int part = 0; part < 3; ++part) {
        const int run_id = rev ? 2 - part : part;
        const int lo = run_id == 0 ? b : imax(b, run_id == 1 ? sth : stt);
        const int hi = run_id == 0 ? imin(e, sth) : (run_id == 1 ? imin(e, stt) : e);
        if (lo >= hi) continue;
        f(s, run_id != 1, hi - lo);
    }
}

template <class F>
L2A_WALK_FN void for_each_segment(const Plan& p, F&& f) {
    for (int s = 0; s < p.nsets; ++s) {
        const int sb = s ? p.r1.tb : p.r0.tb, se = s ? p.r1.te : p.r0.te, rot = s ? p.rot1 : p.rot0;
        if (sb >= se) continue;
        for_each_segment_of(p, s, sb + rot, se, f);  // a reversed set has no rotation: the whole range
        if (rot) for_each_segment_of(p, s, sb, sb + rot, f);
    }
}

}  // namespace walk
}  // namespace l2a
