// The tile walks of the attention kernels (Sec. 4.2: with a fixed compression ratio the visible blocks of every
// query block are known in closed form and need not be stored).  Everything here is integer arithmetic on the
// visibility rule of common.h, usable on the host and on the device: the kernels call these functions for every
// decision about which tiles to visit, which to skip and which need the in-tile mask, and the host exports the
// same functions (unigist_plan_*, unigist_blockmap_build) so that the walk can be checked pair by pair on the CPU.
//
// Two walks cover every visible pair exactly once each:
//   row side (forward, dQ): a tile of query rows walks the compact list of sinks and gists left of its window
//     phase ("gist phase", all of them visible to every row), then the contiguous key steps from the window's first
//     step to the diagonal ("window phase");
//   key side (dK/dV): a query chunk c of MQ rows reaches the compact entries left of far(c) in the gist phase (one
//     workgroup per compact tile of BNK entries and segment of chunks) and every key from far(c) on in the window
//     phase (one workgroup per BNK contiguous keys).
#pragma once
#include <algorithm>

#include "common.h"

namespace unigist {

enum StepKind { STEP_SKIP = 0, STEP_FULL = 1, STEP_MASKED = 2 };  // not visited / every pair visible / in-tile mask

// ------------------------------------------------------------------------------------------ row side
constexpr int kFwdBm = 128, kFwdBn = 32;  // forward: query rows per workgroup, keys per step
constexpr int kDqBm = 128, kDqBn = 64;    // dQ
constexpr int kWaveRows = 32;             // query rows per wave in both

struct RowWalk {
    int wstart;  // first position of the window phase: a step boundary at or left of every window of the tile
    int nfar;    // compact entries (sinks, gists) strictly left of it -- the gist phase, visible to every row
    int ngt;     // steps of the gist phase
    int nwin;    // steps of the window phase (up to the step holding the tile's last row)
};

// the walk of the query rows i0 .. i1 (positions) with steps of Bn keys; s.s0 > 0: K/V hold no position left of s0
__host__ __device__ inline RowWalk row_walk(const AttnShape& s, int i0, int i1, int Bn) {
    RowWalk w;
    const int ws = (win_lo(s, i0) / Bn) * Bn;  // win_lo is non-decreasing: the leftmost window of the tile
    w.wstart = ws > s.s0 ? ws : s.s0;
    w.nfar = count_always(s, w.wstart);
    w.ngt = (w.nfar + Bn - 1) / Bn;
    w.nwin = (i1 - w.wstart) / Bn + 1;
    return w;
}
// first key of step `it`: an index into the compact list in the gist phase, a position in the window phase
__host__ __device__ inline int row_step_first(const RowWalk& w, int it, int Bn) {
    return it < w.ngt ? it * Bn : w.wstart + (it - w.ngt) * Bn;
}
// What the rows row_first .. row_last (a wave's 32 rows in the kernels) do with step `it`; lo_last = win_lo(row_last).
// A window step is skipped when it lies right of every row, and needs no mask when it is causal for the first row
// and inside the window of the last one (win_lo is non-decreasing, so inside every row's window).
__host__ __device__ inline int row_step_kind(const RowWalk& w, int it, int Bn, int row_first, int row_last, int lo_last) {
    if (it < w.ngt) return it * Bn + Bn > w.nfar ? STEP_MASKED : STEP_FULL;  // the tail of the compact list
    const int j0 = w.wstart + (it - w.ngt) * Bn;
    if (j0 > row_last) return STEP_SKIP;
    return (j0 + Bn - 1 <= row_first && j0 >= lo_last) ? STEP_FULL : STEP_MASKED;
}

// ------------------------------------------------------------------------------------------ key side
constexpr int BNK = 128;        // keys (or compact entries) per dK/dV workgroup, 32 per wave
constexpr int MQ = 64;          // query rows per chunk, two blocks of 32
constexpr int kMaxSegs = 32;    // segments per gist tile at most
constexpr int kMaxLateUnits = 512;  // gist-phase units ordered by length at the end of a launch at most

struct BwdPlan {
    int NC;      // query chunks of MQ rows
    int n_gt;    // compact tiles (BNK entries each) seen by some chunk
    int segc;    // chunks per segment
    int nseg;    // segments
    // Slots of the gist-phase partial sums per (batch, kv head): segment sg owns the slots slot0[sg] .. slot0[sg+1]-1,
    // one per compact tile some chunk of the segment reaches (tiles 0 .. slot0[sg+1]-slot0[sg]-1: a tile is reached
    // by every chunk from its first one on).  slot0[nseg] = slots in all.
    int slot0[kMaxSegs + 1];
    // Launch order of the gist-phase workgroups of a dense launch.  First the n_even units that walk their whole
    // segment (the tile is reached from the segment's first chunk on; all of one length), segment-major from the last
    // segment down: even0[i] = such units in the i segments launched first, so the workgroups running together still
    // stream the same Q/dO chunks.  Then the n_late units of the tiles first reached inside their segment, longest
    // first, which fill the end of the launch: late[u] = segment << 10 | tile - (even units of the segment).
    // n_even < 0: plain segment-major order (packed launches, and plans whose late units do not fit the table).
    int n_even = -1, n_late = 0;
    int even0[kMaxSegs + 1];
    unsigned short late[kMaxLateUnits];
    size_t off_lse2, off_part, off_comp, total;  // byte offsets into the workspace (delta sits at 0)
};

// A query chunk c (MQ rows from MQ c) reaches the compact entries at positions left of far(c) in the gist phase and
// everything from far(c) on in the window phase.  far is a multiple of BNK, non-decreasing in c.
__host__ __device__ inline int far_of_chunk(const AttnShape& s, int c) { return (win_lo(s, c * MQ) / BNK) * BNK; }
__host__ __device__ inline int nfar_of_chunk(const AttnShape& s, int c) { return count_always(s, far_of_chunk(s, c)); }

// first chunk in [0, NC] whose gist phase holds more than x entries (NC if none).  The x-th entry of the compact
// list sits at position p, so the condition is far(c) > p; far is monotone in c and the search needs no division
// in the sliding mode.
__host__ __device__ inline int first_chunk_with_more_far(const AttnShape& s, int NC, int x) {
    const int p = pos_of_always(s, x);
    if (!s.umode) {  // win_lo(64 c) = 64 c - W + 1 has to reach the 128-boundary right of p
        const long long c = ((long long)(p / BNK + 1) * BNK + s.W - 1 + MQ - 1) / MQ;
        return c < NC ? (int)c : NC;
    }
    int lo = 0, hi = NC;  // answer in [lo, hi]
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (far_of_chunk(s, mid) > p) hi = mid;
        else lo = mid + 1;
    }
    return lo;
}
// last chunk in [c0, NC) whose window phase still starts at or before position j0 (far <= j0); requires far(c0) <= j0
__host__ __device__ inline int last_chunk_with_far_le(const AttnShape& s, int NC, int c0, int j0) {
    if (!s.umode) {  // win_lo(64 c) = 64 c - W + 1 has to stay left of j0 + 128
        const long long c = ((long long)j0 + BNK + s.W - 2) / MQ;
        return c < NC - 1 ? (int)c : NC - 1;
    }
    int lo = c0, hi = NC - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (far_of_chunk(s, mid) <= j0) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

// The counts of a plan, given the segment length the launch asks for (the workgroups of a packed launch recompute
// them for their document).  No more than kMaxSegs segments per compact tile.
__host__ __device__ inline void plan_counts(const AttnShape& s, BwdPlan& p, int segc) {
    p.NC = (s.L + MQ - 1) / MQ;
    const int nfar_max = nfar_of_chunk(s, p.NC - 1);
    p.n_gt = (nfar_max + BNK - 1) / BNK;
    p.segc = segc;
    while ((p.NC + p.segc - 1) / p.segc > kMaxSegs) p.segc *= 2;
    p.nseg = (p.NC + p.segc - 1) / p.segc;
}
// compact tiles segment sg reaches: those its last chunk reaches (a tile is reached by every chunk from its first on)
__host__ __device__ inline int seg_tiles(const AttnShape& s, const BwdPlan& p, int sg) {
    const int c_last = (sg + 1) * p.segc < p.NC ? (sg + 1) * p.segc - 1 : p.NC - 1;
    return (nfar_of_chunk(s, c_last) + BNK - 1) / BNK;
}
// fills slot0 (host; the workgroups of a packed launch, which derive their document's plan themselves, sum
// seg_tiles instead of indexing a table)
inline void plan_slots(const AttnShape& s, BwdPlan& p) {
    p.slot0[0] = 0;
    for (int sg = 0; sg < p.nseg; ++sg) p.slot0[sg + 1] = p.slot0[sg] + seg_tiles(s, p, sg);
}

// gist-phase unit (workgroup) -> segment and compact tile of a dense launch, in the order described at BwdPlan
__host__ __device__ inline void gist_unit(const BwdPlan& p, int unit, int& seg, int& tile) {
    if (p.n_even < 0) {  // segment-major from the last segment down, the tiles of a segment in order
        const int nslots = p.slot0[p.nseg];
        seg = p.nseg - 1;
        while (seg > 0 && nslots - p.slot0[seg] <= unit) --seg;
        tile = unit - (nslots - p.slot0[seg + 1]);
    } else if (unit < p.n_even) {
        int i = 0;
        while (p.even0[i + 1] <= unit) ++i;
        seg = p.nseg - 1 - i;
        tile = unit - p.even0[i];
    } else {
        const int e = p.late[unit - p.n_even];
        seg = e >> 10;
        const int i = p.nseg - 1 - seg;
        tile = p.even0[i + 1] - p.even0[i] + (e & 1023);
    }
}

// chunks c_lo .. c_hi (inclusive; none if c_lo > c_hi) a dK/dV workgroup streams
struct ChunkRange {
    int c_lo, c_hi;
};
// gist phase: compact tile `tile`, segment `seg`
__host__ __device__ inline ChunkRange gist_tile_chunks(const AttnShape& s, const BwdPlan& p, int tile, int seg) {
    ChunkRange r;
    const int cf = first_chunk_with_more_far(s, p.NC, tile * BNK);
    r.c_lo = cf > seg * p.segc ? cf : seg * p.segc;
    r.c_hi = ((seg + 1) * p.segc < p.NC ? (seg + 1) * p.segc : p.NC) - 1;
    return r;
}
// fills the launch order (host; needs slot0)
inline void plan_order(const AttnShape& s, BwdPlan& p) {
    p.n_even = -1;
    p.n_late = 0;
    int even[kMaxSegs], nl = 0;
    struct Late { int len, code; } late[kMaxLateUnits];
    for (int sg = p.nseg - 1; sg >= 0; --sg) {
        const int nt = p.slot0[sg + 1] - p.slot0[sg];
        const int ne = (nfar_of_chunk(s, sg * p.segc) + BNK - 1) / BNK;  // tiles the segment's first chunk reaches
        even[sg] = ne < nt ? ne : nt;
        for (int t = even[sg]; t < nt; ++t) {
            if (nl == kMaxLateUnits || t - even[sg] > 1023) return;
            const ChunkRange cr = gist_tile_chunks(s, p, t, sg);
            late[nl++] = Late{cr.c_hi - cr.c_lo + 1, sg << 10 | (t - even[sg])};
        }
    }
    std::stable_sort(late, late + nl, [](const Late& a, const Late& b) { return a.len > b.len; });  // longest first
    p.even0[0] = 0;
    for (int i = 0; i < p.nseg; ++i) p.even0[i + 1] = p.even0[i] + even[p.nseg - 1 - i];
    for (int i = p.nseg + 1; i <= kMaxSegs; ++i) p.even0[i] = p.even0[p.nseg];
    for (int i = 0; i < nl; ++i) p.late[i] = (unsigned short)late[i].code;
    for (int i = nl; i < kMaxLateUnits; ++i) p.late[i] = 0;
    p.n_even = p.even0[p.nseg];
    p.n_late = nl;
}

// window phase: the keys BNK tile .. BNK tile + BNK - 1
__host__ __device__ inline ChunkRange window_tile_chunks(const AttnShape& s, const BwdPlan& p, int tile) {
    ChunkRange r;
    r.c_lo = tile * BNK / MQ;
    r.c_hi = last_chunk_with_far_le(s, p.NC, r.c_lo, tile * BNK);
    return r;
}
// What a wave's 32 keys key0 .. key0 + 31 do with the 32 query rows qb0 .. qb0 + 31 of a chunk.
// Gist phase (key0 indexes the compact list, nfar = nfar_of_chunk of the chunk): never skipped; no mask when all 32
// entries are among the chunk's far ones and all 32 rows exist.
// Window phase (key0 a position, hi_w0 = win_hi of the wave's first key): skipped when every row is left of every key;
// no mask when the block is causal for its first row, its last row still has the first key in its window (win_hi
// is non-decreasing, so every key) and all 32 rows exist.
// (Macros: the dK/dV kernels sit exactly at their register budget, and the same expressions wrapped in inline
// functions come out of the register allocator with spills in the loop.  The functions below are for everyone else.)
#define UNIGIST_GIST_BLOCK_MASKED(key0, qb0, nfar, L) ((key0) + 31 >= (nfar) || (qb0) + 31 >= (L))
#define UNIGIST_WINDOW_BLOCK_SKIPPED(key0, qb0) ((qb0) + 31 < (key0))
#define UNIGIST_WINDOW_BLOCK_MASKED(key0, qb0, hi_w0, L) (!((key0) + 31 <= (qb0) && (qb0) + 31 <= (hi_w0) && (qb0) + 31 < (L)))
inline int gist_block_kind(int key0, int qb0, int nfar, int L) {
    return UNIGIST_GIST_BLOCK_MASKED(key0, qb0, nfar, L) ? STEP_MASKED : STEP_FULL;
}
inline int window_block_kind(int key0, int qb0, int hi_w0, int L) {
    if (UNIGIST_WINDOW_BLOCK_SKIPPED(key0, qb0)) return STEP_SKIP;
    return UNIGIST_WINDOW_BLOCK_MASKED(key0, qb0, hi_w0, L) ? STEP_MASKED : STEP_FULL;
}

// plans and workspace layout of a launch (host; attn_bwd_mfma.hip)
BwdPlan make_bwd_plan(const AttnShape& s);

}  // namespace unigist
