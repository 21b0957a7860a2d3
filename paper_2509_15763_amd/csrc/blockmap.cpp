// Host-side view of the tile walks (Sec. 4.2 of the paper: with a fixed compression ratio the set of visible key
// blocks of every query block is known in closed form).  Nothing here has a rule of its own: the block map and
// the plan queries are built from the functions of plan.h, the ones the kernels call for every decision about
// which tiles to visit, skip or mask, so that what the tests check on the CPU is the walk the GPU executes.
//
// Instead of physically moving the gists to one end of the sequence (the paper's "gist shift"), the walks treat
// the sinks and gists left of a query tile's window as a compact virtual list -- entry c < sinks is position c,
// gist g lives at position sinks + (r+1)g + r -- and everything from the window's first tile to the diagonal as
// ordinary contiguous key tiles.
#include <stdlib.h>
#include <string.h>

#include "plan.h"

using namespace unigist;

namespace {

inline int64_t imin(int64_t a, int64_t b) { return a < b ? a : b; }
inline int64_t imax(int64_t a, int64_t b) { return a > b ? a : b; }

constexpr int kMaxL = 1 << 23;  // the limit of the attention entry points

bool shape_ok(int L, int r, int W, int sinks, int window_mode) {
    if (L < 1 || r < 1 || W < 1 || sinks < 0 || L > kMaxL) return false;
    return window_mode == UNIGIST_WINDOW_SLIDING || window_mode == UNIGIST_WINDOW_UNITS;
}

}  // namespace

extern "C" unigist_status unigist_blockmap_build(int L, int r, int W, int Bm, int Bn, unigist_blockmap** out) {
    return unigist_blockmap_build_ex(L, r, W, 0, UNIGIST_WINDOW_SLIDING, Bm, Bn, out);
}

extern "C" unigist_status unigist_blockmap_build_ex(int L, int r, int W, int sinks, int window_mode, int Bm, int Bn,
                                                    unigist_blockmap** out) {
    if (!out || Bm < 1 || Bn < 1 || !shape_ok(L, r, W, sinks, window_mode)) return UNIGIST_EINVAL;
    const AttnShape s = make_shape(1, 1, 1, L, 64, r, W, sinks, window_mode);
    unigist_blockmap* m = (unigist_blockmap*)calloc(1, sizeof(unigist_blockmap));
    if (!m) return UNIGIST_EINVAL;
    m->sinks = sinks;
    m->window_mode = window_mode;
    m->L = L;
    m->r = r;
    m->W = W;
    m->Bm = Bm;
    m->Bn = Bn;
    m->n_qtiles = (int)(((int64_t)L + Bm - 1) / Bm);
    m->n_ktiles = (int)(((int64_t)L + Bn - 1) / Bn);
    m->n_gists = (int)(imax(0, (int64_t)L - s.S) / s.rp1);
    m->win_first = (int*)calloc(m->n_qtiles, sizeof(int));
    m->win_last = (int*)calloc(m->n_qtiles, sizeof(int));
    m->n_far_gists = (int*)calloc(m->n_qtiles, sizeof(int));
    m->n_full = (int*)calloc(m->n_qtiles, sizeof(int));
    m->qt_first = (int*)calloc(m->n_ktiles, sizeof(int));
    m->qt_last = (int*)calloc(m->n_ktiles, sizeof(int));
    if (!m->win_first || !m->win_last || !m->n_far_gists || !m->n_full || !m->qt_first || !m->qt_last) {
        unigist_blockmap_free(m);
        return UNIGIST_EINVAL;
    }

    int64_t max_far = 0;
    for (int t = 0; t < m->n_qtiles; ++t) {
        const int i0 = (int)((int64_t)t * Bm);
        const int i1 = (int)(imin(L, (int64_t)i0 + Bm) - 1);
        const RowWalk w = row_walk(s, i0, i1, Bn);  // the walk of the tile's rows, as the forward and dQ kernels take it
        m->win_first[t] = w.wstart / Bn;
        m->win_last[t] = i1 / Bn;
        m->n_far_gists[t] = w.nfar;
        if (w.nfar > max_far) max_far = w.nfar;
        int full = 0;
        const int lo_last = win_lo(s, i1);
        for (int it = w.ngt; it < w.ngt + w.nwin; ++it)  // the whole tile taken as one group of rows
            if (row_step_kind(w, it, Bn, i0, i1, lo_last) == STEP_FULL) ++full;
        m->n_full[t] = full;
        m->live_tiles += w.nwin + w.ngt;
        m->masked_tiles += w.nwin - full;
        m->causal_tiles += i1 / Bn + 1;
    }
    m->n_gtiles = (int)((max_far + Bn - 1) / Bn);
    m->gist_qt_first = (int*)calloc(m->n_gtiles > 0 ? m->n_gtiles : 1, sizeof(int));
    if (!m->gist_qt_first) {
        unigist_blockmap_free(m);
        return UNIGIST_EINVAL;
    }

    // transposed view
    for (int c = 0; c < m->n_ktiles; ++c) {
        m->qt_first[c] = m->n_qtiles;
        m->qt_last[c] = -1;
    }
    for (int g = 0; g < m->n_gtiles; ++g) m->gist_qt_first[g] = m->n_qtiles;
    for (int t = m->n_qtiles - 1; t >= 0; --t) {
        for (int c = m->win_first[t]; c <= m->win_last[t]; ++c) {
            m->qt_first[c] = t;
            if (m->qt_last[c] < 0) m->qt_last[c] = t;
        }
        const int ngt = (m->n_far_gists[t] + Bn - 1) / Bn;
        for (int g = 0; g < ngt; ++g) m->gist_qt_first[g] = t;
    }

    // visible pairs: keys inside the window plus sinks and gists strictly left of it, per row
    int64_t nv = 0;
    for (int i = 0; i < L; ++i) nv += i - win_lo(s, i) + 1 + count_always(s, win_lo(s, i));
    m->n_vis = nv;
    *out = m;
    return UNIGIST_OK;
}

extern "C" void unigist_blockmap_free(unigist_blockmap* m) {
    if (!m) return;
    free(m->win_first);
    free(m->win_last);
    free(m->n_far_gists);
    free(m->n_full);
    free(m->qt_first);
    free(m->qt_last);
    free(m->gist_qt_first);
    free(m);
}

// ---------------------------------------------------------------- the kernels' walks, step by step
extern "C" unigist_status unigist_plan_row_tile(int L, int r, int W, int sinks, int window_mode, int kernel, int tile,
                                                unigist_row_tile_plan* out, int kind_capacity, signed char* kind) {
    if (!out || !shape_ok(L, r, W, sinks, window_mode)) return UNIGIST_EINVAL;
    if (kernel != UNIGIST_WALK_FWD && kernel != UNIGIST_WALK_DQ) return UNIGIST_EINVAL;
    const int Bm = kernel == UNIGIST_WALK_FWD ? kFwdBm : kDqBm, Bn = kernel == UNIGIST_WALK_FWD ? kFwdBn : kDqBn;
    const int nq = (L + Bm - 1) / Bm;
    if (tile < 0 || tile >= nq) return UNIGIST_EINVAL;
    const AttnShape s = make_shape(1, 1, 1, L, 64, r, W, sinks, window_mode);
    const int i0 = tile * Bm, i1 = (int)imin(L, (int64_t)i0 + Bm) - 1;
    const RowWalk w = row_walk(s, i0, i1, Bn);
    out->Bm = Bm;
    out->Bn = Bn;
    out->rows_per_wave = kWaveRows;
    out->wstart = w.wstart;
    out->nfar = w.nfar;
    out->n_gist_steps = w.ngt;
    out->n_window_steps = w.nwin;
    const int nsteps = w.ngt + w.nwin, nwaves = Bm / kWaveRows;
    if (!kind) return UNIGIST_OK;  // the counts only
    if (kind_capacity < nwaves * nsteps) return UNIGIST_EINVAL;
    for (int wv = 0; wv < nwaves; ++wv) {
        const int wrow0 = i0 + kWaveRows * wv;
        const int lo_wlast = win_lo(s, wrow0 + kWaveRows - 1);  // as the kernels compute it (rows past L included)
        for (int it = 0; it < nsteps; ++it)
            kind[wv * nsteps + it] = (signed char)row_step_kind(w, it, Bn, wrow0, wrow0 + kWaveRows - 1, lo_wlast);
    }
    return UNIGIST_OK;
}

extern "C" unigist_status unigist_bwd_plan_build(int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks,
                                                 int window_mode, unigist_bwd_plan* out) {
    if (!out || B < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || (D < 8 || D > 128 || D % 8 != 0)) return UNIGIST_EINVAL;
    if (!shape_ok(L, r, W, sinks, window_mode)) return UNIGIST_EINVAL;
    const AttnShape s = make_shape(B, Hq, Hkv, L, D, r, W, sinks, window_mode);
    const BwdPlan p = make_bwd_plan(s);
    memset(out, 0, sizeof *out);
    out->key_tile = BNK;
    out->chunk_rows = MQ;
    out->n_chunks = p.NC;
    out->n_key_tiles = (L + BNK - 1) / BNK;
    out->n_gist_tiles = p.n_gt;
    out->seg_chunks = p.segc;
    out->n_segs = p.nseg;
    for (int i = 0; i <= p.nseg; ++i) out->slot0[i] = p.slot0[i];
    out->partial_bytes = (size_t)B * Hkv * p.slot0[p.nseg] * 2 * padded_head_dim(D) * BNK * sizeof(float);
    out->reduced_bytes = (size_t)B * Hkv * p.n_gt * 2 * padded_head_dim(D) * BNK * sizeof(float);
    out->workspace_bytes = p.total;
    return UNIGIST_OK;
}

extern "C" unigist_status unigist_plan_key_tile(int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks,
                                                int window_mode, int gist_phase, int tile, int seg, int* c_lo,
                                                int* c_hi, int capacity, int* nfar, signed char* kind) {
    if (!c_lo || !c_hi || B < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || (D < 8 || D > 128 || D % 8 != 0)) return UNIGIST_EINVAL;
    if (!shape_ok(L, r, W, sinks, window_mode)) return UNIGIST_EINVAL;
    const AttnShape s = make_shape(B, Hq, Hkv, L, D, r, W, sinks, window_mode);
    const BwdPlan p = make_bwd_plan(s);
    ChunkRange cr;
    if (gist_phase) {
        if (seg < 0 || seg >= p.nseg || tile < 0 || tile >= p.slot0[seg + 1] - p.slot0[seg]) return UNIGIST_EINVAL;
        cr = gist_tile_chunks(s, p, tile, seg);
    } else {
        if (tile < 0 || tile >= (L + BNK - 1) / BNK) return UNIGIST_EINVAL;
        cr = window_tile_chunks(s, p, tile);
    }
    *c_lo = cr.c_lo;
    *c_hi = cr.c_hi;
    if (!kind && !nfar) return UNIGIST_OK;
    const int nch = cr.c_hi - cr.c_lo + 1;
    if (nch < 0 || capacity < nch) return UNIGIST_EINVAL;
    for (int c = cr.c_lo; c <= cr.c_hi; ++c) {
        const int nf = gist_phase ? nfar_of_chunk(s, c) : 0;
        if (nfar) nfar[c - cr.c_lo] = nf;
        if (!kind) continue;
        for (int wv = 0; wv < BNK / 32; ++wv) {
            const int key0 = tile * BNK + 32 * wv;
            const int hi_w0 = win_hi(s, key0 < L - 1 ? key0 : L - 1);
            for (int qb = 0; qb < MQ / 32; ++qb) {
                const int qb0 = c * MQ + 32 * qb;
                kind[(wv * nch + (c - cr.c_lo)) * (MQ / 32) + qb] =
                    (signed char)(gist_phase ? gist_block_kind(key0, qb0, nf, L) : window_block_kind(key0, qb0, hi_w0, L));
            }
        }
    }
    return UNIGIST_OK;
}

extern "C" unigist_status unigist_plan_gist_unit(int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks,
                                                 int window_mode, int unit, int* seg, int* tile) {
    if (!seg || !tile || B < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || (D < 8 || D > 128 || D % 8 != 0)) return UNIGIST_EINVAL;
    if (!shape_ok(L, r, W, sinks, window_mode)) return UNIGIST_EINVAL;
    const AttnShape s = make_shape(B, Hq, Hkv, L, D, r, W, sinks, window_mode);
    const BwdPlan p = make_bwd_plan(s);
    if (unit < 0 || unit >= p.slot0[p.nseg]) return UNIGIST_EINVAL;
    gist_unit(p, unit, *seg, *tile);
    return UNIGIST_OK;
}
