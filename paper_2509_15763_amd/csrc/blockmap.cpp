// Host-side block map for gist-masked attention (Sec. 4.2 of the paper: with a fixed
// compression ratio the set of visible key blocks of every query block is known in
// closed form).  The kernels evaluate the same closed forms inline; this builder
// materialises them for tests and for the live-tile report.
//
// Instead of physically moving the gists to one end of the sequence (the paper's
// "gist shift"), the map treats the gists left of a query tile's window as a compact
// virtual list -- gist g lives at position (r+1)g + r -- and everything from the
// window's first tile to the diagonal as ordinary contiguous key tiles.
#include <stdlib.h>
#include <string.h>

#include "unigist.h"

namespace {

inline int64_t imin(int64_t a, int64_t b) { return a < b ? a : b; }
inline int64_t imax(int64_t a, int64_t b) { return a > b ? a : b; }

// The rule of Sec. 4.1 (Eq. 3) as interval arithmetic: a key j <= i is visible to query i iff it is a sink
// or a gist, or lo(i) <= j, where lo(i) is the first position of the local window of i.
struct Rule {
    int64_t L, rp1, W, S;
    bool units;
    int64_t lo(int64_t i) const {
        if (!units) return imax(0, i - W + 1);
        if (i < S) return i;
        return S + imax(0, (i - S) / rp1 - W) * rp1;
    }
    // sinks and gists at positions < x
    int64_t always_below(int64_t x) const { return x <= S ? x : S + (x - S) / rp1; }
};

}  // namespace

extern "C" unigist_status unigist_blockmap_build(int L, int r, int W, int Bm, int Bn, unigist_blockmap** out) {
    return unigist_blockmap_build_ex(L, r, W, 0, UNIGIST_WINDOW_SLIDING, Bm, Bn, out);
}

extern "C" unigist_status unigist_blockmap_build_ex(int L, int r, int W, int sinks, int window_mode, int Bm, int Bn,
                                                    unigist_blockmap** out) {
    if (!out || L < 1 || r < 1 || W < 1 || Bm < 1 || Bn < 1 || sinks < 0) return UNIGIST_EINVAL;
    if (window_mode != UNIGIST_WINDOW_SLIDING && window_mode != UNIGIST_WINDOW_UNITS) return UNIGIST_EINVAL;
    unigist_blockmap* m = (unigist_blockmap*)calloc(1, sizeof(unigist_blockmap));
    if (!m) return UNIGIST_EINVAL;
    const int64_t rp1 = (int64_t)r + 1;
    const Rule rule{L, rp1, imin(W, L), imin(sinks, L), window_mode == UNIGIST_WINDOW_UNITS};
    m->sinks = sinks;
    m->window_mode = window_mode;
    m->L = L;
    m->r = r;
    m->W = W;
    m->Bm = Bm;
    m->Bn = Bn;
    m->n_qtiles = (int)(((int64_t)L + Bm - 1) / Bm);
    m->n_ktiles = (int)(((int64_t)L + Bn - 1) / Bn);
    m->n_gists = (int)(imax(0, (int64_t)L - rule.S) / rp1);
    m->win_first = (int*)calloc(m->n_qtiles, sizeof(int));
    m->win_last = (int*)calloc(m->n_qtiles, sizeof(int));
    m->n_far_gists = (int*)calloc(m->n_qtiles, sizeof(int));
    m->n_full = (int*)calloc(m->n_qtiles, sizeof(int));
    m->qt_first = (int*)calloc(m->n_ktiles, sizeof(int));
    m->qt_last = (int*)calloc(m->n_ktiles, sizeof(int));

    int64_t max_far = 0;
    for (int t = 0; t < m->n_qtiles; ++t) {
        const int64_t i0 = (int64_t)t * Bm;
        const int64_t i1 = imin(L, i0 + Bm) - 1;
        const int64_t lo = rule.lo(i0);  // leftmost position inside any window of the tile (lo is monotone)
        const int64_t ks = (lo / Bn) * Bn;        // window phase starts at a key-tile boundary
        m->win_first[t] = (int)(ks / Bn);
        m->win_last[t] = (int)(i1 / Bn);
        const int64_t far = rule.always_below(ks);  // sinks and gists at positions < ks
        m->n_far_gists[t] = (int)far;
        if (far > max_far) max_far = far;
        int full = 0;
        for (int c = m->win_first[t]; c <= m->win_last[t]; ++c) {
            const int64_t j0 = (int64_t)c * Bn, j1 = j0 + Bn - 1;
            // no mask needed iff every key is causal for the first row and inside the
            // window of the last row
            if (j1 <= i0 && rule.lo(i1) <= j0) ++full;
        }
        m->n_full[t] = full;
        const int64_t nwin = m->win_last[t] - m->win_first[t] + 1;
        const int64_t ngt = (far + Bn - 1) / Bn;
        m->live_tiles += nwin + ngt;
        m->masked_tiles += nwin - full;
        m->causal_tiles += i1 / Bn + 1;
    }
    m->n_gtiles = (int)((max_far + Bn - 1) / Bn);
    m->gist_qt_first = (int*)calloc(m->n_gtiles > 0 ? m->n_gtiles : 1, sizeof(int));

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
    for (int64_t i = 0; i < L; ++i) nv += i - rule.lo(i) + 1 + rule.always_below(rule.lo(i));
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
