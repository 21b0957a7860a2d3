// Compressed KV cache maintenance (Sec. 4.3, Fig. 4 of the paper): raw tokens that have left the local
// window are never attended to again and are dropped; gists are kept for ever.
//
// Cache layout per (batch, kv head): `cap` rows of D elements.  For a state (s, t) the first
// na(s) rows hold the always-visible positions < s -- the sinks, then the gists -- compact and in order
// (na(s) = floor(s / (r+1)) without sinks); the following t - s + 1 rows hold the positions s .. t (raw
// tokens and gists alike).  Every query at a position >= t whose window starts at or after s sees exactly
// these rows.
//
// cache_update builds the state (s_new, t_old + n_new) from the state (s_old, t_old) plus n_new freshly
// computed rows (positions t_old+1 ..): a pure gather, one 16-byte chunk per lane, HBM bound
// (bytes = rows_out * D * elem_bytes read + the same written).
#include "common.h"

namespace unigist {
namespace {

__global__ __launch_bounds__(256) void cache_update_kernel(const char* __restrict__ kc_in, const char* __restrict__ vc_in,
                                                          const char* __restrict__ k_new, const char* __restrict__ v_new,
                                                          char* __restrict__ kc_out, char* __restrict__ vc_out,
                                                          int s_old, int t_old, int cap_in, int new_rows, int s_new,
                                                          int cap_out, int rows_out, AttnShape lay, int row_bytes) {
    const int cpr = row_bytes / 16;                 // 16-byte chunks per row
    const int bh = blockIdx.y;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int n = (int)(idx / cpr), ch = (int)(idx % cpr);
    if (n >= rows_out) return;
    // `lay` carries the layout only (sink count and gist period)
    const int ng_old = count_always(lay, s_old), ng_new = count_always(lay, s_new);
    // position held by output row n
    const int pos = n < ng_new ? pos_of_always(lay, n) : s_new + (n - ng_new);
    const char *ks, *vs;
    size_t off;
    if (pos > t_old) {                              // one of the new rows
        off = ((size_t)bh * new_rows + (pos - t_old - 1)) * row_bytes;
        ks = k_new;
        vs = v_new;
    } else {                                        // already cached: compact gist or window region
        const int row = pos < s_old ? n /* compact entry n < ng_old keeps its row */ : ng_old + (pos - s_old);
        off = ((size_t)bh * cap_in + row) * row_bytes;
        ks = kc_in;
        vs = vc_in;
    }
    const size_t o = ((size_t)bh * cap_out + n) * row_bytes + ch * 16;
    *(u32x4*)(kc_out + o) = *(const u32x4*)(ks + off + ch * 16);
    *(u32x4*)(vc_out + o) = *(const u32x4*)(vs + off + ch * 16);
}

// The same gather with one state per sequence, read from device memory (a serving loop whose sequences are at
// different lengths never has to bring them to the host).  A sequence whose state is inconsistent or does not fit
// the buffers is left alone and reported as -1 rows.
__global__ __launch_bounds__(256) void cache_update_ragged_kernel(
    const char* __restrict__ kc_in, const char* __restrict__ vc_in, const int* __restrict__ s_old_v,
    const int* __restrict__ t_old_v, int cap_in, const char* __restrict__ k_new, const char* __restrict__ v_new,
    const int* __restrict__ n_new_v, int new_rows, char* __restrict__ kc_out, char* __restrict__ vc_out,
    const int* __restrict__ s_new_v, int cap_out, int* __restrict__ rows_out_v, int Hkv, AttnShape lay, int row_bytes,
    int max_pos) {
    const int b = blockIdx.z, bh = b * Hkv + blockIdx.y;
    const int s_old = s_old_v[b], t_old = t_old_v[b], n_new = n_new_v[b], s_new = s_new_v[b];
    bool ok = s_old >= 0 && t_old >= s_old - 1 && n_new >= 0 && n_new <= new_rows && s_new >= s_old &&
              t_old <= max_pos - n_new && s_new <= t_old + n_new + 1;
    int rows_out = -1;
    if (ok) {
        const int rows_in = count_always(lay, s_old) + (t_old - s_old + 1);
        rows_out = count_always(lay, s_new) + (t_old + n_new - s_new + 1);
        if (rows_in > cap_in || rows_out > cap_out) {
            ok = false;
            rows_out = -1;
        }
    }
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) rows_out_v[b] = rows_out;
    if (!ok) return;
    const int cpr = row_bytes / 16;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int n = (int)(idx / cpr), ch = (int)(idx % cpr);
    if (n >= rows_out) return;
    const int ng_old = count_always(lay, s_old), ng_new = count_always(lay, s_new);
    const int pos = n < ng_new ? pos_of_always(lay, n) : s_new + (n - ng_new);
    const char *ks, *vs;
    size_t off;
    if (pos > t_old) {
        off = ((size_t)bh * new_rows + (pos - t_old - 1)) * row_bytes;
        ks = k_new;
        vs = v_new;
    } else {
        const int row = pos < s_old ? n : ng_old + (pos - s_old);
        off = ((size_t)bh * cap_in + row) * row_bytes;
        ks = kc_in;
        vs = vc_in;
    }
    const size_t o = ((size_t)bh * cap_out + n) * row_bytes + ch * 16;
    *(u32x4*)(kc_out + o) = *(const u32x4*)(ks + off + ch * 16);
    *(u32x4*)(vc_out + o) = *(const u32x4*)(vs + off + ch * 16);
}

// ---- ring layouts for token-by-token decoding.  Decode attends to every row of a sequence's slab whatever their
// order, so a new token can take the place of what leaves the window instead of the whole cache being gathered
// again.  In ring state t a slab holds exactly the positions visible to the query at t.
//
// Sliding window of W positions: rows [0, W) hold the window, position p in row p % W; rows [W, W + nf) hold the
// always-visible positions (sinks, gists) that have left the window, in order.  The new token takes the row of the
// position that leaves the window at that moment (which first moves to the far rows if it is a sink or a gist).
//
// Unit-aligned window (the unit of the query plus the W previous units; u = r + 1 positions per unit, units start
// after the S sinks): a whole unit leaves when a new one starts, while the new one fills one token at a time, so
// the unit being filled is kept apart.  With kc the unit of position t and c its positions present:
//   kc <= W: nothing has left the window yet, the slab holds the positions 0 .. t in order;
//   kc >  W: [S sinks | W complete units, unit k in slot k % W | the gists of the units 0 .. kc-W-1 | c rows of unit kc].
// When unit kc+1 starts, the complete unit kc moves into the slot of the unit that leaves (whose gist is saved into
// the far rows first): u rows moved every u tokens.
struct RingLay {
    AttnShape lay;  // sink count, gist period, window mode
    int W;
};
__device__ __forceinline__ int ring_rows(const RingLay& g, int t) {
    const AttnShape& l = g.lay;
    if (t < 0) return 0;
    if (!l.umode) return (t + 1 < g.W ? t + 1 : g.W) + count_always(l, t - g.W + 1 > 0 ? t - g.W + 1 : 0);
    if (t < l.S) return t + 1;
    const int kc = (t - l.S) / l.rp1, c = (t - l.S) % l.rp1 + 1;
    return kc <= g.W ? t + 1 : l.S + g.W * l.rp1 + (kc - g.W) + c;
}
// row of the (visible) position pos in ring state t
__device__ __forceinline__ int ring_row_of_pos(const RingLay& g, int t, int pos) {
    const AttnShape& l = g.lay;
    if (!l.umode) return pos > t - g.W ? pos % g.W : g.W + count_always(l, pos);
    if (t < l.S || pos < l.S) return pos;
    const int u = l.rp1, kc = (t - l.S) / u, k = (pos - l.S) / u, off = (pos - l.S) % u;
    if (kc <= g.W) return pos;
    if (k == kc) return l.S + g.W * u + (kc - g.W) + off;
    if (k >= kc - g.W) return l.S + (k % g.W) * u + off;
    return l.S + g.W * u + k;  // the gist of a unit that has left the window
}
// position held by row n (< ring_rows) in ring state t
__device__ __forceinline__ int ring_pos_of_row(const RingLay& g, int t, int n) {
    const AttnShape& l = g.lay;
    if (!l.umode) {
        const int nwin = t + 1 < g.W ? t + 1 : g.W;
        return n < nwin ? t - (t - n) % g.W : pos_of_always(l, n - g.W);
    }
    if (t < l.S || n < l.S) return n;
    const int u = l.rp1, kc = (t - l.S) / u;
    if (kc <= g.W) return n;
    const int m = n - l.S;
    if (m < g.W * u) {
        const int slot = m / u, k = kc - 1 - (kc - 1 - slot) % g.W;  // the unit in kc-W .. kc-1 with k % W == slot
        return l.S + k * u + m % u;
    }
    const int i = m - g.W * u;
    return i < kc - g.W ? l.S + i * u + u - 1 : l.S + kc * u + (i - (kc - g.W));
}

// TO_RING: ordered state (s[b], t[b]) -> ring state t[b].  !TO_RING: ring state t[b] -> ordered (s[b], t[b]).
// s[b] must be the first position of the window of the query at t[b]: both sides then hold the same positions.
template <bool TO_RING>
__global__ __launch_bounds__(256) void cache_ring_convert_kernel(const char* __restrict__ kc_in, const char* __restrict__ vc_in,
                                                                const int* __restrict__ s_v, const int* __restrict__ t_v,
                                                                int cap_in, char* __restrict__ kc_out, char* __restrict__ vc_out,
                                                                int cap_out, int* __restrict__ rows_out_v, int Hkv, RingLay g,
                                                                int row_bytes, int max_pos) {
    const int b = blockIdx.z, bh = b * Hkv + blockIdx.y;
    const int s = s_v[b], t = t_v[b];
    AttnShape wl = g.lay;  // win_lo wants the window in the shape
    wl.W = g.W;
    bool ok = s >= 0 && t >= -1 && t < max_pos && (t < 0 ? s == 0 : s == win_lo(wl, t));
    int rows = -1;
    if (ok) {
        rows = ring_rows(g, t);  // = count_always(s) + t - s + 1: the same positions on either side
        if (rows > cap_in || rows > cap_out) {
            ok = false;
            rows = -1;
        }
    }
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) rows_out_v[b] = rows;
    if (!ok) return;
    const int cpr = row_bytes / 16;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int n = (int)(idx / cpr), ch = (int)(idx % cpr);
    if (n >= rows) return;
    const int ng = count_always(g.lay, s);
    int src;
    if (TO_RING) {
        const int pos = ring_pos_of_row(g, t, n);
        src = pos < s ? count_always(g.lay, pos) : ng + (pos - s);  // compact entry i sits in row i
    } else {
        const int pos = n < ng ? pos_of_always(g.lay, n) : s + (n - ng);
        src = ring_row_of_pos(g, t, pos);
    }
    const size_t i = ((size_t)bh * cap_in + src) * row_bytes + ch * 16;
    const size_t o = ((size_t)bh * cap_out + n) * row_bytes + ch * 16;
    *(u32x4*)(kc_out + o) = *(const u32x4*)(kc_in + i);
    *(u32x4*)(vc_out + o) = *(const u32x4*)(vc_in + i);
}

// One token per active sequence, in place.  grid (Hkv, B), 64 lanes: lanes 0 .. cpr-1 move K, lanes 32 .. 32+cpr-1 V;
// a lane only ever touches its own 16-byte column of the rows, so its reads and writes are ordered by the program.
__global__ __launch_bounds__(64) void cache_ring_append_kernel(char* __restrict__ kc, char* __restrict__ vc,
                                                              const char* __restrict__ k_new, const char* __restrict__ v_new,
                                                              int new_rows, const int* __restrict__ t_old_v,
                                                              const int* __restrict__ n_new_v, int cap,
                                                              int* __restrict__ rows_out_v, int Hkv, RingLay g, int row_bytes,
                                                              int max_pos) {
    const AttnShape& l = g.lay;
    const int b = blockIdx.y, bh = b * Hkv + blockIdx.x;
    const int t_old = t_old_v[b], act = n_new_v[b];
    int rows = -1;
    const bool ok0 = t_old >= -1 && (act == 0 || act == 1) && t_old < max_pos - act;
    const int t = t_old + act;
    if (ok0) {
        rows = ring_rows(g, t);
        if (rows > cap || ring_rows(g, t_old) > cap) rows = -1;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) rows_out_v[b] = rows;
    if (rows < 0 || act == 0) return;
    const int cpr = row_bytes / 16;
    const int lane = threadIdx.x & 31;
    if (lane >= cpr) return;
    char* c = (threadIdx.x < 32 ? kc : vc) + (size_t)bh * cap * row_bytes + lane * 16;
    const u32x4 nw = *(const u32x4*)((threadIdx.x < 32 ? k_new : v_new) + (size_t)bh * new_rows * row_bytes + lane * 16);
    auto row = [&](int n) { return (u32x4*)(c + (size_t)n * row_bytes); };
    if (!l.umode) {
        const int slot = t % g.W;
        const int p_out = t - g.W;  // leaves the window now; its row is the one the new token takes
        if (p_out >= 0 && is_always(l, p_out)) *row(g.W + count_always(l, p_out)) = *row(slot);
        *row(slot) = nw;
        return;
    }
    const int u = l.rp1;
    const int kc_ = t < l.S ? 0 : (t - l.S) / u, cc = t < l.S ? 0 : (t - l.S) % u + 1;
    if (t < l.S || kc_ <= g.W) {  // nothing has left the window yet: positions in order
        *row(t) = nw;
        return;
    }
    const int base = l.S + g.W * u + (kc_ - g.W);  // first row of the unit being filled
    if (cc > 1) {
        *row(base + cc - 1) = nw;
        return;
    }
    // A new unit starts: the unit kc-1, complete in the rows base-1 .. base+u-2, moves into the slot of the unit
    // kc-1-W, whose gist goes to the far row base-1; then the new token becomes row base.
    const int slot0 = l.S + ((kc_ - 1) % g.W) * u;
    const u32x4 gist = *row(slot0 + u - 1);
    for (int i = 0; i < u; ++i) *row(slot0 + i) = *row(base - 1 + i);
    *row(base - 1) = gist;
    *row(base) = nw;
}

}  // namespace

namespace {
RingLay make_ring_lay(int rp1, int sinks, int W, int umode) {
    RingLay g{};
    g.lay.rp1 = rp1;
    g.lay.S = sinks;
    g.lay.umode = umode;
    g.lay.L = 0x7fffffff;  // win_hi clamps to L - 1; unused here
    g.W = W;
    return g;
}
}  // namespace

hipError_t launch_cache_ring_convert(bool to_ring, const void* kc_in, const void* vc_in, const int* s, const int* t,
                                     int cap_in, void* kc_out, void* vc_out, int cap_out, int* rows_out, int B, int Hkv,
                                     int D, int rp1, int sinks, int W, int umode, int elem_bytes, int max_pos,
                                     hipStream_t st) {
    const RingLay g = make_ring_lay(rp1, sinks, W, umode);
    const int row_bytes = D * elem_bytes;
    const long items = (long)(cap_out < cap_in ? cap_out : cap_in) * (row_bytes / 16);
    dim3 grid((unsigned)((items + 255) / 256), Hkv, B);
    if (to_ring)
        cache_ring_convert_kernel<true><<<grid, 256, 0, st>>>((const char*)kc_in, (const char*)vc_in, s, t, cap_in, (char*)kc_out,
                                                              (char*)vc_out, cap_out, rows_out, Hkv, g, row_bytes, max_pos);
    else
        cache_ring_convert_kernel<false><<<grid, 256, 0, st>>>((const char*)kc_in, (const char*)vc_in, s, t, cap_in, (char*)kc_out,
                                                               (char*)vc_out, cap_out, rows_out, Hkv, g, row_bytes, max_pos);
    return hipGetLastError();
}

hipError_t launch_cache_ring_append(void* kc, void* vc, const void* k_new, const void* v_new, int new_rows, const int* t_old,
                                    const int* n_new, int cap, int* rows_out, int B, int Hkv, int D, int rp1, int sinks,
                                    int W, int umode, int elem_bytes, int max_pos, hipStream_t st) {
    const RingLay g = make_ring_lay(rp1, sinks, W, umode);
    cache_ring_append_kernel<<<dim3(Hkv, B), 64, 0, st>>>((char*)kc, (char*)vc, (const char*)k_new, (const char*)v_new, new_rows,
                                                          t_old, n_new, cap, rows_out, Hkv, g, D * elem_bytes, max_pos);
    return hipGetLastError();
}

hipError_t launch_cache_update_ragged(const void* kc_in, const void* vc_in, const int* s_old, const int* t_old, int cap_in,
                                      const void* k_new, const void* v_new, const int* n_new, int new_rows,
                                      void* kc_out, void* vc_out, const int* s_new, int cap_out, int* rows_out, int B,
                                      int Hkv, int D, int rp1, int sinks, int elem_bytes, int max_pos, hipStream_t st) {
    AttnShape lay{};
    lay.rp1 = rp1;
    lay.S = sinks;
    const int row_bytes = D * elem_bytes;
    const long items = (long)cap_out * (row_bytes / 16);
    dim3 grid((unsigned)((items + 255) / 256), Hkv, B);
    cache_update_ragged_kernel<<<grid, 256, 0, st>>>((const char*)kc_in, (const char*)vc_in, s_old, t_old, cap_in,
                                                     (const char*)k_new, (const char*)v_new, n_new, new_rows,
                                                     (char*)kc_out, (char*)vc_out, s_new, cap_out, rows_out, Hkv, lay,
                                                     row_bytes, max_pos);
    return hipGetLastError();
}

hipError_t launch_cache_update(const void* kc_in, const void* vc_in, int s_old, int t_old, int cap_in,
                               const void* k_new, const void* v_new, int n_new, int new_rows, void* kc_out,
                               void* vc_out, int s_new, int cap_out, int BH, int D, int rp1, int sinks, int elem_bytes,
                               hipStream_t st) {
    AttnShape lay{};
    lay.rp1 = rp1;
    lay.S = sinks;
    const int t_new = t_old + n_new;
    const int rows_out = count_always(lay, s_new) + (t_new - s_new + 1);
    if (rows_out <= 0) return hipSuccess;
    const int row_bytes = D * elem_bytes;
    const long items = (long)rows_out * (row_bytes / 16);
    dim3 grid((unsigned)((items + 255) / 256), BH);
    cache_update_kernel<<<grid, 256, 0, st>>>((const char*)kc_in, (const char*)vc_in, (const char*)k_new,
                                              (const char*)v_new, (char*)kc_out, (char*)vc_out, s_old, t_old, cap_in,
                                              new_rows, s_new, cap_out, rows_out, lay, row_bytes);
    return hipGetLastError();
}

}  // namespace unigist
