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

// ---- ring layout for token-by-token decoding with the sliding window (sinks allowed).  Decode attends to every
// row of a sequence's slab whatever their order, so a new token can take the row of the token that leaves the
// window at the same moment: rows [0, W) hold the window, position p in row p % W; rows [W, W + nf) hold the
// always-visible positions (sinks, gists) that have left the window, in order of position.  Appending a token is
// then one row written (two when the position leaving the window is a sink or a gist, which first moves to the
// far region) instead of a gather of the whole cache.
__device__ __forceinline__ int ring_far(const AttnShape& lay, int W, int t) { return count_always(lay, t - W + 1 > 0 ? t - W + 1 : 0); }
__device__ __forceinline__ int ring_rows(const AttnShape& lay, int W, int t) { return (t + 1 < W ? t + 1 : W) + ring_far(lay, W, t); }

// TO_RING: canonical state (s[b], t[b]) -> ring state t[b].  !TO_RING: ring state t[b] -> canonical (s[b], t[b]).
template <bool TO_RING>
__global__ __launch_bounds__(256) void cache_ring_convert_kernel(const char* __restrict__ kc_in, const char* __restrict__ vc_in,
                                                                const int* __restrict__ s_v, const int* __restrict__ t_v,
                                                                int cap_in, char* __restrict__ kc_out, char* __restrict__ vc_out,
                                                                int cap_out, int* __restrict__ rows_out_v, int Hkv,
                                                                AttnShape lay, int W, int row_bytes, int max_pos) {
    const int b = blockIdx.z, bh = b * Hkv + blockIdx.y;
    const int s = s_v[b], t = t_v[b];
    const int wfirst = t - W + 1 > 0 ? t - W + 1 : 0;  // first position of the window of a query at t
    // the canonical side must hold the whole window (s <= wfirst) and nothing the ring cannot hold (s >= wfirst)
    bool ok = s >= 0 && t >= s - 1 && t < max_pos && (t < 0 ? s == 0 : s == wfirst);
    int rows_out = -1;
    if (ok) {
        const int rows_can = count_always(lay, s) + (t - s + 1), rows_ring = ring_rows(lay, W, t);
        rows_out = TO_RING ? rows_ring : rows_can;
        if ((TO_RING ? rows_can : rows_ring) > cap_in || rows_out > cap_out) {
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
    const int ng = count_always(lay, s);
    const int nwin = t + 1 < W ? t + 1 : W;
    int src;
    if (TO_RING) {
        // position held by ring row n, then its canonical row (compact entry i sits in row i)
        if (n < nwin) {
            const int pos = t - (t - n) % W;
            src = ng + (pos - s);
        } else {
            src = n - W;  // the (n - W)-th always-visible position: left of s, hence compact entry n - W
        }
    } else {
        const int pos = n < ng ? pos_of_always(lay, n) : s + (n - ng);
        src = pos > t - W ? pos % W : W + n;  // far entry n is the n-th always-visible position
    }
    const size_t i = ((size_t)bh * cap_in + src) * row_bytes + ch * 16;
    const size_t o = ((size_t)bh * cap_out + n) * row_bytes + ch * 16;
    *(u32x4*)(kc_out + o) = *(const u32x4*)(kc_in + i);
    *(u32x4*)(vc_out + o) = *(const u32x4*)(vc_in + i);
}

// One token per active sequence, in place.  grid (Hkv, B), 64 lanes: lanes 0 .. cpr-1 move K, lanes 32 .. 32+cpr-1 V.
__global__ __launch_bounds__(64) void cache_ring_append_kernel(char* __restrict__ kc, char* __restrict__ vc,
                                                              const char* __restrict__ k_new, const char* __restrict__ v_new,
                                                              int new_rows, const int* __restrict__ t_old_v,
                                                              const int* __restrict__ n_new_v, int cap,
                                                              int* __restrict__ rows_out_v, int Hkv, AttnShape lay, int W,
                                                              int row_bytes, int max_pos) {
    const int b = blockIdx.y, bh = b * Hkv + blockIdx.x;
    const int t_old = t_old_v[b], act = n_new_v[b];
    int rows = -1;
    const bool ok0 = t_old >= -1 && (act == 0 || act == 1) && t_old < max_pos - act;
    const int t = t_old + act;
    if (ok0) {
        rows = ring_rows(lay, W, t);
        if (rows > cap) rows = -1;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) rows_out_v[b] = rows;
    if (rows < 0 || act == 0) return;
    const int cpr = row_bytes / 16;
    const int lane = threadIdx.x & 31;
    if (lane >= cpr) return;
    char* c = (threadIdx.x < 32 ? kc : vc) + (size_t)bh * cap * row_bytes + lane * 16;
    const char* nw = (threadIdx.x < 32 ? k_new : v_new) + (size_t)bh * new_rows * row_bytes + lane * 16;
    const int slot = t % W;
    const int p_out = t - W;  // leaves the window now; its row is the one the new token takes
    if (p_out >= 0 && is_always(lay, p_out)) {
        const u32x4 keep = *(const u32x4*)(c + (size_t)slot * row_bytes);
        *(u32x4*)(c + (size_t)(W + count_always(lay, p_out)) * row_bytes) = keep;  // read before the slot is overwritten below
    }
    *(u32x4*)(c + (size_t)slot * row_bytes) = *(const u32x4*)nw;
}

}  // namespace

hipError_t launch_cache_ring_convert(bool to_ring, const void* kc_in, const void* vc_in, const int* s, const int* t,
                                     int cap_in, void* kc_out, void* vc_out, int cap_out, int* rows_out, int B, int Hkv,
                                     int D, int rp1, int sinks, int W, int elem_bytes, int max_pos, hipStream_t st) {
    AttnShape lay{};
    lay.rp1 = rp1;
    lay.S = sinks;
    const int row_bytes = D * elem_bytes;
    const long items = (long)cap_out * (row_bytes / 16);
    dim3 grid((unsigned)((items + 255) / 256), Hkv, B);
    if (to_ring)
        cache_ring_convert_kernel<true><<<grid, 256, 0, st>>>((const char*)kc_in, (const char*)vc_in, s, t, cap_in, (char*)kc_out,
                                                              (char*)vc_out, cap_out, rows_out, Hkv, lay, W, row_bytes, max_pos);
    else
        cache_ring_convert_kernel<false><<<grid, 256, 0, st>>>((const char*)kc_in, (const char*)vc_in, s, t, cap_in, (char*)kc_out,
                                                               (char*)vc_out, cap_out, rows_out, Hkv, lay, W, row_bytes, max_pos);
    return hipGetLastError();
}

hipError_t launch_cache_ring_append(void* kc, void* vc, const void* k_new, const void* v_new, int new_rows, const int* t_old,
                                    const int* n_new, int cap, int* rows_out, int B, int Hkv, int D, int rp1, int sinks,
                                    int W, int elem_bytes, int max_pos, hipStream_t st) {
    AttnShape lay{};
    lay.rp1 = rp1;
    lay.S = sinks;
    cache_ring_append_kernel<<<dim3(Hkv, B), 64, 0, st>>>((char*)kc, (char*)vc, (const char*)k_new, (const char*)v_new, new_rows,
                                                          t_old, n_new, cap, rows_out, Hkv, lay, W, D * elem_bytes, max_pos);
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
