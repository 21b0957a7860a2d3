// Internal helpers shared by the libunigist translation units (host + device).
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include "unigist.h"

namespace unigist {

typedef uint16_t bf16_t;  // raw bf16 bits
struct fp8_t {            // one E4M3 code (OCP 8-bit floating point: bias 7, no infinities, max 448)
    uint8_t bits;
};

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }

// round-to-nearest-even f32 -> bf16 (inputs are finite in this library)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// two floats -> packed bf16 pair (lo = a, hi = b), RNE, one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    f32x2 x;
    x[0] = a;
    x[1] = b;
    bf16x2 y = __builtin_convertvector(x, bf16x2);
    return __builtin_bit_cast(uint32_t, y);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// Shape of one attention problem as the kernels see it.
struct AttnShape {
    int B, Hq, Hkv, L, D;
    int rp1;  // r + 1, clamped to L + 1 when there are no gists (so (p+1) % rp1 == 0 never holds)
    int W;    // window: positions (sliding) or previous gist units (unit-aligned); clamped to L
    float scale;
    // Rows between consecutive heads in the caller's tensors (q, out, dout, dq, lse: qhs; k, v, dk, dv: kvhs).
    // Both are L for a plain [B, H, L, D] tensor; a document inside a packed buffer has L = its length and
    // the strides of the whole buffer.  Workspace arrays are always dense (stride L).
    int qhs, kvhs;
    int S;      // sink tokens in front of the first gist unit (Sec. 4.1); always visible
    int umode;  // 0: sliding window of W positions; 1: the unit holding the query plus the W previous units
    // Forward only: the query rows and the K/V rows may be a view of the L positions (chunk-wise prefill
    // over a compressed cache).  Training passes the identity view.
    int Lq;       // query rows held by q/out/lse per head
    int qpos0;    // position of query row 0; the queries are positions qpos0 .. qpos0 + Lq - 1 (= L - 1)
    int kv_rows;  // rows per head in the K/V buffers
    int s0;       // first position stored in the window region of K/V
    int ngb;      // rows in front of it: the gists at positions < s0, compact (gist g in row g)
    // Forward only: K and V stand for K * kscale[kv head] and V * vscale[kv head] (device arrays of Hkv floats; null
    // = 1).  The scales are applied in fp32 to the scores and to the output, never to the bf16 operands.
    const float* kscale;
    const float* vscale;
    // Forward only: explicit strides of q and out in elements (batch, head, row), for tensors laid out otherwise
    // than [B, Hq, qhs, D] -- e.g. [B, L, Hq, D] as projection layers produce them.  q_rs = 0: the dense layout above.
    // lse keeps the dense layout.
    long long q_bs, q_hs;
    int q_rs;
};

// ---- the visibility rule of Sec. 4.1 (Eq. 3) in the closed forms the kernels use.  A key j <= i is visible
// to query i iff it is "always visible" (a sink or a gist) or win_lo(i) <= j, equivalently i <= win_hi(j).
// first position inside the window of query i: non-decreasing in i and <= i
__host__ __device__ inline int win_lo(const AttnShape& s, int i) {
    if (!s.umode) {
        const int lo = i - s.W + 1;
        return lo < 0 ? 0 : lo;
    }
    if (i < s.S) return i;  // a sink query is in no unit: the sinks it sees are always visible anyway
    long long u = (long long)((i - s.S) / s.rp1) - s.W;
    if (u < 0) u = 0;
    return s.S + (int)(u * s.rp1);
}
// last query position that still has key j inside its window (clamped to L - 1): non-decreasing in j, >= j
__host__ __device__ inline int win_hi(const AttnShape& s, int j) {
    long long h;
    if (!s.umode) h = (long long)j + s.W - 1;
    else if (j < s.S) h = j;
    else h = (long long)s.S + ((long long)((j - s.S) / s.rp1) + s.W + 1) * s.rp1 - 1;
    return h > s.L - 1 ? s.L - 1 : (int)h;
}
__host__ __device__ inline bool is_always(const AttnShape& s, int p) { return p < s.S || (p - s.S + 1) % s.rp1 == 0; }
// number of always-visible positions < x, and the position of the c-th of them
__host__ __device__ inline int count_always(const AttnShape& s, int x) { return x <= s.S ? x : s.S + (x - s.S) / s.rp1; }
__host__ __device__ inline int pos_of_always(const AttnShape& s, int c) {
    return c < s.S ? c : s.S + (c - s.S) * s.rp1 + s.rp1 - 1;
}

// The matrix-core kernels are built for head dimensions 64 and 128; a smaller one (a multiple of 8) runs on the next
// of the two with the missing columns treated as zeros.
__host__ __device__ inline int padded_head_dim(int D) { return D <= 64 ? 64 : 128; }

// the shape of a plain [B, H, L, D] problem (host)
inline AttnShape make_shape(int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks = 0,
                     int window_mode = UNIGIST_WINDOW_SLIDING) {
    AttnShape s;
    s.B = B;
    s.Hq = Hq;
    s.Hkv = Hkv;
    s.L = L;
    s.D = D;
    s.rp1 = r >= L ? L + 1 : r + 1;  // r >= L: no position holds a gist
    s.W = W > L ? L : W;
    s.scale = 1.0f / sqrtf((float)D);
    s.S = sinks > L ? L : sinks;
    s.umode = window_mode == UNIGIST_WINDOW_UNITS;
    s.qhs = L;
    s.kvhs = L;
    s.Lq = L;
    s.qpos0 = 0;
    s.kv_rows = L;
    s.s0 = 0;
    s.ngb = 0;
    s.kscale = nullptr;
    s.vscale = nullptr;
    s.q_bs = 0;
    s.q_hs = 0;
    s.q_rs = 0;
    return s;
}

// ---- packed documents: one launch covers up to kMaxDocs documents of a [H, T, D] buffer, each an independent
// sequence (its gist period and window restart at its first row).  The table travels as a kernel argument and is
// read with scalar loads; a workgroup finds its document from its id.
constexpr int kMaxDocs = 64;
struct DocTab {
    int n;                   // documents in this launch (>= 1), none of them empty
    int c0[kMaxDocs];        // first row of the document inside a head of the packed buffers
    int len[kMaxDocs];       // its rows
    int blk0[kMaxDocs + 1];  // first workgroup id of the document in this launch; blk0[n] = grid size
    int part0[kMaxDocs];     // backward: the document's first slot in the array of per-segment gist partials
    int comp0[kMaxDocs];     // backward: the document's first slot in the array of reduced gist sums
};
struct NoDocs {};
// document owning workgroup blk: the last d with blk0[d] <= blk
__device__ __forceinline__ int doc_of_block(const DocTab& t, int blk) {
    int lo = 0, hi = t.n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (t.blk0[mid] <= blk) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}
// the shape of one document of len rows, given the shape of the whole pack (B = 1, L = T, strides T)
__host__ __device__ inline AttnShape doc_view(AttnShape s, int len) {
    s.rp1 = s.rp1 - 1 >= len ? len + 1 : s.rp1;
    s.W = s.W > len ? len : s.W;
    s.S = s.S > len ? len : s.S;
    s.L = len;
    s.Lq = len;
    return s;
}

// ---- chunk-wise prefill of a batch whose sequences are in different states (device arrays of B ints)
struct RaggedSeqs {
    const int* p0;  // position of the sequence's first query row
    const int* n;   // its query rows in this chunk (the first n rows of its slab of q/out/lse)
    const int* s0;  // first position stored in the window region of its cache
    int* rows;      // out: cache rows in use, -1 if the state is invalid (then nothing else is written for it)
};
// The shape of one such sequence, given the launch's shape (L = the largest position count allowed, Lq = rows per
// slab of q, kv_rows = cache capacity).  Needs n >= 1.
__host__ __device__ inline AttnShape seq_view(AttnShape s, int p0, int n, int s0) {
    const int L = p0 + n;
    s.rp1 = s.rp1 - 1 >= L ? L + 1 : s.rp1;
    s.W = s.W > L ? L : s.W;
    s.S = s.S > L ? L : s.S;
    s.L = L;
    s.Lq = n;
    s.qpos0 = p0;
    s.s0 = s0;
    s.ngb = count_always(s, s0);
    return s;
}

// --- launchers implemented in the .hip files (all enqueue on `st`, return hipGetLastError) ---
hipError_t launch_fwd_simple(const void* q, const void* k, const void* v, void* out, float* lse,
                             const AttnShape& s, unigist_dtype dt, hipStream_t st);
hipError_t launch_bwd_simple(const void* q, const void* k, const void* v, const void* out, const float* lse,
                             const void* dout, void* dq, void* dk, void* dv, float* delta,
                             const AttnShape& s, unigist_dtype dt, hipStream_t st);
hipError_t launch_fwd_mfma(const void* q, const void* k, const void* v, void* out, float* lse,
                           const AttnShape& s, hipStream_t st);
// the same over the documents [cu[d], cu[d+1]) of a packed buffer (s: the shape of the whole pack), one launch
// per kMaxDocs documents
hipError_t launch_fwd_mfma_pack(const void* q, const void* k, const void* v, void* out, float* lse,
                                const AttnShape& s, const int* cu, int ndocs, hipStream_t st);
// chunk-wise prefill with per-sequence states (s: the launch's shape, see seq_view; cap = s.kv_rows)
hipError_t launch_fwd_mfma_ragged(const void* q, const void* k, const void* v, void* out, float* lse,
                                  const AttnShape& s, const RaggedSeqs& seqs, hipStream_t st);
size_t bwd_mfma_workspace(const AttnShape& s);
hipError_t launch_bwd_mfma(const void* q, const void* k, const void* v, const void* out, const float* lse,
                           const void* dout, void* dq, void* dk, void* dv, void* ws,
                           const AttnShape& s, unsigned stages, hipStream_t st);
// packed documents (see launch_fwd_mfma_pack); ws: bwd_mfma_pack_workspace bytes (0: the pack is too large)
size_t bwd_mfma_pack_workspace(const AttnShape& s, const int* cu, int ndocs);
hipError_t launch_bwd_mfma_pack(const void* q, const void* k, const void* v, const void* out, const float* lse,
                                const void* dout, void* dq, void* dk, void* dv, void* ws, const AttnShape& s,
                                const int* cu, int ndocs, hipStream_t st);
bool decode_grouped(int Hq, int Hkv, unigist_dtype dt);
int decode_num_splits(int B, int Hq, int Hkv, int Lk, unigist_dtype dt);
hipError_t launch_cache_update(const void* kc_in, const void* vc_in, int s_old, int t_old, int cap_in,
                               const void* k_new, const void* v_new, int n_new, int new_rows,
                               void* kc_out, void* vc_out, int s_new, int cap_out,
                               int BH, int D, int rp1, int sinks, int elem_bytes, hipStream_t st);
hipError_t launch_cache_update_ragged(const void* kc_in, const void* vc_in, const int* s_old, const int* t_old, int cap_in,
                                      const void* k_new, const void* v_new, const int* n_new, int new_rows,
                                      void* kc_out, void* vc_out, const int* s_new, int cap_out, int* rows_out, int B,
                                      int Hkv, int D, int rp1, int sinks, int elem_bytes, int max_pos, hipStream_t st);
// ring layout of the cache for token-by-token decoding (see cache.hip)
hipError_t launch_cache_ring_convert(bool to_ring, const void* kc_in, const void* vc_in, const int* s, const int* t,
                                     int cap_in, void* kc_out, void* vc_out, int cap_out, int* rows_out, int B, int Hkv,
                                     int D, int rp1, int sinks, int W, int umode, int elem_bytes, int max_pos,
                                     hipStream_t st);
hipError_t launch_cache_ring_append(void* kc, void* vc, const void* k_new, const void* v_new, int new_rows, const int* t_old,
                                    const int* n_new, int cap, int* rows_out, int B, int Hkv, int D, int rp1, int sinks,
                                    int W, int umode, int elem_bytes, int max_pos, hipStream_t st);
hipError_t launch_decode(const void* q, const void* kc, const void* vc, void* out, float* lse,
                         int B, int Hq, int Hkv, int Lk, const int* seqlens, int D, unigist_dtype dt,
                         float* ws, hipStream_t st);
// bf16 queries over a cache of E4M3 codes with one scale per kv head (device arrays of Hkv floats)
hipError_t launch_decode_fp8(const void* q, const void* kc, const void* vc, const float* k_scale, const float* v_scale,
                             void* out, float* lse, int B, int Hq, int Hkv, int Lk, const int* seqlens, int D,
                             float* ws, hipStream_t st);
// the first `rows` rows of every [cap, D] slab of E4M3 codes -> bf16 (exact), slabs of `rows` rows; BH slabs
hipError_t launch_widen_e4m3(const void* codes, void* y, int BH, int cap, int rows, int D, hipStream_t st);
// y = e4m3(x / scale[head]) for x [B, H, n, D] (bf16 or fp32), 16 elements per lane
hipError_t launch_quantize_e4m3(const void* x, void* y, const float* scale, int B, int H, int n, int D,
                                unigist_dtype dt_in, hipStream_t st);
hipError_t launch_read_rate(const void* buf, size_t bytes, unsigned* sink, int blocks, hipStream_t st);
hipError_t launch_mfma_rate(const void* operands, long long* clocks, float* sink, int blocks, int iters, hipStream_t st);

}  // namespace unigist
