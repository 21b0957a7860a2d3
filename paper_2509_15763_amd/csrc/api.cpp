// C ABI of libunigist: argument validation and dispatch.  No device memory is
// allocated here and nothing synchronises; kernels are enqueued on the caller's stream
// (the document-by-document packed backward of the fp32 kernels also uses helper streams ordered behind and
// before it, see for_each_doc).
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <vector>

#include "common.h"

using namespace unigist;

namespace {

constexpr int kMaxL = 1 << 23;  // per-head byte offsets (L * D * 2) are kept in 32 bits inside the kernels

// Head dimensions: any multiple of 8 up to 128 (rows are moved in 16-byte pieces; of 16 for one-byte E4M3 codes).  The
// matrix-core kernels are built for 64 and 128 and run smaller ones on the next of the two, the missing columns
// taken as zeros.  Beyond 128 the dK/dV kernel's register budget ends: its dK^T and dV^T accumulators for a wave's
// 32 keys would take 256 registers per lane at D = 256 on top of 128 for the K and V operands.
bool head_dim_ok(int D, unigist_dtype dt) { return D >= 8 && D <= 128 && D % (dt == UNIGIST_E4M3 ? 16 : 8) == 0; }

// Debug switch (unigist_debug_force_plain_alu): bf16 calls take the plain-ALU kernels.  The environment variable
// UNIGIST_DEBUG_PLAIN_ALU=1 sets its initial value; it is read once, when the library is loaded.
std::atomic<int> g_plain_alu{[] {
    const char* e = getenv("UNIGIST_DEBUG_PLAIN_ALU");
    return e && e[0] == '1' ? 1 : 0;
}()};
bool plain_alu_forced() { return g_plain_alu.load(std::memory_order_relaxed) != 0; }

unigist_status check_attn(int B, int Hq, int Hkv, int L, int D, int r, int W, unigist_dtype dt, int sinks = 0,
                          int window_mode = UNIGIST_WINDOW_SLIDING) {
    if (B < 1 || Hq < 1 || Hkv < 1 || L < 1 || D < 1 || r < 1 || W < 1 || sinks < 0) return UNIGIST_EINVAL;
    if (window_mode != UNIGIST_WINDOW_SLIDING && window_mode != UNIGIST_WINDOW_UNITS) return UNIGIST_EINVAL;
    if (Hq % Hkv != 0) return UNIGIST_EINVAL;
    if (dt != UNIGIST_BF16 && dt != UNIGIST_F32) return UNIGIST_EUNSUPPORTED;
    if (!head_dim_ok(D, dt)) return UNIGIST_EUNSUPPORTED;
    if (L > kMaxL || B > 65535 || Hq > 65535) return UNIGIST_EUNSUPPORTED;
    if ((long long)B * Hkv > 65535) return UNIGIST_EUNSUPPORTED;  // (batch, kv head) pairs index a grid's z dimension
    return UNIGIST_OK;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

extern "C" const char* unigist_status_str(unigist_status s) {
    // callers in other languages pass any integer: read it as one (an out-of-range value held in the enum type is
    // undefined behaviour to load in C++)
    int code;
    memcpy(&code, &s, sizeof code);
    switch (code) {
        case UNIGIST_OK: return "ok";
        case UNIGIST_EINVAL: return "invalid argument";
        case UNIGIST_EUNSUPPORTED: return "unsupported head dim, dtype or size";
        case UNIGIST_ELAUNCH: return "HIP launch error";
        case UNIGIST_ESCRATCH: return "problem exceeds the built-in scratch array of the allocation-free entry point";
    }
    return "unknown status";
}

extern "C" int unigist_debug_force_plain_alu(int on) { return g_plain_alu.exchange(on ? 1 : 0); }

extern "C" void unigist_tile_sizes(int D, unigist_dtype dt, int* Bm, int* Bn) {
    (void)D;
    if (Bm) *Bm = dt == UNIGIST_BF16 ? 128 : 64;
    if (Bn) *Bn = dt == UNIGIST_BF16 ? 32 : 1;
}

extern "C" unigist_status unigist_probe_mfma_rate(const void* operands, long long* clocks, float* sink, int blocks,
                                                  int iters, void* hip_stream) {
    if (!operands || !clocks || !sink || blocks < 1 || blocks > 65536 || iters < 1) return UNIGIST_EINVAL;
    return launch_mfma_rate(operands, clocks, sink, blocks, iters, (hipStream_t)hip_stream) == hipSuccess ? UNIGIST_OK
                                                                                                          : UNIGIST_ELAUNCH;
}

extern "C" unigist_status unigist_probe_read_rate(const void* buf, size_t bytes, unsigned* sink, int blocks,
                                                  void* hip_stream) {
    if (!buf || !sink || bytes < 16 || blocks < 1 || blocks > 65536 || ((uintptr_t)buf & 15) != 0) return UNIGIST_EINVAL;
    return launch_read_rate(buf, bytes, sink, blocks, (hipStream_t)hip_stream) == hipSuccess ? UNIGIST_OK : UNIGIST_ELAUNCH;
}

extern "C" unigist_status unigist_attn_fwd(const void* q, const void* k, const void* v, void* out, float* lse,
                                           int B, int Hq, int Hkv, int L, int D, int r, int W, unigist_dtype dt,
                                           void* hip_stream) {
    return unigist_attn_fwd_ex(q, k, v, out, lse, B, Hq, Hkv, L, D, r, W, 0, UNIGIST_WINDOW_SLIDING, dt, hip_stream);
}

extern "C" unigist_status unigist_attn_fwd_ex(const void* q, const void* k, const void* v, void* out, float* lse,
                                              int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks,
                                              int window_mode, unigist_dtype dt, void* hip_stream) {
    unigist_status st = check_attn(B, Hq, Hkv, L, D, r, W, dt, sinks, window_mode);
    if (st != UNIGIST_OK) return st;
    if (!q || !k || !v || !out || !lse) return UNIGIST_EINVAL;
    const AttnShape s = make_shape(B, Hq, Hkv, L, D, r, W, sinks, window_mode);
    hipStream_t stream = (hipStream_t)hip_stream;
    hipError_t e;
    if (dt == UNIGIST_BF16 && !plain_alu_forced())
        e = launch_fwd_mfma(q, k, v, out, lse, s, stream);
    else
        e = launch_fwd_simple(q, k, v, out, lse, s, dt, stream);
    return e == hipSuccess ? UNIGIST_OK : UNIGIST_ELAUNCH;
}

// ---- q, out, dout, dq with explicit strides (k, v, dk, dv, lse dense)
namespace {
unigist_status check_qstrides(const void* a, const void* b, int L, int D, long long q_bs, long long q_hs, long long q_rs,
                              unigist_dtype dt) {
    if (dt != UNIGIST_BF16 || plain_alu_forced()) return UNIGIST_EUNSUPPORTED;  // the bf16 matrix-core kernels only
    // 16-byte vector accesses: strides in multiples of 8 elements, aligned bases; rows must not overlap
    if (q_rs < D || q_hs < 1 || q_bs < 0 || q_rs > 0x7fffffffLL) return UNIGIST_EINVAL;
    if ((q_rs | q_hs | q_bs) & 7) return UNIGIST_EINVAL;
    if (((uintptr_t)a & 15) != 0 || ((uintptr_t)b & 15) != 0) return UNIGIST_EINVAL;
    if ((long long)L * q_rs * 2 > 0xffffffffLL) return UNIGIST_EUNSUPPORTED;  // byte offsets inside a head stay in 32 bits
    return UNIGIST_OK;
}
}  // namespace

extern "C" unigist_status unigist_attn_fwd_strided(const void* q, const void* k, const void* v, void* out, float* lse,
                                                   int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks,
                                                   int window_mode, long long q_batch_stride, long long q_head_stride,
                                                   long long q_row_stride, unigist_dtype dt, void* hip_stream) {
    unigist_status st = check_attn(B, Hq, Hkv, L, D, r, W, dt, sinks, window_mode);
    if (st != UNIGIST_OK) return st;
    if (!q || !k || !v || !out || !lse) return UNIGIST_EINVAL;
    if ((st = check_qstrides(q, out, L, D, q_batch_stride, q_head_stride, q_row_stride, dt)) != UNIGIST_OK) return st;
    AttnShape s = make_shape(B, Hq, Hkv, L, D, r, W, sinks, window_mode);
    s.q_bs = q_batch_stride;
    s.q_hs = q_head_stride;
    s.q_rs = (int)q_row_stride;
    return launch_fwd_mfma(q, k, v, out, lse, s, (hipStream_t)hip_stream) == hipSuccess ? UNIGIST_OK : UNIGIST_ELAUNCH;
}

extern "C" unigist_status unigist_attn_bwd_strided(const void* q, const void* k, const void* v, const void* out,
                                                   const float* lse, const void* dout, void* dq, void* dk, void* dv,
                                                   int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks,
                                                   int window_mode, long long q_batch_stride, long long q_head_stride,
                                                   long long q_row_stride, unigist_dtype dt, void* workspace,
                                                   size_t workspace_bytes, void* hip_stream) {
    unigist_status st = check_attn(B, Hq, Hkv, L, D, r, W, dt, sinks, window_mode);
    if (st != UNIGIST_OK) return st;
    if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv || !workspace) return UNIGIST_EINVAL;
    if ((st = check_qstrides(q, out, L, D, q_batch_stride, q_head_stride, q_row_stride, dt)) != UNIGIST_OK) return st;
    if ((st = check_qstrides(dout, dq, L, D, q_batch_stride, q_head_stride, q_row_stride, dt)) != UNIGIST_OK) return st;
    if (workspace_bytes < unigist_attn_bwd_workspace_ex(B, Hq, Hkv, L, D, r, W, sinks, window_mode, dt))
        return UNIGIST_EINVAL;
    if (((uintptr_t)workspace & 255) != 0) return UNIGIST_EINVAL;
    AttnShape s = make_shape(B, Hq, Hkv, L, D, r, W, sinks, window_mode);
    s.q_bs = q_batch_stride;
    s.q_hs = q_head_stride;
    s.q_rs = (int)q_row_stride;
    return launch_bwd_mfma(q, k, v, out, lse, dout, dq, dk, dv, workspace, s, UNIGIST_BWD_ALL, (hipStream_t)hip_stream) ==
                   hipSuccess
               ? UNIGIST_OK
               : UNIGIST_ELAUNCH;
}

extern "C" size_t unigist_attn_bwd_workspace(int B, int Hq, int Hkv, int L, int D, int r, int W,
                                             unigist_dtype dt) {
    return unigist_attn_bwd_workspace_ex(B, Hq, Hkv, L, D, r, W, 0, UNIGIST_WINDOW_SLIDING, dt);
}

extern "C" size_t unigist_attn_bwd_workspace_ex(int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks,
                                                int window_mode, unigist_dtype dt) {
    if (check_attn(B, Hq, Hkv, L, D, r, W, dt, sinks, window_mode) != UNIGIST_OK) return 0;
    const AttnShape s = make_shape(B, Hq, Hkv, L, D, r, W, sinks, window_mode);
    size_t delta = align256((size_t)B * Hq * L * sizeof(float));
    size_t mfma = dt == UNIGIST_BF16 ? bwd_mfma_workspace(s) : 0;
    return delta > mfma ? delta : mfma;
}

extern "C" unigist_status unigist_attn_bwd_stages(const void* q, const void* k, const void* v, const void* out,
                                                  const float* lse, const void* dout, void* dq, void* dk, void* dv,
                                                  int B, int Hq, int Hkv, int L, int D, int r, int W,
                                                  unigist_dtype dt, void* workspace, size_t workspace_bytes,
                                                  unsigned stages, void* hip_stream) {
    return unigist_attn_bwd_ex(q, k, v, out, lse, dout, dq, dk, dv, B, Hq, Hkv, L, D, r, W, 0,
                               UNIGIST_WINDOW_SLIDING, dt, workspace, workspace_bytes, stages, hip_stream);
}

extern "C" unigist_status unigist_attn_bwd_ex(const void* q, const void* k, const void* v, const void* out,
                                              const float* lse, const void* dout, void* dq, void* dk, void* dv,
                                              int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks,
                                              int window_mode, unigist_dtype dt, void* workspace,
                                              size_t workspace_bytes, unsigned stages, void* hip_stream) {
    unigist_status st = check_attn(B, Hq, Hkv, L, D, r, W, dt, sinks, window_mode);
    if (st != UNIGIST_OK) return st;
    if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv || !workspace) return UNIGIST_EINVAL;
    if (stages == 0 || (stages & ~(unsigned)UNIGIST_BWD_ALL)) return UNIGIST_EINVAL;
    if (workspace_bytes < unigist_attn_bwd_workspace_ex(B, Hq, Hkv, L, D, r, W, sinks, window_mode, dt))
        return UNIGIST_EINVAL;
    if (((uintptr_t)workspace & 255) != 0) return UNIGIST_EINVAL;
    const AttnShape s = make_shape(B, Hq, Hkv, L, D, r, W, sinks, window_mode);
    hipStream_t stream = (hipStream_t)hip_stream;
    hipError_t e;
    if (dt == UNIGIST_BF16 && !plain_alu_forced()) {
        e = launch_bwd_mfma(q, k, v, out, lse, dout, dq, dk, dv, workspace, s, stages, stream);
    } else {
        if (stages != UNIGIST_BWD_ALL) return UNIGIST_EUNSUPPORTED;
        e = launch_bwd_simple(q, k, v, out, lse, dout, dq, dk, dv, (float*)workspace, s, dt, stream);
    }
    return e == hipSuccess ? UNIGIST_OK : UNIGIST_ELAUNCH;
}

extern "C" unigist_status unigist_attn_bwd(const void* q, const void* k, const void* v, const void* out,
                                           const float* lse, const void* dout, void* dq, void* dk, void* dv,
                                           int B, int Hq, int Hkv, int L, int D, int r, int W, unigist_dtype dt,
                                           void* workspace, size_t workspace_bytes, void* hip_stream) {
    return unigist_attn_bwd_stages(q, k, v, out, lse, dout, dq, dk, dv, B, Hq, Hkv, L, D, r, W, dt, workspace,
                                   workspace_bytes, UNIGIST_BWD_ALL, hip_stream);
}

extern "C" size_t unigist_decode_workspace(int B, int Hq, int Hkv, int Lk_max, int D, unigist_dtype dt) {
    if (B < 1 || Hq < 1 || Hkv < 1 || Lk_max < 1 || Hq % Hkv != 0) return 0;
    if (!head_dim_ok(D, dt) || (dt != UNIGIST_BF16 && dt != UNIGIST_F32)) return 0;
    const int ns = decode_num_splits(B, Hq, Hkv, Lk_max, dt);
    return align256((size_t)B * Hq * ns * (padded_head_dim(D) + 2) * sizeof(float));
}

extern "C" unigist_status unigist_decode(const void* q, const void* kcache, const void* vcache, void* out,
                                         float* lse, int B, int Hq, int Hkv, int Lk_max, const int* seqlens, int D,
                                         unigist_dtype dt, void* workspace, size_t workspace_bytes,
                                         void* hip_stream) {
    if (B < 1 || Hq < 1 || Hkv < 1 || Lk_max < 1 || D < 1) return UNIGIST_EINVAL;
    if (Hq % Hkv != 0) return UNIGIST_EINVAL;
    if (dt != UNIGIST_BF16 && dt != UNIGIST_F32) return UNIGIST_EUNSUPPORTED;
    if (!head_dim_ok(D, dt)) return UNIGIST_EUNSUPPORTED;
    if (B > 65535 || Hq > 65535) return UNIGIST_EUNSUPPORTED;
    if (!q || !kcache || !vcache || !out || !workspace) return UNIGIST_EINVAL;
    if (workspace_bytes < unigist_decode_workspace(B, Hq, Hkv, Lk_max, D, dt)) return UNIGIST_EINVAL;
    if (((uintptr_t)workspace & 255) != 0) return UNIGIST_EINVAL;
    hipError_t e = launch_decode(q, kcache, vcache, out, lse, B, Hq, Hkv, Lk_max, seqlens, D, dt,
                                 (float*)workspace, (hipStream_t)hip_stream);
    return e == hipSuccess ? UNIGIST_OK : UNIGIST_ELAUNCH;
}

extern "C" unigist_status unigist_quantize_e4m3(const void* x, void* y, const float* scale, int B, int H, int n, int D,
                                                unigist_dtype dt_in, void* hip_stream) {
    if (B < 1 || H < 1 || n < 0 || D < 1) return UNIGIST_EINVAL;
    if (dt_in != UNIGIST_BF16 && dt_in != UNIGIST_F32) return UNIGIST_EUNSUPPORTED;
    if (!head_dim_ok(D, UNIGIST_E4M3)) return UNIGIST_EUNSUPPORTED;
    if (!scale || (n > 0 && (!x || !y))) return UNIGIST_EINVAL;
    if (((uintptr_t)x & 15) != 0 || ((uintptr_t)y & 15) != 0) return UNIGIST_EINVAL;
    hipError_t e = launch_quantize_e4m3(x, y, scale, B, H, n, D, dt_in, (hipStream_t)hip_stream);
    return e == hipSuccess ? UNIGIST_OK : UNIGIST_ELAUNCH;
}

extern "C" unigist_status unigist_decode_e4m3(const void* q, const void* kcache, const void* vcache,
                                              const float* k_scale, const float* v_scale, void* out, float* lse, int B,
                                              int Hq, int Hkv, int Lk_max, const int* seqlens, int D, void* workspace,
                                              size_t workspace_bytes, void* hip_stream) {
    if (B < 1 || Hq < 1 || Hkv < 1 || Lk_max < 1 || D < 1) return UNIGIST_EINVAL;
    if (Hq % Hkv != 0) return UNIGIST_EINVAL;
    if (!head_dim_ok(D, UNIGIST_E4M3)) return UNIGIST_EUNSUPPORTED;
    if (B > 65535 || Hq > 65535) return UNIGIST_EUNSUPPORTED;
    if (!q || !kcache || !vcache || !k_scale || !v_scale || !out || !workspace) return UNIGIST_EINVAL;
    if (workspace_bytes < unigist_decode_workspace(B, Hq, Hkv, Lk_max, D, UNIGIST_BF16)) return UNIGIST_EINVAL;
    if (((uintptr_t)workspace & 255) != 0) return UNIGIST_EINVAL;
    if (((uintptr_t)kcache & 15) != 0 || ((uintptr_t)vcache & 15) != 0 || ((uintptr_t)q & 15) != 0) return UNIGIST_EINVAL;
    hipError_t e = launch_decode_fp8(q, kcache, vcache, k_scale, v_scale, out, lse, B, Hq, Hkv, Lk_max, seqlens, D,
                                     (float*)workspace, (hipStream_t)hip_stream);
    return e == hipSuccess ? UNIGIST_OK : UNIGIST_ELAUNCH;
}

extern "C" int unigist_window_start(int t, int r, int W, int sinks, int window_mode) {
    if (t < -1 || r < 1 || W < 1 || sinks < 0) return -1;
    if (window_mode != UNIGIST_WINDOW_SLIDING && window_mode != UNIGIST_WINDOW_UNITS) return -1;
    if (t >= kMaxL) return -1;
    if (t == -1) return 0;  // no position yet: the empty cache is in state (0, -1)
    const AttnShape s = make_shape(1, 1, 1, t + 1, 64, r, W, sinks, window_mode);
    return win_lo(s, t);
}

extern "C" int unigist_cache_rows(int s, int t, int r) { return unigist_cache_rows_ex(s, t, r, 0); }

extern "C" int unigist_cache_rows_ex(int s, int t, int r, int sinks) {
    if (s < 0 || r < 1 || sinks < 0 || t < s - 1) return -1;
    const long long na = s <= sinks ? s : sinks + ((long long)s - sinks) / ((long long)r + 1);
    return (int)na + (t - s + 1);
}

extern "C" unigist_status unigist_cache_update(const void* kc_in, const void* vc_in, int s_old, int t_old, int cap_in,
                                               const void* k_new, const void* v_new, int n_new, int new_rows,
                                               void* kc_out, void* vc_out, int s_new, int cap_out, int B, int Hkv,
                                               int D, int r, unigist_dtype dt, void* hip_stream) {
    return unigist_cache_update_ex(kc_in, vc_in, s_old, t_old, cap_in, k_new, v_new, n_new, new_rows, kc_out, vc_out,
                                   s_new, cap_out, B, Hkv, D, r, 0, dt, hip_stream);
}

extern "C" unigist_status unigist_cache_update_ex(const void* kc_in, const void* vc_in, int s_old, int t_old,
                                                  int cap_in, const void* k_new, const void* v_new, int n_new,
                                                  int new_rows, void* kc_out, void* vc_out, int s_new, int cap_out,
                                                  int B, int Hkv, int D, int r, int sinks, unigist_dtype dt,
                                                  void* hip_stream) {
    if (B < 1 || Hkv < 1 || D < 1 || r < 1 || sinks < 0 || n_new < 0 || new_rows < n_new || cap_in < 0 || cap_out < 1)
        return UNIGIST_EINVAL;
    if (dt != UNIGIST_BF16 && dt != UNIGIST_F32 && dt != UNIGIST_E4M3) return UNIGIST_EUNSUPPORTED;
    if (!head_dim_ok(D, dt)) return UNIGIST_EUNSUPPORTED;
    if (s_old < 0 || t_old < s_old - 1 || s_new < s_old) return UNIGIST_EINVAL;
    const long long t_new = (long long)t_old + n_new;
    if (t_new > kMaxL || s_new > t_new + 1) return UNIGIST_EINVAL;
    if ((long long)B * Hkv > 65535) return UNIGIST_EUNSUPPORTED;
    const int rows_in = unigist_cache_rows_ex(s_old, t_old, r, sinks);
    const int rows_out = unigist_cache_rows_ex(s_new, (int)t_new, r, sinks);
    if (rows_in > cap_in || rows_out > cap_out) return UNIGIST_EINVAL;
    if (!kc_out || !vc_out) return UNIGIST_EINVAL;
    if (rows_in > 0 && (!kc_in || !vc_in)) return UNIGIST_EINVAL;
    if (n_new > 0 && (!k_new || !v_new)) return UNIGIST_EINVAL;
    const int rp1 = r >= kMaxL ? kMaxL + 1 : r + 1;
    hipError_t e = launch_cache_update(kc_in, vc_in, s_old, t_old, cap_in, k_new, v_new, n_new, new_rows, kc_out,
                                       vc_out, s_new, cap_out, B * Hkv, D, rp1, sinks > kMaxL ? kMaxL : sinks,
                                       dt == UNIGIST_E4M3 ? 1 : dt == UNIGIST_BF16 ? 2 : 4, (hipStream_t)hip_stream);
    return e == hipSuccess ? UNIGIST_OK : UNIGIST_ELAUNCH;
}

extern "C" unigist_status unigist_cache_update_ragged(const void* kc_in, const void* vc_in, const int* s_old,
                                                      const int* t_old, int cap_in, const void* k_new,
                                                      const void* v_new, const int* n_new, int new_rows, void* kc_out,
                                                      void* vc_out, const int* s_new, int cap_out, int* rows_out, int B,
                                                      int Hkv, int D, int r, int sinks, unigist_dtype dt,
                                                      void* hip_stream) {
    if (B < 1 || Hkv < 1 || D < 1 || r < 1 || sinks < 0 || new_rows < 0 || cap_in < 0 || cap_out < 1) return UNIGIST_EINVAL;
    if (dt != UNIGIST_BF16 && dt != UNIGIST_F32 && dt != UNIGIST_E4M3) return UNIGIST_EUNSUPPORTED;
    if (!head_dim_ok(D, dt)) return UNIGIST_EUNSUPPORTED;
    if (B > 65535 || Hkv > 65535) return UNIGIST_EUNSUPPORTED;
    if (!kc_out || !vc_out || !s_old || !t_old || !n_new || !s_new || !rows_out) return UNIGIST_EINVAL;
    if (cap_in > 0 && (!kc_in || !vc_in)) return UNIGIST_EINVAL;
    if (new_rows > 0 && (!k_new || !v_new)) return UNIGIST_EINVAL;
    const int rp1 = r >= kMaxL ? kMaxL + 1 : r + 1;
    hipError_t e = launch_cache_update_ragged(kc_in, vc_in, s_old, t_old, cap_in, k_new, v_new, n_new, new_rows, kc_out,
                                              vc_out, s_new, cap_out, rows_out, B, Hkv, D, rp1,
                                              sinks > kMaxL ? kMaxL : sinks,
                                              dt == UNIGIST_E4M3 ? 1 : dt == UNIGIST_BF16 ? 2 : 4, kMaxL,
                                              (hipStream_t)hip_stream);
    return e == hipSuccess ? UNIGIST_OK : UNIGIST_ELAUNCH;
}

// ---------------------------------------------------------------- ring layout for token-by-token decoding
namespace {
unigist_status check_ring(int B, int Hkv, int D, int r, int W, int sinks, int window_mode, unigist_dtype dt) {
    if (B < 1 || Hkv < 1 || D < 1 || r < 1 || W < 1 || sinks < 0) return UNIGIST_EINVAL;
    if (window_mode != UNIGIST_WINDOW_SLIDING && window_mode != UNIGIST_WINDOW_UNITS) return UNIGIST_EINVAL;
    if (dt != UNIGIST_BF16 && dt != UNIGIST_F32 && dt != UNIGIST_E4M3) return UNIGIST_EUNSUPPORTED;
    if (!head_dim_ok(D, dt)) return UNIGIST_EUNSUPPORTED;
    if (B > 65535 || Hkv > 65535) return UNIGIST_EUNSUPPORTED;
    return UNIGIST_OK;
}
int dt_bytes(unigist_dtype dt) { return dt == UNIGIST_E4M3 ? 1 : dt == UNIGIST_BF16 ? 2 : 4; }
}  // namespace

extern "C" int unigist_cache_ring_rows(int t, int r, int W, int sinks, int window_mode) {
    if (t < -1 || r < 1 || W < 1 || sinks < 0) return -1;
    if (window_mode != UNIGIST_WINDOW_SLIDING && window_mode != UNIGIST_WINDOW_UNITS) return -1;
    if (window_mode == UNIGIST_WINDOW_SLIDING) {
        const long long left = (long long)t - W + 1 > 0 ? (long long)t - W + 1 : 0;  // positions that have left the window
        const long long far = left <= sinks ? left : sinks + (left - sinks) / ((long long)r + 1);
        return (int)((t + 1 < W ? t + 1 : W) + far);
    }
    if (t < sinks) return t + 1;
    const long long u = (long long)r + 1, kc = (t - sinks) / u, c = (t - sinks) % u + 1;
    // the sinks, the gists of the units left of the window, W complete units, the positions of the current unit
    return kc <= W ? t + 1 : (int)(sinks + (kc - W) + W * u + c);
}

static unigist_status ring_convert(bool to_ring, const void* kc_in, const void* vc_in, const int* s, const int* t,
                                   int cap_in, void* kc_out, void* vc_out, int cap_out, int* rows_out, int B, int Hkv,
                                   int D, int r, int W, int sinks, int window_mode, unigist_dtype dt, void* hip_stream) {
    unigist_status st = check_ring(B, Hkv, D, r, W, sinks, window_mode, dt);
    if (st != UNIGIST_OK) return st;
    if (cap_in < 1 || cap_out < 1) return UNIGIST_EINVAL;
    if (!kc_in || !vc_in || !kc_out || !vc_out || !s || !t || !rows_out) return UNIGIST_EINVAL;
    hipError_t e = launch_cache_ring_convert(to_ring, kc_in, vc_in, s, t, cap_in, kc_out, vc_out, cap_out, rows_out, B, Hkv,
                                             D, r >= kMaxL ? kMaxL + 1 : r + 1, sinks > kMaxL ? kMaxL : sinks,
                                             W > kMaxL ? kMaxL : W, window_mode == UNIGIST_WINDOW_UNITS, dt_bytes(dt),
                                             kMaxL, (hipStream_t)hip_stream);
    return e == hipSuccess ? UNIGIST_OK : UNIGIST_ELAUNCH;
}

extern "C" unigist_status unigist_cache_to_ring(const void* kc_in, const void* vc_in, const int* s, const int* t,
                                                int cap_in, void* kc_out, void* vc_out, int cap_out, int* rows_out,
                                                int B, int Hkv, int D, int r, int W, int sinks, int window_mode,
                                                unigist_dtype dt, void* hip_stream) {
    return ring_convert(true, kc_in, vc_in, s, t, cap_in, kc_out, vc_out, cap_out, rows_out, B, Hkv, D, r, W, sinks,
                        window_mode, dt, hip_stream);
}

extern "C" unigist_status unigist_cache_from_ring(const void* kc_in, const void* vc_in, const int* s, const int* t,
                                                  int cap_in, void* kc_out, void* vc_out, int cap_out, int* rows_out,
                                                  int B, int Hkv, int D, int r, int W, int sinks, int window_mode,
                                                  unigist_dtype dt, void* hip_stream) {
    return ring_convert(false, kc_in, vc_in, s, t, cap_in, kc_out, vc_out, cap_out, rows_out, B, Hkv, D, r, W, sinks,
                        window_mode, dt, hip_stream);
}

extern "C" unigist_status unigist_cache_ring_append(void* kc, void* vc, const void* k_new, const void* v_new,
                                                    int new_rows, const int* t_old, const int* n_new, int cap,
                                                    int* rows_out, int B, int Hkv, int D, int r, int W, int sinks,
                                                    int window_mode, unigist_dtype dt, void* hip_stream) {
    unigist_status st = check_ring(B, Hkv, D, r, W, sinks, window_mode, dt);
    if (st != UNIGIST_OK) return st;
    if (cap < 1 || new_rows < 1) return UNIGIST_EINVAL;
    if (!kc || !vc || !k_new || !v_new || !t_old || !n_new || !rows_out) return UNIGIST_EINVAL;
    hipError_t e = launch_cache_ring_append(kc, vc, k_new, v_new, new_rows, t_old, n_new, cap, rows_out, B, Hkv, D,
                                            r >= kMaxL ? kMaxL + 1 : r + 1, sinks > kMaxL ? kMaxL : sinks,
                                            W > kMaxL ? kMaxL : W, window_mode == UNIGIST_WINDOW_UNITS, dt_bytes(dt), kMaxL,
                                            (hipStream_t)hip_stream);
    return e == hipSuccess ? UNIGIST_OK : UNIGIST_ELAUNCH;
}

extern "C" unigist_status unigist_prefill_chunk(const void* q, const void* kc, const void* vc, void* out, float* lse,
                                                int B, int Hq, int Hkv, int C, int D, int r, int W, int p0, int s,
                                                int cap, unigist_dtype dt, void* hip_stream) {
    return unigist_prefill_chunk_ex(q, kc, vc, out, lse, B, Hq, Hkv, C, D, r, W, 0, UNIGIST_WINDOW_SLIDING, p0, s, cap,
                                    dt, hip_stream);
}

extern "C" unigist_status unigist_prefill_chunk_ex(const void* q, const void* kc, const void* vc, void* out,
                                                   float* lse, int B, int Hq, int Hkv, int C, int D, int r, int W,
                                                   int sinks, int window_mode, int p0, int s, int cap,
                                                   unigist_dtype dt, void* hip_stream) {
    return unigist_prefill_chunk_view(q, kc, vc, out, lse, B, Hq, Hkv, C, C, D, r, W, sinks, window_mode, p0, s, cap, dt,
                                      hip_stream);
}

namespace {
unigist_status prefill_impl(const void* q, const void* kc, const void* vc, void* out, float* lse, int B, int Hq, int Hkv,
                            int C, int q_rows, int D, int r, int W, int sinks, int window_mode, int p0, int s, int cap,
                            long long q_bs, long long q_hs, long long q_rs, unigist_dtype dt, void* hip_stream);
}

extern "C" unigist_status unigist_prefill_chunk_view(const void* q, const void* kc, const void* vc, void* out,
                                                     float* lse, int B, int Hq, int Hkv, int C, int q_rows, int D, int r,
                                                     int W, int sinks, int window_mode, int p0, int s, int cap,
                                                     unigist_dtype dt, void* hip_stream) {
    if (q_rows < C) return UNIGIST_EINVAL;
    if (q_rows > kMaxL) return UNIGIST_EUNSUPPORTED;
    return prefill_impl(q, kc, vc, out, lse, B, Hq, Hkv, C, q_rows, D, r, W, sinks, window_mode, p0, s, cap, 0, 0, 0, dt,
                        hip_stream);
}

extern "C" unigist_status unigist_prefill_chunk_strided(const void* q, const void* kc, const void* vc, void* out,
                                                        float* lse, int B, int Hq, int Hkv, int C, int D, int r, int W,
                                                        int sinks, int window_mode, int p0, int s, int cap,
                                                        long long q_batch_stride, long long q_head_stride,
                                                        long long q_row_stride, unigist_dtype dt, void* hip_stream) {
    // 16-byte vector accesses: strides in multiples of 8 elements, bases aligned; rows must not overlap
    if (q_row_stride < D || q_head_stride < 1 || q_batch_stride < 0 || q_row_stride > 0x7fffffffLL) return UNIGIST_EINVAL;
    if ((q_row_stride | q_head_stride | q_batch_stride) & 7) return UNIGIST_EINVAL;
    if (((uintptr_t)q & 15) != 0 || ((uintptr_t)out & 15) != 0) return UNIGIST_EINVAL;
    return prefill_impl(q, kc, vc, out, lse, B, Hq, Hkv, C, C, D, r, W, sinks, window_mode, p0, s, cap, q_batch_stride,
                        q_head_stride, q_row_stride, dt, hip_stream);
}

namespace {
unigist_status prefill_impl(const void* q, const void* kc, const void* vc, void* out, float* lse, int B, int Hq, int Hkv,
                            int C, int q_rows, int D, int r, int W, int sinks, int window_mode, int p0, int s, int cap,
                            long long q_bs, long long q_hs, long long q_rs, unigist_dtype dt, void* hip_stream) {
    if (C < 1 || p0 < 0 || s < 0 || cap < 1) return UNIGIST_EINVAL;
    const long long Ltot = (long long)p0 + C;
    if (Ltot > kMaxL) return UNIGIST_EUNSUPPORTED;
    unigist_status st = check_attn(B, Hq, Hkv, (int)Ltot, D, r, W, dt, sinks, window_mode);
    if (st != UNIGIST_OK) return st;
    if (dt != UNIGIST_BF16) return UNIGIST_EUNSUPPORTED;
    if (!q || !kc || !vc || !out || !lse) return UNIGIST_EINVAL;
    AttnShape sh = make_shape(B, Hq, Hkv, (int)Ltot, D, r, W, sinks, window_mode);
    // every raw token the first query may see must still be cached
    if (s > win_lo(sh, p0)) return UNIGIST_EINVAL;
    const int rows = unigist_cache_rows_ex(s, (int)Ltot - 1, r, sinks);
    if (rows < 0 || rows > cap) return UNIGIST_EINVAL;
    sh.Lq = C;
    sh.qhs = q_rows;
    sh.qpos0 = p0;
    sh.kv_rows = cap;
    sh.s0 = s;
    sh.ngb = count_always(sh, s);
    sh.q_bs = q_bs;
    sh.q_hs = q_hs;
    sh.q_rs = (int)q_rs;
    hipError_t e = launch_fwd_mfma(q, kc, vc, out, lse, sh, (hipStream_t)hip_stream);
    return e == hipSuccess ? UNIGIST_OK : UNIGIST_ELAUNCH;
}
}  // namespace

extern "C" size_t unigist_prefill_chunk_e4m3_workspace(int B, int Hkv, int D, int s, int t, int r, int sinks) {
    const int rows = unigist_cache_rows_ex(s, t, r, sinks);
    if (B < 1 || Hkv < 1 || D < 1 || rows < 0) return 0;
    return 2 * align256((size_t)B * Hkv * rows * D * 2);  // the rows in use of K and of V, widened to bf16
}

extern "C" unigist_status unigist_prefill_chunk_e4m3(const void* q, const void* kc, const void* vc,
                                                     const float* k_scale, const float* v_scale, void* out, float* lse,
                                                     int B, int Hq, int Hkv, int C, int D, int r, int W, int sinks,
                                                     int window_mode, int p0, int s, int cap, void* workspace,
                                                     size_t workspace_bytes, void* hip_stream) {
    if (C < 1 || p0 < 0 || s < 0 || cap < 1) return UNIGIST_EINVAL;
    const long long Ltot = (long long)p0 + C;
    if (Ltot > kMaxL) return UNIGIST_EUNSUPPORTED;
    unigist_status st = check_attn(B, Hq, Hkv, (int)Ltot, D, r, W, UNIGIST_BF16, sinks, window_mode);
    if (st != UNIGIST_OK) return st;
    if (!head_dim_ok(D, UNIGIST_E4M3)) return UNIGIST_EUNSUPPORTED;
    if (!q || !kc || !vc || !k_scale || !v_scale || !out || !lse || !workspace) return UNIGIST_EINVAL;
    if (((uintptr_t)kc & 15) != 0 || ((uintptr_t)vc & 15) != 0 || ((uintptr_t)workspace & 255) != 0) return UNIGIST_EINVAL;
    AttnShape sh = make_shape(B, Hq, Hkv, (int)Ltot, D, r, W, sinks, window_mode);
    if (s > win_lo(sh, p0)) return UNIGIST_EINVAL;  // every raw token the first query may see must still be cached
    const int rows = unigist_cache_rows_ex(s, (int)Ltot - 1, r, sinks);
    if (rows < 0 || rows > cap) return UNIGIST_EINVAL;
    const size_t need = unigist_prefill_chunk_e4m3_workspace(B, Hkv, D, s, (int)Ltot - 1, r, sinks);
    if (workspace_bytes < need) return UNIGIST_EINVAL;
    // the rows in use, widened (exactly) to bf16, slabs of `rows` rows; the scales go to the kernel
    char* kw = (char*)workspace;
    char* vw = kw + need / 2;
    hipStream_t stream = (hipStream_t)hip_stream;
    if (launch_widen_e4m3(kc, kw, B * Hkv, cap, rows, D, stream) != hipSuccess) return UNIGIST_ELAUNCH;
    if (launch_widen_e4m3(vc, vw, B * Hkv, cap, rows, D, stream) != hipSuccess) return UNIGIST_ELAUNCH;
    sh.Lq = C;
    sh.qhs = C;
    sh.qpos0 = p0;
    sh.kv_rows = rows;
    sh.s0 = s;
    sh.ngb = count_always(sh, s);
    sh.kscale = k_scale;
    sh.vscale = v_scale;
    hipError_t e = launch_fwd_mfma(q, kw, vw, out, lse, sh, stream);
    return e == hipSuccess ? UNIGIST_OK : UNIGIST_ELAUNCH;
}

extern "C" unigist_status unigist_prefill_chunk_ragged(const void* q, const void* kc, const void* vc, void* out,
                                                       float* lse, int B, int Hq, int Hkv, int C, int D, int r, int W,
                                                       int sinks, int window_mode, const int* p0, const int* n,
                                                       const int* s, int cap, int* rows_out, unigist_dtype dt,
                                                       void* hip_stream) {
    if (C < 1 || cap < 1) return UNIGIST_EINVAL;
    unigist_status st = check_attn(B, Hq, Hkv, kMaxL, D, r, W, dt, sinks, window_mode);
    if (st != UNIGIST_OK) return st;
    if (dt != UNIGIST_BF16) return UNIGIST_EUNSUPPORTED;
    if (C > kMaxL || cap > kMaxL) return UNIGIST_EUNSUPPORTED;
    if (!q || !kc || !vc || !out || !lse || !p0 || !n || !s || !rows_out) return UNIGIST_EINVAL;
    // the launch's shape: up to kMaxL positions per sequence; the kernel narrows it to each sequence's state
    AttnShape sh = make_shape(B, Hq, Hkv, kMaxL, D, r, W, sinks, window_mode);
    sh.Lq = C;
    sh.qhs = C;
    sh.kv_rows = cap;
    RaggedSeqs seqs;
    seqs.p0 = p0;
    seqs.n = n;
    seqs.s0 = s;
    seqs.rows = rows_out;
    hipError_t e = launch_fwd_mfma_ragged(q, kc, vc, out, lse, sh, seqs, (hipStream_t)hip_stream);
    return e == hipSuccess ? UNIGIST_OK : UNIGIST_ELAUNCH;
}

// ---------------------------------------------------------------- packed documents
namespace {

unigist_status check_docs(int Hq, int Hkv, int T, int D, int r, int W, int sinks, int window_mode, const int* cu,
                          int ndocs, unigist_dtype dt) {
    if (!cu || ndocs < 1 || T < 1) return UNIGIST_EINVAL;
    if (cu[0] != 0 || cu[ndocs] != T) return UNIGIST_EINVAL;
    for (int d = 0; d < ndocs; ++d)
        if (cu[d + 1] < cu[d]) return UNIGIST_EINVAL;
    return check_attn(1, Hq, Hkv, T, D, r, W, dt, sinks, window_mode);
}

// the document [c0, c0 + len) of a packed [H, T, D] buffer as a shape of its own
AttnShape doc_shape(int Hq, int Hkv, int T, int D, int r, int W, int sinks, int window_mode, int len) {
    AttnShape s = make_shape(1, Hq, Hkv, len, D, r, W, sinks, window_mode);
    s.qhs = T;
    s.kvhs = T;
    s.kv_rows = T;
    return s;
}

size_t elem_bytes(unigist_dtype dt) { return dt == UNIGIST_BF16 ? 2 : 4; }

// The bf16 kernels take a whole pack in one launch (launch_*_mfma_pack).  The fp32 kernels run document by
// document: the documents are independent, and a short document's kernels leave most of the chip idle, so their
// launch sequences are spread over kLanes streams: lane 0 is the caller's stream, the others are
// helper streams (default priority) created once per device and kept for the life of the process -- the only
// state this library holds.  The helpers wait for the caller's stream before their first kernel and the
// caller's stream waits for them after their last one, so to the caller the call still behaves like work
// enqueued on its stream.  If the helpers cannot be created everything goes to the caller's stream.
constexpr int kLanes = 4;

struct Lanes {
    bool tried = false, ok = false;
    hipStream_t st[kLanes - 1];
    hipEvent_t fork, join[kLanes - 1];
};
std::mutex g_lanes_mutex, g_enqueue_mutex;
Lanes g_lanes[16];  // per device ordinal

Lanes* helper_lanes() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return nullptr;
    std::lock_guard<std::mutex> lock(g_lanes_mutex);
    Lanes& l = g_lanes[dev];
    if (!l.tried) {
        l.tried = true;
        bool ok = hipEventCreateWithFlags(&l.fork, hipEventDisableTiming) == hipSuccess;
        for (int i = 0; ok && i < kLanes - 1; ++i)
            ok = hipStreamCreateWithFlags(&l.st[i], hipStreamNonBlocking) == hipSuccess &&
                 hipEventCreateWithFlags(&l.join[i], hipEventDisableTiming) == hipSuccess;
        l.ok = ok;
        if (!ok) (void)hipGetLastError();  // fall back to the caller's stream alone
    }
    return l.ok ? &l : nullptr;
}

// documents in descending length, dealt round-robin to the lanes: lane_of[d], or -1 for an empty document
int assign_lanes(const int* cu, int ndocs, int nlanes, std::vector<int>& order, std::vector<int>& lane_of) {
    order.clear();
    lane_of.assign(ndocs, -1);
    for (int d = 0; d < ndocs; ++d)
        if (cu[d + 1] > cu[d]) order.push_back(d);
    std::stable_sort(order.begin(), order.end(),
                     [&](int a, int b) { return cu[a + 1] - cu[a] > cu[b + 1] - cu[b]; });
    const int used = (int)order.size() < nlanes ? (int)order.size() : nlanes;
    for (size_t i = 0; i < order.size(); ++i) lane_of[order[i]] = (int)(i % (size_t)nlanes);
    return used;
}

// run launch(d, stream, lane) for every non-empty document, longest first; with `spread` over the lanes, joined
// back into `stream`, else all on `stream`
template <typename F>
unigist_status for_each_doc(const int* cu, int ndocs, hipStream_t stream, bool spread, F&& launch) {
    std::vector<int> order, lane_of;
    Lanes* l = spread ? helper_lanes() : nullptr;
    const int nlanes = l ? kLanes : 1;
    const int used = assign_lanes(cu, ndocs, nlanes, order, lane_of);
    // the fork and join events are shared by all calls on a device: one host thread at a time enqueues
    std::unique_lock<std::mutex> enqueue(g_enqueue_mutex, std::defer_lock);
    if (used > 1) enqueue.lock();
    if (used > 1) {
        if (hipEventRecord(l->fork, stream) != hipSuccess) return UNIGIST_ELAUNCH;
        for (int i = 1; i < used; ++i)
            if (hipStreamWaitEvent(l->st[i - 1], l->fork, 0) != hipSuccess) return UNIGIST_ELAUNCH;
    }
    unigist_status rc = UNIGIST_OK;
    for (int d : order) {
        const int lane = lane_of[d];
        if (launch(d, lane == 0 ? stream : l->st[lane - 1], lane) != hipSuccess) {
            rc = UNIGIST_ELAUNCH;
            break;
        }
    }
    for (int i = 1; i < used; ++i)  // always join, also after a failed launch
        if (hipEventRecord(l->join[i - 1], l->st[i - 1]) != hipSuccess ||
            hipStreamWaitEvent(stream, l->join[i - 1], 0) != hipSuccess)
            rc = UNIGIST_ELAUNCH;
    return rc;
}

}  // namespace

extern "C" unigist_status unigist_attn_fwd_varlen(const void* q, const void* k, const void* v, void* out, float* lse,
                                                  int Hq, int Hkv, int T, int D, int r, int W, const int* cu_seqlens,
                                                  int ndocs, unigist_dtype dt, void* hip_stream) {
    return unigist_attn_fwd_varlen_ex(q, k, v, out, lse, Hq, Hkv, T, D, r, W, 0, UNIGIST_WINDOW_SLIDING, cu_seqlens, ndocs,
                                      dt, hip_stream);
}

extern "C" unigist_status unigist_attn_fwd_varlen_ex(const void* q, const void* k, const void* v, void* out,
                                                     float* lse, int Hq, int Hkv, int T, int D, int r, int W, int sinks,
                                                     int window_mode, const int* cu_seqlens, int ndocs,
                                                     unigist_dtype dt, void* hip_stream) {
    unigist_status st = check_docs(Hq, Hkv, T, D, r, W, sinks, window_mode, cu_seqlens, ndocs, dt);
    if (st != UNIGIST_OK) return st;
    if (!q || !k || !v || !out || !lse) return UNIGIST_EINVAL;
    const size_t eb = elem_bytes(dt);
    if (dt == UNIGIST_BF16 && !plain_alu_forced()) {  // one launch, the workgroups look their document up
        const AttnShape s = doc_shape(Hq, Hkv, T, D, r, W, sinks, window_mode, T);
        return launch_fwd_mfma_pack(q, k, v, out, lse, s, cu_seqlens, ndocs, (hipStream_t)hip_stream) == hipSuccess
                   ? UNIGIST_OK
                   : UNIGIST_ELAUNCH;
    }
    return for_each_doc(cu_seqlens, ndocs, (hipStream_t)hip_stream, false, [&](int d, hipStream_t stream, int) {
        const int c0 = cu_seqlens[d], len = cu_seqlens[d + 1] - c0;
        const AttnShape s = doc_shape(Hq, Hkv, T, D, r, W, sinks, window_mode, len);
        const size_t ro = (size_t)c0 * D * eb;  // byte offset of the document's first row inside a head
        const char *qd = (const char*)q + ro, *kd = (const char*)k + ro, *vd = (const char*)v + ro;
        char* od = (char*)out + ro;
        return launch_fwd_simple(qd, kd, vd, od, lse + c0, s, dt, stream);
    });
}

extern "C" unigist_status unigist_attn_fwd_varlen_strided(const void* q, const void* k, const void* v, void* out,
                                                          float* lse, int Hq, int Hkv, int T, int D, int r, int W,
                                                          int sinks, int window_mode, const int* cu_seqlens, int ndocs,
                                                          long long q_head_stride, long long q_row_stride,
                                                          unigist_dtype dt, void* hip_stream) {
    unigist_status st = check_docs(Hq, Hkv, T, D, r, W, sinks, window_mode, cu_seqlens, ndocs, dt);
    if (st != UNIGIST_OK) return st;
    if (!q || !k || !v || !out || !lse) return UNIGIST_EINVAL;
    if ((st = check_qstrides(q, out, T, D, 0, q_head_stride, q_row_stride, dt)) != UNIGIST_OK) return st;
    AttnShape s = doc_shape(Hq, Hkv, T, D, r, W, sinks, window_mode, T);
    s.q_hs = q_head_stride;
    s.q_rs = (int)q_row_stride;
    return launch_fwd_mfma_pack(q, k, v, out, lse, s, cu_seqlens, ndocs, (hipStream_t)hip_stream) == hipSuccess
               ? UNIGIST_OK
               : UNIGIST_ELAUNCH;
}

extern "C" unigist_status unigist_attn_bwd_varlen_strided(const void* q, const void* k, const void* v, const void* out,
                                                          const float* lse, const void* dout, void* dq, void* dk,
                                                          void* dv, int Hq, int Hkv, int T, int D, int r, int W,
                                                          int sinks, int window_mode, const int* cu_seqlens, int ndocs,
                                                          long long q_head_stride, long long q_row_stride,
                                                          unigist_dtype dt, void* workspace, size_t workspace_bytes,
                                                          void* hip_stream) {
    unigist_status st = check_docs(Hq, Hkv, T, D, r, W, sinks, window_mode, cu_seqlens, ndocs, dt);
    if (st != UNIGIST_OK) return st;
    if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv || !workspace) return UNIGIST_EINVAL;
    if ((st = check_qstrides(q, out, T, D, 0, q_head_stride, q_row_stride, dt)) != UNIGIST_OK) return st;
    if ((st = check_qstrides(dout, dq, T, D, 0, q_head_stride, q_row_stride, dt)) != UNIGIST_OK) return st;
    const size_t need = unigist_attn_bwd_varlen_workspace_ex(Hq, Hkv, T, D, r, W, sinks, window_mode, cu_seqlens, ndocs, dt);
    if (workspace_bytes < need) return UNIGIST_EINVAL;
    if (((uintptr_t)workspace & 255) != 0) return UNIGIST_EINVAL;
    AttnShape s = doc_shape(Hq, Hkv, T, D, r, W, sinks, window_mode, T);
    s.q_hs = q_head_stride;
    s.q_rs = (int)q_row_stride;
    return launch_bwd_mfma_pack(q, k, v, out, lse, dout, dq, dk, dv, workspace, s, cu_seqlens, ndocs,
                                (hipStream_t)hip_stream) == hipSuccess
               ? UNIGIST_OK
               : UNIGIST_ELAUNCH;
}

extern "C" size_t unigist_attn_bwd_varlen_workspace(int Hq, int Hkv, int T, int D, int r, int W, const int* cu_seqlens,
                                                    int ndocs, unigist_dtype dt) {
    return unigist_attn_bwd_varlen_workspace_ex(Hq, Hkv, T, D, r, W, 0, UNIGIST_WINDOW_SLIDING, cu_seqlens, ndocs, dt);
}

extern "C" size_t unigist_attn_bwd_varlen_workspace_ex(int Hq, int Hkv, int T, int D, int r, int W, int sinks,
                                                       int window_mode, const int* cu_seqlens, int ndocs,
                                                       unigist_dtype dt) {
    if (check_docs(Hq, Hkv, T, D, r, W, sinks, window_mode, cu_seqlens, ndocs, dt) != UNIGIST_OK) return 0;
    // document-by-document path: one slice per lane, each large enough for the longest document that lane may get
    size_t need = 256;
    for (int d = 0; d < ndocs; ++d) {
        const int len = cu_seqlens[d + 1] - cu_seqlens[d];
        if (len == 0) continue;
        const size_t n = unigist_attn_bwd_workspace_ex(1, Hq, Hkv, len, D, r, W, sinks, window_mode, dt);
        if (n > need) need = n;
    }
    need = align256(need) * kLanes;
    if (dt == UNIGIST_BF16) {
        // single-launch path: delta and lse2 of the whole pack plus every document's gist partial sums.  The larger
        // of the two is asked for, so that the debug switch to the plain-ALU kernels needs no other buffer.
        const size_t pack = bwd_mfma_pack_workspace(doc_shape(Hq, Hkv, T, D, r, W, sinks, window_mode, T), cu_seqlens, ndocs);
        if (pack == 0) return 0;
        need = std::max(need, pack);
    }
    return need;
}

extern "C" unigist_status unigist_attn_bwd_varlen(const void* q, const void* k, const void* v, const void* out,
                                                  const float* lse, const void* dout, void* dq, void* dk, void* dv,
                                                  int Hq, int Hkv, int T, int D, int r, int W, const int* cu_seqlens,
                                                  int ndocs, unigist_dtype dt, void* workspace,
                                                  size_t workspace_bytes, void* hip_stream) {
    return unigist_attn_bwd_varlen_ex(q, k, v, out, lse, dout, dq, dk, dv, Hq, Hkv, T, D, r, W, 0, UNIGIST_WINDOW_SLIDING,
                                      cu_seqlens, ndocs, dt, workspace, workspace_bytes, hip_stream);
}

extern "C" unigist_status unigist_attn_bwd_varlen_ex(const void* q, const void* k, const void* v, const void* out,
                                                     const float* lse, const void* dout, void* dq, void* dk, void* dv,
                                                     int Hq, int Hkv, int T, int D, int r, int W, int sinks,
                                                     int window_mode, const int* cu_seqlens, int ndocs,
                                                     unigist_dtype dt, void* workspace, size_t workspace_bytes,
                                                     void* hip_stream) {
    unigist_status st = check_docs(Hq, Hkv, T, D, r, W, sinks, window_mode, cu_seqlens, ndocs, dt);
    if (st != UNIGIST_OK) return st;
    if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv || !workspace) return UNIGIST_EINVAL;
    const size_t need = unigist_attn_bwd_varlen_workspace_ex(Hq, Hkv, T, D, r, W, sinks, window_mode, cu_seqlens, ndocs, dt);
    if (workspace_bytes < need) return UNIGIST_EINVAL;
    if (((uintptr_t)workspace & 255) != 0) return UNIGIST_EINVAL;
    if (dt == UNIGIST_BF16 && !plain_alu_forced()) {  // one launch per kernel, the workgroups look their document up
        const AttnShape s = doc_shape(Hq, Hkv, T, D, r, W, sinks, window_mode, T);
        return launch_bwd_mfma_pack(q, k, v, out, lse, dout, dq, dk, dv, workspace, s, cu_seqlens, ndocs,
                                    (hipStream_t)hip_stream) == hipSuccess
                   ? UNIGIST_OK
                   : UNIGIST_ELAUNCH;
    }
    size_t slice = 256;
    for (int d = 0; d < ndocs; ++d) {
        const int len = cu_seqlens[d + 1] - cu_seqlens[d];
        if (len > 0) slice = std::max(slice, align256(unigist_attn_bwd_workspace_ex(1, Hq, Hkv, len, D, r, W, sinks, window_mode, dt)));
    }
    const size_t eb = elem_bytes(dt);
    // the documents of one lane run one after the other on its stream and share that lane's workspace slice
    return for_each_doc(cu_seqlens, ndocs, (hipStream_t)hip_stream, true, [&](int d, hipStream_t stream, int lane) {
        const int c0 = cu_seqlens[d], len = cu_seqlens[d + 1] - c0;
        const AttnShape s = doc_shape(Hq, Hkv, T, D, r, W, sinks, window_mode, len);
        const size_t ro = (size_t)c0 * D * eb;
        const char *qd = (const char*)q + ro, *kd = (const char*)k + ro, *vd = (const char*)v + ro;
        const char *od = (const char*)out + ro, *gd = (const char*)dout + ro;
        char *dqd = (char*)dq + ro, *dkd = (char*)dk + ro, *dvd = (char*)dv + ro;
        char* ws = (char*)workspace + slice * lane;
        return launch_bwd_simple(qd, kd, vd, od, lse + c0, gd, dqd, dkd, dvd, (float*)ws, s, dt, stream);
    });
}
