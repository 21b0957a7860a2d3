/*
 * libunigist -- gist-masked causal attention for AMD MI355X (gfx950).
 *
 * The operation is the sparse autoregressive attention of UniGist (Sec. 4.1):
 * the input sequence already carries one gist token after every r raw tokens
 * (Eq. 2, no sink prefix), positions are 0-based, and
 *
 *     gist(p)  <=>  (p + 1) % (r + 1) == 0
 *     vis(i,j) <=>  j <= i  and  ( gist(j)  or  i - j < W )            (Eq. 3)
 *
 * i.e. a query attends to itself, to every earlier gist and to the raw tokens
 * among the W most recent positions (sliding window counted in interleaved
 * positions).  The same rule holds for raw and gist queries.  r >= L means "no
 * gists" (pure sliding window); W >= L means full causal attention.
 *
 * Conventions common to every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *     allocates and frees no device memory, keeps no state (exceptions: the
 *     helper streams of the *_varlen calls, the scratch array of
 *     unigist_decode_noalloc and the switch of unigist_debug_force_plain_alu, see
 *     there), does not synchronise:
 *     work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and the call returns at once.
 *   - Tensors are contiguous, head-major: q, out, dout, dq are [B, Hq, L, D];
 *     k, v, dk, dv are [B, Hkv, L, D]; lse is [B, Hq, L] float.  D is innermost.
 *     Query head h reads kv head h / (Hq / Hkv).
 *   - dt selects the element type of q/k/v/out/dout/dq/dk/dv: bf16 (MFMA kernels,
 *     fp32 accumulation and softmax) or fp32 (plain-ALU debug kernels).  lse and
 *     the workspace are always fp32.
 *   - The softmax scale is 1/sqrt(D) and lse = ln sum_j exp(scale * q_i . k_j)
 *     over the visible j (natural log).
 *   - Outputs are fully overwritten; they need no initialisation.
 *   - Errors are return codes.  Nothing is launched unless UNIGIST_OK is returned,
 *     except that UNIGIST_ELAUNCH reports a HIP launch failure.
 */
#ifndef UNIGIST_H
#define UNIGIST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    UNIGIST_OK = 0,
    UNIGIST_EINVAL = 1,       /* null pointer, non-positive size, Hq % Hkv != 0, workspace too small */
    UNIGIST_EUNSUPPORTED = 2, /* head dim or dtype the kernels are not built for */
    UNIGIST_ELAUNCH = 3,      /* HIP reported an error at launch */
    UNIGIST_ESCRATCH = 4      /* unigist_decode_noalloc: the problem needs more than the built-in scratch array */
} unigist_status;

/*
 * Element types.  UNIGIST_E4M3 (one byte: E4M3 of the OCP 8-bit floating point format, bias 7, no infinities,
 * largest magnitude 448) is a storage type of the compressed cache only: unigist_quantize_e4m3 produces it, the
 * cache maintenance calls (unigist_cache_update, _ex, _ragged, unigist_cache_to_ring / _from_ring / _ring_append)
 * move it, unigist_decode_e4m3 and unigist_prefill_chunk_e4m3 read it; every other call answers
 * UNIGIST_EUNSUPPORTED to it.
 */
typedef enum { UNIGIST_BF16 = 0, UNIGIST_F32 = 1, UNIGIST_E4M3 = 2 } unigist_dtype;

/*
 * How the local window of Eq. 3 is counted (the *_ex entry points):
 *   SLIDING  the W most recent positions (i - j < W), per token;
 *   UNITS    as Sec. 4.1 words it: the gist unit that holds the query (r raw tokens and the gist closing
 *            them) plus the W previous units, counted behind the sink prefix.
 */
typedef enum { UNIGIST_WINDOW_SLIDING = 0, UNIGIST_WINDOW_UNITS = 1 } unigist_window_mode;

/* Human-readable name of a status code (static storage). */
const char* unigist_status_str(unigist_status s);

/*
 * Forward (Sec. 4.1 Eq. 3 mask, Sec. 4.2 block skipping):
 *   out_i = sum_j softmax_j(scale * q_i . k_j | vis(i,j)) v_j,   lse_i as above.
 * q, k, v: in.  out [B,Hq,L,D] (dt), lse [B,Hq,L] (float): out.
 * Requires B, Hq, Hkv, L, W >= 1, r >= 1, Hq % Hkv == 0, and a head dimension D that is a multiple of 8 with
 * 8 <= D <= 128 (every entry point; a multiple of 16 where E4M3 codes are involved), else UNIGIST_EUNSUPPORTED.  The
 * matrix-core kernels are built for D = 64 and D = 128; other head dimensions run on the next of the two with
 * the missing columns taken as zeros, i.e. at the cost of the larger one.
 */
unigist_status unigist_attn_fwd(const void* q, const void* k, const void* v, void* out, float* lse,
                                int B, int Hq, int Hkv, int L, int D, int r, int W,
                                unigist_dtype dt, void* hip_stream);

/*
 * Forward with the full layout of Sec. 4.1: `sinks` >= 0 sink tokens precede the first gist unit (Eq. 2),
 * so gist(p) <=> p >= sinks and (p - sinks + 1) % (r + 1) == 0, every sink is visible to all later
 * queries, and `window_mode` (a unigist_window_mode) selects how W is counted.  A sink query belongs to
 * no unit: in UNITS mode it sees the sinks up to itself.  sinks = 0 with SLIDING is unigist_attn_fwd.
 * Everything else as unigist_attn_fwd; a negative `sinks` or an unknown mode is UNIGIST_EINVAL.
 */
unigist_status unigist_attn_fwd_ex(const void* q, const void* k, const void* v, void* out, float* lse,
                                   int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks,
                                   int window_mode, unigist_dtype dt, void* hip_stream);

/*
 * Backward of l = sum(out * dout) through the forward above.
 * q, k, v, out, lse: the forward's inputs and outputs (in).  dout: in.
 * dq [B,Hq,L,D], dk, dv [B,Hkv,L,D] (dt): out; dk and dv are summed over the
 * Hq/Hkv query heads sharing a kv head.  No atomics are used, so results are
 * bitwise reproducible run to run.
 * workspace: device scratch of at least unigist_attn_bwd_workspace(...) bytes,
 * 256-byte aligned, contents undefined on entry and exit.
 */
unigist_status unigist_attn_bwd(const void* q, const void* k, const void* v, const void* out,
                                const float* lse, const void* dout, void* dq, void* dk, void* dv,
                                int B, int Hq, int Hkv, int L, int D, int r, int W,
                                unigist_dtype dt, void* workspace, size_t workspace_bytes,
                                void* hip_stream);

/*
 * The same backward, restricted to some of its stream-ordered stages (for per-kernel timing and
 * debugging).  `stages` is a bit mask; the stages depend on each other in this order, so a caller
 * running them one by one must keep the order and the same workspace:
 *   UNIGIST_BWD_DELTA        delta_i = dO_i . O_i                      (Sec. 4.1 softmax backward)
 *   UNIGIST_BWD_DKDV_GIST    dK/dV of the pairs whose gist lies left of the query's window phase
 *   UNIGIST_BWD_GIST_REDUCE  fixed-order sum of that phase's partial results
 *   UNIGIST_BWD_DKDV_WINDOW  dK/dV of the window phase, adds the gist phase, writes dk and dv
 *   UNIGIST_BWD_DQ           writes dq
 * unigist_attn_bwd is this call with UNIGIST_BWD_ALL.  Masks other than UNIGIST_BWD_ALL are
 * supported for bf16 only (UNIGIST_EUNSUPPORTED otherwise); stages == 0 is UNIGIST_EINVAL.
 */
enum {
    UNIGIST_BWD_DELTA = 1,
    UNIGIST_BWD_DKDV_GIST = 2,
    UNIGIST_BWD_GIST_REDUCE = 4,
    UNIGIST_BWD_DKDV_WINDOW = 8,
    UNIGIST_BWD_DQ = 16,
    UNIGIST_BWD_ALL = 31
};
unigist_status unigist_attn_bwd_stages(const void* q, const void* k, const void* v, const void* out,
                                       const float* lse, const void* dout, void* dq, void* dk, void* dv,
                                       int B, int Hq, int Hkv, int L, int D, int r, int W,
                                       unigist_dtype dt, void* workspace, size_t workspace_bytes,
                                       unsigned stages, void* hip_stream);

/* Bytes of workspace unigist_attn_bwd needs for this shape (0 on invalid arguments). */
size_t unigist_attn_bwd_workspace(int B, int Hq, int Hkv, int L, int D, int r, int W,
                                  unigist_dtype dt);

/*
 * Backward through unigist_attn_fwd_ex (Sec. 4.1 layout with `sinks` and `window_mode`, see there); the
 * other arguments, the stage mask and the workspace rules are those of unigist_attn_bwd_stages, with the
 * workspace sized by unigist_attn_bwd_workspace_ex for the same (sinks, window_mode).
 */
unigist_status unigist_attn_bwd_ex(const void* q, const void* k, const void* v, const void* out,
                                   const float* lse, const void* dout, void* dq, void* dk, void* dv,
                                   int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks,
                                   int window_mode, unigist_dtype dt, void* workspace,
                                   size_t workspace_bytes, unsigned stages, void* hip_stream);
size_t unigist_attn_bwd_workspace_ex(int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks,
                                     int window_mode, unigist_dtype dt);

/*
 * Forward and backward with explicit strides of the query-side tensors, in elements: element (b, h, i, d) of q, out,
 * dout and dq lies at b * q_batch_stride + h * q_head_stride + i * q_row_stride + d -- e.g. (L * Hq * D, D, Hq * D)
 * for [B, L, Hq, D] tensors as projection layers produce them, which then need no transposing copy (with grouped
 * queries they are the large tensors).  k, v, dk, dv and lse keep the layouts above.  Strides are multiples of 8
 * elements, q_row_stride >= D, the four tensors 16-byte aligned (UNIGIST_EINVAL otherwise), L * q_row_stride below
 * 2^31 elements (UNIGIST_EUNSUPPORTED otherwise); bf16 only.  Same kernels,
 * same arithmetic, same results as unigist_attn_fwd_ex / unigist_attn_bwd_ex; workspace from
 * unigist_attn_bwd_workspace_ex.
 */
unigist_status unigist_attn_fwd_strided(const void* q, const void* k, const void* v, void* out, float* lse,
                                        int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks, int window_mode,
                                        long long q_batch_stride, long long q_head_stride, long long q_row_stride,
                                        unigist_dtype dt, void* hip_stream);
unigist_status unigist_attn_bwd_strided(const void* q, const void* k, const void* v, const void* out,
                                        const float* lse, const void* dout, void* dq, void* dk, void* dv,
                                        int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks, int window_mode,
                                        long long q_batch_stride, long long q_head_stride, long long q_row_stride,
                                        unigist_dtype dt, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Packed documents (Sec. 5.1: several documents share one training sequence and attention never crosses a
 * document boundary).  The tensors hold T tokens per head -- q, out, dout, dq [Hq, T, D]; k, v, dk, dv
 * [Hkv, T, D]; lse [Hq, T] -- and document d occupies the rows cu_seqlens[d] .. cu_seqlens[d+1]-1.  Inside a
 * document everything is as in unigist_attn_fwd / unigist_attn_bwd with L = its length: the gist period and
 * the window restart at the document's first token.  cu_seqlens is a HOST array of ndocs + 1 ints,
 * non-decreasing, cu_seqlens[0] = 0, cu_seqlens[ndocs] = T (UNIGIST_EINVAL otherwise); it is read before the
 * call returns.  Empty documents are allowed.  The documents are independent.
 * bf16: every kernel is launched once for up to 64 documents (the document boundaries travel as a kernel
 * argument and each workgroup looks up the document it belongs to), everything on hip_stream; longer lists of
 * documents take one launch per 64.
 * fp32 (the plain-ALU debug kernels) and bf16 under unigist_debug_force_plain_alu(1): one launch sequence per document;
 * the backward spreads the documents over hip_stream and a few helper streams that the library creates once per
 * device (default priority, kept until the process ends -- the one piece of state this library holds); the
 * helpers start after everything already enqueued on hip_stream and hip_stream continues after them, so the
 * call behaves like work enqueued on hip_stream (under stream capture the helpers join the capture through
 * those events; the streams themselves are created by the first such backward call on a device, which therefore
 * has to happen outside a capture).
 * workspace: size from unigist_attn_bwd_varlen_workspace, 256-byte aligned.  bf16: two floats per (head, token)
 * plus the gist-phase partial sums of every document; fp32: one slice per stream, each sized for the longest
 * document.
 */
unigist_status unigist_attn_fwd_varlen(const void* q, const void* k, const void* v, void* out, float* lse,
                                       int Hq, int Hkv, int T, int D, int r, int W, const int* cu_seqlens,
                                       int ndocs, unigist_dtype dt, void* hip_stream);
unigist_status unigist_attn_bwd_varlen(const void* q, const void* k, const void* v, const void* out,
                                       const float* lse, const void* dout, void* dq, void* dk, void* dv,
                                       int Hq, int Hkv, int T, int D, int r, int W, const int* cu_seqlens,
                                       int ndocs, unigist_dtype dt, void* workspace, size_t workspace_bytes,
                                       void* hip_stream);
size_t unigist_attn_bwd_varlen_workspace(int Hq, int Hkv, int T, int D, int r, int W, const int* cu_seqlens,
                                         int ndocs, unigist_dtype dt);

/*
 * The same for the layout of unigist_attn_fwd_ex inside every document (Sec. 4.1 with the cross-document masking
 * of Sec. 5.1 -- the paper's training setting): each document starts with `sinks` sink tokens (a shorter document
 * is all sinks) and its window is counted per `window_mode`.  (0, UNIGIST_WINDOW_SLIDING) gives the calls above.
 */
unigist_status unigist_attn_fwd_varlen_ex(const void* q, const void* k, const void* v, void* out, float* lse,
                                          int Hq, int Hkv, int T, int D, int r, int W, int sinks, int window_mode,
                                          const int* cu_seqlens, int ndocs, unigist_dtype dt, void* hip_stream);
unigist_status unigist_attn_bwd_varlen_ex(const void* q, const void* k, const void* v, const void* out,
                                          const float* lse, const void* dout, void* dq, void* dk, void* dv,
                                          int Hq, int Hkv, int T, int D, int r, int W, int sinks, int window_mode,
                                          const int* cu_seqlens, int ndocs, unigist_dtype dt, void* workspace,
                                          size_t workspace_bytes, void* hip_stream);
size_t unigist_attn_bwd_varlen_workspace_ex(int Hq, int Hkv, int T, int D, int r, int W, int sinks, int window_mode,
                                            const int* cu_seqlens, int ndocs, unigist_dtype dt);

/*
 * The packed calls with explicit strides of q, out, dout, dq, as unigist_attn_fwd_strided has them: element (h, i, d)
 * lies at h * q_head_stride + i * q_row_stride + d -- (D, Hq * D) for [T, Hq, D] tensors.  k, v, dk, dv stay
 * [Hkv, T, D], lse [Hq, T]; bf16 only; workspace from unigist_attn_bwd_varlen_workspace_ex.
 */
unigist_status unigist_attn_fwd_varlen_strided(const void* q, const void* k, const void* v, void* out, float* lse,
                                               int Hq, int Hkv, int T, int D, int r, int W, int sinks, int window_mode,
                                               const int* cu_seqlens, int ndocs, long long q_head_stride,
                                               long long q_row_stride, unigist_dtype dt, void* hip_stream);
unigist_status unigist_attn_bwd_varlen_strided(const void* q, const void* k, const void* v, const void* out,
                                               const float* lse, const void* dout, void* dq, void* dk, void* dv,
                                               int Hq, int Hkv, int T, int D, int r, int W, int sinks, int window_mode,
                                               const int* cu_seqlens, int ndocs, long long q_head_stride,
                                               long long q_row_stride, unigist_dtype dt, void* workspace,
                                               size_t workspace_bytes, void* hip_stream);

/*
 * Decode over the compressed KV cache (Sec. 4.3, Fig. 4): the raw tokens that have
 * left the window were physically removed, so every cached key of a sequence is
 * visible; the order of the keys in the cache is irrelevant.
 *   q [B,Hq,D]; kcache, vcache [B,Hkv,Lk_max,D] (dt): in.
 *   seqlens: device int32 [B], number of valid keys per sequence (each in
 *            [1, Lk_max]; a sequence given 0 keys gets out = 0 and lse = -inf);
 *            NULL means Lk_max for all.
 *   out [B,Hq,D] (dt): out.  lse [B,Hq] float: out, may be NULL.
 * Split-K over the keys with a log-sum-exp combine (FlashDecoding style).
 * workspace: at least unigist_decode_workspace(...) bytes, 256-byte aligned.
 */
unigist_status unigist_decode(const void* q, const void* kcache, const void* vcache, void* out,
                              float* lse, int B, int Hq, int Hkv, int Lk_max, const int* seqlens,
                              int D, unigist_dtype dt, void* workspace, size_t workspace_bytes,
                              void* hip_stream);

size_t unigist_decode_workspace(int B, int Hq, int Hkv, int Lk_max, int D, unigist_dtype dt);

/*
 * unigist_decode for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, arithmetic and results (bit for bit) as unigist_decode,
 * without the workspace: the split-K partial results go to a fixed array of
 * UNIGIST_DECODE_NOALLOC_SCRATCH_BYTES bytes in the library's device image, which every GPU the library runs on
 * holds until the process ends (its address on the current device is looked up on the first call there; the
 * stream must belong to the current device).  The call allocates and frees nothing.
 * A problem for which unigist_decode_workspace(...) exceeds that size is refused with UNIGIST_ESCRATCH and
 * nothing is launched (the benchmark's serving shape, 64 sequences x 32 heads x 17 408 keys, needs 2.1 MB).
 * All calls on one GPU share the array: calls that may overlap there (different streams, different host threads)
 * race on it and must be ordered by the caller; calls on one stream are ordered by the stream.  Nothing of an
 * earlier call's contents is read: every slot is written before it is used.
 */
#define UNIGIST_DECODE_NOALLOC_SCRATCH_BYTES (8u << 20)
unigist_status unigist_decode_noalloc(const void* q, const void* kcache, const void* vcache, void* out,
                                      float* lse, int B, int Hq, int Hkv, int Lk_max, const int* seqlens,
                                      int D, unigist_dtype dt, void* hip_stream);
size_t unigist_decode_noalloc_scratch_bytes(void);

/*
 * The compressed cache stored in 8 bits (an extension of the decode step of Sec. 4.3, which the paper leaves
 * in the model's dtype; decode streams the cache once from HBM, so halving its bytes halves the time).
 * Storage: E4M3 codes with one positive scale per kv head for K and one for V, element = code * scale.
 *
 * unigist_quantize_e4m3: x [B, H, n, D] (dt_in = bf16 or fp32, DEVICE, 16-byte aligned) -> y, uint8 codes of the
 * same shape: x / scale[h] in binary32 (one correctly rounded division), clamped to [-448, 448], rounded to the
 * nearest E4M3 value, ties to even.  scale: DEVICE, H floats.  n may be 0.
 *
 * unigist_decode_e4m3: unigist_decode with bf16 q and out and with kcache, vcache [B, Hkv, Lk_max, D] holding
 * E4M3 codes (q, kcache, vcache 16-byte aligned), k_scale, v_scale: DEVICE, Hkv floats each.  Same workspace as unigist_decode
 * for bf16.  The cache itself is maintained by unigist_cache_update(_ex) with dt = UNIGIST_E4M3 on quantised rows.
 */
unigist_status unigist_quantize_e4m3(const void* x, void* y, const float* scale, int B, int H, int n, int D,
                                     unigist_dtype dt_in, void* hip_stream);
unigist_status unigist_decode_e4m3(const void* q, const void* kcache, const void* vcache, const float* k_scale,
                                   const float* v_scale, void* out, float* lse, int B, int Hq, int Hkv, int Lk_max,
                                   const int* seqlens, int D, void* workspace, size_t workspace_bytes,
                                   void* hip_stream);

/*
 * Compressed KV cache (Sec. 4.3, Fig. 4: raw tokens outside the local window are never attended to again
 * and can be dropped, chunk by chunk while prefilling and token by token while decoding).
 *
 * Cache layout per (batch, kv head): `cap` rows of D elements, [B, Hkv, cap, D].  In state (s, t) the first
 * floor(s / (r+1)) rows hold the gists at positions < s (gist g in row g) and the next t - s + 1 rows hold
 * the positions s .. t.  unigist_cache_rows(s, t, r) is the number of rows in use.  A query at position
 * i >= t needs s <= max(0, i - W + 1).  The empty cache is (s, t) = (0, -1).
 *
 * unigist_cache_update: state (s_old, t_old) in kc_in/vc_in plus n_new new rows k_new/v_new
 * ([B, Hkv, new_rows, D], positions t_old+1 .. t_old+n_new, n_new <= new_rows) -> state
 * (s_new, t_old + n_new) in kc_out/vc_out.  Requires 0 <= s_old <= s_new <= t_old + n_new + 1, t_old >= s_old - 1,
 * enough capacity, and out buffers that do not overlap the inputs.  kc_in/vc_in may be NULL for the empty
 * cache, k_new/v_new when n_new == 0.  A gather: bit-exact copies, any dtype (UNIGIST_E4M3 included).
 */
int unigist_cache_rows(int s, int t, int r);

/*
 * First position inside the local window of query position t (Sec. 4.1, Eq. 3): max(0, t - W + 1) for the sliding
 * window; for unit windows the first position of the unit W units before t's (t itself for a sink query).  It is
 * the state `s` a cache evicted down to what query t can see is in (0 for t = -1, the empty cache).  Host
 * function; -1 for invalid arguments.
 */
int unigist_window_start(int t, int r, int W, int sinks, int window_mode);
unigist_status unigist_cache_update(const void* kc_in, const void* vc_in, int s_old, int t_old, int cap_in,
                                    const void* k_new, const void* v_new, int n_new, int new_rows,
                                    void* kc_out, void* vc_out, int s_new, int cap_out,
                                    int B, int Hkv, int D, int r, unigist_dtype dt, void* hip_stream);

/*
 * unigist_cache_update_ex for a batch whose sequences are in different states: s_old, t_old, n_new, s_new are
 * DEVICE arrays of B ints (sequence b goes from state (s_old[b], t_old[b]) to (s_new[b], t_old[b] + n_new[b]),
 * taking its first n_new[b] <= new_rows rows of k_new/v_new [B, Hkv, new_rows, D]), so that a serving loop never
 * has to bring the states to the host.  rows_out (DEVICE, B ints, out) receives the rows in use afterwards -- the
 * `seqlens` unigist_decode takes -- or -1 for a sequence whose state violates the conditions of
 * unigist_cache_update or does not fit cap_in / cap_out; such a sequence's output rows are left untouched.  The
 * host checks only what it can see (shapes, pointers, dtype).
 */
unigist_status unigist_cache_update_ragged(const void* kc_in, const void* vc_in, const int* s_old, const int* t_old,
                                           int cap_in, const void* k_new, const void* v_new, const int* n_new,
                                           int new_rows, void* kc_out, void* vc_out, const int* s_new, int cap_out,
                                           int* rows_out, int B, int Hkv, int D, int r, int sinks, unigist_dtype dt,
                                           void* hip_stream);

/*
 * Token-by-token decoding without re-gathering the cache (Sec. 4.3: at every step one token enters the window
 * and tokens leave it; unigist_decode attends to all rows of a slab in whatever order they lie).  In ring state t
 * (the last position held) a slab holds exactly the positions visible to the query at t, in
 * unigist_cache_ring_rows(t, r, W, sinks, window_mode) rows -- the seqlens of unigist_decode for that query.
 * Layout of a slab:
 *   SLIDING: rows [0, W) hold the window, position p in row p % W; rows [W, ..) hold the sinks and gists that
 *     have left the window, in order of position.
 *   UNITS (u = r + 1 positions per unit, after `sinks` sinks; kc = the unit of position t): while kc <= W the
 *     positions 0 .. t in order; afterwards [sinks | W complete units, unit k in slot k % W, u rows each | the
 *     gists of the units 0 .. kc-W-1 | the positions of unit kc present so far].
 *   unigist_cache_to_ring / unigist_cache_from_ring convert between the ordered layout above in state (s[b], t[b])
 *     and ring state t[b] (s, t: DEVICE arrays of B ints; s[b] must be the first position of the window of the
 *     query at t[b], so that both sides hold the same positions; out buffers must not overlap the inputs).  Use
 *     to_ring after the prompt's last prefill chunk and from_ring before prefilling again.
 *   unigist_cache_ring_append, in place: every sequence with n_new[b] = 1 appends row 0 of its slab of k_new/v_new
 *     ([B, Hkv, new_rows, D]) as position t_old[b] + 1.  SLIDING: one row written, two when the position leaving
 *     the window is a sink or a gist (it moves to the far rows first).  UNITS: one row written; when a unit starts,
 *     the r + 1 rows of the unit just completed first move into the slot of the unit that leaves (whose gist is
 *     kept).  n_new[b] = 0 leaves the sequence alone.
 * rows_out (DEVICE, B ints, out): rows in use afterwards, or -1 for a sequence whose state is impossible or does
 * not fit (nothing is written for it).  Any dtype (rows are copied bit for bit).
 */
int unigist_cache_ring_rows(int t, int r, int W, int sinks, int window_mode);
unigist_status unigist_cache_to_ring(const void* kc_in, const void* vc_in, const int* s, const int* t, int cap_in,
                                     void* kc_out, void* vc_out, int cap_out, int* rows_out, int B, int Hkv, int D,
                                     int r, int W, int sinks, int window_mode, unigist_dtype dt, void* hip_stream);
unigist_status unigist_cache_from_ring(const void* kc_in, const void* vc_in, const int* s, const int* t, int cap_in,
                                       void* kc_out, void* vc_out, int cap_out, int* rows_out, int B, int Hkv, int D,
                                       int r, int W, int sinks, int window_mode, unigist_dtype dt, void* hip_stream);
unigist_status unigist_cache_ring_append(void* kc, void* vc, const void* k_new, const void* v_new, int new_rows,
                                         const int* t_old, const int* n_new, int cap, int* rows_out, int B, int Hkv,
                                         int D, int r, int W, int sinks, int window_mode, unigist_dtype dt,
                                         void* hip_stream);

/*
 * Chunk-wise prefill (Sec. 4.3: the prompt is encoded chunk by chunk with the training kernel, dropping
 * the invisible tokens after each chunk).  q holds the C query rows at positions p0 .. p0+C-1, [B, Hq, C, D];
 * kc/vc are caches in state (s, p0+C-1), i.e. already updated with the chunk's own keys, with
 * s <= max(0, p0 - W + 1).  out [B, Hq, C, D], lse [B, Hq, C]: exactly the rows p0 .. p0+C-1 of
 * unigist_attn_fwd on the whole sequence.  bf16 only (UNIGIST_EUNSUPPORTED otherwise).
 */
unigist_status unigist_prefill_chunk(const void* q, const void* kc, const void* vc, void* out, float* lse,
                                     int B, int Hq, int Hkv, int C, int D, int r, int W,
                                     int p0, int s, int cap, unigist_dtype dt, void* hip_stream);

/*
 * The same three calls for the layout of unigist_attn_fwd_ex (Sec. 4.1: `sinks` sink tokens in front, window
 * counted per `window_mode`).  The compact front of the cache then holds the sinks followed by the gists at
 * positions < s, and a query at position i needs s <= the first position of its window (for UNITS: the
 * first position of the unit W units before the one holding i; a sink query needs s <= i).  sinks = 0 with
 * SLIDING gives the calls above.
 */
int unigist_cache_rows_ex(int s, int t, int r, int sinks);
unigist_status unigist_cache_update_ex(const void* kc_in, const void* vc_in, int s_old, int t_old, int cap_in,
                                       const void* k_new, const void* v_new, int n_new, int new_rows,
                                       void* kc_out, void* vc_out, int s_new, int cap_out,
                                       int B, int Hkv, int D, int r, int sinks, unigist_dtype dt, void* hip_stream);
unigist_status unigist_prefill_chunk_ex(const void* q, const void* kc, const void* vc, void* out, float* lse,
                                        int B, int Hq, int Hkv, int C, int D, int r, int W, int sinks,
                                        int window_mode, int p0, int s, int cap, unigist_dtype dt,
                                        void* hip_stream);

/*
 * unigist_prefill_chunk_ex on a slice of larger tensors, so that the chunks of a prompt need not be copied out:
 * q and out point at the chunk's first row of every head inside tensors [B, Hq, q_rows, D] (lse: [B, Hq, q_rows]),
 * i.e. consecutive heads are q_rows >= C rows apart; only the C rows of each head are read and written.
 * q_rows = C is unigist_prefill_chunk_ex.  (The new keys of unigist_cache_update can be such a slice already:
 * pass the pointer to the chunk's first row and new_rows = the rows per head of the tensor it lies in.)
 */
unigist_status unigist_prefill_chunk_view(const void* q, const void* kc, const void* vc, void* out, float* lse,
                                          int B, int Hq, int Hkv, int C, int q_rows, int D, int r, int W, int sinks,
                                          int window_mode, int p0, int s, int cap, unigist_dtype dt,
                                          void* hip_stream);

/*
 * unigist_prefill_chunk_ex with explicit strides of q and out, in elements: element (b, h, i, d) of either lies at
 * b * q_batch_stride + h * q_head_stride + i * q_row_stride + d.  [B, C, Hq, D] tensors, as projection layers
 * produce them, are (C * Hq * D, D, Hq * D).  Strides are multiples of 8 elements, q_row_stride >= D, q and out
 * 16-byte aligned (UNIGIST_EINVAL otherwise); lse stays dense, [B, Hq, C].
 */
unigist_status unigist_prefill_chunk_strided(const void* q, const void* kc, const void* vc, void* out, float* lse,
                                             int B, int Hq, int Hkv, int C, int D, int r, int W, int sinks,
                                             int window_mode, int p0, int s, int cap, long long q_batch_stride,
                                             long long q_head_stride, long long q_row_stride, unigist_dtype dt,
                                             void* hip_stream);

/*
 * unigist_prefill_chunk_ex over a cache of E4M3 codes (as unigist_decode_e4m3 reads it: kc/vc uint8
 * [B, Hkv, cap, D], 16-byte aligned, the value of an element is its code times k_scale / v_scale of its kv head,
 * DEVICE arrays of Hkv positive floats).  q, out bf16.  The rows in use are first widened to bf16 in `workspace`
 * (exact: every E4M3 value is a bf16 value; unigist_prefill_chunk_e4m3_workspace(B, Hkv, D, s, t = p0+C-1, r,
 * sinks) bytes, 256-byte aligned), then the forward kernel runs on them with the scales applied in fp32 to the
 * scores and to the output -- the same arithmetic on the same values as unigist_decode_e4m3.  The result is the
 * rows p0 .. p0+C-1 of attention over the dequantised keys and values.
 */
size_t unigist_prefill_chunk_e4m3_workspace(int B, int Hkv, int D, int s, int t, int r, int sinks);
unigist_status unigist_prefill_chunk_e4m3(const void* q, const void* kc, const void* vc, const float* k_scale,
                                          const float* v_scale, void* out, float* lse, int B, int Hq, int Hkv, int C,
                                          int D, int r, int W, int sinks, int window_mode, int p0, int s, int cap,
                                          void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * unigist_prefill_chunk_ex for a batch whose sequences are in different states (Sec. 4.3, one launch for all of
 * them): p0, n and s are DEVICE arrays of B ints.  Sequence b has n[b] <= C query rows at positions
 * p0[b] .. p0[b]+n[b]-1, the first n[b] rows of its slab of q [B, Hq, C, D]; its slab of kc/vc [B, Hkv, cap, D] is
 * in state (s[b], p0[b]+n[b]-1), e.g. after unigist_cache_update_ragged.  The first n[b] rows of its slab of out
 * and lse are written, the others are left alone.  rows_out (DEVICE, B ints, out) receives the cache rows in use
 * -- what unigist_decode takes as seqlens -- or -1 for a sequence whose state is impossible (negative values,
 * n[b] > C, a window start s[b] right of the first position the first query sees, more rows than cap, more than
 * 2^23 positions); nothing else is written for such a sequence.  n[b] = 0 is allowed.  The host checks only what
 * it can see (shapes, pointers, dtype); bf16 only.
 */
unigist_status unigist_prefill_chunk_ragged(const void* q, const void* kc, const void* vc, void* out, float* lse,
                                            int B, int Hq, int Hkv, int C, int D, int r, int W, int sinks,
                                            int window_mode, const int* p0, const int* n, const int* s, int cap,
                                            int* rows_out, unigist_dtype dt, void* hip_stream);

/*
 * Block map (Sec. 4.2: with a fixed compression ratio the visible blocks are known in
 * closed form and need not be stored; this builder materialises them on the HOST for
 * tests and for the live-tile report, from the functions the kernels walk by).  The sequence is cut into query tiles of Bm rows
 * and key tiles of Bn columns.  Query tile t walks two disjoint phases:
 *   window phase: the contiguous key tiles win_first[t] .. win_last[t] (inclusive), pairs
 *                 inside them are subject to the full predicate vis(i,j);
 *   gist phase:   the first n_far_gists[t] gists of the sequence, taken as a compact
 *                 list (gist g sits at position (r+1)g + r), Bn per tile; every one of
 *                 them lies left of the window phase and is visible to every row of t.
 * Transposed view, for the dK/dV pass: window key tile c is visited by query tiles
 * qt_first[c] .. qt_last[c]; compact gist tile g by query tiles gist_qt_first[g] ..
 * n_qtiles-1 (== n_qtiles if none).
 * All arrays are host memory owned by the map; free with unigist_blockmap_free.
 */
typedef struct unigist_blockmap {
    int L, r, W, Bm, Bn;
    int n_qtiles;        /* ceil(L / Bm) */
    int n_ktiles;        /* ceil(L / Bn) */
    int n_gists;         /* floor(L / (r+1)) */
    int n_gtiles;        /* compact gist tiles any query tile visits */
    int* win_first;      /* [n_qtiles] */
    int* win_last;       /* [n_qtiles] */
    int* n_far_gists;    /* [n_qtiles] */
    int* n_full;         /* [n_qtiles] window tiles needing no mask */
    int* qt_first;       /* [n_ktiles] */
    int* qt_last;        /* [n_ktiles] */
    int* gist_qt_first;  /* [n_gtiles] */
    int64_t live_tiles;    /* window + gist tiles over all query tiles */
    int64_t masked_tiles;  /* of those, window tiles that need the in-tile mask */
    int64_t causal_tiles;  /* tiles a dense causal kernel would visit at the same Bm, Bn */
    int64_t n_vis;         /* visible pairs, closed form */
    int sinks;             /* sink prefix (0 for unigist_blockmap_build) */
    int window_mode;       /* unigist_window_mode */
} unigist_blockmap;

/* Requires L, W, Bm, Bn >= 1, r >= 1.  *out is set only on UNIGIST_OK. */
unigist_status unigist_blockmap_build(int L, int r, int W, int Bm, int Bn, unigist_blockmap** out);
/*
 * The same map for the layout of unigist_attn_fwd_ex.  The compact list then holds the sinks followed
 * by the gists (n_far_gists, n_gtiles and gist_qt_first count both); n_gists still counts gists only.
 */
unigist_status unigist_blockmap_build_ex(int L, int r, int W, int sinks, int window_mode, int Bm, int Bn,
                                         unigist_blockmap** out);
void unigist_blockmap_free(unigist_blockmap* m);

/*
 * The tile walks exactly as the kernels take them (Sec. 4.2: the visible blocks follow from r and W in closed form).
 * unigist_blockmap_build above and the three calls below evaluate, on the HOST, the very functions the kernels
 * call for every decision about which tiles to visit, which to skip and which need the in-tile mask, so that the
 * walks can be checked against the mask rule pair by pair without a GPU.  Step kinds: 0 = not visited (no pair of
 * it is visible), 1 = visited without mask (every pair of it is visible), 2 = visited with the in-tile mask.
 *
 * Row side (forward: 128 query rows per workgroup, 32 keys per step; dQ: 128 rows, 64 keys; a wave owns 32 rows).
 * Query tile `tile` first walks n_gist_steps steps over the first nfar entries of the compact list of sinks and
 * gists (entry c < sinks is position c, gist g is position sinks + (r+1) g + r; all of them lie left of wstart and
 * are visible to every row; only the last step can hold fewer than Bn entries, hence its mask), then
 * n_window_steps steps over the positions wstart, wstart + Bn, ... .  kind (optional, kind_capacity entries
 * available): [Bm / 32 waves][n_gist_steps + n_window_steps].
 */
typedef enum { UNIGIST_WALK_FWD = 0, UNIGIST_WALK_DQ = 1 } unigist_walk_kernel;
typedef struct unigist_row_tile_plan {
    int Bm, Bn, rows_per_wave;
    int wstart, nfar, n_gist_steps, n_window_steps;
} unigist_row_tile_plan;
unigist_status unigist_plan_row_tile(int L, int r, int W, int sinks, int window_mode, int kernel, int tile,
                                     unigist_row_tile_plan* out, int kind_capacity, signed char* kind);
/*
 * Key side (dK/dV; Sec. 4.2 applied in the transposed direction).  Query rows come in chunks of chunk_rows = 64 (two
 * blocks of 32), keys in tiles of key_tile = 128 (32 per wave).  Chunk c reaches the compact entries at positions
 * left of far(c) in the gist phase and every key from far(c) on in the window phase.  The gist phase runs one
 * workgroup per (segment of seg_chunks chunks, compact tile the segment reaches: tiles 0 .. slot0[sg+1]-slot0[sg]-1
 * for segment sg) and leaves one fp32 partial [dK^T | dV^T] block per such pair in slot slot0[sg] + tile, which a
 * reduction sums over the segments in ascending order; the window phase runs one workgroup per key tile.
 * partial_bytes / reduced_bytes: the two parts of unigist_attn_bwd_workspace_ex that hold those blocks
 * (2 * D * 128 floats each), workspace_bytes: all of it (with two floats per query row and head in front).
 */
typedef struct unigist_bwd_plan {
    int key_tile, chunk_rows;
    int n_chunks, n_key_tiles, n_gist_tiles;
    int seg_chunks, n_segs;
    int slot0[33];
    size_t partial_bytes, reduced_bytes, workspace_bytes;
} unigist_bwd_plan;
unigist_status unigist_bwd_plan_build(int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks,
                                      int window_mode, unigist_bwd_plan* out);
/*
 * One dK/dV workgroup of that plan (bf16 kernels): gist_phase != 0: compact tile `tile` of segment `seg`; else key
 * tile `tile` of the window phase (seg ignored).  c_lo .. c_hi (out): the chunks it streams, for every query head
 * of its group.  Optional, for those chunks in order (capacity = chunks the arrays can take): nfar[c] = compact
 * entries chunk c reaches in the gist phase (entry x of the tile counts for chunk c iff 128 tile + x < nfar[c]; 0 in
 * the window phase), kind: [4 waves][chunks][2 blocks of 32 rows].
 */
unigist_status unigist_plan_key_tile(int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks, int window_mode,
                                     int gist_phase, int tile, int seg, int* c_lo, int* c_hi, int capacity, int* nfar,
                                     signed char* kind);

/*
 * Launch order of the gist phase of that plan (dense bf16 launches; Sec. 4.2): workgroup `unit` (0 .. slot0[n_segs]-1
 * per batch entry and kv head) handles compact tile *tile of segment *seg.  Units that walk a whole segment come
 * first, segment-major from the last segment down; the shorter ones (tiles first reached inside their segment) come
 * last, longest first, so that the end of the launch is filled evenly.  Every (segment, tile) slot of the plan occurs
 * exactly once.  UNIGIST_EINVAL for a unit outside the plan or invalid arguments.
 */
unigist_status unigist_plan_gist_unit(int B, int Hq, int Hkv, int L, int D, int r, int W, int sinks, int window_mode,
                                      int unit, int* seg, int* tile);

/* Tile sizes the forward / backward kernels use for head dim D (for the live-tile report). */
void unigist_tile_sizes(int D, unigist_dtype dt, int* Bm, int* Bn);

/*
 * Debug switch, process-wide: with on != 0 every bf16 call of the attention entry points (forward, backward,
 * their _ex and _varlen forms) runs on the plain-ALU kernels of the fp32 build instead of the matrix-core
 * kernels -- a second, independent GPU implementation to compare against (the strided forms, which only the
 * matrix-core kernels have, then answer UNIGIST_EUNSUPPORTED).  Returns the previous setting.  The initial
 * setting is 0, or 1 if the environment variable UNIGIST_DEBUG_PLAIN_ALU=1 was set when the library was
 * loaded; the environment is not consulted afterwards.  Besides the helper streams of the *_varlen calls and the
 * scratch array of unigist_decode_noalloc this flag is the only state the library keeps.
 */
int unigist_debug_force_plain_alu(int on);

/*
 * Measurement aid, not part of the method: the bf16 matrix-core rate the chip sustains on register-resident
 * operands, against which the attention kernels' rates can be read.  `blocks` workgroups of 4 waves each run
 * `iters` rounds of 16 v_mfma_f32_16x16x32_bf16, the shape the attention kernels use (2 * 16 * 16 * 32 flops
 * each, so blocks * 4 * iters * 16 of them in all) on operands read once from `operands` (DEVICE, 32 KiB, any bf16 values: the chip is power-limited and the
 * rate depends on how many bits the operands toggle -- ones and random values give different answers).
 * clocks (DEVICE, 2 * blocks int64): per workgroup the shader-clock cycles and the ticks of the constant-rate
 * (100 MHz) counter the loop took; their ratio is the clock the chip held.  sink (DEVICE, one float) is never
 * written in practice.  The caller times the launch.  1 <= blocks <= 65536, iters >= 1, else UNIGIST_EINVAL.
 */
unigist_status unigist_probe_mfma_rate(const void* operands, long long* clocks, float* sink, int blocks, int iters,
                                       void* hip_stream);

/*
 * Measurement aid, not part of the method: a kernel that does nothing but read `bytes` bytes (a multiple of 16;
 * buf DEVICE, 16-byte aligned) with `blocks` workgroups of 256 lanes, 16 bytes per lane and load, and writes
 * nothing (sink: DEVICE, two zero-initialised 32-bit words, never written in practice).  Timed by the caller, it
 * gives the streaming-read rate the memory system delivers, the ceiling next to which the decode kernel's
 * achieved GB/s can be read.  1 <= blocks <= 65536, else UNIGIST_EINVAL.
 */
unigist_status unigist_probe_read_rate(const void* buf, size_t bytes, unsigned* sink, int blocks, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* UNIGIST_H */
