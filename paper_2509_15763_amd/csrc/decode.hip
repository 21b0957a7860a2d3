// Split-K decode over the compressed KV cache (Sec. 4.3 of the paper: after the raw
// tokens outside the window have been dropped, a new token attends to every cached
// key; the paper notes this is compatible with FlashDecoding-style split-K).
//
// The op streams K and V once from HBM: 4 flops per byte, so it is bandwidth bound.
// Three slice kernels share the workspace format and the combine kernel:
//   decode_split_mfma_kernel      bf16 queries, bf16 or E4M3 cache, query groups of up to 15 heads: contractions on
//                                 the matrix cores (described at the kernel);
//   decode_split_kernel           any dtype (the fp32 debug build) and any group size, plain vector arithmetic.
// Layout of the work of the vector kernel:
//   grid = (splits, kv heads or q heads, B), 256 threads.
//   A workgroup owns one contiguous slice of one sequence's keys for one kv head and
//   serves all G = Hq/Hkv query heads of that group from the same K/V bytes.
//   16 lanes share one key row (each holds D/16 contiguous elements, a 16-byte load
//   for bf16 D=128), so a wave covers 4 rows per load and the workgroup's 4 waves
//   cover 16 adjacent rows (4 KB contiguous for bf16 D=128).
//   Each 16-lane group keeps its own running (max, sum, acc) per query head; the 16
//   groups of a workgroup are merged through LDS and the slice's partial result goes
//   to the workspace as (m, l, acc[D]).  A second kernel merges the slices:
//   lse = ln sum_s l_s e^{m_s}, out = sum_s e^{m_s - m} acc_s / sum_s e^{m_s - m} l_s.
#include <type_traits>

#include "mfma_common.h"

namespace unigist {
namespace {

constexpr int kThreads = 256;
constexpr int kLanesPerRow = 16;
constexpr int kRowsPerIter = kThreads / kLanesPerRow;  // 16
constexpr int kUnroll = 4;

template <typename T, int E> struct RowChunk;  // E contiguous elements of a row -> float[E]
template <int E> struct RowChunk<bf16_t, E> {
    static __device__ __forceinline__ void load(const bf16_t* p, float (&x)[E]) {
        if constexpr (E == 8) {
            u32x4 r = *(const u32x4*)p;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                x[2 * t] = __uint_as_float(r[t] << 16);
                x[2 * t + 1] = __uint_as_float(r[t] & 0xffff0000u);
            }
        } else {
            u32x2 r = *(const u32x2*)p;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                x[2 * t] = __uint_as_float(r[t] << 16);
                x[2 * t + 1] = __uint_as_float(r[t] & 0xffff0000u);
            }
        }
    }
};
template <int E> struct RowChunk<float, E> {
    static __device__ __forceinline__ void load(const float* p, float (&x)[E]) {
#pragma unroll
        for (int t = 0; t < E; t += 4) {
            f32x4 r = *(const f32x4*)(p + t);
            x[t] = r[0];
            x[t + 1] = r[1];
            x[t + 2] = r[2];
            x[t + 3] = r[3];
        }
    }
};

// E4M3 codes -> float, two per v_cvt_pk_f32_fp8
template <int E> struct RowChunk<fp8_t, E> {
    static __device__ __forceinline__ void load(const fp8_t* p, float (&x)[E]) {
        uint32_t r[E / 4];
        if constexpr (E == 8) {
            u32x2 t = *(const u32x2*)p;
            r[0] = t[0];
            r[1] = t[1];
        } else {
            r[0] = *(const uint32_t*)p;
        }
#pragma unroll
        for (int t = 0; t < E / 4; ++t) {
            f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)r[t], false);
            f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)r[t], true);
            x[4 * t] = lo[0];
            x[4 * t + 1] = lo[1];
            x[4 * t + 2] = hi[0];
            x[4 * t + 3] = hi[1];
        }
    }
};

// sum over the 16 lanes of a DPP row; every lane ends with the total
__device__ __forceinline__ float row16_sum(float x) {
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xf, 0xf, false));   // quad_perm [2,3,0,1]
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xf, 0xf, false));  // row_half_mirror
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xf, 0xf, false));  // row_mirror
    return x;
}

// workspace layout per (b, hq, split): [m, l, acc[D]] floats.
// TQ: type of the queries; T: type the cache is stored in.  A cache of E4M3 codes comes with one scale per kv
// head for K and for V (element = code * scale): the K scale is folded into the query, the V scale into the
// slice's partial result.
// D is the head dimension the kernel is built for (64 or 128), Dt <= D (a multiple of 8) the one of the tensors: rows in
// memory are Dt elements long and the lanes holding columns from Dt on work on zeros; the workspace keeps D columns.
template <typename TQ, typename T, int D, int G, int U>
__global__ __launch_bounds__(kThreads) void decode_split_kernel(const TQ* __restrict__ q, const T* __restrict__ kc,
                                                               const T* __restrict__ vc, const int* __restrict__ seqlens,
                                                               const float* __restrict__ k_scale,
                                                               const float* __restrict__ v_scale,
                                                               float* __restrict__ ws, int Hq, int Hkv, int Lk,
                                                               int nsplit, float scale, int Dt) {
    constexpr int E = D / kLanesPerRow;
    const int tid = threadIdx.x;
    const int sub = tid % kLanesPerRow;  // which D/16 chunk of a row
    const int grp = tid / kLanesPerRow;  // which of the 16 rows per iteration
    const int split = blockIdx.x, b = blockIdx.z;
    // G query heads share kv head hk; with G == 1 the grid runs over query heads
    const int hq0 = blockIdx.y * G;
    const int hk = hq0 / (Hq / Hkv);
    const int n = seqlens ? min(max(seqlens[b], 0), Lk) : Lk;  // never past the sequence's slab, whatever the caller wrote
    const int per = (((n + nsplit - 1) / nsplit) + kRowsPerIter - 1) / kRowsPerIter * kRowsPerIter;
    const int k0 = split * per;
    const int k1 = min(n, k0 + per);

    float qr[G][E], acc[G][E], m[G], l[G];
    if (k_scale) scale *= k_scale[hk];
    const float vmul = v_scale ? v_scale[hk] : 1.f;
    const bool have = sub * E < Dt;  // does this lane's piece of a row exist?
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int e = 0; e < E; ++e) qr[g][e] = 0.f;
        if (have) RowChunk<TQ, E>::load(q + ((size_t)b * Hq + hq0 + g) * Dt + sub * E, qr[g]);
        m[g] = -INFINITY;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            qr[g][e] *= scale;
            acc[g][e] = 0.f;
        }
    }
    const T* kb = kc + ((size_t)b * Hkv + hk) * Lk * Dt + (have ? sub * E : 0);  // a lane without a piece re-reads
    const T* vb = vc + ((size_t)b * Hkv + hk) * Lk * Dt + (have ? sub * E : 0);  // the first one; its q is zero

    for (int base = k0; base < k1; base += kRowsPerIter * U) {
        float kx[U][E], vx[U][E];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int row = base + u * kRowsPerIter + grp;
            ok[u] = row < k1;
            int rr = ok[u] ? row : k0;  // k0 < k1 <= n whenever this loop runs: always in bounds
            RowChunk<T, E>::load(kb + (size_t)rr * Dt, kx[u]);
            RowChunk<T, E>::load(vb + (size_t)rr * Dt, vx[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float s = 0.f;
#pragma unroll
                for (int e = 0; e < E; ++e) s += qr[g][e] * kx[u][e];
                s = row16_sum(s);
                if (ok[u]) {
                    if (s > m[g]) {
                        float a = __expf(m[g] - s);
                        l[g] *= a;
#pragma unroll
                        for (int e = 0; e < E; ++e) acc[g][e] *= a;
                        m[g] = s;
                    }
                    float p = __expf(s - m[g]);
                    l[g] += p;
#pragma unroll
                    for (int e = 0; e < E; ++e) acc[g][e] += p * vx[u][e];
                }
            }
        }
    }

    // merge the 16 row groups of the workgroup
    __shared__ float sm[G][kRowsPerIter];
    __shared__ float sl[G][kRowsPerIter];
    __shared__ float sacc[G][kRowsPerIter][D];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (sub == 0) {
            sm[g][grp] = m[g];
            sl[g][grp] = l[g];
        }
#pragma unroll
        for (int e = 0; e < E; ++e) sacc[g][grp][sub * E + e] = acc[g][e];
    }
    __syncthreads();
    for (int idx = tid; idx < G * D; idx += kThreads) {
        const int g = idx / D, d = idx % D;
        float mm = -INFINITY;
#pragma unroll
        for (int t = 0; t < kRowsPerIter; ++t) mm = fmaxf(mm, sm[g][t]);
        float ll = 0.f, a = 0.f;
        if (mm > -INFINITY) {
#pragma unroll
            for (int t = 0; t < kRowsPerIter; ++t) {
                float w = __expf(sm[g][t] - mm);  // exp(-inf) = 0 for groups that saw no key
                ll += w * sl[g][t];
                a += w * sacc[g][t][d];
            }
        }
        float* o = ws + (((size_t)b * Hq + hq0 + g) * nsplit + split) * (D + 2);
        if (d == 0) {
            o[0] = mm;
            o[1] = ll;
        }
        o[2 + d] = a * vmul;
    }
}

template <typename T, int D>
__global__ __launch_bounds__(D) void decode_combine_kernel(const float* __restrict__ ws, T* __restrict__ out,
                                                          float* __restrict__ lse, int nsplit, int Dt) {
    const int bh = blockIdx.x, d = threadIdx.x;
    if (d >= Dt) return;  // columns the tensors do not have
    const float* p = ws + (size_t)bh * nsplit * (D + 2);
    float mm = -INFINITY;
    for (int s = 0; s < nsplit; ++s) mm = fmaxf(mm, p[s * (D + 2)]);
    if (mm == -INFINITY) {  // a sequence of zero keys (outside the contract): the empty sum, not NaN
        Elem<T>::store(out + (size_t)bh * Dt + d, 0.f);
        if (lse && d == 0) lse[bh] = -INFINITY;
        return;
    }
    float ll = 0.f, a = 0.f;
    for (int s = 0; s < nsplit; ++s) {
        float w = __expf(p[s * (D + 2)] - mm);
        ll += w * p[s * (D + 2) + 1];
        a += w * p[s * (D + 2) + 2 + d];
    }
    Elem<T>::store(out + (size_t)bh * Dt + d, a / ll);
    if (lse && d == 0) lse[bh] = mm + __logf(ll);
}

// ---------------------------------------------------------------------------------------------
// bf16 queries, cache in bf16 or as E4M3 codes, query groups of up to 15 heads per kv head: the contractions go to the matrix cores
// (v_mfma_f32_16x16x32_bf16; operand layouts in mfma_common.h), which are idle in this bandwidth-bound op, and the
// vector pipe is left with widening the codes (E4M3 values are exact in bf16; nothing to do for a bf16 cache) and a
// softmax over 16-key columns.
// A wave takes 32 keys per iteration, the workgroup's four waves 128:
//   S^T = K Q^T   A = K: lane (key r16, g4) loads the D/4 elements [D/4 g4, D/4 (g4+1)) of its key's row, k-step ks uses
//                 the eight at offset 8 ks (the contraction order is free as long as Q uses the same one);
//                 B = Q^T: column = query head of the group (columns >= G are zero), in registers;
//   softmax       a head is a column spread over four lanes, each holding 4 of every 16 keys; its running
//                 reference is kept identical on the four lanes and raised lazily, the row sum is a per-lane partial;
//   O^T += V^T P^T  P in place as the B operand (slot 8 g4 + 4 kb + i = key 16 kb + 4 g4 + i); V^T through LDS: the
//                 wave widens its 32 V rows to bf16 into a private swizzled tile and reads it back transposed.
// The four waves' partial (m, l, O) are merged through LDS and written to the workspace like the other kernels'.
template <int D, bool E4M3>
__global__ __launch_bounds__(kThreads) void decode_split_mfma_kernel(const bf16_t* __restrict__ q,
                                                                         const uint8_t* __restrict__ kc,
                                                                         const uint8_t* __restrict__ vc,
                                                                         const int* __restrict__ seqlens,
                                                                         const float* __restrict__ k_scale,
                                                                         const float* __restrict__ v_scale,
                                                                         float* __restrict__ ws, int Hq, int Hkv, int Lk,
                                                                         int nsplit, float scale, int Dt) {
    // Dt <= D: the head dimension of the tensors (rows of Dt elements in memory; a multiple of 8, of 16 for E4M3
    // codes); the K and Q columns from Dt on are zeros, the V columns from Dt on are never stored
    constexpr int KS = D / 32, DB = D / 16, CH = D / 8;  // k-steps, 16-row blocks of O^T, 16-byte chunks per bf16 row
    constexpr int EB = E4M3 ? 1 : 2;                     // bytes per cache element
    constexpr int BPL = D / 4;                           // K elements per lane and key
    constexpr int NKL = BPL * EB / 16;                   // 16-byte loads per lane and key for them
    constexpr int NLV = 32 * D * EB / 1024;              // 16-byte loads per lane for the wave's 32 V rows
    constexpr int LPR = D * EB / 16;                     // lanes per V row
    constexpr float kLog2e = 1.4426950408889634f;
    constexpr float kSlack = 8.f;                        // the reference is raised when a score exceeds it by 2^kSlack
    __shared__ __attribute__((aligned(1024))) char smem[4 * 32 * D * 2];  // per wave: 32 rows of D bf16

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r16 = lane & 15, g4 = lane >> 4;
    const int G = Hq / Hkv;  // <= 15: the merge buffer below holds 4 G (D + 2) floats
    const int split = blockIdx.x, b = blockIdx.z, hk = blockIdx.y, hq0 = hk * G;
    const int n = seqlens ? min(max(seqlens[b], 0), Lk) : Lk;  // never past the sequence's slab, whatever the caller wrote
    const int per = (((n + nsplit - 1) / nsplit) + 127) / 128 * 128;
    const int k0 = split * per;
    const int k1 = min(n, k0 + per);
    const float c = scale * (E4M3 ? k_scale[hk] : 1.f) * kLog2e;  // exp(x) = exp2(x log2 e); the K scale rides along

    // B operand Q^T: lane (column r16 = head of the group, g4) holds Q[head][BPL g4 + 8 ks .. +7]
    bf16x8 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        u32x4 z = {0u, 0u, 0u, 0u};
        if (r16 < G && BPL * g4 + 8 * ks < Dt) z = *(const u32x4*)(q + ((size_t)b * Hq + hq0 + r16) * Dt + BPL * g4 + 8 * ks);
        qf[ks] = __builtin_bit_cast(bf16x8, z);
    }
    f32x4 o[DB];  // O^T: register i of o[db] is d = 16 db + 4 g4 + i, column = head r16
#pragma unroll
    for (int db = 0; db < DB; ++db) o[db] = zero4();
    float m = -INFINITY, l = 0.f;

    const uint8_t* kb = kc + ((size_t)b * Hkv + hk) * Lk * (Dt * EB);
    const uint8_t* vb = vc + ((size_t)b * Hkv + hk) * Lk * (Dt * EB);
    const int row_bytes = Dt * EB;
    char* vt = smem + w * (32 * D * 2);
    int toff[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) toff[db] = tr16_lane_off16<CH>(db);
    // where this lane's V loads go in the tile: load j covers row (64 / LPR) j + lane / LPR and 16 bytes of it -- 16
    // codes, i.e. the bf16 chunks 2 (lane % LPR) and 2 (lane % LPR) + 1 of that row, or the bf16 chunk lane % LPR itself
    constexpr int NVW = E4M3 ? 2 : 1;
    int vwoff[NLV][NVW];
#pragma unroll
    for (int j = 0; j < NLV; ++j) {
        const int row = (64 / LPR) * j + lane / LPR;
#pragma unroll
        for (int t = 0; t < NVW; ++t)
            vwoff[j][t] = row * (CH * 16) + (((NVW * (lane % LPR) + t) ^ swz16<CH>(row)) << 4);
    }

    for (int base = k0 + 32 * w; base < k1; base += 128) {
        // ---- loads: K rows base + 16 kb + r16 (clamped into the slice: clamped keys are masked below), V rows likewise
        u32x4 kw[2][NKL], vw[NLV];
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2) {
            const int row = min(base + 16 * kb2 + r16, k1 - 1);
#pragma unroll
            for (int t = 0; t < NKL; ++t) {
                const int o = BPL * EB * g4 + 16 * t;  // a piece the rows do not have: the first one (its q is zero)
                kw[kb2][t] = *(const u32x4*)(kb + (size_t)row * row_bytes + (o < row_bytes ? o : 0));
            }
        }
#pragma unroll
        for (int j = 0; j < NLV; ++j) {
            const int row = min(base + (64 / LPR) * j + lane / LPR, k1 - 1);
            const int o = 16 * (lane % LPR);
            vw[j] = *(const u32x4*)(vb + (size_t)row * row_bytes + (o < row_bytes ? o : 0));
        }
        // ---- S^T = K Q^T
        f32x4 sa[2];
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2) {
            sa[kb2] = zero4();
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                u32x4 kf;
                if constexpr (E4M3) {
                    const uint32_t w0 = kw[kb2][ks / 2][2 * (ks % 2)], w1 = kw[kb2][ks / 2][2 * (ks % 2) + 1];
                    const f32x2 a0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w0, false), a1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w0, true);
                    const f32x2 a2 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w1, false), a3 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w1, true);
                    kf[0] = pack_bf16x2(a0[0], a0[1]);
                    kf[1] = pack_bf16x2(a1[0], a1[1]);
                    kf[2] = pack_bf16x2(a2[0], a2[1]);
                    kf[3] = pack_bf16x2(a3[0], a3[1]);
                } else {
                    kf = kw[kb2][ks];
                }
                sa[kb2] = mfma16(__builtin_bit_cast(bf16x8, kf), qf[ks], sa[kb2]);
            }
        }
        // ---- V rows (widened to bf16) into the wave's tile
#pragma unroll
        for (int j = 0; j < NLV; ++j) {
            if constexpr (!E4M3) {
                *(u32x4*)(vt + vwoff[j][0]) = vw[j];
                continue;
            }
#pragma unroll
            for (int t = 0; t < NVW; ++t) {
                const uint32_t w0 = vw[j][2 * t], w1 = vw[j][2 * t + 1];
                const f32x2 a0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w0, false), a1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w0, true);
                const f32x2 a2 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w1, false), a3 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w1, true);
                u32x4 x;
                x[0] = pack_bf16x2(a0[0], a0[1]);
                x[1] = pack_bf16x2(a1[0], a1[1]);
                x[2] = pack_bf16x2(a2[0], a2[1]);
                x[3] = pack_bf16x2(a3[0], a3[1]);
                *(u32x4*)(vt + vwoff[j][t]) = x;
            }
        }
        // ---- softmax over the 32 keys; keys past the slice are masked
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (base + 16 * kb2 + 4 * g4 + i >= k1) sa[kb2][i] = -INFINITY;
        float mx = fmaxf(fmaxf(fmaxf(sa[0][0], sa[0][1]), fmaxf(sa[0][2], sa[0][3])),
                         fmaxf(fmaxf(sa[1][0], sa[1][1]), fmaxf(sa[1][2], sa[1][3])));
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        if ((mx - m) * c > kSlack || m == -INFINITY) {  // same decision on the four lanes of a head (same mx, same m)
            if (mx > m) {
                const float alpha = __builtin_amdgcn_exp2f((m - mx) * c);  // m = -inf gives 0
                l *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i = 0; i < 4; ++i) o[db][i] *= alpha;
                m = mx;
            }
        }
        const float mc = (m == -INFINITY ? 0.f : m) * c;
        float p[8];
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
            for (int i = 0; i < 4; ++i) p[4 * kb2 + i] = __builtin_amdgcn_exp2f(fmaf(sa[kb2][i], c, -mc));
        l += ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
        u32x4 pk;
#pragma unroll
        for (int t = 0; t < 4; ++t) pk[t] = pack_bf16x2(p[2 * t], p[2 * t + 1]);
        // ---- O^T += V^T P^T (the tile writes above are this wave's own: LDS operations of a wave complete in order)
#pragma unroll
        for (int db = 0; db < DB; ++db) o[db] = mfma16(tr16_frag16<CH>(vt + toff[db], 0), __builtin_bit_cast(bf16x8, pk), o[db]);
    }

    // ---- merge the four waves (the tiles are dead: their memory takes the partials)
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    __syncthreads();
    float* pm = (float*)smem;              // [4 waves][G]
    float* pl = pm + 4 * G;                // [4 waves][G]
    float* po = pl + 4 * G;                // [4 waves][G][D]
    if (r16 < G) {
        if (g4 == 0) {
            pm[w * G + r16] = m;
            pl[w * G + r16] = l;
        }
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 4; ++i) po[((size_t)w * G + r16) * D + 16 * db + 4 * g4 + i] = o[db][i];
    }
    __syncthreads();
    const float vmul = E4M3 ? v_scale[hk] : 1.f;
    const float ln2 = 0.6931471805599453f;
    for (int idx = tid; idx < G * D; idx += kThreads) {
        const int g = idx / D, d = idx % D;
        float mm = -INFINITY;
#pragma unroll
        for (int t = 0; t < 4; ++t) mm = fmaxf(mm, pm[t * G + g]);
        float ll = 0.f, a = 0.f;
        if (mm > -INFINITY) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float wgt = __builtin_amdgcn_exp2f((pm[t * G + g] - mm) * c);  // exp2(-inf) = 0 for a wave that saw no key
                ll += wgt * pl[t * G + g];
                a += wgt * po[((size_t)t * G + g) * D + d];
            }
        }
        float* outp = ws + (((size_t)b * Hq + hq0 + g) * nsplit + split) * (D + 2);
        if (d == 0) {
            outp[0] = mm * c * ln2;  // the other kernels keep m in natural-log units of the scaled score
            outp[1] = ll;
        }
        outp[2 + d] = a * vmul;
    }
}

template <typename TQ, typename T, int D>
hipError_t decode_launch(const void* q, const void* kc, const void* vc, const float* k_scale, const float* v_scale,
                         void* out, float* lse, int B, int Hq, int Hkv, int Lk, const int* seqlens, int Dt, float* ws,
                         hipStream_t st) {
    constexpr int U = kUnroll;
    constexpr unigist_dtype dt = std::is_same<TQ, float>::value ? UNIGIST_F32 : UNIGIST_BF16;
    const int nsplit = decode_num_splits(B, Hq, Hkv, Lk, dt);
    const float scale = 1.0f / sqrtf((float)Dt);
    if (decode_grouped(Hq, Hkv, dt) && Hq / Hkv == 4) {
        dim3 grid(nsplit, Hkv, B);
        decode_split_kernel<TQ, T, D, 4, U><<<grid, kThreads, 0, st>>>((const TQ*)q, (const T*)kc, (const T*)vc, seqlens,
                                                                       k_scale, v_scale, ws, Hq, Hkv, Lk, nsplit, scale, Dt);
    } else {
        dim3 grid(nsplit, Hq, B);
        decode_split_kernel<TQ, T, D, 1, U><<<grid, kThreads, 0, st>>>((const TQ*)q, (const T*)kc, (const T*)vc, seqlens,
                                                                       k_scale, v_scale, ws, Hq, Hkv, Lk, nsplit, scale, Dt);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    decode_combine_kernel<TQ, D><<<B * Hq, D, 0, st>>>(ws, (TQ*)out, lse, nsplit, Dt);
    return hipGetLastError();
}

}  // namespace

// Does one workgroup serve all query heads of a kv head?  The matrix-core kernel takes groups of up to 15 heads
// (bf16 queries); the vector kernel, which the fp32 build uses, shares the K/V bytes for groups of 4 only.
bool decode_grouped(int Hq, int Hkv, unigist_dtype dt) {
    const int G = Hq / Hkv;
    return dt == UNIGIST_F32 ? G == 4 : G <= 15;
}

// Slices per sequence.  The slice kernel saturates HBM with one workgroup per CU, so the time of a launch goes
// with the number of rounds of 256 workgroups times the slice length: the split is chosen to fill whole rounds
// (a batch of 48 sequences x 8 kv heads = 384 workgroups would leave half of the second round idle), with a
// small price per slice for the partial results the combine kernel has to merge, and never slices shorter than
// 256 keys.  Measured on batches of 1 to 256 sequences: one round is best up to 64 (sequence, head) units, two up
// to 256 units, four beyond.
int decode_num_splits(int B, int Hq, int Hkv, int Lk, unigist_dtype dt) {
    const long units = (long)B * (decode_grouped(Hq, Hkv, dt) ? Hkv : Hq);
    const long target = units <= 64 ? 256 : units <= 256 ? 512 : 1024;
    long nmax = (target + units - 1) / units;
    if (nmax < 4) nmax = 4;
    if (nmax > 64) nmax = 64;
    const long cap = (Lk + 255) / 256;
    if (nmax > cap) nmax = cap;
    if (nmax < 1) nmax = 1;
    int best = 1;
    double best_cost = 1e30;
    for (long n = 1; n <= nmax; ++n) {
        const long wgs = units * n;
        double cost = (double)((wgs + 255) / 256 * 256) / (double)wgs * (1.0 + 0.01 * (double)n);
        if (wgs < target) cost *= 1.05;
        if (cost < best_cost) {
            best_cost = cost;
            best = (int)n;
        }
    }
    return best;
}

namespace {
// bf16 queries over a bf16 or E4M3 cache: the matrix-core kernel when the group fits its columns, else one
// workgroup per query head with the vector kernel
template <bool E4M3>
hipError_t decode_bf16q(const void* q, const void* kc, const void* vc, const float* k_scale, const float* v_scale, void* out,
                        float* lse, int B, int Hq, int Hkv, int Lk, const int* seqlens, int D, float* ws, hipStream_t st) {
    if (!decode_grouped(Hq, Hkv, UNIGIST_BF16)) {
        using T = std::conditional_t<E4M3, fp8_t, bf16_t>;
        return D <= 64 ? decode_launch<bf16_t, T, 64>(q, kc, vc, k_scale, v_scale, out, lse, B, Hq, Hkv, Lk, seqlens, D, ws, st)
                       : decode_launch<bf16_t, T, 128>(q, kc, vc, k_scale, v_scale, out, lse, B, Hq, Hkv, Lk, seqlens, D, ws, st);
    }
    const int nsplit = decode_num_splits(B, Hq, Hkv, Lk, UNIGIST_BF16);
    const float scale = 1.0f / sqrtf((float)D);
    const dim3 grid(nsplit, Hkv, B);
    if (D <= 64)
        decode_split_mfma_kernel<64, E4M3><<<grid, kThreads, 0, st>>>((const bf16_t*)q, (const uint8_t*)kc, (const uint8_t*)vc,
                                                                      seqlens, k_scale, v_scale, ws, Hq, Hkv, Lk, nsplit, scale, D);
    else
        decode_split_mfma_kernel<128, E4M3><<<grid, kThreads, 0, st>>>((const bf16_t*)q, (const uint8_t*)kc, (const uint8_t*)vc,
                                                                       seqlens, k_scale, v_scale, ws, Hq, Hkv, Lk, nsplit, scale, D);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (D <= 64) decode_combine_kernel<bf16_t, 64><<<B * Hq, 64, 0, st>>>(ws, (bf16_t*)out, lse, nsplit, D);
    else decode_combine_kernel<bf16_t, 128><<<B * Hq, 128, 0, st>>>(ws, (bf16_t*)out, lse, nsplit, D);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_decode(const void* q, const void* kc, const void* vc, void* out, float* lse, int B, int Hq,
                         int Hkv, int Lk, const int* seqlens, int D, unigist_dtype dt, float* ws, hipStream_t st) {
    if (dt == UNIGIST_F32)
        return D <= 64 ? decode_launch<float, float, 64>(q, kc, vc, nullptr, nullptr, out, lse, B, Hq, Hkv, Lk, seqlens, D, ws, st)
                       : decode_launch<float, float, 128>(q, kc, vc, nullptr, nullptr, out, lse, B, Hq, Hkv, Lk, seqlens, D, ws, st);
    return decode_bf16q<false>(q, kc, vc, nullptr, nullptr, out, lse, B, Hq, Hkv, Lk, seqlens, D, ws, st);
}

hipError_t launch_decode_fp8(const void* q, const void* kc, const void* vc, const float* k_scale, const float* v_scale,
                             void* out, float* lse, int B, int Hq, int Hkv, int Lk, const int* seqlens, int D,
                             float* ws, hipStream_t st) {
    return decode_bf16q<true>(q, kc, vc, k_scale, v_scale, out, lse, B, Hq, Hkv, Lk, seqlens, D, ws, st);
}

// ---------------------------------------------------------------------------------------------
// Quantisation of new cache rows: y = e4m3(clamp(x / scale[head], -448, 448)), one correctly rounded binary32
// division per element, conversion by v_cvt_pk_fp8_f32 (round to nearest even).  16 elements per lane.
namespace {
template <typename T>
__global__ __launch_bounds__(256) void quantize_e4m3_kernel(const T* __restrict__ x, uint8_t* __restrict__ y,
                                                           const float* __restrict__ scale, int H, long per_head,
                                                           long nchunks) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nchunks) return;
    const long e0 = idx * 16;
    const float c = scale[(e0 / per_head) % H];
    float f[2][8];
    RowChunk<T, 8>::load(x + e0, f[0]);
    RowChunk<T, 8>::load(x + e0 + 8, f[1]);
    u32x4 w;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        float g[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float q = __fdiv_rn(f[t / 2][4 * (t % 2) + i], c);
            g[i] = q != q ? q : fminf(fmaxf(q, -448.f), 448.f);
        }
        int p = 0;
        p = __builtin_amdgcn_cvt_pk_fp8_f32(g[0], g[1], p, false);
        p = __builtin_amdgcn_cvt_pk_fp8_f32(g[2], g[3], p, true);
        w[t] = (uint32_t)p;
    }
    *(u32x4*)(y + e0) = w;
}
// E4M3 codes -> the same values in bf16 (exact: 3 mantissa bits, exponents well inside bf16's), 16 per lane.
// Lane idx covers the elements 16 idx .. 16 idx + 15 of the output, whose slabs hold `rows` of the input slab's `cap` rows.
__global__ __launch_bounds__(256) void widen_e4m3_kernel(const uint8_t* __restrict__ x, bf16_t* __restrict__ y,
                                                        long per_slab_out, long per_slab_in, long nchunks) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nchunks) return;
    const long e0 = idx * 16;
    const long slab = e0 / per_slab_out, within = e0 % per_slab_out;
    const u32x4 w = *(const u32x4*)(x + slab * per_slab_in + within);
    u32x4 lo, hi;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[t], false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[t], true);
        const uint32_t p0 = pack_bf16x2(a[0], a[1]), p1 = pack_bf16x2(b[0], b[1]);
        if (t < 2) {
            lo[2 * t] = p0;
            lo[2 * t + 1] = p1;
        } else {
            hi[2 * (t - 2)] = p0;
            hi[2 * (t - 2) + 1] = p1;
        }
    }
    *(u32x4*)(y + e0) = lo;
    *(u32x4*)(y + e0 + 8) = hi;
}
}  // namespace

hipError_t launch_widen_e4m3(const void* codes, void* y, int BH, int cap, int rows, int D, hipStream_t st) {
    const long per_out = (long)rows * D, per_in = (long)cap * D;
    const long nchunks = (long)BH * per_out / 16;
    if (nchunks <= 0) return hipSuccess;
    const long blocks = (nchunks + 255) / 256;
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    widen_e4m3_kernel<<<dim3((unsigned)blocks), 256, 0, st>>>((const uint8_t*)codes, (bf16_t*)y, per_out, per_in, nchunks);
    return hipGetLastError();
}

hipError_t launch_quantize_e4m3(const void* x, void* y, const float* scale, int B, int H, int n, int D,
                                unigist_dtype dt_in, hipStream_t st) {
    const long per_head = (long)n * D;
    const long nchunks = (long)B * H * per_head / 16;
    if (nchunks <= 0) return hipSuccess;
    const long blocks = (nchunks + 255) / 256;
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    if (dt_in == UNIGIST_F32)
        quantize_e4m3_kernel<float><<<dim3((unsigned)blocks), 256, 0, st>>>((const float*)x, (uint8_t*)y, scale, H, per_head, nchunks);
    else
        quantize_e4m3_kernel<bf16_t><<<dim3((unsigned)blocks), 256, 0, st>>>((const bf16_t*)x, (uint8_t*)y, scale, H, per_head, nchunks);
    return hipGetLastError();
}

}  // namespace unigist
