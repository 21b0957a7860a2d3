// Plain-ALU kernels for gist-masked attention: the fp32 debug build of the library.
//
// One thread owns one query row (forward, dQ) or one key row (dK/dV) and walks the
// rows on the other side one at a time.  The 64 lanes of a wave walk in lockstep
// over the union of their ranges, so every K/V (or Q/dO) row is fetched with a
// wave-uniform address, and apply the visibility rule of Sec. 4.1, Eq. 3 per pair.
// No tiles, no MFMA, fp32 accumulation throughout; slow, but short enough to
// check by eye.  The bf16 instantiations exist so that the MFMA kernels can be
// cross-checked against them on the GPU.  D is the head dimension a kernel is built for
// (64 or 128); the tensors' head dimension s.D may be anything up to it: rows in memory are
// s.D elements long and the loops over d skip the rest.
#include "common.h"

namespace unigist {
namespace {

constexpr int kRows = 64;  // rows per workgroup == one wave

template <typename T, int D>
__device__ __forceinline__ void load_row(const T* __restrict__ p, float (&x)[D]) {
#pragma unroll
    for (int d = 0; d < D; ++d) x[d] = Elem<T>::load(p + d);
}

// ---------------------------------------------------------------- forward
template <typename T, int D>
__global__ __launch_bounds__(kRows) void fwd_simple_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                          const T* __restrict__ v, T* __restrict__ out,
                                                          float* __restrict__ lse, AttnShape s) {
    __shared__ float qs[D][kRows];
    const int lane = threadIdx.x;
    const int h = blockIdx.y, b = blockIdx.z;
    const int hk = h / (s.Hq / s.Hkv);
    const int i_first = blockIdx.x * kRows;
    const int i_last = min(s.L, i_first + kRows) - 1;
    const int i = min(i_first + lane, s.L - 1);  // lanes past the end shadow the last row, never store
    const bool live = i_first + lane < s.L;
    const int Dt = s.D;
    const size_t qoff = (((size_t)b * s.Hq + h) * s.qhs + i) * Dt;
    const T* kb = k + ((size_t)b * s.Hkv + hk) * s.kvhs * Dt;
    const T* vb = v + ((size_t)b * s.Hkv + hk) * s.kvhs * Dt;
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (d < Dt) qs[d][lane] = Elem<T>::load(q + qoff + d) * s.scale;

    float o[D];
#pragma unroll
    for (int d = 0; d < D; ++d) o[d] = 0.f;
    float m = -INFINITY, l = 0.f;

    auto visit = [&](int j) {
        const T* kr = kb + (size_t)j * Dt;
        float sc = 0.f;
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (d < Dt) sc += qs[d][lane] * Elem<T>::load(kr + d);
        if (sc > m) {
            float a = expf(m - sc);
            l *= a;
#pragma unroll
            for (int d = 0; d < D; ++d) o[d] *= a;
            m = sc;
        }
        float p = expf(sc - m);
        l += p;
        const T* vr = vb + (size_t)j * Dt;
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (d < Dt) o[d] += p * Elem<T>::load(vr + d);
    };

    // sinks and gists left of every window of this wave's rows, then the union of the windows
    const int lo_wave = win_lo(s, i_first);
    const int lo_i = win_lo(s, i);
    const int na_wave = count_always(s, lo_wave);  // always-visible positions < lo_wave
    for (int g = 0; g < na_wave; ++g) visit(pos_of_always(s, g));
    for (int j = lo_wave; j <= i_last; ++j) {
        bool ok = j <= i && (is_always(s, j) || j >= lo_i);
        if (ok) visit(j);
    }
    if (live) {
        float inv = 1.f / l;
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (d < Dt) Elem<T>::store(out + qoff + d, o[d] * inv);
        lse[((size_t)b * s.Hq + h) * s.qhs + i] = m + logf(l);
    }
}

// ---------------------------------------------------------------- dQ (+ delta)
template <typename T, int D>
__global__ __launch_bounds__(kRows) void dq_simple_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                         const T* __restrict__ v, const T* __restrict__ out,
                                                         const float* __restrict__ lse, const T* __restrict__ dout,
                                                         T* __restrict__ dq, float* __restrict__ delta, AttnShape s) {
    __shared__ float qs[D][kRows];
    __shared__ float dos[D][kRows];
    const int lane = threadIdx.x;
    const int h = blockIdx.y, b = blockIdx.z;
    const int hk = h / (s.Hq / s.Hkv);
    const int i_first = blockIdx.x * kRows;
    const int i_last = min(s.L, i_first + kRows) - 1;
    const int i = min(i_first + lane, s.L - 1);
    const bool live = i_first + lane < s.L;
    const size_t row = ((size_t)b * s.Hq + h) * s.qhs + i;   // in the caller's tensors
    const size_t wrow = ((size_t)b * s.Hq + h) * s.L + i;    // in the dense workspace
    const int Dt = s.D;
    const size_t qoff = row * Dt;
    const T* kb = k + ((size_t)b * s.Hkv + hk) * s.kvhs * Dt;
    const T* vb = v + ((size_t)b * s.Hkv + hk) * s.kvhs * Dt;
    float dl = 0.f;
#pragma unroll
    for (int d = 0; d < D; ++d) {
        if (d >= Dt) continue;
        qs[d][lane] = Elem<T>::load(q + qoff + d) * s.scale;
        float g = Elem<T>::load(dout + qoff + d);
        dos[d][lane] = g;
        dl += g * Elem<T>::load(out + qoff + d);
    }
    const float ls = lse[row];
    if (live) delta[wrow] = dl;

    float acc[D];
#pragma unroll
    for (int d = 0; d < D; ++d) acc[d] = 0.f;

    auto visit = [&](int j) {
        const T* kr = kb + (size_t)j * Dt;
        const T* vr = vb + (size_t)j * Dt;
        float sc = 0.f, dp = 0.f;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (d >= Dt) continue;
            sc += qs[d][lane] * Elem<T>::load(kr + d);
            dp += dos[d][lane] * Elem<T>::load(vr + d);
        }
        float ds = expf(sc - ls) * (dp - dl);
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (d < Dt) acc[d] += ds * Elem<T>::load(kr + d);
    };

    const int lo_wave = win_lo(s, i_first);
    const int lo_i = win_lo(s, i);
    const int na_wave = count_always(s, lo_wave);
    for (int g = 0; g < na_wave; ++g) visit(pos_of_always(s, g));
    for (int j = lo_wave; j <= i_last; ++j) {
        bool ok = j <= i && (is_always(s, j) || j >= lo_i);
        if (ok) visit(j);
    }
    if (live) {
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (d < Dt) Elem<T>::store(dq + qoff + d, acc[d] * s.scale);
    }
}

// ---------------------------------------------------------------- dK, dV
template <typename T, int D>
__global__ __launch_bounds__(kRows) void dkdv_simple_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                           const T* __restrict__ v, const float* __restrict__ lse,
                                                           const T* __restrict__ dout, const float* __restrict__ delta,
                                                           T* __restrict__ dk, T* __restrict__ dv, AttnShape s) {
    __shared__ float ks[D][kRows];
    __shared__ float vs[D][kRows];
    const int lane = threadIdx.x;
    const int hk = blockIdx.y, b = blockIdx.z;
    const int group = s.Hq / s.Hkv;
    const int j_first = blockIdx.x * kRows;
    const int j_last = min(s.L, j_first + kRows) - 1;
    const int j = min(j_first + lane, s.L - 1);
    const bool live = j_first + lane < s.L;
    const int Dt = s.D;
    const size_t koff = (((size_t)b * s.Hkv + hk) * s.kvhs + j) * Dt;
#pragma unroll
    for (int d = 0; d < D; ++d) {
        if (d >= Dt) continue;
        ks[d][lane] = Elem<T>::load(k + koff + d) * s.scale;
        vs[d][lane] = Elem<T>::load(v + koff + d);
    }
    const bool always_j = is_always(s, j);
    const int hi_j = win_hi(s, j);
    // does any key of this block hold a sink or a gist?  then every later row sees it
    const int first_always = pos_of_always(s, count_always(s, j_first));  // first always-visible position >= j_first
    const bool any_always = first_always <= j_last;
    const int i_end = any_always ? s.L - 1 : win_hi(s, j_last);

    float ak[D], av[D];
#pragma unroll
    for (int d = 0; d < D; ++d) ak[d] = av[d] = 0.f;

    for (int g = 0; g < group; ++g) {
        const int h = hk * group + g;
        const size_t base = ((size_t)b * s.Hq + h) * s.qhs;  // caller's q, dout, lse
        const size_t wbase = ((size_t)b * s.Hq + h) * s.L;   // workspace delta
        for (int i = j_first; i <= i_end; ++i) {
            bool ok = j <= i && (always_j || i <= hi_j);
            if (!ok) continue;
            const T* qr = q + (base + i) * Dt;
            const T* gr = dout + (base + i) * Dt;
            float sc = 0.f, dp = 0.f;
#pragma unroll
            for (int d = 0; d < D; ++d) {
                if (d >= Dt) continue;
                sc += ks[d][lane] * Elem<T>::load(qr + d);
                dp += vs[d][lane] * Elem<T>::load(gr + d);
            }
            float p = expf(sc - lse[base + i]);
            float ds = p * (dp - delta[wbase + i]);
#pragma unroll
            for (int d = 0; d < D; ++d) {
                if (d >= Dt) continue;
                av[d] += p * Elem<T>::load(gr + d);
                ak[d] += ds * Elem<T>::load(qr + d);
            }
        }
    }
    if (live) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (d >= Dt) continue;
            Elem<T>::store(dk + koff + d, ak[d] * s.scale);
            Elem<T>::store(dv + koff + d, av[d]);
        }
    }
}

template <typename T, int D>
hipError_t fwd_launch(const void* q, const void* k, const void* v, void* out, float* lse, const AttnShape& s,
                      hipStream_t st) {
    dim3 grid((s.L + kRows - 1) / kRows, s.Hq, s.B);
    fwd_simple_kernel<T, D><<<grid, kRows, 0, st>>>((const T*)q, (const T*)k, (const T*)v, (T*)out, lse, s);
    return hipGetLastError();
}

template <typename T, int D>
hipError_t bwd_launch(const void* q, const void* k, const void* v, const void* out, const float* lse,
                      const void* dout, void* dq, void* dk, void* dv, float* delta, const AttnShape& s,
                      hipStream_t st) {
    dim3 gq((s.L + kRows - 1) / kRows, s.Hq, s.B);
    dq_simple_kernel<T, D><<<gq, kRows, 0, st>>>((const T*)q, (const T*)k, (const T*)v, (const T*)out, lse,
                                                 (const T*)dout, (T*)dq, delta, s);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 gk((s.L + kRows - 1) / kRows, s.Hkv, s.B);
    dkdv_simple_kernel<T, D><<<gk, kRows, 0, st>>>((const T*)q, (const T*)k, (const T*)v, lse, (const T*)dout,
                                                   delta, (T*)dk, (T*)dv, s);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd_simple(const void* q, const void* k, const void* v, void* out, float* lse,
                             const AttnShape& s, unigist_dtype dt, hipStream_t st) {
    if (dt == UNIGIST_F32)
        return s.D <= 64 ? fwd_launch<float, 64>(q, k, v, out, lse, s, st)
                         : fwd_launch<float, 128>(q, k, v, out, lse, s, st);
    return s.D <= 64 ? fwd_launch<bf16_t, 64>(q, k, v, out, lse, s, st)
                     : fwd_launch<bf16_t, 128>(q, k, v, out, lse, s, st);
}

hipError_t launch_bwd_simple(const void* q, const void* k, const void* v, const void* out, const float* lse,
                             const void* dout, void* dq, void* dk, void* dv, float* delta, const AttnShape& s,
                             unigist_dtype dt, hipStream_t st) {
    if (dt == UNIGIST_F32)
        return s.D <= 64 ? bwd_launch<float, 64>(q, k, v, out, lse, dout, dq, dk, dv, delta, s, st)
                         : bwd_launch<float, 128>(q, k, v, out, lse, dout, dq, dk, dv, delta, s, st);
    return s.D <= 64 ? bwd_launch<bf16_t, 64>(q, k, v, out, lse, dout, dq, dk, dv, delta, s, st)
                     : bwd_launch<bf16_t, 128>(q, k, v, out, lse, dout, dq, dk, dv, delta, s, st);
}

}  // namespace unigist
