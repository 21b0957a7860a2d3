// Forward kernel of gist-masked attention for gfx950: bf16 MFMA, fp32 online softmax.
//
// Mask (Sec. 4.1, Eq. 3): query i sees key j <= i iff j holds a sink or a gist, or j lies inside the local
// window of i (the W most recent positions, or the gist unit of i plus the W previous units).
// Block skipping (Sec. 4.2) is done without moving any data: a query tile walks
//   1. the compact list of gists left of its window (gist g sits at row (r+1)g + r of
//      K/V, gathered by address arithmetic while staging the tile; all of them are
//      visible to every row, so no mask), then
//   2. the contiguous key tiles from the window's first tile to the diagonal, where the
//      full predicate is applied only on tiles that can contain an invisible pair.
//
// Work split: one workgroup = 128 query rows of one head, 4 waves x 32 rows; 64 keys
// per step.  Scores are computed transposed, S^T = K Q^T with v_mfma_f32_32x32x16_bf16,
// so that one lane owns one query column: row max and row sum are in-lane reductions
// plus one exchange between the wave's halves, and the accumulator registers of S^T are
// already the B operand of O^T += V^T P^T.  V^T fragments come straight out of the
// row-major V tile in LDS through ds_read_b64_tr_b16.  K/V tiles are staged with direct
// global->LDS loads into two LDS stages (one barrier per step), 16-byte chunks swizzled.
#include <type_traits>

#include "mfma_common.h"

namespace unigist {
namespace {

constexpr int BM = 128;  // query rows per workgroup
constexpr int BN = 32;   // keys per step
constexpr int NT = 256;  // threads
constexpr float kLazy = 8.f;  // slack of the softmax reference, in exp2 units
constexpr float kBigSum = 16384.f;  // a partial row sum above this sends the step through the maximum search

template <int D>
struct FwdSmem {
    // two stages of a K tile and a V tile, rows unpadded, 16-byte chunks swizzled (see swz())
    char k[2][BN * D * 2];
    char v[2][BN * D * 2];
};

// GEN = false is the layout without sinks and with the sliding window: the mask helpers then fold to their
// short forms at compile time.
template <int D, bool GEN>
__global__ __launch_bounds__(NT, 3) void fwd_mfma_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                        const bf16_t* __restrict__ v, bf16_t* __restrict__ out,
                                                        float* __restrict__ lse, AttnShape s_arg, int nq) {
    AttnShape s = s_arg;
    if constexpr (!GEN) {
        s.S = 0;
        s.umode = 0;
    }
    constexpr int KS = D / 16;            // k-steps of the score MFMA
    constexpr int DB = D / 32;            // 32-row blocks of O^T
    constexpr int CH = D / 8;             // 16-byte chunks per row
    constexpr int RPI = 64 / CH;          // tile rows covered by one direct-load instruction
    constexpr int IPW = BN / RPI / 4;     // such instructions per wave, per matrix, per tile
    constexpr int NKB = BN / 32;          // 32-key blocks per step
    __shared__ __attribute__((aligned(1024))) FwdSmem<D> sm;

    const int tid = threadIdx.x;
    const int lane = tid & 63, w = tid >> 6;
    const int c32 = lane & 31, h = lane >> 5;

    // ---- which (batch, head, query tile): heads of one kv group stay on one XCD, long tiles first
    const int G = s.Hq / s.Hkv;
    const int NP = s.B * s.Hkv;
    int n = blockIdx.x, g, pr, qt;
    if ((NP & 7) == 0) {
        const int xcd = n & 7, mm = n >> 3;
        g = mm % G;
        const int rest = mm / G;
        const int pb = rest % (NP >> 3);
        qt = nq - 1 - rest / (NP >> 3);
        pr = xcd + 8 * pb;
    } else {
        g = n % G;
        const int rest = n / G;
        pr = rest % NP;
        qt = nq - 1 - rest / NP;
    }
    const int b = pr / s.Hkv, hk = pr % s.Hkv;
    const int hq = hk * G + g;

    // Positions are absolute; q/out/lse hold the rows qpos0 .. L-1, K/V hold ngb compact gist rows followed
    // by the positions s0 .. L-1 (training: everything from position 0, no compact rows).
    const int L = s.L, rp1 = s.rp1;
    const int qpos0 = s.qpos0, s0 = s.s0, ngb = s.ngb;
    const int i0 = qpos0 + qt * BM;
    const int i1 = min(L, i0 + BM) - 1;
    const int qrow = i0 + 32 * w + c32;      // this lane's query row
    const int qrow_ld = min(qrow, L - 1);    // rows past the end shadow the last row and are never stored
    const int wrow0 = i0 + 32 * w;           // first row of the wave

    const bf16_t* kb = k + ((size_t)b * s.Hkv + hk) * s.kv_rows * D;
    const bf16_t* vb = v + ((size_t)b * s.Hkv + hk) * s.kv_rows * D;

    // ---- Q fragments (B operand of S^T = K Q^T): lane holds Q[qrow][16 ks + 8 h .. +7]
    bf16x8 qf[KS];
    {
        const bf16_t* qp = q + (((size_t)b * s.Hq + hq) * s.qhs + (qrow_ld - qpos0)) * D + 8 * h;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const bf16x8*)(qp + 16 * ks);
    }

    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) o[db] = zero16();
    float m = -INFINITY, l = 0.f;
    bool need_max = true;  // until every row of the wave has a finite reference
    const float c = s.scale * 1.4426950408889634f;  // exp(x * scale) = exp2(x * c)

    // ---- tile walk
    const int lo = win_lo(s, i0);                 // leftmost position inside any window of the tile
    const int wstart = max((lo / BN) * BN, s0);  // first position of the window phase
    const int nfar = count_always(s, wstart);     // sinks and gists strictly left of the window phase
    const int ngt = (nfar + BN - 1) / BN;
    const int span_q = qrow - win_lo(s, qrow);    // this lane's window reaches span_q positions back
    const int lo_wlast = win_lo(s, wrow0 + 31);   // window start of the wave's last row
    const int nwin = (i1 - wstart) / BN + 1;
    const int ntiles = ngt + nwin;

    // ---- staging: direct global->LDS loads; lane fetches chunk (lane % CH) ^ swz(row) of its row.
    const int lrow = lane / CH;
    const int wv = __builtin_amdgcn_readfirstlane(w);
    int choff[IPW];  // byte offset of the lane's (swizzled) chunk inside its row, per load slot
#pragma unroll
    for (int i = 0; i < IPW; ++i) choff[i] = ((lane % CH) ^ swz<CH>((wv * IPW + i) * RPI + lrow)) * 16;
    const int S = s.S;
    const char* kbytes = (const char*)kb;
    const char* vbytes = (const char*)vb;
    auto issue = [&](int it, int buf) {
        // Tile row rr is, in the gist phase, the (it * BN + rr)-th always-visible position (a sink, or gist g at
        // S + (r+1) g + r), clamped to the last far one; in the window phase position wstart + (it - ngt) * BN + rr,
        // clamped to the last position.  Its row in the buffer: position - s0 + ngb, except for the entries in
        // front (entry c < ngb sits in row c).
        const bool gphase = it < ngt;
#pragma unroll
        for (int i = 0; i < IPW; ++i) {
            const int rr = (wv * IPW + i) * RPI + lrow;
            int row;
            if (gphase) {
                const int c = min(it * BN + rr, nfar - 1);
                const int pos = c < S ? c : S + (c - S) * rp1 + rp1 - 1;
                row = c < ngb ? c : pos - s0 + ngb;
            } else {
                row = min(wstart + (it - ngt) * BN + rr, L - 1) - s0 + ngb;
            }
            const unsigned off = (unsigned)row * (unsigned)(D * 2) + (unsigned)choff[i];  // < 2^32 by the size limit
            g2l16(kbytes + off, &sm.k[buf][(wv * IPW + i) * 1024]);
            g2l16(vbytes + off, &sm.v[buf][(wv * IPW + i) * 1024]);
        }
    };

    // per-lane LDS offsets that do not depend on the tile
    int koff[KS];  // row-wise read of K row c32 (+32), chunk 2 ks + h
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) koff[ks] = swz_off<CH>(c32, 2 * ks + h);
    int voff[DB];  // transposing read of V, 32-column block db
#pragma unroll
    for (int db = 0; db < DB; ++db) voff[db] = tr_lane_off<CH>(db);

    // one step of the walk on LDS stage BUF (a compile-time constant, so that every LDS address is a
    // per-lane register plus an immediate)
    auto tile_step = [&](auto bufc, int it) {
        constexpr int BUF = decltype(bufc)::value;
        const char* kt = sm.k[BUF];
        const char* vt = sm.v[BUF];
        const bool gist_tile = it < ngt;
        const int j0 = gist_tile ? it * BN : wstart + (it - ngt) * BN;  // compact index or position
        // a window tile entirely right of this wave's rows contributes nothing
        if (!gist_tile && j0 > wrow0 + 31) return;

        // ---- S^T = K Q^T : two 32-key blocks
        f32x16 sa[NKB];
#pragma unroll
        for (int kb2 = 0; kb2 < NKB; ++kb2) {
            sa[kb2] = zero16();
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                bf16x8 a = *(const bf16x8*)(kt + kb2 * 32 * CH * 16 + koff[ks]);
                sa[kb2] = mfma32(a, qf[ks], sa[kb2]);
            }
        }

        // ---- mask.  Accumulator element i of block kb2 is key  j0 + 32 kb2 + 8 (i/4) + 4 h + i%4; bit
        // 8 (i/4) + i%4 of vis[kb2] says whether this lane's query sees it.  Visible sets are bit ranges
        // (the tail of the compact list; the window) plus, in the window phase, the sinks and gists.
        bool masked;
        unsigned vis[NKB];
        auto below = [](int n) { return n >= 32 ? ~0u : n <= 0 ? 0u : (1u << n) - 1u; };  // bits 0 .. n-1
        if (gist_tile) {
            masked = j0 + BN > nfar;  // tail of the compact list
#pragma unroll
            for (int kb2 = 0; kb2 < NKB; ++kb2) vis[kb2] = below(nfar - j0 - 4 * h - 32 * kb2);
        } else {
            // unmasked iff all keys are causal for the wave's first row and in the window of its last row
            masked = !(j0 + BN - 1 <= wrow0 && j0 >= lo_wlast);
            if (masked) {
                // bit t of gm: key j0 + 4h + t holds a sink or a gist.  One modulo per lane, shared by ballot.
                const unsigned long long gbits = __builtin_amdgcn_ballot_w64(is_always(s, j0 + lane));
                const unsigned long long gm = gbits >> (4 * h);
                const int d0 = qrow - (j0 + 4 * h);  // distance to the lane's first key
#pragma unroll
                for (int kb2 = 0; kb2 < NKB; ++kb2) {
                    const int d = d0 - 32 * kb2;  // offsets d - span_q .. d are in the window, offsets <= d causal
                    const unsigned causal = below(d + 1);
                    vis[kb2] = (causal & ~below(d - span_q)) | (causal & (unsigned)(gm >> (32 * kb2)));
                }
            }
        }
        if (masked) {
#pragma unroll
            for (int kb2 = 0; kb2 < NKB; ++kb2)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (!((vis[kb2] >> (8 * (i / 4) + (i % 4))) & 1u)) sa[kb2][i] = -INFINITY;
        }

        // ---- online softmax (per query column = per lane).  P = exp2(c S - c m) is summed in fp32 for the row
        // sum (lse stays fp32-accurate) and rounded to bf16 for the second MFMA.  The reference m only has to
        // bound the scores from above within a margin, not be their exact maximum, so the common step does not
        // look for the maximum at all: it exponentiates against the current reference and only if a partial row
        // sum comes out above 2^kBig (or not finite) -- some score exceeded the reference by a lot -- falls back
        // to the step with the maximum.  The quotient O / l is the same either way.
        u32x4 pk[NKB][2];
        float ls;
        auto exps = [&](float mc) __attribute__((always_inline)) {
            ls = 0.f;
#pragma unroll
            for (int kb2 = 0; kb2 < NKB; ++kb2)
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(fmaf(sa[kb2][i], c, -mc));
                    const float p1 = __builtin_amdgcn_exp2f(fmaf(sa[kb2][i + 1], c, -mc));
                    ls += p0 + p1;
                    pk[kb2][i / 8][(i / 2) % 4] = pack_bf16x2(p0, p1);
                }
        };
        bool with_max = need_max;  // wave-uniform: some row of the wave has no reference yet
        if (!with_max) {
            exps(m * c);
            with_max = __builtin_amdgcn_ballot_w64(!(ls <= kBigSum)) != 0ull;
        }
        if (with_max) {
            float mx = sa[0][0];
#pragma unroll
            for (int kb2 = 0; kb2 < NKB; ++kb2)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sa[kb2][i]);
            mx = fmaxf(mx, other_half(mx));
            // the reference is raised (and O, l rescaled) only when a row's maximum exceeds it by more than kLazy
            // in exp2 units, so P <= 2^kLazy here.  A row that has seen nothing yet has m = -inf and grows on its
            // first score; -inf - (-inf) is NaN and compares false.
            const bool grow = (mx - m) * c > kLazy;
            if (__builtin_amdgcn_ballot_w64(grow) != 0ull) {
                const float m_new = grow ? mx : m;
                const float alpha = grow ? __builtin_amdgcn_exp2f((m - m_new) * c) : 1.f;  // m = -inf gives 0
                l *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
                m = m_new;
            }
            exps((m == -INFINITY ? 0.f : m) * c);  // rows with nothing visible so far: every P is exp2(-inf) = 0
            need_max = __builtin_amdgcn_ballot_w64(m == -INFINITY) != 0ull;
        }
        l += ls;

        // ---- O^T += V^T P^T : 16 keys per MFMA, A operand by transposing LDS reads
#pragma unroll
        for (int kb2 = 0; kb2 < NKB; ++kb2)
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const bf16x8 pb = __builtin_bit_cast(bf16x8, pk[kb2][kk]);
#pragma unroll
                for (int db = 0; db < DB; ++db)
                    o[db] = mfma32(tr16_frag_at<CH>(vt + voff[db], 32 * kb2 + 16 * kk), pb, o[db]);
            }
    };

    issue(0, 0);
    for (int it = 0; it < ntiles; it += 2) {
        wait_vmem();      // this wave's part of tile `it` has landed
        __syncthreads();  // ... and everyone's; everyone is also done reading the other stage
        if (it + 1 < ntiles) issue(it + 1, 1);
        tile_step(std::integral_constant<int, 0>{}, it);
        if (it + 1 < ntiles) {
            wait_vmem();
            __syncthreads();
            if (it + 2 < ntiles) issue(it + 2, 0);
            tile_step(std::integral_constant<int, 1>{}, it + 1);
        }
    }

    // ---- epilogue: normalise, store O (row qrow, d = 32 db + 8 (i/4) + 4 h + i%4) and LSE
    const float lt = l + other_half(l);
    const float inv = 1.f / lt;
    if (qrow < L) {
        const size_t orow = ((size_t)b * s.Hq + hq) * s.qhs + (qrow - qpos0);
        bf16_t* op = out + orow * D + 4 * h;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                u32x2 w2;
                w2[0] = pack_bf16x2(o[db][4 * i4] * inv, o[db][4 * i4 + 1] * inv);
                w2[1] = pack_bf16x2(o[db][4 * i4 + 2] * inv, o[db][4 * i4 + 3] * inv);
                *(u32x2*)(op + 32 * db + 8 * i4) = w2;
            }
        if (h == 0) lse[orow] = m * s.scale + __builtin_amdgcn_logf(lt) * 0.6931471805599453f;
    }
}

}  // namespace

hipError_t launch_fwd_mfma(const void* q, const void* k, const void* v, void* out, float* lse, const AttnShape& s,
                           hipStream_t st) {
    const int nq = (s.Lq + BM - 1) / BM;
    const long nblk = (long)nq * s.Hq * s.B;
    if (nblk > 0x7fffffffL) return hipErrorInvalidValue;
    const bool gen = s.S != 0 || s.umode != 0;
    auto go = [&](auto kern) {
        kern<<<dim3((unsigned)nblk), NT, 0, st>>>((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)out, lse,
                                                  s, nq);
    };
    if (s.D == 64) gen ? go(fwd_mfma_kernel<64, true>) : go(fwd_mfma_kernel<64, false>);
    else gen ? go(fwd_mfma_kernel<128, true>) : go(fwd_mfma_kernel<128, false>);
    return hipGetLastError();
}

}  // namespace unigist
