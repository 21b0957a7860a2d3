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
// Work split: one workgroup = 128 query rows of one head, 4 waves x 32 rows; 32 keys per step.
// The matrix instruction is v_mfma_f32_16x16x32_bf16 (D = A * B + C, A 16 x 32, B 32 x 16).  With r16 = lane % 16
// and g4 = lane / 16:
//   A: lane holds A[r16][8 g4 .. 8 g4 + 7]      B: lane holds B[8 g4 .. 8 g4 + 7][r16]
//   C/D: register i holds D[4 g4 + i][r16]
// On random operands the chip, which is power-limited, sustains about 11 % more flops with this shape than with
// 32x32x16; an operand of the same size feeds half as many flops, so every K and V fragment read from LDS is
// used for the wave's two 16-row query blocks, which keeps the LDS and staging traffic per flop where it was.
// Scores are computed transposed, S^T = K Q^T (A = K rows from LDS, B = Q in registers): a query is a column,
// spread over the four lanes r16 + 16 g4, each of which holds 4 of every 16 keys; the running reference of the
// softmax is kept identical on those four lanes and the row sum is a per-lane partial until the epilogue.  The
// accumulator registers of S^T for two 16-key blocks are, after exponentiation and rounding, already the B
// operand of O^T += V^T P^T with the contraction slot 8 g4 + 4 kb + i standing for key 16 kb + 4 g4 + i; the
// matching A operand V^T comes straight out of the row-major V tile in LDS through two ds_read_b64_tr_b16 (rows
// 4 g4 .. 4 g4 + 3 of either 16-key block).  K/V tiles are staged with direct global->LDS loads into two LDS
// stages (one barrier per step), 16-byte chunks swizzled with a period of 16 rows.
#include <string.h>

#include <algorithm>
#include <type_traits>
#include <vector>

#include "mfma_common.h"
#include "plan.h"

namespace unigist {
namespace {

constexpr int BM = kFwdBm;  // query rows per workgroup
constexpr int BN = kFwdBn;  // keys per step
constexpr int NT = 256;  // threads
constexpr float kLazy = 8.f;  // slack of the softmax reference, in exp2 units
constexpr float kBigSum = 16384.f;  // a partial row sum above this sends the step through the maximum search

template <int D>
struct FwdSmem {
    // two stages of a K tile and a V tile, rows unpadded, 16-byte chunks swizzled (see swz16())
    char k[2][BN * D * 2];
    char v[2][BN * D * 2];
};

// GEN = false is the layout without sinks and with the sliding window: the mask helpers then fold to their
// short forms at compile time.
enum { PLAIN = 0, PACK = 1, RAGGED = 2 };
template <int MODE> struct ModeArg { typedef NoDocs type; };
template <> struct ModeArg<PACK> { typedef DocTab type; };
template <> struct ModeArg<RAGGED> { typedef RaggedSeqs type; };

// D is the head dimension the kernel is built for (64 or 128); the tensors' head dimension s.D may be any smaller
// multiple of 8.  Rows in memory are s.D elements long; LDS tiles and fragments have D columns, of which the ones
// from s.D on hold zeros in Q (so they add nothing to the scores) and are never stored on the output side.
// MODE = PACK: the launch covers the documents of a packed buffer (ext), s_arg is the shape of the whole pack.
// MODE = RAGGED: chunk-wise prefill of a batch whose sequences are in different states (ext: device arrays);
// s_arg is the launch's shape and each workgroup derives its sequence's (seq_view).
template <int D, bool GEN, int MODE>
__global__ __launch_bounds__(NT, 3) void fwd_mfma_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                        const bf16_t* __restrict__ v, bf16_t* __restrict__ out,
                                                        float* __restrict__ lse, AttnShape s_arg, int nq,
                                                        typename ModeArg<MODE>::type ext) {
    AttnShape s = s_arg;
    if constexpr (!GEN) {
        s.S = 0;
        s.umode = 0;
    }
    int n = blockIdx.x;
    if constexpr (MODE == PACK) {  // the document becomes the whole problem: its rows, its tiles, its workgroup ids
        const int d = doc_of_block(ext, n);
        n -= ext.blk0[d];
        s = doc_view(s, ext.len[d]);
        nq = (s.L + BM - 1) / BM;
        const size_t ro = (size_t)ext.c0[d] * s.D;
        const size_t qro = s.q_rs ? (size_t)ext.c0[d] * s.q_rs : ro;  // q and out may have explicit strides
        q += qro;
        k += ro;
        v += ro;
        out += qro;
        lse += ext.c0[d];
    }
    constexpr int KS = D / 32;            // k-steps of the score MFMA
    constexpr int DB = D / 16;            // 16-row blocks of O^T
    constexpr int CH = D / 8;             // 16-byte chunks per row
    constexpr int RPI = 64 / CH;          // tile rows covered by one direct-load instruction
    constexpr int IPW = BN / RPI / 4;     // such instructions per wave, per matrix, per tile
    __shared__ __attribute__((aligned(1024))) FwdSmem<D> sm;

    const int tid = threadIdx.x;
    const int lane = tid & 63, w = tid >> 6;
    const int r16 = lane & 15, g4 = lane >> 4;  // MFMA 16x16x32: lane = (row or column r16, k-group g4)

    // ---- which (batch, head, query tile): heads of one kv group stay on one XCD, long tiles first
    const int G = s.Hq / s.Hkv;
    const int NP = s.B * s.Hkv;
    int g, pr, qt;
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
    if constexpr (MODE == RAGGED) {
        // The sequence's state comes from device memory, so it is checked here: a workgroup of a sequence whose
        // state is invalid, or whose tile lies past the sequence's rows, leaves (the whole workgroup, before any
        // barrier); one workgroup per sequence reports the cache rows in use, or -1.
        const int p0 = ext.p0[b], nb = ext.n[b], s0b = ext.s0[b];
        int rows = -1;
        if (p0 >= 0 && nb >= 0 && nb <= s.Lq && s0b >= 0 && (long long)p0 + nb <= s.L) {
            if (nb == 0) {
                if (s0b <= p0) rows = count_always(s, s0b) + (p0 - s0b);
            } else {
                const AttnShape sv = seq_view(s, p0, nb, s0b);
                const int need = sv.ngb + (sv.L - s0b);
                if (s0b <= win_lo(sv, p0) && need <= s.kv_rows) {  // every key the first query sees is cached
                    rows = need;
                    s = sv;
                }
            }
        }
        if (hq == 0 && qt == nq - 1 && threadIdx.x == 0) ext.rows[b] = rows;
        if (rows < 0 || qt * BM >= nb) return;
    }

    // Positions are absolute; q/out/lse hold the rows qpos0 .. L-1, K/V hold ngb compact gist rows followed
    // by the positions s0 .. L-1 (training: everything from position 0, no compact rows).
    const int L = s.L, rp1 = s.rp1, Dt = s.D;
    const int qpos0 = s.qpos0, s0 = s.s0, ngb = s.ngb;
    const int i0 = qpos0 + qt * BM;
    const int i1 = min(L, i0 + BM) - 1;
    const int wrow0 = i0 + 32 * w;           // first row of the wave
    int qrow[2], qrow_ld[2];                 // this lane's two query rows (16-row blocks qb = 0, 1)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        qrow[qb] = wrow0 + 16 * qb + r16;
        qrow_ld[qb] = min(qrow[qb], L - 1);  // rows past the end shadow the last row and are never stored
    }

    const bf16_t* kb = k + ((size_t)b * s.Hkv + hk) * s.kv_rows * Dt;
    const bf16_t* vb = v + ((size_t)b * s.Hkv + hk) * s.kv_rows * Dt;

    // ---- Q fragments (B operand of S^T = K Q^T): lane holds Q[qrow[qb]][32 ks + 8 g4 .. +7]
    bf16x8 qf[2][KS];
    f32x4 o[DB][2];   // O^T blocks: register i of o[db][qb] is d = 16 db + 4 g4 + i, column = query qrow[qb]
    float m[2], l[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const size_t qoff = s.q_rs ? (size_t)b * s.q_bs + (size_t)hq * s.q_hs + (size_t)(qrow_ld[qb] - qpos0) * s.q_rs
                                   : (((size_t)b * s.Hq + hq) * s.qhs + (qrow_ld[qb] - qpos0)) * Dt;
        const bf16_t* qp = q + qoff + 8 * g4;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 z = {0u, 0u, 0u, 0u};  // columns past the tensors' head dimension are zero
            if (32 * ks + 8 * g4 < Dt) z = *(const u32x4*)(qp + 32 * ks);
            qf[qb][ks] = __builtin_bit_cast(bf16x8, z);
        }
#pragma unroll
        for (int db = 0; db < DB; ++db) o[db][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
        m[qb] = -INFINITY;
        l[qb] = 0.f;
    }
    bool need_max = true;  // until every row of the wave has a finite reference
    const float sc = s.kscale ? s.scale * s.kscale[hk] : s.scale;  // softmax scale times the scale of the stored keys
    const float c = sc * 1.4426950408889634f;                       // exp(x * sc) = exp2(x * c)

    // ---- tile walk
    const RowWalk walk = row_walk(s, i0, i1, BN);
    const int wstart = walk.wstart;               // first position of the window phase
    const int nfar = walk.nfar;                   // sinks and gists strictly left of the window phase
    const int ngt = walk.ngt;
    int span_q[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) span_q[qb] = qrow[qb] - win_lo(s, qrow[qb]);  // the window reaches this far back
    const int lo_wlast = win_lo(s, wrow0 + 31);   // window start of the wave's last row
    const int ntiles = ngt + walk.nwin;

    // ---- staging: direct global->LDS loads; lane fetches chunk (lane % CH) ^ swz(row) of its row.
    const int lrow = lane / CH;
    const int wv = __builtin_amdgcn_readfirstlane(w);
    int choff[IPW];  // byte offset of the lane's (swizzled) chunk inside its row, per load slot
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
        const int sc = (lane % CH) ^ swz16<CH>((wv * IPW + i) * RPI + lrow);
        choff[i] = 8 * sc < Dt ? sc * 16 : 0;  // a chunk the rows do not have: any chunk will do (see above)
    }
    const int S = s.S;
    const char* kbytes = (const char*)kb;
    const char* vbytes = (const char*)vb;
    auto issue = [&](int it, int buf) {
        // Tile row rr is, in the gist phase, the (it * BN + rr)-th always-visible position (a sink, or gist g at
        // S + (r+1) g + r), clamped to the last far one; in the window phase position wstart + (it - ngt) * BN + rr,
        // clamped to the last position.  Its row in the buffer: position - s0 + ngb, except for the entries in
        // front (entry c < ngb sits in row c).  The phase only selects wave-uniform parameters, so the per-lane
        // arithmetic has no branch.
        const bool gphase = it < ngt;
        const int a = gphase ? it * BN : wstart + (it - ngt) * BN;
        const int bnd = gphase ? nfar - 1 : L - 1;
        const int first_gist = gphase ? S : 0x7fffffff;  // entries from here on are gists
        const int in_front = gphase ? ngb : 0;           // entries below this sit in the row of their own number
        const int gm = gphase ? rp1 : 1, go = gphase ? 1 : 0;
#pragma unroll
        for (int i = 0; i < IPW; ++i) {
            const int rr = (wv * IPW + i) * RPI + lrow;
            const int c = min(a + rr, bnd);
            int pos;
            if constexpr (GEN)  // entry c >= S is gist c - S at S + (c - S)(r+1) + r; factors < 2^24 by the size limit
                pos = c < first_gist ? c : S + mul24(c - S + 1, rp1) - 1;
            else
                pos = mul24(c + go, gm) - go;
            const int row = c < in_front ? c : pos - s0 + ngb;
            const unsigned off = (unsigned)row * (unsigned)(Dt * 2) + (unsigned)choff[i];  // < 2^32 by the size limit
            g2l16(kbytes + off, &sm.k[buf][(wv * IPW + i) * 1024]);
            g2l16(vbytes + off, &sm.v[buf][(wv * IPW + i) * 1024]);
        }
    };

    // per-lane LDS offsets that do not depend on the tile
    int koff[KS];  // row-wise read of K row r16 (+16 kb), chunk 4 ks + g4
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) koff[ks] = r16 * (CH * 16) + (((4 * ks + g4) ^ swz16<CH>(r16)) << 4);
    // transposing read of V: the 16 lanes of group g4 fetch the 4 x 16 block rows 4 g4 .. +3, columns 16 db .. +15:
    // lane p passes the address of V[4 g4 + p/4][16 db + 4 (p%4)] and receives V[4 g4 .. +3][16 db + p]
    int voff[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) {
        const int rl = 4 * g4 + (r16 >> 2);
        const int ch = 2 * db + ((r16 & 3) >> 1);
        voff[db] = rl * (CH * 16) + ((ch ^ swz16<CH>(rl)) << 4) + (r16 & 1) * 8;
    }

    auto tile_step = [&](auto bufc, int it) {
        constexpr int BUF = decltype(bufc)::value;
        const char* kt = sm.k[BUF];
        const char* vt = sm.v[BUF];
        const bool gist_tile = it < ngt;
        const int j0 = row_step_first(walk, it, BN);  // compact index or position
        const int kind = row_step_kind(walk, it, BN, wrow0, wrow0 + 31, lo_wlast);
        if (kind == STEP_SKIP) return;

        // ---- S^T = K Q^T : sa[kb][qb] register i is key j0 + 16 kb + 4 g4 + i, column = query qrow[qb].
        // The K fragments are read PFK groups ahead of the MFMAs that use them (each feeds both query blocks).
        f32x4 sa[2][2];
        {
            constexpr int N = 2 * KS, PFK = 2;  // group n: key block n / KS, k-step n % KS
            bf16x8 fk[N];
            auto fetch = [&](int n) __attribute__((always_inline)) {
                fk[n] = *(const bf16x8*)(kt + (n / KS) * 16 * CH * 16 + koff[n % KS]);
            };
#pragma unroll
            for (int n = 0; n < PFK; ++n) fetch(n);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int n = 0; n < N; ++n) {
                if (n + PFK < N) fetch(n + PFK);
                const int kb = n / KS, ks = n % KS;
                if (ks == 0) {
                    sa[kb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fk[n], qf[0][ks], f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
                    sa[kb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fk[n], qf[1][ks], f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
                } else {
                    sa[kb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fk[n], qf[0][ks], sa[kb][0], 0, 0, 0);
                    sa[kb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fk[n], qf[1][ks], sa[kb][1], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }

        // ---- mask.  Bit t of vis[qb]: does query qrow[qb] see the key at offset t from j0?  This lane holds the
        // offsets 16 kb + 4 g4 + i.
        if (kind == STEP_MASKED) {
            auto below = [](int n) { return n >= 32 ? ~0u : n <= 0 ? 0u : (1u << n) - 1u; };  // bits 0 .. n-1
            unsigned gm = 0u;
            if (!gist_tile) gm = (unsigned)__builtin_amdgcn_ballot_w64(lane < BN && is_always(s, j0 + lane));
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                unsigned vis;
                if (gist_tile) {
                    vis = below(nfar - j0);
                } else {
                    const int d0 = qrow[qb] - j0;  // offsets d0 - span_q .. d0 are in the window, offsets <= d0 causal
                    vis = below(d0 + 1) & (~below(d0 - span_q[qb]) | gm);
                }
                vis >>= 4 * g4;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (!((vis >> (16 * kb + i)) & 1u)) sa[kb][qb][i] = -INFINITY;
            }
        }

        // ---- online softmax: a query row is spread over the 4 lanes r16 + 16 g4 (4 keys of every 16 each), so the
        // reference m[qb] is kept identical on those lanes and the row sum l[qb] is a per-lane partial
        u32x4 pk[2];
        float ls[2];
        auto exps = [&](int qb, float mc) __attribute__((always_inline)) {
            float p[8];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 4; ++i) p[4 * kb + i] = __builtin_amdgcn_exp2f(fmaf(sa[kb][qb][i], c, -mc));
            ls[qb] = ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
#pragma unroll
            for (int t = 0; t < 4; ++t) pk[qb][t] = pack_bf16x2(p[2 * t], p[2 * t + 1]);
        };
        bool with_max = need_max;
        if (!with_max) {
            exps(0, m[0] * c);
            exps(1, m[1] * c);
            with_max = __builtin_amdgcn_ballot_w64(!(ls[0] <= kBigSum) || !(ls[1] <= kBigSum)) != 0ull;
        }
        if (with_max) {
            bool any_inf = false;
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                float mx = sa[0][qb][0];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) mx = fmaxf(mx, sa[kb][qb][i]);
                mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
                mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
                const bool grow = (mx - m[qb]) * c > kLazy;
                if (__builtin_amdgcn_ballot_w64(grow) != 0ull) {
                    const float m_new = grow ? mx : m[qb];
                    const float alpha = grow ? __builtin_amdgcn_exp2f((m[qb] - m_new) * c) : 1.f;  // m = -inf gives 0
                    l[qb] *= alpha;
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int i = 0; i < 4; ++i) o[db][qb][i] *= alpha;
                    m[qb] = m_new;
                }
                exps(qb, (m[qb] == -INFINITY ? 0.f : m[qb]) * c);
                any_inf = any_inf || m[qb] == -INFINITY;
            }
            need_max = __builtin_amdgcn_ballot_w64(any_inf) != 0ull;
        }
        l[0] += ls[0];
        l[1] += ls[1];

        // ---- O^T += V^T P^T : contraction slot 8 g4 + 4 kb + i is key 16 kb + 4 g4 + i, on both operands.
        // The V^T fragments (two transposing reads each) run PFV blocks ahead of their MFMAs.
        {
            constexpr int PFV = 2;
            s16x4 lo[DB], hi[DB];
            auto fetch = [&](int db) __attribute__((always_inline)) {
                const char* a = vt + voff[db];
                lo[db] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)a);
                hi[db] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(a + 16 * CH * 16));
            };
#pragma unroll
            for (int db = 0; db < PFV; ++db) fetch(db);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                if (db + PFV < DB) fetch(db + PFV);
                const bf16x8 vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo[db], hi[db], 0, 1, 2, 3, 4, 5, 6, 7));
                o[db][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, __builtin_bit_cast(bf16x8, pk[0]), o[db][0], 0, 0, 0);
                o[db][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, __builtin_bit_cast(bf16x8, pk[1]), o[db][1], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
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

    // ---- epilogue: the row sums are spread over the 4 lanes of a query; normalise, store O and LSE
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        float lt = l[qb];
        lt += __shfl_xor(lt, 16, 64);
        lt += __shfl_xor(lt, 32, 64);
        float inv = 1.f / lt;
        if (s.vscale) inv *= s.vscale[hk];  // the stored values stand for V * vscale
        if (qrow[qb] < L) {
            const size_t orow = ((size_t)b * s.Hq + hq) * s.qhs + (qrow[qb] - qpos0);
            const size_t ooff = s.q_rs ? (size_t)b * s.q_bs + (size_t)hq * s.q_hs + (size_t)(qrow[qb] - qpos0) * s.q_rs : orow * Dt;
            bf16_t* op = out + ooff + 4 * g4;
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                if (16 * db + 4 * g4 >= Dt) continue;
                u32x2 w2;
                w2[0] = pack_bf16x2(o[db][qb][0] * inv, o[db][qb][1] * inv);
                w2[1] = pack_bf16x2(o[db][qb][2] * inv, o[db][qb][3] * inv);
                *(u32x2*)(op + 16 * db) = w2;
            }
            if (g4 == 0) lse[orow] = m[qb] * sc + __builtin_amdgcn_logf(lt) * 0.6931471805599453f;
        }
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
                                                  s, nq, NoDocs{});
    };
    if (s.D <= 64) gen ? go(fwd_mfma_kernel<64, true, PLAIN>) : go(fwd_mfma_kernel<64, false, PLAIN>);
    else gen ? go(fwd_mfma_kernel<128, true, PLAIN>) : go(fwd_mfma_kernel<128, false, PLAIN>);
    return hipGetLastError();
}

hipError_t launch_fwd_mfma_ragged(const void* q, const void* k, const void* v, void* out, float* lse, const AttnShape& s,
                                  const RaggedSeqs& seqs, hipStream_t st) {
    const int nq = (s.Lq + BM - 1) / BM;  // tiles of the longest possible chunk; shorter sequences skip theirs
    const long nblk = (long)nq * s.Hq * s.B;
    if (nblk > 0x7fffffffL) return hipErrorInvalidValue;
    const bool gen = s.S != 0 || s.umode != 0;
    auto go = [&](auto kern) {
        kern<<<dim3((unsigned)nblk), NT, 0, st>>>((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)out, lse,
                                                  s, nq, seqs);
    };
    if (s.D <= 64) gen ? go(fwd_mfma_kernel<64, true, RAGGED>) : go(fwd_mfma_kernel<64, false, RAGGED>);
    else gen ? go(fwd_mfma_kernel<128, true, RAGGED>) : go(fwd_mfma_kernel<128, false, RAGGED>);
    return hipGetLastError();
}

hipError_t launch_fwd_mfma_pack(const void* q, const void* k, const void* v, void* out, float* lse, const AttnShape& s,
                                const int* cu, int ndocs, hipStream_t st) {
    // long documents first: their long tiles are the ones that should not start last
    const bool gen = s.S != 0 || s.umode != 0;
    std::vector<int> order;
    for (int d = 0; d < ndocs; ++d)
        if (cu[d + 1] > cu[d]) order.push_back(d);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return cu[a + 1] - cu[a] > cu[b + 1] - cu[b]; });
    for (size_t at = 0; at < order.size(); at += kMaxDocs) {
        DocTab t;
        memset(&t, 0, sizeof t);
        t.n = (int)std::min<size_t>(kMaxDocs, order.size() - at);
        long nblk = 0;
        for (int i = 0; i < t.n; ++i) {
            const int d = order[at + i];
            t.c0[i] = cu[d];
            t.len[i] = cu[d + 1] - cu[d];
            t.blk0[i] = (int)nblk;
            nblk += (long)((t.len[i] + BM - 1) / BM) * s.Hq;
        }
        if (nblk > 0x7fffffffL) return hipErrorInvalidValue;
        t.blk0[t.n] = (int)nblk;
        auto go = [&](auto kern) {
            kern<<<dim3((unsigned)nblk), NT, 0, st>>>((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)out,
                                                      lse, s, 0, t);
        };
        if (s.D <= 64) gen ? go(fwd_mfma_kernel<64, true, PACK>) : go(fwd_mfma_kernel<64, false, PACK>);
        else gen ? go(fwd_mfma_kernel<128, true, PACK>) : go(fwd_mfma_kernel<128, false, PACK>);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace unigist
