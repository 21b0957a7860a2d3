// Backward kernels of gist-masked attention for gfx950 (bf16 MFMA, fp32 accumulation), no atomics.
//
// With P_ij = exp(scale S_ij - lse_i) on the visible pairs of Sec. 4.1, Eq. 3:
//   delta_i = dO_i . O_i                      dV_j = sum_i P_ij dO_i
//   dP_ij   = dO_i . V_j                      dS_ij = P_ij (dP_ij - delta_i)
//   dQ_i    = scale sum_j dS_ij K_j           dK_j = scale sum_i dS_ij Q_i   (summed over the q heads of a group)
//
// Launch sequence (all on the caller's stream):
//   1. delta_kernel         delta = rowsum(dO * O)
//   2. dkdv_kernel<GIST>    one workgroup per (compact gist tile, segment of query chunks): the pairs whose
//                           gist lies left of the query chunk's window phase; fp32 partials to the workspace
//   3. gist_reduce_kernel   sums the segments of a gist tile in a fixed order
//   4. dkdv_kernel<WINDOW>  one workgroup per contiguous 128-key tile: the pairs of the window phase; its
//                           epilogue adds the reduced gist-phase sums to the gist rows and writes dK, dV
//   5. dq_kernel            one workgroup per 128-query tile, same tile walk as the forward
// Every (query, key) pair is handled by exactly one of the two dkdv phases: a query chunk c (64 rows) sees
// the sinks and gists at positions < far(c) = floor(win_lo(64c) / 128) * 128 in the gist phase (win_lo = first
// position of a row's local window) and every key >= far(c) in the window phase.
//
// All contractions run on v_mfma_f32_16x16x32_bf16 (operand layouts in mfma_common.h); a wave always works on
// two 16-wide blocks at once so that every fragment read from LDS feeds two MFMAs.
// dkdv: a wave owns 32 keys as two 16-key blocks (a key is a column, spread over four lanes), K and V fragments
// stay in registers, Q / dO chunks are staged in LDS and read both row-wise (S = Q K^T, dP = dO V^T) and through
// transposing LDS reads (dV^T += dO^T P, dK^T += Q^T dS); the S/dP accumulators of the two 16-row halves of a
// query block are already the B operands of the last two.
// dq: forward-shaped; S^T = K Q^T and dP^T = V dO^T for the wave's two 16-row query blocks, dQ^T += K^T dS^T.
#include <string.h>

#include <algorithm>
#include <type_traits>
#include <vector>

#include "mfma_common.h"
#include "plan.h"

namespace unigist {
namespace {

constexpr int NT = 256;
constexpr int BMQ = kDqBm;  // query rows per dq workgroup
constexpr int BNQ = kDqBn;  // keys per dq step
constexpr int PFS = 2, PFT = 2;  // dq: LDS fragment reads issued this many MFMA groups ahead (S/dP phase, dQ phase)
constexpr float kLog2e = 1.4426950408889634f;

// bits 0 .. n-1 set (none for n <= 0, all for n >= 32)
__device__ __forceinline__ unsigned below_bits(int n) { return n >= 32 ? ~0u : n <= 0 ? 0u : (1u << n) - 1u; }

// chunk steps (per kv head) of the gist phase of one sequence: every gist tile is walked by the chunks from the
// first one that has it left of its window phase to the last
long gist_chunk_steps(const AttnShape& s) {
    BwdPlan p;
    plan_counts(s, p, 32);
    long n = 0;
    for (int t = 0; t < p.n_gt; ++t) n += p.NC - first_chunk_with_more_far(s, p.NC, t * BNK);
    return n;
}

// Segment length (query chunks per gist-phase workgroup) for a launch with `steps` chunk steps in total over all
// (batch, kv head) pairs: 32 chunks (x Hq/Hkv heads = 128 steps per workgroup) balance the last round of a 32K
// sequence; a launch that could not give the 512 workgroup slots of the chip (2 per CU) about five such rounds
// gets segments of 16 (one 8K sequence: 10 % faster, a 32K pack of five documents: 2 %; 8 and 4 were no better,
// their partial sums cost what the balance gains).
int pick_segc(long steps) { return steps / (512 * 5) >= 32 ? 32 : 16; }

BwdPlan make_plan(const AttnShape& s) {
    BwdPlan p;
    plan_counts(s, p, pick_segc(gist_chunk_steps(s) * s.B * s.Hkv));
    plan_slots(s, p);
    plan_order(s, p);
    const size_t a = 255;
    size_t off = ((size_t)s.B * s.Hq * s.L * sizeof(float) + a) & ~a;
    p.off_lse2 = off;  // lse * log2(e), written by the delta pass
    off += ((size_t)s.B * s.Hq * s.L * sizeof(float) + a) & ~a;
    p.off_part = off;  // one [2][D][BNK] fp32 block per (batch, kv head, segment, compact tile the segment reaches)
    off += (size_t)s.B * s.Hkv * p.slot0[p.nseg] * 2 * padded_head_dim(s.D) * BNK * sizeof(float);
    off = (off + a) & ~a;
    p.off_comp = off;  // their sums over the segments: one block per (batch, kv head, compact tile)
    off += (size_t)s.B * s.Hkv * p.n_gt * 2 * padded_head_dim(s.D) * BNK * sizeof(float);
    p.total = (off + a) & ~a;
    return p;
}

// ------------------------------------------------------------------ 1. delta
template <int D>
__global__ __launch_bounds__(NT) void delta_kernel(const bf16_t* __restrict__ out, const bf16_t* __restrict__ dout,
                                                  const float* __restrict__ lse, float* __restrict__ delta,
                                                  float* __restrict__ lse2, long nrows, int L, int qhs, int Hq,
                                                  long long q_bs, long long q_hs, int q_rs, int Dt) {
    constexpr int LPR = D / 8;  // lanes per row, 16 bytes each (Dt <= D elements per row in memory)
    const long row = (long)blockIdx.x * (NT / LPR) + threadIdx.x / LPR;  // dense: (b, h, i) -> (b Hq + h) L + i
    const int sub = threadIdx.x % LPR;
    const long grow = L == qhs ? row : (row / L) * qhs + row % L;        // the same row in the caller's tensors
    float acc = 0.f;
    if (row < nrows) {
        // element offset of the row in out / dout: dense, or with the caller's explicit strides (q_rs != 0)
        const long bh = row / L;
        const long eoff = q_rs ? (bh / Hq) * q_bs + (bh % Hq) * q_hs + (row % L) * (long)q_rs : grow * Dt;
        u32x4 a = {0u, 0u, 0u, 0u}, b = {0u, 0u, 0u, 0u};
        if (sub * 8 < Dt) {
            a = *(const u32x4*)(out + eoff + sub * 8);
            b = *(const u32x4*)(dout + eoff + sub * 8);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            acc += __uint_as_float(a[t] << 16) * __uint_as_float(b[t] << 16);
            acc += __uint_as_float(a[t] & 0xffff0000u) * __uint_as_float(b[t] & 0xffff0000u);
        }
    }
    // reduce over the LPR lanes of a row (LPR is 8 or 16, rows are aligned to LPR lanes)
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) acc += __shfl_xor(acc, off, 64);
    if (row < nrows && sub == 0) {
        delta[row] = -acc;               // stored negated: the consumers add it (dK/dV: as the dP accumulator's start)
        lse2[row] = lse[grow] * kLog2e;  // the exponent base the dK/dV and dQ kernels subtract
    }
}

// ------------------------------------------------------------------ 2./4. dK, dV
template <int D>
struct DkdvSmem {
    // the rows' lse * log2(e) and -delta first: with the two 64 KB of tiles in front of them their addresses would
    // not fit the 16-bit offset field of the LDS instructions and cost a vector instruction per read
    float lse2[2][MQ];
    float delta[2][MQ];
    // two stages of a 64-row Q chunk and dO chunk (rows unpadded, 16-byte chunks swizzled)
    char q[2][MQ * D * 2];
    char g[2][MQ * D * 2];
};

// GEN = false (here and in dq_kernel) is the layout without sinks and with the sliding window: the mask
// helpers then fold to their short forms at compile time.
// PACK = true (here and in dq_kernel): the launch covers the documents of a packed buffer (docs), s_arg is the shape
// of the whole pack, delta and lse2 have the layout of the caller's lse ([Hq, T]), and every document has its
// own run of slots in part and comp.
// QSTR = true: q and dout have the explicit strides of s_arg (q_bs, q_hs, q_rs) instead of the dense layout.  Tensors
// whose head dimension s.D is smaller than the D the kernel is built for (any multiple of 8) also come this way, with
// the strides of their dense layout: rows in memory are s.D elements long, LDS tiles and fragments have D columns,
// of which those from s.D on are zero in the K and V fragments (so they add nothing to S and dP) and are never stored.
template <int D, bool GIST, bool GEN, bool PACK, bool QSTR = false>
__global__ __launch_bounds__(NT, 2) void dkdv_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                    const bf16_t* __restrict__ v, const float* __restrict__ lse2,
                                                    const bf16_t* __restrict__ dout, const float* __restrict__ delta,
                                                    bf16_t* __restrict__ dk, bf16_t* __restrict__ dv,
                                                    float* __restrict__ part, const float* __restrict__ comp,
                                                    AttnShape s_arg, BwdPlan pl,
                                                    std::conditional_t<PACK, DocTab, NoDocs> docs) {
    AttnShape s = s_arg;
    if constexpr (!GEN) {
        s.S = 0;
        s.umode = 0;
    }
    int n = blockIdx.x;
    if constexpr (PACK) {  // the document becomes the whole problem
        const int d = doc_of_block(docs, n);
        n -= docs.blk0[d];
        s = doc_view(s, docs.len[d]);
        plan_counts(s, pl, pl.segc);  // pl arrives with the launch's segment length only
        const size_t ro = (size_t)docs.c0[d] * (QSTR ? s.D : D);
        const size_t qro = QSTR ? (size_t)docs.c0[d] * s.q_rs : ro;
        q += qro;
        k += ro;
        v += ro;
        dout += qro;
        dk += ro;
        dv += ro;
        lse2 += docs.c0[d];
        delta += docs.c0[d];
        part += (size_t)docs.part0[d] * (2 * D * BNK);
        comp += (size_t)docs.comp0[d] * (2 * D * BNK);
    }
    constexpr int KS = D / 32, DB = D / 16, CH = D / 8;  // 16x16x32 MFMA: k-steps of 32, 16-row blocks of dK^T / dV^T
    constexpr int RPI = 64 / CH;        // chunk rows covered by one direct-load instruction
    constexpr int IPW = MQ / RPI / 4;   // such instructions per wave, per matrix, per step
    constexpr int ROWB = CH * 16;       // bytes per row
    __shared__ __attribute__((aligned(1024))) DkdvSmem<D> sm;

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r16 = lane & 15, g4 = lane >> 4;  // the lane's place in a 16x16x32 operand
    const int L = s.L;
    const int G = s.Hq / s.Hkv;
    const float c = s.scale * kLog2e;
    const int Dt = QSTR ? s.D : D;  // elements per row in memory

    // ---- which (batch, kv head) and which unit of work.  Workgroup ids go round-robin over the 8
    // XCDs, so with id % 8 selecting the (batch, kv head) pair every XCD gets the same amount of work
    // and one head's Q/dO stream stays in one XCD's L2.
    const int NP = s.B * s.Hkv;
    int pr, unit;
    if ((NP & 7) == 0) {
        const int mm = n >> 3;
        pr = (n & 7) + 8 * (mm % (NP >> 3));
        unit = mm / (NP >> 3);
    } else {
        pr = n % NP;
        unit = n / NP;
    }
    const int b = pr / s.Hkv, hk = pr % s.Hkv;

    // ---- which keys, which query chunks
    int tile, c_lo, c_hi;  // chunks c_lo .. c_hi inclusive
    int seg = 0;
    int slot = 0, nslots = 0;  // gist phase: the workgroup's slot among the nslots partial sums of its (batch, kv head)
    if (GIST) {
        // One workgroup per (segment, compact tile the segment reaches), segment-major, late (fully populated)
        // segments first: the workgroups running together on an XCD then stream the same Q/dO chunks of the same
        // head through its L2.  A dense launch puts the shorter units -- tiles first reached inside their segment --
        // at the end, longest first, where they even out the last round (gist_unit); a document of a pack counts
        // the slots of its own plan from the last segment down.
        seg = pl.nseg - 1;
        if constexpr (PACK) {  // the document's plan has no table: sum the segments' tile counts
            int rem = unit, nt;
            while ((nt = seg_tiles(s, pl, seg)) <= rem && seg > 0) {
                rem -= nt;
                --seg;
            }
            tile = rem;
            slot = tile;
            for (int sg = 0; sg < seg; ++sg) slot += seg_tiles(s, pl, sg);
            nslots = slot - tile + nt + (unit - rem);
        } else {
            nslots = pl.slot0[pl.nseg];
            gist_unit(pl, unit, seg, tile);
            slot = pl.slot0[seg] + tile;
        }
        const ChunkRange cr = gist_tile_chunks(s, pl, tile, seg);
        c_lo = cr.c_lo;
        c_hi = cr.c_hi;
        if (c_lo > c_hi) return;  // cannot happen for a slot of the plan (uniform exit all the same)
    } else {
        tile = unit;
        const ChunkRange cr = window_tile_chunks(s, pl, tile);
        c_lo = cr.c_lo;
        c_hi = cr.c_hi;
    }
    const int key0 = tile * BNK + 32 * w;      // first key (position, or compact gist index) of the wave
    // The wave's 32 keys are two 16-key blocks kb = 0, 1; this lane's keys are key0 + 16 kb + r16.
    // K, V fragments (B operands): lane holds K[key[kb]][32 ks + 8 g4 .. +7].
    int key[2], span_j[2];
    bool gist_lane[2];
    bf16x8 kf[2][KS], vf[2][KS];
    f32x4 akT[DB][2], avT[DB][2];  // dK^T, dV^T: register i of [db][kb] is d = 16 db + 4 g4 + i, column = key[kb]
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        key[kb] = key0 + 16 * kb + r16;
        int krow;                              // row of K/V holding it
        if (GIST) {
            const int atot = count_always(s, L);  // sinks + gists, >= 1 whenever a gist workgroup exists
            krow = pos_of_always(s, min(key[kb], atot - 1));
        } else {
            krow = min(key[kb], L - 1);
        }
        gist_lane[kb] = GIST ? true : is_always(s, key[kb]);  // a sink or a gist: visible to every later row
        // the key stays in the window for span_j more rows (W - 1 for every key in the sliding mode)
        span_j[kb] = 0;
        if constexpr (!GIST && GEN) span_j[kb] = key[kb] < L ? win_hi(s, key[kb]) - key[kb] : 0;
        const size_t base = (((size_t)b * s.Hkv + hk) * s.kvhs + krow) * Dt + 8 * g4;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 zk = {0u, 0u, 0u, 0u}, zv = {0u, 0u, 0u, 0u};  // columns past the tensors' head dimension are zero
            if (!QSTR || 32 * ks + 8 * g4 < Dt) {
                zk = *(const u32x4*)(k + base + 32 * ks);
                zv = *(const u32x4*)(v + base + 32 * ks);
            }
            kf[kb][ks] = __builtin_bit_cast(bf16x8, zk);
            vf[kb][ks] = __builtin_bit_cast(bf16x8, zv);
        }
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            akT[db][kb] = zero4();
            avT[db][kb] = zero4();
        }
    }
    // last row that has the wave's first key in its window
    int hi_w0 = 0;
    if constexpr (!GIST) hi_w0 = win_hi(s, min(key0, L - 1));

    // ---- staging of the Q / dO chunk: direct global->LDS loads
    const int nch = c_hi - c_lo + 1;
    const int nsteps = nch * G;
    // Load slot i of wave w covers the chunk rows (w * IPW + i) * RPI + lane / CH.  The swizzle repeats every 16 rows and
    // w * IPW * RPI is a multiple of 16, so the lane's byte offset inside the slot's rows takes only NLP different
    // values; everything else of the address is wave-uniform or an immediate.
    // They are recomputed from the lane id at every use: kept in registers across the step they would be
    // spilled, and a reload from scratch waits on the same counter as the direct loads still in flight.
    constexpr int NLP = 16 / RPI;
    static_assert(IPW * RPI == 16 && NLP == IPW, "a wave stages 16 rows per matrix and step");
    auto issue = [&](int g, int cc, int buf) __attribute__((always_inline)) {
        int ln = lane;
        asm volatile("" : "+v"(ln));  // opaque: keeps the address arithmetic below inside this call
        const int lrow_ = ln / CH;
        int lanepart[NLP];
        const unsigned rsb = QSTR ? (unsigned)s.q_rs * 2u : (unsigned)ROWB;  // bytes between consecutive rows in q / dout
#pragma unroll
        for (int i = 0; i < NLP; ++i) {
            int sc = (ln % CH) ^ swz16<CH>(i * RPI + lrow_);  // the source chunk of this lane's LDS position
            if (QSTR && 8 * sc >= Dt) sc = 0;                  // a chunk the rows do not have: any chunk will do
            lanepart[i] = lrow_ * (int)rsb + (sc << 4);
        }
        const size_t hb = ((size_t)b * s.Hq + hk * G + g) * (PACK ? s.qhs : L);  // wave-uniform; workspace rows
        // the head in the caller's tensors
        const size_t hg = QSTR ? (size_t)b * s.q_bs + (size_t)(hk * G + g) * s.q_hs : ((size_t)b * s.Hq + hk * G + g) * s.qhs * D;
        const char* qh = (const char*)(q + hg);
        const char* gh = (const char*)(dout + hg);
        if (cc * MQ + MQ <= L) {  // the whole chunk exists (wave-uniform)
            const size_t cb = (size_t)(cc * MQ + w * IPW * RPI) * rsb;
#pragma unroll
            for (int i = 0; i < IPW; ++i) {
                const unsigned off = (unsigned)lanepart[i % NLP] + (unsigned)(i * RPI) * rsb;
                g2l16(qh + cb + off, &sm.q[buf][(w * IPW + i) * 1024]);
                g2l16(gh + cb + off, &sm.g[buf][(w * IPW + i) * 1024]);
            }
        } else {  // last chunk of a ragged sequence: rows past the end shadow the last row
#pragma unroll
            for (int i = 0; i < IPW; ++i) {
                const int rr = (w * IPW + i) * RPI + lrow_;
                const int row = min(cc * MQ + rr, L - 1);
                const unsigned off = (unsigned)row * rsb + (unsigned)(lanepart[i % NLP] - lrow_ * (int)rsb);
                g2l16(qh + off, &sm.q[buf][(w * IPW + i) * 1024]);
                g2l16(gh + off, &sm.g[buf][(w * IPW + i) * 1024]);
            }
        }
        if (w < 2) {  // wave 0: the 64 rows' lse2, wave 1: their delta (one 4-byte direct load per lane)
            const int row = min(cc * MQ + ln, L - 1);
            const float* src = (w == 0 ? lse2 : delta) + hb + row;
            float* dst = w == 0 ? sm.lse2[buf] : sm.delta[buf];
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)dst, 4, 0, 0);
        }
    };
    // Per-lane LDS offsets.  Row-wise read of chunk row r16 (+16 qs + 32 qb), 16-byte chunk 4 ks + g4: the swizzle
    // XORs the chunk bits, so the offset for k-step ks is roff0 ^ (ks << 6); likewise the transposing read of the
    // 16-column block db sits at toff0 ^ (db << 5).  Only the two bases stay live across the kernel (registers
    // are what this kernel is short of); the XORs are redone per query block.
    const int roff0 = row16_lane_off<CH>(0);
    const int toff0 = tr16_lane_off16<CH>(0);

    // one step on LDS stage BUF (a compile-time constant: LDS addresses = lane register + immediate)
    auto do_step = [&](auto bufc, int cc) __attribute__((always_inline)) {
        constexpr int BUF = decltype(bufc)::value;
        const char* qt = sm.q[BUF];
        const char* gt = sm.g[BUF];
        const int q0 = cc * MQ;

        int nfar = 0;
        if (GIST) nfar = nfar_of_chunk(s, cc);  // compact entries visible to this chunk: index < nfar

#pragma unroll
        for (int qb = 0; qb < MQ / 32; ++qb) {
            const int qb0 = q0 + 32 * qb;  // first query row of the block
            // every row left of every key of the wave: nothing to do (the gist phase never skips)
            if (!GIST && UNIGIST_WINDOW_BLOCK_SKIPPED(key0, qb0)) continue;

            // offsets of this query block; the XORs below touch bits 5..7 only, the block offset bits >= 13
            int rb = roff0 + 32 * qb * ROWB, tb = toff0 + 32 * qb * ROWB;
            asm volatile("" : "+v"(rb), "+v"(tb));  // opaque: the derived offsets are not hoisted out of the loop

            // ---- S = Q K^T, dP = dO V^T for the two 16-row halves qs of the block and the two 16-key blocks kb:
            // register i of sa[qs][kb] is query qb0 + 16 qs + 4 g4 + i, column = key[kb].  Every Q and dO fragment
            // serves both key blocks.  The fragment reads are issued PF groups ahead of the MFMAs that consume them;
            // the scheduling barriers keep the compiler from sinking them back to just before their use, where every
            // MFMA would wait for a full LDS round trip.
            // dP starts from -delta of its rows (the prepass stores delta negated), so dS = P (dP - delta) needs no
            // subtraction afterwards.
            f32x4 sa[2][2], dp[2][2];
#pragma unroll
            for (int qs = 0; qs < 2; ++qs) {
                const f32x4 d4 = *(const f32x4*)(&sm.delta[BUF][32 * qb + 16 * qs + 4 * g4]);
                dp[qs][0] = d4;
                dp[qs][1] = d4;
            }
            {
                constexpr int N = 2 * KS, PF = 1;  // group n: half n / KS, k-step n % KS
                bf16x8 fq[N], fg[N];
                auto fetch = [&](int n) __attribute__((always_inline)) {
                    const int ro = (rb ^ ((n % KS) << 6)) + 16 * (n / KS) * ROWB;
                    fq[n] = *(const bf16x8*)(qt + ro);
                    fg[n] = *(const bf16x8*)(gt + ro);
                };
#pragma unroll
                for (int n = 0; n < PF; ++n) fetch(n);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int n = 0; n < N; ++n) {
                    if (n + PF < N) fetch(n + PF);
                    const int qs = n / KS, ks = n % KS;
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb) {
                        sa[qs][kb] = mfma16(fq[n], kf[kb][ks], ks == 0 ? zero4() : sa[qs][kb]);
                        dp[qs][kb] = mfma16(fg[n], vf[kb][ks], dp[qs][kb]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // ---- P and dS
            bool masked;
            if (GIST) masked = UNIGIST_GIST_BLOCK_MASKED(key0, qb0, nfar, L);
            else masked = UNIGIST_WINDOW_BLOCK_MASKED(key0, qb0, hi_w0, L);
            f32x4 l4[2];
#pragma unroll
            for (int qs = 0; qs < 2; ++qs) l4[qs] = *(const f32x4*)(&sm.lse2[BUF][32 * qb + 16 * qs + 4 * g4]);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int qs = 0; qs < 2; ++qs)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        sa[qs][kb][i] = __builtin_amdgcn_exp2f(fmaf(sa[qs][kb][i], c, -l4[qs][i]));
                if (masked) {
                    // bit t of vis: does query qb0 + t see this lane's key[kb]?  The visible queries are a range of
                    // offsets (those inside the sequence; for a raw key those that still have it in their window),
                    // cut at the diagonal.  This lane holds the offsets 16 qs + 4 g4 + i.
                    unsigned vis;
                    const unsigned inside = below_bits(L - qb0);
                    if (GIST) {
                        vis = key[kb] < nfar ? inside : 0u;
                    } else {
                        const int d0 = qb0 - key[kb];  // distance i - j of the block's first query to the key
                        const int span = GEN ? span_j[kb] : s.W - 1;
                        const unsigned win = gist_lane[kb] ? ~0u : below_bits(span - d0 + 1);
                        vis = inside & win & ~below_bits(-d0);
                    }
                    vis >>= 4 * g4;
#pragma unroll
                    for (int qs = 0; qs < 2; ++qs)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (!((vis >> (16 * qs + i)) & 1u)) sa[qs][kb][i] = 0.f;
                }
#pragma unroll
                for (int qs = 0; qs < 2; ++qs)
#pragma unroll
                    for (int i = 0; i < 4; ++i) dp[qs][kb][i] *= sa[qs][kb][i];
            }
            // ---- dV^T += dO^T P,  dK^T += Q^T dS : contraction slot 8 g4 + 4 qs + i is query 16 qs + 4 g4 + i of the
            // block, on both operands; every dO^T and Q^T fragment serves both key blocks
            bf16x8 pb[2], sb[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                pb[kb] = pack44(sa[0][kb], sa[1][kb]);
                sb[kb] = pack44(dp[0][kb], dp[1][kb]);
            }
            {
                constexpr int PF = 2;
                bf16x8 fg[DB], fq[DB];
                auto fetch = [&](int db) __attribute__((always_inline)) {
                    const int to = tb ^ (db << 5);
                    fg[db] = tr16_frag16<CH>(gt + to, 0);
                    fq[db] = tr16_frag16<CH>(qt + to, 0);
                };
#pragma unroll
                for (int db = 0; db < PF; ++db) fetch(db);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    if (db + PF < DB) fetch(db + PF);
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb) {
                        avT[db][kb] = mfma16(fg[db], pb[kb], avT[db][kb]);
                        akT[db][kb] = mfma16(fq[db], sb[kb], akT[db][kb]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    };

    // Step t handles query chunk c_lo + t % nch of query head t / nch of the group; both walks (the chunk being
    // computed, the chunk being fetched one step ahead) are kept as (head, chunk) counters instead of dividing.
    int gi = 0, ci = c_lo;  // what the next issue() fetches
    int cs = c_lo;          // what the next do_step() computes
    auto next_issue = [&]() __attribute__((always_inline)) {
        if (++ci > c_hi) {
            ci = c_lo;
            ++gi;
        }
    };
    auto next_step = [&]() __attribute__((always_inline)) {
        if (++cs > c_hi) cs = c_lo;
    };
    issue(gi, ci, 0);
    next_issue();
    for (int step = 0; step < nsteps; step += 2) {
        wait_vmem();
        __syncthreads();
        if (step + 1 < nsteps) {
            issue(gi, ci, 1);
            next_issue();
        }
        do_step(std::integral_constant<int, 0>{}, cs);
        next_step();
        if (step + 1 < nsteps) {
            wait_vmem();
            __syncthreads();
            if (step + 2 < nsteps) {
                issue(gi, ci, 0);
                next_issue();
            }
            do_step(std::integral_constant<int, 1>{}, cs);
            next_step();
        }
    }

    // ---- epilogue: register i of [db][kb] is d = 16 db + 4 g4 + i of key[kb]
    if (GIST) {
        // fp32 partials, transposed: [dK^T | dV^T][d][BNK keys]
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            float* o = part + (((size_t)b * s.Hkv + hk) * nslots + slot) * (2 * D * BNK) + 32 * w + 16 * kb + r16;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int d = 16 * db + 4 * g4 + i;
                    o[(size_t)d * BNK] = akT[db][kb][i] * s.scale;
                    o[(size_t)(D + d) * BNK] = avT[db][kb][i];
                }
        }
    } else {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            bool added = false;
            if (gist_lane[kb] && pl.n_gt > 0) {
                // add what the gist phase collected for this row (zero if no chunk saw it from afar)
                const int gi = count_always(s, key[kb]);  // its index in the compact list of sinks and gists
                const int gt = gi / BNK;
                if (gt < pl.n_gt && key[kb] < L) {
                    const float* cp = comp + (((size_t)b * s.Hkv + hk) * pl.n_gt + gt) * (2 * D * BNK) + gi % BNK;
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int d = 16 * db + 4 * g4 + i;
                            akT[db][kb][i] = akT[db][kb][i] * s.scale + cp[(size_t)d * BNK];
                            avT[db][kb][i] += cp[(size_t)(D + d) * BNK];
                        }
                    added = true;
                }
            }
            if (!added) {
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i = 0; i < 4; ++i) akT[db][kb][i] *= s.scale;
            }
            if (key[kb] < L) {
                const size_t base = (((size_t)b * s.Hkv + hk) * s.kvhs + key[kb]) * Dt + 4 * g4;
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    if (QSTR && 16 * db + 4 * g4 >= Dt) continue;
                    u32x2 a, bb;
                    a[0] = pack_bf16x2(akT[db][kb][0], akT[db][kb][1]);
                    a[1] = pack_bf16x2(akT[db][kb][2], akT[db][kb][3]);
                    bb[0] = pack_bf16x2(avT[db][kb][0], avT[db][kb][1]);
                    bb[1] = pack_bf16x2(avT[db][kb][2], avT[db][kb][3]);
                    *(u32x2*)(dk + base + 16 * db) = a;
                    *(u32x2*)(dv + base + 16 * db) = bb;
                }
            }
        }
    }
}

// ------------------------------------------------------------------ 3. sum the segments of each gist tile
__global__ __launch_bounds__(NT) void gist_reduce_kernel(const float* __restrict__ part, float* __restrict__ comp,
                                                        BwdPlan pl, AttnShape s, int per_tile) {
    // grid: x = slices of a tile's 2*D*BNK floats (four per thread, per_tile is a multiple of 4), y = tile,
    // z = (b, hk).  The segments are added in ascending order, so the result does not depend on the launch.
    const int gt = blockIdx.y;
    const int idx = 4 * (blockIdx.x * NT + threadIdx.x);
    if (idx >= per_tile) return;
    const int cf = first_chunk_with_more_far(s, pl.NC, gt * BNK);
    const float* pp = part + (size_t)blockIdx.z * pl.slot0[pl.nseg] * per_tile;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (cf < pl.NC)  // the tile has a slot in every segment from that of its first chunk on
        for (int sg = cf / pl.segc; sg < pl.nseg; ++sg) acc += *(const f32x4*)(pp + (size_t)(pl.slot0[sg] + gt) * per_tile + idx);
    *(f32x4*)(comp + ((size_t)blockIdx.z * pl.n_gt + gt) * per_tile + idx) = acc;
}

// The same for a packed launch.  grid: x = slot of comp (a document's slots are its (kv head, gist tile) pairs,
// docs.blk0 holds the first slot of each document), y = slice of the slot's 2*D*BNK floats.
__global__ __launch_bounds__(NT) void gist_reduce_pack_kernel(const float* __restrict__ part, float* __restrict__ comp,
                                                             AttnShape s_arg, int per_tile, int segc, DocTab docs) {
    const int idx = 4 * (blockIdx.y * NT + threadIdx.x);
    if (idx >= per_tile) return;
    const int d = doc_of_block(docs, blockIdx.x);
    const int t = blockIdx.x - docs.blk0[d];  // (kv head) * n_gt + gist tile
    const AttnShape s = doc_view(s_arg, docs.len[d]);
    BwdPlan pl;
    plan_counts(s, pl, segc);
    const int gt = t % pl.n_gt;
    const int cf = first_chunk_with_more_far(s, pl.NC, gt * BNK);
    int nslots = 0;
    for (int sg = 0; sg < pl.nseg; ++sg) nslots += seg_tiles(s, pl, sg);
    const float* pp = part + ((size_t)docs.part0[d] + (size_t)(t / pl.n_gt) * nslots) * per_tile;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (cf < pl.NC) {
        int base = 0;  // first slot of segment sg
        for (int sg = 0; sg < pl.nseg; ++sg) {
            if (sg >= cf / pl.segc) acc += *(const f32x4*)(pp + (size_t)(base + gt) * per_tile + idx);
            base += seg_tiles(s, pl, sg);
        }
    }
    *(f32x4*)(comp + ((size_t)docs.comp0[d] + t) * per_tile + idx) = acc;
}

// ------------------------------------------------------------------ 5. dQ
template <int D>
struct DqSmem {
    // two stages of a K tile and a V tile, rows unpadded, 16-byte chunks swizzled
    char k[2][BNQ * D * 2];
    char v[2][BNQ * D * 2];
};

template <int D, bool GEN, bool PACK, bool QSTR = false>
__global__ __launch_bounds__(NT, 2) void dq_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                  const bf16_t* __restrict__ v, const float* __restrict__ lse2,
                                                  const bf16_t* __restrict__ dout, const float* __restrict__ delta,
                                                  bf16_t* __restrict__ dq, AttnShape s_arg, int nq,
                                                  std::conditional_t<PACK, DocTab, NoDocs> docs) {
    AttnShape s = s_arg;
    if constexpr (!GEN) {
        s.S = 0;
        s.umode = 0;
    }
    int n = blockIdx.x;
    if constexpr (PACK) {
        const int d = doc_of_block(docs, n);
        n -= docs.blk0[d];
        s = doc_view(s, docs.len[d]);
        nq = (s.L + BMQ - 1) / BMQ;
        const size_t ro = (size_t)docs.c0[d] * (QSTR ? s.D : D);
        const size_t qro = QSTR ? (size_t)docs.c0[d] * s.q_rs : ro;
        q += qro;
        k += ro;
        v += ro;
        dout += qro;
        dq += qro;
        lse2 += docs.c0[d];
        delta += docs.c0[d];
    }
    constexpr int KS = D / 32, DB = D / 16, CH = D / 8;  // 16x16x32 MFMA: k-steps of 32, 16-row blocks of dQ^T
    constexpr int RPI = 64 / CH;
    constexpr int IPW = BNQ / RPI / 4;
    __shared__ __attribute__((aligned(1024))) DqSmem<D> sm;

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int g4 = lane >> 4;  // with r16 = lane % 16: the lane's place in a 16x16x32 operand
    const int G = s.Hq / s.Hkv, NP = s.B * s.Hkv;
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
    const int b = pr / s.Hkv, hk = pr % s.Hkv, hq = hk * G + g;
    const int L = s.L, rp1 = s.rp1;
    const int i0 = qt * BMQ, i1 = min(L, i0 + BMQ) - 1;
    const int wrow0 = i0 + 32 * w;  // first row of the wave; the lane's two rows are wrow0 + 16 qb + r16
    const int Dt = QSTR ? s.D : D;  // elements per row in memory (see dkdv_kernel)
    const char* kbytes = (const char*)(k + ((size_t)b * s.Hkv + hk) * s.kvhs * Dt);
    const char* vbytes = (const char*)(v + ((size_t)b * s.Hkv + hk) * s.kvhs * Dt);
    const float c = s.scale * kLog2e;

    // B operands Q and dO of this lane's two query rows, their lse * log2(e), and -delta in the 4 registers of an
    // accumulator: dP starts from it (the MFMA adds its C operand for free), so dS = P (dP - delta) needs no
    // subtraction.  The registers are made opaque so that they stay 4 registers instead of being rebuilt from one
    // value at every use.
    int qrow[2], span_q[2];
    size_t rowoff[2];
    bf16x8 qf[2][KS], gf[2][KS];
    float ls[2];
    f32x4 ndl[2];
    f32x4 acc[DB][2];  // dQ^T: register i of acc[db][qb] is d = 16 db + 4 g4 + i, column = query qrow[qb]
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        qrow[qb] = wrow0 + 16 * qb + (lane & 15);
        const int qrow_ld = min(qrow[qb], L - 1);
        span_q[qb] = qrow[qb] - win_lo(s, qrow[qb]);  // this row's window reaches span_q positions back
        // element offset of the row in the caller's q, dout and dq
        rowoff[qb] = QSTR ? (size_t)b * s.q_bs + (size_t)hq * s.q_hs + (size_t)qrow_ld * s.q_rs
                          : (((size_t)b * s.Hq + hq) * s.qhs + qrow_ld) * D;
        const size_t wrow = ((size_t)b * s.Hq + hq) * (PACK ? s.qhs : L) + qrow_ld;  // in the workspace
        const bf16_t* qp = q + rowoff[qb] + 8 * g4;
        const bf16_t* gp = dout + rowoff[qb] + 8 * g4;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 zq = {0u, 0u, 0u, 0u}, zg = {0u, 0u, 0u, 0u};  // columns past the tensors' head dimension are zero
            if (!QSTR || 32 * ks + 8 * g4 < Dt) {
                zq = *(const u32x4*)(qp + 32 * ks);
                zg = *(const u32x4*)(gp + 32 * ks);
            }
            qf[qb][ks] = __builtin_bit_cast(bf16x8, zq);
            gf[qb][ks] = __builtin_bit_cast(bf16x8, zg);
        }
        ls[qb] = lse2[wrow];
        const float dl = delta[wrow];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float x = dl;
            asm volatile("" : "+v"(x));
            ndl[qb][i] = x;
        }
#pragma unroll
        for (int db = 0; db < DB; ++db) acc[db][qb] = zero4();
    }

    const RowWalk walk = row_walk(s, i0, i1, BNQ);
    const int wstart = walk.wstart;                // first position of the window phase
    const int nfar = walk.nfar;                    // sinks and gists strictly left of it
    const int ngt = walk.ngt;
    const int ntiles = ngt + walk.nwin;
    const int lo_wlast = win_lo(s, wrow0 + 31);    // window start of the wave's last row
    const int S = s.S;

    // ---- staging (same scheme as the forward kernel)
    const int lrow = lane / CH;
    const int wv = __builtin_amdgcn_readfirstlane(w);
    int choff[IPW];
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
        const int sc = (lane % CH) ^ swz16<CH>((wv * IPW + i) * RPI + lrow);
        choff[i] = (!QSTR || 8 * sc < Dt) ? sc * 16 : 0;  // a chunk the rows do not have: any chunk will do
    }
    auto issue = [&](int it, int buf) {
        // Tile row rr is, in the gist phase, the (it * BNQ + rr)-th always-visible position, clamped to the last far
        // one; in the window phase position wstart + (it - ngt) * BNQ + rr, clamped to the last position.  The phase
        // only selects wave-uniform parameters, so the per-lane arithmetic has no branch.
        const bool gphase = it < ngt;
        const int a = gphase ? it * BNQ : wstart + (it - ngt) * BNQ;
        const int bnd = gphase ? nfar - 1 : L - 1;
        const int first_gist = gphase ? S : 0x7fffffff;  // entries from here on are gists
        const int gm = gphase ? rp1 : 1, go = gphase ? 1 : 0;
#pragma unroll
        for (int i = 0; i < IPW; ++i) {
            const int rr = (wv * IPW + i) * RPI + lrow;
            const int c = min(a + rr, bnd);
            int row;
            if constexpr (GEN)  // entry c >= S is gist c - S at S + (c - S)(r+1) + r; factors < 2^24 by the size limit
                row = c < first_gist ? c : S + mul24(c - S + 1, rp1) - 1;
            else
                row = mul24(c + go, gm) - go;
            const unsigned off = (unsigned)row * (unsigned)(Dt * 2) + (unsigned)choff[i];
            g2l16(kbytes + off, &sm.k[buf][(wv * IPW + i) * 1024]);
            g2l16(vbytes + off, &sm.v[buf][(wv * IPW + i) * 1024]);
        }
    };
    int roff[KS];  // row-wise read of tile row r16 (+16, +32, +48), chunk 4 ks + g4
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) roff[ks] = row16_lane_off<CH>(ks);
    int toff[DB];  // transposing read of K, 16-column block db
#pragma unroll
    for (int db = 0; db < DB; ++db) toff[db] = tr16_lane_off16<CH>(db);

    auto tile_step = [&](auto bufc, int it) {
        constexpr int BUF = decltype(bufc)::value;
        const char* kt = sm.k[BUF];
        const char* vt = sm.v[BUF];
        const bool gist_tile = it < ngt;
        const int j0 = row_step_first(walk, it, BNQ);
        const int kind = row_step_kind(walk, it, BNQ, wrow0, wrow0 + 31, lo_wlast);
        if (kind == STEP_SKIP) return;

        const bool masked = kind == STEP_MASKED;
        unsigned long long gm = 0ull;  // bit t: the key at offset t from j0 holds a sink or a gist
        if (!gist_tile && masked) gm = __builtin_amdgcn_ballot_w64(is_always(s, j0 + lane));

        // S^T, dP^T for the 32 keys of half kb2: register i of sa[kb][qb] is key j0 + 32 kb2 + 16 kb + 4 g4 + i, column =
        // query qrow[qb].  Every K and V fragment serves both query blocks; the reads run PFS groups ahead of their
        // MFMAs and the scheduling barriers keep them there.
        auto sdp = [&](int kb2, f32x4 (&sa)[2][2], f32x4 (&dp)[2][2]) __attribute__((always_inline)) {
            constexpr int N = 2 * KS;  // group n: key block n / KS, k-step n % KS
            bf16x8 fk[N], fv[N];
            auto fetch = [&](int n) __attribute__((always_inline)) {
                const int o = (32 * kb2 + 16 * (n / KS)) * CH * 16 + roff[n % KS];
                fk[n] = *(const bf16x8*)(kt + o);
                fv[n] = *(const bf16x8*)(vt + o);
            };
#pragma unroll
            for (int n = 0; n < PFS; ++n) fetch(n);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int n = 0; n < N; ++n) {
                if (n + PFS < N) fetch(n + PFS);
                const int kb = n / KS, ks = n % KS;
#pragma unroll
                for (int qb = 0; qb < 2; ++qb) {
                    sa[kb][qb] = mfma16(fk[n], qf[qb][ks], ks == 0 ? zero4() : sa[kb][qb]);
                    dp[kb][qb] = mfma16(fv[n], gf[qb][ks], ks == 0 ? ndl[qb] : dp[kb][qb]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // P = exp2(S c - lse), the mask, dS = P (dP - delta) (dP arrives with -delta in it): dp becomes dS
        auto soft = [&](int kb2, f32x4 (&sa)[2][2], f32x4 (&dp)[2][2]) __attribute__((always_inline)) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) sa[kb][qb][i] = __builtin_amdgcn_exp2f(fmaf(sa[kb][qb][i], c, -ls[qb]));
                if (masked) {
                    // bit t of vis: does query qrow[qb] see the key at offset t of this 32-key block?  Visible sets
                    // are bit ranges (the tail of the compact list; the window) plus, in the window phase, the sinks
                    // and gists.  This lane holds the offsets 16 kb + 4 g4 + i.
                    unsigned vis;
                    if (gist_tile) {
                        vis = below_bits(nfar - j0 - 32 * kb2);
                    } else {
                        const int d0 = qrow[qb] - (j0 + 32 * kb2);  // offsets d0 - span_q .. d0: window; <= d0: causal
                        vis = below_bits(d0 + 1) & (~below_bits(d0 - span_q[qb]) | (unsigned)(gm >> (32 * kb2)));
                    }
                    vis >>= 4 * g4;
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (!((vis >> (16 * kb + i)) & 1u)) sa[kb][qb][i] = 0.f;
                }
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) dp[kb][qb][i] *= sa[kb][qb][i];
            }
        };
        // dQ^T += K^T dS^T for half kb2: contraction slot 8 g4 + 4 kb + i is key 16 kb + 4 g4 + i of the half, on both
        // operands
        auto dqm = [&](int kb2, const bf16x8 (&sb)[2]) __attribute__((always_inline)) {
            bf16x8 ft[DB];
#pragma unroll
            for (int db = 0; db < PFT; ++db) ft[db] = tr16_frag16<CH>(kt + toff[db], 32 * kb2);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                if (db + PFT < DB) ft[db + PFT] = tr16_frag16<CH>(kt + toff[db + PFT], 32 * kb2);
                acc[db][0] = mfma16(ft[db], sb[0], acc[db][0]);
                acc[db][1] = mfma16(ft[db], sb[1], acc[db][1]);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2) {
            f32x4 sa[2][2], dp[2][2];
            bf16x8 sb[2];
            sdp(kb2, sa, dp);
            soft(kb2, sa, dp);
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) sb[qb] = pack44(dp[0][qb], dp[1][qb]);
            dqm(kb2, sb);
        }
    };

    issue(0, 0);
    for (int it = 0; it < ntiles; it += 2) {
        wait_vmem();
        __syncthreads();
        if (it + 1 < ntiles) issue(it + 1, 1);
        tile_step(std::integral_constant<int, 0>{}, it);
        if (it + 1 < ntiles) {
            wait_vmem();
            __syncthreads();
            if (it + 2 < ntiles) issue(it + 2, 0);
            tile_step(std::integral_constant<int, 1>{}, it + 1);
        }
    }

#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
        if (qrow[qb] < L) {
            bf16_t* op = dq + rowoff[qb] + 4 * g4;
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                if (QSTR && 16 * db + 4 * g4 >= Dt) continue;
                u32x2 w2;
                w2[0] = pack_bf16x2(acc[db][qb][0] * s.scale, acc[db][qb][1] * s.scale);
                w2[1] = pack_bf16x2(acc[db][qb][2] * s.scale, acc[db][qb][3] * s.scale);
                *(u32x2*)(op + 16 * db) = w2;
            }
        }
}

template <int D>
hipError_t bwd_launch(const bf16_t* q, const bf16_t* k, const bf16_t* v, const bf16_t* out, const float* lse,
                      const bf16_t* dout, bf16_t* dq, bf16_t* dk, bf16_t* dv, char* ws, const AttnShape& s,
                      unsigned stages, hipStream_t st) {
    const BwdPlan pl = make_plan(s);
    const bool gen = s.S != 0 || s.umode != 0;
    const bool qstr = s.q_rs != 0;  // q, out, dout, dq with the caller's explicit strides
    float* delta = (float*)ws;
    float* lse2 = (float*)(ws + pl.off_lse2);
    float* part = (float*)(ws + pl.off_part);
    float* comp = (float*)(ws + pl.off_comp);
    hipError_t e;
    if (stages & UNIGIST_BWD_DELTA) {
        constexpr int rows_per_blk = NT / (D / 8);
        const long nrows = (long)s.B * s.Hq * s.L;
        delta_kernel<D><<<dim3((unsigned)((nrows + rows_per_blk - 1) / rows_per_blk)), NT, 0, st>>>(
            out, dout, lse, delta, lse2, nrows, s.L, s.qhs, s.Hq, s.q_bs, s.q_hs, s.q_rs, s.D);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (pl.n_gt > 0 && (stages & UNIGIST_BWD_DKDV_GIST)) {
        const dim3 grid((unsigned)((long)pl.slot0[pl.nseg] * s.Hkv * s.B));
        if (qstr) {
            if (gen) dkdv_kernel<D, true, true, false, true><<<grid, NT, 0, st>>>(q, k, v, lse2, dout, delta, dk, dv, part, comp, s, pl, NoDocs{});
            else dkdv_kernel<D, true, false, false, true><<<grid, NT, 0, st>>>(q, k, v, lse2, dout, delta, dk, dv, part, comp, s, pl, NoDocs{});
        } else if (gen) dkdv_kernel<D, true, true, false><<<grid, NT, 0, st>>>(q, k, v, lse2, dout, delta, dk, dv, part, comp, s, pl, NoDocs{});
        else dkdv_kernel<D, true, false, false><<<grid, NT, 0, st>>>(q, k, v, lse2, dout, delta, dk, dv, part, comp, s, pl, NoDocs{});
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (pl.n_gt > 0 && (stages & UNIGIST_BWD_GIST_REDUCE)) {
        const int per_tile = 2 * D * BNK;
        gist_reduce_kernel<<<dim3((per_tile / 4 + NT - 1) / NT, pl.n_gt, s.B * s.Hkv), NT, 0, st>>>(part, comp, pl, s, per_tile);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (stages & UNIGIST_BWD_DKDV_WINDOW) {
        const dim3 grid((unsigned)((long)((s.L + BNK - 1) / BNK) * s.Hkv * s.B));
        if (qstr) {
            if (gen) dkdv_kernel<D, false, true, false, true><<<grid, NT, 0, st>>>(q, k, v, lse2, dout, delta, dk, dv, part, comp, s, pl, NoDocs{});
            else dkdv_kernel<D, false, false, false, true><<<grid, NT, 0, st>>>(q, k, v, lse2, dout, delta, dk, dv, part, comp, s, pl, NoDocs{});
        } else if (gen) dkdv_kernel<D, false, true, false><<<grid, NT, 0, st>>>(q, k, v, lse2, dout, delta, dk, dv, part, comp, s, pl, NoDocs{});
        else dkdv_kernel<D, false, false, false><<<grid, NT, 0, st>>>(q, k, v, lse2, dout, delta, dk, dv, part, comp, s, pl, NoDocs{});
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (!(stages & UNIGIST_BWD_DQ)) return hipSuccess;
    const int nq = (s.L + BMQ - 1) / BMQ;
    const long nblk = (long)nq * s.Hq * s.B;
    if (nblk > 0x7fffffffL) return hipErrorInvalidValue;
    if (qstr) {
        if (gen) dq_kernel<D, true, false, true><<<dim3((unsigned)nblk), NT, 0, st>>>(q, k, v, lse2, dout, delta, dq, s, nq, NoDocs{});
        else dq_kernel<D, false, false, true><<<dim3((unsigned)nblk), NT, 0, st>>>(q, k, v, lse2, dout, delta, dq, s, nq, NoDocs{});
    } else if (gen) dq_kernel<D, true, false><<<dim3((unsigned)nblk), NT, 0, st>>>(q, k, v, lse2, dout, delta, dq, s, nq, NoDocs{});
    else dq_kernel<D, false, false><<<dim3((unsigned)nblk), NT, 0, st>>>(q, k, v, lse2, dout, delta, dq, s, nq, NoDocs{});
    return hipGetLastError();
}

// ---- packed documents: the non-empty documents, longest first (their long tiles should not start last), and
// the slots each of them gets in the partial-sum arrays
struct PackPlan {
    std::vector<int> c0, len, part0, comp0;  // per document, in launch order
    int segc;                                // segment length asked of every document's plan
    size_t off_lse2, off_part, off_comp, total;
};

PackPlan make_pack_plan(const AttnShape& s, const int* cu, int ndocs) {
    PackPlan pp;
    std::vector<int> order;
    for (int d = 0; d < ndocs; ++d)
        if (cu[d + 1] > cu[d]) order.push_back(d);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return cu[a + 1] - cu[a] > cu[b + 1] - cu[b]; });
    long steps = 0;
    for (int d : order) steps += gist_chunk_steps(doc_view(s, cu[d + 1] - cu[d]));
    pp.segc = pick_segc(steps * s.Hkv);
    size_t nslot_part = 0, nslot_comp = 0;
    for (int d : order) {
        BwdPlan pl;
        plan_counts(doc_view(s, cu[d + 1] - cu[d]), pl, pp.segc);
        plan_slots(doc_view(s, cu[d + 1] - cu[d]), pl);
        pp.c0.push_back(cu[d]);
        pp.len.push_back(cu[d + 1] - cu[d]);
        pp.part0.push_back((int)nslot_part);
        pp.comp0.push_back((int)nslot_comp);
        nslot_part += (size_t)s.Hkv * pl.slot0[pl.nseg];
        nslot_comp += (size_t)s.Hkv * pl.n_gt;
    }
    const size_t a = 255, per_tile = (size_t)2 * padded_head_dim(s.D) * BNK * sizeof(float);
    size_t off = ((size_t)s.Hq * s.L * sizeof(float) + a) & ~a;  // delta, [Hq, T] like the caller's lse
    pp.off_lse2 = off;
    off += ((size_t)s.Hq * s.L * sizeof(float) + a) & ~a;
    pp.off_part = off;
    off += nslot_part * per_tile;
    pp.off_comp = off;
    off += nslot_comp * per_tile;
    pp.total = (off + a) & ~a;
    if (nslot_part > 0x7fffffffUL) pp.total = 0;  // slot numbers are kept in 32 bits
    return pp;
}

template <int D>
hipError_t bwd_launch_pack(const bf16_t* q, const bf16_t* k, const bf16_t* v, const bf16_t* out, const float* lse,
                           const bf16_t* dout, bf16_t* dq, bf16_t* dk, bf16_t* dv, char* ws, const AttnShape& s,
                           const int* cu, int ndocs, hipStream_t st) {
    const PackPlan pp = make_pack_plan(s, cu, ndocs);
    if (pp.total == 0) return hipErrorInvalidValue;
    float* delta = (float*)ws;
    float* lse2 = (float*)(ws + pp.off_lse2);
    float* part = (float*)(ws + pp.off_part);
    float* comp = (float*)(ws + pp.off_comp);
    hipError_t e;
    {  // delta and lse2 of every row of the pack (a row's delta does not depend on its document)
        constexpr int rows_per_blk = NT / (D / 8);
        const long nrows = (long)s.Hq * s.L;
        delta_kernel<D><<<dim3((unsigned)((nrows + rows_per_blk - 1) / rows_per_blk)), NT, 0, st>>>(
            out, dout, lse, delta, lse2, nrows, s.L, s.qhs, s.Hq, 0, s.q_hs, s.q_rs, s.D);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    const int nd = (int)pp.len.size();
    // one launch of each kernel per kMaxDocs documents; blocks(i) = workgroups (or slots) of document i
    auto for_chunks = [&](auto&& blocks, auto&& launch) -> hipError_t {
        for (int at = 0; at < nd; at += kMaxDocs) {
            DocTab t;
            memset(&t, 0, sizeof t);
            t.n = std::min(kMaxDocs, nd - at);
            long nblk = 0;
            for (int i = 0; i < t.n; ++i) {
                t.c0[i] = pp.c0[at + i];
                t.len[i] = pp.len[at + i];
                t.part0[i] = pp.part0[at + i];
                t.comp0[i] = pp.comp0[at + i];
                t.blk0[i] = (int)nblk;
                nblk += blocks(pp.len[at + i]);
                if (nblk > 0x7fffffffL) return hipErrorInvalidValue;
            }
            t.blk0[t.n] = (int)nblk;
            if (nblk == 0) continue;
            launch(t, (unsigned)nblk);
            const hipError_t err = hipGetLastError();
            if (err != hipSuccess) return err;
        }
        return hipSuccess;
    };
    auto counts = [&](int len) {
        BwdPlan pl;
        plan_counts(doc_view(s, len), pl, pp.segc);
        plan_slots(doc_view(s, len), pl);
        return pl;
    };
    BwdPlan none = {};
    none.segc = pp.segc;
    const bool gen = s.S != 0 || s.umode != 0, qstr = s.q_rs != 0;
    e = for_chunks([&](int len) { const BwdPlan pl = counts(len); return (long)pl.slot0[pl.nseg] * s.Hkv; },
                   [&](const DocTab& t, unsigned nblk) {
                       auto go = [&](auto kern) { kern<<<dim3(nblk), NT, 0, st>>>(q, k, v, lse2, dout, delta, dk, dv, part, comp, s, none, t); };
                       if (qstr) gen ? go(dkdv_kernel<D, true, true, true, true>) : go(dkdv_kernel<D, true, false, true, true>);
                       else gen ? go(dkdv_kernel<D, true, true, true>) : go(dkdv_kernel<D, true, false, true>);
                   });
    if (e != hipSuccess) return e;
    constexpr int per_tile = 2 * D * BNK;
    e = for_chunks([&](int len) { return (long)counts(len).n_gt * s.Hkv; },
                   [&](const DocTab& t, unsigned nblk) {
                       gist_reduce_pack_kernel<<<dim3(nblk, (per_tile / 4 + NT - 1) / NT), NT, 0, st>>>(
                           part, comp, s, per_tile, pp.segc, t);
                   });
    if (e != hipSuccess) return e;
    e = for_chunks([&](int len) { return (long)((len + BNK - 1) / BNK) * s.Hkv; },
                   [&](const DocTab& t, unsigned nblk) {
                       auto go = [&](auto kern) { kern<<<dim3(nblk), NT, 0, st>>>(q, k, v, lse2, dout, delta, dk, dv, part, comp, s, none, t); };
                       if (qstr) gen ? go(dkdv_kernel<D, false, true, true, true>) : go(dkdv_kernel<D, false, false, true, true>);
                       else gen ? go(dkdv_kernel<D, false, true, true>) : go(dkdv_kernel<D, false, false, true>);
                   });
    if (e != hipSuccess) return e;
    return for_chunks([&](int len) { return (long)((len + BMQ - 1) / BMQ) * s.Hq; },
                      [&](const DocTab& t, unsigned nblk) {
                          auto go = [&](auto kern) { kern<<<dim3(nblk), NT, 0, st>>>(q, k, v, lse2, dout, delta, dq, s, 0, t); };
                          if (qstr) gen ? go(dq_kernel<D, true, true, true>) : go(dq_kernel<D, false, true, true>);
                          else gen ? go(dq_kernel<D, true, true>) : go(dq_kernel<D, false, true>);
                      });
}

}  // namespace

size_t bwd_mfma_workspace(const AttnShape& s) { return make_plan(s).total; }

BwdPlan make_bwd_plan(const AttnShape& s) { return make_plan(s); }

size_t bwd_mfma_pack_workspace(const AttnShape& s, const int* cu, int ndocs) { return make_pack_plan(s, cu, ndocs).total; }

// A head dimension below the one the kernels are built for goes through the instantiations for explicit strides of
// q, out, dout and dq, with the strides of the dense layout.
static AttnShape with_dense_strides_if_padded(AttnShape s) {
    if (s.D != padded_head_dim(s.D) && s.q_rs == 0) {
        s.q_rs = s.D;
        s.q_hs = (long long)s.qhs * s.D;
        s.q_bs = (long long)s.Hq * s.q_hs;
    }
    return s;
}

hipError_t launch_bwd_mfma_pack(const void* q, const void* k, const void* v, const void* out, const float* lse,
                                const void* dout, void* dq, void* dk, void* dv, void* ws, const AttnShape& s_in,
                                const int* cu, int ndocs, hipStream_t st) {
    const AttnShape s = with_dense_strides_if_padded(s_in);
    if (s.D <= 64)
        return bwd_launch_pack<64>((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (const bf16_t*)out, lse,
                                   (const bf16_t*)dout, (bf16_t*)dq, (bf16_t*)dk, (bf16_t*)dv, (char*)ws, s, cu, ndocs, st);
    return bwd_launch_pack<128>((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (const bf16_t*)out, lse,
                                (const bf16_t*)dout, (bf16_t*)dq, (bf16_t*)dk, (bf16_t*)dv, (char*)ws, s, cu, ndocs, st);
}

hipError_t launch_bwd_mfma(const void* q, const void* k, const void* v, const void* out, const float* lse,
                           const void* dout, void* dq, void* dk, void* dv, void* ws, const AttnShape& s_in,
                           unsigned stages, hipStream_t st) {
    const AttnShape s = with_dense_strides_if_padded(s_in);
    if (s.D <= 64)
        return bwd_launch<64>((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (const bf16_t*)out, lse,
                              (const bf16_t*)dout, (bf16_t*)dq, (bf16_t*)dk, (bf16_t*)dv, (char*)ws, s, stages, st);
    return bwd_launch<128>((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (const bf16_t*)out, lse,
                           (const bf16_t*)dout, (bf16_t*)dq, (bf16_t*)dk, (bf16_t*)dv, (char*)ws, s, stages, st);
}

}  // namespace unigist
