// Host-side exerciser of libunigist for AddressSanitizer / UndefinedBehaviorSanitizer builds.
// Calls only what runs entirely on the host: the block map, the plan queries, the workspace-size and cache-state
// functions, and the argument validation of every launching entry point with arguments that are refused before
// anything is launched (so no kernel ever runs, with or without a GPU).  Prints "ok <calls>" on success.
#include <stdio.h>
#include <stdlib.h>

#include <vector>

#include "unigist.h"

static long g_calls = 0;
#define CHECK(cond)                                                      \
    do {                                                                 \
        ++g_calls;                                                       \
        if (!(cond)) {                                                   \
            fprintf(stderr, "%s:%d: failed: %s\n", __FILE__, __LINE__, #cond); \
            exit(1);                                                     \
        }                                                                \
    } while (0)

struct Shape {
    int B, Hq, Hkv, L, D, r, W, sinks, mode;
};

static void walk_plans(const Shape& s) {
    for (int kernel = 0; kernel < 2; ++kernel) {
        const int nq = (s.L + 127) / 128;
        for (int t = 0; t < nq; ++t) {
            unigist_row_tile_plan p;
            CHECK(unigist_plan_row_tile(s.L, s.r, s.W, s.sinks, s.mode, kernel, t, &p, 0, nullptr) == UNIGIST_OK);
            const int n = (p.Bm / p.rows_per_wave) * (p.n_gist_steps + p.n_window_steps);
            std::vector<signed char> kind(n);  // exactly as large as documented: an overrun is a finding
            CHECK(unigist_plan_row_tile(s.L, s.r, s.W, s.sinks, s.mode, kernel, t, &p, n, kind.data()) == UNIGIST_OK);
            CHECK(unigist_plan_row_tile(s.L, s.r, s.W, s.sinks, s.mode, kernel, t, &p, n - 1, kind.data()) == UNIGIST_EINVAL);
        }
        unigist_row_tile_plan p;
        CHECK(unigist_plan_row_tile(s.L, s.r, s.W, s.sinks, s.mode, kernel, nq, &p, 0, nullptr) == UNIGIST_EINVAL);
        CHECK(unigist_plan_row_tile(s.L, s.r, s.W, s.sinks, s.mode, kernel, -1, &p, 0, nullptr) == UNIGIST_EINVAL);
    }
    unigist_bwd_plan bp;
    CHECK(unigist_bwd_plan_build(s.B, s.Hq, s.Hkv, s.L, s.D, s.r, s.W, s.sinks, s.mode, &bp) == UNIGIST_OK);
    CHECK(bp.workspace_bytes == unigist_attn_bwd_workspace_ex(s.B, s.Hq, s.Hkv, s.L, s.D, s.r, s.W, s.sinks, s.mode, UNIGIST_BF16));
    for (int phase = 0; phase < 2; ++phase) {
        const int nseg = phase ? bp.n_segs : 1;
        for (int sg = 0; sg < nseg; ++sg) {
            const int nt = phase ? bp.slot0[sg + 1] - bp.slot0[sg] : bp.n_key_tiles;
            for (int t = 0; t < nt; ++t) {
                int lo = 0, hi = -1;
                CHECK(unigist_plan_key_tile(s.B, s.Hq, s.Hkv, s.L, s.D, s.r, s.W, s.sinks, s.mode, phase, t, sg, &lo, &hi, 0,
                                            nullptr, nullptr) == UNIGIST_OK);
                const int n = hi - lo + 1;
                CHECK(n >= 1);
                std::vector<int> nfar(n);
                std::vector<signed char> kind(4 * n * 2);
                CHECK(unigist_plan_key_tile(s.B, s.Hq, s.Hkv, s.L, s.D, s.r, s.W, s.sinks, s.mode, phase, t, sg, &lo, &hi, n,
                                            nfar.data(), kind.data()) == UNIGIST_OK);
                CHECK(unigist_plan_key_tile(s.B, s.Hq, s.Hkv, s.L, s.D, s.r, s.W, s.sinks, s.mode, phase, t, sg, &lo, &hi,
                                            n - 1, nfar.data(), kind.data()) == UNIGIST_EINVAL);
            }
            int lo, hi;
            CHECK(unigist_plan_key_tile(s.B, s.Hq, s.Hkv, s.L, s.D, s.r, s.W, s.sinks, s.mode, phase, nt, sg, &lo, &hi, 0, nullptr,
                                        nullptr) == UNIGIST_EINVAL);
        }
    }
    // the gist phase's launch order: every slot of the plan exactly once
    const int nslots = bp.slot0[bp.n_segs];
    std::vector<char> seen(nslots, 0);
    for (int unit = 0; unit < nslots; ++unit) {
        int sg = -1, t = -1;
        CHECK(unigist_plan_gist_unit(s.B, s.Hq, s.Hkv, s.L, s.D, s.r, s.W, s.sinks, s.mode, unit, &sg, &t) == UNIGIST_OK);
        CHECK(sg >= 0 && sg < bp.n_segs && t >= 0 && t < bp.slot0[sg + 1] - bp.slot0[sg]);
        CHECK(!seen[bp.slot0[sg] + t]);
        seen[bp.slot0[sg] + t] = 1;
    }
    int sg, t;
    CHECK(unigist_plan_gist_unit(s.B, s.Hq, s.Hkv, s.L, s.D, s.r, s.W, s.sinks, s.mode, nslots, &sg, &t) == UNIGIST_EINVAL);
    CHECK(unigist_plan_gist_unit(s.B, s.Hq, s.Hkv, s.L, s.D, s.r, s.W, s.sinks, s.mode, -1, &sg, &t) == UNIGIST_EINVAL);
    CHECK(unigist_plan_gist_unit(s.B, s.Hq, s.Hkv, s.L, s.D, s.r, s.W, s.sinks, s.mode, 0, nullptr, &t) == UNIGIST_EINVAL);
}

static void block_maps(const Shape& s) {
    for (int Bm : {1, 16, 128, 300})
        for (int Bn : {1, 32, 128}) {
            unigist_blockmap* m = nullptr;
            CHECK(unigist_blockmap_build_ex(s.L, s.r, s.W, s.sinks, s.mode, Bm, Bn, &m) == UNIGIST_OK);
            long live = 0;
            for (int t = 0; t < m->n_qtiles; ++t)  // touch every array to its end
                live += m->win_last[t] - m->win_first[t] + 1 + (m->n_far_gists[t] + Bn - 1) / Bn + 0 * m->n_full[t];
            for (int c = 0; c < m->n_ktiles; ++c) CHECK(m->qt_first[c] <= m->qt_last[c]);
            for (int g = 0; g < m->n_gtiles; ++g) CHECK(m->gist_qt_first[g] < m->n_qtiles);
            CHECK(live == m->live_tiles);
            unigist_blockmap_free(m);
        }
}

int main() {
    const Shape shapes[] = {
        {1, 4, 1, 5000, 128, 4, 129, 0, 0},   {2, 8, 8, 9001, 128, 2, 300, 0, 0},  {1, 2, 1, 4097, 64, 8, 1, 0, 0},
        {1, 2, 1, 3000, 64, 4, 1000000, 0, 0}, {1, 2, 2, 2500, 96, 2147483646, 333, 0, 0}, {1, 4, 1, 6000, 128, 4, 25, 128, 1},
        {1, 4, 2, 7000, 128, 3, 1, 5, 1},     {1, 8, 2, 4500, 64, 4, 204, 300, 1}, {1, 2, 1, 63, 8, 1, 3, 0, 0},
        {1, 1, 1, 1, 64, 4, 4, 0, 0},         {1, 32, 8, 32768, 128, 4, 1024, 0, 0}, {1, 2, 1, 70000, 128, 2147483646, 2147483647, 2147483647, 1},
    };
    for (const Shape& s : shapes) {
        walk_plans(s);
        block_maps(s);
    }
    // invalid arguments to the host calls
    unigist_blockmap* m = nullptr;
    CHECK(unigist_blockmap_build(0, 4, 4, 8, 8, &m) == UNIGIST_EINVAL && m == nullptr);
    CHECK(unigist_blockmap_build(8, 4, 4, 8, 8, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_blockmap_build_ex(8, 4, 4, -1, 0, 8, 8, &m) == UNIGIST_EINVAL);
    unigist_blockmap_free(nullptr);
    unigist_bwd_plan bp;
    CHECK(unigist_bwd_plan_build(1, 4, 3, 100, 128, 4, 8, 0, 0, &bp) == UNIGIST_EINVAL);
    CHECK(unigist_bwd_plan_build(1, 4, 2, 100, 100, 4, 8, 0, 0, &bp) == UNIGIST_EINVAL);
    CHECK(unigist_bwd_plan_build(1, 4, 2, 100, 128, 4, 8, 0, 0, nullptr) == UNIGIST_EINVAL);

    // host-only size and state functions, over their edges
    for (int t = -2; t < 300; ++t)
        for (int mode = 0; mode < 2; ++mode) {
            const int s = unigist_window_start(t, 4, 7, 3, mode), rows = unigist_cache_ring_rows(t, 4, 7, 3, mode);
            CHECK(t < -1 ? s == -1 : (s >= 0 && s <= (t < 0 ? 0 : t)));
            CHECK(t < -1 ? rows == -1 : rows >= 0);
            if (t >= 0) CHECK(unigist_cache_rows_ex(s, t, 4, 3) >= 1);
        }
    CHECK(unigist_cache_rows(5, 3, 4) == -1 && unigist_cache_rows_ex(0, 2147483646, 2147483646, 2147483647) > 0);
    CHECK(unigist_window_start(1 << 23, 4, 8, 0, 0) == -1 && unigist_window_start((1 << 23) - 1, 2147483646, 2147483647, 2147483647, 1) >= 0);
    CHECK(unigist_decode_workspace(64, 32, 8, 17408, 128, UNIGIST_BF16) > 0 && unigist_decode_workspace(1, 4, 1, 1, 96, UNIGIST_F32) > 0);
    CHECK(unigist_decode_workspace(1, 4, 3, 10, 128, UNIGIST_BF16) == 0 && unigist_decode_workspace(1, 4, 1, 10, 100, UNIGIST_BF16) == 0);
    CHECK(unigist_decode_noalloc_scratch_bytes() == UNIGIST_DECODE_NOALLOC_SCRATCH_BYTES);
    CHECK(unigist_prefill_chunk_e4m3_workspace(2, 2, 128, 10, 500, 4, 0) > 0 && unigist_prefill_chunk_e4m3_workspace(2, 2, 128, 600, 500, 4, 0) == 0);
    int Bm = 0, Bn = 0;
    unigist_tile_sizes(128, UNIGIST_BF16, &Bm, &Bn);
    unigist_tile_sizes(128, UNIGIST_F32, nullptr, nullptr);
    CHECK(Bm == 128 && Bn == 32);
    for (int st = -1; st < 7; ++st) CHECK(unigist_status_str((unigist_status)st) != nullptr);
    {   // packed documents: the plan of a pack is made on the host
        const int cu[] = {0, 300, 300, 4800, 4801, 9001};
        CHECK(unigist_attn_bwd_varlen_workspace_ex(8, 2, 9001, 128, 4, 64, 0, 0, cu, 5, UNIGIST_BF16) > 0);
        CHECK(unigist_attn_bwd_varlen_workspace_ex(8, 2, 9001, 96, 4, 3, 100, 1, cu, 5, UNIGIST_F32) > 0);
        const int bad[] = {0, 300, 200, 9001};
        CHECK(unigist_attn_bwd_varlen_workspace(8, 2, 9001, 128, 4, 64, bad, 3, UNIGIST_BF16) == 0);
        CHECK(unigist_attn_bwd_varlen_workspace(8, 2, 9000, 128, 4, 64, cu, 5, UNIGIST_BF16) == 0);
        std::vector<int> many(70001);
        for (int i = 0; i <= 70000; ++i) many[i] = i;  // 70 000 one-token documents: more than a thousand launch tables
        CHECK(unigist_attn_bwd_varlen_workspace(4, 4, 70000, 64, 2, 5, many.data(), 70000, UNIGIST_BF16) > 0);
    }

    // every launching entry point, refused before anything is launched
    void* const P = (void*)0x1000;  // never dereferenced
    float* const F = (float*)0x1000;
    int* const I = (int*)0x1000;
    CHECK(unigist_attn_fwd(nullptr, P, P, P, F, 1, 4, 2, 64, 64, 4, 8, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_attn_fwd(P, P, P, P, F, 1, 4, 2, 64, 100, 4, 8, UNIGIST_BF16, nullptr) == UNIGIST_EUNSUPPORTED);
    CHECK(unigist_attn_fwd_ex(P, P, P, P, F, 1, 4, 2, 64, 64, 4, 8, -1, 0, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_attn_fwd_strided(P, P, P, P, F, 1, 4, 2, 64, 64, 4, 8, 0, 0, 0, 64 * 64, 60, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_attn_bwd(P, P, P, P, F, P, P, P, P, 1, 4, 2, 64, 64, 4, 8, UNIGIST_BF16, P, 16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_attn_bwd_ex(P, P, P, P, F, P, P, P, P, 1, 4, 2, 64, 64, 4, 8, 0, 0, UNIGIST_BF16, P, (size_t)1 << 40, 64, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_attn_bwd_strided(P, P, P, P, F, P, P, P, P, 1, 4, 2, 64, 64, 4, 8, 0, 0, 0, 64 * 64, 64, UNIGIST_F32, P, (size_t)1 << 40, nullptr) == UNIGIST_EUNSUPPORTED);
    CHECK(unigist_decode(P, P, P, P, F, 1, 4, 3, 10, nullptr, 128, UNIGIST_BF16, P, 1 << 20, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_decode(P, P, P, P, F, 1, 4, 1, 10, nullptr, 128, UNIGIST_BF16, P, 16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_decode_noalloc(P, P, P, P, F, 4096, 32, 8, 4096, nullptr, 128, UNIGIST_BF16, nullptr) == UNIGIST_ESCRATCH);
    CHECK(unigist_decode_e4m3(P, P, P, F, F, P, F, 1, 4, 1, 10, nullptr, 104, P, 1 << 20, nullptr) == UNIGIST_EUNSUPPORTED);
    CHECK(unigist_quantize_e4m3(P, P, nullptr, 1, 2, 3, 128, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_cache_update(P, P, 5, 3, 100, P, P, 1, 1, P, P, 5, 100, 1, 1, 128, 4, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_cache_update_ex(P, P, 0, 9, 4, P, P, 1, 1, P, P, 0, 100, 1, 1, 128, 4, 0, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_cache_update_ragged(P, P, I, I, 10, P, P, I, 1, P, P, I, 10, nullptr, 2, 2, 128, 4, 0, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_cache_to_ring(P, P, I, I, 0, P, P, 10, I, 1, 1, 128, 4, 8, 0, 0, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_cache_from_ring(P, P, I, I, 10, P, P, 10, I, 1, 1, 128, 4, 8, 0, 3, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_cache_ring_append(P, P, P, P, 0, I, I, 10, I, 1, 1, 128, 4, 8, 0, 0, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_prefill_chunk(P, P, P, P, F, 1, 4, 2, 64, 128, 4, 8, 100, 99, 1000, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_prefill_chunk_ex(P, P, P, P, F, 1, 4, 2, 64, 128, 4, 8, 0, 0, 100, 0, 10, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_prefill_chunk_view(P, P, P, P, F, 1, 4, 2, 64, 32, 128, 4, 8, 0, 0, 0, 0, 1000, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_prefill_chunk_strided(P, P, P, P, F, 1, 4, 2, 64, 128, 4, 8, 0, 0, 0, 0, 1000, 0, 128, 100, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_prefill_chunk_e4m3(P, P, P, F, F, P, F, 1, 4, 2, 64, 128, 4, 8, 0, 0, 0, 0, 1000, P, 16, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_prefill_chunk_ragged(P, P, P, P, F, 2, 4, 2, 64, 128, 4, 8, 0, 0, I, I, nullptr, 100, I, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
    {
        const int cu[] = {0, 30, 64};
        CHECK(unigist_attn_fwd_varlen(P, P, P, P, F, 4, 2, 65, 64, 4, 8, cu, 2, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
        CHECK(unigist_attn_fwd_varlen_ex(P, P, P, nullptr, F, 4, 2, 64, 64, 4, 8, 0, 0, cu, 2, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
        CHECK(unigist_attn_bwd_varlen(P, P, P, P, F, P, P, P, P, 4, 2, 64, 64, 4, 8, cu, 2, UNIGIST_BF16, P, 16, nullptr) == UNIGIST_EINVAL);
        CHECK(unigist_attn_bwd_varlen_ex(P, P, P, P, F, P, P, P, P, 4, 2, 64, 64, 4, 8, 0, 7, cu, 2, UNIGIST_BF16, P, (size_t)1 << 40, nullptr) == UNIGIST_EINVAL);
        CHECK(unigist_attn_fwd_varlen_strided(P, P, P, P, F, 4, 2, 64, 64, 4, 8, 0, 0, cu, 2, 64, 4 * 64 + 4, UNIGIST_BF16, nullptr) == UNIGIST_EINVAL);
        CHECK(unigist_attn_bwd_varlen_strided(P, P, P, P, F, P, P, P, P, 4, 2, 64, 64, 4, 8, 0, 0, cu, 2, 64, 4 * 64, UNIGIST_BF16, P, 16, nullptr) == UNIGIST_EINVAL);
    }
    CHECK(unigist_probe_mfma_rate(nullptr, nullptr, nullptr, 1, 1, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_probe_read_rate(P, 8, (unsigned*)P, 1, nullptr) == UNIGIST_EINVAL);
    CHECK(unigist_debug_force_plain_alu(1) == 0 && unigist_debug_force_plain_alu(0) == 1);
    printf("ok %ld\n", g_calls);
    return 0;
}
