/*
 * Sanitizer run of the CPU oracle (TEST INFRASTRUCTURE ONLY): drives every oracle function on small,
 * deliberately awkward inputs (empty segments, padding rows, ties, budgets 0 and above the count, a
 * destination that is too small) so that AddressSanitizer / UndefinedBehaviorSanitizer see all of its
 * indexing.  Built and run by tests/test_oracle_sanitizers.py:
 *     gcc -std=c11 -g -O1 -fsanitize=address,undefined -fno-sanitize-recover=all -static-libasan selftest.c -lm
 * Exit code 0 = every call returned and the few invariants checked here hold.
 */
#include <stdio.h>

#include "kvtrim_oracle.c"

#define CHECK(cond)                                                            \
    do {                                                                       \
        if (!(cond)) {                                                         \
            fprintf(stderr, "selftest: %s failed (line %d)\n", #cond, __LINE__); \
            return 1;                                                          \
        }                                                                      \
    } while (0)

static uint32_t rng_state = 12345u;
static uint32_t rnd(void) {
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state >> 8;
}

static kvo_cache make_cache(const kvo_shape *sh, int64_t cap, int with_tail) {
    kvo_cache c;
    int64_t nseg = kvo_nseg(sh);
    c.k = (uint16_t *)calloc((size_t)cap * sh->head_dim, 2);
    c.v = (uint16_t *)calloc((size_t)cap * sh->head_dim, 2);
    c.log_beta = (float *)calloc((size_t)cap, 4);
    c.pos = (int32_t *)calloc((size_t)cap, 4);
    c.seg_start = (int64_t *)calloc((size_t)nseg, 8);
    c.seg_len = (int32_t *)calloc((size_t)nseg, 4);
    c.cap = cap;
    c.log_tail = with_tail ? (float *)calloc((size_t)cap, 4) : NULL;
    return c;
}

static void free_cache(kvo_cache *c) {
    free(c->k); free(c->v); free(c->log_beta); free(c->pos); free(c->seg_start); free(c->seg_len); free(c->log_tail);
}

int main(void) {
    const kvo_shape sh = {2, 2, 2, 4, 8};                       /* S, L, Hkv, Hq, D */
    const int64_t nseg = kvo_nseg(&sh);
    const int D = sh.head_dim, room = 12;
    for (int with_tail = 0; with_tail < 2; ++with_tail) {
        kvo_cache c = make_cache(&sh, nseg * room, with_tail);
        for (int64_t g = 0; g < nseg; ++g) c.seg_start[g] = g * room;
        /* three rounds of appends with padding rows; segment 3 never gets a token (stays empty) */
        int32_t next_pos[2] = {0, 0};
        for (int round = 0; round < 3; ++round) {
            const int n_new = 3;
            uint16_t *kn = (uint16_t *)malloc((size_t)nseg * n_new * D * 2), *vn = (uint16_t *)malloc((size_t)nseg * n_new * D * 2);
            float *lb = (float *)malloc((size_t)nseg * n_new * 4), *lt = (float *)malloc((size_t)nseg * n_new * 4);
            int32_t *pn = (int32_t *)malloc((size_t)nseg * n_new * 4);
            for (int64_t i = 0; i < nseg * n_new * D; ++i) { kn[i] = (uint16_t)(0x3c00 + rnd() % 0x400); vn[i] = (uint16_t)(0xbc00 + rnd() % 0x400); }
            for (int64_t g = 0; g < nseg; ++g) {
                const int seq = (int)(g / (sh.n_layers * sh.n_kv_heads));
                const int take = g == 3 ? 0 : (seq == 0 ? 3 : 2);      /* sequence 1 brings fewer tokens: padding */
                for (int r = 0; r < n_new; ++r) {
                    lb[g * n_new + r] = (rnd() % 4 == 0) ? 0.0f : -(float)(rnd() % 3 + 1) * 0.125f;   /* few values: ties */
                    lt[g * n_new + r] = 0.25f;
                    pn[g * n_new + r] = r < take ? next_pos[seq] + r : -1;
                }
            }
            CHECK(kvo_append(&sh, &c, kn, vn, lb, with_tail ? lt : NULL, pn, n_new) == 0);
            next_pos[0] += 3;
            next_pos[1] += 2;
            free(kn); free(vn); free(lb); free(lt); free(pn);
        }
        CHECK(c.seg_len[0] == 9 && c.seg_len[3] == 0 && c.seg_len[nseg - 1] == 6);
        const int32_t now[2] = {next_pos[0] - 1, next_pos[1] - 1};
        float *score = (float *)calloc((size_t)c.cap, 4);
        double *score64 = (double *)calloc((size_t)c.cap, 8);
        kvo_score(&sh, &c, now, score);
        kvo_score_horizon(&sh, &c, now, 2, score64);
        kvo_score_horizon(&sh, &c, now, 0, score64);
        uint8_t *keep = (uint8_t *)calloc((size_t)c.cap, 1);
        int32_t *kept = (int32_t *)calloc((size_t)nseg, 4);
        uint32_t thr[2];
        const int64_t budgets[5][2] = {{0, 1000}, {1, 5}, {17, 11}, {27, 24}, {1000, 0}};
        for (int b = 0; b < 5; ++b) {
            CHECK(kvo_select(&sh, &c, score, budgets[b], keep, kept, thr) == 0);
            for (int seq = 0; seq < 2; ++seq) {
                int64_t total = 0, have = 0;
                for (int64_t g = seq * 4; g < seq * 4 + 4; ++g) { total += kept[g]; have += c.seg_len[g]; }
                CHECK(total == (budgets[b][seq] < have ? budgets[b][seq] : have));
            }
            kvo_cache tight = make_cache(&sh, 1, with_tail);          /* too small unless nothing survives */
            int64_t all = 0;
            for (int64_t g = 0; g < nseg; ++g) all += kept[g];
            CHECK((kvo_compact(&sh, &c, keep, &tight, 0) == 0) == (all <= 1));
            free_cache(&tight);
            kvo_cache dst = make_cache(&sh, all + nseg * 2, with_tail);
            CHECK(kvo_compact(&sh, &c, keep, &dst, 2) == 0);
            uint16_t *q = (uint16_t *)malloc((size_t)sh.n_seq * sh.n_layers * sh.n_q_heads * D * 2);
            for (int i = 0; i < sh.n_seq * sh.n_layers * sh.n_q_heads * D; ++i) q[i] = (uint16_t)(0x3c00 + rnd() % 0x300);
            double *out = (double *)calloc((size_t)sh.n_seq * sh.n_layers * sh.n_q_heads * D, 8);
            double *lse = (double *)calloc((size_t)sh.n_seq * sh.n_layers * sh.n_q_heads, 8);
            kvo_attend(&sh, &dst, q, 0, sh.n_layers, 0.35, out, lse);
            kvo_attend(&sh, &dst, q, 1, 2, 0.35, out, NULL);
            kvo_attend_soft(&sh, &dst, q, now, 0, sh.n_layers, 0.35, out, lse);
            for (int i = 0; i < sh.n_seq * sh.n_layers * sh.n_q_heads * D; ++i) CHECK(out[i] == out[i]);   /* never NaN */
            double occ[2];
            kvo_occupancy(&sh, &dst, now, occ);
            CHECK(occ[0] >= 0 && occ[1] >= 0);
            free(q); free(out); free(lse);
            free_cache(&dst);
        }
        free(score); free(score64); free(keep); free(kept);
        free_cache(&c);
    }
    /* retention gate on non-square shapes, a layer range, both horizon branches */
    {
        const int L = 3, H = 2, dm = 24, dg = 10, dp = 5, n_tok = 4;
        uint16_t *w1 = (uint16_t *)malloc((size_t)L * dg * dm * 2), *w2 = (uint16_t *)malloc((size_t)L * H * dp * dg * 2);
        float *c1 = (float *)malloc((size_t)L * dg * 4), *c2 = (float *)malloc((size_t)L * H * dp * 4), wg[5];
        uint16_t *x = (uint16_t *)malloc((size_t)2 * n_tok * dm * 2);
        for (int i = 0; i < L * dg * dm; ++i) w1[i] = (uint16_t)((rnd() & 1 ? 0x3c00 : 0xbc00) + rnd() % 0x200);
        for (int i = 0; i < L * H * dp * dg; ++i) w2[i] = (uint16_t)((rnd() & 1 ? 0x3c00 : 0xbc00) + rnd() % 0x200);
        for (int i = 0; i < L * dg; ++i) c1[i] = 0.1f;
        for (int i = 0; i < L * H * dp; ++i) c2[i] = -0.1f;
        for (int i = 0; i < dp; ++i) wg[i] = 0.3f;
        for (int i = 0; i < 2 * n_tok * dm; ++i) x[i] = (uint16_t)((rnd() & 1 ? 0x3c00 : 0xbc00) + rnd() % 0x200);
        const kvo_gate g = {L, H, dm, dg, dp, w1, c1, w2, c2, wg, 18.0f};
        double *z = (double *)calloc((size_t)n_tok * L * H, 8), *lb = (double *)calloc((size_t)n_tok * L * H, 8);
        double *lt = (double *)calloc((size_t)n_tok * L * H, 8);
        kvo_gate_forward(&g, x, n_tok, 1, 3, 2, z, lb, lt);
        kvo_gate_forward(&g, x, n_tok, 1, 3, 0, NULL, lb, lt);
        kvo_gate_forward(&g, x, n_tok, 0, 2, 5, z, lb, NULL);
        for (int i = 0; i < n_tok * L * H; ++i) CHECK(lb[i] <= 0.0);
        free(w1); free(w2); free(c1); free(c2); free(x); free(z); free(lb); free(lt);
    }
    CHECK(kvo_key_of_score(-0.0f) < kvo_key_of_score(0.0f));
    printf("selftest ok (%d threads)\n", kvo_threads());
    return 0;
}
