/*
 * CPU oracle for the decode-time hot path of global retention-based KV eviction.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path, and the product path never calls it.
 *
 * What it defines (all citations are to the paper):
 *   kvo_score    Sec. 4.2, Eq. (global_score) in log domain.  At lookahead horizon
 *                T-t = 1: log G~ = (t+1-i) * log(beta), one fp32 multiply.  For a
 *                longer horizon H the cache carries, per entry, the constant
 *                log_tail = log(sum_{k<H} beta^k) fixed when the token was cached,
 *                and log G~ = fma(t+1-i, log(beta), log_tail), one fp32 fused
 *                multiply-add.                                       [pinned]
 *   kvo_score_horizon
 *                Sec. 4.2, Eq. (global_score) for a general horizon H = T-t,
 *                log domain, fp64.                                   [pinned]
 *   kvo_select   Sec. 4.2, eviction rule: keep the M_global entries with the
 *                largest score over all layers and heads of a sequence.
 *                Written as the definition: full sort, take the first B.
 *                                                                    [pinned]
 *   kvo_compact  Sec. 4.2 "Implementation details": every (layer, head) keeps
 *                its own variable-length logical KV sequence.  Written as a
 *                stable filter per segment.                          [pinned]
 *   kvo_attend   Sec. 2.1, Eq. (reform) with r in {0,1}: softmax attention
 *                over the retained entries only, fp64.               [pinned]
 *   kvo_attend_soft  Sec. 2.2: retention-gated (soft) attention, weights
 *                beta^(t-i) e^z, fp64.                               [pinned]
 *   kvo_occupancy    Sec. 4.1: expected occupancy sum of beta^(t-i). [pinned]
 *   kvo_append   bookkeeping: a new token enters every segment's list.
 *   kvo_gate_forward  Sec. 4.1 "Weight-tied retention gates": beta = sigmoid(w_g . Proj_{l,h}(x)
 *                + b_g) for a token entering the cache, fp64, written as the
 *                nested sums of the definition.                      [pinned]
 *
 * Readings of points the paper leaves open (listed again in the design notes):
 *   - elapsed steps = now + 1 - pos  (the score equation, not the t-i of the
 *     training-time retention weight); the newest token has 1.
 *   - total order for the selection: score bits descending (through the usual
 *     order-preserving map of IEEE-754 binary32 to uint32, so -0 < +0), then
 *     layer ascending, head ascending, position ascending.
 *   - budgets are per sequence.
 *   - the appended token competes like every other entry.
 *   - an empty segment attends to nothing: output 0, lse -inf.
 *
 *   - the retention gate: the paper fixes Proj_{l,h} as a two-layer MLP with hidden
 *     width d_g inside a per-block gate, and the tied readout (w_g, b_g); it does not
 *     print the activation, the width of Proj's output or which layer is per head.
 *     Taken here: one first layer per transformer block, shared by its heads,
 *     u = silu(W1_l x + c1_l); a second, linear layer per (block, head),
 *     p = W2_{l,h} u + c2_{l,h} of width d_p; z = w_g . p + b_g; beta = sigmoid(z).
 *
 * Layout of a ragged cache (same meaning as at the library boundary, but these
 * are HOST pointers):
 *   k, v       bf16 bit patterns, [cap][D] row-major
 *   log_beta   fp32 [cap]
 *   log_tail   fp32 [cap] or NULL (NULL = horizon 1): log of the geometric tail sum
 *   pos        int32 [cap], strictly ascending inside a segment
 *   seg_start  int64 [nseg], nseg = S*L*Hkv, segment g = (seq*L + layer)*Hkv + head
 *   seg_len    int32 [nseg]
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t n_seq, n_layers, n_kv_heads, n_q_heads, head_dim;
} kvo_shape;

typedef struct {
    uint16_t *k, *v;
    float *log_beta;
    int32_t *pos;
    int64_t *seg_start;
    int32_t *seg_len;
    int64_t cap;
    float *log_tail;
} kvo_cache;

static int64_t kvo_nseg(const kvo_shape *sh) {
    return (int64_t)sh->n_seq * sh->n_layers * sh->n_kv_heads;
}

static double bf16_to_f64(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* Order-preserving image of a binary32 value in uint32: a < b as floats
 * (with -0 < +0) iff key(a) < key(b) as unsigned integers. */
static uint32_t kvo_key32(float s) {
    uint32_t u;
    memcpy(&u, &s, 4);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

uint32_t kvo_key_of_score(float s) { return kvo_key32(s); }

/* Sec. 4.2, Eq. (global_score).  T-t = 1: G~ = beta^(t+1-i); in log domain this
 * is one binary32 multiply of the (exactly representable) elapsed-step count
 * with log(beta).  With a horizon tail: G~ = beta^(t+1-i) * sum_{k<H} beta^k, in
 * log domain one correctly rounded binary32 fused multiply-add with the cached
 * log of the tail sum. */
void kvo_score(const kvo_shape *sh, const kvo_cache *c, const int32_t *now, float *score_out) {
    int64_t nseg = kvo_nseg(sh);
    int64_t per_seq = (int64_t)sh->n_layers * sh->n_kv_heads;
    for (int64_t g = 0; g < nseg; ++g) {
        int64_t seq = g / per_seq;
        for (int32_t j = 0; j < c->seg_len[g]; ++j) {
            int64_t e = c->seg_start[g] + j;
            int32_t elapsed = now[seq] + 1 - c->pos[e];
            volatile float fe = (float)elapsed; /* volatile: no contraction, no widening */
            if (c->log_tail) {
                score_out[e] = fmaf(fe, c->log_beta[e], c->log_tail[e]);
            } else {
                volatile float s = fe * c->log_beta[e];
                score_out[e] = s;
            }
        }
    }
}

/* Sec. 4.2, Eq. (global_score), general horizon H >= 1 (H <= 0 means the limit
 * H -> infinity):  log G~ = elapsed*log(beta) + log(sum_{k=0}^{H-1} beta^k).
 * fp64 throughout; the geometric sum is written out term by term. */
void kvo_score_horizon(const kvo_shape *sh, const kvo_cache *c, const int32_t *now, int32_t horizon,
                       double *score_out) {
    int64_t nseg = kvo_nseg(sh);
    int64_t per_seq = (int64_t)sh->n_layers * sh->n_kv_heads;
    for (int64_t g = 0; g < nseg; ++g) {
        int64_t seq = g / per_seq;
        for (int32_t j = 0; j < c->seg_len[g]; ++j) {
            int64_t e = c->seg_start[g] + j;
            double lb = (double)c->log_beta[e];
            double beta = exp(lb);
            double elapsed = (double)(now[seq] + 1 - c->pos[e]);
            double tail;
            if (horizon <= 0) {
                tail = -log1p(-beta); /* sum_{k>=0} beta^k = 1/(1-beta) */
            } else {
                double sum = 0.0, term = 1.0;
                for (int32_t k = 0; k < horizon; ++k) {
                    sum += term;
                    term *= beta;
                }
                tail = log(sum);
            }
            score_out[e] = elapsed * lb + tail;
        }
    }
}

typedef struct {
    uint32_t key;
    int32_t layer, head, pos;
    int64_t entry;
} kvo_cand;

static int kvo_cand_cmp(const void *pa, const void *pb) {
    const kvo_cand *a = (const kvo_cand *)pa, *b = (const kvo_cand *)pb;
    if (a->key != b->key) return a->key > b->key ? -1 : 1; /* larger score first */
    if (a->layer != b->layer) return a->layer < b->layer ? -1 : 1;
    if (a->head != b->head) return a->head < b->head ? -1 : 1;
    if (a->pos != b->pos) return a->pos < b->pos ? -1 : 1;
    return 0;
}

/* Sec. 4.2 eviction rule, per sequence: sort every cached entry of the sequence
 * by the total order above and keep the first min(budget, count).
 * keep_out[e] is written (0/1) for every entry inside a segment; kept_out[g] is
 * the number kept in segment g; thr_key_out[seq] (optional) is the key of the
 * last kept entry, or 0xFFFFFFFF when nothing is kept.
 * Returns 0, or -1 if memory for the candidate list cannot be obtained. */
int kvo_select(const kvo_shape *sh, const kvo_cache *c, const float *score, const int64_t *budget,
               uint8_t *keep_out, int32_t *kept_out, uint32_t *thr_key_out) {
    int64_t per_seq = (int64_t)sh->n_layers * sh->n_kv_heads;
    for (int32_t seq = 0; seq < sh->n_seq; ++seq) {
        int64_t count = 0;
        for (int64_t g = seq * per_seq; g < (seq + 1) * per_seq; ++g) count += c->seg_len[g];
        kvo_cand *cand = (kvo_cand *)malloc((size_t)(count > 0 ? count : 1) * sizeof(kvo_cand));
        if (!cand) return -1;
        int64_t n = 0;
        for (int64_t g = seq * per_seq; g < (seq + 1) * per_seq; ++g) {
            int32_t layer = (int32_t)((g - seq * per_seq) / sh->n_kv_heads);
            int32_t head = (int32_t)((g - seq * per_seq) % sh->n_kv_heads);
            kept_out[g] = 0;
            for (int32_t j = 0; j < c->seg_len[g]; ++j) {
                int64_t e = c->seg_start[g] + j;
                cand[n].key = kvo_key32(score[e]);
                cand[n].layer = layer;
                cand[n].head = head;
                cand[n].pos = c->pos[e];
                cand[n].entry = e;
                keep_out[e] = 0;
                ++n;
            }
        }
        qsort(cand, (size_t)n, sizeof(kvo_cand), kvo_cand_cmp);
        int64_t b = budget[seq] < 0 ? 0 : budget[seq];
        int64_t take = b < n ? b : n;
        for (int64_t r = 0; r < take; ++r) {
            keep_out[cand[r].entry] = 1;
            kept_out[(seq * per_seq) + (int64_t)cand[r].layer * sh->n_kv_heads + cand[r].head] += 1;
        }
        if (thr_key_out) thr_key_out[seq] = take > 0 ? cand[take - 1].key : 0xFFFFFFFFu;
        free(cand);
    }
    return 0;
}

/* Stable filter per segment.  dst segment g starts at sum_{g'<g}(kept[g'] + reserve),
 * holds the kept entries of src segment g in their original order, and is followed
 * by `reserve` free slots.  Rows are copied byte for byte.
 * Returns 0, or -4 if dst->cap is too small (nothing is written then). */
int kvo_compact(const kvo_shape *sh, const kvo_cache *src, const uint8_t *keep, kvo_cache *dst,
                int32_t reserve) {
    int64_t nseg = kvo_nseg(sh);
    int D = sh->head_dim;
    int64_t need = 0;
    for (int64_t g = 0; g < nseg; ++g) {
        int64_t kept = 0;
        for (int32_t j = 0; j < src->seg_len[g]; ++j) kept += keep[src->seg_start[g] + j] ? 1 : 0;
        need += kept + reserve;
    }
    if (need > dst->cap) return -4;
    int64_t cursor = 0;
    for (int64_t g = 0; g < nseg; ++g) {
        dst->seg_start[g] = cursor;
        int32_t out = 0;
        for (int32_t j = 0; j < src->seg_len[g]; ++j) {
            int64_t e = src->seg_start[g] + j;
            if (!keep[e]) continue;
            int64_t d = cursor + out;
            memcpy(dst->k + d * D, src->k + e * D, (size_t)D * 2);
            memcpy(dst->v + d * D, src->v + e * D, (size_t)D * 2);
            dst->log_beta[d] = src->log_beta[e];
            if (src->log_tail && dst->log_tail) dst->log_tail[d] = src->log_tail[e];
            dst->pos[d] = src->pos[e];
            ++out;
        }
        dst->seg_len[g] = out;
        cursor += out + reserve;
    }
    return 0;
}

/* Sec. 2.1, Eq. (reform) with r in {0,1}: for KV head h of layer l and each of
 * its G = Hq/Hkv query heads hq = h*G + j,
 *   z_i = (q . k_i) * scale,  alpha = softmax(z),  o = sum_i alpha_i v_i
 * over the entries present in the segment.  q is bf16 [S][L][Hq][D]; out is
 * fp64 [S][L][Hq][D]; lse (optional) is fp64 [S][L][Hq] = log sum_i exp(z_i).
 * Layers outside [layer_begin, layer_end) are not touched. */
static void kvo_attend_impl(const kvo_shape *sh, const kvo_cache *c, const uint16_t *q, const int32_t *now,
                            int32_t layer_begin, int32_t layer_end, double scale, double *out, double *lse) {
    int D = sh->head_dim;
    int G = sh->n_q_heads / sh->n_kv_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t w = 0; w < (int64_t)sh->n_seq * (layer_end - layer_begin) * sh->n_kv_heads; ++w) {
        int32_t head = (int32_t)(w % sh->n_kv_heads);
        int32_t layer = layer_begin + (int32_t)((w / sh->n_kv_heads) % (layer_end - layer_begin));
        int32_t seq = (int32_t)(w / ((int64_t)sh->n_kv_heads * (layer_end - layer_begin)));
        int64_t g = ((int64_t)seq * sh->n_layers + layer) * sh->n_kv_heads + head;
        int32_t n = c->seg_len[g];
        double *z = (double *)malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
        for (int j = 0; j < G; ++j) {
            int64_t hq = ((int64_t)seq * sh->n_layers + layer) * sh->n_q_heads + (int64_t)head * G + j;
            const uint16_t *qv = q + hq * D;
            double *o = out + hq * D;
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            if (n == 0) {
                if (lse) lse[hq] = -INFINITY;
                continue;
            }
            double m = -INFINITY;
            for (int32_t i = 0; i < n; ++i) {
                const uint16_t *kr = c->k + (c->seg_start[g] + i) * D;
                double dot = 0.0;
                for (int d = 0; d < D; ++d) dot += bf16_to_f64(qv[d]) * bf16_to_f64(kr[d]);
                z[i] = dot * scale;
                if (now) /* retention weight beta^(t-i) as a logit bias (t-i) * log(beta) */
                    z[i] += (double)(now[seq] - c->pos[c->seg_start[g] + i]) * (double)c->log_beta[c->seg_start[g] + i];
                if (z[i] > m) m = z[i];
            }
            double denom = 0.0;
            for (int32_t i = 0; i < n; ++i) denom += exp(z[i] - m);
            for (int32_t i = 0; i < n; ++i) {
                double alpha = exp(z[i] - m) / denom;
                const uint16_t *vr = c->v + (c->seg_start[g] + i) * D;
                for (int d = 0; d < D; ++d) o[d] += alpha * bf16_to_f64(vr[d]);
            }
            if (lse) lse[hq] = m + log(denom);
        }
        free(z);
    }
}

void kvo_attend(const kvo_shape *sh, const kvo_cache *c, const uint16_t *q, int32_t layer_begin,
                int32_t layer_end, double scale, double *out, double *lse) {
    kvo_attend_impl(sh, c, q, NULL, layer_begin, layer_end, scale, out, lse);
}

/* Sec. 2.2, retention-gated attention (the soft form the gates are trained with):
 *   alpha~_i = beta_i^(t-i) e^(z_i) / sum_j beta_j^(t-j) e^(z_j),   o~ = sum_i alpha~_i v_i,
 * t = now[seq] the position of the query; same layout and conventions as kvo_attend
 * (lse is the log of the weighted denominator). */
void kvo_attend_soft(const kvo_shape *sh, const kvo_cache *c, const uint16_t *q, const int32_t *now,
                     int32_t layer_begin, int32_t layer_end, double scale, double *out, double *lse) {
    kvo_attend_impl(sh, c, q, now, layer_begin, layer_end, scale, out, lse);
}

/* Sec. 4.1, inner sum of the global capacity loss: the expected cache occupancy of a sequence at
 * step t = now[seq],  occ = sum over its layers, heads and cached entries of beta^(t-i). */
void kvo_occupancy(const kvo_shape *sh, const kvo_cache *c, const int32_t *now, double *occ_out) {
    int64_t per_seq = (int64_t)sh->n_layers * sh->n_kv_heads;
    for (int32_t seq = 0; seq < sh->n_seq; ++seq) {
        double sum = 0.0;
        for (int64_t g = seq * per_seq; g < (seq + 1) * per_seq; ++g)
            for (int32_t j = 0; j < c->seg_len[g]; ++j) {
                int64_t e = c->seg_start[g] + j;
                sum += exp((double)(now[seq] - c->pos[e]) * (double)c->log_beta[e]);
            }
        occ_out[seq] = sum;
    }
}

/* A new token (or n_new consecutive tokens) enters every segment: rows are
 * written behind the segment's current end.  k_new/v_new are [nseg][n_new][D],
 * log_beta_new/log_tail_new/pos_new are [nseg][n_new] (log_tail_new only for caches
 * that carry a horizon tail).  Returns 0, or -4 when a segment has
 * no room before the next segment's start (or the end of the buffer). */
int kvo_append(const kvo_shape *sh, kvo_cache *c, const uint16_t *k_new, const uint16_t *v_new,
               const float *log_beta_new, const float *log_tail_new, const int32_t *pos_new, int32_t n_new) {
    int64_t nseg = kvo_nseg(sh);
    int D = sh->head_dim;
    /* a segment takes its new rows up to the first one with a negative position (padding) */
    for (int64_t g = 0; g < nseg; ++g) {
        int32_t cnt = 0;
        while (cnt < n_new && pos_new[g * n_new + cnt] >= 0) ++cnt;
        int64_t end = c->seg_start[g] + c->seg_len[g];
        int64_t limit = (g + 1 < nseg) ? c->seg_start[g + 1] : c->cap;
        if (end + cnt > limit) return -4;
    }
    for (int64_t g = 0; g < nseg; ++g) {
        int32_t cnt = 0;
        while (cnt < n_new && pos_new[g * n_new + cnt] >= 0) ++cnt;
        for (int32_t r = 0; r < cnt; ++r) {
            int64_t e = c->seg_start[g] + c->seg_len[g] + r;
            memcpy(c->k + e * D, k_new + (g * n_new + r) * D, (size_t)D * 2);
            memcpy(c->v + e * D, v_new + (g * n_new + r) * D, (size_t)D * 2);
            c->log_beta[e] = log_beta_new[g * n_new + r];
            if (c->log_tail && log_tail_new) c->log_tail[e] = log_tail_new[g * n_new + r];
            c->pos[e] = pos_new[g * n_new + r];
        }
        c->seg_len[g] += cnt;
    }
    return 0;
}

/* ---------------------------------------------------------------------------------------------
 * Retention gate (Sec. 4.1, "Weight-tied retention gates"; Sec. 5.1 implementation details:
 * a small MLP per transformer block with hidden width d_g, Proj a two-layer MLP, the final linear
 * layer (w_g, b_g) tied across all layers and heads; Sec. 3.2: beta is computed once, when the
 * token enters the cache).
 *
 * Weights (HOST pointers): w1 bf16 [L][d_g][d_model], c1 fp32 [L][d_g], w2 bf16 [L][H][d_p][d_g],
 * c2 fp32 [L][H][d_p], w_g fp32 [d_p], b_g.  x: bf16 [layer_end - layer_begin][n_tok][d_model], the
 * token representation that enters each block of the layer range.  Outputs, fp64, indexed
 * [(tok * L + layer) * H + head] (for one token per sequence that is segment order); entries of
 * layers outside the range are left alone:
 *   z_out         the gate logit w_g . Proj(x) + b_g
 *   log_beta_out  log sigmoid(z) = -log(1 + e^-z)
 *   log_tail_out  (optional) log sum_{k<H} beta^k for lookahead horizon H (Eq. global_score);
 *                 H = 0 stands for the limit, -log(1 - beta). */
typedef struct {
    int32_t n_layers, n_heads, d_model, d_g, d_p;
    const uint16_t *w1;
    const float *c1;
    const uint16_t *w2;
    const float *c2;
    const float *w_g;
    float b_g;
} kvo_gate;

void kvo_gate_forward(const kvo_gate *g, const uint16_t *x, int32_t n_tok, int32_t layer_begin, int32_t layer_end,
                      int32_t horizon, double *z_out, double *log_beta_out, double *log_tail_out) {
    const int L = g->n_layers, H = g->n_heads, dm = g->d_model, dg = g->d_g, dp = g->d_p;
    double *u = (double *)malloc(sizeof(double) * (size_t)dg);
    for (int layer = layer_begin; layer < layer_end; ++layer) {
        for (int tok = 0; tok < n_tok; ++tok) {
            const uint16_t *xt = x + ((size_t)(layer - layer_begin) * n_tok + tok) * dm;
            for (int j = 0; j < dg; ++j) {                 /* first layer, shared by the heads of the block */
                const uint16_t *row = g->w1 + ((size_t)layer * dg + j) * dm;
                double a = (double)g->c1[(size_t)layer * dg + j];
                for (int k = 0; k < dm; ++k) a += bf16_to_f64(row[k]) * bf16_to_f64(xt[k]);
                u[j] = a / (1.0 + exp(-a));                /* silu */
            }
            for (int h = 0; h < H; ++h) {
                double z = (double)g->b_g;
                for (int i = 0; i < dp; ++i) {             /* Proj's second layer, then the tied readout */
                    const uint16_t *row = g->w2 + (((size_t)layer * H + h) * dp + i) * dg;
                    double p = (double)g->c2[((size_t)layer * H + h) * dp + i];
                    for (int j = 0; j < dg; ++j) p += bf16_to_f64(row[j]) * u[j];
                    z += (double)g->w_g[i] * p;
                }
                const size_t o = ((size_t)tok * L + layer) * H + h;
                const double lb = z >= 0 ? -log1p(exp(-z)) : z - log1p(exp(z));
                if (z_out) z_out[o] = z;
                log_beta_out[o] = lb;
                if (log_tail_out) {
                    if (horizon <= 0) {
                        log_tail_out[o] = -log(-expm1(lb));
                    } else {
                        const double beta = exp(lb);
                        double sum = 0.0, term = 1.0;
                        for (int k = 0; k < horizon; ++k) {
                            sum += term;
                            term *= beta;
                        }
                        log_tail_out[o] = log(sum);
                    }
                }
            }
        }
    }
    free(u);
}

#ifdef _OPENMP
#include <omp.h>
int kvo_threads(void) { return omp_get_max_threads(); }
/* Number of threads the attention loop may use from now on (for timing the oracle on one core and on all). */
void kvo_set_threads(int n) { if (n >= 1) omp_set_num_threads(n); }
#else
int kvo_threads(void) { return 1; }
#endif
