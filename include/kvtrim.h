/*
 * kvtrim: decode-time hot path of global retention-based KV-cache eviction on
 * one MI355X (gfx950).  C ABI; every data pointer is CALLER-OWNED DEVICE memory
 * unless a comment says "host"; `hip_stream` is a hipStream_t passed as void*
 * (NULL = the default stream).
 *
 * One decode / eviction step is
 *     kvtrim_append  (support: the new token enters every segment)
 *  -> kvtrim_score          stage 1      } or both in one call:
 *  -> kvtrim_select_global  stage 2      } kvtrim_score_select
 *  -> kvtrim_compact        stage 3      } or both in one call:
 *  -> kvtrim_decode_attn    stage 4      } kvtrim_compact_attn
 *
 * Common rules
 *  - Every call returns a kvtrim_status; nothing throws or aborts.  Host-visible
 *    argument errors (null pointers, bad shapes, capacity larger than the context
 *    was created for) return KVTRIM_EINVAL before anything is launched.
 *  - The five step calls only enqueue kernels on `hip_stream`: no allocation, no
 *    synchronisation, no host read-back, no memset nodes (a step can be captured
 *    in a HIP graph).  Conditions only the device can see (a destination too
 *    small, a `kept` array that disagrees with the mask) set a sticky device flag;
 *    the kernel that finds the condition writes nothing out of bounds, and later
 *    kernels return early.  The flag is STICKY ACROSS CALLS: while it is set, the
 *    compaction and attention kernels of every later call on the context (also the
 *    replays of a captured graph) do nothing and leave their outputs as they were,
 *    although the host-side status of those calls is KVTRIM_OK - the state the flag
 *    describes is one the next kernels cannot safely build on.  kvtrim_poll_error
 *    reads and clears it: poll after the calls whose device-side errors matter
 *    (an append that may run out of room, a compaction into a tight destination)
 *    and at least once per batch of replayed steps.
 *  - A context owns one workspace (allocated in kvtrim_create) that every call
 *    reuses: calls on one context must be ordered on one stream and come from one
 *    host thread at a time (the context also keeps the last error text and the
 *    profiling state without locks).  Different contexts are independent.
 *
 * Ragged cache (kvtrim_cache)
 *  A "segment" is the logical KV list of one (sequence, layer, KV head); segment
 *  index g = (seq * n_layers + layer) * n_kv_heads + head; nseg = n_seq*n_layers*
 *  n_kv_heads.  Segment g occupies entries [seg_start[g], seg_start[g]+seg_len[g])
 *  of the flat arrays.  Segments are laid out in ascending g without overlap
 *  (seg_start[g] + seg_len[g] <= seg_start[g+1]); free slots may follow a segment.
 *  Inside a segment `pos` is strictly ascending.
 *      k, v       bf16 [cap_entries][head_dim], row-major, 16-byte aligned base
 *      log_beta   fp32 [cap_entries]   log of the retention coefficient, <= 0, not NaN
 *      pos        int32 [cap_entries]  token position of the entry
 *      log_tail   fp32 [cap_entries] or NULL: only for a lookahead horizon H > 1 of the
 *                 score, log(sum_{k<H} beta^k), fixed like beta when the token is cached
 *      seg_start  int64 [nseg]
 *      seg_len    int32 [nseg]
 *  Entries outside every segment are never read; what the calls leave in the
 *  corresponding slots of their outputs is unspecified.
 */
#ifndef KVTRIM_H
#define KVTRIM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kvtrim_ctx kvtrim_ctx; /* opaque */

typedef enum {
    KVTRIM_OK = 0,
    KVTRIM_EINVAL = -1, /* bad argument seen on the host */
    KVTRIM_ENOMEM = -2, /* workspace allocation failed */
    KVTRIM_EHIP = -3,   /* a HIP call failed; text in kvtrim_last_error */
    KVTRIM_ECAP = -4,   /* device-side: destination / segment has no room */
    KVTRIM_EMISMATCH = -5, /* device-side: `kept` does not match the mask */
    KVTRIM_ELAYOUT = -6    /* device-side: segment table inconsistent with cap_entries */
} kvtrim_status;

typedef struct {
    int32_t n_seq;      /* S >= 1 */
    int32_t n_layers;   /* L >= 1 */
    int32_t n_kv_heads; /* Hkv >= 1 */
    int32_t n_q_heads;  /* Hq, a multiple of Hkv, Hq/Hkv <= 8 */
    int32_t head_dim;   /* D: 64 or 128 */
    int64_t max_entries; /* largest cap_entries of any cache passed to this context; 1 .. 2^31 - 4096
                          * (entries of a segment are indexed with 32-bit integers plus a chunk of slack) */
} kvtrim_config;

typedef struct {
    void *k;
    void *v;
    float *log_beta;
    int32_t *pos;
    int64_t *seg_start;
    int32_t *seg_len;
    int64_t cap_entries;
    float *log_tail; /* NULL = lookahead horizon 1 */
} kvtrim_cache;

/* Context life cycle (host side, synchronous).  kvtrim_create allocates the
 * workspace on the current device; kvtrim_workspace_bytes says how large it is.
 * One tuning knob is read from the environment at creation: KVTRIM_ATT_CHUNK = rows per
 * split-K chunk of the stand-alone attention kernel (a multiple of 64 in [256, 65536];
 * default 512, and larger for caches above 8 M entries so that at most 16384 full chunks
 * exist).  It changes the order of floating-point sums in attention, nothing else. */
kvtrim_status kvtrim_create(kvtrim_ctx **out, const kvtrim_config *cfg);
kvtrim_status kvtrim_destroy(kvtrim_ctx *ctx);
size_t kvtrim_workspace_bytes(const kvtrim_config *cfg);
const char *kvtrim_last_error(const kvtrim_ctx *ctx); /* host string, owned by ctx; ctx = NULL: why the calling
                                                         thread's last kvtrim_create failed */

/* Outside the hot loop: waits for `hip_stream`, then returns and clears the
 * sticky device flag (KVTRIM_OK, KVTRIM_ECAP, KVTRIM_EMISMATCH or KVTRIM_ELAYOUT). */
kvtrim_status kvtrim_poll_error(kvtrim_ctx *ctx, void *hip_stream);

/* Stage 1 - retention score, Sec. 4.2 Eq. (global_score), in log domain.
 * Lookahead T-t = 1 (c->log_tail == NULL):
 *     score[e] = float(now[seq] + 1 - pos[e]) * log_beta[e],
 * exactly one IEEE binary32 multiply (round to nearest even).
 * Lookahead T-t = H > 1 or H -> infinity (c->log_tail != NULL; Sec. 5.1 uses H = 2):
 *     score[e] = fma(float(now[seq] + 1 - pos[e]), log_beta[e], log_tail[e]),
 * exactly one correctly rounded binary32 fused multiply-add; log_tail[e] is the
 * log of the factor (1 - beta^H)/(1 - beta) of the equation.
 * now[seq] is the position of the newest token of the sequence (device int32 [n_seq]).
 * score_out: device fp32 [cap_entries]; written for entries inside segments. */
kvtrim_status kvtrim_score(kvtrim_ctx *ctx, const kvtrim_cache *c, const int32_t *now,
                           float *score_out, void *hip_stream);

/* Stage 2 - global eviction rule, Sec. 4.2: per sequence keep the
 * min(budget[seq], count) entries that come first in the total order
 *   (score descending by its IEEE bits mapped order-preservingly to uint32, so
 *    -0 < +0; then layer ascending; head ascending; position ascending).
 * No per-layer or per-head budget exists.  budget: device int64 [n_seq]
 * (negative counts as 0).
 * keep_out: device uint8 [cap_entries], 1 = retained, written for entries inside
 * segments.  kept_out: device int32 [nseg], retained entries per segment.
 * thr_key_out: optional (may be NULL) device uint32 [n_seq], key of the last
 * retained entry in that order, 0xFFFFFFFF when nothing is retained. */
kvtrim_status kvtrim_select_global(kvtrim_ctx *ctx, const kvtrim_cache *c, const float *score,
                                   const int64_t *budget, uint8_t *keep_out, int32_t *kept_out,
                                   uint32_t *thr_key_out, void *hip_stream);

/* Stages 1 + 2 in one call: leaves in score_out, keep_out, kept_out and thr_key_out exactly what
 *     kvtrim_score(c, now) -> kvtrim_select_global(c, score_out, budget)
 * leave there (Sec. 4.2: Eq. (global_score), then the global eviction rule; same total order, same bits), with
 * fewer passes over the cache.  Arguments as in those two calls.
 * evict_hint (host value, a performance hint only - every value gives the same results): about how many entries
 * each sequence loses in this call, e.g. n_layers * n_kv_heads * (tokens appended since the last selection) for a
 * decode step at the budget; 0 = unknown or many (the first eviction after a prefill, a prefill chunk).
 *   hint 0, or one beyond an eighth of the context's candidate list (511 for up to 256 sequences): the radix
 *     passes of kvtrim_select_global, the first of which computes the score as it goes.
 *   otherwise: one pass scores every entry and lists those whose key lies below a bound the context carries from
 *     its previous selection; while a sequence needs k evictions and at least k + 1 entries are listed, the lowest
 *     k + 1 entries of the order are among them and are ranked directly; then the mask pass.  Two kernels.  The
 *     bound follows the threshold from call to call by itself.  A sequence whose list comes up short (no previous
 *     selection on this context, a jump in the budget or the workload) or overflows is selected by a slow single-
 *     block fallback inside the same kernel - correct, but about as slow as a millisecond per 2 M entries, so pass
 *     0 when the number of evictions is not small.
 * Device-side error: KVTRIM_ELAYOUT for a segment table that does not fit cap_entries or overlaps. */
kvtrim_status kvtrim_score_select(kvtrim_ctx *ctx, const kvtrim_cache *c, const int32_t *now, const int64_t *budget,
                                  float *score_out, uint8_t *keep_out, int32_t *kept_out, uint32_t *thr_key_out,
                                  int64_t evict_hint, void *hip_stream);

/* Diagnostics of kvtrim_score_select's decode-step form (outside the hot loop: waits for `hip_stream`): how many
 * per-sequence selections since the context was created were resolved from the candidate list and how many by the
 * slow single-block fallback.  Both are host int64. */
kvtrim_status kvtrim_select_path_counts(kvtrim_ctx *ctx, int64_t *from_list_host, int64_t *fallback_host,
                                        void *hip_stream);

/* Stage 3 - variable-length per-(layer, head) caches, Sec. 4.2 "Implementation
 * details", realised as a stable stream compaction: segment g of dst holds the
 * entries of src segment g with keep[e] != 0 in their original order (K row, V
 * row, log_beta, pos and - if both caches carry it - log_tail copied bit for bit;
 * src->log_tail and dst->log_tail must both be NULL or both be set),
 * dst->seg_len[g] = kept[g] and
 * dst->seg_start[g] = sum_{g' < g} (kept[g'] + reserve), i.e. `reserve` free slots
 * follow every segment.  src and dst must not share buffers.  keep: device uint8
 * [src->cap_entries]; kept: device int32 [nseg] as produced by stage 2.
 * Device-side errors: KVTRIM_ECAP if sum(kept + reserve) > dst->cap_entries (then
 * nothing is written), KVTRIM_EMISMATCH if kept[g] differs from the mask's count. */
kvtrim_status kvtrim_compact(kvtrim_ctx *ctx, const kvtrim_cache *src, const uint8_t *keep,
                             const int32_t *kept, kvtrim_cache *dst, int32_t reserve,
                             void *hip_stream);

/* Stage 4 - decode attention under hard eviction, Sec. 2.1 Eq. (reform) with
 * r in {0,1}: for every segment of layers [layer_begin, layer_end) and each of its
 * G = Hq/Hkv query heads hq = head*G + j,
 *   z_i = (q . k_i) * softmax_scale, alpha = softmax(z), o = sum_i alpha_i v_i
 * over the entries of the segment (bf16 inputs, fp32 accumulation).
 * q: device bf16 [n_seq][n_layers][n_q_heads][head_dim].
 * out: device fp32, same shape; lse: optional (may be NULL) device fp32
 * [n_seq][n_layers][n_q_heads] = log sum_i exp(z_i).  An empty segment gives
 * out = 0 and lse = -inf.  Heads of layers outside the range are not written.
 * The same call on the same cache gives the same bits; the order of the fp32 sums depends
 * on how the call's rows are shared out among the kernel's blocks, so two calls with
 * different layer ranges (or caches of different sizes) may differ in the last bits. */
kvtrim_status kvtrim_decode_attn(kvtrim_ctx *ctx, const kvtrim_cache *c, const void *q,
                                 int32_t layer_begin, int32_t layer_end, float softmax_scale,
                                 float *out, float *lse, void *hip_stream);

/* Retention-gated (soft) attention, Sec. 2.2 - the form the gates are trained with:
 *   alpha~_i = beta_i^(t-i) e^(z_i) / sum_j beta_j^(t-j) e^(z_j),  o~ = sum_i alpha~_i v_i,
 * with t = now[seq] (device int32 [n_seq]) the position of the query; beta = 1 gives
 * kvtrim_decode_attn.  Same arguments, layouts and conventions otherwise; lse is the
 * log of the weighted denominator. */
kvtrim_status kvtrim_decode_attn_soft(kvtrim_ctx *ctx, const kvtrim_cache *c, const void *q,
                                      const int32_t *now, int32_t layer_begin, int32_t layer_end,
                                      float softmax_scale, float *out, float *lse, void *hip_stream);

/* Expected cache occupancy, the inner sum of the global capacity loss of Sec. 4.1:
 *   occ_out[seq] = sum over layers, KV heads and cached entries i of beta^(now[seq] - pos_i).
 * occ_out: device fp64 [n_seq].  Terms are evaluated in fp32 and summed in fp64; the last
 * bits of the sum depend on the order in which the blocks finish. */
kvtrim_status kvtrim_occupancy(kvtrim_ctx *ctx, const kvtrim_cache *c, const int32_t *now,
                               double *occ_out, void *hip_stream);

/* Stages 3 + 4 fused: exactly kvtrim_compact(src -> dst) followed by
 * kvtrim_decode_attn(dst), with the same arguments, results and device-side errors,
 * but every surviving K/V row is read from HBM once: it is used for the attention of
 * its segment while it is moved (q.k on the vector ALU, p.v on the matrix cores with the
 * probabilities split into two bf16 terms: the product is exact to 2^-16 of every term, sums
 * are fp32; the cost does not depend on the number of query heads per KV head).  With a
 * destination of less than a quarter of the source's capacity (few rows can survive) the kernel
 * works a block per chunk of the destination, gathering its rows, instead of a block per chunk
 * of the source.  The library runs the two stages one after the other instead - same results -
 * for a source of more than 67 M entries. */
kvtrim_status kvtrim_compact_attn(kvtrim_ctx *ctx, const kvtrim_cache *src, const uint8_t *keep,
                                  const int32_t *kept, kvtrim_cache *dst, int32_t reserve, const void *q,
                                  int32_t layer_begin, int32_t layer_end, float softmax_scale, float *out,
                                  float *lse, void *hip_stream);

/* Stages 3 + 4 fused, compacting INSIDE the cache: every segment keeps its seg_start, its
 * survivors (keep, kept as produced by kvtrim_select_global for this cache) close up to the
 * front of its region in their order, seg_len becomes kept, and out / lse are the attention
 * over the survivors, as kvtrim_compact_attn gives them.  A row moves only if an entry before it in
 * its segment was evicted, and a row that stays is not written: in a decode step, where one
 * entry in thousands goes, most of the cache is read once for the attention and not written.
 * Segment contents afterwards equal those kvtrim_compact produces; the free slots behind a
 * segment (its room for later kvtrim_append calls) grow and shrink with its length, so a caller
 * runs an out-of-place step (kvtrim_compact_attn with a `reserve`) now and then to even them
 * out - kvtrim_append reports KVTRIM_ECAP when a segment has run out.
 * spare: a second cache structure whose k, v, log_beta, pos (and log_tail if c has one)
 * arrays hold at least c->cap_entries entries and are distinct from c's; the call parks a few
 * rows there while it runs (those that move into a region another thread block may still be
 * reading); its contents afterwards are unspecified, its segment tables are not touched.
 * Served for caches of at most 67 M entries (KVTRIM_EINVAL otherwise).  Device-side errors:
 * KVTRIM_EMISMATCH, KVTRIM_ELAYOUT. */
kvtrim_status kvtrim_compact_attn_inplace(kvtrim_ctx *ctx, kvtrim_cache *c, const uint8_t *keep,
                                          const int32_t *kept, kvtrim_cache *spare, const void *q,
                                          int32_t layer_begin, int32_t layer_end, float softmax_scale,
                                          float *out, float *lse, void *hip_stream);

/* Stage 3 alone, compacting inside the cache: kvtrim_compact_attn_inplace without the attention
 * (same arguments, same rules for `spare`, any cache size the context allows).  Only the rows
 * behind an eviction are touched, so a decode step's compaction costs a fraction of an
 * out-of-place one; kvtrim_decode_attn can then be called layer by layer on the same cache. */
kvtrim_status kvtrim_compact_inplace(kvtrim_ctx *ctx, kvtrim_cache *c, const uint8_t *keep, const int32_t *kept,
                                     kvtrim_cache *spare, void *hip_stream);

/* For callers of the in-place calls: min_room_out[0] (device int32) = the smallest number of free
 * slots behind any segment (up to the next segment's start, or cap_entries for the last one) - how
 * many more tokens per segment kvtrim_append can take for certain before an out-of-place step has
 * to even the room out.  One small kernel; read the result back whenever convenient. */
kvtrim_status kvtrim_min_room(kvtrim_ctx *ctx, const kvtrim_cache *c, int32_t *min_room_out, void *hip_stream);

/* Support - new tokens enter the cache (Sec. 3.2: beta is fixed when the token is
 * first cached).  Appends up to n_new entries to every segment, in order, behind its
 * current end and adds their number to seg_len.  k_new, v_new: device bf16
 * [nseg][n_new][head_dim]; log_beta_new: device fp32 [nseg][n_new]; log_tail_new:
 * device fp32 [nseg][n_new], required iff c->log_tail != NULL (NULL otherwise); pos_new:
 * device int32 [nseg][n_new] (ascending, above the segment's last position).  A
 * segment takes its rows up to the first one with a NEGATIVE position: the sequences
 * of a batch may bring different numbers of tokens (a ragged last chunk of a prefill),
 * the rest of their rows is padding.
 * Device-side error KVTRIM_ECAP if some segment lacks free slots for its rows before
 * the next segment (or the end of the buffer); that segment is then left unchanged. */
kvtrim_status kvtrim_append(kvtrim_ctx *ctx, kvtrim_cache *c, const void *k_new, const void *v_new,
                            const float *log_beta_new, const float *log_tail_new, const int32_t *pos_new,
                            int32_t n_new, void *hip_stream);

/* A decode step on the ragged layout in one call (Sec. 4.2: the new token is cached, every entry rescored, the
 * cache evicted down to the budget and attended).  Leaves in src, score_out, keep_out, kept_out, thr_key_out, dst, out
 * and lse exactly what
 *     kvtrim_append(src, new tokens) -> kvtrim_score_select(src, now, budget, evict_hint)
 *     -> kvtrim_compact_attn(src -> dst, reserve, q)
 * leave there (bit for bit in everything but out / lse, which agree within the attention tolerance: the split of
 * the softmax sums is the same, so in practice they are equal too).  Arguments as in those three calls; keep_out is
 * required.  With a small evict_hint (see kvtrim_score_select), at most 1024 segments per sequence, 1024 sequences
 * and 16 new tokens per segment the step is THREE kernels:
 * one scores, lists the eviction candidates and - in each sequence's last block - ranks them, counts the evicted
 * entries per segment and per chunk of 128 entries and leaves the destination's segment table and, per segment, the
 * indices of its evicted entries (further blocks of the same launch append the new tokens); one moves every
 * surviving row while using it for the attention of its segment (no mask pass, no compaction scan: a block derives
 * its chunk's destination from its segment's record and writes the chunk's mask bytes itself); one merges the
 * partial attention results.  Any other shape or hint runs the three calls one after the other.  Device-side errors as in
 * the three calls. */
kvtrim_status kvtrim_decode_step(kvtrim_ctx *ctx, kvtrim_cache *src, const void *k_new, const void *v_new,
                                 const float *log_beta_new, const float *log_tail_new, const int32_t *pos_new,
                                 int32_t n_new, const int32_t *now, const int64_t *budget, float *score_out,
                                 uint8_t *keep_out, int32_t *kept_out, uint32_t *thr_key_out, kvtrim_cache *dst,
                                 int32_t reserve, const void *q, int32_t layer_begin, int32_t layer_end,
                                 float softmax_scale, float *out, float *lse, int64_t evict_hint, void *hip_stream);

/* The same decode step with stages 3 + 4 done INSIDE the cache (Sec. 4.2).  Leaves in c, score_out, keep_out,
 * kept_out, thr_key_out, out and lse exactly what
 *     kvtrim_append(c, new tokens) -> kvtrim_score_select(c, now, budget, evict_hint)
 *     -> kvtrim_compact_attn_inplace(c, spare, q)
 * leave there; arguments and the rules for `spare` as in those calls (every segment needs free slots for its new
 * tokens behind it: kvtrim_min_room).  Under the conditions of kvtrim_decode_step it is FOUR kernels: the scoring
 * kernel leaves every segment's start where it is, the row mover touches only the rows behind an eviction, a small
 * kernel puts the rows it had to park in `spare` in place, and one merges the partial attention results. */
kvtrim_status kvtrim_decode_step_inplace(kvtrim_ctx *ctx, kvtrim_cache *c, const void *k_new, const void *v_new,
                                         const float *log_beta_new, const float *log_tail_new, const int32_t *pos_new,
                                         int32_t n_new, const int32_t *now, const int64_t *budget, float *score_out,
                                         uint8_t *keep_out, int32_t *kept_out, uint32_t *thr_key_out, kvtrim_cache *spare,
                                         const void *q, int32_t layer_begin, int32_t layer_end, float softmax_scale,
                                         float *out, float *lse, int64_t evict_hint, void *hip_stream);

/* A chunk of a prefill on the ragged layout in one call (the multi-turn flow of Sec. 4.2 / Sec. 5:
 * after every appended chunk of tokens the cache is rescored, selected and compacted).  Leaves in
 * score_out, keep_out, kept_out, thr_key_out and dst exactly what
 *     kvtrim_append(src, new tokens) -> kvtrim_score(src, now) -> kvtrim_select_global(src, budget)
 *     -> kvtrim_compact(src -> dst, reserve)
 * leave there, but the K/V rows of the new tokens go from k_new / v_new straight to their places
 * in dst: only their metadata is appended to src (the score and the selection read nothing else),
 * so the chunk's K/V is written once instead of twice and read once instead of twice.
 * Arguments as in those four calls.  src needs the free slots kvtrim_append needs; afterwards
 * its metadata and seg_len include the new tokens and the K/V rows of those slots are
 * unspecified: src is spent, the live cache is dst.  Device-side errors as in the four calls. */
kvtrim_status kvtrim_append_compact(kvtrim_ctx *ctx, kvtrim_cache *src, const void *k_new, const void *v_new,
                                    const float *log_beta_new, const float *log_tail_new,
                                    const int32_t *pos_new, int32_t n_new, const int32_t *now,
                                    const int64_t *budget, float *score_out, uint8_t *keep_out,
                                    int32_t *kept_out, uint32_t *thr_key_out, kvtrim_cache *dst,
                                    int32_t reserve, void *hip_stream);

/* ------------------------------------------------------------------------------------
 * Paged variant: the layout of Sec. 4.2 "Implementation details" itself.  KV entries live
 * in fixed-size pages of KVTRIM_PAGE_SIZE slots; every (sequence, layer, KV head) segment
 * owns a list of pages (its block table) and so has its own variable length; evicting an
 * entry frees its slot and moves no K/V.  The order of the entries inside a segment is
 * arbitrary (attention does not depend on it); the selection still breaks ties by
 * (layer, head, position), using the stored positions.
 *
 *   k, v         bf16 [n_pages][KVTRIM_PAGE_SIZE][head_dim]
 *   log_beta     fp32 [n_pages][KVTRIM_PAGE_SIZE]
 *   pos          int32 [n_pages][KVTRIM_PAGE_SIZE]; a negative value marks an empty slot
 *   log_tail     fp32 [n_pages][KVTRIM_PAGE_SIZE] or NULL (lookahead horizon, as above)
 *   block_table  int32 [nseg][max_pages_per_seg]  pages of each segment (first seg_pages[g] valid)
 *   seg_pages    int32 [nseg]      pages in the segment's table
 *   seg_live     int32 [nseg]      live entries of the segment
 *   page_owner   int32 [n_pages]   owning segment, negative = free
 *   page_live    int32 [n_pages]   live entries in the page
 *   free_list    int32 [n_pages]   stack of free page ids; n_free int32 [1] its height
 * All of it is caller-owned device memory (k, v, log_beta, pos, log_tail and the score arrays
 * 16-byte aligned, the keep mask 4-byte aligned); kvtrim_paged_build initialises the bookkeeping.
 * Slot s of page p is entry p*KVTRIM_PAGE_SIZE + s of the flat score / keep arrays.
 * n_pages * KVTRIM_PAGE_SIZE must not exceed the context's max_entries, and the calls that run
 * attention need n_pages / 4 + nseg to fit the context's partial-result buffer (always true
 * when n_pages <= 2097152). */
#define KVTRIM_PAGE_SIZE 128
typedef struct {
    void *k;
    void *v;
    float *log_beta;
    int32_t *pos;
    float *log_tail;
    int32_t *block_table;
    int32_t *seg_pages;
    int32_t *seg_live;
    int32_t *page_owner;
    int32_t *page_live;
    int32_t *free_list;
    int32_t *n_free;
    int32_t n_pages;
    int32_t max_pages_per_seg;
} kvtrim_paged_cache;

/* First compression (Fig. "Prefill/compression"): the entries of the ragged cache `src` with
 * keep[e] != 0 (keep, kept as produced by kvtrim_select_global) are gathered, in order, into
 * consecutive pages per segment; the remaining pages go to the free list.  Device-side errors:
 * KVTRIM_ECAP (not enough pages, or a segment needs more than max_pages_per_seg),
 * KVTRIM_EMISMATCH as in kvtrim_compact. */
kvtrim_status kvtrim_paged_build(kvtrim_ctx *ctx, const kvtrim_cache *src, const uint8_t *keep,
                                 const int32_t *kept, kvtrim_paged_cache *dst, void *hip_stream);

/* New tokens enter the pages: up to n_new (1 .. 4096) per segment, laid out as for kvtrim_append
 * (k_new, v_new: bf16 [nseg][n_new][head_dim]; log_beta_new, pos_new: [nseg][n_new]; log_tail_new
 * iff the cache carries log_tail; a segment takes its rows up to the first negative position, the
 * rest is padding).  Tokens take the empty slots of the segment's pages first, then pages from the
 * free list.  KVTRIM_ECAP when the free list or the block table cannot hold a segment's tokens
 * (that segment is then left unchanged). */
kvtrim_status kvtrim_paged_append(kvtrim_ctx *ctx, kvtrim_paged_cache *c, const void *k_new, const void *v_new,
                                  const float *log_beta_new, const float *log_tail_new, const int32_t *pos_new,
                                  int32_t n_new, void *hip_stream);

/* Stage 1 on the paged layout: score_out fp32 [n_pages * KVTRIM_PAGE_SIZE]; the slots of every
 * segment's pages are written (0 for empty slots), free pages are left alone. */
kvtrim_status kvtrim_paged_score(kvtrim_ctx *ctx, const kvtrim_paged_cache *c, const int32_t *now,
                                 float *score_out, void *hip_stream);

/* Stage 2 on the paged layout: same rule and outputs as kvtrim_select_global; keep_out uint8
 * [n_pages * KVTRIM_PAGE_SIZE] is written for the slots of every segment's pages (0 for empty ones). */
kvtrim_status kvtrim_paged_select(kvtrim_ctx *ctx, const kvtrim_paged_cache *c, const float *score,
                                  const int64_t *budget, uint8_t *keep_out, int32_t *kept_out,
                                  uint32_t *thr_key_out, void *hip_stream);

/* Stages 1 + 2 on the paged layout in one call: leaves in score_out, keep_out, kept_out and thr_key_out exactly
 * what kvtrim_paged_score followed by kvtrim_paged_select leave there.  evict_hint as in kvtrim_score_select:
 * 0 runs those two calls' kernels; a small positive value - about the number of entries a sequence loses in this
 * step - takes the decode-step form (Sec. 4.2: a decode step evicts about as many entries as it appended): two
 * kernels that walk every segment's slots through its block table, the first scoring them and ranking the few
 * candidates below a bound carried from the previous call, the second writing the mask.  The result does not
 * depend on the hint; a hint that does not fit costs one slow single-block selection. */
kvtrim_status kvtrim_paged_score_select(kvtrim_ctx *ctx, const kvtrim_paged_cache *c, const int32_t *now,
                                        const int64_t *budget, float *score_out, uint8_t *keep_out, int32_t *kept_out,
                                        uint32_t *thr_key_out, int64_t evict_hint, void *hip_stream);

/* A decode step on the paged layout in one call: leaves in the pages, score_out, keep_out, kept_out, thr_key_out, out
 * and lse what
 *     kvtrim_paged_append(one token per segment) -> kvtrim_paged_score_select(now, budget, evict_hint)
 *     -> kvtrim_paged_evict(keep_out) -> kvtrim_paged_attn(q)
 * leave there (arguments as in those four calls; one row per segment in the new-token arrays) - bit for bit in
 * everything but out / lse, which agree within the attention tolerance: a page that this step's eviction emptied is
 * still listed when the attention's chunk table is built, so the fp32 sums may group differently.  With a small
 * evict_hint the mask kernel of the decode-step selection applies the eviction as it writes the mask (which saves
 * the pass of kvtrim_paged_evict over all pages), its scoring kernel also builds the attention's chunk table, and
 * the attention's merge kernel takes the emptied pages out of the block tables: five kernels per step.  Any other
 * hint runs the four calls. */
kvtrim_status kvtrim_paged_decode_step(kvtrim_ctx *ctx, kvtrim_paged_cache *c, const void *k_new, const void *v_new,
                                       const float *log_beta_new, const float *log_tail_new, const int32_t *pos_new,
                                       const int32_t *now, const int64_t *budget, float *score_out, uint8_t *keep_out,
                                       int32_t *kept_out, uint32_t *thr_key_out, const void *q, int32_t layer_begin,
                                       int32_t layer_end, float softmax_scale, float *out, float *lse, int64_t evict_hint,
                                       void *hip_stream);

/* Stage 3 on the paged layout: live slots with keep[e] == 0 become empty; pages left without a
 * live entry return to the free list and leave their segment's block table.  No K/V moves. */
kvtrim_status kvtrim_paged_evict(kvtrim_ctx *ctx, kvtrim_paged_cache *c, const uint8_t *keep, void *hip_stream);

/* Housekeeping of the paged layout (Sec. 4.2 "Implementation details" describes the layout; the paper does not
 * discuss fragmentation): eviction frees a page only when all of its slots are empty, so over many steps a
 * segment spreads over more pages than its live entries need.  For every segment whose live entries fit into
 * fewer pages, the last pages of its block table are emptied into the free slots of the pages before them
 * (K row, V row, log beta, position and tail constant move together) and return to the free list; afterwards
 * the segment holds ceil(live / KVTRIM_PAGE_SIZE) pages.  The set of entries of every segment is unchanged (a
 * segment's entries have no order inside its pages), so scores, selections and attention outputs are the same
 * as without the call, up to the order of floating-point sums in attention.  Call it when the pool runs low
 * or every few hundred steps; a segment that is already tight costs one look at its page counts. */
kvtrim_status kvtrim_paged_defrag(kvtrim_ctx *ctx, kvtrim_paged_cache *c, void *hip_stream);

/* Stage 4 on the paged layout: as kvtrim_decode_attn, over the live slots of each segment's pages. */
kvtrim_status kvtrim_paged_attn(kvtrim_ctx *ctx, const kvtrim_paged_cache *c, const void *q, int32_t layer_begin,
                                int32_t layer_end, float softmax_scale, float *out, float *lse, void *hip_stream);

/* ---- Retention gate for tokens that enter the cache (Sec. 4.1 "Weight-tied retention gates";
 * Sec. 5.1: a small MLP per transformer block with hidden width d_g = 512, Proj a two-layer MLP,
 * the final linear layer tied across all layers and heads; Sec. 3.2: beta is computed once, when
 * the token is cached).  For layer l, KV head h and token representation x (the input of block l):
 *     u = silu(W1_l x + c1_l)            first layer, one per block, width d_g
 *     p = W2_{l,h} u + c2_{l,h}          second layer of Proj, one per (block, head), width d_p
 *     z = w_g . p + b_g                  tied readout;  beta = sigmoid(z)
 * (the activation, d_p and the sharing of the first layer by the heads of a block are this
 * build's reading; the paper does not print them).
 *
 *   w1   bf16 [n_layers][d_g][d_model]            c1  fp32 [n_layers][d_g]
 *   w2   bf16 [n_layers][n_kv_heads][d_p][d_g]    c2  fp32 [n_layers][n_kv_heads][d_p]
 *   w_g  fp32 [d_p], b_g                          (n_layers, n_kv_heads: the context's)
 * All device pointers, caller-owned, w1 and w2 16-byte aligned; d_model a multiple of 256, d_g a
 * multiple of 64, d_p >= 1. */
typedef struct {
    int32_t d_model, d_g, d_p;
    const void *w1;
    const float *c1;
    const void *w2;
    const float *c2;
    const float *w_g;
    float b_g;
} kvtrim_gate;

/* Bytes of scratch kvtrim_gate_forward needs for n_tok tokens and n_layers layers of a range:
 * n_tok * n_layers * d_g floats (short calls keep the hidden activations u there in fp32; calls of 128 tokens
 * and more keep the folded readout vectors there and, where it fits - from about d_model / 2 tokens on - a
 * copy of W1 in matrix-core operand order); 0 for invalid arguments.  Host-only, no GPU call. */
size_t kvtrim_gate_scratch_bytes(const kvtrim_gate *g, int32_t n_tok, int32_t n_layers);

/* x: bf16 [layer_end - layer_begin][n_tok][d_model], 16-byte aligned, the representation of each
 * token at the input of each block of the range.  Writes, for those layers,
 *   log_beta_out[(tok * n_layers + layer) * n_kv_heads + head] = log sigmoid(z)      (fp32)
 *   log_tail_out[same index] = log(sum_{k<horizon} beta^k), horizon 0 = the limit -log(1 - beta)
 *                              (Eq. global_score; NULL to skip; horizon in [0, 4096])
 * - with one token per sequence this is segment order, the layout kvtrim_append takes.
 * scratch: device memory, 16-byte aligned, at least kvtrim_gate_scratch_bytes(...) bytes, contents
 * undefined afterwards.  Enqueues two or three kernels on the stream; allocates nothing.  Arithmetic:
 * bf16 products accumulated in fp32 on the matrix cores.  Calls below 128 tokens carry u to 16 mantissa
 * bits into the second layer; longer calls use that the second layer and the readout are both linear
 * (z = (W2^T w_g) . u + w_g . c2 + b_g), fold them into one fp32 vector per (layer, head) first and keep u
 * in fp32.  Results agree with an fp64 evaluation to about 1e-5 relative in log beta either way. */
kvtrim_status kvtrim_gate_forward(kvtrim_ctx *ctx, const kvtrim_gate *g, const void *x, int32_t n_tok,
                                  int32_t layer_begin, int32_t layer_end, int32_t horizon, void *scratch,
                                  float *log_beta_out, float *log_tail_out, void *hip_stream);

/* Weights that stay the same from call to call (inference): what kvtrim_gate_forward derives from them inside
 * every call - the folded readout vectors v = W2^T w_g and constants s = w_g . c2 + b_g of every (layer, head),
 * and a copy of W1 in matrix-core operand order - can be computed once and handed to
 * kvtrim_gate_forward_prepared.  kvtrim_gate_prepared_bytes: size of that buffer for a context with n_layers
 * layers and n_kv_heads heads (host-only; 0 for invalid arguments).  kvtrim_gate_prepare: fills `prepared`
 * (device memory, 16-byte aligned, that many bytes, caller-owned) for ALL layers of the context; two kernels on
 * the stream.  The buffer is valid for as long as the weights it was made from are unchanged.
 * kvtrim_gate_forward_prepared: same arguments, outputs and arithmetic contract as kvtrim_gate_forward (g must
 * be the gate the buffer was prepared from; scratch as for kvtrim_gate_forward); calls of every length then read
 * the readout as one dot product per (token, layer, head), and the one-kernel path that kvtrim_gate_forward
 * takes from 128 tokens on is taken from 24 tokens on, reading W1 from the operand-order copy.  Calls of up to 16
 * tokens (with at most 16 KV heads) are one kernel as well; it keeps one arrival counter per layer in the context's
 * workspace, so - as for every call on a context - two gate calls on one context must not run at the same time. */
size_t kvtrim_gate_prepared_bytes(const kvtrim_gate *g, int32_t n_layers, int32_t n_kv_heads);
kvtrim_status kvtrim_gate_prepare(kvtrim_ctx *ctx, const kvtrim_gate *g, void *prepared, void *hip_stream);
kvtrim_status kvtrim_gate_forward_prepared(kvtrim_ctx *ctx, const kvtrim_gate *g, const void *prepared, const void *x,
                                           int32_t n_tok, int32_t layer_begin, int32_t layer_end, int32_t horizon,
                                           void *scratch, float *log_beta_out, float *log_tail_out, void *hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): kvtrim_select_global without a context.  Same selection rule, same kernels, same
 * outputs (keep_out, kept_out, thr_key_out) as kvtrim_select_global; the tables that call keeps in its context's
 * workspace live in one fixed array of KVTRIM_NOALLOC_SCRATCH_BYTES bytes inside the library instead (each GPU
 * the library runs on holds its own copy until the process ends).  The call makes no hipMalloc / hipFree and calls
 * no allocating routine; it only enqueues kernels on `hip_stream`.
 *   cfg         host pointer: the shape (n_seq, n_layers, n_kv_heads, ...) and max_entries >= c->cap_entries.
 *               The tables grow with n_seq (about 200 KB each) and with max_entries (28 bytes per 2048 entries)
 *               plus 12 bytes per segment; a configuration whose tables exceed the array - e.g. more than about
 *               40 sequences - is rejected with KVTRIM_EINVAL before anything is launched.
 *   c, score, budget, keep_out, kept_out, thr_key_out: as in kvtrim_select_global (caller-owned device memory).
 *   status_out  optional device int32 [1]: written by the call's last kernel with KVTRIM_OK, or KVTRIM_ELAYOUT
 *               when the segment table does not fit cap_entries (then keep_out / kept_out are unspecified).
 * All calls on one GPU share that GPU's array: they must be ordered (one stream, or events between streams);
 * calls that overlap on one GPU race.  Nothing carries over from one call to the next. */
#define KVTRIM_NOALLOC_SCRATCH_BYTES 8388608
kvtrim_status kvtrim_select_global_noalloc(const kvtrim_config *cfg, const kvtrim_cache *c, const float *score,
                                           const int64_t *budget, uint8_t *keep_out, int32_t *kept_out,
                                           uint32_t *thr_key_out, int32_t *status_out, void *hip_stream);

/* Instrumentation (for the benchmark; not a step of the method).  Between
 * kvtrim_profile_begin and kvtrim_profile_end every launch of a kernel whose bit is
 * set in `kernel_mask` (bit i = kernel id i, names from kvtrim_kernel_name) is
 * bracketed by a pair of HIP events recorded on the stream the kernel is launched
 * on.  begin allocates the event pool (host side, synchronous; at most
 * KVTRIM_PROFILE_MAX_LAUNCHES launches are bracketed, later ones run unbracketed);
 * end waits for `hip_stream` and writes, per kernel id, the summed duration in
 * milliseconds and the number of bracketed launches into host arrays of
 * KVTRIM_N_KERNELS elements.  Do not capture a HIP graph while profiling is on. */
#define KVTRIM_N_KERNELS 40
#define KVTRIM_PROFILE_MAX_LAUNCHES 4096
kvtrim_status kvtrim_profile_begin(kvtrim_ctx *ctx, uint64_t kernel_mask);
kvtrim_status kvtrim_profile_end(kvtrim_ctx *ctx, void *hip_stream, double *ms_sum_host,
                                 int64_t *launches_host);
const char *kvtrim_kernel_name(int32_t kernel_id); /* NULL when out of range */

#ifdef __cplusplus
}
#endif
#endif /* KVTRIM_H */
