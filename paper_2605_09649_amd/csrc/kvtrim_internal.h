// Internal declarations shared by the translation units of libkvtrim (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvtrim.h"

namespace kvtrim {

// Chunk sizes (entries of one segment handled as a unit).
constexpr int SEL_CHUNK = 2048;      // selection: entries per chunk
constexpr int SEL_SHIFT = 11;        // log2(SEL_CHUNK)
static_assert((1 << SEL_SHIFT) == SEL_CHUNK, "SEL_SHIFT out of step with SEL_CHUNK");
constexpr int CMP_CHUNK = 128;       // compaction: entries per block
constexpr long long CMP_DST_FULL = 1ll << 62;   // flag in ws.cmp_chunk_dst: every entry of the chunk survives
constexpr int CMP_WAVE_ROWS = 16;    // rows a wavefront moves (one batch of loads, one of stores)
constexpr int CMP_THREADS = CMP_CHUNK / CMP_WAVE_ROWS * 64;   // 512: one wavefront per 16 survivors
constexpr int RADIX_BITS0 = 11, RADIX_BITS1 = 11, RADIX_BITS2 = 10;
constexpr int RADIX_BINS = 2048;     // bins of the widest pass
constexpr int HIST_BLOCKS_MAX = 512; // blocks of a histogram pass (few and fat: see k_select.hip)
constexpr int DONE_WORDS = 128;      // 4 sets of 32 counters (three histogram passes, the tie count)
constexpr int HIST_REPLICAS = 8;     // copies of the merged histogram (spreads the device-scope atomics)

// Decode-step selection (k_fastsel.hip): candidates below the carried bound are listed per sequence.
constexpr int FL_CAP_MAX = 4096;     // list entries per sequence (fewer when the context has many sequences)
constexpr int FL_CAP_MIN = 64;
constexpr int FAST_THREADS = 1024;
constexpr int FAST_ENTRIES_PER_BLOCK = 8192;   // entries of a segment one block covers (blocks per segment from the capacity)

constexpr int ERR_CAP = 1;           // bits of the sticky device flag
constexpr int ERR_MISMATCH = 2;
constexpr int ERR_LAYOUT = 4;

struct Shape {
    int32_t n_seq, n_layers, n_kv_heads, n_q_heads, head_dim;
    int32_t nseg, segs_per_seq, group;
};

struct CacheView {                   // device pointers, passed by value to kernels
    const uint16_t* k;
    const uint16_t* v;
    const float* log_beta;
    const int32_t* pos;
    const int64_t* seg_start;
    const int32_t* seg_len;
    int64_t cap;
    const float* log_tail;           // NULL = lookahead horizon 1
};

struct CacheViewMut {
    uint16_t* k;
    uint16_t* v;
    float* log_beta;
    int32_t* pos;
    int64_t* seg_start;
    int32_t* seg_len;
    int64_t cap;
    float* log_tail;
};

// Per-sequence state of the radix select, kept in the workspace.
struct SelState {
    uint32_t prefix;     // digits fixed so far (right aligned)
    uint32_t thr_key;    // final threshold key
    int64_t count;       // candidates of the sequence
    int64_t want;        // min(budget, count)
    int64_t rank;        // entries still to take inside the current bucket
    int64_t tie_quota;   // entries equal to thr_key to keep (in storage order)
    int32_t keep_none;   // want == 0
    int32_t need_rank;   // only some of the entries equal to thr_key fit: they must be ranked in order
};

// Outcome of a selection in the form the decode-step mask kernel reads: entry e of segment g survives iff
// key(e) > key_thr, or key(e) == key_thr and (g, pos(e)) <= (seg_thr, pos_thr) lexicographically - i.e. iff it is
// not behind the last retained entry in the total order (key descending, segment ascending, position ascending).
constexpr int FSEL_NONE = 0, FSEL_ALL = 1, FSEL_THRESHOLD = 2;
struct FastSel {
    int32_t mode;
    uint32_t key_thr;
    int32_t seg_thr;
    int32_t pos_thr;
};

// A paged cache as the decode-step selection walks it: the block tables ([nseg][max_pps] pages of the pool), pages and
// live entries per segment.
struct PagedArgs {
    const int32_t* block_table;
    const int32_t* seg_pages;
    const int32_t* seg_live;
    int32_t n_pages;
    int32_t max_pps;
    // for the mask kernel that also evicts (the paged decode step in one call): what an eviction updates
    int32_t* evict_pos;
    int32_t* evict_seg_live;
    int32_t* evict_page_live;
    int32_t* evict_page_owner;
    // layers [plan_layer_begin, plan_layer_end) whose attention chunk table the scoring kernel also builds (none: no table)
    int32_t plan_layer_begin, plan_layer_end;
};

// The decode step in one call (kvtrim_decode_step): the tokens that enter the cache in this step (laid out as kvtrim_append takes them;
// their rows also go into the source cache) and where the compaction goes.  (pg: the paged form of the decode-step
// selection, which takes neither new tokens nor a destination, hands its tables to the same kernel here.)
struct StepArgs {
    const uint16_t* k_new;
    const uint16_t* v_new;
    const float* lb_new;
    const float* lt_new;
    const int32_t* pos_new;
    int n_new;
    CacheViewMut src;            // the source cache again, writable
    CacheViewMut dst;
    int reserve;
    uint8_t* keep_out;
    PagedArgs pg;
    bool inplace;                // the compaction happens inside src (every segment keeps its start; dst is not used)
};

// One-call decode step: per segment, where its survivors start in the destination and which of its entries go -
// the first STEP_REC_IDX of them here, all of them in ws.step_evl from `off` on (index in the sequence's part).
constexpr int STEP_REC_IDX = 12;
struct alignas(64) StepSegRec {
    int64_t dst_start;
    int32_t cnt;
    int32_t off;
    int32_t idx[STEP_REC_IDX];
};
constexpr uint32_t STEP_CHUNK_DENSE = 0xFFFFFFFFu;
constexpr int STEP_MAX_SEGS = 1024;  // segments per sequence the one-call decode step handles
constexpr int STEP_MAX_EVICT = 1024; // evictions per sequence it lists (more: the keep mask and per-chunk offsets are written by one block)
constexpr int STEP_MAX_SEQS = 1024;  // sequences it handles
constexpr int STEP_MAX_NEW = 16;     // new tokens per segment and step

// One chunk of a segment: entries [first, first + n) of the flat arrays.
struct ChunkDesc {
    int64_t first;
    int32_t n;
    int32_t seg;
};

// The chunk table a selection pass walks: the context's own table of a ragged cache, or one
// chunk per page of a paged cache (then `pos` marks the live slots).
struct SelTables {
    const ChunkDesc* desc;
    const int32_t* prefix;       // [nseg+1] first chunk of each segment
    const int32_t* pos;          // paged only
};

struct Workspace {
    // selection
    int32_t* sel_chunk_prefix;   // [nseg+1] first chunk of each segment
    ChunkDesc* sel_desc;         // [max_sel_chunks]
    int64_t* sel_entry_prefix;   // [nseg+1] entries before each segment
    int4* sel_blk;               // [HIST_BLOCKS_MAX] per histogram block: first chunk, end chunk, first and last sequence
    // paged selection: ties at the threshold, per segment
    int32_t* tie_cnt;            // [nseg]
    int32_t* tie_mode;           // [nseg] 0: no tie survives, 1: all, 2: those with pos <= tie_thr
    int32_t* tie_thr;            // [nseg]
    int64_t* pg_seg_start;       // [nseg] segment table of the page-aligned compaction that builds a paged cache
    int32_t* pg_seg_len;         // [nseg]
    uint32_t* hist;              // [3][HIST_REPLICAS][n_seq][RADIX_BINS]
    SelState* sel;               // [4][n_seq]: final state; state after the plan, after pass 0, after pass 1
    int32_t* chunk_old_len;      // [nseg] kvtrim_append_compact: segment lengths before the chunk was appended
    uint32_t* seq_done;          // [n_seq] blocks of the last histogram pass that have added their counts for the sequence
    uint32_t* done;              // [DONE_WORDS] "last block" counters: per pass one top-level and 16 group counters
    int32_t* chunk_eq;           // [max_sel_chunks] entries equal to the threshold
    int64_t* chunk_tie_base;     // [max_sel_chunks] ties of the sequence before the chunk
    // compaction
    int32_t* cmp_chunk_prefix;   // [nseg+1]
    ChunkDesc* cmp_desc;         // [max_cmp_chunks]
    int64_t* cmp_chunk_dst;      // [max_cmp_chunks] first dst entry of the chunk's survivors (| CMP_DST_FULL)
    int32_t* att_pages;          // [max_att_chunks][4] paged attention: the pages of a chunk, beside its descriptor
    // attention
    int32_t* att_chunk_prefix;   // [nseg+1]
    ChunkDesc* att_desc;         // [max_att_chunks]
    float* att_partial;          // [max_att_chunks][G][D+2]  (m, l, o[D]) per query head
    const int32_t* pg_block_table; // paged attention only: the caller's block tables (set per launch)
    int32_t* err;                // sticky device flag
    // decode-step selection: state carried from call to call, and the per-call candidate lists
    uint32_t* fast_hi;           // [n_seq] entries with key < fast_hi are listed (0: nothing known yet)
    uint32_t* fast_min;          // [n_seq][16] smallest key seen in the call, per group of blocks (0xFFFFFFFF between calls)
    uint32_t* fast_done;         // [n_seq][17] arrivals: top level, 16 groups of blocks (0 between calls)
    uint32_t* fl_count;          // [n_seq][16] candidates per sub-list (beyond its capacity: the list is incomplete; 0 between calls)
    unsigned long long* fast_stat; // [2] sequences resolved from their list / by the single-block select, since the context was created
    FastSel* fast_sel;           // [n_seq] outcome of the call
    uint32_t* fl_key;            // [n_seq][fl_cap] in up to 16 sub-lists of fl_cap / n_sub entries
    int32_t* fl_seg;             // [n_seq][fl_cap]
    int32_t* fl_pos;             // [n_seq][fl_cap]
    int32_t* fl_idx;             // [n_seq][fl_cap] index of the entry in its segment (one-call decode step)
    int32_t fl_cap;
    // one-call decode step
    int32_t* step_len;           // [nseg] segment lengths with the step's new tokens
    StepSegRec* step_rec;        // [nseg] what the row mover needs of a segment to place a chunk's survivors
    int32_t* step_evl;           // [n_seq][STEP_MAX_EVICT] the evicted entries (index in their segment), segment by segment
    uint32_t* step_chunk_ev;     // [max_cmp_chunks] entries a chunk loses in this step (STEP_CHUNK_DENSE: look at the
                                 // keep mask and ws.cmp_chunk_dst instead)
    // gathering fused kernel (sparse selections): the source row of every destination row, CMP_CHUNK slots per
    // destination chunk, written by the compaction scan
    int32_t* gat_src;            // [gat_slots]
    int64_t* att_row_prefix;     // [nseg+1] attention: rows (paged: slots) of the layer range's segments before each segment
    uint32_t* gate_done;         // [n_layers] gate forward: blocks of a layer that have left their part of the readout (zero between calls)
    int64_t gat_slots;
    int64_t max_sel_chunks, max_cmp_chunks, max_att_chunks;
};

}  // namespace kvtrim

namespace kvtrim {
enum KernelId {
    K_SCORE = 0, K_SEL_PLAN, K_SEL_HIST0, K_SEL_HIST1, K_SEL_HIST2, K_SEL_COUNT, K_SEL_MASK,
    K_CMP_SCAN, K_CMP_COPY, K_ATT_PLAN, K_ATT_PARTIAL, K_ATT_COMBINE, K_APPEND, K_CMP_ATTN, K_OCCUPANCY,
    K_PG_INIT, K_PG_APPEND, K_PG_SCORE, K_PG_PLAN, K_PG_COUNT, K_PG_EVICT, K_PG_TIDY, K_PG_ATT_PLAN, K_GATE_HIDDEN, K_GATE_READOUT, K_GATE_FOLD, K_GATE_PREFILL, K_GATE_RETILE, K_PG_DEFRAG, K_GATE_DOT, K_RESERVED_30, K_CMP_UNSTAGE,
    K_FAST_SCAN, K_FAST_MASK, K_RESERVED_34, K_RESERVED_35, K_RESERVED_36, K_RESERVED_37, K_RESERVED_38, K_RESERVED_39, K_COUNT
};
static_assert(K_COUNT == KVTRIM_N_KERNELS, "kernel table out of step with the header");
}  // namespace kvtrim

struct kvtrim_ctx {
    kvtrim_config cfg;
    kvtrim::Shape shape;
    kvtrim::Workspace ws;
    void* ws_base;
    size_t ws_bytes;
    int32_t* err_host;           // pinned mirror of the device flag
    int device;
    int att_chunk_min;           // rows per attention chunk (multiple of 64, >= 256); KVTRIM_ATT_CHUNK overrides
    int att_blocks;              // blocks of the attention kernel's fixed grid; KVTRIM_ATT_BLOCKS overrides
    char last_error[256];
    // instrumentation
    uint64_t prof_mask;
    hipEvent_t* prof_ev;         // [2 * KVTRIM_PROFILE_MAX_LAUNCHES] start/stop pairs
    int8_t* prof_kernel;         // kernel id of each bracketed launch
    int prof_used;
};

namespace kvtrim {

// Upper bound on attention chunks for a cache of `cap` entries, and the chunk size used.
int att_chunk_for(const kvtrim_ctx* ctx, int64_t cap);

kvtrim_status launch_score(kvtrim_ctx*, const CacheView&, const int32_t* now, float* score, hipStream_t);
kvtrim_status launch_select(kvtrim_ctx*, const CacheView&, const float* score, const int64_t* budget,
                            uint8_t* keep, int32_t* kept, uint32_t* thr, hipStream_t);
// Stages 1 + 2 in one call.  General form: the radix passes, the first of which computes the score on the fly and
// writes it out.  Decode-step form (evict_hint small): one pass that scores and lists the candidates below the
// carried bound, resolved by the last block of every sequence, and the mask pass.
kvtrim_status launch_score_select_paged(kvtrim_ctx*, const CacheView& pool, const PagedArgs&, const int32_t* now,
                                        const int64_t* budget, float* score, uint8_t* keep, int32_t* kept, uint32_t* thr,
                                        hipStream_t, bool evict = false);
kvtrim_status launch_score_select(kvtrim_ctx*, const CacheView&, const int32_t* now, const int64_t* budget, float* score,
                                  uint8_t* keep, int32_t* kept, uint32_t* thr, int64_t evict_hint, hipStream_t);
kvtrim_status launch_step_scan(kvtrim_ctx*, const CacheView&, const int32_t* now, const int64_t* budget, float* score,
                               int32_t* kept, uint32_t* thr, const StepArgs& sa, hipStream_t);
// The decode step in one call: append, stages 1 + 2, stages 3 + 4 (three kernels when the step is a decode step).
kvtrim_status launch_decode_step(kvtrim_ctx*, const CacheViewMut& src, const StepArgs& sa, const int32_t* now,
                                 const int64_t* budget, float* score, int32_t* kept, uint32_t* thr, const uint16_t* q,
                                 int32_t layer_begin, int32_t layer_end, float scale, float* out, float* lse,
                                 int64_t evict_hint, hipStream_t);
// The same with stages 3 + 4 inside the cache (four kernels: the row mover is followed by k_cmp_unstage).
kvtrim_status launch_decode_step_inplace(kvtrim_ctx*, const CacheViewMut& c, const StepArgs& sa, const CacheViewMut& stage,
                                         const int32_t* now, const int64_t* budget, float* score, int32_t* kept, uint32_t* thr,
                                         const uint16_t* q, int32_t layer_begin, int32_t layer_end, float scale, float* out,
                                         float* lse, int64_t evict_hint, hipStream_t);
kvtrim_status launch_score_select_general(kvtrim_ctx*, const CacheView&, const int32_t* now, const int64_t* budget,
                                          float* score, uint8_t* keep, int32_t* kept, uint32_t* thr, hipStream_t);
kvtrim_status launch_compact(kvtrim_ctx*, const CacheView& src, const uint8_t* keep, const int32_t* kept,
                             const CacheViewMut& dst, int32_t reserve, hipStream_t);
kvtrim_status launch_attn(kvtrim_ctx*, const CacheView&, const uint16_t* q, const int32_t* soft_now,
                          int32_t layer_begin, int32_t layer_end, float scale, float* out, float* lse, hipStream_t);
void launch_select_passes_paged(kvtrim_ctx*, const float* score, const SelTables&, int hist_blocks, int pass,
                                uint32_t* thr, hipStream_t);
struct PagedView;
// tidy: the merge kernel's launch also takes the pages that an eviction emptied out of the block tables
kvtrim_status launch_attn_paged(kvtrim_ctx*, const CacheView& pool, const int32_t* block_table, const uint16_t* q,
                                int max_chunks,
                                int32_t layer_begin, int32_t layer_end, float scale, float* out, float* lse,
                                hipStream_t, const PagedView* tidy = nullptr);
// gat: also writes the table of the DESTINATION's CMP_CHUNK-row chunks (ws.att_chunk_prefix / ws.att_desc) and the source
// row of every destination row (ws.gat_src) - what the gathering instance of the fused kernel reads.
void launch_cmp_scan_aligned(kvtrim_ctx*, const CacheView& src, const uint8_t* keep, const int32_t* kept,
                             const CacheViewMut& dst, int32_t reserve, int32_t align, hipStream_t, bool gat = false);
// A selection that keeps few entries of every chunk (a destination under a quarter of the source cannot take more than
// one source entry in four) whose tables fit the workspace: the compaction scan then also lists the destination's chunks
// and the source row of every destination row, and the rows are moved a block per chunk of the DESTINATION.
inline bool gather_fits(const kvtrim_ctx* ctx, int64_t src_cap, int64_t dst_cap) {
    const int64_t dst_chunks = dst_cap / kvtrim::CMP_CHUNK + ctx->shape.nseg;
    return dst_cap < src_cap / 4 && dst_chunks <= ctx->ws.max_att_chunks && dst_chunks * kvtrim::CMP_CHUNK <= ctx->ws.gat_slots &&
           src_cap / kvtrim::CMP_CHUNK + ctx->shape.nseg <= ctx->ws.max_cmp_chunks;
}
// The gathering instance of the fused kernel without the attention (the tables of a compaction scan with gat = true
// must be in the workspace).
kvtrim_status launch_gather_rows(kvtrim_ctx*, const CacheView& src, const CacheViewMut& dst, hipStream_t);
kvtrim_status launch_cmp_copy(kvtrim_ctx*, const CacheView& src, const uint8_t* keep, const CacheViewMut& dst,
                              hipStream_t);
kvtrim_status launch_occupancy(kvtrim_ctx*, const CacheView&, const int32_t* now, double* occ, hipStream_t);
void launch_cmp_scan(kvtrim_ctx*, const CacheView& src, const uint8_t* keep, const int32_t* kept,
                     const CacheViewMut& dst, int32_t reserve, hipStream_t);
// persist_nb > 0: the partial results are those of k_att_partial launched with that many blocks (one per block and
// segment; shares start at multiples of round_rows, chunks have chunk_rows rows, extra slots from extra_base on)
kvtrim_status launch_combine(kvtrim_ctx*, const int32_t* chunk_prefix, int32_t layer_begin, int32_t layer_end,
                             float* out, float* lse, hipStream_t, int persist_nb = 0, int round_rows = 1, int chunk_rows = 1,
                             int extra_base = 0);
// ... whose launch also finishes an in-place compaction: the rows parked in `stage` go to their places
kvtrim_status launch_combine_unstage(kvtrim_ctx*, const int32_t* chunk_prefix, int32_t layer_begin, int32_t layer_end,
                                     float* out, float* lse, const CacheViewMut& c, const CacheViewMut& stage,
                                     const int32_t* kept, int64_t max_chunks, hipStream_t);
void launch_cmp_scan_inplace(kvtrim_ctx*, const CacheViewMut& c, const uint8_t* keep, const int32_t* kept, hipStream_t);
// Stage 3 alone inside the cache itself.
kvtrim_status launch_compact_inplace(kvtrim_ctx*, const CacheViewMut& c, const uint8_t* keep, const int32_t* kept,
                                     const CacheViewMut& stage, hipStream_t);
// Stages 3 + 4 inside the cache itself (every segment keeps its start); `stage` lends its row and metadata arrays.
kvtrim_status launch_compact_attn_inplace(kvtrim_ctx*, const CacheViewMut& c, const uint8_t* keep, const int32_t* kept,
                                          const CacheViewMut& stage, const uint16_t* q, int32_t layer_begin,
                                          int32_t layer_end, float scale, float* out, float* lse, hipStream_t);
kvtrim_status launch_compact_attn(kvtrim_ctx*, const CacheView& src, const uint8_t* keep, const int32_t* kept,
                                  const CacheViewMut& dst, int32_t reserve, const uint16_t* q,
                                  int32_t layer_begin, int32_t layer_end, float scale, float* out, float* lse,
                                  hipStream_t, int64_t evict_hint = 0);
// copy_rows = false: only the metadata of the new tokens enters the cache (their K/V rows stay with the caller);
// old_len_out (or NULL) gets every segment's length before the call.
kvtrim_status launch_append(kvtrim_ctx*, const CacheViewMut&, const uint16_t* k_new, const uint16_t* v_new,
                            const float* lb_new, const float* lt_new, const int32_t* pos_new, int32_t n_new,
                            bool copy_rows, int32_t* old_len_out, hipStream_t);
// The row mover for a source whose entries from old_len[seg] on have their K/V rows in k_new / v_new
// ([nseg][n_new][head_dim]) instead of in src (the tables of k_cmp_scan must be in the workspace).
kvtrim_status launch_cmp_copy_new(kvtrim_ctx*, const CacheView& src, const uint8_t* keep, const CacheViewMut& dst,
                                  const uint16_t* k_new, const uint16_t* v_new, int32_t n_new, const int32_t* old_len,
                                  hipStream_t);

kvtrim_status launch_min_room(kvtrim_ctx*, const CacheView&, int32_t* out, hipStream_t);

kvtrim_status hip_fail(kvtrim_ctx* ctx, hipError_t e, const char* what);

// Pieces of the context set-up that the entry point without a context shares: the config check, the shape
// derived from a config, and the layout of a workspace that holds the tables of stage 2 only (returns its size
// in bytes; binds `ws` to `base` when ws is not NULL).
bool config_valid(const kvtrim_config* cfg);
void shape_of(const kvtrim_config* cfg, Shape& sh);
size_t select_workspace(const kvtrim_config* cfg, char* base, Workspace* ws);

#define KVTRIM_HIP(ctx, expr)                                          \
    do {                                                               \
        hipError_t _e = (expr);                                        \
        if (_e != hipSuccess) return ::kvtrim::hip_fail(ctx, _e, #expr); \
    } while (0)

// Brackets the launches made while it is alive with a pair of events when profiling asks for it.
struct ProfScope {
    kvtrim_ctx* ctx;
    hipStream_t st;
    int slot;
    ProfScope(kvtrim_ctx* c, int kernel, hipStream_t s) : ctx(c), st(s), slot(-1) {
        if ((c->prof_mask >> kernel) & 1u) {
            if (c->prof_used < KVTRIM_PROFILE_MAX_LAUNCHES) {
                slot = c->prof_used++;
                c->prof_kernel[slot] = (int8_t)kernel;
                (void)hipEventRecord(c->prof_ev[2 * slot], st);
            }
        }
    }
    ~ProfScope() {
        if (slot >= 0) (void)hipEventRecord(ctx->prof_ev[2 * slot + 1], st);
    }
};

// ---- device helpers --------------------------------------------------------------------
// Digit of pass PASS (11 + 11 + 10 bits, most significant first) and whether the higher digits
// of the key equal the prefix fixed so far.
template <int PASS>
__device__ __forceinline__ bool digit_of(uint32_t key, uint32_t prefix, int* bin) {
    if (PASS == 0) {
        *bin = key >> 21;
        return true;
    } else if (PASS == 1) {
        *bin = (key >> 10) & 2047;
        return (key >> 21) == prefix;
    } else {
        *bin = key & 1023;
        return (key >> 10) == prefix;
    }
}

__device__ __forceinline__ uint32_t key_of_score(float s) {
    uint32_t u = __float_as_uint(s);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// How many retained entries the bound of the decode-step selection is placed above the threshold when a full
// select seeds it: twice the evictions of the call that seeds it, but at least twice a one-token decode step's
// (one entry per segment) and at most a quarter of the candidate list - a first eviction after a prefill evicts
// millions, the decode steps that follow it a few hundred.
__device__ __forceinline__ int64_t seed_distance(int64_t evicted, int segs_per_seq, int fl_cap) {
    int64_t d = 2 * (evicted + 1);
    const int64_t lo = 2 * ((int64_t)segs_per_seq + 1), hi = fl_cap / 4;
    d = d < lo ? lo : d;
    return d > hi ? (hi > 1 ? hi : 1) : d;
}

// number of set bits of `mask` below this lane
__device__ __forceinline__ int mbcnt(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

}  // namespace kvtrim
