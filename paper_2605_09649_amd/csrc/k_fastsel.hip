// Stages 1 + 2 for decode steps (Sec. 4.2: Eq. global_score and the global eviction rule) in two kernels; the
// first of them, in its STEP form, is also the first kernel of the one-call decode step.
//
// A decode step evicts a handful of entries per sequence - as many as it appended - so the selection is the
// search for the FEW LOWEST entries of the total order (key descending, segment ascending, position ascending),
// not a general top-B.  The pass that computes the scores lists every entry whose key lies below a bound `hi`
// carried over from the previous call; if the list holds at least k + 1 entries (k = count - min(budget, count)
// evictions), the k + 1 lowest entries of the whole sequence are the k + 1 lowest of the list, because every entry
// that is not listed has a key >= hi > every listed key.  The last block to finish a sequence ("last block done",
// one arrival counter per sequence) ranks the list - a few hundred entries - and publishes the last retained
// entry of the order as (key, segment, position); the mask kernel compares every entry with that triple.
//
// The bound adapts by itself: the next bound is the key of about the 3(k+1)-th lowest entry of the current
// list.  Scores only decay from step to step (beta <= 1, Eq. global_score) and new tokens enter with the highest
// scores, so the 2(k+1) retained entries below that key are below it at the next step as well: with a steady
// number of evictions per step the list can never come up short.  Nothing depends on the bound for correctness:
// a list that is short (first call, a budget or workload change), too long for its buffer, or with too many equal
// keys at the threshold makes the last block run a plain three-pass radix select over the sequence on its own
// (slow - one block reads every score three times - but rare) which also re-seeds the bound.
#include "kvtrim_paged_device.h"

namespace kvtrim {

constexpr int FAST_ITEMS = FL_CAP_MAX / FAST_THREADS;             // list entries a thread of the resolving block holds
constexpr int FAST_SUB = 16;                                      // sub-lists / group words per sequence
constexpr int FAST_STAGE = 1024;                                  // candidates a block stages in LDS
constexpr int FAST_BATCH = 8;                                     // entries a thread loads before it uses any of them
constexpr int FAST_BIN_DIRECT = 256;                              // a bin of at most this many entries is ranked directly
static_assert(FAST_ITEMS * FAST_THREADS == FL_CAP_MAX, "list capacity must be a multiple of the block size");

// Length of segment g, or 0 with *bad set when its table entry is unusable (negative, beyond the buffers, or
// overlapping its successor).  Every kernel of this file sees a segment through this function.
__device__ __forceinline__ int seg_checked_len(const CacheView& c, int g, int nseg, int64_t* start, bool* bad) {
    const int len = c.seg_len[g];
    const int64_t st = c.seg_start[g];
    const int64_t nxt = g + 1 < nseg ? c.seg_start[g + 1] : c.cap;
    *start = st;
    if (len < 0 || st < 0 || st + len > c.cap || st + len > nxt) {
        *bad = true;
        return 0;
    }
    return len;
}

// A segment as the kernels see it.  STEP: its entries [len_old, len) are this step's new tokens - up to the first
// padding row (negative position), none if the segment has no room for them (kvtrim_append's rule) - whose
// metadata is read from the new-token buffers by every block, never from the cache.
// PAGED: the segment's entries are the slots of its pages in block-table order (entry j = slot j % 128 of the table's
// page j / 128; start = the table's row); slots with a negative position are empty and `live` counts the others.
struct SegView {
    int64_t start;
    int len_old;
    int len;
    int live;
};

constexpr int SCAN_RAGGED = 0, SCAN_STEP = 1, SCAN_PAGED = 2;     // what k_fast_scan walks over

template <int KIND>
__device__ __forceinline__ SegView seg_view(const CacheView& c, int g, int nseg, const StepArgs& sa, bool* bad, bool* nocap) {
    constexpr bool STEP = KIND == SCAN_STEP;
    SegView v;
    if (KIND == SCAN_PAGED) {
        const int npg = sa.pg.seg_pages[g], live = sa.pg.seg_live[g];
        v.start = (int64_t)g * sa.pg.max_pps;
        if (npg < 0 || npg > sa.pg.max_pps || live < 0 || (int64_t)live > (int64_t)npg * KVTRIM_PAGE_SIZE) {
            *bad = true;
            v.len_old = v.len = v.live = 0;
            return v;
        }
        v.len_old = v.len = npg * KVTRIM_PAGE_SIZE;
        v.live = live;
        return v;
    }
    const int len = c.seg_len[g];
    const int64_t st = c.seg_start[g];
    const int64_t nxt = g + 1 < nseg ? c.seg_start[g + 1] : c.cap;
    v.start = st;
    if (len < 0 || st < 0 || st + len > c.cap || st + len > nxt) {
        *bad = true;
        v.len_old = v.len = v.live = 0;
        return v;
    }
    v.len_old = v.len = len;
    if (STEP) {
        int cnt = 0;
        while (cnt < sa.n_new && sa.pos_new[(int64_t)g * sa.n_new + cnt] >= 0) ++cnt;
        if (st + len + cnt > nxt || nxt > c.cap) {
            if (cnt) *nocap = true;
            cnt = 0;
        }
        v.len = len + cnt;
    }
    v.live = v.len;
    return v;
}

// a is evicted before b: lower key first; among equal keys the later (segment, position) first
__device__ __forceinline__ bool evicted_before(uint32_t ka, int sa, int pa, uint32_t kb, int sb, int pb) {
    if (ka != kb) return ka < kb;
    if (sa != sb) return sa > sb;
    return pa > pb;
}

struct ResolveShared {
    uint32_t h[2048];
    int64_t lds64[17];
    int32_t lds32[17];
    uint32_t red_u[16];
    int bin, bin_m, cnt, gather_n, found_seg, found_pos, digit;
    int64_t before, rank_in;
    uint32_t found_key, bin_count;
    uint32_t g_key[FAST_BIN_DIRECT];
    int32_t g_seg[FAST_BIN_DIRECT], g_pos[FAST_BIN_DIRECT];
};

__device__ __forceinline__ uint32_t block_min_u32(uint32_t v, uint32_t* red) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v = min(v, (uint32_t)__shfl_xor((int)v, d, 64));
    __syncthreads();
    if (lane_id() == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    uint32_t r = 0xFFFFFFFFu;
    for (int i = 0; i < (int)(blockDim.x >> 6); ++i) r = min(r, red[i]);
    return r;
}

__device__ __forceinline__ uint32_t block_max_u32(uint32_t v, uint32_t* red) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v = max(v, (uint32_t)__shfl_xor((int)v, d, 64));
    __syncthreads();
    if (lane_id() == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    uint32_t r = 0;
    for (int i = 0; i < (int)(blockDim.x >> 6); ++i) r = max(r, red[i]);
    return r;
}

// Walks an LDS histogram of NB bins from the top bin down to the one that holds the entry of rank `rank`
// (1-based, descending digit order).  Results in sm->digit, sm->rank_in (rank inside the bin), sm->bin_count.
template <int NB>
__device__ __forceinline__ void walk_from_top(ResolveShared* sm, int64_t rank) {
    constexpr int PER = NB / FAST_THREADS;                        // 2 or 1 bins per thread, thread 0 owns the highest
    const int tid = threadIdx.x;
    uint32_t cnt[PER];
    int64_t mine = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        cnt[i] = sm->h[NB - 1 - (tid * PER + i)];
        mine += cnt[i];
    }
    int64_t tot;
    int64_t above = block_excl_scan<int64_t>(mine, sm->lds64, &tot);
    if (above < rank && rank <= above + mine) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            if (rank <= above + cnt[i]) {
                sm->digit = NB - 1 - (tid * PER + i);
                sm->rank_in = rank - above;
                sm->bin_count = cnt[i];
                break;
            }
            above += cnt[i];
        }
    }
    __syncthreads();
}

// Where the key of an entry comes from: computed from log beta and the position (SCORE: stage 1 fused, Eq.
// global_score in log domain - one fp32 multiply, or one fused multiply-add with the cached horizon tail) or
// read from the caller's score array.  Both are inputs of the call, so any block may read any entry at any time.
template <bool SCORE, int KIND>
struct KeySource {
    static constexpr bool STEP = KIND == SCAN_STEP, PAGED = KIND == SCAN_PAGED;
    const float* score_in;
    const float* lb;
    const float* lt;
    const int32_t* pos;
    const float* lb_new;
    const float* lt_new;
    const int32_t* pos_new;
    int n_new;
    int t1;
    const int32_t* bt;                                            // PAGED: the block tables and the pool's page count
    int n_pages;
    // where entry j of the segment lies in the cache's arrays (not for a STEP's new tokens); *bad_page: the block
    // table names a page outside the pool (the page is clamped into it)
    __device__ __forceinline__ int64_t place(const SegView& v, int j, bool* bad_page) const {
        if (!PAGED) return v.start + j;
        int pg = bt[v.start + (j >> 7)];
        if (pg < 0 || pg >= n_pages) {
            *bad_page = true;
            pg = pg < 0 ? 0 : n_pages - 1;
        }
        return (int64_t)pg * KVTRIM_PAGE_SIZE + (j & (KVTRIM_PAGE_SIZE - 1));
    }
    // entry j of segment g: false for an empty slot (PAGED), else its position and score
    __device__ __forceinline__ bool entry_at(int g, const SegView& v, int j, int* p_out, float* s_out) const {
        float b, t = 0.f;
        int p;
        if (STEP && j >= v.len_old) {
            const int64_t i = (int64_t)g * n_new + (j - v.len_old);
            p = pos_new[i];
            b = lb_new[i];
            if (lt) t = lt_new[i];
        } else {
            bool bp = false;
            const int64_t e = place(v, j, &bp);
            p = pos[e];
            if (PAGED && p < 0) return false;
            if (!SCORE) {
                *p_out = p;
                *s_out = score_in[e];
                return true;
            }
            b = lb[e];
            if (lt) t = lt[e];
        }
        *p_out = p;
        if (!SCORE) {
            *s_out = 0.f;                                         // (a STEP always computes its scores)
            return true;
        }
        const float dt = (float)(t1 - p);
        *s_out = lt ? __fmaf_rn(dt, b, t) : __fmul_rn(dt, b);
        return true;
    }
};

// One digit of a most-significant-digit radix select over all entries of the sequence, by this block alone.
template <int PASS, bool SCORE, int KIND>
__device__ __forceinline__ void slow_pass(const KeySource<SCORE, KIND>& ks, const CacheView& c, const Shape& sh,
                                          const StepArgs& sa, int seq, uint32_t prefix, ResolveShared* sm) {
    constexpr int NB = PASS == 2 ? 1024 : 2048;
    const int tid = threadIdx.x;
    __syncthreads();
    for (int i = tid; i < NB; i += FAST_THREADS) sm->h[i] = 0;
    __syncthreads();
    for (int g = seq * sh.segs_per_seq; g < (seq + 1) * sh.segs_per_seq; ++g) {
        bool bad = false, nocap = false;
        const SegView v = seg_view<KIND>(c, g, sh.nseg, sa, &bad, &nocap);
        const int len = v.len;
        for (int j0 = tid; j0 < len; j0 += FAST_THREADS * FAST_BATCH) {
            float sv[FAST_BATCH];
            bool lv[FAST_BATCH];
#pragma unroll
            for (int u = 0; u < FAST_BATCH; ++u) {
                const int j = j0 + u * FAST_THREADS;
                int p;
                sv[u] = 0.f;
                lv[u] = j < len && ks.entry_at(g, v, j, &p, &sv[u]);
            }
#pragma unroll
            for (int u = 0; u < FAST_BATCH; ++u) {
                int bin;
                if (lv[u] && digit_of<PASS>(key_of_score(sv[u]), prefix, &bin)) atomicAdd(&sm->h[bin], 1u);
            }
        }
    }
    __syncthreads();
}

// Key of the entry of rank `rank` (1-based, descending key order) of the sequence; *rank_in = its rank among the
// entries with that key, *ties = how many entries have that key.
template <bool SCORE, int KIND>
__device__ __forceinline__ uint32_t slow_radix(const KeySource<SCORE, KIND>& ks, const CacheView& c, const Shape& sh,
                                               const StepArgs& sa, int seq, int64_t rank, ResolveShared* sm,
                                               int64_t* rank_in, uint32_t* ties) {
    slow_pass<0>(ks, c, sh, sa, seq, 0, sm);
    walk_from_top<2048>(sm, rank);
    uint32_t prefix = (uint32_t)sm->digit;
    rank = sm->rank_in;
    slow_pass<1>(ks, c, sh, sa, seq, prefix, sm);
    walk_from_top<2048>(sm, rank);
    prefix = (prefix << RADIX_BITS1) | (uint32_t)sm->digit;
    rank = sm->rank_in;
    slow_pass<2>(ks, c, sh, sa, seq, prefix, sm);
    walk_from_top<1024>(sm, rank);
    prefix = (prefix << RADIX_BITS2) | (uint32_t)sm->digit;
    *rank_in = sm->rank_in;
    *ties = sm->bin_count;
    __syncthreads();
    return prefix;
}

// One digit of the radix select over the positions of segment g's entries with key == key_thr (taken as
// 0x7fffffff - position, so that the smallest position is the largest): narrows *prefix and *rank.
template <int PASS, bool SCORE, int KIND>
__device__ __forceinline__ void tie_pos_pass(const KeySource<SCORE, KIND>& ks, int g, const SegView& v, uint32_t key_thr,
                                             uint32_t* prefix, int64_t* rank, ResolveShared* sm) {
    constexpr int NB = PASS == 2 ? 1024 : 2048;
    const int tid = threadIdx.x;
    __syncthreads();
    for (int i = tid; i < NB; i += FAST_THREADS) sm->h[i] = 0;
    __syncthreads();
    for (int j = tid; j < v.len; j += FAST_THREADS) {
        int pj, bin;
        float sc;
        if (ks.entry_at(g, v, j, &pj, &sc) && key_of_score(sc) == key_thr &&
            digit_of<PASS>(0x7fffffffu - (uint32_t)pj, *prefix, &bin))
            atomicAdd(&sm->h[bin], 1u);
    }
    __syncthreads();
    walk_from_top<NB>(sm, *rank);
    *prefix = PASS == 0 ? (uint32_t)sm->digit : (*prefix << (PASS == 1 ? RADIX_BITS1 : RADIX_BITS2)) | (uint32_t)sm->digit;
    *rank = sm->rank_in;
}

// The `quota`-th entry (1-based) with key == key_thr in (segment ascending, position ascending) order:
// result in sm->found_seg / sm->found_pos.  The caller guarantees that it exists.
template <bool SCORE, int KIND>
__device__ __forceinline__ void slow_tie_walk(const KeySource<SCORE, KIND>& ks, const CacheView& c, const Shape& sh,
                                              const StepArgs& sa, int seq, uint32_t key_thr, int64_t quota,
                                              ResolveShared* sm) {
    const int tid = threadIdx.x;
    int64_t need = quota;
    auto is_tie = [&](int g, const SegView& v, int j, int* p) {
        float sc;
        return j < v.len && ks.entry_at(g, v, j, p, &sc) && key_of_score(sc) == key_thr;
    };
    for (int g = seq * sh.segs_per_seq; g < (seq + 1) * sh.segs_per_seq; ++g) {
        bool bad = false, nocap = false;
        const SegView v = seg_view<KIND>(c, g, sh.nseg, sa, &bad, &nocap);
        const int len = v.len;
        int mine = 0, p;
        for (int j = tid; j < len; j += FAST_THREADS) mine += is_tie(g, v, j, &p);
        const int in_seg = block_sum<int32_t>(mine, sm->lds32);
        if (need > in_seg) {
            need -= in_seg;
            continue;
        }
        if (KIND == SCAN_PAGED) {
            // the entry is in this segment, whose slots are in no particular order: the need-th smallest position
            // among its ties is the need-th largest of 0x7fffffff - position - three digits, as for the keys
            uint32_t prefix = 0;
            int64_t rank = need;
            tie_pos_pass<0>(ks, g, v, key_thr, &prefix, &rank, sm);
            tie_pos_pass<1>(ks, g, v, key_thr, &prefix, &rank, sm);
            tie_pos_pass<2>(ks, g, v, key_thr, &prefix, &rank, sm);
            __syncthreads();
            if (tid == 0) {
                sm->found_seg = g;
                sm->found_pos = (int)(0x7fffffffu - prefix);
            }
            __syncthreads();
            return;
        }
        // the entry is in this segment: entries are stored in position order
        int64_t running = 0;
        for (int base = 0; base < len; base += FAST_THREADS) {    // uniform trip count
            const int j = base + tid;
            int pj = 0;
            const int is_eq = is_tie(g, v, j, &pj);
            int32_t tot;
            const int32_t ex = block_excl_scan<int32_t>(is_eq, sm->lds32, &tot);
            if (is_eq && running + ex == need - 1) {
                sm->found_seg = g;
                sm->found_pos = pj;
            }
            running += tot;
            if (running >= need) break;                           // uniform: tot comes from LDS
        }
        __syncthreads();
        return;
    }
    __syncthreads();
}

// loads and stores that bypass the caches which are not coherent across the chip (what one block writes this way
// and has seen acknowledged, another block reads this way without any fence)
template <typename T>
__device__ __forceinline__ T ld_dev(const T* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
template <typename T>
__device__ __forceinline__ void st_dev(T* p, T v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// SCORE: stage 1 is computed here (and written to score_out); otherwise the scores are read from score_in.
// STEP (implies SCORE): the decode step in one call.  Every block scores a segment's new tokens from the new-token
// buffers; one more block per segment, behind the scanning blocks of the grid, writes their rows and metadata into
// the source cache and the segment's part of the row mover's chunk table.  The last block of a sequence also leaves
// what the compaction needs: survivors per segment, the destination's segment table and - when the evicted entries
// are on the candidate list - per chunk of 128 entries the number of entries it loses and per segment a record with
// the start of its survivors in the destination and the indices of its evicted entries, from which a block of the
// row mover places its chunk's survivors itself (and writes its mask bytes).  After the single-block select, or
// with more evictions than the lists hold, it writes the whole mask and a destination offset per chunk instead.
//
// Cross-block traffic inside the kernel: the candidate lists, their counters, the lowest keys and the arrival
// counters.  All of it is written with device-scope atomics or write-through stores whose acknowledgement the
// writer waits for before it arrives, and read with device-scope loads - so no block needs a fence, which on this
// chip means a write-back of a whole L2.  The scores written here are read by the NEXT kernel only; the
// single-block select, which has to look at every entry, recomputes them from the call's inputs.
template <bool SCORE, int KIND>
__global__ __launch_bounds__(FAST_THREADS) void k_fast_scan(CacheView c, const int32_t* __restrict__ now,
                                                            const float* score_in, float* score_out,
                                                            const int64_t* __restrict__ budget, Shape sh, Workspace ws,
                                                            int bps, int32_t* __restrict__ kept_out,
                                                            uint32_t* __restrict__ thr_out, StepArgs sa) {
    constexpr bool STEP = KIND == SCAN_STEP, PAGED = KIND == SCAN_PAGED;
    static_assert(!STEP || SCORE, "the one-call step computes the scores itself");
    __shared__ ResolveShared sm;
    __shared__ int s_last, s_ncand;
    __shared__ uint32_t s_base;
    // this block's candidates, before they go to the list; the last block of a sequence reuses the space (STEP)
    __shared__ int32_t s_pool[(STEP ? 3 : 2) * FAST_STAGE];
    uint32_t* c_key = reinterpret_cast<uint32_t*>(s_pool);
    int32_t* c_pos = s_pool + FAST_STAGE;
    int32_t* c_idx = s_pool + (STEP ? 2 : 1) * FAST_STAGE;
    __shared__ int s_ev[STEP ? STEP_MAX_SEGS : 1], s_off[STEP ? STEP_MAX_SEGS : 1];
    __shared__ int s_seqcnt[STEP ? STEP_MAX_SEQS : 1];
    static_assert(STEP_MAX_SEGS <= FAST_STAGE && STEP_MAX_SEGS <= FAST_THREADS && STEP_MAX_EVICT <= FAST_STAGE, "the step's tables reuse the staging space, one segment per thread");
    const int tid = threadIdx.x;
    // PAGED, when the caller attends next: behind the scanning blocks the grid has PG_TABLE_BLOCKS blocks that build the
    // attention's chunk table.  The table depends on the block tables only, which this step's eviction leaves alone (a
    // page that it empties stays listed until it is tidied away, and a reader finds all its slots empty).
    if (PAGED && (int)blockIdx.x >= sh.nseg * bps) {
        PagedView pc{};
        pc.block_table = const_cast<int32_t*>(sa.pg.block_table);
        pc.seg_pages = const_cast<int32_t*>(sa.pg.seg_pages);
        pc.seg_live = const_cast<int32_t*>(sa.pg.seg_live);
        pc.n_pages = sa.pg.n_pages;
        pc.max_pps = sa.pg.max_pps;
        const int H = sh.n_kv_heads, L = sh.n_layers, lb = sa.pg.plan_layer_begin, le = sa.pg.plan_layer_end;
        auto in_range = [=](int g) {
            const int layer = (g / H) % L;
            return layer >= lb && layer < le;
        };
        build_page_table<ATT_PAGE_GROUP>(pc, sh.nseg, in_range, ws.att_chunk_prefix, ws.att_desc, ws.max_att_chunks, nullptr,
                                         ws.err, (int)blockIdx.x - sh.nseg * bps, (int)gridDim.x - sh.nseg * bps, ws.att_pages,
                                         ws.att_row_prefix);
        return;
    }
    // STEP: behind the scanning blocks the grid has one block per segment that only writes the segment's tables
    const bool tables_only = STEP && (int)blockIdx.x >= sh.nseg * bps;
    const int seg = tables_only ? (int)blockIdx.x - sh.nseg * bps : (int)blockIdx.x / bps;
    const int part = tables_only ? 0 : (int)blockIdx.x % bps;
    const int seq = seg / sh.segs_per_seq;
    // Device-scope atomics on one address are served one after the other (tens of nanoseconds each), so the
    // blocks of a sequence do not meet on one word: the list is kept in up to FAST_SUB sub-lists with a counter
    // each, the lowest key and the arrivals in FAST_SUB group words (then one top-level arrival per group).
    const int blk_in_seq = (seg - seq * sh.segs_per_seq) * bps + part;
    const int nblk = sh.segs_per_seq * bps;
    const int nsub = nblk < FAST_SUB ? nblk : FAST_SUB;
    const int sub = blk_in_seq % nsub;
    if (tid == 0) s_ncand = 0;
    __syncthreads();
    bool bad = false, nocap = false;
    const SegView sv0 = seg_view<KIND>(c, seg, sh.nseg, sa, &bad, &nocap);
    const int64_t start = sv0.start;
    const int len = sv0.len;
    if (tid == 0 && part == 0 && !tables_only && (bad || nocap)) atomicOr(ws.err, bad ? ERR_LAYOUT : ERR_CAP);
    const uint32_t hi = ws.fast_hi[seq];
    const uint32_t cap = (uint32_t)ws.fl_cap;
    const uint32_t subcap = cap / (uint32_t)nsub;                 // entries per sub-list
    uint32_t* lk = ws.fl_key + (size_t)seq * cap;
    int32_t* ls = ws.fl_seg + (size_t)seq * cap;
    int32_t* lp = ws.fl_pos + (size_t)seq * cap;
    int32_t* li = ws.fl_idx + (size_t)seq * cap;
    uint32_t* sub_count = ws.fl_count + (size_t)seq * FAST_SUB;
    uint32_t* grp_min = ws.fast_min + (size_t)seq * FAST_SUB;
    uint32_t* done = ws.fast_done + (size_t)seq * (FAST_SUB + 1);
    KeySource<SCORE, KIND> ks;
    ks.bt = sa.pg.block_table;
    ks.n_pages = sa.pg.n_pages;
    ks.score_in = score_in;
    ks.lb = c.log_beta;
    ks.lt = c.log_tail;
    ks.pos = c.pos;
    ks.lb_new = sa.lb_new;
    ks.lt_new = sa.lt_new;
    ks.pos_new = sa.pos_new;
    ks.n_new = sa.n_new;
    ks.t1 = SCORE ? now[seq] + 1 : 0;

    // STEP, the segment's tables-only block (it takes no part in the scan, so the sequence's last block never waits
    // for this): the segment's new tokens enter the source cache, and the segment's part of the row mover's chunk
    // table is written.  Both are read by the next kernel only.
    if (tables_only) {
        // ---- this segment's new tokens enter the source cache (rows: 16 bytes per thread; metadata)
        const int cnt_new = sv0.len - sv0.len_old;
        const int vpr = sh.head_dim / 8;
        const uint4* kn = reinterpret_cast<const uint4*>(sa.k_new) + (int64_t)seg * sa.n_new * vpr;
        const uint4* vn = reinterpret_cast<const uint4*>(sa.v_new) + (int64_t)seg * sa.n_new * vpr;
        uint4* kd = reinterpret_cast<uint4*>(sa.src.k) + (start + sv0.len_old) * vpr;
        uint4* vd = reinterpret_cast<uint4*>(sa.src.v) + (start + sv0.len_old) * vpr;
        for (int i = tid; i < cnt_new * vpr; i += FAST_THREADS) {
            kd[i] = kn[i];
            vd[i] = vn[i];
        }
        for (int i = tid; i < cnt_new; i += FAST_THREADS) {
            const int64_t e = start + sv0.len_old + i, ni = (int64_t)seg * sa.n_new + i;
            sa.src.log_beta[e] = sa.lb_new[ni];
            if (c.log_tail) sa.src.log_tail[e] = sa.lt_new[ni];
            sa.src.pos[e] = sa.pos_new[ni];
        }
        // ---- and its part of the row mover's chunk table: the chunks of the segments before it are counted here
        int before = 0;
        for (int g = tid; g < seg; g += FAST_THREADS) {
            bool b2 = false, n2 = false;
            const SegView v = seg_view<KIND>(c, g, sh.nseg, sa, &b2, &n2);
            before += (v.len + CMP_CHUNK - 1) / CMP_CHUNK;
        }
        before = block_sum<int32_t>(before, sm.lds32);
        const int nch = (len + CMP_CHUNK - 1) / CMP_CHUNK;
        for (int ch = tid; ch < nch; ch += FAST_THREADS) {
            ChunkDesc d;
            d.first = start + (int64_t)ch * CMP_CHUNK;
            d.n = min(CMP_CHUNK, len - ch * CMP_CHUNK);
            d.seg = seg;
            ws.cmp_desc[before + ch] = d;
        }
        if (tid == 0) {
            ws.cmp_chunk_prefix[seg] = before;
            if (seg == sh.nseg - 1) ws.cmp_chunk_prefix[sh.nseg] = before + nch;
            if (!sa.inplace) ws.step_len[seg] = len;              // (in place: the sequence's last block leaves the survivors' count there)
        }
        return;
    }

    // ---- every entry of this block's share: score, and onto the list if its key is below the bound
    {
        uint32_t mn = 0xFFFFFFFFu;
        // batches of FAST_BATCH entries per thread: all loads of a batch are issued before any of them is used
        for (int j0 = part * FAST_THREADS + tid; j0 < len; j0 += bps * FAST_THREADS * FAST_BATCH) {
            float sv[FAST_BATCH];
            int pv[FAST_BATCH];
            int64_t at[FAST_BATCH];                               // where the entry lies in the arrays
            bool bad_page = false;
#pragma unroll
            for (int u = 0; u < FAST_BATCH; ++u) {
                const int j = j0 + u * bps * FAST_THREADS;
                const bool isnew = STEP && j >= sv0.len_old;
                at[u] = isnew ? (int64_t)seg * sa.n_new + (j - sv0.len_old) : (j < len ? ks.place(sv0, j, &bad_page) : 0);
            }
            if (PAGED && bad_page) atomicOr(ws.err, ERR_LAYOUT);
            if (SCORE) {
                float lbv[FAST_BATCH], ltv[FAST_BATCH];
#pragma unroll
                for (int u = 0; u < FAST_BATCH; ++u) {
                    const int j = j0 + u * bps * FAST_THREADS;
                    const bool in = j < len;
                    const bool isnew = STEP && j >= sv0.len_old;
                    pv[u] = in ? (isnew ? sa.pos_new : c.pos)[at[u]] : 0;
                    lbv[u] = in ? (isnew ? sa.lb_new : c.log_beta)[at[u]] : 0.f;
                    ltv[u] = (in && c.log_tail) ? (isnew ? sa.lt_new : c.log_tail)[at[u]] : 0.f;
                }
#pragma unroll
                for (int u = 0; u < FAST_BATCH; ++u) {
                    const int j = j0 + u * bps * FAST_THREADS;
                    const float dt = (float)(ks.t1 - pv[u]);
                    sv[u] = c.log_tail ? __fmaf_rn(dt, lbv[u], ltv[u]) : __fmul_rn(dt, lbv[u]);
                    if (PAGED && pv[u] < 0) sv[u] = 0.f;          // an empty slot's score reads 0
                    if (j < len) score_out[STEP ? start + j : at[u]] = sv[u];
                }
            } else {
#pragma unroll
                for (int u = 0; u < FAST_BATCH; ++u) {
                    const int j = j0 + u * bps * FAST_THREADS;
                    sv[u] = j < len ? score_in[at[u]] : 0.f;
                    pv[u] = (PAGED && j < len) ? c.pos[at[u]] : 0;
                }
            }
#pragma unroll
            for (int u = 0; u < FAST_BATCH; ++u) {
                const int j = j0 + u * bps * FAST_THREADS;
                const uint32_t key = key_of_score(sv[u]);
                const bool live = j < len && (!PAGED || pv[u] >= 0);
                if (live) mn = min(mn, key);
                if (live && key < hi) {                           // rare: a few hundred entries per sequence and call
                    const int slot = atomicAdd(&s_ncand, 1);
                    if (slot < FAST_STAGE) {
                        c_key[slot] = key;
                        c_pos[slot] = (SCORE || PAGED) ? pv[u] : c.pos[at[u]];
                        if (STEP) c_idx[slot] = j;
                    }
                }
            }
        }
        mn = block_min_u32(mn, sm.red_u);                         // (its barriers also complete s_ncand and the staged entries)
        const int ncand = s_ncand;
        if (tid == 0) {
            if (mn != 0xFFFFFFFFu) atomicMin(&grp_min[sub], mn);
            // one reservation per block; a block with more candidates than it can stage makes its sub-list overflow
            if (ncand > 0) s_base = atomicAdd(&sub_count[sub], ncand > FAST_STAGE ? cap + 1u : (uint32_t)ncand);
        }
        __syncthreads();
        if (ncand > 0 && ncand <= FAST_STAGE) {
            const uint32_t base = s_base;
            for (int i = tid; i < ncand; i += FAST_THREADS) {
                const uint32_t slot = base + (uint32_t)i;
                if (slot < subcap) {
                    const size_t at = (size_t)sub * subcap + slot;
                    st_dev(&lk[at], c_key[i]);
                    st_dev(&ls[at], (int32_t)seg);
                    st_dev(&lp[at], c_pos[i]);
                    if (STEP) st_dev(&li[at], c_idx[i]);
                }
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");              // this thread's list entries are acknowledged ...
    __syncthreads();                                              // ... and so are the whole block's, before it arrives
    if (tid == 0) {
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");   // (thread 0's own atomics above have returned)
        const int grp = blk_in_seq % FAST_SUB;
        const unsigned gsize = (unsigned)(nblk - grp + FAST_SUB - 1) / FAST_SUB;   // blocks of the sequence with this group number
        int last = 0;
        if (atomicAdd(&done[1 + grp], 1u) == gsize - 1u) {
            const unsigned ngroups = nblk < FAST_SUB ? (unsigned)nblk : (unsigned)FAST_SUB;
            last = atomicAdd(&done[0], 1u) == ngroups - 1u;
        }
        s_last = last;
    }
    __syncthreads();
    if (!s_last) return;

    // ---- the last block of the sequence: everything of the sequence has been scored and listed.
    // All it needs is requested at once: the sub-list counters, the lowest keys, every slot of the list (whether
    // a slot holds an entry is known once the counters are here), the segment lengths, the budget.
    uint32_t sub_n[FAST_SUB];
    uint32_t min_key = 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < FAST_SUB; ++i) {
        sub_n[i] = i < nsub ? ld_dev(&sub_count[i]) : 0u;
        min_key = min(min_key, ld_dev(&grp_min[i]));
    }
    uint32_t key[FAST_ITEMS];
    int sg[FAST_ITEMS], ps[FAST_ITEMS], ix[FAST_ITEMS];
    uint32_t slot_sub[FAST_ITEMS], slot_idx[FAST_ITEMS];
#pragma unroll
    for (int u = 0; u < FAST_ITEMS; ++u) {
        const uint32_t i = (uint32_t)tid + (uint32_t)u * FAST_THREADS;   // slot i of the flat list buffer
        slot_sub[u] = i / subcap;
        slot_idx[u] = i - slot_sub[u] * subcap;
        key[u] = 0;
        sg[u] = ps[u] = ix[u] = 0;
        if (i < cap && slot_sub[u] < (uint32_t)nsub) {
            key[u] = ld_dev(&lk[i]);
            sg[u] = ld_dev(&ls[i]);
            ps[u] = ld_dev(&lp[i]);
            if (STEP) ix[u] = ld_dev(&li[i]);
        }
    }
    const int g0 = seq * sh.segs_per_seq;
    int64_t cnt = 0;
    int64_t step_before = 0, step_total = 0;                      // STEP: destination entries before this sequence / of all sequences
    int step_chunks_before = 0;                                   // STEP: chunks of the sequences before this one
    int my_len = 0;                                               // STEP: length of segment g0 + tid (one segment of the sequence per thread)
    int32_t step_cex = 0, step_ctot = 0;                          // STEP: chunks of the sequence's segments before that one / of all of them
    if (STEP) {
        // entries per sequence of the whole batch (the destination of a sequence starts behind all earlier ones)
        for (int i = tid; i < sh.n_seq; i += FAST_THREADS) s_seqcnt[i] = 0;
        __syncthreads();
        int chunks_before = 0;
        for (int g = tid; g < sh.nseg; g += FAST_THREADS) {
            bool b2 = false, n2 = false;
            const SegView v = seg_view<KIND>(c, g, sh.nseg, sa, &b2, &n2);
            if (v.len) atomicAdd(&s_seqcnt[g / sh.segs_per_seq], v.len);
            if (g < g0) chunks_before += (v.len + CMP_CHUNK - 1) / CMP_CHUNK;
            if (g >= g0 && g < g0 + sh.segs_per_seq) {
                kept_out[g] = 0;
                s_pool[FAST_STAGE + (g - g0)] = v.len;            // (the staging space is free once the block has arrived)
            }
        }
        step_chunks_before = block_sum<int32_t>(chunks_before, sm.lds32);
        int64_t need = 0;
        if (tid < sh.n_seq) {                                     // (n_seq <= FAST_THREADS here)
            int64_t b = budget[tid];
            if (b < 0) b = 0;
            const int64_t n = s_seqcnt[tid];
            need = (b < n ? b : n) + (int64_t)sa.reserve * sh.segs_per_seq;
        }
        int64_t tot;
        const int64_t ex = block_excl_scan<int64_t>(need, sm.lds64, &tot);
        if (tid == seq) sm.before = ex;
        __syncthreads();
        step_before = sm.before;
        step_total = tot;
        // The per-chunk eviction counts of this sequence are cleared NOW, long before they are needed: the stores
        // (write-through: the counts are added with device-scope atomics) complete while the candidates are ranked.
        if (tid < sh.segs_per_seq) my_len = s_pool[FAST_STAGE + tid];
        step_cex = block_excl_scan<int32_t>((my_len + CMP_CHUNK - 1) / CMP_CHUNK, sm.lds32, &step_ctot);
        if (sa.inplace || step_total <= sa.dst.cap)
            for (int i = tid; i < step_ctot; i += FAST_THREADS) st_dev(&ws.step_chunk_ev[step_chunks_before + i], 0u);
        cnt = s_seqcnt[seq];
        __syncthreads();
    } else {
        for (int g = g0 + tid; g < g0 + sh.segs_per_seq; g += FAST_THREADS) {
            bool b2 = false, n2 = false;
            cnt += seg_view<KIND>(c, g, sh.nseg, sa, &b2, &n2).live;
            kept_out[g] = 0;                                      // the mask kernel adds its counts
        }
    }
    int64_t bud = budget[seq];
    if (bud < 0) bud = 0;
    bool sub_overflow = false;
    uint32_t n_list = 0;
#pragma unroll
    for (int i = 0; i < FAST_SUB; ++i) {
        sub_overflow = sub_overflow || sub_n[i] > subcap;
        n_list += sub_n[i] > subcap ? subcap : sub_n[i];
    }
    bool valid[FAST_ITEMS], listed[FAST_ITEMS];
    uint32_t lo = 0xFFFFFFFFu, hi_k = 0;
#pragma unroll
    for (int u = 0; u < FAST_ITEMS; ++u) {
        uint32_t n_here = 0;
#pragma unroll
        for (int q = 0; q < FAST_SUB; ++q) n_here = slot_sub[u] == (uint32_t)q ? sub_n[q] : n_here;
        valid[u] = (uint32_t)tid + (uint32_t)u * FAST_THREADS < cap && slot_sub[u] < (uint32_t)nsub && slot_idx[u] < n_here;
        listed[u] = valid[u];
        if (valid[u]) {
            lo = min(lo, key[u]);
            hi_k = max(hi_k, key[u]);
        }
    }
    __syncthreads();                                              // every thread has read the per-call words
    if (tid <= FAST_SUB) {                                        // ... which go back to "between calls"
        atomicExch(&done[tid], 0u);
        if (tid < FAST_SUB) {
            atomicExch(&sub_count[tid], 0u);
            atomicExch(&grp_min[tid], 0xFFFFFFFFu);
        }
    }
    {   // entries of the sequence, lowest and highest listed key: one reduction
        if (!STEP) cnt = wave_sum(cnt);
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            lo = min(lo, (uint32_t)__shfl_xor((int)lo, d, 64));
            hi_k = max(hi_k, (uint32_t)__shfl_xor((int)hi_k, d, 64));
        }
        if (lane_id() == 0) {
            sm.lds64[tid >> 6] = cnt;
            sm.red_u[tid >> 6] = lo;
            sm.h[tid >> 6] = hi_k;
        }
        __syncthreads();
        if (!STEP) cnt = 0;
        for (int i = 0; i < FAST_THREADS / 64; ++i) {
            if (!STEP) cnt += sm.lds64[i];
            lo = min(lo, sm.red_u[i]);
            hi_k = max(hi_k, sm.h[i]);
        }
    }
    const int64_t want = bud < cnt ? bud : cnt;
    const int64_t k = cnt - want;                                 // entries to evict
    FastSel out;
    out.mode = FSEL_THRESHOLD;
    out.key_thr = 0xFFFFFFFFu;
    out.seg_thr = 0x7fffffff;
    out.pos_thr = 0x7fffffff;
    uint32_t next_hi = hi;
    bool used_fallback = false;
    if (want == 0) {
        out.mode = FSEL_NONE;
    } else if (k == 0) {
        out.mode = FSEL_ALL;
        out.key_thr = min_key;                                    // key of the last entry of the order
    } else {
        bool solved = false;
        if (!sub_overflow && (int64_t)n_list >= k + 1 && n_list <= cap) {
            // -- rank the list: the entry of rank k (0-based, eviction order) is the last retained one
            int64_t r = k;
            bool first = true;
            for (int round = 0; round < 5; ++round) {             // every round narrows the key range by a factor of 1024
                const uint32_t range = hi_k - lo;
                const int shift = range < 1024u ? 0 : 32 - __clz(range) - 10;
                __syncthreads();
                sm.h[tid] = 0;
                if (tid == 0) sm.gather_n = 0;
                __syncthreads();
#pragma unroll
                for (int u = 0; u < FAST_ITEMS; ++u)
                    if (valid[u]) atomicAdd(&sm.h[(key[u] - lo) >> shift], 1u);
                __syncthreads();
                const int32_t v = (int32_t)sm.h[tid];
                int32_t tot;
                const int32_t ex = block_excl_scan<int32_t>(v, sm.lds32, &tot);
                if (ex <= r && r < (int64_t)ex + v) {
                    sm.bin = tid;
                    sm.before = ex;
                    sm.cnt = v;
                }
                if (first) {
                    const int64_t m3 = 3 * (k + 1);
                    const int64_t m = m3 < (int64_t)tot - 1 ? m3 : (int64_t)tot - 1;
                    if (ex <= m && m < (int64_t)ex + v) sm.bin_m = tid;
                }
                __syncthreads();
                const int bin = sm.bin, bcnt = sm.cnt;
                const int64_t before = sm.before;
                if (first) {
                    // next bound: the upper edge of the bin that holds the entry of rank min(3(k+1), n - 1);
                    // doubled distance from the threshold's bin when the list was too short to reach that rank
                    uint64_t edge = (uint64_t)lo + (((uint64_t)sm.bin_m + 1) << shift);
                    if ((int64_t)tot - 1 < 3 * (k + 1)) edge += edge - ((uint64_t)lo + ((uint64_t)bin << shift));
                    next_hi = edge > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)edge;
                    first = false;
                }
                if (bcnt <= FAST_BIN_DIRECT) {
                    // few entries in the bin: rank them directly on the whole triple
#pragma unroll
                    for (int u = 0; u < FAST_ITEMS; ++u) {
                        if (valid[u] && (int)((key[u] - lo) >> shift) == bin) {
                            const int slot = atomicAdd(&sm.gather_n, 1);
                            sm.g_key[slot] = key[u];
                            sm.g_seg[slot] = sg[u];
                            sm.g_pos[slot] = ps[u];
                        }
                    }
                    __syncthreads();
                    {
                        // four threads to an entry (bcnt <= 256 = a quarter of the block), each against every fourth
                        // of the others; the triples are compared without branches, so the loop's LDS reads do not
                        // wait for one another (with the short-circuit form an iteration took three dependent reads)
                        static_assert(4 * FAST_BIN_DIRECT <= FAST_THREADS, "four threads rank one entry");
                        const int me = min(tid >> 2, bcnt - 1);
                        const uint32_t mk = sm.g_key[me];
                        const int ms = sm.g_seg[me], mp = sm.g_pos[me];
                        int rank = 0;
                        for (int j = tid & 3; j < bcnt; j += 4) {
                            const uint32_t kj = sm.g_key[j];
                            const int sj = sm.g_seg[j], pj = sm.g_pos[j];
                            rank += (int)((kj < mk) | ((kj == mk) & ((sj > ms) | ((sj == ms) & (pj > mp)))));
                        }
                        rank += __shfl_xor(rank, 1, 64);
                        rank += __shfl_xor(rank, 2, 64);
                        if ((tid >> 2) < bcnt && (tid & 3) == 0 && rank == (int)(r - before)) {
                            sm.found_key = mk;
                            sm.found_seg = ms;
                            sm.found_pos = mp;
                        }
                    }
                    __syncthreads();
                    out.key_thr = sm.found_key;
                    out.seg_thr = sm.found_seg;
                    out.pos_thr = sm.found_pos;
                    solved = true;
                    break;
                }
                if (shift == 0) break;                            // too many equal keys at the threshold: the plain select below
                const uint32_t nlo = lo + ((uint32_t)bin << shift);
#pragma unroll
                for (int u = 0; u < FAST_ITEMS; ++u) valid[u] = valid[u] && (int)((key[u] - lo) >> shift) == bin;
                lo = nlo;
                const uint64_t top = (uint64_t)nlo + ((1ull << shift) - 1ull);
                hi_k = top < (uint64_t)hi_k ? (uint32_t)top : hi_k;
                r -= before;
            }
        }
        if (!solved) {
            // -- plain radix select by this block alone; also the bound for the next call
            used_fallback = true;
            __syncthreads();
            int64_t rank_in;
            uint32_t ties;
            const uint32_t key_thr = slow_radix(ks, c, sh, sa, seq, want, &sm, &rank_in, &ties);
            out.key_thr = key_thr;
            if (rank_in < (int64_t)ties) {                        // only the first rank_in of the equal keys survive
                slow_tie_walk(ks, c, sh, sa, seq, key_thr, rank_in, &sm);
                out.seg_thr = sm.found_seg;
                out.pos_thr = sm.found_pos;
            }
            __syncthreads();
            const int64_t above = seed_distance(k, sh.segs_per_seq, ws.fl_cap);
            const int64_t rank_b = want - above >= 1 ? want - above : 1;
            int64_t unused_r;
            uint32_t unused_t;
            const uint32_t key_b = slow_radix(ks, c, sh, sa, seq, rank_b, &sm, &unused_r, &unused_t);
            next_hi = key_b == 0xFFFFFFFFu ? key_b : key_b + 1u;
        }
    }
    if (tid == 0) {
        if (out.mode == FSEL_THRESHOLD) atomicAdd(&ws.fast_stat[used_fallback ? 1 : 0], 1ull);
        ws.fast_sel[seq] = out;
        if (thr_out) thr_out[seq] = out.mode == FSEL_NONE ? 0xFFFFFFFFu : out.key_thr;
        if (out.mode == FSEL_THRESHOLD) ws.fast_hi[seq] = next_hi;
    }
    if (!STEP) return;

    // ---- STEP: what the row mover needs: survivors per segment, the destination's segment table, a destination
    // offset per chunk of 128 entries (flagged when the chunk loses nothing) and the keep mask of the chunks that do
    // lose entries.  Entry (g, position p, key) survives iff it is not behind the last retained entry `out`.
    if (STEP) {
        if (!sa.inplace && step_total > sa.dst.cap) {             // every sequence's last block takes the same decision
            if (tid == 0) atomicOr(ws.err, ERR_CAP);
            return;
        }
        const int nsg = sh.segs_per_seq;
        // The evicted entries are among the listed ones unless the single-block select ran; they are handed over as
        // lists, so there must not be too many (nothing retained at all also takes the other route).
        const bool sparse = out.mode == FSEL_ALL || (out.mode == FSEL_THRESHOLD && !used_fallback && k <= STEP_MAX_EVICT);
        int* s_cb = s_pool;                                       // first chunk of the segment, counted inside the sequence
        uint32_t* s_fill = sm.h;                                  // fill counters of the scatter
        const int32_t cex = step_cex, ctot = step_ctot;
        uint32_t* chunk_ev = ws.step_chunk_ev + step_chunks_before;   // this sequence's chunks
        if (sparse) {
            // What the row mover gets: per chunk the number of entries it loses (a byte; almost all 0), per segment a
            // record - where its survivors start in the destination, and the indices of its evicted entries.  From
            // these a block of the row mover places its chunk itself: survivors of chunk ch of segment g start at
            // dst_start[g] + 128 ch - (evicted entries of g before the chunk).
            __syncthreads();
            if (tid < nsg) {
                s_ev[tid] = 0;
                s_cb[tid] = cex;
            }
            s_fill[tid] = 0;
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // the zeros written above are in place before any count is added
            __syncthreads();
            bool ev[FAST_ITEMS];
#pragma unroll
            for (int u = 0; u < FAST_ITEMS; ++u) {
                ev[u] = out.mode == FSEL_THRESHOLD && listed[u] && evicted_before(key[u], sg[u], ps[u], out.key_thr, out.seg_thr, out.pos_thr);
                if (ev[u]) {
                    const int sl = sg[u] - g0;
                    atomicAdd(&s_ev[sl], 1);
                    atomicAdd(&chunk_ev[s_cb[sl] + ix[u] / CMP_CHUNK], 1u);
                }
            }
            __syncthreads();
            const int my_ev = tid < nsg ? s_ev[tid] : 0;
            int32_t etot;
            const int32_t eex = block_excl_scan<int32_t>(my_ev, sm.lds32, &etot);
            int64_t ntot;
            const int64_t nex = block_excl_scan<int64_t>(tid < nsg ? (int64_t)(my_len - my_ev) + sa.reserve : 0, sm.lds64, &ntot);
            if (tid < nsg) {
                const int g = g0 + tid;
                s_off[tid] = eex;
                kept_out[g] = my_len - my_ev;
                StepSegRec* rec = ws.step_rec + g;
                if (sa.inplace) {                                 // the segment keeps its start; the row mover commits the new length
                    rec->dst_start = c.seg_start[g];
                    ws.step_len[g] = my_len - my_ev;
                } else {
                    sa.dst.seg_start[g] = step_before + nex;
                    sa.dst.seg_len[g] = my_len - my_ev;
                    rec->dst_start = step_before + nex;
                }
                rec->cnt = my_ev;
                rec->off = eex;
            }
            __syncthreads();
            int32_t* evl = ws.step_evl + (size_t)seq * STEP_MAX_EVICT;
#pragma unroll
            for (int u = 0; u < FAST_ITEMS; ++u) {
                if (ev[u]) {
                    const int sl = sg[u] - g0;
                    const int slot = (int)atomicAdd(&s_fill[sl], 1u);
                    evl[s_off[sl] + slot] = ix[u];
                    if (slot < STEP_REC_IDX) ws.step_rec[g0 + sl].idx[slot] = ix[u];
                }
            }
        } else {
            // after the single-block select (or with very many evictions) the evicted entries are not listed: one more
            // pass over the sequence leaves the keep mask and, per chunk of 128 entries, where its survivors go
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // (the zeros written earlier have landed)
            __syncthreads();
            for (int i = tid; i < ctot; i += FAST_THREADS) st_dev(&chunk_ev[i], STEP_CHUNK_DENSE);   // "look at the mask and the table"
            int64_t cursor = step_before;
            int cb = step_chunks_before;
            const int lane = lane_id(), wave = tid >> 6;
            for (int g = g0; g < g0 + nsg; ++g) {
                bool b2 = false, n2 = false;
                const SegView v = seg_view<KIND>(c, g, sh.nseg, sa, &b2, &n2);
                if (sa.inplace) cursor = v.start;                 // the segment keeps its start
                int64_t running = 0;
                for (int t0 = 0; t0 < v.len; t0 += FAST_THREADS) {   // tiles of 8 chunks
                    const int j = t0 + tid;
                    bool kf = false;
                    if (j < v.len) {
                        if (out.mode == FSEL_THRESHOLD) {
                            int pj;
                            float sj;
                            ks.entry_at(g, v, j, &pj, &sj);
                            const uint32_t kk = key_of_score(sj);
                            kf = !evicted_before(kk, g, pj, out.key_thr, out.seg_thr, out.pos_thr);
                        } else {
                            kf = out.mode == FSEL_ALL;
                        }
                        sa.keep_out[v.start + j] = kf;
                    }
                    const int wc = __popcll(__ballot(kf));
                    __syncthreads();
                    if (lane == 0) sm.h[wave] = wc;               // 16 wavefronts = 8 chunks of two
                    __syncthreads();
                    if (tid < FAST_THREADS / CMP_CHUNK) {
                        const int chl = t0 / CMP_CHUNK + tid;     // chunk of the segment
                        if (chl * CMP_CHUNK < v.len) {
                            int64_t ex = 0;
                            for (int i = 0; i < tid; ++i) ex += sm.h[2 * i] + sm.h[2 * i + 1];
                            const int here = sm.h[2 * tid] + sm.h[2 * tid + 1];
                            const int n = min(CMP_CHUNK, v.len - chl * CMP_CHUNK);
                            ws.cmp_chunk_dst[cb + chl] = (cursor + running + ex) | (here == n ? CMP_DST_FULL : 0);
                        }
                    }
                    int tile = 0;
                    for (int i = 0; i < FAST_THREADS / 64; ++i) tile += sm.h[i];
                    running += tile;
                }
                if (tid == 0) {
                    kept_out[g] = (int32_t)running;
                    if (sa.inplace) {
                        ws.step_len[g] = (int32_t)running;
                    } else {
                        sa.dst.seg_start[g] = cursor;
                        sa.dst.seg_len[g] = (int32_t)running;
                    }
                }
                cursor += running + sa.reserve;
                cb += (v.len + CMP_CHUNK - 1) / CMP_CHUNK;
            }
        }
    }
}

// keep[e] from the published triple; survivors per segment are added to kept_out (zeroed by k_fast_scan).
// PAGED: the segment's slots through its block table; an empty slot's byte is 0.
// EVICT (PAGED only; the paged decode step in one call): stage 3 of the paged layout rides along - a live slot that
// is not kept becomes empty (position -1), the live counts of its page and segment go down, and a page left without
// a live entry is marked for release (owner -2), exactly as k_pg_evict does from the mask.
template <bool PAGED, bool EVICT = false>
__global__ __launch_bounds__(FAST_THREADS) void k_fast_mask(CacheView c, const float* __restrict__ score, Shape sh,
                                                            Workspace ws, int bps, uint8_t* __restrict__ keep,
                                                            int32_t* __restrict__ kept_out, PagedArgs pg) {
    __shared__ int32_t lds32[17];
    const int tid = threadIdx.x;
    const int seg = blockIdx.x / bps, part = blockIdx.x % bps;
    const int seq = seg / sh.segs_per_seq;
    StepArgs sa{};
    sa.pg = pg;
    bool bad = false, nocap = false;
    const SegView v = seg_view<PAGED ? SCAN_PAGED : SCAN_RAGGED>(c, seg, sh.nseg, sa, &bad, &nocap);
    const int len = v.len;
    KeySource<false, PAGED ? SCAN_PAGED : SCAN_RAGGED> ks;
    ks.bt = pg.block_table;
    ks.n_pages = pg.n_pages;
    const FastSel fs = ws.fast_sel[seq];
    int n = 0;
    const bool seg_before = seg < fs.seg_thr, seg_same = seg == fs.seg_thr;
    for (int j0 = part * FAST_THREADS + tid; j0 < len; j0 += bps * FAST_THREADS * FAST_BATCH) {
        int64_t at[FAST_BATCH];
        bool bp = false;
#pragma unroll
        for (int u = 0; u < FAST_BATCH; ++u) {
            const int j = j0 + u * bps * FAST_THREADS;
            at[u] = j < len ? ks.place(v, j, &bp) : 0;
        }
        float sv[FAST_BATCH];
        int pv[FAST_BATCH];
#pragma unroll
        for (int u = 0; u < FAST_BATCH; ++u) {
            const int j = j0 + u * bps * FAST_THREADS;
            sv[u] = (j < len && fs.mode == FSEL_THRESHOLD) ? score[at[u]] : 0.f;
            pv[u] = (PAGED && j < len) ? c.pos[at[u]] : 0;
        }
#pragma unroll
        for (int u = 0; u < FAST_BATCH; ++u) {
            const int j = j0 + u * bps * FAST_THREADS;
            bool kf = false;
            if (j < len) {
                kf = fs.mode == FSEL_ALL;
                if (fs.mode == FSEL_THRESHOLD) {
                    const uint32_t key = key_of_score(sv[u]);
                    kf = key > fs.key_thr;
                    if (key == fs.key_thr) kf = seg_before || (seg_same && (PAGED ? pv[u] : c.pos[at[u]]) <= fs.pos_thr);
                }
                if (PAGED && pv[u] < 0) kf = false;
                keep[at[u]] = kf;
                n += kf;
            }
            if (EVICT) {
                // a wavefront holds 64 consecutive slots of one page here (or none: a segment's slots come in whole pages)
                const bool gone = j < len && pv[u] >= 0 && !kf;
                const int n_gone = __popcll(__ballot(gone));
                if (gone) pg.evict_pos[at[u]] = -1;
                if (n_gone && lane_id() == 0) {
                    const int page = (int)(at[u] / KVTRIM_PAGE_SIZE);
                    const int left = atomicSub(&pg.evict_page_live[page], n_gone) - n_gone;
                    atomicSub(&pg.evict_seg_live[seg], n_gone);
                    if (left <= 0) pg.evict_page_owner[page] = -2;
                }
            }
        }
    }
    n = block_sum<int32_t>(n, lds32);
    if (tid == 0 && n) atomicAdd(&kept_out[seg], n);
}

kvtrim_status launch_score_select(kvtrim_ctx* ctx, const CacheView& c, const int32_t* now, const int64_t* budget,
                                  float* score, uint8_t* keep, int32_t* kept, uint32_t* thr, int64_t evict_hint,
                                  hipStream_t st) {
    const Shape& sh = ctx->shape;
    const Workspace& ws = ctx->ws;
    // the list has to hold about 3 (k + 1) entries for k evictions, spread unevenly over its sub-lists
    if (evict_hint <= 0 || 8 * (evict_hint + 1) > (int64_t)ws.fl_cap)
        return launch_score_select_general(ctx, c, now, budget, score, keep, kept, thr, st);
    int64_t bps = c.cap / ((int64_t)sh.nseg * FAST_ENTRIES_PER_BLOCK);
    bps = bps < 1 ? 1 : (bps > 64 ? 64 : bps);
    const dim3 grid((unsigned)(sh.nseg * bps)), block(FAST_THREADS);
    { ProfScope prof(ctx, K_FAST_SCAN, st);
      hipLaunchKernelGGL((k_fast_scan<true, SCAN_RAGGED>), grid, block, 0, st, c, now, (const float*)nullptr, score, budget, sh, ws, (int)bps, kept, thr, StepArgs()); }
    { ProfScope prof(ctx, K_FAST_MASK, st);
      hipLaunchKernelGGL(k_fast_mask<false>, grid, block, 0, st, c, (const float*)score, sh, ws, (int)bps, keep, kept, PagedArgs()); }
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

// The decode-step form over a paged cache (`pool`: the page pool's arrays, cap = its slots): the same two kernels,
// walking every segment's slots through its block table.  The caller has checked that the hint fits the list.
kvtrim_status launch_score_select_paged(kvtrim_ctx* ctx, const CacheView& pool, const PagedArgs& pg, const int32_t* now,
                                        const int64_t* budget, float* score, uint8_t* keep, int32_t* kept, uint32_t* thr,
                                        hipStream_t st, bool evict) {
    const Shape& sh = ctx->shape;
    const Workspace& ws = ctx->ws;
    int64_t bps = pool.cap / ((int64_t)sh.nseg * FAST_ENTRIES_PER_BLOCK);
    bps = bps < 1 ? 1 : (bps > 64 ? 64 : bps);
    const dim3 grid((unsigned)(sh.nseg * bps)), block(FAST_THREADS);
    const bool plan = pg.plan_layer_end > pg.plan_layer_begin;
    const dim3 scan_grid((unsigned)(sh.nseg * bps + (plan ? PG_TABLE_BLOCKS : 0)));
    StepArgs sa{};
    sa.pg = pg;
    { ProfScope prof(ctx, K_FAST_SCAN, st);
      hipLaunchKernelGGL((k_fast_scan<true, SCAN_PAGED>), scan_grid, block, 0, st, pool, now, (const float*)nullptr, score, budget, sh, ws, (int)bps, kept, thr, sa); }
    { ProfScope prof(ctx, K_FAST_MASK, st);
      if (evict)
          hipLaunchKernelGGL((k_fast_mask<true, true>), grid, block, 0, st, pool, (const float*)score, sh, ws, (int)bps, keep, kept, pg);
      else
          hipLaunchKernelGGL((k_fast_mask<true, false>), grid, block, 0, st, pool, (const float*)score, sh, ws, (int)bps, keep, kept, pg); }
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

// The scoring kernel of the one-call decode step (the caller has checked that the step fits its limits).
kvtrim_status launch_step_scan(kvtrim_ctx* ctx, const CacheView& c, const int32_t* now, const int64_t* budget, float* score,
                               int32_t* kept, uint32_t* thr, const StepArgs& sa, hipStream_t st) {
    const Shape& sh = ctx->shape;
    int64_t bps = c.cap / ((int64_t)sh.nseg * FAST_ENTRIES_PER_BLOCK);
    bps = bps < 1 ? 1 : (bps > 64 ? 64 : bps);
    ProfScope prof(ctx, K_FAST_SCAN, st);
    hipLaunchKernelGGL((k_fast_scan<true, SCAN_STEP>), dim3((unsigned)(sh.nseg * bps + sh.nseg)), dim3(FAST_THREADS), 0, st, c, now,
                       (const float*)nullptr, score, budget, sh, ctx->ws, (int)bps, kept, thr, sa);
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

}  // namespace kvtrim
