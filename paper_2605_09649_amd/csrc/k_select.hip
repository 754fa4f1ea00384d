// Stage 2: one global top-B selection per sequence (Sec. 4.2, eviction rule) - the general form, for any
// number of evictions (the decode-step form, which looks only for the few lowest entries, is in k_fastsel.hip).
//
// Exact selection by a three-pass most-significant-digit radix select (11 + 11 + 10 bits)
// on the order-preserving uint32 image of the fp32 score.  Each pass builds per-block
// histograms in LDS and merges them with device-scope atomics into replicated global histograms.
// Every block of pass p + 1 finds the digit of pass p itself, by walking the merged histogram of
// pass p in its prologue; only the last pass uses "last block done" (per sequence: the last block
// that holds entries of the sequence fixes the final digit, the threshold key and the tie quota).
// The first pass can compute the score on the fly (stage 1 fused: it reads log beta and the
// position instead of a score array and writes the score out as it goes).
// Entries above the threshold are kept; entries equal to it are kept in storage order
// (segment ascending, position ascending = layer, head, position) until the budget is
// met.  When every entry equal to the threshold fits (the usual case) the mask is a plain
// comparison; otherwise an ordered count of ties per chunk and an exclusive scan over the
// chunks rank them.
#include "kvtrim_device.h"

namespace kvtrim {

constexpr int SEL_THREADS = 256;      // mask kernel: one chunk per block, 8 entries per thread
constexpr int CNT_THREADS = 1024;
constexpr int HIST_THREADS = 1024;    // histogram passes: few fat blocks, so that few device-scope
constexpr int HIST_BLOCKS = HIST_BLOCKS_MAX;   // atomics meet on one address when the LDS histograms are merged
                                      // (the merged histogram is also kept in HIST_REPLICAS copies)
constexpr int PLAN_ZERO_BLOCKS = 8;   // extra blocks of the plan kernel that clear the histograms

__global__ __launch_bounds__(1024) void k_sel_plan(CacheView c, Shape sh, const int64_t* __restrict__ budget,
                                                   Workspace ws, int32_t* __restrict__ kept_out,
                                                   uint32_t* __restrict__ thr_out, int hist_blocks) {
    if (blockIdx.x > 0) {                      // clear the (replicated) histograms of the three passes
        const int64_t n = (int64_t)3 * HIST_REPLICAS * sh.n_seq * RADIX_BINS;   // 65536 sequences: 3.2 G words
        for (int64_t i = (blockIdx.x - 1) * blockDim.x + threadIdx.x; i < n; i += (gridDim.x - 1) * blockDim.x)
            ws.hist[i] = 0;
        return;
    }
    for (int i = threadIdx.x; i < DONE_WORDS; i += blockDim.x) ws.done[i] = 0;
    for (int g = threadIdx.x; g < sh.nseg; g += blockDim.x) kept_out[g] = 0;
    const int total = build_chunk_table(c.seg_len, c.seg_start, sh.nseg, [](int) { return true; }, SEL_CHUNK, c.cap,
                                        ws.sel_chunk_prefix, ws.sel_desc, ws.max_sel_chunks, ws.sel_entry_prefix, ws.err);
    if ((int)threadIdx.x < hist_blocks) {                         // chunk range of every histogram block
        const int cpb = (total + hist_blocks - 1) / hist_blocks;
        const int c0 = min(total, (int)threadIdx.x * cpb), c1 = min(total, c0 + cpb);
        int4 r = make_int4(c0, c1, 0, -1);
        if (c0 < c1) {
            r.z = ws.sel_desc[c0].seg / sh.segs_per_seq;
            r.w = ws.sel_desc[c1 - 1].seg / sh.segs_per_seq;
        }
        ws.sel_blk[threadIdx.x] = r;
    }
    for (int seq = threadIdx.x; seq < sh.n_seq; seq += blockDim.x) {
        const int64_t n = ws.sel_entry_prefix[(seq + 1) * sh.segs_per_seq] - ws.sel_entry_prefix[seq * sh.segs_per_seq];
        int64_t b = budget[seq];
        if (b < 0) b = 0;
        SelState st;
        st.prefix = 0;
        st.thr_key = 0xFFFFFFFFu;
        st.count = n;
        st.want = b < n ? b : n;
        st.rank = st.want;
        st.tie_quota = 0;
        st.keep_none = st.want == 0;
        st.need_rank = 0;
        ws.sel[seq] = st;                                         // final slot (what the count and mask kernels read)
        ws.sel[sh.n_seq + seq] = st;                              // state before the first digit
        ws.seq_done[seq] = 0;
        if (thr_out) thr_out[seq] = 0xFFFFFFFFu;                  // stands for a sequence that keeps nothing
    }
}

// One digit of the threshold key: walks the merged histogram of pass P (the sum of its replicas) of sequence
// `seq` from the top bin down to the bin that holds the entry of rank st.rank (1-based, descending key order)
// and returns the state with that digit appended.  Called by all threads of a 1024-thread block; `cnt_out`
// gets the population of the chosen bin.
template <int P>
__device__ __forceinline__ SelState next_digit(const uint32_t* __restrict__ hist_pass, int n_seq, int seq, SelState st,
                                               int64_t* lds64, SelState* s_state, uint32_t* cnt_out) {
    constexpr int NB = P == 2 ? 1024 : 2048;
    constexpr int PER = NB / 1024;                                // bins per thread (1 or 2), thread 0 owns the highest bins
    const int tid = threadIdx.x;
    uint32_t cnt[PER];
    int64_t mine = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int bin = NB - 1 - (tid * PER + i);
        uint32_t v = 0;
#pragma unroll
        for (int r = 0; r < HIST_REPLICAS; ++r) v += hist_pass[((size_t)r * n_seq + seq) * RADIX_BINS + bin];
        cnt[i] = v;
        mine += v;
    }
    int64_t tot;
    int64_t above = block_excl_scan<int64_t>(mine, lds64, &tot);
    if (above < st.rank && st.rank <= above + mine) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            if (st.rank <= above + cnt[i]) {
                const uint32_t bin = NB - 1 - (tid * PER + i);
                const int bits = P == 2 ? RADIX_BITS2 : (P == 1 ? RADIX_BITS1 : RADIX_BITS0);
                SelState o = st;
                o.prefix = (st.prefix << bits) | bin;
                o.rank = st.rank - above;
                *s_state = o;
                *cnt_out = cnt[i];
                break;
            }
            above += cnt[i];
        }
    }
    __syncthreads();
    const SelState o = *s_state;
    __syncthreads();                                              // s_state may be written again by the next call
    return o;
}

// Histogram of the next digit over the entries whose higher digits equal the prefix found so
// far.  A block takes a contiguous range of chunks and walks it as a flat range of entry slots
// (every load independent of the previous one); its LDS histogram is flushed per sequence.
// Only one thread per block issues the device-scope fence (a fence per wavefront costs an L2
// write-back each and dominated the pass).
// SHIFT = log2 of the chunk size of the table (2048-entry chunks of a ragged cache, 128-slot pages of a
// paged one); PAGED: a slot counts only if its position is not negative.
// SCORE (first pass of a ragged cache only): the score is computed here from log beta and the position (Eq.
// global_score in log domain, exactly as k_score does) and written to score_w; `score` is not read.
// VEC (ragged caches whose arrays are all 16-byte aligned): a chunk is walked in ALIGNED groups of four entries -
// 16-byte loads, four times the bytes in flight of the entry-by-entry walk.  A group may begin before the chunk or
// end behind it (segments start anywhere): what lies outside [first, first + n) is loaded and ignored; the one group
// that would reach past the end of the arrays is read entry by entry.
struct Quad {
    int64_t a;        // first entry of the aligned group
    int lo, hi;       // its entries a + lo .. a + hi - 1 belong to the chunk (lo == hi: none)
    bool whole;       // all four can be loaded (the group ends inside the arrays)
};
__device__ __forceinline__ Quad quad_of(const ChunkDesc& d, int q, int64_t cap) {
    Quad r;
    r.a = (d.first & ~(int64_t)3) + 4 * (int64_t)q;
    const int64_t end = d.first + d.n;
    r.lo = (int)(d.first > r.a ? d.first - r.a : 0);
    const int64_t h = end - r.a;
    r.hi = h < r.lo ? r.lo : (h < 4 ? (int)h : 4);
    r.whole = r.a + 4 <= cap;
    return r;
}
template <typename T>
__device__ __forceinline__ void load_quad(const T* __restrict__ base, const Quad& q, T (&v)[4]) {
    struct alignas(16) T4 { T x, y, z, w; };
    // (a group with nothing of the chunk, or reaching past the arrays, loads the arrays' first four entries instead)
    const T4 x = *reinterpret_cast<const T4*>(base + ((q.whole && q.lo < q.hi) ? q.a : 0));
    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
}
template <typename T>
__device__ __forceinline__ void reload_quad_tail(const T* __restrict__ base, const Quad& q, T (&v)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (i >= q.lo && i < q.hi) v[i] = base[q.a + i];
}

template <int PASS, int SHIFT, bool PAGED, bool SCORE = false>
__global__ __launch_bounds__(HIST_THREADS, 8) void k_sel_hist(const float* __restrict__ score, Shape sh,
                                                           Workspace ws, SelTables tb,
                                                           uint32_t* __restrict__ thr_out, CacheView c,
                                                           const int32_t* __restrict__ now,
                                                           float* __restrict__ score_w, bool vec) {
    static_assert(!SCORE || (PASS == 0 && !PAGED), "the score is fused into the first pass over a ragged cache only");
    constexpr int NB = PASS == 2 ? 1024 : 2048;
    constexpr int HIST_TILE = 64;
    __shared__ uint32_t h[NB];
    __shared__ ChunkDesc s_desc[HIST_TILE];
    __shared__ int64_t lds64[17];
    __shared__ SelState s_state;
    __shared__ uint32_t s_cnt;
    __shared__ int is_last;
    const int tid = threadIdx.x;
    const int4 rng = ws.sel_blk[blockIdx.x];
    const int c0 = rng.x, c1 = rng.y;
    uint32_t* hist_pass = ws.hist + (size_t)PASS * HIST_REPLICAS * sh.n_seq * RADIX_BINS;
    uint32_t* hist = hist_pass + (size_t)(blockIdx.x % HIST_REPLICAS) * sh.n_seq * RADIX_BINS;

    if (c0 < c1) {
        for (int i = tid; i < NB; i += HIST_THREADS) h[i] = 0;
        const int seq_lo = rng.z, seq_hi = rng.w;
        for (int seq = seq_lo; seq <= seq_hi; ++seq) {
            const int a = max(c0, tb.prefix[seq * sh.segs_per_seq]);
            const int b = min(c1, tb.prefix[(seq + 1) * sh.segs_per_seq]);
            if (a >= b) continue;
            if (!SCORE && ws.sel[seq].keep_none) continue;        // (with SCORE the pass still has the scores to write)
            const int t1 = SCORE ? now[seq] + 1 : 0;
            // The digits fixed so far: every block derives them itself from the previous pass's merged histogram
            // (a few microseconds of L2 reads, the same for all blocks) instead of waiting for that pass's last
            // block to do it, which put "last block done" detection and the walk on the critical path of every pass.
            // (slots of ws.sel: [0] final, [1] after the plan, [2] after the first digit, [3] after the second)
            SelState st = ws.sel[(size_t)(PASS > 1 ? PASS : 1) * sh.n_seq + seq];
            if (PASS > 0) {
                uint32_t unused;
                st = next_digit<(PASS > 0 ? PASS - 1 : 0)>(ws.hist + (size_t)(PASS - 1) * HIST_REPLICAS * sh.n_seq * RADIX_BINS,
                                                          sh.n_seq, seq, st, lds64, &s_state, &unused);
            }
            if (PASS > 0 && tid == 0) ws.sel[(size_t)(PASS + 1) * sh.n_seq + seq] = st;   // the same value from every block
            const uint32_t prefix = st.prefix;
            // the descriptors of a tile of chunks go through LDS so that the score loads of a
            // thread do not depend on anything loaded inside the loop and are all in flight at once
            for (int t0 = a; t0 < b; t0 += HIST_TILE) {
                const int nt = min(HIST_TILE, b - t0);
                __syncthreads();
                if (tid < nt) s_desc[tid] = tb.desc[t0 + tid];
                __syncthreads();
                if (PAGED) {
                    // pages are whole, 16-byte aligned chunks: four slots per load
#pragma unroll 4
                    for (int s4 = tid; s4 < (nt << (SHIFT - 2)); s4 += HIST_THREADS) {
                        const ChunkDesc d = s_desc[s4 >> (SHIFT - 2)];
                        const int64_t e = d.first + ((s4 & ((1 << (SHIFT - 2)) - 1)) << 2);
                        const float4 sc = *reinterpret_cast<const float4*>(score + e);
                        const float v[4] = {sc.x, sc.y, sc.z, sc.w};
                        int bin[4];
                        bool hit[4];
                        bool any = false;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            hit[i] = digit_of<PASS>(key_of_score(v[i]), prefix, &bin[i]);
                            any |= hit[i];
                        }
                        if (any) {                                // the positions are looked at only where a prefix matches
                            const int4 ps = *reinterpret_cast<const int4*>(tb.pos + e);
                            const int p[4] = {ps.x, ps.y, ps.z, ps.w};
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                if (hit[i] && p[i] >= 0) atomicAdd(&h[bin[i]], 1u);
                        }
                    }
                } else if (vec) {
                    constexpr int QPC = (1 << (SHIFT - 2)) + 1;   // aligned groups of four that can overlap a chunk
                    constexpr int U = SCORE ? 2 : 4;              // groups a thread has in flight
                    for (int q0 = tid; q0 < nt * QPC; q0 += HIST_THREADS * U) {
                        Quad qd[U];
                        float sv[U][4];
                        int pv[U][4];
                        float lbv[U][4], ltv[U][4];
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            const int qi = q0 + u * HIST_THREADS;
                            const int cidx = qi < nt * QPC ? qi / QPC : 0;
                            ChunkDesc d = s_desc[cidx];
                            if (qi >= nt * QPC) d.n = 0;
                            qd[u] = quad_of(d, qi - cidx * QPC, c.cap);
                            if (SCORE) {
                                load_quad(c.pos, qd[u], pv[u]);
                                load_quad(c.log_beta, qd[u], lbv[u]);
                                if (c.log_tail) load_quad(c.log_tail, qd[u], ltv[u]);
                            } else {
                                load_quad(score, qd[u], sv[u]);
                            }
                        }
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            const Quad& q = qd[u];
                            if (q.lo >= q.hi) continue;
                            if (!q.whole) {                       // (once per array at most)
                                if (SCORE) {
                                    reload_quad_tail(c.pos, q, pv[u]);
                                    reload_quad_tail(c.log_beta, q, lbv[u]);
                                    if (c.log_tail) reload_quad_tail(c.log_tail, q, ltv[u]);
                                } else {
                                    reload_quad_tail(score, q, sv[u]);
                                }
                            }
                            if (SCORE) {
#pragma unroll
                                for (int i = 0; i < 4; ++i) {
                                    const float dt = (float)(t1 - pv[u][i]);
                                    sv[u][i] = c.log_tail ? __fmaf_rn(dt, lbv[u][i], ltv[u][i]) : __fmul_rn(dt, lbv[u][i]);
                                }
                                if (q.whole && q.lo == 0 && q.hi == 4) {
                                    *reinterpret_cast<float4*>(score_w + q.a) = make_float4(sv[u][0], sv[u][1], sv[u][2], sv[u][3]);
                                } else {
#pragma unroll
                                    for (int i = 0; i < 4; ++i)
                                        if (i >= q.lo && i < q.hi) score_w[q.a + i] = sv[u][i];
                                }
                            }
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                int bin;
                                if (i >= q.lo && i < q.hi && digit_of<PASS>(key_of_score(sv[u][i]), prefix, &bin)) atomicAdd(&h[bin], 1u);
                            }
                        }
                    }
                } else {
#pragma unroll 8
                    for (int slot = tid; slot < (nt << SHIFT); slot += HIST_THREADS) {
                        const ChunkDesc d = s_desc[slot >> SHIFT];
                        const int j = slot & ((1 << SHIFT) - 1);
                        if (j < d.n) {
                            int bin;
                            float sv;
                            if (SCORE) {
                                const int64_t e = d.first + j;
                                const float dt = (float)(t1 - c.pos[e]);
                                sv = c.log_tail ? __fmaf_rn(dt, c.log_beta[e], c.log_tail[e]) : __fmul_rn(dt, c.log_beta[e]);
                                score_w[e] = sv;
                            } else {
                                sv = score[d.first + j];
                            }
                            if (digit_of<PASS>(key_of_score(sv), prefix, &bin)) atomicAdd(&h[bin], 1u);
                        }
                    }
                }
            }
            __syncthreads();
            for (int i = tid; i < NB; i += HIST_THREADS) {
                const uint32_t v = h[i];
                if (v) {
                    atomicAdd(&hist[(size_t)seq * RADIX_BINS + i], v);
                    h[i] = 0;
                }
            }
            if (PASS < 2) continue;                               // the next pass finds this pass's digit itself

            // Last pass: the block that is last to add its counts for THIS sequence takes the final digit, hence
            // the threshold key, how many of the entries equal to it survive, and whether those have to be ranked
            // in order.  (One "last block" per sequence, so the sequences of a batch finish side by side.)
            __syncthreads();
            if (tid == 0) {
                __threadfence();
                const int p0 = tb.prefix[seq * sh.segs_per_seq], p1 = tb.prefix[(seq + 1) * sh.segs_per_seq];
                const int cpb = (tb.prefix[sh.nseg] + (int)gridDim.x - 1) / (int)gridDim.x;   // chunks per block, as in the plan
                const unsigned nblk = (unsigned)((p1 - 1) / cpb - p0 / cpb + 1);              // blocks that meet [p0, p1)
                is_last = atomicAdd(&ws.seq_done[seq], 1u) == nblk - 1;
            }
            __syncthreads();
            if (!is_last) continue;
            __threadfence();
            SelState fin = next_digit<2>(hist_pass, sh.n_seq, seq, st, lds64, &s_state, &s_cnt);
            if (tid == 0) {
                fin.thr_key = fin.prefix;
                fin.tie_quota = fin.rank;
                fin.need_rank = fin.rank < (int64_t)s_cnt;        // fewer survive than tie at the threshold
                if (fin.need_rank) atomicOr((int*)&ws.done[127], 1);
                if (thr_out) thr_out[seq] = fin.thr_key;
                ws.sel[seq] = fin;
            }
            // The bound the decode-step selection starts from at its next call (k_fastsel.hip): a key with about
            // 2 (k + 1) retained entries between it and the threshold (seed_distance).  The entry of
            // that rank is walked down the three histograms as far as it shares the threshold's digits (below that
            // the histograms count other buckets); where it leaves them, the upper edge of its bucket is taken.
            if (ws.fl_cap > 0 && st.count > st.want) {
                SelState sb = ws.sel[(size_t)sh.n_seq + seq];     // state before the first digit
                const int64_t above = seed_distance(st.count - st.want, sh.segs_per_seq, ws.fl_cap);
                sb.rank = st.want - above >= 1 ? st.want - above : 1;
                uint32_t unused;
                uint64_t seed;
                sb = next_digit<0>(ws.hist, sh.n_seq, seq, sb, lds64, &s_state, &unused);
                if (sb.prefix != (fin.prefix >> 21)) {
                    seed = ((uint64_t)sb.prefix + 1) << 21;
                } else {
                    sb = next_digit<1>(ws.hist + (size_t)1 * HIST_REPLICAS * sh.n_seq * RADIX_BINS, sh.n_seq, seq, sb, lds64, &s_state, &unused);
                    if (sb.prefix != (fin.prefix >> 10)) {
                        seed = ((uint64_t)sb.prefix + 1) << 10;
                    } else {
                        sb = next_digit<2>(hist_pass, sh.n_seq, seq, sb, lds64, &s_state, &unused);
                        seed = (uint64_t)sb.prefix + 1;
                    }
                }
                if (tid == 0) ws.fast_hi[seq] = seed > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)seed;
            }
        }
    }
}

// Only runs when, for some sequence, the entries equal to the threshold do not all fit.  Per
// chunk of such a sequence: entries above the threshold (credited to the segment) and entries
// equal to it; the last block then turns the per-chunk tie counts into exclusive prefixes per
// sequence and credits the ties that fit into the quota to their segments.
__global__ __launch_bounds__(CNT_THREADS) void k_sel_count(const float* __restrict__ score, Shape sh,
                                                           Workspace ws, SelTables tb,
                                                           int32_t* __restrict__ kept_out) {
    __shared__ int64_t lds64[17];
    __shared__ int32_t lds32[17];
    __shared__ int s_list[CNT_THREADS];
    __shared__ int s_n, is_last;
    if (ws.done[127] == 0) return;                                // uniform over the grid
    const int tid = threadIdx.x;
    for_each_ranked_seq(ws.sel, sh.n_seq, s_list, &s_n, [&](int seq) {
        const uint32_t thr_key = ws.sel[seq].thr_key;
        const int cb = tb.prefix[seq * sh.segs_per_seq], ce = tb.prefix[(seq + 1) * sh.segs_per_seq];
        for (int ch = cb + blockIdx.x; ch < ce; ch += gridDim.x) {
            const ChunkDesc d = tb.desc[ch];
            int gt = 0, eq = 0;
            for (int j = tid; j < d.n; j += CNT_THREADS) {
                const uint32_t key = key_of_score(score[d.first + j]);
                gt += key > thr_key;
                eq += key == thr_key;
            }
            gt = block_sum<int32_t>(gt, lds32);
            eq = block_sum<int32_t>(eq, lds32);
            if (tid == 0) {
                if (gt) atomicAdd(&kept_out[d.seg], gt);
                ws.chunk_eq[ch] = eq;
            }
        }
    });
    __syncthreads();
    if (tid == 0) is_last = arrive_last(ws.done + 32 * 3);
    __syncthreads();
    if (!is_last) return;
    __threadfence();

    for_each_ranked_seq(ws.sel, sh.n_seq, s_list, &s_n, [&](int seq) {
        const int cb = tb.prefix[seq * sh.segs_per_seq];
        const int ce = tb.prefix[(seq + 1) * sh.segs_per_seq];
        const int64_t quota = ws.sel[seq].tie_quota;
        int64_t running = 0;
        for (int base = cb; base < ce; base += CNT_THREADS) {
            const int cc = base + tid;
            int64_t v = cc < ce ? (int64_t)__hip_atomic_load(&ws.chunk_eq[cc], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
            int64_t tot;
            int64_t ex = block_excl_scan<int64_t>(v, lds64, &tot);
            if (cc < ce) {
                const int64_t tbase = running + ex;
                ws.chunk_tie_base[cc] = tbase;
                if (v > 0 && tbase < quota) {
                    const int64_t take = min(v, quota - tbase);
                    atomicAdd(&kept_out[tb.desc[cc].seg], (int32_t)take);
                }
            }
            running += tot;
        }
    });
}

// keep[e] = key > thr, or key == thr and the entry is among the first `quota` ties of its
// sequence in (segment, position) order.  When every tie fits (the usual case) the kernel also
// counts the survivors of its chunk into kept_out; otherwise the count kernel has done that.
// A segment is stored in position order, so the ties are ranked by storage order (exclusive tie
// counts per chunk).
__global__ __launch_bounds__(SEL_THREADS) void k_sel_mask(const float* __restrict__ score, Shape sh,
                                                          Workspace ws, SelTables tb, uint8_t* __restrict__ keep,
                                                          int32_t* __restrict__ kept_out) {
    __shared__ int32_t lds32[17];
    const int tid = threadIdx.x;
    const int total = tb.prefix[sh.nseg];
    const int ch = blockIdx.x;
    if (ch >= total) return;
    const ChunkDesc d = tb.desc[ch];
    const SelState st = ws.sel[d.seg / sh.segs_per_seq];
    const float* s = score + d.first;
    uint8_t* kp = keep + d.first;
    if (st.keep_none) {
        for (int j = tid; j < d.n; j += SEL_THREADS) kp[j] = 0;
        return;
    }
    if (!st.need_rank) {                                          // every tie survives
        int n = 0;
#pragma unroll 8
        for (int j = tid; j < d.n; j += SEL_THREADS) {
            const bool k = key_of_score(s[j]) >= st.thr_key;
            kp[j] = k;
            n += k;
        }
        n = block_sum<int32_t>(n, lds32);
        if (tid == 0 && n) atomicAdd(&kept_out[d.seg], n);
        return;
    }
    const int64_t tbase = ws.chunk_tie_base[ch];
    const int eq_total = ws.chunk_eq[ch];
    if (eq_total == 0 || tbase + eq_total <= st.tie_quota) {     // every tie of this chunk survives
        for (int j = tid; j < d.n; j += SEL_THREADS) kp[j] = key_of_score(s[j]) >= st.thr_key;
        return;
    }
    if (tbase >= st.tie_quota) {                                  // no tie of this chunk survives
        for (int j = tid; j < d.n; j += SEL_THREADS) kp[j] = key_of_score(s[j]) > st.thr_key;
        return;
    }
    // the quota runs out inside this chunk: rank the ties in order
    int64_t running = tbase;
    for (int base = 0; base < d.n; base += SEL_THREADS) {         // uniform trip count
        const int j = base + tid;
        uint32_t key = 0;
        int is_eq = 0;
        if (j < d.n) {
            key = key_of_score(s[j]);
            is_eq = key == st.thr_key;
        }
        int32_t tot;
        int32_t ex = block_excl_scan<int32_t>(is_eq, lds32, &tot);
        if (j < d.n) kp[j] = key > st.thr_key || (is_eq && running + ex < st.tie_quota);
        running += tot;
    }
}

// The three histogram passes over a paged cache whose chunk table (one chunk per page) is in tb;
// the plan, the tie count and the mask of the paged layout live in k_paged.hip.
void launch_select_passes_paged(kvtrim_ctx* ctx, const float* score, const SelTables& tb, int hist_blocks,
                                int pass, uint32_t* thr, hipStream_t st) {
    const Shape& sh = ctx->shape;
    const Workspace& ws = ctx->ws;
    if (pass == 0) {
        ProfScope prof(ctx, K_SEL_HIST0, st);
        hipLaunchKernelGGL((k_sel_hist<0, 7, true>), dim3(hist_blocks), dim3(HIST_THREADS), 0, st, score, sh, ws, tb, thr, CacheView(), nullptr, nullptr, false);
    } else if (pass == 1) {
        ProfScope prof(ctx, K_SEL_HIST1, st);
        hipLaunchKernelGGL((k_sel_hist<1, 7, true>), dim3(hist_blocks), dim3(HIST_THREADS), 0, st, score, sh, ws, tb, thr, CacheView(), nullptr, nullptr, false);
    } else {
        ProfScope prof(ctx, K_SEL_HIST2, st);
        hipLaunchKernelGGL((k_sel_hist<2, 7, true>), dim3(hist_blocks), dim3(HIST_THREADS), 0, st, score, sh, ws, tb, thr, CacheView(), nullptr, nullptr, false);
    }
}

// now != NULL: stage 1 is fused into the first pass, which writes the scores to score_w.
static kvtrim_status launch_select_impl(kvtrim_ctx* ctx, const CacheView& c, const float* score, const int32_t* now,
                                        float* score_w, const int64_t* budget, uint8_t* keep, int32_t* kept,
                                        uint32_t* thr, hipStream_t st) {
    const Shape& sh = ctx->shape;
    const Workspace& ws = ctx->ws;
    const int64_t max_chunks = c.cap / SEL_CHUNK + sh.nseg;      // bound on the chunk count
    const int n_chunk_blocks = (int)max_chunks;
    const int hist_blocks = (int)(max_chunks < HIST_BLOCKS ? (max_chunks < 1 ? 1 : max_chunks) : HIST_BLOCKS);
    SelTables tb;
    tb.desc = ws.sel_desc;
    tb.prefix = ws.sel_chunk_prefix;
    tb.pos = nullptr;
    // 16-byte loads need every array they touch aligned (and at least one group of four entries)
    const bool vec = c.cap >= 4 && ((((uintptr_t)score) | ((uintptr_t)score_w) | ((uintptr_t)c.pos) | ((uintptr_t)c.log_beta) |
                                     ((uintptr_t)c.log_tail)) & 15) == 0;
    { ProfScope prof(ctx, K_SEL_PLAN, st);
      hipLaunchKernelGGL(k_sel_plan, dim3(1 + PLAN_ZERO_BLOCKS), dim3(1024), 0, st, c, sh, budget, ws, kept, thr, hist_blocks); }
    { ProfScope prof(ctx, K_SEL_HIST0, st);
      if (now)
          hipLaunchKernelGGL((k_sel_hist<0, SEL_SHIFT, false, true>), dim3(hist_blocks), dim3(HIST_THREADS), 0, st, (const float*)nullptr, sh, ws, tb, thr, c, now, score_w, vec);
      else
          hipLaunchKernelGGL((k_sel_hist<0, SEL_SHIFT, false>), dim3(hist_blocks), dim3(HIST_THREADS), 0, st, score, sh, ws, tb, thr, c, nullptr, nullptr, vec); }
    { ProfScope prof(ctx, K_SEL_HIST1, st);
      hipLaunchKernelGGL((k_sel_hist<1, SEL_SHIFT, false>), dim3(hist_blocks), dim3(HIST_THREADS), 0, st, score, sh, ws, tb, thr, c, nullptr, nullptr, vec); }
    { ProfScope prof(ctx, K_SEL_HIST2, st);
      hipLaunchKernelGGL((k_sel_hist<2, SEL_SHIFT, false>), dim3(hist_blocks), dim3(HIST_THREADS), 0, st, score, sh, ws, tb, thr, c, nullptr, nullptr, vec); }
    { ProfScope prof(ctx, K_SEL_COUNT, st);
      hipLaunchKernelGGL(k_sel_count, dim3(n_chunk_blocks < 256 ? n_chunk_blocks : 256), dim3(CNT_THREADS), 0, st, score, sh, ws, tb, kept); }
    { ProfScope prof(ctx, K_SEL_MASK, st);
      hipLaunchKernelGGL(k_sel_mask, dim3(n_chunk_blocks), dim3(SEL_THREADS), 0, st, score, sh, ws, tb, keep, kept); }
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

kvtrim_status launch_select(kvtrim_ctx* ctx, const CacheView& c, const float* score, const int64_t* budget,
                            uint8_t* keep, int32_t* kept, uint32_t* thr, hipStream_t st) {
    return launch_select_impl(ctx, c, score, nullptr, nullptr, budget, keep, kept, thr, st);
}

kvtrim_status launch_score_select_general(kvtrim_ctx* ctx, const CacheView& c, const int32_t* now, const int64_t* budget,
                                          float* score, uint8_t* keep, int32_t* kept, uint32_t* thr, hipStream_t st) {
    return launch_select_impl(ctx, c, score, now, score, budget, keep, kept, thr, st);
}

}  // namespace kvtrim
