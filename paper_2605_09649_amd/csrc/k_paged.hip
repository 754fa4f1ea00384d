// Paged variant (the layout of Sec. 4.2 "Implementation details"): fixed-size pages, a block
// table per (sequence, layer, KV head) segment, eviction that frees slots and moves no K/V.
//
// The selection and the attention reuse the kernels of the ragged path: a page is a chunk of
// KVTRIM_PAGE_SIZE slots whose descriptor {first slot, size, segment} comes from the block tables,
// and a slot takes part only if its position is not negative.  This file holds what is specific
// to pages: building them from a ragged cache, appending into free slots, the chunk tables, the
// tie rule by position (a segment's slots are in no particular order), eviction and the
// bookkeeping of free pages.
#include "kvtrim_paged_device.h"

namespace kvtrim {

// ---------------------------------------------------------------------------------------------
// Build: the page-aligned compaction has written the survivors of segment g to the slots
// [seg_start[g], seg_start[g] + seg_len[g]) with seg_start a multiple of the page size.  Blocks
// [0, nseg) set up the segment's pages, the remaining blocks the free pages.
__global__ __launch_bounds__(256) void k_pg_init(PagedView pc, Shape sh, Workspace ws) {
    if (__hip_atomic_load(ws.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
    const int tid = threadIdx.x;
    const int last = sh.nseg - 1;
    const int used = (int)((ws.pg_seg_start[last] + ((int64_t)ws.pg_seg_len[last] + P - 1) / P * P) / P);
    if ((int)blockIdx.x < sh.nseg) {
        const int g = blockIdx.x;
        const int len = ws.pg_seg_len[g];
        const int first = (int)(ws.pg_seg_start[g] / P);
        const int npg = (len + P - 1) / P;
        if (npg > pc.max_pps || first + npg > pc.n_pages) {          // uniform over the block
            if (tid == 0) {
                atomicOr(ws.err, ERR_CAP);
                pc.seg_pages[g] = 0;
                pc.seg_live[g] = 0;
            }
            return;
        }
        for (int i = tid; i < npg; i += 256) {
            pc.block_table[(int64_t)g * pc.max_pps + i] = first + i;
            pc.page_owner[first + i] = g;
            pc.page_live[first + i] = min(P, len - i * P);
        }
        if (npg > 0)                                                 // empty tail of the last page
            for (int j = len - (npg - 1) * P + tid; j < P; j += 256) pc.pos[(int64_t)(first + npg - 1) * P + j] = -1;
        if (tid == 0) {
            pc.seg_pages[g] = npg;
            pc.seg_live[g] = len;
        }
        return;
    }
    const int nfree = pc.n_pages - used;
    const int fb = blockIdx.x - sh.nseg, nfb = gridDim.x - sh.nseg;
    if (fb == 0 && tid == 0) *pc.n_free = nfree;
    for (int i = fb; i < nfree; i += nfb) {                          // page used + i; popped in ascending order
        const int page = used + i;
        if (tid == 0) {
            pc.page_owner[page] = -1;
            pc.page_live[page] = 0;
            pc.free_list[nfree - 1 - i] = page;
        }
        if (tid < P) pc.pos[(int64_t)page * P + tid] = -1;
    }
}

// ---------------------------------------------------------------------------------------------
// Append: one wavefront per segment.
__global__ __launch_bounds__(256) void k_pg_append(PagedView pc, const uint16_t* __restrict__ k_new,
                                                   const uint16_t* __restrict__ v_new,
                                                   const float* __restrict__ lb_new, const float* __restrict__ lt_new,
                                                   const int32_t* __restrict__ pos_new, int nseg, int head_dim,
                                                   int32_t* err) {
    const int lane = lane_id();
    const int g = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (g >= nseg) return;                                           // uniform over the wavefront
    if (pos_new[g] < 0) return;                                      // padding: this segment brings no token
    const int npg = pc.seg_pages[g];
    if (npg < 0 || npg > pc.max_pps) {
        if (lane == 0) atomicOr(err, ERR_LAYOUT);
        return;
    }
    const int32_t* bt = pc.block_table + (int64_t)g * pc.max_pps;
    int found = -1;
    for (int base = 0; base < npg && found < 0; base += 64) {
        const int i = base + lane;
        bool ok = false;
        if (i < npg) {
            const int pg = bt[i];
            ok = pg >= 0 && pg < pc.n_pages && pc.page_live[pg] < P;
        }
        const uint64_t m = __ballot(ok);
        if (m) found = base + __ffsll((long long)m) - 1;
    }
    int page = -1, slot = 0;
    if (found >= 0) {
        page = bt[found];
        const uint64_t m0 = __ballot(pc.pos[(int64_t)page * P + lane] < 0);
        const uint64_t m1 = __ballot(pc.pos[(int64_t)page * P + 64 + lane] < 0);
        if (m0) slot = __ffsll((long long)m0) - 1;
        else if (m1) slot = 64 + __ffsll((long long)m1) - 1;
        else {
            if (lane == 0) atomicOr(err, ERR_LAYOUT);                // page_live disagrees with the slots
            return;
        }
    } else {
        if (npg >= pc.max_pps) {
            if (lane == 0) atomicOr(err, ERR_CAP);
            return;
        }
        int got = -1;
        if (lane == 0) {
            const int idx = atomicSub(pc.n_free, 1) - 1;
            if (idx < 0) {
                atomicAdd(pc.n_free, 1);
                atomicOr(err, ERR_CAP);
            } else {
                got = pc.free_list[idx];
                if (got < 0 || got >= pc.n_pages) {
                    atomicOr(err, ERR_LAYOUT);
                    got = -1;
                }
            }
        }
        page = __shfl(got, 0, 64);
        if (page < 0) return;
        if (lane == 0) {
            pc.block_table[(int64_t)g * pc.max_pps + npg] = page;
            pc.page_owner[page] = g;
            pc.seg_pages[g] = npg + 1;
        }
        slot = 0;
    }
    const int64_t e = (int64_t)page * P + slot;
    const int vpr = head_dim / 8;
    const uint4* ks = reinterpret_cast<const uint4*>(k_new) + (int64_t)g * vpr;
    const uint4* vs = reinterpret_cast<const uint4*>(v_new) + (int64_t)g * vpr;
    uint4* kd = reinterpret_cast<uint4*>(pc.k) + e * vpr;
    uint4* vd = reinterpret_cast<uint4*>(pc.v) + e * vpr;
    for (int i = lane; i < vpr; i += 64) {
        kd[i] = ks[i];
        vd[i] = vs[i];
    }
    if (lane == 0) {
        pc.log_beta[e] = lb_new[g];
        if (pc.log_tail) pc.log_tail[e] = lt_new[g];
        pc.pos[e] = pos_new[g];
        pc.page_live[page] += 1;
        pc.seg_live[g] += 1;
    }
}

// Append of up to n_new tokens per segment (a prefill chunk): one block per segment.  The segment's
// tokens - its rows up to the first negative position - first fill the empty slots of its pages, in
// page order, and the rest goes to pages popped from the free stack in one step.  Whether the pages
// are there is decided before anything is written, so a segment without room is left unchanged.
constexpr int PGA_THREADS = 256;
constexpr int PGA_MAX_NEW = 4096;          // tokens per segment and call (the slot of every token sits in LDS)

__global__ __launch_bounds__(PGA_THREADS) void k_pg_append_n(PagedView pc, const uint16_t* __restrict__ k_new,
                                                             const uint16_t* __restrict__ v_new,
                                                             const float* __restrict__ lb_new,
                                                             const float* __restrict__ lt_new,
                                                             const int32_t* __restrict__ pos_new, int n_new, int head_dim,
                                                             int32_t* err) {
    __shared__ int32_t s_entry[PGA_MAX_NEW];                         // slot (flat entry index) of every token
    __shared__ int32_t lds32[17];
    __shared__ int s_cnt, s_first_new, s_ok;
    const int tid = threadIdx.x, g = blockIdx.x;
    if (tid == 0) s_cnt = n_new;
    __syncthreads();
    for (int i = tid; i < n_new; i += PGA_THREADS)
        if (pos_new[(int64_t)g * n_new + i] < 0) atomicMin(&s_cnt, i);
    __syncthreads();
    const int cnt = s_cnt;                                           // tokens before the first padding row
    if (cnt == 0) return;
    const int npg = pc.seg_pages[g];
    if (npg < 0 || npg > pc.max_pps) {
        if (tid == 0) atomicOr(err, ERR_LAYOUT);
        return;
    }
    int32_t* bt = pc.block_table + (int64_t)g * pc.max_pps;

    // free slots of the segment's pages
    int32_t free_total = 0;
    for (int base = 0; base < npg; base += PGA_THREADS) {
        const int i = base + tid;
        int32_t f = 0;
        if (i < npg) {
            const int pg = bt[i];
            if (pg >= 0 && pg < pc.n_pages) f = max(0, P - pc.page_live[pg]);
        }
        free_total += block_sum<int32_t>(f, lds32);
    }
    const int fill = min(cnt, (int)free_total);                      // tokens that go into holes
    const int np = (cnt - fill + P - 1) / P;                         // new pages
    if (tid == 0) {
        s_ok = 1;
        s_first_new = 0;
        if (np > 0) {
            if (npg + np > pc.max_pps) {
                s_ok = 0;
            } else {
                const int idx = atomicSub(pc.n_free, np) - np;       // our pages: free_list[idx .. idx + np)
                if (idx < 0) {
                    atomicAdd(pc.n_free, np);
                    s_ok = 0;
                } else {
                    s_first_new = idx;
                }
            }
            if (!s_ok) atomicOr(err, ERR_CAP);
        }
    }
    __syncthreads();
    if (!s_ok) return;

    // holes: page i takes the tokens [before_i, before_i + take_i), one thread per page walks its slots
    int32_t before = 0;
    for (int base = 0; base < npg && before < fill; base += PGA_THREADS) {
        const int i = base + tid;
        int pg = -1;
        int32_t f = 0;
        if (i < npg) {
            pg = bt[i];
            if (pg >= 0 && pg < pc.n_pages) f = max(0, P - pc.page_live[pg]);
            else pg = -1;
        }
        int32_t tot;
        const int32_t ex = before + block_excl_scan<int32_t>(f, lds32, &tot);
        if (pg >= 0 && f > 0 && ex < fill) {
            const int take = min((int)f, fill - (int)ex);
            int done = 0;
            for (int sl = 0; sl < P && done < take; ++sl) {
                const int64_t e = (int64_t)pg * P + sl;
                if (pc.pos[e] < 0) s_entry[ex + done++] = (int32_t)e;
            }
            if (done != take) atomicOr(err, ERR_LAYOUT);             // page_live disagrees with the slots
            for (int d = done; d < take; ++d) s_entry[ex + d] = (int32_t)((int64_t)pg * P);   // stay in bounds
            pc.page_live[pg] += take;
        }
        before += tot;
    }
    // new pages, popped from the top of the stack downwards
    const int rest = cnt - fill;
    for (int j = tid; j < np; j += PGA_THREADS) {
        int pg = pc.free_list[s_first_new + np - 1 - j];
        if (pg < 0 || pg >= pc.n_pages) {
            atomicOr(err, ERR_LAYOUT);
            pg = 0;
        }
        bt[npg + j] = pg;
        pc.page_owner[pg] = g;
        pc.page_live[pg] = min(P, rest - j * P);
    }
    __syncthreads();
    for (int t = tid; t < rest; t += PGA_THREADS) s_entry[fill + t] = bt[npg + t / P] * P + t % P;
    __syncthreads();

    // rows and per-entry metadata
    const int vpr = head_dim / 8;
    const uint4* ks = reinterpret_cast<const uint4*>(k_new) + (int64_t)g * n_new * vpr;
    const uint4* vs = reinterpret_cast<const uint4*>(v_new) + (int64_t)g * n_new * vpr;
    uint4* kd = reinterpret_cast<uint4*>(pc.k);
    uint4* vd = reinterpret_cast<uint4*>(pc.v);
    for (int i = tid; i < cnt * vpr; i += PGA_THREADS) {
        const int t = i / vpr, c = i - t * vpr;
        const int64_t e = s_entry[t];
        kd[e * vpr + c] = ks[i];
        vd[e * vpr + c] = vs[i];
    }
    for (int t = tid; t < cnt; t += PGA_THREADS) {
        const int64_t e = s_entry[t];
        pc.log_beta[e] = lb_new[(int64_t)g * n_new + t];
        if (pc.log_tail) pc.log_tail[e] = lt_new[(int64_t)g * n_new + t];
        pc.pos[e] = pos_new[(int64_t)g * n_new + t];
    }
    if (tid == 0) {
        pc.seg_pages[g] = npg + np;
        pc.seg_live[g] += cnt;
    }
}

// ---------------------------------------------------------------------------------------------
// Score: a block takes PG_PER_BLOCK pages; a thread takes four consecutive slots (16-byte loads
// and stores).  Empty slots of a segment's pages get 0; free pages are skipped.
constexpr int PG_PER_BLOCK = 8;
constexpr int PG4_THREADS = PG_PER_BLOCK * P / 4;    // one thread per four slots

__global__ __launch_bounds__(PG4_THREADS) void k_pg_score(PagedView pc, const int32_t* __restrict__ now,
                                                          float* __restrict__ score, int segs_per_seq, int nseg) {
    const int page = blockIdx.x * PG_PER_BLOCK + (threadIdx.x >> 5);
    if (page >= pc.n_pages) return;
    const int owner = pc.page_owner[page];
    if (owner < 0 || owner >= nseg) return;
    const int64_t e = (int64_t)page * P + (threadIdx.x & 31) * 4;
    const int4 ps = *reinterpret_cast<const int4*>(pc.pos + e);
    const float4 lb = *reinterpret_cast<const float4*>(pc.log_beta + e);
    const int t1 = now[owner / segs_per_seq] + 1;
    float4 r;
    if (pc.log_tail) {
        const float4 lt = *reinterpret_cast<const float4*>(pc.log_tail + e);
        r.x = __fmaf_rn((float)(t1 - ps.x), lb.x, lt.x);
        r.y = __fmaf_rn((float)(t1 - ps.y), lb.y, lt.y);
        r.z = __fmaf_rn((float)(t1 - ps.z), lb.z, lt.z);
        r.w = __fmaf_rn((float)(t1 - ps.w), lb.w, lt.w);
    } else {
        r.x = __fmul_rn((float)(t1 - ps.x), lb.x);
        r.y = __fmul_rn((float)(t1 - ps.y), lb.y);
        r.z = __fmul_rn((float)(t1 - ps.z), lb.z);
        r.w = __fmul_rn((float)(t1 - ps.w), lb.w);
    }
    if (ps.x < 0) r.x = 0.f;
    if (ps.y < 0) r.y = 0.f;
    if (ps.z < 0) r.z = 0.f;
    if (ps.w < 0) r.w = 0.f;
    *reinterpret_cast<float4*>(score + e) = r;
}

constexpr int PG_PLAN_ZERO_BLOCKS = 8;

// segment that owns chunk c: the last g with prefix[g] <= c (prefix[nseg] > c)
__device__ __forceinline__ int seg_of_chunk(const int32_t* prefix, int nseg, int c) {
    int lo = 0, hi = nseg;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (prefix[mid] > c) hi = mid;
        else lo = mid + 1;
    }
    return lo - 1;
}

// Plan of the paged selection: blocks [0, PG_TABLE_BLOCKS) build the chunk table (in the
// compaction's table slots of the workspace, which a paged step does not otherwise use); block 0
// also sets the chunk range of every histogram block and the per-sequence state; the remaining
// blocks clear the histograms.
__global__ __launch_bounds__(1024) void k_pg_plan(PagedView pc, Shape sh, const int64_t* __restrict__ budget,
                                                  Workspace ws, int32_t* __restrict__ kept_out,
                                                  uint32_t* __restrict__ thr_out, int hist_blocks) {
    if (blockIdx.x >= PG_TABLE_BLOCKS) {
        const int64_t n = (int64_t)3 * HIST_REPLICAS * sh.n_seq * RADIX_BINS;
        const int zb = blockIdx.x - PG_TABLE_BLOCKS, nzb = gridDim.x - PG_TABLE_BLOCKS;
        for (int64_t i = zb * blockDim.x + threadIdx.x; i < n; i += nzb * blockDim.x) ws.hist[i] = 0;
        return;
    }
    const int tid = threadIdx.x;
    if (blockIdx.x == 0) {
        for (int i = tid; i < DONE_WORDS; i += blockDim.x) ws.done[i] = 0;
        for (int g = tid; g < sh.nseg; g += blockDim.x) {
            kept_out[g] = 0;
            ws.tie_cnt[g] = 0;
            ws.tie_mode[g] = 0;
            ws.tie_thr[g] = 0;
        }
    }
    const int total = build_page_table<1>(pc, sh.nseg, [](int) { return true; }, ws.cmp_chunk_prefix, ws.cmp_desc,
                                          ws.max_cmp_chunks, ws.sel_entry_prefix, ws.err, blockIdx.x, PG_TABLE_BLOCKS);
    if (blockIdx.x != 0) return;
    if (tid < hist_blocks) {
        const int cpb = (total + hist_blocks - 1) / hist_blocks;
        const int c0 = min(total, tid * cpb), c1 = min(total, c0 + cpb);
        int4 r = make_int4(c0, c1, 0, -1);
        if (c0 < c1) {
            r.z = seg_of_chunk(ws.cmp_chunk_prefix, sh.nseg, c0) / sh.segs_per_seq;
            r.w = seg_of_chunk(ws.cmp_chunk_prefix, sh.nseg, c1 - 1) / sh.segs_per_seq;
        }
        ws.sel_blk[tid] = r;
    }
    for (int seq = tid; seq < sh.n_seq; seq += blockDim.x) {
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
        ws.sel[seq] = st;                                            // final slot (what the count and mask kernels read)
        ws.sel[sh.n_seq + seq] = st;                                 // state before the first digit
        ws.seq_done[seq] = 0;
        if (thr_out) thr_out[seq] = 0xFFFFFFFFu;
    }
}

__global__ __launch_bounds__(1024) void k_pg_att_plan(PagedView pc, Shape sh, Workspace ws, int layer_begin,
                                                      int layer_end) {
    const int H = sh.n_kv_heads, L = sh.n_layers;
    auto in_range = [=](int g) {
        const int layer = (g / H) % L;
        return layer >= layer_begin && layer < layer_end;
    };
    static_assert(ATT_PAGE_GROUP == 4, "ws.att_pages holds four pages per chunk");
    build_page_table<ATT_PAGE_GROUP>(pc, sh.nseg, in_range, ws.att_chunk_prefix, ws.att_desc, ws.max_att_chunks, nullptr,
                                     ws.err, blockIdx.x, gridDim.x, ws.att_pages, ws.att_row_prefix);
}

// Mask of the paged selection: a block takes PG_PER_BLOCK pages, a thread four consecutive slots
// (32 lanes to a page).  The survivors are credited to their segment with one device-scope atomic
// per run of pages of the same segment (a block mostly holds pages of one segment): atomics that
// meet on one cache line are served one after the other, and one per wavefront made this kernel
// ten times slower.
__global__ __launch_bounds__(PG4_THREADS) void k_pg_mask(PagedView pc, const float* __restrict__ score, Shape sh,
                                                         Workspace ws, uint8_t* __restrict__ keep,
                                                         int32_t* __restrict__ kept_out) {
    __shared__ int s_n[PG_PER_BLOCK], s_seg[PG_PER_BLOCK];
    const int total = ws.cmp_chunk_prefix[sh.nseg];
    const int pib = threadIdx.x >> 5;                                // page of the block
    const int ch = blockIdx.x * PG_PER_BLOCK + pib;
    int n = 0, seg = -1;
    if (ch < total) {
        const ChunkDesc d = ws.cmp_desc[ch];
        const SelState st = ws.sel[d.seg / sh.segs_per_seq];
        const int64_t e = d.first + (threadIdx.x & 31) * 4;
        const int4 p4 = *reinterpret_cast<const int4*>(pc.pos + e);
        const float4 s4 = *reinterpret_cast<const float4*>(score + e);
        const int ps[4] = {p4.x, p4.y, p4.z, p4.w};
        const float sc[4] = {s4.x, s4.y, s4.z, s4.w};
        int mode = 0, pthr = 0;
        if (st.need_rank) {                                          // 0: no tie survives, 1: all, 2: positions <= tie_thr
            mode = ws.tie_mode[d.seg];
            pthr = ws.tie_thr[d.seg];
        }
        uint32_t packed = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            bool k = false;
            if (ps[j] >= 0 && !st.keep_none) {
                const uint32_t key = key_of_score(sc[j]);
                k = st.need_rank ? (key > st.thr_key || (key == st.thr_key && (mode == 1 || (mode == 2 && ps[j] <= pthr))))
                                 : key >= st.thr_key;
            }
            packed |= (uint32_t)k << (8 * j);
            n += k;
        }
        *reinterpret_cast<uint32_t*>(keep + e) = packed;
        if (!st.need_rank) seg = d.seg;                              // otherwise the count kernel has credited the segments
    }
#pragma unroll
    for (int dlt = 16; dlt >= 1; dlt >>= 1) n += __shfl_xor(n, dlt, 64);   // sum over the 32 lanes of the page
    if ((threadIdx.x & 31) == 0) {
        s_n[pib] = n;
        s_seg[pib] = seg;
    }
    __syncthreads();
    if (threadIdx.x < PG_PER_BLOCK) {
        const int w = threadIdx.x, sg = s_seg[w];
        if (sg >= 0 && (w == 0 || s_seg[w - 1] != sg)) {             // first page of a run
            int sum = 0;
            for (int j = w; j < PG_PER_BLOCK && s_seg[j] == sg; ++j) sum += s_n[j];
            if (sum) atomicAdd(&kept_out[sg], sum);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Ties that do not all fit.  Per page of such a sequence: slots above the threshold are credited
// to the segment, slots equal to it are counted per segment.  The last block to finish turns the
// quota of every sequence into a rule per segment - in (layer, head) order the ties of a segment
// all survive, or none does, and in at most one segment only the q ties with the smallest
// positions survive; that position bound is found by a radix select over the segment's ties.
__device__ __forceinline__ bool is_tie(const PagedView& pc, const float* score, int64_t e, uint32_t thr, int* pos_out) {
    const int ps = pc.pos[e];
    *pos_out = ps;
    return ps >= 0 && key_of_score(score[e]) == thr;
}

constexpr int PGC_THREADS = 256;           // two pages per block and sweep
constexpr int PGC_BINS_PER_THREAD = 2048 / PGC_THREADS;

__global__ __launch_bounds__(PGC_THREADS) void k_pg_count(PagedView pc, const float* __restrict__ score, Shape sh,
                                                          Workspace ws, int32_t* __restrict__ kept_out) {
    if (ws.done[127] == 0) return;                                   // uniform over the grid: every tie fits
    __shared__ int64_t lds64[17];
    __shared__ int32_t lds32[17];
    __shared__ uint32_t h[2048];
    __shared__ int s_list[PGC_THREADS];
    __shared__ int s_n, is_last, s_part_seg, s_part_q, s_digit, s_rank;
    const int tid = threadIdx.x;
    for_each_ranked_seq(ws.sel, sh.n_seq, s_list, &s_n, [&](int seq) {
        const uint32_t thr_key = ws.sel[seq].thr_key;
        const int cb = ws.cmp_chunk_prefix[seq * sh.segs_per_seq], ce = ws.cmp_chunk_prefix[(seq + 1) * sh.segs_per_seq];
        for (int ch = cb + blockIdx.x * 2 + (tid >> 7); ch < ce; ch += gridDim.x * 2) {   // uniform over the wavefront
            const ChunkDesc d = ws.cmp_desc[ch];
            const int64_t e = d.first + (tid & (P - 1));
            bool gt = false, eq = false;
            if (pc.pos[e] >= 0) {
                const uint32_t key = key_of_score(score[e]);
                gt = key > thr_key;
                eq = key == thr_key;
            }
            const int ngt = __popcll(__ballot(gt)), neq = __popcll(__ballot(eq));
            if (lane_id() == 0) {
                if (ngt) atomicAdd(&kept_out[d.seg], ngt);
                if (neq) atomicAdd(&ws.tie_cnt[d.seg], neq);
            }
        }
    });
    __syncthreads();
    if (tid == 0) is_last = arrive_last(ws.done + 32 * 3);
    __syncthreads();
    if (!is_last) return;
    __threadfence();

    for_each_ranked_seq(ws.sel, sh.n_seq, s_list, &s_n, [&](int seq) {
        const SelState st = ws.sel[seq];
        if (tid == 0) s_part_seg = -1;
        __syncthreads();
        int64_t running = 0;
        for (int base = 0; base < sh.segs_per_seq; base += PGC_THREADS) {
            const int i = base + tid;
            const int g = seq * sh.segs_per_seq + i;
            const int64_t v = i < sh.segs_per_seq
                                  ? (int64_t)__hip_atomic_load(&ws.tie_cnt[g], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
            int64_t tot;
            const int64_t ex = block_excl_scan<int64_t>(v, lds64, &tot);
            if (i < sh.segs_per_seq && v > 0) {
                const int64_t before = running + ex;
                if (before + v <= st.tie_quota) {
                    ws.tie_mode[g] = 1;
                    atomicAdd(&kept_out[g], (int32_t)v);
                } else if (before < st.tie_quota) {
                    s_part_seg = g;
                    s_part_q = (int)(st.tie_quota - before);
                }                                                    // else mode 0 (set by the plan)
            }
            running += tot;
        }
        __syncthreads();
        const int g = s_part_seg;
        if (g < 0) return;                                           // uniform over the block
        // the q-th smallest position among the ties of segment g: 11 + 10 + 10 bits, most significant first
        const int npg = pc.seg_pages[g];
        const int32_t* bt = pc.block_table + (int64_t)g * pc.max_pps;
        if (tid == 0) s_rank = s_part_q;
        uint32_t prefix = 0;
        for (int pass = 0; pass < 3; ++pass) {
            const int shift = pass == 0 ? 20 : (pass == 1 ? 10 : 0);
            const int nb = pass == 0 ? 2048 : 1024;
            for (int i = tid; i < 2048; i += PGC_THREADS) h[i] = 0;
            __syncthreads();
            for (int64_t s = tid; s < (int64_t)npg * P; s += PGC_THREADS) {
                const int pg = min(max(bt[s / P], 0), pc.n_pages - 1);
                const int64_t e = (int64_t)pg * P + (s % P);
                int ps;
                if (is_tie(pc, score, e, st.thr_key, &ps)) {
                    const uint32_t up = (uint32_t)ps;
                    const bool match = pass == 0 ? true : (pass == 1 ? (up >> 20) == prefix : (up >> 10) == prefix);
                    if (match) atomicAdd(&h[(up >> shift) & (nb - 1)], 1u);
                }
            }
            __syncthreads();
            // ascending walk: thread t owns bins [t * PGC_BINS_PER_THREAD, (t + 1) * PGC_BINS_PER_THREAD)
            int32_t mine = 0;
#pragma unroll
            for (int i = 0; i < PGC_BINS_PER_THREAD; ++i) mine += (int32_t)h[tid * PGC_BINS_PER_THREAD + i];
            int32_t tot;
            int32_t below = block_excl_scan<int32_t>(mine, lds32, &tot);
            const int rank = s_rank;
            __syncthreads();
            if (below < rank && rank <= below + mine) {
#pragma unroll
                for (int i = 0; i < PGC_BINS_PER_THREAD; ++i) {
                    const int32_t c = (int32_t)h[tid * PGC_BINS_PER_THREAD + i];
                    if (rank <= below + c) {
                        s_digit = tid * PGC_BINS_PER_THREAD + i;
                        s_rank = rank - below;
                        break;
                    }
                    below += c;
                }
            }
            __syncthreads();
            prefix = (prefix << (pass == 0 ? 11 : 10)) | (uint32_t)s_digit;
        }
        if (tid == 0) {
            ws.tie_mode[g] = 2;
            ws.tie_thr[g] = (int32_t)prefix;
            atomicAdd(&kept_out[g], s_part_q);
        }
        __syncthreads();
    });
}

// ---------------------------------------------------------------------------------------------
// Eviction: a block takes PG_PER_BLOCK pages, a thread four consecutive slots (16-byte loads of the
// positions, 4-byte loads of the mask), so a page is the business of one half wavefront.  A page left
// without a live entry is marked for release (owner -2); tidying (k_pg_tidy, or the tidy blocks of the
// attention's merge kernel) takes it out of its segment's block table and pushes it on the free list.
__global__ __launch_bounds__(PG4_THREADS) void k_pg_evict(PagedView pc, const uint8_t* __restrict__ keep, int nseg) {
    const int page = blockIdx.x * PG_PER_BLOCK + (threadIdx.x >> 5);
    const int owner = page < pc.n_pages ? pc.page_owner[page] : -1;
    const bool mine = owner >= 0 && owner < nseg;                    // the same in the 32 lanes of a page
    int n = 0;
    if (mine) {
        const int64_t e = (int64_t)page * P + (threadIdx.x & 31) * 4;
        int4 ps = *reinterpret_cast<const int4*>(pc.pos + e);
        const uint32_t kp = *reinterpret_cast<const uint32_t*>(keep + e);
        const bool e0 = ps.x >= 0 && (kp & 0x000000FFu) == 0, e1 = ps.y >= 0 && (kp & 0x0000FF00u) == 0;
        const bool e2 = ps.z >= 0 && (kp & 0x00FF0000u) == 0, e3 = ps.w >= 0 && (kp & 0xFF000000u) == 0;
        n = (int)e0 + (int)e1 + (int)e2 + (int)e3;
        if (n) {
            if (e0) ps.x = -1;
            if (e1) ps.y = -1;
            if (e2) ps.z = -1;
            if (e3) ps.w = -1;
            *reinterpret_cast<int4*>(pc.pos + e) = ps;
        }
    }
    // sum over the 32 lanes of the page (the exchanges stay inside each half of the wavefront)
#pragma unroll
    for (int d = 16; d >= 1; d >>= 1) n += __shfl_xor(n, d, 64);
    if (mine && n && (threadIdx.x & 31) == 0) {
        const int left = atomicSub(&pc.page_live[page], n) - n;
        atomicSub(&pc.seg_live[owner], n);
        if (left <= 0) pc.page_owner[page] = -2;
    }
}

// One block per segment: the pages that an eviction emptied leave the segment's block table.
__global__ __launch_bounds__(256) void k_pg_tidy(PagedView pc, int32_t* err) { tidy_segment<256>(pc, blockIdx.x, err); }

// ---------------------------------------------------------------------------------------------
// Defragmentation (housekeeping of the paged layout, not a step of the method): eviction frees a page only
// when all of its slots are empty, so a segment slowly spreads over more pages than its live entries need.
// One block per segment: if the live entries fit into fewer pages, the last pages of the block table are
// emptied into the free slots of the pages before them - K row, V row, log beta, position, tail constant
// move together - and return to the free list; the table is cut.  A segment's entries have no order inside
// its pages, so nothing else changes; segments that are already as tight as they can be are left alone.
// Works in passes of at most PGD_LIST moves: whole pages of entries to move (from the table's end backwards)
// and the free slots that take them (from its start forwards) are listed in LDS, then every wavefront
// moves one entry at a time.
constexpr int PGD_THREADS = 256, PGD_LIST = 1024;

__global__ __launch_bounds__(PGD_THREADS) void k_pg_defrag(PagedView pc, int head_dim, int32_t* err) {
    __shared__ int32_t lds32[17];
    __shared__ int64_t s_from[PGD_LIST], s_to[PGD_LIST];
    __shared__ int s_bad;
    const int g = blockIdx.x, tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int npg = pc.seg_pages[g];
    if (npg < 0 || npg > pc.max_pps) {
        if (tid == 0) atomicOr(err, ERR_LAYOUT);
        return;
    }
    if (npg == 0) return;
    int32_t* bt = pc.block_table + (int64_t)g * pc.max_pps;
    if (tid == 0) s_bad = 0;
    __syncthreads();
    int mine = 0;
    for (int i = tid; i < npg; i += PGD_THREADS) {
        const int page = bt[i];
        if (page < 0 || page >= pc.n_pages || pc.page_owner[page] != g) s_bad = 1;
        else mine += pc.page_live[page];
    }
    const int total = block_sum<int32_t>(mine, lds32);               // its barriers also publish s_bad
    if (s_bad || total < 0 || total > npg * P) {
        if (tid == 0) atomicOr(err, ERR_LAYOUT);
        return;
    }
    const int keep_pages = (total + P - 1) / P;
    if (keep_pages >= npg) return;                                   // as tight as it can be

    const int words = head_dim >> 1;                                 // 32-bit words of a K or V row
    uint32_t* k32 = reinterpret_cast<uint32_t*>(pc.k);
    uint32_t* v32 = reinterpret_cast<uint32_t*>(pc.v);
    int rc = 0;                                                      // next page that may still have free slots
    int dc = npg - 1;                                                // next page to empty
    while (dc >= keep_pages) {                                       // every quantity that steers the loops is the same in all threads
        // entries to move: whole pages while the list has room for one more
        int nf = 0;
        while (dc >= keep_pages && nf + P <= PGD_LIST) {
            const int page = bt[dc];
            const int64_t e = (int64_t)page * P + tid;
            const bool live = tid < P && pc.pos[e] >= 0;
            int32_t tot;
            const int32_t ex = block_excl_scan<int32_t>(live ? 1 : 0, lds32, &tot);
            if (live) s_from[nf + ex] = e;
            nf += tot;
            --dc;
        }
        // as many free slots of the pages that stay
        int nh = 0;
        while (nh < nf && rc < keep_pages) {
            const int page = bt[rc];
            const int64_t e = (int64_t)page * P + tid;
            const bool hole = tid < P && pc.pos[e] < 0;
            int32_t tot;
            const int32_t ex = block_excl_scan<int32_t>(hole ? 1 : 0, lds32, &tot);
            if (hole && nh + ex < nf) s_to[nh + ex] = e;
            if (nh + tot <= nf) ++rc;                                // the page is full after this pass
            nh = min(nf, nh + tot);
        }
        if (nh < nf) {                                               // the live counts did not describe the pages
            if (tid == 0) atomicOr(err, ERR_MISMATCH);
            return;
        }
        __syncthreads();
        for (int m = wave; m < nf; m += PGD_THREADS / 64) {
            const int64_t src = s_from[m], dst = s_to[m];
            for (int i = lane; i < words; i += 64) {
                k32[dst * words + i] = k32[src * words + i];
                v32[dst * words + i] = v32[src * words + i];
            }
            if (lane == 0) {
                pc.log_beta[dst] = pc.log_beta[src];
                if (pc.log_tail) pc.log_tail[dst] = pc.log_tail[src];
                pc.pos[dst] = pc.pos[src];
                pc.pos[src] = -1;
                atomicAdd(&pc.page_live[(int)(dst / P)], 1);
                atomicSub(&pc.page_live[(int)(src / P)], 1);
            }
        }
        __syncthreads();                                             // the next pass looks at the slots again
    }
    for (int i = keep_pages + tid; i < npg; i += PGD_THREADS) {     // the emptied pages go back to the free list
        const int page = bt[i];
        pc.page_owner[page] = -1;
        pc.page_live[page] = 0;
        const int idx = atomicAdd(pc.n_free, 1);
        if (idx >= 0 && idx < pc.n_pages) pc.free_list[idx] = page;
    }
    if (tid == 0) pc.seg_pages[g] = keep_pages;
}

// ---------------------------------------------------------------------------------------------
static PagedView view_of(const kvtrim_paged_cache* c) {
    PagedView v;
    v.k = (uint16_t*)c->k;
    v.v = (uint16_t*)c->v;
    v.log_beta = c->log_beta;
    v.pos = c->pos;
    v.log_tail = c->log_tail;
    v.block_table = c->block_table;
    v.seg_pages = c->seg_pages;
    v.seg_live = c->seg_live;
    v.page_owner = c->page_owner;
    v.page_live = c->page_live;
    v.free_list = c->free_list;
    v.n_free = c->n_free;
    v.n_pages = c->n_pages;
    v.max_pps = c->max_pages_per_seg;
    return v;
}

static CacheView pool_view(const kvtrim_paged_cache* c) {
    CacheView v;
    v.k = (const uint16_t*)c->k;
    v.v = (const uint16_t*)c->v;
    v.log_beta = c->log_beta;
    v.pos = c->pos;
    v.seg_start = nullptr;
    v.seg_len = nullptr;
    v.cap = (int64_t)c->n_pages * P;
    v.log_tail = c->log_tail;
    return v;
}

// what is wrong with the arguments of an attention call over pages (NULL if nothing)
static const char* paged_attn_problem(const kvtrim_ctx* ctx, const kvtrim_paged_cache* c, const void* q, int32_t layer_begin,
                                      int32_t layer_end, float softmax_scale, const float* out) {
    if (!q || !out) return "q / out is NULL";
    if (((uintptr_t)q) & 15) return "q not 16-byte aligned";
    if (layer_begin < 0 || layer_end > ctx->cfg.n_layers || layer_begin >= layer_end) return "empty or out-of-range layer range";
    if (!(softmax_scale == softmax_scale)) return "softmax_scale is NaN";
    if ((int64_t)c->n_pages / ATT_PAGE_GROUP + ctx->shape.nseg > ctx->ws.max_att_chunks)
        return "too many pages for the partial-result buffer of this context";
    return nullptr;
}

static const char* paged_problem(const kvtrim_ctx* ctx, const kvtrim_paged_cache* c) {
    if (!c) return "paged cache is NULL";
    if (!c->k || !c->v || !c->log_beta || !c->pos || !c->block_table || !c->seg_pages || !c->seg_live ||
        !c->page_owner || !c->page_live || !c->free_list || !c->n_free)
        return "paged cache has a NULL pointer";
    if ((((uintptr_t)c->k) | ((uintptr_t)c->v) | ((uintptr_t)c->log_beta) | ((uintptr_t)c->pos) | ((uintptr_t)c->log_tail)) & 15)
        return "k / v / log_beta / pos / log_tail not 16-byte aligned";
    if (c->n_pages < 1 || c->max_pages_per_seg < 1) return "n_pages / max_pages_per_seg < 1";
    if ((int64_t)c->n_pages * P > ctx->cfg.max_entries) return "n_pages * page size exceeds max_entries";
    return nullptr;
}

static kvtrim_status bad(kvtrim_ctx* ctx, const char* why) {
    snprintf(ctx->last_error, sizeof(ctx->last_error), "invalid argument: %s", why);
    return KVTRIM_EINVAL;
}

}  // namespace kvtrim

using namespace kvtrim;

extern "C" {

kvtrim_status kvtrim_paged_build(kvtrim_ctx* ctx, const kvtrim_cache* src, const uint8_t* keep, const int32_t* kept,
                                 kvtrim_paged_cache* dst, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = paged_problem(ctx, dst)) return bad(ctx, p);
    if (!src || !src->k || !src->v || !src->log_beta || !src->pos || !src->seg_start || !src->seg_len || !keep || !kept)
        return bad(ctx, "src / keep / kept has a NULL pointer");
    if (src->cap_entries < 1 || src->cap_entries > ctx->cfg.max_entries) return bad(ctx, "src cap_entries outside [1, max_entries]");
    if ((src->log_tail == nullptr) != (dst->log_tail == nullptr)) return bad(ctx, "log_tail must be set in both caches or in neither");
    if (src->k == dst->k || src->v == dst->v || src->log_beta == dst->log_beta || src->pos == dst->pos)
        return bad(ctx, "src and dst share a buffer");
    hipStream_t st = (hipStream_t)hip_stream;
    CacheView sv;
    sv.k = (const uint16_t*)src->k;
    sv.v = (const uint16_t*)src->v;
    sv.log_beta = src->log_beta;
    sv.pos = src->pos;
    sv.seg_start = src->seg_start;
    sv.seg_len = src->seg_len;
    sv.cap = src->cap_entries;
    sv.log_tail = src->log_tail;
    CacheViewMut dv;
    dv.k = (uint16_t*)dst->k;
    dv.v = (uint16_t*)dst->v;
    dv.log_beta = dst->log_beta;
    dv.pos = dst->pos;
    dv.seg_start = ctx->ws.pg_seg_start;
    dv.seg_len = ctx->ws.pg_seg_len;
    dv.cap = (int64_t)dst->n_pages * P;
    dv.log_tail = dst->log_tail;
    launch_cmp_scan_aligned(ctx, sv, keep, kept, dv, 0, P, st, gather_fits(ctx, sv.cap, dv.cap));
    kvtrim_status rc = launch_cmp_copy(ctx, sv, keep, dv, st);
    if (rc != KVTRIM_OK) return rc;
    {
        ProfScope prof(ctx, K_PG_INIT, st);
        const int free_blocks = dst->n_pages < 1024 ? dst->n_pages : 1024;
        hipLaunchKernelGGL(k_pg_init, dim3(ctx->shape.nseg + free_blocks), dim3(256), 0, st, view_of(dst), ctx->shape, ctx->ws);
    }
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

kvtrim_status kvtrim_paged_append(kvtrim_ctx* ctx, kvtrim_paged_cache* c, const void* k_new, const void* v_new,
                                  const float* log_beta_new, const float* log_tail_new, const int32_t* pos_new,
                                  int32_t n_new, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = paged_problem(ctx, c)) return bad(ctx, p);
    if (!k_new || !v_new || !log_beta_new || !pos_new) return bad(ctx, "a new-token pointer is NULL");
    if ((((uintptr_t)k_new) | ((uintptr_t)v_new)) & 15) return bad(ctx, "k_new / v_new not 16-byte aligned");
    if ((c->log_tail == nullptr) != (log_tail_new == nullptr))
        return bad(ctx, "log_tail_new is required exactly when the cache carries log_tail");
    if (n_new < 1 || n_new > PGA_MAX_NEW) return bad(ctx, "n_new outside [1, 4096]");
    hipStream_t st = (hipStream_t)hip_stream;
    ProfScope prof(ctx, K_PG_APPEND, st);
    if (n_new == 1)
        hipLaunchKernelGGL(k_pg_append, dim3((ctx->shape.nseg + 3) / 4), dim3(256), 0, st, view_of(c), (const uint16_t*)k_new,
                           (const uint16_t*)v_new, log_beta_new, log_tail_new, pos_new, ctx->shape.nseg, ctx->shape.head_dim,
                           ctx->ws.err);
    else
        hipLaunchKernelGGL(k_pg_append_n, dim3(ctx->shape.nseg), dim3(PGA_THREADS), 0, st, view_of(c), (const uint16_t*)k_new,
                           (const uint16_t*)v_new, log_beta_new, log_tail_new, pos_new, n_new, ctx->shape.head_dim, ctx->ws.err);
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

kvtrim_status kvtrim_paged_score(kvtrim_ctx* ctx, const kvtrim_paged_cache* c, const int32_t* now, float* score_out,
                                 void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = paged_problem(ctx, c)) return bad(ctx, p);
    if (!now || !score_out) return bad(ctx, "now / score_out is NULL");
    if (((uintptr_t)score_out) & 15) return bad(ctx, "score_out not 16-byte aligned");
    hipStream_t st = (hipStream_t)hip_stream;
    ProfScope prof(ctx, K_PG_SCORE, st);
    hipLaunchKernelGGL(k_pg_score, dim3((c->n_pages + PG_PER_BLOCK - 1) / PG_PER_BLOCK), dim3(PG4_THREADS), 0, st, view_of(c),
                       now, score_out, ctx->shape.segs_per_seq, ctx->shape.nseg);
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

kvtrim_status kvtrim_paged_select(kvtrim_ctx* ctx, const kvtrim_paged_cache* c, const float* score, const int64_t* budget,
                                  uint8_t* keep_out, int32_t* kept_out, uint32_t* thr_key_out, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = paged_problem(ctx, c)) return bad(ctx, p);
    if (!score || !budget || !keep_out || !kept_out) return bad(ctx, "score / budget / keep_out / kept_out is NULL");
    if ((((uintptr_t)score) & 15) || (((uintptr_t)keep_out) & 3)) return bad(ctx, "score not 16-byte or keep_out not 4-byte aligned");
    hipStream_t st = (hipStream_t)hip_stream;
    const PagedView pv = view_of(c);
    const int hist_blocks = c->n_pages < HIST_BLOCKS_MAX ? c->n_pages : HIST_BLOCKS_MAX;
    {
        ProfScope prof(ctx, K_PG_PLAN, st);
        hipLaunchKernelGGL(k_pg_plan, dim3(PG_TABLE_BLOCKS + PG_PLAN_ZERO_BLOCKS), dim3(1024), 0, st, pv, ctx->shape, budget, ctx->ws,
                           kept_out, thr_key_out, hist_blocks);
    }
    SelTables tb;
    tb.desc = ctx->ws.cmp_desc;
    tb.prefix = ctx->ws.cmp_chunk_prefix;
    tb.pos = c->pos;
    for (int pass = 0; pass < 3; ++pass) launch_select_passes_paged(ctx, score, tb, hist_blocks, pass, thr_key_out, st);
    {
        ProfScope prof(ctx, K_PG_COUNT, st);
        const int pairs = (c->n_pages + 1) / 2;
        hipLaunchKernelGGL(k_pg_count, dim3(pairs < 1024 ? pairs : 1024), dim3(PGC_THREADS), 0, st, pv, score, ctx->shape,
                           ctx->ws, kept_out);
    }
    {
        ProfScope prof(ctx, K_SEL_MASK, st);
        hipLaunchKernelGGL(k_pg_mask, dim3((c->n_pages + PG_PER_BLOCK - 1) / PG_PER_BLOCK), dim3(PG4_THREADS), 0, st, pv, score,
                           ctx->shape, ctx->ws, keep_out, kept_out);
    }
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

kvtrim_status kvtrim_paged_score_select(kvtrim_ctx* ctx, const kvtrim_paged_cache* c, const int32_t* now, const int64_t* budget,
                                        float* score_out, uint8_t* keep_out, int32_t* kept_out, uint32_t* thr_key_out,
                                        int64_t evict_hint, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = paged_problem(ctx, c)) return bad(ctx, p);
    if (!now || !budget || !score_out || !keep_out || !kept_out) return bad(ctx, "now / budget / score_out / keep_out / kept_out is NULL");
    if ((((uintptr_t)score_out) & 15) || (((uintptr_t)keep_out) & 3)) return bad(ctx, "score_out not 16-byte or keep_out not 4-byte aligned");
    // the list has to hold about 3 (k + 1) entries for k evictions, spread unevenly over its sub-lists
    if (evict_hint <= 0 || 8 * (evict_hint + 1) > (int64_t)ctx->ws.fl_cap) {
        const kvtrim_status rc = kvtrim_paged_score(ctx, c, now, score_out, hip_stream);
        if (rc != KVTRIM_OK) return rc;
        return kvtrim_paged_select(ctx, c, score_out, budget, keep_out, kept_out, thr_key_out, hip_stream);
    }
    PagedArgs pg{};
    pg.block_table = c->block_table;
    pg.seg_pages = c->seg_pages;
    pg.seg_live = c->seg_live;
    pg.n_pages = c->n_pages;
    pg.max_pps = c->max_pages_per_seg;
    pg.evict_pos = pg.evict_seg_live = pg.evict_page_live = pg.evict_page_owner = nullptr;
    return launch_score_select_paged(ctx, pool_view(c), pg, now, budget, score_out, keep_out, kept_out, thr_key_out,
                                     (hipStream_t)hip_stream);
}

kvtrim_status kvtrim_paged_decode_step(kvtrim_ctx* ctx, kvtrim_paged_cache* c, const void* k_new, const void* v_new,
                                       const float* log_beta_new, const float* log_tail_new, const int32_t* pos_new,
                                       const int32_t* now, const int64_t* budget, float* score_out, uint8_t* keep_out,
                                       int32_t* kept_out, uint32_t* thr_key_out, const void* q, int32_t layer_begin,
                                       int32_t layer_end, float softmax_scale, float* out, float* lse, int64_t evict_hint,
                                       void* hip_stream) {
    kvtrim_status rc = kvtrim_paged_append(ctx, c, k_new, v_new, log_beta_new, log_tail_new, pos_new, 1, hip_stream);
    if (rc != KVTRIM_OK) return rc;
    if (evict_hint <= 0 || 8 * (evict_hint + 1) > (int64_t)ctx->ws.fl_cap) {
        rc = kvtrim_paged_score_select(ctx, c, now, budget, score_out, keep_out, kept_out, thr_key_out, evict_hint, hip_stream);
        if (rc != KVTRIM_OK) return rc;
        rc = kvtrim_paged_evict(ctx, c, keep_out, hip_stream);
        if (rc != KVTRIM_OK) return rc;
    } else {
        // the decode-step selection, whose mask kernel also applies the eviction ...
        if (!now || !budget || !score_out || !keep_out || !kept_out) return bad(ctx, "now / budget / score_out / keep_out / kept_out is NULL");
        if ((((uintptr_t)score_out) & 15) || (((uintptr_t)keep_out) & 3)) return bad(ctx, "score_out not 16-byte or keep_out not 4-byte aligned");
        hipStream_t st = (hipStream_t)hip_stream;
        PagedArgs pg{};
        pg.block_table = c->block_table;
        pg.seg_pages = c->seg_pages;
        pg.seg_live = c->seg_live;
        pg.n_pages = c->n_pages;
        pg.max_pps = c->max_pages_per_seg;
        pg.evict_pos = c->pos;
        pg.evict_seg_live = c->seg_live;
        pg.evict_page_live = c->page_live;
        pg.evict_page_owner = c->page_owner;
        // ... whose scoring kernel also builds the attention's chunk table; the merge kernel of the attention tidies
        // the block tables afterwards: five kernels in all
        if (const char* p = paged_attn_problem(ctx, c, q, layer_begin, layer_end, softmax_scale, out)) return bad(ctx, p);
        pg.plan_layer_begin = layer_begin;
        pg.plan_layer_end = layer_end;
        rc = launch_score_select_paged(ctx, pool_view(c), pg, now, budget, score_out, keep_out, kept_out, thr_key_out, st, true);
        if (rc != KVTRIM_OK) return rc;
        const PagedView pv = view_of(c);
        const int max_chunks = c->n_pages / ATT_PAGE_GROUP + ctx->shape.nseg;
        return launch_attn_paged(ctx, pool_view(c), c->block_table, (const uint16_t*)q, max_chunks, layer_begin, layer_end,
                                 softmax_scale, out, lse, st, &pv);
    }
    return kvtrim_paged_attn(ctx, c, q, layer_begin, layer_end, softmax_scale, out, lse, hip_stream);
}

kvtrim_status kvtrim_paged_evict(kvtrim_ctx* ctx, kvtrim_paged_cache* c, const uint8_t* keep, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = paged_problem(ctx, c)) return bad(ctx, p);
    if (!keep) return bad(ctx, "keep is NULL");
    if (((uintptr_t)keep) & 3) return bad(ctx, "keep not 4-byte aligned");
    hipStream_t st = (hipStream_t)hip_stream;
    const PagedView pv = view_of(c);
    {
        ProfScope prof(ctx, K_PG_EVICT, st);
        hipLaunchKernelGGL(k_pg_evict, dim3((c->n_pages + PG_PER_BLOCK - 1) / PG_PER_BLOCK), dim3(PG4_THREADS), 0, st, pv, keep,
                           ctx->shape.nseg);
    }
    {
        ProfScope prof(ctx, K_PG_TIDY, st);
        hipLaunchKernelGGL(k_pg_tidy, dim3(ctx->shape.nseg), dim3(256), 0, st, pv, ctx->ws.err);
    }
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

kvtrim_status kvtrim_paged_defrag(kvtrim_ctx* ctx, kvtrim_paged_cache* c, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = paged_problem(ctx, c)) return bad(ctx, p);
    hipStream_t st = (hipStream_t)hip_stream;
    {
        ProfScope prof(ctx, K_PG_DEFRAG, st);
        hipLaunchKernelGGL(k_pg_defrag, dim3(ctx->shape.nseg), dim3(PGD_THREADS), 0, st, view_of(c), ctx->shape.head_dim,
                           ctx->ws.err);
    }
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

kvtrim_status kvtrim_paged_attn(kvtrim_ctx* ctx, const kvtrim_paged_cache* c, const void* q, int32_t layer_begin,
                                int32_t layer_end, float softmax_scale, float* out, float* lse, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (const char* p = paged_problem(ctx, c)) return bad(ctx, p);
    if (const char* p = paged_attn_problem(ctx, c, q, layer_begin, layer_end, softmax_scale, out)) return bad(ctx, p);
    hipStream_t st = (hipStream_t)hip_stream;
    {
        ProfScope prof(ctx, K_PG_ATT_PLAN, st);
        hipLaunchKernelGGL(k_pg_att_plan, dim3(PG_TABLE_BLOCKS), dim3(1024), 0, st, view_of(c), ctx->shape, ctx->ws,
                           layer_begin, layer_end);
    }
    const int max_chunks = c->n_pages / ATT_PAGE_GROUP + ctx->shape.nseg;   // sum over segments of ceil(pages / group)
    return launch_attn_paged(ctx, pool_view(c), c->block_table, (const uint16_t*)q, max_chunks, layer_begin, layer_end,
                             softmax_scale, out, lse, st);
}

}  // extern "C"
