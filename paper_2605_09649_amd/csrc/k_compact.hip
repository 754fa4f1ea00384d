// Stage 3: stable stream compaction of the retained entries into a tight ragged cache.
//
// k_cmp_scan  one block per segment: counts the mask per 128-entry chunk (wavefront ballot),
//             scans the counts inside the segment and derives the destination segment table
//             from `kept`.
// k_cmp_copy  one block of 8 wavefronts per chunk: a ballot/prefix over the chunk's mask
//             ranks the survivors; every wavefront then moves at most 16 rows in ONE batch of
//             loads followed by one batch of stores (16 bytes per lane, whole rows per 16
//             lanes, non-temporal) and ends.  Short-lived wavefronts measured ~10 % faster on
//             this chip than wavefronts that loop over several batches.
#include "kvtrim_device.h"

namespace kvtrim {

constexpr int SCAN_THREADS = 1024;
constexpr int SCAN_BATCH = 8;          // chunks whose mask bytes a wavefront requests before it counts any

// Sums N values over the block with one pair of barriers; every thread gets every sum.
template <int N>
__device__ __forceinline__ void block_sum_n(int64_t (&v)[N], int64_t* lds /* [16 * N] */) {
    const int lane = lane_id(), wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
#pragma unroll
    for (int k = 0; k < N; ++k) v[k] = wave_sum(v[k]);
    __syncthreads();
    if (lane == 0) {
#pragma unroll
        for (int k = 0; k < N; ++k) lds[wave * N + k] = v[k];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < N; ++k) {
        int64_t s = 0;
        for (int w = 0; w < nw; ++w) s += lds[w * N + k];
        v[k] = s;
    }
}

// With many segments the per-block reduction over all segments below costs more than a launch: one block
// then scans the segments once and leaves, per segment, the first chunk (ws.cmp_chunk_prefix) and the first
// destination entry (dst.seg_start) - the two values k_cmp_scan would otherwise derive in every block.
// inplace: the survivors stay in their segment's own region (dst is the same cache): the segment starts stand as
// they are and there is no capacity to check.
__global__ __launch_bounds__(SCAN_THREADS) void k_cmp_prefix(CacheView src, const int32_t* __restrict__ kept,
                                                             CacheViewMut dst, int reserve, int align, Shape sh,
                                                             Workspace ws, int inplace, int gat) {
    __shared__ int64_t lds64[17];
    __shared__ int s_bad_layout, s_bad_kept;
    const int tid = threadIdx.x, nseg = sh.nseg;
    if (tid == 0) s_bad_layout = s_bad_kept = 0;
    __syncthreads();
    int64_t chunks = 0, entries = 0, runs = 0;
    for (int base = 0; base < nseg; base += SCAN_THREADS) {
        const int i = base + tid;
        int64_t nch = 0, need = 0, nrun = 0;
        if (i < nseg) {
            const int len = src.seg_len[i];
            const int64_t st = src.seg_start[i];
            const int kp = kept[i];
            const int64_t nxt = i + 1 < nseg ? src.seg_start[i + 1] : src.cap;
            if (len < 0 || st < 0 || st + len > src.cap || st + len > nxt) s_bad_layout = 1;
            if (kp < 0 || kp > len) s_bad_kept = 1;
            nch = len > 0 ? ((int64_t)len + CMP_CHUNK - 1) / CMP_CHUNK : 0;
            need = ((int64_t)kp + reserve + align - 1) / align * align;
            nrun = gat && len > 0 ? ((int64_t)kp + CMP_CHUNK - 1) / CMP_CHUNK : 0;
        }
        int64_t tot_c, tot_e;
        const int64_t ex_c = block_excl_scan<int64_t>(nch, lds64, &tot_c);
        const int64_t ex_e = block_excl_scan<int64_t>(need, lds64, &tot_e);
        if (i < nseg) {
            ws.cmp_chunk_prefix[i] = (int32_t)min(chunks + ex_c, (int64_t)0x7fffffff);
            // (parked in the workspace: the destination is written only once the capacity check below has passed)
            if (!inplace) ws.pg_seg_start[i] = entries + ex_e;
        }
        chunks += tot_c;
        entries += tot_e;
        if (gat) {                                                // uniform over the block
            int64_t tot_r;
            const int64_t ex_r = block_excl_scan<int64_t>(nrun, lds64, &tot_r);
            if (i < nseg) ws.att_chunk_prefix[i] = (int32_t)min(runs + ex_r, (int64_t)0x7fffffff);
            runs += tot_r;
        }
    }
    __syncthreads();
    const bool bad_layout = s_bad_layout || chunks > ws.max_cmp_chunks || runs > ws.max_att_chunks, bad_kept = s_bad_kept != 0;
    if (tid == 0) {
        if (bad_layout || bad_kept || (!inplace && entries > dst.cap)) {
            atomicOr(ws.err, bad_layout ? ERR_LAYOUT : (bad_kept ? ERR_MISMATCH : ERR_CAP));
            ws.cmp_chunk_prefix[nseg] = 0;
            if (gat) ws.att_chunk_prefix[nseg] = 0;
        } else {
            ws.cmp_chunk_prefix[nseg] = (int32_t)chunks;
            if (gat) ws.att_chunk_prefix[nseg] = (int32_t)runs;
        }
    }
    if (!inplace && !(bad_layout || bad_kept || entries > dst.cap)) {
        __syncthreads();                                          // the parked starts are this block's own writes
        for (int i = tid; i < nseg; i += SCAN_THREADS) dst.seg_start[i] = ws.pg_seg_start[i];
    }
}

// PRE: k_cmp_prefix has run (segment prefixes and the checks over all segments are done).
// gat: the table of the DESTINATION's 128-row chunks (ws.att_chunk_prefix / ws.att_desc) and the source row of every
// destination row (ws.gat_src) are written as well, for the gathering instance of the fused kernel that follows.
template <bool PRE>
__global__ __launch_bounds__(SCAN_THREADS) void k_cmp_scan(CacheView src, const uint8_t* __restrict__ keep,
                                                           const int32_t* __restrict__ kept, CacheViewMut dst,
                                                           int reserve, int align, Shape sh, Workspace ws, int inplace,
                                                           int gat) {
    __shared__ int64_t lds64[17];
    __shared__ int64_t lds_n[16 * 8];
    __shared__ int s_cnt[SCAN_THREADS];
    __shared__ int s_ex[SCAN_THREADS];
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int g = blockIdx.x;
    const int nseg = sh.nseg;

    // Order of the memory traffic: (1) this segment's own table entry; (2) in one round, the table entries of all
    // segments (for the prefixes; !PRE) and the mask bytes of this segment's first SCAN_THREADS chunks; then
    // arithmetic only; (3) the stores.  A decode-step segment is done after two dependent round trips.
    const int len_raw = src.seg_len[g];
    const int64_t start = src.seg_start[g];
    const bool own_ok = len_raw >= 0 && start >= 0 && start + len_raw <= src.cap;   // (checked for all segments below / by k_cmp_prefix)
    const int len = own_ok ? len_raw : 0;
    const int nch = len > 0 ? (len + CMP_CHUNK - 1) / CMP_CHUNK : 0;
    const uint8_t* kp = keep + start;

    int64_t chunks_before, dst_before, runs_before = 0;
    int o_len = 0, o_kp = 0;                                      // !PRE: table entry of segment `tid`
    int64_t o_st = 0;
    if (PRE) {
        // One decision for the whole block: another block of this launch may raise the flag (a mask that disagrees
        // with `kept`) between the reads of two wavefronts, and a block that lost some of its wavefronts would scan
        // counts that were never written.
        __shared__ int s_err;
        if (tid == 0) s_err = __hip_atomic_load(ws.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (s_err != 0) return;
        chunks_before = ws.cmp_chunk_prefix[g];
        dst_before = dst.seg_start[g];
        if (gat) runs_before = ws.att_chunk_prefix[g];
    } else if (tid < nseg) {                                      // (nseg <= SCAN_THREADS without k_cmp_prefix)
        o_len = src.seg_len[tid];
        o_st = src.seg_start[tid];
        o_kp = kept[tid];
    }

    // survivors per chunk of one tile of SCAN_THREADS chunks into s_cnt: one wavefront per chunk, two coalesced byte
    // loads per lane; a wavefront requests the bytes of up to SCAN_BATCH of its chunks before it counts any
    uint8_t b[SCAN_BATCH][CMP_CHUNK / 64];
    auto request = [&](int tile0, int tile_n, int c0) {
#pragma unroll
        for (int u = 0; u < SCAN_BATCH; ++u) {
            const int ch = tile0 + c0 + u * (SCAN_THREADS / 64);
#pragma unroll
            for (int r = 0; r < CMP_CHUNK / 64; ++r) {
                const int64_t j = (int64_t)ch * CMP_CHUNK + r * 64 + lane;
                b[u][r] = (c0 + u * (SCAN_THREADS / 64) < tile_n && j < len) ? kp[j] : (uint8_t)0;
            }
        }
    };
    auto count = [&](int tile_n, int c0) {
#pragma unroll
        for (int u = 0; u < SCAN_BATCH; ++u) {
            int cnt = 0;
#pragma unroll
            for (int r = 0; r < CMP_CHUNK / 64; ++r) cnt += __popcll(__ballot(b[u][r] != 0));
            const int cl = c0 + u * (SCAN_THREADS / 64);
            if (lane == 0 && cl < tile_n) s_cnt[cl] = cnt;
        }
    };
    request(0, min(SCAN_THREADS, nch), wave);                     // in flight while the prefixes are summed

    if (!PRE) {
        // chunks and destination entries of the segments before g, and the totals
        int64_t acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};   // chunks_before, dst_before, dst_total, chunks_total, bad_layout, bad_kept, runs_before, runs_total
        if (tid < nseg) {
            const int i = tid;
            const int64_t o_nxt = i + 1 < nseg ? src.seg_start[i + 1] : src.cap;
            acc[4] |= (o_len < 0 || o_st < 0 || o_st + o_len > src.cap || o_st + o_len > o_nxt);
            acc[5] |= (o_kp < 0 || o_kp > o_len);
            const int64_t nc = o_len > 0 ? ((int64_t)o_len + CMP_CHUNK - 1) / CMP_CHUNK : 0;
            const int64_t need = ((int64_t)o_kp + reserve + align - 1) / align * align;   // align = 1 unless pages are built
            const int64_t nrun = gat && o_len > 0 ? ((int64_t)o_kp + CMP_CHUNK - 1) / CMP_CHUNK : 0;
            acc[3] += nc;
            acc[2] += need;
            acc[7] += nrun;
            if (i < g) {
                acc[0] += nc;
                acc[1] += need;
                acc[6] += nrun;
            }
        }
        block_sum_n<8>(acc, lds_n);
        chunks_before = acc[0];
        dst_before = acc[1];
        runs_before = acc[6];
        const int64_t dst_total = acc[2], chunks_total = acc[3];
        const bool bad_layout = acc[4] != 0 || chunks_total > ws.max_cmp_chunks || acc[7] > ws.max_att_chunks, bad_kept = acc[5] != 0;
        if (inplace) dst_before = start;                          // the segment keeps its place
        if (bad_layout || bad_kept || (!inplace && dst_total > dst.cap)) {   // every block takes the same decision
            if (tid == 0) {
                atomicOr(ws.err, bad_layout ? ERR_LAYOUT : (bad_kept ? ERR_MISMATCH : ERR_CAP));
                if (g == 0) {
                    ws.cmp_chunk_prefix[nseg] = 0;
                    if (gat) ws.att_chunk_prefix[nseg] = 0;
                }
            }
            return;
        }
    }

    const int cbase = (int)chunks_before;
    int64_t gat_slots = 0;                                        // gat: slots of this segment in ws.gat_src
    if (gat) {                                                    // the chunks of the DESTINATION segment, for the gathering fused kernel
        const int rlen = own_ok ? kept[g] : 0;
        const int nrun = len > 0 && rlen > 0 ? (rlen + CMP_CHUNK - 1) / CMP_CHUNK : 0;
        gat_slots = (int64_t)nrun * CMP_CHUNK;
        for (int u = tid; u < nrun; u += SCAN_THREADS) {
            ChunkDesc d;
            d.first = dst_before + (int64_t)u * CMP_CHUNK;
            d.n = min(CMP_CHUNK, rlen - u * CMP_CHUNK);
            d.seg = g;
            ws.att_desc[runs_before + u] = d;
        }
        if (tid == 0 && !PRE) {
            ws.att_chunk_prefix[g] = (int32_t)runs_before;
            if (g == nseg - 1) ws.att_chunk_prefix[nseg] = (int32_t)(runs_before + nrun);
        }
    }

    // Tiles of SCAN_THREADS chunks: counts (phase 1, above), then a thread per chunk - exclusive scan of the counts,
    // destination offset and descriptor of every chunk (phase 2).
    int64_t running = 0;
    for (int tile0 = 0; tile0 < nch; tile0 += SCAN_THREADS) {
        const int tile_n = min(SCAN_THREADS, nch - tile0);
        __syncthreads();                                          // s_cnt of the previous tile has been read
        for (int c0 = wave; c0 < tile_n; c0 += (SCAN_THREADS / 64) * SCAN_BATCH) {
            if (tile0 > 0 || c0 > wave) request(tile0, tile_n, c0);   // (the first batch of the first tile is already here)
            count(tile_n, c0);
        }
        __syncthreads();
        const int ch = tile0 + tid;
        const int64_t v = tid < tile_n ? s_cnt[tid] : 0;
        int64_t tot;
        const int64_t ex = block_excl_scan<int64_t>(v, lds64, &tot);
        if (tid < tile_n) {
            const int n = min(CMP_CHUNK, len - ch * CMP_CHUNK);
            // a chunk that loses nothing is marked: its mover needs neither the mask nor the ranks
            ws.cmp_chunk_dst[cbase + ch] = (dst_before + running + ex) | (v == n ? CMP_DST_FULL : 0);
            ChunkDesc d;
            d.first = start + (int64_t)ch * CMP_CHUNK;
            d.n = n;
            d.seg = g;
            ws.cmp_desc[cbase + ch] = d;
        }
        if (gat) {
            // the source row of every destination row, in slots of CMP_CHUNK per destination chunk (the segment's
            // chunks are consecutive, so row r of the segment has slot runs_before * CMP_CHUNK + r): a wavefront per
            // source chunk ranks its survivors again (the mask bytes come from the cache this time)
            s_ex[tid] = (int)(running + ex);
            __syncthreads();
            int32_t* slots = ws.gat_src + runs_before * CMP_CHUNK;
            for (int c0 = wave; c0 < tile_n; c0 += (SCAN_THREADS / 64) * SCAN_BATCH) {
                request(tile0, tile_n, c0);
#pragma unroll
                for (int u = 0; u < SCAN_BATCH; ++u) {
                    const int cl = c0 + u * (SCAN_THREADS / 64);
                    if (cl >= tile_n) break;                      // uniform over the wavefront
                    const uint64_t m0 = __ballot(b[u][0] != 0), m1 = __ballot(b[u][1] != 0);
                    const int r0 = s_ex[cl] + mbcnt(m0), r1 = s_ex[cl] + __popcll(m0) + mbcnt(m1);
                    const int32_t row = (int32_t)(start + (int64_t)(tile0 + cl) * CMP_CHUNK + lane);
                    // (a mask with more survivors than `kept` says - reported below - must not leave the segment's slots)
                    if (b[u][0] != 0 && r0 >= 0 && r0 < gat_slots) slots[r0] = row;
                    if (b[u][1] != 0 && r1 >= 0 && r1 < gat_slots) slots[r1] = row + 64;
                }
            }
        }
        running += tot;
    }
    if (gat) {
        // the slots behind the segment's last row, up to the end of its last chunk, name a row that exists
        for (int64_t r = running + tid; r < gat_slots; r += SCAN_THREADS) ws.gat_src[runs_before * CMP_CHUNK + r] = (int32_t)start;
    }
    if (tid == 0) {
        if (running != kept[g]) atomicOr(ws.err, ERR_MISMATCH);
        if (!inplace) {                                           // (in place the other blocks are still reading the lengths:
            dst.seg_start[g] = dst_before;                        //  the mover's last kernel commits them)
            dst.seg_len[g] = kept[g];
        }
        if (!PRE) {
            ws.cmp_chunk_prefix[g] = cbase;
            if (g == nseg - 1) ws.cmp_chunk_prefix[nseg] = cbase + nch;
        }
    }
}

typedef unsigned v4u __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint4 ld16_nt(const uint4* p) {
    v4u t = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void st16_nt(uint4* p, uint4 v) {
    v4u t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<v4u*>(p));
}

// NEW: the K/V rows of a segment's entries from old_len[seg] on are not in src but in k_new / v_new
// ([nseg][n_new][D], entry old_len + i of segment g = row g * n_new + i): a chunk of tokens whose metadata has
// been appended to src goes from the caller's buffers straight to its place in dst.
template <int D, bool NEW>
__global__ __launch_bounds__(CMP_THREADS) void k_cmp_copy(CacheView src, const uint8_t* __restrict__ keep,
                                                          CacheViewMut dst, Shape sh, Workspace ws,
                                                          const uint16_t* __restrict__ k_new,
                                                          const uint16_t* __restrict__ v_new, int n_new,
                                                          const int32_t* __restrict__ old_len) {
    constexpr int VPR = D / 8;                    // 16-byte vectors per row
    constexpr int RPI = 64 / VPR;                 // rows moved by one wavefront instruction
    constexpr int BATCH = CMP_WAVE_ROWS / RPI;    // instructions per wavefront: 4 (D=128) or 2 (D=64)
    __shared__ int wave_cnt[CMP_CHUNK / 64];
    __shared__ int list[CMP_CHUNK];
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    if (__hip_atomic_load(ws.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
    const int total = ws.cmp_chunk_prefix[sh.nseg];
    const int ch = blockIdx.x;
    if (ch >= total) return;
    const ChunkDesc d = ws.cmp_desc[ch];
    const int64_t sbase = d.first;                                // first source entry of the chunk
    const int64_t dbase = ws.cmp_chunk_dst[ch] & ~CMP_DST_FULL;   // first destination entry of its survivors
    // the first CMP_CHUNK threads rank the survivors
    int rank = 0;
    bool flag = false;
    if (tid < CMP_CHUNK) {
        flag = tid < d.n && keep[sbase + tid] != 0;
        const uint64_t mask = __ballot(flag);
        rank = mbcnt(mask);
        if (lane == 0) wave_cnt[wave] = __popcll(mask);
    }
    __syncthreads();
    int cnt = 0;
#pragma unroll
    for (int w = 0; w < CMP_CHUNK / 64; ++w) {
        if (w < wave && tid < CMP_CHUNK) rank += wave_cnt[w];
        cnt += wave_cnt[w];
    }
    if (flag) {
        list[rank] = tid;
        dst.log_beta[dbase + rank] = src.log_beta[sbase + tid];
        if (src.log_tail) dst.log_tail[dbase + rank] = src.log_tail[sbase + tid];
        dst.pos[dbase + rank] = src.pos[sbase + tid];
    }
    __syncthreads();
    const int r0 = wave * CMP_WAVE_ROWS;                          // this wavefront's rows of the survivor list
    if (r0 >= cnt) return;
    const uint4* sk = reinterpret_cast<const uint4*>(src.k);
    const uint4* sv = reinterpret_cast<const uint4*>(src.v);
    uint4* dk = reinterpret_cast<uint4*>(dst.k);
    uint4* dv = reinterpret_cast<uint4*>(dst.v);
    const int sub = lane / VPR, col = lane % VPR;
    uint4 kk[BATCH], vv[BATCH];
    // NEW: index of the chunk's first entry in its segment, and where the segment's new entries begin
    const int64_t seg_off = NEW ? sbase - src.seg_start[d.seg] : 0;
    const int64_t first_new = NEW ? old_len[d.seg] : 0;
    const int64_t new_base = NEW ? (int64_t)d.seg * n_new - first_new : 0;   // + index in the segment = row of k_new
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
        const int r = min(r0 + u * RPI + sub, cnt - 1);           // clamped: loads stay on live rows
        const int64_t j = seg_off + list[r];
        if (NEW && j >= first_new) {
            const int64_t ne = (new_base + j) * VPR + col;
            kk[u] = ld16_nt(reinterpret_cast<const uint4*>(k_new) + ne);
            vv[u] = ld16_nt(reinterpret_cast<const uint4*>(v_new) + ne);
        } else {
            const int64_t se = (sbase + list[r]) * VPR + col;
            kk[u] = ld16_nt(sk + se);
            vv[u] = ld16_nt(sv + se);
        }
    }
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
        const int r = r0 + u * RPI + sub;
        if (r < cnt) {
            const int64_t de = (dbase + r) * VPR + col;
            st16_nt(dk + de, kk[u]);
            st16_nt(dv + de, vv[u]);
        }
    }
}

void launch_cmp_scan_aligned(kvtrim_ctx* ctx, const CacheView& src, const uint8_t* keep, const int32_t* kept,
                             const CacheViewMut& dst, int32_t reserve, int32_t align, hipStream_t st, bool gat) {
    ProfScope prof(ctx, K_CMP_SCAN, st);
    const int g = gat ? 1 : 0;
    if (ctx->shape.nseg > 1024) {                                 // see k_cmp_prefix
        hipLaunchKernelGGL(k_cmp_prefix, dim3(1), dim3(SCAN_THREADS), 0, st, src, kept, dst, reserve, align, ctx->shape, ctx->ws, 0, g);
        hipLaunchKernelGGL(k_cmp_scan<true>, dim3(ctx->shape.nseg), dim3(SCAN_THREADS), 0, st, src, keep, kept, dst, reserve,
                           align, ctx->shape, ctx->ws, 0, g);
    } else {
        hipLaunchKernelGGL(k_cmp_scan<false>, dim3(ctx->shape.nseg), dim3(SCAN_THREADS), 0, st, src, keep, kept, dst, reserve,
                           align, ctx->shape, ctx->ws, 0, g);
    }
}

// The tables for a compaction inside the cache itself: every segment keeps its start, chunk ch's survivors go to
// ws.cmp_chunk_dst[ch] = seg_start + survivors of the segment's earlier chunks; nothing of the cache is written.
void launch_cmp_scan_inplace(kvtrim_ctx* ctx, const CacheViewMut& c, const uint8_t* keep, const int32_t* kept, hipStream_t st) {
    ProfScope prof(ctx, K_CMP_SCAN, st);
    CacheView src;
    src.k = c.k; src.v = c.v; src.log_beta = c.log_beta; src.pos = c.pos;
    src.seg_start = c.seg_start; src.seg_len = c.seg_len; src.cap = c.cap; src.log_tail = c.log_tail;
    if (ctx->shape.nseg > 1024) {
        hipLaunchKernelGGL(k_cmp_prefix, dim3(1), dim3(SCAN_THREADS), 0, st, src, kept, c, 0, 1, ctx->shape, ctx->ws, 1, 0);
        hipLaunchKernelGGL(k_cmp_scan<true>, dim3(ctx->shape.nseg), dim3(SCAN_THREADS), 0, st, src, keep, kept, c, 0, 1,
                           ctx->shape, ctx->ws, 1, 0);
    } else {
        hipLaunchKernelGGL(k_cmp_scan<false>, dim3(ctx->shape.nseg), dim3(SCAN_THREADS), 0, st, src, keep, kept, c, 0, 1,
                           ctx->shape, ctx->ws, 1, 0);
    }
}

void launch_cmp_scan(kvtrim_ctx* ctx, const CacheView& src, const uint8_t* keep, const int32_t* kept,
                     const CacheViewMut& dst, int32_t reserve, hipStream_t st) {
    launch_cmp_scan_aligned(ctx, src, keep, kept, dst, reserve, 1, st);
}

kvtrim_status launch_compact(kvtrim_ctx* ctx, const CacheView& src, const uint8_t* keep, const int32_t* kept,
                             const CacheViewMut& dst, int32_t reserve, hipStream_t st) {
    launch_cmp_scan_aligned(ctx, src, keep, kept, dst, reserve, 1, st, gather_fits(ctx, src.cap, dst.cap));
    return launch_cmp_copy(ctx, src, keep, dst, st);
}

// The row mover alone (the tables of k_cmp_scan must be in the workspace - with gat = gather_fits(...), which decides
// here which mover runs).
kvtrim_status launch_cmp_copy(kvtrim_ctx* ctx, const CacheView& src, const uint8_t* keep, const CacheViewMut& dst,
                              hipStream_t st) {
    const Shape& sh = ctx->shape;
    const Workspace& ws = ctx->ws;
    const int64_t max_chunks = src.cap / CMP_CHUNK + sh.nseg;
    if (max_chunks > 0) {
        ProfScope prof(ctx, K_CMP_COPY, st);
        const dim3 grid((unsigned)max_chunks), block(CMP_THREADS);
        if (gather_fits(ctx, src.cap, dst.cap))                   // few survivors per chunk: a block per chunk of the destination
            return launch_gather_rows(ctx, src, dst, st);
        if (sh.head_dim == 128)
            hipLaunchKernelGGL((k_cmp_copy<128, false>), grid, block, 0, st, src, keep, dst, sh, ws, nullptr, nullptr, 0, nullptr);
        else
            hipLaunchKernelGGL((k_cmp_copy<64, false>), grid, block, 0, st, src, keep, dst, sh, ws, nullptr, nullptr, 0, nullptr);
    }
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

kvtrim_status launch_cmp_copy_new(kvtrim_ctx* ctx, const CacheView& src, const uint8_t* keep, const CacheViewMut& dst,
                                  const uint16_t* k_new, const uint16_t* v_new, int32_t n_new, const int32_t* old_len,
                                  hipStream_t st) {
    const Shape& sh = ctx->shape;
    const Workspace& ws = ctx->ws;
    const int64_t max_chunks = src.cap / CMP_CHUNK + sh.nseg;
    if (max_chunks > 0) {
        ProfScope prof(ctx, K_CMP_COPY, st);
        const dim3 grid((unsigned)max_chunks), block(CMP_THREADS);
        if (sh.head_dim == 128)
            hipLaunchKernelGGL((k_cmp_copy<128, true>), grid, block, 0, st, src, keep, dst, sh, ws, k_new, v_new, n_new, old_len);
        else
            hipLaunchKernelGGL((k_cmp_copy<64, true>), grid, block, 0, st, src, keep, dst, sh, ws, k_new, v_new, n_new, old_len);
    }
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

}  // namespace kvtrim
