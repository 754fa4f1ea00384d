// Stage 3: stable stream compaction of the retained entries into a tight ragged cache.
//
// k_cmp_scan  one block per segment: counts the mask per 256-entry chunk, scans the counts
//             inside the segment and derives the destination segment table from `kept`.
// k_cmp_copy  one block per chunk: wavefront ballot/prefix ranks the survivors and the
//             rows are streamed 16 bytes per lane, whole rows per 16 (D=128) or 8 (D=64) lanes.
#include "kvtrim_device.h"

namespace kvtrim {

constexpr int CMP_THREADS = 256;

__global__ __launch_bounds__(CMP_THREADS) void k_cmp_scan(CacheView src, const uint8_t* __restrict__ keep,
                                                          const int32_t* __restrict__ kept, CacheViewMut dst,
                                                          int reserve, Shape sh, Workspace ws) {
    __shared__ int64_t lds64[17];
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int g = blockIdx.x;
    const int nseg = sh.nseg;

    // chunks and destination entries of the segments before g, and the totals
    int64_t chunks_before = 0, dst_before = 0, dst_total = 0, chunks_total = 0;
    int64_t bad_layout = 0, bad_kept = 0;
    for (int i = tid; i < nseg; i += CMP_THREADS) {
        const int len = src.seg_len[i];
        const int64_t st = src.seg_start[i];
        const int kp = kept[i];
        bad_layout |= (len < 0 || st < 0 || st + len > src.cap);
        bad_kept |= (kp < 0 || kp > len);
        const int64_t nch = len > 0 ? (len + CMP_CHUNK - 1) / CMP_CHUNK : 0;
        const int64_t need = (int64_t)kp + reserve;
        chunks_total += nch;
        dst_total += need;
        if (i < g) {
            chunks_before += nch;
            dst_before += need;
        }
    }
    chunks_before = block_sum<int64_t>(chunks_before, lds64);
    dst_before = block_sum<int64_t>(dst_before, lds64);
    dst_total = block_sum<int64_t>(dst_total, lds64);
    chunks_total = block_sum<int64_t>(chunks_total, lds64);
    bad_layout = block_sum<int64_t>(bad_layout, lds64);
    bad_kept = block_sum<int64_t>(bad_kept, lds64);
    if (bad_layout || chunks_total > ws.max_cmp_chunks) {
        bad_layout = 1;
    }
    if (bad_layout || bad_kept || dst_total > dst.cap) {       // every block takes the same decision
        if (tid == 0) {
            atomicOr(ws.err, bad_layout ? ERR_LAYOUT : (bad_kept ? ERR_MISMATCH : ERR_CAP));
            if (g == 0) ws.cmp_chunk_prefix[nseg] = 0;
        }
        return;
    }

    const int len = src.seg_len[g];
    const int nch = len > 0 ? (len + CMP_CHUNK - 1) / CMP_CHUNK : 0;
    const uint8_t* kp = keep + src.seg_start[g];
    const int cbase = (int)chunks_before;

    // phase 1: survivors per chunk (one wavefront per chunk, four coalesced byte loads)
    for (int ch = wave; ch < nch; ch += CMP_THREADS / 64) {
        int cnt = 0;
#pragma unroll
        for (int r = 0; r < CMP_CHUNK / 64; ++r) {
            const int j = ch * CMP_CHUNK + r * 64 + lane;
            const bool f = j < len && kp[j] != 0;
            cnt += __popcll(__ballot(f));
        }
        if (lane == 0) {
            ws.cmp_chunk_dst[cbase + ch] = cnt;
            ChunkDesc d;
            d.first = src.seg_start[g] + (int64_t)ch * CMP_CHUNK;
            d.n = min(CMP_CHUNK, len - ch * CMP_CHUNK);
            d.seg = g;
            ws.cmp_desc[cbase + ch] = d;
        }
    }
    __syncthreads();
    // phase 2: exclusive scan of the counts inside the segment
    int64_t running = 0;
    for (int base = 0; base < nch; base += CMP_THREADS) {
        const int ch = base + tid;
        const int64_t v = ch < nch ? ws.cmp_chunk_dst[cbase + ch] : 0;
        int64_t tot;
        const int64_t ex = block_excl_scan<int64_t>(v, lds64, &tot);
        if (ch < nch) ws.cmp_chunk_dst[cbase + ch] = dst_before + running + ex;
        running += tot;
    }
    if (tid == 0) {
        if (running != kept[g]) atomicOr(ws.err, ERR_MISMATCH);
        dst.seg_start[g] = dst_before;
        dst.seg_len[g] = kept[g];
        ws.cmp_chunk_prefix[g] = cbase;
        if (g == nseg - 1) ws.cmp_chunk_prefix[nseg] = cbase + nch;
    }
}

typedef unsigned v4u __attribute__((ext_vector_type(4)));

template <bool NT>
__device__ __forceinline__ uint4 ld16(const uint4* p) {
    if (NT) {
        v4u t = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p));
        return make_uint4(t.x, t.y, t.z, t.w);
    }
    return *p;
}
template <bool NT>
__device__ __forceinline__ void st16(uint4* p, uint4 v) {
    if (NT) {
        v4u t = {v.x, v.y, v.z, v.w};
        __builtin_nontemporal_store(t, reinterpret_cast<v4u*>(p));
    } else {
        *p = v;
    }
}

template <int D, int UNROLL, bool NT>
__global__ __launch_bounds__(CMP_THREADS) void k_cmp_copy(CacheView src, const uint8_t* __restrict__ keep,
                                                          CacheViewMut dst, Shape sh, Workspace ws) {
    constexpr int VPR = D / 8;            // 16-byte vectors per row
    constexpr int RPI = 64 / VPR;         // rows moved by one wavefront instruction
    __shared__ int wave_cnt[4];
    __shared__ int list[4][64];
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    if (__hip_atomic_load(ws.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
    const int total = ws.cmp_chunk_prefix[sh.nseg];
    const int ch = blockIdx.x;
    if (ch >= total) return;
    const ChunkDesc d = ws.cmp_desc[ch];
    const int64_t sbase = d.first;                                // first source entry of the chunk
    const bool flag = tid < d.n && keep[sbase + tid] != 0;
    const uint64_t mask = __ballot(flag);
    const int rank = mbcnt(mask);
    const int cnt = __popcll(mask);
    if (lane == 0) wave_cnt[wave] = cnt;
    if (flag) list[wave][rank] = tid;
    __syncthreads();
    int wbase = 0;
    for (int w = 0; w < wave; ++w) wbase += wave_cnt[w];
    const int64_t dbase = ws.cmp_chunk_dst[ch] + wbase;           // first destination entry of this wavefront
    if (flag) {
        dst.log_beta[dbase + rank] = src.log_beta[sbase + tid];
        dst.pos[dbase + rank] = src.pos[sbase + tid];
    }
    const uint4* sk = reinterpret_cast<const uint4*>(src.k);
    const uint4* sv = reinterpret_cast<const uint4*>(src.v);
    uint4* dk = reinterpret_cast<uint4*>(dst.k);
    uint4* dv = reinterpret_cast<uint4*>(dst.v);
    const int sub = lane / VPR, col = lane % VPR;
    for (int r0 = 0; r0 < cnt; r0 += RPI * UNROLL) {
        uint4 kk[UNROLL], vv[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int r = r0 + u * RPI + sub;
            if (r < cnt) {
                const int64_t se = (sbase + list[wave][r]) * VPR + col;
                kk[u] = ld16<NT>(sk + se);
                vv[u] = ld16<NT>(sv + se);
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int r = r0 + u * RPI + sub;
            if (r < cnt) {
                const int64_t de = (dbase + r) * VPR + col;
                st16<NT>(dk + de, kk[u]);
                st16<NT>(dv + de, vv[u]);
            }
        }
    }
}

void launch_cmp_scan(kvtrim_ctx* ctx, const CacheView& src, const uint8_t* keep, const int32_t* kept,
                     const CacheViewMut& dst, int32_t reserve, hipStream_t st) {
    ProfScope prof(ctx, K_CMP_SCAN, st);
    hipLaunchKernelGGL(k_cmp_scan, dim3(ctx->shape.nseg), dim3(CMP_THREADS), 0, st, src, keep, kept, dst, reserve,
                       ctx->shape, ctx->ws);
}

kvtrim_status launch_compact(kvtrim_ctx* ctx, const CacheView& src, const uint8_t* keep, const int32_t* kept,
                             const CacheViewMut& dst, int32_t reserve, hipStream_t st) {
    const Shape& sh = ctx->shape;
    const Workspace& ws = ctx->ws;
    const int64_t max_chunks = src.cap / CMP_CHUNK + sh.nseg;
    launch_cmp_scan(ctx, src, keep, kept, dst, reserve, st);
    if (max_chunks > 0) {
        ProfScope prof(ctx, K_CMP_COPY, st);
        const dim3 grid((unsigned)max_chunks), block(CMP_THREADS);
#define KVTRIM_COPY(D_, U_, NT_) hipLaunchKernelGGL((k_cmp_copy<D_, U_, NT_>), grid, block, 0, st, src, keep, dst, sh, ws)
#define KVTRIM_COPY_U(D_, NT_)                                       \
    switch (ctx->cmp_unroll) {                                       \
        case 1: KVTRIM_COPY(D_, 1, NT_); break;                      \
        case 2: KVTRIM_COPY(D_, 2, NT_); break;                      \
        default: KVTRIM_COPY(D_, 4, NT_); break;                     \
    }
        if (sh.head_dim == 128) {
            if (ctx->cmp_nt) { KVTRIM_COPY_U(128, true) } else { KVTRIM_COPY_U(128, false) }
        } else {
            if (ctx->cmp_nt) { KVTRIM_COPY_U(64, true) } else { KVTRIM_COPY_U(64, false) }
        }
#undef KVTRIM_COPY_U
#undef KVTRIM_COPY
    }
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

}  // namespace kvtrim
