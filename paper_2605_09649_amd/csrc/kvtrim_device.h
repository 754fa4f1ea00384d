// Block-level device utilities: scans, reductions, the chunk table of a ragged cache.
#pragma once
#include "kvtrim_internal.h"

namespace kvtrim {

// Inclusive scan over the 64 lanes of a wavefront.
template <typename T>
__device__ __forceinline__ T wave_incl_scan(T v) {
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        T o = __shfl_up(v, d, 64);
        if (lane >= d) v += o;
    }
    return v;
}

template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// Exclusive scan over the threads of a block (blockDim.x a multiple of 64, at most 1024).
// `lds` needs 17 elements.  Returns the exclusive prefix; *total gets the block sum.
template <typename T>
__device__ __forceinline__ T block_excl_scan(T v, T* lds, T* total) {
    const int lane = lane_id(), wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    T inc = wave_incl_scan(v);
    __syncthreads();                       // lds may still be read from a previous call
    if (lane == 63) lds[wave] = inc;
    __syncthreads();
    if (wave == 0) {
        T w = lane < nw ? lds[lane] : T(0);
        T wi = wave_incl_scan(w);
        if (lane < nw) lds[lane] = wi - w; // exclusive wave offsets
        if (lane == nw - 1) lds[16] = wi;
    }
    __syncthreads();
    *total = lds[16];
    return lds[wave] + inc - v;
}

template <typename T>
__device__ __forceinline__ T block_sum(T v, T* lds) {
    const int lane = lane_id(), wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    v = wave_sum(v);
    __syncthreads();
    if (lane == 0) lds[wave] = v;
    __syncthreads();
    T s = T(0);
    for (int i = 0; i < nw; ++i) s += lds[i];
    return s;
}

// "Last block done" detection, called by one thread per block after the block's results are
// written.  Device-scope atomics on ONE address are served one after the other (tens of
// nanoseconds each), so 256 blocks do not meet on one counter: 16 group counters first, then the
// last block of each group on the top-level counter.  counters: [0] top level, [1..16] groups.
__device__ __forceinline__ bool arrive_last(uint32_t* counters) {
    __threadfence();
    const unsigned grp = blockIdx.x & 15u;
    const unsigned gsize = (gridDim.x - grp + 15u) / 16u;        // blocks with this group number
    if (atomicAdd(&counters[1 + grp], 1u) != gsize - 1) return false;
    __threadfence();
    const unsigned ngroups = gridDim.x < 16u ? gridDim.x : 16u;
    return atomicAdd(&counters[0], 1u) == ngroups - 1;
}

// Calls body(seq) - by all threads of the block, one sequence after the other - for every sequence whose ties at
// the threshold have to be ranked (need_rank in its final selection state).  The flags of blockDim.x sequences
// are read at once, so a batch of many sequences of which few (usually none) need it costs one round of loads
// instead of one dependent load per sequence.  s_list needs blockDim.x elements.
template <typename Body>
__device__ __forceinline__ void for_each_ranked_seq(const SelState* __restrict__ sel, int n_seq, int* s_list, int* s_n,
                                                    Body body) {
    for (int base = 0; base < n_seq; base += blockDim.x) {
        __syncthreads();
        if (threadIdx.x == 0) *s_n = 0;
        __syncthreads();
        const int sq = base + threadIdx.x;
        if (sq < n_seq && sel[sq].need_rank) s_list[atomicAdd(s_n, 1)] = sq;
        __syncthreads();
        const int n = *s_n;
        for (int k = 0; k < n; ++k) body(s_list[k]);
    }
}

// Chunk table of a ragged cache, built by ONE block (blockDim.x <= 1024): segment g with
// in_range(g) is cut into ceil(seg_len[g] / chunk) chunks (none for the other segments);
// prefix[g] = first chunk of segment g, prefix[nseg] = number of chunks, desc[c] = entries and
// segment of chunk c.  Returns the number of chunks.  Every segment is checked against `cap`
// and its successor, the chunk count against `max_chunks` (ERR_LAYOUT; the table is then left
// empty).  Optionally writes entry_prefix[g] = entries of the in-range segments before g
// (entry_prefix[nseg] = all of them).
// Segments with few chunks are filled by the thread that scanned them; long ones are queued
// in LDS and filled by whole wavefronts.  The table may be built by `nparts` blocks: every block
// scans all segments, block `part` fills the descriptors of the segments g = part (mod nparts),
// and block 0 writes the prefixes.
template <typename InRange>
__device__ __forceinline__ int build_chunk_table(const int32_t* __restrict__ seg_len,
                                                 const int64_t* __restrict__ seg_start, int nseg,
                                                 InRange in_range, int chunk, int64_t cap,
                                                 int32_t* prefix, ChunkDesc* desc, int64_t max_chunks,
                                                 int64_t* entry_prefix, int32_t* err, int part = 0, int nparts = 1) {
    constexpr int SMALL = 16;
    __shared__ uint64_t s_scan[17];
    __shared__ int s_bad, s_nbig;
    __shared__ int s_big_g[1024], s_big_c0[1024];
    if (threadIdx.x == 0) s_bad = 0;
    __syncthreads();
    // pass 1: validate and count (chunks in the low, entries in the high 32 bits of one scan)
    uint64_t carry = 0;
    for (int base = 0; base < nseg; base += blockDim.x) {
        const int g = base + threadIdx.x;
        uint64_t v = 0;
        if (g < nseg) {
            const int len = seg_len[g];
            const int64_t st = seg_start[g];
            const int64_t nxt = (g + 1 < nseg) ? seg_start[g + 1] : cap;
            if (len < 0 || st < 0 || st + len > cap || st + len > nxt) s_bad = 1;
            else if (in_range(g) && len > 0) v = ((uint64_t)len << 32) | (uint64_t)(((int64_t)len + chunk - 1) / chunk);
        }
        uint64_t tot;
        block_excl_scan<uint64_t>(v, s_scan, &tot);
        carry += tot;
    }
    __syncthreads();
    const int64_t total = (int64_t)(carry & 0xffffffffu);
    if (s_bad || total > max_chunks || (carry >> 32) > (uint64_t)cap) {
        if (threadIdx.x == 0) atomicOr(err, ERR_LAYOUT);
        if (part == 0) {
            for (int g = threadIdx.x; g <= nseg; g += blockDim.x) {
                prefix[g] = 0;
                if (entry_prefix) entry_prefix[g] = 0;
            }
        }
        __syncthreads();
        return 0;
    }
    // pass 2: prefixes and descriptors
    carry = 0;
    for (int base = 0; base < nseg; base += blockDim.x) {
        const int g = base + threadIdx.x;
        uint64_t v = 0;
        int len = 0;
        int64_t st = 0;
        if (g < nseg) {
            len = seg_len[g];
            st = seg_start[g];
            if (in_range(g) && len > 0) v = ((uint64_t)len << 32) | (uint64_t)(((int64_t)len + chunk - 1) / chunk);
        }
        if (threadIdx.x == 0) s_nbig = 0;
        uint64_t tot;
        const uint64_t ex = carry + block_excl_scan<uint64_t>(v, s_scan, &tot);
        carry += tot;
        const int c0 = (int)(ex & 0xffffffffu);
        const int n = (int)(v & 0xffffffffu);
        if (g < nseg && part == 0) {
            prefix[g] = c0;
            if (entry_prefix) entry_prefix[g] = (int64_t)(ex >> 32);
        }
        if (g < nseg && g % nparts == part) {
            if (n > SMALL) {
                const int slot = atomicAdd(&s_nbig, 1);
                s_big_g[slot] = g;
                s_big_c0[slot] = c0;
            } else {
                for (int i = 0; i < n; ++i) {
                    ChunkDesc d;
                    d.first = st + (int64_t)i * chunk;
                    d.n = min(chunk, len - i * chunk);
                    d.seg = g;
                    desc[c0 + i] = d;
                }
            }
        }
        __syncthreads();
        const int lane = lane_id(), wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
        for (int b = wave; b < s_nbig; b += nw) {
            const int gg = s_big_g[b], cc = s_big_c0[b];
            const int ll = seg_len[gg];
            const int64_t ss = seg_start[gg];
            const int nn = (int)(((int64_t)ll + chunk - 1) / chunk);
            for (int i = lane; i < nn; i += 64) {
                ChunkDesc d;
                d.first = ss + (int64_t)i * chunk;
                d.n = min(chunk, ll - i * chunk);
                d.seg = gg;
                desc[cc + i] = d;
            }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0 && part == 0) {
        prefix[nseg] = (int32_t)(carry & 0xffffffffu);
        if (entry_prefix) entry_prefix[nseg] = (int64_t)(carry >> 32);
    }
    __syncthreads();
    return (int)total;
}

// After the in-place row mover: the survivors of chunk `ch` whose place lies before the chunk's own range (as many
// as were evicted before the chunk in its segment, at most all of its survivors) wait in `stage` at their final
// index; the calling wavefront puts them there (in a decode step most chunks have nothing parked and the call
// returns at once).  The wavefront of a segment's first chunk also commits the segment's new length, which no
// kernel of the call reads any more.
template <int D>
__device__ __forceinline__ void unstage_chunk(const CacheViewMut& c, const CacheViewMut& stage, const int32_t* __restrict__ kept,
                                              const Shape& sh, const Workspace& ws, int ch) {
    constexpr int VPR = D / 8;                                    // 16-byte vectors per row
    const int lane = lane_id();
    if (__hip_atomic_load(ws.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
    if (ch >= ws.cmp_chunk_prefix[sh.nseg]) return;
    const ChunkDesc cd = ws.cmp_desc[ch];
    const int seg = cd.seg;
    const int64_t dbase = ws.cmp_chunk_dst[ch] & ~CMP_DST_FULL;
    const int first_ch = ws.cmp_chunk_prefix[seg];
    if (ch == first_ch && lane == 0) c.seg_len[seg] = kept[seg];
    if (cd.first == dbase) return;                                // nothing was evicted before this chunk
    const bool last = ch + 1 >= ws.cmp_chunk_prefix[seg + 1];
    const int64_t dnext = last ? c.seg_start[seg] + kept[seg] : (ws.cmp_chunk_dst[ch + 1] & ~CMP_DST_FULL);
    const int64_t staged = min(cd.first - dbase, dnext - dbase);  // survivors that belong before the chunk's own range
    const uint4* sk = reinterpret_cast<const uint4*>(stage.k) + dbase * VPR;
    const uint4* sv = reinterpret_cast<const uint4*>(stage.v) + dbase * VPR;
    uint4* dk = reinterpret_cast<uint4*>(c.k) + dbase * VPR;
    uint4* dv = reinterpret_cast<uint4*>(c.v) + dbase * VPR;
    for (int64_t i = lane; i < staged * VPR; i += 64) {
        dk[i] = sk[i];
        dv[i] = sv[i];
    }
    for (int64_t i = lane; i < staged; i += 64) {
        c.log_beta[dbase + i] = stage.log_beta[dbase + i];
        if (c.log_tail) c.log_tail[dbase + i] = stage.log_tail[dbase + i];
        c.pos[dbase + i] = stage.pos[dbase + i];
    }
}

}  // namespace kvtrim
