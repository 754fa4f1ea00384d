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

// Chunk table of a ragged cache, built by ONE block: segment g with in_range(g) has
// ceil(seg_len[g] / chunk) chunks (0 for the other segments);
// prefix[g] = first chunk of segment g, prefix[nseg] = number of chunks, chunk_seg[c] = segment
// of chunk c.  Also checks every segment against `cap` and the chunk count against `max_chunks`
// (ERR_LAYOUT; the table is then left empty).  `lds64` needs 17 int64.
template <typename InRange>
__device__ __forceinline__ void build_chunk_table(const int32_t* __restrict__ seg_len,
                                                  const int64_t* __restrict__ seg_start, int nseg,
                                                  InRange in_range, int chunk, int64_t cap,
                                                  int32_t* prefix, int32_t* chunk_seg, int64_t max_chunks,
                                                  int32_t* err, int64_t* lds64) {
    __shared__ int bad;
    if (threadIdx.x == 0) bad = 0;
    __syncthreads();
    int64_t carry = 0;
    for (int base = 0; base < nseg; base += blockDim.x) {
        int g = base + threadIdx.x;
        int64_t n = 0;
        if (g < nseg) {
            int len = seg_len[g];
            int64_t st = seg_start[g];
            int64_t nxt = (g + 1 < nseg) ? seg_start[g + 1] : cap;
            if (len < 0 || st < 0 || st + len > cap || st + len > nxt) bad = 1;
            if (in_range(g) && len > 0) n = (len + chunk - 1) / chunk;
        }
        int64_t tot;
        int64_t ex = block_excl_scan<int64_t>(n, lds64, &tot);
        if (g < nseg) prefix[g] = (int32_t)min(carry + ex, (int64_t)0x7fffffff);
        carry += tot;
    }
    __syncthreads();
    if (bad || carry > max_chunks) {
        if (threadIdx.x == 0) atomicOr(err, ERR_LAYOUT);
        for (int g = threadIdx.x; g <= nseg; g += blockDim.x) prefix[g] = 0;
        __syncthreads();
        return;
    }
    if (threadIdx.x == 0) prefix[nseg] = (int32_t)carry;
    __syncthreads();
    // one wavefront per segment, lanes stride over its chunks
    const int lane = lane_id(), wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    for (int g = wave; g < nseg; g += nw) {
        if (!in_range(g)) continue;
        int c0 = prefix[g];
        int len = seg_len[g];
        int n = len > 0 ? (len + chunk - 1) / chunk : 0;
        for (int i = lane; i < n; i += 64) chunk_seg[c0 + i] = g;
    }
    __syncthreads();
}

}  // namespace kvtrim
