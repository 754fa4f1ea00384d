// Device code of the paged layout that more than one kernel file uses: the view of a paged cache, the chunk
// table over its block tables, and the tidying of a block table after an eviction.
#pragma once
#include "kvtrim_device.h"

namespace kvtrim {

constexpr int P = KVTRIM_PAGE_SIZE;

struct PagedView {
    uint16_t* k;
    uint16_t* v;
    float* log_beta;
    int32_t* pos;
    float* log_tail;
    int32_t* block_table;
    int32_t* seg_pages;
    int32_t* seg_live;
    int32_t* page_owner;
    int32_t* page_live;
    int32_t* free_list;
    int32_t* n_free;
    int32_t n_pages;
    int32_t max_pps;
};

constexpr int PG_TABLE_BLOCKS = 16;        // blocks that share the building of a chunk table
constexpr int ATT_PAGE_GROUP = 4;          // pages per attention chunk (512 rows, the ragged path's chunk)

// ---------------------------------------------------------------------------------------------
// Chunk table of a paged cache: the pages of every segment with in_range(g), in segment order,
// GROUP pages to a chunk.  prefix[g] = first chunk of segment g, prefix[nseg] = number of chunks;
// entry_prefix (optional) counts the live entries of the segments before g.
//   GROUP == 1: desc = {first slot of the page, page size, segment}           (selection)
//   GROUP  > 1: desc = {index of the group's first block-table entry, slots of the group, segment},
//               pages_out[chunk][GROUP] = the group's pages (clamped into the pool), so that the reader
//               has them with the descriptor and not one dependent load later  (attention)
// Built by `nparts` blocks: every block scans the per-segment counts (a few thousand integers),
// block `part` fills the descriptors of the segments g = part (mod nparts), one wavefront per
// segment, and block 0 writes the prefixes (slot_prefix, optional: the slots - pages times the page size - of the
// in-range segments before g).  Returns the number of chunks.  Counts that do not
// fit raise ERR_LAYOUT and leave the table empty; a page id out of range raises it too and is
// clamped, so that no reader leaves the pool.
template <int GROUP, typename InRange>
__device__ __forceinline__ int build_page_table(const PagedView& pc, int nseg, InRange in_range, int32_t* prefix,
                                                ChunkDesc* desc, int64_t max_chunks, int64_t* entry_prefix,
                                                int32_t* err, int part, int nparts, int32_t* pages_out = nullptr,
                                                int64_t* slot_prefix = nullptr) {
    __shared__ uint64_t s_scan[17];
    __shared__ int s_bad;
    __shared__ int s_c0[1024], s_n[1024];
    const int tid = threadIdx.x;
    if (tid == 0) s_bad = 0;
    __syncthreads();
    uint64_t carry = 0, slot_carry = 0;
    for (int base = 0; base < nseg; base += blockDim.x) {
        const int g = base + tid;
        uint64_t v = 0;
        int npg = 0;
        if (g < nseg) {
            npg = pc.seg_pages[g];
            const int live = pc.seg_live[g];
            if (npg < 0 || npg > pc.max_pps || live < 0 || (int64_t)live > (int64_t)npg * P) {
                s_bad = 1;
                npg = 0;
            } else if (in_range(g)) {
                v = ((uint64_t)live << 32) | (uint64_t)((npg + GROUP - 1) / GROUP);
            } else {
                npg = 0;
            }
        }
        uint64_t tot;
        const uint64_t ex = carry + block_excl_scan<uint64_t>(v, s_scan, &tot);
        carry += tot;
        const int c0 = (int)(ex & 0xffffffffu);
        if (g < nseg && part == 0) {
            prefix[g] = c0;
            if (entry_prefix) entry_prefix[g] = (int64_t)(ex >> 32);
        }
        if (slot_prefix) {                                           // slots of the in-range segments before g
            uint64_t stot;
            const uint64_t sex = slot_carry + block_excl_scan<uint64_t>((uint64_t)npg * P, s_scan, &stot);
            slot_carry += stot;
            if (g < nseg && part == 0) slot_prefix[g] = (int64_t)sex;
        }
        s_c0[tid] = c0;
        s_n[tid] = npg;
        __syncthreads();
        if (!s_bad && (int64_t)(carry & 0xffffffffu) <= max_chunks) {
            const int lane = lane_id(), wave = tid >> 6, nw = blockDim.x >> 6;
            const int ntile = min((int)blockDim.x, nseg - base);
            const int first_t = ((part - base) % nparts + nparts) % nparts;      // first t with (base + t) = part (mod nparts)
            for (int t = first_t + wave * nparts; t < ntile; t += nw * nparts) {
                const int gg = base + t, cc = s_c0[t], nn = s_n[t];
                const int64_t row = (int64_t)gg * pc.max_pps;
                bool bad_page = false;
                for (int i = lane; i < nn; i += 64) {
                    const int pg = pc.block_table[row + i];
                    bad_page |= pg < 0 || pg >= pc.n_pages;
                    ChunkDesc d;
                    d.seg = gg;
                    if (GROUP == 1) {
                        d.first = (int64_t)min(max(pg, 0), pc.n_pages - 1) * P;
                        d.n = P;
                        desc[cc + i] = d;
                    } else {
                        if (pages_out) pages_out[(int64_t)(cc + i / GROUP) * GROUP + i % GROUP] = min(max(pg, 0), pc.n_pages - 1);
                        if (i % GROUP == 0) {
                            d.first = row + i;
                            d.n = P * min(GROUP, nn - i);
                            desc[cc + i / GROUP] = d;
                        }
                    }
                }
                if (__any(bad_page) && lane == 0) atomicOr(err, ERR_LAYOUT);
            }
        }
        __syncthreads();
    }
    const int64_t total = (int64_t)(carry & 0xffffffffu);
    if (s_bad || total > max_chunks) {
        if (part == 0) {
            if (tid == 0) atomicOr(err, ERR_LAYOUT);
            for (int g = tid; g <= nseg; g += blockDim.x) {
                prefix[g] = 0;
                if (entry_prefix) entry_prefix[g] = 0;
                if (slot_prefix) slot_prefix[g] = 0;
            }
        }
        __syncthreads();
        return 0;
    }
    if (tid == 0 && part == 0) {
        prefix[nseg] = (int32_t)total;
        if (entry_prefix) entry_prefix[nseg] = (int64_t)(carry >> 32);
        if (slot_prefix) slot_prefix[nseg] = (int64_t)slot_carry;
    }
    __syncthreads();
    return (int)total;
}

// A block of THREADS threads tidies segment g: the pages marked for release leave its block table (order of
// the others kept) and return to the free list.  A released page that is still in the table is harmless to a
// reader - every slot of it is empty - so this may run any time after the eviction and before the next append.
template <int THREADS>
__device__ __forceinline__ void tidy_segment(const PagedView& pc, int g, int32_t* err) {
    __shared__ int32_t lds32[17];
    __shared__ int32_t s_page[THREADS];
    const int tid = threadIdx.x;
    const int npg = pc.seg_pages[g];
    if (npg < 0 || npg > pc.max_pps) {
        if (tid == 0) atomicOr(err, ERR_LAYOUT);
        return;
    }
    int32_t* bt = pc.block_table + (int64_t)g * pc.max_pps;
    int out = 0;
    for (int base = 0; base < npg; base += THREADS) {                    // read a tile, then write it: out <= base
        const int i = base + tid;
        int page = -1;
        bool alive = false;
        if (i < npg) {
            page = bt[i];
            if (page >= 0 && page < pc.n_pages) {
                alive = pc.page_owner[page] == g;
                if (!alive && pc.page_owner[page] == -2) {          // release
                    pc.page_owner[page] = -1;
                    pc.page_live[page] = 0;
                    const int idx = atomicAdd(pc.n_free, 1);
                    if (idx >= 0 && idx < pc.n_pages) pc.free_list[idx] = page;
                }
            }
        }
        int32_t tot;
        const int32_t ex = block_excl_scan<int32_t>(alive ? 1 : 0, lds32, &tot);
        s_page[tid] = page;
        __syncthreads();
        if (alive) bt[out + ex] = s_page[tid];
        __syncthreads();
        out += tot;
    }
    if (tid == 0) pc.seg_pages[g] = out;
}

}  // namespace kvtrim
