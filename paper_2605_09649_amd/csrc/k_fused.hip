// Stages 3 + 4 in one pass over the retained rows: while a surviving K/V row travels from
// the source cache to its slot in the compacted cache it is also used for the decode
// attention of its segment (Sec. 2.1, Eq. reform with r in {0,1}), so K and V are read from
// HBM once per step instead of twice.  Result is the same as compaction followed by
// attention over the compacted cache.
//
// One block of 8 wavefronts per 128-entry chunk of a source segment (the chunk table and the
// destination offsets come from k_cmp_scan).  A ballot/prefix over the chunk's mask ranks the
// survivors (a chunk that k_cmp_scan has marked as losing nothing skips the mask and the ranks
// and asks for its rows at once: 0.378 -> 0.371 ms at the long-context workload, where a step
// evicts 256 of 2.1 M entries); every wavefront then takes at most 16 of them, moves them with ONE batch of
// loads and one batch of stores, four rows per instruction (16 lanes x 16 bytes = one
// 256-byte row, so loads and stores are whole rows), and ends - short-lived wavefronts
// measured ~10 % faster on this chip than wavefronts that loop over several batches.  In
// that layout a lane owns the same 8-element column slice of the K rows and of the V rows of 4 rows:
//   q.k   4 packed two-element bf16 dot products per query head, row and lane, then a 16-lane
//         all-reduce with DPP
//   p.v   one MFMA per column of the slice: the lane's 4 rows are 4 consecutive slots of the
//         reduction dimension, and the MFMA sums over the wavefront's 16 rows for all query heads
// A wavefront takes one softmax partial per query head over its 16 rows; the wavefronts of the
// block are merged through LDS, and the chunks of a segment by k_att_combine.
//
// The same kernel has an instance that compacts INSIDE the cache (segments keep their starts; only the rows
// behind an eviction move), followed by k_cmp_unstage; k_cmp_move_inplace is that instance without the
// attention (it is bracketed under the row mover's name, k_cmp_copy, when kernels are timed).
#include "kvtrim_device.h"

namespace kvtrim {

constexpr int FUS_THREADS = CMP_THREADS;

typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

// acc + a.lo * b.lo + a.hi * b.hi on a pair of packed bf16 values (products and sum in fp32)
__device__ __forceinline__ float dot2_bf16(unsigned a, unsigned b, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), acc, false);
}

template <int D>
struct Row;
template <>
struct Row<128> {
    typedef uint4 vec;
    static constexpr int E = 8;
    static __device__ __forceinline__ vec ld(const vec* p) {
        v4u t = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p));
        return make_uint4(t.x, t.y, t.z, t.w);
    }
    static __device__ __forceinline__ void st(vec* p, vec v) {
        v4u t = {v.x, v.y, v.z, v.w};
        __builtin_nontemporal_store(t, reinterpret_cast<v4u*>(p));
    }
    static __device__ __forceinline__ unsigned word(vec x, int w) { return w == 0 ? x.x : (w == 1 ? x.y : (w == 2 ? x.z : x.w)); }
    static __device__ __forceinline__ float dot(vec a, vec b) {   // the lane's 8-element slice of q . k
        return dot2_bf16(a.w, b.w, dot2_bf16(a.z, b.z, dot2_bf16(a.y, b.y, dot2_bf16(a.x, b.x, 0.f))));
    }
};
template <>
struct Row<64> {
    typedef uint2 vec;
    static constexpr int E = 4;
    static __device__ __forceinline__ vec ld(const vec* p) {
        v2u t = __builtin_nontemporal_load(reinterpret_cast<const v2u*>(p));
        return make_uint2(t.x, t.y);
    }
    static __device__ __forceinline__ void st(vec* p, vec v) {
        v2u t = {v.x, v.y};
        __builtin_nontemporal_store(t, reinterpret_cast<v2u*>(p));
    }
    static __device__ __forceinline__ unsigned word(vec x, int w) { return w == 0 ? x.x : x.y; }
    static __device__ __forceinline__ float dot(vec a, vec b) { return dot2_bf16(a.y, b.y, dot2_bf16(a.x, b.x, 0.f)); }
};

// sum over the 16 lanes of a row group, result in every lane
__device__ __forceinline__ float row16_sum(float x) {
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xF, 0xF, false));  // row_half_mirror
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x140, 0xF, 0xF, false));  // row_mirror
    return x;
}

// INPLACE: src and dst are the same cache and every segment keeps its start (tables from launch_cmp_scan_inplace),
// so survivor r of a chunk moves left by the number of entries evicted before it, or not at all.  A block may
// overwrite its own chunk's entries once all of its wavefronts hold their rows in registers; the (few) survivors
// whose destination lies in an earlier chunk's range - which another block may still be reading - go to the same
// index of `stage` instead, and k_cmp_unstage puts them in place after this kernel has ended.  Rows that do not move
// are not written at all.
// STEP (the one-call decode step, kvtrim_decode_step and its in-place form): the tables come from the step's scoring
// kernel instead of a compaction scan - the same per-chunk descriptors, but no destination per chunk: the number of
// entries the chunk loses and a record per segment, from which the block derives where its survivors go and, in
// the few chunks that lose entries, which they are.  The kernel then also writes the keep mask (`keep` is the
// caller's output array) and commits the source segment's new length (step_seg_len = the source cache's seg_len
// array; the new token was appended by the scoring kernel).  After the scoring kernel's single-block select the
// per-chunk word says "dense": destination offsets and mask are in memory, as after a compaction scan.
// GATHER (a selection that keeps few entries of every chunk - the first eviction after a long prefill; out of place
// only): a block per 128-row chunk of the DESTINATION.  The compaction scan has listed the chunks (ws.att_desc) and
// the source row of every destination row (ws.gat_src, 128 slots per chunk, the slots behind a ragged chunk's last
// row naming a live row), so a block asks for its row numbers at once, together with its descriptor, and for the
// rows as soon as the numbers are there; neither the mask nor the source's chunk table is read.
template <int D, int G, bool INPLACE, bool STEP = false, bool GATHER = false>
__global__ __launch_bounds__(FUS_THREADS) void k_cmp_attn(CacheView src, const uint8_t* keep,
                                                          CacheViewMut dst, CacheViewMut stage,
                                                          const uint16_t* __restrict__ q,
                                                          Shape sh, Workspace ws, float scale_log2,
                                                          int layer_begin, int layer_end, int32_t* step_seg_len = nullptr) {
    static_assert(!(GATHER && (INPLACE || STEP)), "the gathering instance compacts out of place, from a keep mask");
    typedef Row<D> R;
    typedef typename R::vec vec;
    constexpr int E = R::E;
    constexpr int VPR = 16;                                       // lanes (vectors) per row
    constexpr int NW = FUS_THREADS / 64;                          // 8 wavefronts
    __shared__ int wave_cnt[CMP_CHUNK / 64];
    __shared__ int list[CMP_CHUNK];
    __shared__ float s_m[NW][G], s_l[NW][G];
    constexpr int SO = D + 8;                                     // floats per (wavefront, head) in s_o: a 32-byte skew between heads
    __shared__ __attribute__((aligned(16))) float s_o[NW][G][SO];

    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int ch = blockIdx.x;
    // descriptor and destination are fetched together with the two grid-wide words (the grid never exceeds the
    // tables; what they hold at or beyond `total` is not used)
    const ChunkDesc cd = GATHER ? ws.att_desc[ch] : ws.cmp_desc[ch];
    int64_t dflag = STEP ? 0 : (GATHER ? CMP_DST_FULL : ws.cmp_chunk_dst[ch]);
    const uint32_t step_ev = STEP ? ws.step_chunk_ev[ch] : 0u;    // STEP: entries the chunk loses (or "see the table")
    // GATHER: the source rows of this thread's rows (the slots exist for every block of the grid; what they hold at
    // or beyond the last chunk is not used)
    int gat_row[4] = {0, 0, 0, 0}, gat_md = 0;
    if (GATHER) {
        const int32_t* slots = ws.gat_src + (int64_t)ch * CMP_CHUNK;
#pragma unroll
        for (int u = 0; u < 4; ++u) gat_row[u] = slots[(tid >> 6) * CMP_WAVE_ROWS + u * 4 + ((tid & 63) >> 4)];
        if (tid < CMP_CHUNK) gat_md = slots[tid];
    }
    if (__hip_atomic_load(ws.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
    if (ch >= (GATHER ? ws.att_chunk_prefix : ws.cmp_chunk_prefix)[sh.nseg]) return;
    const int64_t sbase = GATHER ? 0 : cd.first;                  // (GATHER: row numbers are absolute)
    // STEP: the scoring kernel leaves no destination per chunk (one block would write 16 K of them) but a record per
    // SEGMENT - where the segment's survivors start and which of its entries go - from which the chunk's block
    // places its survivors itself: they start at dst_start + (chunk's first index) - (evicted entries before it).
    // Everything here is uniform over the block (scalar loads); the record is only needed for the stores and, in
    // the few chunks that lose entries, for the survivor list.
    const bool step_listed = STEP && step_ev != STEP_CHUNK_DENSE;
    int step_idx0 = 0, step_cnt = 0, step_recw = 0;               // step_recw: lane l holds 32-bit word l of the segment's record
    const int32_t* step_more = nullptr;                           // the segment's evicted entries beyond those in the record
    int64_t dbase = GATHER ? cd.first : dflag & ~CMP_DST_FULL;
    if (STEP && !step_listed) {
        dflag = ws.cmp_chunk_dst[ch];
        dbase = dflag & ~CMP_DST_FULL;
    }
    // Called by whole wavefronts, for a full chunk AFTER its rows have been requested: the record comes with one
    // vector load of 16 lanes - vector loads return in order, so the wait for the rows does not wait for it, whereas
    // a scalar load would make every later scalar wait, and the row requests behind it, wait for the record.
    auto step_load = [&]() {
        static_assert(sizeof(StepSegRec) == 64 && STEP_REC_IDX == 12, "one word per lane: dst_start, cnt, off, twelve indices");
        const int32_t* rw = reinterpret_cast<const int32_t*>(ws.step_rec + cd.seg);
        step_recw = lane < 16 ? rw[lane] : 0;
    };
    auto step_resolve = [&]() {
        // (the segment's start is read here and not with the record: it is a scalar load that depends on the descriptor,
        // and the wait for it would stand between the descriptor and the requests for the rows)
        step_idx0 = (int)(sbase - src.seg_start[cd.seg]);
        step_cnt = __builtin_amdgcn_readlane(step_recw, 2);
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane(step_recw, 0), hi = (uint32_t)__builtin_amdgcn_readlane(step_recw, 1);
        step_more = ws.step_evl + (size_t)(cd.seg / sh.segs_per_seq) * STEP_MAX_EVICT + __builtin_amdgcn_readlane(step_recw, 3);
        int before = __popcll(__ballot(lane >= 4 && lane < 4 + min(step_cnt, STEP_REC_IDX) && step_recw < step_idx0));
        for (int i = STEP_REC_IDX; i < step_cnt; ++i) before += step_more[i] < step_idx0;
        dbase = (int64_t)(((uint64_t)hi << 32) | lo) + step_idx0 - before;
    };
    auto step_place = [&]() {
        step_load();
        step_resolve();
    };
    // Every entry of the chunk survives (almost every chunk of a decode step): row r of the survivors is row r of
    // the chunk, so the rows are requested right away instead of after the mask has arrived and been ranked.
    const bool full = step_listed ? step_ev == 0u : (dflag & CMP_DST_FULL) != 0;   // uniform over the block
    int cnt = 0;
    float md_lb = 0.f, md_lt = 0.f;
    int md_pos = 0, md_rank = tid;
    // this thread carries an entry's metadata in registers (INPLACE: not if the chunk stays as it is)
    // (a listed chunk of an in-place STEP learns its place only after its rows have been requested: it asks for the
    // metadata then, if it moves at all)
    bool md_mine = full && tid < cd.n && !(INPLACE && (step_listed || dbase == sbase));
    if (full) {
        cnt = cd.n;
        if (md_mine) {
            const int64_t e = GATHER ? (int64_t)gat_md : sbase + tid;
            md_lb = src.log_beta[e];
            if (src.log_tail) md_lt = src.log_tail[e];
            md_pos = src.pos[e];
        }
        if (STEP && tid < cd.n) const_cast<uint8_t*>(keep)[sbase + tid] = 1;   // (chunks that lose entries have their mask already)
    } else {
        int rank = 0;
        bool flag = false;
        if (step_listed) step_place();                            // (a chunk that loses entries needs the list first)
        if (tid < CMP_CHUNK) {
            if (step_listed) {                                    // the mask of this chunk from the segment's list
                flag = tid < cd.n;
#pragma unroll
                for (int i = 0; i < STEP_REC_IDX; ++i)
                    flag = flag & !((i < step_cnt) & (__builtin_amdgcn_readlane(step_recw, 4 + i) == step_idx0 + tid));
                for (int i = STEP_REC_IDX; i < step_cnt; ++i) flag = flag && step_more[i] != step_idx0 + tid;
                if (tid < cd.n) const_cast<uint8_t*>(keep)[sbase + tid] = flag;
            } else {
                flag = tid < cd.n && keep[sbase + tid] != 0;
            }
            const uint64_t mask = __ballot(flag);
            rank = mbcnt(mask);
            if (lane == 0) wave_cnt[wave] = __popcll(mask);
        }
        __syncthreads();
#pragma unroll
        for (int w = 0; w < CMP_CHUNK / 64; ++w) {
            if (w < wave && tid < CMP_CHUNK) rank += wave_cnt[w];
            cnt += wave_cnt[w];
        }
        if (flag) {
            list[rank] = tid;
            if (INPLACE) {                                        // written after the whole block has read its entries
                md_mine = true;
                md_rank = rank;
                md_lb = src.log_beta[sbase + tid];
                if (src.log_tail) md_lt = src.log_tail[sbase + tid];
                md_pos = src.pos[sbase + tid];
            } else {
                dst.log_beta[dbase + rank] = src.log_beta[sbase + tid];
                if (src.log_tail) dst.log_tail[dbase + rank] = src.log_tail[sbase + tid];
                dst.pos[dbase + rank] = src.pos[sbase + tid];
            }
        }
        __syncthreads();
    }

    const int seg = cd.seg;
    const int seq = seg / sh.segs_per_seq, lh = seg % sh.segs_per_seq;
    const int layer = lh / sh.n_kv_heads, head = lh % sh.n_kv_heads;
    const bool attend = layer >= layer_begin && layer < layer_end;   // uniform over the block
    const int sub = lane >> 4, col = lane & 15;
    const int r0 = wave * CMP_WAVE_ROWS;                          // this wavefront's rows of the survivor list
    const bool has_rows = r0 < cnt;                               // uniform over the wavefront

    const vec* sk = reinterpret_cast<const vec*>(src.k);
    const vec* sv = reinterpret_cast<const vec*>(src.v);
    // the three steps of a wavefront that has rows: fetch rows and queries, write the rows out, attend
    auto fetch = [&](vec (&kk)[4], vec (&vv)[4], int (&srow)[4], vec (&qp)[G]) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = min(r0 + u * 4 + sub, cnt - 1);         // clamped: loads stay on live rows
            srow[u] = GATHER ? gat_row[u] : (full ? r : list[r]); // the chunk entry the row comes from
            const int64_t se = (sbase + srow[u]) * VPR + col;
            kk[u] = R::ld(sk + se);
            vv[u] = R::ld(sv + se);
        }
        if (attend) {
            const int64_t hq0 = ((int64_t)seq * sh.n_layers + layer) * sh.n_q_heads + (int64_t)head * G;
#pragma unroll
            for (int g = 0; g < G; ++g) qp[g] = reinterpret_cast<const vec*>(q + (hq0 + g) * D)[col];   // (stays packed: q.k is a packed dot product)
        }
    };
    auto write_rows = [&](const vec (&kk)[4], const vec (&vv)[4], const int (&srow)[4]) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = r0 + u * 4 + sub;
            if (r < cnt && (!INPLACE || dbase + r != sbase + srow[u])) {   // INPLACE: a row that stays is not written
                const int64_t de = (dbase + r) * VPR + col;
                const bool own = !INPLACE || dbase + r >= sbase;  // inside this chunk's own range (or another buffer)
                R::st(reinterpret_cast<vec*>(own ? dst.k : stage.k) + de, kk[u]);
                R::st(reinterpret_cast<vec*>(own ? dst.v : stage.v) + de, vv[u]);
            }
        }
    };
    auto write_metadata = [&]() {
        const int64_t de = dbase + md_rank;
        if (!INPLACE || de != sbase + tid) {
            const CacheViewMut& t = (!INPLACE || de >= sbase) ? dst : stage;
            t.log_beta[de] = md_lb;
            if (src.log_tail) t.log_tail[de] = md_lt;
            t.pos[de] = md_pos;
        }
    };
    // Attention of this wavefront's 16 rows.
    //   q.k   on the vector ALU, packed: 4 (2) two-element bf16 dot products per query head, row and lane, then a
    //         16-lane all-reduce with DPP - every lane ends up with the logits of its 4 rows for every head.
    //   p.v   on the matrix cores.  A lane holds the same 8 (4) columns of 4 rows, i.e. for one column 4 values along
    //         the reduction (row) dimension - the operand layout of a 16x16x32 MFMA with m = the lane's column block
    //         (lane & 15), k = 8 (lane >> 4) + j: slots j = 0..3 carry the lane's rows u = j, slots 4..7 the same rows
    //         again.  The other operand carries, for n = head (lane & 15 again: lane (sub, g) serves head g), the
    //         probabilities of those rows as TWO bf16 values each, rounded value in slots 0..3 and the rounded
    //         remainder in 4..7, so that the product is exact to 2^-16 of every term (V is bf16 anyway, sums are
    //         fp32).  One MFMA per column of the lane's slice sums over all 16 rows of the wavefront and all G heads
    //         at once; its result - lane (sub, g): columns 8 (4 sub + i) + e, i = 0..3, of head g - goes to LDS.
    //         (On the vector ALU the same product took 128 instructions per head; the in-place instance, which moves
    //         few rows, was bound by them from G = 4 on.)
    auto attend_rows = [&](const vec (&kk)[4], const vec (&vv)[4], const vec (&qp)[G]) {
        float zs[4];                                              // logits of this lane's head (lane & 15; lanes >= G: head G - 1, unused)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const bool valid = r0 + u * 4 + sub < cnt;
            float zu = 0.f;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float s = row16_sum(R::dot(qp[g], kk[u]));
                zu = (g == 0 || col >= g) ? s : zu;               // (ends as head min(col, G - 1))
            }
            zs[u] = valid ? zu * scale_log2 : -INFINITY;
        }
        const float mx = fmaxf(fmaxf(zs[0], zs[1]), fmaxf(zs[2], zs[3]));
        float m_all = fmaxf(mx, __shfl_xor(mx, 16, 64));
        m_all = fmaxf(m_all, __shfl_xor(m_all, 32, 64));          // maximum over the wavefront's 16 rows
        const float m_fin = m_all == -INFINITY ? 0.f : m_all;
        float p[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) p[u] = __builtin_amdgcn_exp2f(zs[u] - m_fin);
        float l_all = (p[0] + p[1]) + (p[2] + p[3]);
        l_all += __shfl_xor(l_all, 16, 64);
        l_all += __shfl_xor(l_all, 32, 64);
        if (sub == 0 && col < G) {
            s_m[wave][col] = m_all;
            s_l[wave][col] = l_all;
        }
        // p = hi + lo + O(2^-16 p), both bf16 (round to nearest even)
        const bf16x2 h01 = {(__bf16)p[0], (__bf16)p[1]}, h23 = {(__bf16)p[2], (__bf16)p[3]};
        const bf16x2 l01 = {(__bf16)(p[0] - (float)h01.x), (__bf16)(p[1] - (float)h01.y)};
        const bf16x2 l23 = {(__bf16)(p[2] - (float)h23.x), (__bf16)(p[3] - (float)h23.y)};
        const uint4 pb = make_uint4(__builtin_bit_cast(unsigned, h01), __builtin_bit_cast(unsigned, h23),
                                    __builtin_bit_cast(unsigned, l01), __builtin_bit_cast(unsigned, l23));
        float4v acc[E];
#pragma unroll
        for (int w = 0; w < E / 2; ++w) {
            const unsigned x0 = R::word(vv[0], w), x1 = R::word(vv[1], w), x2 = R::word(vv[2], w), x3 = R::word(vv[3], w);
            // columns 2 w (low halves) and 2 w + 1 (high halves) of the four rows
            const unsigned a01 = __builtin_amdgcn_perm(x1, x0, 0x05040100u), a23 = __builtin_amdgcn_perm(x3, x2, 0x05040100u);
            const unsigned b01 = __builtin_amdgcn_perm(x1, x0, 0x07060302u), b23 = __builtin_amdgcn_perm(x3, x2, 0x07060302u);
            const float4v zero = {0.f, 0.f, 0.f, 0.f};
            acc[2 * w] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, make_uint4(a01, a23, a01, a23)),
                                                                 __builtin_bit_cast(bf16x8, pb), zero, 0, 0, 0);
            acc[2 * w + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, make_uint4(b01, b23, b01, b23)),
                                                                     __builtin_bit_cast(bf16x8, pb), zero, 0, 0, 0);
        }
        if (col < G) {
            // s_o[wave][head][(4 i + sub) E + e] = column E (4 sub + i) + e: the four lanes of a head write 4 E contiguous floats
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float* o = &s_o[wave][col][(4 * i + sub) * E];
#pragma unroll
                for (int e4 = 0; e4 < E; e4 += 4)
                    *reinterpret_cast<float4*>(o + e4) = make_float4(acc[e4][i], acc[e4 + 1][i], acc[e4 + 2][i], acc[e4 + 3][i]);
            }
        }
    };

    if (!INPLACE) {
        if (has_rows) {
            vec kk[4], vv[4];
            int srow[4];
            vec qp[G];
            fetch(kk, vv, srow, qp);
            if (step_listed && full) step_place();
            write_rows(kk, vv, srow);
            if (md_mine) write_metadata();                        // (wavefronts 0 and 1, which have rows whenever they have entries)
            if (attend) attend_rows(kk, vv, qp);
        }
    } else {
        vec kk[4], vv[4];
        int srow[4];
        vec qp[G];
        // (in place a chunk that stays writes nothing, so its record is asked for BEFORE its rows: it is there first,
        // and the attention can start on the first rows that arrive)
        if (step_listed && full) step_load();
        if (has_rows) fetch(kk, vv, srow, qp);
        if (step_listed && full) step_resolve();                  // (every wavefront: the decision below is the block's)
        // nothing of this chunk moves when it loses nothing and nothing was evicted before it in its segment
        const bool moves = !(full && dbase == sbase);             // uniform over the block
        if (STEP && step_listed && full && moves && tid < cd.n) {
            md_mine = true;
            md_lb = src.log_beta[sbase + tid];
            if (src.log_tail) md_lt = src.log_tail[sbase + tid];
            md_pos = src.pos[sbase + tid];
        }
        // STEP: the chunk's place goes into the table k_cmp_unstage reads (a compaction scan would have left it there)
        if (STEP && step_listed && tid == 0) ws.cmp_chunk_dst[ch] = dbase | (full ? CMP_DST_FULL : 0);
        if (moves) {
            // every wavefront of the block holds its rows and metadata in registers before any of them overwrites an entry
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (md_mine) write_metadata();
        }
        if (has_rows) {
            if (moves) write_rows(kk, vv, srow);
            if (attend) attend_rows(kk, vv, qp);
        }
    }
    // the segment's first chunk commits the source segment's new length (after the rows have been asked for: the look
    // at the segment's start is a load that depends on the descriptor)
    if (STEP && tid == 0 && sbase == src.seg_start[seg]) step_seg_len[seg] = ws.step_len[seg];
    if (!attend) return;

    // the partials of the wavefronts that had rows are merged by all threads
    __syncthreads();
    const int nw = min(NW, (cnt + CMP_WAVE_ROWS - 1) / CMP_WAVE_ROWS);
    float* part = ws.att_partial + (size_t)ch * G * (D + 2);
    for (int idx = tid; idx < G * D; idx += FUS_THREADS) {
        const int g = idx / D, d = idx % D;
        const int cb = d / E;                                     // column block 4 sub + i sits at 4 i + sub (see attend_rows)
        const int so_at = (4 * (cb & 3) + (cb >> 2)) * E + d % E;
        float M = -INFINITY;
#pragma unroll
        for (int s = 0; s < NW; ++s)
            if (s < nw) M = fmaxf(M, s_m[s][g]);
        const float Ms = M == -INFINITY ? 0.f : M;
        float accd = 0.f, lsum = 0.f;
#pragma unroll
        for (int s = 0; s < NW; ++s) {
            if (s < nw) {
                const float w = __builtin_amdgcn_exp2f(s_m[s][g] - Ms);
                accd += s_o[s][g][so_at] * w;
                lsum += s_l[s][g] * w;
            }
        }
        part[g * (D + 2) + 2 + d] = accd;
        if (d == 0) {
            part[g * (D + 2)] = M;
            part[g * (D + 2) + 1] = lsum;
        }
    }
}

template <int D, bool INPLACE>
static bool dispatch_fused(int G, dim3 grid, hipStream_t st, const CacheView& src, const uint8_t* keep,
                           const CacheViewMut& dst, const CacheViewMut& stage, const uint16_t* q, const Shape& sh,
                           const Workspace& ws, float scale_log2, int lb, int le) {
    switch (G) {
#define KVTRIM_CASE(g) \
    case g: hipLaunchKernelGGL((k_cmp_attn<D, g, INPLACE>), grid, dim3(FUS_THREADS), 0, st, src, keep, dst, stage, q, sh, ws, scale_log2, lb, le); return true;
        KVTRIM_CASE(1) KVTRIM_CASE(2) KVTRIM_CASE(3) KVTRIM_CASE(4) KVTRIM_CASE(5) KVTRIM_CASE(6) KVTRIM_CASE(7) KVTRIM_CASE(8)
#undef KVTRIM_CASE
        default: return false;
    }
}

template <int D>
static bool dispatch_gather(int G, dim3 grid, hipStream_t st, const CacheView& src, const CacheViewMut& dst,
                            const uint16_t* q, const Shape& sh, const Workspace& ws, float scale_log2, int lb, int le) {
    switch (G) {
#define KVTRIM_CASE(g) \
    case g: hipLaunchKernelGGL((k_cmp_attn<D, g, false, false, true>), grid, dim3(FUS_THREADS), 0, st, src, nullptr, dst, dst, q, sh, ws, scale_log2, lb, le); return true;
        KVTRIM_CASE(1) KVTRIM_CASE(2) KVTRIM_CASE(3) KVTRIM_CASE(4) KVTRIM_CASE(5) KVTRIM_CASE(6) KVTRIM_CASE(7) KVTRIM_CASE(8)
#undef KVTRIM_CASE
        default: return false;
    }
}

// Stage 3 alone for a sparse selection: the gathering instance with no layer to attend (it then reads no query and
// writes no partial result).
kvtrim_status launch_gather_rows(kvtrim_ctx* ctx, const CacheView& src, const CacheViewMut& dst, hipStream_t st) {
    const Shape& sh = ctx->shape;
    const dim3 grid((unsigned)(dst.cap / CMP_CHUNK + sh.nseg));
    if (sh.head_dim == 128)
        hipLaunchKernelGGL((k_cmp_attn<128, 1, false, false, true>), grid, dim3(FUS_THREADS), 0, st, src, nullptr, dst, dst, nullptr, sh, ctx->ws, 0.f, 0, 0);
    else
        hipLaunchKernelGGL((k_cmp_attn<64, 1, false, false, true>), grid, dim3(FUS_THREADS), 0, st, src, nullptr, dst, dst, nullptr, sh, ctx->ws, 0.f, 0, 0);
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

// After k_cmp_attn<.., INPLACE>: the survivors of a chunk whose place lies before the chunk's own range (as many
// as were evicted before the chunk in its segment, at most all of its survivors) wait in `stage` at their final
// index; one wavefront per chunk puts them there (in a decode step most chunks have nothing parked and their
// wavefront ends at once).  The wavefront of a segment's first chunk also commits the segment's new length, which
// no kernel of the call reads any more.
constexpr int UNS_THREADS = 256;

template <int D>
__global__ __launch_bounds__(UNS_THREADS) void k_cmp_unstage(CacheViewMut c, CacheViewMut stage,
                                                             const int32_t* __restrict__ kept, Shape sh, Workspace ws) {
    unstage_chunk<D>(c, stage, kept, sh, ws, (int)(blockIdx.x * (UNS_THREADS / 64) + (threadIdx.x >> 6)));
}

// Stage 3 alone inside the cache: k_cmp_attn<.., INPLACE> without the attention.  A chunk that loses nothing and
// stays where it is - almost every chunk of a decode step - ends after reading its descriptor, so the kernel
// touches only the rows behind an eviction.  Non-temporal loads and stores matter here: with plain ones the mover
// took 0.129 instead of 0.094 ms and the attention that reads the cache next 0.237 instead of 0.203 ms.  (A fixed
// grid of 512 ... 8192 blocks walking over the chunks measured slower than a block per chunk.)
template <int D>
__global__ __launch_bounds__(CMP_THREADS) void k_cmp_move_inplace(CacheViewMut c, const uint8_t* __restrict__ keep,
                                                                  CacheViewMut stage, Shape sh, Workspace ws) {
    constexpr int VPR = D / 8;                    // 16-byte vectors per row
    constexpr int RPI = 64 / VPR;                 // rows moved by one wavefront instruction
    constexpr int BATCH = CMP_WAVE_ROWS / RPI;    // instructions per wavefront: 4 (D=128) or 2 (D=64)
    __shared__ int wave_cnt[CMP_CHUNK / 64];
    __shared__ int list[CMP_CHUNK];
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int ch = blockIdx.x;
    const ChunkDesc cd = ws.cmp_desc[ch];
    const int64_t dflag = ws.cmp_chunk_dst[ch];
    if (__hip_atomic_load(ws.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
    if (ch >= ws.cmp_chunk_prefix[sh.nseg]) return;
    const int64_t sbase = cd.first, dbase = dflag & ~CMP_DST_FULL;
    const bool full = (dflag & CMP_DST_FULL) != 0;
    if (full && dbase == sbase) return;                           // nothing of this chunk moves
    int cnt = cd.n, rank = tid;
    bool mine = tid < cd.n;                                       // this thread carries an entry's metadata
    if (!full) {
        rank = 0;
        mine = false;
        if (tid < CMP_CHUNK) {
            mine = tid < cd.n && keep[sbase + tid] != 0;
            const uint64_t mask = __ballot(mine);
            rank = mbcnt(mask);
            if (lane == 0) wave_cnt[wave] = __popcll(mask);
        }
        __syncthreads();
        cnt = 0;
#pragma unroll
        for (int w = 0; w < CMP_CHUNK / 64; ++w) {
            if (w < wave && tid < CMP_CHUNK) rank += wave_cnt[w];
            cnt += wave_cnt[w];
        }
        if (mine) list[rank] = tid;
        __syncthreads();
    }
    float md_lb = 0.f, md_lt = 0.f;
    int md_pos = 0;
    if (mine) {
        md_lb = c.log_beta[sbase + tid];
        if (c.log_tail) md_lt = c.log_tail[sbase + tid];
        md_pos = c.pos[sbase + tid];
    }
    const int r0 = wave * CMP_WAVE_ROWS;                          // this wavefront's rows of the survivor list
    const int sub = lane / VPR, col = lane % VPR;
    uint4 kk[BATCH], vv[BATCH];
    int srow[BATCH];
    if (r0 < cnt) {
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int r = min(r0 + u * RPI + sub, cnt - 1);       // clamped: loads stay on live rows
            srow[u] = full ? r : list[r];
            const int64_t se = (sbase + srow[u]) * VPR + col;
            kk[u] = Row<128>::ld(reinterpret_cast<const uint4*>(c.k) + se);   // non-temporal, as in the fused kernel
            vv[u] = Row<128>::ld(reinterpret_cast<const uint4*>(c.v) + se);
        }
    }
    // every wavefront of the block holds its rows and metadata in registers before any of them overwrites an entry
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (mine) {
        const int64_t de = dbase + rank;
        if (de != sbase + tid) {
            const CacheViewMut& t = de >= sbase ? c : stage;
            t.log_beta[de] = md_lb;
            if (c.log_tail) t.log_tail[de] = md_lt;
            t.pos[de] = md_pos;
        }
    }
    if (r0 < cnt) {
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int r = r0 + u * RPI + sub;
            if (r < cnt && dbase + r != sbase + srow[u]) {
                const int64_t de = (dbase + r) * VPR + col;
                const bool own = dbase + r >= sbase;
                Row<128>::st(reinterpret_cast<uint4*>(own ? c.k : stage.k) + de, kk[u]);
                Row<128>::st(reinterpret_cast<uint4*>(own ? c.v : stage.v) + de, vv[u]);
            }
        }
    }
}

kvtrim_status launch_compact_inplace(kvtrim_ctx* ctx, const CacheViewMut& c, const uint8_t* keep, const int32_t* kept,
                                     const CacheViewMut& stage, hipStream_t st) {
    const Shape& sh = ctx->shape;
    const Workspace& ws = ctx->ws;
    const int64_t max_chunks = c.cap / CMP_CHUNK + sh.nseg;
    launch_cmp_scan_inplace(ctx, c, keep, kept, st);
    {
        ProfScope prof(ctx, K_CMP_COPY, st);
        if (sh.head_dim == 128)
            hipLaunchKernelGGL(k_cmp_move_inplace<128>, dim3((unsigned)max_chunks), dim3(CMP_THREADS), 0, st, c, keep, stage, sh, ws);
        else
            hipLaunchKernelGGL(k_cmp_move_inplace<64>, dim3((unsigned)max_chunks), dim3(CMP_THREADS), 0, st, c, keep, stage, sh, ws);
    }
    {
        ProfScope prof(ctx, K_CMP_UNSTAGE, st);
        const dim3 grid((unsigned)((max_chunks + UNS_THREADS / 64 - 1) / (UNS_THREADS / 64)));
        if (sh.head_dim == 128)
            hipLaunchKernelGGL(k_cmp_unstage<128>, grid, dim3(UNS_THREADS), 0, st, c, stage, kept, sh, ws);
        else
            hipLaunchKernelGGL(k_cmp_unstage<64>, grid, dim3(UNS_THREADS), 0, st, c, stage, kept, sh, ws);
    }
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

kvtrim_status launch_compact_attn(kvtrim_ctx* ctx, const CacheView& src, const uint8_t* keep, const int32_t* kept,
                                  const CacheViewMut& dst, int32_t reserve, const uint16_t* q, int32_t layer_begin,
                                  int32_t layer_end, float scale, float* out, float* lse, hipStream_t st,
                                  int64_t evict_hint) {
    const Shape& sh = ctx->shape;
    const Workspace& ws = ctx->ws;
    const int64_t max_chunks = src.cap / CMP_CHUNK + sh.nseg;
    // (The fused kernel's time does not depend on the group of query heads: 2.1 M retained entries, G = 1..8: 366-378 us
    // at head_dim 128, 180-199 us at head_dim 64 - p.v runs on the matrix cores for all heads at once.)
    // Few survivors per source chunk?  A caller that names the evictions of the step (kvtrim_decode_step's evict_hint)
    // has said so itself: a positive hint means a decode step, every chunk nearly whole.  Without a hint the
    // capacities decide, in the one direction in which they can: a destination under a quarter of the source cannot
    // take more than one source entry in four.
    const bool sparse = evict_hint > 0 ? false : dst.cap < src.cap / 4;
    const int64_t dst_chunks = dst.cap / CMP_CHUNK + sh.nseg;    // upper bound on the destination's chunks
    if (sparse && gather_fits(ctx, src.cap, dst.cap)) {
        // Few survivors per source chunk: the fused kernel's gathering instance, a block per chunk of the destination
        // (a block per source chunk would write one partial result per 128 source entries for a handful of survivors
        // each).  The compaction scan lists the destination's chunks and the source row of each of their rows.
        launch_cmp_scan_aligned(ctx, src, keep, kept, dst, reserve, 1, st, true);
        bool ok;
        {
            ProfScope prof(ctx, K_CMP_ATTN, st);
            const float scale_log2 = scale * 1.4426950408889634f;
            ok = sh.head_dim == 128
                     ? dispatch_gather<128>(sh.group, dim3((unsigned)dst_chunks), st, src, dst, q, sh, ws, scale_log2, layer_begin, layer_end)
                     : dispatch_gather<64>(sh.group, dim3((unsigned)dst_chunks), st, src, dst, q, sh, ws, scale_log2, layer_begin, layer_end);
        }
        if (!ok) return KVTRIM_EINVAL;
        return launch_combine(ctx, ws.att_chunk_prefix, layer_begin, layer_end, out, lse, st);
    }
    if (max_chunks > ws.max_att_chunks || sparse) {
        // Run the two stages one after the other, which computes the same thing: when there are too many source
        // chunks for the partial-result buffer, and for a sparse selection the gathering instance cannot take.
        kvtrim_status rc = launch_compact(ctx, src, keep, kept, dst, reserve, st);
        if (rc != KVTRIM_OK) return rc;
        CacheView d;
        d.k = dst.k; d.v = dst.v; d.log_beta = dst.log_beta; d.pos = dst.pos;
        d.seg_start = dst.seg_start; d.seg_len = dst.seg_len; d.cap = dst.cap; d.log_tail = dst.log_tail;
        return launch_attn(ctx, d, q, nullptr, layer_begin, layer_end, scale, out, lse, st);
    }
    launch_cmp_scan(ctx, src, keep, kept, dst, reserve, st);
    bool ok;
    {
        ProfScope prof(ctx, K_CMP_ATTN, st);
        const float scale_log2 = scale * 1.4426950408889634f;
        ok = sh.head_dim == 128
                 ? dispatch_fused<128, false>(sh.group, dim3((unsigned)max_chunks), st, src, keep, dst, dst, q, sh, ws, scale_log2, layer_begin, layer_end)
                 : dispatch_fused<64, false>(sh.group, dim3((unsigned)max_chunks), st, src, keep, dst, dst, q, sh, ws, scale_log2, layer_begin, layer_end);
    }
    if (!ok) return KVTRIM_EINVAL;
    return launch_combine(ctx, ws.cmp_chunk_prefix, layer_begin, layer_end, out, lse, st);
}

kvtrim_status launch_compact_attn_inplace(kvtrim_ctx* ctx, const CacheViewMut& c, const uint8_t* keep, const int32_t* kept,
                                          const CacheViewMut& stage, const uint16_t* q, int32_t layer_begin,
                                          int32_t layer_end, float scale, float* out, float* lse, hipStream_t st) {
    const Shape& sh = ctx->shape;
    const Workspace& ws = ctx->ws;
    const int64_t max_chunks = c.cap / CMP_CHUNK + sh.nseg;      // <= ws.max_att_chunks, checked by the caller
    CacheView src;
    src.k = c.k; src.v = c.v; src.log_beta = c.log_beta; src.pos = c.pos;
    src.seg_start = c.seg_start; src.seg_len = c.seg_len; src.cap = c.cap; src.log_tail = c.log_tail;
    launch_cmp_scan_inplace(ctx, c, keep, kept, st);
    bool ok;
    {
        ProfScope prof(ctx, K_CMP_ATTN, st);
        const float scale_log2 = scale * 1.4426950408889634f;
        ok = sh.head_dim == 128
                 ? dispatch_fused<128, true>(sh.group, dim3((unsigned)max_chunks), st, src, keep, c, stage, q, sh, ws, scale_log2, layer_begin, layer_end)
                 : dispatch_fused<64, true>(sh.group, dim3((unsigned)max_chunks), st, src, keep, c, stage, q, sh, ws, scale_log2, layer_begin, layer_end);
    }
    if (!ok) return KVTRIM_EINVAL;
    // the parked rows go to their places in the launch of the merge kernel (nothing there reads them)
    return launch_combine_unstage(ctx, ws.cmp_chunk_prefix, layer_begin, layer_end, out, lse, c, stage, kept, max_chunks, st);
}

kvtrim_status launch_decode_step(kvtrim_ctx* ctx, const CacheViewMut& srcm, const StepArgs& sa, const int32_t* now,
                                 const int64_t* budget, float* score, int32_t* kept, uint32_t* thr, const uint16_t* q,
                                 int32_t layer_begin, int32_t layer_end, float scale, float* out, float* lse,
                                 int64_t evict_hint, hipStream_t st) {
    const Shape& sh = ctx->shape;
    const Workspace& ws = ctx->ws;
    CacheView src;
    src.k = srcm.k; src.v = srcm.v; src.log_beta = srcm.log_beta; src.pos = srcm.pos;
    src.seg_start = srcm.seg_start; src.seg_len = srcm.seg_len; src.cap = srcm.cap; src.log_tail = srcm.log_tail;
    const int64_t max_chunks = src.cap / CMP_CHUNK + sh.nseg;
    // Three kernels (score + resolve, move + attend, merge) when this is a decode step the candidate list can carry;
    // otherwise the calls it stands for, one after the other.
    const bool three = evict_hint > 0 && 8 * (evict_hint + 1) <= (int64_t)ws.fl_cap &&
                       sh.segs_per_seq <= STEP_MAX_SEGS && sh.n_seq <= STEP_MAX_SEQS && sa.n_new <= STEP_MAX_NEW &&
                       max_chunks <= ws.max_att_chunks && max_chunks <= ws.max_cmp_chunks;
    if (!three) {
        kvtrim_status rc = launch_append(ctx, srcm, sa.k_new, sa.v_new, sa.lb_new, sa.lt_new, sa.pos_new, sa.n_new, true, nullptr, st);
        if (rc != KVTRIM_OK) return rc;
        rc = launch_score_select(ctx, src, now, budget, score, sa.keep_out, kept, thr, evict_hint, st);
        if (rc != KVTRIM_OK) return rc;
        return launch_compact_attn(ctx, src, sa.keep_out, kept, sa.dst, sa.reserve, q, layer_begin, layer_end, scale, out, lse, st,
                                   evict_hint);
    }
    kvtrim_status rc = launch_step_scan(ctx, src, now, budget, score, kept, thr, sa, st);
    if (rc != KVTRIM_OK) return rc;
    {
        ProfScope prof(ctx, K_CMP_ATTN, st);
        const float scale_log2 = scale * 1.4426950408889634f;
        const dim3 grid((unsigned)max_chunks), block(FUS_THREADS);
        switch (sh.head_dim * 16 + sh.group) {
#define KVTRIM_CASE(d, g) \
    case d * 16 + g: hipLaunchKernelGGL((k_cmp_attn<d, g, false, true>), grid, block, 0, st, src, (const uint8_t*)sa.keep_out, sa.dst, sa.dst, q, sh, ws, scale_log2, layer_begin, layer_end, srcm.seg_len); break;
            KVTRIM_CASE(128, 1) KVTRIM_CASE(128, 2) KVTRIM_CASE(128, 3) KVTRIM_CASE(128, 4) KVTRIM_CASE(128, 5) KVTRIM_CASE(128, 6) KVTRIM_CASE(128, 7) KVTRIM_CASE(128, 8)
            KVTRIM_CASE(64, 1) KVTRIM_CASE(64, 2) KVTRIM_CASE(64, 3) KVTRIM_CASE(64, 4) KVTRIM_CASE(64, 5) KVTRIM_CASE(64, 6) KVTRIM_CASE(64, 7) KVTRIM_CASE(64, 8)
#undef KVTRIM_CASE
            default: return KVTRIM_EINVAL;
        }
    }
    return launch_combine(ctx, ws.cmp_chunk_prefix, layer_begin, layer_end, out, lse, st);
}

// The decode step in one call with stages 3 + 4 inside the cache: four kernels (score + resolve, move + attend, the
// rows parked in `stage` put in place, merge) when this is a decode step the candidate list can carry; otherwise the
// calls it stands for, one after the other.
kvtrim_status launch_decode_step_inplace(kvtrim_ctx* ctx, const CacheViewMut& c, const StepArgs& sa, const CacheViewMut& stage,
                                         const int32_t* now, const int64_t* budget, float* score, int32_t* kept, uint32_t* thr,
                                         const uint16_t* q, int32_t layer_begin, int32_t layer_end, float scale, float* out,
                                         float* lse, int64_t evict_hint, hipStream_t st) {
    const Shape& sh = ctx->shape;
    const Workspace& ws = ctx->ws;
    CacheView src;
    src.k = c.k; src.v = c.v; src.log_beta = c.log_beta; src.pos = c.pos;
    src.seg_start = c.seg_start; src.seg_len = c.seg_len; src.cap = c.cap; src.log_tail = c.log_tail;
    const int64_t max_chunks = src.cap / CMP_CHUNK + sh.nseg;    // <= ws.max_att_chunks, checked by the caller
    const bool four = evict_hint > 0 && 8 * (evict_hint + 1) <= (int64_t)ws.fl_cap && sh.segs_per_seq <= STEP_MAX_SEGS &&
                      sh.n_seq <= STEP_MAX_SEQS && sa.n_new <= STEP_MAX_NEW && max_chunks <= ws.max_cmp_chunks;
    if (!four) {
        kvtrim_status rc = launch_append(ctx, c, sa.k_new, sa.v_new, sa.lb_new, sa.lt_new, sa.pos_new, sa.n_new, true, nullptr, st);
        if (rc != KVTRIM_OK) return rc;
        rc = launch_score_select(ctx, src, now, budget, score, sa.keep_out, kept, thr, evict_hint, st);
        if (rc != KVTRIM_OK) return rc;
        return launch_compact_attn_inplace(ctx, c, sa.keep_out, kept, stage, q, layer_begin, layer_end, scale, out, lse, st);
    }
    kvtrim_status rc = launch_step_scan(ctx, src, now, budget, score, kept, thr, sa, st);
    if (rc != KVTRIM_OK) return rc;
    {
        ProfScope prof(ctx, K_CMP_ATTN, st);
        const float scale_log2 = scale * 1.4426950408889634f;
        const dim3 grid((unsigned)max_chunks), block(FUS_THREADS);
        switch (sh.head_dim * 16 + sh.group) {
#define KVTRIM_CASE(d, g) \
    case d * 16 + g: hipLaunchKernelGGL((k_cmp_attn<d, g, true, true>), grid, block, 0, st, src, (const uint8_t*)sa.keep_out, c, stage, q, sh, ws, scale_log2, layer_begin, layer_end, c.seg_len); break;
            KVTRIM_CASE(128, 1) KVTRIM_CASE(128, 2) KVTRIM_CASE(128, 3) KVTRIM_CASE(128, 4) KVTRIM_CASE(128, 5) KVTRIM_CASE(128, 6) KVTRIM_CASE(128, 7) KVTRIM_CASE(128, 8)
            KVTRIM_CASE(64, 1) KVTRIM_CASE(64, 2) KVTRIM_CASE(64, 3) KVTRIM_CASE(64, 4) KVTRIM_CASE(64, 5) KVTRIM_CASE(64, 6) KVTRIM_CASE(64, 7) KVTRIM_CASE(64, 8)
#undef KVTRIM_CASE
            default: return KVTRIM_EINVAL;
        }
    }
    // the parked rows go to their places in the launch of the merge kernel (nothing there reads them)
    return launch_combine_unstage(ctx, ws.cmp_chunk_prefix, layer_begin, layer_end, out, lse, c, stage, kept, max_chunks, st);
}

}  // namespace kvtrim
