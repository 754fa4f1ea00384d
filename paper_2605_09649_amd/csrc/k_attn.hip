// Stage 4: GQA decode attention over the ragged retained caches (Sec. 2.1, Eq. reform, r in {0,1}).
//
// Split-K over fixed-size chunks of each segment so that very unequal segment lengths still
// fill the chip: a fixed grid of blocks shares the rows of the chunk table equally, each block
// walking a contiguous stretch of it.  Inside a chunk a wavefront walks tiles of 16 rows:
//   Q.K^T  one MFMA 16x16 accumulator per tile (rows = 16 keys, columns = the G query heads,
//          padded to 16); K fragments are loaded straight from HBM in the operand layout
//          (lane = key row, four lanes share 64 contiguous bytes of the row).
//   P.V    one MFMA 16x16x32 per column of a lane's slice: a lane owns one 16-byte column slice of
//          4 rows of the tile (rows 4b..4b+3 for its row group b), so V is read fully coalesced
//          (16 lanes = one 256-byte row) and the lane holds, per column, 4 consecutive slots of
//          the MFMA's reduction dimension; the probabilities of those rows for query head c are
//          what the Q.K^T accumulator of lane (b, c) holds - the other operand, as two bf16 terms.
// A wavefront keeps one online-softmax stream per query head (the maximum over the tile's 16
// rows) for as long as the block stays inside one segment; then the four wavefronts are merged
// through LDS, and the partial results of a segment by k_att_combine.  Logits are kept in base-2
// units.
#include "kvtrim_paged_device.h"

namespace kvtrim {

constexpr int ATT_THREADS = 256;
constexpr int ATT_PLAN_BLOCKS = 16;         // blocks that share the filling of the chunk table

typedef __attribute__((ext_vector_type(4))) float float4v;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) unsigned v4u;
typedef __attribute__((ext_vector_type(2))) unsigned v2u;

__global__ __launch_bounds__(1024) void k_att_plan(CacheView c, Shape sh, Workspace ws, int chunk,
                                                   int layer_begin, int layer_end, int64_t max_chunks) {
    const int H = sh.n_kv_heads, L = sh.n_layers;
    auto in_range = [=](int g) {
        const int layer = (g / H) % L;
        return layer >= layer_begin && layer < layer_end;
    };
    build_chunk_table(c.seg_len, c.seg_start, sh.nseg, in_range, chunk, c.cap, ws.att_chunk_prefix,
                      ws.att_desc, max_chunks, ws.att_row_prefix, ws.err, (int)blockIdx.x, (int)gridDim.x);
}

template <int D>
struct Frag;
template <>
struct Frag<128> {
    typedef uint4 vec;                       // 8 bf16
    static constexpr int E = 8;
    static __device__ __forceinline__ float4v mma(vec a, vec b, float4v c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ vec zero() { return make_uint4(0, 0, 0, 0); }
    static __device__ __forceinline__ vec ld(const vec* p) {     // K and V rows are read once per call: a streaming load
        const v4u t = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p));
        return make_uint4(t.x, t.y, t.z, t.w);
    }
    static __device__ __forceinline__ unsigned word(vec x, int w) { return w == 0 ? x.x : (w == 1 ? x.y : (w == 2 ? x.z : x.w)); }
};
template <>
struct Frag<64> {
    typedef uint2 vec;                       // 4 bf16
    static constexpr int E = 4;
    static __device__ __forceinline__ float4v mma(vec a, vec b, float4v c) {
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(short4v, a), __builtin_bit_cast(short4v, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ vec zero() { return make_uint2(0, 0); }
    static __device__ __forceinline__ vec ld(const vec* p) {
        const v2u t = __builtin_nontemporal_load(reinterpret_cast<const v2u*>(p));
        return make_uint2(t.x, t.y);
    }
    static __device__ __forceinline__ unsigned word(vec x, int w) { return w == 0 ? x.x : x.y; }
};

// partial layout: [slot][G][D + 2] = (m in base-2 units, l, o[D] unnormalised)
// SOFT: retention-gated attention of Sec. 2.2 - the logit of entry i gets the bias (t - i) log(beta_i),
// t = now[seq] (the weights beta^(t-i) e^z of the soft form); otherwise hard eviction, no bias.
// PAGED: the chunk is a run of pages of a paged cache - cd.first indexes the first of them in the block
// tables, cd.n counts their slots; slots with a negative position are empty and take no part (their
// logit is -inf and their V row, which may hold anything, is replaced by zeros).
template <int D, int G, bool SOFT, bool PAGED>
__global__ __launch_bounds__(ATT_THREADS) void k_att_partial(CacheView c, const uint16_t* __restrict__ q,
                                                             Shape sh, Workspace ws, int chunk,
                                                             float scale_log2, const int32_t* __restrict__ now,
                                                             int round_rows, int extra_base) {
    typedef Frag<D> F;
    typedef typename F::vec vec;
    constexpr int E = F::E;
    constexpr int NSTREAM = ATT_THREADS / 64;
    __shared__ float s_m[NSTREAM][G], s_l[NSTREAM][G];
    constexpr int SO = D + 8;                                     // a 32-byte skew between heads
    __shared__ __attribute__((aligned(16))) float s_o[NSTREAM][G][SO];

    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    // The grid is fixed (a few blocks per compute unit).  The rows of the layer range's segments, one segment after the
    // other (ws.att_row_prefix; N rows in all), are shared out equally: block b starts at the row b N / nb, rounded down
    // to a multiple of round_rows inside its segment (64: a round of the four wavefronts; a whole chunk when the
    // partial-result buffer has no extra slots to spare), and ends where block b + 1 starts.  A
    // block keeps ONE online-softmax state for as long as its rows belong to the same segment: a partial result is
    // written per (block, segment) run and not per chunk - at the slot of the chunk that the run starts with, or at
    // slot extra_base + b when the run starts inside a chunk (the block before it owns that chunk's slot).
    // On this GPU a stream of reads slows down by far more than the bytes suggest when result writes are mixed into
    // it (8.5 MB of writes in a 1.1 GB read stream cost 12 us of 170), so the fewer partial results the better.
    const int total = ws.att_chunk_prefix[sh.nseg];
    const int nb = min((int)gridDim.x, total);
    if ((int)blockIdx.x >= nb) return;
    const int64_t* rp = ws.att_row_prefix;
    const int64_t N = rp[sh.nseg];
    // where the rows e0 <= e1 of the concatenation lie: the segment s with rp[s] <= e < rp[s + 1] (nseg behind the last row)
    // and the round of rows inside it.  A 64-way search, both rows at once: every lane looks at one point of each
    // remaining range, so 4096 segments take two rounds of one load instead of twelve loads one after the other.
    int seg_b, row_b, seg_e, row_e;
    {
        const int64_t e0 = (int64_t)blockIdx.x * N / nb, e1 = (int64_t)(blockIdx.x + 1) * N / nb;
        int lo0 = 0, hi0 = sh.nseg, lo1 = 0, hi1 = sh.nseg;        // invariant: rp[lo] <= e < rp[hi]   (rp[0] = 0, rp[nseg] = N)
        while (hi0 - lo0 > 1 || hi1 - lo1 > 1) {
            const int st0 = (hi0 - lo0 + 63) / 64, st1 = (hi1 - lo1 + 63) / 64;   // lane l probes lo + (l + 1) stride
            const int i0 = lo0 + (lane + 1) * st0, i1 = lo1 + (lane + 1) * st1;
            const bool in0 = i0 < hi0 && rp[min(i0, sh.nseg)] <= e0, in1 = i1 < hi1 && rp[min(i1, sh.nseg)] <= e1;
            const int n0 = __popcll(__ballot(in0)), n1 = __popcll(__ballot(in1));   // (monotone: the first n lanes)
            hi0 = min(hi0, lo0 + (n0 + 1) * st0);
            lo0 += n0 * st0;
            hi1 = min(hi1, lo1 + (n1 + 1) * st1);
            lo1 += n1 * st1;
        }
        seg_b = e0 >= N ? sh.nseg : lo0;
        row_b = e0 >= N ? 0 : (int)(e0 - rp[lo0]) / round_rows * round_rows;
        seg_e = e1 >= N ? sh.nseg : lo1;
        row_e = e1 >= N ? 0 : (int)(e1 - rp[lo1]) / round_rows * round_rows;
    }
    if (seg_b == seg_e && row_b == row_e) return;                 // (shares of less than a round: a later block has the rows)
    const int c16 = lane & 15, b4 = lane >> 4;
    const vec* kp = reinterpret_cast<const vec*>(c.k);
    const vec* vp = reinterpret_cast<const vec*>(c.v);
    constexpr int VPR = D / E;                                    // vectors per row = 16

    // o[e][i] = unnormalised output of head c16, column E (4 b4 + i) + e (the MFMA accumulators of P.V)
    float4v o[E];
    float m, l;                                                   // m: running maximum of head c16 (the same in the four row groups)
    vec qf[4];
    int t_now = 0;
    auto reset = [&]() {
#pragma unroll
        for (int e = 0; e < E; ++e) o[e] = float4v{0.f, 0.f, 0.f, 0.f};
        m = -INFINITY;
        l = 0.f;
    };
    // the run's partial result goes to slot `slot`: the wavefronts' partials (the MFMAs have summed over a wavefront's
    // row groups already) meet in LDS, s_o[wave][head][(4 i + b4) E + e] = column E (4 b4 + i) + e, and are merged
    auto flush = [&](int slot) {
        float l_all = l;
        l_all += __shfl_xor(l_all, 16, 64);
        l_all += __shfl_xor(l_all, 32, 64);
        if (c16 < G) {
            if (b4 == 0) {
                s_m[wave][c16] = m;
                s_l[wave][c16] = l_all;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float* so = &s_o[wave][c16][(4 * i + b4) * E];
#pragma unroll
                for (int e4 = 0; e4 < E; e4 += 4)
                    *reinterpret_cast<float4*>(so + e4) = make_float4(o[e4][i], o[e4 + 1][i], o[e4 + 2][i], o[e4 + 3][i]);
            }
        }
        __syncthreads();
        float* part = ws.att_partial + (size_t)slot * G * (D + 2);
        for (int idx = tid; idx < G * D; idx += ATT_THREADS) {
            const int g = idx / D, d = idx % D;
            const int cb = d / E;
            const int so_at = (4 * (cb & 3) + (cb >> 2)) * E + d % E;
            float M = -INFINITY;
#pragma unroll
            for (int s2 = 0; s2 < NSTREAM; ++s2) M = fmaxf(M, s_m[s2][g]);
            const float Ms = M == -INFINITY ? 0.f : M;
            float accd = 0.f, lsum = 0.f;
#pragma unroll
            for (int s2 = 0; s2 < NSTREAM; ++s2) {
                const float w = __builtin_amdgcn_exp2f(s_m[s2][g] - Ms);
                accd += s_o[s2][g][so_at] * w;
                lsum += s_l[s2][g] * w;
            }
            part[g * (D + 2) + 2 + d] = accd;
            if (d == 0) {
                part[g * (D + 2)] = M;
                part[g * (D + 2) + 1] = lsum;
            }
        }
        __syncthreads();                                          // (the next run's partials may overwrite LDS)
    };
    for (int seg = seg_b; seg <= seg_e && seg < sh.nseg; ++seg) {
    const int c0 = ws.att_chunk_prefix[seg], c1 = ws.att_chunk_prefix[seg + 1];
    const int run_lo = seg == seg_b ? row_b : 0;                  // this block's rows of the segment: [run_lo, run_hi)
    const int run_hi = seg == seg_e ? row_e : (int)(rp[seg + 1] - rp[seg]);
    if (c0 >= c1 || run_lo >= run_hi) continue;                   // (uniform over the block)
    const int run_slot = run_lo % chunk == 0 ? c0 + run_lo / chunk : extra_base + (int)blockIdx.x;
    reset();
    {   // query fragments: lane (query c16, k-group b4), MFMA step j covers elements (4j + b4)*E ..
        const int seq = seg / sh.segs_per_seq, lh = seg % sh.segs_per_seq;
        const int layer = lh / sh.n_kv_heads, head = lh % sh.n_kv_heads;
        const int64_t qrow = ((int64_t)seq * sh.n_layers + layer) * sh.n_q_heads + (int64_t)head * G + c16;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            qf[j] = c16 < G ? reinterpret_cast<const vec*>(q + qrow * D)[4 * j + b4] : F::zero();
        t_now = SOFT ? now[seq] : 0;
    }
    const int ch_first = c0 + run_lo / chunk, ch_last = min(c1 - 1, c0 + (run_hi - 1) / chunk);
    for (int ch = ch_first; ch <= ch_last; ++ch) {
    const ChunkDesc cd = ws.att_desc[ch];
    int4 pgs = make_int4(0, 0, 0, 0);
    if (PAGED) pgs = reinterpret_cast<const int4*>(ws.att_pages)[ch];   // the chunk's pages, beside its descriptor
    const int ch_row0 = (ch - c0) * chunk;                        // the chunk's first row in the segment's numbering
    const int row_end = cd.n;                                     // the chunk's rows are [0, n) counted from cd.first ...
    const int off = max(run_lo - ch_row0, 0), row_stop = min(row_end, run_hi - ch_row0);   // ... and this block's are [off, row_stop)
    const int64_t base = cd.first;

    // PAGED: the (at most four) pages of the run come from the plan's table beside the descriptors, so no
    // load of the loop waits for a look-up in the block table
    int pg0 = 0, pg1 = 0, pg2 = 0, pg3 = 0;
    if (PAGED) {
        const int np = row_end >> 7, hi = (int)(c.cap >> 7) - 1;
        pg0 = min(max(pgs.x, 0), hi);
        pg1 = np > 1 ? min(max(pgs.y, 0), hi) : 0;
        pg2 = np > 2 ? min(max(pgs.z, 0), hi) : 0;
        pg3 = np > 3 ? min(max(pgs.w, 0), hi) : 0;
    }

    for (int r0 = off + wave * 16; r0 < row_stop; r0 += 64) {
        const int last = row_end - 1;
        int64_t rbase = base;                                     // entry of row 0 in this 16-row group's numbering
        if (PAGED) {                                              // 16 | page size: the group lies in one page
            const int pi = r0 >> 7;
            const int pg = pi == 0 ? pg0 : (pi == 1 ? pg1 : (pi == 2 ? pg2 : pg3));
            rbase = (int64_t)pg * KVTRIM_PAGE_SIZE - (r0 & ~(KVTRIM_PAGE_SIZE - 1));
        }
        // K in MFMA operand layout: lane -> row r0 + c16, vectors 4j + b4
        const int64_t krow = rbase + min(r0 + c16, last);
        vec kf[4], vf[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) kf[j] = F::ld(kp + krow * VPR + 4 * j + b4);
        // V coalesced: lane -> row r0 + 4*b4 + i, vector c16
#pragma unroll
        for (int i = 0; i < 4; ++i) vf[i] = F::ld(vp + (rbase + min(r0 + 4 * b4 + i, last)) * VPR + c16);
        int ps[4] = {0, 0, 0, 0};                                 // PAGED: the positions of the lane's slots, asked for with the rows
        if (PAGED) {
#pragma unroll
            for (int i = 0; i < 4; ++i) ps[i] = c.pos[rbase + min(r0 + 4 * b4 + i, last)];
        }

        float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) acc = F::mma(kf[j], qf[j], acc);
        // acc[i] = q(c16) . k(r0 + 4*b4 + i)
        float z[4];
        float tmax = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = r0 + 4 * b4 + i;
            const int64_t e = rbase + min(row, last);
            float zi = acc[i] * scale_log2;
            if (SOFT) zi = fmaf((float)(t_now - c.pos[e]) * c.log_beta[e], 1.4426950408889634f, zi);
            bool valid = row < row_end;
            if (PAGED) {                                          // an empty slot takes no part
                valid = valid && ps[i] >= 0;
                if (!valid) vf[i] = F::zero();
            }
            z[i] = valid ? zi : -INFINITY;
            tmax = fmaxf(tmax, z[i]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));             // over the tile's 16 rows: P.V sums over all of them
        const float m_new = fmaxf(m, tmax);
        const float m_safe = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m - m_safe);   // m = -inf gives 0; l and o are 0 then
        float p[4];
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            p[i] = __builtin_amdgcn_exp2f(z[i] - m_safe);
            psum += p[i];
        }
        l = l * alpha + psum;                                     // (this row group's share; summed over the groups at the end)
        m = m_new;
        if (__any(alpha != 1.0f)) {
#pragma unroll
            for (int e = 0; e < E; ++e) o[e] *= alpha;
        }
        // P.V on the matrix cores: lane (b4, c16) holds, for every column of its slice, the values of its 4 rows - 4
        // consecutive slots of the reduction dimension of a 16x16x32 MFMA with m = the column block c16 - and the
        // probabilities of the same rows for head c16, the other operand (n = c16).  A probability goes in as two
        // bf16 terms, the rounded value (slots 0..3) and the rounded remainder (slots 4..7, against the same V values
        // again), so every product is exact to 2^-16; the sums are fp32.  One MFMA per column of the slice.
        const bf16x2 h01 = {(__bf16)p[0], (__bf16)p[1]}, h23 = {(__bf16)p[2], (__bf16)p[3]};
        const bf16x2 l01 = {(__bf16)(p[0] - (float)h01.x), (__bf16)(p[1] - (float)h01.y)};
        const bf16x2 l23 = {(__bf16)(p[2] - (float)h23.x), (__bf16)(p[3] - (float)h23.y)};
        const uint4 pb = make_uint4(__builtin_bit_cast(unsigned, h01), __builtin_bit_cast(unsigned, h23),
                                    __builtin_bit_cast(unsigned, l01), __builtin_bit_cast(unsigned, l23));
#pragma unroll
        for (int w = 0; w < E / 2; ++w) {
            const unsigned x0 = F::word(vf[0], w), x1 = F::word(vf[1], w), x2 = F::word(vf[2], w), x3 = F::word(vf[3], w);
            // columns 2 w (low halves) and 2 w + 1 (high halves) of the four rows
            const unsigned a01 = __builtin_amdgcn_perm(x1, x0, 0x05040100u), a23 = __builtin_amdgcn_perm(x3, x2, 0x05040100u);
            const unsigned b01 = __builtin_amdgcn_perm(x1, x0, 0x07060302u), b23 = __builtin_amdgcn_perm(x3, x2, 0x07060302u);
            o[2 * w] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, make_uint4(a01, a23, a01, a23)),
                                                               __builtin_bit_cast(bf16x8, pb), o[2 * w], 0, 0, 0);
            o[2 * w + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, make_uint4(b01, b23, b01, b23)),
                                                                   __builtin_bit_cast(bf16x8, pb), o[2 * w + 1], 0, 0, 0);
        }
    }

    }                                                             // (chunks of the run)
    flush(run_slot);
    }                                                             // (segments of the block)
}

// One block per segment of the layer range: merges the partial results of its chunks, a tile
// of COMB_TILE chunks at a time.  Phase A brings the tile's (m, l) pairs into LDS and turns
// them into weights 2^(m - M); phase B lets every thread sum "its" (query head, d) column over
// the tile with loads that do not depend on each other, so all of them are in flight at once.
constexpr int COMB_TILE = 128;
constexpr int COMB_THREADS = 512;
static_assert(COMB_THREADS / 64 >= 8, "one wavefront of the merge kernel per query head of a group");
// Housekeeping that nothing in this launch reads rides behind the merging blocks of the grid, so that it needs no
// launch of its own:
//   EXTRA_TIDY (the paged decode step in one call): one block per segment takes the pages emptied by the step's
//              eviction out of the segment's block table;
//   EXTRA_UNSTAGE (the in-place compaction with attention): one wavefront per chunk of the row mover's table puts the
//              rows that the mover parked into their places.
constexpr int EXTRA_NONE = 0, EXTRA_TIDY = 1, EXTRA_UNSTAGE = 2;
struct CombineExtra {
    PagedView tidy;
    CacheViewMut c, stage;
    const int32_t* kept;
};

// PERSIST: the partial results come from k_att_partial's fixed grid of persist_nb blocks - one per (block, segment)
// run, at the slot of the run's first chunk or, for a run that starts inside a chunk, at slot extra_base + block -
// and not one per chunk (the fused row mover's partials).
template <int D, int EXTRA, bool PERSIST>
__global__ __launch_bounds__(COMB_THREADS) void k_att_combine(Shape sh, Workspace ws,
                                                              const int32_t* __restrict__ chunk_prefix,
                                                              int layer_begin, int layer_end,
                                                              float* __restrict__ out, float* __restrict__ lse,
                                                              CombineExtra ex, int persist_nb, int round_rows,
                                                              int chunk_rows, int extra_base) {
    __shared__ float s_m[COMB_TILE][8], s_w[COMB_TILE][8], s_l[COMB_TILE][8];
    __shared__ float s_M[8], s_a[8], s_L[8];
    const int G = sh.group;
    const int nl = layer_end - layer_begin;
    const int per = nl * sh.n_kv_heads;
    if (EXTRA != EXTRA_NONE && (int)blockIdx.x >= sh.n_seq * per) {
        const int xb = (int)blockIdx.x - sh.n_seq * per;
        if (EXTRA == EXTRA_TIDY) tidy_segment<COMB_THREADS>(ex.tidy, xb, ws.err);
        if (EXTRA == EXTRA_UNSTAGE) unstage_chunk<D>(ex.c, ex.stage, ex.kept, sh, ws, xb * (COMB_THREADS / 64) + (int)(threadIdx.x >> 6));
        return;
    }
    const int seq = blockIdx.x / per, r = blockIdx.x % per;
    const int layer = layer_begin + r / sh.n_kv_heads, head = r % sh.n_kv_heads;
    const int seg = (seq * sh.n_layers + layer) * sh.n_kv_heads + head;
    if (__hip_atomic_load(ws.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;   // tables may be stale
    const int c0 = chunk_prefix[seg];
    const int c1 = min(chunk_prefix[seg + 1], (int)ws.max_att_chunks);
    const int64_t hq0 = ((int64_t)seq * sh.n_layers + layer) * sh.n_q_heads + (int64_t)head * G;
    const float LN2 = 0.6931471805599453f;
    constexpr int PAIRS = (8 * D + COMB_THREADS - 1) / COMB_THREADS;   // (query head, d) pairs per thread, G <= 8
    const int tid = threadIdx.x;
    float acc[PAIRS];
#pragma unroll
    for (int p = 0; p < PAIRS; ++p) acc[p] = 0.f;
    if (tid < 8) {
        s_M[tid] = -INFINITY;
        s_L[tid] = 0.f;
    }
    const size_t stride = (size_t)G * (D + 2);
    // entries to merge: entry e sits at slot_of(e).  PERSIST: block b of the attention kernel started at row b N / nb of
    // the concatenated segments (ws.att_row_prefix), rounded down to a multiple of round_rows inside its segment, and
    // ended where block b + 1 started.  The blocks that had rows of this segment are b0 - the last one that starts at
    // or before the segment's first row - up to b1, the last one that starts inside it; each left one partial result:
    // b0 at slot c0, a later one at the slot of the chunk it started with or, if it started inside a chunk, at its own
    // extra slot.  (A block whose start and end round to the same row had nothing to do: weight zero.)
    int n = c1 - c0, b0 = 0, nb = 1;
    int64_t N = 0, r0s = 0, r1s = 0;                              // rows of all segments / before this one / up to its end
    if (PERSIST) {
        const int64_t total = chunk_prefix[sh.nseg];
        N = ws.att_row_prefix[sh.nseg];
        r0s = ws.att_row_prefix[seg];
        r1s = ws.att_row_prefix[seg + 1];
        nb = (int)min((int64_t)persist_nb, total);
        if (c1 > c0 && r1s > r0s) {
            const int64_t lim0 = min(r0s + round_rows, r1s);      // starts below this row round down to the segment's first
            b0 = (int)((lim0 * nb + N - 1) / N) - 1;
            n = (int)((r1s * nb + N - 1) / N) - 1 - b0 + 1;
        } else {
            n = 0;
        }
    }
    __shared__ int s_slot[PERSIST ? COMB_TILE : 1];               // PERSIST: the slots of the tile's entries (-1: nothing there)
    auto slot_of = [&](int e) -> int {
        if (!PERSIST) return c0 + e;
        if (e == 0) return c0;
        const int b = b0 + e;
        const int64_t eb = (int64_t)b * N / nb, en = (int64_t)(b + 1) * N / nb;
        const int row = (int)(eb - r0s) / round_rows * round_rows;
        if (en < r1s && (int)(en - r0s) / round_rows * round_rows == row) return -1;   // an empty share
        return row % chunk_rows == 0 ? c0 + row / chunk_rows : extra_base + b;
    };
    for (int t0 = 0; t0 < n; t0 += COMB_TILE) {
        const int nt = min(COMB_TILE, n - t0);
        __syncthreads();
        for (int i = tid; i < nt * G; i += COMB_THREADS) {
            const int slot = slot_of(t0 + i / G);
            if (PERSIST && i % G == 0) s_slot[i / G] = max(slot, c0);           // (an empty share: any slot, with weight zero)
            const float* p = ws.att_partial + (size_t)max(slot, c0) * stride + (size_t)(i % G) * (D + 2);
            s_m[i / G][i % G] = slot < 0 ? -INFINITY : p[0];
            s_l[i / G][i % G] = slot < 0 ? 0.f : p[1];
        }
        __syncthreads();
        const int wv = tid >> 6, ln = tid & 63;                    // wavefront g of the block serves query head g (G <= 8 wavefronts)
        if (wv < G) {                                             // running maximum and rescale factor per query head
            float tm = -INFINITY;
            for (int i = ln; i < nt; i += 64) tm = fmaxf(tm, s_m[i][wv]);
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) tm = fmaxf(tm, __shfl_xor(tm, d, 64));
            if (ln == 0) {
                const float old = s_M[wv];
                tm = fmaxf(tm, old);
                const float ms = tm == -INFINITY ? 0.f : tm;
                s_a[wv] = __builtin_amdgcn_exp2f(old - ms);
                s_M[wv] = tm;
            }
        }
        __syncthreads();
        for (int i = tid; i < nt * G; i += COMB_THREADS) {
            const float M = s_M[i % G];
            s_w[i / G][i % G] = __builtin_amdgcn_exp2f(s_m[i / G][i % G] - (M == -INFINITY ? 0.f : M));
        }
        __syncthreads();
        if (wv < G) {
            float lv = 0.f;
            for (int i = ln; i < nt; i += 64) lv += s_l[i][wv] * s_w[i][wv];
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) lv += __shfl_xor(lv, d, 64);
            if (ln == 0) s_L[wv] = s_L[wv] * s_a[wv] + lv;
        }
#pragma unroll
        for (int p = 0; p < PAIRS; ++p) {
            const int idx = tid + p * COMB_THREADS;
            if (idx >= G * D) break;
            const int g = idx / D, d = idx % D;
            const float* base = ws.att_partial + (size_t)g * (D + 2) + 2 + d;
            float av = acc[p] * s_a[g];
            int i = 0;
            for (; i + 8 <= nt; i += 8) {
                float x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = base[(size_t)(PERSIST ? s_slot[i + u] : c0 + t0 + i + u) * stride];
#pragma unroll
                for (int u = 0; u < 8; ++u) av = fmaf(x[u], s_w[i + u][g], av);
            }
            if (PERSIST) {                                        // (a handful of entries: all of them in flight at once)
                float x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = base[(size_t)s_slot[min(i + u, nt - 1)] * stride];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (i + u < nt) av = fmaf(x[u], s_w[i + u][g], av);
            } else {
                for (; i < nt; ++i) av = fmaf(base[(size_t)(c0 + t0 + i) * stride], s_w[i][g], av);
            }
            acc[p] = av;
        }
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < PAIRS; ++p) {
        const int idx = tid + p * COMB_THREADS;
        if (idx >= G * D) break;
        const int g = idx / D, d = idx % D;
        const float L = s_L[g];
        out[(hq0 + g) * D + d] = L > 0.f ? acc[p] / L : 0.f;
        if (d == 0 && lse) lse[hq0 + g] = L > 0.f ? (s_M[g] + __builtin_amdgcn_logf(L)) * LN2 : -INFINITY;
    }
}

template <int D, int G>
static void launch_partial(const CacheView& c, const uint16_t* q, const Shape& sh, const Workspace& ws,
                           int chunk, float scale_log2, const int32_t* now, bool paged, unsigned blocks,
                           int round_rows, int extra_base, hipStream_t st) {
    if (paged)
        hipLaunchKernelGGL((k_att_partial<D, G, false, true>), dim3(blocks), dim3(ATT_THREADS), 0, st, c, q, sh, ws, chunk, scale_log2, now, round_rows, extra_base);
    else if (now)
        hipLaunchKernelGGL((k_att_partial<D, G, true, false>), dim3(blocks), dim3(ATT_THREADS), 0, st, c, q, sh, ws, chunk, scale_log2, now, round_rows, extra_base);
    else
        hipLaunchKernelGGL((k_att_partial<D, G, false, false>), dim3(blocks), dim3(ATT_THREADS), 0, st, c, q, sh, ws, chunk, scale_log2, now, round_rows, extra_base);
}

template <int D>
static bool dispatch_partial(int G, const CacheView& c, const uint16_t* q, const Shape& sh, const Workspace& ws,
                             int chunk, float scale_log2, const int32_t* now, bool paged, unsigned blocks,
                             int round_rows, int extra_base, hipStream_t st) {
    switch (G) {
#define KVTRIM_CASE(g) case g: launch_partial<D, g>(c, q, sh, ws, chunk, scale_log2, now, paged, blocks, round_rows, extra_base, st); return true;
        KVTRIM_CASE(1) KVTRIM_CASE(2) KVTRIM_CASE(3) KVTRIM_CASE(4) KVTRIM_CASE(5) KVTRIM_CASE(6) KVTRIM_CASE(7) KVTRIM_CASE(8)
#undef KVTRIM_CASE
        default: return false;
    }
}

// The fixed grid of k_att_partial for a table of at most max_chunks chunks of `chunk` rows: nb blocks, whose shares
// start at multiples of 64 rows when the partial-result buffer has nb slots to spare behind the chunks' own (for the
// runs that start inside a chunk), else at whole chunks.
struct AttGrid {
    int nb, round_rows, chunk_rows, extra_base;
};
static AttGrid att_grid(const kvtrim_ctx* ctx, int64_t max_chunks, int chunk) {
    AttGrid g;
    g.nb = (int)(max_chunks < ctx->att_blocks ? max_chunks : ctx->att_blocks);
    g.extra_base = (int)max_chunks;
    g.chunk_rows = chunk;
    g.round_rows = max_chunks + g.nb <= ctx->ws.max_att_chunks && chunk % 64 == 0 ? 64 : chunk;
    return g;
}

int att_chunk_for(const kvtrim_ctx* ctx, int64_t cap) {
    int64_t chunk = (cap / 16384 + 63) / 64 * 64;
    return (int)(chunk < ctx->att_chunk_min ? ctx->att_chunk_min : chunk);
}

kvtrim_status launch_attn(kvtrim_ctx* ctx, const CacheView& c, const uint16_t* q, const int32_t* soft_now,
                          int32_t layer_begin, int32_t layer_end, float scale, float* out, float* lse,
                          hipStream_t st) {
    const Shape& sh = ctx->shape;
    const Workspace& ws = ctx->ws;
    const int chunk = att_chunk_for(ctx, c.cap);
    const int64_t max_chunks = c.cap / chunk + sh.nseg;
    const AttGrid ag = att_grid(ctx, max_chunks, chunk);
    const int nb = ag.nb;
    const float scale_log2 = scale * 1.4426950408889634f;
    { ProfScope prof(ctx, K_ATT_PLAN, st);
      hipLaunchKernelGGL(k_att_plan, dim3(ATT_PLAN_BLOCKS), dim3(1024), 0, st, c, sh, ws, chunk, layer_begin, layer_end, max_chunks); }
    bool ok;
    {
        ProfScope prof(ctx, K_ATT_PARTIAL, st);
        ok = sh.head_dim == 128
                  ? dispatch_partial<128>(sh.group, c, q, sh, ws, chunk, scale_log2, soft_now, false, (unsigned)nb, ag.round_rows, ag.extra_base, st)
                  : dispatch_partial<64>(sh.group, c, q, sh, ws, chunk, scale_log2, soft_now, false, (unsigned)nb, ag.round_rows, ag.extra_base, st);
    }
    if (!ok) return KVTRIM_EINVAL;
    return launch_combine(ctx, ws.att_chunk_prefix, layer_begin, layer_end, out, lse, st, nb, ag.round_rows, ag.chunk_rows, ag.extra_base);
}

// Attention over the page runs listed in ws.att_desc / ws.att_chunk_prefix (built by the paged plan
// kernel; the pages themselves are looked up in block_table): one block per run, then the
// per-segment merge.
kvtrim_status launch_attn_paged(kvtrim_ctx* ctx, const CacheView& pool, const int32_t* block_table, const uint16_t* q,
                                int max_chunks, int32_t layer_begin, int32_t layer_end, float scale, float* out,
                                float* lse, hipStream_t st, const PagedView* tidy) {
    const Shape& sh = ctx->shape;
    Workspace ws = ctx->ws;
    ws.pg_block_table = block_table;
    constexpr int chunk = ATT_PAGE_GROUP * KVTRIM_PAGE_SIZE;
    const AttGrid ag = att_grid(ctx, max_chunks, chunk);
    const int nb = ag.nb;
    const float scale_log2 = scale * 1.4426950408889634f;
    bool ok;
    {
        ProfScope prof(ctx, K_ATT_PARTIAL, st);
        ok = sh.head_dim == 128
                 ? dispatch_partial<128>(sh.group, pool, q, sh, ws, chunk, scale_log2, nullptr, true, (unsigned)nb, ag.round_rows, ag.extra_base, st)
                 : dispatch_partial<64>(sh.group, pool, q, sh, ws, chunk, scale_log2, nullptr, true, (unsigned)nb, ag.round_rows, ag.extra_base, st);
    }
    if (!ok) return KVTRIM_EINVAL;
    if (!tidy) return launch_combine(ctx, ws.att_chunk_prefix, layer_begin, layer_end, out, lse, st, nb, ag.round_rows, ag.chunk_rows, ag.extra_base);
    // the merge, and in the same launch one block per segment that tidies its block table
    CombineExtra ex{};
    ex.tidy = *tidy;
    const unsigned nblk = (unsigned)(sh.n_seq * (layer_end - layer_begin) * sh.n_kv_heads + sh.nseg);
    ProfScope prof(ctx, K_ATT_COMBINE, st);
    if (sh.head_dim == 128)
        hipLaunchKernelGGL((k_att_combine<128, EXTRA_TIDY, true>), dim3(nblk), dim3(COMB_THREADS), 0, st, sh, ws, ws.att_chunk_prefix, layer_begin, layer_end, out, lse, ex, nb, ag.round_rows, ag.chunk_rows, ag.extra_base);
    else
        hipLaunchKernelGGL((k_att_combine<64, EXTRA_TIDY, true>), dim3(nblk), dim3(COMB_THREADS), 0, st, sh, ws, ws.att_chunk_prefix, layer_begin, layer_end, out, lse, ex, nb, ag.round_rows, ag.chunk_rows, ag.extra_base);
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

// Merges the per-chunk partial results in ws.att_partial; chunk_prefix[g] .. chunk_prefix[g+1]
// are the chunks of segment g.
kvtrim_status launch_combine(kvtrim_ctx* ctx, const int32_t* chunk_prefix, int32_t layer_begin,
                             int32_t layer_end, float* out, float* lse, hipStream_t st, int persist_nb, int round_rows,
                             int chunk_rows, int extra_base) {
    const Shape& sh = ctx->shape;
    const Workspace& ws = ctx->ws;
    const unsigned nblk = (unsigned)(sh.n_seq * (layer_end - layer_begin) * sh.n_kv_heads);
    ProfScope prof(ctx, K_ATT_COMBINE, st);
    if (persist_nb > 0) {
        if (sh.head_dim == 128)
            hipLaunchKernelGGL((k_att_combine<128, EXTRA_NONE, true>), dim3(nblk), dim3(COMB_THREADS), 0, st, sh, ws, chunk_prefix, layer_begin, layer_end, out, lse, CombineExtra{}, persist_nb, round_rows, chunk_rows, extra_base);
        else
            hipLaunchKernelGGL((k_att_combine<64, EXTRA_NONE, true>), dim3(nblk), dim3(COMB_THREADS), 0, st, sh, ws, chunk_prefix, layer_begin, layer_end, out, lse, CombineExtra{}, persist_nb, round_rows, chunk_rows, extra_base);
    } else if (sh.head_dim == 128)
        hipLaunchKernelGGL((k_att_combine<128, EXTRA_NONE, false>), dim3(nblk), dim3(COMB_THREADS), 0, st, sh, ws, chunk_prefix, layer_begin, layer_end, out, lse, CombineExtra{}, 0, 1, 1, 0);
    else
        hipLaunchKernelGGL((k_att_combine<64, EXTRA_NONE, false>), dim3(nblk), dim3(COMB_THREADS), 0, st, sh, ws, chunk_prefix, layer_begin, layer_end, out, lse, CombineExtra{}, 0, 1, 1, 0);
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

// The merge after the in-place row mover: the launch also puts the rows that the mover parked in `stage` into their
// places (one wavefront per chunk of the mover's table, max_chunks of them) and commits the segments' new lengths.
kvtrim_status launch_combine_unstage(kvtrim_ctx* ctx, const int32_t* chunk_prefix, int32_t layer_begin, int32_t layer_end,
                                     float* out, float* lse, const CacheViewMut& c, const CacheViewMut& stage,
                                     const int32_t* kept, int64_t max_chunks, hipStream_t st) {
    const Shape& sh = ctx->shape;
    const Workspace& ws = ctx->ws;
    CombineExtra ex{};
    ex.c = c;
    ex.stage = stage;
    ex.kept = kept;
    const int64_t per_block = COMB_THREADS / 64;
    const unsigned nblk = (unsigned)(sh.n_seq * (layer_end - layer_begin) * sh.n_kv_heads + (max_chunks + per_block - 1) / per_block);
    ProfScope prof(ctx, K_ATT_COMBINE, st);
    if (sh.head_dim == 128)
        hipLaunchKernelGGL((k_att_combine<128, EXTRA_UNSTAGE, false>), dim3(nblk), dim3(COMB_THREADS), 0, st, sh, ws, chunk_prefix, layer_begin, layer_end, out, lse, ex, 0, 1, 1, 0);
    else
        hipLaunchKernelGGL((k_att_combine<64, EXTRA_UNSTAGE, false>), dim3(nblk), dim3(COMB_THREADS), 0, st, sh, ws, chunk_prefix, layer_begin, layer_end, out, lse, ex, 0, 1, 1, 0);
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

}  // namespace kvtrim
