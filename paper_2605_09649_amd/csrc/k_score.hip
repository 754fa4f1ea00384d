// Stage 1 (retention score in log domain) and the append support kernel.
#include "kvtrim_device.h"

namespace kvtrim {

// Sec. 4.2, Eq. (global_score) in log domain.  Lookahead 1: log G~ = (now + 1 - pos) * log(beta),
// one fp32 multiply.  Longer lookahead: the cached log of the tail sum is added by the same
// instruction, one correctly rounded fp32 fused multiply-add.  `bps` blocks share a segment and
// stride over its entries.
__global__ __launch_bounds__(256) void k_score(CacheView c, const int32_t* __restrict__ now,
                                               float* __restrict__ score, int segs_per_seq, int bps) {
    const int seg = blockIdx.x / bps, part = blockIdx.x % bps;
    const int len = c.seg_len[seg];
    const int64_t start = c.seg_start[seg];
    if (len < 0 || start < 0 || start + len > c.cap) return;     // never index outside the buffers
    const int t1 = now[seg / segs_per_seq] + 1;
    const float* lb = c.log_beta + start;
    const int32_t* pos = c.pos + start;
    float* out = score + start;
    if (c.log_tail) {
        const float* lt = c.log_tail + start;
        for (int64_t j = part * 256 + threadIdx.x; j < len; j += bps * 256)
            out[j] = __fmaf_rn((float)(t1 - pos[j]), lb[j], lt[j]);
    } else {
        for (int64_t j = part * 256 + threadIdx.x; j < len; j += bps * 256)
            out[j] = __fmul_rn((float)(t1 - pos[j]), lb[j]);
    }
}

kvtrim_status launch_score(kvtrim_ctx* ctx, const CacheView& c, const int32_t* now, float* score,
                           hipStream_t st) {
    const Shape& sh = ctx->shape;
    int64_t bps = c.cap / ((int64_t)sh.nseg * 1024);
    bps = bps < 1 ? 1 : (bps > 64 ? 64 : bps);
    ProfScope prof(ctx, K_SCORE, st);
    hipLaunchKernelGGL(k_score, dim3((unsigned)(sh.nseg * bps)), dim3(256), 0, st, c, now, score,
                       sh.segs_per_seq, (int)bps);
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

// Sec. 4.1, inner sum of the global capacity loss: occ[seq] = sum over the cached entries of the
// sequence of beta^(t - i) = exp((now - pos) log(beta)).  fp32 per entry, fp64 from the wavefront
// sum on; the blocks add into occ[seq] with fp64 atomics (so the last bits depend on their order).
__global__ __launch_bounds__(256) void k_occ_zero(double* __restrict__ occ, int n_seq) {
    for (int i = threadIdx.x; i < n_seq; i += 256) occ[i] = 0.0;
}

__global__ __launch_bounds__(256) void k_occupancy(CacheView c, const int32_t* __restrict__ now,
                                                   double* __restrict__ occ, int segs_per_seq, int bps) {
    __shared__ double lds[17];
    const int seg = blockIdx.x / bps, part = blockIdx.x % bps;
    const int len = c.seg_len[seg];
    const int64_t start = c.seg_start[seg];
    if (len < 0 || start < 0 || start + len > c.cap) return;     // uniform over the block
    const int seq = seg / segs_per_seq;
    const int t = now[seq];
    const float* lb = c.log_beta + start;
    const int32_t* pos = c.pos + start;
    double sum = 0.0;
    for (int64_t j = part * 256 + threadIdx.x; j < len; j += bps * 256)
        sum += (double)__builtin_amdgcn_exp2f((float)(t - pos[j]) * lb[j] * 1.4426950408889634f);
    sum = block_sum<double>(sum, lds);
    if (threadIdx.x == 0 && sum != 0.0) atomicAdd(&occ[seq], sum);
}

kvtrim_status launch_occupancy(kvtrim_ctx* ctx, const CacheView& c, const int32_t* now, double* occ,
                               hipStream_t st) {
    const Shape& sh = ctx->shape;
    int64_t bps = c.cap / ((int64_t)sh.nseg * 1024);
    bps = bps < 1 ? 1 : (bps > 64 ? 64 : bps);
    ProfScope prof(ctx, K_OCCUPANCY, st);
    hipLaunchKernelGGL(k_occ_zero, dim3(1), dim3(256), 0, st, occ, sh.n_seq);
    hipLaunchKernelGGL(k_occupancy, dim3((unsigned)(sh.nseg * bps)), dim3(256), 0, st, c, now, occ,
                       sh.segs_per_seq, (int)bps);
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

// One block per segment: copies the segment's new rows behind its end (16 bytes per lane) and the
// per-entry metadata, then bumps seg_len.  A segment takes its rows up to the first one with a
// negative position (sequences of a batch may bring different numbers of tokens: the others are
// padding).  A segment without room is left alone.
__global__ __launch_bounds__(256) void k_append(CacheViewMut c, const uint16_t* __restrict__ k_new,
                                                const uint16_t* __restrict__ v_new,
                                                const float* __restrict__ lb_new,
                                                const float* __restrict__ lt_new,
                                                const int32_t* __restrict__ pos_new, int n_new, int nseg,
                                                int head_dim, bool copy_rows, int32_t* __restrict__ old_len_out,
                                                int32_t* err) {
    __shared__ int s_cnt;
    const int seg = blockIdx.x;
    const int len = c.seg_len[seg];
    if (threadIdx.x == 0) {
        s_cnt = n_new;
        if (old_len_out) old_len_out[seg] = len;                  // whatever happens below: the entries before `len` are the old ones
    }
    __syncthreads();
    for (int i = threadIdx.x; i < n_new; i += blockDim.x)
        if (pos_new[(int64_t)seg * n_new + i] < 0) atomicMin(&s_cnt, i);
    __syncthreads();
    const int cnt = s_cnt;                                        // rows before the first padding row
    if (cnt == 0) return;
    const int64_t start = c.seg_start[seg];
    const int64_t limit = (seg + 1 < nseg) ? c.seg_start[seg + 1] : c.cap;
    if (len < 0 || start < 0 || limit > c.cap || start + len + cnt > limit) {
        if (threadIdx.x == 0) atomicOr(err, ERR_CAP);
        return;
    }
    const int vec_per_row = head_dim / 8;                         // uint4 (8 bf16) per row
    const uint4* ks = reinterpret_cast<const uint4*>(k_new) + (int64_t)seg * n_new * vec_per_row;
    const uint4* vs = reinterpret_cast<const uint4*>(v_new) + (int64_t)seg * n_new * vec_per_row;
    uint4* kd = reinterpret_cast<uint4*>(c.k) + (start + len) * vec_per_row;
    uint4* vd = reinterpret_cast<uint4*>(c.v) + (start + len) * vec_per_row;
    if (copy_rows) {
        for (int i = threadIdx.x; i < cnt * vec_per_row; i += blockDim.x) {
            kd[i] = ks[i];
            vd[i] = vs[i];
        }
    }
    for (int i = threadIdx.x; i < cnt; i += blockDim.x) {
        c.log_beta[start + len + i] = lb_new[(int64_t)seg * n_new + i];
        if (c.log_tail) c.log_tail[start + len + i] = lt_new[(int64_t)seg * n_new + i];
        c.pos[start + len + i] = pos_new[(int64_t)seg * n_new + i];
    }
    __syncthreads();
    if (threadIdx.x == 0) c.seg_len[seg] = len + cnt;
}

// min over the segments of the free slots behind them (up to the next segment's start, or the end of the buffers)
__global__ __launch_bounds__(1024) void k_min_room(CacheView c, int nseg, int32_t* __restrict__ out) {
    __shared__ int s_min;
    if (threadIdx.x == 0) s_min = 0x7fffffff;
    __syncthreads();
    int64_t mine = 0x7fffffff;
    for (int g = threadIdx.x; g < nseg; g += blockDim.x) {
        const int64_t end = c.seg_start[g] + c.seg_len[g];
        const int64_t limit = g + 1 < nseg ? c.seg_start[g + 1] : c.cap;
        mine = min(mine, limit - end);
    }
    atomicMin(&s_min, (int)max(min(mine, (int64_t)0x7fffffff), (int64_t)-0x7fffffff));
    __syncthreads();
    if (threadIdx.x == 0) out[0] = s_min;
}

kvtrim_status launch_min_room(kvtrim_ctx* ctx, const CacheView& c, int32_t* out, hipStream_t st) {
    hipLaunchKernelGGL(k_min_room, dim3(1), dim3(1024), 0, st, c, ctx->shape.nseg, out);
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

kvtrim_status launch_append(kvtrim_ctx* ctx, const CacheViewMut& c, const uint16_t* k_new, const uint16_t* v_new,
                            const float* lb_new, const float* lt_new, const int32_t* pos_new, int32_t n_new,
                            bool copy_rows, int32_t* old_len_out, hipStream_t st) {
    const Shape& sh = ctx->shape;
    ProfScope prof(ctx, K_APPEND, st);
    hipLaunchKernelGGL(k_append, dim3(sh.nseg), dim3(256), 0, st, c, k_new, v_new, lb_new, lt_new, pos_new, n_new,
                       sh.nseg, sh.head_dim, copy_rows, old_len_out, ctx->ws.err);
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

}  // namespace kvtrim
