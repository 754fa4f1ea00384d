// Retention gate for tokens that enter the cache (Sec. 4.1, "Weight-tied retention gates";
// Sec. 3.2: beta is computed once, at insertion):
//     u = silu(W1_l x + c1_l)                       one first layer per transformer block, width d_g
//     p = W2_{l,h} u + c2_{l,h}                     second layer of Proj per (block, KV head), width d_p
//     z = w_g . p + b_g,  beta = sigmoid(z)         readout tied across all layers and heads
// The outputs are log(beta) and, for a lookahead horizon H != 1, log(sum_{k<H} beta^k) - the two
// per-entry constants the score stage reads.
//
// Both layers are dense contractions and run on the matrix cores (MFMA 16x16x32 bf16, fp32
// accumulation); with one token per sequence they are bound by streaming the weights once from
// HBM, and the unused token columns of the MFMA tile cost nothing.
//   k_gate_hidden   a block owns 16 rows of W1 of one layer and up to 64 tokens; its four
//                   wavefronts split the contraction over d_model, are summed through LDS, and
//                   write u in fp32.
//   k_gate_readout  a block owns one (layer, head) and 16 tokens; u is split into two bf16 numbers
//                   (u = hi + lo to 2^-17 relative) so that the second layer keeps fp32-like
//                   accuracy on the bf16 matrix cores; every wavefront takes 16-row tiles of W2,
//                   folds its rows with w_g, and the block adds b_g and applies log-sigmoid.
// The contraction index may be permuted freely as long as both operands use the same permutation:
// a lane loads 32 contiguous bytes of its row per 64-wide step (so four lanes read one full
// 128-byte line) and feeds the two halves to two MFMAs.
#include "kvtrim_device.h"

namespace kvtrim {

typedef __attribute__((ext_vector_type(4))) float gate_f4;
typedef __attribute__((ext_vector_type(8))) __bf16 gate_bf8;

__device__ __forceinline__ gate_f4 mma_bf16(uint4 a, uint4 b, gate_f4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(gate_bf8, a), __builtin_bit_cast(gate_bf8, b), c, 0, 0, 0);
}

struct GateView {
    const uint16_t* w1;      // [L][d_g][d_model]
    const float* c1;         // [L][d_g]
    const uint16_t* w2;      // [L][H][d_p][d_g]
    const float* c2;         // [L][H][d_p]
    const float* w_g;        // [d_p]
    float b_g;
    int d_model, d_g, d_p;
};

constexpr int GH_THREADS = 256;          // four wavefronts split d_model
constexpr int GH_ROWS = 16;

// x: bf16 [layers of the range][n_tok][d_model]; u: fp32 [layers of the range][n_tok][d_g]
template <int NT>
__global__ __launch_bounds__(GH_THREADS) void k_gate_hidden(GateView g, const uint16_t* __restrict__ x, int n_tok,
                                                            int layer_begin, float* __restrict__ u) {
    __shared__ float s_part[4][NT][16][17];
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int r16 = lane & 15, g4 = lane >> 4;
    const int row0 = blockIdx.x * GH_ROWS;
    const int lr = blockIdx.y;                                       // layer of the range
    const int layer = layer_begin + lr;
    const int tok0 = blockIdx.z * 16 * NT;
    const int kw = g.d_model >> 2;                                   // contraction share of a wavefront
    const int k_begin = wave * kw;

    const uint4* arow = reinterpret_cast<const uint4*>(g.w1 + ((size_t)layer * g.d_g + row0 + r16) * g.d_model + k_begin + 16 * g4);
    const uint4* brow[NT];
    bool bval[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int tok = tok0 + 16 * t + r16;
        bval[t] = tok < n_tok;
        brow[t] = reinterpret_cast<const uint4*>(x + ((size_t)lr * n_tok + (bval[t] ? tok : 0)) * g.d_model + k_begin + 16 * g4);
    }
    gate_f4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = gate_f4{0.f, 0.f, 0.f, 0.f};

    // 64 contraction indices per step (8 uint4 of a row); four steps of weights are loaded ahead
    constexpr int AHEAD = 4;
    const int steps = kw >> 6;                                       // kw is a multiple of 64
    for (int s0 = 0; s0 < steps; s0 += AHEAD) {
        uint4 a[AHEAD][2];
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) {
            if (s0 + i < steps) {
                a[i][0] = arow[(s0 + i) * 8];
                a[i][1] = arow[(s0 + i) * 8 + 1];
            } else {
                a[i][0] = a[i][1] = make_uint4(0, 0, 0, 0);
            }
        }
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) {
            if (s0 + i < steps) {
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    uint4 b0 = make_uint4(0, 0, 0, 0), b1 = b0;
                    if (bval[t]) {
                        b0 = brow[t][(s0 + i) * 8];
                        b1 = brow[t][(s0 + i) * 8 + 1];
                    }
                    acc[t] = mma_bf16(a[i][0], b0, acc[t]);
                    acc[t] = mma_bf16(a[i][1], b1, acc[t]);
                }
            }
        }
    }
    // acc[t][r] = partial of (row 4*g4 + r, token r16 of tile t)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) s_part[wave][t][4 * g4 + r][r16] = acc[t][r];
    __syncthreads();
    for (int idx = tid; idx < NT * 256; idx += GH_THREADS) {
        const int t = idx >> 8, tk = (idx >> 4) & 15, row = idx & 15;
        const int tok = tok0 + 16 * t + tk;
        if (tok < n_tok) {
            const float a = s_part[0][t][row][tk] + s_part[1][t][row][tk] + s_part[2][t][row][tk] + s_part[3][t][row][tk] +
                            g.c1[(size_t)layer * g.d_g + row0 + row];
            u[((size_t)lr * n_tok + tok) * g.d_g + row0 + row] = a / (1.0f + __expf(-a));
        }
    }
}

// The same first layer for many tokens (prefill, chunked prefill): a 128 x 128 output tile per block,
// 64-wide steps of both operands staged through LDS (the next step's global loads are in flight in
// registers while the current one is multiplied), 2 x 2 wavefronts of 64 x 64, i.e. 4 x 4 MFMA tiles
// each.  Both operands are contiguous along the contraction, so global loads, LDS rows and MFMA
// operands all use the same 16-byte pieces; LDS rows are padded by 16 bytes against bank conflicts.
// Measured (4096 tokens, the metric model): 175 TFLOP/s, 7 % of the MFMA peak - the matrix pipe is busy 7 % of
// the time and the L2 misses fetch 10.8 GB for 1.2 GB of distinct operands (a 128-token tile is shared by only
// four blocks, and the 4 MB of W1_l do not stay in a 4 MB L2 while tokens stream through it).  Re-mapping blocks
// so that a layer stays on one XCD, a second register stage, and rotating the start of the contraction per block
// changed nothing or made it slower; the fix is a tile that spans all rows of W1_l.  Not built: this kernel only
// serves prefill-sized calls, which are not on the decode path.
constexpr int GG_BM = 128, GG_BN = 128, GG_BK = 64, GG_LD = GG_BK + 8;

__global__ __launch_bounds__(256) void k_gate_hidden_gemm(GateView g, const uint16_t* __restrict__ x, int n_tok,
                                                          int layer_begin, float* __restrict__ u) {
    __shared__ __align__(16) uint16_t sA[GG_BM][GG_LD], sB[GG_BN][GG_LD];
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int r16 = lane & 15, g4 = lane >> 4;
    const int wm = wave >> 1, wn = wave & 1;
    const int bm = blockIdx.x * GG_BM, bn = blockIdx.y * GG_BN;
    const int lr = blockIdx.z;
    const int layer = layer_begin + lr;
    const uint16_t* abase = g.w1 + (size_t)layer * g.d_g * g.d_model;
    const uint16_t* bbase = x + (size_t)lr * n_tok * g.d_model;

    // this thread's four 16-byte pieces of each operand tile: row = piece / 8, column piece % 8
    const uint4* ap[4];
    const uint4* bp[4];
    bool av[4], bv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int piece = tid + 256 * i, row = piece >> 3, cc = piece & 7;
        av[i] = bm + row < g.d_g;
        bv[i] = bn + row < n_tok;
        ap[i] = reinterpret_cast<const uint4*>(abase + (size_t)(av[i] ? bm + row : 0) * g.d_model + cc * 8);
        bp[i] = reinterpret_cast<const uint4*>(bbase + (size_t)(bv[i] ? bn + row : 0) * g.d_model + cc * 8);
    }
    gate_f4 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = gate_f4{0.f, 0.f, 0.f, 0.f};

    const uint4 zero = make_uint4(0, 0, 0, 0);
    const int steps = g.d_model / GG_BK;
    auto fetch = [&](int kt, uint4 (&ra)[4], uint4 (&rb)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            ra[i] = av[i] ? ap[i][kt * (GG_BK / 8)] : zero;
            rb[i] = bv[i] ? bp[i][kt * (GG_BK / 8)] : zero;
        }
    };
    auto stage = [&](const uint4 (&ra)[4], const uint4 (&rb)[4]) {
        __syncthreads();                                             // the previous step's LDS reads are done
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int piece = tid + 256 * i, row = piece >> 3, cc = piece & 7;
            *reinterpret_cast<uint4*>(&sA[row][cc * 8]) = ra[i];
            *reinterpret_cast<uint4*>(&sB[row][cc * 8]) = rb[i];
        }
        __syncthreads();
    };
    auto multiply = [&]() {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            uint4 a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = *reinterpret_cast<const uint4*>(&sA[wm * 64 + i * 16 + r16][s * 32 + 8 * g4]);
                b[i] = *reinterpret_cast<const uint4*>(&sB[wn * 64 + i * 16 + r16][s * 32 + 8 * g4]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = mma_bf16(a[i], b[j], acc[i][j]);
        }
    };
    uint4 ra[4], rb[4];
    fetch(0, ra, rb);
    for (int kt = 0; kt < steps; ++kt) {
        stage(ra, rb);
        if (kt + 1 < steps) fetch(kt + 1, ra, rb);                   // in flight while this step is multiplied
        multiply();
    }
    // acc[i][j][r] = (row bm + wm*64 + i*16 + 4*g4 + r, token bn + wn*64 + j*16 + r16)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int tok = bn + wn * 64 + j * 16 + r16;
        if (tok >= n_tok) continue;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = bm + wm * 64 + i * 16 + 4 * g4;
            if (row >= g.d_g) continue;                              // d_g is a multiple of 64: whole groups of four
            const float4 c = *reinterpret_cast<const float4*>(g.c1 + (size_t)layer * g.d_g + row);
            float4 o;
            float t;
            t = acc[i][j][0] + c.x; o.x = t / (1.0f + __expf(-t));
            t = acc[i][j][1] + c.y; o.y = t / (1.0f + __expf(-t));
            t = acc[i][j][2] + c.z; o.z = t / (1.0f + __expf(-t));
            t = acc[i][j][3] + c.w; o.w = t / (1.0f + __expf(-t));
            *reinterpret_cast<float4*>(u + ((size_t)lr * n_tok + tok) * g.d_g + row) = o;
        }
    }
}

constexpr int GR_THREADS = 512;          // eight wavefronts share the 16-row tiles of W2
constexpr int GR_KC = 512;               // contraction chunk staged in LDS
constexpr int GR_LD = GR_KC + 8;         // padded row of the staged chunk (elements)

__device__ __forceinline__ uint16_t bf16_rne(float f) {
    uint32_t b = __float_as_uint(f);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return (uint16_t)(b >> 16);
}

__device__ __forceinline__ float log_sigmoid(float z) {
    return z >= 0.f ? -log1pf(expf(-z)) : z - log1pf(expf(z));
}

// log sum_{k<H} beta^k from log(beta); H <= 0: the limit -log(1 - beta)
__device__ __forceinline__ float log_tail_of(float lb, int horizon) {
    if (horizon <= 0) return -logf(-expm1f(lb));
    const float beta = expf(lb);
    float sum = 0.f, term = 1.f;
    for (int k = 0; k < horizon; ++k) {
        sum += term;
        term *= beta;
    }
    return logf(sum);
}

__global__ __launch_bounds__(GR_THREADS) void k_gate_readout(GateView g, const float* __restrict__ u, int n_tok,
                                                             int layer_begin, int n_layers, int n_heads, int horizon,
                                                             float* __restrict__ log_beta_out,
                                                             float* __restrict__ log_tail_out) {
    __shared__ __align__(16) uint16_t s_hi[16][GR_LD], s_lo[16][GR_LD];
    __shared__ float s_z[GR_THREADS / 64][16];
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int r16 = lane & 15, g4 = lane >> 4;
    const int head = blockIdx.x, lr = blockIdx.y, layer = layer_begin + lr;
    const int tok0 = blockIdx.z * 16;
    const int row_tiles = (g.d_p + 15) >> 4;
    const uint16_t* w2 = g.w2 + ((size_t)layer * n_heads + head) * g.d_p * g.d_g;
    const float* c2 = g.c2 + ((size_t)layer * n_heads + head) * g.d_p;

    float zacc = 0.f;                                                // sum over this lane's rows of w_g[row] * (p[row]) for token r16
    for (int kc = 0; kc < g.d_g; kc += GR_KC) {
        const int kn = min(GR_KC, g.d_g - kc);                       // multiple of 64
        __syncthreads();
        for (int idx = tid; idx < 16 * kn; idx += GR_THREADS) {      // stage u[tok0 .. tok0+16)[kc .. kc+kn) as hi + lo
            const int tk = idx / kn, k = idx - tk * kn;
            const int tok = tok0 + tk;
            const float f = tok < n_tok ? u[((size_t)lr * n_tok + tok) * g.d_g + kc + k] : 0.f;
            const uint16_t hi = bf16_rne(f);
            s_hi[tk][k] = hi;
            s_lo[tk][k] = bf16_rne(f - __uint_as_float((uint32_t)hi << 16));
        }
        __syncthreads();
        for (int rt = wave; rt < row_tiles; rt += GR_THREADS / 64) {
            const int row = rt * 16 + r16;
            const bool rv = row < g.d_p;
            const uint4* arow = reinterpret_cast<const uint4*>(w2 + (size_t)(rv ? row : 0) * g.d_g + kc + 16 * g4);
            gate_f4 acc = {0.f, 0.f, 0.f, 0.f};
            for (int s = 0; s < (kn >> 6); ++s) {
                uint4 a0 = make_uint4(0, 0, 0, 0), a1 = a0;
                if (rv) {
                    a0 = arow[s * 8];
                    a1 = arow[s * 8 + 1];
                }
                const int kk = s * 64 + 16 * g4;
                const uint4 h0 = *reinterpret_cast<const uint4*>(&s_hi[r16][kk]);
                const uint4 h1 = *reinterpret_cast<const uint4*>(&s_hi[r16][kk + 8]);
                const uint4 l0 = *reinterpret_cast<const uint4*>(&s_lo[r16][kk]);
                const uint4 l1 = *reinterpret_cast<const uint4*>(&s_lo[r16][kk + 8]);
                acc = mma_bf16(a0, h0, acc);
                acc = mma_bf16(a1, h1, acc);
                acc = mma_bf16(a0, l0, acc);
                acc = mma_bf16(a1, l1, acc);
            }
            // acc[r] = contribution of this chunk to p[row 16*rt + 4*g4 + r] for token r16
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int pr = rt * 16 + 4 * g4 + r;
                if (pr < g.d_p) zacc = fmaf(g.w_g[pr], acc[r] + (kc == 0 ? c2[pr] : 0.f), zacc);
            }
        }
    }
    zacc += __shfl_xor(zacc, 16, 64);
    zacc += __shfl_xor(zacc, 32, 64);
    if (lane < 16) s_z[wave][lane] = zacc;
    __syncthreads();
    if (tid < 16) {
        const int tok = tok0 + tid;
        if (tok < n_tok) {
            float z = g.b_g;
#pragma unroll
            for (int w = 0; w < GR_THREADS / 64; ++w) z += s_z[w][tid];
            const float lb = log_sigmoid(z);
            const size_t o = ((size_t)tok * n_layers + layer) * n_heads + head;
            log_beta_out[o] = lb;
            if (log_tail_out) log_tail_out[o] = log_tail_of(lb, horizon);
        }
    }
}

kvtrim_status launch_gate(kvtrim_ctx* ctx, const GateView& g, const uint16_t* x, int n_tok, int layer_begin, int layer_end,
                          int horizon, float* scratch, float* log_beta_out, float* log_tail_out, hipStream_t st) {
    const int nl = layer_end - layer_begin;
    {
        ProfScope prof(ctx, K_GATE_HIDDEN, st);
        const dim3 grid1(g.d_g / GH_ROWS, nl, 1);
        if (n_tok <= 16)
            hipLaunchKernelGGL(k_gate_hidden<1>, dim3(grid1.x, nl, 1), dim3(GH_THREADS), 0, st, g, x, n_tok, layer_begin, scratch);
        else if (n_tok <= 32)
            hipLaunchKernelGGL(k_gate_hidden<2>, dim3(grid1.x, nl, 1), dim3(GH_THREADS), 0, st, g, x, n_tok, layer_begin, scratch);
        else if (n_tok < 256)                                        // below that the tiled kernel cannot fill the chip
            hipLaunchKernelGGL(k_gate_hidden<4>, dim3(grid1.x, nl, (n_tok + 63) / 64), dim3(GH_THREADS), 0, st, g, x, n_tok,
                               layer_begin, scratch);
        else
            hipLaunchKernelGGL(k_gate_hidden_gemm, dim3((g.d_g + GG_BM - 1) / GG_BM, (n_tok + GG_BN - 1) / GG_BN, nl), dim3(256), 0,
                               st, g, x, n_tok, layer_begin, scratch);
    }
    {
        ProfScope prof(ctx, K_GATE_READOUT, st);
        hipLaunchKernelGGL(k_gate_readout, dim3(ctx->shape.n_kv_heads, nl, (n_tok + 15) / 16), dim3(GR_THREADS), 0, st, g, scratch,
                           n_tok, layer_begin, ctx->shape.n_layers, ctx->shape.n_kv_heads, horizon, log_beta_out, log_tail_out);
    }
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

}  // namespace kvtrim

using namespace kvtrim;

extern "C" {

size_t kvtrim_gate_scratch_bytes(const kvtrim_gate* g, int32_t n_tok, int32_t n_layers) {
    if (!g || n_tok < 1 || n_layers < 1 || g->d_g < 1) return 0;
    return (size_t)n_tok * (size_t)n_layers * (size_t)g->d_g * sizeof(float);
}

kvtrim_status kvtrim_gate_forward(kvtrim_ctx* ctx, const kvtrim_gate* g, const void* x, int32_t n_tok, int32_t layer_begin,
                                  int32_t layer_end, int32_t horizon, void* scratch, float* log_beta_out,
                                  float* log_tail_out, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    auto bad = [&](const char* why) {
        snprintf(ctx->last_error, sizeof(ctx->last_error), "invalid argument: %s", why);
        return KVTRIM_EINVAL;
    };
    if (!g || !g->w1 || !g->c1 || !g->w2 || !g->c2 || !g->w_g) return bad("gate or one of its weight pointers is NULL");
    if (!x || !scratch || !log_beta_out) return bad("x / scratch / log_beta_out is NULL");
    if (g->d_model < 256 || g->d_model % 256) return bad("d_model must be a positive multiple of 256");
    if (g->d_g < 64 || g->d_g % 64) return bad("d_g must be a positive multiple of 64");
    if (g->d_p < 1) return bad("d_p < 1");
    if (n_tok < 1) return bad("n_tok < 1");
    if ((int64_t)n_tok > 65535 * 16) return bad("n_tok too large for one call");
    if ((((uintptr_t)g->c1) | ((uintptr_t)g->w_g)) & 15) return bad("c1 / w_g not 16-byte aligned");
    if (layer_begin < 0 || layer_end > ctx->cfg.n_layers || layer_begin >= layer_end) return bad("empty or out-of-range layer range");
    if (horizon < 0 || horizon > 4096) return bad("horizon outside [0, 4096] (0 = infinite)");
    if ((((uintptr_t)x) | ((uintptr_t)g->w1) | ((uintptr_t)g->w2) | ((uintptr_t)scratch)) & 15)
        return bad("x / w1 / w2 / scratch not 16-byte aligned");
    if (!(g->b_g == g->b_g)) return bad("b_g is NaN");
    GateView v;
    v.w1 = (const uint16_t*)g->w1;
    v.c1 = g->c1;
    v.w2 = (const uint16_t*)g->w2;
    v.c2 = g->c2;
    v.w_g = g->w_g;
    v.b_g = g->b_g;
    v.d_model = g->d_model;
    v.d_g = g->d_g;
    v.d_p = g->d_p;
    return launch_gate(ctx, v, (const uint16_t*)x, n_tok, layer_begin, layer_end, horizon, (float*)scratch, log_beta_out,
                       log_tail_out, (hipStream_t)hip_stream);
}

}  // extern "C"
