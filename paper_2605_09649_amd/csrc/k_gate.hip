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
//   k_gate_hidden   a block owns 16 rows of W1 of one layer (64 rows when a call brings more than 16
//                   tokens) and up to 64 tokens; its four wavefronts split the contraction over
//                   d_model, are summed through LDS, and write u in fp32.
//   k_gate_readout  a block owns one (layer, head) and 16 tokens; u is split into two bf16 numbers
//                   (u = hi + lo to 2^-17 relative) so that the second layer keeps fp32-like
//                   accuracy on the bf16 matrix cores; every wavefront takes 16-row tiles of W2,
//                   folds its rows with w_g, and the block adds b_g and applies log-sigmoid.
//   k_gate_fold, k_gate_retile, k_gate_prefill   calls of 128 tokens and more: see further down.
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

constexpr int GH_THREADS = 256;          // four wavefronts split d_model
constexpr int GH_ROWS = 16;

// x: bf16 [layers of the range][n_tok][d_model]; u: fp32 [layers of the range][n_tok][d_g]
// NT: 16-token tiles per block; MT: 16-row tiles of W1 per block.  Every wavefront load of x fetches an operand
// straight from row-major memory, the slow way through the vector L1, and every block reads all of its tokens'
// rows: with more than 16 tokens a block takes MT = 4 tiles of W1 so that x is read by a quarter of the blocks.
// TILED: W1 comes from the operand-order copy of a prepared buffer (`tiled` points at the first layer of the
// range: [layer][16-row tile][64-wide step][half][lane] 16-byte pieces), so a wavefront load reads 1 KB in one piece.
// DOT (one tile of tokens, one tile of rows, prepared weights): the readout from the folded vectors happens here as
// well, so u never goes to memory and the call is one kernel.  z = v . u + s is a sum over the hidden units, of which
// a block holds 16: it leaves its part of every (token, head) sum in `part` ([layer][block][head][token], the
// caller's scratch buffer), and the block of a layer that arrives last (one counter per layer, left at zero) adds
// the parts in block order - the same order whichever block that is.
struct GateDot {
    const float* v;          // [layers of the range][heads][d_g]
    const float* s;          // [layers of the range][heads]
    float* part;
    uint32_t* done;          // [layers of the range]
    float* log_beta_out;
    float* log_tail_out;
    int n_heads, n_layers, horizon;
};

template <int NT, int MT, bool TILED, bool DOT>
__global__ __launch_bounds__(GH_THREADS) void k_gate_hidden(GateView g, const uint16_t* __restrict__ x, int n_tok,
                                                            int layer_begin, const uint4* __restrict__ tiled,
                                                            float* __restrict__ u, GateDot dot) {
    static_assert(!DOT || (NT == 1 && MT == 1 && TILED), "the readout rides in the 16 x 16 instance only");
    __shared__ float s_part[4][NT][16 * MT][17];
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int r16 = lane & 15, g4 = lane >> 4;
    const int row0 = blockIdx.x * GH_ROWS * MT;
    const int lr = blockIdx.y;                                       // layer of the range
    const int layer = layer_begin + lr;
    const int tok0 = blockIdx.z * 16 * NT;
    const int kw = g.d_model >> 2;                                   // contraction share of a wavefront
    const int k_begin = wave * kw;

    // piece p (0, 1) of step s of row tile m sits at arow[m * a_tile + s * a_step + p * a_half]
    const uint4* arow = TILED ? tiled + (((size_t)lr * (g.d_g >> 4) + (size_t)blockIdx.x * MT) * (g.d_model >> 6) + (k_begin >> 6)) * 128 + lane
                              : reinterpret_cast<const uint4*>(g.w1 + ((size_t)layer * g.d_g + row0 + r16) * g.d_model + k_begin + 16 * g4);
    constexpr int a_step = TILED ? 128 : 8, a_half = TILED ? 64 : 1;
    const size_t a_tile = TILED ? (size_t)(g.d_model >> 6) * 128 : (size_t)2 * g.d_model;
    const uint4* brow[NT];
    bool bval[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int tok = tok0 + 16 * t + r16;
        bval[t] = tok < n_tok;
        brow[t] = reinterpret_cast<const uint4*>(x + ((size_t)lr * n_tok + (bval[t] ? tok : 0)) * g.d_model + k_begin + 16 * g4);
    }
    gate_f4 acc[MT][NT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[m][t] = gate_f4{0.f, 0.f, 0.f, 0.f};
    // DOT: the folded vectors' entries for this thread's hidden unit, asked for before the stream of W1 starts
    constexpr int DOT_HEADS = DOT ? 16 : 1;
    float vh[DOT_HEADS];
    if (DOT) {
#pragma unroll
        for (int h = 0; h < DOT_HEADS; ++h)
            vh[h] = h < dot.n_heads ? dot.v[((size_t)lr * dot.n_heads + h) * g.d_g + row0 + (tid & 15)] : 0.f;
    }

    // 64 contraction indices per step (8 uint4 of a row); AHEAD steps of weights are loaded ahead
    constexpr int AHEAD = MT == 1 ? 4 : 2;
    const int steps = kw >> 6;                                       // kw is a multiple of 64
    for (int s0 = 0; s0 < steps; s0 += AHEAD) {
        uint4 a[AHEAD][MT][2];
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) {
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                if (s0 + i < steps) {
                    a[i][m][0] = arow[m * a_tile + (s0 + i) * a_step];
                    a[i][m][1] = arow[m * a_tile + (s0 + i) * a_step + a_half];
                } else {
                    a[i][m][0] = a[i][m][1] = make_uint4(0, 0, 0, 0);
                }
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
#pragma unroll
                    for (int m = 0; m < MT; ++m) {
                        acc[m][t] = mma_bf16(a[i][m][0], b0, acc[m][t]);
                        acc[m][t] = mma_bf16(a[i][m][1], b1, acc[m][t]);
                    }
                }
            }
        }
    }
    // acc[m][t][r] = partial of (row 16*m + 4*g4 + r, token r16 of tile t)
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) s_part[wave][t][16 * m + 4 * g4 + r][r16] = acc[m][t][r];
    __syncthreads();
    constexpr int ROWS = 16 * MT;
    if (DOT) {
        static_assert(GH_THREADS == 256, "one (hidden unit, token) pair per thread");
        __shared__ int s_last;
        const int row = tid & 15, tok = tid >> 4;                   // (a token's 16 hidden units sit in 16 neighbouring lanes)
        const int nblk = gridDim.x;
        float su = 0.f;
        if (tok < n_tok) {
            const float a = s_part[0][0][row][tok] + s_part[1][0][row][tok] + s_part[2][0][row][tok] + s_part[3][0][row][tok] +
                            g.c1[(size_t)layer * g.d_g + row0 + row];
            su = a / (1.0f + __expf(-a));
        }
#pragma unroll
        for (int h = 0; h < DOT_HEADS; ++h) {
            if (h >= dot.n_heads) break;                          // (uniform)
            float p = su * vh[h];
            p += __shfl_xor(p, 1, 64);
            p += __shfl_xor(p, 2, 64);
            p += __shfl_xor(p, 4, 64);
            p += __shfl_xor(p, 8, 64);
            if (row == 0 && tok < n_tok)
                __hip_atomic_store(&dot.part[(((size_t)lr * nblk + blockIdx.x) * dot.n_heads + h) * n_tok + tok], p, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // this thread's parts are acknowledged ...
        __syncthreads();                                          // ... and so are the whole block's, before it arrives
        if (tid == 0) s_last = atomicAdd(&dot.done[lr], 1u) == (unsigned)nblk - 1u;
        __syncthreads();
        if (!s_last) return;
        if (tid == 0) __hip_atomic_store(&dot.done[lr], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // (for the next call)
        for (int item = tid; item < n_tok * dot.n_heads; item += GH_THREADS) {
            const int tk = item / dot.n_heads, h = item % dot.n_heads;
            float z = 0.f;
            for (int b0 = 0; b0 < nblk; b0 += 16) {               // 16 parts asked for at once, added in block order
                float pt[16];
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    pt[i] = b0 + i < nblk ? __hip_atomic_load(&dot.part[(((size_t)lr * nblk + b0 + i) * dot.n_heads + h) * n_tok + tk],
                                                              __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                          : 0.f;
#pragma unroll
                for (int i = 0; i < 16; ++i) z += pt[i];
            }
            const float lb = log_sigmoid(z + dot.s[(size_t)lr * dot.n_heads + h]);
            const size_t o = ((size_t)tk * dot.n_layers + layer_begin + lr) * dot.n_heads + h;
            dot.log_beta_out[o] = lb;
            if (dot.log_tail_out) dot.log_tail_out[o] = log_tail_of(lb, dot.horizon);
        }
        return;
    }
    for (int idx = tid; idx < NT * 16 * ROWS; idx += GH_THREADS) {
        const int row = idx % ROWS, tk = (idx / ROWS) & 15, t = idx / (16 * ROWS);
        const int tok = tok0 + 16 * t + tk;
        if (tok < n_tok) {
            const float a = s_part[0][t][row][tk] + s_part[1][t][row][tk] + s_part[2][t][row][tk] + s_part[3][t][row][tk] +
                            g.c1[(size_t)layer * g.d_g + row0 + row];
            u[((size_t)lr * n_tok + tok) * g.d_g + row0 + row] = a / (1.0f + __expf(-a));
        }
    }
}

// The first layer alone for many tokens when the hidden width does not fit the folded prefill kernel below
// (not a multiple of 128, or above 512): a 128 x 128 output tile per block, 64-wide steps of both operands
// staged through LDS (the next step's global loads are in flight in registers while the current one is
// multiplied), 2 x 2 wavefronts of 64 x 64, i.e. 4 x 4 MFMA tiles each.  Both operands are contiguous along
// the contraction, so global loads, LDS rows and MFMA operands all use the same 16-byte pieces; LDS rows are
// padded by 16 bytes against bank conflicts.  Measured (4096 tokens, the metric model): 175 TFLOP/s, 7 % of the
// MFMA peak - a 128-token tile is shared by only four blocks and every block re-reads its W1 rows.
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

// ---- Many tokens per call (a prefill chunk): the second layer and the tied readout are both linear, so
//     z = w_g . (W2 u + c2) + b_g = v . u + s,   v = W2^T w_g  (d_g numbers per (layer, head)),  s = w_g . c2 + b_g
// k_gate_fold computes v and s for the call's weights (one pass over W2), and k_gate_prefill then needs no
// second contraction: a block owns 128 tokens and ALL d_g hidden units of one layer, keeps u in its MFMA
// accumulators, and finishes with eight dot products per token on the vector ALU - u never goes to memory
// and every token row is read once.
//
// Fold: one block per (layer, head).  A wavefront reads whole rows of W2 (a lane owns 8 columns, 16 bytes, of
// every 512-column stretch), the eight wavefronts take every eighth row, and their partial vectors meet in LDS.
constexpr int GF_THREADS = 512, GF_COLS = 512;

__global__ __launch_bounds__(GF_THREADS) void k_gate_fold(GateView g, int layer_begin, int n_heads, float* __restrict__ v,
                                                          float* __restrict__ s) {
    __shared__ __align__(16) float s_part[GF_THREADS / 64][GF_COLS];
    __shared__ float s_red[GF_THREADS / 64];
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int head = blockIdx.x, lr = blockIdx.y, layer = layer_begin + lr;
    const uint16_t* w2 = g.w2 + ((size_t)layer * n_heads + head) * g.d_p * g.d_g;
    const float* c2 = g.c2 + ((size_t)layer * n_heads + head) * g.d_p;
    float* vout = v + ((size_t)lr * n_heads + head) * g.d_g;
    for (int c0 = 0; c0 < g.d_g; c0 += GF_COLS) {                    // d_g is a multiple of 64: a lane's 8 columns are all in or all out
        const int col = c0 + 8 * lane;
        float a[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) a[e] = 0.f;
        if (col < g.d_g) {
#pragma unroll 4
            for (int j = wave; j < g.d_p; j += GF_THREADS / 64) {
                const uint4 w = *reinterpret_cast<const uint4*>(w2 + (size_t)j * g.d_g + col);
                const float wg = g.w_g[j];
                const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    a[2 * e] = fmaf(wg, __uint_as_float(ww[e] << 16), a[2 * e]);
                    a[2 * e + 1] = fmaf(wg, __uint_as_float(ww[e] & 0xFFFF0000u), a[2 * e + 1]);
                }
            }
        }
        __syncthreads();                                             // the previous stretch has been summed
        *reinterpret_cast<float4*>(&s_part[wave][8 * lane]) = make_float4(a[0], a[1], a[2], a[3]);
        *reinterpret_cast<float4*>(&s_part[wave][8 * lane + 4]) = make_float4(a[4], a[5], a[6], a[7]);
        __syncthreads();
        if (tid < GF_COLS && c0 + tid < g.d_g) {
            float t = 0.f;
#pragma unroll
            for (int w = 0; w < GF_THREADS / 64; ++w) t += s_part[w][tid];
            vout[c0 + tid] = t;
        }
    }
    float part = 0.f;
    for (int j = tid; j < g.d_p; j += GF_THREADS) part = fmaf(g.w_g[j], c2[j], part);
    part = wave_sum(part);
    if (lane == 0) s_red[wave] = part;
    __syncthreads();
    if (tid == 0) {
        float t = g.b_g;
#pragma unroll
        for (int w = 0; w < GF_THREADS / 64; ++w) t += s_red[w];
        s[(size_t)lr * n_heads + head] = t;
    }
}

// Operand layout and the memory system.  A wavefront load that fetches an MFMA operand straight from a
// row-major matrix touches 16 different rows in every group of 16 lanes; the vector L1 then serves about
// 15 bytes per clock and compute unit (measured), against 50 for loads whose 16-lane groups read 256
// contiguous bytes.  Hence:
//   k_gate_retile  copies W1 once per call into tiles of 16 rows x 64 columns (2 KB) stored in lane order - the
//                  two 16-byte halves a lane feeds to the two MFMAs of a step at [half][lane] - when the call
//                  is long enough to pay for the pass and the scratch buffer has room;
//   token rows     are loaded coalesced (8 lanes cover the 128 bytes of a row and step) and scattered into
//                  operand order inside LDS, which they pass through anyway.
// The contraction index of a step is permuted (both operands alike): lane group g of half h holds columns
// 16 g + 8 h .. + 8.
//
// Retile: one wavefront per (layer, 16-row tile, 4 steps); reads in operand layout, writes 1 KB contiguous.
constexpr int GT_THREADS = 256;

__global__ __launch_bounds__(GT_THREADS) void k_gate_retile(GateView g, int layer_begin, uint4* __restrict__ tiled) {
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int r16 = lane & 15, g4 = lane >> 4;
    const int steps = g.d_model >> 6;
    const int tile = blockIdx.y, lr = blockIdx.z;
    const int s0 = (blockIdx.x * (GT_THREADS / 64) + wave) * 4;      // steps is a multiple of 4
    if (s0 >= steps) return;
    const uint4* src = reinterpret_cast<const uint4*>(g.w1 + ((size_t)(layer_begin + lr) * g.d_g + 16 * tile + r16) * g.d_model +
                                                      64 * s0 + 16 * g4);
    uint4* dst = tiled + (((size_t)lr * (g.d_g >> 4) + tile) * steps + s0) * 128 + lane;
    uint4 v[4][2];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        v[u][0] = src[8 * u];
        v[u][1] = src[8 * u + 1];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        dst[128 * u] = v[u][0];
        dst[128 * u + 64] = v[u][1];
    }
}

// Prefill: 512 threads = 8 wavefronts.  Wavefront w owns hidden units [w*16*HT, (w+1)*16*HT) (d_g = 128*HT)
// for all 16*TT tokens of the block: HT x TT accumulator tiles of 16 x 16 (TT = 8 for long calls; 4 or 2 when
// 128-token blocks would be too few to fill the chip).  Its W1 operands go from global memory to registers,
// one step ahead: from the tiled copy (TILED) or straight from the rows (a lane loads 32 contiguous bytes of
// its row per 64-wide step and feeds the halves to two MFMAs).  The token rows are shared by all wavefronts:
// wavefront j < TT loads token tile j and parks it in LDS in operand order; a fragment half is 4 lane groups
// of 256 bytes, 16 bytes of padding after each and 64 after the half, which spreads the 8 pieces of a row
// over 32 banks when they are parked (the reads then see two-way conflicts between lane groups; measured, that
// costs less than eight-way conflicts on the parking side: 562 against 595 us for 4096 tokens).  Steps go in pairs with one barrier per pair and three pair buffers.  Block ids are mapped so
// that the blocks an XCD runs at one time belong to one layer (ids are dealt to the eight XCDs in turn), so
// W1_l is shared through that XCD's L2.
constexpr int GP_THREADS = 512, GP_HEADS_MAX = 8;
constexpr int GP_GROUP_BYTES = 272, GP_HALF_BYTES = 4 * GP_GROUP_BYTES, GP_TILE_BYTES = 2 * GP_HALF_BYTES;   // 272, 1088, 2176

template <int HT, int TT, bool TILED>
__global__ __launch_bounds__(GP_THREADS) void k_gate_prefill(GateView g, const uint16_t* __restrict__ x, int n_tok,
                                                             int layer_begin, int nl, int n_layers, int n_heads, int horizon,
                                                             const uint4* __restrict__ tiled, const float* __restrict__ v,
                                                             const float* __restrict__ sconst,
                                                             float* __restrict__ log_beta_out,
                                                             float* __restrict__ log_tail_out) {
    constexpr int GP_TOK = 16 * TT;
    constexpr int STEP_BYTES = TT * GP_TILE_BYTES;
    // three buffers of [step of the pair][token tile] tiles of 2176 bytes; after the loop [wave][head][token] floats, 4 TT KB
    __shared__ __align__(16) char s_x[6 * STEP_BYTES];
    const int tid = threadIdx.x, lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);       // uniform: addresses below stay scalar base + lane offset
    const int r16 = lane & 15, g4 = lane >> 4;
    const int tiles = (n_tok + GP_TOK - 1) / GP_TOK;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int lr = (slot / tiles) * 8 + xcd;
    if (lr >= nl) return;                                            // whole block, before any barrier
    const int tok0 = (slot % tiles) * GP_TOK;
    const int layer = layer_begin + lr;
    const int hid0 = wave * 16 * HT;
    const int steps = g.d_model >> 6;                                // 64 contraction indices = 128 bytes of a row per step

    // W1: uniform base + 32-bit lane offset, in bytes
    const uint32_t row_bytes = 2u * (uint32_t)g.d_model;
    const char* wbase;
    uint32_t aoff, a_tile_stride;
    if (TILED) {
        wbase = reinterpret_cast<const char*>(tiled + ((size_t)lr * (g.d_g >> 4) + (hid0 >> 4)) * steps * 128);
        aoff = 16u * (uint32_t)lane;
        a_tile_stride = (uint32_t)steps * 2048u;
    } else {
        wbase = reinterpret_cast<const char*>(g.w1 + ((size_t)layer * g.d_g + hid0) * g.d_model);
        aoff = (uint32_t)r16 * row_bytes + 32u * (uint32_t)g4;
        a_tile_stride = 16u * row_bytes;
    }
    // token rows: lane l takes the 16-byte piece l % 8 of rows l / 8 and l / 8 + 8 of its tile; rows past the end
    // repeat the last token and are never written
    const int tile_tok0 = tok0 + 16 * min(wave, TT - 1);
    const int xr_a = min(tile_tok0 + (lane >> 3), n_tok - 1), xr_b = min(tile_tok0 + (lane >> 3) + 8, n_tok - 1);
    const char* xbase = reinterpret_cast<const char*>(x + (size_t)lr * n_tok * g.d_model) + 16 * (lane & 7);
    const size_t xoff_a = (size_t)xr_a * row_bytes, xoff_b = (size_t)xr_b * row_bytes;
    // where those pieces go inside a parked tile, and where this lane reads its operand from
    const int park_off = min(wave, TT - 1) * GP_TILE_BYTES + (lane & 1) * GP_HALF_BYTES + ((lane & 7) >> 1) * GP_GROUP_BYTES + (lane >> 3) * 16;
    const int read_off = g4 * GP_GROUP_BYTES + r16 * 16;

    gate_f4 acc[HT][TT];
#pragma unroll
    for (int i = 0; i < HT; ++i)
#pragma unroll
        for (int j = 0; j < TT; ++j) acc[i][j] = gate_f4{0.f, 0.f, 0.f, 0.f};

    uint4 a0[HT][2], a1[HT][2], xr[2][2];
    auto load_a = [&](int kt, uint4 (&a)[HT][2]) {
#pragma unroll
        for (int i = 0; i < HT; ++i) {
            if (TILED) {
                const uint4* p = reinterpret_cast<const uint4*>(wbase + (size_t)i * a_tile_stride + (size_t)kt * 2048 + aoff);
                a[i][0] = p[0];
                a[i][1] = p[64];
            } else {
                const uint4* p = reinterpret_cast<const uint4*>(wbase + (size_t)i * a_tile_stride + (size_t)kt * 128 + aoff);
                a[i][0] = p[0];
                a[i][1] = p[1];
            }
        }
    };
    // uniform per wavefront; a compile-time "true" in the full-size variant keeps its loop free of branches
    const bool loader = TT == 8 || wave < TT;
    xr[0][0] = xr[0][1] = xr[1][0] = xr[1][1] = make_uint4(0, 0, 0, 0);
    auto load_x = [&](int kt) {                                      // the token rows of steps kt and kt + 1
        if (TT == 8 || loader) {
            const char* p = xbase + (size_t)kt * 128;
            xr[0][0] = *reinterpret_cast<const uint4*>(p + xoff_a);
            xr[0][1] = *reinterpret_cast<const uint4*>(p + xoff_b);
            xr[1][0] = *reinterpret_cast<const uint4*>(p + xoff_a + 128);
            xr[1][1] = *reinterpret_cast<const uint4*>(p + xoff_b + 128);
        }
    };
    auto park_x = [&](int buf) {                                     // buf: one of the three pair buffers
        if (TT == 8 || loader) {
            char* p = s_x + buf * 2 * STEP_BYTES + park_off;
            *reinterpret_cast<uint4*>(p) = xr[0][0];
            *reinterpret_cast<uint4*>(p + 128) = xr[0][1];           // row + 8
            *reinterpret_cast<uint4*>(p + STEP_BYTES) = xr[1][0];
            *reinterpret_cast<uint4*>(p + STEP_BYTES + 128) = xr[1][1];
        }
    };
    // One step: 2 TT fragments (fragment f = half f / TT of token tile f % TT), each multiplied into HT accumulator
    // tiles.  The reads run two fragments ahead of the MFMAs and continue into the next step (`next`), also across
    // the barrier between pairs, so the matrix pipe does not wait for LDS when a step or a pair begins.
    uint4 b0, b1;
    auto frag = [&](const char* base, int f) {
        return *reinterpret_cast<const uint4*>(base + (f % TT) * GP_TILE_BYTES + (f / TT) * GP_HALF_BYTES);
    };
    auto multiply = [&](const char* base, const char* next, const uint4 (&a)[HT][2]) {
#pragma unroll
        for (int f = 0; f < 2 * TT; ++f) {
            const uint4 b2 = f + 2 < 2 * TT ? frag(base, f + 2) : frag(next, f + 2 - 2 * TT);
#pragma unroll
            for (int i = 0; i < HT; ++i) acc[i][f % TT] = mma_bf16(a[i][f / TT], b0, acc[i][f % TT]);
            b0 = b1;
            b1 = b2;
            __builtin_amdgcn_sched_barrier(0);                       // keeps the compiler from hoisting all the reads (spills)
        }
    };
    // Steps go in pairs, the token rows of a pair are parked together, one barrier per pair, three pair buffers.
    // During pair P: its rows are read from buffer P % 3 (parked during pair P - 2), the rows of pair P + 2 wait in
    // registers and are parked at the end into buffer (P + 2) % 3 - which pair P - 1 was read from, before the
    // previous barrier - and the W1 operands of the next step arrive.  The loop has no branches: past the end the
    // loads repeat the last pair, into registers and buffers nobody reads any more.
    const int last = steps - 2;                                      // steps is a multiple of 4
    load_x(0);
    load_a(0, a0);
    load_a(1, a1);
    park_x(0);
    load_x(min(2, last));
    park_x(1);
    __syncthreads();
    load_x(min(4, last));
    int cur = 0;                                                     // buffer of the current pair
    b0 = frag(s_x + read_off, 0);
    b1 = frag(s_x + read_off, 1);
    for (int kt = 0; kt < steps; kt += 2) {
        const int nxt = cur == 2 ? 0 : cur + 1, nn = nxt == 2 ? 0 : nxt + 1;
        const char* base = s_x + cur * 2 * STEP_BYTES + read_off;
        multiply(base, base + STEP_BYTES, a0);
        load_a(min(kt + 2, last), a0);
        multiply(base + STEP_BYTES, s_x + nxt * 2 * STEP_BYTES + read_off, a1);
        load_a(min(kt + 3, last + 1), a1);
        park_x(nn);
        __syncthreads();
        load_x(min(kt + 6, last));
        cur = nxt;
    }

    // acc[i][j][r] = pre-activation of (hidden hid0 + 16 i + 4 g4 + r, token tok0 + 16 j + r16).
    // The folded readout vectors of this layer (heads x d_g floats, at most 16 KB) are fetched while the
    // activation is applied and staged in LDS behind the [wave][head][token] partial sums.
    float* s_z = reinterpret_cast<float*>(s_x);                      // every wavefront is past the last barrier of the loop
    float4* s_v = reinterpret_cast<float4*>(s_x + 4096 * TT);
    const int v_f4 = (n_heads * g.d_g) >> 2;                         // <= 1024: two per thread
    const float4* vsrc = reinterpret_cast<const float4*>(v + (size_t)lr * n_heads * g.d_g);
    float4 v0 = make_float4(0.f, 0.f, 0.f, 0.f), v1 = v0;
    if (tid < v_f4) v0 = vsrc[tid];
    if (tid + GP_THREADS < v_f4) v1 = vsrc[tid + GP_THREADS];
#pragma unroll
    for (int i = 0; i < HT; ++i) {
        const float4 c = *reinterpret_cast<const float4*>(g.c1 + (size_t)layer * g.d_g + hid0 + 16 * i + 4 * g4);
        const float cc[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
        for (int j = 0; j < TT; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float t = acc[i][j][r] + cc[r];
                acc[i][j][r] = t * __builtin_amdgcn_rcpf(1.0f + __expf(-t));   // silu; the reciprocal is good to 1 ulp
            }
    }
    if (tid < v_f4) s_v[tid] = v0;
    if (tid + GP_THREADS < v_f4) s_v[tid + GP_THREADS] = v1;
    __syncthreads();
    for (int h = 0; h < n_heads; ++h) {
        const float4* vh = s_v + ((h * g.d_g + hid0) >> 2) + g4;
        float zp[TT];
#pragma unroll
        for (int j = 0; j < TT; ++j) zp[j] = 0.f;
#pragma unroll
        for (int i = 0; i < HT; ++i) {
            const float4 w = vh[4 * i];
            const float ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int j = 0; j < TT; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) zp[j] = fmaf(ww[r], acc[i][j][r], zp[j]);
        }
#pragma unroll
        for (int j = 0; j < TT; ++j) {
            float t = zp[j];
            t += __shfl_xor(t, 16, 64);
            t += __shfl_xor(t, 32, 64);
            if (g4 == 0) s_z[(wave * GP_HEADS_MAX + h) * GP_TOK + 16 * j + r16] = t;
        }
    }
    __syncthreads();
    for (int idx = tid; idx < n_heads * GP_TOK; idx += GP_THREADS) {
        const int h = idx / GP_TOK, tk = idx - h * GP_TOK;
        const int tok = tok0 + tk;
        if (tok >= n_tok) continue;
        float z = sconst[(size_t)lr * n_heads + h];
#pragma unroll
        for (int w = 0; w < 8; ++w) z += s_z[(w * GP_HEADS_MAX + h) * GP_TOK + tk];
        const float lb = log_sigmoid(z);
        const size_t o = ((size_t)tok * n_layers + layer) * n_heads + h;
        log_beta_out[o] = lb;
        if (log_tail_out) log_tail_out[o] = log_tail_of(lb, horizon);
    }
}

// Below this many tokens the fold's extra pass over W2 and the few blocks of the prefill kernel do not pay.
#ifndef KVTRIM_GATE_PREFILL_MIN_TOK
#define KVTRIM_GATE_PREFILL_MIN_TOK 128
#endif
constexpr int GP_MIN_TOK = KVTRIM_GATE_PREFILL_MIN_TOK;
constexpr int GP_MIN_TOK_PREPARED = 24;

static bool prefill_shape(const kvtrim_ctx* ctx, const GateView& g) {
    return g.d_g % 128 == 0 && g.d_g <= 512 && ctx->shape.n_kv_heads <= GP_HEADS_MAX;
}

// Readout from folded vectors for calls that went through the per-token first-layer kernels: one wavefront
// per (token, layer, head) forms z = v . u + s - every dot product is one trip to memory, all of them at once.
constexpr int GD_THREADS = 256;

__global__ __launch_bounds__(GD_THREADS) void k_gate_dot(const float* __restrict__ u, const float* __restrict__ v,
                                                         const float* __restrict__ sconst, int n_tok, int d_g,
                                                         int layer_begin, int n_layers, int n_heads, int horizon,
                                                         float* __restrict__ log_beta_out,
                                                         float* __restrict__ log_tail_out) {
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int64_t item = (int64_t)blockIdx.x * (GD_THREADS / 64) + wave;    // (token, head) of layer blockIdx.y
    const int lr = blockIdx.y;
    if (item >= (int64_t)n_tok * n_heads) return;
    const int tok = (int)(item / n_heads), h = (int)(item % n_heads);
    const float* urow = u + ((size_t)lr * n_tok + tok) * d_g;
    const float* vh = v + ((size_t)lr * n_heads + h) * d_g;
    float acc = 0.f;
    for (int k = lane; k < d_g; k += 64) acc = fmaf(urow[k], vh[k], acc);
    acc = wave_sum(acc);
    if (lane == 0) {
        const float lb = log_sigmoid(acc + sconst[(size_t)lr * n_heads + h]);
        const size_t o = ((size_t)tok * n_layers + layer_begin + lr) * n_heads + h;
        log_beta_out[o] = lb;
        if (log_tail_out) log_tail_out[o] = log_tail_of(lb, horizon);
    }
}

// Layout of a prepared buffer (kvtrim_gate_prepare): v [L][heads][d_g], s [L][heads], padding to 16 bytes, then
// W1 of all L layers in operand-order tiles.
static size_t prepared_fold_floats(const GateView& g, int n_layers, int n_heads) {
    return ((size_t)n_layers * n_heads * (g.d_g + 1) + 3) & ~(size_t)3;
}

kvtrim_status launch_gate_prepare(kvtrim_ctx* ctx, const GateView& g, float* prepared, hipStream_t st) {
    const int L = ctx->shape.n_layers, n_heads = ctx->shape.n_kv_heads;
    float* v = prepared;
    float* sconst = prepared + (size_t)L * n_heads * g.d_g;
    uint4* tiled = reinterpret_cast<uint4*>(prepared + prepared_fold_floats(g, L, n_heads));
    {
        ProfScope prof(ctx, K_GATE_FOLD, st);
        hipLaunchKernelGGL(k_gate_fold, dim3(n_heads, L), dim3(GF_THREADS), 0, st, g, 0, n_heads, v, sconst);
    }
    {
        ProfScope prof(ctx, K_GATE_RETILE, st);
        const int steps = g.d_model >> 6;
        hipLaunchKernelGGL(k_gate_retile, dim3((steps / 4 + GT_THREADS / 64 - 1) / (GT_THREADS / 64), g.d_g / 16, L),
                           dim3(GT_THREADS), 0, st, g, 0, tiled);
    }
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

// prepared: NULL (everything is derived from the weights inside the call) or a buffer filled by launch_gate_prepare
// for the same weights.
kvtrim_status launch_gate(kvtrim_ctx* ctx, const GateView& g, const float* prepared, const uint16_t* x, int n_tok,
                          int layer_begin, int layer_end, int horizon, float* scratch, float* log_beta_out,
                          float* log_tail_out, hipStream_t st) {
    const int nl = layer_end - layer_begin;
    const int L = ctx->shape.n_layers, n_heads = ctx->shape.n_kv_heads;
    // the folded vectors and the tiled W1 of the layer range, when prepared
    const float* pv = prepared ? prepared + (size_t)layer_begin * n_heads * g.d_g : nullptr;
    const float* ps = prepared ? prepared + (size_t)L * n_heads * g.d_g + (size_t)layer_begin * n_heads : nullptr;
    const uint4* ptiled = prepared ? reinterpret_cast<const uint4*>(prepared + prepared_fold_floats(g, L, n_heads)) +
                                         (size_t)layer_begin * (g.d_g >> 4) * (g.d_model >> 6) * 128
                                   : nullptr;
    // with prepared weights the folded kernel has no per-call passes to pay for and wins from 24 tokens on
    // (measured: 17 tokens 55 us per-token kernels, 24 tokens 58 / 58 us folded, 32 tokens 60 / 58, 64 tokens 80 / 58)
    if (n_tok >= (prepared ? GP_MIN_TOK_PREPARED : GP_MIN_TOK) && prefill_shape(ctx, g)) {
        const float* v = pv;
        const float* sconst = ps;
        const uint4* tiled = ptiled;
        bool use_tiled = prepared != nullptr;
        if (!prepared) {
            // scratch: v [nl][heads][d_g], s [nl][heads], then (16-byte aligned) the tiled copy of W1 if the buffer
            // - n_tok * nl * d_g floats - has room for it, which also means the call is long enough for the pass to pay
            float* sv = scratch;
            float* ss = scratch + (size_t)nl * n_heads * g.d_g;
            const size_t fold_floats = ((size_t)nl * n_heads * (g.d_g + 1) + 3) & ~(size_t)3;
            const size_t tiled_floats = (size_t)nl * g.d_g * g.d_model / 2;
            use_tiled = fold_floats + tiled_floats <= (size_t)n_tok * nl * g.d_g;
            uint4* st_tiled = reinterpret_cast<uint4*>(scratch + fold_floats);
            {
                ProfScope prof(ctx, K_GATE_FOLD, st);
                hipLaunchKernelGGL(k_gate_fold, dim3(n_heads, nl), dim3(GF_THREADS), 0, st, g, layer_begin, n_heads, sv, ss);
            }
            if (use_tiled) {
                ProfScope prof(ctx, K_GATE_RETILE, st);
                const int steps = g.d_model >> 6;
                hipLaunchKernelGGL(k_gate_retile, dim3((steps / 4 + GT_THREADS / 64 - 1) / (GT_THREADS / 64), g.d_g / 16, nl),
                                   dim3(GT_THREADS), 0, st, g, layer_begin, st_tiled);
            }
            v = sv;
            sconst = ss;
            tiled = st_tiled;
        }
        {
            ProfScope prof(ctx, K_GATE_PREFILL, st);
            // tokens per block: 128, or 64 / 32 while that is what it takes to have a block for every compute unit
            int tt = 8;
            while (tt > 2 && (int64_t)nl * ((n_tok + 16 * tt - 1) / (16 * tt)) < 256) tt >>= 1;
            const int tiles = (n_tok + 16 * tt - 1) / (16 * tt);
            const dim3 grid(8u * (unsigned)((nl + 7) / 8) * (unsigned)tiles);
#define KVTRIM_GATE_PREFILL(HT, TT, TILED)                                                                                    \
    hipLaunchKernelGGL((k_gate_prefill<HT, TT, TILED>), grid, dim3(GP_THREADS), 0, st, g, x, n_tok, layer_begin, nl, L,       \
                       n_heads, horizon, tiled, v, sconst, log_beta_out, log_tail_out)
#define KVTRIM_GATE_PREFILL_TT(HT)                                                                                            \
    do {                                                                                                                      \
        if (use_tiled && tt == 8) KVTRIM_GATE_PREFILL(HT, 8, true);                                                           \
        else if (use_tiled && tt == 4) KVTRIM_GATE_PREFILL(HT, 4, true);                                                      \
        else if (use_tiled) KVTRIM_GATE_PREFILL(HT, 2, true);                                                                 \
        else if (tt == 8) KVTRIM_GATE_PREFILL(HT, 8, false);                                                                  \
        else if (tt == 4) KVTRIM_GATE_PREFILL(HT, 4, false);                                                                  \
        else KVTRIM_GATE_PREFILL(HT, 2, false);                                                                               \
    } while (0)
            switch (g.d_g / 128) {
                case 1: KVTRIM_GATE_PREFILL_TT(1); break;
                case 2: KVTRIM_GATE_PREFILL_TT(2); break;
                case 3: KVTRIM_GATE_PREFILL_TT(3); break;
                default: KVTRIM_GATE_PREFILL_TT(4); break;
            }
#undef KVTRIM_GATE_PREFILL_TT
#undef KVTRIM_GATE_PREFILL
        }
        KVTRIM_HIP(ctx, hipGetLastError());
        return KVTRIM_OK;
    }
    // up to 16 tokens with prepared weights: the readout rides in the first-layer kernel (its parts of the sums,
    // heads * d_g / 16 numbers per token and layer, fit the scratch buffer's d_g when there are at most 16 heads)
    if (prepared && n_tok <= 16 && n_heads <= 16) {
        ProfScope prof(ctx, K_GATE_HIDDEN, st);
        GateDot dot;
        dot.v = pv;
        dot.s = ps;
        dot.part = scratch;
        dot.done = ctx->ws.gate_done;
        dot.log_beta_out = log_beta_out;
        dot.log_tail_out = log_tail_out;
        dot.n_heads = n_heads;
        dot.n_layers = L;
        dot.horizon = horizon;
        hipLaunchKernelGGL((k_gate_hidden<1, 1, true, true>), dim3(g.d_g / GH_ROWS, nl, 1), dim3(GH_THREADS), 0, st, g, x, n_tok,
                           layer_begin, ptiled, nullptr, dot);
        KVTRIM_HIP(ctx, hipGetLastError());
        return KVTRIM_OK;
    }
    {
        ProfScope prof(ctx, K_GATE_HIDDEN, st);
        const dim3 grid1(g.d_g / GH_ROWS, nl, 1);
        const dim3 grid4(g.d_g / (4 * GH_ROWS), nl, 1);              // d_g is a multiple of 64
        if (n_tok <= 16 && prepared)
            hipLaunchKernelGGL((k_gate_hidden<1, 1, true, false>), grid1, dim3(GH_THREADS), 0, st, g, x, n_tok, layer_begin, ptiled, scratch, GateDot{});
        else if (n_tok <= 32 && prepared)
            hipLaunchKernelGGL((k_gate_hidden<2, 4, true, false>), grid4, dim3(GH_THREADS), 0, st, g, x, n_tok, layer_begin, ptiled, scratch, GateDot{});
        else if (n_tok <= 64 && prepared)
            hipLaunchKernelGGL((k_gate_hidden<4, 4, true, false>), grid4, dim3(GH_THREADS), 0, st, g, x, n_tok, layer_begin, ptiled, scratch, GateDot{});
        else if (n_tok <= 16)
            hipLaunchKernelGGL((k_gate_hidden<1, 1, false, false>), grid1, dim3(GH_THREADS), 0, st, g, x, n_tok, layer_begin, ptiled, scratch, GateDot{});
        else if (n_tok <= 32)
            hipLaunchKernelGGL((k_gate_hidden<2, 4, false, false>), grid4, dim3(GH_THREADS), 0, st, g, x, n_tok, layer_begin, ptiled, scratch, GateDot{});
        else if (n_tok < 256)                                        // below that the tiled kernel cannot fill the chip
            hipLaunchKernelGGL((k_gate_hidden<4, 4, false, false>), dim3(grid4.x, nl, (n_tok + 63) / 64), dim3(GH_THREADS), 0, st, g, x, n_tok,
                               layer_begin, ptiled, scratch, GateDot{});
        else
            hipLaunchKernelGGL(k_gate_hidden_gemm, dim3((g.d_g + GG_BM - 1) / GG_BM, (n_tok + GG_BN - 1) / GG_BN, nl), dim3(256), 0,
                               st, g, x, n_tok, layer_begin, scratch);
    }
    if (prepared) {
        ProfScope prof(ctx, K_GATE_DOT, st);
        const int64_t items = (int64_t)n_tok * n_heads;
        hipLaunchKernelGGL(k_gate_dot, dim3((unsigned)((items + GD_THREADS / 64 - 1) / (GD_THREADS / 64)), nl), dim3(GD_THREADS), 0,
                           st, scratch, pv, ps, n_tok, g.d_g, layer_begin, L, n_heads, horizon, log_beta_out, log_tail_out);
    } else {
        ProfScope prof(ctx, K_GATE_READOUT, st);
        hipLaunchKernelGGL(k_gate_readout, dim3(n_heads, nl, (n_tok + 15) / 16), dim3(GR_THREADS), 0, st, g, scratch,
                           n_tok, layer_begin, L, n_heads, horizon, log_beta_out, log_tail_out);
    }
    KVTRIM_HIP(ctx, hipGetLastError());
    return KVTRIM_OK;
}

}  // namespace kvtrim

using namespace kvtrim;

extern "C" {

size_t kvtrim_gate_scratch_bytes(const kvtrim_gate* g, int32_t n_tok, int32_t n_layers) {
    if (!g || n_tok < 1 || n_layers < 1 || g->d_g < 1) return 0;
    // u for the per-token kernels; the prefill kernels keep (heads <= 8) * (d_g + 1) numbers per layer there and
    // run only from GP_MIN_TOK tokens on, so they always fit
    return (size_t)n_tok * (size_t)n_layers * (size_t)g->d_g * sizeof(float);
}

// argument checks shared by the gate entry points; returns NULL when the gate itself is usable
static const char* gate_problem(const kvtrim_gate* g) {
    if (!g || !g->w1 || !g->c1 || !g->w2 || !g->c2 || !g->w_g) return "gate or one of its weight pointers is NULL";
    if (g->d_model < 256 || g->d_model % 256) return "d_model must be a positive multiple of 256";
    if (g->d_g < 64 || g->d_g % 64) return "d_g must be a positive multiple of 64";
    if (g->d_p < 1) return "d_p < 1";
    if ((((uintptr_t)g->c1) | ((uintptr_t)g->w_g)) & 15) return "c1 / w_g not 16-byte aligned";
    if ((((uintptr_t)g->w1) | ((uintptr_t)g->w2)) & 15) return "w1 / w2 not 16-byte aligned";
    if (!(g->b_g == g->b_g)) return "b_g is NaN";
    return nullptr;
}

static GateView gate_view(const kvtrim_gate* g) {
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
    return v;
}

static kvtrim_status gate_forward(kvtrim_ctx* ctx, const kvtrim_gate* g, const void* prepared, const void* x, int32_t n_tok,
                                  int32_t layer_begin, int32_t layer_end, int32_t horizon, void* scratch,
                                  float* log_beta_out, float* log_tail_out, void* hip_stream) {
    auto bad = [&](const char* why) {
        snprintf(ctx->last_error, sizeof(ctx->last_error), "invalid argument: %s", why);
        return KVTRIM_EINVAL;
    };
    if (const char* p = gate_problem(g)) return bad(p);
    if (!x || !scratch || !log_beta_out) return bad("x / scratch / log_beta_out is NULL");
    if (n_tok < 1) return bad("n_tok < 1");
    if ((int64_t)n_tok > 65535 * 16) return bad("n_tok too large for one call");
    if (layer_begin < 0 || layer_end > ctx->cfg.n_layers || layer_begin >= layer_end) return bad("empty or out-of-range layer range");
    if (horizon < 0 || horizon > 4096) return bad("horizon outside [0, 4096] (0 = infinite)");
    if ((((uintptr_t)x) | ((uintptr_t)scratch) | ((uintptr_t)prepared)) & 15) return bad("x / scratch / prepared not 16-byte aligned");
    return launch_gate(ctx, gate_view(g), (const float*)prepared, (const uint16_t*)x, n_tok, layer_begin, layer_end, horizon,
                       (float*)scratch, log_beta_out, log_tail_out, (hipStream_t)hip_stream);
}

kvtrim_status kvtrim_gate_forward(kvtrim_ctx* ctx, const kvtrim_gate* g, const void* x, int32_t n_tok, int32_t layer_begin,
                                  int32_t layer_end, int32_t horizon, void* scratch, float* log_beta_out,
                                  float* log_tail_out, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    return gate_forward(ctx, g, nullptr, x, n_tok, layer_begin, layer_end, horizon, scratch, log_beta_out, log_tail_out,
                        hip_stream);
}

size_t kvtrim_gate_prepared_bytes(const kvtrim_gate* g, int32_t n_layers, int32_t n_kv_heads) {
    if (gate_problem(g) || n_layers < 1 || n_kv_heads < 1) return 0;
    const size_t fold = ((size_t)n_layers * n_kv_heads * ((size_t)g->d_g + 1) + 3) & ~(size_t)3;
    return fold * sizeof(float) + (size_t)n_layers * g->d_g * g->d_model * 2;
}

kvtrim_status kvtrim_gate_prepare(kvtrim_ctx* ctx, const kvtrim_gate* g, void* prepared, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    auto bad = [&](const char* why) {
        snprintf(ctx->last_error, sizeof(ctx->last_error), "invalid argument: %s", why);
        return KVTRIM_EINVAL;
    };
    if (const char* p = gate_problem(g)) return bad(p);
    if (!prepared || (((uintptr_t)prepared) & 15)) return bad("prepared is NULL or not 16-byte aligned");
    return launch_gate_prepare(ctx, gate_view(g), (float*)prepared, (hipStream_t)hip_stream);
}

kvtrim_status kvtrim_gate_forward_prepared(kvtrim_ctx* ctx, const kvtrim_gate* g, const void* prepared, const void* x,
                                           int32_t n_tok, int32_t layer_begin, int32_t layer_end, int32_t horizon,
                                           void* scratch, float* log_beta_out, float* log_tail_out, void* hip_stream) {
    if (!ctx) return KVTRIM_EINVAL;
    if (!prepared) {
        snprintf(ctx->last_error, sizeof(ctx->last_error), "invalid argument: prepared is NULL");
        return KVTRIM_EINVAL;
    }
    return gate_forward(ctx, g, prepared, x, n_tok, layer_begin, layer_end, horizon, scratch, log_beta_out, log_tail_out,
                        hip_stream);
}

}  // extern "C"
