// Learnable affine re-parameterisation of a projection (section 3.1.2):
//     X W + b  ->  ((X - delta) / s) Q(W * s) + b + delta W
// with W stored [N, K] (out x in), s and delta per input feature [K].  The pieces around the quantized
// layer, all HBM-bound:
//   mq_affine_weight  Ws = W * s (what the quantizer is given) and c = b + W delta (the bias of the
//                     transformed layer), one pass over W
//   mq_affine_input   Xt = bf16((X - delta) / s)
//   mq_affine_bwd     gradients with respect to delta and s from what the straight-through backward of
//                     the transformed layer returns (column reductions over tokens and over channels)
// The bias itself enters the forward in its epilogue (mq_linear_fwd_multi_l2).
#include "mq_common.h"

namespace mq {

namespace {

// One workgroup per output channel: Ws[n, :] = W[n, :] * s, c[n] = b[n] + sum_k W[n, k] delta[k].
__global__ __launch_bounds__(256) void affine_weight_kernel(const float *__restrict__ W, int64_t ldw, int K,
                                                            const float *__restrict__ s, const float *__restrict__ delta,
                                                            const float *__restrict__ b, float *__restrict__ Ws,
                                                            float *__restrict__ c) {
    __shared__ double red[4];
    const int n = blockIdx.x;
    const float *w = W + (size_t)n * ldw;
    float dot = 0.f;
    for (int k = threadIdx.x * 4; k < K; k += 1024) {
        const f32x4 wv = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(w + k));
        if (Ws) {
            f32x4 o = wv;
            if (s) {
                const f32x4 sv = *reinterpret_cast<const f32x4 *>(s + k);
#pragma unroll
                for (int j = 0; j < 4; ++j) o[j] = __fmul_rn(wv[j], sv[j]);
            }
            *reinterpret_cast<f32x4 *>(Ws + (size_t)n * K + k) = o;
        }
        if (delta) {
            const f32x4 dv = *reinterpret_cast<const f32x4 *>(delta + k);
#pragma unroll
            for (int j = 0; j < 4; ++j) dot += wv[j] * dv[j];
        }
    }
    if (!c) return;
    double d = dot;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) d += __shfl_xor(d, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = d;
    __syncthreads();
    if (threadIdx.x == 0) c[n] = (float)((b ? (double)b[n] : 0.0) + red[0] + red[1] + red[2] + red[3]);
}

// Xt = bf16((X - delta) / s), eight elements per thread (K is a multiple of 8)
__global__ __launch_bounds__(256) void affine_input_kernel(const uint16_t *__restrict__ X, int64_t chunks, int K,
                                                           const float *__restrict__ s, const float *__restrict__ delta,
                                                           uint16_t *__restrict__ Xt) {
    const int64_t ch = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (ch >= chunks) return;
    const int k = (int)((ch * 8) % K);
    const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(X) + ch);
    float sv[8], dv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) sv[j] = 1.0f, dv[j] = 0.0f;
    if (s) {  // (K is a multiple of 8 and the vectors are 16-byte aligned: two 16-byte loads each)
        *reinterpret_cast<f32x4 *>(sv) = *reinterpret_cast<const f32x4 *>(s + k);
        *reinterpret_cast<f32x4 *>(sv + 4) = *reinterpret_cast<const f32x4 *>(s + k + 4);
    }
    if (delta) {
        *reinterpret_cast<f32x4 *>(dv) = *reinterpret_cast<const f32x4 *>(delta + k);
        *reinterpret_cast<f32x4 *>(dv + 4) = *reinterpret_cast<const f32x4 *>(delta + k + 4);
    }
    u32x4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float lo = __fdiv_rn(__fsub_rn(bf16_lo(x[j]), dv[2 * j]), sv[2 * j]);
        const float hi = __fdiv_rn(__fsub_rn(bf16_hi(x[j]), dv[2 * j + 1]), sv[2 * j + 1]);
        o[j] = pack_bf16x2(lo, hi);
    }
    __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(Xt) + ch);
}

// Column reductions.  A workgroup covers 256 columns (64 column threads x 4 columns) and one range of
// rows (4 row threads step through it); partial[split][which][col] holds its sums, finished by a second
// pass in a fixed order.
constexpr int kColsPerBlock = 256;

struct ColArgs {
    const uint16_t *A16[3];  // bf16 [rows, cols] inputs
    const float *A32[2];     // fp32 [rows, ld] inputs
    const float *rowvec;     // per-row fp32 factor
    float lam[3];
    int64_t ld32;
    int rows, cols, rows_per_split, nr;
    float *partial;          // [splits][2][cols]
};

// mode 0: out0 = sum_r lam_r sum_rows A16[r]                              (dc)
// mode 1: out0 = sum_rows A16[0], out1 = sum_rows A16[0] * A16[1]          (dXt, dXt * X)
// mode 2: out0 = sum_rows rowvec * A32[0], out1 = sum_rows A32[1] * A32[0] (dc W, dWs W)
template <int MODE>
__global__ __launch_bounds__(256) void colreduce_kernel(ColArgs a) {
    __shared__ float red[2][4][kColsPerBlock];
    const int ct = threadIdx.x & 63, rt = threadIdx.x >> 6;
    const int col = blockIdx.x * kColsPerBlock + ct * 4;
    const int r0 = blockIdx.y * a.rows_per_split, r1 = min(r0 + a.rows_per_split, a.rows);
    float s0[4] = {0.f, 0.f, 0.f, 0.f}, s1[4] = {0.f, 0.f, 0.f, 0.f};
    if (col < a.cols) {
        for (int r = r0 + rt; r < r1; r += 4) {
            if (MODE == 0) {
                for (int i = 0; i < a.nr; ++i) {
                    const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(a.A16[i] + (size_t)r * a.cols + col));
                    s0[0] += a.lam[i] * bf16_lo(v.x);
                    s0[1] += a.lam[i] * bf16_hi(v.x);
                    s0[2] += a.lam[i] * bf16_lo(v.y);
                    s0[3] += a.lam[i] * bf16_hi(v.y);
                }
            } else if (MODE == 1) {
                const u32x2 g = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(a.A16[0] + (size_t)r * a.cols + col));
                const u32x2 x = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(a.A16[1] + (size_t)r * a.cols + col));
                const float gv[4] = {bf16_lo(g.x), bf16_hi(g.x), bf16_lo(g.y), bf16_hi(g.y)};
                const float xv[4] = {bf16_lo(x.x), bf16_hi(x.x), bf16_lo(x.y), bf16_hi(x.y)};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    s0[j] += gv[j];
                    s1[j] += gv[j] * xv[j];
                }
            } else {
                const f32x4 w = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(a.A32[0] + (size_t)r * a.ld32 + col));
                const f32x4 g = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(a.A32[1] + (size_t)r * a.cols + col));
                const float f = a.rowvec[r];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    s0[j] += f * w[j];
                    s1[j] += g[j] * w[j];
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        red[0][rt][ct * 4 + j] = s0[j];
        red[1][rt][ct * 4 + j] = s1[j];
    }
    __syncthreads();
    const int c = blockIdx.x * kColsPerBlock + threadIdx.x;
    if (c < a.cols) {
        const int t = threadIdx.x;
        float *out = a.partial + (size_t)blockIdx.y * 2 * a.cols;
        out[c] = (red[0][0][t] + red[0][1][t]) + (red[0][2][t] + red[0][3][t]);
        out[a.cols + c] = (red[1][0][t] + red[1][1][t]) + (red[1][2][t] + red[1][3][t]);
    }
}

// Sum over the splits of partial[split][which][c] for 16 columns per workgroup: thread (c, q) adds the
// splits q, q + 16, ... in fp64, the sixteen lanes of a column meet in LDS (a fixed order).
constexpr int kFinishCols = 16;
__device__ __forceinline__ double split_sum(const float *partial, int splits, int cols, int which, int c, int q,
                                            double (*red)[kFinishCols]) {
    double v = 0.0;
    if (c < cols)
        for (int sp = q; sp < splits; sp += 16) v += (double)partial[((size_t)sp * 2 + which) * cols + c];
    __syncthreads();  // (the previous use of red is over)
    const int t = threadIdx.x & (kFinishCols - 1);
    red[q][t] = v;
    __syncthreads();
    double r = 0.0;
#pragma unroll
    for (int i = 0; i < 16; ++i) r += red[i][t];
    return r;
}

__global__ __launch_bounds__(256) void colfinish_dc_kernel(const float *partial, int splits, int cols, float *dc) {
    __shared__ double red[16][kFinishCols];
    const int c = blockIdx.x * kFinishCols + (threadIdx.x & (kFinishCols - 1)), q = threadIdx.x >> 4;
    const double v = split_sum(partial, splits, cols, 0, c, q, red);
    if (q == 0 && c < cols) dc[c] = (float)v;
}

// ddelta_k = -(1/s_k) P0 + R0,  ds_k = -(1/s_k^2) (P1 - delta_k P0) + R1
__global__ __launch_bounds__(256) void affine_bwd_finish_kernel(const float *px, int sx, const float *pw, int sw, int K,
                                                                const float *s, const float *delta, float *ddelta,
                                                                float *ds) {
    __shared__ double red[16][kFinishCols];
    const int k = blockIdx.x * kFinishCols + (threadIdx.x & (kFinishCols - 1)), q = threadIdx.x >> 4;
    const double p0 = split_sum(px, sx, K, 0, k, q, red), p1 = split_sum(px, sx, K, 1, k, q, red);
    const double r0 = split_sum(pw, sw, K, 0, k, q, red), r1 = split_sum(pw, sw, K, 1, k, q, red);
    if (q != 0 || k >= K) return;
    const double sv = s ? (double)s[k] : 1.0, dv = delta ? (double)delta[k] : 0.0;
    if (ddelta) ddelta[k] = (float)(-p0 / sv + r0);
    if (ds) ds[k] = (float)(-(p1 - dv * p0) / (sv * sv) + r1);
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// row ranges so that about 2048 workgroups exist
inline int splits_for(int64_t rows, int64_t cols) {
    const int64_t colblocks = cdiv(cols, kColsPerBlock);
    int64_t sp = std::max<int64_t>(1, std::min<int64_t>(cdiv(2048, colblocks), cdiv(rows, 16)));
    return (int)std::min<int64_t>(sp, 128);
}

struct AffineLayout {
    size_t pdy, px, pw, dc, total;
    int sdy, sx, sw;
};
inline AffineLayout affine_layout(int64_t M, int64_t N, int64_t K) {
    AffineLayout l;
    l.sdy = splits_for(M, N);
    l.sx = splits_for(M, K);
    l.sw = splits_for(N, K);
    size_t off = 0;
    l.pdy = off, off += align256((size_t)l.sdy * 2 * N * 4);
    l.px = off, off += align256((size_t)l.sx * 2 * K * 4);
    l.pw = off, off += align256((size_t)l.sw * 2 * K * 4);
    l.dc = off, off += align256((size_t)N * 4);
    l.total = off;
    return l;
}

}  // namespace

size_t affine_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    if (M < 0 || N < 0 || K < 0) return 0;
    return affine_layout(M, N, K).total + 256;
}

}  // namespace mq

extern "C" mq_status mq_affine_weight(const float *W, int64_t N, int64_t K, int64_t ldw, const float *s,
                                      const float *delta, const float *b, float *Ws, float *c, void *hip_stream) {
    using namespace mq;
    if (N < 0 || K < 1 || ldw < K || N > 0x7FFFFFF0 || K > (1 << 22)) return MQ_ERR_SHAPE;
    if (K % 4 != 0 || ldw % 4 != 0) return MQ_ERR_ALIGN;
    if (N == 0) return MQ_OK;
    if (!W || (!Ws && !c)) return MQ_ERR_NULL;
    if (!aligned16(W) || (Ws && !aligned16(Ws)) || (s && !aligned16(s)) || (delta && !aligned16(delta))) return MQ_ERR_ALIGN;
    affine_weight_kernel<<<dim3((unsigned)N), dim3(256), 0, static_cast<hipStream_t>(hip_stream)>>>(W, ldw, (int)K, s, delta,
                                                                                                    b, Ws, c);
    return launch_status();
}

extern "C" mq_status mq_affine_input(const uint16_t *X, int64_t M, int64_t K, const float *s, const float *delta,
                                     uint16_t *Xt, void *hip_stream) {
    using namespace mq;
    if (M < 0 || K < 1 || K > (1 << 22) || M > 0x7FFFFFF0) return MQ_ERR_SHAPE;
    if (K % 8 != 0) return MQ_ERR_ALIGN;
    if (M == 0) return MQ_OK;
    if (!X || !Xt) return MQ_ERR_NULL;
    if (!aligned16(X) || !aligned16(Xt) || (s && !aligned16(s)) || (delta && !aligned16(delta))) return MQ_ERR_ALIGN;
    const int64_t chunks = M * K / 8;
    if (cdiv(chunks, 256) > 0x7FFFFFFF) return MQ_ERR_SHAPE;
    affine_input_kernel<<<dim3((unsigned)cdiv(chunks, 256)), dim3(256), 0, static_cast<hipStream_t>(hip_stream)>>>(
        X, chunks, (int)K, s, delta, Xt);
    return launch_status();
}

extern "C" mq_status mq_affine_bwd(const uint16_t *X, const uint16_t *dXt, const float *W, int64_t ldw, const float *dWs,
                                   const uint16_t *const *dY, const float *lambda, int nr, int64_t M, int64_t N,
                                   int64_t K, const float *s, const float *delta, float *ddelta, float *ds, float *dc,
                                   void *ws, size_t ws_bytes, void *hip_stream) {
    using namespace mq;
    if (nr < 1 || nr > 3) return MQ_ERR_BITS;
    if (M < 1 || N < 1 || K < 1 || ldw < K) return MQ_ERR_SHAPE;
    if (M > (1 << 22) || N > (1 << 22) || K > (1 << 22)) return MQ_ERR_SHAPE;
    if (K % 4 != 0 || N % 4 != 0 || ldw % 4 != 0) return MQ_ERR_ALIGN;
    if (!X || !dXt || !W || !dWs || !dY || (!ddelta && !ds && !dc)) return MQ_ERR_NULL;
    for (int i = 0; i < nr; ++i)
        if (!dY[i]) return MQ_ERR_NULL;
    if (!aligned16(X) || !aligned16(dXt) || !aligned16(W) || !aligned16(dWs)) return MQ_ERR_ALIGN;
    for (int i = 0; i < nr; ++i)
        if (!aligned16(dY[i])) return MQ_ERR_ALIGN;
    const AffineLayout lay = affine_layout(M, N, K);
    if (!ws || ws_bytes < lay.total + 256) return MQ_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    uint8_t *base = reinterpret_cast<uint8_t *>((reinterpret_cast<uintptr_t>(ws) + 255) & ~(uintptr_t)255);
    float *pdy = reinterpret_cast<float *>(base + lay.pdy), *px = reinterpret_cast<float *>(base + lay.px);
    float *pw = reinterpret_cast<float *>(base + lay.pw);
    float *dcv = dc ? dc : reinterpret_cast<float *>(base + lay.dc);

    ColArgs a{};
    // dc[n] = sum_r lambda_r sum_m dY_r[m, n]
    for (int i = 0; i < nr; ++i) {
        a.A16[i] = dY[i];
        a.lam[i] = lambda ? lambda[i] : 1.0f;
    }
    a.nr = nr;
    a.rows = (int)M;
    a.cols = (int)N;
    a.rows_per_split = (int)cdiv(M, lay.sdy);
    a.partial = pdy;
    colreduce_kernel<0><<<dim3((unsigned)cdiv(N, kColsPerBlock), (unsigned)lay.sdy), dim3(256), 0, st>>>(a);
    colfinish_dc_kernel<<<dim3((unsigned)cdiv(N, kFinishCols)), dim3(256), 0, st>>>(pdy, lay.sdy, (int)N, dcv);
    if (!ddelta && !ds) return launch_status();

    // over the tokens: sum dXt, sum dXt * X
    ColArgs x{};
    x.A16[0] = dXt;
    x.A16[1] = X;
    x.rows = (int)M;
    x.cols = (int)K;
    x.rows_per_split = (int)cdiv(M, lay.sx);
    x.partial = px;
    colreduce_kernel<1><<<dim3((unsigned)cdiv(K, kColsPerBlock), (unsigned)lay.sx), dim3(256), 0, st>>>(x);
    // over the channels: sum dc W, sum dWs W
    ColArgs w{};
    w.A32[0] = W;
    w.A32[1] = dWs;
    w.ld32 = ldw;
    w.rowvec = dcv;
    w.rows = (int)N;
    w.cols = (int)K;
    w.rows_per_split = (int)cdiv(N, lay.sw);
    w.partial = pw;
    colreduce_kernel<2><<<dim3((unsigned)cdiv(K, kColsPerBlock), (unsigned)lay.sw), dim3(256), 0, st>>>(w);
    affine_bwd_finish_kernel<<<dim3((unsigned)cdiv(K, kFinishCols)), dim3(256), 0, st>>>(px, lay.sx, pw, lay.sw, (int)K, s, delta,
                                                                                 ddelta, ds);
    return launch_status();
}
