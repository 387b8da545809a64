// mq_linear_bwd_clip: gradients of the MatQuant objective with respect to the clip factors gamma, beta
// of the quantizer of section 3.1.2 (alpha = (gamma max - beta min) / 255, z = -beta min / alpha), under
// the straight-through estimator: the rounding to the 8-bit code and the rounding inside the slicing
// operator of section 3.2 pass the gradient unchanged, the clamp to 0..255 and the clamp of a slice to
// its top code pass it only where they do not act.  With u = w / alpha + z and What_r = alpha (S_r - z):
//     d What_r / d alpha = (S_r - z) - m_r w / alpha          d What_r / d z = -alpha (1 - m_r)
// where m_r = 1 where neither clamp acts.  Unlike dW, where every bit-width has the same derivative and the
// gradients are summed before one contraction, these coefficients differ per bit-width: each r takes its
// own dY_r^T X contraction (the matrix-core kernel of the backward, into a scratch matrix), followed by a
// row reduction against the coefficients (HBM-bound: 4 + 4 + 1 bytes per weight and bit-width).
#include "mq_common.h"

namespace mq {

namespace {

struct ClipArgs {
    const float *W;       // [N, ldw]
    const uint8_t *Q;     // [N, K]
    const float *G;       // [N, K]: lambda_r dY_r^T X
    const float *alpha, *zero;
    const float *gamma, *beta;  // [N] or null (= 1)
    float *acc;           // [N][2]: running d alpha, d z over the bit-widths
    float *dgamma, *dbeta, *dalpha, *dzero;
    int64_t ldw;
    int N, K;
    int r, ep;
    int first, last;
};

// One workgroup per output channel.  Four weights per thread and step; fp32 products, per-thread fp32
// sums over at most K / 1024 steps, fp64 across the workgroup.
__global__ __launch_bounds__(256) void clip_reduce_kernel(ClipArgs a) {
    __shared__ double red[4][4];
    const int n = blockIdx.x;
    const float al = a.alpha[n], ze = a.zero[n];
    const float *w = a.W + (size_t)n * a.ldw;
    const float *g = a.G + (size_t)n * a.K;
    const uint8_t *q = a.Q + (size_t)n * a.K;
    const int s = 8 - a.r, half = (1 << s) >> 1, top = (1 << a.r) - 1;
    float sa = 0.f, sz = 0.f, mn = INFINITY, mx = -INFINITY;
    for (int k = threadIdx.x * 4; k < a.K; k += 1024) {
        const f32x4 wv = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(w + k));
        const f32x4 gv = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(g + k));
        const uint32_t qv = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(q + k));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // the quantizer's own operations, in its order, decide whether its clamp acted
            const float t = __fdiv_rn(wv[j], al);
            const float rounded = rintf(__fadd_rn(t, ze));
            const bool inside = rounded >= 0.0f && rounded <= 255.0f;
            const int code8 = (int)((qv >> (8 * j)) & 0xFFu);
            const int raw = (code8 + half) >> s;
            const bool clamped = !a.ep && raw > top;
            const float S = (float)((clamped ? top : raw) << s);
            const bool m = inside && !clamped;
            sa += gv[j] * ((S - ze) - (m ? t : 0.0f));
            sz += m ? 0.0f : gv[j] * -al;
            mn = fminf(mn, wv[j]);
            mx = fmaxf(mx, wv[j]);
        }
    }
    double da = sa, dz = sz;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        da += __shfl_xor(da, o);
        dz += __shfl_xor(dz, o);
        mn = fminf(mn, __shfl_xor(mn, o));
        mx = fmaxf(mx, __shfl_xor(mx, o));
    }
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
        red[wave][0] = da;
        red[wave][1] = dz;
        red[wave][2] = mn;
        red[wave][3] = mx;
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    da = red[0][0] + red[1][0] + red[2][0] + red[3][0];
    dz = red[0][1] + red[1][1] + red[2][1] + red[3][1];
    if (!a.first) {
        da += (double)a.acc[2 * n];
        dz += (double)a.acc[2 * n + 1];
    }
    if (!a.last) {
        a.acc[2 * n] = (float)da;
        a.acc[2 * n + 1] = (float)dz;
        return;
    }
    const double lo = fmin(fmin(red[0][2], red[1][2]), fmin(red[2][2], red[3][2]));
    const double hi = fmax(fmax(red[0][3], red[1][3]), fmax(red[2][3], red[3][3]));
    // chain rule through alpha(gamma, beta) and z(beta, alpha), with beta min = -z alpha.  A row whose
    // clipped range is empty (the quantizer's own fp32 test) was given alpha = 1 and carries no gradient.
    const float lo32 = (float)lo, hi32 = (float)hi;
    const bool degenerate = (a.gamma ? __fmul_rn(a.gamma[n], hi32) : hi32) == (a.beta ? __fmul_rn(a.beta[n], lo32) : lo32);
    const double A = al, Z = ze;
    const double da_dg = hi / 255.0, da_db = -lo / 255.0;
    const double bmin_a2 = -Z / A;  // beta min / alpha^2
    const double dz_dg = bmin_a2 * da_dg;
    const double dz_db = -lo / A + bmin_a2 * da_db;
    if (a.dalpha) a.dalpha[n] = (float)da;
    if (a.dzero) a.dzero[n] = (float)dz;
    a.dgamma[n] = degenerate ? 0.0f : (float)(da * da_dg + dz * dz_dg);
    a.dbeta[n] = degenerate ? 0.0f : (float)(da * da_db + dz * dz_db);
}

__global__ void clip_zero_kernel(float *a, float *b, float *c, float *d, int n) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    a[i] = 0.f;
    b[i] = 0.f;
    if (c) c[i] = 0.f;
    if (d) d[i] = 0.f;
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace

size_t clip_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    return align256((size_t)N * K * 4) + align256((size_t)N * 8) + mq_workspace_bytes(MQ_OP_LINEAR_BWD, M, N, K, 1) + 256;
}

}  // namespace mq

extern "C" mq_status mq_linear_bwd_clip(const float *W, int64_t ldw, const uint16_t *X, const uint8_t *Q,
                                        const float *alpha, const float *zero, const float *gamma,
                                        const float *beta, const uint16_t *const *dY, const float *lambda, int64_t M,
                                        int64_t N, int64_t K, const int *rs, int nr, uint32_t flags, float *dgamma,
                                        float *dbeta, float *dalpha, float *dzero, void *ws, size_t ws_bytes,
                                        void *hip_stream) {
    using namespace mq;
    if (nr < 1 || nr > 3 || !rs) return MQ_ERR_BITS;
    for (int i = 0; i < nr; ++i) {
        if (rs[i] < 1 || rs[i] > 8) return MQ_ERR_BITS;
        for (int j = 0; j < i; ++j)
            if (rs[j] == rs[i]) return MQ_ERR_BITS;
    }
    if (M < 0 || N < 0 || K < 1 || ldw < K) return MQ_ERR_SHAPE;
    if (M > (1 << 22) || N > (1 << 22) || K > (1 << 22)) return MQ_ERR_SHAPE;
    if (K % 16 != 0 || N % 16 != 0 || ldw % 4 != 0) return MQ_ERR_ALIGN;
    if (N == 0) return MQ_OK;
    if (!W || !Q || !alpha || !zero || !dgamma || !dbeta || (M > 0 && (!X || !dY))) return MQ_ERR_NULL;
    for (int i = 0; i < nr && M > 0; ++i)
        if (!dY[i]) return MQ_ERR_NULL;
    if (!aligned16(W) || !aligned16(Q)) return MQ_ERR_ALIGN;
    if (!ws || ws_bytes < clip_workspace_bytes(M, N, K) || !aligned16(ws)) return MQ_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);

    uint8_t *base = reinterpret_cast<uint8_t *>((reinterpret_cast<uintptr_t>(ws) + 255) & ~(uintptr_t)255);
    float *G = reinterpret_cast<float *>(base);
    float *acc = reinterpret_cast<float *>(base + align256((size_t)N * K * 4));
    uint8_t *bws = base + align256((size_t)N * K * 4) + align256((size_t)N * 8);
    const size_t bws_bytes = mq_workspace_bytes(MQ_OP_LINEAR_BWD, M, N, K, 1);

    if (M == 0) {  // no tokens: the objective does not depend on the weights
        clip_zero_kernel<<<dim3((unsigned)cdiv(N, 256)), dim3(256), 0, st>>>(dgamma, dbeta, dalpha, dzero, (int)N);
        return launch_status();
    }
    for (int i = 0; i < nr; ++i) {
        const float lam = lambda ? lambda[i] : 1.0f;
        // G = lambda_r dY_r^T X through the dW path of the backward, one bit-width at a time
        mq_status s = mq_linear_bwd(X, nullptr, nullptr, nullptr, dY + i, &lam, M, N, K, rs + i, 1, 0, nullptr, G, bws,
                                    bws_bytes, hip_stream);
        if (s != MQ_OK) return s;
        ClipArgs a{};
        a.W = W;
        a.Q = Q;
        a.G = G;
        a.alpha = alpha;
        a.zero = zero;
        a.gamma = gamma;
        a.beta = beta;
        a.acc = acc;
        a.dgamma = dgamma;
        a.dbeta = dbeta;
        a.dalpha = dalpha;
        a.dzero = dzero;
        a.ldw = ldw;
        a.N = (int)N;
        a.K = (int)K;
        a.r = rs[i];
        a.ep = (flags & MQ_FLAG_EXTRA_PRECISION) ? 1 : 0;
        a.first = i == 0;
        a.last = i + 1 == nr;
        clip_reduce_kernel<<<dim3((unsigned)N), dim3(256), 0, st>>>(a);
        if ((s = launch_status()) != MQ_OK) return s;
    }
    return MQ_OK;
}
