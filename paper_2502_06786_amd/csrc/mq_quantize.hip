// mq_quantize_int8: per-output-channel MinMax quantizer to 8 bits (section 3.1.1; with gamma/beta
// the clipped form of section 3.1.2).  HBM-bound: each row is read once into registers, reduced to
// its min/max with wavefront shuffles, and quantized from the registers, so the algorithmic traffic
// is 4 B read + 1 B written per weight.
#include "mq_common.h"

namespace mq {

constexpr int kQuantVecMax = 16;  // float4 per thread held in registers

__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// alpha and z of one row from its min and max: one IEEE fp32 operation per symbol.
__device__ __forceinline__ void scale_zero(float mn, float mx, const float *gamma, const float *beta,
                                           int64_t n, float &a, float &z) {
    const float hi = gamma ? __fmul_rn(gamma[n], mx) : mx;
    const float lo = beta ? __fmul_rn(beta[n], mn) : mn;
    if (hi == lo) {
        a = 1.0f;
        z = -lo;
    } else {
        a = __fdiv_rn(__fsub_rn(hi, lo), 255.0f);
        z = __fdiv_rn(-lo, a);
    }
}

__device__ __forceinline__ uint32_t quant1(float w, float a, float z) {
    float r = rintf(__fadd_rn(__fdiv_rn(w, a), z));  // round half to even
    r = fminf(fmaxf(r, 0.0f), 255.0f);
    return (uint32_t)r;
}

// TPR threads cooperate on one row; a block of BLOCK threads holds BLOCK / TPR rows.
// Requires K % 4 == 0, ldw % 4 == 0, K / 4 <= TPR * kQuantVecMax.
template <int TPR, int BLOCK>
__global__ __launch_bounds__(BLOCK) void quantize_rows_kernel(const float *__restrict__ W, int64_t N,
                                                              int64_t K, int64_t ldw,
                                                              const float *__restrict__ gamma,
                                                              const float *__restrict__ beta,
                                                              uint8_t *__restrict__ Q,
                                                              float *__restrict__ alpha,
                                                              float *__restrict__ zero) {
    constexpr int ROWS = BLOCK / TPR;
    constexpr int WAVES_PER_ROW = TPR / 64;
    __shared__ float red_min[BLOCK / 64], red_max[BLOCK / 64];

    const int t = threadIdx.x % TPR;
    const int row_in_block = threadIdx.x / TPR;
    const int64_t n = (int64_t)blockIdx.x * ROWS + row_in_block;
    const bool live = n < N;
    const int nv = (int)(K >> 2);

    f32x4 v[kQuantVecMax];
    float mn = INFINITY, mx = -INFINITY;
    if (live) {
        const f32x4 *src = reinterpret_cast<const f32x4 *>(W + n * ldw);
#pragma unroll
        for (int i = 0; i < kQuantVecMax; ++i) {
            const int idx = t + i * TPR;
            if (idx < nv) {
                v[i] = __builtin_nontemporal_load(src + idx);
                mn = fminf(fminf(fminf(mn, v[i].x), fminf(v[i].y, v[i].z)), v[i].w);
                mx = fmaxf(fmaxf(fmaxf(mx, v[i].x), fmaxf(v[i].y, v[i].z)), v[i].w);
            }
        }
    }
    mn = wave_min(mn);
    mx = wave_max(mx);
    if constexpr (WAVES_PER_ROW > 1) {
        const int wave = threadIdx.x / 64;
        if ((threadIdx.x & 63) == 0) {
            red_min[wave] = mn;
            red_max[wave] = mx;
        }
        __syncthreads();
        const int first = row_in_block * WAVES_PER_ROW;
        mn = red_min[first];
        mx = red_max[first];
#pragma unroll
        for (int w = 1; w < WAVES_PER_ROW; ++w) {
            mn = fminf(mn, red_min[first + w]);
            mx = fmaxf(mx, red_max[first + w]);
        }
    }
    if (!live) return;
    float a, z;
    scale_zero(mn, mx, gamma, beta, n, a, z);
    if (t == 0) {
        alpha[n] = a;
        zero[n] = z;
    }
    uint32_t *dst = reinterpret_cast<uint32_t *>(Q + n * K);
#pragma unroll
    for (int i = 0; i < kQuantVecMax; ++i) {
        const int idx = t + i * TPR;
        if (idx < nv) {
            const uint32_t p = quant1(v[i].x, a, z) | (quant1(v[i].y, a, z) << 8) |
                               (quant1(v[i].z, a, z) << 16) | (quant1(v[i].w, a, z) << 24);
            __builtin_nontemporal_store(p, dst + idx);
        }
    }
}

// Any K and stride: one block per row, the row is read twice (second read normally hits L2).
__global__ __launch_bounds__(256) void quantize_rows_generic_kernel(const float *__restrict__ W, int64_t N,
                                                                    int64_t K, int64_t ldw,
                                                                    const float *__restrict__ gamma,
                                                                    const float *__restrict__ beta,
                                                                    uint8_t *__restrict__ Q,
                                                                    float *__restrict__ alpha,
                                                                    float *__restrict__ zero) {
    __shared__ float red_min[4], red_max[4];
    const int64_t n = blockIdx.x;
    const float *w = W + n * ldw;
    float mn = INFINITY, mx = -INFINITY;
    for (int64_t k = threadIdx.x; k < K; k += 256) {
        mn = fminf(mn, w[k]);
        mx = fmaxf(mx, w[k]);
    }
    mn = wave_min(mn);
    mx = wave_max(mx);
    if ((threadIdx.x & 63) == 0) {
        red_min[threadIdx.x / 64] = mn;
        red_max[threadIdx.x / 64] = mx;
    }
    __syncthreads();
    mn = fminf(fminf(red_min[0], red_min[1]), fminf(red_min[2], red_min[3]));
    mx = fmaxf(fmaxf(red_max[0], red_max[1]), fmaxf(red_max[2], red_max[3]));
    float a, z;
    scale_zero(mn, mx, gamma, beta, n, a, z);
    if (threadIdx.x == 0) {
        alpha[n] = a;
        zero[n] = z;
    }
    for (int64_t k = threadIdx.x; k < K; k += 256) Q[n * K + k] = (uint8_t)quant1(w[k], a, z);
}

// fp32 -> bf16 (round to nearest even) of the per-channel scale and zero-point for the decode path
__global__ __launch_bounds__(256) void params_to_bf16_kernel(const float *__restrict__ alpha,
                                                             const float *__restrict__ zero, int64_t N,
                                                             uint16_t *__restrict__ alpha_bf16,
                                                             uint16_t *__restrict__ zero_bf16) {
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n < N) {
        alpha_bf16[n] = (uint16_t)float_to_bf16_bits(alpha[n]);
        zero_bf16[n] = (uint16_t)float_to_bf16_bits(zero[n]);
    }
}

}  // namespace mq

extern "C" mq_status mq_params_to_bf16(const float *alpha, const float *zero, int64_t N, uint16_t *alpha_bf16,
                                       uint16_t *zero_bf16, void *hip_stream) {
    using namespace mq;
    if (N < 0 || N > 0x7FFFFFFF) return MQ_ERR_SHAPE;
    if (N == 0) return MQ_OK;
    if (!alpha || !zero || !alpha_bf16 || !zero_bf16) return MQ_ERR_NULL;
    params_to_bf16_kernel<<<dim3((unsigned)cdiv(N, 256)), dim3(256), 0, static_cast<hipStream_t>(hip_stream)>>>(
        alpha, zero, N, alpha_bf16, zero_bf16);
    return launch_status();
}

extern "C" mq_status mq_quantize_int8(const float *W, int64_t N, int64_t K, int64_t ldw,
                                      const float *gamma, const float *beta, uint8_t *Q,
                                      float *alpha, float *zero, void *hip_stream) {
    using namespace mq;
    if (N < 0 || K < 0 || ldw < K) return MQ_ERR_SHAPE;
    if (N == 0) return MQ_OK;
    if (K == 0) return MQ_ERR_SHAPE;
    if (N > 0x7FFFFFFF) return MQ_ERR_SHAPE;
    if (!W || !Q || !alpha || !zero) return MQ_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const bool vec = (K % 4 == 0) && (ldw % 4 == 0) && aligned16(W) && aligned16(Q) &&
                     (K / 4 <= 1024 * kQuantVecMax);
    if (!vec) {
        quantize_rows_generic_kernel<<<dim3((unsigned)N), dim3(256), 0, st>>>(W, N, K, ldw, gamma, beta, Q,
                                                                            alpha, zero);
    } else if (K / 4 <= 64 * kQuantVecMax) {
        quantize_rows_kernel<64, 256><<<dim3((unsigned)cdiv(N, 4)), dim3(256), 0, st>>>(W, N, K, ldw, gamma,
                                                                                      beta, Q, alpha, zero);
    } else if (K / 4 <= 256 * kQuantVecMax) {
        quantize_rows_kernel<256, 256><<<dim3((unsigned)N), dim3(256), 0, st>>>(W, N, K, ldw, gamma, beta, Q,
                                                                              alpha, zero);
    } else {
        quantize_rows_kernel<1024, 1024><<<dim3((unsigned)N), dim3(1024), 0, st>>>(W, N, K, ldw, gamma, beta,
                                                                                 Q, alpha, zero);
    }
    return launch_status();
}
