// mq_matquant_l2_loss: the weighted sum over the bit-widths of the layer-wise L2 reconstruction losses
// (joint objective of section 3.2 with the loss of section 3.1.2) and its co-distillation variants
// (section 5.2), together with the gradients dY_i that the straight-through backward consumes.
//
// HBM-bound: every Y_i and the target are read once, every dY_i written once (2 (2 nr + 1) bytes per
// output element); the nr sums are reduced per workgroup and finished by a second, one-workgroup
// kernel in a fixed order (no atomics: the losses are reproducible bit for bit).
#include "mq_common.h"

namespace mq {

namespace {

constexpr int kLossBlock = 256;
constexpr int kLossPerThread = 2;  // 16-byte chunks per thread

struct LossArgs {
    const uint16_t *Y[3];
    const uint16_t *target;
    uint16_t *dY[3];
    int teacher[3];
    float coef[3];  // lambda_i * 2 / (M N)
    int nr;
    int mix;
    int64_t chunks;  // 16-byte chunks per tensor
    float *partial;  // [blocks][4]
};

__global__ __launch_bounds__(kLossBlock) void l2_loss_kernel(LossArgs a) {
    __shared__ float red[kLossBlock / 64][4];
    float sum[3] = {0.f, 0.f, 0.f};
    const int64_t base = ((int64_t)blockIdx.x * kLossBlock + threadIdx.x) * kLossPerThread;
#pragma unroll
    for (int c = 0; c < kLossPerThread; ++c) {
        const int64_t ch = base + c;
        if (ch >= a.chunks) break;
        u32x4 y[3], t = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < 3; ++i)
            if (i < a.nr) y[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.Y[i]) + ch);
        if (a.target) t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.target) + ch);
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            if (i >= a.nr) break;
            const int th = a.teacher[i];
            const u32x4 tt = th < 0 ? t : (th == 0 ? y[0] : (th == 1 ? y[1] : y[2]));
            u32x4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float y0 = bf16_lo(y[i][j]), y1 = bf16_hi(y[i][j]);
                float d0 = y0 - bf16_lo(tt[j]), d1 = y1 - bf16_hi(tt[j]);
                float s = d0 * d0 + d1 * d1;
                if (a.mix && th >= 0) {  // teacher and ground truth, weighted equally
                    const float e0 = y0 - bf16_lo(t[j]), e1 = y1 - bf16_hi(t[j]);
                    s = 0.5f * (s + e0 * e0 + e1 * e1);
                    d0 = 0.5f * (d0 + e0);
                    d1 = 0.5f * (d1 + e1);
                }
                sum[i] += s;
                o[j] = pack_bf16x2(a.coef[i] * d0, a.coef[i] * d1);
            }
            reinterpret_cast<u32x4 *>(a.dY[i])[ch] = o;
        }
    }
    // workgroup sums, fixed order
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        float v = sum[i];
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m);
        if (lane == 0) red[wave][i] = v;
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        float v = 0.f;
        for (int w = 0; w < kLossBlock / 64; ++w) v += red[w][threadIdx.x];
        a.partial[(size_t)blockIdx.x * 4 + threadIdx.x] = v;
    }
}

__global__ __launch_bounds__(256) void l2_loss_finish_kernel(const float *partial, int64_t blocks, int nr, float inv_mn,
                                                             float *losses) {
    __shared__ double red[256];
    for (int i = 0; i < nr; ++i) {
        double v = 0.0;
        for (int64_t b = threadIdx.x; b < blocks; b += 256) v += (double)partial[b * 4 + i];
        red[threadIdx.x] = v;
        __syncthreads();
        for (int s = 128; s > 0; s >>= 1) {
            if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
            __syncthreads();
        }
        if (threadIdx.x == 0) losses[i] = (float)(red[0] * (double)inv_mn);
        __syncthreads();
    }
}

inline int64_t loss_blocks(int64_t M, int64_t N) {
    const int64_t chunks = M * N / 8;
    return cdiv(chunks, (int64_t)kLossBlock * kLossPerThread);
}

}  // namespace

mq_status launch_loss_finish(const float *partial, int64_t blocks, int nr, float inv_mn, float *losses,
                             hipStream_t st) {
    l2_loss_finish_kernel<<<dim3(1), dim3(256), 0, st>>>(partial, blocks, nr, inv_mn, losses);
    return launch_status();
}

size_t loss_workspace_bytes(int64_t M, int64_t N) {
    if (M < 0 || N < 0) return 0;
    return (size_t)loss_blocks(M, N) * 16 + 512;
}

}  // namespace mq

extern "C" mq_status mq_matquant_l2_loss(const uint16_t *const *Y, const uint16_t *target, const int *teacher,
                                         const float *lambda, int64_t M, int64_t N, int nr, uint32_t flags,
                                         uint16_t *const *dY, float *losses, void *ws, size_t ws_bytes,
                                         void *hip_stream) {
    using namespace mq;
    if (nr < 1 || nr > 3) return MQ_ERR_BITS;
    if (M < 0 || N < 0 || (M > 0 && N > (int64_t)0x7FFFFFFFFFFFll / M)) return MQ_ERR_SHAPE;
    if ((M * N) % 8 != 0) return MQ_ERR_ALIGN;
    const bool mix = (flags & MQ_FLAG_LOSS_MIX) != 0;
    bool need_target = mix;
    if (teacher)
        for (int i = 0; i < nr; ++i) {
            if (teacher[i] < -1 || teacher[i] >= nr || teacher[i] == i) return MQ_ERR_SHAPE;
            if (teacher[i] < 0) need_target = true;
        }
    else
        need_target = true;
    if (M * N == 0) return MQ_OK;
    if (!Y || !dY || !losses || (need_target && !target)) return MQ_ERR_NULL;
    for (int i = 0; i < nr; ++i) {
        if (!Y[i] || !dY[i]) return MQ_ERR_NULL;
        if (!aligned16(Y[i]) || !aligned16(dY[i])) return MQ_ERR_ALIGN;
    }
    if (target && !aligned16(target)) return MQ_ERR_ALIGN;
    if (!ws || ws_bytes < loss_workspace_bytes(M, N)) return MQ_ERR_WORKSPACE;

    LossArgs a{};
    const double mn = (double)M * (double)N;
    for (int i = 0; i < nr; ++i) {
        a.Y[i] = Y[i];
        a.dY[i] = dY[i];
        a.teacher[i] = teacher ? teacher[i] : -1;
        a.coef[i] = (float)((lambda ? (double)lambda[i] : 1.0) * 2.0 / mn);
    }
    a.target = target;
    a.nr = nr;
    a.mix = mix ? 1 : 0;
    a.chunks = M * N / 8;
    a.partial = reinterpret_cast<float *>((reinterpret_cast<uintptr_t>(ws) + 255) & ~(uintptr_t)255);
    const int64_t blocks = loss_blocks(M, N);
    if (blocks > 0x7FFFFFFF) return MQ_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    l2_loss_kernel<<<dim3((unsigned)blocks), dim3(kLossBlock), 0, st>>>(a);
    mq_status s = launch_status();
    if (s != MQ_OK) return s;
    return launch_loss_finish(a.partial, blocks, nr, (float)(1.0 / mn), losses, st);
}
