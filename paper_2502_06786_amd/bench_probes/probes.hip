// Measurement helpers: what this GPU sustains on a loop that does nothing but bf16 matrix-core
// products, and on a kernel that does nothing but read.  They put the roofline fractions of the
// method's kernels next to a measured ceiling as well as the published one; they compute nothing
// of the method.
#include "../csrc/mq_common.h"
#include "probes.h"

namespace mq {

// 256 threads = one wave per SIMD, 12 independent 32x32 accumulators per wave (the register budget
// of the fused kernels), operands taken from `ops` (so that their bit patterns - and with them the
// power the products draw - are the caller's choice) and rotated every iteration.
__global__ __launch_bounds__(256) void probe_mfma_kernel(const u32x4 *__restrict__ ops, int64_t iters,
                                                         float *__restrict__ sink) {
    constexpr int NACC = 12;
    f32x16 acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    Frag8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i].u = ops[(threadIdx.x * 8 + i) & 4095];
        b[i].u = ops[(threadIdx.x * 8 + 4 + i) & 4095];
    }
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < NACC; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 3].b, b[(i + (int)it) & 3].b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
}

// The same loop on the other bf16 shape, 16x16x32, with two waves per SIMD (512 threads) and 24
// independent 16x16 accumulators per wave: per product half the flops of a 32x32x16 one for the same
// operand registers and a quarter of the accumulator registers.  One wave per SIMD issues these
// products at little more than half rate, two waves at nearly full rate, and on N(0,1) operands the
// loop sustains more than the 32x32x16 loop at any occupancy (the chip is power-limited there).
__global__ __launch_bounds__(512) void probe_mfma16_kernel(const u32x4 *__restrict__ ops, int64_t iters,
                                                           float *__restrict__ sink) {
    constexpr int NACC = 24;
    f32x4 acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    Frag8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i].u = ops[(threadIdx.x * 8 + i) & 4095];
        b[i].u = ops[(threadIdx.x * 8 + 4 + i) & 4095];
    }
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < NACC; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 3].b, b[(i + (int)it) & 3].b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NACC; ++i) s += (acc[i][0] + acc[i][1]) + (acc[i][2] + acc[i][3]);
    sink[blockIdx.x * 512 + threadIdx.x] = s;
}

// Each wave reads whole kilobytes (16 bytes per lane), four non-temporal loads in flight, grid-stride
// (non-temporal loads stream 7-9 % faster than plain ones on buffers beyond the caches).
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4 *__restrict__ src, int64_t chunks,
                                                         uint32_t *__restrict__ sink) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; c + 3 * stride < chunks; c += 4 * stride) {
        const u32x4 v0 = __builtin_nontemporal_load(src + c), v1 = __builtin_nontemporal_load(src + c + stride);
        const u32x4 v2 = __builtin_nontemporal_load(src + c + 2 * stride), v3 = __builtin_nontemporal_load(src + c + 3 * stride);
        acc += v0 ^ v1;
        acc += v2 ^ v3;
    }
    for (; c < chunks; c += stride) acc += src[c];
    // (the sum is data dependent, so the loads cannot be dropped; the store almost never happens)
    if (acc.x + acc.y + acc.z + acc.w == 0x9E3779B9u) sink[0] = acc.x;
}

}  // namespace mq

extern "C" int mq_probe_mfma(const uint16_t *operands_bf16, int64_t iters, float *sink, void *hip_stream) {
    using namespace mq;
    if (!operands_bf16 || !sink) return MQ_ERR_NULL;
    if (iters < 1 || iters > (1ll << 24)) return MQ_ERR_SHAPE;
    if (!aligned16(operands_bf16)) return MQ_ERR_ALIGN;
    probe_mfma_kernel<<<dim3(256), dim3(256), 0, static_cast<hipStream_t>(hip_stream)>>>(
        reinterpret_cast<const u32x4 *>(operands_bf16), iters, sink);
    return launch_status();
}

extern "C" int mq_probe_mfma16(const uint16_t *operands_bf16, int64_t iters, float *sink, void *hip_stream) {
    using namespace mq;
    if (!operands_bf16 || !sink) return MQ_ERR_NULL;
    if (iters < 1 || iters > (1ll << 24)) return MQ_ERR_SHAPE;
    if (!aligned16(operands_bf16)) return MQ_ERR_ALIGN;
    probe_mfma16_kernel<<<dim3(256), dim3(512), 0, static_cast<hipStream_t>(hip_stream)>>>(
        reinterpret_cast<const u32x4 *>(operands_bf16), iters, sink);
    return launch_status();
}

extern "C" int mq_probe_read(const void *src, int64_t bytes, uint32_t *sink, void *hip_stream) {
    using namespace mq;
    if (!src || !sink) return MQ_ERR_NULL;
    if (bytes < 16 || (bytes & 15)) return MQ_ERR_SHAPE;
    if (!aligned16(src)) return MQ_ERR_ALIGN;
    const int64_t chunks = bytes >> 4;
    int64_t blocks = cdiv(chunks, 256 * 4);
    if (blocks > 256 * 8) blocks = 256 * 8;
    probe_read_kernel<<<dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream)>>>(
        reinterpret_cast<const u32x4 *>(src), chunks, sink);
    return launch_status();
}
