// mq_ffn_mixnmatch: a stack of gated feed-forward layers on the decode path, every layer at its own
// bit-width (layer-wise Mix'n'Match, section 4.3 and appendix B).  The matrix-vector products are the
// decode GEMVs of mq_gemv_sliced (the gate and up rows are one stacked plane, so both come out of a
// single pass over the activations); the gate activation and the optional residual are two small
// element-wise kernels.
#include "mq_common.h"

namespace mq {

namespace {

__device__ __forceinline__ float gelu_tanh(float v) {
    // 0.5 v (1 + tanh(sqrt(2 / pi) (v + 0.044715 v^3)))
    const float t = 0.7978845608028654f * (v + 0.044715f * v * v * v);
    return 0.5f * v * (1.0f + tanhf(t));
}
__device__ __forceinline__ float silu(float v) { return v / (1.0f + __expf(-v)); }

// a[b, f] = act(gu[b, f]) * gu[b, F + f], eight elements per thread
template <bool SILU>
__global__ __launch_bounds__(256) void gate_kernel(const uint16_t *__restrict__ gu, uint16_t *__restrict__ a, int B, int F) {
    const int per_row = F >> 3;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= B * per_row) return;
    const int b = idx / per_row, f = (idx - b * per_row) << 3;
    const u32x4 g = *reinterpret_cast<const u32x4 *>(gu + (size_t)b * 2 * F + f);
    const u32x4 u = *reinterpret_cast<const u32x4 *>(gu + (size_t)b * 2 * F + F + f);
    u32x4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float g0 = __uint_as_float(g[j] << 16), g1 = __uint_as_float(g[j] & 0xFFFF0000u);
        const float u0 = __uint_as_float(u[j] << 16), u1 = __uint_as_float(u[j] & 0xFFFF0000u);
        const float a0 = (SILU ? silu(g0) : gelu_tanh(g0)) * u0, a1 = (SILU ? silu(g1) : gelu_tanh(g1)) * u1;
        o[j] = pack_bf16x2(a0, a1);
    }
    *reinterpret_cast<u32x4 *>(a + (size_t)b * F + f) = o;
}

// out[i] = bf16(h[i] + o[i]), eight elements per thread
__global__ __launch_bounds__(256) void residual_kernel(const uint16_t *__restrict__ h, const uint16_t *__restrict__ o,
                                                       uint16_t *__restrict__ out, int n8) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= n8) return;
    const u32x4 a = reinterpret_cast<const u32x4 *>(h)[idx], b = reinterpret_cast<const u32x4 *>(o)[idx];
    u32x4 r;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        r[j] = pack_bf16x2(__uint_as_float(a[j] << 16) + __uint_as_float(b[j] << 16),
                           __uint_as_float(a[j] & 0xFFFF0000u) + __uint_as_float(b[j] & 0xFFFF0000u));
    reinterpret_cast<u32x4 *>(out)[idx] = r;
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct FfnLayout {
    size_t gu, act, h0, h1, o, total;
};
inline FfnLayout ffn_layout(int64_t B, int64_t F, int64_t d) {
    FfnLayout l;
    size_t off = 0;
    l.gu = off, off += align256((size_t)B * 2 * F * 2);
    l.act = off, off += align256((size_t)B * F * 2);
    l.h0 = off, off += align256((size_t)B * d * 2);
    l.h1 = off, off += align256((size_t)B * d * 2);
    l.o = off, off += align256((size_t)B * d * 2);
    l.total = off;
    return l;
}

}  // namespace

size_t ffn_workspace_bytes(int64_t B, int64_t F, int64_t d) {
    if (B < 1 || B > 16 || F < 1 || d < 1) return 0;
    return ffn_layout(B, F, d).total + 256;
}

}  // namespace mq

extern "C" mq_status mq_ffn_mixnmatch(const uint16_t *x, const mq_ffn_layer *layers, int n_layers, int64_t B, int64_t d,
                                      int64_t F, uint32_t flags, uint16_t *y, void *ws, size_t ws_bytes,
                                      void *hip_stream) {
    using namespace mq;
    if (n_layers < 0 || B < 1 || B > 16 || d < 1 || F < 1 || d > 0x3FFFFFF0 || F > 0x3FFFFFF0) return MQ_ERR_SHAPE;
    if (F % 8 != 0 || d % 8 != 0) return MQ_ERR_ALIGN;
    if (!x || !y || (n_layers > 0 && !layers)) return MQ_ERR_NULL;
    if (x == y) return MQ_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(y)) return MQ_ERR_ALIGN;
    for (int l = 0; l < n_layers; ++l) {
        const mq_ffn_layer &L = layers[l];
        if (L.r != 8 && L.r != 6 && L.r != 4 && L.r != 3 && L.r != 2) return MQ_ERR_BITS;
        if (!L.gate_up || !L.down || !L.alpha_gu || !L.zero_gu || !L.alpha_dn || !L.zero_dn) return MQ_ERR_NULL;
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (n_layers == 0) {
        if (hipMemcpyAsync(y, x, (size_t)B * d * 2, hipMemcpyDeviceToDevice, st) != hipSuccess) return MQ_ERR_DEVICE;
        return MQ_OK;
    }
    const FfnLayout lay = ffn_layout(B, F, d);
    if (!ws || ws_bytes < lay.total + 256) return MQ_ERR_WORKSPACE;
    uint8_t *base = reinterpret_cast<uint8_t *>((reinterpret_cast<uintptr_t>(ws) + 255) & ~(uintptr_t)255);
    uint16_t *gu = reinterpret_cast<uint16_t *>(base + lay.gu), *act = reinterpret_cast<uint16_t *>(base + lay.act);
    uint16_t *hbuf[2] = {reinterpret_cast<uint16_t *>(base + lay.h0), reinterpret_cast<uint16_t *>(base + lay.h1)};
    uint16_t *obuf = reinterpret_cast<uint16_t *>(base + lay.o);
    const bool residual = (flags & MQ_FLAG_FFN_RESIDUAL) != 0, use_silu = (flags & MQ_FLAG_FFN_SILU) != 0;

    const uint16_t *h = x;
    for (int l = 0; l < n_layers; ++l) {
        const mq_ffn_layer &L = layers[l];
        const bool last = l + 1 == n_layers;
        uint16_t *hn = last ? y : hbuf[l & 1];  // (never the buffer h lives in)
        mq_status s = mq_gemv_sliced(h, L.gate_up, L.alpha_gu, L.zero_gu, nullptr, B, 2 * F, d, L.r, gu, hip_stream);
        if (s != MQ_OK) return s;
        const int n_act = (int)(B * (F >> 3));
        if (use_silu)
            gate_kernel<true><<<dim3((n_act + 255) / 256), dim3(256), 0, st>>>(gu, act, (int)B, (int)F);
        else
            gate_kernel<false><<<dim3((n_act + 255) / 256), dim3(256), 0, st>>>(gu, act, (int)B, (int)F);
        if ((s = launch_status()) != MQ_OK) return s;
        s = mq_gemv_sliced(act, L.down, L.alpha_dn, L.zero_dn, nullptr, B, d, F, L.r, residual ? obuf : hn, hip_stream);
        if (s != MQ_OK) return s;
        if (residual) {
            const int n8 = (int)(B * d / 8);
            residual_kernel<<<dim3((n8 + 255) / 256), dim3(256), 0, st>>>(h, obuf, hn, n8);
            if ((s = launch_status()) != MQ_OK) return s;
        }
        h = hn;
    }
    return MQ_OK;
}
