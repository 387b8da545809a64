// Internal interface between the two decode-GEMV kernels (not part of the public ABI).
#pragma once

#include "mq_common.h"

namespace mq {

struct GemvArgs {
    const uint16_t *x;        // [B, K] bf16
    const uint8_t *packed;    // [N, KB]
    const uint16_t *alpha;    // [N] bf16
    const uint16_t *zero;     // [N] bf16
    uint16_t *y;              // [B, N] bf16
    int add_y;                // != 0: y holds, packed by ovf_sum_pack, a per-output addend to the sum of code * x
                              // (the overflow sums of the extra-precision slice), read before y is overwritten
    int B, N, K;
    int KB;       // bytes per packed row
    float scale;  // 2^s: one step of the stored codes on the int8 grid
    // What the epilogue does with the product o[b, n] (rounded to bf16 first in every case):
    //   kPostNone      y[b, n] = o
    //   kPostResidual  y[b, n] = bf16(res[b, n] + o)
    //   kPostGelu/Silu rows come in (gate, up) pairs, gate at the even row:
    //                  y[b, n / 2] = bf16(act(o[b, n]) * o[b, n + 1]), y is [B, N / 2]
    int post;
    const uint16_t *res;  // [B, N] bf16, kPostResidual only
};

enum { kPostNone = 0, kPostResidual = 1, kPostGelu = 2, kPostSilu = 3 };

// 1 / (1 + exp(-t)) with the hardware exponential and reciprocal (about 1e-6 relative: far below the bf16 rounding
// that follows every use)
__device__ __forceinline__ float sigmoid_fast(float t) { return __frcp_rn(1.0f + __expf(-t)); }
__device__ __forceinline__ float gelu_tanh(float v) {
    // 0.5 v (1 + tanh(t)) = v sigmoid(2 t),  t = sqrt(2 / pi) (v + 0.044715 v^3)
    const float t = 0.7978845608028654f * (v + 0.044715f * v * v * v);
    return v * sigmoid_fast(2.0f * t);
}
__device__ __forceinline__ float silu(float v) { return v * sigmoid_fast(v); }
// derivative of the gate activation (GELU in its tanh form, or SiLU)
__device__ __forceinline__ float act_grad(float g, bool use_silu) {
    if (use_silu) {
        const float sig = sigmoid_fast(g);
        return sig * (1.0f + g * (1.0f - sig));
    }
    const float c = 0.7978845608028654f;
    const float th = 2.0f * sigmoid_fast(2.0f * c * (g + 0.044715f * g * g * g)) - 1.0f;  // tanh
    return 0.5f * (1.0f + th) + 0.5f * g * (1.0f - th * th) * c * (1.0f + 3.0f * 0.044715f * g * g);
}
// the two gradients of a (gate, up) pair of the gated unit a = act(g) u, rounded to bf16 as a pair (dg, du)
__device__ __forceinline__ uint32_t gated_pair_grad(float g, float u, float da, bool use_silu) {
    return pack_bf16x2(da * u * act_grad(g, use_silu), da * (use_silu ? silu(g) : gelu_tanh(g)));
}
__device__ __forceinline__ float bf16_rounded(float v) { return __uint_as_float(float_to_bf16_bits(v) << 16); }
// one gated output from the (gate, up) pair of products
__device__ __forceinline__ uint16_t gated_bf16(float gate, float up, int post) {
    const float g = bf16_rounded(gate), u = bf16_rounded(up);
    return (uint16_t)float_to_bf16_bits((post == kPostSilu ? silu(g) : gelu_tanh(g)) * u);
}
__device__ __forceinline__ uint16_t residual_bf16(uint16_t res, float o) {
    return (uint16_t)float_to_bf16_bits(__uint_as_float((uint32_t)res << 16) + bf16_rounded(o));
}

// The decode GEMV with an epilogue of the list above (the public mq_gemv_sliced is kPostNone).
mq_status gemv_sliced_post(const uint16_t *x, const uint8_t *packed, const uint16_t *alpha_bf16,
                           const uint16_t *zero_bf16, int64_t B, int64_t N, int64_t K, int r, uint16_t *y, int post,
                           const uint16_t *res, void *hip_stream, void *split_ws = nullptr, size_t split_ws_bytes = 0);

// The host-side checks of such a call that do not involve x or y (callers that enqueue several
// GEMVs run them for every one before the first launch).
mq_status gemv_sliced_check(const uint8_t *packed, int64_t B, int64_t N, int64_t K, int r, int post);

// The overflow sums of the extra-precision GEMV travel from the kernel that forms them to the dense kernel's
// epilogue inside the output buffer y, 16 bits per output: IEEE half precision of sum / 256 (11 significant bits,
// sums up to 1.6e7 in magnitude, saturating beyond; an absolute step of 2^-16 for tiny sums).  Small integers,
// e.g. the sums of one-hot activations, pass exactly.
__device__ __forceinline__ uint16_t ovf_sum_pack(float sum) {
    const float scaled = fminf(fmaxf(sum * 0.00390625f, -65504.0f), 65504.0f);
    return __builtin_bit_cast(uint16_t, (_Float16)scaled);
}
__device__ __forceinline__ float ovf_sum_unpack(uint16_t bits) { return 256.0f * (float)__builtin_bit_cast(_Float16, bits); }

// y[b, n] <- ovf_sum_pack(sum of x[b, k] over the overflow columns k of row n) (mq_gemv_ovf.hip); K <= 65536
mq_status launch_overflow_sums(const uint16_t *x, const int32_t *row_ptr, const uint16_t *col_idx, int64_t capacity,
                               int64_t B, int64_t N, int64_t K, uint16_t *y, hipStream_t st);

// Small-batch kernel (B <= 4, r = 4 or 2): activations live in registers.
// Returns MQ_OK with *handled = false when the shape is outside what it covers.
mq_status launch_gemv_quad(const GemvArgs &a, int r, hipStream_t st, bool *handled);

// Batches of 5 .. 16 on tall int4 / int2 planes (no residual epilogue restriction): activations in registers as
// 16x16x32 matrix-core operands.  Same convention for *handled.
mq_status launch_gemv_reg(const GemvArgs &a, int r, hipStream_t st, bool *handled);

// The same kernel with K split over workgroups and a second kernel that adds the parts (any number of rows; for long
// rows and few of them).  ws: gemv_split_workspace_bytes() bytes of device memory (0 = shape not covered).
size_t gemv_split_workspace_bytes(int64_t B, int64_t N, int64_t K, int r);
mq_status launch_gemv_reg_split(const GemvArgs &a, int r, void *ws, size_t ws_bytes, hipStream_t st, bool *handled);

}  // namespace mq
