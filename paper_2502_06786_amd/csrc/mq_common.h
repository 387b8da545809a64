// Shared host/device helpers of the gfx950 kernels (not part of the public ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mq.h"

namespace mq {

typedef uint32_t u32;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

union Frag8 {  // eight bf16 = one MFMA operand register quad
    u32x4 u;
    bf16x8 b;
};

__device__ __forceinline__ float bf16_bits_to_float(uint32_t h) { return __uint_as_float(h << 16); }

// fp32 -> bf16, round to nearest even, two at a time: gfx950 converts a pair in one instruction
// (v_cvt_pk_bf16_f32), which the compiler selects for this vector conversion.
typedef __bf16 bf16pair_t __attribute__((ext_vector_type(2)));
typedef float f32pair_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32pair_t{lo, hi}, bf16pair_t));
}

__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) { return pack_bf16x2(f, 0.0f) & 0xFFFFu; }
// the two bf16 values of a 32-bit word
__device__ __forceinline__ float bf16_lo(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t v) { return __uint_as_float(v & 0xFFFF0000u); }

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline mq_status launch_status() { return hipGetLastError() == hipSuccess ? MQ_OK : MQ_ERR_DEVICE; }

inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// workspace of mq_ffn_mixnmatch (mq_ffn.hip)
size_t ffn_workspace_bytes(int64_t B, int64_t F, int64_t d);
// workspace of mq_matquant_l2_loss (mq_loss.hip)
size_t loss_workspace_bytes(int64_t M, int64_t N);
// workspace of mq_linear_bwd_clip (mq_clip.hip)
size_t clip_workspace_bytes(int64_t M, int64_t N, int64_t K);
// workspace of mq_affine_bwd (mq_affine.hip)
size_t affine_workspace_bytes(int64_t M, int64_t N, int64_t K);
// losses[i] = inv_mn * sum over the workgroups of partial[workgroup][i] (rows of 4 floats), in a
// fixed order; one small launch on `st` (mq_loss.hip)
mq_status launch_loss_finish(const float *partial, int64_t blocks, int nr, float inv_mn, float *losses,
                             hipStream_t st);

// Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  This maps the hardware
// id to a logical id such that each XCD owns one contiguous range of logical ids, so that tiles
// which share operands are co-resident under one L2.
__device__ __forceinline__ uint32_t xcd_contiguous_id(uint32_t hw_id, uint32_t count) {
    const uint32_t xcd = hw_id & 7u, slot = hw_id >> 3;
    const uint32_t per = count >> 3, extra = count & 7u;
    return xcd * per + (xcd < extra ? xcd : extra) + slot;
}

}  // namespace mq
