// Internal interface between the two decode-GEMV kernels (not part of the public ABI).
#pragma once

#include "mq_common.h"

namespace mq {

struct GemvArgs {
    const uint16_t *x;        // [B, K] bf16
    const uint8_t *packed;    // [N, KB]
    const uint16_t *alpha;    // [N] bf16
    const uint16_t *zero;     // [N] bf16
    const int32_t *row_ptr;   // [N + 1] or null
    const uint16_t *col_idx;  // overflow columns
    uint16_t *y;              // [B, N] bf16
    int B, N, K;
    int KB;       // bytes per packed row
    float scale;  // 2^s: one step of the stored codes on the int8 grid
};

// Small-batch kernel (B <= 4, r = 4 or 2, no overflow list): activations live in registers.
// Returns MQ_OK with *handled = false when the shape is outside what it covers.
mq_status launch_gemv_quad(const GemvArgs &a, int r, hipStream_t st, bool *handled);

}  // namespace mq
