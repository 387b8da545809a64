/*
 * mq.h - C ABI of the MI355X (gfx950) nested quantized linear layer of
 * Matryoshka Quantization (arXiv 2502.06786).
 *
 * One int8 code per weight, one (alpha, z) pair per output channel; every lower
 * bit-width r is read out of the same int8 code with the paper's slicing
 * operator and shares alpha and z.  The five operations below are the whole
 * hot path: quantize, slice (+pack), fused multi-precision forward, the
 * straight-through backward used in co-training, and the weight-only decode
 * GEMV.
 *
 * Conventions
 *   - Weight W[N][K] row-major: N output channels, K input features.  M tokens.
 *   - s = 8 - r, half = 2^(s-1) (0 for r = 8).
 *   - bf16 tensors are passed as uint16_t bit patterns.
 *   - EVERY pointer is a DEVICE pointer unless its comment says "host".
 *   - The caller owns every buffer.  The library allocates nothing, frees
 *     nothing and never synchronises: all work is enqueued on `hip_stream`
 *     (a hipStream_t passed as void*, NULL = the default stream).  Scratch
 *     memory comes from a caller-provided workspace sized by
 *     mq_workspace_bytes().
 *   - Errors are return codes; arguments are checked on the host before any
 *     launch and nothing is enqueued when a call fails.  After a failure no
 *     output is defined.
 *   - Device pointers must be 16-byte aligned and all matrices are dense
 *     (row stride = row length) except W, which has `ldw`.
 *   - Reentrant: no mutable global state.  Two calls may run concurrently on
 *     different streams when their buffers (workspace included) do not overlap.
 */
#ifndef MQ_H
#define MQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MQ_OK = 0,
    MQ_ERR_NULL = 1,      /* a required pointer is NULL                                    */
    MQ_ERR_SHAPE = 2,     /* negative size, size beyond a documented limit                 */
    MQ_ERR_BITS = 3,      /* r outside the accepted set, duplicate r, nr out of range      */
    MQ_ERR_ALIGN = 4,     /* pointer not 16-byte aligned or a row length not a legal multiple */
    MQ_ERR_WORKSPACE = 5, /* workspace NULL or smaller than mq_workspace_bytes()           */
    MQ_ERR_CAPACITY = 6,  /* mq_overflow.capacity negative.  A capacity that turns out too
                             small is not an error of the call: see mq_overflow.nnz          */
    MQ_ERR_DEVICE = 7     /* a HIP call failed (launch error)                              */
} mq_status;

enum {
    MQ_FLAG_EXTRA_PRECISION = 1, /* errata section: slice without the clamp (2^r + 1 levels) */
    MQ_FLAG_PACKED = 2,          /* mq_slice: write 8/r codes per byte instead of one        */
    MQ_FLAG_ACCUM_DW = 4,        /* mq_linear_bwd: dW += instead of dW =                     */
    MQ_FLAG_EP_DENSE = 8         /* mq_slice, with the two flags above: one plane of r + 1 bits
                                    per code that keeps code 2^r, instead of plane + list     */
};

enum { MQ_OP_LINEAR_FWD = 0, MQ_OP_LINEAR_BWD = 1, MQ_OP_FFN_DECODE = 2, MQ_OP_L2_LOSS = 3, MQ_OP_LINEAR_FWD_L2 = 4,
       MQ_OP_LINEAR_BWD_CLIP = 5, MQ_OP_AFFINE_BWD = 6, MQ_OP_GEMV = 7 };

/*
 * Extra-precision overflow set (errata section: weights whose rounded r-bit
 * code equals 2^r need "an extra bit").  The paper gives no storage format;
 * this one is CSR over output channels: the columns k of row n with
 * q[n,k] >= 256 - half, ascending, are col_idx[row_ptr[n] .. row_ptr[n+1]).
 * K <= 65536 so a column fits uint16_t.
 */
typedef struct {
    int32_t *row_ptr;  /* device [N+1]                                                    */
    uint16_t *col_idx; /* device [capacity]                                               */
    int64_t capacity;  /* in: number of entries col_idx can hold                          */
    int64_t *nnz;      /* device scalar, out: total size of the set.  If it exceeds
                          `capacity`, col_idx holds only the first `capacity` entries in
                          row order and row_ptr still describes the full set; the caller
                          checks after the stream has completed.  mq_gemv_sliced given
                          such a list uses exactly the entries that were stored (list
                          positions >= capacity are dropped, nothing past col_idx is
                          read).                                                          */
} mq_overflow;

/*
 * MinMax quantizer to c = 8 bits, one (alpha, z) per output channel
 * (section 3.1.1, MinMax equation; with gamma/beta the OmniQuant form of
 * section 3.1.2):
 *     hi = gamma_n * max_k W[n,k]     lo = beta_n * min_k W[n,k]
 *     alpha_n = (hi - lo) / 255       z_n = -lo / alpha_n
 *     Q[n,k]  = clamp(round(W[n,k] / alpha_n + z_n), 0, 255)
 * fp32 throughout, one IEEE operation per symbol in that order (division is
 * correctly rounded, the add is not fused), round = half-to-even.  A row with
 * hi == lo takes alpha = 1, z = -lo (all codes 0).  W must be finite.
 *   W      [N, ldw] fp32, ldw >= K
 *   gamma  [N] fp32 or NULL (= 1)      beta [N] fp32 or NULL (= 1)
 *   Q      [N, K] uint8 out            alpha, zero [N] fp32 out
 * K >= 1 when N > 0.  N == 0 is a no-op.
 */
mq_status mq_quantize_int8(const float *W, int64_t N, int64_t K, int64_t ldw,
                           const float *gamma, const float *beta,
                           uint8_t *Q, float *alpha, float *zero, void *hip_stream);

/*
 * Per-channel scale and zero-point rounded to bf16 (nearest even) for the decode path, which keeps
 * them in bf16 next to the packed low-bit plane.  alpha, zero [N] fp32 -> alpha_bf16, zero_bf16 [N].
 * (The paper fixes no storage type for them; the decode GEMV consumes exactly these arrays.)
 */
mq_status mq_params_to_bf16(const float *alpha, const float *zero, int64_t N, uint16_t *alpha_bf16,
                            uint16_t *zero_bf16, void *hip_stream);

/*
 * Slicing operator S(q, r) of section 3.2 (slicing equation; appendix A for
 * the rounding):  code = min((q + half) >> s, 2^r - 1), S = code << s.
 *   Q    [N, K] uint8
 *   r    1..8 (r = 8 is the identity)
 *   out  without MQ_FLAG_PACKED: [N, K] uint8, the codes (NOT shifted back up);
 *        with MQ_FLAG_PACKED (r in {8, 6, 4, 3, 2}, K*r a multiple of 8):
 *        [N, K*r/8] bytes, each row a little-endian bit stream of r bits per
 *        code: code k at stream bits [r*k, r*k + r), stream bit t = bit t mod 8
 *        of byte t / 8 (for r in {8, 4, 2}: element k in byte k/(8/r) at bit
 *        offset r * (k mod 8/r); r = 6 and r = 3, the interpolated bit-widths
 *        of section 4.2, put 4 resp. 8 codes into 3 bytes).  The packing order
 *        is this library's definition.
 *   ovf  required iff MQ_FLAG_EXTRA_PRECISION (errata section): the dense plane
 *        written to `out` is the clamped one (bit-identical to the plain
 *        slice) and the weights whose unclamped code is 2^r are listed in *ovf.
 *        `ovf` itself is a host struct holding device pointers.  Needs K <= 65536.
 *        With MQ_FLAG_EP_DENSE as well (and MQ_FLAG_PACKED): no list; `out` is
 *        [N, K*(r+1)/8], the same bit-stream format with r + 1 bits per code,
 *        holding the unclamped codes 0 .. 2^r (r + 1 in {2, 3, 4, 6, 8}); this is
 *        the layout of choice where the overflow bucket is dense (about 5 % of
 *        the weights at r = 2 in the paper's Table 7) and ovf may be NULL.
 */
mq_status mq_slice(const uint8_t *Q, int64_t N, int64_t K, int r, uint32_t flags,
                   uint8_t *out, const mq_overflow *ovf, void *hip_stream);

/*
 * Several packed planes of the same codes in one call (the nested model of section 3.2 is served at several
 * bit-widths from one set of int8 codes): out[i] = the packed rs[i]-bit plane exactly as mq_slice with
 * MQ_FLAG_PACKED writes it.  The int4 and int2 planes and the sizes of the overflow set are produced by a single
 * pass over Q (rows that are whole 16-byte chunks), so slicing a layer for decode reads the codes twice (planes
 * and counts, then the columns of the list) instead of once per kernel of every plane.
 *   rs         host int[nr], distinct values out of {8, 6, 4, 3, 2}; nr in 1..3
 *   out        host array of nr device pointers, out[i] [N, K*rs[i]/8]
 *   flags      0, or MQ_FLAG_EXTRA_PRECISION: the overflow set of bit-width rs[ovf_index] is also listed in *ovf
 *              (every plane is the clamped one); MQ_FLAG_EP_DENSE is not accepted here
 *   ovf_index  index into rs (ignored without MQ_FLAG_EXTRA_PRECISION; pass -1)
 * Status codes and limits as for mq_slice.
 */
mq_status mq_slice_multi(const uint8_t *Q, int64_t N, int64_t K, const int *rs, int nr, uint32_t flags,
                         uint8_t *const *out, int ovf_index, const mq_overflow *ovf, void *hip_stream);

/*
 * Fused multi-precision forward, the F(S(Q(theta, c), r), x) of the MatQuant
 * objective (section 3.2) for every r in rs[] in ONE pass over X and Q:
 *     Y_i[m,n] = sum_k X[m,k] * alpha_n * (S(Q[n,k], rs[i]) - z_n)
 * bf16 x bf16 -> fp32 matrix-core accumulation, rounded once to bf16.
 *   X      [M, K] bf16               Q [N, K] uint8        alpha, zero [N] fp32
 *   rs     host int[nr], distinct values in 1..8; nr in 1..3
 *   flags  MQ_FLAG_EXTRA_PRECISION: slices use the unclamped code
 *   Y      host array of nr device pointers, each [M, N] bf16 out
 *   ws     workspace of at least mq_workspace_bytes(MQ_OP_LINEAR_FWD, M, N, K, nr)
 * K must be a multiple of 16 and N a multiple of 8 (16-byte rows).  M is free.
 * M == 0 or N == 0 is a no-op.  Limits (MQ_ERR_SHAPE beyond): M, N below 2^31 - 256,
 * K <= 2^22, ceil(M / 128) * ceil(N / 128) below 2^31.
 */
mq_status mq_linear_fwd_multi(const uint16_t *X, const uint8_t *Q, const float *alpha,
                              const float *zero, int64_t M, int64_t N, int64_t K,
                              const int *rs, int nr, uint32_t flags,
                              uint16_t *const *Y, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * mq_linear_fwd_multi for callers that cannot allocate or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and limits
 * as mq_linear_fwd_multi without `ws`; the per-token sums of X that the forward keeps between its
 * pre-pass and its epilogue live in a fixed device array inside the library (1 MiB, one copy per GPU,
 * held until the process ends).  No hipMalloc, hipFree or other allocating call is made.
 *   - M <= 262144 tokens (MQ_ERR_SHAPE beyond: the built-in scratch holds one float per token).
 *   - Every call on one GPU uses that GPU's array: calls that overlap in time on the same GPU (two
 *     streams, two host threads) race and must be serialised by the caller.  Calls on different GPUs
 *     are independent.  Nothing is kept between calls.
 *   - The device address of the array is looked up once per GPU at the first call made with that GPU
 *     current; make that first call outside a graph capture.
 */
mq_status mq_linear_fwd_multi_noalloc(const uint16_t *X, const uint8_t *Q, const float *alpha,
                                      const float *zero, int64_t M, int64_t N, int64_t K,
                                      const int *rs, int nr, uint32_t flags,
                                      uint16_t *const *Y, void *hip_stream);

/*
 * Straight-through backward of the same layer (sections 3.1.1 / 3.1.2 use an
 * STE through the quantizer; identity through both rounds and both clamps,
 * alpha and z held constant) for the weighted sum of per-bit-width losses of
 * the MatQuant objective (section 3.2):
 *     dX[m,k] = sum_i lambda_i sum_n dY_i[m,n] * alpha_n * (S(Q[n,k], rs[i]) - z_n)
 *     dW[n,k] = sum_m (sum_i lambda_i dY_i[m,n]) * X[m,k]
 *   dY      host array of nr device pointers, each [M, N] bf16
 *   lambda  host float[nr] or NULL (= 1)
 *   dX      [M, K] bf16 out, or NULL to skip
 *   dW      [N, K] fp32 out (accumulated into with MQ_FLAG_ACCUM_DW), or NULL to skip
 *   ws      workspace of at least mq_workspace_bytes(MQ_OP_LINEAR_BWD, M, N, K, nr)
 * K must be a multiple of 16 and N a multiple of 16.  M is free.
 * M == 0: dW (a sum over no tokens) is set to zero unless MQ_FLAG_ACCUM_DW; N == 0: dX is set to zero.
 * The bf16 rounding of lambda_i * alpha_n * dY_i (dX) and of
 * sum_i lambda_i dY_i (dW) before the matrix-core contraction is part of the
 * stated tolerance.
 */
mq_status mq_linear_bwd(const uint16_t *X, const uint8_t *Q, const float *alpha, const float *zero,
                        const uint16_t *const *dY, const float *lambda,
                        int64_t M, int64_t N, int64_t K, const int *rs, int nr, uint32_t flags,
                        uint16_t *dX, float *dW, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Weight-only decode GEMV on a packed r-bit plane (section 1: decode is bound
 * by moving the weights out of HBM; the errata section asks for sparse
 * additions of the extra bits):
 *     y[b,n] = alpha_n * (2^s * (sum_k code[n,k] x[b,k] + sum_{k in O_n} x[b,k])
 *                         - z_n * sum_k x[b,k])
 *   x       [B, K] bf16, 1 <= B <= 16
 *   packed  [N, K*r/8] as written by mq_slice with MQ_FLAG_PACKED, r in {8, 6, 4, 3, 2}
 *   alpha_bf16, zero_bf16  [N] bf16
 *   ovf     host struct or NULL (= plain slice); row_ptr/col_idx as written by mq_slice, capacity =
 *           entries col_idx holds (list positions beyond it are ignored; negative: MQ_ERR_CAPACITY);
 *           nnz is not read
 *   y       [B, N] bf16 out
 * A packed row must be a whole number of 16-byte units (K*r a multiple of 128 bits; for
 * r = 6 and r = 3 of 12-byte units, K*r a multiple of 96 bits; else MQ_ERR_ALIGN); B*K <= 2^29 and, with an overflow list, K <= 65536 (else MQ_ERR_SHAPE).
 * N == 0 is a no-op.
 */
mq_status mq_gemv_sliced(const uint16_t *x, const uint8_t *packed, const uint16_t *alpha_bf16,
                         const uint16_t *zero_bf16, const mq_overflow *ovf,
                         int64_t B, int64_t N, int64_t K, int r, uint16_t *y, void *hip_stream);

/*
 * mq_gemv_sliced for callers that can lend scratch memory (section 1: the decode GEMV moves the weights out of
 * HBM once; with few rows and a long K, e.g. the down projection at B = 16, one workgroup per row block leaves
 * most of the chip idle, so K is also split over workgroups and a second kernel adds the parts in a fixed order).
 * Same arguments, result to the same tolerance (the order of the fp32 additions differs), plus
 *   ws      device, 16-byte aligned, at least mq_workspace_bytes(MQ_OP_GEMV, B, N, K, r) bytes (else
 *           MQ_ERR_WORKSPACE); contents undefined on entry and exit; calls that share it must not overlap
 * Shapes the split form is not used for (B <= 4, r not in {4, 2}, packed rows that are not whole 128-byte lines or
 * shorter than 1664 bytes, more than 8192 rows) run exactly as mq_gemv_sliced does and leave ws untouched.
 */
mq_status mq_gemv_sliced_ws(const uint16_t *x, const uint8_t *packed, const uint16_t *alpha_bf16,
                            const uint16_t *zero_bf16, const mq_overflow *ovf,
                            int64_t B, int64_t N, int64_t K, int r, uint16_t *y,
                            void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The same GEMV on a dense extra-precision plane (mq_slice with MQ_FLAG_EXTRA_PRECISION |
 * MQ_FLAG_PACKED | MQ_FLAG_EP_DENSE): codes 0 .. 2^r stored with r + 1 bits, one code step
 * still 2^(8-r) (errata section: int2 with the extra bucket has the levels 0, 64, 128, 192, 256).
 *   packed  [N, K*(r+1)/8], r + 1 in {2, 3, 4, 6, 8}; alignment as for a plain (r+1)-bit plane
 */
mq_status mq_gemv_sliced_dense_ep(const uint16_t *x, const uint8_t *packed, const uint16_t *alpha_bf16,
                                  const uint16_t *zero_bf16, int64_t B, int64_t N, int64_t K, int r,
                                  uint16_t *y, void *hip_stream);

/*
 * The MatQuant objective with the layer-wise L2 reconstruction loss (section 3.2, joint objective over
 * the bit-widths, with the loss of section 3.1.2: the output of the quantized layer against the output
 * y' of the full-precision layer), and its co-distillation variants (section 5.2: the output of a
 * higher-precision slice as the target of a lower one, alone or next to y' with equal weights):
 *     loss_i   = 1/(M N) * sum_{m,n} (Y_i - T_i)^2        T_i = target (teacher[i] < 0) or Y_teacher[i]
 *     loss_i   = 1/2 of each of the two when teacher[i] >= 0 and MQ_FLAG_LOSS_MIX
 *     total    = sum_i lambda_i loss_i
 *     dY_i     = d total / d Y_i with the teachers held constant (stop-gradient)
 *              = lambda_i * 2 (Y_i - T_i) / (M N)         (the mean of the two differences when mixed)
 *   Y        host array of nr device pointers, each [M, N] bf16 (the outputs of mq_linear_fwd_multi)
 *   target   [M, N] bf16, y'; may be NULL when every i has a teacher and MQ_FLAG_LOSS_MIX is not set
 *   teacher  host int[nr] or NULL (= all -1); teacher[i] in -1 .. nr-1, teacher[i] != i
 *   lambda   host float[nr] or NULL (= 1)
 *   dY       host array of nr device pointers, each [M, N] bf16 out: what mq_linear_bwd takes
 *   losses   device float[nr] out: loss_i (unweighted)
 *   ws       workspace of at least mq_workspace_bytes(MQ_OP_L2_LOSS, M, N, 0, nr)
 * M * N must be a multiple of 8; 1 <= nr <= 3.  M * N == 0 is a no-op.
 */
enum { MQ_FLAG_LOSS_MIX = 64 };
mq_status mq_matquant_l2_loss(const uint16_t *const *Y, const uint16_t *target, const int *teacher,
                              const float *lambda, int64_t M, int64_t N, int nr, uint32_t flags,
                              uint16_t *const *dY, float *losses, void *ws, size_t ws_bytes,
                              void *hip_stream);

/*
 * mq_linear_fwd_multi and mq_matquant_l2_loss in one pass: the training step of section 3.2 needs
 * the outputs Y_i only to form the loss and its gradients, so the objective is evaluated on the
 * rounded bf16 outputs while a tile is still on chip, and the Y_i need not travel to memory and
 * back.  Per element the arithmetic is that of the two calls in sequence: the dY_i are bit-identical
 * to theirs, the losses agree up to the order of the fp32 partial sums.
 *   X, Q, alpha, zero, M, N, K, rs, nr   as for mq_linear_fwd_multi
 *   target, teacher, lambda, dY, losses  as for mq_matquant_l2_loss (indices in the order of rs)
 *   flags    MQ_FLAG_EXTRA_PRECISION and / or MQ_FLAG_LOSS_MIX
 *   bias     [N] fp32 or NULL: added to every output before it is rounded to bf16 (the bias of the
 *            layer; with the affine re-parameterisation of section 3.1.2 the vector c of mq_affine_weight)
 *   Y        NULL, or a host array of nr device pointers of which any may be NULL: an output
 *            whose pointer is NULL is not stored
 *   ws       workspace of at least mq_workspace_bytes(MQ_OP_LINEAR_FWD_L2, M, N, K, nr)
 * Alignment and size limits as for mq_linear_fwd_multi.  M == 0 or N == 0 is a no-op.
 */
mq_status mq_linear_fwd_multi_l2(const uint16_t *X, const uint8_t *Q, const float *alpha,
                                 const float *zero, int64_t M, int64_t N, int64_t K,
                                 const int *rs, int nr, uint32_t flags, const float *bias,
                                 const uint16_t *target, const int *teacher, const float *lambda,
                                 uint16_t *const *Y, uint16_t *const *dY, float *losses,
                                 void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Gradients of the MatQuant objective with respect to the clip factors gamma, beta that the
 * quantizer takes (section 3.1.2: alpha = (gamma max - beta min) / 255, z = -beta min / alpha; these
 * are the parameters that the OmniQuant base algorithm trains through the layer-wise L2 loss), for
 * the gradients dY_r of mq_matquant_l2_loss / mq_linear_fwd_multi_l2:
 *     dgamma_n = sum_r lambda_r sum_{m,k} dY_r[m,n] X[m,k] * d What_r[n,k] / d gamma_n   (dbeta alike)
 * under the straight-through estimator the section names, read as: the rounding to the 8-bit code
 * and the rounding inside the slicing operator pass the gradient unchanged; the clamp to 0..255 and
 * the clamp of a slice to its top code 2^r - 1 (absent with MQ_FLAG_EXTRA_PRECISION) pass it only
 * where they do not act.  With u = w / alpha + z and What_r = alpha (S(q, r) - z):
 *     d What_r / d alpha = (S(q, r) - z) - m_r w / alpha         d What_r / d z = -alpha (1 - m_r)
 * (m_r = 1 where neither clamp acts), chained through alpha(gamma, beta), z(beta, alpha).  A row with
 * gamma max == beta min (alpha set to 1 by the quantizer) gets zero gradients.
 *   W        [N, ldw] fp32 master weights, ldw a multiple of 4
 *   X        [M, K] bf16           Q [N, K] uint8, alpha, zero [N] fp32 as mq_quantize_int8 wrote them
 *   gamma, beta  [N] fp32 or NULL (= 1): what the quantizer was called with
 *   dY, lambda, rs, nr  as for mq_linear_bwd
 *   dgamma, dbeta  [N] fp32 out;  dalpha, dzero  [N] fp32 out or NULL (the gradients with respect to
 *            alpha and z, before the chain rule)
 *   ws       workspace of at least mq_workspace_bytes(MQ_OP_LINEAR_BWD_CLIP, M, N, K, nr)
 * Alignment and size limits as for mq_linear_bwd.  N == 0 is a no-op; M == 0 writes zeros.
 */
mq_status mq_linear_bwd_clip(const float *W, int64_t ldw, const uint16_t *X, const uint8_t *Q,
                             const float *alpha, const float *zero, const float *gamma, const float *beta,
                             const uint16_t *const *dY, const float *lambda,
                             int64_t M, int64_t N, int64_t K, const int *rs, int nr, uint32_t flags,
                             float *dgamma, float *dbeta, float *dalpha, float *dzero,
                             void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Learnable affine re-parameterisation of a projection (section 3.1.2, the second OmniQuant equation):
 *     X W + b  ->  ((X - delta) / s) Q(W * s) + b + delta W
 * with W stored [N, K] (output channels x input features), s and delta per input feature.  Three
 * bandwidth-bound operations around the quantized layer; the layer itself is mq_quantize_int8 on Ws,
 * mq_linear_fwd_multi_l2 on Xt with bias c, mq_linear_bwd (and mq_linear_bwd_clip) on Xt.
 *
 * mq_affine_weight:  Ws[n,k] = W[n,k] * s[k] (one fp32 product: the quantizer's input, bit for bit)
 *                    c[n]    = b[n] + sum_k W[n,k] delta[k]
 *   W [N, ldw] fp32;  s, delta [K] fp32 or NULL (= 1, = 0);  b [N] fp32 or NULL (= 0)
 *   Ws [N, K] fp32 out or NULL;  c [N] fp32 out or NULL (at least one of the two)
 *   K and ldw multiples of 4.
 * mq_affine_input:   Xt[m,k] = bf16((X[m,k] - delta[k]) / s[k]);  X, Xt [M, K] bf16, K a multiple of 8
 *                    (s and delta 16-byte aligned like every other pointer; M K below 2^42 elements,
 *                    MQ_ERR_SHAPE beyond)
 * mq_affine_bwd:     with dXt = d objective / d Xt (the dX of mq_linear_bwd), dWs = d objective / d Ws
 *                    (its dW: the straight-through estimator is the identity through the quantizer) and
 *                    dc[n] = sum_r lambda_r sum_m dY_r[m,n]:
 *                      ddelta[k] = -(1/s[k]) sum_m dXt[m,k] + sum_n dc[n] W[n,k]
 *                      ds[k]     = -(1/s[k]^2) sum_m dXt[m,k] (X[m,k] - delta[k]) + sum_n dWs[n,k] W[n,k]
 *                    (the range of the quantizer follows s through max and min of Ws without a gradient,
 *                    as in mq_linear_bwd_clip)
 *   X, dXt [M, K] bf16;  W [N, ldw] fp32;  dWs [N, K] fp32;  dY, lambda, nr as for mq_linear_bwd
 *   ddelta, ds [K] fp32 out, dc [N] fp32 out; any may be NULL (not all)
 *   ws       workspace of at least mq_workspace_bytes(MQ_OP_AFFINE_BWD, M, N, K, nr)
 *   M, N, K >= 1; N, K, ldw multiples of 4.
 */
mq_status mq_affine_weight(const float *W, int64_t N, int64_t K, int64_t ldw, const float *s,
                           const float *delta, const float *b, float *Ws, float *c, void *hip_stream);
mq_status mq_affine_input(const uint16_t *X, int64_t M, int64_t K, const float *s, const float *delta,
                          uint16_t *Xt, void *hip_stream);
mq_status mq_affine_bwd(const uint16_t *X, const uint16_t *dXt, const float *W, int64_t ldw,
                        const float *dWs, const uint16_t *const *dY, const float *lambda, int nr,
                        int64_t M, int64_t N, int64_t K, const float *s, const float *delta,
                        float *ddelta, float *ds, float *dc, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Layer-wise Mix'n'Match on the decode path (section 4.3 "Mix'n'Match", section 5.1.3 and appendix B:
 * every feed-forward layer of the stack is served at its own bit-width, e.g. int2 in the first and
 * last layers and int8 in the middle, "Pyramid"): a stack of gated feed-forward layers, each reading
 * the r_l-bit planes sliced from its own 8-bit codes,
 *     h_0 = x;   g, u = W_gate h_l, W_up h_l;   a = act(g) * u;   o = W_down a;
 *     h_(l+1) = o   (or h_l + o with MQ_FLAG_FFN_RESIDUAL);          y = h_L
 * with every matrix-vector product computed as mq_gemv_sliced does and every intermediate (g, u, a, o,
 * h) rounded to bf16.  The paper does not write the block out; Gemma-2 uses act = GELU (tanh form),
 * the default here, Mistral SiLU (MQ_FLAG_FFN_SILU).
 *   x        [B, d] bf16, 1 <= B <= 16
 *   layers   HOST array of n_layers descriptors; all pointers in them are device pointers:
 *              gate_up   packed plane [2F, d*r/8] of the gate and the up rows, interleaved: row 2 f is
 *                        gate row f, row 2 f + 1 is up row f (the two products of a pair then meet in
 *                        one thread's epilogue; this order is this library's definition)
 *              down      packed plane [d, F*r/8]
 *              alpha_gu, zero_gu  bf16 [2F], in the row order of gate_up;  alpha_dn, zero_dn  bf16 [d]
 *              r         bits of this layer's planes: 8, 6, 4, 3 or 2
 *   y        [B, d] bf16 out (may not alias x)
 *   ws       workspace of at least mq_workspace_bytes(MQ_OP_FFN_DECODE, B, F, d, 1)
 * Alignment of the planes as for mq_gemv_sliced; F a multiple of 8.
 */
typedef struct {
    const uint8_t *gate_up;
    const uint8_t *down;
    const uint16_t *alpha_gu, *zero_gu;
    const uint16_t *alpha_dn, *zero_dn;
    int r;
} mq_ffn_layer;
enum { MQ_FLAG_FFN_SILU = 16, MQ_FLAG_FFN_RESIDUAL = 32 };
mq_status mq_ffn_mixnmatch(const uint16_t *x, const mq_ffn_layer *layers, int n_layers,
                           int64_t B, int64_t d, int64_t F, uint32_t flags, uint16_t *y,
                           void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The gate of the feed-forward block on the training path (the block of section 5 whose weights the
 * paper quantizes; section 3.1.2 optimizes the error of whole layers).  The gate and up projections are
 * one quantized linear layer over the stacked weight [2F, d] with the rows of a pair next to each other
 * (row 2 f = gate row f, row 2 f + 1 = up row f, as in mq_ffn_mixnmatch), so that one
 * mq_linear_fwd_multi call over the shared input yields GU_r [M, 2F] for every bit-width; then
 *     A_r[m, f]  = bf16(act(GU_r[m, 2f]) * GU_r[m, 2f+1])                     (mq_gated_unit_fwd)
 * feeds the down projection (one mq_linear_fwd_multi / _l2 call per bit-width, their inputs differ), and
 *     dGU_r[m, 2f]   = bf16(dA_r[m, f] * GU_r[m, 2f+1] * act'(GU_r[m, 2f]))
 *     dGU_r[m, 2f+1] = bf16(dA_r[m, f] * act(GU_r[m, 2f]))                   (mq_gated_unit_bwd)
 * takes the down projection's dX_r back to the stacked layer's mq_linear_bwd.  act = GELU in its tanh
 * form, or SiLU with MQ_FLAG_FFN_SILU.  All nr (1..3) tensors are processed in one launch.
 *   GU, dGU  host arrays of nr device pointers, each [M, 2F] bf16;  A, dA  each [M, F] bf16
 * F must be a multiple of 8.  M == 0 is a no-op.
 */
mq_status mq_gated_unit_fwd(const uint16_t *const *GU, int nr, int64_t M, int64_t F, uint32_t flags,
                            uint16_t *const *A, void *hip_stream);
mq_status mq_gated_unit_bwd(const uint16_t *const *GU, const uint16_t *const *dA, int nr, int64_t M,
                            int64_t F, uint32_t flags, uint16_t *const *dGU, void *hip_stream);

/*
 * mq_linear_fwd_multi of the stacked gate / up layer and mq_gated_unit_fwd in one call: the gated products are
 * formed from the rounded outputs while a tile is still on chip (the arithmetic of mq_gated_unit_fwd: the A_r are
 * bit-identical to the two calls in sequence), so the GU_r are not read back.
 *   X [M, K] bf16;  Q [2F, K] uint8, alpha, zero [2F] fp32 (rows (gate f, up f) pairs);  rs, nr as usual
 *   GU       NULL, or host array of nr device pointers, each [M, 2F] bf16 out or NULL (an output whose pointer
 *            is NULL is not stored; the backward of the block needs them)
 *   A        host array of nr device pointers, each [M, F] bf16 out
 *   flags    MQ_FLAG_EXTRA_PRECISION, MQ_FLAG_FFN_SILU (GELU-tanh otherwise)
 *   ws       workspace of at least mq_workspace_bytes(MQ_OP_LINEAR_FWD, M, 2F, K, nr)
 * K a multiple of 16, F a multiple of 4; A rows 8-byte aligned.
 */
mq_status mq_linear_fwd_multi_gated(const uint16_t *X, const uint8_t *Q, const float *alpha, const float *zero,
                                    int64_t M, int64_t F, int64_t K, const int *rs, int nr, uint32_t flags,
                                    uint16_t *const *GU, uint16_t *const *A, void *ws, size_t ws_bytes,
                                    void *hip_stream);

/*
 * mq_gated_unit_bwd and mq_linear_bwd of the stacked gate / up layer in one call: the gradients dGU_r of the
 * gated unit are formed (and rounded to bf16, exactly as mq_gated_unit_bwd writes them) inside the pass that
 * prepares the operands of the backward, so they never travel to memory and back (section 3.1 straight-through
 * backward of the layer; the block of section 5).  Results are bit-identical to the two calls in sequence.
 *   X        [M, K] bf16, the input of the stacked layer;  Q [2F, K] uint8, alpha, zero [2F] fp32
 *   GU       host array of nr device pointers, each [M, 2F] bf16: the outputs of the stacked layer per bit-width
 *   dA       host array of nr device pointers, each [M, F] bf16: the gradients of the gated products
 *   lambda, rs, nr, dX, dW, ws  as for mq_linear_bwd with N = 2F (workspace of MQ_OP_LINEAR_BWD at N = 2F)
 *   flags    MQ_FLAG_EXTRA_PRECISION, MQ_FLAG_ACCUM_DW, MQ_FLAG_FFN_SILU (GELU-tanh otherwise)
 * K a multiple of 16, F a multiple of 8 (2F of 16).
 */
mq_status mq_linear_bwd_gated(const uint16_t *X, const uint8_t *Q, const float *alpha, const float *zero,
                              const uint16_t *const *GU, const uint16_t *const *dA, const float *lambda,
                              int64_t M, int64_t F, int64_t K, const int *rs, int nr, uint32_t flags,
                              uint16_t *dX, float *dW, void *ws, size_t ws_bytes, void *hip_stream);

/* Bytes of workspace `op` needs at these sizes (0 on invalid arguments).  MQ_OP_FFN_DECODE: M = B, N = F, K = d.
 * MQ_OP_GEMV: M = B, nr = r (bits per code). */
size_t mq_workspace_bytes(int op, int64_t M, int64_t N, int64_t K, int nr);

/* Static, human-readable name of a status code. */
const char *mq_status_string(mq_status status);

#ifdef __cplusplus
}
#endif
#endif /* MQ_H */
