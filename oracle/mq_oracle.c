/*
 * CPU oracle for the Matryoshka-Quantization nested quantized linear layer
 * (arXiv 2502.06786).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, definition-level
 * reference the HIP kernels are checked against.  Nothing in the product path
 * may call it; it shares no code, header, table or helper with the HIP path.
 *
 * Every function takes HOST pointers.  Floating point is evaluated in fp64
 * except where the quantizer itself is defined in fp32 (section 3.1.1, MinMax
 * quantizer), where each operation is a single IEEE fp32 operation in the
 * order written below (compile with -ffp-contract=off, no fast-math).
 *
 * Conventions: weight W[N][K] row-major, N output channels, K input features,
 * one (alpha, z) pair per output channel.  c = 8 throughout.  bf16 tensors are
 * passed as raw uint16 bit patterns.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py
 * against values the paper prints, closed forms, brute force or a library
 * routine.  What the paper leaves open (packing order, overflow-list format,
 * identity STE) is this repository's definition and is "parity unpinned" by
 * the paper itself; see the notes beside each function.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double bf16_bits_to_f64(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* ------------------------------------------------------------------------
 * MinMax quantizer, section 3.1.1 (first equation), with the optional
 * OmniQuant clip factors of section 3.1.2 (gamma scales the max, beta the
 * min; NULL means 1).  Per output channel n:
 *     hi = gamma_n * max_k W[n,k],  lo = beta_n * min_k W[n,k]
 *     alpha = (hi - lo) / 255,      z = -lo / alpha
 *     q = clamp(round(W/alpha + z), 0, 255)
 * fp32, one IEEE operation per arithmetic symbol; round = half-to-even
 * (the paper does not name a tie rule for this equation).  A constant row
 * (hi == lo) would divide by zero; it takes alpha = 1, z = -lo so that
 * q = 0 and alpha * (q - z) returns the constant.
 * ---------------------------------------------------------------------- */
void mqo_quantize_int8(const float *W, int64_t N, int64_t K, int64_t ldw,
                       const float *gamma, const float *beta,
                       uint8_t *Q, float *alpha, float *zero) {
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const float *w = W + n * ldw;
        float mn = w[0], mx = w[0];
        for (int64_t k = 1; k < K; ++k) {
            if (w[k] < mn) mn = w[k];
            if (w[k] > mx) mx = w[k];
        }
        float hi = gamma ? gamma[n] * mx : mx;
        float lo = beta ? beta[n] * mn : mn;
        float a, z;
        if (hi == lo) {
            a = 1.0f;
            z = -lo;
        } else {
            a = (hi - lo) / 255.0f;
            z = -lo / a;
        }
        alpha[n] = a;
        zero[n] = z;
        for (int64_t k = 0; k < K; ++k) {
            float t = w[k] / a;
            float u = t + z;
            float r = rintf(u); /* round-half-to-even in the default mode */
            if (r < 0.0f) r = 0.0f;
            if (r > 255.0f) r = 255.0f;
            Q[n * K + k] = (uint8_t)r;
        }
    }
}

/* ------------------------------------------------------------------------
 * Slicing operator S(q, r), section 3.2 (slicing equation) and appendix A:
 *     code = clamp(round(q / 2^(8-r)), 0, 2^r - 1),  S = code * 2^(8-r)
 * The appendix describes the rounding at bit level (look at the bit below
 * the kept ones and push up when it is set), which is round-half-UP on a
 * non-negative integer: floor(q / 2^s + 1/2).  The extra-precision variant
 * of the errata section drops the clamp, so the code may reach 2^r.
 * Evaluated here literally in double precision; q / 2^s and + 0.5 are exact.
 * ---------------------------------------------------------------------- */
static int slice_code(int q, int r, int ep) {
    int s = 8 - r;
    double scaled = (double)q / (double)(1 << s);
    int code = (int)floor(scaled + 0.5);
    if (!ep) {
        int top = (1 << r) - 1;
        if (code < 0) code = 0;
        if (code > top) code = top;
    }
    return code;
}

/* code[i] for every element; ep != 0 gives the unclamped code (max 2^r). */
void mqo_slice_codes(const uint8_t *Q, int64_t count, int r, int ep, uint8_t *code) {
    for (int64_t i = 0; i < count; ++i) code[i] = (uint8_t)slice_code(Q[i], r, ep);
}

/* S(q, r) on the int8 grid (needs 9 bits in the extra-precision case). */
void mqo_slice_values(const uint8_t *Q, int64_t count, int r, int ep, uint16_t *value) {
    for (int64_t i = 0; i < count; ++i)
        value[i] = (uint16_t)(slice_code(Q[i], r, ep) << (8 - r));
}

/* ------------------------------------------------------------------------
 * Packing (format is this repository's; the paper gives none).  A row is a
 * little-endian bit stream of r bits per code: code k occupies stream bits
 * [r k, r k + r), least significant bit first, and stream bit t is bit t mod 8
 * of byte t / 8.  For r in {8, 4, 2} this is "8/r codes per byte, element k in
 * byte k / (8/r) at bit offset r (k mod 8/r)"; r = 6 and r = 3 (the
 * interpolated bit-widths of section 4.2) put 4 resp. 8 codes into 3 bytes.
 * K r must be a multiple of 8.
 * ---------------------------------------------------------------------- */
void mqo_pack(const uint8_t *code, int64_t N, int64_t K, int r, uint8_t *out) {
    int64_t kb = K * r / 8;
    memset(out, 0, (size_t)(N * kb));
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            for (int j = 0; j < r; ++j) {
                int64_t t = k * r + j;
                if ((code[n * K + k] >> j) & 1) out[n * kb + t / 8] |= (uint8_t)(1u << (t % 8));
            }
}

static int stream_code(const uint8_t *row, int64_t k, int r) {
    int c = 0;
    for (int j = 0; j < r; ++j) {
        int64_t t = k * r + j;
        c |= ((row[t / 8] >> (t % 8)) & 1) << j;
    }
    return c;
}

void mqo_unpack(const uint8_t *packed, int64_t N, int64_t K, int r, uint8_t *code) {
    int64_t kb = K * r / 8;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) code[n * K + k] = (uint8_t)stream_code(packed + n * kb, k, r);
}

/* ------------------------------------------------------------------------
 * Extra-precision overflow set (errata section: "an extra bit" for the values
 * that land in bucket 2^r).  Format is this repository's: CSR over rows,
 * ascending uint16 columns.  row_ptr has N+1 entries.  Returns the total
 * count; writes at most `capacity` columns.
 * ---------------------------------------------------------------------- */
int64_t mqo_overflow_csr(const uint8_t *Q, int64_t N, int64_t K, int r,
                         int32_t *row_ptr, uint16_t *col_idx, int64_t capacity) {
    int64_t nnz = 0;
    int top = (1 << r) - 1;
    for (int64_t n = 0; n < N; ++n) {
        row_ptr[n] = (int32_t)nnz;
        for (int64_t k = 0; k < K; ++k) {
            if (slice_code(Q[n * K + k], r, 1) > top) {
                if (nnz < capacity) col_idx[nnz] = (uint16_t)k;
                ++nnz;
            }
        }
    }
    row_ptr[N] = (int32_t)nnz;
    return nnz;
}

/* ------------------------------------------------------------------------
 * Dequantized weight: What_r[n,k] = alpha_n * (S(q[n,k], r) - z_n), the same
 * alpha, z for every r (that is what the * 2^(c-r) in the slicing equation
 * is for; the paper's int2 level set 0, 64, 128, 192 lives on the int8 grid).
 * ---------------------------------------------------------------------- */
static double what(const uint8_t *Q, const float *alpha, const float *zero,
                   int64_t n, int64_t k, int64_t K, int r, int ep) {
    int S = slice_code(Q[n * K + k], r, ep) << (8 - r);
    return (double)alpha[n] * ((double)S - (double)zero[n]);
}

void mqo_dequant(const uint8_t *Q, const float *alpha, const float *zero,
                 int64_t N, int64_t K, int r, int ep, double *What) {
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) What[n * K + k] = what(Q, alpha, zero, n, k, K, r, ep);
}

/* ------------------------------------------------------------------------
 * Forward of one linear at one bit-width (the F(S(Q(theta,c),r), x) inside
 * the MatQuant objective, section 3.2):  Y[m,n] = sum_k X[m,k] * What_r[n,k].
 * ---------------------------------------------------------------------- */
void mqo_linear_fwd(const uint16_t *X, const uint8_t *Q, const float *alpha, const float *zero,
                    int64_t M, int64_t N, int64_t K, int r, int ep, double *Y) {
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double *wrow = (double *)malloc((size_t)K * sizeof(double));
        for (int64_t k = 0; k < K; ++k) wrow[k] = what(Q, alpha, zero, n, k, K, r, ep);
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) acc += bf16_bits_to_f64(X[m * K + k]) * wrow[k];
            Y[m * N + n] = acc;
        }
        free(wrow);
    }
}

/* Same sum for a list of (m, n) pairs only; out[i] = Y[ms[i], ns[i]]. */
void mqo_linear_fwd_sampled(const uint16_t *X, const uint8_t *Q, const float *alpha,
                            const float *zero, int64_t M, int64_t N, int64_t K, int r, int ep,
                            const int64_t *ms, const int64_t *ns, int64_t count, double *out) {
    (void)M;
    (void)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        int64_t m = ms[i], n = ns[i];
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k)
            acc += bf16_bits_to_f64(X[m * K + k]) * what(Q, alpha, zero, n, k, K, r, ep);
        out[i] = acc;
    }
}

/* ------------------------------------------------------------------------
 * Straight-through backward (sections 3.1.1 and 3.1.2 only say that an STE
 * carries gradients through the quantizer; the identity STE with alpha, z
 * held constant is this repository's reading).  With per-bit-width output
 * gradients dY_r and loss weights lambda_r (section 3.2, MatQuant objective):
 *     dX[m,k] = sum_r lambda_r sum_n dY_r[m,n] * What_r[n,k]
 *     dW[n,k] = sum_m (sum_r lambda_r dY_r[m,n]) * X[m,k]
 * ---------------------------------------------------------------------- */
void mqo_linear_bwd_dx(const uint8_t *Q, const float *alpha, const float *zero,
                       const uint16_t *const *dY, const float *lambda,
                       int64_t M, int64_t N, int64_t K, const int *rs, int nr, int ep,
                       double *dX) {
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < K; ++k) {
        double *wcol = (double *)malloc((size_t)N * sizeof(double));
        for (int64_t m = 0; m < M; ++m) dX[m * K + k] = 0.0;
        for (int i = 0; i < nr; ++i) {
            double lam = lambda ? (double)lambda[i] : 1.0;
            for (int64_t n = 0; n < N; ++n) wcol[n] = what(Q, alpha, zero, n, k, K, rs[i], ep);
            for (int64_t m = 0; m < M; ++m) {
                double acc = 0.0;
                for (int64_t n = 0; n < N; ++n) acc += bf16_bits_to_f64(dY[i][m * N + n]) * wcol[n];
                dX[m * K + k] += lam * acc;
            }
        }
        free(wcol);
    }
}

void mqo_linear_bwd_dx_sampled(const uint8_t *Q, const float *alpha, const float *zero,
                               const uint16_t *const *dY, const float *lambda,
                               int64_t M, int64_t N, int64_t K, const int *rs, int nr, int ep,
                               const int64_t *ms, const int64_t *ks, int64_t count, double *out) {
    (void)M;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < count; ++j) {
        int64_t m = ms[j], k = ks[j];
        double total = 0.0;
        for (int i = 0; i < nr; ++i) {
            double lam = lambda ? (double)lambda[i] : 1.0;
            double acc = 0.0;
            for (int64_t n = 0; n < N; ++n)
                acc += bf16_bits_to_f64(dY[i][m * N + n]) * what(Q, alpha, zero, n, k, K, rs[i], ep);
            total += lam * acc;
        }
        out[j] = total;
    }
}

void mqo_linear_bwd_dw(const uint16_t *X, const uint16_t *const *dY, const float *lambda,
                       int64_t M, int64_t N, int64_t K, int nr, double *dW) {
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double *g = (double *)malloc((size_t)M * sizeof(double));
        for (int64_t m = 0; m < M; ++m) {
            double s = 0.0;
            for (int i = 0; i < nr; ++i)
                s += (lambda ? (double)lambda[i] : 1.0) * bf16_bits_to_f64(dY[i][m * N + n]);
            g[m] = s;
        }
        for (int64_t k = 0; k < K; ++k) {
            double acc = 0.0;
            for (int64_t m = 0; m < M; ++m) acc += g[m] * bf16_bits_to_f64(X[m * K + k]);
            dW[n * K + k] = acc;
        }
        free(g);
    }
}

void mqo_linear_bwd_dw_sampled(const uint16_t *X, const uint16_t *const *dY, const float *lambda,
                               int64_t M, int64_t N, int64_t K, int nr,
                               const int64_t *ns, const int64_t *ks, int64_t count, double *out) {
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < count; ++j) {
        int64_t n = ns[j], k = ks[j];
        double acc = 0.0;
        for (int64_t m = 0; m < M; ++m) {
            double g = 0.0;
            for (int i = 0; i < nr; ++i)
                g += (lambda ? (double)lambda[i] : 1.0) * bf16_bits_to_f64(dY[i][m * N + n]);
            acc += g * bf16_bits_to_f64(X[m * K + k]);
        }
        out[j] = acc;
    }
}

/* ------------------------------------------------------------------------
 * Weight-only decode GEMV from a packed r-bit plane (section 1 motivates it:
 * decode is bound by moving weights out of HBM; section 5.4 and the errata
 * mention the kernels without describing them):
 *     y[b,n] = sum_k x[b,k] * alpha_n * (S[n,k] - z_n)
 * where S = code << (8-r) is read back from the packed plane, alpha and z
 * are bf16, and, when an overflow list is given (extra precision), S gains
 * one more 2^(8-r) at every listed column.  `shift` < 0 means s = 8 - r; a
 * dense extra-precision plane (codes 0 .. 2^rv stored with r = rv + 1 bits,
 * errata section) is read with shift = 8 - rv.
 * ---------------------------------------------------------------------- */
void mqo_gemv_sliced(const uint16_t *x, const uint8_t *packed, const uint16_t *alpha_bf16,
                     const uint16_t *zero_bf16, const int32_t *row_ptr, const uint16_t *col_idx,
                     int64_t B, int64_t N, int64_t K, int r, int shift, double *y) {
    int64_t kb = K * r / 8;
    int s = shift < 0 ? 8 - r : shift;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double a = bf16_bits_to_f64(alpha_bf16[n]);
        double z = bf16_bits_to_f64(zero_bf16[n]);
        int *S = (int *)malloc((size_t)K * sizeof(int));
        for (int64_t k = 0; k < K; ++k) S[k] = stream_code(packed + n * kb, k, r) << s;
        if (row_ptr)
            for (int32_t p = row_ptr[n]; p < row_ptr[n + 1]; ++p) S[col_idx[p]] += 1 << s;
        for (int64_t b = 0; b < B; ++b) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += bf16_bits_to_f64(x[b * K + k]) * (a * ((double)S[k] - z));
            y[b * N + n] = acc;
        }
        free(S);
    }
}

int mqo_num_threads(void) {
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
