// mq_gemv_sliced: weight-only decode GEMV on a packed r-bit plane (section 1: decode is bound by
// streaming the weights out of HBM), plus the sparse overflow additions the errata section asks for.
//
// HBM-bound: N*K*r/8 weight bytes are read exactly once with 16-byte loads; everything else is
// small.  The multiply-accumulate runs on the 16x16x32 bf16 matrix core (16 weight rows x up to 16
// batch entries), because at int2 rates a VALU multiply per weight and batch entry would not keep
// up with HBM.  Codes are turned into bf16 without integer->float conversion: a 2- or 4-bit field
// that sits at mantissa bit p of a bf16 whose exponent is 2^(7-p) reads as 2^(7-p) + code, so one
// AND-OR per two codes does the unpack; the constant 2^(7-p) offsets are summed by one extra
// matrix-core product with a constant operand and subtracted in the epilogue.
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
    int KB;  // bytes per packed row
};

constexpr uint32_t kOne2 = 0x3F803F80u;                                 // (1.0, 1.0)
constexpr uint32_t kB128 = 0x43004300u, kB32 = 0x42004200u, kB8 = 0x41004100u;  // (128,128) (32,32) (8,8)

__device__ __forceinline__ f32x4 mfma16(const u32x4 &a, const u32x4 &b, const f32x4 &c) {
    Frag8 fa, fb;
    fa.u = a;
    fb.u = b;
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa.b, fb.b, c, 0, 0, 0);
}

// (lo halves) and (hi halves) of two registers of packed bf16 pairs
__device__ __forceinline__ uint32_t pair_lo(uint32_t first, uint32_t second) {
    return __builtin_amdgcn_perm(second, first, 0x05040100u);
}
__device__ __forceinline__ uint32_t pair_hi(uint32_t first, uint32_t second) {
    return __builtin_amdgcn_perm(second, first, 0x07060302u);
}

// One workgroup = NW waves on one block of 16 * RG weight rows; the waves interleave over the
// 64-byte row segments and their partial sums meet in LDS.  Lane (i, g) = (lane % 16, lane / 16)
// owns weight row i of each of the RG row groups and bytes [16 g, 16 g + 16) of every segment,
// and batch entry b = i of the activations for the same k range.
template <int R, int RG>
__global__ __launch_bounds__(512) void gemv_kernel(GemvArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int NW = blockDim.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int n0 = blockIdx.x * (16 * RG);
    constexpr int KPB = 8 / R;          // codes per byte
    constexpr int SLOTS = RG + 1;       // accumulators per lane: RG row groups + the constant operand

    f32x4 acc[RG];
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) acc[rg] = f32x4{0.f, 0.f, 0.f, 0.f};
    f32x4 acc_c = {0.f, 0.f, 0.f, 0.f};  // row 0: sum_k x, row 1 (int2): sum_k x * offset_k

    const int iters = (a.KB + 63) >> 6;
    const bool xlive = i < a.B;
    const uint16_t *xrow = a.x + (size_t)(xlive ? i : 0) * a.K;

    for (int it = wave; it < iters; it += NW) {
        const int off = it * 64 + g * 16;  // byte offset inside the packed row
        const bool inside = off < a.KB;
        u32x4 wt[RG];
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) {
            const int row = n0 + rg * 16 + i;
            wt[rg] = u32x4{0u, 0u, 0u, 0u};
            if (inside && row < a.N)
                wt[rg] = __builtin_nontemporal_load(
                    reinterpret_cast<const u32x4 *>(a.packed + (size_t)row * a.KB + off));
        }
        const int kx = off * KPB;  // first k of this lane's 16 bytes
        const bool xl = inside && xlive;

        if constexpr (R == 2) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                u32x4 x0 = {0u, 0u, 0u, 0u}, x1 = {0u, 0u, 0u, 0u};
                if (xl) {
                    x0 = *reinterpret_cast<const u32x4 *>(xrow + kx + 16 * w);
                    x1 = *reinterpret_cast<const u32x4 *>(xrow + kx + 16 * w + 8);
                }
                // codes j and j + 8 of the dword share a register; pair the activations the same way
                const u32x4 xb0 = {pair_lo(x0.x, x1.x), pair_hi(x0.x, x1.x), pair_lo(x0.y, x1.y), pair_hi(x0.y, x1.y)};
                const u32x4 xb1 = {pair_lo(x0.z, x1.z), pair_hi(x0.z, x1.z), pair_lo(x0.w, x1.w), pair_hi(x0.w, x1.w)};
#pragma unroll
                for (int rg = 0; rg < RG; ++rg) {
                    const uint32_t d = wt[rg][w], d6 = d >> 6, d12 = d >> 12;
                    const u32x4 a0 = {(d & 0x00030003u) | kB128, (d & 0x000C000Cu) | kB32,
                                      (d & 0x00300030u) | kB8, (d6 & 0x00030003u) | kB128};
                    const u32x4 a1 = {(d6 & 0x000C000Cu) | kB32, (d6 & 0x00300030u) | kB8,
                                      (d12 & 0x00030003u) | kB128, (d12 & 0x000C000Cu) | kB32};
                    acc[rg] = mfma16(a0, xb0, acc[rg]);
                    acc[rg] = mfma16(a1, xb1, acc[rg]);
                }
                // constant operand: row 0 = ones, row 1 = the offsets of the fields above
                u32x4 c0 = {0u, 0u, 0u, 0u}, c1 = {0u, 0u, 0u, 0u};
                if (i == 0) {
                    c0 = u32x4{kOne2, kOne2, kOne2, kOne2};
                    c1 = c0;
                } else if (i == 1) {
                    c0 = u32x4{kB128, kB32, kB8, kB128};
                    c1 = u32x4{kB32, kB8, kB128, kB32};
                }
                acc_c = mfma16(c0, xb0, acc_c);
                acc_c = mfma16(c1, xb1, acc_c);
            }
        } else if constexpr (R == 4) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                u32x4 x0 = {0u, 0u, 0u, 0u};
                if (xl) x0 = *reinterpret_cast<const u32x4 *>(xrow + kx + 8 * w);
                // codes j and j + 4 of the dword share a register
                const u32x4 xb = {pair_lo(x0.x, x0.z), pair_hi(x0.x, x0.z), pair_lo(x0.y, x0.w), pair_hi(x0.y, x0.w)};
#pragma unroll
                for (int rg = 0; rg < RG; ++rg) {
                    const uint32_t d = wt[rg][w];
                    const u32x4 a0 = {(d & 0x000F000Fu) | kB128, ((d >> 4) & 0x000F000Fu) | kB128,
                                      ((d >> 8) & 0x000F000Fu) | kB128, ((d >> 12) & 0x000F000Fu) | kB128};
                    acc[rg] = mfma16(a0, xb, acc[rg]);
                }
                u32x4 c0 = {0u, 0u, 0u, 0u};
                if (i == 0) c0 = u32x4{kOne2, kOne2, kOne2, kOne2};
                acc_c = mfma16(c0, xb, acc_c);
            }
        } else {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                u32x4 xb = {0u, 0u, 0u, 0u};
                if (xl) xb = *reinterpret_cast<const u32x4 *>(xrow + kx + 8 * u);
#pragma unroll
                for (int rg = 0; rg < RG; ++rg) {
                    const uint32_t d0 = wt[rg][2 * u], d1 = wt[rg][2 * u + 1];
                    auto two = [](uint32_t lo, uint32_t hi) {  // two small integers -> packed bf16 (exact)
                        return __builtin_amdgcn_perm(__float_as_uint((float)hi), __float_as_uint((float)lo), 0x07060302u);
                    };
                    const u32x4 a0 = {two(d0 & 0xFFu, (d0 >> 8) & 0xFFu), two((d0 >> 16) & 0xFFu, d0 >> 24),
                                      two(d1 & 0xFFu, (d1 >> 8) & 0xFFu), two((d1 >> 16) & 0xFFu, d1 >> 24)};
                    acc[rg] = mfma16(a0, xb, acc[rg]);
                }
                u32x4 c0 = {0u, 0u, 0u, 0u};
                if (i == 0) c0 = u32x4{kOne2, kOne2, kOne2, kOne2};
                acc_c = mfma16(c0, xb, acc_c);
            }
        }
    }

    // ---- cross-wave reduction in LDS --------------------------------------------------------
    // part[wave][slot][lane] (float4), then total[slot][lane], then ovf[row][b]
    f32x4 *part = reinterpret_cast<f32x4 *>(lds);
    f32x4 *total = part + NW * SLOTS * 64;
    float *ovf = reinterpret_cast<float *>(total + SLOTS * 64);
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) part[(wave * SLOTS + rg) * 64 + lane] = acc[rg];
    part[(wave * SLOTS + RG) * 64 + lane] = acc_c;

    // ---- extra precision: sum of x over each row's overflow columns ---------------------------
    if (a.row_ptr) {
        for (int r = wave; r < 16 * RG; r += NW) {
            const int row = n0 + r;
            float s[16];
#pragma unroll
            for (int b = 0; b < 16; ++b) s[b] = 0.f;
            if (row < a.N) {
                const int lo = a.row_ptr[row], hi = a.row_ptr[row + 1];
                for (int p = lo + lane; p < hi; p += 64) {
                    const int col = a.col_idx[p];
#pragma unroll
                    for (int b = 0; b < 16; ++b)
                        if (b < a.B) s[b] += bf16_bits_to_float(a.x[(size_t)b * a.K + col]);
                }
            }
#pragma unroll
            for (int b = 0; b < 16; ++b) {
                if (b < a.B) {
#pragma unroll
                    for (int o = 32; o > 0; o >>= 1) s[b] += __shfl_xor(s[b], o, 64);
                }
                if (lane == 0) ovf[r * 16 + b] = s[b];
            }
        }
    }
    __syncthreads();
    for (int t = threadIdx.x; t < SLOTS * 64; t += blockDim.x) {
        f32x4 sum = part[t];
        for (int w = 1; w < NW; ++w) {
            const f32x4 p = part[w * SLOTS * 64 + t];
            sum.x += p.x;
            sum.y += p.y;
            sum.z += p.z;
            sum.w += p.w;
        }
        total[t] = sum;
    }
    __syncthreads();

    // ---- epilogue: y[b, n] = alpha_n * (2^s * (codes.x [+ overflow]) - z_n * sum_k x) -----------
    // matrix-core output layout: lane = column b + 16 * (row / 4), component = row % 4
    const float *tot = reinterpret_cast<const float *>(total);
    constexpr float kScale = (float)(1 << (8 - R));
    for (int t = threadIdx.x; t < 16 * RG * 16; t += blockDim.x) {
        const int b = t / (16 * RG), r = t % (16 * RG);
        const int row = n0 + r;
        if (b >= a.B || row >= a.N) continue;
        const int rg = r >> 4, ri = r & 15;
        float dot = tot[(rg * 64 + b + 16 * (ri >> 2)) * 4 + (ri & 3)];
        const float xsum = tot[(RG * 64 + b) * 4 + 0];
        float offset;
        if constexpr (R == 2) {
            offset = tot[(RG * 64 + b) * 4 + 1];
        } else if constexpr (R == 4) {
            offset = 128.0f * xsum;
        } else {
            offset = 0.0f;
        }
        dot -= offset;
        if (a.row_ptr) dot += ovf[r * 16 + b];
        const float al = bf16_bits_to_float(a.alpha[row]), z = bf16_bits_to_float(a.zero[row]);
        const float yv = al * (kScale * dot - z * xsum);
        a.y[(size_t)b * a.N + row] = (uint16_t)float_to_bf16_bits(yv);
    }
}

template <int R, int RG>
static void launch_gemv(const GemvArgs &a, int nw, hipStream_t st) {
    const int blocks = (int)cdiv(a.N, 16 * RG);
    const size_t lds = (size_t)(nw + 1) * (RG + 1) * 64 * 16 + (size_t)16 * RG * 16 * 4;
    gemv_kernel<R, RG><<<dim3(blocks), dim3(64 * nw), lds, st>>>(a);
}

}  // namespace mq

extern "C" mq_status mq_gemv_sliced(const uint16_t *x, const uint8_t *packed, const uint16_t *alpha_bf16,
                                    const uint16_t *zero_bf16, const mq_overflow *ovf, int64_t B, int64_t N,
                                    int64_t K, int r, uint16_t *y, void *hip_stream) {
    using namespace mq;
    if (r != 8 && r != 4 && r != 2) return MQ_ERR_BITS;
    if (B < 1 || B > 16 || N < 0 || K < 1 || N > 0x7FFFFFF0 || K > 0x7FFFFFF0) return MQ_ERR_SHAPE;
    if (ovf && K > 65536) return MQ_ERR_SHAPE;
    const int64_t kb = K * r / 8;
    if ((K * r) % 128 != 0) return MQ_ERR_ALIGN;  // packed rows are whole 16-byte units
    if (N == 0) return MQ_OK;
    if (!x || !packed || !alpha_bf16 || !zero_bf16 || !y) return MQ_ERR_NULL;
    if (ovf && (!ovf->row_ptr || !ovf->col_idx)) return MQ_ERR_NULL;
    if (!aligned16(x) || !aligned16(packed)) return MQ_ERR_ALIGN;

    GemvArgs a;
    a.x = x;
    a.packed = packed;
    a.alpha = alpha_bf16;
    a.zero = zero_bf16;
    a.row_ptr = ovf ? ovf->row_ptr : nullptr;
    a.col_idx = ovf ? ovf->col_idx : nullptr;
    a.y = y;
    a.B = (int)B;
    a.N = (int)N;
    a.K = (int)K;
    a.KB = (int)kb;

    // rows per workgroup: as many as still leave two workgroups per compute unit
    int rg = 4;
    while (rg > 1 && cdiv(N, 16 * rg) < 512) rg >>= 1;
    // waves per workgroup: each should see at least two 64-byte segments of its rows
    const int64_t iters = cdiv(kb, 64);
    int nw = 8;
    while (nw > 1 && iters < 2 * nw) nw >>= 1;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
#define MQ_GEMV_CASE(R_, RG_)                    \
    if (r == R_ && rg == RG_) {                  \
        launch_gemv<R_, RG_>(a, nw, st);         \
        return launch_status();                  \
    }
    MQ_GEMV_CASE(2, 1) MQ_GEMV_CASE(2, 2) MQ_GEMV_CASE(2, 4)
    MQ_GEMV_CASE(4, 1) MQ_GEMV_CASE(4, 2) MQ_GEMV_CASE(4, 4)
    MQ_GEMV_CASE(8, 1) MQ_GEMV_CASE(8, 2) MQ_GEMV_CASE(8, 4)
#undef MQ_GEMV_CASE
    return MQ_ERR_BITS;
}
