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

// Eight (R = 2), four (R = 4) or two (R = 8) MFMAs on the 16 bytes `d` a lane holds of one weight
// row, against the activations x0/x1 of the same k range; `acc_c` gathers the products with the
// constant operand c (row 0 = ones, for int2 row 1 = the field offsets).
template <int R, int RG>
__device__ __forceinline__ void gemv_segment(const u32x4 (&wt)[RG], const u32x4 *xs, int i, f32x4 (&acc)[RG],
                                             f32x4 &acc_c) {
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    const u32x4 ones = {kOne2, kOne2, kOne2, kOne2};
    if constexpr (R == 2) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const u32x4 x0 = xs[2 * w], x1 = xs[2 * w + 1];
            // codes j and j + 8 of the dword share a register; pair the activations the same way
            const u32x4 xb0 = {pair_lo(x0.x, x1.x), pair_hi(x0.x, x1.x), pair_lo(x0.y, x1.y), pair_hi(x0.y, x1.y)};
            const u32x4 xb1 = {pair_lo(x0.z, x1.z), pair_hi(x0.z, x1.z), pair_lo(x0.w, x1.w), pair_hi(x0.w, x1.w)};
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) {
                const uint32_t d = wt[rg][w], d6 = d >> 6, d12 = d >> 12;
                const u32x4 a0 = {(d & 0x00030003u) | kB128, (d & 0x000C000Cu) | kB32, (d & 0x00300030u) | kB8,
                                  (d6 & 0x00030003u) | kB128};
                const u32x4 a1 = {(d6 & 0x000C000Cu) | kB32, (d6 & 0x00300030u) | kB8, (d12 & 0x00030003u) | kB128,
                                  (d12 & 0x000C000Cu) | kB32};
                acc[rg] = mfma16(a0, xb0, acc[rg]);
                acc[rg] = mfma16(a1, xb1, acc[rg]);
            }
            const u32x4 c0 = i == 0 ? ones : (i == 1 ? u32x4{kB128, kB32, kB8, kB128} : zero4);
            const u32x4 c1 = i == 0 ? ones : (i == 1 ? u32x4{kB32, kB8, kB128, kB32} : zero4);
            acc_c = mfma16(c0, xb0, acc_c);
            acc_c = mfma16(c1, xb1, acc_c);
        }
    } else if constexpr (R == 4) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const u32x4 x0 = xs[w];
            // codes j and j + 4 of the dword share a register
            const u32x4 xb = {pair_lo(x0.x, x0.z), pair_hi(x0.x, x0.z), pair_lo(x0.y, x0.w), pair_hi(x0.y, x0.w)};
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) {
                const uint32_t d = wt[rg][w];
                const u32x4 a0 = {(d & 0x000F000Fu) | kB128, ((d >> 4) & 0x000F000Fu) | kB128,
                                  ((d >> 8) & 0x000F000Fu) | kB128, ((d >> 12) & 0x000F000Fu) | kB128};
                acc[rg] = mfma16(a0, xb, acc[rg]);
            }
            acc_c = mfma16(i == 0 ? ones : zero4, xb, acc_c);
        }
    } else {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const u32x4 xb = xs[u];
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
            acc_c = mfma16(i == 0 ? ones : zero4, xb, acc_c);
        }
    }
}

// One workgroup = NW waves on one block of 16 * RG weight rows; the waves interleave over the
// 64-byte row segments and their partial sums meet in LDS.  Lane (i, g) = (lane % 16, lane / 16)
// owns weight row i of each of the RG row groups and bytes [16 g, 16 g + 16) of every segment,
// and batch entry b = i of the activations for the same k range.  A wave requests the weights and
// activations of IT segments at once before it computes, so that a whole small matrix is in
// flight after one round trip to memory.
template <int R, int RG, int IT>
__global__ __launch_bounds__(1024) void gemv_kernel(GemvArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int NW = blockDim.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int n0 = blockIdx.x * (16 * RG);
    constexpr int KPB = 8 / R;             // codes per byte
    constexpr int SLOTS = RG + 1;          // accumulators per lane: RG row groups + the constant operand
    constexpr int XV = R == 2 ? 8 : (R == 4 ? 4 : 2);  // 16-byte activation loads per lane and segment

    // epilogue parameters of this thread's first output, requested before anything else so that
    // their latency is hidden behind the weight stream
    constexpr int OUTS = 16 * RG * 16;  // outputs of the workgroup: (b, row) = (t / (16 RG), t % (16 RG))
    uint16_t e_alpha = 0, e_zero = 0;
    if (threadIdx.x < OUTS && n0 + (int)(threadIdx.x % (16 * RG)) < a.N) {
        e_alpha = a.alpha[n0 + threadIdx.x % (16 * RG)];
        e_zero = a.zero[n0 + threadIdx.x % (16 * RG)];
    }

    f32x4 acc[RG];
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) acc[rg] = f32x4{0.f, 0.f, 0.f, 0.f};
    f32x4 acc_c = {0.f, 0.f, 0.f, 0.f};  // row 0: sum_k x, row 1 (int2): sum_k x * offset_k

    const int segs = (a.KB + 63) >> 6;
    const bool xlive = i < a.B;
    const uint16_t *xrow = a.x + (size_t)(xlive ? i : 0) * a.K;

    for (int s0 = wave; s0 < segs; s0 += NW * IT) {
        u32x4 wt[IT][RG];
        u32x4 xs[IT][XV];
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int off = (s0 + it * NW) * 64 + g * 16;  // byte offset inside the packed row
            const bool inside = off < a.KB;
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) {
                const int row = n0 + rg * 16 + i;
                wt[it][rg] = u32x4{0u, 0u, 0u, 0u};
                if (inside && row < a.N)
                    wt[it][rg] = __builtin_nontemporal_load(
                        reinterpret_cast<const u32x4 *>(a.packed + (size_t)row * a.KB + off));
            }
        }
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int off = (s0 + it * NW) * 64 + g * 16;
            const bool xl = off < a.KB && xlive;
            const u32x4 *xp = reinterpret_cast<const u32x4 *>(xrow + off * KPB);
#pragma unroll
            for (int v = 0; v < XV; ++v) xs[it][v] = xl ? xp[v] : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int it = 0; it < IT; ++it) gemv_segment<R, RG>(wt[it], xs[it], i, acc, acc_c);
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
    for (int t = threadIdx.x; t < OUTS; t += blockDim.x) {
        const int b = t / (16 * RG), er = t % (16 * RG), erow = n0 + er;
        if (b >= a.B || erow >= a.N) continue;
        if (t != (int)threadIdx.x) {  // only workgroups with fewer threads than outputs come here
            e_alpha = a.alpha[erow];
            e_zero = a.zero[erow];
        }
        const int rg = er >> 4, ri = er & 15;
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
        if (a.row_ptr) dot += ovf[er * 16 + b];
        const float al = bf16_bits_to_float(e_alpha), z = bf16_bits_to_float(e_zero);
        const float yv = al * (kScale * dot - z * xsum);
        a.y[(size_t)b * a.N + erow] = (uint16_t)float_to_bf16_bits(yv);
    }
}

template <int R, int RG, int IT>
static void launch_gemv(const GemvArgs &a, int nw, hipStream_t st) {
    const int blocks = (int)cdiv(a.N, 16 * RG);
    const size_t lds = (size_t)(nw + 1) * (RG + 1) * 64 * 16 + (size_t)16 * RG * 16 * 4;
    gemv_kernel<R, RG, IT><<<dim3(blocks), dim3(64 * nw), lds, st>>>(a);
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

    // Rows per workgroup (16 RG): each activation value is fetched once per workgroup, so a larger
    // batch wants more rows behind every fetch; small batches keep RG = 1 for more workgroups.
    const int rg = B <= 2 ? 1 : (B <= 8 ? 2 : 4);
    // Waves per workgroup split the 64-byte segments of the rows; each wave takes up to IT of them
    // per round trip to memory.
    const int64_t segs = cdiv(kb, 64);
    int nw = 16;
    while (nw > 1 && segs < nw) nw >>= 1;
    int it = segs >= 2 * nw ? 2 : 1;
    if (r == 2 && rg == 4) it = 1;  // 64 int2 weights per lane and segment: registers allow one segment
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
#define MQ_GEMV_CASE(R_, RG_, IT_)                 \
    if (r == R_ && rg == RG_ && it == IT_) {       \
        launch_gemv<R_, RG_, IT_>(a, nw, st);      \
        return launch_status();                    \
    }
    MQ_GEMV_CASE(2, 1, 1) MQ_GEMV_CASE(2, 2, 1) MQ_GEMV_CASE(2, 4, 1)
    MQ_GEMV_CASE(2, 1, 2) MQ_GEMV_CASE(2, 2, 2)
    MQ_GEMV_CASE(4, 1, 1) MQ_GEMV_CASE(4, 2, 1) MQ_GEMV_CASE(4, 4, 1)
    MQ_GEMV_CASE(4, 1, 2) MQ_GEMV_CASE(4, 2, 2) MQ_GEMV_CASE(4, 4, 2)
    MQ_GEMV_CASE(8, 1, 1) MQ_GEMV_CASE(8, 2, 1) MQ_GEMV_CASE(8, 4, 1)
    MQ_GEMV_CASE(8, 1, 2) MQ_GEMV_CASE(8, 2, 2) MQ_GEMV_CASE(8, 4, 2)
#undef MQ_GEMV_CASE
    return MQ_ERR_BITS;
}
