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
#include <type_traits>

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

// Sum over the 64 lanes without the LDS crossbar: three DPP steps inside a row of 16, then the four
// rows through scalar reads.  The result is wave-uniform.
__device__ __forceinline__ float wave_sum(float v) {
    auto dpp_add = [](float x, auto ctrl) {
        const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value, 0xF, 0xF, true);
        return x + __int_as_float(moved);
    };
    v = dpp_add(v, std::integral_constant<int, 0xB1>{});   // quad_perm [1,0,3,2]
    v = dpp_add(v, std::integral_constant<int, 0x4E>{});   // quad_perm [2,3,0,1]
    v = dpp_add(v, std::integral_constant<int, 0x141>{});  // row_half_mirror: the other quad of 8
    v = dpp_add(v, std::integral_constant<int, 0x140>{});  // row_mirror: the other half of 16
    const int bits = __float_as_int(v);
    return __int_as_float(__builtin_amdgcn_readlane(bits, 0)) + __int_as_float(__builtin_amdgcn_readlane(bits, 16)) +
           __int_as_float(__builtin_amdgcn_readlane(bits, 32)) + __int_as_float(__builtin_amdgcn_readlane(bits, 48));
}

// The MFMAs of one 64-byte row segment: the 16 bytes a lane holds of each of its RG weight rows
// against the activations of the same k range, read from LDS (xs[v * xstride] = v-th operand of
// the lane's k range, already in the element order of the unpacked codes).
template <int R, int RG>
__device__ __forceinline__ void gemv_segment(const u32x4 (&wt)[RG], const u32x4 *xs, int xstride, f32x4 (&acc)[RG]) {
    if constexpr (R == 2) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const u32x4 xb0 = xs[(2 * w) * xstride], xb1 = xs[(2 * w + 1) * xstride];
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) {
                // codes j and j + 8 of a dword share a register; fields at bits 0-1, 2-3, 4-5 of a
                // 16-bit lane read as 128 + c, 32 + c, 8 + c under the exponents below
                const uint32_t d = wt[rg][w], d6 = d >> 6, d12 = d >> 12;
                const u32x4 a0 = {(d & 0x00030003u) | kB128, (d & 0x000C000Cu) | kB32, (d & 0x00300030u) | kB8,
                                  (d6 & 0x00030003u) | kB128};
                const u32x4 a1 = {(d6 & 0x000C000Cu) | kB32, (d6 & 0x00300030u) | kB8, (d12 & 0x00030003u) | kB128,
                                  (d12 & 0x000C000Cu) | kB32};
                acc[rg] = mfma16(a0, xb0, acc[rg]);
                acc[rg] = mfma16(a1, xb1, acc[rg]);
            }
        }
    } else if constexpr (R == 4) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const u32x4 xb = xs[w * xstride];
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) {
                const uint32_t d = wt[rg][w];  // codes j and j + 4 of the dword share a register
                const u32x4 a0 = {(d & 0x000F000Fu) | kB128, ((d >> 4) & 0x000F000Fu) | kB128,
                                  ((d >> 8) & 0x000F000Fu) | kB128, ((d >> 12) & 0x000F000Fu) | kB128};
                acc[rg] = mfma16(a0, xb, acc[rg]);
            }
        }
    } else {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const u32x4 xb = xs[u * xstride];
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
        }
    }
}

// One workgroup = KS * RW waves.  Wave (ks, rw) = (wave % KS, wave / KS) streams block rw of
// 16 * RG weight rows and takes every KS-th 64-byte segment of those rows; the KS partial sums of a
// row block meet in LDS.  Lane (i, g) = (lane % 16, lane / 16) owns weight row i of each of the RG
// row groups and bytes [16 g, 16 g + 16) of a segment, and batch entry b = i of the activations
// for the same k range.
//
// The activations are staged in LDS once per workgroup, already paired the way the unpacked codes
// are (in chunks of at most kXChunk bytes when B * K is large) and shared by all its waves; while
// they sit there, sum_k x and (int2) sum_k x * offset_k are taken once per workgroup, which is
// what removes the 128 / 32 / 8 offsets of the unpack and applies the zero-point.  The weights
// stream through a register ring that keeps D - 1 segments per wave in flight behind the one
// being computed.  Few rows -> large KS (the whole matrix is in flight after one round trip);
// many rows -> KS = 1 and every wave streams its own rows.
//
// Lanes are never masked in the hot loop: rows past N re-read row N - 1 and batch entries past B
// re-read entry i % bp; both only feed outputs that are not stored.  A lane whose 16 bytes lie
// past the end of the row re-reads the row's last 16 bytes; any bit pattern unpacks to finite
// numbers, and those meet activations that were staged as zeros.
constexpr int kXChunk = 65536;
constexpr int kSumBytes = 2048;  // per-wave partial sums of x: [2][16 batch entries][16 waves] floats, in front of the staging area

template <int R, int RG, int D, bool EP>
__global__ __launch_bounds__(1024) void gemv_kernel(GemvArgs a, int bp, int chunk_segs, int KS) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int NW = blockDim.x >> 6;
    const int RW = NW / KS;
    const int ks = wave % KS, rw = wave / KS;
    const int i = lane & 15, g = lane >> 4;
    constexpr int ROWS = 16 * RG;          // rows of one row block
    const int nb = blockIdx.x * RW * ROWS; // first row of the workgroup
    const int n0 = nb + rw * ROWS;         // first row of this wave
    constexpr int KPB = 8 / R;             // codes per byte
    constexpr int XV = R == 2 ? 8 : (R == 4 ? 4 : 2);  // 16-byte activation operands per lane and segment
    constexpr int SEGK = 64 * KPB;         // k values per segment
    constexpr int UNITK = R == 2 ? 16 : 8; // k values one staging step handles
    constexpr int UPS = SEGK / UNITK;      // staging steps per segment and batch entry

    float *sums = lds;  // [b * 16 + wave]: part of sum_k x[b, k]; [256 + b * 16 + wave]: part of sum_k x[b, k] * offset_k
    u32x4 *xl = reinterpret_cast<u32x4 *>(reinterpret_cast<uint8_t *>(lds) + kSumBytes);
    for (int t = threadIdx.x; t < 512; t += blockDim.x) sums[t] = 0.f;

    f32x4 acc[RG];
    u32x4 w[D][RG];
    const uint8_t *rp[RG];
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) {
        acc[rg] = f32x4{0.f, 0.f, 0.f, 0.f};
        rp[rg] = a.packed + (size_t)min(n0 + rg * 16 + i, a.N - 1) * a.KB;
#pragma unroll
        for (int d = 0; d < D; ++d) w[d][rg] = u32x4{0u, 0u, 0u, 0u};
    }
    int off = ks * 64 + g * 16;  // byte offset, inside the packed row, of the next segment to request
    // Unconditional (an offset past the row is clamped into it), so that the number of loads in
    // flight is known at compile time and a use only waits for its own load.
    const int off_last = a.KB - 16;
    auto fetch_next = [&](u32x4 (&dst)[RG]) {
        const int o = min(off, off_last);
#pragma unroll
        for (int rg = 0; rg < RG; ++rg)
            dst[rg] = *reinterpret_cast<const u32x4 *>(rp[rg] + o);  // (plain loads: non-temporal ones measured slower here)
        off += KS * 64;
    };
    const int segs = (a.KB + 63) >> 6;
    const u32x4 *xlane = xl + g * bp + (i & (bp - 1));
    const int step = KS * D;  // segments one turn of the ring covers (all KS waves of a row block)

    // The code below is kept small on purpose: a decode GEMV runs for a few microseconds, and
    // instruction fetch of a cold kernel is a visible part of that.
#pragma unroll
    for (int d = 0; d + 1 < D; ++d) fetch_next(w[d]);

    int s = ks;
    for (int c0 = 0; c0 < segs; c0 += chunk_segs) {
        const int c1 = min(c0 + chunk_segs, segs);
        const int units_per_row = (c1 - c0) * UPS;
        if (c0 > 0) __syncthreads();  // the previous chunk of x has been consumed
        // ---- stage x[:, c0 * SEGK : c1 * SEGK) in operand order: (ls, v, g, b) ------------------
        for (int t = threadIdx.x; t < units_per_row * a.B; t += blockDim.x) {
            const int b = t / units_per_row, un = t % units_per_row;
            const int k = c0 * SEGK + un * UNITK;
            const int ls = un / UPS, in = un % UPS;
            u32x4 x0 = {0u, 0u, 0u, 0u}, x1 = {0u, 0u, 0u, 0u};
            if (k < a.K) {  // a partial last segment is completed with zeros
                const uint16_t *src = a.x + (size_t)b * a.K + k;
                x0 = *reinterpret_cast<const u32x4 *>(src);
                if constexpr (R == 2) x1 = *reinterpret_cast<const u32x4 *>(src + 8);
            }
            if constexpr (R == 2) {
                const int gg = in >> 2, ww = in & 3;  // k = seg * 256 + gg * 64 + ww * 16
                // codes j and j + 8 of a dword share a register: pair the activations the same way
                xl[((ls * XV + 2 * ww) * 4 + gg) * bp + b] =
                    u32x4{pair_lo(x0.x, x1.x), pair_hi(x0.x, x1.x), pair_lo(x0.y, x1.y), pair_hi(x0.y, x1.y)};
                xl[((ls * XV + 2 * ww + 1) * 4 + gg) * bp + b] =
                    u32x4{pair_lo(x0.z, x1.z), pair_hi(x0.z, x1.z), pair_lo(x0.w, x1.w), pair_hi(x0.w, x1.w)};
            } else {
                const int gg = in / XV, vv = in % XV;  // k = seg * SEGK + gg * (SEGK / 4) + vv * 8
                if constexpr (R == 4)  // codes j and j + 4 of a dword share a register
                    x0 = u32x4{pair_lo(x0.x, x0.z), pair_hi(x0.x, x0.z), pair_lo(x0.y, x0.w), pair_hi(x0.y, x0.w)};
                xl[((ls * XV + vv) * 4 + gg) * bp + b] = x0;
            }
        }
        __syncthreads();
        // ---- this wave's share of sum_k x and sum_k x * offset_k of the chunk, in a fixed order ----
        {
            const int Q = (c1 - c0) * XV * 4, per = (Q + NW - 1) / NW;
            const int qlo = wave * per, qhi = min(qlo + per, Q);
            for (int b = 0; b < a.B; ++b) {
                float s1 = 0.f, s2 = 0.f;
                for (int q = qlo + lane; q < qhi; q += 64) {
                    const u32x4 v = xl[q * bp + b];
                    const bool odd = (q >> 2) & 1;  // operand index v within the segment
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        const float e = __uint_as_float(v[jj] << 16) + __uint_as_float(v[jj] & 0xFFFF0000u);
                        s1 += e;
                        if constexpr (R == 2) {
                            const int cls = ((odd ? 4 : 0) + jj) % 3;  // field position inside the 16-bit lane
                            s2 += e * (cls == 0 ? 128.f : (cls == 1 ? 32.f : 8.f));
                        }
                    }
                }
                s1 = wave_sum(s1);
                if constexpr (R == 2) s2 = wave_sum(s2);
                if (lane == 0) {
                    sums[b * 16 + wave] += s1;
                    sums[256 + b * 16 + wave] += s2;
                }
            }
        }
        // ---- the wave's segments of this chunk --------------------------------------------------
        // The load of the segment D - 1 ahead is unconditional (so that the number in flight stays
        // known and a use waits for its own load only); the arithmetic of a segment past the end
        // is skipped by a wave-uniform branch.  The ring is unrolled D times: moving registers
        // whose loads are still in flight would force a wait for them.
        for (; s < c1; s += step) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                fetch_next(w[(d + D - 1) % D]);
                if (s + d * KS < c1) gemv_segment<R, RG>(w[d], xlane + (s + d * KS - c0) * XV * 4 * bp, 4 * bp, acc);
            }
        }
    }
    __syncthreads();  // the staging area is reused by the reduction below

    // ---- reduction over the KS waves of a row block, in LDS ------------------------------------
    // part[wave][rg][lane] (float4), then ovf[row][b]; the sum is left in part[rw * KS][..]
    f32x4 *part = reinterpret_cast<f32x4 *>(xl);
    float *ovf = reinterpret_cast<float *>(part + NW * RG * 64);
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) part[(wave * RG + rg) * 64 + lane] = acc[rg];

    // ---- extra precision: sum of x over each row's overflow columns ---------------------------
    if constexpr (EP) {
        for (int r = wave; r < RW * ROWS; r += NW) {
            const int row = nb + r;
            float sx[16];
#pragma unroll
            for (int b = 0; b < 16; ++b) sx[b] = 0.f;
            if (row < a.N) {
                const int lo = a.row_ptr[row], hi = a.row_ptr[row + 1];
                for (int p = lo + lane; p < hi; p += 64) {
                    const int col = a.col_idx[p];
#pragma unroll
                    for (int b = 0; b < 16; ++b)
                        if (b < a.B) sx[b] += bf16_bits_to_float(a.x[(size_t)b * a.K + col]);
                }
            }
#pragma unroll
            for (int b = 0; b < 16; ++b) {
                if (b < a.B) {
#pragma unroll
                    for (int o = 32; o > 0; o >>= 1) sx[b] += __shfl_xor(sx[b], o, 64);
                }
                if (lane == 0) ovf[r * 16 + b] = sx[b];
            }
        }
    }
    __syncthreads();
    if (KS > 1) {
        for (int t = threadIdx.x; t < RW * RG * 64; t += blockDim.x) {
            const int q = t / (RG * 64), e = t % (RG * 64);
            f32x4 *base = part + (size_t)q * KS * RG * 64 + e;
            f32x4 sum = base[0];
            for (int kk = 1; kk < KS; ++kk) {
                const f32x4 pv = base[kk * RG * 64];
                sum.x += pv.x;
                sum.y += pv.y;
                sum.z += pv.z;
                sum.w += pv.w;
            }
            base[0] = sum;
        }
        __syncthreads();
    }

    // ---- epilogue: y[b, n] = alpha_n * (2^s * (codes.x [+ overflow]) - z_n * sum_k x) -----------
    // matrix-core output layout: lane = column b + 16 * (row / 4), component = row % 4
    constexpr float kScale = (float)(1 << (8 - R));
    for (int t = threadIdx.x; t < RW * ROWS * 16; t += blockDim.x) {
        const int b = t / (RW * ROWS), r = t % (RW * ROWS), row = nb + r;
        if (b >= a.B || row >= a.N) continue;
        const int q = r / ROWS, er = r % ROWS, rg = er >> 4, ri = er & 15;
        const float *tot = reinterpret_cast<const float *>(part + (size_t)q * KS * RG * 64);
        float dot = tot[(rg * 64 + b + 16 * (ri >> 2)) * 4 + (ri & 3)];
        float xsum = 0.f, xoff = 0.f;
        for (int wv = 0; wv < NW; ++wv) {
            xsum += sums[b * 16 + wv];
            xoff += sums[256 + b * 16 + wv];
        }
        if constexpr (R == 2) dot -= xoff;
        if constexpr (R == 4) dot -= 128.0f * xsum;
        if constexpr (EP) dot += ovf[r * 16 + b];
        const float al = bf16_bits_to_float(a.alpha[row]), z = bf16_bits_to_float(a.zero[row]);
        const float yv = al * (kScale * dot - z * xsum);
        a.y[(size_t)b * a.N + row] = (uint16_t)float_to_bf16_bits(yv);
    }
}

template <int R, int RG, int D>
static mq_status launch_gemv(const GemvArgs &a, int nw, int ks, hipStream_t st) {
    int bp = 1;
    while (bp < a.B) bp <<= 1;
    const int segk = 64 * (8 / R), segs = (a.KB + 63) / 64;
    const int seg_bytes = segk * 2 * bp;  // staged activations of one segment
    // Segments of x per staging chunk.  Everything at once when it fits 128 KB; otherwise chunks of
    // about kXChunk bytes that are a multiple of KS * D segments, so that the register ring of
    // every wave is in the same phase at each chunk boundary.
    // Segments of x per staging chunk.  Everything at once when it fits 128 KB; otherwise chunks of
    // about kXChunk bytes that are a multiple of KS * D segments, so that the register ring of
    // every wave is in the same phase at each chunk boundary.
    int chunk_segs = segs;
    if ((size_t)segs * seg_bytes > 131072) {
        while (ks > 1 && ks * D * seg_bytes > 131072) ks >>= 1;
        const int step = ks * D;
        chunk_segs = kXChunk / seg_bytes / step * step;
        if (chunk_segs < step) chunk_segs = step;
    }
    if (nw < ks) nw = ks;
    const int rw = nw / ks;
    const int blocks = (int)cdiv(a.N, 16 * RG * rw);
    const size_t xbytes = (size_t)chunk_segs * seg_bytes;
    const size_t red = (size_t)nw * RG * 64 * 16 + (size_t)rw * 16 * RG * 16 * 4;
    const size_t lds = kSumBytes + (xbytes > red ? xbytes : red);
    auto go = [&](auto kern) -> mq_status {
        if (lds > 65536 && hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return MQ_ERR_DEVICE;
        kern<<<dim3(blocks), dim3(64 * nw), lds, st>>>(a, bp, chunk_segs, ks);
        return launch_status();
    };
    return a.row_ptr ? go(gemv_kernel<R, RG, D, true>) : go(gemv_kernel<R, RG, D, false>);
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
    // K-split: enough waves in total (about 16 per compute unit) when there are few row blocks,
    // none when the rows alone provide them.  Workgroups have 8 waves (KS of them per row block),
    // or KS when that is larger.
    const int64_t segs = cdiv(kb, 64);
    const int64_t row_blocks = cdiv(N, 16 * rg);
    int ks = 1;
    while (ks < 16 && row_blocks * ks < 4096 && 2 * ks <= segs) ks <<= 1;
    const int nw = ks > 8 ? ks : 8;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
#define MQ_GEMV_CASE(R_, RG_, D_) \
    if (r == R_ && rg == RG_) return launch_gemv<R_, RG_, D_>(a, nw, ks, st);
    MQ_GEMV_CASE(2, 1, 4) MQ_GEMV_CASE(2, 2, 3) MQ_GEMV_CASE(2, 4, 2)
    MQ_GEMV_CASE(4, 1, 4) MQ_GEMV_CASE(4, 2, 3) MQ_GEMV_CASE(4, 4, 2)
    MQ_GEMV_CASE(8, 1, 4) MQ_GEMV_CASE(8, 2, 3) MQ_GEMV_CASE(8, 4, 2)
#undef MQ_GEMV_CASE
    return MQ_ERR_BITS;
}
