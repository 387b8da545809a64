// mq_slice: the slicing operator S(q, r) of section 3.2 (round half up at bit level as appendix A
// describes, clamp to 2^r - 1), optional packing to 8/r codes per byte, and the extra-precision
// overflow set of the errata section as a CSR list.  Integer-only and HBM-bound:
// 1 B read + r/8 B written per weight when packed.
#include <algorithm>

#include "mq_common.h"

namespace mq {

// Four int8 codes in a dword -> four r-bit codes in the same byte positions.
// Works on the two 16-bit lanes that hold bytes (0, 2) and (1, 3), so q + half cannot overflow.
__device__ __forceinline__ uint32_t slice4(uint32_t d, uint32_t half2, uint32_t s, uint32_t top2) {
    uint32_t even = d & 0x00FF00FFu;
    uint32_t odd = (d >> 8) & 0x00FF00FFu;
    even = ((even + half2) >> s) & 0x01FF01FFu;  // a 16-bit lane holds at most 255 + 64 < 512
    odd = ((odd + half2) >> s) & 0x01FF01FFu;
    // per-lane min with the top code
    const uint32_t e_lo = min(even & 0xFFFFu, top2 & 0xFFFFu), e_hi = min(even >> 16, top2 >> 16);
    const uint32_t o_lo = min(odd & 0xFFFFu, top2 & 0xFFFFu), o_hi = min(odd >> 16, top2 >> 16);
    return e_lo | (o_lo << 8) | (e_hi << 16) | (o_hi << 24);
}

__device__ __forceinline__ uint32_t slice1(uint32_t q, uint32_t s, uint32_t top) {
    const uint32_t half = (1u << s) >> 1;
    return min((q + half) >> s, top);
}

// 16 codes per thread.  MODE 0: one code per byte; MODE 4 / 2: packed nibbles / crumbs.
// s = 8 - r, top = the largest code (2^r - 1, or 2^r when the clamp is dropped for a dense
// extra-precision plane, which is then packed one bit wider than r).
template <int MODE>
__global__ __launch_bounds__(256) void slice_kernel(const uint8_t *__restrict__ Q, int64_t count, uint32_t s,
                                                    uint32_t top, uint8_t *__restrict__ out) {
    const uint32_t half = (1u << s) >> 1;
    const uint32_t half2 = half | (half << 16), top2 = top | (top << 16);
    const int64_t chunks = count >> 4;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < chunks; c += stride) {
        u32x4 d = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(Q) + c);
        u32x4 o;
        o.x = slice4(d.x, half2, s, top2);
        o.y = slice4(d.y, half2, s, top2);
        o.z = slice4(d.z, half2, s, top2);
        o.w = slice4(d.w, half2, s, top2);
        if constexpr (MODE == 0) {
            __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(out) + c);
        } else if constexpr (MODE == 4) {
            // bytes (b0 b1 b2 b3) of codes < 16 -> two bytes (b0 | b1 << 4), (b2 | b3 << 4)
            auto nib = [](uint32_t x) {
                uint32_t y = (x | (x >> 4)) & 0x00FF00FFu;  // byte0 | byte1 << 4 in each 16-bit lane
                return (y | (y >> 8)) & 0xFFFFu;
            };
            u32x2 p;
            p.x = nib(o.x) | (nib(o.y) << 16);
            p.y = nib(o.z) | (nib(o.w) << 16);
            __builtin_nontemporal_store(p, reinterpret_cast<u32x2 *>(out) + c);
        } else {
            // bytes of codes < 4 -> one byte b0 | b1 << 2 | b2 << 4 | b3 << 6
            auto crumb = [](uint32_t x) {
                uint32_t y = (x | (x >> 6)) & 0x000F000Fu;  // (b0 | b1 << 2) in each 16-bit lane
                return (y | (y >> 12)) & 0xFFu;
            };
            const uint32_t p = crumb(o.x) | (crumb(o.y) << 8) | (crumb(o.z) << 16) | (crumb(o.w) << 24);
            __builtin_nontemporal_store(p, reinterpret_cast<uint32_t *>(out) + c);
        }
    }
    // tail shorter than 16 codes: one thread, element by element (packing groups never straddle it
    // because count is a multiple of 8 / r in the packed modes)
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const int64_t done = chunks << 4;
        if constexpr (MODE == 0) {
            for (int64_t i = done; i < count; ++i) out[i] = (uint8_t)slice1(Q[i], s, top);
        } else {
            constexpr int PER = 8 / MODE;
            for (int64_t i = done; i < count; i += PER) {
                uint32_t b = 0;
                for (int j = 0; j < PER; ++j) b |= slice1(Q[i + j], s, top) << (MODE * j);
                out[i / PER] = (uint8_t)b;
            }
        }
    }
}

// Packed r-bit planes for bit-widths that do not divide 8 (r = 6, 3: the interpolated bit-widths of
// section 4.2): a little-endian bit stream, code k at stream bits [r k, r k + r).  32 codes per
// thread become exactly R dwords.
template <int R>
__global__ __launch_bounds__(256) void slice_stream_kernel(const uint8_t *__restrict__ Q, int64_t count, uint32_t s,
                                                           uint32_t top, uint8_t *__restrict__ out) {
    const uint32_t half = (1u << s) >> 1;
    const uint32_t half2 = half | (half << 16), top2 = top | (top << 16);
    const int64_t groups = count >> 5;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < groups; c += stride) {
        const u32x4 d0 = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(Q) + 2 * c);
        const u32x4 d1 = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(Q) + 2 * c + 1);
        uint32_t codes[8];  // four codes per dword, one per byte
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            codes[w] = slice4(d0[w], half2, s, top2);
            codes[4 + w] = slice4(d1[w], half2, s, top2);
        }
        uint32_t *dst = reinterpret_cast<uint32_t *>(out) + c * R;
        uint64_t acc = 0;
        int have = 0, word = 0;  // (compile-time after unrolling)
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            const uint64_t code = (codes[k >> 2] >> (8 * (k & 3))) & 0xFFu;
            acc |= code << have;
            have += R;
            if (have >= 32) {
                __builtin_nontemporal_store((uint32_t)acc, dst + word);
                ++word;
                acc >>= 32;
                have -= 32;
            }
        }
    }
    // tail shorter than 32 codes (a whole number of bytes, since count * R is a multiple of 8): one
    // thread, bit by bit
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const int64_t done = groups << 5;
        uint32_t acc = 0;
        int have = 0;
        int64_t byte = done * R / 8;
        for (int64_t i = done; i < count; ++i) {
            acc |= slice1(Q[i], s, top) << have;
            have += R;
            while (have >= 8) {
                out[byte++] = (uint8_t)acc;
                acc >>= 8;
                have -= 8;
            }
        }
    }
}

// ---- extra-precision overflow set -----------------------------------------------------------
// Number of codes >= threshold among the four bytes of d.
__device__ __forceinline__ int count_ge4(uint32_t d, uint32_t thr) {
    return ((d & 0xFFu) >= thr) + (((d >> 8) & 0xFFu) >= thr) + (((d >> 16) & 0xFFu) >= thr) + ((d >> 24) >= thr);
}

// One block per row: row_ptr[n + 1] = number of codes >= thr in row n (row_ptr[0] = 0).
__global__ __launch_bounds__(256) void overflow_count_kernel(const uint8_t *__restrict__ Q, int64_t K,
                                                             uint32_t thr, int32_t *__restrict__ row_ptr) {
    __shared__ int red[4];
    const int64_t n = blockIdx.x;
    const uint8_t *row = Q + n * K;
    int cnt = 0;
    if ((K & 15) == 0) {  // rows are whole 16-byte chunks (Q itself is 16-byte aligned)
        const u32x4 *row16 = reinterpret_cast<const u32x4 *>(row);
        for (int64_t c = threadIdx.x; c < (K >> 4); c += 256) {
            const u32x4 d = row16[c];
            cnt += count_ge4(d.x, thr) + count_ge4(d.y, thr) + count_ge4(d.z, thr) + count_ge4(d.w, thr);
        }
    } else {
        for (int64_t k = threadIdx.x; k < K; k += 256) cnt += row[k] >= thr;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x / 64] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        row_ptr[n + 1] = red[0] + red[1] + red[2] + red[3];
        if (n == 0) row_ptr[0] = 0;
    }
}

// Several products of one pass over the codes (mq_slice_multi): the packed int4 plane, the packed int2 plane and
// the per-row size of the overflow set of one of them, any subset.  A wave owns a row (rows are whole 16-byte
// chunks), so the count is a wave reduction and the planes leave as 8- and 4-byte pieces next to each other.
template <bool P4, bool P2, bool CNT>
__global__ __launch_bounds__(256) void slice_multi_kernel(const uint8_t *__restrict__ Q, int64_t N, int64_t K,
                                                          uint8_t *__restrict__ out4, uint8_t *__restrict__ out2,
                                                          uint32_t thr, int32_t *__restrict__ row_ptr) {
    const int lane = threadIdx.x & 63;
    const int64_t n = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;
    const u32x4 *row = reinterpret_cast<const u32x4 *>(Q + n * K);
    const int64_t chunks = K >> 4;
    constexpr uint32_t kHalf4 = 8u | (8u << 16), kTop4 = 15u | (15u << 16), kHalf2 = 32u | (32u << 16), kTop2 = 3u | (3u << 16);
    int cnt = 0;
    for (int64_t c = lane; c < chunks; c += 64) {
        const u32x4 d = __builtin_nontemporal_load(row + c);
        if constexpr (P4) {
            auto nib = [](uint32_t x) {
                const uint32_t y = (x | (x >> 4)) & 0x00FF00FFu;
                return (y | (y >> 8)) & 0xFFFFu;
            };
            u32x2 p;
            p.x = nib(slice4(d.x, kHalf4, 4, kTop4)) | (nib(slice4(d.y, kHalf4, 4, kTop4)) << 16);
            p.y = nib(slice4(d.z, kHalf4, 4, kTop4)) | (nib(slice4(d.w, kHalf4, 4, kTop4)) << 16);
            __builtin_nontemporal_store(p, reinterpret_cast<u32x2 *>(out4 + n * (K >> 1)) + c);
        }
        if constexpr (P2) {
            auto crumb = [](uint32_t x) {
                const uint32_t y = (x | (x >> 6)) & 0x000F000Fu;
                return (y | (y >> 12)) & 0xFFu;
            };
            const uint32_t p = crumb(slice4(d.x, kHalf2, 6, kTop2)) | (crumb(slice4(d.y, kHalf2, 6, kTop2)) << 8) |
                               (crumb(slice4(d.z, kHalf2, 6, kTop2)) << 16) | (crumb(slice4(d.w, kHalf2, 6, kTop2)) << 24);
            __builtin_nontemporal_store(p, reinterpret_cast<uint32_t *>(out2 + n * (K >> 2)) + c);
        }
        if constexpr (CNT) cnt += count_ge4(d.x, thr) + count_ge4(d.y, thr) + count_ge4(d.z, thr) + count_ge4(d.w, thr);
    }
    if constexpr (CNT) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
        if (lane == 0) {
            row_ptr[n + 1] = cnt;
            if (n == 0) row_ptr[0] = 0;
        }
    }
}

// Single block, in place: row_ptr[1..N] counts -> inclusive prefix sums; *nnz = total.  Every thread sums
// its run of counts, the 1024 sums are scanned inside the waves with lane shuffles and across the 16 waves
// through LDS (two barriers in all).
__global__ __launch_bounds__(1024) void overflow_scan_kernel(int32_t *__restrict__ row_ptr, int64_t N,
                                                             int64_t *__restrict__ nnz) {
    __shared__ int64_t wave_total[16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t per = (N + 1023) / 1024;
    const int64_t lo = 1 + threadIdx.x * per;
    const int64_t hi = lo + per < N + 1 ? lo + per : N + 1;
    int64_t sum = 0;
    for (int64_t i = lo; i < hi; ++i) sum += row_ptr[i];
    int64_t incl = sum;  // inclusive scan over the lanes of the wave
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int64_t up = __shfl_up(incl, o, 64);
        if (lane >= o) incl += up;
    }
    if (lane == 63) wave_total[wave] = incl;
    __syncthreads();
    int64_t before = 0;
    for (int w = 0; w < wave; ++w) before += wave_total[w];
    int64_t run = before + incl - sum;  // total of the threads before this one
    for (int64_t i = lo; i < hi; ++i) {
        run += row_ptr[i];
        row_ptr[i] = (int32_t)run;
    }
    if (threadIdx.x == 1023) *nnz = before + incl;
}

// One block per row: columns with code >= thr, ascending, written at row_ptr[n] (bounded by capacity).
__global__ __launch_bounds__(256) void overflow_fill_kernel(const uint8_t *__restrict__ Q, int64_t K,
                                                            uint32_t thr, const int32_t *__restrict__ row_ptr,
                                                            uint16_t *__restrict__ col_idx, int64_t capacity) {
    __shared__ int wave_tot[4];
    const int64_t n = blockIdx.x;
    const uint8_t *row = Q + n * K;
    int64_t base = row_ptr[n];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int64_t k0 = 0; k0 < K; k0 += 256) {
        const int64_t k = k0 + threadIdx.x;
        const bool hit = k < K && row[k] >= thr;
        const uint64_t ballot = __ballot(hit);
        if (lane == 0) wave_tot[wave] = __popcll(ballot);
        __syncthreads();
        int before = __popcll(ballot & ((1ull << lane) - 1ull));
        for (int w = 0; w < wave; ++w) before += wave_tot[w];
        const int total = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
        if (hit && base + before < capacity) col_idx[base + before] = (uint16_t)k;
        base += total;
        __syncthreads();
    }
}

// Same result for rows that are whole 16-byte chunks: a thread takes 16 consecutive columns, the
// position of its first hit comes from a prefix sum over the hit counts of the threads before it.
__global__ __launch_bounds__(256) void overflow_fill16_kernel(const uint8_t *__restrict__ Q, int64_t K,
                                                              uint32_t thr, const int32_t *__restrict__ row_ptr,
                                                              uint16_t *__restrict__ col_idx, int64_t capacity) {
    __shared__ int wave_tot[4];
    const int64_t n = blockIdx.x;
    const u32x4 *row16 = reinterpret_cast<const u32x4 *>(Q + n * K);
    int64_t base = row_ptr[n];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t chunks = K >> 4;
    for (int64_t c0 = 0; c0 < chunks; c0 += 256) {
        const int64_t c = c0 + threadIdx.x;
        uint32_t hits = 0;  // bit j: column 16 c + j overflows
        if (c < chunks) {
            const u32x4 d = row16[c];
#pragma unroll
            for (int w = 0; w < 4; ++w)
#pragma unroll
                for (int b = 0; b < 4; ++b) hits |= (uint32_t)(((d[w] >> (8 * b)) & 0xFFu) >= thr) << (4 * w + b);
        }
        const int cnt = __popc(hits);
        int incl = cnt;  // inclusive prefix sum over the lanes of the wave
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        int before = incl - cnt;
        for (int w = 0; w < wave; ++w) before += wave_tot[w];
        const int total = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
        int64_t pos = base + before;
        while (hits) {
            const int j = __ffs(hits) - 1;
            hits &= hits - 1;
            if (pos < capacity) col_idx[pos] = (uint16_t)(c * 16 + j);
            ++pos;
        }
        base += total;
        __syncthreads();
    }
}

}  // namespace mq

extern "C" mq_status mq_slice(const uint8_t *Q, int64_t N, int64_t K, int r, uint32_t flags, uint8_t *out,
                              const mq_overflow *ovf, void *hip_stream) {
    using namespace mq;
    if (N < 0 || K < 0) return MQ_ERR_SHAPE;
    if (r < 1 || r > 8) return MQ_ERR_BITS;
    const bool packed = flags & MQ_FLAG_PACKED, ep = flags & MQ_FLAG_EXTRA_PRECISION;
    const bool dense_ep = flags & MQ_FLAG_EP_DENSE;
    if (dense_ep && !(packed && ep)) return MQ_ERR_BITS;
    const int rp = dense_ep ? r + 1 : r;  // bits per stored code
    if (packed && !(rp == 8 || rp == 6 || rp == 4 || rp == 3 || rp == 2)) return MQ_ERR_BITS;
    if (packed && ((K * rp) % 8) != 0) return MQ_ERR_ALIGN;  // rows are whole bytes
    if (ep && !dense_ep) {
        if (!ovf) return MQ_ERR_NULL;
        if (N > 0 && (!ovf->row_ptr || !ovf->nnz || (ovf->capacity > 0 && !ovf->col_idx))) return MQ_ERR_NULL;
        if (ovf->capacity < 0) return MQ_ERR_CAPACITY;
        if (K > 65536 || N > 0x7FFFFFFE || (N > 0 && K > 0x7FFFFFFF / N)) return MQ_ERR_SHAPE;
    }
    if (N == 0 || K == 0) {
        return MQ_OK;
    }
    if (!Q || !out) return MQ_ERR_NULL;
    if (!aligned16(Q) || !aligned16(out)) return MQ_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int64_t count = N * K;
    const int64_t chunks = count >> 4;
    int64_t blocks = cdiv(chunks > 0 ? chunks : 1, 256);
    if (blocks > 256 * 32) blocks = 256 * 32;  // grid-stride beyond 32 blocks per CU
    const uint32_t sh = (uint32_t)(8 - r);
    const uint32_t top = dense_ep ? (1u << r) : (1u << r) - 1;  // a dense extra-precision plane keeps code 2^r
    if (packed && (rp == 6 || rp == 3)) {
        int64_t sblocks = cdiv(std::max<int64_t>(count >> 5, 1), 256);
        if (sblocks > 256 * 32) sblocks = 256 * 32;
        if (rp == 6)
            slice_stream_kernel<6><<<dim3((unsigned)sblocks), dim3(256), 0, st>>>(Q, count, sh, top, out);
        else
            slice_stream_kernel<3><<<dim3((unsigned)sblocks), dim3(256), 0, st>>>(Q, count, sh, top, out);
    } else if (!packed || rp == 8) {
        slice_kernel<0><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(Q, count, sh, top, out);
    } else if (rp == 4) {
        slice_kernel<4><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(Q, count, sh, top, out);
    } else {
        slice_kernel<2><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(Q, count, sh, top, out);
    }
    if (ep && !dense_ep) {
        const uint32_t half = (1u << (8 - r)) >> 1;
        const uint32_t thr = r == 8 ? 256u : 256u - half;  // r = 8: nothing overflows
        overflow_count_kernel<<<dim3((unsigned)N), dim3(256), 0, st>>>(Q, K, thr, ovf->row_ptr);
        overflow_scan_kernel<<<dim3(1), dim3(1024), 0, st>>>(ovf->row_ptr, N, ovf->nnz);
        if ((K & 15) == 0)
            overflow_fill16_kernel<<<dim3((unsigned)N), dim3(256), 0, st>>>(Q, K, thr, ovf->row_ptr, ovf->col_idx,
                                                                           ovf->capacity);
        else
            overflow_fill_kernel<<<dim3((unsigned)N), dim3(256), 0, st>>>(Q, K, thr, ovf->row_ptr, ovf->col_idx,
                                                                         ovf->capacity);
    }
    return launch_status();
}

extern "C" mq_status mq_slice_multi(const uint8_t *Q, int64_t N, int64_t K, const int *rs, int nr, uint32_t flags,
                                    uint8_t *const *out, int ovf_index, const mq_overflow *ovf, void *hip_stream) {
    using namespace mq;
    if (N < 0 || K < 0) return MQ_ERR_SHAPE;
    if (!rs || nr < 1 || nr > 3) return MQ_ERR_BITS;
    const bool ep = flags & MQ_FLAG_EXTRA_PRECISION;
    if ((flags & MQ_FLAG_EP_DENSE) || (ep && (ovf_index < 0 || ovf_index >= nr)) || (!ep && ovf_index >= 0 && ovf)) return MQ_ERR_BITS;
    for (int i = 0; i < nr; ++i) {
        if (rs[i] != 8 && rs[i] != 6 && rs[i] != 4 && rs[i] != 3 && rs[i] != 2) return MQ_ERR_BITS;
        for (int j = 0; j < i; ++j)
            if (rs[j] == rs[i]) return MQ_ERR_BITS;
        if ((K * rs[i]) % 8 != 0) return MQ_ERR_ALIGN;
    }
    if (ep) {
        if (!ovf) return MQ_ERR_NULL;
        if (N > 0 && (!ovf->row_ptr || !ovf->nnz || (ovf->capacity > 0 && !ovf->col_idx))) return MQ_ERR_NULL;
        if (ovf->capacity < 0) return MQ_ERR_CAPACITY;
        if (K > 65536 || N > 0x7FFFFFFE || (N > 0 && K > 0x7FFFFFFF / N)) return MQ_ERR_SHAPE;
    }
    if (N == 0 || K == 0) return MQ_OK;
    if (!Q || !out) return MQ_ERR_NULL;
    for (int i = 0; i < nr; ++i) {
        if (!out[i]) return MQ_ERR_NULL;
        if (!aligned16(out[i])) return MQ_ERR_ALIGN;
    }
    if (!aligned16(Q)) return MQ_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    // The int4 and int2 planes and the size of the overflow set come out of one pass over the codes when rows are whole
    // 16-byte chunks; every other plane (and every plane of a ragged matrix) takes the single-plane route.
    uint8_t *p4 = nullptr, *p2 = nullptr;
    bool fused[3] = {false, false, false};
    if ((K & 15) == 0)
        for (int i = 0; i < nr; ++i) {
            if (rs[i] == 4) p4 = out[i], fused[i] = true;
            if (rs[i] == 2) p2 = out[i], fused[i] = true;
        }
    const int r_ovf = ep ? rs[ovf_index] : 8;
    const bool count_fused = ep && (K & 15) == 0 && (p4 || p2);
    for (int i = 0; i < nr; ++i) {
        if (fused[i]) continue;
        const bool with_list = ep && i == ovf_index && !count_fused;
        const mq_status s = mq_slice(Q, N, K, rs[i], MQ_FLAG_PACKED | (with_list ? MQ_FLAG_EXTRA_PRECISION : 0), out[i],
                                     with_list ? ovf : nullptr, hip_stream);
        if (s != MQ_OK) return s;
    }
    if (p4 || p2) {
        const uint32_t half = (1u << (8 - r_ovf)) >> 1, thr = r_ovf == 8 ? 256u : 256u - half;
        const dim3 grid((unsigned)cdiv(N, 4)), block(256);
        int32_t *rp = count_fused ? ovf->row_ptr : nullptr;
#define MQ_SM(P4_, P2_) \
    if ((p4 != nullptr) == P4_ && (p2 != nullptr) == P2_) { \
        if (count_fused) slice_multi_kernel<P4_, P2_, true><<<grid, block, 0, st>>>(Q, N, K, p4, p2, thr, rp); \
        else slice_multi_kernel<P4_, P2_, false><<<grid, block, 0, st>>>(Q, N, K, p4, p2, thr, rp); \
    }
        MQ_SM(true, true) MQ_SM(true, false) MQ_SM(false, true)
#undef MQ_SM
        if (count_fused) {
            overflow_scan_kernel<<<dim3(1), dim3(1024), 0, st>>>(ovf->row_ptr, N, ovf->nnz);
            overflow_fill16_kernel<<<dim3((unsigned)N), dim3(256), 0, st>>>(Q, K, thr, ovf->row_ptr, ovf->col_idx, ovf->capacity);
        }
    }
    return launch_status();
}
