// The sparse additions of the extra-precision GEMV (errata section: weights whose r-bit code rounds up to 2^r
// carry "an extra bit"; the section asks for sparse additions of those bits on top of the dense low-bit plane):
//     osum[b, n] = sum over the overflow columns k of row n of x[b, k]
// for every output, written as a 16-bit number (ovf_sum_pack: half precision of the sum / 256) into the output
// buffer y itself, where the GEMV kernel that follows on the same stream picks it up in its epilogue
// (y[b, n] = alpha_n (2^s (codes . x + osum) - z_n sum x)) before it overwrites y.  No scratch memory is needed
// that way; the price is that the overflow sum is rounded to 11 significant bits on the way (2^-11 relative, on a
// term that is a few per cent of the output at the paper's overflow densities; exact whenever the sum is a small
// integer, e.g. for one-hot activations).
//
// The list is a CSR over output channels with ascending uint16 columns.  Sixteen neighbouring lanes own a row
// at a time (rows are handed out inside a workgroup through an LDS counter, so uneven rows balance) and read its
// columns as 16-byte pieces, eight per lane, 256 contiguous bytes per step.  The activations sit in LDS
// TRANSPOSED, xT[k][b] with the BP batch entries of a column next to each other, so that one entry costs one
// LDS read of 2 BP bytes and BP additions, and no lane ever waits for another: the sixteen partial sums of a row
// meet in a butterfly at its end.  Entries outside the row (a 16-byte piece may straddle its ends) point at a row
// of zeros behind the last column instead of being masked.  When K * B activations do not fit, the batch is
// processed BP entries at a time (the workgroup's part of the list then comes out of L2 again).
#include <algorithm>

#include "mq_gemv.h"

namespace mq {

namespace {

struct OvfArgs {
    const uint16_t *x;        // [B, K] bf16
    const int32_t *row_ptr;   // [N + 1]
    const uint16_t *col_idx;  // [cap]
    uint16_t *y;              // [B, N] bf16: receives the sums
    int B, N, K;
    int cap;                  // entries col_idx holds
    int rows_per_wg;
};

// xT row r lives at slot r ^ (r / 8 % 8) (BP > 1): the staging writes of a wave (rows 8 apart) then spread over the banks
template <int BP>
__device__ __forceinline__ uint32_t xt_slot(uint32_t r) { return BP == 1 ? r : (r ^ ((r >> 3) & 7u)); }

template <int BP>
__global__ __launch_bounds__(1024) void ovf_sum_kernel(OvfArgs a) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    constexpr int ROWB = 2 * BP;  // bytes of one xT row
    const int tid = threadIdx.x, lane16 = tid & 15, grp = tid >> 4, ngrp = blockDim.x >> 4;
    const int R0 = blockIdx.x * a.rows_per_wg, R1 = min(R0 + a.rows_per_wg, a.N);
    const int KZ = (a.K + 7) & ~7;  // the row of zeros (and the padding up to it)
    int *rp = reinterpret_cast<int *>(lds + (size_t)(KZ + 8) * ROWB);  // [rows of the workgroup + 1], behind xT
    // (columns are read in whole dwords: with an odd capacity the last dword reaches two bytes past the last entry,
    // inside the same aligned dword; that half is never used)
    const __amdgpu_buffer_rsrc_t rcol = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.col_idx), 0, (int)std::min<int64_t>(((int64_t)a.cap * 2 + 3) & ~3ll, 0x7FFFFFFF), 0x00020000);
    typedef __bf16 bfp __attribute__((ext_vector_type(2)));
    // acc + one half of a bf16 pair: a dot product with (1, 0) or (0, 1).  The selectors are kept in vector registers
    // (as literal operands of the packed instruction they were observed to select the wrong half)
    uint32_t sel_lo = 0x00003F80u, sel_hi = 0x3F800000u;
    asm volatile("" : "+v"(sel_lo), "+v"(sel_hi));
    auto add_lo = [&](uint32_t v, float acc) {
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bfp, v), __builtin_bit_cast(bfp, sel_lo), acc, false);
    };
    auto add_hi = [&](uint32_t v, float acc) {
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bfp, v), __builtin_bit_cast(bfp, sel_hi), acc, false);
    };

    for (int b0 = 0; b0 < a.B; b0 += BP) {
        if (b0 > 0) __syncthreads();  // the previous batch group is done with xT
        // ---- stage xT for batch entries [b0, b0 + BP) ----------------------------------------------------
        // A thread takes 8 consecutive k of a pair of batch entries (two 16-byte loads; sixteen neighbouring
        // threads read 256 contiguous bytes of a batch row) and writes eight dwords (entry 2 p, entry 2 p + 1) of
        // eight xT rows.  BP = 1: xT is x itself.
        {
            auto load8 = [&](int b, int k) -> u32x4 {  // x[b, k .. k + 8), zeros past the batch or the row
                u32x4 v = {0u, 0u, 0u, 0u};
                if (b < a.B && k + 8 <= a.K) {
                    v = *reinterpret_cast<const u32x4 *>(a.x + (size_t)b * a.K + k);
                } else if (b < a.B && k < a.K) {  // ragged end of a row
                    uint32_t t[8];
                    for (int j = 0; j < 8; ++j) t[j] = k + j < a.K ? a.x[(size_t)b * a.K + k + j] : 0u;
                    v = u32x4{t[0] | (t[1] << 16), t[2] | (t[3] << 16), t[4] | (t[5] << 16), t[6] | (t[7] << 16)};
                }
                return v;
            };
            if constexpr (BP == 1) {
                for (int k = tid * 8; k < KZ + 8; k += (int)blockDim.x * 8)
                    *reinterpret_cast<u32x4 *>(lds + (size_t)k * 2) = load8(b0, k);
            } else {
                constexpr int PAIRS = BP / 2;
                const int kgl = tid & 15, pr = (tid >> 4) % PAIRS, kgo = (tid >> 4) / PAIRS;
                const int kg_step = 16 * ((int)(blockDim.x >> 4) / PAIRS);
                for (int kg = kgo * 16 + kgl; kg * 8 < KZ + 8; kg += kg_step) {
                    const int k = kg * 8;
                    const u32x4 v0 = load8(b0 + 2 * pr, k), v1 = load8(b0 + 2 * pr + 1, k);
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const uint32_t d = (j & 1) ? __builtin_amdgcn_perm(v1[j >> 1], v0[j >> 1], 0x07060302u)
                                                   : __builtin_amdgcn_perm(v1[j >> 1], v0[j >> 1], 0x05040100u);
                        *reinterpret_cast<uint32_t *>(lds + xt_slot<BP>((uint32_t)(k + j)) * ROWB + pr * 4) = d;
                    }
                }
            }
        }
        // the list positions of the workgroup's rows, clamped to what col_idx holds (once: they do not depend on the batch group)
        if (b0 == 0)
            for (int t = tid; t <= R1 - R0; t += (int)blockDim.x) rp[t] = min(a.row_ptr[R0 + t], a.cap);
        __syncthreads();

        // ---- walk: a group of 16 lanes per row, rows dealt round-robin to the groups ---------------------------
        // A row's columns are requested four windows (4 x 128 entries) at a time, and the first four windows of the
        // group's next row before the current row is summed, so that a group waits for memory once, not per window.
        constexpr int W = 4;
        u32x4 cur[W], nxt[W];
        auto request = [&](u32x4 (&dst)[W], int p0, int p1, int first_window) {
#pragma unroll
            for (int w = 0; w < W; ++w) {
                const int idx0 = (p0 & ~7) + (first_window + w) * 128 + lane16 * 8;
                // (a window past the row is not requested: the offset is moved out of range, which returns zeros)
                const uint32_t off = idx0 < p1 ? (uint32_t)idx0 * 2u : 0x80000000u;
                dst[w] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rcol, off, 0, 0));
            }
        };
        int rl = grp;  // row of the workgroup this group is at
        if (rl < R1 - R0) request(cur, rp[rl], rp[rl + 1], 0);
        while (rl < R1 - R0) {
            const int row = R0 + rl;
            const int p0 = rp[rl], p1 = rp[rl + 1];
            const int rn = rl + ngrp;
            if (rn < R1 - R0) request(nxt, rp[rn], rp[rn + 1], 0);
            float s[BP];
#pragma unroll
            for (int b = 0; b < BP; ++b) s[b] = 0.f;
            for (int w0 = 0; (p0 & ~7) + w0 * 128 < p1; w0 += W) {
                if (w0 > 0) request(cur, p0, p1, w0);  // (rows of more than 512 entries: these waits are not hidden)
#pragma unroll
                for (int w = 0; w < W; ++w) {
                    const int idx0 = (p0 & ~7) + (w0 + w) * 128 + lane16 * 8;
                    if ((p0 & ~7) + (w0 + w) * 128 >= p1) break;   // uniform over the group
                    const u32x4 cv = cur[w];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const int idx = idx0 + j;
                        const uint32_t col = (j & 1) ? (cv[j >> 1] >> 16) : (cv[j >> 1] & 0xFFFFu);
                        const uint32_t r = (idx >= p0 && idx < p1) ? col : (uint32_t)KZ;
                        const uint8_t *src = lds + xt_slot<BP>(r) * ROWB;
                        if constexpr (BP == 16) {
                            const u32x4 v0 = *reinterpret_cast<const u32x4 *>(src), v1 = *reinterpret_cast<const u32x4 *>(src + 16);
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                s[2 * q] = add_lo(v0[q], s[2 * q]);
                                s[2 * q + 1] = add_hi(v0[q], s[2 * q + 1]);
                                s[8 + 2 * q] = add_lo(v1[q], s[8 + 2 * q]);
                                s[8 + 2 * q + 1] = add_hi(v1[q], s[8 + 2 * q + 1]);
                            }
                        } else if constexpr (BP == 8) {
                            const u32x4 v0 = *reinterpret_cast<const u32x4 *>(src);
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                s[2 * q] = add_lo(v0[q], s[2 * q]);
                                s[2 * q + 1] = add_hi(v0[q], s[2 * q + 1]);
                            }
                        } else if constexpr (BP == 4) {
                            const u32x2 v0 = *reinterpret_cast<const u32x2 *>(src);
                            s[0] = add_lo(v0.x, s[0]);
                            s[1] = add_hi(v0.x, s[1]);
                            s[2] = add_lo(v0.y, s[2]);
                            s[3] = add_hi(v0.y, s[3]);
                        } else if constexpr (BP == 2) {
                            const uint32_t v0 = *reinterpret_cast<const uint32_t *>(src);
                            s[0] = add_lo(v0, s[0]);
                            s[1] = add_hi(v0, s[1]);
                        } else {
                            s[0] += bf16_bits_to_float(*reinterpret_cast<const uint16_t *>(src));
                        }
                    }
                }
            }
            // the sixteen partial sums of every batch entry meet: halve the set of entries a lane keeps while
            // more than one is left, then plain butterflies; lane l ends with the total of entry l / (16 / BP)
            int V = BP;
#pragma unroll
            for (int m = 8; m >= 1; m >>= 1) {
                if (V > 1) {
                    const int H = V / 2;
                    const bool upper = (lane16 & m) != 0;
#pragma unroll
                    for (int j = 0; j < BP / 2; ++j) {
                        if (j < H) {
                            const float keep = upper ? s[j + H] : s[j], send = upper ? s[j] : s[j + H];
                            s[j] = keep + __shfl_xor(send, m, 64);
                        }
                    }
                    V = H;
                } else {
                    s[0] += __shfl_xor(s[0], m, 64);
                }
            }
            constexpr int DUP = 16 / BP;  // lanes that hold the same total
            const int b = b0 + lane16 / DUP;
            if ((lane16 % DUP) == 0 && b < a.B) a.y[(size_t)b * a.N + row] = ovf_sum_pack(s[0]);
            // next row of this group: its first windows are on their way
            rl = rn;
#pragma unroll
            for (int w = 0; w < W; ++w) cur[w] = nxt[w];
        }
    }
}

}  // namespace

// Enqueues the kernel above: y[b, n] <- ovf_sum_pack(sum of x[b, k] over the overflow columns of row n).  K <= 65536.
mq_status launch_overflow_sums(const uint16_t *x, const int32_t *row_ptr, const uint16_t *col_idx, int64_t capacity,
                               int64_t B, int64_t N, int64_t K, uint16_t *y, hipStream_t st) {
    if (N == 0) return MQ_OK;
    OvfArgs a;
    a.x = x;
    a.row_ptr = row_ptr;
    a.col_idx = col_idx;
    a.y = y;
    a.B = (int)B;
    a.N = (int)N;
    a.K = (int)K;
    a.cap = (int)std::min<int64_t>(capacity, 0x3FFFFFFF);
    // batch entries per pass: the largest power of two (at most the padded batch) whose transposed activations fit
    const size_t rows = (size_t)((K + 7) & ~7) + 8;  // columns, padding, the row of zeros
    int bp = 1;
    while (bp < B) bp <<= 1;
    while (bp > 1 && rows * 2 * bp > 150 * 1024) bp >>= 1;
    if (rows * 2 * bp > 150 * 1024) return MQ_ERR_SHAPE;  // (cannot happen for K <= 65536)
    const size_t xt_bytes = rows * 2 * bp;
    // one workgroup of 16 waves per compute unit and pass when the activations are large, more when they are small
    const int per_cu = xt_bytes > 72 * 1024 ? 1 : 2;
    int grid = (int)std::min<int64_t>(256 * per_cu, cdiv(N, 64));
    if (grid < 1) grid = 1;
    a.rows_per_wg = (int)cdiv(N, grid);
    grid = (int)cdiv(N, a.rows_per_wg);
    const size_t lds = xt_bytes + ((size_t)a.rows_per_wg + 1) * 4;
    if (lds > 160 * 1024) return MQ_ERR_SHAPE;  // (cannot happen: N < 2^31 rows over 256 workgroups would need K * B beyond the cap above)
    auto go = [&](auto kern) -> mq_status {
        if (lds > 65536 && hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                               (int)lds) != hipSuccess)
            return MQ_ERR_DEVICE;
        kern<<<dim3(grid), dim3(1024), lds, st>>>(a);
        return launch_status();
    };
    switch (bp) {
        case 16: return go(ovf_sum_kernel<16>);
        case 8: return go(ovf_sum_kernel<8>);
        case 4: return go(ovf_sum_kernel<4>);
        case 2: return go(ovf_sum_kernel<2>);
        default: return go(ovf_sum_kernel<1>);
    }
}

}  // namespace mq
