// mq_gemv_sliced for small batches (B <= 4) on int4 / int2 planes: the activations of a wave's K
// slice live in registers, so the hot loop touches LDS only to change the lane layout of the weight
// lines it streams (section 1: decode is bound by moving the weights out of HBM).
//
// Products run on v_mfma_f32_4x4x4_16b_bf16 with an A-operand broadcast (cbsz = 2): the 64 lanes are
// four k-groups g of 16 lanes; lane (g, i) holds 16 bytes of weight row i as the B operand (column =
// its own row), and block `abid` of its k-group (lanes 16 g + 4 abid + b, b = batch entry) supplies
// the A operand, four activations per batch entry.  One register pair of activations therefore
// serves four products (abid = 0..3) and a whole K slice of 2048 int2 codes costs 64 registers; the
// result of a product is y[b] of the lane's own row in accumulator register b.  Nothing is shared
// between lanes until a row block is finished.
//
// A wave owns NL consecutive 128-byte lines of every row (its K slice, index ks) and walks over row
// blocks of 16 rows ("visits"); the KS slices of a row block sit in one workgroup and meet in LDS at
// the end.  Weight lines are fetched as whole 128-byte lines by eight neighbouring lanes through
// buffer loads (a request past the wave's last visit is out of range: it returns zeros and costs no
// traffic, so the number of loads in flight is the same in every iteration), two visits ahead, and
// change lanes through a 2 KB LDS tile per wave one step before they are used.
//
// Codes become bf16 numbers with one AND-OR per two codes: a field at mantissa bits 0-1 / 2-3 / 4-5
// under the exponent of 128 / 32 / 8 reads as 128 + c, 32 + c, 8 + c.  The offsets leave in the
// epilogue through sum_k x_k * offset_k, which every workgroup computes once next to sum_k x_k (the
// zero-point term).
#include <algorithm>
#include <cstdlib>

#include "mq_gemv.h"

namespace mq {

namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kE128 = 0x43004300u, kE32 = 0x42004200u, kE8 = 0x41004100u;  // (128,128) (32,32) (8,8)
constexpr uint32_t kOutOfRange = 0x80000000u;
constexpr int kSumsBytes = 1024;  // float [16 waves][4 batch entries][2]
constexpr int kTileBytes = 2048;  // per wave
constexpr int kXPad = 32;         // row pitch of the staged activations = whole 1 KB blocks + this (bank shift per batch entry)
typedef __attribute__((address_space(3))) void *lds_ptr;

template <int ABID>
__device__ __forceinline__ f32x4 mfma_quad(const u32x2 &x, uint32_t w0, uint32_t w1, const f32x4 &c) {
    return __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(s16x4, x), __builtin_bit_cast(s16x4, u32x2{w0, w1}),
                                                  c, 2, ABID, 0);
}

// (v & mask) | magic; selected as one v_and_or_b32 when the mask is scalar and the magic a register
__device__ __forceinline__ uint32_t and_or(uint32_t v, uint32_t mask_s, uint32_t magic_v) {
    return (v & mask_s) | magic_v;
}

struct QuadConsts {
    uint32_t m0, m1, m2;     // scalar: field masks
    uint32_t e128, e32, e8;  // vector: exponent patterns
};

template <int R>
__device__ __forceinline__ QuadConsts quad_consts() {
    QuadConsts c;
    c.m0 = R == 2 ? 0x00030003u : 0x000F000Fu;
    c.m1 = 0x000C000Cu;
    c.m2 = 0x00300030u;
    c.e128 = kE128;
    c.e32 = kE32;
    c.e8 = kE8;
    asm volatile("" : "+s"(c.m0), "+s"(c.m1), "+s"(c.m2));
    asm volatile("" : "+v"(c.e128), "+v"(c.e32), "+v"(c.e8));
    return c;
}

// One dword of a lane's piece against the activations that belong to it.  `dwi` = index of the
// dword among the eight of the lane's two pieces of the line; xr = the line's activation registers.
template <int R, int XP>
__device__ __forceinline__ void quad_dword(uint32_t d, int dwi, const u32x2 (&xr)[XP], const QuadConsts &qc,
                                           f32x4 &acc0, f32x4 &acc1) {
    if constexpr (R == 2) {
        // codes j and j + 8 of the dword share a register; quad u = codes (2u, 2u + 8, 2u + 1, 2u + 9)
        const uint32_t d6 = d >> 6, d12 = d >> 12;
        const u32x2 &x = xr[dwi];
        acc0 = mfma_quad<0>(x, and_or(d, qc.m0, qc.e128), and_or(d, qc.m1, qc.e32), acc0);
        acc1 = mfma_quad<1>(x, and_or(d, qc.m2, qc.e8), and_or(d6, qc.m0, qc.e128), acc1);
        acc0 = mfma_quad<2>(x, and_or(d6, qc.m1, qc.e32), and_or(d6, qc.m2, qc.e8), acc0);
        acc1 = mfma_quad<3>(x, and_or(d12, qc.m0, qc.e128), and_or(d12, qc.m1, qc.e32), acc1);
    } else {
        // codes j and j + 4 of the dword share a register; quad u = codes (2u, 2u + 4, 2u + 1, 2u + 5);
        // two dwords share an activation register pair
        const u32x2 &x = xr[dwi >> 1];
        const uint32_t r0 = and_or(d, qc.m0, qc.e128), r1 = and_or(d >> 4, qc.m0, qc.e128);
        const uint32_t r2 = and_or(d >> 8, qc.m0, qc.e128), r3 = and_or(d >> 12, qc.m0, qc.e128);
        if (dwi & 1) {
            acc0 = mfma_quad<2>(x, r0, r1, acc0);
            acc1 = mfma_quad<3>(x, r2, r3, acc1);
        } else {
            acc0 = mfma_quad<0>(x, r0, r1, acc0);
            acc1 = mfma_quad<1>(x, r2, r3, acc1);
        }
    }
}

// R = bits per code (4 or 2), NL = 128-byte lines of a row per K slice.  Workgroup = KS * RW waves;
// wave (ks, rw) = (wave % KS, wave / KS) takes slice ks of row blocks rb0 + rw, rb0 + rw + RW, ...
// of the CH row blocks [rb0, rb0 + CH) that the workgroup owns.
template <int R, int NL>
__global__ __launch_bounds__(512) void gemv_quad_kernel(GemvArgs a, int KS, int RW, int CH) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    constexpr int CPD = 32 / R;      // codes per dword
    constexpr int QD = CPD / 4;      // quads per dword
    constexpr int XP = 2 * QD;       // activation register pairs per line
    constexpr int CPB = 8 / R;       // codes per byte

    const int tid = threadIdx.x, lane = tid & 63, nthreads = blockDim.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int NW = nthreads >> 6;
    const int ks = wave % KS, rw = wave / KS;
    const int li = lane >> 3, lc = lane & 7;       // fetch: row li (+ 8), piece lc of the line
    const int i = lane & 15, g = lane >> 4;        // compute: row i, pieces g and g + 4
    const int t = (lane >> 2) & 3, b = lane & 3;   // activations: block t, batch entry b

    const int NRB = (a.N + 15) >> 4;
    const int rb0 = blockIdx.x * CH, rb1 = min(rb0 + CH, NRB);
    const int row0 = rb0 * 16;
    const int rows_wg = min(rb1 * 16, a.N) - row0;  // >= 1 (the grid covers exactly the row blocks)
    const int line0 = ks * NL;

    float *sums = reinterpret_cast<float *>(lds);
    uint8_t *tile = lds + kSumsBytes + wave * kTileBytes;
    f32x4 *ypart = reinterpret_cast<f32x4 *>(lds + kSumsBytes + NW * kTileBytes);  // [KS][CH * 16]
    // activations of the whole workgroup: row b at b * xpitch, natural order, zero-filled up to a whole 512-k block
    const int kblocks = (a.K + 511) >> 9;
    const int xpitch = kblocks * 1024 + kXPad;
    uint8_t *xbuf = lds + kSumsBytes + NW * kTileBytes + KS * CH * 16 * (int)sizeof(f32x4);

    const __amdgpu_buffer_rsrc_t rwt = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(a.packed + (size_t)row0 * a.KB), 0, (int)((uint32_t)rows_wg * (uint32_t)a.KB), 0x00020000);
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.x), 0, (int)((uint32_t)a.B * (uint32_t)a.K * 2u), 0x00020000);

    // ---- activations -> LDS (direct loads, 1 KB = 512 k of one batch entry per wave instruction) --------
    for (int j = wave; j < a.B * kblocks; j += NW) {
        const int bj = j / kblocks, kb = j - bj * kblocks;
        const int k = kb * 512 + lane * 8;
        const uint32_t vo = k < a.K ? ((uint32_t)bj * (uint32_t)a.K + (uint32_t)k) * 2u : kOutOfRange;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_ptr)(xbuf + bj * xpitch + kb * 1024), 16, vo, 0, 0, 0);
    }

    // ---- weight ring: raw[slot][line][first / second eight rows], two visits deep ---------------------
    u32x4 raw[2][NL][2];
    uint32_t piece_off[NL];  // byte offset of the lane's piece inside a row (clamped into the row)
#pragma unroll
    for (int ln = 0; ln < NL; ++ln) piece_off[ln] = (uint32_t)min((line0 + ln) * 128 + lc * 16, a.KB - 16);
    const int nv = max(0, (rb1 - rb0 - rw + RW - 1) / RW);  // visits of this wave (wave-uniform)
    auto issue = [&](int visit, u32x4 (&dst)[2], int ln) {
        const int rb = rb0 + rw + visit * RW;
        // bit 31 of the offset set when the visit does not exist (arithmetic on purpose: a branch
        // around a load would make the number of loads in flight depend on the path)
        const uint32_t gone = (uint32_t)((rb1 - 1 - rb) >> 31) << 31;
        const uint32_t r_a = (uint32_t)(min(rb * 16 + li, a.N - 1) - row0) * (uint32_t)a.KB;
        const uint32_t r_b = (uint32_t)(min(rb * 16 + li + 8, a.N - 1) - row0) * (uint32_t)a.KB;
        dst[0] = __builtin_amdgcn_raw_buffer_load_b128(rwt, (r_a + piece_off[ln]) | gone, 0, 0);
        dst[1] = __builtin_amdgcn_raw_buffer_load_b128(rwt, (r_b + piece_off[ln]) | gone, 0, 0);
    };
#pragma unroll
    for (int ln = 0; ln < NL; ++ln) issue(0, raw[0][ln], ln);

#pragma unroll
    for (int ln = 0; ln < NL; ++ln) issue(1, raw[1][ln], ln);
    // the staged activations are older than the 4 NL weight loads requested since, and loads return in order
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(4 * NL) : "memory");
    __syncthreads();

    // ---- activations of the slice -> registers ------------------------------------------------------
    // pair p of line ln, lane (g, t, b): quad 4 p + t of the lane's stream of the line, i.e. the dwords
    // of x that hold codes (2u, 2u + 1) and (2u + CPD/2, 2u + 1 + CPD/2) of the quad's weight dword
    u32x2 xr[NL][XP];
    {
        const uint8_t *xrow = xbuf + min(b, a.B - 1) * xpitch;
#pragma unroll
        for (int ln = 0; ln < NL; ++ln)
#pragma unroll
            for (int p = 0; p < XP; ++p) {
                const int qi = 4 * p + t, dwi = qi / QD, u = qi % QD, h = dwi >> 2, w = dwi & 3;
                const int byte_in_row = (line0 + ln) * 128 + (g + 4 * h) * 16 + 4 * w;
                const bool valid = byte_in_row < a.KB && b < a.B;
                const uint32_t *q = reinterpret_cast<const uint32_t *>(xrow + (valid ? (byte_in_row * CPB + 2 * u) * 2 : 0));
                const uint32_t first = q[0], second = q[CPD / 4];
                xr[ln][p].x = valid ? first : 0u;
                xr[ln][p].y = valid ? second : 0u;
            }
    }

    // alpha and z of the first outputs this thread will write, requested ahead
    const int total_out = rows_wg * a.B;
    constexpr int PF = 2;
    float pal[PF], pze[PF];
#pragma unroll
    for (int m = 0; m < PF; ++m) {
        const int idx = tid + m * nthreads;
        const int row = row0 + (idx < total_out ? idx % rows_wg : 0);
        pal[m] = bf16_bits_to_float(a.alpha[row]);
        pze[m] = bf16_bits_to_float(a.zero[row]);
    }

    // The operand order of a quad is (2u, 2u + CPD/2, 2u + 1, 2u + 1 + CPD/2).  sum_k x and
    // sum_k x * offset_k of the slice come out of the same registers (every activation of the slice
    // sits in exactly one lane); line ln is summed by the wave with rw == ln % RW.
    {
        // offset of code position k % 8 at int2: 128 32 8 128 32 8 128 32; lane t holds positions 2t, 2t + 1
        const float off_a = R != 2 ? 128.f : (t == 1 ? 8.f : (t == 2 ? 32.f : 128.f));
        const float off_b = R != 2 ? 128.f : (t == 1 ? 128.f : (t == 2 ? 8.f : 32.f));
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int ln = 0; ln < NL; ++ln) {
#pragma unroll
            for (int p = 0; p < XP; ++p) {
                const uint32_t first = xr[ln][p].x, second = xr[ln][p].y;
                xr[ln][p] = u32x2{__builtin_amdgcn_perm(second, first, 0x05040100u),   // (first.lo, second.lo)
                                  __builtin_amdgcn_perm(second, first, 0x07060302u)};  // (first.hi, second.hi)
            }
            if (ln % RW == rw) {
#pragma unroll
                for (int p = 0; p < XP; ++p) {
                    const float ea = __uint_as_float(xr[ln][p].x << 16) + __uint_as_float(xr[ln][p].x & 0xFFFF0000u);
                    const float eb = __uint_as_float(xr[ln][p].y << 16) + __uint_as_float(xr[ln][p].y & 0xFFFF0000u);
                    s1 += ea + eb;
                    s2 += ea * off_a + eb * off_b;
                }
            }
        }
#pragma unroll
        for (int m = 4; m < 64; m <<= 1) {  // over the lanes of one batch entry
            s1 += __shfl_xor(s1, m);
            s2 += __shfl_xor(s2, m);
        }
        if (lane < 4) {
            sums[(wave * 4 + lane) * 2] = s1;
            sums[(wave * 4 + lane) * 2 + 1] = s2;
        }
    }

    // ---- main loop ------------------------------------------------------------------------------------
    // tile [row][piece ^ (row / 2 % 8)]: conflict-free for the line-shaped writes and the row-shaped reads
    const uint32_t wslot0 = (uint32_t)(8 * li + (lc ^ ((li >> 1) & 7))) << 4;
    const uint32_t wslot1 = (uint32_t)(8 * (li + 8) + (lc ^ (((li + 8) >> 1) & 7))) << 4;
    const uint32_t rslot0 = (uint32_t)(8 * i + (g ^ ((i >> 1) & 7))) << 4;
    const uint32_t rslot1 = (uint32_t)(8 * i + ((4 + g) ^ ((i >> 1) & 7))) << 4;
    // LDS operations of one wave execute in order, so the tile needs no barrier
    auto transpose = [&](const u32x4 (&src)[2], u32x4 (&dst)[2]) {
        *reinterpret_cast<u32x4 *>(tile + wslot0) = src[0];
        *reinterpret_cast<u32x4 *>(tile + wslot1) = src[1];
        dst[0] = *reinterpret_cast<const u32x4 *>(tile + rslot0);
        dst[1] = *reinterpret_cast<const u32x4 *>(tile + rslot1);
    };
    const QuadConsts qc = quad_consts<R>();
    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    u32x4 wt[2][2];
    transpose(raw[0][0], wt[0]);
    issue(2, raw[0][0], 0);
    for (int v = 0; v < nv; v += 2) {
#pragma unroll
        for (int vv = 0; vv < 2; ++vv) {
            const bool active = v + vv < nv;
#pragma unroll
            for (int ln = 0; ln < NL; ++ln) {
                const int par = (vv * NL + ln) & 1;
                // the step after this one changes lanes now and is used in the next step; its ring
                // registers are requested again at once, for the visit two further on
                const int nln = ln + 1 == NL ? 0 : ln + 1, nvv = ln + 1 == NL ? vv + 1 : vv;
                transpose(raw[nvv & 1][nln], wt[par ^ 1]);
                issue(v + nvv + 2, raw[nvv & 1][nln], nln);
                __builtin_amdgcn_sched_barrier(0);
                if (active) {
#pragma unroll
                    for (int dwi = 0; dwi < 8; ++dwi)
                        quad_dword<R, XP>(wt[par][dwi >> 2][dwi & 3], dwi, xr[ln], qc, acc0, acc1);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (active) {
                // accumulator register b = y[b] of row i, k-group g: add the four k-groups
                f32x4 s = acc0 + acc1;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    s[c] += __shfl_xor(s[c], 16);
                    s[c] += __shfl_xor(s[c], 32);
                }
                const int rbl = rw + (v + vv) * RW;  // row block inside the workgroup's range
                if (g == 0) ypart[(ks * CH + rbl) * 16 + i] = s;
                acc0 = acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
    }

    // ---- epilogue: y[b, n] = alpha_n * (2^s * (sum_k (offset_k + code) x - sum_k offset_k x) - z_n * sum_k x) --
    __syncthreads();
    const float kScale = a.scale;
    for (int idx = tid, m = 0; idx < total_out; idx += nthreads, ++m) {
        const int bb = idx / rows_wg, r = idx - bb * rows_wg;
        float xsum = 0.f, xoff = 0.f;
        for (int w = 0; w < NW; ++w) {
            xsum += sums[(w * 4 + bb) * 2];
            xoff += sums[(w * 4 + bb) * 2 + 1];
        }
        float dot = 0.f;
        for (int k = 0; k < KS; ++k) dot += ypart[k * CH * 16 + r][bb];
        float al, ze;
        if (m < PF) {
            al = m == 0 ? pal[0] : pal[1];
            ze = m == 0 ? pze[0] : pze[1];
        } else {
            al = bf16_bits_to_float(a.alpha[row0 + r]);
            ze = bf16_bits_to_float(a.zero[row0 + r]);
        }
        const float yv = al * (kScale * (dot - xoff) - ze * xsum);
        a.y[(size_t)bb * a.N + row0 + r] = (uint16_t)float_to_bf16_bits(yv);
    }
}

struct QuadPlan {
    int nl, ks, rw, ch, grid;
    size_t lds;
};

template <int R, int NL>
mq_status launch_quad(const GemvArgs &a, const QuadPlan &p, hipStream_t st) {
    auto kern = gemv_quad_kernel<R, NL>;
    if (p.lds > 65536 && hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.lds) != hipSuccess)
        return MQ_ERR_DEVICE;
    kern<<<dim3(p.grid), dim3(64 * p.ks * p.rw), p.lds, st>>>(a, p.ks, p.rw, p.ch);
    return launch_status();
}

}  // namespace

mq_status launch_gemv_quad(const GemvArgs &a, int r, hipStream_t st, bool *handled) {
    *handled = false;
    if (a.B > 4 || (r != 2 && r != 4) || a.row_ptr) return MQ_OK;
    const int lines = (a.KB + 127) / 128;
    const int nrb = (a.N + 15) / 16;
    // Lines per slice: the widest slice (fewest activation reloads per byte of weights) that wastes
    // no more than one line in ten on padding and leaves at least about a thousand waves.
    QuadPlan p{};
    p.nl = 0;
    for (int nl = 4; nl >= 1; --nl) {
        const int ks = (lines + nl - 1) / nl;
        if (ks > 8) break;
        const bool enough = (int64_t)nrb * ks >= 1024 || nl == 1;
        if (10 * (ks * nl - lines) <= lines && enough) {
            p.nl = nl;
            p.ks = ks;
            break;
        }
        if (p.nl == 0 || nl == 1) {  // fallback if nothing passes both tests
            p.nl = nl;
            p.ks = ks;
        }
    }
    if (p.nl == 0) return MQ_OK;  // K too long for one workgroup of slices: the general kernel takes it
    int wpc = 8;                   // waves per compute unit the grid is sized for
#ifdef MQ_GEMV_TUNE
    if (const char *e = getenv("MQ_GEMVQ_NL")) {
        p.nl = atoi(e);
        p.ks = (lines + p.nl - 1) / p.nl;
        if (p.nl < 1 || p.nl > 4 || p.ks > 8) return MQ_ERR_SHAPE;
    }
    if (const char *e = getenv("MQ_GEMVQ_WPC")) wpc = atoi(e);
#endif
    // Row-block waves per workgroup and row blocks per workgroup: the whole grid resident at once
    // (wpc waves per compute unit), every wave the same number of visits where the shape allows.
    p.rw = std::max(1, std::min(8 / p.ks, wpc / p.ks));
#ifdef MQ_GEMV_TUNE
    if (const char *e = getenv("MQ_GEMVQ_RW")) p.rw = atoi(e);
    if (p.rw < 1 || p.rw * p.ks > 8) return MQ_ERR_SHAPE;
#endif
    const int nw = p.ks * p.rw;
    const int per_cu = std::max(1, wpc / nw);
    const int capacity = 256 * per_cu;
    int visits = (int)cdiv(nrb, (int64_t)capacity * p.rw);  // per wave
    p.ch = visits * p.rw;
#ifdef MQ_GEMV_TUNE
    if (const char *e = getenv("MQ_GEMVQ_CH")) p.ch = atoi(e);
    if (p.ch < 1) return MQ_ERR_SHAPE;
#endif
    p.grid = (int)cdiv(nrb, p.ch);
    p.lds = kSumsBytes + (size_t)nw * kTileBytes + (size_t)p.ks * p.ch * 16 * sizeof(f32x4) +
            (size_t)a.B * (((size_t)a.K + 511) / 512 * 1024 + kXPad);
    if (p.lds > 160 * 1024 || (int64_t)p.ch * 16 * a.KB > 0x7FFFFFFFll || (int64_t)a.B * a.K * 2 > 0x7FFFFFFFll)
        return MQ_OK;
    *handled = true;
#define MQ_QUAD_CASE(R_, NL_) \
    if (r == R_ && p.nl == NL_) return launch_quad<R_, NL_>(a, p, st);
    MQ_QUAD_CASE(2, 1) MQ_QUAD_CASE(2, 2) MQ_QUAD_CASE(2, 3) MQ_QUAD_CASE(2, 4)
    MQ_QUAD_CASE(4, 1) MQ_QUAD_CASE(4, 2) MQ_QUAD_CASE(4, 3) MQ_QUAD_CASE(4, 4)
#undef MQ_QUAD_CASE
    *handled = false;
    return MQ_OK;
}

}  // namespace mq
