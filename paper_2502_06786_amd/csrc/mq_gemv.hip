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
#include <algorithm>
#include <type_traits>

#include "mq_gemv.h"

namespace mq {


__device__ __forceinline__ void wait_all_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

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

// One workgroup = KS * RW waves.  Wave (ks, rw) = (wave % KS, wave / KS) streams block rw of
// 16 * RG weight rows and takes every KS-th 64-byte segment of those rows; the KS partial sums of a
// row block meet in LDS.  Lane (i, g) = (lane % 16, lane / 16) owns weight row i of each of the RG
// row groups and bytes [16 g, 16 g + 16) of a segment, and batch entry b = i of the activations
// for the same k range.  A workgroup walks over groups of RW row blocks (grid-stride), so that the
// whole grid is resident at once and no second, mostly empty round of workgroups is needed.
//
// Activations: x is brought into LDS by direct global->LDS loads (asynchronous, all in flight at
// once) as 1 KB blocks of 512 consecutive k of one batch entry; 16-byte slot L of the block of
// batch entry b is kept at slot L ^ b, so that the 16 lanes of a matrix-core operand read (16
// batch entries, same k) hit 16 different bank groups.  A second, LDS-local pass pairs the values
// the way the unpacked codes are paired and takes sum_k x and (int2) sum_k x * offset_k, which is
// what removes the 128 / 32 / 8 offsets of the unpack and applies the zero-point.  When all of x
// fits it is staged once per workgroup; otherwise in chunks, per group of row blocks.
//
// Weights stream through a register ring that keeps D - 1 segments per wave in flight behind the
// one being computed.  Few rows -> large KS (the whole matrix is in flight after one round trip);
// many rows -> KS = 1 and every wave streams its own rows.
//
// Lanes are never masked in the hot loop: rows past N re-read row N - 1 and batch entries past B
// re-read whatever LDS holds for them; both only feed outputs that are not stored (a column of the
// product depends on its own batch entry only).  A lane whose 16 bytes lie past the end of the row
// re-reads the row's last 16 bytes; any bit pattern unpacks to finite numbers, and those meet
// activations that were staged as zeros.
constexpr int kSumBytes = 1024;  // [0, 32): per-half-wave parts of sum_k x; [32, 64): of sum_k x * offset_k
constexpr uint32_t kOOB = 0x80000000u;
typedef __attribute__((address_space(3))) void *lds_ptr;

// The operands of one 64-byte segment: XV 16-byte slots per lane; slot L = sb * 4 XV + g * XV + v of
// the block, kept at L ^ b.
// (v & mask) | magic.  The fused v_and_or_b32 takes at most one scalar operand and no literals, so it
// is only selected when the masks already live in scalar registers and the exponent patterns in
// vector registers (see unpack_consts); with literal constants the compiler emits two instructions.
// (Plain C on purpose: hazards around instructions inside inline assembly are not tracked.)
__device__ __forceinline__ uint32_t and_or(uint32_t v, uint32_t mask_s, uint32_t magic_v) {
    return (v & mask_s) | magic_v;
}

// Geometry per bit-width.  A weight "line" is what eight neighbouring lanes fetch of one row in one
// load: 128 bytes (16 per lane) for r = 8, 4, 2, and 96 bytes (12 per lane) for the bit streams of
// r = 6 and r = 3, whose codes straddle any power-of-two boundary but fill 12 bytes exactly
// (16 resp. 32 codes).  A lane's piece unpacks to XV matrix-core operands of 8 codes each.
constexpr int line_bytes(int r) { return (r == 6 || r == 3) ? 96 : 128; }
constexpr int piece_bytes(int r) { return line_bytes(r) / 8; }
constexpr int line_codes(int r) { return line_bytes(r) * 8 / r; }            // k values per line
constexpr int operands_per_piece(int r) { return line_codes(r) / 8 / 8; }    // XV
typedef uint32_t u32x3_a4 __attribute__((ext_vector_type(3), aligned(4)));  // a 12-byte piece as one load

// Order in which the 32 codes of a 3-bit piece (12 bytes) enter its four matrix-core operands:
// kOrder3[8 v + 2 p + h] = code that operand v holds in half h of register p.  Codes that sit at the
// same position of the two 16-bit halves of a dword once each half is shifted by its own amount
// share a register (one packed shift serves two registers: the codes at bits 0-2 read as 128 + c,
// the next ones at bits 3-5 as 16 + c); the six codes that straddle a half or lie alone go last.
__device__ constexpr uint8_t kOrder3[32] = {0, 6, 1, 7, 2, 8, 3, 9,          11, 16, 12, 17, 13, 18, 14, 19,
                                            22, 27, 23, 28, 24, 29, 25, 30,  15, 20, 4, 5, 10, 21, 26, 31};
// offset under which element (v, p) of the 3-bit order reads: 16 for the registers fed from bits 3-5
__host__ __device__ constexpr float offset3(int v, int p) { return (v < 3 && (p & 1)) ? 16.f : 128.f; }
constexpr uint32_t kB16 = 0x41804180u;  // (16, 16)

// Constants of the unpack, pinned in registers once per kernel.
struct UnpackConsts {
    uint32_t m0, m1, m2;     // scalar: field masks
    uint32_t e128, e32, e8;  // vector: (128,128), (32,32), (8,8) as bf16 pairs
};
template <int R>
__device__ __forceinline__ UnpackConsts unpack_consts() {
    UnpackConsts c;
    c.m0 = R == 2 ? 0x00030003u : (R == 4 ? 0x000F000Fu : (R == 6 ? 0x0000003Fu : 0x00070007u));
    c.m1 = R == 2 ? 0x000C000Cu : (R == 6 ? 0x003F0000u : 0x00380038u);
    c.m2 = R == 3 ? 0x00070000u : 0x00300030u;
    c.e128 = kB128;
    c.e32 = R == 3 ? kB16 : kB32;
    c.e8 = kB8;
    asm volatile("" : "+s"(c.m0), "+s"(c.m1), "+s"(c.m2));
    asm volatile("" : "+v"(c.e128), "+v"(c.e32), "+v"(c.e8));
    return c;
}

// The operands of one 64-byte segment: XV 16-byte slots per lane; slot L = sb * 4 XV + g * XV + v of
// the block, kept at L ^ b.
template <int R, int RG>
__device__ __forceinline__ void gemv_segment(const u32x4 (&wt)[RG], const uint8_t *blk, uint32_t slot0,
                                             const UnpackConsts &uc, f32x4 (&acc)[RG]) {
    // slot0 = (sb * 4 XV + g * XV) ^ b, shifted to bytes; v < XV only touches bits that b may flip too
    auto operand = [&](int v) { return *reinterpret_cast<const u32x4 *>(blk + (slot0 ^ (uint32_t)(v << 4))); };
    if constexpr (R == 2) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const u32x4 xb0 = operand(2 * w), xb1 = operand(2 * w + 1);
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) {
                // codes j and j + 8 of a dword share a register; fields at bits 0-1, 2-3, 4-5 of a
                // 16-bit lane read as 128 + c, 32 + c, 8 + c under the exponents of e128, e32, e8
                const uint32_t d = wt[rg][w], d6 = d >> 6, d12 = d >> 12;
                const u32x4 a0 = {and_or(d, uc.m0, uc.e128), and_or(d, uc.m1, uc.e32), and_or(d, uc.m2, uc.e8),
                                  and_or(d6, uc.m0, uc.e128)};
                const u32x4 a1 = {and_or(d6, uc.m1, uc.e32), and_or(d6, uc.m2, uc.e8), and_or(d12, uc.m0, uc.e128),
                                  and_or(d12, uc.m1, uc.e32)};
                acc[rg] = mfma16(a0, xb0, acc[rg]);
                acc[rg] = mfma16(a1, xb1, acc[rg]);
            }
        }
    } else if constexpr (R == 4) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const u32x4 xb = operand(w);
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) {
                const uint32_t d = wt[rg][w];  // codes j and j + 4 of the dword share a register
                const u32x4 a0 = {and_or(d, uc.m0, uc.e128), and_or(d >> 4, uc.m0, uc.e128),
                                  and_or(d >> 8, uc.m0, uc.e128), and_or(d >> 12, uc.m0, uc.e128)};
                acc[rg] = mfma16(a0, xb, acc[rg]);
            }
        }
    } else if constexpr (R == 3) {
        // 32 codes in 96 bits, operands in the order of kOrder3 (see there)
        u32x4 xb[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) xb[v] = operand(v);
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) {
            u32x4 ops[4];
            const uint32_t d0 = wt[rg].x, d1 = wt[rg].y, d2 = wt[rg].z;
            auto halves = [](uint32_t d, int lo, int hi) {  // each 16-bit half shifted right by its own amount
                const u16x2 t = __builtin_bit_cast(u16x2, d) >> u16x2{(unsigned short)lo, (unsigned short)hi};
                return __builtin_bit_cast(uint32_t, t);
            };
            const uint32_t a0 = halves(d0, 0, 2), a1 = halves(d0, 6, 8);
            ops[0] = u32x4{and_or(a0, uc.m0, uc.e128), and_or(a0, uc.m1, uc.e32), and_or(a1, uc.m0, uc.e128),
                               and_or(a1, uc.m1, uc.e32)};
            const uint32_t b0 = halves(d1, 1, 0), b1 = halves(d1, 7, 6);
            ops[1] = u32x4{and_or(b0, uc.m0, uc.e128), and_or(b0, uc.m1, uc.e32), and_or(b1, uc.m0, uc.e128),
                               and_or(b1, uc.m1, uc.e32)};
            const uint32_t c0 = halves(d2, 2, 1), c1 = halves(d2, 8, 7);
            ops[2] = u32x4{and_or(c0, uc.m0, uc.e128), and_or(c0, uc.m1, uc.e32), and_or(c1, uc.m0, uc.e128),
                               and_or(c1, uc.m1, uc.e32)};
            // (15, 20): bits 13-15 and 28-30 of d1; (4, 5): bits 12-14 and 15-17 of d0;
            // (10, 21): bits 30-32 and 63-65 of the piece; (26, 31): bits 14-16 and 29-31 of d2
            const uint32_t lo7 = uc.m0 & 0xFFFFu;  // 0x7 in the low half only
            ops[3] = u32x4{and_or(halves(d1, 13, 12), uc.m0, uc.e128),
                               and_or(d0 << 1, uc.m2, and_or(d0 >> 12, lo7, uc.e128)),
                               and_or(__builtin_amdgcn_alignbit(d2, d1, 15), uc.m2,
                                      and_or(__builtin_amdgcn_alignbit(d1, d0, 30), lo7, uc.e128)),
                               and_or(d2 >> 13, uc.m2, and_or(d2 >> 14, lo7, uc.e128))};
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[rg] = mfma16(ops[v], xb[v], acc[rg]);
        }
    } else if constexpr (R == 6) {
        // bit stream: code j of the 96-bit piece sits at bits [6 j, 6 j + 6); operand v takes codes
        // 8 v .. 8 v + 7 in their natural order, two per register (low half, high half), each read
        // as 128 + code under the exponent of e128
        constexpr int XVP = operands_per_piece(R);
#pragma unroll
        for (int v = 0; v < XVP; ++v) {
            const u32x4 xb = operand(v);
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) {
                const u32x4 d = wt[rg];
                auto field_at = [&](int j, int pos) -> uint32_t {  // code j moved to bit `pos`, unmasked
                    const int bit = R * j, idx = bit >> 5, sh = bit & 31;
                    if (sh + R > 32) return __builtin_amdgcn_alignbit(d[(idx + 1) & 3], d[idx], (uint32_t)(sh - pos));
                    return sh >= pos ? d[idx] >> (sh - pos) : d[idx] << (pos - sh);
                };
                u32x4 a0;
#pragma unroll
                for (int p2 = 0; p2 < 4; ++p2) {
                    const int j = 8 * v + 2 * p2;
                    a0[p2] = and_or(field_at(j + 1, 16), uc.m1, and_or(field_at(j, 0), uc.m0, uc.e128));
                }
                acc[rg] = mfma16(a0, xb, acc[rg]);
            }
        }
    } else {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const u32x4 xb = operand(u);
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

// CB = 512-k blocks of x per chunk.  LDS: [sums][area A][x], where area A starts with the 2 KB per
// wave through which weight lines are transposed and also takes the reduction data once the main
// loop is over.  single != 0: all of x is staged once per workgroup and stays (area A then is as
// large as the reduction data); single == 0: x is restaged (in one or more chunks) for every group
// of row blocks and the reduction data may run over it.
template <int R, int RG, int D>
__global__ __launch_bounds__(1024) void gemv_kernel(GemvArgs a, int bp, int CB, int KS, int ngroups, int x_off,
                                                    int single_flag) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int NW = blockDim.x >> 6;
    const int RW = NW / KS;
    const int ks = wave % KS, rw = wave / KS;
    const int i = lane & 15, g = lane >> 4;
    constexpr int ROWS = 16 * RG;          // rows of one row block
    constexpr int LINEB = line_bytes(R), PIECE = piece_bytes(R);
    constexpr int XV = operands_per_piece(R);     // 16-byte activation operands per lane and segment
    constexpr int SSPB = 512 / line_codes(R);     // weight lines (two segments each) per 512-k block of x

    float *sums = reinterpret_cast<float *>(lds);
    uint8_t *area = lds + kSumBytes;
    uint8_t *xbuf = area + x_off;
    const int segs = (a.KB + LINEB - 1) / LINEB;  // weight lines per row
    const int chunk_segs = CB * SSPB;
    const bool single = single_flag != 0;
    const int bb = i & (bp - 1), b15 = bb & 15;
    const uint8_t *xlane = xbuf + bb * 1024;
    const uint32_t lane_slot = (uint32_t)((g * XV) ^ b15);

    // Weights are fetched as whole 128-byte lines: lane (li, lc) = (lane / 8, lane % 8) takes 16-byte
    // piece lc of the line of row li (first load) and row li + 8 (second load) of a 16-row group, so
    // that eight neighbouring lanes cover one line.  The matrix core wants lane (i, g) to hold piece
    // 4 * sgm + g of row i for segment sgm of the line: the pieces change lanes through a 2 KB LDS
    // tile per wave, [row][piece ^ (row / 2 % 8)], which both the writes and the reads hit without
    // bank conflicts.  LDS operations of one wave execute in order, so the tile needs no barrier.
    const int li = lane >> 3, lc = lane & 7;
    uint8_t *tb = area + wave * 2048;
    const uint32_t wslot0 = (uint32_t)(8 * li + (lc ^ ((li >> 1) & 7))) << 4;
    const uint32_t wslot1 = (uint32_t)(8 * (li + 8) + (lc ^ (((li + 8) >> 1) & 7))) << 4;
    const uint32_t rslot0 = (uint32_t)(8 * i + (g ^ ((i >> 1) & 7))) << 4;
    const uint32_t rslot1 = (uint32_t)(8 * i + ((4 + g) ^ ((i >> 1) & 7))) << 4;

    const uint64_t xbytes = (uint64_t)a.B * a.K * 2;
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.x), 0, (int)(xbytes > 0x7FFFFFFFull ? 0x7FFFFFFFull : xbytes), 0x00020000);

    // chunk c of x -> LDS: block j = (kb, b) by wave j % NW
    auto issue_x = [&](int c) {
        for (int j = wave; j < CB * bp; j += NW) {
            const int kb = j / bp, b = j % bp;
            if (b < a.B) {
                const int k = (c * CB + kb) * 512 + ((lane ^ (b & 15)) << 3);
                const uint32_t vo = k < a.K ? ((uint32_t)b * (uint32_t)a.K + (uint32_t)k) * 2u : kOOB;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_ptr)(xbuf + j * 1024), 16, vo, 0, 0, 0);
            }
        }
    };
    // LDS-local pass over the staged chunk: pair the activations like the codes, accumulate the sums
    float s1 = 0.f, s2 = 0.f;
    auto pair_pass = [&](bool with_sums) {
        const int hw = wave * 2 + (lane >> 5), u = lane & 31;
        for (int j = hw; j < CB * bp; j += 2 * NW) {
            const int b = j % bp;
            if (b >= a.B) continue;
            uint8_t *blk = xbuf + j * 1024;
            if constexpr (R == 2) {
                u32x4 *p0 = reinterpret_cast<u32x4 *>(blk + (((2 * u) ^ (b & 15)) << 4));
                u32x4 *p1 = reinterpret_cast<u32x4 *>(blk + (((2 * u + 1) ^ (b & 15)) << 4));
                const u32x4 x0 = *p0, x1 = *p1;
                // codes j and j + 8 of a dword share a register: pair the activations the same way
                const u32x4 o0 = {pair_lo(x0.x, x1.x), pair_hi(x0.x, x1.x), pair_lo(x0.y, x1.y), pair_hi(x0.y, x1.y)};
                const u32x4 o1 = {pair_lo(x0.z, x1.z), pair_hi(x0.z, x1.z), pair_lo(x0.w, x1.w), pair_hi(x0.w, x1.w)};
                *p0 = o0;
                *p1 = o1;
                if (with_sums) {
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        const float e0 = __uint_as_float(o0[jj] << 16) + __uint_as_float(o0[jj] & 0xFFFF0000u);
                        const float e1 = __uint_as_float(o1[jj] << 16) + __uint_as_float(o1[jj] & 0xFFFF0000u);
                        s1 += e0 + e1;
                        // field position inside the 16-bit lane: 0, 1, 2, 0 then 1, 2, 0, 1
                        s2 += e0 * (jj % 3 == 0 ? 128.f : (jj % 3 == 1 ? 32.f : 8.f));
                        s2 += e1 * ((jj + 4) % 3 == 0 ? 128.f : ((jj + 4) % 3 == 1 ? 32.f : 8.f));
                    }
                }
            } else if constexpr (R == 3) {
                if (u < 16) {  // a 1 KB block holds 16 units of 32 activations (four slots)
                    uint32_t src[16], dst[16];
#pragma unroll
                    for (int sl = 0; sl < 4; ++sl) {
                        const u32x4 t = *reinterpret_cast<const u32x4 *>(blk + (((4 * u + sl) ^ (b & 15)) << 4));
                        src[4 * sl] = t.x, src[4 * sl + 1] = t.y, src[4 * sl + 2] = t.z, src[4 * sl + 3] = t.w;
                    }
#pragma unroll
                    for (int o = 0; o < 16; ++o) {  // register o of the unit: operand o / 4, register o % 4
                        const int ea = kOrder3[2 * o], eb = kOrder3[2 * o + 1];  // low half, high half
                        const uint32_t lo = (ea & 1) ? src[ea >> 1] >> 16 : src[ea >> 1] & 0xFFFFu;
                        const uint32_t hi = (eb & 1) ? src[eb >> 1] & 0xFFFF0000u : src[eb >> 1] << 16;
                        dst[o] = lo | hi;
                        if (with_sums) {
                            const float e = __uint_as_float(dst[o] << 16) + __uint_as_float(dst[o] & 0xFFFF0000u);
                            s1 += e;
                            s2 += e * offset3(o >> 2, o & 3);
                        }
                    }
#pragma unroll
                    for (int sl = 0; sl < 4; ++sl)
                        *reinterpret_cast<u32x4 *>(blk + (((4 * u + sl) ^ (b & 15)) << 4)) =
                            u32x4{dst[4 * sl], dst[4 * sl + 1], dst[4 * sl + 2], dst[4 * sl + 3]};
                }
            } else {
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    u32x4 *p = reinterpret_cast<u32x4 *>(blk + (((u + 32 * half) ^ (b & 15)) << 4));
                    u32x4 x0 = *p;
                    if constexpr (R == 4) {  // codes j and j + 4 of a dword share a register
                        x0 = u32x4{pair_lo(x0.x, x0.z), pair_hi(x0.x, x0.z), pair_lo(x0.y, x0.w), pair_hi(x0.y, x0.w)};
                        *p = x0;
                    }
                    if (with_sums) {
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj)
                            s1 += __uint_as_float(x0[jj] << 16) + __uint_as_float(x0[jj] & 0xFFFF0000u);
                    }
                }
            }
        }
    };
    // sum over a half-wave, left in its lane 0 (lanes 0 and 32 of the wave)
    auto half_wave_sum = [&](float v) {
        auto dpp_add = [](float x, auto ctrl) {
            const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value, 0xF, 0xF, true);
            return x + __int_as_float(moved);
        };
        v = dpp_add(v, std::integral_constant<int, 0xB1>{});
        v = dpp_add(v, std::integral_constant<int, 0x4E>{});
        v = dpp_add(v, std::integral_constant<int, 0x141>{});
        v = dpp_add(v, std::integral_constant<int, 0x140>{});
        const int bits = __float_as_int(v);
        const float lo = __int_as_float(__builtin_amdgcn_readlane(bits, 0)) + __int_as_float(__builtin_amdgcn_readlane(bits, 16));
        const float hi = __int_as_float(__builtin_amdgcn_readlane(bits, 32)) + __int_as_float(__builtin_amdgcn_readlane(bits, 48));
        return lane < 32 ? lo : hi;
    };

    // `ring` = weight loads that were requested after the activations and may stay in flight (loads
    // return in order, so waiting for all but the newest `ring` is waiting for the activations)
    auto stage = [&](int c, bool with_sums, auto ring) {
        if constexpr (decltype(ring)::value == 0)
            wait_all_loads();
        else
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(decltype(ring)::value) : "memory");
        __syncthreads();
        pair_pass(with_sums);
        if (with_sums) {  // running totals; complete after the last chunk's pass
            const float t1 = half_wave_sum(s1), t2 = (R == 2 || R == 3) ? half_wave_sum(s2) : 0.f;
            if ((lane & 31) == 0) {
                sums[wave * 2 + (lane >> 5)] = t1;
                sums[32 + wave * 2 + (lane >> 5)] = t2;
            }
        }
        __syncthreads();
    };
    const UnpackConsts uc = unpack_consts<R>();
    bool first = true;
    for (int grp = blockIdx.x; grp < ngroups; grp += gridDim.x) {
        const int nb = grp * RW * ROWS;  // first row of the group
        const int n0 = nb + rw * ROWS;   // first row of this wave
        f32x4 acc[RG];
        u32x4 w[D][2][RG];  // [ring slot][first / second load][row group]
        const int n0c = min(n0, a.N - 1);
        const uint8_t *wbase = a.packed + (size_t)n0c * a.KB;  // wave-uniform
        uint32_t roff[RG][2];
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) {
            acc[rg] = f32x4{0.f, 0.f, 0.f, 0.f};
            roff[rg][0] = (uint32_t)(min(n0 + rg * 16 + li, a.N - 1) - n0c) * (uint32_t)a.KB;
            roff[rg][1] = (uint32_t)(min(n0 + rg * 16 + li + 8, a.N - 1) - n0c) * (uint32_t)a.KB;
#pragma unroll
            for (int d = 0; d < D; ++d) w[d][0][rg] = w[d][1][rg] = u32x4{0u, 0u, 0u, 0u};
        }
        // alpha and z of the rows this lane will write: requested now and used after the main loop
        float pal[RG][4], pze[RG][4];
        auto load_params = [&]() {
#pragma unroll
            for (int rg = 0; rg < RG; ++rg)
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) {
                    const int row = min(n0 + rg * 16 + 4 * g + cc, a.N - 1);
                    pal[rg][cc] = bf16_bits_to_float(a.alpha[row]);
                    pze[rg][cc] = bf16_bits_to_float(a.zero[row]);
                }
        };
        load_params();
        int off = ks * LINEB + lc * PIECE;  // byte offset, inside the packed row, of the next piece to request
        // Unconditional (an offset past the row is clamped into it), so that the number of loads in
        // flight is known at compile time and a use only waits for its own load.
        const int off_last = a.KB - PIECE;
        auto fetch_next = [&](u32x4 (&dst)[2][RG]) {
            const uint32_t o = (uint32_t)min(off, off_last);
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) {
                if constexpr (PIECE == 16) {
                    // (non-temporal: every weight byte is read once)
                    dst[0][rg] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wbase + (roff[rg][0] + o)));
                    dst[1][rg] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wbase + (roff[rg][1] + o)));
                } else {  // 12-byte pieces, 4-byte aligned
                    const u32x3_a4 p0 = __builtin_nontemporal_load(reinterpret_cast<const u32x3_a4 *>(wbase + (roff[rg][0] + o)));
                    const u32x3_a4 p1 = __builtin_nontemporal_load(reinterpret_cast<const u32x3_a4 *>(wbase + (roff[rg][1] + o)));
                    dst[0][rg] = u32x4{p0.x, p0.y, p0.z, 0u};
                    dst[1][rg] = u32x4{p1.x, p1.y, p1.z, 0u};
                }
            }
            off += KS * LINEB;
        };
        // one 128-byte line of each of the wave's 16 RG rows: transpose through LDS, then two segments
        auto compute_line = [&](const u32x4 (&raw)[2][RG], int sr) {
            u32x4 wt0[RG], wt1[RG];
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) {
                *reinterpret_cast<u32x4 *>(tb + wslot0) = raw[0][rg];
                *reinterpret_cast<u32x4 *>(tb + wslot1) = raw[1][rg];
                wt0[rg] = *reinterpret_cast<const u32x4 *>(tb + rslot0);
                wt1[rg] = *reinterpret_cast<const u32x4 *>(tb + rslot1);
            }
            const uint8_t *blk = xlane + (sr / SSPB) * bp * 1024;
            const uint32_t sb = (uint32_t)(sr % SSPB) * 2u;  // first segment of the line inside the x block
            gemv_segment<R, RG>(wt0, blk, ((sb * 4 * XV) ^ lane_slot) << 4, uc, acc);
            __builtin_amdgcn_sched_barrier(0);  // keeps the operand reads of the second segment out of the first
            gemv_segment<R, RG>(wt1, blk, (((sb + 1) * 4 * XV) ^ lane_slot) << 4, uc, acc);
        };
        // The activations of the first chunk are requested before the weights of the ring: they come
        // from L2 and are paired while the first weight lines are still on their way from HBM.
        const bool stage_first = first || !single;
        if (stage_first) {
            if (!first) __syncthreads();  // the previous group is done with the x area
            issue_x(0);
        }
#pragma unroll
        for (int d = 0; d + 1 < D; ++d) fetch_next(w[d]);

        // Line sb + ks is this wave's line in the current step; sb is the same for all waves of the
        // workgroup, so the switch to the next chunk of x (a barrier) happens in the same step for
        // all of them: chunk boundaries are multiples of KS.  The load of the line D - 1 steps ahead
        // is unconditional; the arithmetic of a line past the end is skipped by a wave-uniform
        // branch.  The ring is unrolled D times: moving registers whose loads are still in flight
        // would force a wait for them.
        int c = 0, c0 = 0, c1 = min(chunk_segs, segs);
        if (stage_first) stage(0, first, std::integral_constant<int, (D - 1) * 2 * RG>{});
        for (int sb = 0; sb < segs;) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                if (sb >= c1 && c1 < segs) {  // (only when x does not fit: restaged per group, chunk by chunk)
                    __syncthreads();          // the chunk has been consumed
                    ++c;
                    c0 = c1;
                    c1 = min(c0 + chunk_segs, segs);
                    issue_x(c);
                    stage(c, first, std::integral_constant<int, 0>{});
                }
                fetch_next(w[(d + D - 1) % D]);
                if (sb + ks < c1) compute_line(w[d], sb + ks - c0);
                sb += KS;
            }
        }
        first = false;

        // ---- after the main loop ------------------------------------------------------------------
        // Wave ks == 0 of a row block ends up with the sums of its rows in the matrix-core output
        // layout (lane = batch entry b + 16 * (row / 4), component = row % 4) and writes them out
        // itself.  With KS == 1 nothing is shared between waves here, so they run on without a barrier;
        // otherwise the partial sums meet in LDS.
        f32x4 *part = reinterpret_cast<f32x4 *>(area);                    // [wave][rg][lane], over the tiles
        const bool shared = KS > 1;
        if (KS > 1) {
            __syncthreads();  // every wave is done with its transposition tile
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) part[(wave * RG + rg) * 64 + lane] = acc[rg];
        }
        if (shared) __syncthreads();
        if (ks == 0) {
            if (KS > 1) {
#pragma unroll
                for (int rg = 0; rg < RG; ++rg)
                    for (int kk = 1; kk < KS; ++kk) {
                        const f32x4 pv = part[((wave + kk) * RG + rg) * 64 + lane];
                        acc[rg].x += pv.x;
                        acc[rg].y += pv.y;
                        acc[rg].z += pv.z;
                        acc[rg].w += pv.w;
                    }
            }
            // y[b, n] = alpha_n * (2^s * (codes.x [+ overflow]) - z_n * sum_k x)
            const float kScale = a.scale;
            const int b = lane & 15;
            if (b < a.B) {
                float xsum = 0.f, xoff = 0.f;
                for (int hw = b; hw < 2 * NW; hw += bp) {  // the half-waves that staged batch entry b
                    xsum += sums[hw];
                    xoff += sums[32 + hw];
                }
#pragma unroll
                for (int rg = 0; rg < RG; ++rg) {
                    float yv[4];
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) {
                        const int rl = rg * 16 + 4 * g + cc;
                        float dot = acc[rg][cc];
                        if constexpr (R == 2 || R == 3) dot -= xoff;
                        if constexpr (R == 4 || R == 6) dot -= 128.0f * xsum;
                        // extra precision: the overflow sum of this output waits in y (written by the kernel
                        // that ran before this one on the stream)
                        if (a.add_y && n0 + rl < a.N) dot += ovf_sum_unpack(a.y[(size_t)b * a.N + n0 + rl]);
                        yv[cc] = pal[rg][cc] * (kScale * dot - pze[rg][cc] * xsum);
                    }
                    const int row0 = n0 + rg * 16 + 4 * g;  // the lane's four consecutive rows
                    if (a.post >= kPostGelu) {              // two (gate, up) pairs (N is even)
#pragma unroll
                        for (int cc = 0; cc < 4; cc += 2)
                            if (row0 + cc < a.N)
                                a.y[(size_t)b * (a.N >> 1) + ((row0 + cc) >> 1)] = gated_bf16(yv[cc], yv[cc + 1], a.post);
                    } else {
#pragma unroll
                        for (int cc = 0; cc < 4; ++cc) {
                            const size_t at = (size_t)b * a.N + row0 + cc;
                            if (row0 + cc < a.N)
                                a.y[at] = a.post == kPostResidual ? residual_bf16(a.res[at], yv[cc])
                                                                  : (uint16_t)float_to_bf16_bits(yv[cc]);
                        }
                    }
                }
            }
        }
        // the next group's tiles or (restaged) x area start behind a barrier
        if (shared && single && grp + (int)gridDim.x < ngroups) __syncthreads();
    }
}

template <int R, int RG, int D>
static mq_status launch_gemv(const GemvArgs &a, int nw, int ks, hipStream_t st) {
    int bp = 1;
    while (bp < a.B) bp <<= 1;
    constexpr int SSPB = 512 / line_codes(R);  // weight lines per 512-k block of x
    const int lines = (a.KB + line_bytes(R) - 1) / line_bytes(R);
    const int blocks_all = (lines + SSPB - 1) / SSPB;  // 512-k blocks that cover K
    // area A: the 2 KB transposition tiles of the waves (reused for the K-split partial sums, which
    // need RG <= 2 KB per wave)
    static_assert(RG <= 2, "partial sums are laid over the transposition tiles");
    auto area_bytes = [&](int nw_, int) { return (size_t)nw_ * 2048; };
    constexpr size_t kLdsMax = 160 * 1024 - kSumBytes;
    // all of x at once when it fits behind the reduction data; otherwise chunks that are a multiple of
    // KS * D lines, so that the register ring of every wave is in the same phase at each chunk
    // boundary, restaged for every group of row blocks, with the reduction data laid over them
    int CB = blocks_all, single = 1;
    size_t x_off = area_bytes(nw, ks);
    size_t lds = kSumBytes + x_off + (size_t)blocks_all * bp * 1024;
    if (lds > kLdsMax + kSumBytes) {
        single = 0;
        // chunks of whole 512-k blocks whose line count is a multiple of KS; eight waves per workgroup
        // (more row-block groups, a smaller area A), the largest KS whose chunk still fits
        nw = 8;
        if (ks > nw) ks = nw;
        int cap_blocks = 0;
        for (;; ks >>= 1) {
            cap_blocks = (int)(std::min<size_t>(131072, kLdsMax - area_bytes(nw, ks)) / (bp * 1024));
            if (ks == 1 || cap_blocks * SSPB >= ks) break;
        }
        const int unit = std::max(ks, SSPB);  // (both are powers of two)
        CB = cap_blocks * SSPB / unit * unit / SSPB;
        if (CB < 1) return MQ_ERR_SHAPE;  // (cannot happen: at KS = 1 at least seven 16 KB blocks fit)
        x_off = area_bytes(nw, ks);
        lds = kSumBytes + x_off + (size_t)CB * bp * 1024;
    }
    const int rw = nw / ks;
    const int ngroups = (int)cdiv(a.N, 16 * RG * rw);
    // resident workgroups: 16 waves and 160 KB of LDS per compute unit, 256 compute units
    const int wpc = 16;
    const int per_cu = std::max(1, std::min(wpc / nw, (int)((160 * 1024) / lds)));
    const int capacity = 256 * per_cu;
    const int rounds = (ngroups + capacity - 1) / capacity;
    const int grid = (ngroups + rounds - 1) / rounds;
    auto go = [&](auto kern) -> mq_status {
        if (lds > 65536 && hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return MQ_ERR_DEVICE;
        kern<<<dim3(grid), dim3(64 * nw), lds, st>>>(a, bp, CB, ks, ngroups, (int)x_off, single);
        return launch_status();
    };
    return go(gemv_kernel<R, RG, D>);
}

}  // namespace mq

// Everything about one GEMV that can be refused before a launch and does not depend on x or y: bit-width,
// sizes, row alignment of the plane, the plane pointer.  `post` as in GemvArgs.
mq_status mq::gemv_sliced_check(const uint8_t *packed, int64_t B, int64_t N, int64_t K, int r, int post) {
    if (post >= kPostGelu && N % 2 != 0) return MQ_ERR_SHAPE;
    if (r != 8 && r != 6 && r != 4 && r != 3 && r != 2) return MQ_ERR_BITS;
    if (B < 1 || B > 16 || N < 0 || K < 1 || N > 0x7FFFFFF0 || K > 0x7FFFFFF0) return MQ_ERR_SHAPE;
    if (B * K > (1ll << 29)) return MQ_ERR_SHAPE;  // 32-bit byte offsets into x
    // packed rows are whole 16-byte units (12-byte units for the bit streams of r = 6 and r = 3)
    if ((K * r) % (8 * piece_bytes(r)) != 0) return MQ_ERR_ALIGN;
    if (N == 0) return MQ_OK;
    if (!packed) return MQ_ERR_NULL;
    if (!aligned16(packed)) return MQ_ERR_ALIGN;
    return MQ_OK;
}

// r = bits per stored code, shift = s of the grid the codes live on (8 - r for a plain plane)
static mq_status gemv_dispatch(const uint16_t *x, const uint8_t *packed, const uint16_t *alpha_bf16,
                               const uint16_t *zero_bf16, const mq_overflow *ovf, int64_t B, int64_t N, int64_t K,
                               int r, int shift, uint16_t *y, void *hip_stream, int post = mq::kPostNone,
                               const uint16_t *res = nullptr, void *ws = nullptr, size_t ws_bytes = 0) {
    using namespace mq;
    if (post == kPostResidual && !res && N > 0) return MQ_ERR_NULL;
    if (ovf && K > 65536) return MQ_ERR_SHAPE;
    if (post >= kPostGelu && ovf) return MQ_ERR_SHAPE;
    const mq_status cs = gemv_sliced_check(packed, B, N, K, r, post);
    if (cs != MQ_OK) return cs;
    const int64_t kb = K * r / 8;
    if (N == 0) return MQ_OK;
    if (!x || !alpha_bf16 || !zero_bf16 || !y) return MQ_ERR_NULL;
    if (ovf && (!ovf->row_ptr || !ovf->col_idx)) return MQ_ERR_NULL;
    if (ovf && ovf->capacity < 0) return MQ_ERR_CAPACITY;
    if (!aligned16(x)) return MQ_ERR_ALIGN;

    GemvArgs a;
    a.x = x;
    a.packed = packed;
    a.alpha = alpha_bf16;
    a.zero = zero_bf16;
    a.add_y = ovf ? 1 : 0;
    a.y = y;
    a.B = (int)B;
    a.N = (int)N;
    a.K = (int)K;
    a.KB = (int)kb;
    a.scale = (float)(1 << shift);
    a.post = post;
    a.res = res;

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (ovf) {
        // extra precision: the sparse additions first, as 16-bit sums into y; the dense kernel below adds them to
        // its products before it scales and overwrites y
        const mq_status os = launch_overflow_sums(x, ovf->row_ptr, ovf->col_idx, ovf->capacity, B, N, K, y, st);
        if (os != MQ_OK) return os;
    }
    if (ws) {
        bool handled = false;
        const mq_status ss = launch_gemv_reg_split(a, r, ws, ws_bytes, st, &handled);
        if (ss != MQ_OK || handled) return ss;
    }
    {
        bool handled = false;
        const mq_status qs = launch_gemv_quad(a, r, st, &handled);
        if (qs != MQ_OK || handled) return qs;
        const mq_status rs = launch_gemv_reg(a, r, st, &handled);
        if (rs != MQ_OK || handled) return rs;
    }

    // Rows per wave (16 RG): every activation operand read from LDS serves RG matrix-core products, so
    // tall matrices take two row groups; short ones keep RG = 1 for more waves (measured on the decode
    // shapes at B = 4 and 16: 4096 rows run 10-25 % faster with RG = 1, 14336 rows level or faster with 2;
    // at B = 1 the columns are idle anyway and 11008 and 14336 rows run 6-13 % faster with RG = 1.  A
    // deeper ring did not help at any of these sizes: D = 4 and 5 were 2-10 % slower than 3).
    const int rg = (N >= 8192 && (B > 2 || N >= 16384)) ? 2 : 1;
    // K-split: about 2048 waves in total (8 per compute unit measured best across the decode shapes:
    // enough loads in flight, and the whole grid resident at once) when there are few row blocks,
    // none when the rows alone provide them.  Workgroups have 8 waves (KS of them per row block),
    // or KS when that is larger.
    const int64_t segs = cdiv(kb, line_bytes(r));  // weight lines per row
    const int64_t row_blocks = cdiv(N, 16 * rg);
    int ks = 1;
    // (short matrices with batched activations: shorter slices pay off; at 14336 rows they cost 15-25 %)
    const int64_t wave_budget = (B >= 4 && rg == 1) ? 4096 : 2048;
    while (ks < 16 && row_blocks * ks * 2 <= wave_budget && 2 * ks <= segs) ks <<= 1;
    const int nw = ks > 8 ? ks : 8;
#define MQ_GEMV_CASE(R_, RG_, D_) \
    if (r == R_ && rg == RG_) return launch_gemv<R_, RG_, D_>(a, nw, ks, st);
    MQ_GEMV_CASE(2, 1, 3) MQ_GEMV_CASE(2, 2, 2)
    MQ_GEMV_CASE(4, 1, 4) MQ_GEMV_CASE(4, 2, 2)
    MQ_GEMV_CASE(8, 1, 4) MQ_GEMV_CASE(8, 2, 2)
    MQ_GEMV_CASE(6, 1, 4) MQ_GEMV_CASE(6, 2, 2)
    MQ_GEMV_CASE(3, 1, 4) MQ_GEMV_CASE(3, 2, 2)
#undef MQ_GEMV_CASE
    return MQ_ERR_BITS;
}

mq_status mq::gemv_sliced_post(const uint16_t *x, const uint8_t *packed, const uint16_t *alpha_bf16,
                               const uint16_t *zero_bf16, int64_t B, int64_t N, int64_t K, int r, uint16_t *y, int post,
                               const uint16_t *res, void *hip_stream, void *split_ws, size_t split_ws_bytes) {
    if (r < 1 || r > 8) return MQ_ERR_BITS;
    const bool split = split_ws && gemv_split_workspace_bytes(B, N, K, r) != 0;
    return gemv_dispatch(x, packed, alpha_bf16, zero_bf16, nullptr, B, N, K, r, 8 - r, y, hip_stream, post, res,
                         split ? split_ws : nullptr, split_ws_bytes);
}

extern "C" mq_status mq_gemv_sliced(const uint16_t *x, const uint8_t *packed, const uint16_t *alpha_bf16,
                                    const uint16_t *zero_bf16, const mq_overflow *ovf, int64_t B, int64_t N,
                                    int64_t K, int r, uint16_t *y, void *hip_stream) {
    if (r < 1 || r > 8) return MQ_ERR_BITS;
    return gemv_dispatch(x, packed, alpha_bf16, zero_bf16, ovf, B, N, K, r, 8 - r, y, hip_stream);
}

extern "C" mq_status mq_gemv_sliced_ws(const uint16_t *x, const uint8_t *packed, const uint16_t *alpha_bf16,
                                       const uint16_t *zero_bf16, const mq_overflow *ovf, int64_t B, int64_t N,
                                       int64_t K, int r, uint16_t *y, void *ws, size_t ws_bytes, void *hip_stream) {
    if (r < 1 || r > 8) return MQ_ERR_BITS;
    const size_t need = mq::gemv_split_workspace_bytes(B, N, K, r);
    if (!ws || ws_bytes < std::max<size_t>(256, need) || !mq::aligned16(ws)) return MQ_ERR_WORKSPACE;
    return gemv_dispatch(x, packed, alpha_bf16, zero_bf16, ovf, B, N, K, r, 8 - r, y, hip_stream, mq::kPostNone, nullptr,
                         need ? ws : nullptr, ws_bytes);
}

extern "C" mq_status mq_gemv_sliced_dense_ep(const uint16_t *x, const uint8_t *packed, const uint16_t *alpha_bf16,
                                             const uint16_t *zero_bf16, int64_t B, int64_t N, int64_t K, int r,
                                             uint16_t *y, void *hip_stream) {
    if (r < 1 || r > 7) return MQ_ERR_BITS;
    // codes 0 .. 2^r of the r-bit extra-precision slice, stored with r + 1 bits, one step = 2^(8 - r)
    return gemv_dispatch(x, packed, alpha_bf16, zero_bf16, nullptr, B, N, K, r + 1, 8 - r, y, hip_stream);
}
