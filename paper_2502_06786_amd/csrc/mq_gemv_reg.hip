// mq_gemv_sliced for batches of 5 .. 16 on tall int4 / int2 planes: the activations of a wave's K slice live in
// registers as 16x16x32 bf16 matrix-core operands, so the hot loop touches LDS only to change the lane layout of
// the weight tiles it streams (section 1: decode is bound by moving the weights out of HBM).
//
// A wave owns NL consecutive 128-byte lines of every row (a K slice) and walks over row blocks of 16 rows; all
// slices of a row block sit in one workgroup and meet in LDS at the end.  Weight tiles (16 rows x 128 bytes) are
// fetched as whole lines by eight neighbouring lanes, by direct global->LDS loads into a ring of S tiles per wave
// (a request past the wave's last step is out of range and moves no data, so the number of loads in flight is the
// same in every iteration); lane (i, g) reads pieces g and g + 4 of row i back out of the tile one step before
// use.  Codes become bf16 numbers with one AND-OR per two codes (a field at mantissa bits 0-1 / 2-3 / 4-5 under
// the exponent of 128 / 32 / 8 reads as 128 + c, 32 + c, 8 + c); the offsets leave in the epilogue through
// sum_k x_k offset_k, which comes out of the activation registers next to sum_k x_k (the zero-point term).
#include <algorithm>

#include "mq_gemv.h"

namespace mq {

namespace {
typedef __attribute__((address_space(3))) void *lds_ptr;
constexpr uint32_t kE128 = 0x43004300u, kE32 = 0x42004200u, kE8 = 0x41004100u;
constexpr int kTile = 2048;      // 16 rows x 128 bytes
constexpr int kStreamed = 2;     // non-temporal weight loads

__device__ __forceinline__ f32x4 mfma16(const u32x4 &a, const u32x4 &b, const f32x4 &c) {
    Frag8 fa, fb;
    fa.u = a;
    fb.u = b;
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa.b, fb.b, c, 0, 0, 0);
}
__device__ __forceinline__ uint32_t and_or(uint32_t v, uint32_t mask_s, uint32_t magic_v) { return (v & mask_s) | magic_v; }
__device__ __forceinline__ uint32_t pair_lo(uint32_t first, uint32_t second) { return __builtin_amdgcn_perm(second, first, 0x05040100u); }
__device__ __forceinline__ uint32_t pair_hi(uint32_t first, uint32_t second) { return __builtin_amdgcn_perm(second, first, 0x07060302u); }

struct Consts {
    uint32_t m0, m1, m2;
    uint32_t e128, e32, e8;
};
template <int R>
__device__ __forceinline__ Consts consts() {
    Consts c;
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

// operands per line and lane: int2: 2 pieces x 4 dwords x 2 = 16; int4: 2 x 4 x 1 = 8
template <int R>
constexpr int ops_per_line() { return R == 2 ? 16 : 8; }

// Outputs of rows row0 .. row0 + 3 for batch entry b from the sum of (offset + code) x, the offsets' share xoff and
// the activations' sum xsum.
__device__ __forceinline__ void finish_outputs(const GemvArgs &a, int b, int row0, const f32x4 &dot, float xsum, float xoff,
                                               const float (&al)[4], const float (&ze)[4]) {
    float yv[4];
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
        float d = dot[cc] - xoff;
        // extra precision: the overflow sum of this output waits in y (the kernel before this one wrote it)
        if (a.add_y && row0 + cc < a.N) d += ovf_sum_unpack(a.y[(size_t)b * a.N + row0 + cc]);
        yv[cc] = al[cc] * (a.scale * d - ze[cc] * xsum);
    }
    if (a.post >= kPostGelu) {
#pragma unroll
        for (int cc = 0; cc < 4; cc += 2)
            if (row0 + cc < a.N) a.y[(size_t)b * (a.N >> 1) + ((row0 + cc) >> 1)] = gated_bf16(yv[cc], yv[cc + 1], a.post);
    } else {
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            const size_t at = (size_t)b * a.N + row0 + cc;
            if (row0 + cc < a.N)
                a.y[at] = a.post == kPostResidual ? residual_bf16(a.res[at], yv[cc]) : (uint16_t)float_to_bf16_bits(yv[cc]);
        }
    }
}

// R = bits per code (2 or 4); NL = 128-byte lines per K slice; S = ring depth (tiles per wave)
// Workgroup = KS * RW waves; wave (ks, rw).  Slices ks, ks + KS, ... (rounds) of row blocks rw, rw + RW, ... of the
// workgroup's CH row blocks c * G + blockIdx.
// SPLIT: blockIdx.y picks a group of KS slices (one round); the workgroup leaves its partial products and activation
// sums in global memory (pdot [groups][row blocks][64] x 4 floats, psum [groups][16][2]) for split_reduce_kernel.
template <int R, int NL, int S, int MAXT, bool SPLIT>
__global__ __launch_bounds__(MAXT) void gemv_reg_kernel(GemvArgs a, int KS, int RW, int CH, int NSL_all, f32x4 *pdot,
                                                        float *psum) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    constexpr int OPL = ops_per_line<R>();
    constexpr int CPB = 8 / R;  // codes per byte

    const int tid = threadIdx.x, lane = tid & 63, nthreads = blockDim.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int NW = nthreads >> 6;
    const int ks = wave % KS, rw = wave / KS;
    const int li = lane >> 3, lc = lane & 7;   // fetch: row li (+ 8), piece lc
    const int i = lane & 15, g = lane >> 4;    // compute: row i (A operand) / batch entry i (B operand), k-group g

    const int NRB = (a.N + 15) >> 4;
    const int G = gridDim.x, wg = blockIdx.x;
    const int nblk = (NRB - wg + G - 1) / G;            // row blocks of this workgroup (>= 1)
    const int nv = max(0, (nblk - rw + RW - 1) / RW);   // visits per round (wave-uniform)
    const int SB = SPLIT ? (int)blockIdx.y * KS : 0;    // first slice of this workgroup
    const int NSL = SPLIT ? min(KS, NSL_all - SB) : NSL_all;
    const int nr = (NSL - ks + KS - 1) / KS;            // rounds of this wave
    const int nsteps = nr * nv * NL;

    float *sums = reinterpret_cast<float *>(lds);                                   // [NSL][16][2]
    const int sums_bytes = NSL * 16 * 2 * 4;
    uint8_t *ring = lds + sums_bytes + wave * (S * kTile);
    f32x4 *ypart = reinterpret_cast<f32x4 *>(lds + sums_bytes + NW * S * kTile);    // [NSL][CH][64]

    const __amdgpu_buffer_rsrc_t rwt = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(a.packed), 0, (int)(uint32_t)((size_t)a.N * a.KB), 0x00020000);

    // ---- weight ring --------------------------------------------------------------------------------
    const int lp0 = lc ^ ((li >> 1) & 7), lp1 = lc ^ (((li + 8) >> 1) & 7);
    int iround = 0, ivisit = 0, iln = 0, islot = 0;
    auto issue_next = [&]() {
        const int c = rw + ivisit * RW, rb = c * G + wg;
        const uint32_t gone = (uint32_t)(((nblk - 1 - c) | (nr - 1 - iround)) >> 31) << 31;
        const uint32_t sbase = gone ? 0u : (uint32_t)rb * 16u * (uint32_t)a.KB;
        const int last = a.N - 1 - rb * 16;
        const uint32_t r_a = (uint32_t)max(min(li, last), 0) * (uint32_t)a.KB;
        const uint32_t r_b = (uint32_t)max(min(li + 8, last), 0) * (uint32_t)a.KB;
        const int lb = ((SB + ks + KS * iround) * NL + iln) * 128;
        const uint32_t p_a = (uint32_t)max(min(lb + lp0 * 16, a.KB - 16), 0);
        const uint32_t p_b = (uint32_t)max(min(lb + lp1 * 16, a.KB - 16), 0);
        uint8_t *dst = ring + islot * kTile;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rwt, (lds_ptr)dst, 16, (r_a + p_a) | gone, sbase, 0, kStreamed);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rwt, (lds_ptr)(dst + 1024), 16, (r_b + p_b) | gone, sbase, 0, kStreamed);
        if (++iln == NL) {
            iln = 0;
            if (++ivisit >= nv) ivisit = 0, ++iround;
        }
        islot = islot + 1 == S ? 0 : islot + 1;
    };

    // ---- activations of a slice -> registers (straight from memory: they sit in L2 after the first wave) -------
    // lane (j, g) = (batch entry, k-group) holds, for line ln, piece h (pieces g and g + 4 of the line) and dword w,
    // the activations of the dword's codes in the order the unpack produces them
    u32x4 xr[NL][OPL];
    float s1 = 0.f, s2 = 0.f;
    typedef __bf16 bfp __attribute__((ext_vector_type(2)));
    auto dot2 = [](uint32_t v, uint32_t c, float acc) {
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bfp, v), __builtin_bit_cast(bfp, c), acc, false);
    };
    const bool has_b = i < a.B;
    const uint16_t *xrow = a.x + (size_t)(has_b ? i : 0) * a.K;
    auto load_x = [&](int slice) {
#pragma unroll
        for (int ln = 0; ln < NL; ++ln) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int byte0 = (slice * NL + ln) * 128 + (g + 4 * h) * 16;   // first byte of the piece in the packed row
                if constexpr (R == 2) {
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        const int bytew = byte0 + 4 * w;
                        const bool valid = has_b && bytew < a.KB;
                        const u32x4 *q = reinterpret_cast<const u32x4 *>(xrow + (valid ? bytew * CPB : 0));
                        u32x4 x0 = q[0], x1 = q[1];
                        if (!valid) x0 = x1 = u32x4{0u, 0u, 0u, 0u};
                        xr[ln][(h * 4 + w) * 2] = u32x4{pair_lo(x0.x, x1.x), pair_hi(x0.x, x1.x), pair_lo(x0.y, x1.y), pair_hi(x0.y, x1.y)};
                        xr[ln][(h * 4 + w) * 2 + 1] = u32x4{pair_lo(x0.z, x1.z), pair_hi(x0.z, x1.z), pair_lo(x0.w, x1.w), pair_hi(x0.w, x1.w)};
                    }
                } else if constexpr (R == 4) {
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        const int bytew = byte0 + 4 * w;
                        const bool valid = has_b && bytew < a.KB;
                        const u32x4 *q = reinterpret_cast<const u32x4 *>(xrow + (valid ? bytew * CPB : 0));
                        u32x4 x0 = q[0];
                        if (!valid) x0 = u32x4{0u, 0u, 0u, 0u};
                        xr[ln][h * 4 + w] = u32x4{pair_lo(x0.x, x0.z), pair_hi(x0.x, x0.z), pair_lo(x0.y, x0.w), pair_hi(x0.y, x0.w)};
                    }
                }
            }
#pragma unroll
            for (int o = 0; o < OPL; ++o) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    s1 = dot2(xr[ln][o][c], 0x3F803F80u, s1);
                    if constexpr (R == 2) {
                        // offsets of the registers of an operand pair: 128 32 8 128 | 32 8 128 32
                        const int pos = (o & 1) * 4 + c;
                        const uint32_t off = pos % 3 == 0 ? kE128 : (pos % 3 == 1 ? kE32 : kE8);
                        s2 = dot2(xr[ln][o][c], off, s2);
                    }
                }
            }
        }
    };

    // (requested first: loads return in order, and the waits below count the ring loads only)
    // alpha, z of the first epilogue item of this thread (item = (row block c, output lane): 4 rows x 1 batch entry)
    const int items = nblk * 64;
    float pal[4], pze[4];
    if constexpr (!SPLIT) {
        const int it = tid < items ? tid : 0;
        const int c = it >> 6, ol = it & 63;
        const int row0 = (c * G + wg) * 16 + 4 * (ol >> 4);
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            const int row = min(row0 + cc, a.N - 1);
            pal[cc] = bf16_bits_to_float(a.alpha[row]);
            pze[cc] = bf16_bits_to_float(a.zero[row]);
        }
    }

    if (nr > 0 && nv > 0) load_x(SB + ks);
#pragma unroll
    for (int st = 0; st < S; ++st) issue_next();


    // ---- main loop -------------------------------------------------------------------------------------
    static_assert(S >= 2 && S <= 16, "ring depth");
    constexpr int U = (NL % 2 == 0) ? NL : 2 * NL;
    const uint32_t rslot0 = (uint32_t)(8 * i + (g ^ ((i >> 1) & 7))) << 4;
    const uint32_t rslot1 = (uint32_t)(8 * i + ((4 + g) ^ ((i >> 1) & 7))) << 4;
    auto read_tile = [&](int slot, u32x4 (&dst)[2]) {
        const uint8_t *tile = ring + slot * kTile;
        dst[0] = *reinterpret_cast<const u32x4 *>(tile + rslot0);
        dst[1] = *reinterpret_cast<const u32x4 *>(tile + rslot1);
    };
    const Consts qc = consts<R>();
    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    u32x4 wt[2][2];
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * (S - 1)) : "memory");
    read_tile(0, wt[0]);
    int nslot = 1;
    int vcur = 0, rcur = 0;
    for (int s0 = 0; s0 < nsteps; s0 += U) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int ln = u % NL, par = u & 1;
            const bool active = s0 + u < nsteps;
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * (S - 2)) : "memory");
            read_tile(nslot, wt[par ^ 1]);
            asm volatile("s_waitcnt lgkmcnt(2)" ::: "memory");
            issue_next();
            nslot = nslot + 1 == S ? 0 : nslot + 1;
            __builtin_amdgcn_sched_barrier(0);
            if (active) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    if constexpr (R == 2) {
#pragma unroll
                        for (int w = 0; w < 4; ++w) {
                            const uint32_t d = wt[par][h][w], d6 = d >> 6, d12 = d >> 12;
                            const u32x4 a0 = {and_or(d, qc.m0, qc.e128), and_or(d, qc.m1, qc.e32), and_or(d, qc.m2, qc.e8),
                                              and_or(d6, qc.m0, qc.e128)};
                            const u32x4 a1 = {and_or(d6, qc.m1, qc.e32), and_or(d6, qc.m2, qc.e8), and_or(d12, qc.m0, qc.e128),
                                              and_or(d12, qc.m1, qc.e32)};
                            acc0 = mfma16(a0, xr[ln][(h * 4 + w) * 2], acc0);
                            acc1 = mfma16(a1, xr[ln][(h * 4 + w) * 2 + 1], acc1);
                        }
                    } else if constexpr (R == 4) {
#pragma unroll
                        for (int w = 0; w < 4; ++w) {
                            const uint32_t d = wt[par][h][w];
                            const u32x4 a0 = {and_or(d, qc.m0, qc.e128), and_or(d >> 4, qc.m0, qc.e128),
                                              and_or(d >> 8, qc.m0, qc.e128), and_or(d >> 12, qc.m0, qc.e128)};
                            if (w & 1) acc1 = mfma16(a0, xr[ln][h * 4 + w], acc1);
                            else acc0 = mfma16(a0, xr[ln][h * 4 + w], acc0);
                        }
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (ln == NL - 1 && active) {
                const f32x4 sum = acc0 + acc1;
                const int cblk = rw + vcur * RW;
                ypart[((ks + KS * rcur) * CH + cblk) * 64 + lane] = sum;
                acc0 = acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
                if (++vcur == nv) {
                    vcur = 0;
                    // the sums of this slice's activations: over the four k-groups of a batch entry
                    s1 += __shfl_xor(s1, 16);
                    s1 += __shfl_xor(s1, 32);
                    s2 += __shfl_xor(s2, 16);
                    s2 += __shfl_xor(s2, 32);
                    if (lane < 16 && rw == 0) {
                        sums[((ks + KS * rcur) * 16 + lane) * 2] = s1;
                        sums[((ks + KS * rcur) * 16 + lane) * 2 + 1] = R == 2 ? s2 : 128.f * s1;
                    }
                    s1 = s2 = 0.f;
                    if (++rcur < nr) load_x(SB + ks + KS * rcur);
                }
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // ---- epilogue ---------------------------------------------------------------------------------------
    __syncthreads();
    for (int it = tid, m = 0; it < items; it += nthreads, ++m) {
        const int c = it >> 6, ol = it & 63, b = ol & 15;
        if (b >= a.B) continue;
        const int row0 = (c * G + wg) * 16 + 4 * (ol >> 4);
        if (row0 >= a.N) continue;
        float xsum = 0.f, xoff = 0.f;
        f32x4 dot = {0.f, 0.f, 0.f, 0.f};
        for (int sl0 = 0; sl0 < NSL; sl0 += 8) {   // eight slices at a time: their LDS reads are independent
            float xs[8], xo[8];
            f32x4 dp[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int sl = min(sl0 + q, NSL - 1);
                xs[q] = sums[(sl * 16 + b) * 2];
                xo[q] = sums[(sl * 16 + b) * 2 + 1];
                dp[q] = ypart[(sl * CH + c) * 64 + ol];
            }
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (sl0 + q < NSL) {
                    xsum += xs[q];
                    xoff += xo[q];
                    dot += dp[q];
                }
        }
        if constexpr (SPLIT) {
            pdot[((size_t)blockIdx.y * NRB + (c * G + wg)) * 64 + ol] = dot;
            if (wg == 0 && c == 0 && ol < 16) {
                psum[(blockIdx.y * 16 + b) * 2] = xsum;
                psum[(blockIdx.y * 16 + b) * 2 + 1] = xoff;
            }
        } else {
            float al[4], ze[4];
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                if (m == 0) {
                    al[cc] = pal[cc], ze[cc] = pze[cc];
                } else {
                    const int row = min(row0 + cc, a.N - 1);
                    al[cc] = bf16_bits_to_float(a.alpha[row]), ze[cc] = bf16_bits_to_float(a.zero[row]);
                }
            }
            finish_outputs(a, b, row0, dot, xsum, xoff, al, ze);
        }
    }
}

// second kernel of the split form: adds the groups' partial results in a fixed order and finishes the outputs
__global__ __launch_bounds__(256) void split_reduce_kernel(GemvArgs a, int SG, const f32x4 *pdot, const float *psum) {
    const int NRB = (a.N + 15) >> 4;
    const int it = blockIdx.x * 256 + threadIdx.x;
    if (it >= NRB * 64) return;
    const int rb = it >> 6, ol = it & 63, b = ol & 15;
    const int row0 = rb * 16 + 4 * (ol >> 4);
    if (b >= a.B || row0 >= a.N) return;
    float al[4], ze[4];
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
        const int row = min(row0 + cc, a.N - 1);
        al[cc] = bf16_bits_to_float(a.alpha[row]), ze[cc] = bf16_bits_to_float(a.zero[row]);
    }
    float xsum = 0.f, xoff = 0.f;
    f32x4 dot = {0.f, 0.f, 0.f, 0.f};
    for (int g0 = 0; g0 < SG; g0 += 8) {
        f32x4 dp[8];
        float xs[8], xo[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int sg = min(g0 + q, SG - 1);
            dp[q] = pdot[((size_t)sg * NRB + rb) * 64 + ol];
            xs[q] = psum[(sg * 16 + b) * 2];
            xo[q] = psum[(sg * 16 + b) * 2 + 1];
        }
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if (g0 + q < SG) {
                dot += dp[q];
                xsum += xs[q];
                xoff += xo[q];
            }
    }
    finish_outputs(a, b, row0, dot, xsum, xoff, al, ze);
}


struct RegPlan {
    int nl, nsl, ks, ch, grid, depth;
    size_t lds;
};

template <int R, int NL, int S, int MAXT>
mq_status launch_reg(const GemvArgs &a, const RegPlan &p, hipStream_t st) {
    auto kern = gemv_reg_kernel<R, NL, S, MAXT, false>;
    if (p.lds > 65536 && hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                             (int)p.lds) != hipSuccess)
        return MQ_ERR_DEVICE;
    kern<<<dim3(p.grid), dim3(64 * p.ks), p.lds, st>>>(a, p.ks, 1, p.ch, p.nsl, nullptr, nullptr);
    return launch_status();
}

// the split form: groups of p.ks slices in blockIdx.y, then the reduction
template <int R, int NL, int S>
mq_status launch_reg_split(const GemvArgs &a, const RegPlan &p, int groups, void *ws, hipStream_t st) {
    auto kern = gemv_reg_kernel<R, NL, S, 256, true>;
    if (p.lds > 65536 && hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                             (int)p.lds) != hipSuccess)
        return MQ_ERR_DEVICE;
    const int nrb = (a.N + 15) / 16;
    f32x4 *pdot = static_cast<f32x4 *>(ws);
    float *psum = reinterpret_cast<float *>(pdot + (size_t)groups * nrb * 64);
    kern<<<dim3(p.grid, groups), dim3(64 * p.ks), p.lds, st>>>(a, p.ks, 1, p.ch, p.nsl, pdot, psum);
    mq_status s = launch_status();
    if (s != MQ_OK) return s;
    split_reduce_kernel<<<dim3((nrb * 64 + 255) / 256), dim3(256), 0, st>>>(a, groups, pdot, psum);
    return launch_status();
}

// Split plan: workgroups of four waves (four slices), every wave visiting p.ch row blocks; about one workgroup per
// compute unit (measured best on 4096 x 14336 and 4608 x 36864 at B = 8 and 16: 13 us against 25, 25 against 94; two
// to four per compute unit cost 10-35 % more, their activation loads grow with the number of workgroups).
// Used for long rows and few of them: at least four groups of slices and at most 8192 rows; elsewhere the one-kernel
// forms are level or faster (4096 x 4096, 14336 x 4096 and taller: 1.0-1.5x the time).
bool split_plan(const GemvArgs &a, int r, RegPlan *p, int *groups) {
    if (a.B <= 4 || (r != 2 && r != 4) || (a.KB & 127) != 0 || (int64_t)a.N * a.KB > 0x7FFFFFFFll) return false;
    const int lines = a.KB >> 7, nrb = (a.N + 15) / 16;
    p->nl = r == 2 ? 1 : 2;
    if (lines % p->nl) p->nl = 1;
    p->nsl = lines / p->nl;
    p->ks = std::min(4, p->nsl);
    *groups = (p->nsl + p->ks - 1) / p->ks;
    if (*groups < 4 || a.N > 8192) return false;
    p->depth = 3;
    const int row_groups = std::max(1, 256 / *groups);
    p->ch = (nrb + row_groups - 1) / row_groups;
    p->grid = (nrb + p->ch - 1) / p->ch;
    p->lds = (size_t)p->ks * 128 + (size_t)p->ks * p->depth * kTile + (size_t)p->ks * p->ch * 1024;
    return p->lds <= 160 * 1024;
}

}  // namespace

// Returns MQ_OK with *handled = false when the shape is outside what this kernel is used for.
mq_status launch_gemv_reg(const GemvArgs &a, int r, hipStream_t st, bool *handled) {
    *handled = false;
    if (a.B <= 4 || (r != 2 && r != 4) || (a.KB & 127) != 0) return MQ_OK;
    const int lines = a.KB >> 7, nrb = (a.N + 15) / 16;
    // Measured against the general kernel at B = 16: 0.8x its time on 36864 x 4608 (int2 and int4), level on
    // 28672 x 4096, slower on 14336 rows and below (too few row blocks per wave for the activation registers to pay).
    if (nrb < 2048) return MQ_OK;
    RegPlan p{};
    p.nl = r == 2 ? 1 : 2;                 // 64 activation registers per int2 line, 32 per int4 line
    if (lines % p.nl) p.nl = 1;
    p.nsl = lines / p.nl;
    if (p.nsl > 16) return MQ_OK;          // one wave per slice, at most 16 waves
    p.ks = p.nsl;
    // The whole grid resident at once, as many workgroups per compute unit as LDS and the 16 wave slots allow; planes
    // with so many row blocks that a workgroup's partial outputs would not fit LDS run in two to four equal rounds.
    p.depth = 0;
    for (int rounds = 1; rounds <= 4 && !p.depth; ++rounds)
        for (int depth : {3, 2}) {
            for (int per_cu = std::max(1, 16 / p.ks); per_cu >= 1 && !p.depth; --per_cu) {
                const int grid = std::min(nrb, 256 * per_cu * rounds), ch = (nrb + grid - 1) / grid;
                const size_t lds = (size_t)p.nsl * 128 + (size_t)p.ks * depth * kTile + (size_t)p.nsl * ch * 1024;
                if (lds * per_cu <= 160 * 1024) {
                    p.depth = depth;
                    p.ch = ch;
                    p.grid = (nrb + ch - 1) / ch;
                    p.lds = lds;
                }
            }
            if (p.depth) break;
        }
    if (!p.depth || (int64_t)a.N * a.KB > 0x7FFFFFFFll) return MQ_OK;
    *handled = true;
#define MQ_REG_CASE(R_, NL_)                                                   \
    if (r == R_ && p.nl == NL_) {                                              \
        if (p.depth == 3) return launch_reg<R_, NL_, 3, 1024>(a, p, st);       \
        return launch_reg<R_, NL_, 2, 1024>(a, p, st);                         \
    }
    MQ_REG_CASE(2, 1) MQ_REG_CASE(4, 1) MQ_REG_CASE(4, 2)
#undef MQ_REG_CASE
    *handled = false;
    return MQ_OK;
}

size_t gemv_split_workspace_bytes(int64_t B, int64_t N, int64_t K, int r) {
    if (B < 1 || N < 1 || K < 1 || (r != 2 && r != 4) || (K * r) % 8 != 0) return 0;
    const int64_t kb = K * r / 8;
    if (kb & 127) return 0;
    const int64_t lines = kb >> 7, nl = (r == 4 && lines % 2 == 0) ? 2 : 1, nsl = lines / nl;
    const int64_t groups = (nsl + 3) / 4, nrb = (N + 15) / 16;
    if (B <= 4 || groups < 4 || N > 8192) return 0;   // (the conditions of split_plan)
    return (size_t)(groups * nrb * 1024 + groups * 128);
}

mq_status launch_gemv_reg_split(const GemvArgs &a, int r, void *ws, size_t ws_bytes, hipStream_t st, bool *handled) {
    *handled = false;
    RegPlan p{};
    int groups = 0;
    if (!split_plan(a, r, &p, &groups)) return MQ_OK;
    if (!ws || ws_bytes < gemv_split_workspace_bytes(a.B, a.N, a.K, r) || !aligned16(ws)) return MQ_ERR_WORKSPACE;
    *handled = true;
    if (r == 2) return launch_reg_split<2, 1, 3>(a, p, groups, ws, st);
    if (p.nl == 2) return launch_reg_split<4, 2, 3>(a, p, groups, ws, st);
    return launch_reg_split<4, 1, 3>(a, p, groups, ws, st);
}

}  // namespace mq
