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
// A wave owns NL consecutive 128-byte lines of every row (a K slice) and walks over row blocks of 16
// rows ("visits"); all slices of a row block sit in one workgroup and meet in LDS at the end.  Weight
// lines are fetched as whole 128-byte lines by eight neighbouring lanes, by direct global->LDS loads
// into a ring of 2 KB tiles per wave, a few steps ahead (a request past the wave's last step is out
// of range: it moves no data, so the number of loads in flight is the same in every iteration); the
// compute layout (lane = row and 16-byte piece) is read back out of the tile one step before use.
//
// Codes become bf16 numbers with one AND-OR per two codes: a field at mantissa bits 0-1 / 2-3 / 4-5
// under the exponent of 128 / 32 / 8 reads as 128 + c, 32 + c, 8 + c.  The offsets leave in the
// epilogue through sum_k x_k * offset_k, which comes out of the activation registers next to
// sum_k x_k (the zero-point term).
#include <algorithm>

#include "mq_gemv.h"

namespace mq {

namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kE128 = 0x43004300u, kE32 = 0x42004200u, kE8 = 0x41004100u;  // (128,128) (32,32) (8,8)
constexpr uint32_t kOutOfRange = 0x80000000u;
constexpr int kStreamed = 2;  // cache policy of the weight loads: non-temporal (each byte is read once; measured 7-9 % more read bandwidth)
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

// R = bits per code (4 or 2), NL = 128-byte lines of a row per K slice, S = tiles in a wave's ring.
// Workgroup = KS * RW waves; wave (ks, rw) = (wave % KS, wave / KS) takes the slices ks, ks + KS, ...
// (one "round" each) of the workgroup's row blocks number rw, rw + RW, ...  The workgroup owns every
// G-th row block (G = workgroups in the grid): its c-th one is row block c * G + blockIdx, c < CH, so
// that at any time the requests of the whole grid fall into one narrow window of the matrix that
// moves from its first row to its last.
template <int R, int NL, int S>
__global__ __launch_bounds__(512) void gemv_quad_kernel(GemvArgs a, int KS, int RW, int CH, int NSL) {
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
    const int G = gridDim.x, wg = blockIdx.x;
    const int nblk = (NRB - wg + G - 1) / G;             // row blocks of this workgroup (>= 1)
    const int nv = max(0, (nblk - rw + RW - 1) / RW);    // visits per round of this wave (wave-uniform)
    const int nr = (NSL - ks + KS - 1) / KS;             // rounds of this wave: slices ks + KS r < NSL
    const int nsteps = nr * nv * NL;

    float *sums = reinterpret_cast<float *>(lds);
    uint8_t *ring = lds + kSumsBytes + wave * (S * kTileBytes);                          // S tiles of 16 rows x 128 bytes
    f32x4 *ypart = reinterpret_cast<f32x4 *>(lds + kSumsBytes + NW * S * kTileBytes);    // [NSL][CH * 16]
    // activations of the whole workgroup: row b at b * xpitch, natural order, zero-filled up to a whole 512-k block
    const int kblocks = (a.K + 511) >> 9;
    const int xpitch = kblocks * 1024 + kXPad;
    const uint8_t *xbuf = lds + kSumsBytes + NW * S * kTileBytes + NSL * CH * 16 * (int)sizeof(f32x4);

    const __amdgpu_buffer_rsrc_t rwt = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(a.packed), 0, (int)(uint32_t)((size_t)a.N * a.KB), 0x00020000);
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(a.x), 0, (int)((uint32_t)a.B * (uint32_t)a.K * 2u), 0x00020000);

    // ---- activations -> LDS (direct loads, 1 KB = 512 k of one batch entry per wave instruction) --------
    for (int j = wave; j < a.B * kblocks; j += NW) {
        const int bj = j / kblocks, kb = j - bj * kblocks;
        const int k = kb * 512 + lane * 8;
        const uint32_t vo = k < a.K ? ((uint32_t)bj * (uint32_t)a.K + (uint32_t)k) * 2u : kOutOfRange;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_ptr)(const_cast<uint8_t *>(xbuf) + bj * xpitch + kb * 1024), 16,
                                                 vo, 0, 0, 0);
    }

    // alpha and z of the first outputs this thread will write, requested ahead.
    // output idx = (b * nblk + c) * 16 + i: row (c * G + wg) * 16 + i of batch entry b
    const int total_out = a.B * nblk * 16;
    auto out_row = [&](int idx) { return (((idx >> 4) % nblk) * G + wg) * 16 + (idx & 15); };
    constexpr int PF = 2;
    float pal[PF], pze[PF];
#pragma unroll
    for (int m = 0; m < PF; ++m) {
        const int idx = tid + m * nthreads;
        const int row = min(out_row(idx < total_out ? idx : 0), a.N - 1);
        pal[m] = bf16_bits_to_float(a.alpha[row]);
        pze[m] = bf16_bits_to_float(a.zero[row]);
    }

    // ---- weight ring: S tiles per wave in LDS, filled by direct loads ----------------------------------
    // Step s of the wave = line s % NL of visit (s / NL) % nv of round s / (NL nv).  Lane l of a load
    // lands at byte 16 l of its half of the tile; it fetches piece (l % 8) ^ swz(row) of row l / 8
    // (+ 8), so that the tile reads [row][piece ^ swz(row)], swz(row) = row / 2 % 8: whole 128-byte
    // lines on the memory side, and the row-shaped reads of the compute layout hit every bank once.
    const int lp0 = lc ^ ((li >> 1) & 7), lp1 = lc ^ (((li + 8) >> 1) & 7);  // pieces this lane fetches
    int iround = 0, ivisit = 0, iln = 0, islot = 0;  // the next step to request and the slot it goes to
    auto issue_next = [&]() {
        const int c = rw + ivisit * RW, rb = c * G + wg;
        // bit 31 of the offset set when the step does not exist: such a request is out of range, moves
        // no data and still counts as a load in flight (arithmetic on purpose, no branch)
        const uint32_t gone = (uint32_t)(((nblk - 1 - c) | (nr - 1 - iround)) >> 31) << 31;
        // the row block's first byte goes into the scalar offset; rows past the last one re-read it
        const uint32_t sbase = gone ? 0u : (uint32_t)rb * 16u * (uint32_t)a.KB;
        const int last = a.N - 1 - rb * 16;
        const uint32_t r_a = (uint32_t)max(min(li, last), 0) * (uint32_t)a.KB;
        const uint32_t r_b = (uint32_t)max(min(li + 8, last), 0) * (uint32_t)a.KB;
        const int lb = ((ks + KS * iround) * NL + iln) * 128;
        const uint32_t p_a = (uint32_t)max(min(lb + lp0 * 16, a.KB - 16), 0);
        const uint32_t p_b = (uint32_t)max(min(lb + lp1 * 16, a.KB - 16), 0);
        uint8_t *dst = ring + islot * kTileBytes;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rwt, (lds_ptr)dst, 16, (r_a + p_a) | gone, sbase, 0, kStreamed);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rwt, (lds_ptr)(dst + 1024), 16, (r_b + p_b) | gone, sbase, 0, kStreamed);
        if (++iln == NL) {
            iln = 0;
            if (++ivisit >= nv) ivisit = 0, ++iround;
        }
        islot = islot + 1 == S ? 0 : islot + 1;
    };
#pragma unroll
    for (int st = 0; st < S; ++st) issue_next();  // the first S steps are requested now
    // the staged activations are older than the 2 S weight loads requested since, and loads return in order
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * S) : "memory");
    // (the bare barrier: a fence here would wait for the tiles still on their way, which no other wave reads)
    __builtin_amdgcn_s_barrier();

    // ---- activations of a slice -> registers --------------------------------------------------------
    // pair p of line ln, lane (g, t, b): quad 4 p + t of the lane's stream of the line, i.e. the dwords
    // of x that hold codes (2u, 2u + 1) and (2u + CPD/2, 2u + 1 + CPD/2) of the quad's weight dword,
    // rearranged to the operand order (2u, 2u + CPD/2, 2u + 1, 2u + 1 + CPD/2).  sum_k x and
    // sum_k x * offset_k come out of the same registers (every activation of the slice sits in
    // exactly one lane); line ln is summed by the wave with rw == ln % RW.
    u32x2 xr[NL][XP];
    float s1 = 0.f, s2 = 0.f;
    // offset of code position k % 8 at int2: 128 32 8 128 32 8 128 32; lane t holds positions 2t, 2t + 1 in
    // its first register (both halves) and its second
    const float off_a = R != 2 ? 128.f : (t == 1 ? 8.f : (t == 2 ? 32.f : 128.f));
    const float off_b = R != 2 ? 128.f : (t == 1 ? 128.f : (t == 2 ? 8.f : 32.f));
    const uint32_t offs_a = pack_bf16x2(off_a, off_a), offs_b = pack_bf16x2(off_b, off_b);
    typedef __bf16 bfp __attribute__((ext_vector_type(2)));
    auto dot2 = [](uint32_t v, uint32_t c, float acc) {
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bfp, v), __builtin_bit_cast(bfp, c), acc, false);
    };
    const uint8_t *xrow = xbuf + min(b, a.B - 1) * xpitch;
    auto load_x = [&](int slice) {
#pragma unroll
        for (int ln = 0; ln < NL; ++ln) {
#pragma unroll
            for (int p = 0; p < XP; ++p) {
                const int qi = 4 * p + t, dwi = qi / QD, u = qi % QD, h = dwi >> 2, w = dwi & 3;
                const int byte_in_row = (slice * NL + ln) * 128 + (g + 4 * h) * 16 + 4 * w;
                const bool valid = byte_in_row < a.KB && b < a.B;
                const uint32_t *q = reinterpret_cast<const uint32_t *>(xrow + (valid ? (byte_in_row * CPB + 2 * u) * 2 : 0));
                const uint32_t first = valid ? q[0] : 0u, second = valid ? q[CPD / 4] : 0u;
                xr[ln][p] = u32x2{__builtin_amdgcn_perm(second, first, 0x05040100u),   // (first.lo, second.lo)
                                  __builtin_amdgcn_perm(second, first, 0x07060302u)};  // (first.hi, second.hi)
            }
            if (ln % RW == rw) {
#pragma unroll
                for (int p = 0; p < XP; ++p) {
                    s1 = dot2(xr[ln][p].x, 0x3F803F80u, s1);
                    s1 = dot2(xr[ln][p].y, 0x3F803F80u, s1);
                    if constexpr (R == 2) {
                        s2 = dot2(xr[ln][p].x, offs_a, s2);
                        s2 = dot2(xr[ln][p].y, offs_b, s2);
                    }
                }
            }
        }
    };
    if (nr > 0) load_x(ks);

    // ---- main loop ------------------------------------------------------------------------------------
    // In the iteration of step s: the tile of step s + 1 has landed (all but the 2 (S - 2) newest loads
    // are back; loads return in order) and is read into the other register set; the reads of step s,
    // issued an iteration ago, are complete by then, so its slot is requested again for step s + S;
    // then step s is computed.  LDS operations of one wave execute in order.
    static_assert(S >= 2 && S <= 16, "ring depth");
    constexpr int U = (NL % 2 == 0) ? NL : 2 * NL;  // steps per unrolled iteration: line and register set known
    const uint32_t rslot0 = (uint32_t)(8 * i + (g ^ ((i >> 1) & 7))) << 4;
    const uint32_t rslot1 = (uint32_t)(8 * i + ((4 + g) ^ ((i >> 1) & 7))) << 4;
    auto read_tile = [&](int slot, u32x4 (&dst)[2]) {
        const uint8_t *tile = ring + slot * kTileBytes;
        dst[0] = *reinterpret_cast<const u32x4 *>(tile + rslot0);
        dst[1] = *reinterpret_cast<const u32x4 *>(tile + rslot1);
    };
    const QuadConsts qc = quad_consts<R>();
    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    u32x4 wt[2][2];
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * (S - 1)) : "memory");  // step 0 has landed
    read_tile(0, wt[0]);
    int nslot = 1;            // slot of step s + 1 (islot = slot of step s + S = slot of step s)
    int vcur = 0, rcur = 0;   // visit and round of step s
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
                for (int dwi = 0; dwi < 8; ++dwi)
                    quad_dword<R, XP>(wt[par][dwi >> 2][dwi & 3], dwi, xr[ln], qc, acc0, acc1);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (ln == NL - 1 && active) {
                // accumulator register b = y[b] of row i, k-group g: add the four k-groups
                f32x4 sum = acc0 + acc1;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    sum[c] += __shfl_xor(sum[c], 16);
                    sum[c] += __shfl_xor(sum[c], 32);
                }
                const int cblk = rw + vcur * RW;  // row block inside the workgroup's list
                if (g == 0) ypart[((ks + KS * rcur) * CH + cblk) * 16 + i] = sum;
                acc0 = acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
                if (++vcur == nv) {  // next round: the activations of the next slice
                    vcur = 0;
                    if (++rcur < nr) load_x(ks + KS * rcur);
                }
            }
        }
    }
    // every request of this wave (the last ones are out of range) is back before its tiles are given up
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int m = 4; m < 64; m <<= 1) {  // over the lanes of one batch entry
        s1 += __shfl_xor(s1, m);
        s2 += __shfl_xor(s2, m);
    }
    if (lane < 4) {
        sums[(wave * 4 + lane) * 2] = s1;
        sums[(wave * 4 + lane) * 2 + 1] = R == 2 ? s2 : 128.f * s1;
    }

    // ---- epilogue: y[b, n] = alpha_n * (2^s * (sum_k (offset_k + code) x - sum_k offset_k x) - z_n * sum_k x) --
    __syncthreads();
    const float kScale = a.scale;
    for (int idx = tid, m = 0; idx < total_out; idx += nthreads, ++m) {
        const int bb = idx / (nblk * 16), r = idx - bb * (nblk * 16), row = out_row(idx);
        const bool live = row < a.N;
        if (!live && a.post < kPostGelu) continue;
        float xsum = 0.f, xoff = 0.f;
        for (int w = 0; w < NW; ++w) {
            xsum += sums[(w * 4 + bb) * 2];
            xoff += sums[(w * 4 + bb) * 2 + 1];
        }
        float dot = 0.f;
        for (int k = 0; k < NSL; ++k) dot += ypart[k * CH * 16 + r][bb];
        // extra precision: the overflow sum of this output waits in y (the kernel before this one wrote it)
        if (a.add_y && live) dot += ovf_sum_unpack(a.y[(size_t)bb * a.N + row]);
        float al, ze;
        if (m < PF) {
            al = m == 0 ? pal[0] : pal[1];
            ze = m == 0 ? pze[0] : pze[1];
        } else {
            al = live ? bf16_bits_to_float(a.alpha[row]) : 0.f;
            ze = live ? bf16_bits_to_float(a.zero[row]) : 0.f;
        }
        const float yv = al * (kScale * (dot - xoff) - ze * xsum);
        if (a.post >= kPostGelu) {
            // neighbouring threads hold neighbouring rows of one 16-row block: the even one of a
            // (gate, up) pair takes the up value from its neighbour (the trip count of this loop is
            // the same for both, total_out and the thread count being even)
            const float up = __shfl_xor(yv, 1);
            if (live && !(row & 1)) a.y[(size_t)bb * (a.N >> 1) + (row >> 1)] = gated_bf16(yv, up, a.post);
        } else {
            a.y[(size_t)bb * a.N + row] = (uint16_t)float_to_bf16_bits(yv);
        }
    }
}

struct QuadPlan {
    int nl, nsl, ks, rw, ch, grid, depth;
    size_t lds;
};

template <int R, int NL, int S>
mq_status launch_quad(const GemvArgs &a, const QuadPlan &p, hipStream_t st) {
    auto kern = gemv_quad_kernel<R, NL, S>;
    if (p.lds > 65536 && hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.lds) != hipSuccess)
        return MQ_ERR_DEVICE;
    kern<<<dim3(p.grid), dim3(64 * p.ks * p.rw), p.lds, st>>>(a, p.ks, p.rw, p.ch, p.nsl);
    return launch_status();
}

}  // namespace

mq_status launch_gemv_quad(const GemvArgs &a, int r, hipStream_t st, bool *handled) {
    *handled = false;
    if (a.B > 4 || (r != 2 && r != 4) || a.post == kPostResidual) return MQ_OK;
    const int lines = (a.KB + 127) / 128;
    const int nrb = (a.N + 15) / 16;
    // Measured against the general kernel on 4096..36864 rows: 0.85-0.9x the time at 36864 x 4608, level or
    // slower at 14336 rows and below, where a launch is bound by latencies and not by bytes.
    if (nrb < 1024) return MQ_OK;
    // Lines per slice: no padded lines if possible, then about four slices per row (measured over the
    // decode shapes: fewer leave a workgroup with too few waves, more spend their time filling activation
    // registers), one round.
    QuadPlan p{};
    {
        int best = -1, best_cost = 0;
        for (int nl = 1; nl <= 4; ++nl) {
            const int nsl = (lines + nl - 1) / nl, pad = nsl * nl - lines;
            const int cost = pad * 8 + (nsl > 8 ? 4 : 0) + std::abs(nsl - 4);
            if (best < 0 || cost < best_cost) best = nl, best_cost = cost;
        }
        p.nl = best;
        if (p.nl < 1 || p.nl > 4) return MQ_ERR_SHAPE;
    }
    p.nsl = (lines + p.nl - 1) / p.nl;
    // Slices per round: all of them up to eight waves, otherwise the largest divisor (every wave the
    // same number of rounds), otherwise eight.
    p.ks = std::min(p.nsl, 8);
    if (p.nsl > 8)
        for (int d = 8; d >= 5; --d)
            if (p.nsl % d == 0) {
                p.ks = d;
                break;
            }
    if (p.ks < 1 || p.ks > 8) return MQ_ERR_SHAPE;
    // waves per compute unit the grid is sized for (measured on 16384..73728 rows: 12 is best at B = 1, within 2 % of the
    // best everywhere; at B = 4, where a wave's activation registers take four times as long to fill, 8 is 5-10 % faster
    // on the tall planes; 6, 16 and 24 are slower)
    const int wpc = a.B > 2 ? 8 : 12;
    // Row-block waves per workgroup and row blocks per workgroup: the whole grid resident at once
    // (wpc waves per compute unit), every wave the same number of visits where the shape allows.
    p.rw = 1;
    if (p.rw < 1 || p.rw * p.ks > 8) return MQ_ERR_SHAPE;
    const int nw = p.ks * p.rw;
    const int per_cu = std::max(1, wpc / nw);
    const int capacity = 256 * per_cu;
    const int visits = (int)cdiv(nrb, (int64_t)capacity * p.rw);  // per wave and round
    p.ch = visits * p.rw;
    if (p.ch < 1) return MQ_ERR_SHAPE;
    p.grid = (int)cdiv(nrb, p.ch);
    p.ch = (int)cdiv(nrb, p.grid);  // (the most row blocks any workgroup gets)
    // Ring depth, as far as the LDS of a compute unit (160 KB, shared by per_cu workgroups) allows.
    const size_t fixed = kSumsBytes + (size_t)p.nsl * p.ch * 16 * sizeof(f32x4) +
                         (size_t)a.B * (((size_t)a.K + 511) / 512 * 1024 + kXPad);
    const size_t budget = (size_t)160 * 1024 / per_cu;
    p.depth = 0;
    for (int d : {3, 2}) {  // (deeper rings measured slower: three steps in flight per wave are enough)
        if (fixed + (size_t)nw * d * kTileBytes > budget) continue;
        p.depth = d;
        break;
    }
    if (p.depth == 0) return MQ_OK;
    p.lds = fixed + (size_t)nw * p.depth * kTileBytes;
    if (p.lds > 160 * 1024 || (int64_t)a.N * a.KB > 0x7FFFFFFFll || (int64_t)a.B * a.K * 2 > 0x7FFFFFFFll)
        return MQ_OK;
    *handled = true;
#define MQ_QUAD_CASE(R_, NL_)                                             \
    if (r == R_ && p.nl == NL_) {                                         \
        if (p.depth == 3) return launch_quad<R_, NL_, 3>(a, p, st);       \
        if (p.depth == 2) return launch_quad<R_, NL_, 2>(a, p, st);       \
    }
    MQ_QUAD_CASE(2, 1) MQ_QUAD_CASE(2, 2) MQ_QUAD_CASE(2, 3) MQ_QUAD_CASE(2, 4)
    MQ_QUAD_CASE(4, 1) MQ_QUAD_CASE(4, 2) MQ_QUAD_CASE(4, 3) MQ_QUAD_CASE(4, 4)
#undef MQ_QUAD_CASE
    *handled = false;
    return MQ_OK;
}

}  // namespace mq
