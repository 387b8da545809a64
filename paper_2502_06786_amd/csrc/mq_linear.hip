// mq_linear_fwd_multi / mq_linear_bwd: the nested quantized linear on the bf16 matrix cores.
//
// Forward (MatQuant objective, section 3.2: the same input goes through the layer once per
// bit-width): ONE pass over X and the int8 codes.  A workgroup (256 threads, one wave per SIMD) owns
// 128 output channels x 32 MB tokens (MB = 4 or 5); four LDS stages of a [32 MB x 64] bf16 tile of X
// and a [128 x 64] tile of int8 codes are filled by direct global->LDS loads, every wave turns the
// codes of its 32 channels into one bf16 operand per requested bit-width in registers and issues
// 32x32x16 MFMAs into one accumulator set per bit-width.
//
//   r = 8     : int8 -> fp32 -> bf16 (exact, codes <= 255).
//   r < 8     : the slicing operator of section 3.2 on 16-bit lanes.  The byte is placed in the high
//               half of a 16-bit lane, a saturating add of half << 8 implements min(q + half, 255)
//               (the clamp of the slicing equation), a shift leaves the r-bit code, and OR-ing
//               0x4300 makes the bf16 number 128 + code.  The 128 is removed in the epilogue with
//               the per-token sum of X.  Extra precision (errata section) skips the saturation.
//
// Epilogue: Y = alpha_n * (2^s * acc - (2^s * 128 + z_n) * sum_k X[m,k]).
//
// Backward (identity STE): dX reuses the same in-register slicing on a transposed copy of the
// codes, with one pre-scaled gradient operand per bit-width accumulated into a single accumulator;
// dW is a plain bf16 GEMM of the lambda-weighted gradient sum against X.
#include <algorithm>
#include <mutex>
#include <type_traits>

#include "mq_gemv.h"

namespace mq {

typedef __attribute__((address_space(3))) void *lds_ptr;

constexpr int BKT = 64;                  // contraction elements per LDS stage
constexpr uint32_t kOOB = 0x80000000u;   // buffer offset beyond any descriptor built here
constexpr uint32_t kMagic128 = 0x43004300u;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint64_t bytes) {
    const uint32_t rec = bytes > 0x7FFFFFFFull ? 0x7FFFFFFFu : (uint32_t)bytes;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)rec, 0x00020000);
}

__device__ __forceinline__ void wait_vm0() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ f32x16 mfma32(const u32x4 &a, const u32x4 &b, const f32x16 &c) {
    Frag8 fa, fb;
    fa.u = a;
    fb.u = b;
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.b, fb.b, c, 0, 0, 0);
}

// ---- LDS tiles ------------------------------------------------------------------------------
// bf16 tile: ROWS x 64 elements, 128-byte rows of eight 16-byte chunks; chunk c of row r is stored
// at chunk position c ^ ((r >> 1) & 7).  u8 tile: ROWS x 64 bytes, four chunks per row; chunk c of
// row r at position c ^ ((r >> 2) & 3).  The LDS has 64 four-byte banks and serves a 16-byte read
// sixteen lanes at a time, so sixteen consecutive rows must land on sixteen distinct 16-byte bank
// groups of a 256-byte window; both swizzles do that (measured: same rate as a contiguous read).  A direct-to-LDS load writes lane l of a wave at base + 16 l, so the swizzle is
// applied by choosing which global chunk each lane fetches.

// Per-lane byte offset (row * ld_bytes + chunk * 16) of instruction `inst` of this wave for a bf16
// tile, and the element column of the chunk (for the tail predicate).
template <int NWAVES>
__device__ __forceinline__ void bf16_tile_lane(int wave, int lane, int inst, uint32_t ld_bytes,
                                               uint32_t &voff, int &col) {
    const int slot = (wave + inst * NWAVES) * 64 + lane;
    const int row = slot >> 3, p = slot & 7, c = p ^ ((row >> 1) & 7);
    voff = (uint32_t)row * ld_bytes + (uint32_t)c * 16u;
    col = c * 8;
}
template <int NWAVES>
__device__ __forceinline__ void u8_tile_lane(int wave, int lane, int inst, uint32_t ld_bytes,
                                             uint32_t &voff, int &col) {
    const int slot = (wave + inst * NWAVES) * 64 + lane;
    const int row = slot >> 2, p = slot & 3, c = p ^ ((row >> 2) & 3);
    voff = (uint32_t)row * ld_bytes + (uint32_t)c * 16u;
    col = c * 16;
}

// ---- code -> bf16 operand conversions ---------------------------------------------------------
// Eight int8 codes (two dwords, k ascending) -> eight bf16 of the same value.
__device__ __forceinline__ u32x4 codes_to_bf16_r8(uint32_t d0, uint32_t d1) {
    auto two = [](float lo, float hi) {
        return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
    };
    return u32x4{two((float)(d0 & 0xFFu), (float)((d0 >> 8) & 0xFFu)),
                 two((float)((d0 >> 16) & 0xFFu), (float)(d0 >> 24)),
                 two((float)(d1 & 0xFFu), (float)((d1 >> 8) & 0xFFu)),
                 two((float)((d1 >> 16) & 0xFFu), (float)(d1 >> 24))};
}

// Bytes of two dwords placed in 16-bit lanes, k ascending.  HIGH: byte << 8 (for the saturating
// add), else byte in the low half.
template <bool HIGH>
__device__ __forceinline__ u32x4 place_bytes(uint32_t d0, uint32_t d1) {
    constexpr uint32_t s01 = HIGH ? 0x010C000Cu : 0x0C010C00u;
    constexpr uint32_t s23 = HIGH ? 0x030C020Cu : 0x0C030C02u;
    return u32x4{__builtin_amdgcn_perm(0u, d0, s01), __builtin_amdgcn_perm(0u, d0, s23),
                 __builtin_amdgcn_perm(0u, d1, s01), __builtin_amdgcn_perm(0u, d1, s23)};
}

// r-bit slice of section 3.2 as bf16(128 + code), from bytes placed by place_bytes<!EP>.
// half2 = half in both 16-bit lanes (shifted left by 8 unless EP); sh = s (+ 8 unless EP).
template <bool EP>
__device__ __forceinline__ u32x4 sliced_to_bf16(const u32x4 &placed, uint32_t half2, uint32_t sh) {
    u32x4 out;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if constexpr (EP) {
            out[i] = (((placed[i] + half2) >> sh) & 0x00FF00FFu) | kMagic128;
        } else {
            const uint32_t pv = placed[i];
            u16x2 t = __builtin_elementwise_add_sat(__builtin_bit_cast(u16x2, pv), __builtin_bit_cast(u16x2, half2));
            const unsigned short s16 = (unsigned short)sh;
            t = t >> u16x2{s16, s16};
            out[i] = __builtin_bit_cast(uint32_t, t) | kMagic128;
        }
    }
    return out;
}

struct SliceParam {  // wave-uniform per bit-width
    uint32_t half2;  // half (<< 8 unless EP) in both 16-bit lanes
    uint32_t sh;     // shift that leaves the code
};

template <bool EP>
__device__ __forceinline__ SliceParam slice_param(int r) {
    const uint32_t s = 8 - r, half = (1u << s) >> 1;
    SliceParam p;
    if constexpr (EP) {
        p.half2 = half | (half << 16);
        p.sh = s;
    } else {
        p.half2 = (half << 8) | (half << 24);
        p.sh = s + 8;
    }
    return p;
}

// ============================================================================================
// forward
// ============================================================================================
struct FwdArgs {
    const uint16_t *X;
    const uint8_t *Q;
    const float *alpha, *zero, *rowsum;
    uint16_t *Y[3];
    int M, N, K;
    int r[3];  // bit-width per slot; slot 0 is the r = 8 slot when HAS8
    int tiles_m, tiles_n;
    // LOSS kernels only (slot order as Y): the L2 objective is evaluated on the rounded outputs
    // while they sit in the staging tiles.  Y[i] may then be NULL (that output is not stored).
    const uint16_t *T;
    uint16_t *dY[3];
    int teacher[3];  // slot of the teacher, or -1 for the target T
    float coef[3];   // lambda_i * 2 / (M N)
    int mix;
    float *partial;  // [workgroup][4] sums of squared differences
    const float *bias;  // [N] added to every output before it is rounded, or null
    // plain kernels only: the layer is the stacked gate / up projection of a gated unit (channels (g, u) pairs)
    // and A[i] [M, N / 2] receives act(g) u of the rounded outputs; gate = 0 none, 1 GELU-tanh, 2 SiLU
    uint16_t *A[3];
    int gate;
};

constexpr int FWD_BN = 128;
constexpr int FWD_Q_TILE = FWD_BN * 64;
constexpr int FWD_STAGES = 4;
// 32-token blocks per wave: the accumulators (16 NR MB registers) must leave room for the operands
constexpr int fwd_mb(int nr) { return nr == 3 ? 5 : 6; }
constexpr int fwd_lds(int mb, int nr) {
    const int stages = FWD_STAGES * (mb * 32 * 128 + FWD_Q_TILE), staging = nr * mb * 32 * (FWD_BN * 2 + 8);
    return stages > staging ? stages : staging;
}

// One workgroup = 4 waves (one per SIMD, so each may use the whole 512-entry register file) on a
// (32 MB)-token x 128-channel tile; wave w owns channels [32 w, 32 w + 32) for all tokens, i.e.
// MB x NR accumulator blocks of 32 x 32.  The converted code operand of a wave is then reused by
// MB MFMAs per bit-width, which keeps the VALU slicing work at a fraction of the MFMA time.
// LDS holds four stages of 64 k: stage kt is computed while stage kt + 1 is resident (the operands
// of the next 16-wide k step are fetched into registers behind the MFMAs of the current one, also
// across the stage boundary) and stages kt + 2, kt + 3 are in flight, so a load has two full
// iterations to arrive.
template <int NR, bool HAS8, bool EP, int MB, bool LOSS>
__global__ __launch_bounds__(256) void fwd_kernel(FwdArgs a) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    constexpr int BM = 32 * MB;
    constexpr int X_TILE = BM * 128;
    constexpr int STAGE = X_TILE + FWD_Q_TILE;
    constexpr int LPS = MB + 2;  // direct-to-LDS loads per wave and stage
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int h = lane >> 5, l32 = lane & 31;

    // What the epilogue needs from the kernel arguments is fetched now, into scalar registers that stay
    // live through the main loop: read where it is used, each costs a scalar-memory round trip with
    // nothing to hide it (one wave per SIMD).
    const float *k_alpha = a.alpha, *k_zero = a.zero, *k_rowsum = a.rowsum, *k_bias = LOSS ? a.bias : nullptr;
    const uint16_t *k_T = LOSS ? a.T : nullptr;
    uint16_t *k_Y[NR], *k_dY[NR];
    float k_coef[NR];
    int k_teacher[NR], k_mix = LOSS ? a.mix : 0;
    uint16_t *k_A[NR];
    int k_gate = LOSS ? 0 : a.gate;
    asm volatile("" : "+s"(k_alpha), "+s"(k_zero), "+s"(k_rowsum));
#pragma unroll
    for (int i = 0; i < NR; ++i) {
        k_Y[i] = a.Y[i];
        asm volatile("" : "+s"(k_Y[i]));
        k_A[i] = LOSS ? nullptr : a.A[i];
        if constexpr (!LOSS) asm volatile("" : "+s"(k_A[i]));
        if constexpr (LOSS) {
            k_dY[i] = a.dY[i];
            k_coef[i] = a.coef[i];
            k_teacher[i] = a.teacher[i];
            asm volatile("" : "+s"(k_dY[i]), "+s"(k_coef[i]), "+s"(k_teacher[i]));
        }
    }
    if constexpr (LOSS) asm volatile("" : "+s"(k_bias), "+s"(k_T), "+s"(k_mix));
    if constexpr (!LOSS) asm volatile("" : "+s"(k_gate));

    // XCD-aware tile order: each XCD walks groups of 4 token tiles across the channel tiles
    const uint32_t lid = xcd_contiguous_id(blockIdx.x, gridDim.x);
    constexpr int GROUP = 4;
    const int width = GROUP * a.tiles_n;
    const int first_m = (int)(lid / width) * GROUP;
    const int gsz = min(a.tiles_m - first_m, GROUP);
    const int tm = first_m + (int)(lid % width) % gsz;
    const int tn = (int)(lid % width) / gsz;
    const int m0 = tm * BM, n0 = tn * FWD_BN;

    const __amdgpu_buffer_rsrc_t rX = make_rsrc(a.X + (size_t)m0 * a.K, (uint64_t)(a.M - m0) * a.K * 2);
    const __amdgpu_buffer_rsrc_t rQ = make_rsrc(a.Q + (size_t)n0 * a.K, (uint64_t)(a.N - n0) * a.K);

    // global -> LDS: lane offsets of the wave's first X / Q instruction; instruction i is 32 (X) or
    // 64 (Q) rows further down with the same chunk
    uint32_t xoff0, qoff0;
    int xcol, qcol;
    bf16_tile_lane<4>(wave, lane, 0, (uint32_t)a.K * 2u, xoff0, xcol);
    u8_tile_lane<4>(wave, lane, 0, (uint32_t)a.K, qoff0, qcol);
    const uint32_t xstep = 32u * (uint32_t)a.K * 2u, qstep = 64u * (uint32_t)a.K;

    // Stage kt -> LDS buffer kt % 4, as MB + 2 loads per wave (MB of X, then 2 of Q).  Branch-free:
    // a stage past the end of K (or a chunk past K in the last stage) is requested at an
    // out-of-range offset, which the buffer unit answers with zeros without touching memory, so
    // the number of loads in flight is the same in every iteration.
    auto issue_one = [&](int kt, int i) {
        const int k0 = kt * BKT;
        uint8_t *xs = smem + (kt & 3) * STAGE;
        if (i < MB) {
            // (an out-of-range base stays out of range: kOOB + i * xstep < 2^32 for every legal K)
            const uint32_t xb = (k0 + xcol < a.K) ? xoff0 + (uint32_t)k0 * 2u : kOOB;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rX, (lds_ptr)(xs + (wave + i * 4) * 1024), 16,
                                                     xb + (uint32_t)i * xstep, 0, 0, 0);
        } else {
            const uint32_t qb = (k0 + qcol < a.K) ? qoff0 + (uint32_t)k0 : kOOB;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rQ, (lds_ptr)(xs + X_TILE + (wave + (i - MB) * 4) * 1024), 16,
                                                     qb + (uint32_t)(i - MB) * qstep, 0, 0, 0);
        }
    };
    auto issue = [&](int kt) {
#pragma unroll
        for (int i = 0; i < MB + 2; ++i) issue_one(kt, i);
    };

    // LDS fragment addresses (byte offsets inside a stage)
    const int nl = wave * 32 + l32;
    const uint32_t qa0 = X_TILE + nl * 64 + ((h ^ ((nl >> 2) & 3)) << 4);
    const uint32_t qa1 = X_TILE + nl * 64 + (((h + 2) ^ ((nl >> 2) & 3)) << 4);
    uint32_t xa[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int cx = 2 * h + 4 * (t >> 1) + (t & 1);
        xa[t] = l32 * 128 + ((cx ^ ((l32 >> 1) & 7)) << 4);
    }

    SliceParam sp[NR];
#pragma unroll
    for (int i = 0; i < NR; ++i) sp[i] = slice_param<EP>(a.r[i]);

    // Dword w (two consecutive k) of the code operand of slot i, from the 8 code bytes (d0, d1).
    auto convert_piece = [&](int i, int w, uint32_t d0, uint32_t d1) -> uint32_t {
        const uint32_t d = w < 2 ? d0 : d1;
        if (HAS8 && i == 0) {
            const float lo = (w & 1) ? (float)((d >> 16) & 0xFFu) : (float)(d & 0xFFu);
            const float hi = (w & 1) ? (float)(d >> 24) : (float)((d >> 8) & 0xFFu);
            return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
        }
        if constexpr (EP) {
            const uint32_t placed = __builtin_amdgcn_perm(0u, d, (w & 1) ? 0x0C030C02u : 0x0C010C00u);
            return (((placed + sp[i].half2) >> sp[i].sh) & 0x00FF00FFu) | kMagic128;
        } else {
            const uint32_t placed = __builtin_amdgcn_perm(0u, d, (w & 1) ? 0x030C020Cu : 0x010C000Cu);
            u16x2 t = __builtin_elementwise_add_sat(__builtin_bit_cast(u16x2, placed),
                                                    __builtin_bit_cast(u16x2, sp[i].half2));
            const unsigned short s16 = (unsigned short)sp[i].sh;
            t = t >> u16x2{s16, s16};
            return __builtin_bit_cast(uint32_t, t) | kMagic128;
        }
    };

    f32x16 acc[NR][MB];
#pragma unroll
    for (int i = 0; i < NR; ++i)
#pragma unroll
        for (int j = 0; j < MB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nkt = (a.K + BKT - 1) / BKT;
    issue(0);
    issue(1);
    issue(2);
    // stage 0 must have landed before the first operand fetch; stages 1 and 2 may stay in flight
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LPS) : "memory");
    __syncthreads();

    u32x4 xf[MB];      // activation operands of the current k step (refilled as soon as they are consumed)
    u32x4 raw[2];      // 32 code bytes of this lane's channel: four k steps of one stage
    u32x4 wf[NR];      // code operands of the current k step
    raw[0] = *reinterpret_cast<const u32x4 *>(smem + qa0);
    raw[1] = *reinterpret_cast<const u32x4 *>(smem + qa1);
#pragma unroll
    for (int j = 0; j < MB; ++j) xf[j] = *reinterpret_cast<const u32x4 *>(smem + xa[0] + j * 4096);
#pragma unroll
    for (int i = 0; i < NR; ++i)
#pragma unroll
        for (int w = 0; w < 4; ++w) wf[i][w] = convert_piece(i, w, raw[0][0], raw[0][1]);

    // One stage of 64 k: four 16-wide steps of NR * MB MFMAs.  A wave issues in order, so whatever
    // is queued behind an MFMA that waits for the matrix pipe waits with it; the other work of a
    // step is therefore cut into one small group per MFMA, fenced so that the compiler keeps it
    // there:  group q < MB requests operand block q of step t + 1 from LDS (it then has the rest
    // of the step to arrive), groups 1 .. 4 NR each produce one dword of the next code operands,
    // the last groups of step 0 issue the global loads of stage kt + 3, and step 2 fetches the
    // code bytes of the next stage.  MORE (compile time): there is a next stage.
    auto tile = [&](auto more_tag, int kt) {
        constexpr bool MORE = decltype(more_tag)::value;
        constexpr int NM = NR * MB;
        static_assert(4 * NR <= NM, "not enough MFMAs to hide the operand work");
        constexpr int CQ = 4 * NR + 1 <= NM ? 1 : 0;  // first group that carries a conversion
        constexpr int LPG = (LPS + NM - 1) / NM;  // global loads per group in step 0
        const uint8_t *cur = smem + (kt & 3) * STAGE;
        const uint8_t *nxt = smem + ((kt + 1) & 3) * STAGE;
        u32x4 rawn[2];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const bool pre = t < 3 || MORE;  // is there a next step
            const uint8_t *src = t < 3 ? cur + xa[(t + 1) & 3] : nxt + xa[0];
            // code bytes of the next step
            uint32_t d0 = t == 3 ? rawn[0][0] : (t + 1 < 2 ? raw[0][2 * (t + 1)] : raw[1][2 * (t + 1 - 2)]);
            uint32_t d1 = t == 3 ? rawn[0][1] : (t + 1 < 2 ? raw[0][2 * (t + 1) + 1] : raw[1][2 * (t + 1 - 2) + 1]);
            // pin the conversions of this step to this step (the optimizer would otherwise collect
            // them across the loop back-edge)
            if (pre) asm volatile("" : "+v"(d0), "+v"(d1));
            u32x4 xfn[MB];
            u32x4 wfn[NR];
#pragma unroll
            for (int q = 0; q < NM; ++q) {
                const int j = q / NR, i = q % NR;
                acc[i][j] = mfma32(wf[i], xf[j], acc[i][j]);
                if (pre && q < MB) xfn[q] = *reinterpret_cast<const u32x4 *>(src + q * 4096);
                if (pre && q >= CQ && q - CQ < 4 * NR) {
                    uint32_t piece = convert_piece((q - CQ) / 4, (q - CQ) % 4, d0, d1);
                    asm volatile("" : "+v"(piece));  // keeps the conversion inside this group
                    wfn[(q - CQ) / 4][(q - CQ) % 4] = piece;
                }
                if (MORE && t == 2 && q >= NM - 2) rawn[q - (NM - 2)] = *reinterpret_cast<const u32x4 *>(nxt + (q == NM - 2 ? qa0 : qa1));
                if (MORE && t == 0) {
#pragma unroll
                    for (int u = 0; u < LPG; ++u) {
                        const int ld = (NM - 1 - q) * LPG + u;  // the last groups carry the loads
                        if (ld < LPS) issue_one(kt + 3, ld);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (pre) {
#pragma unroll
                for (int i = 0; i < NR; ++i) wf[i] = wfn[i];
#pragma unroll
                for (int j = 0; j < MB; ++j) xf[j] = xfn[j];
            }
        }
        if (MORE) {
            raw[0] = rawn[0];
            raw[1] = rawn[1];
        }
    };

    for (int kt = 0; kt + 1 < nkt; ++kt) {
        // Stage kt + 1 must be resident for the operand prefetch at the end of this iteration; the
        // loads of stage kt + 2 may stay in flight.  After the barrier every wave is done with
        // stage kt - 1, whose buffer stage kt + 3 reuses.
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPS) : "memory");
        __syncthreads();
        tile(std::true_type{}, kt);
    }
    tile(std::false_type{}, nkt - 1);
    wait_vm0();  // zero-fill loads of dead stages must not land in the staging area below

    // ---- epilogue ---------------------------------------------------------------------------
    // accumulator v = 4 g + e of a lane holds row (channel) 8 g + 4 h + e, column (token) l32.
    // A lane therefore owns only 4 consecutive channels of a token; the tile is first assembled in
    // LDS ([token][channel] bf16, rows padded by 8 bytes so that both the 8-byte writes and the
    // read-back are bank-conflict free) and then stored as whole 256-byte rows.
    constexpr int OS = FWD_BN * 2 + 8;  // staging row stride in bytes
    constexpr int OT = BM * OS;         // one bit-width
    __syncthreads();                    // every wave is done with the operand stages
    float rs[MB];
#pragma unroll
    for (int j = 0; j < MB; ++j) {
        const int m = m0 + j * 32 + l32;
        rs[j] = m < a.M ? k_rowsum[m] : 0.f;
    }
    f32x4 alv[4], zev[4], bv[LOSS ? 4 : 1];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int nloc = wave * 32 + 8 * g + 4 * h;
        alv[g] = f32x4{0.f, 0.f, 0.f, 0.f};
        zev[g] = f32x4{0.f, 0.f, 0.f, 0.f};
        if constexpr (LOSS) bv[g] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (n0 + nloc < a.N) {
            alv[g] = *reinterpret_cast<const f32x4 *>(k_alpha + n0 + nloc);
            zev[g] = *reinterpret_cast<const f32x4 *>(k_zero + n0 + nloc);
            if constexpr (LOSS)
                if (k_bias) bv[g] = *reinterpret_cast<const f32x4 *>(k_bias + n0 + nloc);
        }
    }
    // LOSS: the lane's chunks of the target are requested now, behind the parameter loads, and
    // arrive while the accumulators are converted and staged.  With the largest accumulator sets
    // there are registers for some of them only (the counts below are the largest that compile
    // without spills); the others are requested after the staging and arrive while the first ones
    // are consumed.
    constexpr int CHUNKS = BM * 16 / 256;
    constexpr int EARLY = NR * MB > 12 ? 2 : (NR * MB == 12 ? CHUNKS / 2 : CHUNKS);
    u32x4 tpre[LOSS ? CHUNKS : 1];
    auto request_target = [&](int it) {
        const int c = it * 256 + threadIdx.x;
        const int m = m0 + (c >> 4), n = n0 + (c & 15) * 8;
        tpre[it] = u32x4{0u, 0u, 0u, 0u};
        if (k_T && m < a.M && n < a.N)
            tpre[it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(k_T + (size_t)m * a.N + n));
    };
    if constexpr (LOSS) {
#pragma unroll
        for (int it = 0; it < EARLY; ++it) request_target(it);
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int nloc = wave * 32 + 8 * g + 4 * h;
        const f32x4 al = alv[g], ze = zev[g];
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            const bool is8 = HAS8 && i == 0;
            const float mult = is8 ? 1.0f : (float)(1 << (8 - a.r[i]));
            const float bias = is8 ? 0.0f : 128.0f * mult;
            float bz[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) bz[e] = bias + ze[e];
#pragma unroll
            for (int j = 0; j < MB; ++j) {
                float y[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // (mult is a power of two, so the fused form rounds exactly like mult * acc - t)
                    const float t = bz[e] * rs[j];
                    const float inner = is8 ? acc[i][j][4 * g + e] - t : __builtin_fmaf(mult, acc[i][j][4 * g + e], -t);
                    y[e] = LOSS ? __builtin_fmaf(al[e], inner, bv[g][e]) : al[e] * inner;
                }
                const u32x2 o = {pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
                *reinterpret_cast<u32x2 *>(smem + i * OT + (j * 32 + l32) * OS + nloc * 2) = o;
            }
        }
    }
    if constexpr (LOSS) {
#pragma unroll
        for (int it = EARLY; it < CHUNKS; ++it) request_target(it);
    }
    __syncthreads();
    if constexpr (!LOSS) {
#pragma unroll
        for (int i = 0; i < NR; ++i) {
#pragma unroll
            for (int it = 0; it < BM * 16 / 256; ++it) {
                const int c = it * 256 + threadIdx.x;
                const int row = c >> 4, ch = c & 15;
                const int m = m0 + row, n = n0 + ch * 8;
                if (m < a.M && n < a.N) {
                    const uint8_t *src = smem + i * OT + row * OS + ch * 16;
                    const u32x2 lo = *reinterpret_cast<const u32x2 *>(src);
                    const u32x2 hi = *reinterpret_cast<const u32x2 *>(src + 8);
                    if (k_Y[i])
                        __builtin_nontemporal_store(u32x4{lo.x, lo.y, hi.x, hi.y},
                                                    reinterpret_cast<u32x4 *>(k_Y[i] + (size_t)m * a.N + n));
                    if (k_gate) {
                        // the gated unit on the rounded outputs, pair by pair (the arithmetic of mq_gated_unit_fwd)
                        const bool use_silu = k_gate == 2;
                        auto gated = [&](uint32_t pair) {
                            const float g = bf16_lo(pair), u = bf16_hi(pair);
                            return (use_silu ? silu(g) : gelu_tanh(g)) * u;
                        };
                        const u32x2 o = {pack_bf16x2(gated(lo.x), gated(lo.y)), pack_bf16x2(gated(hi.x), gated(hi.y))};
                        __builtin_nontemporal_store(o, reinterpret_cast<u32x2 *>(k_A[i] + (size_t)m * (a.N >> 1) + (n >> 1)));
                    }
                }
            }
        }
    } else {
        // L2 objective on the staged tile (section 3.2 with the loss of section 3.1.2, co-distillation
        // targets of section 5.2): a lane takes the same 8 channels of a token from every bit-width
        // and from the target, adds (Y_i - T_i)^2 to its sums and stores dY_i = coef_i (Y_i - T_i);
        // the arithmetic per element is that of the stand-alone loss kernel, on the same rounded Y.
        float sum[NR];
#pragma unroll
        for (int i = 0; i < NR; ++i) sum[i] = 0.f;
        // The parameters of the objective are read once into vector registers (left to itself the compiler
        // reloads them from the kernel arguments for every chunk, a scalar-memory round trip each time):
        // the factor, the lane's addresses in dY_i / Y_i, and the choice of the teacher as bit masks.
        const int crow = threadIdx.x >> 4, cch = threadIdx.x & 15;  // chunk `it` is row crow + 16 it, channels 8 cch ..
        const size_t at0 = (size_t)(m0 + crow) * a.N + n0 + cch * 8;
        const bool cols_ok = n0 + cch * 8 < a.N;
        float cf[NR];
        uint32_t pick[NR][NR], mixed_slot[NR];
        uint16_t *pd[NR], *py[NR];
        int stored = 0, taught = 0;  // wave-uniform: bit i = Y_i is stored / slot i has a teacher
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            cf[i] = k_coef[i];
            pd[i] = k_dY[i] + at0;
            py[i] = k_Y[i] ? k_Y[i] + at0 : nullptr;
            stored |= k_Y[i] ? 1 << i : 0;
            taught |= k_teacher[i] >= 0 ? 1 << i : 0;
            mixed_slot[i] = k_teacher[i] >= 0 ? 0xFFFFFFFFu : 0u;
            asm volatile("" : "+v"(cf[i]), "+v"(pd[i]), "+v"(py[i]), "+v"(mixed_slot[i]));
#pragma unroll
            for (int u = 0; u < NR; ++u) {
                pick[i][u] = k_teacher[i] == u ? 0xFFFFFFFFu : 0u;
                asm volatile("" : "+v"(pick[i][u]));
            }
        }
        stored = __builtin_amdgcn_readfirstlane(stored);
        taught = __builtin_amdgcn_readfirstlane(taught);
        asm volatile("" : "+s"(stored), "+s"(taught));
        const size_t chunk_step = (size_t)16 * a.N;  // elements between a lane's consecutive chunks
        // The equal-weight mix of teacher and target, and the presence of any teacher at all, are variants
        // of the whole loop, chosen once: without teachers every bit-width is compared with the target and
        // the selection of the reference disappears.
        auto chunks = [&](auto mixed, auto teach) {
            constexpr bool MIX = decltype(mixed)::value, TEACH = decltype(teach)::value;
            // the staged values of chunk it + 1 are read (every chunk lies inside the tile) before chunk it is
            // worked on, outside the bounds test, so that the LDS latency hides behind arithmetic
            auto staged = [&](int it, u32x4 (&dst)[NR]) {
#pragma unroll
                for (int i = 0; i < NR; ++i) {
                    const uint8_t *src = smem + i * OT + (crow + 16 * it) * OS + cch * 16;
                    const u32x2 lo = *reinterpret_cast<const u32x2 *>(src);
                    const u32x2 hi = *reinterpret_cast<const u32x2 *>(src + 8);
                    dst[i] = u32x4{lo.x, lo.y, hi.x, hi.y};
                }
            };
            u32x4 ynext[NR];
            staged(0, ynext);
#pragma unroll
            for (int it = 0; it < CHUNKS; ++it) {
                const int row = crow + 16 * it;
                u32x4 y[NR];
#pragma unroll
                for (int i = 0; i < NR; ++i) y[i] = ynext[i];
                if (it + 1 < CHUNKS) staged(it + 1, ynext);
                if (cols_ok && m0 + row < a.M) {
                    const u32x4 t = tpre[it];
#pragma unroll
                    for (int i = 0; i < NR; ++i) {
                        u32x4 tt = t;
                        if constexpr (TEACH) {
#pragma unroll
                            for (int u = 0; u < NR; ++u)
                                if (u != i) {
#pragma unroll
                                    for (int j = 0; j < 4; ++j) tt[j] = (y[u][j] & pick[i][u]) | (tt[j] & ~pick[i][u]);
                                }
                        }
                        u32x4 o;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const float y0 = bf16_lo(y[i][j]), y1 = bf16_hi(y[i][j]);
                            float d0 = y0 - bf16_lo(tt[j]), d1 = y1 - bf16_hi(tt[j]);
                            if (MIX && mixed_slot[i]) {  // teacher and ground truth, weighted equally
                                const float e0 = y0 - bf16_lo(t[j]), e1 = y1 - bf16_hi(t[j]);
                                sum[i] += 0.5f * (d0 * d0 + d1 * d1 + e0 * e0 + e1 * e1);
                                d0 = 0.5f * (d0 + e0);
                                d1 = 0.5f * (d1 + e1);
                            } else {
                                sum[i] = __builtin_fmaf(d1, d1, __builtin_fmaf(d0, d0, sum[i]));
                            }
                            o[j] = pack_bf16x2(cf[i] * d0, cf[i] * d1);
                        }
                        __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(pd[i] + it * chunk_step));
                        if (stored & (1 << i))
                            __builtin_nontemporal_store(y[i], reinterpret_cast<u32x4 *>(py[i] + it * chunk_step));
                    }
                }
            }
        };
        if (k_mix)
            chunks(std::true_type{}, std::true_type{});
        else if (taught)
            chunks(std::false_type{}, std::true_type{});
        else
            chunks(std::false_type{}, std::false_type{});
        // workgroup sums in a fixed order; the staging tiles are dead after the barrier
        __syncthreads();
        float *red = reinterpret_cast<float *>(smem);
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            float v = sum[i];
#pragma unroll
            for (int msk = 1; msk < 64; msk <<= 1) v += __shfl_xor(v, msk);
            if (lane == 0) red[wave * 4 + i] = v;
        }
        __syncthreads();
        if (threadIdx.x < 4) {
            float v = 0.f;
            if ((int)threadIdx.x < NR)
                for (int w = 0; w < 4; ++w) v += red[w * 4 + threadIdx.x];
            a.partial[(size_t)blockIdx.x * 4 + threadIdx.x] = v;
        }
    }
}

// out[i] = in[slot_i]: the losses of the fused forward, from slot order back to the caller's order
__global__ void permute3_kernel(const float *in, float *out, int nr, int s0, int s1, int s2) {
    if (threadIdx.x == 0 && nr > 0) out[0] = in[s0];
    if (threadIdx.x == 1 && nr > 1) out[1] = in[s1];
    if (threadIdx.x == 2 && nr > 2) out[2] = in[s2];
}

// sum_k X[m, k] in fp32, one wave per row
__global__ __launch_bounds__(256) void rowsum_kernel(const uint16_t *__restrict__ X, int M, int K,
                                                     float *__restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (m >= M) return;
    const u32x4 *row = reinterpret_cast<const u32x4 *>(X + (size_t)m * K);
    float s = 0.f;
    for (int c = lane; c < K / 8; c += 64) {
        const u32x4 v = row[c];
#pragma unroll
        for (int i = 0; i < 4; ++i) s += __uint_as_float(v[i] << 16) + __uint_as_float(v[i] & 0xFFFF0000u);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) out[m] = s;
}

// ============================================================================================
// backward, preparation (HBM-bound): one pass over the nr gradient tensors produces
//   As_i[m, n] = bf16(lambda_i * alpha_n * 2^s_i * dY_i[m, n])     (operand of the dX contraction)
//   c[m]       = sum_i sum_n As_i[m, n] * (bias_i + z_n / 2^s_i)   (what the 128 + code form and z add to dX[m, :])
//   GT[n, m]   = bf16(sum_i lambda_i * dY_i[m, n])                  (transposed operand of the dW GEMM, in token blocks)
// ============================================================================================
struct PrepArgs {
    const uint16_t *dY[3];
    // GATED kernels: the layer is the stacked gate / up projection of a gated unit a = act(g) u and its output
    // gradients are formed here from GU_i [M, N] (columns (g, u) pairs) and dA_i [M, N / 2] instead of read from dY_i
    const uint16_t *GU[3];
    const uint16_t *dA[3];
    int silu;
    uint16_t *As[3];     // null pointers when dX is not wanted
    const float *alpha, *zero;
    float lam[3];
    float mult[3];       // 2^s_i
    float bias[3];       // 128 for sliced slots, 0 for the r = 8 slot
    float *cpart;        // [nsplit][M] partial sums of c over column ranges, or null
    uint16_t *GT;        // [M / 32][N][32] (blocks of 32 tokens; see DwArgs) or null; tokens M .. ldm - 1 are written as zeros
    int nr, M, N;
    int ldm;             // M rounded up to a multiple of 8
    int cols_per_split;  // multiple of 64
};

constexpr int PREP_ROWS = 32;
constexpr int PREP_MAX_SPLIT = 16;

// Workgroup (strip, split) walks 32 token rows across one range of columns in 32 x 64 tiles: thread
// (r, ch) = (t / 8, t % 8) owns eight consecutive columns of row r, so a row segment is one 128-byte
// line per gradient tensor.  The summed gradient tile is turned through LDS and leaves as 64-byte
// row segments of GT.
template <bool GATED>
__global__ __launch_bounds__(256) void bwd_prep_kernel(PrepArgs a) {
    __shared__ uint16_t tile[64][PREP_ROWS + 2];
    const int t = threadIdx.x, r = t >> 3, ch = t & 7;
    const int m0 = blockIdx.x * PREP_ROWS, m = m0 + r;
    const int nbeg = blockIdx.y * a.cols_per_split, nend = min(nbeg + a.cols_per_split, a.N);
    const bool want_as = a.As[0] != nullptr;
    float c = 0.f;
    for (int n0 = nbeg; n0 < nend; n0 += 64) {
        const int n = n0 + ch * 8;
        float g[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) g[j] = 0.f;
        if (m < a.M && n < a.N) {
            float al[8], ze[8];
            if (want_as) {
                *reinterpret_cast<f32x4 *>(al) = *reinterpret_cast<const f32x4 *>(a.alpha + n);
                *reinterpret_cast<f32x4 *>(al + 4) = *reinterpret_cast<const f32x4 *>(a.alpha + n + 4);
                *reinterpret_cast<f32x4 *>(ze) = *reinterpret_cast<const f32x4 *>(a.zero + n);
                *reinterpret_cast<f32x4 *>(ze + 4) = *reinterpret_cast<const f32x4 *>(a.zero + n + 4);
            }
            u32x4 dy[3];
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                if (i >= a.nr) break;
                if constexpr (GATED) {
                    // the gradient of the gated unit, pair by pair, rounded to bf16 like mq_gated_unit_bwd does
                    const u32x4 gu = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.GU[i] + (size_t)m * a.N + n));
                    const u32x2 da = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(a.dA[i] + (size_t)m * (a.N >> 1) + (n >> 1)));
#pragma unroll
                    for (int w = 0; w < 4; ++w)
                        dy[i][w] = gated_pair_grad(bf16_lo(gu[w]), bf16_hi(gu[w]), (w & 1) ? bf16_hi(da[w >> 1]) : bf16_lo(da[w >> 1]),
                                                   a.silu != 0);
                } else {
                    dy[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.dY[i] + (size_t)m * a.N + n));
                }
            }
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                if (i >= a.nr) break;
                const float f = a.lam[i] * a.mult[i], inv = 1.0f / a.mult[i];
                u32x4 o;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const float dlo = bf16_bits_to_float(dy[i][w] & 0xFFFFu), dhi = bf16_bits_to_float(dy[i][w] >> 16);
                    g[2 * w] += a.lam[i] * dlo;
                    g[2 * w + 1] += a.lam[i] * dhi;
                    if (want_as) {
                        o[w] = pack_bf16x2(dlo * (f * al[2 * w]), dhi * (f * al[2 * w + 1]));
                        c += bf16_bits_to_float(o[w] & 0xFFFFu) * (a.bias[i] + ze[2 * w] * inv);
                        c += bf16_bits_to_float(o[w] >> 16) * (a.bias[i] + ze[2 * w + 1] * inv);
                    }
                }
                if (want_as) *reinterpret_cast<u32x4 *>(a.As[i] + (size_t)m * a.N + n) = o;
            }
        }
        if (a.GT) {
            __syncthreads();  // the previous tile has been written out
#pragma unroll
            for (int j = 0; j < 8; ++j) tile[ch * 8 + j][r] = (uint16_t)float_to_bf16_bits(g[j]);
            __syncthreads();
            const int nn = t >> 2, part = t & 3;  // 64 rows of GT, four 16-byte pieces each
            if (n0 + nn < a.N && m0 + part * 8 < a.M) {  // (a piece that straddles M ends with zeros)
                const uint32_t *src = reinterpret_cast<const uint32_t *>(&tile[nn][part * 8]);
                *reinterpret_cast<u32x4 *>(a.GT + ((size_t)blockIdx.x * a.N + n0 + nn) * 32 + part * 8) =
                    u32x4{src[0], src[1], src[2], src[3]};
            }
        }
    }
    if (a.cpart) {
        c += __shfl_xor(c, 1, 64);
        c += __shfl_xor(c, 2, 64);
        c += __shfl_xor(c, 4, 64);
        if (ch == 0 && m < a.M) a.cpart[(size_t)blockIdx.y * a.M + m] = c;
    }
}

// out[c, r] = in[r, c] for a [rows, cols] matrix of 1- or 2-byte elements; cols is a multiple of 16
// bytes' worth of elements, the rows of out are ld_out elements apart (rows rounded up to such a
// multiple) and end with zeros.  64 x (64 bytes) tiles, 16-byte global accesses on both sides, the
// turn happens in LDS.
// BLOCKED (2-byte elements): out is [rows / 32][cols][32] instead, i.e. element (c, r) sits at ((r / 32) cols + c) 32 + r % 32
// (the operand layout of dw_kernel).
template <typename T, bool BLOCKED = false>
__global__ __launch_bounds__(256) void transpose_kernel(const T *__restrict__ in, T *__restrict__ out, int rows,
                                                        int cols, int ld_out) {
    constexpr int E = 16 / sizeof(T);  // elements per 16 bytes
    constexpr int TC = 4 * E;          // tile columns (64 bytes)
    constexpr int S = 64 + 4 / sizeof(T);  // padded row of the turned tile (a multiple of 4 bytes)
    __shared__ T tile[TC][S];
    const int t = threadIdx.x;
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * TC;
    {
        const int r = t >> 2, chunk = t & 3;
        if (c0 + chunk * E < cols) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (r0 + r < rows) v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(in + (size_t)(r0 + r) * cols + c0 + chunk * E));
            T e[E];
            __builtin_memcpy(e, &v, 16);
#pragma unroll
            for (int j = 0; j < E; ++j) tile[chunk * E + j][r] = e[j];
        }
    }
    __syncthreads();
    {
        constexpr int PIECES = 64 / E;  // 16-byte pieces per row of the turned tile
        const int c = t / PIECES, piece = t % PIECES;
        if (c < TC && c0 + c < cols && r0 + piece * E < rows) {
            const uint32_t *src = reinterpret_cast<const uint32_t *>(&tile[c][piece * E]);
            const int r = r0 + piece * E;
            const size_t at = BLOCKED ? ((size_t)(r >> 5) * cols + c0 + c) * 32 + (r & 31) : (size_t)(c0 + c) * ld_out + r;
            *reinterpret_cast<u32x4 *>(out + at) = u32x4{src[0], src[1], src[2], src[3]};
        }
    }
}

// ============================================================================================
// backward dX: dX[m, k] = sum_i sum_n As_i[m, n] * V_i[n, k] - c[m], V_i = the bf16 operand of slot i
// Rows of the matrix-core product are k (from the transposed codes QT[K, N]), columns are tokens,
// the contraction runs over n and, within each n tile, over the bit-widths.
// ============================================================================================
struct DxArgs {
    const uint16_t *As[3];  // [M, N] bf16, slot order (the r = 8 slot first when HAS8)
    const uint8_t *QT;      // [K, N] u8
    const float *cvec;      // [nsplit][M]: partial sums of c[m] over column ranges
    int nsplit;
    uint16_t *dX;           // [M, K] bf16
    int M, N, K;
    int r[3];               // bit-width per slot
    int tiles_m, tiles_k;
};

constexpr int DX_MB = 5;                        // 32-token blocks per wave
constexpr int DX_RB = 2;                        // 32-row blocks of k per wave
constexpr int DX_BM = 32 * DX_MB;               // tokens per workgroup
constexpr int DX_BK = 4 * 32 * DX_RB;           // k rows per workgroup (4 waves)
constexpr int DX_A_TILE = DX_BM * 128, DX_Q_TILE = DX_BK * 64;
constexpr int DX_STAGE = DX_A_TILE + DX_Q_TILE;
constexpr int DX_OS = DX_BK * 2 + 8;            // row stride of the output staging tile
constexpr int dx_lds() {
    const int stages = 4 * DX_STAGE, staging = DX_BM * DX_OS;
    return stages > staging ? stages : staging;
}

// Same pipeline as the forward kernel (one wave per SIMD, four LDS stages, one small fenced group
// of operand work per MFMA), with the roles changed: a stage is one 64-wide tile of n for ONE
// bit-width, i.e. the gradient operand As_slot[tokens, n tile] and the transposed codes
// QT[k rows, n tile]; the NRS bit-widths of an n tile follow each other and all accumulate into the
// same accumulators.  Wave w owns k rows [64 w, 64 w + 64) for all 160 tokens of the tile.  The
// stage loop is unrolled over the bit-widths so that the kind of code conversion is a compile-time
// property of each copy of the stage body.
template <int NRS, bool HAS8, bool EP>
__global__ __launch_bounds__(256) void dx_kernel(DxArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    constexpr int MB = DX_MB, RB = DX_RB;
    constexpr int QL = DX_BK / 64;       // direct-to-LDS loads per wave and stage for the codes (16 rows each)
    constexpr int LPS = MB + QL;         // loads per wave and stage
    constexpr int NM = RB * MB;          // MFMAs per 16-wide step
    static_assert(4 * RB + 1 <= NM && LPS <= NM, "not enough MFMAs to hide the operand work");
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int h = lane >> 5, l32 = lane & 31;

    const uint32_t lid = xcd_contiguous_id(blockIdx.x, gridDim.x);
    constexpr int GROUP = 4;
    const int width = GROUP * a.tiles_k;
    const int first_m = (int)(lid / width) * GROUP;
    const int gsz = min(a.tiles_m - first_m, GROUP);
    const int tm = first_m + (int)(lid % width) % gsz;
    const int tk = (int)(lid % width) / gsz;
    const int m0 = tm * DX_BM, k0 = tk * DX_BK;

    __amdgpu_buffer_rsrc_t rA[NRS];
#pragma unroll
    for (int i = 0; i < NRS; ++i) rA[i] = make_rsrc(a.As[i] + (size_t)m0 * a.N, (uint64_t)(a.M - m0) * a.N * 2);
    const __amdgpu_buffer_rsrc_t rQ = make_rsrc(a.QT + (size_t)k0 * a.N, (uint64_t)(a.K - k0) * a.N);

    uint32_t aoff0, qoff0;
    int acol, qcol;
    bf16_tile_lane<4>(wave, lane, 0, (uint32_t)a.N * 2u, aoff0, acol);
    u8_tile_lane<4>(wave, lane, 0, (uint32_t)a.N, qoff0, qcol);
    const uint32_t astep = 32u * (uint32_t)a.N * 2u, qstep = 64u * (uint32_t)a.N;

    // load i of stage (n tile nt, bit-width slot) into LDS buffer `buf`; out-of-range requests
    // (a tile past N) are answered with zeros, so the loads in flight are the same every stage
    auto issue_one = [&](int nt, auto slot_tag, int buf, int i) {
        constexpr int SLOT = decltype(slot_tag)::value;
        const int n0 = nt * BKT;
        uint8_t *as = smem + buf * DX_STAGE;
        if (i < MB) {
            const uint32_t ab = (n0 + acol < a.N) ? aoff0 + (uint32_t)n0 * 2u : kOOB;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rA[SLOT], (lds_ptr)(as + (wave + i * 4) * 1024), 16,
                                                     ab + (uint32_t)i * astep, 0, 0, 0);
        } else {
            // The code bytes of an n tile are fetched with its first bit-width only: the other bit-widths
            // of the tile slice the same bytes, which the lanes then still hold in registers.  Their
            // requests go out of range (no traffic) so that every stage has the same number of loads.
            const uint32_t qb = (SLOT == 0 && n0 + qcol < a.N) ? qoff0 + (uint32_t)n0 : kOOB;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rQ, (lds_ptr)(as + DX_A_TILE + (wave + (i - MB) * 4) * 1024), 16,
                                                     qb + (uint32_t)(i - MB) * qstep, 0, 0, 0);
        }
    };

    // LDS fragment addresses (byte offsets inside a stage)
    uint32_t qa[RB][2];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int kl = wave * (32 * RB) + rb * 32 + l32;
        qa[rb][0] = DX_A_TILE + kl * 64 + ((h ^ ((kl >> 2) & 3)) << 4);
        qa[rb][1] = DX_A_TILE + kl * 64 + (((h + 2) ^ ((kl >> 2) & 3)) << 4);
    }
    uint32_t xa[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int cx = 2 * h + 4 * (t >> 1) + (t & 1);
        xa[t] = l32 * 128 + ((cx ^ ((l32 >> 1) & 7)) << 4);
    }

    SliceParam sp[NRS];
#pragma unroll
    for (int i = 0; i < NRS; ++i) sp[i] = slice_param<EP>(a.r[i]);

    // dword w (two consecutive n) of the code operand of bit-width SLOT from 8 code bytes (d0, d1)
    auto convert_piece = [&](auto slot_tag, int w, uint32_t d0, uint32_t d1) -> uint32_t {
        constexpr int SLOT = decltype(slot_tag)::value;
        const uint32_t d = w < 2 ? d0 : d1;
        if constexpr (HAS8 && SLOT == 0) {
            const float lo = (w & 1) ? (float)((d >> 16) & 0xFFu) : (float)(d & 0xFFu);
            const float hi = (w & 1) ? (float)(d >> 24) : (float)((d >> 8) & 0xFFu);
            return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
        } else if constexpr (EP) {
            const uint32_t placed = __builtin_amdgcn_perm(0u, d, (w & 1) ? 0x0C030C02u : 0x0C010C00u);
            return (((placed + sp[SLOT].half2) >> sp[SLOT].sh) & 0x00FF00FFu) | kMagic128;
        } else {
            const uint32_t placed = __builtin_amdgcn_perm(0u, d, (w & 1) ? 0x030C020Cu : 0x010C000Cu);
            u16x2 t = __builtin_elementwise_add_sat(__builtin_bit_cast(u16x2, placed),
                                                    __builtin_bit_cast(u16x2, sp[SLOT].half2));
            const unsigned short s16 = (unsigned short)sp[SLOT].sh;
            t = t >> u16x2{s16, s16};
            return __builtin_bit_cast(uint32_t, t) | kMagic128;
        }
    };

    f32x16 acc[RB][MB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int j = 0; j < MB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[rb][j][v] = 0.f;

    const int nnt = (a.N + BKT - 1) / BKT;
    // prologue: stages 0, 1, 2 (n tile st / NRS, bit-width st % NRS)
    {
        auto issue_stage = [&](auto st_tag) {
            constexpr int ST = decltype(st_tag)::value;
#pragma unroll
            for (int i = 0; i < LPS; ++i) issue_one(ST / NRS, std::integral_constant<int, ST % NRS>{}, ST & 3, i);
        };
        issue_stage(std::integral_constant<int, 0>{});
        issue_stage(std::integral_constant<int, 1>{});
        issue_stage(std::integral_constant<int, 2>{});
    }
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LPS) : "memory");
    __syncthreads();

    u32x4 xf[MB];         // gradient operands of the current step
    u32x4 raw[RB][2];     // 32 code bytes per k row of this lane: four steps of one stage
    u32x4 wf[RB];         // code operands of the current step
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        raw[rb][0] = *reinterpret_cast<const u32x4 *>(smem + qa[rb][0]);
        raw[rb][1] = *reinterpret_cast<const u32x4 *>(smem + qa[rb][1]);
#pragma unroll
        for (int w = 0; w < 4; ++w) wf[rb][w] = convert_piece(std::integral_constant<int, 0>{}, w, raw[rb][0][0], raw[rb][0][1]);
    }
#pragma unroll
    for (int j = 0; j < MB; ++j) xf[j] = *reinterpret_cast<const u32x4 *>(smem + xa[0] + j * 4096);

    // One stage: four 16-wide steps.  st = index of this stage, nt3 / the slot of stage st + 3 are
    // what the loads issued in step 0 fetch.
    auto tile = [&](auto slot_tag, auto more_tag, int st, int nt) {
        constexpr int SLOT = decltype(slot_tag)::value;
        constexpr bool MORE = decltype(more_tag)::value;
        constexpr int NEXT = (SLOT + 1) % NRS;
        const uint8_t *cur = smem + (st & 3) * DX_STAGE;
        const uint8_t *nxt = smem + ((st + 1) & 3) * DX_STAGE;
        u32x4 rawn[RB][2];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const bool pre = t < 3 || MORE;
            const uint8_t *src = t < 3 ? cur + xa[(t + 1) & 3] : nxt + xa[0];
            uint32_t d0[RB], d1[RB];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                d0[rb] = t == 3 ? rawn[rb][0][0] : (t + 1 < 2 ? raw[rb][0][2 * (t + 1)] : raw[rb][1][2 * (t + 1 - 2)]);
                d1[rb] = t == 3 ? rawn[rb][0][1] : (t + 1 < 2 ? raw[rb][0][2 * (t + 1) + 1] : raw[rb][1][2 * (t + 1 - 2) + 1]);
                if (pre) asm volatile("" : "+v"(d0[rb]), "+v"(d1[rb]));  // pins the conversions to this step
            }
            u32x4 xfn[MB];
            u32x4 wfn[RB];
#pragma unroll
            for (int q = 0; q < NM; ++q) {
                const int j = q / RB, rb = q % RB;
                acc[rb][j] = mfma32(wf[rb], xf[j], acc[rb][j]);
                if (pre && q < MB) xfn[q] = *reinterpret_cast<const u32x4 *>(src + q * 4096);
                if (pre && q >= 1 && q - 1 < 4 * RB) {
                    const int prb = (q - 1) / 4, pw = (q - 1) % 4;
                    uint32_t piece = t < 3 ? convert_piece(std::integral_constant<int, SLOT>{}, pw, d0[prb], d1[prb])
                                           : convert_piece(std::integral_constant<int, NEXT>{}, pw, d0[prb], d1[prb]);
                    asm volatile("" : "+v"(piece));  // keeps the conversion inside this group
                    wfn[prb][pw] = piece;
                }
                if (MORE && t == 2 && q >= NM - 2 * RB) {
                    const int e = q - (NM - 2 * RB);
                    if constexpr (NEXT == 0)  // a new n tile: its code bytes
                        rawn[e / 2][e % 2] = *reinterpret_cast<const u32x4 *>(nxt + qa[e / 2][e % 2]);
                    else                      // the next bit-width of this n tile: the bytes at hand
                        rawn[e / 2][e % 2] = raw[e / 2][e % 2];
                }
                if (MORE && t == 0 && NM - 1 - q < LPS)
                    issue_one(nt + (SLOT + 3) / NRS, std::integral_constant<int, (SLOT + 3) % NRS>{}, (st + 3) & 3, NM - 1 - q);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (pre) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) wf[rb] = wfn[rb];
#pragma unroll
                for (int j = 0; j < MB; ++j) xf[j] = xfn[j];
            }
        }
        if (MORE) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                raw[rb][0] = rawn[rb][0];
                raw[rb][1] = rawn[rb][1];
            }
        }
    };
    auto stage = [&](auto slot_tag, auto more_tag, int st, int nt) {
        // stage st + 1 must be resident (operand prefetch at the end of this stage); the loads of
        // stage st + 2 may stay in flight; after the barrier the buffer of stage st - 1 is free
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPS) : "memory");
        __syncthreads();
        tile(slot_tag, more_tag, st, nt);
    };

    int st = 0;
    for (int nt = 0; nt + 1 < nnt; ++nt) {
        stage(std::integral_constant<int, 0>{}, std::true_type{}, st++, nt);
        if constexpr (NRS > 1) stage(std::integral_constant<int, 1>{}, std::true_type{}, st++, nt);
        if constexpr (NRS > 2) stage(std::integral_constant<int, 2>{}, std::true_type{}, st++, nt);
    }
    {
        const int nt = nnt - 1;
        if constexpr (NRS == 1) {
            stage(std::integral_constant<int, 0>{}, std::false_type{}, st++, nt);
        } else if constexpr (NRS == 2) {
            stage(std::integral_constant<int, 0>{}, std::true_type{}, st++, nt);
            stage(std::integral_constant<int, 1>{}, std::false_type{}, st++, nt);
        } else {
            stage(std::integral_constant<int, 0>{}, std::true_type{}, st++, nt);
            stage(std::integral_constant<int, 1>{}, std::true_type{}, st++, nt);
            stage(std::integral_constant<int, 2>{}, std::false_type{}, st++, nt);
        }
    }
    wait_vm0();  // zero-fill loads of dead stages must not land in the staging area below

    // ---- epilogue: rows of the product are k, columns tokens; dX = acc - c[m] --------------------
    // assembled in LDS as [token][k] bf16 (rows padded by 8 bytes) and stored as whole 512-byte rows
    __syncthreads();
    // c[m] = sum over the column ranges of the prep kernel, in their order.  The partial sums of all the
    // lane's tokens are requested four ranges at a time (20 loads in flight: one memory round trip per
    // group instead of one per value, which with nothing else to run cost more than the stores).
    float cs[MB];
#pragma unroll
    for (int j = 0; j < MB; ++j) cs[j] = 0.f;
    for (int sp0 = 0; sp0 < a.nsplit; sp0 += 4) {
        float part[4][MB];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int j = 0; j < MB; ++j) {
                const int m = m0 + j * 32 + l32;
                part[u][j] = (sp0 + u < a.nsplit && m < a.M) ? a.cvec[(size_t)(sp0 + u) * a.M + m] : 0.f;
            }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int j = 0; j < MB; ++j) cs[j] += part[u][j];
    }
#pragma unroll
    for (int j = 0; j < MB; ++j) {
        const float c = cs[j];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int kloc = wave * (32 * RB) + rb * 32 + 8 * g + 4 * h;
                const u32x2 o = {pack_bf16x2(acc[rb][j][4 * g] - c, acc[rb][j][4 * g + 1] - c),
                                 pack_bf16x2(acc[rb][j][4 * g + 2] - c, acc[rb][j][4 * g + 3] - c)};
                *reinterpret_cast<u32x2 *>(smem + (j * 32 + l32) * DX_OS + kloc * 2) = o;
            }
    }
    __syncthreads();
    constexpr int CPR = DX_BK / 8;  // 16-byte chunks per row
#pragma unroll
    for (int it = 0; it < DX_BM * CPR / 256; ++it) {
        const int c = it * 256 + threadIdx.x;
        const int row = c / CPR, ch = c % CPR;
        const int m = m0 + row, k = k0 + ch * 8;
        if (m < a.M && k < a.K) {
            const uint8_t *src = smem + row * DX_OS + ch * 16;
            const u32x2 lo = *reinterpret_cast<const u32x2 *>(src);
            const u32x2 hi = *reinterpret_cast<const u32x2 *>(src + 8);
            __builtin_nontemporal_store(u32x4{lo.x, lo.y, hi.x, hi.y},
                                        reinterpret_cast<u32x4 *>(a.dX + (size_t)m * a.K + k));
        }
    }
#else
    (void)a;
#endif
}

// ============================================================================================
// backward dW: dW[n, k] (+)= sum_m GT[n, m] * XT[k, m]   (plain bf16 GEMM, fp32 out)
// ============================================================================================
struct DwArgs {
    // Both operands come in blocks of 32 tokens, [M / 32][rows][32]: the 64-byte row segments that one LDS stage takes
    // from a tile's 256 rows are then one contiguous 16 KB piece of memory, i.e. whole 128-byte lines.  (With rows of
    // M tokens a stage would use half of every line it touches and the other half 32 tokens later, when the line has
    // left the first-level cache: twice the traffic between the caches.)
    const uint16_t *GT;  // [M / 32][N][32]
    const uint16_t *XT;  // [M / 32][K][32]
    float *dW;           // [N, K]
    float *part;         // [split tiles][parts][256][256]: partial tiles of the split last round
    int M, N, K;
    int ldm;             // M rounded up to a multiple of 8; tokens M .. ldm - 1 hold zeros
    int accumulate;
    int tiles_n, tiles_k;
    int whole;           // work items [0, whole) are whole tiles; the others are token ranges of the remaining tiles
    int parts;           // token ranges per remaining tile
};

constexpr int DW_RB = 4;                   // 32-row blocks of n per wave
constexpr int DW_MB = 4;                   // 32-column blocks of k per wave
constexpr int DW_BN = 2 * 32 * DW_RB;      // rows of n per workgroup (2 x 2 waves)
constexpr int DW_BK = 2 * 32 * DW_MB;      // columns of k per workgroup
constexpr int DW_BM = 32;                  // contraction elements (tokens) per stage: 64-byte rows
constexpr int DW_A_TILE = DW_BN * 64, DW_B_TILE = DW_BK * 64;
constexpr int DW_STAGE = DW_A_TILE + DW_B_TILE;
constexpr int DW_NST = 5;                  // LDS stages
constexpr int DW_LDS = DW_NST * DW_STAGE;
constexpr int DW_CUS = 256;                // compute units a round of workgroups fills

// How the tiles of dW are dealt to workgroups.  Whole rounds of 256 tiles run one tile per workgroup; the tiles of a
// last partial round (at most half a round) are cut along the tokens into `parts` ranges each, so that the round
// still occupies every compute unit for 1 / parts of a tile's time; the ranges leave fp32 partial tiles in the
// workspace and dw_reduce_kernel adds them in a fixed order.
struct DwPlan {
    int tiles_n, tiles_k, whole, rest, parts;
    size_t part_bytes;
};
static DwPlan dw_plan(int64_t M, int64_t N, int64_t K) {
    DwPlan p;
    p.tiles_n = (int)cdiv(N, DW_BN);
    p.tiles_k = (int)cdiv(K, DW_BK);
    const int64_t tiles = (int64_t)p.tiles_n * p.tiles_k;
    const int64_t stages = cdiv(M, DW_BM);
    int rest = (int)(tiles % DW_CUS);
    int parts = rest > 0 ? DW_CUS / rest : 1;
    parts = (int)std::min<int64_t>(parts, std::max<int64_t>(1, stages / 8));   // at least eight stages per range
    if (tiles < DW_CUS || parts < 2) rest = 0, parts = 1;
    p.whole = (int)(tiles - rest);
    p.rest = rest;
    p.parts = parts;
    p.part_bytes = (size_t)rest * parts * DW_BN * DW_BK * 4;
    return p;
}

// Same pipeline as the forward and dX kernels (one wave per SIMD, direct-to-LDS stages, one small fenced group of
// operand work per MFMA), without any code conversion: both operands are bf16 rows with the contraction index
// (tokens) contiguous.  The four waves form a 2 x 2 grid over the 256 x 256 tile, 128 x 128 each: 16 accumulators
// (all 256 accumulator registers), 8 operand reads per 16 MFMAs - the square wave tile is what keeps the LDS traffic
// (32 KB read + 16 KB written per 16-token step and compute unit, 94 bytes per clock at the matrix-core rate) under
// the 128 bytes per clock the LDS delivers.  Stages are 32 tokens deep (64-byte rows); five of them fill the LDS.
__global__ __launch_bounds__(256) void dw_kernel(DwArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    constexpr int RB = DW_RB, MB = DW_MB, NM = RB * MB;
    constexpr int AL = DW_BN / 64, BL = DW_BK / 64;  // direct-to-LDS loads per wave and stage (16 rows each)
    constexpr int LPS = AL + BL;
    static_assert(RB + MB <= NM && LPS <= NM, "not enough MFMAs to hide the operand work");
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wn = wave >> 1, wk = wave & 1;
    const int h = lane >> 5, l32 = lane & 31;

    // work item -> tile and token range
    const int nmt_all = (a.M + DW_BM - 1) / DW_BM;
    uint32_t lid;
    int mt0 = 0, mt1 = nmt_all;
    float *dst = a.dW;
    bool to_part = false;
    if ((int)blockIdx.x < a.whole) {
        lid = xcd_contiguous_id(blockIdx.x, (uint32_t)a.whole);
    } else {
        const int idx = (int)blockIdx.x - a.whole, part = idx % a.parts;
        lid = (uint32_t)(a.whole + idx / a.parts);
        mt0 = (int)((int64_t)nmt_all * part / a.parts);
        mt1 = (int)((int64_t)nmt_all * (part + 1) / a.parts);
        dst = a.part + (size_t)idx * (DW_BN * DW_BK);
        to_part = true;
    }
    constexpr int GROUP = 4;
    const int width = GROUP * a.tiles_k;
    const int first_n = (int)(lid / width) * GROUP;
    const int gsz = min(a.tiles_n - first_n, GROUP);
    const int tn = first_n + (int)(lid % width) % gsz;
    const int tk = (int)(lid % width) / gsz;
    const int n0 = tn * DW_BN, k0 = tk * DW_BK;

    uint32_t off0;
    int colb;  // byte column of this lane's 16-byte piece inside a 64-byte row
    u8_tile_lane<4>(wave, lane, 0, 64u, off0, colb);
    const uint32_t rstep = 64u * 64u;  // 64 rows further down

    // load i of the stage of token block mt into LDS buffer `buf`.  The descriptor of a stage starts at the tile's
    // first row inside that block and ends with the block, so rows past N (K) are out of range; a block or a piece
    // past M is requested at an out-of-range offset.  Both are answered with zeros without touching memory, so the
    // loads in flight are the same every stage.
    auto issue_one = [&](int mt, int buf, int i) {
        const int mm = mt * DW_BM;
        uint8_t *base = smem + buf * DW_STAGE;
        const uint32_t o = (mm + colb / 2 < a.M) ? off0 : kOOB;
        if (i < AL) {
            const __amdgpu_buffer_rsrc_t rG = make_rsrc(a.GT + ((size_t)mt * a.N + n0) * 32, (uint64_t)(a.N - n0) * 64);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rG, (lds_ptr)(base + (wave + i * 4) * 1024), 16,
                                                     o + (uint32_t)i * rstep, 0, 0, 0);
        } else {
            const __amdgpu_buffer_rsrc_t rX = make_rsrc(a.XT + ((size_t)mt * a.K + k0) * 32, (uint64_t)(a.K - k0) * 64);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rX, (lds_ptr)(base + DW_A_TILE + (wave + (i - AL) * 4) * 1024), 16,
                                                     o + (uint32_t)(i - AL) * rstep, 0, 0, 0);
        }
    };

    // LDS fragment offsets inside a stage for the two 16-token steps of a stage
    uint32_t ab[2], bb[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const uint32_t chunk = (uint32_t)((2 * t + h) ^ ((l32 >> 2) & 3)) << 4;
        ab[t] = (uint32_t)(wn * 128 + l32) * 64u + chunk;
        bb[t] = (uint32_t)DW_A_TILE + (uint32_t)(wk * 128 + l32) * 64u + chunk;
    }

    f32x16 acc[RB][MB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int j = 0; j < MB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[rb][j][v] = 0.f;

    const int nmt = mt1 - mt0;   // >= 1 (the host plans at least eight stages per range)
#pragma unroll
    for (int st = 0; st < DW_NST - 1; ++st)
#pragma unroll
        for (int i = 0; i < LPS; ++i) issue_one(mt0 + st, st, i);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DW_NST - 2) * LPS) : "memory");
    __syncthreads();

    u32x4 af[RB], bf[MB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) af[rb] = *reinterpret_cast<const u32x4 *>(smem + ab[0] + rb * 2048);
#pragma unroll
    for (int j = 0; j < MB; ++j) bf[j] = *reinterpret_cast<const u32x4 *>(smem + bb[0] + j * 2048);

    // one stage: two 16-token steps; cb = LDS buffer of this stage
    auto tile = [&](auto more_tag, int mt, int cb) {
        constexpr bool MORE = decltype(more_tag)::value;
        const int nb = cb + 1 == DW_NST ? 0 : cb + 1;   // buffer of the next stage
        const int ib = cb == 0 ? DW_NST - 1 : cb - 1;   // buffer of stage mt + NST - 1 (= the one of stage mt - 1)
        const uint8_t *cur = smem + cb * DW_STAGE;
        const uint8_t *nxt = smem + nb * DW_STAGE;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const bool pre = t == 0 || MORE;
            const uint8_t *src = t == 0 ? cur : nxt;
            const int tn_ = t == 0 ? 1 : 0;
            u32x4 afn[RB], bfn[MB];
#pragma unroll
            for (int q = 0; q < NM; ++q) {
                const int rb = q % RB, j = q / RB;
                acc[rb][j] = mfma32(af[rb], bf[j], acc[rb][j]);
                if (pre && q < RB) afn[q] = *reinterpret_cast<const u32x4 *>(src + ab[tn_] + q * 2048);
                if (pre && q >= RB && q < RB + MB)
                    bfn[q - RB] = *reinterpret_cast<const u32x4 *>(src + bb[tn_] + (q - RB) * 2048);
                if (MORE && t == 0 && q >= NM - LPS) issue_one(mt + DW_NST - 1, ib, q - (NM - LPS));
                __builtin_amdgcn_sched_barrier(0);
            }
            if (pre) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) af[rb] = afn[rb];
#pragma unroll
                for (int j = 0; j < MB; ++j) bf[j] = bfn[j];
            }
        }
    };

    int cb = 0;
    for (int mt = 0; mt + 1 < nmt; ++mt) {
        // stage mt + 1 must be resident (operand prefetch at the end of this stage); the loads of
        // stages mt + 2 and mt + 3 may stay in flight; after the barrier the buffer of stage mt - 1
        // is free for stage mt + 4
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DW_NST - 3) * LPS) : "memory");
        __syncthreads();
        tile(std::true_type{}, mt0 + mt, cb);
        cb = cb + 1 == DW_NST ? 0 : cb + 1;
    }
    tile(std::false_type{}, mt0 + nmt - 1, cb);
    wait_vm0();  // loads of stages that nobody consumes must have landed before the workgroup ends

    // Rows of the product are n, columns k: a store instruction writes 32 consecutive k (one 128-byte line)
    // of two rows.  Branch-free: every store goes through a buffer descriptor that starts at the first
    // element of the wave's 32-row block and ends with the destination, so rows past N fall out of range and are
    // dropped by the memory unit; a column past K is sent out of range explicitly.  The row part of the
    // address (wave-uniform) travels in the scalar offset, the lane part in one register per k block.
    // A token range of a split tile writes its whole 256 x 256 partial tile instead (row length 256, no edges).
    // When accumulating, the old values of four rows are requested together, one memory round trip per 16 values.
    const int ld = to_part ? DW_BK : a.K;              // row length of the destination
    const int rows = to_part ? DW_BN : a.N - n0;       // rows and columns of the destination from this tile's origin
    const int cols = to_part ? DW_BK : a.K - k0;
    float *origin = to_part ? dst : dst + (int64_t)n0 * a.K + k0;
    auto store_tile = [&](auto accumulate_tag) {
        constexpr bool ACCUMULATE = decltype(accumulate_tag)::value;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int r0 = wn * 128 + rb * 32;                      // first row of the block inside the tile
            const int64_t left = ((int64_t)rows - r0) * ld - (to_part ? 0 : k0);  // elements to the end of the destination
            const __amdgpu_buffer_rsrc_t rW = make_rsrc(origin + (int64_t)r0 * ld, left > 0 ? (uint64_t)left * 4u : 0u);
            uint32_t voff[MB];
#pragma unroll
            for (int j = 0; j < MB; ++j) {
                const int c = wk * 128 + j * 32 + l32;
                voff[j] = c < cols ? ((uint32_t)(4 * h) * (uint32_t)ld + (uint32_t)c) * 4u : kOOB;
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint32_t old[ACCUMULATE ? 4 : 1][MB];
                if constexpr (ACCUMULATE) {  // the values of four rows are requested together
#pragma unroll
                    for (int e = 0; e < 4; ++e)
#pragma unroll
                        for (int j = 0; j < MB; ++j)
                            old[e][j] = __builtin_amdgcn_raw_buffer_load_b32(rW, voff[j], (uint32_t)(8 * g + e) * (uint32_t)ld * 4u, 0);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t row = (uint32_t)(8 * g + e) * (uint32_t)ld * 4u;
#pragma unroll
                    for (int j = 0; j < MB; ++j) {
                        float v = acc[rb][j][4 * g + e];
                        if constexpr (ACCUMULATE) v = __uint_as_float(old[e][j]) + v;
                        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rW, voff[j], row, 0);
                    }
                }
            }
        }
    };
    if (a.accumulate && !to_part)
        store_tile(std::true_type{});
    else
        store_tile(std::false_type{});
#else
    (void)a;
#endif
}

// dW tile (+)= the partial tiles of its token ranges, added in the order of the ranges.  One workgroup per 16 rows of
// a split tile, a thread per four columns.
__global__ __launch_bounds__(256) void dw_reduce_kernel(DwArgs a) {
    const int t = blockIdx.x / (DW_BN / 16), r16 = blockIdx.x % (DW_BN / 16);   // split tile, 16-row block
    const uint32_t lid = (uint32_t)(a.whole + t);
    constexpr int GROUP = 4;
    const int width = GROUP * a.tiles_k;
    const int first_n = (int)(lid / width) * GROUP;
    const int gsz = min(a.tiles_n - first_n, GROUP);
    const int tn = first_n + (int)(lid % width) % gsz;
    const int tk = (int)(lid % width) / gsz;
    const int row = r16 * 16 + (threadIdx.x >> 6) * 4, col = (threadIdx.x & 63) * 4;
    const int k = tk * DW_BK + col;
    if (k >= a.K) return;   // (K is a multiple of 8: four columns are inside or outside together)
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int n = tn * DW_BN + row + rr;
        if (n >= a.N) return;
        const float *src = a.part + (size_t)t * a.parts * (DW_BN * DW_BK) + (size_t)(row + rr) * DW_BK + col;
        f32x4 sum = *reinterpret_cast<const f32x4 *>(src);
        for (int p = 1; p < a.parts; ++p) sum += *reinterpret_cast<const f32x4 *>(src + (size_t)p * (DW_BN * DW_BK));
        f32x4 *out = reinterpret_cast<f32x4 *>(a.dW + (size_t)n * a.K + k);
        if (a.accumulate) sum += *out;
        *out = sum;
    }
}

// ============================================================================================
// host side
// ============================================================================================
static size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

struct BwdWorkspace {
    size_t cvec, as[3], gt, xt, qt, dwp, total;
};

static BwdWorkspace bwd_layout(int64_t M, int64_t N, int64_t K, int nr) {
    BwdWorkspace w;
    size_t o = 0;
    w.cvec = o;
    o += align256((size_t)PREP_MAX_SPLIT * M * 4);
    for (int i = 0; i < 3; ++i) {
        w.as[i] = o;
        if (i < nr) o += align256((size_t)M * N * 2);
    }
    const size_t m32 = ((size_t)M + 31) & ~(size_t)31;   // the transposed operands of dW come in blocks of 32 tokens
    w.gt = o;
    o += align256(m32 * N * 2);
    w.xt = o;
    o += align256(m32 * K * 2);
    w.qt = o;
    o += align256((size_t)N * K);
    w.dwp = o;
    o += align256(dw_plan(M, N, K).part_bytes);
    w.total = o;
    return w;
}

static mq_status check_rs(const int *rs, int nr) {
    if (!rs) return MQ_ERR_NULL;
    if (nr < 1 || nr > 3) return MQ_ERR_BITS;
    for (int i = 0; i < nr; ++i) {
        if (rs[i] < 1 || rs[i] > 8) return MQ_ERR_BITS;
        for (int j = 0; j < i; ++j)
            if (rs[j] == rs[i]) return MQ_ERR_BITS;
    }
    return MQ_OK;
}

template <typename Kern>
static bool allow_lds(Kern kern, int bytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                               bytes) == hipSuccess;
}

template <int NR, bool HAS8, bool EP, int MB, bool LOSS>
static mq_status launch_fwd_mb(FwdArgs a, hipStream_t st, int64_t *blocks) {
    a.tiles_m = (int)cdiv(a.M, 32 * MB);
    a.tiles_n = (int)cdiv(a.N, FWD_BN);
    *blocks = (int64_t)a.tiles_m * a.tiles_n;
    if (!allow_lds(fwd_kernel<NR, HAS8, EP, MB, LOSS>, fwd_lds(MB, NR))) return MQ_ERR_DEVICE;
    fwd_kernel<NR, HAS8, EP, MB, LOSS><<<dim3(a.tiles_m * a.tiles_n), dim3(256), fwd_lds(MB, NR), st>>>(a);
    return launch_status();
}

// Token-tile height: the tallest tile amortises the code conversion and the epilogue best, but the
// number of tiles rarely divides evenly over the 256 compute units; one block less can save a whole
// round of workgroups.  Cost of a choice = rounds x (main loop + epilogue) in matrix-core cycles
// (32 per MFMA, plus about 180 cycles per 64-wide k stage and bit-width that do not shrink with the tile:
// conversions and the stage barrier - fitted on the 9B gate shape, where 160 tokens run 2.5-4 % faster than
// 128 although both fill their rounds; prologue and epilogue constants measured on the Gemma-2-2B shapes).
template <int NR, bool HAS8, bool EP, bool LOSS>
static mq_status launch_fwd(const FwdArgs &a, hipStream_t st, int64_t *blocks) {
    constexpr int HI = fwd_mb(NR), LO = HI - 1;
    auto cost = [&](int mb) {
        const int64_t tiles = cdiv(a.M, 32 * mb) * cdiv(a.N, FWD_BN);
        const int64_t rounds = cdiv(tiles, 256);
        const int64_t per_tile = cdiv(a.K, BKT) * (NR * mb * 128 + 180 * NR) + 3000 + 890 * NR * mb;
        return rounds * per_tile;
    };
    return cost(LO) < cost(HI) ? launch_fwd_mb<NR, HAS8, EP, LO, LOSS>(a, st, blocks)
                               : launch_fwd_mb<NR, HAS8, EP, HI, LOSS>(a, st, blocks);
}

template <int NR, bool HAS8, bool LOSS>
static mq_status launch_fwd_ep(const FwdArgs &a, bool ep, hipStream_t st, int64_t *blocks) {
    return ep ? launch_fwd<NR, HAS8, true, LOSS>(a, st, blocks) : launch_fwd<NR, HAS8, false, LOSS>(a, st, blocks);
}

template <bool LOSS>
static mq_status launch_fwd_any(const FwdArgs &a, int nr, bool has8, bool ep, hipStream_t st, int64_t *blocks) {
    if (nr == 1)
        return has8 ? launch_fwd_ep<1, true, LOSS>(a, ep, st, blocks) : launch_fwd_ep<1, false, LOSS>(a, ep, st, blocks);
    if (nr == 2)
        return has8 ? launch_fwd_ep<2, true, LOSS>(a, ep, st, blocks) : launch_fwd_ep<2, false, LOSS>(a, ep, st, blocks);
    return has8 ? launch_fwd_ep<3, true, LOSS>(a, ep, st, blocks) : launch_fwd_ep<3, false, LOSS>(a, ep, st, blocks);
}

// workgroups of the forward kernel at its smallest token tile (128 tokens): bound for the partial sums
static int64_t fwd_max_blocks(int64_t M, int64_t N) { return cdiv(M, 128) * cdiv(N, FWD_BN); }

template <int NRS, bool HAS8, bool EP>
static mq_status launch_dx_one(const DxArgs &d, hipStream_t st) {
    if (!allow_lds(dx_kernel<NRS, HAS8, EP>, dx_lds())) return MQ_ERR_DEVICE;
    dx_kernel<NRS, HAS8, EP><<<dim3(d.tiles_m * d.tiles_k), dim3(256), dx_lds(), st>>>(d);
    return launch_status();
}

template <int NRS>
static mq_status launch_dx_nrs(const DxArgs &d, bool has8, bool ep, hipStream_t st) {
    if (has8) return ep ? launch_dx_one<NRS, true, true>(d, st) : launch_dx_one<NRS, true, false>(d, st);
    return ep ? launch_dx_one<NRS, false, true>(d, st) : launch_dx_one<NRS, false, false>(d, st);
}

static mq_status launch_dx(const DxArgs &d, int nr, bool has8, bool ep, hipStream_t st) {
    if (nr == 1) return launch_dx_nrs<1>(d, has8, ep, st);
    if (nr == 2) return launch_dx_nrs<2>(d, has8, ep, st);
    return launch_dx_nrs<3>(d, has8, ep, st);
}

}  // namespace mq

extern "C" size_t mq_workspace_bytes(int op, int64_t M, int64_t N, int64_t K, int nr) {
    using namespace mq;
    if (op == MQ_OP_GEMV)  // M = B, nr = bits per code
        return M < 1 || M > 16 || N < 0 || K < 1 || nr < 1 || nr > 8 ? 0 : std::max<size_t>(256, gemv_split_workspace_bytes(M, N, K, nr));
    if (M < 0 || N < 0 || K < 0 || nr < 1 || nr > 3) return 0;
    if (op == MQ_OP_LINEAR_FWD) return align256((size_t)M * 4) + 256;
    if (op == MQ_OP_LINEAR_FWD_L2) return align256((size_t)M * 4) + (size_t)fwd_max_blocks(M, N) * 16 + 256;
    if (op == MQ_OP_LINEAR_BWD) return bwd_layout(M, N, K, nr).total + 256;
    if (op == MQ_OP_FFN_DECODE) return ffn_workspace_bytes(M, N, K);
    if (op == MQ_OP_L2_LOSS) return loss_workspace_bytes(M, N);
    if (op == MQ_OP_LINEAR_BWD_CLIP) return clip_workspace_bytes(M, N, K);
    if (op == MQ_OP_AFFINE_BWD) return affine_workspace_bytes(M, N, K);
    return 0;
}

namespace mq {

// the L2 objective evaluated in the forward epilogue (user order; mapped to slots below)
struct FwdLoss {
    const uint16_t *target;
    const int *teacher;
    const float *lambda;
    uint16_t *const *dY;
    float *losses;
    uint32_t mix;
    const float *bias;
};

static mq_status fwd_run(const uint16_t *X, const uint8_t *Q, const float *alpha, const float *zero, int64_t M,
                         int64_t N, int64_t K, const int *rs, int nr, uint32_t flags, uint16_t *const *Y,
                         const FwdLoss *loss, void *ws, size_t ws_bytes, void *hip_stream,
                         bool check_only = false, uint16_t *const *gated_out = nullptr, int gate = 0) {
    if (M < 0 || N < 0 || K < 1) return MQ_ERR_SHAPE;
    if (M > 0x7FFFFF00 || N > 0x7FFFFF00 || K > (1 << 22)) return MQ_ERR_SHAPE;
    if (cdiv(M, 128) * cdiv(N, FWD_BN) > 0x7FFFFFFF) return MQ_ERR_SHAPE;  // tiles of one launch
    mq_status s = check_rs(rs, nr);
    if (s != MQ_OK) return s;
    if (K % 16 != 0 || N % 8 != 0) return MQ_ERR_ALIGN;
    bool need_target = false;
    if (loss) {
        need_target = loss->mix || !loss->teacher;
        if (loss->teacher)
            for (int i = 0; i < nr; ++i) {
                if (loss->teacher[i] < -1 || loss->teacher[i] >= nr || loss->teacher[i] == i) return MQ_ERR_SHAPE;
                if (loss->teacher[i] < 0) need_target = true;
            }
    }
    if (M == 0 || N == 0) return MQ_OK;
    if (!X || !Q || !alpha || !zero) return MQ_ERR_NULL;
    if (!loss && !Y && !gate) return MQ_ERR_NULL;
    if (gate && !gated_out) return MQ_ERR_NULL;
    for (int i = 0; i < nr; ++i) {
        uint16_t *yi = Y ? Y[i] : nullptr;
        if (!loss && !gate && !yi) return MQ_ERR_NULL;
        if (yi && !aligned16(yi)) return MQ_ERR_ALIGN;
        if (gate && !gated_out[i]) return MQ_ERR_NULL;
        if (gate && (reinterpret_cast<uintptr_t>(gated_out[i]) & 7u)) return MQ_ERR_ALIGN;
    }
    if (loss) {
        if (!loss->dY || !loss->losses || (need_target && !loss->target)) return MQ_ERR_NULL;
        for (int i = 0; i < nr; ++i) {
            if (!loss->dY[i]) return MQ_ERR_NULL;
            if (!aligned16(loss->dY[i])) return MQ_ERR_ALIGN;
        }
        if (loss->target && !aligned16(loss->target)) return MQ_ERR_ALIGN;
        if (loss->bias && !aligned16(loss->bias)) return MQ_ERR_ALIGN;
    }
    if (!aligned16(X) || !aligned16(Q) || !aligned16(alpha) || !aligned16(zero)) return MQ_ERR_ALIGN;
    const int op = loss ? MQ_OP_LINEAR_FWD_L2 : MQ_OP_LINEAR_FWD;
    if (check_only) return MQ_OK;  // every argument but the workspace is fine
    if (!ws || ws_bytes < mq_workspace_bytes(op, M, N, K, nr) || !aligned16(ws)) return MQ_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);

    FwdArgs a{};
    a.X = X;
    a.Q = Q;
    a.alpha = alpha;
    a.zero = zero;
    a.rowsum = static_cast<float *>(ws);
    a.M = (int)M;
    a.N = (int)N;
    a.K = (int)K;
    // slot order: the r = 8 slot (if any) first
    int has8 = 0, pos = 0;
    int slot_of[3] = {0, 0, 0};
    for (int i = 0; i < 3; ++i) {
        a.Y[i] = nullptr;
        a.A[i] = nullptr;
        a.r[i] = 8;
    }
    a.gate = gate;
    for (int i = 0; i < nr; ++i)
        if (rs[i] == 8) {
            has8 = 1;
            slot_of[i] = 0;
        }
    pos = has8;
    for (int i = 0; i < nr; ++i)
        if (rs[i] != 8) slot_of[i] = pos++;
    for (int i = 0; i < nr; ++i) {
        a.Y[slot_of[i]] = Y ? Y[i] : nullptr;
        a.A[slot_of[i]] = gate ? gated_out[i] : nullptr;
        a.r[slot_of[i]] = rs[i];
    }
    const double mn = (double)M * (double)N;
    if (loss) {
        a.T = loss->target;
        a.bias = loss->bias;
        a.mix = loss->mix ? 1 : 0;
        a.partial = reinterpret_cast<float *>(static_cast<uint8_t *>(ws) + align256((size_t)M * 4));
        for (int i = 0; i < nr; ++i) {
            const int sl = slot_of[i];
            a.dY[sl] = loss->dY[i];
            const int th = loss->teacher ? loss->teacher[i] : -1;
            a.teacher[sl] = th < 0 ? -1 : slot_of[th];
            a.coef[sl] = (float)((loss->lambda ? (double)loss->lambda[i] : 1.0) * 2.0 / mn);
        }
    }

    rowsum_kernel<<<dim3((unsigned)cdiv(M, 4)), dim3(256), 0, st>>>(X, (int)M, (int)K, static_cast<float *>(ws));
    const bool ep = flags & MQ_FLAG_EXTRA_PRECISION;
    int64_t blocks = 0;
    if (!loss) return launch_fwd_any<false>(a, nr, has8, ep, st, &blocks);
    s = launch_fwd_any<true>(a, nr, has8, ep, st, &blocks);
    if (s != MQ_OK) return s;
    // the kernel's sums are in slot order: where that is not the caller's order (an r = 8 that is
    // not first) they are finished into the tail of the workspace and permuted
    float *slot_losses = a.partial + (size_t)fwd_max_blocks(M, N) * 4;
    bool same = true;
    for (int i = 0; i < nr; ++i) same = same && slot_of[i] == i;
    s = launch_loss_finish(a.partial, blocks, nr, (float)(1.0 / mn), same ? loss->losses : slot_losses, st);
    if (s != MQ_OK || same) return s;
    permute3_kernel<<<dim3(1), dim3(64), 0, st>>>(slot_losses, loss->losses, nr, slot_of[0], slot_of[1], slot_of[2]);
    return launch_status();
}

// 16-byte chunks of zeros (a kernel, not a memset node: callers may capture the stream into a graph)
__global__ __launch_bounds__(256) void zero_fill_kernel(u32x4 *__restrict__ dst, int64_t chunks) {
    for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < chunks; c += (int64_t)gridDim.x * 256)
        dst[c] = u32x4{0u, 0u, 0u, 0u};
}

}  // namespace mq

extern "C" mq_status mq_linear_fwd_multi(const uint16_t *X, const uint8_t *Q, const float *alpha,
                                         const float *zero, int64_t M, int64_t N, int64_t K, const int *rs,
                                         int nr, uint32_t flags, uint16_t *const *Y, void *ws, size_t ws_bytes,
                                         void *hip_stream) {
    return mq::fwd_run(X, Q, alpha, zero, M, N, K, rs, nr, flags, Y, nullptr, ws, ws_bytes, hip_stream);
}

extern "C" mq_status mq_linear_fwd_multi_gated(const uint16_t *X, const uint8_t *Q, const float *alpha,
                                               const float *zero, int64_t M, int64_t F, int64_t K, const int *rs,
                                               int nr, uint32_t flags, uint16_t *const *GU, uint16_t *const *A,
                                               void *ws, size_t ws_bytes, void *hip_stream) {
    if (F < 0 || F > 0x3FFFFF00) return MQ_ERR_SHAPE;
    if (F % 4 != 0) return MQ_ERR_ALIGN;  // rows of A start on 8-byte boundaries
    return mq::fwd_run(X, Q, alpha, zero, M, 2 * F, K, rs, nr, flags, GU, nullptr, ws, ws_bytes, hip_stream, false, A,
                       (flags & MQ_FLAG_FFN_SILU) ? 2 : 1);
}

// ---- the forward for callers that cannot allocate --------------------------------------------------
// Scratch of mq_linear_fwd_multi_noalloc: the per-token sums of X that the forward's pre-pass writes and
// its epilogue reads, in device memory that belongs to the library image (one copy per GPU, held until
// the process ends) instead of a caller workspace.
namespace mq {
constexpr int64_t kNoAllocMaxTokens = 1 << 18;
constexpr int kNoAllocMaxDevices = 64;
static __device__ __align__(256) float scratch[kNoAllocMaxTokens + 64];
// device address of `scratch` per GPU (the array's name is only a host-side handle), looked up once per device
static void *g_scratch_addr[kNoAllocMaxDevices];
static std::mutex g_scratch_mutex;

static mq_status noalloc_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kNoAllocMaxDevices) return MQ_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_addr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MQ_ERR_DEVICE;
        g_scratch_addr[dev] = ptr;
    }
    *out = g_scratch_addr[dev];
    return MQ_OK;
}
}  // namespace mq

extern "C" mq_status mq_linear_fwd_multi_noalloc(const uint16_t *X, const uint8_t *Q, const float *alpha,
                                                 const float *zero, int64_t M, int64_t N, int64_t K, const int *rs,
                                                 int nr, uint32_t flags, uint16_t *const *Y, void *hip_stream) {
    using namespace mq;
    if (M > kNoAllocMaxTokens) return MQ_ERR_SHAPE;  // more tokens than the built-in scratch holds
    const size_t need = M >= 0 && nr >= 1 && nr <= 3 ? mq_workspace_bytes(MQ_OP_LINEAR_FWD, M, N, K, nr) : 0;
    if (need > sizeof(float) * (kNoAllocMaxTokens + 64)) return MQ_ERR_SHAPE;
    // the arguments are checked before the device is touched; an empty call launches nothing and needs no scratch
    mq_status s = fwd_run(X, Q, alpha, zero, M, N, K, rs, nr, flags, Y, nullptr, nullptr, 0, hip_stream, true);
    if (s != MQ_OK || M == 0 || N == 0) return s;
    void *ws = nullptr;
    s = noalloc_scratch(&ws);
    if (s != MQ_OK) return s;
    return fwd_run(X, Q, alpha, zero, M, N, K, rs, nr, flags, Y, nullptr, ws, sizeof(float) * (kNoAllocMaxTokens + 64),
                   hip_stream);
}

extern "C" mq_status mq_linear_fwd_multi_l2(const uint16_t *X, const uint8_t *Q, const float *alpha,
                                            const float *zero, int64_t M, int64_t N, int64_t K, const int *rs,
                                            int nr, uint32_t flags, const float *bias, const uint16_t *target,
                                            const int *teacher, const float *lambda, uint16_t *const *Y,
                                            uint16_t *const *dY, float *losses, void *ws, size_t ws_bytes,
                                            void *hip_stream) {
    const mq::FwdLoss loss{target, teacher, lambda, dY, losses, flags & MQ_FLAG_LOSS_MIX, bias};
    return mq::fwd_run(X, Q, alpha, zero, M, N, K, rs, nr, flags, Y, &loss, ws, ws_bytes, hip_stream);
}

namespace mq {
// gated: the output gradients come from GU and dA (see PrepArgs) instead of dY
static mq_status bwd_run(bool gated, const uint16_t *X, const uint8_t *Q, const float *alpha, const float *zero,
                         const uint16_t *const *dY, const uint16_t *const *GU, const uint16_t *const *dA,
                         const float *lambda, int64_t M, int64_t N, int64_t K, const int *rs, int nr, uint32_t flags,
                         uint16_t *dX, float *dW, void *ws, size_t ws_bytes, void *hip_stream) {
    if (M < 0 || N < 0 || K < 1) return MQ_ERR_SHAPE;
    if (M > (1 << 22) || N > (1 << 22) || K > (1 << 22)) return MQ_ERR_SHAPE;
    mq_status s = check_rs(rs, nr);
    if (s != MQ_OK) return s;
    if (K % 16 != 0 || N % 16 != 0) return MQ_ERR_ALIGN;
    if (M == 0 || N == 0) {
        // empty sums: dW (over no tokens) and dX (over no channels) are zero
        hipStream_t st0 = static_cast<hipStream_t>(hip_stream);
        const bool zero_dw = M == 0 && N > 0 && dW && !(flags & MQ_FLAG_ACCUM_DW), zero_dx = N == 0 && M > 0 && dX;
        if (!zero_dw && !zero_dx) return MQ_OK;
        if (M == 0 && N > 0 && dW && !(flags & MQ_FLAG_ACCUM_DW)) {
            if (!aligned16(dW)) return MQ_ERR_ALIGN;
            zero_fill_kernel<<<dim3((unsigned)std::min<int64_t>(cdiv(N * K / 4, 256), 65536)), dim3(256), 0, st0>>>(
                reinterpret_cast<u32x4 *>(dW), N * K / 4);
        }
        if (N == 0 && M > 0 && dX) {
            if (!aligned16(dX)) return MQ_ERR_ALIGN;
            zero_fill_kernel<<<dim3((unsigned)std::min<int64_t>(cdiv(M * K / 8, 256), 65536)), dim3(256), 0, st0>>>(
                reinterpret_cast<u32x4 *>(dX), M * K / 8);
        }
        return launch_status();
    }
    if (gated) {
        if (!GU || !dA) return MQ_ERR_NULL;
        for (int i = 0; i < nr; ++i) {
            if (!GU[i] || !dA[i]) return MQ_ERR_NULL;
            if (!aligned16(GU[i]) || !aligned16(dA[i])) return MQ_ERR_ALIGN;
        }
    } else {
        if (!dY) return MQ_ERR_NULL;
        for (int i = 0; i < nr; ++i) {
            if (!dY[i]) return MQ_ERR_NULL;
            if (!aligned16(dY[i])) return MQ_ERR_ALIGN;
        }
    }
    if (dX && (!Q || !alpha || !zero)) return MQ_ERR_NULL;
    if (dW && !X) return MQ_ERR_NULL;
    if ((dX && !aligned16(dX)) || (dW && !aligned16(dW)) || (X && !aligned16(X)) || (Q && !aligned16(Q)) ||
        (alpha && !aligned16(alpha)) || (zero && !aligned16(zero)))
        return MQ_ERR_ALIGN;
    if (!ws || ws_bytes < mq_workspace_bytes(MQ_OP_LINEAR_BWD, M, N, K, nr) || !aligned16(ws))
        return MQ_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const BwdWorkspace lay = bwd_layout(M, N, K, nr);
    uint8_t *base = static_cast<uint8_t *>(ws);
    const bool ep = flags & MQ_FLAG_EXTRA_PRECISION;

    // one pass over the gradients: scaled operands + c for dX, transposed sum for dW
    PrepArgs p;
    for (int i = 0; i < 3; ++i) {
        const int j = i < nr ? i : 0;
        p.dY[i] = gated ? nullptr : dY[j];
        p.GU[i] = gated ? GU[j] : nullptr;
        p.dA[i] = gated ? dA[j] : nullptr;
        p.As[i] = dX ? reinterpret_cast<uint16_t *>(base + lay.as[j]) : nullptr;
        p.lam[i] = lambda ? lambda[j] : 1.0f;
        p.mult[i] = rs[j] == 8 ? 1.0f : (float)(1 << (8 - rs[j]));
        p.bias[i] = rs[j] == 8 ? 0.0f : 128.0f;
    }
    p.alpha = alpha;
    p.zero = zero;
    p.cpart = dX ? reinterpret_cast<float *>(base + lay.cvec) : nullptr;
    p.GT = dW ? reinterpret_cast<uint16_t *>(base + lay.gt) : nullptr;
    p.nr = nr;
    p.M = (int)M;
    p.N = (int)N;
    p.ldm = (int)((M + 7) & ~(int64_t)7);
    // column ranges so that about a thousand workgroups exist; c[m] is summed over them in the dX epilogue
    const int64_t strips = cdiv(M, PREP_ROWS);
    int nsplit = (int)std::min<int64_t>(std::min<int64_t>(PREP_MAX_SPLIT, cdiv(N, 64)), std::max<int64_t>(1, cdiv(1024, strips)));
    p.cols_per_split = (int)(cdiv(cdiv(N, nsplit), 64) * 64);
    nsplit = (int)cdiv(N, p.cols_per_split);
    p.silu = (flags & MQ_FLAG_FFN_SILU) ? 1 : 0;
    if (gated)
        bwd_prep_kernel<true><<<dim3((unsigned)strips, (unsigned)nsplit), dim3(256), 0, st>>>(p);
    else
        bwd_prep_kernel<false><<<dim3((unsigned)strips, (unsigned)nsplit), dim3(256), 0, st>>>(p);

    if (dX) {
        uint8_t *QT = base + lay.qt;
        transpose_kernel<uint8_t><<<dim3((unsigned)cdiv(K, 64), (unsigned)cdiv(N, 64)), dim3(256), 0, st>>>(
            Q, QT, (int)N, (int)K, (int)N);

        // slot order of the kernel: the r = 8 bit-width (if any) first
        DxArgs d;
        int order[3] = {0, 0, 0}, has8 = 0, pos = 0;
        for (int i = 0; i < nr; ++i)
            if (rs[i] == 8) {
                has8 = 1;
                order[pos++] = i;
            }
        for (int i = 0; i < nr; ++i)
            if (rs[i] != 8) order[pos++] = i;
        for (int i = 0; i < 3; ++i) {
            const int j = order[i < nr ? i : 0];
            d.As[i] = p.As[j];
            d.r[i] = rs[j];
        }
        d.QT = QT;
        d.cvec = p.cpart;
        d.nsplit = nsplit;
        d.dX = dX;
        d.M = (int)M;
        d.N = (int)N;
        d.K = (int)K;
        d.tiles_m = (int)cdiv(M, DX_BM);
        d.tiles_k = (int)cdiv(K, DX_BK);
        const mq_status ds = launch_dx(d, nr, has8 != 0, ep, st);
        if (ds != MQ_OK) return ds;
    }
    if (dW) {
        uint16_t *XT = reinterpret_cast<uint16_t *>(base + lay.xt);
        transpose_kernel<uint16_t, true><<<dim3((unsigned)cdiv(K, 32), (unsigned)cdiv(M, 64)), dim3(256), 0, st>>>(
            X, XT, (int)M, (int)K, p.ldm);
        DwArgs w;
        w.GT = p.GT;
        w.XT = XT;
        w.dW = dW;
        w.M = (int)M;
        w.N = (int)N;
        w.K = (int)K;
        w.ldm = p.ldm;
        w.accumulate = (flags & MQ_FLAG_ACCUM_DW) ? 1 : 0;
        const DwPlan plan = dw_plan(M, N, K);
        w.tiles_n = plan.tiles_n;
        w.tiles_k = plan.tiles_k;
        w.whole = plan.whole;
        w.parts = plan.parts;
        w.part = reinterpret_cast<float *>(base + lay.dwp);
        if (!allow_lds(dw_kernel, DW_LDS)) return MQ_ERR_DEVICE;
        dw_kernel<<<dim3(plan.whole + plan.rest * plan.parts), dim3(256), DW_LDS, st>>>(w);
        if (plan.rest > 0) dw_reduce_kernel<<<dim3(plan.rest * (DW_BN / 16)), dim3(256), 0, st>>>(w);
    }
    return launch_status();
}
}  // namespace mq

extern "C" mq_status mq_linear_bwd(const uint16_t *X, const uint8_t *Q, const float *alpha, const float *zero,
                                   const uint16_t *const *dY, const float *lambda, int64_t M, int64_t N,
                                   int64_t K, const int *rs, int nr, uint32_t flags, uint16_t *dX, float *dW,
                                   void *ws, size_t ws_bytes, void *hip_stream) {
    return mq::bwd_run(false, X, Q, alpha, zero, dY, nullptr, nullptr, lambda, M, N, K, rs, nr, flags, dX, dW, ws, ws_bytes,
                       hip_stream);
}

extern "C" mq_status mq_linear_bwd_gated(const uint16_t *X, const uint8_t *Q, const float *alpha, const float *zero,
                                         const uint16_t *const *GU, const uint16_t *const *dA, const float *lambda,
                                         int64_t M, int64_t F, int64_t K, const int *rs, int nr, uint32_t flags,
                                         uint16_t *dX, float *dW, void *ws, size_t ws_bytes, void *hip_stream) {
    if (F < 0 || F > (1 << 21)) return MQ_ERR_SHAPE;
    return mq::bwd_run(true, X, Q, alpha, zero, nullptr, GU, dA, lambda, M, 2 * F, K, rs, nr, flags, dX, dW, ws, ws_bytes,
                       hip_stream);
}

extern "C" const char *mq_status_string(mq_status status) {
    switch (status) {
        case MQ_OK: return "ok";
        case MQ_ERR_NULL: return "null pointer";
        case MQ_ERR_SHAPE: return "bad shape";
        case MQ_ERR_BITS: return "bad bit-width";
        case MQ_ERR_ALIGN: return "bad alignment";
        case MQ_ERR_WORKSPACE: return "workspace too small";
        case MQ_ERR_CAPACITY: return "overflow list capacity exceeded";
        case MQ_ERR_DEVICE: return "device error";
    }
    return "unknown status";
}
