// mq_ffn_mixnmatch: a stack of gated feed-forward layers on the decode path, every layer at its own
// bit-width (layer-wise Mix'n'Match, section 4.3 and appendix B).  A layer is two launches of the
// decode GEMV: the gate and up rows are one plane with the rows of a pair next to each other, so both
// products come out of a single pass over the activations and meet in the epilogue, which applies the
// gate activation; the epilogue of the down product adds the residual.  (As separate element-wise
// kernels the two small operations cost about a quarter of a layer's time at batch 1.)
#include <algorithm>

#include "mq_gemv.h"

namespace mq {

namespace {

// ---- the gate on the training path: [M, 2F] outputs of the stacked gate / up projection, the columns of a
// pair next to each other, for up to three bit-widths in one launch (HBM-bound: 6 bytes per gated element
// forward, 10 backward) ----
struct GateArgs {
    const uint16_t *GU[3];
    const uint16_t *dA[3];
    uint16_t *out[3];  // forward: A [M, F]; backward: dGU [M, 2F]
    int64_t chunks;    // chunks of 8 gated elements per tensor
    int nr, silu;
};

template <bool BWD>
__global__ __launch_bounds__(256) void gate_train_kernel(GateArgs a) {
    const int64_t ch = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (ch >= a.chunks) return;
    for (int i = 0; i < a.nr; ++i) {
        const u32x4 p0 = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.GU[i]) + 2 * ch);
        const u32x4 p1 = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.GU[i]) + 2 * ch + 1);
        const uint32_t pairs[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};  // (gate, up) per dword
        if constexpr (!BWD) {
            u32x4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float g0 = bf16_lo(pairs[2 * j]), u0 = bf16_hi(pairs[2 * j]);
                const float g1 = bf16_lo(pairs[2 * j + 1]), u1 = bf16_hi(pairs[2 * j + 1]);
                o[j] = pack_bf16x2((a.silu ? silu(g0) : gelu_tanh(g0)) * u0, (a.silu ? silu(g1) : gelu_tanh(g1)) * u1);
            }
            reinterpret_cast<u32x4 *>(a.out[i])[ch] = o;
        } else {
            const u32x4 d = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.dA[i]) + ch);
            uint32_t o[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float g = bf16_lo(pairs[j]), u = bf16_hi(pairs[j]);
                const float da = (j & 1) ? bf16_hi(d[j >> 1]) : bf16_lo(d[j >> 1]);
                o[j] = gated_pair_grad(g, u, da, a.silu != 0);
            }
            reinterpret_cast<u32x4 *>(a.out[i])[2 * ch] = u32x4{o[0], o[1], o[2], o[3]};
            reinterpret_cast<u32x4 *>(a.out[i])[2 * ch + 1] = u32x4{o[4], o[5], o[6], o[7]};
        }
    }
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct FfnLayout {
    size_t act, h0, h1, split, split_bytes, total;
};
inline FfnLayout ffn_layout(int64_t B, int64_t F, int64_t d) {
    FfnLayout l;
    size_t off = 0;
    l.act = off, off += align256((size_t)B * F * 2);
    l.h0 = off, off += align256((size_t)B * d * 2);
    l.h1 = off, off += align256((size_t)B * d * 2);
    // parts of the down product when its K (= F) is split over workgroups
    l.split_bytes = std::max(gemv_split_workspace_bytes(B, d, F, 4), gemv_split_workspace_bytes(B, d, F, 2));
    l.split = off, off += align256(l.split_bytes);
    l.total = off;
    return l;
}

}  // namespace

size_t ffn_workspace_bytes(int64_t B, int64_t F, int64_t d) {
    if (B < 1 || B > 16 || F < 1 || d < 1) return 0;
    return ffn_layout(B, F, d).total + 256;
}

}  // namespace mq

extern "C" mq_status mq_ffn_mixnmatch(const uint16_t *x, const mq_ffn_layer *layers, int n_layers, int64_t B, int64_t d,
                                      int64_t F, uint32_t flags, uint16_t *y, void *ws, size_t ws_bytes,
                                      void *hip_stream) {
    using namespace mq;
    if (n_layers < 0 || B < 1 || B > 16 || d < 1 || F < 1 || d > 0x3FFFFFF0 || F > 0x3FFFFFF0) return MQ_ERR_SHAPE;
    if (F % 8 != 0 || d % 8 != 0) return MQ_ERR_ALIGN;
    if (!x || !y || (n_layers > 0 && !layers)) return MQ_ERR_NULL;
    if (x == y) return MQ_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(y)) return MQ_ERR_ALIGN;
    for (int l = 0; l < n_layers; ++l) {
        const mq_ffn_layer &L = layers[l];
        if (L.r != 8 && L.r != 6 && L.r != 4 && L.r != 3 && L.r != 2) return MQ_ERR_BITS;
        if (!L.gate_up || !L.down || !L.alpha_gu || !L.zero_gu || !L.alpha_dn || !L.zero_dn) return MQ_ERR_NULL;
        // both products of the layer are checked now, so that no layer is enqueued when a later one is refused
        mq_status s = gemv_sliced_check(L.gate_up, B, 2 * F, d, L.r, kPostGelu);
        if (s == MQ_OK) s = gemv_sliced_check(L.down, B, d, F, L.r, kPostNone);
        if (s != MQ_OK) return s;
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (n_layers == 0) {
        if (hipMemcpyAsync(y, x, (size_t)B * d * 2, hipMemcpyDeviceToDevice, st) != hipSuccess) return MQ_ERR_DEVICE;
        return MQ_OK;
    }
    const FfnLayout lay = ffn_layout(B, F, d);
    if (!ws || ws_bytes < lay.total + 256) return MQ_ERR_WORKSPACE;
    uint8_t *base = reinterpret_cast<uint8_t *>((reinterpret_cast<uintptr_t>(ws) + 255) & ~(uintptr_t)255);
    uint16_t *act = reinterpret_cast<uint16_t *>(base + lay.act);
    uint16_t *hbuf[2] = {reinterpret_cast<uint16_t *>(base + lay.h0), reinterpret_cast<uint16_t *>(base + lay.h1)};
    const bool residual = (flags & MQ_FLAG_FFN_RESIDUAL) != 0, use_silu = (flags & MQ_FLAG_FFN_SILU) != 0;

    const uint16_t *h = x;
    for (int l = 0; l < n_layers; ++l) {
        const mq_ffn_layer &L = layers[l];
        const bool last = l + 1 == n_layers;
        uint16_t *hn = last ? y : hbuf[l & 1];  // (never the buffer h lives in)
        mq_status s = gemv_sliced_post(h, L.gate_up, L.alpha_gu, L.zero_gu, B, 2 * F, d, L.r, act,
                                       use_silu ? kPostSilu : kPostGelu, nullptr, hip_stream);
        if (s != MQ_OK) return s;
        s = gemv_sliced_post(act, L.down, L.alpha_dn, L.zero_dn, B, d, F, L.r, hn, residual ? kPostResidual : kPostNone,
                             residual ? h : nullptr, hip_stream, lay.split_bytes ? base + lay.split : nullptr, lay.split_bytes);
        if (s != MQ_OK) return s;
        h = hn;
    }
    return MQ_OK;
}

static mq_status gated_unit(const uint16_t *const *GU, const uint16_t *const *dA, int nr, int64_t M, int64_t F,
                            uint32_t flags, uint16_t *const *out, bool bwd, void *hip_stream) {
    using namespace mq;
    if (nr < 1 || nr > 3) return MQ_ERR_BITS;
    if (M < 0 || F < 1 || F > 0x3FFFFFF0 || (M > 0 && F > (int64_t)0x3FFFFFFFFFFFll / M)) return MQ_ERR_SHAPE;
    if (F % 8 != 0) return MQ_ERR_ALIGN;
    if (M == 0) return MQ_OK;
    if (!GU || !out || (bwd && !dA)) return MQ_ERR_NULL;
    GateArgs a{};
    for (int i = 0; i < nr; ++i) {
        if (!GU[i] || !out[i] || (bwd && !dA[i])) return MQ_ERR_NULL;
        if (!aligned16(GU[i]) || !aligned16(out[i]) || (bwd && !aligned16(dA[i]))) return MQ_ERR_ALIGN;
        a.GU[i] = GU[i];
        a.dA[i] = bwd ? dA[i] : nullptr;
        a.out[i] = out[i];
    }
    a.chunks = M * F / 8;
    a.nr = nr;
    a.silu = (flags & MQ_FLAG_FFN_SILU) ? 1 : 0;
    const int64_t blocks = cdiv(a.chunks, 256);
    if (blocks > 0x7FFFFFFF) return MQ_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (bwd)
        gate_train_kernel<true><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(a);
    else
        gate_train_kernel<false><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(a);
    return launch_status();
}

extern "C" mq_status mq_gated_unit_fwd(const uint16_t *const *GU, int nr, int64_t M, int64_t F, uint32_t flags,
                                       uint16_t *const *A, void *hip_stream) {
    return gated_unit(GU, nullptr, nr, M, F, flags, A, false, hip_stream);
}

extern "C" mq_status mq_gated_unit_bwd(const uint16_t *const *GU, const uint16_t *const *dA, int nr, int64_t M, int64_t F,
                                       uint32_t flags, uint16_t *const *dGU, void *hip_stream) {
    return gated_unit(GU, dA, nr, M, F, flags, dGU, true, hip_stream);
}

