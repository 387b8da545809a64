// mq_ffn_mixnmatch: a stack of gated feed-forward layers on the decode path, every layer at its own
// bit-width (layer-wise Mix'n'Match, section 4.3 and appendix B).  A layer is two launches of the
// decode GEMV: the gate and up rows are one plane with the rows of a pair next to each other, so both
// products come out of a single pass over the activations and meet in the epilogue, which applies the
// gate activation; the epilogue of the down product adds the residual.  (As separate element-wise
// kernels the two small operations cost about a quarter of a layer's time at batch 1.)
#include "mq_gemv.h"

namespace mq {

namespace {

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct FfnLayout {
    size_t act, h0, h1, total;
};
inline FfnLayout ffn_layout(int64_t B, int64_t F, int64_t d) {
    FfnLayout l;
    size_t off = 0;
    l.act = off, off += align256((size_t)B * F * 2);
    l.h0 = off, off += align256((size_t)B * d * 2);
    l.h1 = off, off += align256((size_t)B * d * 2);
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
                             residual ? h : nullptr, hip_stream);
        if (s != MQ_OK) return s;
        h = hn;
    }
    return MQ_OK;
}
