// The linear layers of one decoder block as one call: each GEMM fed by the operator that
// produces its input with the activation quantizer fused in (paper Section 4.1.3), the
// activation width chosen per linear (Section 4.1.2: 8 bits for the down projection,
// 6 bits elsewhere).  Host code only: it strings together the library's own launches.
#include "api_internal.h"
#include "flexq_kernels.h"

namespace {

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool bits_ok(int b) { return b == 6 || b == 8; }

struct Carve {
    int8_t *xq;      // [M, max(H, F)] codes of the stage being fed
    uint16_t *sx;    // [M]
    void *gemm;      // workspace of the GEMM calls (counter area first)
    size_t gemm_bytes;
};

size_t gemm_ws_bytes(const flexq_layer *L, int M)
{
    size_t need = 0;
    const int shapes[4][2] = {{L->QKV, L->H}, {L->H, L->H}, {2 * L->F, L->H}, {L->H, L->F}};
    for (const auto &s : shapes) {
        const size_t b = flexq_workspace_bytes(M, s[0], s[1]);
        if (b == 0) return 0;
        if (b > need) need = b;
    }
    return need;
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

size_t flexq_layer_workspace_bytes(const flexq_layer *L, int M)
{
    if (!L || M < 1 || L->H < 1 || L->F < 1 || L->QKV < 1) return 0;
    const size_t g = gemm_ws_bytes(L, M);
    if (g == 0) return 0;
    const int widest = L->H > L->F ? L->H : L->F;
    // (fewer than 32 tokens: room for one block of 32-token tiles)
    return g + round_up((size_t)(M < 32 ? 32 : M) * widest, 256) + round_up((size_t)M * 2, 256);
}

flexq_status flexq_layer_linears(const flexq_layer *L, int M, const flexq_layer_io *io, int first_stage,
                                 int last_stage, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!L || !io || M < 1) return FLEXQ_EINVAL;
    if (first_stage < 0 || last_stage > 3 || first_stage > last_stage) return FLEXQ_EINVAL;
    if (L->H < 1 || L->F < 1 || L->QKV < 1 || (L->group != 0 && L->group != 128) || !(L->eps > 0.0f))
        return FLEXQ_EINVAL;
    if (!bits_ok(L->bits_qkv) || !bits_ok(L->bits_o) || !bits_ok(L->bits_gate_up) || !bits_ok(L->bits_down))
        return FLEXQ_EINVAL;
    const size_t need = flexq_layer_workspace_bytes(L, M);
    if (need == 0) return FLEXQ_ESHAPE;
    // everything a stage in [first_stage, last_stage] touches is checked before any launch
    for (int s = first_stage; s <= last_stage; ++s) {
        const void *w = s == 0 ? L->w_qkv : s == 1 ? L->w_o : s == 2 ? L->w_gate_up : L->w_down;
        const void *in = s == 0 ? (const void *)io->x : s == 1 ? (const void *)io->attn
                       : s == 2 ? (const void *)io->x_ffn : (const void *)io->gate_up;
        const void *out = s == 0 ? (void *)io->qkv : s == 1 ? (void *)io->o : s == 2 ? (void *)io->gate_up
                                                                                     : (void *)io->down;
        const void *gamma = s == 0 ? L->gamma_attn : s == 2 ? L->gamma_ffn : (const void *)w;
        const void *h = s == 0 ? io->h_attn_norm : s == 2 ? io->h_ffn_norm : s == 3 ? io->h_swiglu : nullptr;
        if (!w || !in || !out || !gamma) return FLEXQ_EINVAL;
        if (!aligned16(w) || !aligned16(in) || !aligned16(out) || !aligned16(gamma) || (h && !aligned16(h)))
            return FLEXQ_EALIGN;
    }
    if (!workspace || workspace_bytes < need) return FLEXQ_EWORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return FLEXQ_EALIGN;

    Carve c;
    c.gemm_bytes = gemm_ws_bytes(L, M);
    c.gemm = workspace;                                       // its counter area leads the workspace
    uint8_t *p = (uint8_t *)workspace + c.gemm_bytes;
    const int widest = L->H > L->F ? L->H : L->F;
    c.xq = (int8_t *)p;
    c.sx = (uint16_t *)(p + round_up((size_t)(M < 32 ? 32 : M) * widest, 256));

    hipStream_t st = (hipStream_t)stream;
    const flexq::Tuning automatic{};
    auto gemm = [&](int bits, const void *w, const int8_t *xq, const uint16_t *sx, const uint16_t *x_fp16,
                    int N, int K, uint16_t *y, int xt) {
        return flexq::linear_impl(automatic, bits, w, L->group, xq, sx, x_fp16, M, N, K, y, nullptr, c.gemm,
                                  c.gemm_bytes, stream, nullptr, 0, nullptr, xt);
    };
    // batches of 17 to 32 tokens: the producers write their codes in tile order (packed at
    // 6 bits) where the streaming kernel reads them faster that way
    auto layout = [&](int bits, int N, int K) {
        return flexq::linear_wants_tiles(bits, M, N, K, L->group) ? bits : 0;
    };
    for (int s = first_stage; s <= last_stage; ++s) {
        flexq_status r = FLEXQ_OK;
        if (s == 0) {            // RMS norm + quantize -> fused QKV
            const int lay = layout(L->bits_qkv, L->QKV, L->H);
            if (flexq::launch_rmsnorm_quant(io->x, L->gamma_attn, L->eps, M, L->H, L->bits_qkv, c.xq, c.sx,
                                            io->h_attn_norm, st, lay) != hipSuccess)
                return FLEXQ_EHIP;
            r = gemm(L->bits_qkv, L->w_qkv, c.xq, c.sx, nullptr, L->QKV, L->H, io->qkv, lay);
        } else if (s == 1) {     // quantize node -> attention output projection (fp16 in: decode
                                 // batches quantize inside the streaming kernel)
            r = gemm(L->bits_o, L->w_o, nullptr, nullptr, io->attn, L->H, L->H, io->o, 0);
        } else if (s == 2) {     // RMS norm + quantize -> fused gate | up
            const int lay = layout(L->bits_gate_up, 2 * L->F, L->H);
            if (flexq::launch_rmsnorm_quant(io->x_ffn, L->gamma_ffn, L->eps, M, L->H, L->bits_gate_up, c.xq,
                                            c.sx, io->h_ffn_norm, st, lay) != hipSuccess)
                return FLEXQ_EHIP;
            r = gemm(L->bits_gate_up, L->w_gate_up, c.xq, c.sx, nullptr, 2 * L->F, L->H, io->gate_up, lay);
        } else {                 // SiLU(gate) * up + quantize -> down projection
            const int lay = layout(L->bits_down, L->H, L->F);
            if (flexq::launch_swiglu_quant(io->gate_up, M, L->F, L->bits_down, c.xq, c.sx, io->h_swiglu, st,
                                           lay) != hipSuccess)
                return FLEXQ_EHIP;
            r = gemm(L->bits_down, L->w_down, c.xq, c.sx, nullptr, L->H, L->F, io->down, lay);
        }
        if (r != FLEXQ_OK) return r;
    }
    return FLEXQ_OK;
}

}  // extern "C"
#pragma GCC visibility pop
