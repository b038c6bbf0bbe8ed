// C ABI of the library: argument checks on the host, then kernel dispatch.
// Nothing here allocates, frees or synchronizes.
#include "../../include/flexq.h"
#include "flexq_kernels.h"

#include "api_internal.h"

// The library keeps no mutable state: every choice below is a function of the call's
// arguments (and, in the development build only, of the Tuning passed with the call).

namespace {

using flexq::Tuning;

constexpr int kMaxRowBlocks = FLEXQ_WORKSPACE_COUNTER_BYTES / 4;
constexpr int kSkinnyMaxM = 128;

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

flexq_status check_shape(int N, int K, int group)
{
    if (N < 1 || K < 1) return FLEXQ_EINVAL;
    if (group != 0 && group != 128) return FLEXQ_EINVAL;
    if (N % 32 != 0 || K % 128 != 0 || K > FLEXQ_MAX_K || N / 32 > kMaxRowBlocks) return FLEXQ_ESHAPE;
    return FLEXQ_OK;
}

size_t scale_count(int N, int K, int group) { return group == 0 ? (size_t)N : (size_t)N * (K / 128); }

// K splits of the streaming kernel.  Measured on MI355X: one workgroup of
// eight wavefronts per 32-row block streams fastest as soon as there are enough
// of them for half the CUs (at N = 4096, 128 blocks unsplit beat 256 split ones:
// the cross-workgroup hand-off costs more than the idle CUs); splitting K
// further only adds hand-offs.  So split just enough to reach 128 workgroups,
// keep at least two tiles per wavefront, and keep the partial-sum traffic (8 bytes
// per split, token and column) under a ninth of the weight stream.
int choose_split(int M, int N, int K, int forced = 0)
{
    const int kt = K / 128;
    int ks;
    if (forced > 0) {
        ks = forced;
    } else {
        const int row_blocks = N / 32;
        ks = (128 + row_blocks - 1) / row_blocks;
        const int by_traffic = (int)((long)K / (96L * M));
        if (ks > by_traffic) ks = by_traffic;
        if (ks > kt / 16) ks = kt / 16;
    }
    if (ks > kt) ks = kt;
    if (ks > 64) ks = 64;
    if (ks < 1) ks = 1;
    return ks;
}

// K splits of the tiled kernel for mid-size M: with fewer than one 128x128 output
// tile per CU the blocks are long latency chains on a mostly idle chip, so K is
// split until there is about one block per CU (measured optimum on MI355X: 4 splits
// at M = 128, 2 at M = 256), keeping at least four 128-k stages per block and the
// partial-sum traffic (8 bytes per split and output) under the weight bytes.
int choose_gemm_split(int M, int N, int K, int forced = 0)
{
    const int kt = K / 128;
    int ks;
    if (forced > 0) {
        ks = forced;
    } else {
        const long tiles = (long)((M + 127) / 128) * ((N + 127) / 128);
        // about one block per CU; two per CU once there are several row tiles and K is
        // long enough for the partial sums to stay a small share of the traffic
        // (measured: 28672-deep down projection at 256 and 512 tokens)
        const long target = (K >= 16384 && tiles >= 128) ? 512 : 256;
        if (tiles >= target) return 1;
        ks = (int)(target / tiles);
        if (ks > kt / 4) ks = kt / 4;
        const int by_traffic = K / (11 * M);
        if (ks > by_traffic) ks = by_traffic;
        if (ks > 16) ks = 16;
    }
    if (ks > kt) ks = kt;
    return ks < 1 ? 1 : ks;
}

// Wavefronts per workgroup of the streaming kernel.
int choose_waves(int M, int N, int K, int ks, int forced = 0)
{
    if (forced > 0) return forced;
    const int tiles = K / 128 / ks;
    // few row blocks and long rows (the 7B / 13B down projections at one to four tokens):
    // sixteen wavefronts per workgroup keep more of the chip streaming (measured: 10-20 %)
    if (M <= 4 && (long)(N / 32) * ks < 256 && tiles >= 64) return 16;
    // between one and two workgroups per CU (LLaMA-2-70B's 10240-wide QKV: 320 row blocks)
    // workgroups of eight wavefronts run in one and a quarter rounds; from 16 tokens on,
    // where a workgroup's time is long enough to matter, four wavefronts per workgroup let
    // every row block start at once (measured: 19 vs 21 us at 16 tokens, 26 vs 27 at 32)
    const long wgs = (long)(N / 32) * ks;
    if (M >= 16 && wgs > 256 && wgs < 512 && tiles >= 16) return 4;
    // wide layers with short rows at one to four tokens (the gate+up projections of
    // LLaMA-2-7B and 13B: 688 and 864 row blocks of 32 and 40 tiles): with four wavefronts
    // per workgroup every row block is resident from the start (measured at 640 to 1792
    // row blocks: 13-20 % faster up to 32 tiles per row at one to four tokens, 17-20 % at
    // 40 to 56 tiles at one token, 3 % at four; no gain from 64 tiles on or from 8 tokens)
    if (wgs >= 640 && ((tiles <= 32 && M <= 4) || (tiles < 64 && M <= 2))) return 4;
    return tiles >= 16 ? 8 : 4;
}

struct Workspace {
    unsigned *counters;
    int8_t *xq;
    uint16_t *sx;
    void *partial;
    size_t partial_capacity;  // bytes
};

// quantized activations of the prologue: row-major, or (up to 32 tokens) one block of tiles
size_t xq_bytes(int M, int K) { return round_up((size_t)(M < 32 ? 32 : M) * K, 256); }

size_t fixed_bytes(int M, int K)
{
    return FLEXQ_WORKSPACE_COUNTER_BYTES + xq_bytes(M, K) + round_up((size_t)M * 2, 256);
}

size_t act_tiles_bytes(int act_bits, int M, int K)
{
    return (size_t)((M + 31) / 32) * (K / 128) * (act_bits == 6 ? 3072 : 4096);
}

Workspace carve(void *ws, size_t bytes, int M, int K)
{
    Workspace w;
    uint8_t *p = (uint8_t *)ws;
    w.counters = (unsigned *)p;
    p += FLEXQ_WORKSPACE_COUNTER_BYTES;
    w.xq = (int8_t *)p;
    p += xq_bytes(M, K);
    w.sx = (uint16_t *)p;
    p += round_up((size_t)M * 2, 256);
    w.partial = p;
    w.partial_capacity = bytes - fixed_bytes(M, K);
    return w;
}

size_t workspace_bytes_for(int M, int N, int K)
{
    if (M < 1 || check_shape(N, K, 0) != FLEXQ_OK) return 0;
    size_t partial = 0;
    const int top = M < kSkinnyMaxM ? M : kSkinnyMaxM;
    for (int m = 1; m <= top; ++m) {
        const int ks = choose_split(m, N, K);
        const size_t b = ks > 1 ? (size_t)ks * m * N * 4 : 0;
        if (b > partial) partial = b;
    }
    {
        const int gs = choose_gemm_split(M, N, K);
        const size_t b = gs > 1 ? (size_t)gs * M * N * 4 : 0;
        if (b > partial) partial = b;
    }
    if (const int pieces = flexq::low_cut_pieces(M, N, K); pieces != 0) {   // 128x256 tiles cut along K
        const size_t b = flexq::low_cut_bytes((N + 255) / 256 * pieces);
        if (b > partial) partial = b;
    }
    if (M > kSkinnyMaxM) {   // the 256x256 kernel's tail cut along K
        const size_t b = flexq::streamk_plan(M, N, K).partial_bytes;
        if (b > partial) partial = b;
    }
    return fixed_bytes(M, K) + round_up(partial, 256);
}

}  // namespace

namespace flexq {

namespace {

// the tiled kernel addresses both operands with 32-bit buffer offsets
bool tiled_addressable(int M, int N, int K)
{
    return (long)(M + 256) * K < (1L << 32) && (long)N * K / 4 * 3 < (1L << 32);
}

// Measured cross-over between the streaming kernel and the tiled kernel with K splits:
// the streaming kernel re-reads the activations once per 32 output channels (and past
// 32 tokens needs a second MFMA row tile), while the tiled kernel's time stays flat up
// to 128 tokens but carries the fixed cost of its K splits on small layers.  So: up to
// 32 tokens stream (24 on very wide layers unless the activations are, or can be written
// as, packed 6-bit tiles: the 57344-wide gate+up at 25 to 32 tokens takes 73 us tiled,
// 77-91 us streaming from row-major codes, 72-75 us from 8-bit tiles and 67-69 us from
// packed 6-bit tiles), up to 64 on layers of at most 2^25 weights (2^26 with group-wise
// scales, which have no 64-row tile), up to 128 on layers of at most 2^24 (LLaMA-2-7B's
// 4096 x 4096: 24 vs 31 us at 128 tokens).
bool streams_by_choice(int M, int N, int K, int group, bool packed_tiles = false)
{
    const long weights = (long)N * K;
    return M <= 24 || (M <= 32 && (N < 32768 || packed_tiles)) ||
           (M <= 64 && weights <= (group == 0 ? (1L << 25) : (1L << 26))) ||
           (M <= 128 && weights <= (1L << 24)) || (M <= 64 && !tiled_addressable(M, N, K));
}

// Seventeen to 32 tokens (24 to 32 for 8-bit activations) whose slice of the activations
// does not fit the streaming kernel's LDS staging: the quantizer writes them in tile
// order (6-bit activations packed like the weights), which the kernel reads with
// coalesced loads instead of a scattered 128-byte line per token and k-step.  A tile
// always carries 32 token rows, so the time no longer depends on the token count
// (measured on the LLaMA-2-70B layers, quantize + GEMV from fp16: 25 / 19 / 46 us on
// qkv / o / down for any count up to 32, against 30 / 21 / 52 us row-major at 32 tokens
// and 23 / 17 / 38 us at 16).
bool tiles_pay(int act_bits, int M, int K, int split_k)
{
    return M <= 32 && M >= (act_bits == 6 ? 17 : 24) && !flexq::skinny_slice_fits(M, K, split_k);
}

}  // namespace

bool linear_wants_tiles(int act_bits, int M, int N, int K, int group)
{
    return streams_by_choice(M, N, K, group, act_bits == 6) && tiles_pay(act_bits, M, K, choose_split(M, N, K));
}

flexq_status linear_check(const void *packed, int group, const int8_t *xq, const uint16_t *sx,
                          const uint16_t *x_fp16, int M, int N, int K, const uint16_t *y,
                          const int32_t *acc_out, const void *workspace, size_t workspace_bytes,
                          const uint16_t *sxg, int sxg_stride)
{
    if (!packed || !y || M < 1) return FLEXQ_EINVAL;
    if (sxg) {   // scales per token and group: pre-quantized activations, group-128 weights
        if (!xq || x_fp16 || acc_out || group != 128 || sxg_stride < M) return FLEXQ_EINVAL;
    } else if (!x_fp16 && (!xq || !sx)) {
        return FLEXQ_EINVAL;
    }
    flexq_status s = check_shape(N, K, group);
    if (s != FLEXQ_OK) return s;
    if (group != 0 && acc_out) return FLEXQ_EINVAL;
    if (!aligned16(packed) || !aligned16(y) || (acc_out && !aligned16(acc_out)) ||
        (x_fp16 && !aligned16(x_fp16)) || (!x_fp16 && !aligned16(xq)))
        return FLEXQ_EALIGN;
    if (!workspace || workspace_bytes < workspace_bytes_for(M, N, K)) return FLEXQ_EWORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return FLEXQ_EALIGN;
    return FLEXQ_OK;
}

flexq_status linear_impl(const Tuning &tune, int act_bits, const void *packed, int group,
                         const int8_t *xq, const uint16_t *sx, const uint16_t *x_fp16, int M, int N, int K,
                         uint16_t *y, int32_t *acc_out, void *workspace, size_t workspace_bytes,
                         void *stream, const uint16_t *sxg, int sxg_stride, int *dispatched, int xt)
{
    if (dispatched) *dispatched = 0;
    if (xt != 0 && (xt != act_bits || M > 32 || sxg || x_fp16)) return FLEXQ_EINVAL;
    if (flexq_status s = linear_check(packed, group, xq, sx, x_fp16, M, N, K, y, acc_out, workspace,
                                      workspace_bytes, sxg, sxg_stride);
        s != FLEXQ_OK)
        return s;

    hipStream_t st = (hipStream_t)stream;
    Workspace ws = carve(workspace, workspace_bytes, M, K);

    const int forced = tune.kernel;
    const bool tiled_ok = tiled_addressable(M, N, K);
    // fp16 activations at 6 bits can be written as packed tiles, which the streaming kernel
    // reads fastest
    const bool may_tile = x_fp16 && !sxg && tune.tiles != 2 && tune.ablate == 0;
    bool stream_kernel = streams_by_choice(M, N, K, group, may_tile && act_bits == 6);
    // group-wise activation scales reach the tiled kernel by 4-byte DMA loads: even stride
    if (sxg && (sxg_stride % 2 != 0 || !tiled_ok)) stream_kernel = true;
    if (forced == 1) stream_kernel = true;
    if (forced == 2) stream_kernel = false;
    if (xt != 0) stream_kernel = true;

    // Single-token decode: the streaming kernel quantizes the activations itself.  (Each
    // workgroup then scans the token's whole fp16 row, which pays off while a CU runs only
    // a few workgroups -- measured break-even near 1024 workgroups -- and for one token
    // only: over the four LLaMA-2-70B layers the fused form takes 120 us against 122 us for
    // quantize launch + GEMV at one token, but 132 against 125 at two and 157 against 131
    // at eight.  The kernel can do up to eight; tune.fuse = 1 asks for that.)
    const int ks0 = choose_split(M, N, K, tune.split_k);
    const bool fuse = x_fp16 && stream_kernel && tune.fuse != 2 && flexq::skinny_can_fuse(M, K, ks0) &&
                      (tune.fuse == 1 || (M == 1 && (long)(N / 32) * ks0 <= 1024));
    if (may_tile && !fuse && stream_kernel && M <= 32 && (tune.tiles == 1 || tiles_pay(act_bits, M, K, ks0)))
        xt = act_bits;
    if (x_fp16 && !fuse) {
        if (flexq::launch_quant_act(x_fp16, M, K, act_bits, ws.xq, ws.sx, st, xt) != hipSuccess)
            return FLEXQ_EHIP;
        xq = ws.xq;
        sx = ws.sx;
    }

    flexq::LinearArgs a;
    a.packed = packed;
    a.scales = (const uint16_t *)((const uint8_t *)packed + (size_t)N * K * 6 / 8);
    a.N = N;
    a.K = K;
    a.group = group;
    a.counters = ws.counters;
    a.partial = ws.partial;
    a.partial_bytes = ws.partial_capacity;
    a.x_fp16 = fuse ? x_fp16 : nullptr;
    a.qmax = act_bits == 6 ? 31.0f : 127.0f;
    a.sxg = nullptr;
    a.sxg_stride = sxg_stride;
    a.ablate = tune.ablate;
    a.xt = xt;
    if (tune.spin != 0) a.spin = tune.spin < 0 ? 0 : tune.spin;

    if (!stream_kernel) {
        // the tiled kernel addresses both operands with 32-bit buffer offsets
        if (!tiled_ok) return FLEXQ_ESHAPE;
        a.xq = xq;
        a.sx = sx;
        a.sxg = sxg;
        a.M = M;
        a.y = y;
        a.acc_out = acc_out;
        a.split_k = choose_gemm_split(M, N, K, tune.split_k);
        const size_t per_split = (size_t)M * N * 4;
        if ((size_t)a.split_k * per_split > ws.partial_capacity)
            a.split_k = (int)(ws.partial_capacity / per_split);
        if ((size_t)a.split_k * per_split >= ((size_t)1 << 32)) a.split_k = 1;   // 32-bit buffer offsets
        if (a.split_k < 2) a.split_k = 1;
        int cfg = tune.gemm_cfg;
        const int kt_max = K / 128;
        if (cfg == 0 && tune.split_k > 0 && a.split_k > 1) cfg = 8;   // a forced split is honoured
        // (13: a forced split is the number of pieces per cut tile; the bounds above do not apply)
        if (cfg == 13 || cfg == 16) a.split_k = tune.split_k > 1 ? (tune.split_k < kt_max ? tune.split_k : kt_max) : 1;
        int chosen = 0, tail_runs = 0;
        const hipError_t e = flexq::launch_gemm(a, cfg, st, &chosen, &tail_runs);
        if (dispatched) *dispatched = chosen * 1000 + (chosen >= 13 ? tail_runs : a.split_k);
        return e == hipSuccess ? FLEXQ_OK : FLEXQ_EHIP;
    }
    for (int m0 = 0; m0 < M; m0 += kSkinnyMaxM) {
        const int rows = M - m0 < kSkinnyMaxM ? M - m0 : kSkinnyMaxM;
        a.xq = xq + (size_t)m0 * K;
        a.sx = sx ? sx + m0 : nullptr;
        a.sxg = sxg ? sxg + m0 : nullptr;
        a.M = rows;
        a.y = y + (size_t)m0 * N;
        a.acc_out = acc_out ? acc_out + (size_t)m0 * N : nullptr;
        a.split_k = choose_split(rows, N, K, tune.split_k);
        // never outgrow the partial-sum area the caller provided
        const size_t per_split = (size_t)rows * N * 4;
        if ((size_t)a.split_k * per_split > ws.partial_capacity)
            a.split_k = (int)(ws.partial_capacity / per_split);
        if (a.split_k < 1) a.split_k = 1;
        if (flexq::launch_skinny(a, choose_waves(rows, N, K, a.split_k, tune.waves), st) != hipSuccess)
            return FLEXQ_EHIP;
        if (dispatched) *dispatched = 1000 + a.split_k + (xt != 0 ? 500 : 0);
    }
    return FLEXQ_OK;
}

}  // namespace flexq

namespace {

const flexq::Tuning kAuto{};

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

const char *flexq_status_string(flexq_status s)
{
    switch (s) {
    case FLEXQ_OK: return "ok";
    case FLEXQ_EINVAL: return "invalid argument";
    case FLEXQ_ESHAPE: return "unsupported shape (need N % 32 == 0, K % 128 == 0, K <= 65536)";
    case FLEXQ_EALIGN: return "pointer not sufficiently aligned";
    case FLEXQ_EHIP: return "HIP runtime error";
    case FLEXQ_EWORKSPACE: return "workspace missing or too small";
    default: return "unknown status";
    }
}

int flexq_layout_version(void) { return 1; }

size_t flexq_packed_bytes(int N, int K, int group)
{
    if (check_shape(N, K, group) != FLEXQ_OK) return 0;
    return round_up((size_t)N * K * 6 / 8 + 2 * scale_count(N, K, group), 256);
}

flexq_status flexq_quant_w6(const float *w, int N, int K, int group, int8_t *wq, uint16_t *sw,
                            void *stream)
{
    if (!w || !wq || !sw) return FLEXQ_EINVAL;
    flexq_status s = check_shape(N, K, group);
    if (s != FLEXQ_OK) return s;
    return flexq::launch_quant_w6(w, N, K, group, wq, sw, (hipStream_t)stream) == hipSuccess
               ? FLEXQ_OK
               : FLEXQ_EHIP;
}

flexq_status flexq_pack_w6(const int8_t *wq, const uint16_t *sw, int N, int K, int group,
                           void *packed, void *stream)
{
    if (!wq || !sw || !packed) return FLEXQ_EINVAL;
    flexq_status s = check_shape(N, K, group);
    if (s != FLEXQ_OK) return s;
    if (!aligned16(wq) || !aligned16(packed)) return FLEXQ_EALIGN;
    return flexq::launch_pack_w6(wq, sw, N, K, group, packed, (hipStream_t)stream) == hipSuccess
               ? FLEXQ_OK
               : FLEXQ_EHIP;
}

flexq_status flexq_unpack_w6(const void *packed, int N, int K, int group, int8_t *wq, uint16_t *sw,
                             void *stream)
{
    if (!wq || !sw || !packed) return FLEXQ_EINVAL;
    flexq_status s = check_shape(N, K, group);
    if (s != FLEXQ_OK) return s;
    if (!aligned16(wq) || !aligned16(packed)) return FLEXQ_EALIGN;
    return flexq::launch_unpack_w6(packed, N, K, group, wq, sw, (hipStream_t)stream) == hipSuccess
               ? FLEXQ_OK
               : FLEXQ_EHIP;
}

flexq_status flexq_quant_act(const uint16_t *x, int M, int K, int act_bits, int8_t *xq, uint16_t *sx,
                             void *stream)
{
    if (!x || !xq || !sx || M < 1) return FLEXQ_EINVAL;
    if (act_bits != 6 && act_bits != 8) return FLEXQ_EINVAL;
    if (K < 1) return FLEXQ_EINVAL;
    if (K % 128 != 0 || K > FLEXQ_MAX_K) return FLEXQ_ESHAPE;
    if (!aligned16(x) || !aligned16(xq)) return FLEXQ_EALIGN;
    return flexq::launch_quant_act(x, M, K, act_bits, xq, sx, (hipStream_t)stream) == hipSuccess
               ? FLEXQ_OK
               : FLEXQ_EHIP;
}

size_t flexq_act_tiles_bytes(int act_bits, int M, int K)
{
    if ((act_bits != 6 && act_bits != 8) || M < 1 || K < 1 || K % 128 != 0 || K > FLEXQ_MAX_K) return 0;
    return act_tiles_bytes(act_bits, M, K);
}

flexq_status flexq_quant_act_tiles(const uint16_t *x, int M, int K, int act_bits, void *xt, uint16_t *sx,
                                   void *stream)
{
    if (!x || !xt || !sx || M < 1 || K < 1) return FLEXQ_EINVAL;
    if (act_bits != 6 && act_bits != 8) return FLEXQ_EINVAL;
    if (K % 128 != 0 || K > FLEXQ_MAX_K) return FLEXQ_ESHAPE;
    if (!aligned16(x) || !aligned16(xt)) return FLEXQ_EALIGN;
    return flexq::launch_quant_act(x, M, K, act_bits, (int8_t *)xt, sx, (hipStream_t)stream, act_bits) ==
                   hipSuccess
               ? FLEXQ_OK
               : FLEXQ_EHIP;
}

flexq_status flexq_untile_act(const void *xt, int M, int K, int act_bits, int8_t *xq, void *stream)
{
    if (!xt || !xq || M < 1 || K < 1) return FLEXQ_EINVAL;
    if (act_bits != 6 && act_bits != 8) return FLEXQ_EINVAL;
    if (K % 128 != 0 || K > FLEXQ_MAX_K) return FLEXQ_ESHAPE;
    if (!aligned16(xt) || !aligned16(xq)) return FLEXQ_EALIGN;
    return flexq::launch_untile_act((const uint8_t *)xt, act_bits, M, K, xq, (hipStream_t)stream) == hipSuccess
               ? FLEXQ_OK
               : FLEXQ_EHIP;
}

flexq_status flexq_gemv_tiles(int act_bits, const void *packed, int group, const void *xt,
                              const uint16_t *sx, int M, int N, int K, uint16_t *y, int32_t *acc_out,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    if (act_bits != 6 && act_bits != 8) return FLEXQ_EINVAL;
    if (M > 32) return FLEXQ_EINVAL;
    return flexq::linear_impl(kAuto, act_bits, packed, group, (const int8_t *)xt, sx, nullptr, M, N, K, y,
                              acc_out, workspace, workspace_bytes, stream, nullptr, 0, nullptr, act_bits);
}

flexq_status flexq_rmsnorm_quant(const uint16_t *x, const uint16_t *gamma, float eps, int M, int K,
                                 int act_bits, int8_t *xq, uint16_t *sx, uint16_t *h_out,
                                 void *stream)
{
    if (!x || !gamma || !xq || !sx || M < 1 || K < 1) return FLEXQ_EINVAL;
    if (act_bits != 6 && act_bits != 8) return FLEXQ_EINVAL;
    if (!(eps > 0.0f)) return FLEXQ_EINVAL;
    if (K % 128 != 0 || K > FLEXQ_MAX_K) return FLEXQ_ESHAPE;
    if (!aligned16(x) || !aligned16(gamma) || !aligned16(xq) || (h_out && !aligned16(h_out)))
        return FLEXQ_EALIGN;
    return flexq::launch_rmsnorm_quant(x, gamma, eps, M, K, act_bits, xq, sx, h_out,
                                       (hipStream_t)stream) == hipSuccess
               ? FLEXQ_OK
               : FLEXQ_EHIP;
}

flexq_status flexq_swiglu_quant(const uint16_t *gate_up, int M, int F, int act_bits, int8_t *xq,
                                uint16_t *sx, uint16_t *h_out, void *stream)
{
    if (!gate_up || !xq || !sx || M < 1 || F < 1) return FLEXQ_EINVAL;
    if (act_bits != 6 && act_bits != 8) return FLEXQ_EINVAL;
    if (F % 128 != 0 || F > FLEXQ_MAX_K) return FLEXQ_ESHAPE;
    if (!aligned16(gate_up) || !aligned16(xq) || (h_out && !aligned16(h_out))) return FLEXQ_EALIGN;
    return flexq::launch_swiglu_quant(gate_up, M, F, act_bits, xq, sx, h_out,
                                      (hipStream_t)stream) == hipSuccess
               ? FLEXQ_OK
               : FLEXQ_EHIP;
}

flexq_status flexq_quant_act_g128(const uint16_t *x, int M, int K, int act_bits, int8_t *xq,
                                  uint16_t *sxg, int sxg_stride, void *stream)
{
    if (!x || !xq || !sxg || M < 1 || K < 1 || sxg_stride < M) return FLEXQ_EINVAL;
    if (act_bits != 6 && act_bits != 8) return FLEXQ_EINVAL;
    if (K % 128 != 0 || K > FLEXQ_MAX_K) return FLEXQ_ESHAPE;
    if (!aligned16(x) || !aligned16(xq)) return FLEXQ_EALIGN;
    return flexq::launch_quant_act_g128(x, M, K, act_bits, xq, sxg, sxg_stride,
                                        (hipStream_t)stream) == hipSuccess
               ? FLEXQ_OK
               : FLEXQ_EHIP;
}

flexq_status flexq_linear_g128(const void *packed, const int8_t *xq, const uint16_t *sxg,
                               int sxg_stride, int M, int N, int K, uint16_t *y, void *workspace,
                               size_t workspace_bytes, void *stream)
{
    if (!sxg) return FLEXQ_EINVAL;
    return flexq::linear_impl(kAuto, 8, packed, 128, xq, nullptr, nullptr, M, N, K, y, nullptr, workspace,
                              workspace_bytes, stream, sxg, sxg_stride, nullptr);
}

size_t flexq_workspace_bytes(int M, int N, int K) { return workspace_bytes_for(M, N, K); }

flexq_status flexq_workspace_init(void *workspace, size_t workspace_bytes, void *stream)
{
    if (!workspace) return FLEXQ_EINVAL;
    if (workspace_bytes < FLEXQ_WORKSPACE_COUNTER_BYTES) return FLEXQ_EWORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return FLEXQ_EALIGN;
    return flexq::launch_fill_zero(workspace, FLEXQ_WORKSPACE_COUNTER_BYTES, (hipStream_t)stream) ==
                   hipSuccess
               ? FLEXQ_OK
               : FLEXQ_EHIP;
}

flexq_status flexq_gemm_w6a6(const void *packed, int group, const int8_t *xq, const uint16_t *sx,
                             const uint16_t *x_fp16, int M, int N, int K, uint16_t *y,
                             int32_t *acc_out, void *workspace, size_t workspace_bytes, void *stream)
{
    return flexq::linear_impl(kAuto, 6, packed, group, xq, sx, x_fp16, M, N, K, y, acc_out, workspace,
                              workspace_bytes, stream, nullptr, 0, nullptr);
}

flexq_status flexq_gemm_w6a8(const void *packed, int group, const int8_t *xq, const uint16_t *sx,
                             const uint16_t *x_fp16, int M, int N, int K, uint16_t *y,
                             int32_t *acc_out, void *workspace, size_t workspace_bytes, void *stream)
{
    return flexq::linear_impl(kAuto, 8, packed, group, xq, sx, x_fp16, M, N, K, y, acc_out, workspace,
                              workspace_bytes, stream, nullptr, 0, nullptr);
}

flexq_status flexq_gemv_w6a6(const void *packed, int group, const int8_t *xq, const uint16_t *sx,
                             const uint16_t *x_fp16, int M, int N, int K, uint16_t *y,
                             int32_t *acc_out, void *workspace, size_t workspace_bytes, void *stream)
{
    return flexq::linear_impl(kAuto, 6, packed, group, xq, sx, x_fp16, M, N, K, y, acc_out, workspace,
                              workspace_bytes, stream, nullptr, 0, nullptr);
}

flexq_status flexq_gemv_w6a8(const void *packed, int group, const int8_t *xq, const uint16_t *sx,
                             const uint16_t *x_fp16, int M, int N, int K, uint16_t *y,
                             int32_t *acc_out, void *workspace, size_t workspace_bytes, void *stream)
{
    return flexq::linear_impl(kAuto, 8, packed, group, xq, sx, x_fp16, M, N, K, y, acc_out, workspace,
                              workspace_bytes, stream, nullptr, 0, nullptr);
}

}  // extern "C"
#pragma GCC visibility pop
