// C ABI of the NestedFP library: argument validation, workspace layout and dispatch to
// the streaming (decode) or tiled (prefill) kernel family.  See include/nestedfp.h for
// the contract of every entry point.
#include "../../include/nestedfp.h"
#include "nfp_host.h"

#include <string.h>

namespace nfp {

Tuning &tuning() {
    static Tuning t = {-1, -1, -1, -1, -1, -1, -1, -1, -1, -1, 1, -1};
    return t;
}

bool use_small_gemm(int64_t M) {
    int64_t lim = tuning().small_max_m >= 0 ? tuning().small_max_m : 64;
    if (lim > 64) lim = 64;
    return M <= lim;
}

static inline bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
static inline size_t round256(size_t b) { return (b + 255) & ~(size_t)255; }

// workspace layout: [Xq : M*K bytes][scales : M floats][split-K partials]
struct Workspace {
    uint8_t *xq;
    float *scales;
    float *partials;
    size_t partial_bytes;
};

static bool route_small(int kind, int64_t M, int64_t N, int64_t K, int64_t ldw) {
    if (!use_small_gemm(M) || !small_gemm_supports(kind, M, N, K, ldw)) return false;
    // measured: with three or four token tiles per wave the streaming kernel falls behind the
    // tiled NestedFP kernel (whose weights bypass LDS) on the widest layers (gate/up projections)
    if (kind == kNestedF16 && M > 32 && N >= 16384 && tuning().small_max_m < 0) return false;
    // and from 49 tokens on everywhere but on the smallest layers (64-token tiles, split along K)
    if (kind == kNestedF16 && M > 48 && (N > 4096 || K > 4096) && tuning().small_max_m < 0) return false;
    // the plain FP16 kernels: the same from 49 tokens on, and from 33 on where both N and K are large
    if (kind == kPlainF16 && tuning().small_max_m < 0 &&
        ((M > 48 && (N > 4096 || K > 4096)) || (M > 32 && N >= 8192 && K >= 8192))) return false;
    // E4M3 weights: where the layer is large enough for the 64-token tiles to pay, from 33 tokens on
    // on the widest layers, from 49 on those with a long K
    if (kind == kE4M3 && tuning().small_max_m < 0 && ((M > 32 && N >= 16384) || (M > 48 && K >= 14336))) return false;
    return true;
}

static size_t partial_bytes_for(int kind, int64_t M, int64_t N, int64_t K) {
    return route_small(kind, M, N, K, K) ? small_gemm_partial_bytes(kind, M, N, K)
                                   : large_gemm_partial_bytes(kind, M, N, K);
}

static size_t workspace_bytes_for(int kind, int64_t M, int64_t N, int64_t K, bool quantize) {
    size_t b = round256(partial_bytes_for(kind, M, N, K));
    if (quantize) b += round256((size_t)M * (size_t)K) + round256((size_t)M * sizeof(float));
    return b;
}

static bool carve(void *ws, size_t ws_bytes, int kind, int64_t M, int64_t N, int64_t K, bool quantize,
                  Workspace &out) {
    size_t need = workspace_bytes_for(kind, M, N, K, quantize);
    if (need > 0 && (ws == nullptr || ws_bytes < need || !aligned(ws, 16))) return false;
    uint8_t *p = static_cast<uint8_t *>(ws);
    out.xq = nullptr;
    out.scales = nullptr;
    if (quantize) {
        out.xq = p;  p += round256((size_t)M * (size_t)K);
        out.scales = reinterpret_cast<float *>(p);  p += round256((size_t)M * sizeof(float));
    }
    out.partials = reinterpret_cast<float *>(p);
    out.partial_bytes = partial_bytes_for(kind, M, N, K);
    return true;
}

static int check_mat(const void *ptr, int64_t rows, int64_t cols, int64_t ld, int64_t ld_mult) {
    if (ptr == nullptr || rows < 0 || cols < 0) return kErrArg;
    if (ld < cols || (ld % ld_mult) != 0 || !aligned(ptr, 16)) return kErrShape;
    return kOk;
}

static int run_gemm(int kind, const GemmArgs &a, hipStream_t stream) {
    return route_small(kind, a.M, a.N, a.K, a.ldw) ? launch_small_gemm(kind, a, stream)
                                       : launch_large_gemm(kind, a, stream);
}

static int check_dims(int64_t M, int64_t N, int64_t K) {
    if (M < 0 || N < 0 || K <= 0) return kErrArg;
    if ((K % 16) != 0) return kErrShape;
    if (M > 0x3fffffff || N > 0x3fffffff || K > 0x3fffffff) return kErrShape;
    return kOk;
}

static int check_out(const uint16_t *Y, int64_t N, int64_t ldy) {
    if (Y == nullptr) return kErrArg;
    if (ldy < N || !aligned(Y, 2)) return kErrShape;
    return kOk;
}

// FP8-mode GEMM straight from FP16 activations where the streaming kernel can quantise them
// itself (decode batches whose K fits one workgroup pass); returns -1 if it cannot.
static int fp8_gemm_fused(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const float *act_scale,
                          const uint8_t *Wq, int64_t N, float w_scale, uint16_t *Y, int64_t ldy,
                          hipStream_t stream) {
    if (!route_small(kE4M3, M, N, K, K) || !small_gemm_fuses_quant(M, N, K)) return -1;
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.X = X;  a.ldx = ldx;  a.static_scale = act_scale;  a.w_scale = w_scale;
    a.W0 = Wq;  a.W1 = nullptr;  a.ldw = K;
    a.M = M;  a.N = N;  a.K = K;  a.Y = Y;  a.ldy = ldy;
    return launch_small_gemm(kE4M3Quant, a, stream);
}

static int fp8_gemm(const uint8_t *Xq, const float *scales, int64_t M, int64_t K, const uint8_t *Wq,
                    int64_t N, float w_scale, uint16_t *Y, int64_t ldy, float *partials,
                    size_t partial_bytes, hipStream_t stream) {
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.X = Xq;  a.ldx = K;  a.scales = scales;  a.w_scale = w_scale;
    a.W0 = Wq;  a.W1 = nullptr;  a.ldw = K;
    a.M = M;  a.N = N;  a.K = K;  a.Y = Y;  a.ldy = ldy;
    a.partials = partials;  a.partial_bytes = partial_bytes;
    return run_gemm(kE4M3, a, stream);
}

}  // namespace nfp

using namespace nfp;

extern "C" {

int nestedfp_version(void) { return 200; }

const char *nestedfp_status_string(int status) {
    switch (status) {
        case NESTEDFP_OK: return "ok";
        case NESTEDFP_ERR_ARG: return "invalid argument (NULL pointer, negative size or unknown mode)";
        case NESTEDFP_ERR_SHAPE: return "unsupported shape (K % 16, leading dimension or alignment)";
        case NESTEDFP_ERR_RANGE: return "weights outside the NestedFP range (|w| > 1.75, Inf or NaN)";
        case NESTEDFP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case NESTEDFP_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

static int finish_count(uint64_t *dev, uint64_t *host, hipStream_t stream) {
    if (host == nullptr) return NESTEDFP_OK;
    if (hipMemcpyAsync(host, dev, sizeof(uint64_t), hipMemcpyDeviceToHost, stream) != hipSuccess)
        return NESTEDFP_ERR_HIP;
    if (hipStreamSynchronize(stream) != hipSuccess) return NESTEDFP_ERR_HIP;
    return *host == 0 ? NESTEDFP_OK : NESTEDFP_ERR_RANGE;
}

int nestedfp_range_check(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint64_t *out_of_range,
                         uint64_t *out_of_range_host, void *stream) {
    if (out_of_range == nullptr) return NESTEDFP_ERR_ARG;
    int st = check_dims(0, N, K);
    if (st != kOk) return st;
    st = check_mat(W, N, K, ldw, 8);
    if (st != kOk) return st;
    if (!aligned(out_of_range, 8)) return NESTEDFP_ERR_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = launch_range_check(W, N, K, ldw, out_of_range, s);
    if (st != kOk) return st;
    return finish_count(out_of_range, out_of_range_host, s);
}

int nestedfp_decompose(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint8_t *upper,
                       uint8_t *lower, uint64_t *out_of_range, uint64_t *out_of_range_host,
                       void *stream) {
    if (out_of_range_host != nullptr && out_of_range == nullptr) return NESTEDFP_ERR_ARG;
    int st = check_dims(0, N, K);
    if (st != kOk) return st;
    if (N == 0) {                                     // empty layer: nothing to read or write
        hipStream_t s0 = static_cast<hipStream_t>(stream);
        if (out_of_range && launch_zero_u64(out_of_range, s0) != kOk) return NESTEDFP_ERR_HIP;
        return finish_count(out_of_range, out_of_range_host, s0);
    }
    if (upper == nullptr || lower == nullptr) return NESTEDFP_ERR_ARG;
    st = check_mat(W, N, K, ldw, 8);
    if (st != kOk) return st;
    if (!aligned(upper, 16) || !aligned(lower, 16)) return NESTEDFP_ERR_SHAPE;
    if (out_of_range && !aligned(out_of_range, 8)) return NESTEDFP_ERR_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = launch_decompose(W, N, K, ldw, upper, lower, out_of_range, s);
    if (st != kOk) return st;
    return finish_count(out_of_range, out_of_range_host, s);
}

int nestedfp_reconstruct(const uint8_t *upper, const uint8_t *lower, int64_t N, int64_t K, uint16_t *W,
                         int64_t ldw, void *stream) {
    int st = check_dims(0, N, K);
    if (st != kOk) return st;
    if (N == 0) return NESTEDFP_OK;
    if (upper == nullptr || lower == nullptr) return NESTEDFP_ERR_ARG;
    st = check_mat(W, N, K, ldw, 8);
    if (st != kOk) return st;
    if (!aligned(upper, 16) || !aligned(lower, 16)) return NESTEDFP_ERR_SHAPE;
    return launch_reconstruct(upper, lower, N, K, W, ldw, static_cast<hipStream_t>(stream));
}

size_t nestedfp_plane_bytes(int64_t N, int64_t K) {
    if (check_dims(0, N, K) != kOk) return 0;
    return plane_bytes(N, K);
}

int nestedfp_pack_plane(const uint8_t *src, int64_t N, int64_t K, int64_t ld, uint8_t *dst, void *stream) {
    int st = check_dims(0, N, K);
    if (st != kOk) return st;
    if (N == 0) return NESTEDFP_OK;
    if (src == nullptr || dst == nullptr) return NESTEDFP_ERR_ARG;
    if (ld < K || (ld & 15) != 0 || !aligned(src, 16) || !aligned(dst, 16)) return NESTEDFP_ERR_SHAPE;
    return launch_pack_plane(src, N, K, ld, dst, static_cast<hipStream_t>(stream));
}

int nestedfp_unpack_plane(const uint8_t *src, int64_t N, int64_t K, uint8_t *dst, int64_t ld, void *stream) {
    int st = check_dims(0, N, K);
    if (st != kOk) return st;
    if (N == 0) return NESTEDFP_OK;
    if (src == nullptr || dst == nullptr) return NESTEDFP_ERR_ARG;
    if (ld < K || (ld & 15) != 0 || !aligned(src, 16) || !aligned(dst, 16)) return NESTEDFP_ERR_SHAPE;
    return launch_unpack_plane(src, N, K, dst, ld, static_cast<hipStream_t>(stream));
}

int nestedfp_quantize_act(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const float *static_scale,
                          uint8_t *Xq, float *scales, void *stream) {
    if (Xq == nullptr || scales == nullptr) return NESTEDFP_ERR_ARG;
    int st = check_dims(M, 0, K);
    if (st != kOk) return st;
    st = check_mat(X, M, K, ldx, 8);
    if (st != kOk) return st;
    if (!aligned(Xq, 16) || !aligned(scales, 4)) return NESTEDFP_ERR_SHAPE;
    if (M == 0) return NESTEDFP_OK;
    return launch_quantize_act(X, M, K, ldx, static_scale, Xq, scales, static_cast<hipStream_t>(stream));
}

size_t nestedfp_gemm_workspace_size(int64_t M, int64_t N, int64_t K, int mode) {
    if (check_dims(M, N, K) != kOk) return 0;
    if (mode != NESTEDFP_MODE_FP16 && mode != NESTEDFP_MODE_FP8) return 0;
    if (M == 0 || N == 0) return 0;
    if (mode == NESTEDFP_MODE_FP16) {
        // the plain baseline takes the same query; its launch shape may differ from the nested one
        const size_t a = workspace_bytes_for(kNestedF16, M, N, K, false), b = workspace_bytes_for(kPlainF16, M, N, K, false);
        return a > b ? a : b;
    }
    return workspace_bytes_for(kE4M3, M, N, K, true);
}

int nestedfp_gemm(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const uint8_t *upper,
                  const uint8_t *lower, int64_t N, int mode, const float *act_scale, uint16_t *Y,
                  int64_t ldy, void *workspace, size_t workspace_bytes, void *stream) {
    if (mode != NESTEDFP_MODE_FP16 && mode != NESTEDFP_MODE_FP8) return NESTEDFP_ERR_ARG;
    int st = check_dims(M, N, K);
    if (st != kOk) return st;
    if (M == 0 || N == 0) return NESTEDFP_OK;         // nothing to read or write: no pointer is looked at
    if (upper == nullptr) return NESTEDFP_ERR_ARG;
    if (mode == NESTEDFP_MODE_FP16 && lower == nullptr) return NESTEDFP_ERR_ARG;
    st = check_mat(X, M, K, ldx, 8);
    if (st != kOk) return st;
    st = check_out(Y, N, ldy);
    if (st != kOk) return st;
    if (!aligned(upper, 16) || (mode == NESTEDFP_MODE_FP16 && !aligned(lower, 16))) return NESTEDFP_ERR_SHAPE;
    if (M == 0 || N == 0) return NESTEDFP_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Workspace ws;
    if (mode == NESTEDFP_MODE_FP16) {
        if (!carve(workspace, workspace_bytes, kNestedF16, M, N, K, false, ws)) return NESTEDFP_ERR_WORKSPACE;
        GemmArgs a;
        memset(&a, 0, sizeof(a));
        a.X = X;  a.ldx = ldx;  a.W0 = upper;  a.W1 = lower;  a.ldw = K;
        a.M = M;  a.N = N;  a.K = K;  a.Y = Y;  a.ldy = ldy;
        a.partials = ws.partials;  a.partial_bytes = ws.partial_bytes;
        return run_gemm(kNestedF16, a, s);
    }
    if (!carve(workspace, workspace_bytes, kE4M3, M, N, K, true, ws)) return NESTEDFP_ERR_WORKSPACE;
    // Sec. 4.1: the upper plane read as E4M3 is the weight times 2^8
    st = fp8_gemm_fused(X, M, K, ldx, act_scale, upper, N, 0.00390625f, Y, ldy, s);
    if (st >= 0) return st;
    st = launch_quantize_act(X, M, K, ldx, act_scale, ws.xq, ws.scales, s);
    if (st != kOk) return st;
    return fp8_gemm(ws.xq, ws.scales, M, K, upper, N, 0.00390625f, Y, ldy, ws.partials, ws.partial_bytes, s);
}

int nestedfp_plain_gemm_fp16(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const uint16_t *W,
                             int64_t N, int64_t ldw, uint16_t *Y, int64_t ldy, void *workspace,
                             size_t workspace_bytes, void *stream) {
    int st = check_dims(M, N, K);
    if (st != kOk) return st;
    if (M == 0 || N == 0) return NESTEDFP_OK;
    st = check_mat(X, M, K, ldx, 8);
    if (st != kOk) return st;
    st = check_mat(W, N, K, ldw, 8);
    if (st != kOk) return st;
    st = check_out(Y, N, ldy);
    if (st != kOk) return st;
    if (M == 0 || N == 0) return NESTEDFP_OK;
    Workspace ws;
    if (!carve(workspace, workspace_bytes, kPlainF16, M, N, K, false, ws)) return NESTEDFP_ERR_WORKSPACE;
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.X = X;  a.ldx = ldx;  a.W0 = W;  a.W1 = nullptr;  a.ldw = ldw;
    a.M = M;  a.N = N;  a.K = K;  a.Y = Y;  a.ldy = ldy;
    a.partials = ws.partials;  a.partial_bytes = ws.partial_bytes;
    return run_gemm(kPlainF16, a, static_cast<hipStream_t>(stream));
}

int nestedfp_plain_gemm_fp8(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const uint8_t *Wq,
                            int64_t N, float w_scale, const float *act_scale, uint16_t *Y, int64_t ldy,
                            void *workspace, size_t workspace_bytes, void *stream) {
    int st = check_dims(M, N, K);
    if (st != kOk) return st;
    if (M == 0 || N == 0) return NESTEDFP_OK;
    if (Wq == nullptr) return NESTEDFP_ERR_ARG;
    st = check_mat(X, M, K, ldx, 8);
    if (st != kOk) return st;
    st = check_out(Y, N, ldy);
    if (st != kOk) return st;
    if (!aligned(Wq, 16)) return NESTEDFP_ERR_SHAPE;
    if (M == 0 || N == 0) return NESTEDFP_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Workspace ws;
    if (!carve(workspace, workspace_bytes, kE4M3, M, N, K, true, ws)) return NESTEDFP_ERR_WORKSPACE;
    st = fp8_gemm_fused(X, M, K, ldx, act_scale, Wq, N, w_scale, Y, ldy, s);
    if (st >= 0) return st;
    st = launch_quantize_act(X, M, K, ldx, act_scale, ws.xq, ws.scales, s);
    if (st != kOk) return st;
    return fp8_gemm(ws.xq, ws.scales, M, K, Wq, N, w_scale, Y, ldy, ws.partials, ws.partial_bytes, s);
}

int nestedfp_gemm_fp8_prequantized(const uint8_t *Xq, const float *scales, int64_t M, int64_t K,
                                   const uint8_t *upper, int64_t N, float w_scale, uint16_t *Y,
                                   int64_t ldy, void *workspace, size_t workspace_bytes, void *stream) {
    int st = check_dims(M, N, K);
    if (st != kOk) return st;
    if (M == 0 || N == 0) return NESTEDFP_OK;
    if (Xq == nullptr || scales == nullptr || upper == nullptr) return NESTEDFP_ERR_ARG;
    st = check_out(Y, N, ldy);
    if (st != kOk) return st;
    if (!aligned(Xq, 16) || !aligned(upper, 16) || !aligned(scales, 4)) return NESTEDFP_ERR_SHAPE;
    if (M == 0 || N == 0) return NESTEDFP_OK;
    Workspace ws;
    if (!carve(workspace, workspace_bytes, kE4M3, M, N, K, false, ws)) return NESTEDFP_ERR_WORKSPACE;
    return fp8_gemm(Xq, scales, M, K, upper, N, w_scale, Y, ldy, ws.partials, ws.partial_bytes,
                    static_cast<hipStream_t>(stream));
}

int nestedfp_layer_prepare(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint8_t *upper,
                           uint8_t *lower, uint64_t *out_of_range, nestedfp_layer *layer_host, void *stream) {
    if (layer_host == nullptr || out_of_range == nullptr) return NESTEDFP_ERR_ARG;
    uint64_t count = 0;
    int st = nestedfp_decompose(W, N, K, ldw, upper, lower, out_of_range, &count, stream);
    if (st != NESTEDFP_OK && st != NESTEDFP_ERR_RANGE) return st;
    memset(layer_host, 0, sizeof(*layer_host));
    layer_host->N = N;
    layer_host->K = K;
    layer_host->out_of_range = count;
    if (st == NESTEDFP_ERR_RANGE) {
        layer_host->is_exception = 1;
        layer_host->W = W;
        layer_host->ldw = ldw;
    } else {
        layer_host->upper = upper;
        layer_host->lower = lower;
    }
    return NESTEDFP_OK;
}

size_t nestedfp_linear_workspace_size(int64_t M, const nestedfp_layer *layer_host, int mode) {
    if (layer_host == nullptr) return 0;
    if (layer_host->is_exception) mode = NESTEDFP_MODE_FP16;
    return nestedfp_gemm_workspace_size(M, layer_host->N, layer_host->K, mode);
}

int nestedfp_linear(const uint16_t *X, int64_t M, int64_t ldx, const nestedfp_layer *layer_host, int mode,
                    const float *act_scale, uint16_t *Y, int64_t ldy, void *workspace,
                    size_t workspace_bytes, void *stream) {
    if (layer_host == nullptr) return NESTEDFP_ERR_ARG;
    if (mode != NESTEDFP_MODE_FP16 && mode != NESTEDFP_MODE_FP8) return NESTEDFP_ERR_ARG;
    const nestedfp_layer &L = *layer_host;
    if (L.is_exception)
        return nestedfp_plain_gemm_fp16(X, M, L.K, ldx, L.W, L.N, L.ldw, Y, ldy, workspace, workspace_bytes, stream);
    return nestedfp_gemm(X, M, L.K, ldx, L.upper, L.lower, L.N, mode, act_scale, Y, ldy, workspace,
                         workspace_bytes, stream);
}

static const char *const kKnobs[] = {"small_max_m", "small_split", "small_spw", "small_tiles", "small_interleave",
                                     "large_split", "large_bm", "large_bn", "large_epilogue", "small_fuse_quant", "quant_hw", "large_xcd_map",
                                     nullptr};

const char *nestedfp_tune_name(int index) {
    if (index < 0 || index >= (int)(sizeof(kKnobs) / sizeof(kKnobs[0]))) return nullptr;
    return kKnobs[index];
}

int nestedfp_tune(const char *knob, int64_t value) {
    if (knob == nullptr) return NESTEDFP_ERR_ARG;
    Tuning &t = tuning();
    if (value < 0) value = -1;
    if (!strcmp(knob, "small_max_m")) t.small_max_m = value;
    else if (!strcmp(knob, "small_split")) t.small_split = value;
    else if (!strcmp(knob, "small_spw")) t.small_spw = value;
    else if (!strcmp(knob, "small_tiles")) t.small_tiles = value;
    else if (!strcmp(knob, "small_interleave")) t.small_interleave = value;
    else if (!strcmp(knob, "large_split")) t.large_split = value;
    else if (!strcmp(knob, "large_bm")) t.large_bm = value;
    else if (!strcmp(knob, "large_bn")) t.large_bn = value;
    else if (!strcmp(knob, "large_epilogue")) t.large_epilogue = value;
    else if (!strcmp(knob, "small_fuse_quant")) t.small_fuse_quant = value;
    else if (!strcmp(knob, "quant_hw")) t.quant_hw = value < 0 ? 1 : value;
    else if (!strcmp(knob, "large_xcd_map")) t.large_xcd_map = value;
    else return NESTEDFP_ERR_ARG;
    return NESTEDFP_OK;
}

}  // extern "C"
