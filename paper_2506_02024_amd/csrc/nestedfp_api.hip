// C ABI of the NestedFP library: argument validation, workspace layout and dispatch to
// the streaming (decode) or tiled (prefill) kernel family.  See include/nestedfp.h for
// the contract of every entry point.
#include "../../include/nestedfp.h"
#include "nfp_host.h"

#include <string.h>

#include <mutex>

namespace nfp {

Tuning &tuning() {
    static Tuning t = {-1, -1, -1, -1, -1, -1, -1, -1, -1, -1, 1, -1, -1, -1, -1, -1};
    return t;
}

bool use_small_gemm(int64_t M) {
    int64_t lim = tuning().small_max_m >= 0 ? tuning().small_max_m : 64;
    if (lim > 64) lim = 64;
    return M <= lim;
}

static inline bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
static inline size_t round256(size_t b) { return (b + 255) & ~(size_t)255; }

constexpr int64_t kMaxK = (int64_t)1 << 21;            // K and leading dimensions: 256 rows stay below 2^31 bytes

// workspace layout: [arrival counters : kCounterBytes][Xq : M*K bytes][scales : M floats][split-K partials]
struct Workspace {
    uint32_t *counters;
    uint8_t *xq;
    float *scales;
    float *partials;
    size_t partial_bytes;
};

static bool route_small(int kind, int64_t M, int64_t N, int64_t K, int64_t ldw) {
    if (!use_small_gemm(M) || !small_gemm_supports(kind, M, N, K, ldw)) return false;
    if (tuning().small_max_m >= 0) return true;
    const int cls = kind_class(kind);
    // Timed on the 18 layer shapes of the paper's five models at 12 ... 64 tokens, all three classes:
    // with three or four token tiles per wave (33 tokens and more) the streaming kernel is behind
    // the 64-token tiles of the tiled kernels (split along K) on every shape, by 9-97 %;
    if (M > 32) return false;
    // with two token tiles (17 ... 32 tokens) it is behind by 5-30 % except on the smallest layers
    // (and, for plain row-major FP16 weights, on layers of 4096 rows); up to 16 tokens it stays
    const int64_t weights = N * K;
    if (M > 16) {
        if (cls == 1 && weights >= ((int64_t)20 << 20)) return false;
        if (cls == 2 && weights >= ((int64_t)50 << 20)) return false;
        if (cls == 0 && N >= 5120) return false;
    }
    return true;
}

static size_t partial_bytes_for(int kind, int64_t M, int64_t N, int64_t K) {
    return route_small(kind, M, N, K, K) ? small_gemm_partial_bytes(kind, M, N, K)
                                   : large_gemm_partial_bytes(kind, M, N, K);
}

static size_t workspace_bytes_for(int kind, int64_t M, int64_t N, int64_t K, bool quantize) {
    size_t b = round256(partial_bytes_for(kind, M, N, K));
    if (quantize) b += round256((size_t)M * (size_t)K) + round256((size_t)M * sizeof(float));
    return b > 0 ? b + kCounterBytes : 0;
}

static bool carve(void *ws, size_t ws_bytes, int kind, int64_t M, int64_t N, int64_t K, bool quantize,
                  Workspace &out) {
    size_t need = workspace_bytes_for(kind, M, N, K, quantize);
    if (need > 0 && (ws == nullptr || ws_bytes < need || !aligned(ws, 16))) return false;
    out.counters = nullptr;
    out.xq = nullptr;
    out.scales = nullptr;
    out.partials = nullptr;
    out.partial_bytes = 0;
    if (need == 0) return true;
    uint8_t *p = static_cast<uint8_t *>(ws);
    out.counters = reinterpret_cast<uint32_t *>(p);  p += kCounterBytes;
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
    if (ld < cols || ld > kMaxK || (ld % ld_mult) != 0 || !aligned(ptr, 16)) return kErrShape;
    return kOk;
}

static int run_gemm(int kind, const GemmArgs &a, hipStream_t stream) {
    return route_small(kind, a.M, a.N, a.K, a.ldw) ? launch_small_gemm(kind, a, stream)
                                       : launch_large_gemm(kind, a, stream);
}

static int check_dims(int64_t M, int64_t N, int64_t K) {
    if (M < 0 || N < 0 || K <= 0) return kErrArg;
    if ((K % 16) != 0) return kErrShape;
    if (M > 0x3fffffff || N > 0x3fffffff || K > kMaxK) return kErrShape;
    return kOk;
}

static int check_out(const uint16_t *Y, int64_t N, int64_t ldy) {
    if (Y == nullptr) return kErrArg;
    if (ldy < N || !aligned(Y, 2)) return kErrShape;
    return kOk;
}

static bool valid_mode(int mode) { return mode == NESTEDFP_MODE_FP16 || mode == NESTEDFP_MODE_FP8; }
static bool valid_layout(int layout) { return layout == NESTEDFP_LAYOUT_ROWMAJOR || layout == NESTEDFP_LAYOUT_PACKED; }

// FP8-mode GEMM straight from FP16 activations where the streaming kernel can quantise them
// itself (decode batches whose K fits one workgroup pass, packed planes); returns -1 if it cannot.
static int fp8_gemm_fused(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const float *act_scale,
                          const uint8_t *Wq, int64_t N, int w_kind, float w_scale, uint16_t *Y, int64_t ldy,
                          hipStream_t stream) {
    if (w_kind != kE4M3 || !route_small(kE4M3, M, N, K, K) || !small_gemm_fuses_quant(M, N, K)) return -1;
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.X = X;  a.ldx = ldx;  a.static_scale = act_scale;  a.w_scale = w_scale;
    a.W0 = Wq;  a.W1 = nullptr;  a.ldw = K;
    a.M = M;  a.N = N;  a.K = K;  a.Y = Y;  a.ldy = ldy;
    return launch_small_gemm(kE4M3Quant, a, stream);
}

static int fp8_gemm(const uint8_t *Xq, const float *scales, int64_t M, int64_t K, const uint8_t *Wq,
                    int64_t N, int w_kind, float w_scale, uint16_t *Y, int64_t ldy, const Workspace &ws,
                    hipStream_t stream) {
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.X = Xq;  a.ldx = K;  a.scales = scales;  a.w_scale = w_scale;
    a.W0 = Wq;  a.W1 = nullptr;  a.ldw = K;
    a.M = M;  a.N = N;  a.K = K;  a.Y = Y;  a.ldy = ldy;
    a.partials = ws.partials;  a.partial_bytes = ws.partial_bytes;  a.counters = ws.counters;
    return run_gemm(w_kind, a, stream);
}

static int finish_count(uint64_t *dev, uint64_t *host, hipStream_t stream) {
    if (host == nullptr) return NESTEDFP_OK;
    if (hipMemcpyAsync(host, dev, sizeof(uint64_t), hipMemcpyDeviceToHost, stream) != hipSuccess)
        return NESTEDFP_ERR_HIP;
    if (hipStreamSynchronize(stream) != hipSuccess) return NESTEDFP_ERR_HIP;
    return *host == 0 ? NESTEDFP_OK : NESTEDFP_ERR_RANGE;
}

static int decompose_impl(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint8_t *upper, uint8_t *lower,
                          uint64_t *out_of_range, uint64_t *out_of_range_host, bool packed, void *stream) {
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
    st = launch_decompose(W, N, K, ldw, upper, lower, out_of_range, packed, s);
    if (st != kOk) return st;
    return finish_count(out_of_range, out_of_range_host, s);
}

static int reconstruct_impl(const uint8_t *upper, const uint8_t *lower, int64_t N, int64_t K, uint16_t *W,
                            int64_t ldw, bool packed, void *stream) {
    int st = check_dims(0, N, K);
    if (st != kOk) return st;
    if (N == 0) return NESTEDFP_OK;
    if (upper == nullptr || lower == nullptr) return NESTEDFP_ERR_ARG;
    st = check_mat(W, N, K, ldw, 8);
    if (st != kOk) return st;
    if (!aligned(upper, 16) || !aligned(lower, 16)) return NESTEDFP_ERR_SHAPE;
    return launch_reconstruct(upper, lower, N, K, W, ldw, packed, static_cast<hipStream_t>(stream));
}

static size_t gemm_workspace_size(int64_t M, int64_t N, int64_t K, int mode) {
    if (check_dims(M, N, K) != kOk) return 0;
    if (!valid_mode(mode)) return 0;
    if (M == 0 || N == 0) return 0;
    // one query serves both plane layouts and the plain baselines; their launch shapes may differ
    size_t need = 0;
    if (mode == NESTEDFP_MODE_FP16) {
        for (int kind : {kNestedF16, kNestedF16Row, kPlainF16, kPlainF16Packed}) {
            const size_t b = workspace_bytes_for(kind, M, N, K, false);
            if (b > need) need = b;
        }
    } else {
        for (int kind : {kE4M3, kE4M3Row}) {
            const size_t b = workspace_bytes_for(kind, M, N, K, true);
            if (b > need) need = b;
        }
    }
    return need;
}

static int gemm_impl(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const uint8_t *upper,
                     const uint8_t *lower, int64_t N, int layout, int mode, const float *act_scale, uint16_t *Y,
                     int64_t ldy, void *workspace, size_t workspace_bytes, void *stream) {
    if (!valid_mode(mode) || !valid_layout(layout)) return NESTEDFP_ERR_ARG;
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
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool packed = layout == NESTEDFP_LAYOUT_PACKED;
    Workspace ws;
    if (mode == NESTEDFP_MODE_FP16) {
        const int kind = packed ? kNestedF16 : kNestedF16Row;
        if (!carve(workspace, workspace_bytes, kind, M, N, K, false, ws)) return NESTEDFP_ERR_WORKSPACE;
        GemmArgs a;
        memset(&a, 0, sizeof(a));
        a.X = X;  a.ldx = ldx;  a.W0 = upper;  a.W1 = lower;  a.ldw = K;
        a.M = M;  a.N = N;  a.K = K;  a.Y = Y;  a.ldy = ldy;
        a.partials = ws.partials;  a.partial_bytes = ws.partial_bytes;  a.counters = ws.counters;
        return run_gemm(kind, a, s);
    }
    const int kind = packed ? kE4M3 : kE4M3Row;
    if (!carve(workspace, workspace_bytes, kind, M, N, K, true, ws)) return NESTEDFP_ERR_WORKSPACE;
    // Sec. 4.1: the upper plane read as E4M3 is the weight times 2^8
    st = fp8_gemm_fused(X, M, K, ldx, act_scale, upper, N, kind, 0.00390625f, Y, ldy, s);
    if (st >= 0) return st;
    st = launch_quantize_act(X, M, K, ldx, act_scale, ws.xq, ws.scales, s);
    if (st != kOk) return st;
    return fp8_gemm(ws.xq, ws.scales, M, K, upper, N, kind, 0.00390625f, Y, ldy, ws, s);
}

static int plain_fp16_impl(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const void *W, int64_t N,
                           int64_t ldw, bool packed, uint16_t *Y, int64_t ldy, void *workspace,
                           size_t workspace_bytes, void *stream) {
    int st = check_dims(M, N, K);
    if (st != kOk) return st;
    if (M == 0 || N == 0) return NESTEDFP_OK;
    st = check_mat(X, M, K, ldx, 8);
    if (st != kOk) return st;
    st = packed ? (W == nullptr ? kErrArg : (aligned(W, 16) ? kOk : kErrShape)) : check_mat(W, N, K, ldw, 8);
    if (st != kOk) return st;
    st = check_out(Y, N, ldy);
    if (st != kOk) return st;
    const int kind = packed ? kPlainF16Packed : kPlainF16;
    Workspace ws;
    if (!carve(workspace, workspace_bytes, kind, M, N, K, false, ws)) return NESTEDFP_ERR_WORKSPACE;
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.X = X;  a.ldx = ldx;  a.W0 = W;  a.W1 = nullptr;  a.ldw = packed ? K : ldw;
    a.M = M;  a.N = N;  a.K = K;  a.Y = Y;  a.ldy = ldy;
    a.partials = ws.partials;  a.partial_bytes = ws.partial_bytes;  a.counters = ws.counters;
    return run_gemm(kind, a, static_cast<hipStream_t>(stream));
}

static int plain_fp8_impl(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const uint8_t *Wq, int64_t N,
                          bool packed, float w_scale, const float *act_scale, uint16_t *Y, int64_t ldy,
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
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int kind = packed ? kE4M3 : kE4M3Row;
    Workspace ws;
    if (!carve(workspace, workspace_bytes, kind, M, N, K, true, ws)) return NESTEDFP_ERR_WORKSPACE;
    st = fp8_gemm_fused(X, M, K, ldx, act_scale, Wq, N, kind, w_scale, Y, ldy, s);
    if (st >= 0) return st;
    st = launch_quantize_act(X, M, K, ldx, act_scale, ws.xq, ws.scales, s);
    if (st != kOk) return st;
    return fp8_gemm(ws.xq, ws.scales, M, K, Wq, N, kind, w_scale, Y, ldy, ws, s);
}

}  // namespace nfp

// ---- scratch of the entry point that takes no workspace ------------------------------------------
// A fixed array in the library's device image: every GPU that loads the library holds its own copy
// at its own address until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the address it returns (per device) is what kernels and fills are given.
static __device__ __align__(256) unsigned char scratch[NESTEDFP_STATIC_SCRATCH_BYTES];

namespace nfp {

constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];               // device address of `scratch`, per device
static std::mutex g_scratch_mutex;

// Address of this device's scratch array; on first use its arrival counters are cleared (the image
// starts zeroed and every call leaves them zero; the fill makes that independent of the loader).
static int static_scratch(void **out, hipStream_t stream) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return kErrHip;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return kErrHip;
        if (launch_zero_words(static_cast<uint32_t *>(ptr), kMaxCounters, stream) != kOk) return kErrHip;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return kOk;
}

}  // namespace nfp

using namespace nfp;

extern "C" {

int nestedfp_version(void) { return 300; }

const char *nestedfp_status_string(int status) {
    switch (status) {
        case NESTEDFP_OK: return "ok";
        case NESTEDFP_ERR_ARG: return "invalid argument (NULL pointer, negative size, unknown mode or layout)";
        case NESTEDFP_ERR_SHAPE: return "unsupported shape (K % 16, leading dimension, size limit or alignment)";
        case NESTEDFP_ERR_RANGE: return "weights outside the NestedFP range (|w| > 1.75, Inf or NaN)";
        case NESTEDFP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case NESTEDFP_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
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
    return decompose_impl(W, N, K, ldw, upper, lower, out_of_range, out_of_range_host, false, stream);
}

int nestedfp_decompose_packed(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint8_t *upper,
                              uint8_t *lower, uint64_t *out_of_range, uint64_t *out_of_range_host,
                              void *stream) {
    return decompose_impl(W, N, K, ldw, upper, lower, out_of_range, out_of_range_host, true, stream);
}

int nestedfp_reconstruct(const uint8_t *upper, const uint8_t *lower, int64_t N, int64_t K, uint16_t *W,
                         int64_t ldw, void *stream) {
    return reconstruct_impl(upper, lower, N, K, W, ldw, false, stream);
}

int nestedfp_reconstruct_packed(const uint8_t *upper, const uint8_t *lower, int64_t N, int64_t K, uint16_t *W,
                                int64_t ldw, void *stream) {
    return reconstruct_impl(upper, lower, N, K, W, ldw, true, stream);
}

size_t nestedfp_plane_bytes(int64_t N, int64_t K) {
    if (check_dims(0, N, K) != kOk) return 0;
    return plane_bytes(N, K);
}

size_t nestedfp_packed_fp16_bytes(int64_t N, int64_t K) {
    if (check_dims(0, N, K) != kOk) return 0;
    return 2 * plane_bytes(N, K);
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

int nestedfp_pack_fp16(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint8_t *dst, void *stream) {
    int st = check_dims(0, N, K);
    if (st != kOk) return st;
    if (N == 0) return NESTEDFP_OK;
    if (dst == nullptr) return NESTEDFP_ERR_ARG;
    st = check_mat(W, N, K, ldw, 8);
    if (st != kOk) return st;
    if (!aligned(dst, 16)) return NESTEDFP_ERR_SHAPE;
    return launch_pack_fp16(W, N, K, ldw, dst, static_cast<hipStream_t>(stream));
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
    return gemm_workspace_size(M, N, K, mode);
}

int nestedfp_workspace_init(void *workspace, size_t workspace_bytes, void *stream) {
    if (workspace == nullptr) return workspace_bytes == 0 ? NESTEDFP_OK : NESTEDFP_ERR_ARG;
    if (!aligned(workspace, 16)) return NESTEDFP_ERR_SHAPE;
    const size_t n = workspace_bytes < kCounterBytes ? workspace_bytes : kCounterBytes;
    return launch_zero_words(static_cast<uint32_t *>(workspace), (int)(n / 4), static_cast<hipStream_t>(stream));
}

int nestedfp_gemm(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const uint8_t *upper,
                  const uint8_t *lower, int64_t N, int mode, const float *act_scale, uint16_t *Y,
                  int64_t ldy, void *workspace, size_t workspace_bytes, void *stream) {
    return gemm_impl(X, M, K, ldx, upper, lower, N, NESTEDFP_LAYOUT_ROWMAJOR, mode, act_scale, Y, ldy, workspace,
                     workspace_bytes, stream);
}

int nestedfp_gemm_packed(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const uint8_t *upper,
                         const uint8_t *lower, int64_t N, int mode, const float *act_scale, uint16_t *Y,
                         int64_t ldy, void *workspace, size_t workspace_bytes, void *stream) {
    return gemm_impl(X, M, K, ldx, upper, lower, N, NESTEDFP_LAYOUT_PACKED, mode, act_scale, Y, ldy, workspace,
                     workspace_bytes, stream);
}

int nestedfp_gemm_static(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const uint8_t *upper,
                         const uint8_t *lower, int64_t N, int mode, const float *act_scale, uint16_t *Y,
                         int64_t ldy, void *stream) {
    if (!valid_mode(mode)) return NESTEDFP_ERR_ARG;
    int st = check_dims(M, N, K);
    if (st != kOk) return st;
    if (M == 0 || N == 0) return NESTEDFP_OK;
    // the scratch this problem needs in this plane layout and mode, against the fixed array
    const int kind = mode == NESTEDFP_MODE_FP16 ? kNestedF16Row : kE4M3Row;
    const size_t need = workspace_bytes_for(kind, M, N, K, mode == NESTEDFP_MODE_FP8);
    if (need > (size_t)NESTEDFP_STATIC_SCRATCH_BYTES) return NESTEDFP_ERR_WORKSPACE;
    void *ws = nullptr;
    if (need > 0) {
        st = static_scratch(&ws, static_cast<hipStream_t>(stream));
        if (st != kOk) return st;
    }
    return gemm_impl(X, M, K, ldx, upper, lower, N, NESTEDFP_LAYOUT_ROWMAJOR, mode, act_scale, Y, ldy, ws,
                     need > 0 ? (size_t)NESTEDFP_STATIC_SCRATCH_BYTES : 0, stream);
}

int nestedfp_plain_gemm_fp16(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const uint16_t *W,
                             int64_t N, int64_t ldw, uint16_t *Y, int64_t ldy, void *workspace,
                             size_t workspace_bytes, void *stream) {
    return plain_fp16_impl(X, M, K, ldx, W, N, ldw, false, Y, ldy, workspace, workspace_bytes, stream);
}

int nestedfp_plain_gemm_fp16_packed(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const uint8_t *Wp,
                                    int64_t N, uint16_t *Y, int64_t ldy, void *workspace,
                                    size_t workspace_bytes, void *stream) {
    return plain_fp16_impl(X, M, K, ldx, Wp, N, K, true, Y, ldy, workspace, workspace_bytes, stream);
}

int nestedfp_plain_gemm_fp8(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const uint8_t *Wq,
                            int64_t N, float w_scale, const float *act_scale, uint16_t *Y, int64_t ldy,
                            void *workspace, size_t workspace_bytes, void *stream) {
    return plain_fp8_impl(X, M, K, ldx, Wq, N, false, w_scale, act_scale, Y, ldy, workspace, workspace_bytes, stream);
}

int nestedfp_plain_gemm_fp8_packed(const uint16_t *X, int64_t M, int64_t K, int64_t ldx, const uint8_t *Wq,
                                   int64_t N, float w_scale, const float *act_scale, uint16_t *Y, int64_t ldy,
                                   void *workspace, size_t workspace_bytes, void *stream) {
    return plain_fp8_impl(X, M, K, ldx, Wq, N, true, w_scale, act_scale, Y, ldy, workspace, workspace_bytes, stream);
}

int nestedfp_gemm_fp8_prequantized(const uint8_t *Xq, const float *scales, int64_t M, int64_t K,
                                   const uint8_t *upper, int64_t N, int layout, float w_scale, uint16_t *Y,
                                   int64_t ldy, void *workspace, size_t workspace_bytes, void *stream) {
    if (!valid_layout(layout)) return NESTEDFP_ERR_ARG;
    int st = check_dims(M, N, K);
    if (st != kOk) return st;
    if (M == 0 || N == 0) return NESTEDFP_OK;
    if (Xq == nullptr || scales == nullptr || upper == nullptr) return NESTEDFP_ERR_ARG;
    st = check_out(Y, N, ldy);
    if (st != kOk) return st;
    if (!aligned(Xq, 16) || !aligned(upper, 16) || !aligned(scales, 4)) return NESTEDFP_ERR_SHAPE;
    const int kind = layout == NESTEDFP_LAYOUT_PACKED ? kE4M3 : kE4M3Row;
    Workspace ws;
    if (!carve(workspace, workspace_bytes, kind, M, N, K, false, ws)) return NESTEDFP_ERR_WORKSPACE;
    return fp8_gemm(Xq, scales, M, K, upper, N, kind, w_scale, Y, ldy, ws, static_cast<hipStream_t>(stream));
}

int nestedfp_layer_prepare(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, int layout, uint8_t *upper,
                           uint8_t *lower, uint64_t *out_of_range, nestedfp_layer *layer_host, void *stream) {
    if (layer_host == nullptr || out_of_range == nullptr || !valid_layout(layout)) return NESTEDFP_ERR_ARG;
    uint64_t count = 0;
    int st = decompose_impl(W, N, K, ldw, upper, lower, out_of_range, &count, layout == NESTEDFP_LAYOUT_PACKED, stream);
    if (st != NESTEDFP_OK && st != NESTEDFP_ERR_RANGE) return st;
    memset(layer_host, 0, sizeof(*layer_host));
    layer_host->N = N;
    layer_host->K = K;
    layer_host->layout = layout;
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
    return gemm_workspace_size(M, layer_host->N, layer_host->K, mode);
}

int nestedfp_linear(const uint16_t *X, int64_t M, int64_t ldx, const nestedfp_layer *layer_host, int mode,
                    const float *act_scale, uint16_t *Y, int64_t ldy, void *workspace,
                    size_t workspace_bytes, void *stream) {
    if (layer_host == nullptr) return NESTEDFP_ERR_ARG;
    if (!valid_mode(mode)) return NESTEDFP_ERR_ARG;
    const nestedfp_layer &L = *layer_host;
    if (L.is_exception)
        return nestedfp_plain_gemm_fp16(X, M, L.K, ldx, L.W, L.N, L.ldw, Y, ldy, workspace, workspace_bytes, stream);
    return gemm_impl(X, M, L.K, ldx, L.upper, L.lower, L.N, L.layout, mode, act_scale, Y, ldy, workspace,
                     workspace_bytes, stream);
}

int nestedfp_select_mode(int64_t tokens, int64_t threshold) {
    return tokens > threshold ? NESTEDFP_MODE_FP8 : NESTEDFP_MODE_FP16;
}

int nestedfp_probe_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream) {
    if (src == nullptr || sink == nullptr) return NESTEDFP_ERR_ARG;
    if (bytes == 0 || (bytes & 65535) != 0 || !aligned(src, 16) || bytes / 65536 > 0x7fffffffu) return NESTEDFP_ERR_SHAPE;
    return launch_probe_stream_read(src, bytes, sink, static_cast<hipStream_t>(stream));
}

int nestedfp_probe_stream_read_sparse(const void *src, size_t bytes, uint32_t *sink, void *stream) {
    if (src == nullptr || sink == nullptr) return NESTEDFP_ERR_ARG;
    if (bytes == 0 || (bytes & 131071) != 0 || !aligned(src, 16) || bytes / 131072 > 0x7fffffffu) return NESTEDFP_ERR_SHAPE;
    return launch_probe_stream_read_sparse(src, bytes, sink, static_cast<hipStream_t>(stream));
}

int nestedfp_probe_mfma(const void *operands, int fp8, int iters, uint32_t *sink, double *flops_host, void *stream) {
    if (operands == nullptr || sink == nullptr || iters <= 0) return NESTEDFP_ERR_ARG;
    if (!aligned(operands, 16)) return NESTEDFP_ERR_SHAPE;
    return launch_probe_mfma(operands, fp8 != 0, iters, sink, flops_host, static_cast<hipStream_t>(stream));
}

static const char *const kKnobs[] = {"small_max_m", "small_split", "small_spw", "small_tiles", "small_interleave",
                                     "large_split", "large_bm", "large_bn", "large_epilogue", "small_fuse_quant", "quant_hw", "large_xcd_map",
                                     "fused_reduce", "large_deep", "tuned_table", "quant_onepass", nullptr};

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
    else if (!strcmp(knob, "fused_reduce")) t.fused_reduce = value;
    else if (!strcmp(knob, "large_deep")) t.large_deep = value;
    else if (!strcmp(knob, "tuned_table")) t.tuned_table = value;
    else if (!strcmp(knob, "quant_onepass")) t.quant_onepass = value;
    else return NESTEDFP_ERR_ARG;
    return NESTEDFP_OK;
}

}  // extern "C"
