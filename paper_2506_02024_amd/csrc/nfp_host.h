// Host-side declarations shared by the NestedFP library's translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <atomic>

namespace nfp {

// status codes mirror include/nestedfp.h
enum { kOk = 0, kErrArg = 1, kErrShape = 2, kErrRange = 3, kErrWorkspace = 4, kErrHip = 5 };

inline int hip_ok(hipError_t e) { return e == hipSuccess ? kOk : kErrHip; }

// weight operand kinds of the GEMM kernels
//   kPlainF16      : FP16 weights, row-major [N,K] (row stride ldw)
//   kNestedF16     : the two byte planes in packed 1 KB blocks
//   kE4M3          : E4M3 bytes (the upper plane) in packed 1 KB blocks
//   kE4M3Quant     : as kE4M3, FP16 activations quantised per token inside the kernel
//   kNestedF16Row  : the two byte planes row-major [N,K], regrouped into operand order in flight
//   kE4M3Row       : E4M3 bytes row-major [N,K]
//   kPlainF16Packed: FP16 weights in packed 2 KB blocks (the like-for-like partner of kNestedF16)
enum WeightKind { kPlainF16 = 0, kNestedF16 = 1, kE4M3 = 2, kE4M3Quant = 3,
                  kNestedF16Row = 4, kE4M3Row = 5, kPlainF16Packed = 6, kNumKinds = 7 };

constexpr bool kind_is_fp8(int k) { return k == kE4M3 || k == kE4M3Quant || k == kE4M3Row; }
constexpr bool kind_is_nested(int k) { return k == kNestedF16 || k == kNestedF16Row; }
// weights stored in blocks of 16 rows x 64 columns, lane order inside
constexpr bool kind_is_packed(int k) { return k == kNestedF16 || k == kE4M3 || k == kE4M3Quant || k == kPlainF16Packed; }
// bytes of one weight in the array(s) the kernel reads
constexpr int kind_elem_bytes(int k) { return (k == kPlainF16 || k == kPlainF16Packed) ? 2 : 1; }
// which cost table / routing rule a kind follows: 0 plain FP16 through LDS, 1 FP16 operands through
// registers (both plane layouts, packed FP16), 2 E4M3
constexpr int kind_class(int k) { return k == kPlainF16 ? 0 : (kind_is_fp8(k) ? 2 : 1); }

// bytes of one weight array of an [N,K] layer as the kernels address it (plain row-major FP16:
// row stride ldw elements; row-major planes are dense; packed kinds are padded to whole blocks)
inline int64_t weight_array_bytes(int kind, int64_t N, int64_t K, int64_t ldw) {
    if (N <= 0) return 0;
    if (kind_is_packed(kind)) return ((N + 15) / 16 * 16) * ((K + 63) / 64 * 64) * kind_elem_bytes(kind);
    if (kind == kPlainF16) return (N - 1) * 2 * ldw + 2 * K;
    return N * K;
}

struct GemmArgs {
    // activations: fp16 X (kPlainF16 / kNestedF16) or E4M3 Xq with per-row scales (kE4M3)
    const void *X;        // uint16_t* or uint8_t*
    int64_t ldx;          // elements
    const float *scales;  // [M], kE4M3 only
    const float *static_scale;  // kE4M3Quant: optional per-tensor activation scale (device float)
    float w_scale;        // kE4M3 only
    // weights
    const void *W0;       // fp16 W, or upper plane, or E4M3 weights
    const void *W1;       // lower plane (kNestedF16 only)
    int64_t ldw;          // elements (plain fp16 only; planes are dense)
    int64_t M, N, K;
    uint16_t *Y;
    int64_t ldy;
    float *partials;      // split-K scratch (may be NULL if split == 1)
    size_t partial_bytes;
    uint32_t *counters;   // kMaxCounters arrival counters, all zero between calls (NULL: reduce in a second launch)
};

// arrival counters at the start of every workspace: one per output tile of a split launch
constexpr int kMaxCounters = 4096;
constexpr size_t kCounterBytes = kMaxCounters * sizeof(uint32_t);

// tuning knobs (negative = built-in choice)
struct Tuning {
    int64_t small_max_m;     // largest M routed to the streaming kernel
    int64_t small_split;     // grid-level split-K of the streaming kernel
    int64_t small_spw;       // K-steps per wave (2 or 4)
    int64_t small_tiles;     // 16-row weight tiles per workgroup
    int64_t small_interleave;  // 1: a workgroup's tiles are strided by the grid size
    int64_t large_split;     // grid-level split-K of the tiled kernel
    int64_t large_bm;        // tokens per tile of the tiled kernel (64, 128 or 256)
    int64_t large_bn;        // weight rows per tile (128 or 256; unset: same as large_bm)
    int64_t large_epilogue;  // 0: store results straight from the MFMA layout instead of row-wise through LDS
    int64_t small_fuse_quant;  // 1: quantise activations inside the streaming kernel where it can
    int64_t quant_hw;        // 1: hardware E4M3 convert, 0: integer rounding
    int64_t large_xcd_map;   // 0: tiles in launch order instead of grouped by XCD (tiled kernels)
    int64_t fused_reduce;    // 0: split-K partials are summed by a second launch instead of the last workgroup
    int64_t large_deep;      // 1 / 0: force / forbid the deeper load pipelines of the tiled kernels (tiles below 256 x 256)
    int64_t tuned_table;     // 0: the tiled kernels' launch shape always comes from the cost model, never from the table of timed shapes
    int64_t quant_onepass;   // 1 / 0: force / forbid the single-pass activation quantisation (rows kept in registers) where it fits
};
Tuning &tuning();

int launch_decompose(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint8_t *upper,
                     uint8_t *lower, uint64_t *counter, bool packed, hipStream_t stream);
int launch_range_check(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint64_t *counter,
                       hipStream_t stream);
int launch_zero_u64(uint64_t *p, hipStream_t stream);
int launch_reconstruct(const uint8_t *upper, const uint8_t *lower, int64_t N, int64_t K,
                       uint16_t *W, int64_t ldw, bool packed, hipStream_t stream);
int launch_pack_fp16(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint8_t *dst, hipStream_t stream);
int launch_zero_words(uint32_t *p, int n, hipStream_t stream);
size_t plane_bytes(int64_t N, int64_t K);
int launch_pack_plane(const uint8_t *src, int64_t N, int64_t K, int64_t ld, uint8_t *dst, hipStream_t stream);
int launch_unpack_plane(const uint8_t *src, int64_t N, int64_t K, uint8_t *dst, int64_t ld, hipStream_t stream);
int launch_quantize_act(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                        const float *static_scale, uint8_t *Xq, float *scales, hipStream_t stream);

// streaming (small-M) and tiled (large-M) GEMM families
bool small_gemm_supports(int kind, int64_t M, int64_t N, int64_t K, int64_t ldw);
bool small_gemm_fuses_quant(int64_t M, int64_t N, int64_t K);
size_t small_gemm_partial_bytes(int kind, int64_t M, int64_t N, int64_t K);
int launch_small_gemm(int kind, const GemmArgs &a, hipStream_t stream);
size_t large_gemm_partial_bytes(int kind, int64_t M, int64_t N, int64_t K);
int launch_large_gemm(int kind, const GemmArgs &a, hipStream_t stream);

int launch_splitk_reduce(const float *partials, int S, int64_t M, int64_t N, const float *scales,
                         float w_scale, uint16_t *Y, int64_t ldy, hipStream_t stream);

bool large_gemm_supports(int kind, int64_t K, int64_t ldx, int64_t ldw);
int launch_probe_stream_read(const void *src, size_t bytes, uint32_t *sink, hipStream_t stream);
int launch_probe_stream_read_sparse(const void *src, size_t bytes, uint32_t *sink, hipStream_t stream);
int launch_probe_mfma(const void *operands, int fp8, int iters, uint32_t *sink, double *flops_host,
                      hipStream_t stream);

bool use_small_gemm(int64_t M);

}  // namespace nfp
