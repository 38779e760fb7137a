// Host-side declarations shared by the NestedFP library's translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace nfp {

// status codes mirror include/nestedfp.h
enum { kOk = 0, kErrArg = 1, kErrShape = 2, kErrRange = 3, kErrWorkspace = 4, kErrHip = 5 };

inline int hip_ok(hipError_t e) { return e == hipSuccess ? kOk : kErrHip; }

// weight operand kinds of the GEMM kernels
// kE4M3Quant: packed E4M3 weights, FP16 activations quantised per token inside the kernel
enum WeightKind { kPlainF16 = 0, kNestedF16 = 1, kE4M3 = 2, kE4M3Quant = 3 };

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
};

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
};
Tuning &tuning();

int launch_decompose(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint8_t *upper,
                     uint8_t *lower, uint64_t *counter, hipStream_t stream);
int launch_range_check(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint64_t *counter,
                       hipStream_t stream);
int launch_zero_u64(uint64_t *p, hipStream_t stream);
int launch_reconstruct(const uint8_t *upper, const uint8_t *lower, int64_t N, int64_t K,
                       uint16_t *W, int64_t ldw, hipStream_t stream);
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

bool use_small_gemm(int64_t M);

}  // namespace nfp
