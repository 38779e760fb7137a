/*
 * nestedfp.h -- C ABI of the NestedFP hot path for AMD MI355X (gfx950).
 *
 * NestedFP (arxiv 2506.02024) stores every FP16 weight of a linear layer once, as two
 * byte planes of the weight's shape (Sec. 4 "Overview"): `upper` is a valid E4M3 number
 * equal to the weight times 2^8 rounded to nearest-even, `lower` is the low mantissa byte
 * (Sec. 4.1).  A GEMM call then runs in one of two modes on the same planes: FP16 mode
 * rebuilds the exact FP16 weights on the fly (Sec. 4.2), FP8 mode reads only `upper`.
 *
 * Conventions shared by every call
 *   - All tensor pointers are DEVICE pointers unless the parameter name ends in `_host`.
 *     The caller owns every buffer; the library never allocates or frees device memory
 *     and never writes to an input.
 *   - FP16 data travels as uint16_t bit patterns.  W is [N,K] row-major (K contiguous,
 *     row stride ldw elements), X is [M,K] (row stride ldx), Y is [M,N] (row stride ldy);
 *     Y = X * W^T.  Quantised activations are dense row-major bytes.
 *   - BYTE PLANES ARE ROW-MAJOR: `upper` and `lower` (and the E4M3 weights of the plain FP8
 *     baseline) are dense [N,K] byte matrices, element (n,k) at n*K + k -- the two tensors of
 *     Sec. 4 "Overview" as they are.  The upper plane on its own is an ordinary E4M3 weight
 *     tensor that any FP8 GEMM can take (Sec. 4 "Challenge 2").  The GEMM kernels regroup the
 *     bytes into their operand order while loading them.
 *   - PACKED STORAGE IS AN OPT-IN PRE-PACK of the same bytes (the entry points whose names end
 *     in `_packed`): with Np = 16*ceil(N/16) and Kp = 64*ceil(K/64) a packed plane takes Np*Kp
 *     bytes (nestedfp_plane_bytes) and consists of 1024-byte blocks, one per 16-row by
 *     64-column sub-matrix; block (i,j) starts at ((i * Kp/64) + j) * 1024 and holds the
 *     16-byte chunk of row 16i+r, columns 64j+16g .. 64j+16g+15 at chunk index r + 16g
 *     (r = 0..15, g = 0..3), bytes in column order.  Rows >= N and columns >= K are zero.
 *     That is the order in which the 64 lanes of a wave hold an MFMA operand, so one 128-bit
 *     load per lane reads a block front to back; the weight stream of a decode-sized batch
 *     runs 10-30 % faster from it than from row-major planes.  nestedfp_pack_plane /
 *     nestedfp_unpack_plane convert; footprint and contents are otherwise the same.
 *   - K must be a positive multiple of 16 and at most 2^21; ldw, ldx must be multiples of 8,
 *     >= K and at most 2^21; ldy must be a multiple of 4 and >= N when N % 4 == 0, else any
 *     ldy >= N is taken by a slower store path; W, X, planes, Xq and workspace pointers must
 *     be 16-byte aligned, Y 8-byte aligned.  M >= 1 and N >= 1 are otherwise arbitrary (no
 *     padding is asked of the caller).  M == 0 or N == 0 is a no-op that returns NESTEDFP_OK
 *     (the GEMM entry points then look at no pointer: empty operands may be NULL).
 *   - WORKSPACE.  The GEMM entry points take caller-provided scratch (size from the matching
 *     size query).  Its first NESTEDFP_WORKSPACE_COUNTER_BYTES bytes are arrival counters of
 *     the split-K kernels: pass every new workspace to nestedfp_workspace_init once (and again
 *     if anything else wrote to it); every call leaves the counters cleared.  Calls that share
 *     a workspace must not overlap in time (different streams need different workspaces).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls are
 *     asynchronous on that stream except where stated.
 *   - Argument errors are found before anything is launched and reported as a status
 *     code; nothing aborts or throws.
 *   - Thread safety: calls may be made from several host threads as long as nestedfp_tune is
 *     not in use (its knobs are process-wide and unsynchronised; leave them alone outside
 *     benchmarks and tests).
 */
#ifndef NESTEDFP_H
#define NESTEDFP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    NESTEDFP_OK = 0,
    NESTEDFP_ERR_ARG = 1,       /* NULL pointer, negative size, unknown mode            */
    NESTEDFP_ERR_SHAPE = 2,     /* K % 16 != 0, leading dimension too small or too large, misaligned */
    NESTEDFP_ERR_RANGE = 3,     /* some |w| > 1.75, Inf or NaN: layer is not applicable  */
    NESTEDFP_ERR_WORKSPACE = 4, /* workspace missing or smaller than the size query says */
    NESTEDFP_ERR_HIP = 5        /* a HIP call or launch failed                           */
} nestedfp_status;

typedef enum {
    NESTEDFP_MODE_FP16 = 0,     /* both planes, exact FP16 weights, fp16 MFMA            */
    NESTEDFP_MODE_FP8 = 1       /* upper plane only, E4M3 x E4M3 MFMA, scale 2^-8        */
} nestedfp_mode;

typedef enum {
    NESTEDFP_LAYOUT_ROWMAJOR = 0,   /* planes are dense [N,K] byte matrices               */
    NESTEDFP_LAYOUT_PACKED = 1      /* planes are pre-packed into 1 KB blocks (see above) */
} nestedfp_layout;

#define NESTEDFP_WORKSPACE_COUNTER_BYTES 16384

int nestedfp_version(void);
const char *nestedfp_status_string(int status);

/*
 * Applicability test (Sec. 4.1 "Opportunities", "Handling Exception Layers"): a layer
 * can be stored in the format iff every weight has |w| <= 1.75 (so the FP16 exponent MSB
 * is zero and rounding cannot leave E4M3's finite range).  Counts the words that do not
 * fit (Inf and NaN included) into *out_of_range (device, 8 bytes, overwritten).
 * If out_of_range_host is non-NULL the call also waits for the stream, copies the count
 * there and returns NESTEDFP_ERR_RANGE when it is non-zero.
 */
int nestedfp_range_check(const uint16_t *W, int64_t N, int64_t K, int64_t ldw,
                         uint64_t *out_of_range, uint64_t *out_of_range_host, void *stream);

/*
 * Decomposition (Sec. 4.1 "Our Proposal"), done once, offline: for each weight
 *   upper = S | RNE_7(E[3:0]|M[1:10] -> E[3:0]|M[1:3])   (carry may enter the exponent)
 *   lower = M[3:10]
 * written to the row-major byte planes `upper` and `lower` (N*K bytes each).  Words that
 * fail the applicability test are counted into *out_of_range (device, 8 bytes,
 * overwritten; may be NULL to skip counting) and their plane entries are written as 0.  With
 * out_of_range_host non-NULL (needs out_of_range too) the call waits for the stream,
 * copies the count and returns NESTEDFP_ERR_RANGE if it is non-zero: the caller then
 * keeps the layer in FP16 (an "exception layer") and runs nestedfp_plain_gemm_fp16.
 * nestedfp_decompose_packed writes packed planes instead (nestedfp_plane_bytes(N,K) bytes
 * each, padding included, all of it overwritten).
 */
int nestedfp_decompose(const uint16_t *W, int64_t N, int64_t K, int64_t ldw,
                       uint8_t *upper, uint8_t *lower,
                       uint64_t *out_of_range, uint64_t *out_of_range_host, void *stream);
int nestedfp_decompose_packed(const uint16_t *W, int64_t N, int64_t K, int64_t ldw,
                              uint8_t *upper, uint8_t *lower,
                              uint64_t *out_of_range, uint64_t *out_of_range_host, void *stream);

/*
 * Lossless reconstruction (Sec. 4.1 "FP16 Reconstruction", Sec. 4.2 Alg. 1): rebuilds the
 * FP16 words from the (row-major / packed) planes; if the LSB of upper differs from the MSB
 * of lower the rounding is undone first.  Exact inverse of nestedfp_decompose on planes it
 * produced; for byte pairs that no in-range weight produces the result is unspecified.
 */
int nestedfp_reconstruct(const uint8_t *upper, const uint8_t *lower, int64_t N, int64_t K,
                         uint16_t *W, int64_t ldw, void *stream);
int nestedfp_reconstruct_packed(const uint8_t *upper, const uint8_t *lower, int64_t N, int64_t K,
                                uint16_t *W, int64_t ldw, void *stream);

/*
 * Packed storage (see the conventions above; it serves the kernels of Sec. 4.2, whose lanes
 * each own 16 consecutive weights of one row).
 * plane_bytes: size of one packed plane of an [N,K] layer; 0 for invalid arguments.
 * pack_plane:  row-major bytes src[N][ld] (ld >= K, multiple of 16) -> packed dst.  Padding is zeroed.
 * unpack_plane: packed src -> row-major dst[N][ld].
 * packed_fp16_bytes / pack_fp16: the same block order for FP16 weights (2 * plane_bytes; a
 *   block is two halves of 1 KB, lane chunk l of the first half holding columns 16g .. 16g+7
 *   and of the second half columns 16g+8 .. 16g+15 of row r, l = r + 16g): the operand of
 *   nestedfp_plain_gemm_fp16_packed.
 */
size_t nestedfp_plane_bytes(int64_t N, int64_t K);
int nestedfp_pack_plane(const uint8_t *src, int64_t N, int64_t K, int64_t ld, uint8_t *dst, void *stream);
int nestedfp_unpack_plane(const uint8_t *src, int64_t N, int64_t K, uint8_t *dst, int64_t ld, void *stream);
size_t nestedfp_packed_fp16_bytes(int64_t N, int64_t K);
int nestedfp_pack_fp16(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint8_t *dst, void *stream);

/*
 * Activation quantisation for FP8 mode (Sec. 2.2 "E4M3 Format": dynamic per-token or
 * static per-tensor scaling; Sec. 5.1 uses per-token).  For each row m of X:
 *   scale[m] = amax_k |X[m,k]| / 448   (one binary32 division; 1 if the row is all zero)
 *   Xq[m,k]  = E4M3_RNE_saturating( binary32(X[m,k]) / scale[m] )
 * With static_scale non-NULL (device, one float) that value is used for every row.
 * Xq is dense [M,K] bytes, scales is [M] floats.  X must be finite.
 */
int nestedfp_quantize_act(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                          const float *static_scale, uint8_t *Xq, float *scales, void *stream);

/*
 * Bytes of caller-provided scratch that nestedfp_gemm (or a plain baseline, which take
 * the same query with the corresponding mode; either plane layout) needs for this problem:
 * arrival counters, split-K partial sums and, in FP8 mode, the quantised activations with
 * their scales.  Grows with M*K and M*N, never with N*K: no weight copy is ever made.
 * Returns 0 for invalid arguments and for empty problems.
 * workspace_init clears the arrival counters at the start of a workspace (a small kernel on
 * `stream`, safe inside a stream capture); see WORKSPACE above.
 */
size_t nestedfp_gemm_workspace_size(int64_t M, int64_t N, int64_t K, int mode);
int nestedfp_workspace_init(void *workspace, size_t workspace_bytes, void *stream);

/*
 * The linear layer Y = X * W^T over the two planes (Sec. 4 "Overview", Sec. 4.2).
 *   FP16 mode: streams both planes, merges them into exact FP16 weights inside the
 *     kernel, fp16 MFMA with fp32 accumulation, fp16 output.  Bitwise equal to
 *     nestedfp_plain_gemm_fp16 on the original weights whenever the two run with the same
 *     launch shape (the built-in choice is made per kernel and may differ; the knobs
 *     small_max_m, small_spw, large_bm / large_bn / large_split of nestedfp_tune pin it).
 *   FP8 mode: quantises X per token (or with *act_scale, device float, if non-NULL),
 *     multiplies E4M3 activations by the upper plane read as E4M3, fp32 accumulation,
 *     scales by scale[m] * 2^-8 (Sec. 4.1: the upper plane is the weight times 2^8),
 *     fp16 output: the FP32 sum times the FP32 scale is rounded to FP32, then to FP16, in
 *     every kernel and launch shape.  `lower` is never read and may be NULL.
 * workspace must hold at least nestedfp_gemm_workspace_size(M,N,K,mode) bytes.
 * nestedfp_gemm takes row-major planes, nestedfp_gemm_packed packed ones; same results bit
 * for bit.
 */
int nestedfp_gemm(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                  const uint8_t *upper, const uint8_t *lower, int64_t N,
                  int mode, const float *act_scale,
                  uint16_t *Y, int64_t ldy,
                  void *workspace, size_t workspace_bytes, void *stream);
int nestedfp_gemm_packed(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                         const uint8_t *upper, const uint8_t *lower, int64_t N,
                         int mode, const float *act_scale,
                         uint16_t *Y, int64_t ldy,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * nestedfp_gemm for callers that cannot allocate device memory or pass a workspace (code
 * under HIP graph capture that owns no scratch, tight serving loops, harnesses that forbid
 * hipMalloc): row-major planes, same arguments without the workspace, same results.  The
 * scratch is a fixed array inside the library's device image (NESTEDFP_STATIC_SCRATCH_BYTES
 * per GPU, held until the process ends); a problem whose workspace query exceeds it is
 * refused with NESTEDFP_ERR_WORKSPACE.  The call itself allocates nothing.  All calls on one
 * GPU share that array: calls that may overlap in time on one GPU (different streams) race.
 */
#define NESTEDFP_STATIC_SCRATCH_BYTES (32u << 20)
int nestedfp_gemm_static(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                         const uint8_t *upper, const uint8_t *lower, int64_t N,
                         int mode, const float *act_scale,
                         uint16_t *Y, int64_t ldy, void *stream);

/*
 * Plain baselines of the same kernel family, for the comparison of Sec. 5.2 (NestedFP
 * FP16 mode against an FP16 GEMM that reads ordinary FP16 weights) and its FP8 analogue.
 * plain_gemm_fp16: W is ordinary row-major FP16 [N,K].
 * plain_gemm_fp16_packed: Wp is FP16 in packed storage (nestedfp_pack_fp16): the same kernel
 *   as FP16 mode over packed planes minus the reconstruction, i.e. the like-for-like partner
 *   that isolates the cost of Alg. 1.
 * plain_gemm_fp8:  Wq is any row-major E4M3 [N,K] tensor (plain_gemm_fp8_packed: in packed
 *   plane storage) with one host-side float scale;
 *   Y = scale[m] * w_scale * sum_k e4m3(Xq) * e4m3(Wq).  Feeding it the upper plane with
 *   w_scale = 2^-8 is, by Sec. 4 "Challenge 2", exactly FP8 mode.
 */
int nestedfp_plain_gemm_fp16(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                             const uint16_t *W, int64_t N, int64_t ldw,
                             uint16_t *Y, int64_t ldy,
                             void *workspace, size_t workspace_bytes, void *stream);
int nestedfp_plain_gemm_fp16_packed(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                                    const uint8_t *Wp, int64_t N,
                                    uint16_t *Y, int64_t ldy,
                                    void *workspace, size_t workspace_bytes, void *stream);
int nestedfp_plain_gemm_fp8(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                            const uint8_t *Wq, int64_t N, float w_scale,
                            const float *act_scale,
                            uint16_t *Y, int64_t ldy,
                            void *workspace, size_t workspace_bytes, void *stream);
int nestedfp_plain_gemm_fp8_packed(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                                   const uint8_t *Wq, int64_t N, float w_scale,
                                   const float *act_scale,
                                   uint16_t *Y, int64_t ldy,
                                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * FP8-mode GEMM from activations that are already quantised (Xq dense row-major [M,K] E4M3 bytes,
 * scales [M] floats), e.g. by nestedfp_quantize_act; lets a caller quantise once and
 * reuse the result for several linears that share X.  Same arithmetic as FP8 mode.
 * `layout` (nestedfp_layout) says how `upper` is stored.
 */
int nestedfp_gemm_fp8_prequantized(const uint8_t *Xq, const float *scales, int64_t M, int64_t K,
                                   const uint8_t *upper, int64_t N, int layout, float w_scale,
                                   uint16_t *Y, int64_t ldy,
                                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * Exception layers (Sec. 4.1 "Handling Exception Layers", App. Table 4): a layer with any
 * |w| > 1.75 cannot be stored in the format and stays in FP16; it then runs the FP16 GEMM
 * in BOTH modes while every other layer follows the requested mode.
 * nestedfp_layer describes one linear either way (a plain struct in HOST memory; the
 * pointers inside are device pointers owned by the caller).
 * layer_prepare: decomposes W into upper/lower (in `layout`, as nestedfp_decompose /
 *   nestedfp_decompose_packed), waits for the stream and fills *layer: is_exception = 0 with
 *   the planes, or, if some weight is out of range, is_exception = 1 with W/ldw (the planes
 *   then hold nothing useful and may be released; W must stay alive instead).
 *   *out_of_range is device scratch (8 bytes).  Returns NESTEDFP_OK in both cases.
 * linear_workspace_size / linear: Y = X * W^T for the layer in `mode`; an exception layer
 *   ignores the mode (and act_scale) and multiplies its FP16 weights.
 */
typedef struct {
    int64_t N, K;
    int32_t is_exception;
    int32_t layout;             /* nestedfp_layout of the planes */
    const uint8_t *upper;       /* planes when is_exception == 0 */
    const uint8_t *lower;
    const uint16_t *W;          /* row-major FP16 weights when is_exception == 1 */
    int64_t ldw;
    uint64_t out_of_range;      /* count found by layer_prepare */
} nestedfp_layer;

int nestedfp_layer_prepare(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, int layout,
                           uint8_t *upper, uint8_t *lower, uint64_t *out_of_range,
                           nestedfp_layer *layer_host, void *stream);
size_t nestedfp_linear_workspace_size(int64_t M, const nestedfp_layer *layer_host, int mode);
int nestedfp_linear(const uint16_t *X, int64_t M, int64_t ldx, const nestedfp_layer *layer_host,
                    int mode, const float *act_scale, uint16_t *Y, int64_t ldy,
                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * Load-aware mode selection (Sec. 5.4): an iteration runs in FP8 mode when the number of
 * tokens it has to process exceeds `threshold` (1024 in the paper's experiment), otherwise in
 * FP16 mode.  Pure host function; returns a nestedfp_mode.
 */
int nestedfp_select_mode(int64_t tokens, int64_t threshold);

/*
 * Measurement aids for the benchmark (no part of the method): what this chip sustains for
 * the two resources the GEMMs are bound by, measured with the library's own instruction mix.
 * probe_stream_read: every wave reads `bytes` (a multiple of 65536) of `src` once with 128-bit
 *   loads, many in flight, and keeps nothing (a checksum of a few lanes goes to *sink, device,
 *   4 bytes): the rate a weight stream can reach at best.
 * probe_stream_read_sparse: the same read (`bytes` a multiple of 131072) with 16 KB per wave and at
 *   most 8 waves per CU; fewer, longer-lived waves read faster than the many small workgroups of the
 *   probe above, so this is the higher of the two rates.
 * probe_mfma: `iters` rounds of dependent-free MFMAs on operands filled from `operands`
 *   (device, at least 65536 bytes, the caller's choice of bit patterns) on every CU;
 *   fp8 = 0: v_mfma_f32_16x16x32_f16, fp8 = 1: v_mfma_f32_16x16x128_f8f6f4.  *flops_host
 *   receives the flops one call performs.  Results go to *sink (device, 4 bytes).
 */
int nestedfp_probe_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream);
int nestedfp_probe_stream_read_sparse(const void *src, size_t bytes, uint32_t *sink, void *stream);
int nestedfp_probe_mfma(const void *operands, int fp8, int iters, uint32_t *sink,
                        double *flops_host, void *stream);

/*
 * Tuning hook for benchmark sweeps and tests: overrides one launch parameter process-wide
 * (not thread-safe; a call that runs while another thread changes a knob may size its
 * workspace for one launch shape and launch another).  knob names are listed in
 * nestedfp_tune_name(i), i = 0.. until NULL.  value < 0 restores the built-in choice.
 * Returns NESTEDFP_ERR_ARG for unknown knobs.
 */
int nestedfp_tune(const char *knob, int64_t value);
const char *nestedfp_tune_name(int index);

#ifdef __cplusplus
}
#endif
#endif /* NESTEDFP_H */
