// Streaming GEMM for decode-sized batches (M <= 64): Y = X * W^T with the weight stream
// read exactly once from HBM and nothing staged in LDS (no weight reuse across waves).
// The paper's sweep starts at M = 32 with T_m >= 16 (Sec. 5.2, App. C); below that the
// linear layer is bound by HBM bandwidth, so the kernel is built around 128-bit loads of
// the byte planes with many loads in flight, K split across the waves of a workgroup,
// activations held in registers, and a fixed-order reduction.
//
// Weight rows are the MFMA "A" operand (lane l: row l%16 of a 16-row tile, K-group l/16),
// tokens (MT tiles of 16) the "B" operand, so each lane ends up with 4 consecutive output
// columns of one token: 8-byte stores of fp16.
//   plain FP16 : lane loads 32 B of FP16 weights              -> 2 x v_mfma_f32_16x16x32_f16
//   NestedFP16 : lane loads 16 B upper + 16 B lower, merges them (Sec. 4.2, Alg. 1) -> same
//   E4M3       : lane loads 2 x 16 B of E4M3 bytes (upper plane) -> 1 x v_mfma_f32_16x16x128_f8f6f4
// Every kind exists for two storage orders of the weights: row-major [N,K] (the two byte tensors
// of Sec. 4 "Overview" as they are: a lane's 16 bytes are 16 consecutive columns of its row, a wave
// instruction gathers 64-byte pieces of 16 rows) and packed blocks of 16 rows x 64 columns whose
// chunk order is the lane order, so that every load of a wave is one contiguous kilobyte.
// Columns past K and rows past N are never multiplied: their loads are sent out of the buffer's
// range and return zero, whatever the memory behind them holds.
#include <algorithm>

#include "nfp_device.h"
#include "nfp_host.h"

namespace nfp {

struct SmallParams {
    const uint8_t *X;       // fp16 X (as bytes) or E4M3 Xq
    int64_t x_row_bytes;    // row stride of X in bytes
    const float *scales;    // [M] (kE4M3) or NULL
    const float *static_scale;  // kE4M3Quant: per-tensor activation scale or NULL (per token)
    int quant_hw;           // kE4M3Quant: hardware or integer E4M3 encoder
    float w_scale;
    const uint8_t *W0;      // fp16 W (bytes) / upper plane / E4M3 weights
    const uint8_t *W1;      // lower plane
    uint32_t w_row_bytes;   // row-major kinds: row stride of W0 (and W1) in bytes
    uint32_t tile_bytes;    // distance between consecutive 16-row tiles in bytes
    uint32_t w_bytes;       // addressable bytes of W0 (and W1), < 2^31
    int M, N, K;
    uint16_t *Y;
    int64_t ldy;
    float *partials;        // [S][M][N] when S > 1
    uint32_t *counters;     // one arrival counter per workgroup column (zero between launches), or NULL
    int k_passes;           // K slices each wave walks through in turn
    int tiles_per_wg;       // 16-row weight tiles each workgroup walks through
    int tile_stride;        // distance between a workgroup's consecutive tiles (1 or gridDim.x)
    int vec_store;          // 1: 8-byte fp16 stores allowed
};

template <int KIND> struct StepK { static constexpr int value = kind_is_fp8(KIND) ? 128 : 64; };

// One K-step of weights for one 16-row tile, as loaded (32 bytes per lane).
struct WItem { u32x4 a, b; };   // plain: 32 B fp16; nested: upper, lower; e4m3: 32 B

// Buffer resource over a weight array: raw (unstructured) addressing with a byte range
// check, so reads past the end (N tail, look-ahead past the last tile) return zero
// without touching memory.  The arrays are smaller than 2 GiB (checked on the host), so an
// offset with bit 31 set is out of range by construction.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t weight_rsrc(const uint8_t *base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(base), 0, bytes, 0x00020000);
}

constexpr uint32_t kDead = 0x80000000u;               // an offset no weight array reaches

// Where the weights of a K-step sit.  `voff` = lane part + tile part + the wave's slice; step S adds
// an immediate.  Row-major kinds: lane l = row l % 16, columns 16 (l / 16) .. + 15 of the step's 64
// (E4M3: of each 64-column half of the step's 128).  Packed kinds: lane l = chunk l of the block.
template <int KIND> struct WLayout {
    static constexpr bool PACKED = kind_is_packed(KIND);
    static constexpr int EB = kind_elem_bytes(KIND);
    static constexpr int KSTEP = StepK<KIND>::value;
    // bytes between consecutive K-steps of one tile
    static constexpr int STEP = PACKED ? (KSTEP / 64) * 1024 * EB : KSTEP * EB;
    // the second 16 bytes of a lane's step, relative to the first (NestedFP: the other plane, same offset)
    static constexpr int SECOND = kind_is_nested(KIND) ? 0
                                  : (KIND == kPlainF16 ? 16 : (PACKED ? 1024 : 64));
    // Cache policy of the weight loads.  Every weight is read once per launch.  Packed kinds fetch whole
    // 128-byte lines (a contiguous kilobyte per instruction) and mark them non-temporal (nt, bit 1),
    // so that they pass through L2 without displacing the activations and partial sums: the decode step
    // runs 5-8 % faster.  Row-major kinds take 64-byte pieces of a line, the other half follows in a
    // later instruction, and the same hint makes them 4-12 % slower (measured), so they keep the default.
#ifndef NFP_SMALL_POLICY
#define NFP_SMALL_POLICY 2
#endif
    static constexpr int POLICY = PACKED ? NFP_SMALL_POLICY : 0;
};

// Weights of K-step `S` of the wave's slice.  The whole offset is in the range-checked VGPR part of
// the address (the scalar offset is not range-checked).  va / vb: the lane's columns of the first /
// second 16 bytes lie inside K; otherwise the load is sent out of range and returns zero.
template <int KIND, int S>
__device__ __forceinline__ void load_w(WItem &r, __amdgpu_buffer_rsrc_t r0, __amdgpu_buffer_rsrc_t r1,
                                       uint32_t voff, bool va, bool vb) {
    typedef WLayout<KIND> L;
    const uint32_t oa = va ? voff : kDead, ob = vb ? voff : kDead;
    r.a = __builtin_amdgcn_raw_buffer_load_b128(r0, oa + S * L::STEP, 0, L::POLICY);
    r.b = __builtin_amdgcn_raw_buffer_load_b128(r1, ob + S * L::STEP + L::SECOND, 0, L::POLICY);
}

// Activations of one K-step for 16 tokens (32 bytes per lane); zero outside M and K.
template <int KIND>
__device__ __forceinline__ void load_x(u32x4 &xa, u32x4 &xb, const SmallParams &p, int m, int k) {
    const u32x4 zero = {0u, 0u, 0u, 0u};
    bool row_ok = m < p.M;
    if (kind_is_fp8(KIND)) {
        // same column order as the weight operand: 16 columns of each 64-column half
        const uint8_t *src = p.X + (int64_t)m * p.x_row_bytes + k;
        xa = (row_ok && k < p.K) ? *reinterpret_cast<const u32x4 *>(src) : zero;
        xb = (row_ok && (k + 64) < p.K) ? *reinterpret_cast<const u32x4 *>(src + 64) : zero;
    } else {
        const uint8_t *src = p.X + (int64_t)m * p.x_row_bytes + 2 * (int64_t)k;
        bool ok = row_ok && k < p.K;
        xa = ok ? *reinterpret_cast<const u32x4 *>(src) : zero;
        xb = ok ? *reinterpret_cast<const u32x4 *>(src + 16) : zero;
    }
}

__device__ __forceinline__ half8 as_half8(const u32x4 &v) {
    union { u32x4 u; half8 h; } c;
    c.u = v;
    return c.h;
}

// Turns the raw weight bytes of one step into MFMA operands (merges the planes if nested).
template <int KIND>
__device__ __forceinline__ void prep_w(const WItem &w, u32x4 &w_lo, u32x4 &w_hi) {
    if (kind_is_nested(KIND)) {
        merge16(w.a, w.b, w_lo, w_hi);             // Sec. 4.2, Alg. 1
    } else {
        w_lo = w.a;
        w_hi = w.b;
    }
}

template <int KIND>
__device__ __forceinline__ floatx4 mma_step(const u32x4 &w_lo, const u32x4 &w_hi, const u32x4 &xa,
                                            const u32x4 &xb, floatx4 acc) {
    if (kind_is_fp8(KIND)) {
        intx8 a, b;
        a[0] = w_lo.x; a[1] = w_lo.y; a[2] = w_lo.z; a[3] = w_lo.w;
        a[4] = w_hi.x; a[5] = w_hi.y; a[6] = w_hi.z; a[7] = w_hi.w;
        b[0] = xa.x; b[1] = xa.y; b[2] = xa.z; b[3] = xa.w;
        b[4] = xb.x; b[5] = xb.y; b[6] = xb.z; b[7] = xb.w;
        // E4M3 x E4M3, unit block scales
        return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, acc, 0, 0, 0, 0, 0, 0);
    } else {
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(w_lo), as_half8(xa), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(w_hi), as_half8(xb), acc, 0, 0, 0);
        return acc;
    }
}

template <int KIND, int SPW, int S = 0>
struct FetchTile {
    static __device__ __forceinline__ void run(WItem (&w)[SPW], __amdgpu_buffer_rsrc_t r0,
                                               __amdgpu_buffer_rsrc_t r1, uint32_t voff,
                                               const bool (&va)[SPW], const bool (&vb)[SPW]) {
        if constexpr (KIND == kNestedF16 && S == 0) {
            // packed planes: the tile's blocks of the upper plane first, then those of the lower plane,
            // two runs of consecutive kilobytes instead of an alternation between two distant arrays
            // (about 1 % on the decode step, timed against the plain kernel of the same run as control)
            typedef WLayout<KIND> L;
#pragma unroll
            for (int q = 0; q < SPW; ++q)
                w[q].a = __builtin_amdgcn_raw_buffer_load_b128(r0, (va[q] ? voff : kDead) + q * L::STEP, 0, L::POLICY);
#pragma unroll
            for (int q = 0; q < SPW; ++q)
                w[q].b = __builtin_amdgcn_raw_buffer_load_b128(r1, (vb[q] ? voff : kDead) + q * L::STEP + L::SECOND, 0, L::POLICY);
        } else {
            load_w<KIND, S>(w[S], r0, r1, voff, va[S], vb[S]);
            FetchTile<KIND, SPW, S + 1>::run(w, r0, r1, voff, va, vb);
        }
    }
};
template <int KIND, int SPW>
struct FetchTile<KIND, SPW, SPW> {
    static __device__ __forceinline__ void run(WItem (&)[SPW], __amdgpu_buffer_rsrc_t, __amdgpu_buffer_rsrc_t,
                                               uint32_t, const bool (&)[SPW], const bool (&)[SPW]) {}
};

// Activation-stationary streaming kernel.
//   workgroup = up to 16 waves; wave w owns the K-slice [w*SPW*KSTEP, (w+1)*SPW*KSTEP) of
//   grid slice blockIdx.y and keeps the activations of that slice in registers for the whole
//   kernel; the workgroup walks through `tiles_per_wg` 16-row weight tiles, so each wave
//   streams 16 rows x (SPW*KSTEP) contiguous K per tile.  Two tile buffers swap roles
//   (no copies, no branch in the loop body): the loads of tile t+1 are in flight while
//   tile t is merged and multiplied.  Per-tile partial sums go to LDS and are reduced
//   across the waves once, at the end, in fixed wave order.
template <int KIND, int MT, int SPW, bool MULTIPASS>
__global__ void __launch_bounds__((MT == 4 || SPW == 8) ? 512 : 1024)
small_gemm_kernel(SmallParams p) {
    extern __shared__ float lds[];                    // [tile][wave][MT][64] x float4
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int waves = blockDim.x >> 6;
    const int g = lane >> 4;
    const int r16 = lane & 15;
    const int slice = blockIdx.y;
    constexpr int KSTEP = StepK<KIND>::value;
    constexpr int KLANE = 16;                         // first column of lane group g within a step: 16*g
    const int tiles_total = (p.N + 15) >> 4;
    // a workgroup's tiles: a contiguous chunk (stride 1) or interleaved with the other
    // workgroups (stride gridDim.x), so that the chip sweeps the weights front to back
    const int tstride = p.tile_stride;
    const int tile0 = tstride == 1 ? blockIdx.x * p.tiles_per_wg : blockIdx.x;
    const int T = tstride == 1 ? min(p.tiles_per_wg, tiles_total - tile0)
                               : (tiles_total - tile0 + tstride - 1) / tstride;
    floatx4 *slots = reinterpret_cast<floatx4 *>(lds);
    const __amdgpu_buffer_rsrc_t rs0 = weight_rsrc(p.W0, p.w_bytes);
    const __amdgpu_buffer_rsrc_t rs1 = weight_rsrc(kind_is_nested(KIND) ? p.W1 : p.W0, p.w_bytes);
    const uint32_t tile_bytes = p.tile_bytes;
    typedef WLayout<KIND> L;

    // with several K passes this wave's partial tiles live in LDS and start at zero
    // (the spare slot of an odd T included)
    if (MULTIPASS)
        for (int tile = 0; tile < ((T + 1) & ~1); ++tile)
#pragma unroll
            for (int i = 0; i < MT; ++i)
                slots[((tile * waves + wave) * MT + i) * 64 + lane] = floatx4{0.f, 0.f, 0.f, 0.f};

    // Long rows take several passes: in pass q the wave owns K-slice (slice*passes + q)*waves
    // + wave, reloads the activations of that slice and walks the same tiles again, adding
    // to its partial tiles in LDS.
    u32x4 xa[SPW][MT], xb[SPW][MT];
    uint32_t voff = 0;
    bool va[SPW], vb[SPW];                            // this lane's columns of step s lie inside K

    auto fetch = [&](WItem (&w)[SPW], int tile) {
        // past the last tile every lane is sent out of range
        const uint32_t base = tile < T ? voff + (uint32_t)(tile0 + tile * tstride) * tile_bytes : kDead;
        FetchTile<KIND, SPW>::run(w, rs0, rs1, base, va, vb);
    };
    auto consume = [&](const WItem (&w)[SPW], int tile) {
        floatx4 acc[MT];
#pragma unroll
        for (int i = 0; i < MT; ++i)
            acc[i] = MULTIPASS ? slots[((tile * waves + wave) * MT + i) * 64 + lane] : floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < SPW; ++s) {
            u32x4 w_lo, w_hi;
            prep_w<KIND>(w[s], w_lo, w_hi);
#pragma unroll
            for (int i = 0; i < MT; ++i) acc[i] = mma_step<KIND>(w_lo, w_hi, xa[s][i], xb[s][i], acc[i]);
        }
#pragma unroll
        for (int i = 0; i < MT; ++i) slots[((tile * waves + wave) * MT + i) * 64 + lane] = acc[i];
    };

    WItem buf0[SPW], buf1[SPW];
    __shared__ uint32_t row_max[16 * 16];             // kE4M3Quant: per wave and token row
    float row_scale = 1.0f;
    const int passes = MULTIPASS ? p.k_passes : 1;
    for (int pass = 0; pass < passes; ++pass) {
        const int k_wave = ((slice * passes + pass) * waves + wave) * (SPW * KSTEP) + KLANE * g;
        if (L::PACKED) voff = (uint32_t)lane * 16u + (uint32_t)((k_wave - KLANE * g) >> 6) * (1024u * L::EB);   // block column of the slice
        else voff = (uint32_t)r16 * p.w_row_bytes + (uint32_t)k_wave * (uint32_t)L::EB;
#pragma unroll
        for (int s = 0; s < SPW; ++s) {
            va[s] = k_wave + s * KSTEP < p.K;
            vb[s] = kind_is_fp8(KIND) ? k_wave + s * KSTEP + 64 < p.K : va[s];
        }
        if (KIND == kE4M3Quant) {
            // Fused activation quantisation (Sec. 2.2 per-token scaling; one token tile, the
            // workgroup covers all of K): every wave loads the FP16 activations of its own slice,
            // the row maxima are combined through LDS, and each lane converts what it holds --
            // the same divisions and conversions as the stand-alone kernel, no Xq round trip.
            u32x4 xr[SPW][4];
            const bool row_ok = r16 < p.M;
#pragma unroll
            for (int s = 0; s < SPW; ++s) {
                const int k = k_wave + s * KSTEP;
                const uint8_t *src = p.X + (int64_t)r16 * p.x_row_bytes + 2 * (int64_t)k;
                const bool ok0 = row_ok && k < p.K, ok1 = row_ok && (k + 64) < p.K;
                const u32x4 zero = {0u, 0u, 0u, 0u};
                xr[s][0] = ok0 ? *reinterpret_cast<const u32x4 *>(src) : zero;
                xr[s][1] = ok0 ? *reinterpret_cast<const u32x4 *>(src + 16) : zero;
                xr[s][2] = ok1 ? *reinterpret_cast<const u32x4 *>(src + 128) : zero;
                xr[s][3] = ok1 ? *reinterpret_cast<const u32x4 *>(src + 144) : zero;
            }
            fetch(buf0, 0);                            // the weights travel during the reduction
            float sc;
            if (p.static_scale) {
                sc = *p.static_scale;
            } else {
                uint32_t amax_bits = 0;                // |x| as an integer compare on the magnitude bits
#pragma unroll
                for (int s = 0; s < SPW; ++s)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const uint32_t w[4] = {xr[s][q].x, xr[s][q].y, xr[s][q].z, xr[s][q].w};
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            amax_bits = max(amax_bits, max(w[e] & 0x7fffu, (w[e] >> 16) & 0x7fffu));
                    }
                amax_bits = max(amax_bits, (uint32_t)__shfl_xor((int)amax_bits, 16, 64));
                amax_bits = max(amax_bits, (uint32_t)__shfl_xor((int)amax_bits, 32, 64));
                if (g == 0) row_max[wave * 16 + r16] = amax_bits;
                __syncthreads();
                uint32_t all = 0;
                for (int w2 = 0; w2 < waves; ++w2) all = max(all, row_max[w2 * 16 + r16]);
                const float amax = half_bits_to_float(all);
                sc = (amax == 0.0f) ? 1.0f : amax / 448.0f;
            }
            row_scale = sc;
            const float rc = 1.0f / sc;                // correctly rounded; see div_by_scale
#pragma unroll
            for (int s = 0; s < SPW; ++s) {
                if (p.quant_hw) {
                    xa[s][0] = u32x4{quant4<true>(xr[s][0].x, xr[s][0].y, sc, rc), quant4<true>(xr[s][0].z, xr[s][0].w, sc, rc),
                                     quant4<true>(xr[s][1].x, xr[s][1].y, sc, rc), quant4<true>(xr[s][1].z, xr[s][1].w, sc, rc)};
                    xb[s][0] = u32x4{quant4<true>(xr[s][2].x, xr[s][2].y, sc, rc), quant4<true>(xr[s][2].z, xr[s][2].w, sc, rc),
                                     quant4<true>(xr[s][3].x, xr[s][3].y, sc, rc), quant4<true>(xr[s][3].z, xr[s][3].w, sc, rc)};
                } else {
                    xa[s][0] = u32x4{quant4<false>(xr[s][0].x, xr[s][0].y, sc, rc), quant4<false>(xr[s][0].z, xr[s][0].w, sc, rc),
                                     quant4<false>(xr[s][1].x, xr[s][1].y, sc, rc), quant4<false>(xr[s][1].z, xr[s][1].w, sc, rc)};
                    xb[s][0] = u32x4{quant4<false>(xr[s][2].x, xr[s][2].y, sc, rc), quant4<false>(xr[s][2].z, xr[s][2].w, sc, rc),
                                     quant4<false>(xr[s][3].x, xr[s][3].y, sc, rc), quant4<false>(xr[s][3].z, xr[s][3].w, sc, rc)};
                }
            }
        } else {
#pragma unroll
            for (int s = 0; s < SPW; ++s)
#pragma unroll
                for (int i = 0; i < MT; ++i) load_x<KIND>(xa[s][i], xb[s][i], p, 16 * i + r16, k_wave + s * KSTEP);
            fetch(buf0, 0);
        }
        // The scheduling barriers keep the compiler from sinking the look-ahead loads below the
        // multiplies (which would turn every wait into a full drain).  For odd T the last
        // half-trip multiplies zeros into a spare slot.
        for (int tile = 0; tile < T; tile += 2) {
            fetch(buf1, tile + 1);
            __builtin_amdgcn_sched_barrier(0);
            consume(buf0, tile);
            __builtin_amdgcn_sched_barrier(0);
            fetch(buf0, tile + 2);
            __builtin_amdgcn_sched_barrier(0);
            consume(buf1, tile + 1);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    __syncthreads();

    // ---- fixed-order reduction over the waves of the workgroup -----------------------------
    auto store_y = [&](floatx4 sum, int m, int n) {
        if (kind_is_fp8(KIND)) {
            float sc = (KIND == kE4M3Quant ? row_scale : p.scales[m]) * p.w_scale;
            sum.x = scale_f32(sum.x, sc); sum.y = scale_f32(sum.y, sc); sum.z = scale_f32(sum.z, sc); sum.w = scale_f32(sum.w, sc);
        }
        uint16_t *dst = p.Y + (int64_t)m * p.ldy + n;
        if (p.vec_store && n + 3 < p.N) {
            u32x2 o;
            o.x = float2_to_half2_bits(sum.x, sum.y);
            o.y = float2_to_half2_bits(sum.z, sum.w);
            *reinterpret_cast<u32x2 *>(dst) = o;
        } else {
            float v[4] = {sum.x, sum.y, sum.z, sum.w};
            for (int q = 0; q < 4 && n + q < p.N; ++q) {
                union { _Float16 f; uint16_t u; } cv;
                cv.f = (_Float16)v[q];
                dst[q] = cv.u;
            }
        }
    };
    // Partial sums of a grid-level K split.  Where the last workgroup to arrive finishes the sum
    // (p.counters), they are written through to memory and read back past the caches (cache policy
    // sc0 sc1, system scope): every XCD has an L2 of its own, and the alternative -- a release fence
    // in every workgroup, which writes back the whole L2, and an acquire fence, which invalidates
    // it -- made the kernel four times slower (measured).
    const bool fused = gridDim.y > 1 && p.counters != nullptr;
    constexpr int kThrough = 1 | 16;                  // buffer cache policy: sc0 | sc1
    const bool part_vec = (p.N & 3) == 0;
    const int64_t slice_elems = (int64_t)p.M * p.N;
    const __amdgpu_buffer_rsrc_t rpart = __builtin_amdgcn_make_buffer_rsrc(
        p.partials, 0, fused ? (uint32_t)(gridDim.y * slice_elems * 4) : 0u, 0x00020000);
    for (int item = wave; item < T * MT; item += waves) {
        const int tile = item / MT, i = item - tile * MT;
        floatx4 sum = slots[((tile * waves) * MT + i) * 64 + lane];
        for (int w2 = 1; w2 < waves; ++w2) {
            floatx4 v = slots[((tile * waves + w2) * MT + i) * 64 + lane];
            sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
        }
        const int m = 16 * i + r16;
        const int n = (tile0 + tile * tstride) * 16 + 4 * g;
        if (m >= p.M || n >= p.N) continue;
        if (gridDim.y > 1) {
            const int64_t e = ((int64_t)slice * p.M + m) * p.N + n;
            if (fused) {
                const uint32_t off = (uint32_t)(e * 4);
                if (part_vec) {
                    __builtin_amdgcn_raw_buffer_store_b128(u32x4{__float_as_uint(sum.x), __float_as_uint(sum.y),
                                                                 __float_as_uint(sum.z), __float_as_uint(sum.w)},
                                                           rpart, off, 0, kThrough);
                } else {
                    const float v[4] = {sum.x, sum.y, sum.z, sum.w};
                    for (int q = 0; q < 4 && n + q < p.N; ++q)
                        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v[q]), rpart, off + 4 * q, 0, kThrough);
                }
            } else {
                float *dst = p.partials + e;
                if (part_vec) {
                    *reinterpret_cast<floatx4 *>(dst) = sum;
                } else {
                    float v[4] = {sum.x, sum.y, sum.z, sum.w};
                    for (int q = 0; q < 4 && n + q < p.N; ++q) dst[q] = v[q];
                }
            }
        } else {
            store_y(sum, m, n);
        }
    }
    if (!fused) return;

    // ---- grid-level K split finished by the last workgroup to arrive -------------------------
    // Every workgroup of a tile column waits until its partial sums have reached memory, then takes
    // a ticket; the one that draws the last ticket adds the slices in slice order -- the order of
    // the stand-alone reduction kernel, so the result does not depend on who came last -- and
    // leaves the counter at zero for the next launch.  Nobody waits for anybody.
    __shared__ uint32_t ticket;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this lane's write-through stores are done
    __syncthreads();
    if (threadIdx.x == 0)
        ticket = __hip_atomic_fetch_add(&p.counters[blockIdx.x], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (ticket != gridDim.y - 1) return;
    for (int item = wave; item < T * MT; item += waves) {
        const int tile = item / MT, i = item - tile * MT;
        const int m = 16 * i + r16;
        const int n = (tile0 + tile * tstride) * 16 + 4 * g;
        if (m >= p.M || n >= p.N) continue;
        const uint32_t off = (uint32_t)(((int64_t)m * p.N + n) * 4);
        const uint32_t sstep = (uint32_t)(slice_elems * 4);
        floatx4 sum;
        if (part_vec) {
            u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rpart, off, 0, kThrough);
            sum = floatx4{__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
            for (int s2 = 1; s2 < (int)gridDim.y; ++s2) {
                v = __builtin_amdgcn_raw_buffer_load_b128(rpart, off + s2 * sstep, 0, kThrough);
                sum.x += __uint_as_float(v.x); sum.y += __uint_as_float(v.y);
                sum.z += __uint_as_float(v.z); sum.w += __uint_as_float(v.w);
            }
        } else {
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            for (int q = 0; q < 4 && n + q < p.N; ++q) {
                v[q] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rpart, off + 4 * q, 0, kThrough));
                for (int s2 = 1; s2 < (int)gridDim.y; ++s2)
                    v[q] += __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rpart, off + s2 * sstep + 4 * q, 0, kThrough));
            }
            sum = floatx4{v[0], v[1], v[2], v[3]};
        }
        store_y(sum, m, n);
    }
    if (threadIdx.x == 0) __hip_atomic_store(&p.counters[blockIdx.x], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Sums the S split-K partials in slice order, applies the FP8-mode scale, writes fp16.
// VEC: four consecutive columns per lane (needs N % 4 == 0 and 8-byte aligned output rows).
template <bool VEC>
__global__ void __launch_bounds__(256)
splitk_reduce_kernel(const float *__restrict__ partials, int S, int M, int N, const float *scales,
                     float w_scale, uint16_t *__restrict__ Y, int64_t ldy) {
    constexpr int W = VEC ? 4 : 1;
    const int64_t total = (int64_t)M * N;
    const int64_t idx = ((int64_t)blockIdx.x * 256 + threadIdx.x) * W;
    if (idx >= total) return;
    const int m = (int)(idx / N), n = (int)(idx - (int64_t)m * N);
    float v[W];
    if (VEC) {
        floatx4 t = *reinterpret_cast<const floatx4 *>(partials + idx);
        v[0] = t.x; v[W > 1 ? 1 : 0] = t.y; v[W > 2 ? 2 : 0] = t.z; v[W > 3 ? 3 : 0] = t.w;
        for (int s = 1; s < S; ++s) {
            floatx4 u = *reinterpret_cast<const floatx4 *>(partials + (int64_t)s * total + idx);
            v[0] += u.x; v[W > 1 ? 1 : 0] += u.y; v[W > 2 ? 2 : 0] += u.z; v[W > 3 ? 3 : 0] += u.w;
        }
    } else {
        v[0] = partials[idx];
        for (int s = 1; s < S; ++s) v[0] += partials[(int64_t)s * total + idx];
    }
    const float sc = scales ? scales[m] * w_scale : 1.0f;
    uint16_t *dst = Y + (int64_t)m * ldy + n;
    if (VEC) {
        u32x2 o;
        o.x = float2_to_half2_bits(scales ? scale_f32(v[0], sc) : v[0], scales ? scale_f32(v[W > 1 ? 1 : 0], sc) : v[W > 1 ? 1 : 0]);
        o.y = float2_to_half2_bits(scales ? scale_f32(v[W > 2 ? 2 : 0], sc) : v[W > 2 ? 2 : 0],
                                   scales ? scale_f32(v[W > 3 ? 3 : 0], sc) : v[W > 3 ? 3 : 0]);
        *reinterpret_cast<u32x2 *>(dst) = o;
    } else {
        union { _Float16 f; uint16_t u; } c;
        c.f = (_Float16)(scales ? scale_f32(v[0], sc) : v[0]);
        dst[0] = c.u;
    }
}

int launch_splitk_reduce(const float *partials, int S, int64_t M, int64_t N, const float *scales,
                         float w_scale, uint16_t *Y, int64_t ldy, hipStream_t stream) {
    const int64_t total = M * N;
    const bool vec = (N & 3) == 0 && (ldy & 3) == 0 && (reinterpret_cast<uintptr_t>(Y) & 7) == 0 &&
                     (reinterpret_cast<uintptr_t>(partials) & 15) == 0;
    if (vec)
        splitk_reduce_kernel<true><<<(unsigned)((total / 4 + 255) / 256), 256, 0, stream>>>(
            partials, S, (int)M, (int)N, scales, w_scale, Y, ldy);
    else
        splitk_reduce_kernel<false><<<(unsigned)((total + 255) / 256), 256, 0, stream>>>(
            partials, S, (int)M, (int)N, scales, w_scale, Y, ldy);
    return hip_ok(hipGetLastError());
}

// ---- host-side configuration ---------------------------------------------------------
struct SmallConfig { int mt, spw, waves, split, passes, tiles_per_wg; };

// Launch shapes of the streaming kernel that were timed faster than the rules below choose, on the
// layer shapes of the models the paper evaluates (Sec. 5.1), for batches of up to 16 tokens.
struct TunedSmall { int cls, N, K, spw, split, tiles; };
static const TunedSmall kTunedSmall[] = {
#include "tuned_small.inc"
    {-1, 0, 0, 0, 0, 0},
};

static SmallConfig choose_small(int kind, int64_t M, int64_t N, int64_t K) {
    const Tuning &t = tuning();
    SmallConfig c;
    c.mt = M <= 16 ? 1 : (M <= 32 ? 2 : 4);
    // knobs first; with none set, the table of timed shapes; otherwise the rules
    int64_t k_spw = t.small_spw, k_split = t.small_split, k_tiles = t.small_tiles;
    if (k_spw <= 0 && k_split <= 0 && k_tiles <= 0 && t.tuned_table != 0 && c.mt == 1) {
        for (const TunedSmall &e : kTunedSmall)
            if (e.cls == kind_class(kind) && e.N == N && e.K == K) {
                k_spw = e.spw;  k_split = e.split;  k_tiles = e.tiles;
                break;
            }
    }
    const bool fp8 = kind_is_fp8(kind), nested = kind_class(kind) == 1;
    const int kstep = fp8 ? 128 : 64;
    const int steps = (int)((K + kstep - 1) / kstep);
    // Row-major FP16 weights (the plain baseline) stream best in long runs per row: 8 K-steps per
    // wave (512 contiguous bytes of each row), 8 waves (measured: 8-10 % faster than 4 x 16);
    // the packed planes are contiguous per tile whatever the slice and gain nothing from it.
    const bool can_long = (kind == kPlainF16 || kind == kNestedF16Row) && M <= 16 && (K + 63) / 64 >= 64;
    const bool long_slices = can_long && (k_spw == 8 || (kind == kPlainF16 && k_spw <= 0));
    const int max_waves = (c.mt == 4 || long_slices) ? 8 : 16;     // four token tiles need 256 VGPRs per wave
    const int64_t tiles = (N + 15) / 16;
    // K-steps per wave: 2 with several token tiles (their activations need the registers) and
    // for large layers (measured: two passes of short slices beat one pass of long ones);
    // otherwise 4, or 2 if that still lets one workgroup cover all of K
    c.spw = 4;
    if ((steps + 3) / 4 < 16 && steps >= 2) c.spw = 2;
    if (tiles >= 1024 && !nested) c.spw = 2;
    if (k_spw == 2 || k_spw == 4) c.spw = (int)k_spw;
    if (c.mt > 1) c.spw = 2;
    if (long_slices) c.spw = 8;
    const int slices = (steps + c.spw - 1) / c.spw;               // wave-sized K slices
    // Grid-level split of K (fp32 partials + a second kernel): small layers run faster as
    // about a thousand short workgroups than as a few hundred wide ones, so K is split by
    // the largest power of two that keeps tiles*split <= 1024 (at most 8: the scratch stays
    // below 8*M*N floats).  What 16 waves x split do not cover is walked in passes.
    const int rounds = (slices + max_waves - 1) / max_waves;
    // E4M3 layers move half the bytes: half as many workgroups, unless K needs passes anyway
    const int64_t wg_target = (fp8 && rounds == 1) ? 512 : 1024;
    int split = 1;
    while (split < 8 && tiles * (split * 2) <= wg_target) split *= 2;
    // measured with packed planes: a single token tile whose K fits one pass is as fast
    // unsplit once there is a tile per CU, and saves the reduction launch
    if (c.mt == 1 && rounds == 1 && tiles >= 256) split = 1;
    // ... except FP16 weights on layers of one or two tiles per CU: two K slices per tile column and
    // twice the tiles per workgroup leave the workgroup count alone, halve the activations every
    // workgroup has to fetch, and the last workgroup of a column sums the two slices itself
    // (measured on 4096 x 4096 and 6144 x 4096 at 16 tokens: 13.3 -> 12.0 and 16.1 -> 15.3 us per call)
    const bool pair_slices = !fp8 && c.mt == 1 && rounds == 1 && tiles >= 256 && tiles <= 512 && slices >= 2 &&
                             t.fused_reduce != 0;
    if (pair_slices) split = 2;
    if (k_split > 0) split = (int)k_split;
    if (split > slices) split = slices;
    c.split = split;
    c.passes = (rounds + split - 1) / split;
    c.waves = (slices + split * c.passes - 1) / (split * c.passes);
    if (c.waves > max_waves) {                                    // cannot happen; keep the launch legal
        c.waves = max_waves;
        c.passes = (slices + split * max_waves - 1) / (split * max_waves);
    }
    // Tiles per workgroup.  A workgroup keeps a kilobyte of partial sums per tile and wave in LDS (an
    // even number of slots, 128 KB at most).  The launch runs in rounds of one workgroup per CU and is
    // bound by the weight stream, which 224 workgroups fill; with fewer each one gets faster, but only
    // up to about twice as fast on an empty chip.  A round of R workgroups therefore costs its tiles
    // times R / 256 from 224 workgroups on and 0.875 (1 - 0.43 (224 - R) / 224) below (fitted to
    // timings of 1 ... 12 tiles per workgroup on eight layer shapes), plus half a tile for its ramp and
    // tail.  Cheapest wins, the larger count on a tie (fewer workgroups fetch the activations).
    const int slots_max = 128 / (c.waves * c.mt);
    int per_max = slots_max & ~1;                      // (an odd count takes a spare slot)
    if (per_max < 1) per_max = 1;
    if (per_max > 16) per_max = 16;
    int64_t per = 1;
    double best = 1e30;
    for (int cand = 1; cand <= per_max; ++cand) {
        const int64_t wgs = ((tiles + cand - 1) / cand) * c.split;
        const int64_t full = wgs / 256, rem = wgs % 256;
        const double part = rem >= 224 ? (double)rem / 256.0 : 0.875 * (1.0 - 0.43 * (double)(224 - rem) / 224.0);
        double cost = (double)cand * ((double)full + (rem ? part : 0.0)) + 0.5 * (double)(full + (rem ? 1 : 0));
        if (cost <= best) { best = cost;  per = cand; }
    }
    if (pair_slices && k_split <= 0) per = 2 * ((tiles + 255) / 256);
    if (k_tiles > 0) per = k_tiles;
    if (per > per_max) per = per_max;
    if (per < 1) per = 1;
    c.tiles_per_wg = (int)per;
    return c;
}

bool small_gemm_supports(int kind, int64_t M, int64_t N, int64_t K, int64_t ldw) {
    // the weight array must be addressable with 31-bit byte offsets (bit 31 marks a load as dead),
    // a few tiles of slack included
    (void)M;
    return weight_array_bytes(kind, N + 48, K, ldw) < ((int64_t)1 << 31);
}

size_t small_gemm_partial_bytes(int kind, int64_t M, int64_t N, int64_t K) {
    SmallConfig c = choose_small(kind, M, N, K);
    return c.split > 1 ? (size_t)c.split * (size_t)M * (size_t)N * sizeof(float) : 0;
}

template <int KIND, int MT, int SPW>
static void launch_small_t(const SmallParams &p, const SmallConfig &c, dim3 grid, hipStream_t stream) {
    size_t lds = (size_t)((c.tiles_per_wg + 1) & ~1) * c.waves * MT * 64 * sizeof(floatx4);
    auto kern1 = small_gemm_kernel<KIND, MT, SPW, false>;
    auto kernp = small_gemm_kernel<KIND, MT, SPW, true>;
    static std::atomic<bool> attr_set{false};                    // once per instantiation
    if (!attr_set.load(std::memory_order_acquire)) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern1),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernp),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
        attr_set.store(true, std::memory_order_release);
    }
    if (c.passes > 1) kernp<<<grid, c.waves * 64, lds, stream>>>(p);
    else kern1<<<grid, c.waves * 64, lds, stream>>>(p);
}

// The fused-quantisation kind exists for one token tile, one K pass and no grid split only.
static void launch_small_quant(const SmallParams &p, const SmallConfig &c, dim3 grid, hipStream_t stream) {
    size_t lds = (size_t)((c.tiles_per_wg + 1) & ~1) * c.waves * 64 * sizeof(floatx4);
    auto k2 = small_gemm_kernel<kE4M3Quant, 1, 2, false>;
    auto k4 = small_gemm_kernel<kE4M3Quant, 1, 4, false>;
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k2), hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k4), hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
        attr_set.store(true, std::memory_order_release);
    }
    if (c.spw == 2) k2<<<grid, c.waves * 64, lds, stream>>>(p);
    else k4<<<grid, c.waves * 64, lds, stream>>>(p);
}

bool small_gemm_fuses_quant(int64_t M, int64_t N, int64_t K) {
    // Off unless asked for: every workgroup has to convert all of its 16 x K activations
    // itself, which costs more VALU time per CU (measured 3-6 us per call at K = 4096) than
    // the separate quantisation launch it saves.
    if (tuning().small_fuse_quant <= 0) return false;
    SmallConfig c = choose_small(kE4M3, M, N, K);
    return c.mt == 1 && c.split == 1 && c.passes == 1;
}

template <int KIND>
static void launch_small_k(const SmallParams &p, const SmallConfig &c, dim3 grid, hipStream_t stream) {
    if constexpr (KIND == kPlainF16 || KIND == kNestedF16Row) {
        if (c.mt == 1 && c.spw == 8) { launch_small_t<KIND, 1, 8>(p, c, grid, stream);  return; }
    }
    switch (c.mt * 10 + c.spw) {
        case 14: launch_small_t<KIND, 1, 4>(p, c, grid, stream); break;
        case 12: launch_small_t<KIND, 1, 2>(p, c, grid, stream); break;
        case 22: launch_small_t<KIND, 2, 2>(p, c, grid, stream); break;
        default: launch_small_t<KIND, 4, 2>(p, c, grid, stream); break;
    }
}

int launch_small_gemm(int kind, const GemmArgs &a, hipStream_t stream) {
    SmallConfig c = choose_small(kind, a.M, a.N, a.K);
    SmallParams p;
    p.X = static_cast<const uint8_t *>(a.X);
    p.x_row_bytes = (kind == kE4M3 || kind == kE4M3Row) ? a.ldx : 2 * a.ldx;
    p.scales = a.scales;
    p.static_scale = a.static_scale;
    p.quant_hw = tuning().quant_hw != 0 ? 1 : 0;
    p.w_scale = a.w_scale;
    p.W0 = static_cast<const uint8_t *>(a.W0);
    p.W1 = static_cast<const uint8_t *>(a.W1);
    if (kind_is_packed(kind)) {
        // 16 rows of a tile take 16 * Kp contiguous elements (Kp = K rounded up to 64)
        p.w_row_bytes = 0;
        p.tile_bytes = (uint32_t)(((a.K + 63) / 64) * 1024 * kind_elem_bytes(kind));
    } else {
        p.w_row_bytes = (uint32_t)(kind == kPlainF16 ? 2 * a.ldw : a.K);
        p.tile_bytes = 16u * p.w_row_bytes;
    }
    p.w_bytes = (uint32_t)weight_array_bytes(kind, a.N, a.K, a.ldw);
    p.M = (int)a.M;  p.N = (int)a.N;  p.K = (int)a.K;
    p.Y = a.Y;  p.ldy = a.ldy;
    p.partials = a.partials;
    p.tiles_per_wg = c.tiles_per_wg;
    const int64_t tiles = (a.N + 15) / 16;
    const unsigned grid_x = (unsigned)((tiles + c.tiles_per_wg - 1) / c.tiles_per_wg);
    // the last workgroup of a tile column sums the K slices itself where there is a counter for it
    const bool fused_reduce = c.split > 1 && a.counters != nullptr && grid_x <= (unsigned)kMaxCounters &&
                              (int64_t)c.split * a.M * a.N * 4 < ((int64_t)1 << 32) && tuning().fused_reduce != 0;
    p.counters = fused_reduce ? a.counters : nullptr;
    p.k_passes = c.passes;
    p.tile_stride = (tuning().small_interleave != 0 && c.tiles_per_wg > 1) ? (int)grid_x : 1;
    p.vec_store = ((a.N & 3) == 0 && (a.ldy & 3) == 0 && (reinterpret_cast<uintptr_t>(a.Y) & 7) == 0) ? 1 : 0;
    if (c.split > 1 && (a.partials == nullptr ||
                        a.partial_bytes < (size_t)c.split * a.M * a.N * sizeof(float)))
        return kErrWorkspace;
    dim3 grid(grid_x, (unsigned)c.split);
    if (kind == kE4M3Quant && !(c.mt == 1 && c.split == 1 && c.passes == 1)) return kErrArg;   // caller checks first
    switch (kind) {
        case kPlainF16: launch_small_k<kPlainF16>(p, c, grid, stream); break;
        case kPlainF16Packed: launch_small_k<kPlainF16Packed>(p, c, grid, stream); break;
        case kNestedF16: launch_small_k<kNestedF16>(p, c, grid, stream); break;
        case kNestedF16Row: launch_small_k<kNestedF16Row>(p, c, grid, stream); break;
        case kE4M3Quant: launch_small_quant(p, c, grid, stream); break;
        case kE4M3Row: launch_small_k<kE4M3Row>(p, c, grid, stream); break;
        case kE4M3: launch_small_k<kE4M3>(p, c, grid, stream); break;
        default: return kErrArg;
    }
    if (hipGetLastError() != hipSuccess) return kErrHip;
    if (c.split > 1 && !fused_reduce)
        return launch_splitk_reduce(a.partials, c.split, a.M, a.N, kind_is_fp8(kind) ? a.scales : nullptr,
                                    a.w_scale, a.Y, a.ldy, stream);
    return kOk;
}

}  // namespace nfp
