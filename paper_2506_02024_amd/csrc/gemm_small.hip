// Streaming GEMM for decode-sized batches (M <= 64): Y = X * W^T with the weight stream
// read exactly once from HBM and nothing staged in LDS (no weight reuse across waves).
// The paper's sweep starts at M = 32 with T_m >= 16 (Sec. 5.2, App. C); below that the
// linear layer is bound by HBM bandwidth, so the kernel is built around 128-bit loads of
// the byte planes with many loads in flight, K split across the waves of a workgroup and
// a fixed-order reduction.
//
// One wave owns NT tiles of 16 weight rows and MT tiles of 16 tokens.  Weight rows are the
// MFMA "A" operand (lane l: row l%16, K-group l/16), tokens the "B" operand, so each lane
// ends up with 4 consecutive output columns of one token: 8-byte stores of fp16.
//   kPlainF16 : lane loads 32 B of FP16 weights             -> 2 x v_mfma_f32_16x16x32_f16
//   kNestedF16: lane loads 16 B upper + 16 B lower, merges them (Sec. 4.2, Alg. 1) -> same
//   kE4M3     : lane loads 32 B of E4M3 bytes (upper plane)  -> 1 x v_mfma_f32_16x16x128_f8f6f4
#include "nfp_device.h"
#include "nfp_host.h"

namespace nfp {

struct SmallParams {
    const uint8_t *X;       // fp16 X (as bytes) or E4M3 Xq
    int64_t x_row_bytes;    // row stride of X in bytes
    const float *scales;    // [M] (kE4M3) or NULL
    float w_scale;
    const uint8_t *W0;      // fp16 W (bytes) / upper plane / E4M3 weights
    const uint8_t *W1;      // lower plane
    int64_t w_row_bytes;    // row stride of W0 (and W1) in bytes
    int M, N, K;
    uint16_t *Y;
    int64_t ldy;
    float *partials;        // [S][M][N] when S > 1
    int steps_total;        // K-steps over the whole K
    int steps_per_part;     // K-steps per (slice, wave) part
    int vec_store;          // 1: 8-byte fp16 stores allowed
};

template <int KIND> struct StepK { static constexpr int value = (KIND == kE4M3) ? 128 : 64; };

// Raw per-step operands of one lane.
template <int KIND> struct WRaw { u32x4 a, b; };   // plain: 32 B fp16; nested: upper, lower; e4m3: 32 B

template <int KIND>
__device__ __forceinline__ void load_w(WRaw<KIND> &r, const SmallParams &p, int row, int k0, int g,
                                       bool row_ok) {
    // k0: first K index of the step; g: lane's K-group (0..3)
    const u32x4 zero = {0u, 0u, 0u, 0u};
    if (KIND == kPlainF16) {
        int k = k0 + 16 * g;
        bool ok = row_ok && k < p.K;
        const u32x4 *src = reinterpret_cast<const u32x4 *>(p.W0 + (int64_t)row * p.w_row_bytes + 2 * (int64_t)k);
        r.a = ok ? __builtin_nontemporal_load(src) : zero;
        r.b = ok ? __builtin_nontemporal_load(src + 1) : zero;
    } else if (KIND == kNestedF16) {
        int k = k0 + 16 * g;
        bool ok = row_ok && k < p.K;
        int64_t off = (int64_t)row * p.w_row_bytes + k;
        r.a = ok ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p.W0 + off)) : zero;
        r.b = ok ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p.W1 + off)) : zero;
    } else {
        int k = k0 + 32 * g;
        int64_t off = (int64_t)row * p.w_row_bytes + k;
        bool ok0 = row_ok && k < p.K, ok1 = row_ok && (k + 16) < p.K;
        r.a = ok0 ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p.W0 + off)) : zero;
        r.b = ok1 ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p.W0 + off + 16)) : zero;
    }
}

template <int KIND>
__device__ __forceinline__ void load_x(u32x4 &xa, u32x4 &xb, const SmallParams &p, int m, int k0, int g) {
    const u32x4 zero = {0u, 0u, 0u, 0u};
    bool row_ok = m < p.M;
    if (KIND == kE4M3) {
        int k = k0 + 32 * g;
        const uint8_t *src = p.X + (int64_t)m * p.x_row_bytes + k;
        xa = (row_ok && k < p.K) ? *reinterpret_cast<const u32x4 *>(src) : zero;
        xb = (row_ok && (k + 16) < p.K) ? *reinterpret_cast<const u32x4 *>(src + 16) : zero;
    } else {
        int k = k0 + 16 * g;
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
__device__ __forceinline__ void prep_w(const WRaw<KIND> &w, u32x4 &w_lo, u32x4 &w_hi) {
    if (KIND == kNestedF16) {
        merge16(w.a, w.b, w_lo, w_hi);
    } else {
        w_lo = w.a;
        w_hi = w.b;
    }
}

template <int KIND>
__device__ __forceinline__ floatx4 mma_step(const u32x4 &w_lo, const u32x4 &w_hi, const u32x4 &xa,
                                            const u32x4 &xb, floatx4 acc) {
    if (KIND == kE4M3) {
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

// Wave cap per workgroup: 16, or 8 where the accumulators and two steps of operands need
// more than 128 VGPRs (8 or more 16x16 tiles per wave).
constexpr int small_max_waves(int mt, int nt) { return mt * nt >= 8 ? 8 : 16; }

template <int KIND, int MT, int NT, int U>
__global__ void __launch_bounds__(64 * small_max_waves(MT, NT))
small_gemm_kernel(SmallParams p) {
    extern __shared__ float lds[];                    // [waves][MT*NT][64][4]
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int waves = blockDim.x >> 6;
    const int g = lane >> 4;
    const int r16 = lane & 15;
    const int n_base = blockIdx.x * (NT * 16);
    const int slice = blockIdx.y;
    constexpr int KSTEP = StepK<KIND>::value;

    // this wave's contiguous range of K-steps
    const int part = slice * waves + wave;
    int t_begin = part * p.steps_per_part;
    int t_end = min(t_begin + p.steps_per_part, p.steps_total);

    floatx4 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    int rows[NT];
    bool rows_ok[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        rows[j] = n_base + 16 * j + r16;
        rows_ok[j] = rows[j] < p.N;
    }

    for (int t0 = t_begin; t0 < t_end; t0 += U) {
        WRaw<KIND> w[U][NT];
        u32x4 xa[U][MT], xb[U][MT];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int k0 = (t0 + u) * KSTEP;
            bool live = (t0 + u) < t_end;
#pragma unroll
            for (int j = 0; j < NT; ++j) load_w<KIND>(w[u][j], p, rows[j], k0, g, rows_ok[j] && live);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int k0 = (t0 + u) * KSTEP;
            // dead steps read X in bounds of K or get zeros from the K guard; weights are zero
#pragma unroll
            for (int i = 0; i < MT; ++i) load_x<KIND>(xa[u][i], xb[u][i], p, 16 * i + r16, k0, g);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                u32x4 w_lo, w_hi;
                prep_w<KIND>(w[u][j], w_lo, w_hi);
#pragma unroll
                for (int i = 0; i < MT; ++i)
                    acc[i][j] = mma_step<KIND>(w_lo, w_hi, xa[u][i], xb[u][i], acc[i][j]);
            }
    }

    // ---- fixed-order reduction over the waves of the workgroup --------------------------
    constexpr int TILES = MT * NT;
    floatx4 *slots = reinterpret_cast<floatx4 *>(lds);
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) slots[(wave * TILES + i * NT + j) * 64 + lane] = acc[i][j];
    __syncthreads();
    for (int tile = wave; tile < TILES; tile += waves) {
        const int i = tile / NT, j = tile - i * NT;
        floatx4 sum = slots[tile * 64 + lane];
        for (int w2 = 1; w2 < waves; ++w2) {
            floatx4 v = slots[(w2 * TILES + tile) * 64 + lane];
            sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
        }
        const int m = 16 * i + r16;
        const int n = n_base + 16 * j + 4 * g;
        if (m >= p.M || n >= p.N) continue;
        if (gridDim.y > 1) {
            float *dst = p.partials + ((int64_t)slice * p.M + m) * p.N + n;
            if (n + 3 < p.N && (p.N & 3) == 0) {
                *reinterpret_cast<floatx4 *>(dst) = sum;
            } else {
                float v[4] = {sum.x, sum.y, sum.z, sum.w};
                for (int q = 0; q < 4 && n + q < p.N; ++q) dst[q] = v[q];
            }
        } else {
            if (KIND == kE4M3) {
                float s = p.scales[m] * p.w_scale;
                sum.x *= s; sum.y *= s; sum.z *= s; sum.w *= s;
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
                    union { _Float16 f; uint16_t u; } c;
                    c.f = (_Float16)v[q];
                    dst[q] = c.u;
                }
            }
        }
    }
}

// Sums the S split-K partials in slice order, applies the FP8-mode scale, writes fp16.
__global__ void __launch_bounds__(256)
splitk_reduce_kernel(const float *__restrict__ partials, int S, int M, int N, const float *scales,
                     float w_scale, uint16_t *__restrict__ Y, int64_t ldy) {
    int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t total = (int64_t)M * N;
    if (idx >= total) return;
    int m = (int)(idx / N), n = (int)(idx - (int64_t)m * N);
    float sum = partials[idx];
    for (int s = 1; s < S; ++s) sum += partials[(int64_t)s * total + idx];
    if (scales) sum *= scales[m] * w_scale;
    union { _Float16 f; uint16_t u; } c;
    c.f = (_Float16)sum;
    Y[(int64_t)m * ldy + n] = c.u;
}

int launch_splitk_reduce(const float *partials, int S, int64_t M, int64_t N, const float *scales,
                         float w_scale, uint16_t *Y, int64_t ldy, hipStream_t stream) {
    int64_t total = M * N;
    splitk_reduce_kernel<<<(unsigned)((total + 255) / 256), 256, 0, stream>>>(partials, S, (int)M, (int)N,
                                                                              scales, w_scale, Y, ldy);
    return hip_ok(hipGetLastError());
}

// ---- host-side configuration ---------------------------------------------------------
struct SmallConfig { int mt, nt, waves, split, u; };

static SmallConfig choose_small(int kind, int64_t M, int64_t N, int64_t K) {
    SmallConfig c;
    c.mt = M <= 16 ? 1 : (M <= 32 ? 2 : 4);
    c.nt = c.mt;                      // keeps activation reads (L2) equal to weight reads
    const Tuning &t = tuning();
    if (t.small_nt > 0) c.nt = (int)t.small_nt;
    if (c.nt != 1 && c.nt != 2 && c.nt != 4) c.nt = c.mt;
    int kstep = (kind == kE4M3) ? 128 : 64;
    int steps = (int)((K + kstep - 1) / kstep);
    int64_t groups = (N + 16 * c.nt - 1) / (16 * c.nt);
    // aim for ~4096 waves on the chip (16 per CU), at least 2 K-steps per wave
    int64_t want_parts = (4096 + groups - 1) / groups;
    int64_t max_parts = steps / 2 > 0 ? steps / 2 : 1;
    if (want_parts > max_parts) want_parts = max_parts;
    if (want_parts < 1) want_parts = 1;
    int max_waves = small_max_waves(c.mt, c.nt);      // LDS slots: waves * tiles KB <= 128 KB
    c.waves = (int)(want_parts < max_waves ? want_parts : max_waves);
    c.split = (int)((want_parts + c.waves - 1) / c.waves);
    if (c.split > 8) c.split = 8;
    if (t.small_waves > 0) c.waves = (int)(t.small_waves < max_waves ? t.small_waves : max_waves);
    if (t.small_split > 0) c.split = (int)t.small_split;
    if ((int64_t)c.waves * c.split > steps) {        // never more parts than K-steps
        c.split = 1;
        if (c.waves > steps) c.waves = steps;
    }
    c.u = 2;
    return c;
}

size_t small_gemm_partial_bytes(int kind, int64_t M, int64_t N, int64_t K) {
    SmallConfig c = choose_small(kind, M, N, K);
    return c.split > 1 ? (size_t)c.split * (size_t)M * (size_t)N * sizeof(float) : 0;
}

template <int KIND, int MT, int NT>
static void launch_small_t(const SmallParams &p, const SmallConfig &c, dim3 grid, hipStream_t stream) {
    size_t lds = (size_t)c.waves * MT * NT * 64 * sizeof(floatx4);
    auto kern = small_gemm_kernel<KIND, MT, NT, 2>;
    static bool attr_set = false;                    // once per instantiation
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
        attr_set = true;
    }
    kern<<<grid, c.waves * 64, lds, stream>>>(p);
}

template <int KIND>
static void launch_small_k(const SmallParams &p, const SmallConfig &c, dim3 grid, hipStream_t stream) {
    switch (c.mt * 10 + c.nt) {
        case 11: launch_small_t<KIND, 1, 1>(p, c, grid, stream); break;
        case 12: launch_small_t<KIND, 1, 2>(p, c, grid, stream); break;
        case 14: launch_small_t<KIND, 1, 4>(p, c, grid, stream); break;
        case 21: launch_small_t<KIND, 2, 1>(p, c, grid, stream); break;
        case 22: launch_small_t<KIND, 2, 2>(p, c, grid, stream); break;
        case 24: launch_small_t<KIND, 2, 4>(p, c, grid, stream); break;
        case 41: launch_small_t<KIND, 4, 1>(p, c, grid, stream); break;
        case 42: launch_small_t<KIND, 4, 2>(p, c, grid, stream); break;
        default: launch_small_t<KIND, 4, 4>(p, c, grid, stream); break;
    }
}

int launch_small_gemm(int kind, const GemmArgs &a, hipStream_t stream) {
    SmallConfig c = choose_small(kind, a.M, a.N, a.K);
    SmallParams p;
    p.X = static_cast<const uint8_t *>(a.X);
    p.x_row_bytes = (kind == kE4M3) ? a.ldx : 2 * a.ldx;
    p.scales = a.scales;
    p.w_scale = a.w_scale;
    p.W0 = static_cast<const uint8_t *>(a.W0);
    p.W1 = static_cast<const uint8_t *>(a.W1);
    p.w_row_bytes = (kind == kPlainF16) ? 2 * a.ldw : a.K;
    p.M = (int)a.M;  p.N = (int)a.N;  p.K = (int)a.K;
    p.Y = a.Y;  p.ldy = a.ldy;
    p.partials = a.partials;
    int kstep = (kind == kE4M3) ? 128 : 64;
    p.steps_total = (int)((a.K + kstep - 1) / kstep);
    int parts = c.waves * c.split;
    p.steps_per_part = (p.steps_total + parts - 1) / parts;
    p.vec_store = ((a.N & 3) == 0 && (a.ldy & 3) == 0 && (reinterpret_cast<uintptr_t>(a.Y) & 7) == 0) ? 1 : 0;
    if (c.split > 1 && (a.partials == nullptr ||
                        a.partial_bytes < (size_t)c.split * a.M * a.N * sizeof(float)))
        return kErrWorkspace;
    dim3 grid((unsigned)((a.N + 16 * c.nt - 1) / (16 * c.nt)), (unsigned)c.split);
    switch (kind) {
        case kPlainF16: launch_small_k<kPlainF16>(p, c, grid, stream); break;
        case kNestedF16: launch_small_k<kNestedF16>(p, c, grid, stream); break;
        default: launch_small_k<kE4M3>(p, c, grid, stream); break;
    }
    if (hipGetLastError() != hipSuccess) return kErrHip;
    if (c.split > 1)
        return launch_splitk_reduce(a.partials, c.split, a.M, a.N, kind == kE4M3 ? a.scales : nullptr,
                                    a.w_scale, a.Y, a.ldy, stream);
    return kOk;
}

}  // namespace nfp
