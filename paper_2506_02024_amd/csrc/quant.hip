// Per-token activation quantisation to E4M3 for FP8 mode (Sec. 2.2 "E4M3 Format",
// Sec. 5.1 "Methodology").  One workgroup per token row: pass 1 finds the row's largest
// magnitude, pass 2 (the row is still in cache) divides and converts.  HBM-bound:
// 2 bytes read + 1 byte written per activation.
#include "nfp_device.h"
#include "nfp_host.h"

namespace nfp {

constexpr int kQuantThreads = 256;

template <bool HW>
__global__ void __launch_bounds__(kQuantThreads)
quantize_act_kernel(const uint16_t *__restrict__ X, int64_t K, int64_t ldx,
                    const float *__restrict__ static_scale, uint8_t *__restrict__ Xq,
                    float *__restrict__ scales) {
    const int64_t m = blockIdx.x;
    const u32x4 *row = reinterpret_cast<const u32x4 *>(X + m * ldx);
    const int chunks = (int)(K / 8);                 // 8 halves per 16-byte chunk
    __shared__ uint32_t red[kQuantThreads / 64];
    float s;
    if (static_scale) {
        s = *static_scale;
    } else {
        // |x| as an integer compare on the magnitude bits: monotone for finite halves
        uint32_t amax_bits = 0;
        for (int c = threadIdx.x; c < chunks; c += kQuantThreads) {
            u32x4 v = row[c];
            uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint32_t lo = w[i] & 0x7fffu, hi = (w[i] >> 16) & 0x7fffu;
                amax_bits = max(amax_bits, max(lo, hi));
            }
        }
        for (int off = 32; off > 0; off >>= 1)
            amax_bits = max(amax_bits, (uint32_t)__shfl_xor((int)amax_bits, off, 64));
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = amax_bits;
        __syncthreads();
        uint32_t all = 0;
#pragma unroll
        for (int i = 0; i < kQuantThreads / 64; ++i) all = max(all, red[i]);
        float amax = half_bits_to_float(all);
        s = (amax == 0.0f) ? 1.0f : amax / 448.0f;
    }
    if (threadIdx.x == 0) scales[m] = s;
    const float y = 1.0f / s;                        // correctly rounded; see div_by_scale
    u32x2 *out = reinterpret_cast<u32x2 *>(Xq + m * K);
    for (int c = threadIdx.x; c < chunks; c += kQuantThreads) {
        u32x4 v = row[c];
        u32x2 q;
        q.x = quant4<HW>(v.x, v.y, s, y);
        q.y = quant4<HW>(v.z, v.w, s, y);
        out[c] = q;
    }
}

// Single-pass variant for rows that fit in registers (K <= 32768): every lane keeps its
// 16-byte chunks between the maximum and the conversion, so the row is read once and the
// kernel is one load latency shorter -- what matters for decode-sized batches, where this
// kernel is pure latency, and for long rows, whose second read no longer comes from the cache.
template <int CPT, bool HW>
__global__ void __launch_bounds__(1024)
quantize_act_onepass_kernel(const uint16_t *__restrict__ X, int64_t K, int64_t ldx,
                            const float *__restrict__ static_scale, uint8_t *__restrict__ Xq,
                            float *__restrict__ scales) {
    const int64_t m = blockIdx.x;
    const u32x4 *row = reinterpret_cast<const u32x4 *>(X + m * ldx);
    const int chunks = (int)(K / 8);
    __shared__ uint32_t red[16];
    u32x4 v[CPT];
    uint32_t amax_bits = 0;
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        int c = threadIdx.x + i * blockDim.x;
        v[i] = c < chunks ? row[c] : u32x4{0u, 0u, 0u, 0u};
        uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
        for (int q = 0; q < 4; ++q) amax_bits = max(amax_bits, max(w[q] & 0x7fffu, (w[q] >> 16) & 0x7fffu));
    }
    float s;
    if (static_scale) {
        s = *static_scale;
    } else {
        for (int off = 32; off > 0; off >>= 1)
            amax_bits = max(amax_bits, (uint32_t)__shfl_xor((int)amax_bits, off, 64));
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = amax_bits;
        __syncthreads();
        uint32_t all = 0;
        const int waves = blockDim.x >> 6;
        for (int i = 0; i < waves; ++i) all = max(all, red[i]);
        float amax = half_bits_to_float(all);
        s = (amax == 0.0f) ? 1.0f : amax / 448.0f;
    }
    if (threadIdx.x == 0) scales[m] = s;
    const float y = 1.0f / s;                        // correctly rounded; see div_by_scale
    u32x2 *out = reinterpret_cast<u32x2 *>(Xq + m * K);
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        int c = threadIdx.x + i * blockDim.x;
        if (c < chunks) {
            u32x2 q;
            q.x = quant4<HW>(v[i].x, v[i].y, s, y);
            q.y = quant4<HW>(v[i].z, v[i].w, s, y);
            out[c] = q;
        }
    }
}

template <int CPT>
static void launch_onepass(bool hw, int threads, const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                           const float *static_scale, uint8_t *Xq, float *scales, hipStream_t stream) {
    dim3 grid((unsigned)M);
    if (hw)
        quantize_act_onepass_kernel<CPT, true><<<grid, threads, 0, stream>>>(X, K, ldx, static_scale, Xq, scales);
    else
        quantize_act_onepass_kernel<CPT, false><<<grid, threads, 0, stream>>>(X, K, ldx, static_scale, Xq, scales);
}

int launch_quantize_act(const uint16_t *X, int64_t M, int64_t K, int64_t ldx,
                        const float *static_scale, uint8_t *Xq, float *scales, hipStream_t stream) {
    bool hw = tuning().quant_hw != 0;
    const int64_t chunks = K / 8;
    const int64_t onepass = tuning().quant_onepass;
    // one pass for decode-sized batches (latency) and for long rows at any batch (measured at 8192
    // tokens: 5.1-5.4 TB/s against 3.9 for K = 14336 / 28672, equal at K = 8192, 4 % behind at 4096)
    if (chunks <= 4096 && (onepass > 0 || (onepass < 0 && (M <= 256 || chunks >= 1024)))) {
        // as many lanes as the row has chunks (up to 1024, 4 chunks each)
        int cpt = chunks <= 1024 ? 1 : (chunks <= 2048 ? 2 : 4);
        int threads = (int)(((chunks + cpt - 1) / cpt + 63) / 64 * 64);
        if (cpt == 1) launch_onepass<1>(hw, threads, X, M, K, ldx, static_scale, Xq, scales, stream);
        else if (cpt == 2) launch_onepass<2>(hw, threads, X, M, K, ldx, static_scale, Xq, scales, stream);
        else launch_onepass<4>(hw, threads, X, M, K, ldx, static_scale, Xq, scales, stream);
        return hip_ok(hipGetLastError());
    }
    dim3 grid((unsigned)M);
    if (hw)
        quantize_act_kernel<true><<<grid, kQuantThreads, 0, stream>>>(X, K, ldx, static_scale, Xq, scales);
    else
        quantize_act_kernel<false><<<grid, kQuantThreads, 0, stream>>>(X, K, ldx, static_scale, Xq, scales);
    return hip_ok(hipGetLastError());
}

}  // namespace nfp
