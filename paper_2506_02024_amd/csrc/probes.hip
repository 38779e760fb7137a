// Measurement aids for the benchmark: what the chip sustains for the two resources the GEMM
// kernels are bound by (HBM reads, MFMA issue), measured with their instruction mix.
// No part of the method.
#include "nfp_device.h"
#include "nfp_host.h"

namespace nfp {

// Every wave reads 8 KB with eight 128-bit loads per lane (a contiguous kilobyte per
// instruction, all eight in flight) and exits: the access pattern of the streaming GEMM
// without its arithmetic.  The store never happens for real data; it keeps the loads alive.
__global__ void __launch_bounds__(1024)
stream_read_kernel(const uint8_t *__restrict__ src, uint32_t *__restrict__ sink) {
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    const u32x4 *p = reinterpret_cast<const u32x4 *>(src + wave * 8192 + lane * 16);
    u32x4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = __builtin_nontemporal_load(p + i * 64);
    uint32_t x = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) x ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
    if (x == 0x9e3779b9u && lane == 63) *sink = x;
}

// The same read with 16 KB per wave and at most one workgroup of 8 waves per CU (a dynamic LDS
// allocation of 160 KB that nothing touches keeps a second one out).  The kernel above is held back by
// the turnover of its many small workgroups, not by memory: fewer and longer-lived waves read faster.
__global__ void __launch_bounds__(512)
stream_read_sparse_kernel(const uint8_t *__restrict__ src, uint32_t *__restrict__ sink) {
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    const u32x4 *p = reinterpret_cast<const u32x4 *>(src + wave * 16384 + lane * 16);
    u32x4 v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = __builtin_nontemporal_load(p + i * 64);
    uint32_t x = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) x ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
    if (x == 0x9e3779b9u && lane == 63) *sink = x;
}

int launch_probe_stream_read_sparse(const void *src, size_t bytes, uint32_t *sink, hipStream_t stream) {
    constexpr int lds = 160 * 1024;
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(stream_read_sparse_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr_set.store(true, std::memory_order_release);
    }
    // bytes is a multiple of 131072: whole workgroups of 8 waves x 16 KB
    stream_read_sparse_kernel<<<(unsigned)(bytes / 131072), 512, lds, stream>>>(static_cast<const uint8_t *>(src), sink);
    return hip_ok(hipGetLastError());
}

int launch_probe_stream_read(const void *src, size_t bytes, uint32_t *sink, hipStream_t stream) {
    const size_t waves = bytes / 8192;                 // bytes is a multiple of 65536: whole workgroups of 8 waves
    stream_read_kernel<<<(unsigned)(waves / 8), 512, 0, stream>>>(static_cast<const uint8_t *>(src), sink);
    return hip_ok(hipGetLastError());
}

// Nothing but MFMAs: 16 independent accumulators per wave, operands rotating through four
// register sets so that the multiplier inputs change from one instruction to the next (the
// chip's clock under load depends on the data).  4 waves per SIMD.
constexpr int kProbeBlocks = 1024, kProbeThreads = 256, kProbeChains = 16;

template <bool FP8>
__global__ void __launch_bounds__(kProbeThreads)
mfma_probe_kernel(const uint8_t *__restrict__ operands, int iters, uint32_t *__restrict__ sink) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    intx8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // 8 KB per register set and operand side; the buffer holds 65536 bytes
        const intx4 *pa = reinterpret_cast<const intx4 *>(operands + (i * 2) * 8192 + ((wave * 64 + lane) & 255) * 32);
        const intx4 *pb = reinterpret_cast<const intx4 *>(operands + (i * 2 + 1) * 8192 + ((wave * 64 + lane) & 255) * 32);
        const intx4 a0 = pa[0], a1 = pa[1], b0 = pb[0], b1 = pb[1];
        a[i] = intx8{a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
        b[i] = intx8{b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
    }
    floatx4 acc[kProbeChains];
#pragma unroll
    for (int c = 0; c < kProbeChains; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < kProbeChains; ++c) {
            if (FP8) {
                acc[c] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[c & 3], b[(c >> 2) & 3], acc[c], 0, 0, 0, 0, 0, 0);
            } else {
                union { intx4 v; half8 h; } ua, ub;
                ua.v = intx4{a[c & 3][0], a[c & 3][1], a[c & 3][2], a[c & 3][3]};
                ub.v = intx4{b[(c >> 2) & 3][0], b[(c >> 2) & 3][1], b[(c >> 2) & 3][2], b[(c >> 2) & 3][3]};
                acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ua.h, ub.h, acc[c], 0, 0, 0);
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < kProbeChains; ++c) s += acc[c].x + acc[c].y + acc[c].z + acc[c].w;
    if (s == 1.2345678e-30f) *sink = __float_as_uint(s);
}

int launch_probe_mfma(const void *operands, int fp8, int iters, uint32_t *sink, double *flops_host,
                      hipStream_t stream) {
    const double per_mfma = fp8 ? 2.0 * 16 * 16 * 128 : 2.0 * 16 * 16 * 32;
    if (flops_host)
        *flops_host = per_mfma * kProbeChains * (double)iters * (kProbeBlocks * (kProbeThreads / 64));
    if (fp8)
        mfma_probe_kernel<true><<<kProbeBlocks, kProbeThreads, 0, stream>>>(static_cast<const uint8_t *>(operands), iters, sink);
    else
        mfma_probe_kernel<false><<<kProbeBlocks, kProbeThreads, 0, stream>>>(static_cast<const uint8_t *>(operands), iters, sink);
    return hip_ok(hipGetLastError());
}

}  // namespace nfp
