// Element-wise kernels of the NestedFP format (Sec. 4.1): applicability count,
// decomposition into byte planes, lossless reconstruction.  All three are HBM-bound:
// every lane moves 16 weights per step with 128-bit loads and stores.
#include "nfp_device.h"
#include "nfp_host.h"

namespace nfp {

constexpr int kPlaneThreads = 256;

// chunk c (16 weights) -> (row, first column)
struct ChunkMap {
    int64_t chunks_per_row;   // K / 16
    int64_t total;            // N * K / 16
};

__device__ __forceinline__ void add_count(uint64_t *counter, uint32_t bad) {
    // wave reduction, then one vector atomic per wave
    for (int off = 32; off > 0; off >>= 1) bad += __shfl_down(bad, off, 64);
    if ((threadIdx.x & 63) == 0 && bad != 0)
        atomicAdd(reinterpret_cast<unsigned long long *>(counter), (unsigned long long)bad);
}

__global__ void __launch_bounds__(kPlaneThreads)
decompose_kernel(const uint16_t *__restrict__ W, int64_t ldw, ChunkMap map,
                 uint8_t *__restrict__ upper, uint8_t *__restrict__ lower,
                 uint64_t *__restrict__ counter) {
    uint32_t bad = 0;
    const int64_t stride = (int64_t)gridDim.x * kPlaneThreads;
    for (int64_t c = (int64_t)blockIdx.x * kPlaneThreads + threadIdx.x; c < map.total; c += stride) {
        int64_t row = c / map.chunks_per_row;
        int64_t col = (c - row * map.chunks_per_row) * 16;
        const u32x4 *src = reinterpret_cast<const u32x4 *>(W + row * ldw + col);
        u32x4 a = __builtin_nontemporal_load(src);
        u32x4 b = __builtin_nontemporal_load(src + 1);
        uint32_t u[8], l[8];
        decompose2(a.x, u[0], l[0], bad);
        decompose2(a.y, u[1], l[1], bad);
        decompose2(a.z, u[2], l[2], bad);
        decompose2(a.w, u[3], l[3], bad);
        decompose2(b.x, u[4], l[4], bad);
        decompose2(b.y, u[5], l[5], bad);
        decompose2(b.z, u[6], l[6], bad);
        decompose2(b.w, u[7], l[7], bad);
        u32x4 up, lo;
        up.x = pack_even_bytes(u[0], u[1]);  lo.x = pack_even_bytes(l[0], l[1]);
        up.y = pack_even_bytes(u[2], u[3]);  lo.y = pack_even_bytes(l[2], l[3]);
        up.z = pack_even_bytes(u[4], u[5]);  lo.z = pack_even_bytes(l[4], l[5]);
        up.w = pack_even_bytes(u[6], u[7]);  lo.w = pack_even_bytes(l[6], l[7]);
        __builtin_nontemporal_store(up, reinterpret_cast<u32x4 *>(upper + c * 16));
        __builtin_nontemporal_store(lo, reinterpret_cast<u32x4 *>(lower + c * 16));
    }
    if (counter) add_count(counter, bad);
}

__global__ void __launch_bounds__(kPlaneThreads)
range_check_kernel(const uint16_t *__restrict__ W, int64_t ldw, ChunkMap map,
                   uint64_t *__restrict__ counter) {
    uint32_t bad = 0;
    const int64_t stride = (int64_t)gridDim.x * kPlaneThreads;
    for (int64_t c = (int64_t)blockIdx.x * kPlaneThreads + threadIdx.x; c < map.total; c += stride) {
        int64_t row = c / map.chunks_per_row;
        int64_t col = (c - row * map.chunks_per_row) * 16;
        const u32x4 *src = reinterpret_cast<const u32x4 *>(W + row * ldw + col);
        u32x4 a = __builtin_nontemporal_load(src);
        u32x4 b = __builtin_nontemporal_load(src + 1);
        uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t m = w[i] & 0x7fff7fffu;
            bad += ((m & 0xffffu) > 0x3f00u) + ((m >> 16) > 0x3f00u);
        }
    }
    add_count(counter, bad);
}

__global__ void __launch_bounds__(kPlaneThreads)
reconstruct_kernel(const uint8_t *__restrict__ upper, const uint8_t *__restrict__ lower,
                   ChunkMap map, uint16_t *__restrict__ W, int64_t ldw) {
    const int64_t stride = (int64_t)gridDim.x * kPlaneThreads;
    for (int64_t c = (int64_t)blockIdx.x * kPlaneThreads + threadIdx.x; c < map.total; c += stride) {
        u32x4 u = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(upper + c * 16));
        u32x4 l = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(lower + c * 16));
        u32x4 w0, w1;
        merge16(u, l, w0, w1);
        int64_t row = c / map.chunks_per_row;
        int64_t col = (c - row * map.chunks_per_row) * 16;
        u32x4 *dst = reinterpret_cast<u32x4 *>(W + row * ldw + col);
        __builtin_nontemporal_store(w0, dst);
        __builtin_nontemporal_store(w1, dst + 1);
    }
}

__global__ void zero_u64_kernel(uint64_t *p) { *p = 0; }

int launch_zero_u64(uint64_t *p, hipStream_t stream) {
    zero_u64_kernel<<<1, 1, 0, stream>>>(p);
    return hip_ok(hipGetLastError());
}

static int plane_grid(int64_t total_chunks) {
    // one chunk per lane for small tensors; up to four per lane (grid-stride) for large ones
    int64_t blocks = (total_chunks + kPlaneThreads - 1) / kPlaneThreads;
    if (blocks > 4096) blocks = (blocks / 4 > 4096) ? blocks / 4 : 4096;
    if (blocks < 1) blocks = 1;
    return (int)(blocks > 0x7fffffff ? 0x7fffffff : blocks);
}

int launch_decompose(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint8_t *upper,
                     uint8_t *lower, uint64_t *counter, hipStream_t stream) {
    ChunkMap map{K / 16, N * (K / 16)};
    if (counter) zero_u64_kernel<<<1, 1, 0, stream>>>(counter);
    decompose_kernel<<<plane_grid(map.total), kPlaneThreads, 0, stream>>>(W, ldw, map, upper, lower,
                                                                         counter);
    return hip_ok(hipGetLastError());
}

int launch_range_check(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint64_t *counter,
                       hipStream_t stream) {
    ChunkMap map{K / 16, N * (K / 16)};
    zero_u64_kernel<<<1, 1, 0, stream>>>(counter);
    range_check_kernel<<<plane_grid(map.total), kPlaneThreads, 0, stream>>>(W, ldw, map, counter);
    return hip_ok(hipGetLastError());
}

int launch_reconstruct(const uint8_t *upper, const uint8_t *lower, int64_t N, int64_t K,
                       uint16_t *W, int64_t ldw, hipStream_t stream) {
    ChunkMap map{K / 16, N * (K / 16)};
    reconstruct_kernel<<<plane_grid(map.total), kPlaneThreads, 0, stream>>>(upper, lower, map, W, ldw);
    return hip_ok(hipGetLastError());
}

}  // namespace nfp
