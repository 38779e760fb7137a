// Element-wise kernels of the NestedFP format (Sec. 4.1): applicability count,
// decomposition into byte planes, lossless reconstruction.  All three are HBM-bound:
// every lane moves 16 weights per step with 128-bit loads and stores.  The planes are
// row-major [N,K] byte matrices (the two tensors of Sec. 4 "Overview" as they are); the
// packed form below is an optional pre-pack of the same bytes for the GEMM kernels.
#include "nfp_device.h"
#include "nfp_host.h"

namespace nfp {

constexpr int kPlaneThreads = 256;

// Packed plane layout: a plane of an [N,K] byte matrix is a sequence of 1 KB blocks, one per
// 16-row x 64-column sub-matrix, block (i,j) at ((i * kblocks) + j) * 1024.  Inside a block
// the 16-byte chunk of row r (0..15), column group g (0..3) sits at chunk index r + 16*g:
// exactly the order in which the 64 lanes of a wave hold an MFMA operand (row = lane % 16,
// K group = lane / 16), so one 128-bit load per lane reads the block front to back.
// Rows past N and columns past K are stored as zeros.
struct BlockMap {
    int64_t N, K;
    int64_t kblocks;          // ceil(K / 64)
    int64_t blocks;           // ceil(N / 16) * kblocks
};

static BlockMap block_map(int64_t N, int64_t K) {
    BlockMap m;
    m.N = N;  m.K = K;
    m.kblocks = (K + 63) / 64;
    m.blocks = ((N + 15) / 16) * m.kblocks;
    return m;
}

__device__ __forceinline__ void add_count(uint64_t *counter, uint32_t bad) {
    // wave reduction, then one vector atomic per wave
    for (int off = 32; off > 0; off >>= 1) bad += __shfl_down(bad, off, 64);
    if ((threadIdx.x & 63) == 0 && bad != 0)
        atomicAdd(reinterpret_cast<unsigned long long *>(counter), (unsigned long long)bad);
}

// One wave per block and trip: lane l owns chunk l of the block, i.e. row 16*i + l%16 and
// columns 64*j + 16*(l/16) .. +15 of the matrix.
struct LaneChunk {
    int64_t row, col;
    int64_t offset;           // byte offset of the chunk in the packed plane
    bool inside;
};

__device__ __forceinline__ LaneChunk lane_chunk(const BlockMap &m, int64_t block, int lane) {
    LaneChunk c;
    const int64_t i = block / m.kblocks, j = block - i * m.kblocks;
    c.row = 16 * i + (lane & 15);
    c.col = 64 * j + 16 * (lane >> 4);
    c.offset = block * 1024 + lane * 16;
    c.inside = c.row < m.N && c.col < m.K;
    return c;
}

__global__ void __launch_bounds__(kPlaneThreads)
decompose_kernel(const uint16_t *__restrict__ W, int64_t ldw, BlockMap map,
                 uint8_t *__restrict__ upper, uint8_t *__restrict__ lower,
                 uint64_t *__restrict__ counter) {
    uint32_t bad = 0;
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * kPlaneThreads + threadIdx.x) >> 6;
    const int64_t waves = ((int64_t)gridDim.x * kPlaneThreads) >> 6;
    for (int64_t blk = wave; blk < map.blocks; blk += waves) {
        const LaneChunk c = lane_chunk(map, blk, lane);
        u32x4 up = {0, 0, 0, 0}, lo = {0, 0, 0, 0};
        if (c.inside) {
            const u32x4 *src = reinterpret_cast<const u32x4 *>(W + c.row * ldw + c.col);
            u32x4 a = __builtin_nontemporal_load(src);
            u32x4 b = __builtin_nontemporal_load(src + 1);
            decompose16(a, b, up, lo, bad);
        }
        __builtin_nontemporal_store(up, reinterpret_cast<u32x4 *>(upper + c.offset));
        __builtin_nontemporal_store(lo, reinterpret_cast<u32x4 *>(lower + c.offset));
    }
    if (counter) add_count(counter, bad);
}

// chunk c (16 weights) of a row-major matrix -> (row, first column)
struct ChunkMap {
    int64_t chunks_per_row;   // K / 16
    int64_t total;            // N * K / 16
};

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
                   BlockMap map, uint16_t *__restrict__ W, int64_t ldw) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * kPlaneThreads + threadIdx.x) >> 6;
    const int64_t waves = ((int64_t)gridDim.x * kPlaneThreads) >> 6;
    for (int64_t blk = wave; blk < map.blocks; blk += waves) {
        const LaneChunk c = lane_chunk(map, blk, lane);
        if (!c.inside) continue;
        u32x4 u = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(upper + c.offset));
        u32x4 l = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(lower + c.offset));
        u32x4 w0, w1;
        merge16(u, l, w0, w1);
        u32x4 *dst = reinterpret_cast<u32x4 *>(W + c.row * ldw + c.col);
        __builtin_nontemporal_store(w0, dst);
        __builtin_nontemporal_store(w1, dst + 1);
    }
}

// ---- row-major planes: chunk c (16 weights) of the matrix is row c / (K/16), columns 16 * (c % (K/16)) .. +15
__global__ void __launch_bounds__(kPlaneThreads)
decompose_rows_kernel(const uint16_t *__restrict__ W, int64_t ldw, ChunkMap map, int64_t K,
                      uint8_t *__restrict__ upper, uint8_t *__restrict__ lower,
                      uint64_t *__restrict__ counter) {
    uint32_t bad = 0;
    const int64_t stride = (int64_t)gridDim.x * kPlaneThreads;
    for (int64_t c = (int64_t)blockIdx.x * kPlaneThreads + threadIdx.x; c < map.total; c += stride) {
        const int64_t row = c / map.chunks_per_row;
        const int64_t col = (c - row * map.chunks_per_row) * 16;
        const u32x4 *src = reinterpret_cast<const u32x4 *>(W + row * ldw + col);
        const u32x4 a = __builtin_nontemporal_load(src);
        const u32x4 b = __builtin_nontemporal_load(src + 1);
        u32x4 up, lo;
        decompose16(a, b, up, lo, bad);
        __builtin_nontemporal_store(up, reinterpret_cast<u32x4 *>(upper + row * K + col));
        __builtin_nontemporal_store(lo, reinterpret_cast<u32x4 *>(lower + row * K + col));
    }
    if (counter) add_count(counter, bad);
}

__global__ void __launch_bounds__(kPlaneThreads)
reconstruct_rows_kernel(const uint8_t *__restrict__ upper, const uint8_t *__restrict__ lower,
                        ChunkMap map, int64_t K, uint16_t *__restrict__ W, int64_t ldw) {
    const int64_t stride = (int64_t)gridDim.x * kPlaneThreads;
    for (int64_t c = (int64_t)blockIdx.x * kPlaneThreads + threadIdx.x; c < map.total; c += stride) {
        const int64_t row = c / map.chunks_per_row;
        const int64_t col = (c - row * map.chunks_per_row) * 16;
        const u32x4 u = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(upper + row * K + col));
        const u32x4 l = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(lower + row * K + col));
        u32x4 w0, w1;
        merge16(u, l, w0, w1);
        u32x4 *dst = reinterpret_cast<u32x4 *>(W + row * ldw + col);
        __builtin_nontemporal_store(w0, dst);
        __builtin_nontemporal_store(w1, dst + 1);
    }
}

// FP16 weights in packed storage: one 2 KB block per 16-row x 64-column sub-matrix, made of two
// halves of 1 KB; lane l (row l % 16, column group l / 16) owns chunk l of each half: columns
// 16 g .. 16 g + 7 in the first, 16 g + 8 .. 16 g + 15 in the second -- what a lane of the
// NestedFP kernels holds after merging its 16 bytes of each plane.  Padding is zero.
__global__ void __launch_bounds__(kPlaneThreads)
pack_fp16_kernel(const uint16_t *__restrict__ W, int64_t ldw, BlockMap map, uint8_t *__restrict__ dst) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * kPlaneThreads + threadIdx.x) >> 6;
    const int64_t waves = ((int64_t)gridDim.x * kPlaneThreads) >> 6;
    for (int64_t blk = wave; blk < map.blocks; blk += waves) {
        const LaneChunk c = lane_chunk(map, blk, lane);
        u32x4 a = {0, 0, 0, 0}, b = {0, 0, 0, 0};
        if (c.inside) {
            const u32x4 *src = reinterpret_cast<const u32x4 *>(W + c.row * ldw + c.col);
            a = __builtin_nontemporal_load(src);
            b = __builtin_nontemporal_load(src + 1);
        }
        __builtin_nontemporal_store(a, reinterpret_cast<u32x4 *>(dst + blk * 2048 + lane * 16));
        __builtin_nontemporal_store(b, reinterpret_cast<u32x4 *>(dst + blk * 2048 + 1024 + lane * 16));
    }
}

// Row-major bytes <-> packed plane (for E4M3 weights that do not come from a decomposition,
// and for reading a plane back in matrix order).
template <bool PACK>
__global__ void __launch_bounds__(kPlaneThreads)
repack_kernel(const uint8_t *__restrict__ src, uint8_t *__restrict__ dst, int64_t ld, BlockMap map) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * kPlaneThreads + threadIdx.x) >> 6;
    const int64_t waves = ((int64_t)gridDim.x * kPlaneThreads) >> 6;
    for (int64_t blk = wave; blk < map.blocks; blk += waves) {
        const LaneChunk c = lane_chunk(map, blk, lane);
        if (PACK) {
            u32x4 v = {0, 0, 0, 0};
            if (c.inside) v = *reinterpret_cast<const u32x4 *>(src + c.row * ld + c.col);
            *reinterpret_cast<u32x4 *>(dst + c.offset) = v;
        } else if (c.inside) {
            *reinterpret_cast<u32x4 *>(dst + c.row * ld + c.col) = *reinterpret_cast<const u32x4 *>(src + c.offset);
        }
    }
}

__global__ void zero_u64_kernel(uint64_t *p) { *p = 0; }

__global__ void zero_words_kernel(uint32_t *p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

int launch_zero_words(uint32_t *p, int n, hipStream_t stream) {
    if (n <= 0) return kOk;
    zero_words_kernel<<<(n + 255) / 256, 256, 0, stream>>>(p, n);
    return hip_ok(hipGetLastError());
}

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

size_t plane_bytes(int64_t N, int64_t K) {
    return (size_t)(((N + 15) / 16) * 16) * (size_t)(((K + 63) / 64) * 64);
}

int launch_decompose(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint8_t *upper,
                     uint8_t *lower, uint64_t *counter, bool packed, hipStream_t stream) {
    if (counter) zero_u64_kernel<<<1, 1, 0, stream>>>(counter);
    if (packed) {
        BlockMap map = block_map(N, K);
        decompose_kernel<<<plane_grid(map.blocks * 64), kPlaneThreads, 0, stream>>>(W, ldw, map, upper, lower,
                                                                                  counter);
    } else {
        ChunkMap map{K / 16, N * (K / 16)};
        decompose_rows_kernel<<<plane_grid(map.total), kPlaneThreads, 0, stream>>>(W, ldw, map, K, upper, lower,
                                                                                 counter);
    }
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
                       uint16_t *W, int64_t ldw, bool packed, hipStream_t stream) {
    if (packed) {
        BlockMap map = block_map(N, K);
        reconstruct_kernel<<<plane_grid(map.blocks * 64), kPlaneThreads, 0, stream>>>(upper, lower, map, W, ldw);
    } else {
        ChunkMap map{K / 16, N * (K / 16)};
        reconstruct_rows_kernel<<<plane_grid(map.total), kPlaneThreads, 0, stream>>>(upper, lower, map, K, W, ldw);
    }
    return hip_ok(hipGetLastError());
}

int launch_pack_fp16(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint8_t *dst, hipStream_t stream) {
    BlockMap map = block_map(N, K);
    pack_fp16_kernel<<<plane_grid(map.blocks * 64), kPlaneThreads, 0, stream>>>(W, ldw, map, dst);
    return hip_ok(hipGetLastError());
}

int launch_pack_plane(const uint8_t *src, int64_t N, int64_t K, int64_t ld, uint8_t *dst, hipStream_t stream) {
    BlockMap map = block_map(N, K);
    repack_kernel<true><<<plane_grid(map.blocks * 64), kPlaneThreads, 0, stream>>>(src, dst, ld, map);
    return hip_ok(hipGetLastError());
}

int launch_unpack_plane(const uint8_t *src, int64_t N, int64_t K, uint8_t *dst, int64_t ld, hipStream_t stream) {
    BlockMap map = block_map(N, K);
    repack_kernel<false><<<plane_grid(map.blocks * 64), kPlaneThreads, 0, stream>>>(src, dst, ld, map);
    return hip_ok(hipGetLastError());
}

}  // namespace nfp
