// LDS-tiled MFMA GEMMs for prefill-sized batches: Y = X * W^T, compute-bound.
//
// Three kernels.  large_gemm_kernel multiplies plain FP16 weights or E4M3 weights (FP8 mode: the
// upper plane as it is, row-major or in packed blocks): TM tokens x TN weight rows x 128 bytes of K
// per row (64 halves or 128 E4M3 bytes) per stage, two LDS stages, 8 waves.  nested_bypass_kernel is FP16 mode: Sec. 4.2
// puts the FP16 reconstruction between the shared-memory-to-register copy and the tensor-core
// instruction of every warp and hides it with a third pipeline stage; here every weight belongs
// to exactly one wave, which loads its 16 bytes of each plane per lane (from row-major planes or
// from packed blocks) into registers, merges them there (Alg. 1) and feeds them to the MFMA -- the
// weights never pass through LDS; the same kernel without the merge multiplies FP16 weights stored
// in packed blocks, the like-for-like baseline of Sec. 5.2.  e4m3_bypass_kernel
// is the same register path for E4M3 weights, used for batches of 49 .. 64 tokens, where the
// weight stream is the bound.
//
// In all of them, weight rows are the MFMA "A" operand and tokens the "B" operand, so a lane holds 4
// consecutive output columns of one token.  Tokens and plain / E4M3 weights reach LDS by
// direct-to-LDS buffer loads; FP16 rows are 128 bytes with the 16-byte chunk index XOR-swizzled
// with the row so that the MFMA fragment reads are free of bank conflicts, packed E4M3 blocks
// are copied as they are.
#include <type_traits>

#include "nfp_device.h"
#include "nfp_host.h"

namespace nfp {

struct LargeParams {
    const uint8_t *X;       // fp16 X (bytes) or E4M3 Xq
    int64_t x_row_bytes;    // 256 rows of it stay below 2^31 (checked on the host): bit 31 of a tile-local offset marks a dead load
    const float *scales;
    float w_scale;
    const uint8_t *W0;
    const uint8_t *W1;
    int64_t w_row_bytes;    // bytes per row of W0 for row-major weights (plain: 2*ldw, planes / E4M3: K); same limit
    int M, N, K;
    int k_bytes;            // bytes per row along K for 8-chunk operands (2K or K)
    int kblocks;            // 64-column blocks per row tile of a packed plane: ceil(K / 64)
    uint16_t *Y;
    int64_t ldy;
    float *partials;
    int tiles_m, tiles_n;
    int ktiles_total, ktiles_per_split;
    int vec_store;
    int row_store;          // Y rows can be written 16 bytes per lane (N, ldy multiples of 8, Y 16-byte aligned)
    int xcd_map;            // group the token tiles of a weight tile on one XCD (see tile_of_block)
};

// Which tile a workgroup takes.  The hardware deals consecutive workgroups to the 8 XCDs in turn,
// and every XCD has an L2 of its own.  With few token tiles per weight tile (batches of up to about
// 1000 tokens) the launch order "token tile fastest" puts the token tiles of one weight tile on
// different XCDs, so each of them fetches those weights from memory again; instead, workgroup
// b of XCD b % 8 takes token tile (b / 8) % tiles_m of weight tile 8 * ((b / 8) / tiles_m) + b % 8:
// all token tiles of a weight tile follow each other on one XCD.  The last tiles_n % 8 weight tiles
// keep the launch order.  With many token tiles per weight tile the launch order already gives
// every XCD a near-square block of tiles (tiles_m / 8 token tiles x 8 weight tiles at a time).
__device__ __forceinline__ void tile_of_block(const LargeParams &p, int b, int &tm, int &tn) {
    const int grouped = 8 * p.tiles_m * (p.tiles_n >> 3);
    if (p.xcd_map && b < grouped) {
        const int j = b >> 3;
        tm = j % p.tiles_m;
        tn = (j / p.tiles_m) * 8 + (b & 7);
    } else if (p.xcd_map) {
        const int r = b - grouped;
        tm = r % p.tiles_m;
        tn = (p.tiles_n & ~7) + r / p.tiles_m;
    } else {
        tm = b % p.tiles_m;
        tn = b / p.tiles_m;
    }
}

// LDS tiles are rows of 128 bytes; the 16-byte chunk index is XOR-ed with (row >> 1) & 7.
// gfx950 serves ds_read_b128 at 256 B/clk only if 16 consecutive lanes hit 64 distinct
// 4-byte banks: rows r, r+1 then share a swizzle and fill one 256-byte bank line, and the
// pairs of 16 consecutive rows take the 8 different swizzles.  The 128-bit writes of the
// global->LDS copy (8 lanes per row) are conflict-free under the same map.
__device__ __forceinline__ int swz(int row, int chunk) { return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4); }

// FP16 tiles: which 16-byte chunk of a 128-byte global row the physical chunk slot p of an LDS row
// holds (before the XOR swizzle).  The sum over k does not care about the order of k as long as
// both operands agree.  The register-path NestedFP kernel gets its weights 16 consecutive columns
// per lane (lane group g = l / 16 holds columns 16 g .. 16 g + 15 of a packed block), so substep
// s of a K-tile multiplies halves 16 g + 8 s .. + 7, i.e. chunk 2 g + s of the row; all FP16 kernels
// use that order, so that they add up alike and FP16 mode equals the plain FP16 GEMM bit for bit.
// In LDS the four lane groups must read ADJACENT chunks (a stride of two chunks between the
// groups halves the LDS read rate: bank conflicts), so chunk 2 g + s is stored in slot 4 s + g.
__device__ __forceinline__ int fp16_chunk_of_slot(int p) { return ((p & 3) << 1) | (p >> 2); }

__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_rsrc(const uint8_t *base, int64_t row0, int rows,
                                                            int64_t row_bytes, int k_bytes) {
    // raw buffer over the rows of one tile; anything past the last valid byte reads as zero
    uint32_t bytes = rows > 0 ? (uint32_t)((rows - 1) * row_bytes + k_bytes) : 0u;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(base + row0 * row_bytes), 0, bytes, 0x00020000);
}

// raw buffer over the 16-row tiles of a packed plane (blocks of block_bytes) that hold rows row0 .. row0+rows-1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t plane_rsrc(const uint8_t *base, int64_t row0, int rows, int kblocks,
                                                             int block_bytes) {
    const int64_t tile_bytes = (int64_t)kblocks * block_bytes;
    uint32_t bytes = rows > 0 ? (uint32_t)(((rows + 15) >> 4) * tile_bytes) : 0u;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(base + (row0 >> 4) * tile_bytes), 0, bytes, 0x00020000);
}

// ---- writing a workgroup's result tile ------------------------------------------------------------
// MB: rows of an MFMA block (16 or 32).  Accumulator layout: lane l holds token l % MB of a block
// and, for v = 0 .. MB*MB/256 - 1, the four consecutive weight rows
// (MB == 32 ? 8 v + 4 (l / 32) : 4 (l / 16)) .. +3.
template <int KIND, int TM, int TN, int WAVES_M, int WAVES_N, int MB_ = (kind_is_fp8(KIND) ? 32 : 16)>
struct TileStore {
    static constexpr int WAVES = WAVES_M * WAVES_N;
    static constexpr int WTM = TM / WAVES_M, WTN = TN / WAVES_N;
    static constexpr int MB = MB_;
    static constexpr int FMB = WTM / MB, FNB = WTN / MB;
    typedef typename std::conditional<MB == 32, floatx16, floatx4>::type AccT;

    // Result tile through LDS: the MFMA layout leaves a lane with 4 consecutive outputs of one
    // token, so direct stores are 8-byte pieces scattered over 16 or 32 rows per instruction.  Written
    // to LDS as FP16 first (16-byte chunks XOR-swizzled with the row), the tile goes out as
    // whole rows, 16 bytes per lane, every store instruction covering complete 128-byte lines.
    // The caller guarantees that no wave still reads the operand stages.
    static constexpr int OCH = TN * 2 / 16;            // 16-byte chunks per output row
        static constexpr int NV = MB == 32 ? 4 : 1;
    static __device__ __forceinline__ float scaled(float x, float s) { return kind_is_fp8(KIND) ? scale_f32(x, s) : x; }
    static __device__ __forceinline__ int acc_col(int lane, int v) { return MB == 32 ? 8 * v + 4 * (lane >> 5) : 4 * (lane >> 4); }

    static __device__ __forceinline__ void epilogue_lds(const LargeParams &p, AccT (&acc)[FNB][FMB], int m0, int n0,
                                                        int wm, int wn, int lane, int wave, uint8_t *lds) {
        const int r = lane % MB;
#pragma unroll
        for (int j = 0; j < FMB; ++j) {
            const int row = wm * WTM + MB * j + r;
            float s = 1.0f;
            if (kind_is_fp8(KIND)) {
                const int m = m0 + row;
                s = (m < p.M ? p.scales[m] : 0.f) * p.w_scale;
            }
#pragma unroll
            for (int i = 0; i < FNB; ++i)
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const int col = wn * WTN + MB * i + acc_col(lane, v);
                    const int chunk = col >> 3;
                    u32x2 o;
                    o.x = float2_to_half2_bits(scaled(acc[i][j][4 * v], s), scaled(acc[i][j][4 * v + 1], s));
                    o.y = float2_to_half2_bits(scaled(acc[i][j][4 * v + 2], s), scaled(acc[i][j][4 * v + 3], s));
                    *reinterpret_cast<u32x2 *>(lds + row * (TN * 2) + ((chunk ^ (row & (OCH - 1))) << 4) + 8 * ((col >> 2) & 1)) = o;
                }
        }
        __syncthreads();
        constexpr int RPI = 64 / OCH;                  // rows per store instruction
        constexpr int ROWS = TM / WAVES;               // rows per wave
        const int chunk = lane % OCH;
        const int n = n0 + chunk * 8;
#pragma unroll
        for (int it = 0; it < ROWS / RPI; ++it) {
            const int row = wave * ROWS + it * RPI + lane / OCH;
            const u32x4 v = *reinterpret_cast<const u32x4 *>(lds + row * (TN * 2) + ((chunk ^ (row & (OCH - 1))) << 4));
            const int m = m0 + row;
            if (m < p.M && n < p.N) *reinterpret_cast<u32x4 *>(p.Y + (int64_t)m * p.ldy + n) = v;
        }
    }

    static __device__ __forceinline__ void epilogue(const LargeParams &p, AccT (&acc)[FNB][FMB], int m0, int n0,
                                                    int wm, int wn, int lane, int split) {
        const int r = lane % MB;
#pragma unroll
        for (int j = 0; j < FMB; ++j) {
            const int m = m0 + wm * WTM + MB * j + r;
            if (m >= p.M) continue;
            float s = 1.0f;
            if (kind_is_fp8(KIND) && gridDim.y == 1) s = p.scales[m] * p.w_scale;
#pragma unroll
            for (int i = 0; i < FNB; ++i)
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const int n = n0 + wn * WTN + MB * i + acc_col(lane, v);
                    if (n >= p.N) continue;
                    const float x[4] = {acc[i][j][4 * v], acc[i][j][4 * v + 1], acc[i][j][4 * v + 2], acc[i][j][4 * v + 3]};
                    if (gridDim.y > 1) {
                        float *dst = p.partials + ((int64_t)split * p.M + m) * p.N + n;
                        if ((p.N & 3) == 0) {
                            *reinterpret_cast<floatx4 *>(dst) = floatx4{x[0], x[1], x[2], x[3]};
                        } else {
                            for (int e = 0; e < 4 && n + e < p.N; ++e) dst[e] = x[e];
                        }
                    } else {
                        uint16_t *dst = p.Y + (int64_t)m * p.ldy + n;
                        if (p.vec_store) {
                            u32x2 o;
                            o.x = float2_to_half2_bits(scaled(x[0], s), scaled(x[1], s));
                            o.y = float2_to_half2_bits(scaled(x[2], s), scaled(x[3], s));
                            *reinterpret_cast<u32x2 *>(dst) = o;
                        } else {
                            for (int e = 0; e < 4 && n + e < p.N; ++e) {
                                union { _Float16 f; uint16_t u; } cv;
                                cv.f = (_Float16)scaled(x[e], s);
                                dst[e] = cv.u;
                            }
                        }
                    }
                }
        }
    }
};

// NST: LDS stages.  Two are enough where a K-tile's MFMAs outlast the latency of the next K-tile's
// loads (256 x 256 tiles) or two workgroups share a CU; a launch with at most one workgroup per CU
// and smaller tiles takes three or four, so that loads run NST - 1 K-tiles ahead.
template <int KIND, int TM, int TN, int WAVES_M, int WAVES_N, int NST = 2>
struct LargeKernel {
    static_assert(KIND == kPlainF16 || KIND == kE4M3 || KIND == kE4M3Row, "NestedFP16 has a kernel of its own");
    static constexpr bool FP8 = kind_is_fp8(KIND);
    static constexpr bool PACKED_W = KIND == kE4M3;    // weight stage = packed 1 KB blocks as they are
    static constexpr int WAVES = WAVES_M * WAVES_N;
    static_assert(WAVES == 8, "two waves per SIMD: one loading (older), one not");
    static constexpr int THREADS = 64 * WAVES;
    static constexpr int WTM = TM / WAVES_M, WTN = TN / WAVES_N;
    static constexpr int STAGE = (TM + TN) * 128;      // bytes per LDS stage
    static constexpr int LDS_BYTES = NST * STAGE;
    static_assert(NST >= 2 && LDS_BYTES <= 160 * 1024, "LDS stages");
    typedef TileStore<KIND, TM, TN, WAVES_M, WAVES_N> Store;
    static_assert(TM * TN * 2 <= LDS_BYTES, "output tile must fit into the operand stages");

    // ---- MFMA tiling ------------------------------------------------------------------------
    // FP16 kinds: v_mfma_f32_16x16x32_f16.  Under the chip's power limit (which, not the issue
    // rate, bounds a full-chip FP16 GEMM on random operands) it sustains about 15 % more flops
    // than 32x32x16: it moves half as many accumulator registers per flop.  E4M3:
    // v_mfma_scale_f32_32x32x64_f8f6f4 (the 16x16x128 shape would need more fragment registers
    // than a wave with a 128x64 tile has).  A wave's tile is FNB x FMB blocks of MB weight rows x
    // MB tokens; a K-tile (128 bytes per row) is two substeps of 64 bytes per row; a fragment is
    // NCH 16-byte chunks per lane: lane l supplies row l % MB and bytes 16 * NCH * (l / MB) .. of
    // the substep's 64.
    static constexpr int MB = FP8 ? 32 : 16;
    static constexpr int SUBS = 2;
    static constexpr int NCH = FP8 ? 2 : 1;
    static constexpr int FMB = WTM / MB, FNB = WTN / MB;
    static constexpr int MF = FMB * FNB;                             // MFMAs per substep
    typedef typename std::conditional<MB == 32, floatx16, floatx4>::type AccT;
    // Slot plan of a substep.  The MFMAs run token block by token block (the FNB weight
    // fragments stay, the token fragments stream).  The first NPRE fragments of a substep (all
    // weight fragments, up to two token fragments) are fetched in the tail of the substep before
    // it, the other token fragments early in the substep itself, about two token blocks ahead of
    // their use.  The one barrier of a K-tile sits in its second substep behind the last read of
    // the current stage (slot QB): from there on the stage is free for K-tile kt+2; the loads of
    // kt+2 and the first reads of kt+1 follow it.
    static constexpr int NB0 = FMB < 2 ? FMB : 2;
    static constexpr int NPRE = FNB + NB0;
    static constexpr int NREST = FMB - NB0;
    static constexpr int RSTR = (3 * FNB) / 4 > 0 ? (3 * FNB) / 4 : 1;        // slots between the early token reads
    static constexpr int QB = NREST > 0 ? (NREST - 1) * RSTR + (MB == 32 ? 2 : 3) : 0;   // slot that starts with the barrier
    static constexpr int RPT = (NPRE + (MF - QB) - 1) / (MF - QB);            // look-ahead reads per tail slot
    static constexpr int TSLOTS = (NPRE + RPT - 1) / RPT;                     // tail slots that read
    static constexpr int TSTR = (MF - QB) / TSLOTS;                           // slots between them
    static constexpr int TAIL0 = MF - TSLOTS * TSTR;
    static_assert(QB < MF && TAIL0 >= QB && TSTR >= 1, "slot plan");

    struct Frags { intx4 a[FNB][NCH]; intx4 b[FMB][NCH]; };

    // the chunk slot of an LDS row that lane group g reads in substep s (see fp16_chunk_of_slot)
    static __device__ __forceinline__ int k_chunk(int s, int g, int q) { return 4 * s + NCH * g + q; }

    // LDS address of chunk q of a weight fragment: row, substep s, lane group g = l / MB.
    // Row-major weights: rows of 128 bytes, XOR-swizzled.  Packed E4M3: the stage holds the 1 KB blocks
    // as they are in memory, [row tile][2 blocks]; a substep is one block, and 16 lanes with
    // consecutive rows read 256 consecutive bytes.
    static __device__ __forceinline__ int w_addr(int row, int s, int g, int q) {
        if (PACKED_W) return (((row >> 4) * 2 + s) << 10) + (((row & 15) + 16 * (NCH * g + q)) << 4);
        return swz(row, k_chunk(s, g, q));
    }

    // fragment R of substep s in the order of first use: weight blocks 0..FNB-1, token blocks 0..FMB-1
    template <int R>
    static __device__ __forceinline__ void read_frag(Frags &f, const uint8_t *stage, int wm, int wn, int lane, int s) {
        const int r = lane % MB, g = lane / MB;
#pragma unroll
        for (int q = 0; q < NCH; ++q) {
            if constexpr (R < FNB)
                f.a[R][q] = *reinterpret_cast<const intx4 *>(stage + w_addr(wn * WTN + MB * R + r, s, g, q));
            else
                f.b[R - FNB][q] = *reinterpret_cast<const intx4 *>(
                    stage + TN * 128 + swz(wm * WTM + MB * (R - FNB) + r, k_chunk(s, g, q)));
        }
    }

    template <int R, int END>
    static __device__ __forceinline__ void read_frags(Frags &f, const uint8_t *stage, int wm, int wn, int lane, int s) {
        if constexpr (R < END) {
            read_frag<R>(f, stage, wm, wn, lane, s);
            read_frags<R + 1, END>(f, stage, wm, wn, lane, s);
        }
    }

    // weight rows are the "A" operand, tokens the "B" operand: a lane gets one token of the block
    // and groups of four consecutive weight rows
    template <int Q>
    static __device__ __forceinline__ void mfma_one(const Frags &f, AccT (&acc)[FNB][FMB]) {
        constexpr int j = Q / FNB, i = Q % FNB;
        if constexpr (FP8) {
            intx8 a = {f.a[i][0].x, f.a[i][0].y, f.a[i][0].z, f.a[i][0].w, f.a[i][NCH - 1].x, f.a[i][NCH - 1].y, f.a[i][NCH - 1].z, f.a[i][NCH - 1].w};
            intx8 b = {f.b[j][0].x, f.b[j][0].y, f.b[j][0].z, f.b[j][0].w, f.b[j][NCH - 1].x, f.b[j][NCH - 1].y, f.b[j][NCH - 1].z, f.b[j][NCH - 1].w};
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[i][j], 0, 0, 0, 0, 0, 0);
        } else {
            union { intx4 v; half8 h; } a, b;
            a.v = f.a[i][0];
            b.v = f.b[j][0];
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a.h, b.h, acc[i][j], 0, 0, 0);
        }
    }

    // ---- direct-to-LDS loads (buffer_load ... lds) -------------------------------------------
    // One wave instruction fills 1 KB of LDS = 8 tile rows in lane order (lane l -> row l/8,
    // physical chunk l%8), so the XOR swizzle is applied on the global side: lane l fetches
    // the logical chunk (l%8) ^ ((row>>1)&7) of its row.  No VGPR staging, no ds_write.
    // With two waves per SIMD the older one wins every arbitration and reaches the barrier long
    // before the younger one.  The loads are therefore issued by the older four waves only:
    // a load instruction blocks the issue of whatever is behind it while the address queue is
    // full, and those waves have the time to spare.
    static constexpr int DW = 4;                       // waves that issue direct-to-LDS loads
    static constexpr int XG = TM / 8 / DW;             // 8-row groups per loading wave, token tile
    static constexpr int WG8 = TN / 8 / DW;            // 8-row groups per loading wave, weight tile
    static constexpr int DMAS = XG + WG8;              // loads per loading wave per K-tile
    static constexpr int DPS = (DMAS + (MF - QB) - 1) / (MF - QB);     // loads per slot behind the barrier

    struct DmaOffsets {
        uint32_t x[XG], w[WG8];
        uint32_t kpos;                                 // this lane's K byte position in a K-tile
        int wbit;                                      // E4M3: which of a K-tile's two block columns this wave loads
    };

    static __device__ __forceinline__ void make_dma_offsets(DmaOffsets &o, const LargeParams &p, int wave, int lane) {
        const int pc = lane & 7;
        const int slot = pc ^ ((((wave & 1) << 2) + (lane >> 4)) & 7);  // (row >> 1) & 7 for row = gid*8 + lane/8
        const int c = FP8 ? slot : fp16_chunk_of_slot(slot);
        o.kpos = 16u * c;
#pragma unroll
        for (int i = 0; i < XG; ++i) o.x[i] = (uint32_t)((i * DW + wave) * 8 + (lane >> 3)) * (uint32_t)p.x_row_bytes + 16u * c;
#pragma unroll
        for (int i = 0; i < WG8; ++i) {
            if (PACKED_W) {
                // packed upper plane: load i of wave w is block b = i*DW + w of the stage, i.e. block
                // column (2*kt + b%2) of row tile b/2; lane l fetches chunk l
                const int b = i * DW + wave;
                o.w[i] = (uint32_t)((b >> 1) * p.kblocks + (b & 1)) * 1024u + 16u * lane;
            } else {
                o.w[i] = (uint32_t)((i * DW + wave) * 8 + (lane >> 3)) * (uint32_t)p.w_row_bytes + 16u * c;
            }
        }
        o.wbit = wave & 1;
    }

    typedef __attribute__((address_space(3))) uint8_t lds_byte;

    // the i-th of a wave's XG + WG8 direct-to-LDS loads of one K-tile (token rows first);
    // i is a constant at every call site
    static __device__ __forceinline__ void dma_one(int i, const DmaOffsets &o, uint32_t x_lim, uint32_t w_lim,
                                                   __amdgpu_buffer_rsrc_t rx, __amdgpu_buffer_rsrc_t rw,
                                                   lds_byte *stage, int wave, int kt) {
        const uint32_t kb = (uint32_t)kt * 128u;
        if (i < XG) {
            const uint32_t kill = (kb + o.kpos < x_lim) ? 0u : 0x80000000u;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (__attribute__((address_space(3))) void *)(stage + TN * 128 + (i * DW + wave) * 1024),
                                                     16, (o.x[i] + kb) | kill, 0, 0, 0);
        } else {
            const int j = i - XG;
            if (PACKED_W) {
                // w_lim = block columns of the plane; past them the load is sent out of range
                const uint32_t kill = ((uint32_t)(2 * kt + o.wbit) < w_lim) ? 0u : 0x80000000u;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (__attribute__((address_space(3))) void *)(stage + (j * DW + wave) * 1024),
                                                         16, (o.w[j] + (uint32_t)kt * 2048u) | kill, 0, 0, 0);
            } else {
                const uint32_t kill = (kb + o.kpos < w_lim) ? 0u : 0x80000000u;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (__attribute__((address_space(3))) void *)(stage + (j * DW + wave) * 1024),
                                                         16, (o.w[j] + kb) | kill, 0, 0, 0);
            }
        }
    }

    // ---- the K loop as an explicit instruction schedule ---------------------------------------
    // Every MFMA is followed by the few other instructions assigned to its slot and a scheduling
    // fence, so the order below is the order in the binary.  OLDER: one of the DW waves that
    // issue the direct-to-LDS loads; the loop exists once per role so that it has no branches
    // inside.  PAR: which of the two fragment sets the substep multiplies.
    struct Ctx {
        AccT (&acc)[FNB][FMB];
        Frags (&fr)[2];
        const DmaOffsets &dof;
        __amdgpu_buffer_rsrc_t rx, rw;
        uint8_t *lds;
        lds_byte *lds3;
        uint32_t x_lim, w_lim;
        int wave, lane, wm, wn;
        int kt, cur, nxt;                               // K-tile, its LDS stage, the next K-tile's
    };

    template <bool OLDER, int S, int PAR, int Q>
    static __device__ __forceinline__ void slot(Ctx &c) {
        constexpr bool last = (S == SUBS - 1);
        if constexpr (last && Q == QB) {
            // every read of the current stage has been issued; once all waves are here and their
            // loads of the next K-tile have landed (those of the NST - 2 K-tiles after it may stay
            // in flight), the stage is free and the next one complete
            if constexpr (OLDER) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((NST - 2) * DMAS) : "memory");
            else asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if constexpr (NST == 2) {
                __syncthreads();
            } else {
                // a bare barrier: the fence of __syncthreads() would drain the loads in flight.  What
                // it would order is ordered by the waits above: the next stage's loads have landed,
                // and every LDS read of the stage that is refilled next has returned.
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        mfma_one<Q>(c.fr[PAR], c.acc);
        if constexpr (Q % RSTR == 0 && Q / RSTR < NREST)
            read_frag<FNB + NB0 + Q / RSTR>(c.fr[PAR], c.lds + c.cur * STAGE, c.wm, c.wn, c.lane, S);
        if constexpr (Q >= TAIL0 && (Q - TAIL0) % TSTR == 0 && (Q - TAIL0) / TSTR < TSLOTS) {
            constexpr int r0 = (Q - TAIL0) / TSTR * RPT;
            read_frags<r0, (r0 + RPT < NPRE ? r0 + RPT : NPRE)>(c.fr[PAR ^ 1], c.lds + (last ? c.nxt : c.cur) * STAGE, c.wm, c.wn,
                                                                c.lane, last ? 0 : S + 1);
        }
        if constexpr (last && OLDER && Q >= QB) {
#pragma unroll
            for (int d = (Q - QB) * DPS; d < (Q - QB + 1) * DPS && d < DMAS; ++d)
                dma_one(d, c.dof, c.x_lim, c.w_lim, c.rx, c.rw, c.lds3 + c.cur * STAGE, c.wave, c.kt + NST);
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (Q + 1 < MF) slot<OLDER, S, PAR, Q + 1>(c);
    }

    template <bool OLDER>
    static __device__ __forceinline__ void k_loop(Ctx &c, int kt_begin, int kt_end) {
        int cur = 0;
        for (int kt = kt_begin; kt < kt_end; ++kt) {
            c.kt = kt;
            c.cur = cur;
            cur = cur + 1 == NST ? 0 : cur + 1;
            c.nxt = cur;
            __builtin_amdgcn_sched_barrier(0);
            slot<OLDER, 0, 0, 0>(c);
            slot<OLDER, 1, 1, 0>(c);
        }
    }

    static __device__ __forceinline__ void run(const LargeParams &p, uint8_t *lds, lds_byte *lds3) {
        const int lane = threadIdx.x & 63;
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const int wm = wave % WAVES_M, wn = wave / WAVES_M;
        int tm, tn;
        tile_of_block(p, blockIdx.x, tm, tn);
        const int m0 = tm * TM, n0 = tn * TN;
        const int split = blockIdx.y;
        const int kt_begin = split * p.ktiles_per_split;
        const int kt_end = min(kt_begin + p.ktiles_per_split, p.ktiles_total);

        const __amdgpu_buffer_rsrc_t rx = tile_rsrc(p.X, m0, min(TM, p.M - m0), p.x_row_bytes, p.k_bytes);
        const __amdgpu_buffer_rsrc_t rw = PACKED_W
            ? plane_rsrc(p.W0, n0, min(TN, p.N - n0), p.kblocks, 1024)
            : tile_rsrc(p.W0, n0, min(TN, p.N - n0), p.w_row_bytes, p.k_bytes);
        DmaOffsets dof;
        make_dma_offsets(dof, p, wave, lane);
        const uint32_t x_lim = (uint32_t)p.k_bytes;
        const uint32_t w_lim = PACKED_W ? (uint32_t)p.kblocks : (uint32_t)p.k_bytes;

        // NST LDS stages; tokens and weights go straight from global memory into LDS.
        if (wave < DW) {
#pragma unroll
            for (int st = 0; st < NST; ++st)
#pragma unroll
                for (int i = 0; i < DMAS; ++i)
                    dma_one(i, dof, x_lim, w_lim, rx, rw, lds3 + st * STAGE, wave, kt_begin + st);
        }
        // the loads of K-tile kt_begin (a wave that issued none passes straight through)
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NST - 1) * DMAS) : "memory");
        __syncthreads();

        AccT acc[FNB][FMB];
#pragma unroll
        for (int i = 0; i < FNB; ++i)
#pragma unroll
            for (int j = 0; j < FMB; ++j)
#pragma unroll
                for (int q = 0; q < (MB == 32 ? 16 : 4); ++q) acc[i][j][q] = 0.f;
        Frags fr[2];
        Ctx c{acc, fr, dof, rx, rw, lds, lds3, x_lim, w_lim, wave, lane, wm, wn, kt_begin, 0, 0};
        read_frags<0, NPRE>(fr[0], lds, wm, wn, lane, 0);
        if (wave < DW) k_loop<true>(c, kt_begin, kt_end);
        else k_loop<false>(c, kt_begin, kt_end);
        // the loads of the K-tiles past the end are still in flight: they must have landed
        // before the LDS is reused for the output tile or handed back
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (p.row_store && gridDim.y == 1) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // the look-ahead fragment reads
            __syncthreads();
            Store::epilogue_lds(p, acc, m0, n0, wm, wn, lane, wave, lds);
        } else {
            Store::epilogue(p, acc, m0, n0, wm, wn, lane, split);
        }
    }

};

template <int KIND, int TM, int TN, int WAVES_M, int WAVES_N, int NST>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N)
large_gemm_kernel(LargeParams p) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
    typedef LargeKernel<KIND, TM, TN, WAVES_M, WAVES_N, NST> Kern;
    Kern::run(p, lds_raw, (typename Kern::lds_byte *)lds_raw);
}

// ---- NestedFP16 with the weights kept out of LDS ------------------------------------------------
// Eight waves side by side along the weight rows: a wave owns TN/8 weight rows and all TM tokens
// of the tile, so every weight is needed by exactly one wave.  The wave loads 16 bytes of each
// plane per lane straight into registers (lane l: row l % 16, columns 16 * (l / 16) .. +15 of a
// 64-column block -- 16 rows x 64 bytes per instruction from row-major planes, one contiguous
// kilobyte from packed ones), merges them there (Sec. 4.2, Alg. 1) and feeds the result to the MFMA
// as it is (WK = kPlainF16Packed: FP16 weights in packed blocks, no merge): the sum over k
// does not care about the order of k, so substep s of a K-tile takes columns 16 g + 8 s .. + 7
// from lane group g, and the token fragments are read from LDS in the same order (chunk
// 2 g + s of the 128-byte row, see fp16_chunk_of_slot).  No ds_write, no weight tile in LDS; LDS holds four stages of
// the token tile only (loads run three K-tiles ahead), and the one barrier per K-tile sits
// at its end and waits for no LDS read.
// DEEP: a ring of eight token stages with the token loads six and the plane loads four K-tiles ahead
// (tiles of at most 128 tokens, launches that do not fill the chip: there a K-tile's MFMAs are
// short against the latency of a load) instead of four stages and three / two K-tiles.
template <int TM, int TN, int WK, bool DEEP = false, bool NT = false>
struct BypassKernel {
    static_assert(WK == kNestedF16 || WK == kNestedF16Row || WK == kPlainF16Packed, "weights that go through registers");
    static constexpr bool MERGE = kind_is_nested(WK);
    static constexpr bool ROWMAJOR = WK == kNestedF16Row;
    // NT: the launch has one token tile, so every weight is read once; packed blocks (whole lines per
    // instruction) are then marked non-temporal, as in the streaming kernel.  The 64-token tiles always
    // are; the 128-token tiles on the large layers (timed: 6-10 % faster from about 100 Mi weights on at
    // M = 96 and 128, a few per cent slower on the small ones).
    static constexpr int POLICY = (!ROWMAJOR && (NT || TM == 64)) ? 2 : 0;
    static constexpr int BLOCK_BYTES = 1024 * kind_elem_bytes(WK);   // packed kinds: one 16 x 64 block
    typedef TileStore<kNestedF16, TM, TN, 1, 8> Store;
    static constexpr int DW = 4;                               // waves that issue the token loads
    static constexpr int WTN = TN / 8;
    static constexpr int FMB = TM / 16, FNB = WTN / 16;
    static constexpr int MF = FMB * FNB;                       // MFMAs per substep
    // (a ring of eight stages with the token loads six and the plane loads three K-tiles ahead was
    // no faster for the 64-token tiles)
    static constexpr int NST = DEEP ? 8 : 4;                   // LDS stages of the token tile
    static constexpr int XA = DEEP ? 6 : 3;                    // token loads run this many K-tiles ahead
    static constexpr int NRAW = DEEP ? 4 : 2;                  // plane blocks are loaded this many K-tiles ahead
    static_assert(XA >= 3 && XA < NST && NRAW <= XA && NRAW >= 2, "the stage being filled is neither the one in use nor the next");
    static_assert(NST * TM * 128 <= 160 * 1024, "LDS stages");
    static constexpr int STAGE = TM * 128;
    static constexpr int LDS_BYTES = NST * STAGE > TM * TN * 2 ? NST * STAGE : TM * TN * 2;
    static constexpr int XG = TM / 8 / DW;                     // loads per loading wave per K-tile
    static constexpr int LEAD = 2;                             // token fragments are read this many blocks ahead
    static constexpr int NMQ = 2 * FNB;                        // merges of four weights per substep
    static constexpr int MQS = MF / NMQ;                       // slots between them
    static constexpr int DQS = MF / XG;                        // slots between token loads
    static_assert(FNB <= 2 && FMB > LEAD && MF % NMQ == 0 && MF % XG == 0 && MQS >= 2, "slot plan");
    typedef __attribute__((address_space(3))) uint8_t lds_byte;

    // one K-tile of the wave's weights: 16 bytes of each plane, or the two halves of a packed FP16 block
    struct Raw { u32x4 u[FNB], l[FNB]; };

    struct Ctx {
        floatx4 (&acc)[FNB][FMB];
        intx4 (&a)[2][FNB];                                    // merged weight fragments of substeps 0 / 1
        intx4 (&b)[2][FMB];                                    // token fragments (a few are live at a time)
        Raw (&raw)[NRAW];
        __amdgpu_buffer_rsrc_t rx, rw0, rw1;
        uint32_t x_off, x_step, x_kpos, x_lim;               // offset of the wave's first load, step between its loads
        uint32_t w_off, w_istep, w_kpos, w_lim;              // lane + wave part, step between row tiles, column test
        const uint8_t *lds;
        lds_byte *lds3;
        int wave, lane;
        int kt, st;                                            // K-tile, its LDS stage
    };

    template <int J>
    static __device__ __forceinline__ void read_b(intx4 &dst, const uint8_t *stage, int lane, int s) {
        dst = *reinterpret_cast<const intx4 *>(stage + swz(16 * J + (lane & 15), 4 * s + (lane >> 4)));
    }

    // the lane's columns of K-tile kt lie inside K (w_kpos = 16 (l / 16) for row-major planes, whose
    // rows have no padding; 0 for packed blocks, which are zero-padded to whole blocks); otherwise
    // the load is sent out of the buffer's range and returns zero
    static __device__ __forceinline__ void load_raw(Raw &r, const Ctx &c, int kt) {
        const uint32_t kill = ((uint32_t)kt * 64u + c.w_kpos < c.w_lim) ? 0u : 0x80000000u;
#pragma unroll
        for (int i = 0; i < FNB; ++i) {
            const uint32_t off = (c.w_off + (uint32_t)i * c.w_istep + (uint32_t)kt * (ROWMAJOR ? 64u : (uint32_t)BLOCK_BYTES)) | kill;
            r.u[i] = __builtin_amdgcn_raw_buffer_load_b128(c.rw0, off, 0, POLICY);
            if (MERGE) r.l[i] = __builtin_amdgcn_raw_buffer_load_b128(c.rw1, off, 0, POLICY);
            else r.l[i] = __builtin_amdgcn_raw_buffer_load_b128(c.rw0, off + 1024u, 0, POLICY);
        }
    }

    // four weights of row tile I: dwords H (substep 0) or 2 + H (substep 1) of the lane's chunk of
    // each plane; packed FP16 weights are taken as they are (first half block = substep 0)
    template <int S, int I, int H>
    static __device__ __forceinline__ void merge_part(intx4 &dst, const Raw &r) {
        if constexpr (MERGE) {
            uint32_t w01, w23;
            merge4(r.u[I][2 * S + H], r.l[I][2 * S + H], w01, w23);
            dst[2 * H] = (int)w01;
            dst[2 * H + 1] = (int)w23;
        } else {
            dst[2 * H] = (int)(S == 0 ? r.u[I][2 * H] : r.l[I][2 * H]);
            dst[2 * H + 1] = (int)(S == 0 ? r.u[I][2 * H + 1] : r.l[I][2 * H + 1]);
        }
    }

    static __device__ __forceinline__ void dma_x(const Ctx &c, int i, int kt) {
        const uint32_t kb = (uint32_t)kt * 128u;
        const uint32_t kill = (kb + c.x_kpos < c.x_lim) ? 0u : 0x80000000u;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(c.rx, (__attribute__((address_space(3))) void *)(c.lds3 + (kt & (NST - 1)) * STAGE + (i * DW + c.wave) * 1024),
                                                 16, (c.x_off + (uint32_t)i * c.x_step + kb) | kill, 0, 0, 0);
    }

    // PAR: which register set holds the plane blocks of this K-tile (the one after it holds the next)
    template <bool OLDER, int S, int PAR, int Q>
    static __device__ __forceinline__ void slot(Ctx &c) {
        constexpr int j = Q / FNB, i = Q % FNB;
        {
            union { intx4 v; half8 h; } a, b;
            a.v = c.a[S][i];
            b.v = c.b[S][j];
            c.acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a.h, b.h, c.acc[i][j], 0, 0, 0);
        }
        if constexpr (i == 0) {
            // token fragment LEAD blocks ahead: this substep, the next one, or the next K-tile
            if constexpr (j + LEAD < FMB) read_b<j + LEAD>(c.b[S][j + LEAD], c.lds + c.st * STAGE, c.lane, S);
            else if constexpr (S == 0) read_b<j + LEAD - FMB>(c.b[1][j + LEAD - FMB], c.lds + c.st * STAGE, c.lane, 1);
            else read_b<j + LEAD - FMB>(c.b[0][j + LEAD - FMB], c.lds + ((c.st + 1) & (NST - 1)) * STAGE, c.lane, 0);
        }
        if constexpr (Q % MQS == MQS - 1) {
            // substep 0 merges this K-tile's second half, substep 1 the next K-tile's first half
            constexpr int m = Q / MQS;
            if constexpr (S == 0) merge_part<1, m / 2, m % 2>(c.a[1][m / 2], c.raw[PAR]);
            else merge_part<0, m / 2, m % 2>(c.a[0][m / 2], c.raw[(PAR + 1) % NRAW]);
        }
        if constexpr (OLDER && S == 0 && Q % DQS == 0) dma_x(c, Q / DQS, c.kt + XA);
        if constexpr (S == 1 && Q == 0) load_raw(c.raw[PAR], c, c.kt + NRAW);  // its blocks are merged
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (Q + 1 < MF) slot<OLDER, S, PAR, Q + 1>(c);
    }

    template <bool OLDER, int PAR>
    static __device__ __forceinline__ void k_tile(Ctx &c) {
        __builtin_amdgcn_sched_barrier(0);
        slot<OLDER, 0, PAR, 0>(c);
        slot<OLDER, 1, PAR, 0>(c);
        // The token loads of K-tile kt+2 (issued during kt+2-XA) must have landed before anybody
        // reads them (from the tail of kt+1 on).  Younger than them in this wave, and allowed to
        // be in flight: the plane loads of that K-tile and all loads of the XA-2 K-tiles since
        // (for XA = 3 the count is rounded down to this K-tile's loads).
        if constexpr (OLDER) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(XA == 3 ? XG + 2 * FNB : 2 * FNB + (XA - 2) * (XG + 2 * FNB)) : "memory");
        // a bare barrier: __syncthreads() carries a release fence, which would drain the token loads
        // issued in this K-tile.  What the fence would order is ordered by the wait above (loads
        // that have to be visible) and by the MFMAs, which have consumed every LDS read of the
        // stage that is refilled next.
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    }

    template <bool OLDER>
    static __device__ __forceinline__ void k_loop(Ctx &c, int kt_begin, int kt_end) {
        // no branch inside the loop body: the compiler then counts the loads in flight exactly
        // instead of draining them at the loop head
        int kt = kt_begin;
        for (; kt + NRAW <= kt_end; kt += NRAW) k_tiles<OLDER, 0, NRAW>(c, kt);
        tail<OLDER, 0>(c, kt, kt_end);
    }

    // K-tiles kt + P .. kt + END - 1, on register sets P .. END - 1
    template <bool OLDER, int P, int END>
    static __device__ __forceinline__ void k_tiles(Ctx &c, int kt) {
        c.kt = kt + P;
        c.st = (kt + P) & (NST - 1);
        k_tile<OLDER, P>(c);
        if constexpr (P + 1 < END) k_tiles<OLDER, P + 1, END>(c, kt);
    }

    // the last 0 .. NRAW - 1 K-tiles
    template <bool OLDER, int P>
    static __device__ __forceinline__ void tail(Ctx &c, int kt, int kt_end) {
        if constexpr (P + 1 < NRAW) {
            if (kt + P < kt_end) {
                k_tiles<OLDER, P, P + 1>(c, kt);
                tail<OLDER, P + 1>(c, kt, kt_end);
            }
        }
    }

    static __device__ __forceinline__ void run(const LargeParams &p, uint8_t *lds, lds_byte *lds3) {
        const int lane = threadIdx.x & 63;
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        int tm, tn;
        tile_of_block(p, blockIdx.x, tm, tn);
        const int m0 = tm * TM, n0 = tn * TN;
        const int split = blockIdx.y;
        // the LDS stage of a K-tile is kt % 4: start the slice on a multiple of 4 as far as the ring goes
        const int kt_begin = split * p.ktiles_per_split;
        const int kt_end = min(kt_begin + p.ktiles_per_split, p.ktiles_total);

        floatx4 acc[FNB][FMB];
#pragma unroll
        for (int i = 0; i < FNB; ++i)
#pragma unroll
            for (int j = 0; j < FMB; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
        intx4 a[2][FNB], b[2][FMB];
        Raw raw[NRAW];
        const int w_rows = min(TN, p.N - n0);
        Ctx c{acc, a, b, raw,
              tile_rsrc(p.X, m0, min(TM, p.M - m0), p.x_row_bytes, p.k_bytes),
              ROWMAJOR ? tile_rsrc(p.W0, n0, w_rows, p.w_row_bytes, p.K) : plane_rsrc(p.W0, n0, w_rows, p.kblocks, BLOCK_BYTES),
              ROWMAJOR ? tile_rsrc(p.W1, n0, w_rows, p.w_row_bytes, p.K)
                       : plane_rsrc(MERGE ? p.W1 : p.W0, n0, w_rows, p.kblocks, BLOCK_BYTES),
              0u, (uint32_t)(DW * 8) * (uint32_t)p.x_row_bytes, 0u, (uint32_t)p.k_bytes, 0u, 0u, 0u, 0u, lds, lds3, wave, lane,
              kt_begin, 0};
        {
            const int pc = lane & 7;
            const int ch = fp16_chunk_of_slot(pc ^ ((((wave & 1) << 2) + (lane >> 4)) & 7));   // (row >> 1) & 7 for row = gid*8 + lane/8
            c.x_kpos = 16u * ch;
            c.x_off = (uint32_t)(wave * 8 + (lane >> 3)) * (uint32_t)p.x_row_bytes + 16u * ch;
            if (ROWMAJOR) {
                c.w_off = (uint32_t)(FNB * wave * 16 + (lane & 15)) * (uint32_t)p.w_row_bytes + 16u * (uint32_t)(lane >> 4);
                c.w_istep = 16u * (uint32_t)p.w_row_bytes;
                c.w_kpos = 16u * (uint32_t)(lane >> 4);
                c.w_lim = (uint32_t)p.K;
            } else {
                c.w_off = (uint32_t)(FNB * wave * p.kblocks) * (uint32_t)BLOCK_BYTES + (uint32_t)lane * 16u;
                c.w_istep = (uint32_t)p.kblocks * (uint32_t)BLOCK_BYTES;
                c.w_kpos = 0u;
                c.w_lim = (uint32_t)p.kblocks * 64u;
            }
        }
        // token tiles of the first XA K-tiles, plane blocks of the first NRAW
        if (wave < DW) {
#pragma unroll
            for (int d = 0; d < XA; ++d)
#pragma unroll
                for (int i = 0; i < XG; ++i) dma_x(c, i, kt_begin + d);
        }
#pragma unroll
        for (int d = 0; d < NRAW; ++d) load_raw(raw[d], c, kt_begin + d);
        // (in order: once the first plane blocks are here, the token loads issued before them are too)
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NRAW - 1) * 2 * FNB) : "memory");
        merge_part<0, 0, 0>(a[0][0], raw[0]);
        merge_part<0, 0, 1>(a[0][0], raw[0]);
        if constexpr (FNB > 1) {
            merge_part<0, FNB - 1, 0>(a[0][FNB - 1], raw[0]);
            merge_part<0, FNB - 1, 1>(a[0][FNB - 1], raw[0]);
        }
        __syncthreads();
        c.st = kt_begin & (NST - 1);
        {
            const uint8_t *st0 = lds + c.st * STAGE;
            read_b<0>(b[0][0], st0, lane, 0);
            if (LEAD > 1) read_b<1>(b[0][1], st0, lane, 0);
            if (LEAD > 2) read_b<2>(b[0][2], st0, lane, 0);
            if (LEAD > 3) read_b<3>(b[0][3], st0, lane, 0);
        }
        if (wave < DW) k_loop<true>(c, kt_begin, kt_end);
        else k_loop<false>(c, kt_begin, kt_end);
        // token loads of K-tiles past the end are still in flight: they must have landed before the
        // LDS is reused for the output tile or handed back
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        // (keeps the epilogue's address arithmetic behind the loop, where registers are free)
        int lane_out = lane;
        asm volatile("" : "+v"(lane_out));
        if (p.row_store && gridDim.y == 1) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // the look-ahead fragment reads
            __syncthreads();
            Store::epilogue_lds(p, acc, m0, n0, 0, wave, lane_out, wave, lds);
        } else {
            Store::epilogue(p, acc, m0, n0, 0, wave, lane_out, split);
        }
    }
};

template <int TM, int TN, int WK, bool DEEP, bool NT>
__global__ void __launch_bounds__(512)
nested_bypass_kernel(LargeParams p) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
    typedef BypassKernel<TM, TN, WK, DEEP, NT> Kern;
    Kern::run(p, lds_raw, (typename Kern::lds_byte *)lds_raw);
}

// ---- FP8 mode on at most 64 tokens per tile: E4M3 weights through registers ---------------------
// The same layout of work as nested_bypass_kernel (eight waves side by side along the weight rows,
// packed 1 KB blocks loaded 16 bytes per lane, token tile in a ring of four LDS stages), for
// batches where the weight stream is the bound.  A K-tile is 128 bytes of a token row and two
// blocks of the upper plane; lane group g = l / 16 holds columns 16 g .. + 15 of both blocks, 32
// bytes, which is one operand of v_mfma_f32_16x16x128_f8f6f4, and reads the same bytes of its token
// (chunks g and 4 + g of the row).  A token block's fragment of K-tile kt + 1 is read right behind
// the block's MFMAs of K-tile kt, into the same registers.
template <int TM, int TN, bool ROWMAJOR>
struct E4m3BypassKernel {
    typedef TileStore<kE4M3, TM, TN, 1, 8, 16> Store;
    static constexpr int DW = 4;                               // waves that issue the token loads
    static constexpr int WTN = TN / 8;
    static constexpr int FMB = TM / 16, FNB = WTN / 16;
    static constexpr int NST = 8;                              // LDS stages of the token tile
    static constexpr int XA = 6;                               // token loads run this many K-tiles ahead
    static constexpr int NRAW = 4;                             // plane blocks are loaded this many K-tiles ahead
    static constexpr int STAGE = TM * 128;
    static constexpr int LDS_BYTES = NST * STAGE > TM * TN * 2 ? NST * STAGE : TM * TN * 2;
    static constexpr int XG = TM / 8 / DW;                     // loads per loading wave per K-tile
    static_assert(XG >= 1 && FNB >= 1 && FNB <= 2, "tile shape");
    static_assert(XA >= 3 && XA < NST && NRAW <= XA, "the stage being filled is neither the one in use nor the next");
    typedef __attribute__((address_space(3))) uint8_t lds_byte;

    static constexpr int POLICY = (!ROWMAJOR && TM == 64) ? 2 : 0;   // packed blocks, read once per launch: non-temporal
    struct Raw { intx4 u[FNB][2]; };                           // one K-tile of the wave's plane blocks
    struct Tok { intx4 q[FMB][2]; };                           // one K-tile of token fragments

    struct Ctx {
        floatx4 (&acc)[FNB][FMB];
        Raw (&raw)[NRAW];
        Tok &tok;                                              // block J is re-read for the next K-tile right behind its MFMAs
        __amdgpu_buffer_rsrc_t rx, rw;
        uint32_t x_off, x_step, x_kpos, x_lim;
        uint32_t w_off, w_istep, w_kpos, w_lim;              // as in the NestedFP16 kernel
        const uint8_t *lds;
        lds_byte *lds3;
        int wave, lane;
        int kt;
    };

    static __device__ __forceinline__ void load_raw(Raw &r, const Ctx &c, int kt) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t kill = ((uint32_t)(2 * kt + h) * 64u + c.w_kpos < c.w_lim) ? 0u : 0x80000000u;
#pragma unroll
            for (int i = 0; i < FNB; ++i)
                r.u[i][h] = __builtin_bit_cast(intx4, __builtin_amdgcn_raw_buffer_load_b128(
                    c.rw, (c.w_off + (uint32_t)i * c.w_istep + (uint32_t)(2 * kt + h) * (ROWMAJOR ? 64u : 1024u)) | kill, 0, POLICY));
        }
    }

    static __device__ __forceinline__ void dma_x(const Ctx &c, int i, int kt) {
        const uint32_t kb = (uint32_t)kt * 128u;
        const uint32_t kill = (kb + c.x_kpos < c.x_lim) ? 0u : 0x80000000u;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(c.rx, (__attribute__((address_space(3))) void *)(c.lds3 + (kt & (NST - 1)) * STAGE + (i * DW + c.wave) * 1024),
                                                 16, (c.x_off + (uint32_t)i * c.x_step + kb) | kill, 0, 0, 0);
    }

    template <int J>
    static __device__ __forceinline__ void read_tok(Tok &t, const uint8_t *stage, int lane) {
        t.q[J][0] = *reinterpret_cast<const intx4 *>(stage + swz(16 * J + (lane & 15), lane >> 4));
        t.q[J][1] = *reinterpret_cast<const intx4 *>(stage + swz(16 * J + (lane & 15), 4 + (lane >> 4)));
    }

    template <int J>
    static __device__ __forceinline__ void block(Ctx &c, const Raw &r, const uint8_t *next_stage) {
        const intx8 b = __builtin_shufflevector(c.tok.q[J][0], c.tok.q[J][1], 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
        for (int i = 0; i < FNB; ++i) {
            const intx8 a = __builtin_shufflevector(r.u[i][0], r.u[i][1], 0, 1, 2, 3, 4, 5, 6, 7);
            c.acc[i][J] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c.acc[i][J], 0, 0, 0, 0, 0, 0);
        }
        read_tok<J>(c.tok, next_stage, c.lane);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (J + 1 < FMB) block<J + 1>(c, r, next_stage);
    }

    // PAR: which register set holds this K-tile's plane blocks
    template <bool OLDER, int PAR>
    static __device__ __forceinline__ void k_tile(Ctx &c) {
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (OLDER) {
#pragma unroll
            for (int i = 0; i < XG; ++i) dma_x(c, i, c.kt + XA);
        }
        block<0>(c, c.raw[PAR], c.lds + ((c.kt + 1) & (NST - 1)) * STAGE);
        load_raw(c.raw[PAR], c, c.kt + NRAW);                  // its blocks are used up
        // The token loads of K-tile kt+2 (issued during kt+2-XA) must have landed before anybody
        // reads them (during kt+1).  Younger than them in this wave, and allowed to be in flight:
        // the plane loads of that K-tile and all loads of the XA-2 K-tiles since.
        if constexpr (OLDER) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * FNB + (XA - 2) * (XG + 2 * FNB)) : "memory");
        // a bare barrier: __syncthreads() carries a release fence, which would drain the token loads
        // just issued.  What the fence would order is ordered by the wait above (loads that have to
        // be visible) and by the MFMAs that consumed every LDS read of the stage refilled next.
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    }

    template <bool OLDER>
    static __device__ __forceinline__ void k_loop(Ctx &c, int kt_begin, int kt_end) {
        static_assert(NRAW == 4, "unrolled by the number of register sets");
        int kt = kt_begin;
        for (; kt + 4 <= kt_end; kt += 4) {
            c.kt = kt;
            k_tile<OLDER, 0>(c);
            c.kt = kt + 1;
            k_tile<OLDER, 1>(c);
            c.kt = kt + 2;
            k_tile<OLDER, 2>(c);
            c.kt = kt + 3;
            k_tile<OLDER, 3>(c);
        }
        if (kt < kt_end) {
            c.kt = kt;
            k_tile<OLDER, 0>(c);
            if (kt + 1 < kt_end) {
                c.kt = kt + 1;
                k_tile<OLDER, 1>(c);
                if (kt + 2 < kt_end) {
                    c.kt = kt + 2;
                    k_tile<OLDER, 2>(c);
                }
            }
        }
    }

    static __device__ __forceinline__ void run(const LargeParams &p, uint8_t *lds, lds_byte *lds3) {
        const int lane = threadIdx.x & 63;
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        int tm, tn;
        tile_of_block(p, blockIdx.x, tm, tn);
        const int m0 = tm * TM, n0 = tn * TN;
        const int split = blockIdx.y;
        const int kt_begin = split * p.ktiles_per_split;
        const int kt_end = min(kt_begin + p.ktiles_per_split, p.ktiles_total);

        floatx4 acc[FNB][FMB];
#pragma unroll
        for (int i = 0; i < FNB; ++i)
#pragma unroll
            for (int j = 0; j < FMB; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
        Raw raw[NRAW];
        Tok tok;
        const int w_rows = min(TN, p.N - n0);
        Ctx c{acc, raw, tok,
              tile_rsrc(p.X, m0, min(TM, p.M - m0), p.x_row_bytes, p.k_bytes),
              ROWMAJOR ? tile_rsrc(p.W0, n0, w_rows, p.w_row_bytes, p.K) : plane_rsrc(p.W0, n0, w_rows, p.kblocks, 1024),
              0u, (uint32_t)(DW * 8) * (uint32_t)p.x_row_bytes, 0u, (uint32_t)p.k_bytes, 0u, 0u, 0u, 0u, lds, lds3, wave, lane,
              kt_begin};
        {
            const int ch = (lane & 7) ^ ((((wave & 1) << 2) + (lane >> 4)) & 7);    // (row >> 1) & 7 for row = gid*8 + lane/8
            c.x_kpos = 16u * ch;
            c.x_off = (uint32_t)(wave * 8 + (lane >> 3)) * (uint32_t)p.x_row_bytes + 16u * ch;
            if (ROWMAJOR) {
                c.w_off = (uint32_t)(FNB * wave * 16 + (lane & 15)) * (uint32_t)p.w_row_bytes + 16u * (uint32_t)(lane >> 4);
                c.w_istep = 16u * (uint32_t)p.w_row_bytes;
                c.w_kpos = 16u * (uint32_t)(lane >> 4);
                c.w_lim = (uint32_t)p.K;
            } else {
                c.w_off = (uint32_t)(FNB * wave * p.kblocks) * 1024u + (uint32_t)lane * 16u;
                c.w_istep = (uint32_t)p.kblocks * 1024u;
                c.w_kpos = 0u;
                c.w_lim = (uint32_t)p.kblocks * 64u;
            }
        }
        // token tiles of the first XA K-tiles, plane blocks of the first NRAW
        if (wave < DW) {
#pragma unroll
            for (int d = 0; d < XA; ++d)
#pragma unroll
                for (int i = 0; i < XG; ++i) dma_x(c, i, kt_begin + d);
        }
#pragma unroll
        for (int d = 0; d < NRAW; ++d) load_raw(raw[d], c, kt_begin + d);
        // the token tiles of the first two K-tiles: in order, everything but the later token loads
        // and the plane loads has landed
        if (wave < DW) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((XA - 2) * XG + NRAW * 2 * FNB) : "memory");
        __syncthreads();
        {
            const uint8_t *st0 = lds + (kt_begin & (NST - 1)) * STAGE;
            read_tok<0>(tok, st0, lane);
            if constexpr (FMB > 1) read_tok<1>(tok, st0, lane);
            if constexpr (FMB > 2) read_tok<2>(tok, st0, lane);
            if constexpr (FMB > 3) read_tok<3>(tok, st0, lane);
            static_assert(FMB <= 4, "prologue reads");
        }
        if (wave < DW) k_loop<true>(c, kt_begin, kt_end);
        else k_loop<false>(c, kt_begin, kt_end);
        // token loads of K-tiles past the end are still in flight: they must have landed before the
        // LDS is reused for the output tile or handed back
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (p.row_store && gridDim.y == 1) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // the look-ahead fragment reads
            __syncthreads();
            Store::epilogue_lds(p, acc, m0, n0, 0, wave, lane, wave, lds);
        } else {
            Store::epilogue(p, acc, m0, n0, 0, wave, lane, split);
        }
    }
};

template <int TM, int TN, bool ROWMAJOR>
__global__ void __launch_bounds__(512)
e4m3_bypass_kernel(LargeParams p) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
    typedef E4m3BypassKernel<TM, TN, ROWMAJOR> Kern;
    Kern::run(p, lds_raw, (typename Kern::lds_byte *)lds_raw);
}

struct LargeConfig { int tm, tn, split, deep; };

// Tile shape and K split from a small cost model.  The workgroups are dealt round-robin to the
// 256 CUs; a workgroup costs a fixed part plus a time per K-tile that depends on the tile shape
// and the weight kind; two 128x128 workgroups share a CU and together run s2 times faster than
// one after the other; a layer cannot finish before its weights have crossed the memory bus
// once; a split adds a reduction launch plus the traffic of the fp32 partials.  The constants
// are a least-squares fit (microseconds) to sweeps of every shape and split over M = 128 ...
// 4096 on the four Llama-3-8B layer shapes and a square 8192 layer.
struct TileCost { double tk, tfix; };                  // per K-tile, per workgroup
static const int kTileShapes[4][2] = {{256, 256}, {256, 128}, {128, 256}, {128, 128}};   // tokens x weight rows
static const TileCost kTileCost[3][4] = {
    {{1.353, 0.0}, {1.053, 0.07}, {1.098, 0.0}, {0.848, 0.0}},      // plain FP16
    {{1.242, 2.30}, {0.873, 0.75}, {0.887, 0.17}, {0.542, 0.0}},    // NestedFP16
    {{1.317, 4.39}, {1.061, 2.10}, {1.089, 2.28}, {0.864, 1.01}},   // E4M3
};
static const double kPairSpeedup[3] = {1.58, 1.02, 1.51};
// The same tile shapes with the deeper load pipeline (three or four LDS stages, one workgroup per
// CU, no pair speed-up): per K-tile about a quarter cheaper for the kernels whose weights go through
// LDS, at a higher fixed cost; nothing gained on the register path (NestedFP16), which does not use it.
// Least-squares fit to a sweep of every shape, split and pipeline depth over M = 128 ... 2048 on six
// Llama-3 8B / 70B layer shapes.
static const TileCost kDeepTileCost[3][4] = {
    {{0, 0}, {0.863, 1.56}, {0.900, 1.71}, {0.585, 2.50}},         // plain FP16
    {{0, 0}, {0, 0}, {0, 0}, {0, 0}},                               // NestedFP16: not used
    {{0, 0}, {0.978, 2.96}, {0.938, 2.77}, {0.606, 2.61}},         // E4M3
};
static const int kSplits[] = {1, 2, 3, 4, 6, 8};

// split-K cost: the reduction kernel's launch plus its traffic
static double split_cost(int64_t M, int64_t N, int slices, double launch_us, double bytes_per_us) {
    return launch_us + 8.0 * (double)M * (double)N * slices / bytes_per_us;
}

// At most 64 tokens: one 64 x 128 tile shape per weight kind and only the split to choose.  Such a
// launch is bound by the weight stream, whose rate depends on how many workgroups pull on it.
// Constants from timings of the four splits on six layer shapes at M = 64.
struct Tile64Cost {
    double tk, tfix;        // microseconds per K-tile and per workgroup
    int slots;              // workgroups the chip holds at a time
    double rate, rate512;   // bytes per microsecond of the weight stream (from 512 workgroups on)
    double few;             // exponent of the rate's fall below 256 workgroups
};
static const Tile64Cost kTile64Cost[3] = {
    {0.7, 0.4, 512, 4.5e6, 5.5e6, 0.5},       // plain FP16 (LDS kernel, three workgroups per CU)
    {0.466, 0.4, 512, 5.25e6, 5.5e6, 0.5},    // NestedFP16 (register path, two per CU)
    {0.35, 0.4, 256, 5.5e6, 5.5e6, 0.3},      // E4M3 (register path, one per CU)
};
static LargeConfig choose_tile64(int cls, int64_t M, int64_t N, int kt) {
    const Tuning &t = tuning();
    const Tile64Cost &tc = kTile64Cost[cls];
    LargeConfig c;
    c.tm = 64;  c.tn = 128;  c.split = 1;  c.deep = 0;
    const int64_t tiles = ((M + 63) / 64) * ((N + 127) / 128);
    double best = 1e30;
    for (int split : {1, 2, 3, 4, 6, 8}) {
        if (t.large_split > 0) split = (int)(t.large_split < kt ? t.large_split : kt);
        else if (split > 1 && split > kt / 4) break;
        const int per = (kt + split - 1) / split;
        const int slices = (kt + per - 1) / per;
        const int64_t wgs = tiles * slices;
        const int64_t rounds = (wgs + tc.slots - 1) / tc.slots;
        double time = (double)rounds * (tc.tfix + per * tc.tk);
        double floor_t = (double)N * (double)kt * 128.0 / (wgs < 512 ? tc.rate : tc.rate512);
        if (wgs < 256) floor_t *= std::pow(256.0 / (double)wgs, tc.few);
        // the weight stream is shared per CU: workgroups beyond one per CU that do not make a whole
        // further round leave most CUs waiting for a few (measured: 320 workgroups take 1.3-1.5 times
        // as long as 240 with the same bytes)
        if (wgs > 256) floor_t *= (double)(((wgs + 255) / 256) * 256) / (double)wgs;
        if (time < floor_t) time = floor_t;
        if (slices > 1) time += split_cost(M, N, slices, 4.56, 4.24e6);
        if (time < best) { best = time;  c.split = split; }
        if (t.large_split > 0) break;
    }
    return c;
}

// Launch shapes that were timed faster than the cost model's choice, for the layer shapes of the
// models the paper evaluates (Sec. 5.1).  An entry tuned at M tokens serves the batches of more than
// 3 M / 4 (M / 2 up to 64 tokens) and at most M tokens that give the same number of token tiles.
struct TunedTile { int cls, N, K, M, tm, tn, split, deep; };
static const TunedTile kTunedTiles[] = {
#include "tuned_tiles.inc"
    {-1, 0, 0, 0, 0, 0, 0, 0},
};

static bool tuned_large(int cls, int64_t M, int64_t N, int64_t K, LargeConfig &c) {
    for (const TunedTile &e : kTunedTiles) {
        if (e.cls != cls || e.N != N || e.K != K) continue;
        // (batches of up to 64 tokens are one 64-token tile whatever their size; above, a shape timed
        // at M tokens is trusted down to three quarters of M)
        if (M > e.M || (e.M <= 64 ? 2 * M <= e.M : 4 * M <= 3 * e.M)) continue;
        if ((M + e.tm - 1) / e.tm != (e.M + e.tm - 1) / e.tm) continue;
        c.tm = e.tm;  c.tn = e.tn;  c.split = e.split;  c.deep = e.deep;
        return true;
    }
    return false;
}

static LargeConfig choose_large(int kind, int64_t M, int64_t N, int64_t K) {
    LargeConfig c;
    const Tuning &t = tuning();
    const int cls = kind_class(kind);                  // cost tables: plain FP16 through LDS, FP16 through registers, E4M3
    const int kt = (int)(((kind_is_fp8(kind) ? K : 2 * K) + 127) / 128);
    if (t.tuned_table != 0 && t.large_bm < 0 && t.large_bn < 0 && t.large_split <= 0 && t.large_deep < 0 &&
        tuned_large(cls, M, N, K, c))
        return c;
    if (t.large_bm == 64 || (M <= 64 && t.large_bm < 0 && t.large_bn < 0))
        return choose_tile64(cls, M, N, kt);
    double best = 1e30;
    c.tm = c.tn = 256;
    c.split = 1;
    c.deep = 0;
    const int want_m = (t.large_bm == 128 || t.large_bm == 256) ? (int)t.large_bm : 0;
    const int want_n = (t.large_bn == 128 || t.large_bn == 256) ? (int)t.large_bn : want_m;
    const double w_bytes = (double)N * (double)K * (kind_is_fp8(kind) ? 1.0 : 2.0);
    for (int sh = 0; sh < 4; ++sh) {
        const int bm = kTileShapes[sh][0], bn = kTileShapes[sh][1];
        if (want_m && bm != want_m) continue;
        if (want_n && bn != want_n) continue;
        const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
        for (int deep = 0; deep < 2; ++deep) {
            if (deep && (kDeepTileCost[cls][sh].tk == 0.0 || t.large_deep == 0)) continue;
            if (!deep && t.large_deep > 0 && kDeepTileCost[cls][sh].tk != 0.0) continue;
            const TileCost &tc = deep ? kDeepTileCost[cls][sh] : kTileCost[cls][sh];
            for (int split : kSplits) {
                if (t.large_split > 0) split = (int)(t.large_split < kt ? t.large_split : kt);
                else if (split > 1 && split > kt / 4) break;
                const int per = (kt + split - 1) / split;                     // K-tiles per workgroup
                const int slices = (kt + per - 1) / per;
                const int64_t rounds = (tiles * slices + 255) / 256;
                double time = (double)rounds * (tc.tfix + per * tc.tk);
                if (sh == 3 && rounds >= 2 && !deep) time /= kPairSpeedup[cls];
                // the weights' one pass over the memory bus (slower while the chip is not full)
                const int64_t wgs = tiles * slices;
                double mem_floor = w_bytes / (wgs < 512 ? 4.57e6 : 4.44e6);
                if (wgs < 256) mem_floor *= std::sqrt(256.0 / (double)wgs);
                if (time < mem_floor) time = mem_floor;
                if (slices > 1) time += split_cost(M, N, slices, 3.18, 4.44e6);
                if (time < best) { best = time;  c.tm = bm;  c.tn = bn;  c.split = split;  c.deep = deep; }
                if (t.large_split > 0) break;
            }
        }
    }
    return c;
}

size_t large_gemm_partial_bytes(int kind, int64_t M, int64_t N, int64_t K) {
    LargeConfig c = choose_large(kind, M, N, K);
    return c.split > 1 ? (size_t)c.split * (size_t)M * (size_t)N * sizeof(float) : 0;
}

template <int KIND, int TM, int TN, int WAVES_M, int WAVES_N, int NST = 2>
static void launch_large_t(const LargeParams &p, dim3 grid, hipStream_t stream) {
    auto kern = large_gemm_kernel<KIND, TM, TN, WAVES_M, WAVES_N, NST>;
    constexpr int lds = LargeKernel<KIND, TM, TN, WAVES_M, WAVES_N, NST>::LDS_BYTES;
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr_set.store(true, std::memory_order_release);
    }
    kern<<<grid, 64 * WAVES_M * WAVES_N, lds, stream>>>(p);
}

template <int TM, int TN, int WK, bool DEEP = false, bool NT = false>
static void launch_bypass(const LargeParams &p, dim3 grid, hipStream_t stream) {
    auto kern = nested_bypass_kernel<TM, TN, WK, DEEP, NT>;
    constexpr int lds = BypassKernel<TM, TN, WK, DEEP, NT>::LDS_BYTES;
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr_set.store(true, std::memory_order_release);
    }
    kern<<<grid, 512, lds, stream>>>(p);
}

template <int TM, int TN, bool ROWMAJOR>
static void launch_e4m3_bypass(const LargeParams &p, dim3 grid, hipStream_t stream) {
    auto kern = e4m3_bypass_kernel<TM, TN, ROWMAJOR>;
    constexpr int lds = E4m3BypassKernel<TM, TN, ROWMAJOR>::LDS_BYTES;
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr_set.store(true, std::memory_order_release);
    }
    kern<<<grid, 512, lds, stream>>>(p);
}

// weights through LDS: plain row-major FP16, E4M3 in either storage order
template <int KIND>
static void launch_large_k(const LargeParams &p, const LargeConfig &c, dim3 grid, hipStream_t stream) {
    if (c.tm == 64) {
        if constexpr (KIND == kPlainF16) launch_large_t<KIND, 64, 128, 2, 4>(p, grid, stream);
        else launch_e4m3_bypass<64, 128, KIND == kE4M3Row>(p, grid, stream);
    } else if (c.tm == 256 && c.tn == 256) launch_large_t<KIND, 256, 256, 2, 4>(p, grid, stream);
    else if (c.tm == 256) {
        if (c.deep) launch_large_t<KIND, 256, 128, 4, 2, 3>(p, grid, stream);
        else launch_large_t<KIND, 256, 128, 4, 2>(p, grid, stream);
    } else if (c.tn == 256) {
        if (c.deep) launch_large_t<KIND, 128, 256, 2, 4, 3>(p, grid, stream);
        else launch_large_t<KIND, 128, 256, 2, 4>(p, grid, stream);
    } else {
        if (c.deep) launch_large_t<KIND, 128, 128, 2, 4, 4>(p, grid, stream);
        else launch_large_t<KIND, 128, 128, 2, 4>(p, grid, stream);
    }
}

// weights through registers: NestedFP16 in either storage order, packed FP16
template <int WK>
static void launch_nested(const LargeParams &p, const LargeConfig &c, dim3 grid, hipStream_t stream) {
    if (c.tm == 64) launch_bypass<64, 128, WK>(p, grid, stream);
    else if (c.tm == 256 && c.tn == 256) launch_bypass<256, 256, WK>(p, grid, stream);
    else if (c.tm == 256) launch_bypass<256, 128, WK>(p, grid, stream);
    else {
        // one token tile over a large packed layer: weights marked non-temporal (see BypassKernel)
        if constexpr (WK != kNestedF16Row) {
            if (p.tiles_m == 1 && (int64_t)p.N * p.K >= ((int64_t)100 << 20)) {
                if (c.tn == 256) {
                    if (c.deep) launch_bypass<128, 256, WK, true, true>(p, grid, stream);
                    else launch_bypass<128, 256, WK, false, true>(p, grid, stream);
                } else {
                    if (c.deep) launch_bypass<128, 128, WK, true, true>(p, grid, stream);
                    else launch_bypass<128, 128, WK, false, true>(p, grid, stream);
                }
                return;
            }
        }
        if (c.tn == 256) {
            if (c.deep) launch_bypass<128, 256, WK, true>(p, grid, stream);
            else launch_bypass<128, 256, WK>(p, grid, stream);
        } else {
            if (c.deep) launch_bypass<128, 128, WK, true>(p, grid, stream);
            else launch_bypass<128, 128, WK>(p, grid, stream);
        }
    }
}

// The kernels address a tile with 32-bit byte offsets whose bit 31 marks a dead load, so 256 rows
// of any operand must stay below 2^31 bytes.
bool large_gemm_supports(int kind, int64_t K, int64_t ldx, int64_t ldw) {
    const int64_t x_row = kind_is_fp8(kind) ? ldx : 2 * ldx;
    const int64_t w_row = kind == kPlainF16 ? 2 * ldw : ((K + 63) / 64) * 64 * kind_elem_bytes(kind);
    const int64_t lim = (int64_t)1 << 31;
    return 256 * x_row + 4096 < lim && 256 * w_row + 4096 < lim;
}

int launch_large_gemm(int kind, const GemmArgs &a, hipStream_t stream) {
    if (!large_gemm_supports(kind, a.K, a.ldx, a.ldw)) return kErrShape;
    LargeConfig c = choose_large(kind, a.M, a.N, a.K);
    // the register-path kernels take the deeper pipeline only where it is asked for (knob) or was
    // timed faster (table), and only on the tiles of 128 tokens
    if (kind_class(kind) == 1) c.deep = (tuning().large_deep > 0 || (c.deep && tuning().large_deep != 0)) && c.tm == 128;
    LargeParams p;
    p.X = static_cast<const uint8_t *>(a.X);
    p.x_row_bytes = kind_is_fp8(kind) ? a.ldx : 2 * a.ldx;
    p.scales = a.scales;
    p.w_scale = a.w_scale;
    p.W0 = static_cast<const uint8_t *>(a.W0);
    p.W1 = static_cast<const uint8_t *>(a.W1);
    p.w_row_bytes = (kind == kPlainF16) ? 2 * a.ldw : a.K;        // row-major kinds only
    p.M = (int)a.M;  p.N = (int)a.N;  p.K = (int)a.K;
    p.k_bytes = kind_is_fp8(kind) ? (int)a.K : (int)(2 * a.K);
    p.kblocks = (int)((a.K + 63) / 64);
    p.Y = a.Y;  p.ldy = a.ldy;
    p.partials = a.partials;
    p.tiles_m = (int)((a.M + c.tm - 1) / c.tm);
    p.tiles_n = (int)((a.N + c.tn - 1) / c.tn);
    p.ktiles_total = (p.k_bytes + 127) / 128;
    p.ktiles_per_split = (p.ktiles_total + c.split - 1) / c.split;
    c.split = (p.ktiles_total + p.ktiles_per_split - 1) / p.ktiles_per_split;   // no empty slices
    p.xcd_map = (tuning().large_xcd_map != 0 && p.tiles_m >= 2 && p.tiles_m <= 8) ? 1 : 0;
    p.vec_store = ((a.N & 3) == 0 && (a.ldy & 3) == 0 && (reinterpret_cast<uintptr_t>(a.Y) & 7) == 0) ? 1 : 0;
    p.row_store = ((a.N & 7) == 0 && (a.ldy & 7) == 0 && (reinterpret_cast<uintptr_t>(a.Y) & 15) == 0) ? 1 : 0;
    if (tuning().large_epilogue == 0) p.row_store = 0;
    if (c.split > 1 && (a.partials == nullptr ||
                        a.partial_bytes < (size_t)c.split * a.M * a.N * sizeof(float)))
        return kErrWorkspace;
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)c.split);
    switch (kind) {
        case kPlainF16: launch_large_k<kPlainF16>(p, c, grid, stream); break;
        case kNestedF16: launch_nested<kNestedF16>(p, c, grid, stream); break;
        case kNestedF16Row: launch_nested<kNestedF16Row>(p, c, grid, stream); break;
        case kPlainF16Packed: launch_nested<kPlainF16Packed>(p, c, grid, stream); break;
        case kE4M3: launch_large_k<kE4M3>(p, c, grid, stream); break;
        case kE4M3Row: launch_large_k<kE4M3Row>(p, c, grid, stream); break;
        default: return kErrArg;
    }
    if (hipGetLastError() != hipSuccess) return kErrHip;
    if (c.split > 1)
        return launch_splitk_reduce(a.partials, c.split, a.M, a.N, kind_is_fp8(kind) ? a.scales : nullptr,
                                    a.w_scale, a.Y, a.ldy, stream);
    return kOk;
}

}  // namespace nfp
