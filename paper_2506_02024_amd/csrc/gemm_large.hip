// LDS-tiled MFMA GEMM for prefill-sized batches: Y = X * W^T, compute-bound.
//
// Sec. 4.2 puts the FP16 reconstruction between the shared-memory-to-register copy and
// the tensor-core instruction of every warp and hides it with a third pipeline stage.
// Here the planes are merged ONCE per workgroup on their way from HBM to LDS
// (global -> VGPR -> Alg. 1 -> ds_write of finished FP16), so the MFMA loop that follows
// is the plain FP16 loop and the merge costs 2 VALU ops per weight per workgroup instead
// of per wave.
//
// Tile: TM tokens x TN weight rows x 128 bytes of K per row (64 halves or 128 E4M3 bytes),
// two LDS stages, 8 waves as 2 (tokens) x 4 (weight rows).  Weight rows are the MFMA "A"
// operand and tokens the "B" operand, so a lane holds 4 consecutive output columns of one
// token.  Tokens and plain / E4M3 weights reach LDS by direct-to-LDS buffer loads; FP16 rows
// are 128 bytes with the 16-byte chunk index XOR-swizzled with the row so that the MFMA
// fragment reads are free of bank conflicts, packed E4M3 blocks are copied as they are.
#include "nfp_device.h"
#include "nfp_host.h"

namespace nfp {

constexpr int kLargeThreads = 512;

struct LargeParams {
    const uint8_t *X;       // fp16 X (bytes) or E4M3 Xq
    int64_t x_row_bytes;    // < 2^24 (checked on the host): tile-local offsets fit in 31 bits
    const float *scales;
    float w_scale;
    const uint8_t *W0;
    const uint8_t *W1;
    int64_t w_row_bytes;    // bytes per row of W0 (plain: 2*ldw, planes / E4M3: K)
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
};

// LDS tiles are rows of 128 bytes; the 16-byte chunk index is XOR-ed with (row >> 1) & 7.
// gfx950 serves ds_read_b128 at 256 B/clk only if 16 consecutive lanes hit 64 distinct
// 4-byte banks: rows r, r+1 then share a swizzle and fill one 256-byte bank line, and the
// pairs of 16 consecutive rows take the 8 different swizzles.  The 128-bit writes of the
// global->LDS copy (8 lanes per row) are conflict-free under the same map.
__device__ __forceinline__ int swz(int row, int chunk) { return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4); }

__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_rsrc(const uint8_t *base, int64_t row0, int rows,
                                                            int64_t row_bytes, int k_bytes) {
    // raw buffer over the rows of one tile; anything past the last valid byte reads as zero
    uint32_t bytes = rows > 0 ? (uint32_t)((rows - 1) * row_bytes + k_bytes) : 0u;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(base + row0 * row_bytes), 0, bytes, 0x00020000);
}

// raw buffer over the 16-row tiles of a packed plane that hold rows row0 .. row0+rows-1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t plane_rsrc(const uint8_t *base, int64_t row0, int rows, int kblocks) {
    const int64_t tile_bytes = (int64_t)kblocks * 1024;
    uint32_t bytes = rows > 0 ? (uint32_t)(((rows + 15) >> 4) * tile_bytes) : 0u;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(base + (row0 >> 4) * tile_bytes), 0, bytes, 0x00020000);
}

template <int KIND, int TM, int TN, int WAVES_M, int WAVES_N>
struct LargeKernel {
    static constexpr int THREADS = 64 * WAVES_M * WAVES_N;
    static constexpr int WTM = TM / WAVES_M, WTN = TN / WAVES_N;
    static constexpr int FM = WTM / 32, FN = WTN / 32;
    static constexpr int STAGE = (TM + TN) * 128;      // bytes per LDS stage
    static constexpr int LDS_BYTES = 2 * STAGE;
    static constexpr int SUBSTEPS = 2;                 // E4M3 loop: two substeps of 64 bytes
    // slot plan of the FP16 loop (see there)
    static constexpr int FM16 = WTM / 16, FN16 = WTN / 16;
    static constexpr int MF = FM16 * FN16;                           // MFMAs per substep
    static constexpr int NPRE = FN16 + 2;
    static constexpr int NREST = FM16 - 2;
    static constexpr int RSTR = (3 * FN16) / 4 > 0 ? (3 * FN16) / 4 : 1;      // slots between the early token reads
    static constexpr int QB = (NREST - 1) * RSTR + 3;                // slot that starts with the barrier
    static constexpr int TSTR = (MF - QB) / NPRE > 0 ? (MF - QB) / NPRE : 1;  // slots between the look-ahead reads
    static constexpr int TAIL0 = MF - NPRE * TSTR;

    // MFMA operand fragments of one K substep (16 halves / 64 E4M3 bytes per row)
    struct Frags {
        intx4 a[FN][KIND == kE4M3 ? 2 : 1];
        intx4 b[FM][KIND == kE4M3 ? 2 : 1];
    };

    // The r-th LDS read of a substep's fragments, in the order the MFMAs need them:
    // a[0], b[0..FM-1], a[1..FN-1] (NC reads each).
    template <int R>
    static __device__ __forceinline__ void read_one(Frags &f, const uint8_t *stage, int wm, int wn, int lane, int s) {
        constexpr int NC = KIND == kE4M3 ? 2 : 1;
        constexpr int F = R / NC, Q = R % NC;              // fragment index in issue order, chunk within it
        const uint8_t *sW = stage, *sX = stage + TN * 128;
        const int r32 = lane & 31, h = lane >> 5;
        const int c = NC * (2 * s + h) + Q;
        if (F == 0) f.a[0][Q] = *reinterpret_cast<const intx4 *>(sW + w_addr(wn * WTN + r32, s, h, Q));
        else if (F <= FM) f.b[F - 1][Q] = *reinterpret_cast<const intx4 *>(sX + swz(wm * WTM + 32 * (F - 1) + r32, c));
        else f.a[F - FM][Q] = *reinterpret_cast<const intx4 *>(sW + w_addr(wn * WTN + 32 * (F - FM) + r32, s, h, Q));
    }

    // LDS address of a weight fragment chunk.  FP16 kinds: rows of 128 bytes, XOR-swizzled.
    // E4M3: the stage holds the packed 1 KB blocks as they are in memory, [row tile][2 blocks];
    // a substep is one block, and 16 lanes with consecutive rows read 256 consecutive bytes.
    static __device__ __forceinline__ int w_addr(int row, int s, int h, int q) {
        if (KIND == kE4M3) return (((row >> 4) * 2 + s) << 10) + (((row & 15) + 16 * (2 * h + q)) << 4);
        return swz(row, 2 * s + h);
    }

    template <int Q>
    static __device__ __forceinline__ void mfma_one(const Frags &f, floatx16 (&acc)[FN][FM]) {
        constexpr int i = Q / FM, j = Q % FM;
        if (KIND == kE4M3) {
            intx8 a = {f.a[i][0].x, f.a[i][0].y, f.a[i][0].z, f.a[i][0].w,
                       f.a[i][NC1].x, f.a[i][NC1].y, f.a[i][NC1].z, f.a[i][NC1].w};
            intx8 b = {f.b[j][0].x, f.b[j][0].y, f.b[j][0].z, f.b[j][0].w,
                       f.b[j][NC1].x, f.b[j][NC1].y, f.b[j][NC1].z, f.b[j][NC1].w};
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[i][j], 0, 0, 0, 0, 0, 0);
        } else {
            union { intx4 v; half8 h; } a, b;
            a.v = f.a[i][0];
            b.v = f.b[j][0];
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a.h, b.h, acc[i][j], 0, 0, 0);
        }
    }

    static constexpr int NC1 = KIND == kE4M3 ? 1 : 0;

    // ---- direct-to-LDS loads (buffer_load ... lds) -------------------------------------------
    // One wave instruction fills 1 KB of LDS = 8 tile rows in lane order (lane l -> row l/8,
    // physical chunk l%8), so the XOR swizzle is applied on the global side: lane l fetches
    // the logical chunk (l%8) ^ ((row>>1)&7) of its row.  No VGPR staging, no ds_write.
    static constexpr int WAVES = WAVES_M * WAVES_N;
    // With two waves per SIMD the older one wins every arbitration and reaches the barrier long
    // before the younger one.  The loads are therefore issued by the older four waves only:
    // a load instruction blocks the issue of whatever is behind it while the address queue is
    // full, and those waves have the time to spare.
    static constexpr int DW = WAVES == 8 ? 4 : WAVES;  // waves that issue direct-to-LDS loads
    static constexpr bool kTwoRoles = WAVES != DW;
    // The planes are loaded, merged and written to LDS one packed 1 KB block of each plane at a
    // time (a "piece": 16 rows x 64 columns; lane l holds chunk l, i.e. row l % 16, columns
    // 16 * (l / 16) .. +15).  16 consecutive lanes then write one chunk column of 16 consecutive
    // rows, the bank pattern of the fragment reads.  The older wave of a SIMD wins every
    // arbitration and has time to spare, so the loading waves take three of every four pieces
    // (measured: 3:1 beats 2:2 and 4:0); a weight tile of 128 rows is merged by them alone.
    static constexpr int NPO = TN == 256 ? 3 : 2;         // pieces of an older (loading) wave
    static constexpr int NPY = TN / 64 - NPO;             // pieces of a younger wave
    static constexpr int NPW = NPO > NPY ? NPO : NPY;
    template <bool OLDER> static constexpr int pieces() { return OLDER ? NPO : NPY; }
    struct PlaneRegs { u32x4 u[NPW], l[NPW]; };
    struct PlaneOffsets { uint32_t lane_off; uint32_t lds_off; uint32_t lim; };
    static constexpr int XG = TM / 8 / DW;             // 8-row groups per loading wave, token tile
    static constexpr int WG8 = TN / 8 / DW;            // 8-row groups per loading wave, weight tile

    struct DmaOffsets {
        uint32_t x[XG], w[WG8];
        uint32_t kpos;                                 // this lane's K byte position in a K-tile
        int wbit;                                      // E4M3: which of a K-tile's two block columns this wave loads
    };

    static __device__ __forceinline__ void make_dma_offsets(DmaOffsets &o, const LargeParams &p, int wave, int lane) {
        const int pc = lane & 7;
        const int c = pc ^ ((((wave & 1) << 2) + (lane >> 4)) & 7);     // (row >> 1) & 7 for row = gid*8 + lane/8
        o.kpos = 16u * c;
#pragma unroll
        for (int i = 0; i < XG; ++i) o.x[i] = (uint32_t)((i * DW + wave) * 8 + (lane >> 3)) * (uint32_t)p.x_row_bytes + 16u * c;
#pragma unroll
        for (int i = 0; i < WG8; ++i) {
            if (KIND == kE4M3) {
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
            if (KIND == kE4M3) {
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
    // Every MFMA of a substep is followed by the few other instructions assigned to its slot
    // and a scheduling fence, so the order below is the order in the binary:
    //   * LDS reads of the next substep's fragments, one (FP16) or two (E4M3) per MFMA, in the
    //     order the MFMAs will need them;
    //   * the direct-to-LDS loads, spread over three substeps so that the eight waves never
    //     fill the texture-address queue (a wave that cannot issue its load cannot issue the
    //     MFMA behind it either);
    //   * for the planes: merge + LDS write + reload, one 16-weight piece at a time.
    static constexpr int READS = (FN + FM) * (KIND == kE4M3 ? 2 : 1);
    static constexpr int MFMAS = FN * FM;
    static constexpr int RPS = (READS + MFMAS - 1) / MFMAS;            // reads per slot
    static constexpr int DMAS = XG + (KIND == kNestedF16 ? 0 : WG8);   // loads per wave per K-tile
    static constexpr int DPS = (DMAS + MFMAS - 1) / MFMAS;             // loads per slot of the last substep

    struct Ctx {
        floatx16 (&acc)[FN][FM];
        Frags (&fr)[2];
        const DmaOffsets &dof;
        __amdgpu_buffer_rsrc_t rx, rw0;
        uint8_t *lds;
        lds_byte *lds3;
        uint32_t x_lim, w_lim;
        int wave, lane, wm, wn;
        int kt, cur;
    };

    static __device__ __forceinline__ void make_plane_offsets(PlaneOffsets &o, const LargeParams &p, int wave, int lane) {
        const int r = lane & 15, c4 = lane >> 4;
        const int tile0 = wave < DW ? wave * NPO : DW * NPO + (wave - DW) * NPY;      // first row tile of the wave
        o.lane_off = (uint32_t)(tile0 * p.kblocks) * 1024u + (uint32_t)lane * 16u;
        // FP16 stage: row 16 * row tile + r, 16-byte chunks 2 * c4 and 2 * c4 + 1 (XOR-swizzled)
        o.lds_off = (uint32_t)(tile0 * 16 + r) * 128u + (uint32_t)(((2 * c4) ^ ((r >> 1) & 7)) << 4);
        o.lim = (uint32_t)p.kblocks;                    // block columns of the plane
    }

    template <int P>
    static __device__ __forceinline__ void load_piece(PlaneRegs &pf, const PlaneOffsets &o, __amdgpu_buffer_rsrc_t rw0,
                                                      __amdgpu_buffer_rsrc_t rw1, int kblocks, int kt) {
        const uint32_t kill = ((uint32_t)kt < o.lim) ? 0u : 0x80000000u;
        const uint32_t soff = (uint32_t)(P * kblocks + kt) * 1024u;
        pf.u[P] = __builtin_amdgcn_raw_buffer_load_b128(rw0, (o.lane_off + soff) | kill, 0, 0);
        pf.l[P] = __builtin_amdgcn_raw_buffer_load_b128(rw1, (o.lane_off + soff) | kill, 0, 0);
    }

    // Sec. 4.2, Alg. 1 on the J-th four weights of piece P (8 VALU instructions); every second
    // quarter completes a 16-byte chunk of the FP16 row, which goes into the tile of `stage`
    template <int P, int J>
    static __device__ __forceinline__ void merge_quarter(const PlaneRegs &pf, const PlaneOffsets &o, u32x4 &merged, uint8_t *stage) {
        uint32_t w01, w23;
        merge4(pf.u[P][J], pf.l[P][J], w01, w23);
        merged[2 * (J & 1)] = w01;
        merged[2 * (J & 1) + 1] = w23;
        if constexpr ((J & 1) == 1)
            *reinterpret_cast<u32x4 *>(stage + ((o.lds_off ^ (uint32_t)((J >> 1) << 4)) + P * 2048)) = merged;
    }

    // When the quarters of a wave's pieces run.  The registers of a piece hold K-tile kt+1 while
    // K-tile kt is multiplied; it goes into the other stage (free since the barrier of kt-1) and
    // the registers are reloaded with kt+2 right behind the piece's last quarter, most of a
    // K-tile before they are needed again.  Older waves: pieces 0 and 1 in the first substep, 2
    // in the head of the second (before the barrier), one quarter every few slots; younger
    // waves: their piece spread over the first substep.
    template <bool OLDER> static constexpr int piece_sub(int p) { return OLDER && p >= 2 ? 1 : 0; }
    template <bool OLDER> static constexpr int piece_stride(int p) { return OLDER ? (MF >= 32 ? 4 : 1) : MF / 4; }
    template <bool OLDER> static constexpr int piece_slot(int p) { return OLDER ? ((p & 1) ? MF / 2 : 0) : MF / 8; }
    static_assert(NPO <= 3 && NPY <= 1 && NPY >= 0, "merge slots");
    static_assert(KIND != kNestedF16 || NPO < 3 || 3 * piece_stride<true>(2) < QB, "merge slots");
    // (piece * 4 + quarter) that runs at slot q of substep s, or -1
    template <bool OLDER> static constexpr int quarter_at(int s, int q) {
        for (int p = 0; p < pieces<OLDER>(); ++p)
            if (piece_sub<OLDER>(p) == s && q >= piece_slot<OLDER>(p) && (q - piece_slot<OLDER>(p)) % piece_stride<OLDER>(p) == 0 &&
                (q - piece_slot<OLDER>(p)) / piece_stride<OLDER>(p) < 4)
                return 4 * p + (q - piece_slot<OLDER>(p)) / piece_stride<OLDER>(p);
        return -1;
    }

    template <bool OLDER, int G, class C>
    static __device__ __forceinline__ void plane_quarter(C &c) {
        constexpr int P = G / 4, J = G % 4;
        merge_quarter<P, J>(c.pf, c.off, c.merged, c.lds + (c.cur ^ 1) * STAGE);
        if constexpr (J == 3) load_piece<P>(c.pf, c.off, c.rw0, c.rw1, c.kblocks, c.kt + 2);
    }

    // stage 0 is merged here; stage 1 is written in the first K-tile of the loop, as in every later one
    template <bool OLDER, int P>
    static __device__ __forceinline__ void plane_prologue(PlaneRegs &pf, const PlaneOffsets &o, __amdgpu_buffer_rsrc_t rw0,
                                                          __amdgpu_buffer_rsrc_t rw1, int kblocks, int kt_begin, uint8_t *lds) {
        if constexpr (P < pieces<OLDER>()) {
            u32x4 merged;
            load_piece<P>(pf, o, rw0, rw1, kblocks, kt_begin);
            merge_quarter<P, 0>(pf, o, merged, lds);  merge_quarter<P, 1>(pf, o, merged, lds);
            merge_quarter<P, 2>(pf, o, merged, lds);  merge_quarter<P, 3>(pf, o, merged, lds);
            load_piece<P>(pf, o, rw0, rw1, kblocks, kt_begin + 1);
            plane_prologue<OLDER, P + 1>(pf, o, rw0, rw1, kblocks, kt_begin, lds);
        }
    }

    // OLDER: one of the DW waves that issue the direct-to-LDS loads.  The K loop exists once per
    // role so that it has no branches inside.
    template <bool OLDER, int S, int Q>
    static __device__ __forceinline__ void slot(Ctx &c) {
        constexpr bool last = (S == SUBSTEPS - 1);
        mfma_one<Q>(c.fr[S & 1], c.acc);
        {   // fragments of the following substep (of the next K-tile after the barrier)
            const uint8_t *src = c.lds + (last ? c.cur ^ 1 : c.cur) * STAGE;
            constexpr int s_next = last ? 0 : S + 1;
            Frags &dst = c.fr[(S + 1) & 1];
            read_range<Q * RPS, (Q + 1) * RPS < READS ? (Q + 1) * RPS : READS>(dst, src, c.wm, c.wn, c.lane, s_next);
        }
        if constexpr (last) {
            if constexpr (OLDER) {
#pragma unroll
                for (int d = Q * DPS; d < (Q + 1) * DPS && d < DMAS; ++d)
                    dma_one(d, c.dof, c.x_lim, c.w_lim, c.rx, c.rw0, c.lds3 + c.cur * STAGE, c.wave, c.kt + 2);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (Q + 1 < MFMAS) slot<OLDER, S, Q + 1>(c);
    }

    template <bool OLDER, int S>
    static __device__ __forceinline__ void substeps(Ctx &c) {
        if constexpr (S == SUBSTEPS - 1) {
            // Everything this wave still needs from the current stage is in registers.  Once all
            // waves are here and their loads of the next K-tile have landed, the current stage
            // is free and the next one complete.
            if constexpr (OLDER) asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            else asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
        }
        slot<OLDER, S, 0>(c);
        if constexpr (S + 1 < SUBSTEPS) substeps<OLDER, S + 1>(c);
    }

    template <bool OLDER>
    static __device__ __forceinline__ void k_loop(Ctx &c, int kt_begin, int kt_end) {
        for (int kt = kt_begin; kt < kt_end; ++kt) {
            c.kt = kt;
            c.cur = (kt - kt_begin) & 1;
            __builtin_amdgcn_sched_barrier(0);
            substeps<OLDER, 0>(c);
        }
    }

    // ---- FP16 kinds: the same loop on v_mfma_f32_16x16x32_f16 --------------------------------
    // Under the chip's power limit (which, not the issue rate, bounds a full-chip FP16 GEMM on
    // random operands) the 16x16x32 instruction sustains about 15 % more flops than 32x32x16: it
    // moves half as many accumulator registers per flop.  A K-tile is two substeps of 32 halves;
    // a wave's tile is FN16 x FM16 blocks of 16 weight rows x 16 tokens, the MFMAs of a substep
    // run token block by token block (the FN16 weight fragments stay, the token fragments
    // stream).  LDS reads: the first NPRE fragments of a substep (all weight fragments, two token
    // fragments) are fetched in the tail of the substep before it, the other token fragments
    // early in the substep itself, about two token blocks ahead of their use.  The barrier of
    // the K-tile sits in the second substep behind the last read of the current stage (slot QB);
    // loads of K-tile kt+2, the older waves' plane merge and the reads of K-tile kt+1 follow it.
    static constexpr int DPS16 = (DMAS + (MF - QB) - 1) / (MF - QB);
    static_assert(KIND == kE4M3 || (FM16 >= 3 && TAIL0 >= QB && QB < MF), "slot plan of the 16x16x32 loop");
    struct Frags16 { intx4 a[FN16]; intx4 b[FM16]; };

    struct Ctx16 {
        floatx4 (&acc)[FN16][FM16];
        Frags16 (&fr)[2];
        PlaneRegs &pf;
        u32x4 merged;                                   // FP16 chunk being assembled by the plane merge
        const PlaneOffsets &off;
        const DmaOffsets &dof;
        __amdgpu_buffer_rsrc_t rx, rw0, rw1;
        uint8_t *lds;
        lds_byte *lds3;
        uint32_t x_lim, w_lim;
        int wave, lane, wm, wn;
        int kblocks;
        int kt, cur;
    };

    // fragment R of substep s in the order of first use: weight blocks 0..FN16-1, token blocks 0..FM16-1;
    // lane l takes row l % 16, halves 32*s + 8*(l/16) .. +7 (16x16x32 operand layout)
    template <int R>
    static __device__ __forceinline__ void read16(Frags16 &f, const uint8_t *stage, int wm, int wn, int lane, int s) {
        const int r16 = lane & 15, c = 4 * s + (lane >> 4);
        if constexpr (R < FN16) f.a[R] = *reinterpret_cast<const intx4 *>(stage + swz(wn * WTN + 16 * R + r16, c));
        else f.b[R - FN16] = *reinterpret_cast<const intx4 *>(stage + TN * 128 + swz(wm * WTM + 16 * (R - FN16) + r16, c));
    }

    template <int R, int END>
    static __device__ __forceinline__ void read16_range(Frags16 &f, const uint8_t *stage, int wm, int wn, int lane, int s) {
        if constexpr (R < END) {
            read16<R>(f, stage, wm, wn, lane, s);
            read16_range<R + 1, END>(f, stage, wm, wn, lane, s);
        }
    }

    template <bool OLDER, int S, int Q>
    static __device__ __forceinline__ void slot16(Ctx16 &c) {
        constexpr bool last = (S == 1);
        if constexpr (last && Q == QB) {
            // every read of the current stage has been issued; once all waves are here and their
            // loads of the next K-tile have landed, the stage is free and the next one complete
            // (the loading waves' plane loads of this K-tile are younger than those and may still fly)
            if constexpr (OLDER) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(KIND == kNestedF16 ? 2 * NPO : 0) : "memory");
            else asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
        }
        {
            constexpr int j = Q / FN16, i = Q % FN16;
            union { intx4 v; half8 h; } a, b;
            a.v = c.fr[S].a[i];
            b.v = c.fr[S].b[j];
            c.acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a.h, b.h, c.acc[i][j], 0, 0, 0);
        }
        if constexpr (Q % RSTR == 0 && Q / RSTR < NREST)
            read16<FN16 + 2 + Q / RSTR>(c.fr[S], c.lds + c.cur * STAGE, c.wm, c.wn, c.lane, S);
        if constexpr (Q >= TAIL0 && (Q - TAIL0) % TSTR == 0 && (Q - TAIL0) / TSTR < NPRE)
            read16<(Q - TAIL0) / TSTR>(c.fr[S ^ 1], c.lds + (last ? c.cur ^ 1 : c.cur) * STAGE, c.wm, c.wn, c.lane, last ? 0 : 1);
        if constexpr (last && Q >= QB) {
            if constexpr (OLDER) {
#pragma unroll
                for (int d = (Q - QB) * DPS16; d < (Q - QB + 1) * DPS16 && d < DMAS; ++d)
                    dma_one(d, c.dof, c.x_lim, c.w_lim, c.rx, c.rw0, c.lds3 + c.cur * STAGE, c.wave, c.kt + 2);
            }
        }
        if constexpr (KIND == kNestedF16 && quarter_at<OLDER>(S, Q) >= 0) plane_quarter<OLDER, quarter_at<OLDER>(S, Q)>(c);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (Q + 1 < MF) slot16<OLDER, S, Q + 1>(c);
    }

    template <bool OLDER>
    static __device__ __forceinline__ void k_loop16(Ctx16 &c, int kt_begin, int kt_end) {
        for (int kt = kt_begin; kt < kt_end; ++kt) {
            c.kt = kt;
            c.cur = (kt - kt_begin) & 1;
            __builtin_amdgcn_sched_barrier(0);
            slot16<OLDER, 0, 0>(c);
            slot16<OLDER, 1, 0>(c);
        }
    }

    template <int R, int END>
    static __device__ __forceinline__ void read_range(Frags &f, const uint8_t *stage, int wm, int wn, int lane, int s) {
        if constexpr (R < END) {
            read_one<R>(f, stage, wm, wn, lane, s);
            read_range<R + 1, END>(f, stage, wm, wn, lane, s);
        }
    }

    template <int R>
    static __device__ __forceinline__ void read_all(Frags &f, const uint8_t *stage, int wm, int wn, int lane) {
        if constexpr (R < READS) {
            read_one<R>(f, stage, wm, wn, lane, 0);
            read_all<R + 1>(f, stage, wm, wn, lane);
        }
    }

    static __device__ __forceinline__ void run(const LargeParams &p, uint8_t *lds, lds_byte *lds3) {
        const int lane = threadIdx.x & 63;
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const int wm = wave % WAVES_M, wn = wave / WAVES_M;
        const int tile = blockIdx.x;
        const int tm = tile % p.tiles_m, tn = tile / p.tiles_m;
        const int m0 = tm * TM, n0 = tn * TN;
        const int split = blockIdx.y;
        const int kt_begin = split * p.ktiles_per_split;
        const int kt_end = min(kt_begin + p.ktiles_per_split, p.ktiles_total);

        const __amdgpu_buffer_rsrc_t rx = tile_rsrc(p.X, m0, min(TM, p.M - m0), p.x_row_bytes, p.k_bytes);
        const __amdgpu_buffer_rsrc_t rw0 = KIND == kPlainF16
            ? tile_rsrc(p.W0, n0, min(TN, p.N - n0), p.w_row_bytes, p.k_bytes)
            : plane_rsrc(p.W0, n0, min(TN, p.N - n0), p.kblocks);
        const __amdgpu_buffer_rsrc_t rw1 = KIND == kNestedF16 ? plane_rsrc(p.W1, n0, min(TN, p.N - n0), p.kblocks) : rw0;
        DmaOffsets dof;
        make_dma_offsets(dof, p, wave, lane);
        PlaneOffsets off;
        if (KIND == kNestedF16) make_plane_offsets(off, p, wave, lane);
        PlaneRegs pf;
        const uint32_t x_lim = (uint32_t)p.k_bytes;
        const uint32_t w_lim = KIND == kE4M3 ? (uint32_t)p.kblocks : (uint32_t)p.k_bytes;

        // Two LDS stages.  Tokens (and plain / E4M3 weights) go straight from global memory
        // into LDS; the planes take the register path (they have to pass through the merge).
        // There is one barrier per K-tile, placed where every wave has fetched the last
        // fragments of the current stage: from there on the stage is free for K-tile kt+2,
        // and the first fragments of K-tile kt+1 are fetched underneath the last MFMAs.
        if (wave < DW) {
#pragma unroll
            for (int st = 0; st < 2; ++st)
#pragma unroll
                for (int i = 0; i < DMAS; ++i)
                    dma_one(i, dof, x_lim, w_lim, rx, rw0, lds3 + st * STAGE, wave, kt_begin + st);
        }
        if (KIND == kNestedF16) {
            if (wave < DW) plane_prologue<true, 0>(pf, off, rw0, rw1, p.kblocks, kt_begin, lds);
            else plane_prologue<false, 0>(pf, off, rw0, rw1, p.kblocks, kt_begin, lds);
            // everything but the plane loads issued last (the token loads came before them all)
            if (wave < DW) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(2 * NPO) : "memory");
            else asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(2 * NPY) : "memory");
        } else {
            // the loads of K-tile kt_begin (a wave that issued none passes straight through)
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(DMAS) : "memory");
        }
        __syncthreads();

        if constexpr (KIND == kE4M3) {
            floatx16 acc[FN][FM];
#pragma unroll
            for (int i = 0; i < FN; ++i)
#pragma unroll
                for (int j = 0; j < FM; ++j)
#pragma unroll
                    for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;
            Frags fr[2];
            Ctx c{acc, fr, dof, rx, rw0, lds, lds3, x_lim, w_lim, wave, lane, wm, wn, kt_begin, 0};
            read_all<0>(fr[0], lds, wm, wn, lane);
            if (!kTwoRoles || wave < DW) k_loop<true>(c, kt_begin, kt_end);
            else k_loop<false>(c, kt_begin, kt_end);
            if (p.row_store && gridDim.y == 1) {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // the look-ahead fragment reads
                __syncthreads();
                epilogue_lds(p, acc, m0, n0, wm, wn, lane, wave, lds);
            } else {
                epilogue(p, acc, m0, n0, wm, wn, lane, split);
            }
        } else {
            floatx4 acc[FN16][FM16];
#pragma unroll
            for (int i = 0; i < FN16; ++i)
#pragma unroll
                for (int j = 0; j < FM16; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
            Frags16 fr[2];
            Ctx16 c{acc, fr, pf, u32x4{0, 0, 0, 0}, off, dof, rx, rw0, rw1, lds, lds3, x_lim, w_lim,
                    wave, lane, wm, wn, p.kblocks, kt_begin, 0};
            read16_range<0, NPRE>(fr[0], lds, wm, wn, lane, 0);
            if (!kTwoRoles || wave < DW) k_loop16<true>(c, kt_begin, kt_end);
            else k_loop16<false>(c, kt_begin, kt_end);
            if (p.row_store && gridDim.y == 1) {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __syncthreads();
                epilogue_lds16(p, acc, m0, n0, wm, wn, lane, wave, lds);
            } else {
                epilogue16(p, acc, m0, n0, wm, wn, lane, split);
            }
        }
    }

    // Result tile through LDS: the MFMA layout leaves a lane with 4 consecutive outputs of one
    // token, so direct stores are 8-byte pieces scattered over 32 rows per instruction.  Written
    // to LDS as FP16 first (16-byte chunks XOR-swizzled with the row), the tile goes out as
    // whole rows, 16 bytes per lane, every store instruction covering complete 128-byte lines.
    // The caller guarantees that no wave still reads the operand stages.
    static constexpr int OCH = TN * 2 / 16;            // 16-byte chunks per output row
    static_assert(TM * TN * 2 <= LDS_BYTES, "output tile must fit into the operand stages");
    static __device__ __forceinline__ void epilogue_lds(const LargeParams &p, floatx16 (&acc)[FN][FM], int m0, int n0,
                                                        int wm, int wn, int lane, int wave, uint8_t *lds) {
        const int r32 = lane & 31, h = lane >> 5;
#pragma unroll
        for (int j = 0; j < FM; ++j) {
            const int row = wm * WTM + 32 * j + r32;
            float s = 1.0f;
            if (KIND == kE4M3) {
                const int m = m0 + row;
                s = (m < p.M ? p.scales[m] : 0.f) * p.w_scale;
            }
#pragma unroll
            for (int i = 0; i < FN; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int chunk = wn * (WTN / 8) + 4 * i + q;
                    u32x2 o;
                    o.x = float2_to_half2_bits(acc[i][j][4 * q] * s, acc[i][j][4 * q + 1] * s);
                    o.y = float2_to_half2_bits(acc[i][j][4 * q + 2] * s, acc[i][j][4 * q + 3] * s);
                    *reinterpret_cast<u32x2 *>(lds + row * (TN * 2) + ((chunk ^ (row & (OCH - 1))) << 4) + 8 * h) = o;
                }
        }
        store_tile_rows(p, m0, n0, lane, wave, lds);
    }

    // the FP16 tile in LDS goes out as whole rows, 16 bytes per lane
    static __device__ __forceinline__ void store_tile_rows(const LargeParams &p, int m0, int n0, int lane, int wave,
                                                           const uint8_t *lds) {
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

    // 16x16x32 accumulators: lane l holds token l % 16 and the four consecutive weight rows
    // 4 * (l / 16) .. +3 of every 16x16 block
    static __device__ __forceinline__ void epilogue_lds16(const LargeParams &p, floatx4 (&acc)[FN16][FM16], int m0, int n0,
                                                          int wm, int wn, int lane, int wave, uint8_t *lds) {
        const int r16 = lane & 15, q4 = lane >> 4;
#pragma unroll
        for (int j = 0; j < FM16; ++j) {
            const int row = wm * WTM + 16 * j + r16;
#pragma unroll
            for (int i = 0; i < FN16; ++i) {
                const int col = wn * WTN + 16 * i + 4 * q4;
                const int chunk = col >> 3;
                u32x2 o;
                o.x = float2_to_half2_bits(acc[i][j][0], acc[i][j][1]);
                o.y = float2_to_half2_bits(acc[i][j][2], acc[i][j][3]);
                *reinterpret_cast<u32x2 *>(lds + row * (TN * 2) + ((chunk ^ (row & (OCH - 1))) << 4) + 8 * (q4 & 1)) = o;
            }
        }
        store_tile_rows(p, m0, n0, lane, wave, lds);
    }

    static __device__ __forceinline__ void epilogue16(const LargeParams &p, floatx4 (&acc)[FN16][FM16], int m0, int n0,
                                                      int wm, int wn, int lane, int split) {
        const int r16 = lane & 15, q4 = lane >> 4;
#pragma unroll
        for (int j = 0; j < FM16; ++j) {
            const int m = m0 + wm * WTM + 16 * j + r16;
            if (m >= p.M) continue;
#pragma unroll
            for (int i = 0; i < FN16; ++i) {
                const int n = n0 + wn * WTN + 16 * i + 4 * q4;
                if (n >= p.N) continue;
                const floatx4 v = acc[i][j];
                if (gridDim.y > 1) {
                    float *dst = p.partials + ((int64_t)split * p.M + m) * p.N + n;
                    if ((p.N & 3) == 0) {
                        *reinterpret_cast<floatx4 *>(dst) = v;
                    } else {
                        for (int e = 0; e < 4 && n + e < p.N; ++e) dst[e] = v[e];
                    }
                } else {
                    uint16_t *dst = p.Y + (int64_t)m * p.ldy + n;
                    if (p.vec_store) {
                        u32x2 o;
                        o.x = float2_to_half2_bits(v[0], v[1]);
                        o.y = float2_to_half2_bits(v[2], v[3]);
                        *reinterpret_cast<u32x2 *>(dst) = o;
                    } else {
                        for (int e = 0; e < 4 && n + e < p.N; ++e) {
                            union { _Float16 f; uint16_t u; } cv;
                            cv.f = (_Float16)v[e];
                            dst[e] = cv.u;
                        }
                    }
                }
            }
        }
    }

    static __device__ __forceinline__ void epilogue(const LargeParams &p, floatx16 (&acc)[FN][FM], int m0, int n0,
                                                    int wm, int wn, int lane, int split) {
        const int r32 = lane & 31, h = lane >> 5;
#pragma unroll
        for (int j = 0; j < FM; ++j) {
            const int m = m0 + wm * WTM + 32 * j + r32;
            if (m >= p.M) continue;
            float s = 1.0f;
            if (KIND == kE4M3 && gridDim.y == 1) s = p.scales[m] * p.w_scale;
#pragma unroll
            for (int i = 0; i < FN; ++i) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = n0 + wn * WTN + 32 * i + 8 * q + 4 * h;
                    if (n >= p.N) continue;
                    float v[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                                  acc[i][j][4 * q + 3]};
                    if (gridDim.y > 1) {
                        float *dst = p.partials + ((int64_t)split * p.M + m) * p.N + n;
                        if ((p.N & 3) == 0) {
                            *reinterpret_cast<floatx4 *>(dst) = floatx4{v[0], v[1], v[2], v[3]};
                        } else {
                            for (int e = 0; e < 4 && n + e < p.N; ++e) dst[e] = v[e];
                        }
                    } else {
                        uint16_t *dst = p.Y + (int64_t)m * p.ldy + n;
                        if (p.vec_store) {
                            u32x2 o;
                            o.x = float2_to_half2_bits(v[0] * s, v[1] * s);
                            o.y = float2_to_half2_bits(v[2] * s, v[3] * s);
                            *reinterpret_cast<u32x2 *>(dst) = o;
                        } else {
                            for (int e = 0; e < 4 && n + e < p.N; ++e) {
                                union { _Float16 f; uint16_t u; } c;
                                c.f = (_Float16)(v[e] * s);
                                dst[e] = c.u;
                            }
                        }
                    }
                }
            }
        }
    }
};

template <int KIND, int TM, int TN, int WAVES_M, int WAVES_N>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N)
large_gemm_kernel(LargeParams p) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
    typedef LargeKernel<KIND, TM, TN, WAVES_M, WAVES_N> Kern;
    Kern::run(p, lds_raw, (typename Kern::lds_byte *)lds_raw);
}

struct LargeConfig { int tm, tn, split; };

// Tile shape and K split from a small cost model.  The workgroups are dealt round-robin to the
// 256 CUs; a workgroup costs a fixed part plus a time per K-tile that depends on the tile shape
// and the weight kind; two 128x128 workgroups share a CU and together run s2 times faster than
// one after the other; a layer cannot finish before its weights have crossed the memory bus
// once; a split adds a reduction launch plus the traffic of the fp32 partials.  The constants
// are a least-squares fit (microseconds) to sweeps of every shape and split over M = 128 ...
// 4096 on the four Llama-3-8B layer shapes and a square 8192 layer.
struct TileCost { double tk, tfix; };                  // per K-tile, per workgroup
static const int kTileShapes[4][2] = {{256, 256}, {256, 128}, {128, 256}, {128, 128}};    // tokens x weight rows
static const TileCost kTileCost[3][4] = {
    {{1.321, 0.69}, {1.019, 0.0}, {1.096, 0.50}, {0.811, 0.0}},     // plain FP16
    {{1.408, 0.95}, {1.080, 0.0}, {1.013, 1.74}, {0.866, 0.0}},     // NestedFP16
    {{1.337, 7.28}, {1.085, 1.12}, {1.110, 2.62}, {0.864, 0.85}},   // E4M3
};
static const double kPairSpeedup[3] = {1.46, 1.37, 1.41};

static LargeConfig choose_large(int kind, int64_t M, int64_t N, int64_t K) {
    LargeConfig c;
    const Tuning &t = tuning();
    const int kt = (int)((((kind == kE4M3) ? K : 2 * K) + 127) / 128);
    double best = 1e30;
    c.tm = c.tn = 256;
    c.split = 1;
    const int want_m = (t.large_bm == 128 || t.large_bm == 256) ? (int)t.large_bm : 0;
    const int want_n = (t.large_bn == 128 || t.large_bn == 256) ? (int)t.large_bn : want_m;
    const double mem_floor = (double)N * (double)K * (kind == kE4M3 ? 1.0 : 2.0) / 4.47e6;
    for (int sh = 0; sh < 4; ++sh) {
        const int bm = kTileShapes[sh][0], bn = kTileShapes[sh][1];
        if (want_m && bm != want_m) continue;
        if (want_n && bn != want_n) continue;
        const TileCost &tc = kTileCost[kind > 2 ? 2 : kind][sh];
        const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
        for (int split = 1; split <= 8; split *= 2) {
            if (t.large_split > 0) split = (int)(t.large_split < kt ? t.large_split : kt);
            else if (split > 1 && split > kt / 4) break;
            const int per = (kt + split - 1) / split;                     // K-tiles per workgroup
            const int slices = (kt + per - 1) / per;
            const int64_t rounds = (tiles * slices + 255) / 256;
            double time = (double)rounds * (tc.tfix + per * tc.tk);
            if (sh == 3 && rounds >= 2) time /= kPairSpeedup[kind > 2 ? 2 : kind];
            if (time < mem_floor) time = mem_floor;
            if (slices > 1) time += 4.32 + 8.0 * (double)M * (double)N * slices / 4.32e6;
            if (time < best) { best = time;  c.tm = bm;  c.tn = bn;  c.split = split; }
            if (t.large_split > 0) break;
        }
    }
    return c;
}

size_t large_gemm_partial_bytes(int kind, int64_t M, int64_t N, int64_t K) {
    LargeConfig c = choose_large(kind, M, N, K);
    return c.split > 1 ? (size_t)c.split * (size_t)M * (size_t)N * sizeof(float) : 0;
}

template <int KIND, int TM, int TN, int WAVES_M, int WAVES_N>
static void launch_large_t(const LargeParams &p, dim3 grid, hipStream_t stream) {
    auto kern = large_gemm_kernel<KIND, TM, TN, WAVES_M, WAVES_N>;
    constexpr int lds = LargeKernel<KIND, TM, TN, WAVES_M, WAVES_N>::LDS_BYTES;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr_set = true;
    }
    kern<<<grid, 64 * WAVES_M * WAVES_N, lds, stream>>>(p);
}

template <int KIND>
static void launch_large_k(const LargeParams &p, const LargeConfig &c, dim3 grid, hipStream_t stream) {
    if (c.tm == 256 && c.tn == 256) launch_large_t<KIND, 256, 256, 2, 4>(p, grid, stream);
    else if (c.tm == 256) launch_large_t<KIND, 256, 128, 4, 2>(p, grid, stream);
    else if (c.tn == 256) launch_large_t<KIND, 128, 256, 2, 4>(p, grid, stream);
    else launch_large_t<KIND, 128, 128, 2, 4>(p, grid, stream);
}

int launch_large_gemm(int kind, const GemmArgs &a, hipStream_t stream) {
    LargeConfig c = choose_large(kind, a.M, a.N, a.K);
    LargeParams p;
    p.X = static_cast<const uint8_t *>(a.X);
    p.x_row_bytes = (kind == kE4M3) ? a.ldx : 2 * a.ldx;
    p.scales = a.scales;
    p.w_scale = a.w_scale;
    p.W0 = static_cast<const uint8_t *>(a.W0);
    p.W1 = static_cast<const uint8_t *>(a.W1);
    p.w_row_bytes = (kind == kPlainF16) ? 2 * a.ldw : a.K;
    p.M = (int)a.M;  p.N = (int)a.N;  p.K = (int)a.K;
    p.k_bytes = (kind == kE4M3) ? (int)a.K : (int)(2 * a.K);
    p.kblocks = (int)((a.K + 63) / 64);
    p.Y = a.Y;  p.ldy = a.ldy;
    p.partials = a.partials;
    p.tiles_m = (int)((a.M + c.tm - 1) / c.tm);
    p.tiles_n = (int)((a.N + c.tn - 1) / c.tn);
    p.ktiles_total = (p.k_bytes + 127) / 128;
    p.ktiles_per_split = (p.ktiles_total + c.split - 1) / c.split;
    c.split = (p.ktiles_total + p.ktiles_per_split - 1) / p.ktiles_per_split;   // no empty slices
    p.vec_store = ((a.N & 3) == 0 && (a.ldy & 3) == 0 && (reinterpret_cast<uintptr_t>(a.Y) & 7) == 0) ? 1 : 0;
    p.row_store = ((a.N & 7) == 0 && (a.ldy & 7) == 0 && (reinterpret_cast<uintptr_t>(a.Y) & 15) == 0) ? 1 : 0;
    if (tuning().large_epilogue == 0) p.row_store = 0;
    if (c.split > 1 && (a.partials == nullptr ||
                        a.partial_bytes < (size_t)c.split * a.M * a.N * sizeof(float)))
        return kErrWorkspace;
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)c.split);
    switch (kind) {
        case kPlainF16: launch_large_k<kPlainF16>(p, c, grid, stream); break;
        case kNestedF16: launch_large_k<kNestedF16>(p, c, grid, stream); break;
        default: launch_large_k<kE4M3>(p, c, grid, stream); break;
    }
    if (hipGetLastError() != hipSuccess) return kErrHip;
    if (c.split > 1)
        return launch_splitk_reduce(a.partials, c.split, a.M, a.N, kind == kE4M3 ? a.scales : nullptr,
                                    a.w_scale, a.Y, a.ldy, stream);
    return kOk;
}

}  // namespace nfp
