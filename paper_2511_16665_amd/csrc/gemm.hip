// C[M][N] (op)= A[M][K] . W[N][K]^T  -- every projection of the decoder block, the LM head and the
// drafter's input projection.  Both operands are K-contiguous, which is what the MFMA operand
// layout wants: a lane feeds 8 consecutive k values of one row.
//
// bf16 path (gfx950): v_mfma_f32_32x32x16_bf16, fp32 accumulation.  A workgroup of 4 waves (2x2)
// owns a (64*WTM) x (64*WTN) tile; each wave owns WTM x WTN MFMA tiles of 32x32.  K is walked in
// steps of 64 through rings of LDS slots (SA for the activation rows, SB for the weight rows) filled
// by direct global->LDS loads (no staging registers, no ds_write).  Workgroups are persistent: as
// many as the chip holds at once, each walking several tiles with the load pipeline running across
// tile boundaries; ids are remapped so that each XCD (ids are dealt round-robin over the 8 XCDs) walks
// a contiguous range of tiles, M fastest: neighbours on one XCD share the same weight tile in that
// XCD's L2.
// Measured on MI355X, and what shapes the kernel: a register-only MFMA loop with one wave per SIMD
// reaches ~2.0 PFLOP/s; the chip clocks down to ~1.6-1.8 GHz under sustained MFMA load; a CU's
// vector-memory front end moves ~50 B/clk of global->LDS traffic when rows are fetched as whole
// 128-byte lines (~110 GB/s per CU, half that for 64-byte pieces), so the 64 KB a 256x256 tile
// needs per K step occupy it for ~1300 of the step's 2048 MFMA clocks.  With the output stores
// switched off the 256x256 kernel runs at 1.34-1.42 PFLOP/s on the M = 1536 shapes; the stores of a
// tile are not overlapped with compute (all workgroups finish their tiles together and the burst
// runs at the HBM write rate, ~5-6 TB/s whatever the store shape), which costs 8-15 %.
//
// Generic path (fp32 mode, odd shapes): 64x64 LDS-tiled FMA kernel with full bounds checks.
#include "dev_common.h"
#include <cmath>
#include "kernels.h"

namespace tlt {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;  // 16-byte register vector (HIP's uint4 struct defeats SROA)

constexpr int kBK = 64;

template <int OUT>
__device__ __forceinline__ void store_out(void* C, int64_t idx, float v) {
    if (OUT == OUT_T)
        ((bf16*)C)[idx] = from_float<bf16>(v);
    else if (OUT == OUT_F32 || OUT == OUT_SPLIT_F32)
        ((float*)C)[idx] = v;
    else if (OUT == OUT_ADD_F32)
        ((float*)C)[idx] += v;
    else if (OUT == OUT_ATOMIC_ADD_F32)
        unsafeAtomicAdd((float*)C + idx, v);   // split-K partial sums: hardware fp32 add at the L2
}

constexpr uint32_t vmcnt_imm(int n) { return 0x0F70u | (uint32_t)(n & 15) | ((uint32_t)(n >> 4) << 14); }

// ------------------------------------------------------------------------------------------------
// The main loop is software-pipelined by hand.  What the schedule has to respect on this chip:
//  * one wave per SIMD issues in order, so anything that blocks the wave blocks its matrix pipe;
//  * the vector-memory front end accepts one 1 KB global->LDS wave instruction every ~20 clocks and
//    a wave that issues one while it is busy waits for its turn, so the loads are never issued as a
//    burst: every MFMA row (WTN MFMAs) is followed by exactly one load, all step long;
//  * a slot can only be refilled after the barrier that frees it and must have landed before the
//    barrier that publishes it.  The activation rows get one slot more than the weight rows (3 + 2
//    slots of 32 KB = the whole 160 KB LDS for a 256x256 tile): weight loads are issued in the first
//    half of that window and have the second half to land, activation loads are issued in the
//    second half and have a whole further step.
// Per K step t (four 16-wide slices, fragment register sets F0/F1):
//    slice 0 on F0 | LDS reads of slice 1 -> F1 | W tile t-1+SB, second half
//    slice 1 on F1 | LDS reads of slice 2 -> F0 | A tile t-1+SA, first half
//    slice 2 on F0 | LDS reads of slice 3 -> F1 | A tile t-1+SA, second half
//    wait for the reads and for tile t+1, barrier                 (tile t's slots are free from here)
//    slice 3 on F1 | LDS reads of (t+1, slice 0) -> F0 | W tile t+SB, first half
// so the last slice's MFMAs cover the barrier skew and the first reads of the next tile.  The loads
// are issued from inline assembly (buffer descriptor + 32-bit per-lane byte offset + scalar K offset) and waited for
// explicitly: the compiler does not see them and so cannot order them against the LDS reads with a
// full vmcnt(0).
// LDS layout: tile rows unpadded (128 B = 8 chunks of 16 B), chunk c of row r at c ^ ((r >> 1) & 7).
// The LDS has 64 banks (256 B per clock): a 16-byte fragment read is served 16 lanes at a time, and
// with this swizzle 16 consecutive rows hit 16 distinct 16-byte columns (SQ_LDS_BANK_CONFLICT = 0;
// swizzling with r & 7 instead costs a two-way conflict on every read).
__device__ __forceinline__ void dma_buf_16(u32x4_t rsrc, uint32_t voff_bytes, uint32_t soff_bytes,
                                           uint32_t lds_bytes) {
    asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, %2 offen lds"
                 :
                 : "v"(voff_bytes), "s"(rsrc), "s"(soff_bytes), "s"(lds_bytes)
                 : "memory", "m0");
}
// the same load marked non-temporal: for weight rows that no other workgroup reads, see NTW below
__device__ __forceinline__ void dma_buf_16_nt(u32x4_t rsrc, uint32_t voff_bytes, uint32_t soff_bytes,
                                              uint32_t lds_bytes) {
    asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, %2 offen nt lds"
                 :
                 : "v"(voff_bytes), "s"(rsrc), "s"(soff_bytes), "s"(lds_bytes)
                 : "memory", "m0");
}

// GLU = true: the fused gate/up projection.  A workgroup's BN weight rows are BN/2 rows of W (gate)
// followed by the same BN/2 rows of W2 (up); each wave multiplies both halves for its columns and
// the epilogue stores silu(gate) * up, so C is [M][N] with N counting gate columns and the two
// intermediate matrices never exist.
// (The kernel's N is only the row stride of C: which column tiles exist is decided by total_tiles, and ncols,
// a multiple of 32, is where the launch's output columns end: the last column tile may reach past it.)
// NTW = true: the weight rows are fetched with the non-temporal hint.  For a single row of tiles that is not cut
// along K every weight row is read by one workgroup, once, and the hint keeps the stream from displacing what the
// caches hold of the activations and of the neighbouring kernels' data: the LM head at 40-256 rows 5-8 % faster
// (233 -> 221 us, 207 -> 193), gate/up at 256 rows 2-3 %, the small kernels around them 1-4 %.  With several row
// tiles per weight tile, or with K cuts, the same hint costs 1-5 % (o projection at 1536 rows 46.7 -> 48.1 us, the
// down projection's 8 cuts at 256 rows 45.2 -> 47.6): those launches do not take it, except the K cuts of 128x128
// tiles at up to 128 rows (one row of tiles: 14.8 -> 14.1 us at 40 rows, plain decoding at batch 32 5.60 -> 5.56 ms).
// (Kernel traces of both builds on one box.)
template <int WGM, int WGN, int WTM, int WTN, int SA, int SB, int OUT, bool GLU = false, bool NTW = false>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_pipe_k(int M, int N, int K, const uint16_t* __restrict__ A,
                                                        const uint16_t* __restrict__ W, const uint16_t* __restrict__ W2,
                                                        void* __restrict__ C, int nbm, int total_tiles, int per_xcd,
                                                        int ksplit, int wg_per_xcd, int32_t* __restrict__ C2, int kskew,
                                                        int64_t split_stride, int ncols) {
    constexpr int NW = WGM * WGN;
    constexpr int BKS = 64;
    constexpr int BM = 32 * WTM * WGM, BN = 32 * WTN * WGN;
    constexpr int ASZ = BM * BKS, BSZ = BN * BKS;      // elements per A slot / W slot
    constexpr int LA = BM / 8 / NW, LB = BN / 8 / NW;  // 1 KB DMA instructions per wave per tile: A part, W part
    constexpr int NR = WTM + WTN;                     // fragment reads per slice
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile rows must split evenly over the waves");
    static_assert(LA % 2 == 0 && LB % 2 == 0 && WTM >= 2, "schedule: each operand's loads are split over two slices");
    static_assert(SA >= 2 && SB >= 2, "at least double buffering");
    constexpr int RQ = (NR + WTM / 2 - 1) / (WTM / 2);   // fragment reads issued by each of the first WTM/2 MFMA rows
    // loads that may still be in flight when tile t+1 must be complete (issue order per step: W, then A)
    constexpr int kInFlightA = (SA - 2) * (LA + LB), kInFlightB = (SB - 1) * LA + (SB - 2) * LB;
    constexpr int kInFlight = kInFlightA < kInFlightB ? kInFlightA : kInFlightB;
    constexpr int BNO = GLU ? BN / 2 : BN;            // output columns per workgroup
    // widths that do not divide the 128 columns every launch is a multiple of: the last column tile may be partial
    constexpr bool kPartialN = BNO % 64 != 0;
    static_assert(!GLU || (NW % 2 == 0 && WTN % 2 == 0), "gate and up halves split over waves and over a wave's column tiles");
    extern __shared__ __align__(16) uint16_t lds[];   // SA A slots, then SB W slots

    // Persistent workgroups: XCD x (ids are dealt round-robin over the XCDs) owns the logical tiles
    // x*per_xcd .. (x+1)*per_xcd-1 and its wg_per_xcd workgroups walk them with that stride, so at any
    // time an XCD works on a contiguous run of tiles (M fastest: neighbours share a weight tile in L2).
    // The K steps of all of a workgroup's tiles form one sequence that the slot rings run through
    // without draining: while the last steps of a tile compute, the first K tiles of the next one load.
    const int pid = blockIdx.x;
    const int xcd = pid & 7, wslot = pid >> 3;
    const int first = xcd * per_xcd + wslot;
    int range_end = total_tiles - xcd * per_xcd;
    range_end = range_end < per_xcd ? range_end : per_xcd;
    if (wslot >= range_end) return;
    const int n_my = (range_end - wslot + wg_per_xcd - 1) / wg_per_xcd;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int nk_all = K / BKS;
    const bool up_wave = GLU && wave >= NW / 2;

    // tile j of this workgroup: M fastest, then N, then the K split.  An XCD's run of tiles then lies in one K split
    // (or two): its workgroups walk the same K range together and share the activation K tiles in its L2, where
    // with the split inside N every XCD would fetch the activation rows of every K range.
    struct TileInfo { int m0, n0, kt0, nt, split; };
    const int nbn_all = total_tiles / (nbm * ksplit);
    auto tile_info = [&](int j) {
        const int logical = first + j * wg_per_xcd;
        const int tile_m = logical % nbm, tile_n = (logical / nbm) % nbn_all, split = logical / (nbm * nbn_all);
        TileInfo ti;
        // (integer division runs on the vector ALU: pin the uniform results back into scalar registers)
        ti.m0 = __builtin_amdgcn_readfirstlane(tile_m * BM);
        ti.n0 = __builtin_amdgcn_readfirstlane(tile_n * BNO);
        // K tiles of split i: an even cut, or (kskew > 0) lengths that rise linearly from the mean - kskew
        // to the mean + kskew, so that the splits of a one-round launch end at different times and the
        // partial tiles of the early ones are added while the others still multiply
        auto kbound = [&](int i) {   // (nk_all * ksplit < 2^31 by the shape check)
            int k = nk_all * i / ksplit;
            if (kskew > 0) k += kskew * (i * (i - 1) - i * (ksplit - 1)) / (ksplit - 1);
            return k;
        };
        ti.kt0 = __builtin_amdgcn_readfirstlane(kbound(split));
        ti.nt = __builtin_amdgcn_readfirstlane(kbound(split + 1)) - ti.kt0;
        ti.split = __builtin_amdgcn_readfirstlane(split);
        return ti;
    };
    // raw buffer descriptors (four scalar words: base, base high bits, size in bytes, format) over a
    // tile's two row panels.  The activation panel's size is its valid rows: lanes that would fetch rows
    // past M are out of range and fetch nothing (their accumulator rows are never stored).  Every
    // in-range offset is below 2^31 by the launcher's shape check.
    auto desc = [&](const uint16_t* base, uint32_t bytes) {
        const uint64_t p = (uint64_t)(uintptr_t)base;
        u32x4_t d;
        d[0] = __builtin_amdgcn_readfirstlane((uint32_t)p);
        d[1] = __builtin_amdgcn_readfirstlane((uint32_t)(p >> 32) & 0xffffu);
        d[2] = bytes;
        d[3] = 0x00020000u;
        return d;
    };
    auto desc_a = [&](const TileInfo& ti) {
        int rows = M - ti.m0;
        rows = rows < BM ? rows : BM;
        return desc(A + (int64_t)ti.m0 * K, (uint32_t)(rows * K * 2));
    };
    // (GLU: the first half of the waves fetch the gate rows, the second half the up rows; a wave's
    // LB blocks are BN / NW consecutive tile rows, so they never straddle the two halves)
    // Where the last column tile of a launch may be partial (kPartialN), the weight panel's size is its valid rows
    // as well: rows past ncols fetch nothing, and the columns they would make are never stored.
    auto desc_b = [&](const TileInfo& ti) {
        const uint16_t* base = up_wave ? W2 + ((int64_t)ti.n0 - BN / 2) * K : W + (int64_t)ti.n0 * K;
        if constexpr (!kPartialN) return desc(base, 0x7fffffffu);
        int cols = ncols - ti.n0;
        cols = cols < BNO ? cols : BNO;
        return desc(base, (uint32_t)(((up_wave ? BN / 2 : 0) + cols) * K * 2));
    };

    // DMA addressing: wave w fills 1 KB blocks w*LA .. of an A slot (8 tile rows each) and w*LB .. of
    // a W slot; lane -> (row r of the block, stored chunk c) fetches the logical chunk that the
    // swizzle places there
    const int r = lane >> 3, c = lane & 7;
    uint32_t offA[LA], offB[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int trow = (wave * LA + i) * 8 + r;
        offA[i] = ((uint32_t)trow * (uint32_t)K + (c ^ ((trow >> 1) & 7)) * 8) * 2u;
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int trow = (wave * LB + i) * 8 + r;
        offB[i] = ((uint32_t)trow * (uint32_t)K + (c ^ ((trow >> 1) & 7)) * 8) * 2u;
    }
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t*)lds;
    const uint32_t lds_waveA = lds_base + (uint32_t)(wave * LA) * 1024u;
    const uint32_t lds_waveB = lds_base + (uint32_t)(SA * ASZ * 2) + (uint32_t)(wave * LB) * 1024u;

    // load cursors: the next K tile each operand fetches, in the order the compute side consumes them
    // (descriptor, absolute K tile index, end of the tile's K range).  When a cursor reaches the end of
    // its tile it jumps to the `next` triple, which the compute loop points at its following tile, or,
    // after the last one, back at the last K tile (harmless re-fetches keep the schedule uniform).  All
    // of it is scalar selects: the K loop stays one basic block.  A cursor runs at most SA-1 K tiles
    // ahead, so with at least SA K tiles per tile (the launcher's condition for giving a workgroup more
    // than one) it never needs more than the one following tile.
    const TileInfo ti0 = tile_info(0);
    u32x4_t rsA = desc_a(ti0), rsB = desc_b(ti0), rsA_nx = rsA, rsB_nx = rsB;
    int a_kt = ti0.kt0, a_end = ti0.kt0 + ti0.nt, b_kt = a_kt, b_end = a_end;
    int nx_kt0 = a_end - 1, nx_end = a_end;
    uint32_t kA2 = (uint32_t)a_kt * (BKS * 2), kB2 = kA2;   // byte offset of the cursor's K tile in a row
    auto advance_a = [&]() {
        ++a_kt;
        const bool wrap = a_kt == a_end;
#pragma unroll
        for (int w = 0; w < 3; ++w) rsA[w] = wrap ? rsA_nx[w] : rsA[w];
        a_kt = wrap ? nx_kt0 : a_kt;
        a_end = wrap ? nx_end : a_end;
        kA2 = (uint32_t)a_kt * (BKS * 2);
    };
    auto advance_b = [&]() {
        ++b_kt;
        const bool wrap = b_kt == b_end;
#pragma unroll
        for (int w = 0; w < 3; ++w) rsB[w] = wrap ? rsB_nx[w] : rsB[w];
        b_kt = wrap ? nx_kt0 : b_kt;
        b_end = wrap ? nx_end : b_end;
        kB2 = (uint32_t)b_kt * (BKS * 2);
    };
    // point `next` at tile j+1 (call while both cursors are inside tile j)
    auto set_next = [&](int j, const TileInfo& tj) {
        if (j + 1 < n_my) {
            const TileInfo tn = tile_info(j + 1);
            rsA_nx = desc_a(tn);
            rsB_nx = desc_b(tn);
            nx_kt0 = tn.kt0;
            nx_end = tn.kt0 + tn.nt;
        } else {
            rsA_nx = desc_a(tj);
            rsB_nx = desc_b(tj);
            nx_kt0 = tj.kt0 + tj.nt - 1;
            nx_end = tj.kt0 + tj.nt;
        }
    };
    set_next(0, ti0);

#define TLT_DMA_A(slot, d) dma_buf_16(rsA, offA[d], kA2, lds_waveA + (uint32_t)((slot) * ASZ * 2 + (d) * 1024));
#define TLT_DMA_B(slot, d)                                                                                        \
    {                                                                                                             \
        if constexpr (NTW) dma_buf_16_nt(rsB, offB[d], kB2, lds_waveB + (uint32_t)((slot) * BSZ * 2 + (d) * 1024)); \
        else dma_buf_16(rsB, offB[d], kB2, lds_waveB + (uint32_t)((slot) * BSZ * 2 + (d) * 1024));                \
    }

    f32x16_t acc[WTM][WTN];
#pragma unroll
    for (int i = 0; i < WTM; ++i)
#pragma unroll
        for (int j = 0; j < WTN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // prologue: K tile 0 first, then A tiles 1 .. SA-2, W tiles 1 .. SB-2 and the first half of W tile SB-1
#pragma unroll
    for (int d = 0; d < LA; ++d) TLT_DMA_A(0, d)
    advance_a();
#pragma unroll
    for (int d = 0; d < LB; ++d) TLT_DMA_B(0, d)
    advance_b();
#pragma unroll
    for (int st = 1; st < SA - 1; ++st) {
#pragma unroll
        for (int d = 0; d < LA; ++d) TLT_DMA_A(st, d)
        advance_a();
    }
#pragma unroll
    for (int st = 1; st < SB - 1; ++st) {
#pragma unroll
        for (int d = 0; d < LB; ++d) TLT_DMA_B(st, d)
        advance_b();
    }
#pragma unroll
    for (int d = 0; d < LB / 2; ++d) TLT_DMA_B(SB - 1, d)

    const int fragA = (wm * (WTM * 32) + l32) * BKS;
    // tile row of column tile j of this wave (GLU: j < WTN/2 are gate rows, the rest the matching up rows)
    auto colrow = [&](int j) {
        return GLU ? (j / (WTN / 2)) * (BN / 2) + (j % (WTN / 2)) * 32 : j * 32;
    };
    const int fragB = ((GLU ? wn * (WTN / 2 * 32) : wn * (WTN * 32)) + l32) * BKS;
    const int sw = (l32 >> 1) & 7;

    bf16x8_t fa[2][WTM], fb[2][WTN];
    // read q of a slice's NR fragment reads: the W fragments first (every MFMA row needs them all)
#define TLT_READ1(buf, pa, pb, kk, q)                                                                             \
    {                                                                                                             \
        const int ch = ((2 * (kk) + lhi) ^ sw) * 8;                                                               \
        if ((q) < WTN) fb[buf][q] = __builtin_bit_cast(bf16x8_t, *(const u32x4_t*)((pb) + fragB + colrow(q) * BKS + ch)); \
        else fa[buf][(q) - WTN] = __builtin_bit_cast(bf16x8_t, *(const u32x4_t*)((pa) + fragA + ((q) - WTN) * 32 * BKS + ch)); \
    }
#define TLT_MFMA(buf, i, j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
    // one slice: the MFMA rows on fragment set `buf`; the reads of the next slice into the other set
    // in its first rows; the H loads base .. base+H-1 of operand OP (0 = A, 1 = W) spread evenly
    // over the rows, each issued after its row's MFMAs.  Odd rows run their columns backwards, so that
    // consecutive MFMAs always share one operand (the launches run against the power limit: 0.4 % of
    // the verification GEMMs' time, measured)
#define TLT_SLICE(buf, pa, pb, rkk, OP, slot, base, H)                                                            \
    _Pragma("unroll") for (int i = 0; i < WTM; ++i) {                                                              \
        if (i < WTM / 2) {                                                                                        \
            _Pragma("unroll") for (int q = i * RQ; q < (i + 1) * RQ && q < NR; ++q) TLT_READ1((buf) ^ 1, pa, pb, rkk, q) \
        }                                                                                                         \
        _Pragma("unroll") for (int j = 0; j < WTN; ++j) TLT_MFMA(buf, i, ((i & 1) ? WTN - 1 - j : j))              \
        __builtin_amdgcn_sched_barrier(0);                                                                        \
        _Pragma("unroll") for (int d = (i * (H)) / WTM; d < ((i + 1) * (H)) / WTM; ++d) {                          \
            if ((OP) == 0) TLT_DMA_A(slot, (base) + d) else TLT_DMA_B(slot, (base) + d)                            \
        }                                                                                                         \
        __builtin_amdgcn_sched_barrier(0);                                                                        \
    }

    __builtin_amdgcn_s_waitcnt(vmcnt_imm((SA - 2) * LA + (SB - 2) * LB + LB / 2));   // K tile 0 has landed
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int q = 0; q < NR; ++q) TLT_READ1(0, lds, lds + SA * ASZ, 0, q)

    // slot of the current K tile in each ring; pa_/pb_ = slot of the one before (refilled during this step)
    int sa = 0, sb = 0, pa_ = SA - 1, pb_ = SB - 1;
    for (int j = 0; j < n_my; ++j) {
        const TileInfo ti = tile_info(j);
        if (j > 0) set_next(j, ti);
        for (int t = 0; t < ti.nt; ++t) {
            const uint16_t* pa = lds + sa * ASZ;
            const uint16_t* pb = lds + SA * ASZ + sb * BSZ;
            const int na = sa + 1 == SA ? 0 : sa + 1, nb = sb + 1 == SB ? 0 : sb + 1;
            // the first slice's fragments were requested a whole slice ago; waiting here, before the next
            // reads are issued, keeps the compiler from waiting for those as well
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            TLT_SLICE(0, pa, pb, 1, 1, pb_, LB / 2, LB / 2)           // W cursor, second half
            advance_b();
            TLT_SLICE(1, pa, pb, 2, 0, pa_, 0, LA / 2)                // A cursor, first half
            TLT_SLICE(0, pa, pb, 3, 0, pa_, LA / 2, LA / 2)           //           second half
            advance_a();
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(kInFlight));        // the next K tile has landed
            __builtin_amdgcn_s_barrier();                            // ... for every wave; this one's slots are free
            __builtin_amdgcn_sched_barrier(0);
            TLT_SLICE(1, lds + na * ASZ, lds + SA * ASZ + nb * BSZ, 0, 1, sb, 0, LB / 2)   // W cursor, first half
            pa_ = sa; pb_ = sb; sa = na; sb = nb;
        }
        // the tile is complete: store it and clear the accumulators while the next tile's loads land
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (OUT == OUT_ROWMAX) {
            // best (value, column) of each of this wave's WTM*32 rows over its WTN*32 columns: first over a
            // lane's own WTN columns of the row, then across the 32 lanes that hold the row's other
            // columns.  That second reduction is a reduce-scatter: every exchange halves the rows a lane
            // still carries, so it costs 2*NV exchanges instead of 5*NV; a lane ends with rows
            // k = lane32*NV/32 .. of the wave's NV = WTM*16 (row index k = i*16 + v within its half).
            constexpr int NV = WTM * 16;
            float bv[NV];
            int bi[NV];
#pragma unroll
            for (int i = 0; i < WTM; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float m = acc[i][0][v];
                    int mi = ti.n0 + wn * (WTN * 32) + l32;
#pragma unroll
                    for (int jj = 1; jj < WTN; ++jj)
                        if (acc[i][jj][v] > m) {   // strictly greater: the lower column wins a tie
                            m = acc[i][jj][v];
                            mi = ti.n0 + wn * (WTN * 32) + jj * 32 + l32;
                        }
                    bv[i * 16 + v] = m;
                    bi[i * 16 + v] = mi;
                }
#pragma unroll
            for (int H = NV / 2, mask = 16; mask >= 1; H >>= 1, mask >>= 1) {
                const bool upper = (l32 & mask) != 0;   // this lane keeps the upper half of what it carries
#pragma unroll
                for (int k = 0; k < (H > 0 ? H : 1); ++k) {
                    if (H > 0) {
                        const float send_v = upper ? bv[k] : bv[k + H];
                        const int send_i = upper ? bi[k] : bi[k + H];
                        const float keep_v = upper ? bv[k + H] : bv[k];
                        const int keep_i = upper ? bi[k + H] : bi[k];
                        const float ov = __shfl_xor(send_v, mask, 64);
                        const int oi = __shfl_xor(send_i, mask, 64);
                        const bool take = ov > keep_v || (ov == keep_v && oi < keep_i);
                        bv[k] = take ? ov : keep_v;
                        bi[k] = take ? oi : keep_i;
                    }
                }
            }
            constexpr int PER = NV / 32;   // rows a lane ends with
            const int P = N;               // partial blocks per row of the whole product
#pragma unroll
            for (int e = 0; e < PER; ++e) {
                const int k = l32 * PER + e, i = k >> 4, v = k & 15;
                const int row = ti.m0 + wm * (WTM * 32) + i * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3);
                if (row < M) {
                    const int64_t o = (int64_t)row * P + ti.n0 / (WTN * 32) + wn;
                    ((float*)C)[o] = bv[e];
                    C2[o] = bi[e];
                }
            }
        } else if constexpr (GLU && OUT == OUT_T) {
            // A lane holds one column of four consecutive rows (v = 4 vq .. 4 vq + 3) of each 32x32 block: stored
            // as they lie, that is 2 bytes per lane and store instruction, and the tile's 512 of those cost
            // more than its arithmetic.  The four lanes of a quad trade values instead (two exchanges of fp32 with
            // the neighbour, one of a packed pair with the lane two over) until each holds four adjacent
            // columns of one row, and stores them as 8 bytes (gate/up at M = 1536: 408 -> 394 us, at M = 128: 95 -> 88;
            // the same trade for fp32 output, or for a plain bf16 product, gains nothing: measured).
            const int q4 = lane & 3;
            const bool odd = (q4 & 1) != 0, hi2 = (q4 & 2) != 0;
            auto swap1 = [](float x) {   // value of the neighbouring lane (quad permutation 1, 0, 3, 2)
                return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xF, 0xF, false));
            };
            auto swap2 = [](uint32_t x) {   // value of the lane two over (quad permutation 2, 3, 0, 1)
                return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xF, 0xF, false);
            };
#pragma unroll
            for (int i = 0; i < WTM; ++i) {
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    const int row = ti.m0 + wm * (WTM * 32) + i * 32 + 8 * vq + 4 * lhi + q4;   // the row this lane stores
#pragma unroll
                    for (int jj = 0; jj < WTN / 2; ++jj) {
                        float r[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            // (the accumulators leave their registers here and nowhere earlier: left to itself the
                            // compiler copies most of the tile out first and spills)
                            float g, u;
                            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(g) : "a"(acc[i][jj][4 * vq + e]));
                            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(u) : "a"(acc[i][jj + WTN / 2][4 * vq + e]));
                            // (hardware reciprocal, 1 ulp: the result is rounded to bf16 anyway, and an IEEE division
                            // per element costs the tile epilogue several microseconds)
                            r[e] = g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;
                        }
                        // rows 0/1 and 2/3: an even lane keeps the lower row and gets the neighbour's column of it
                        const float n01 = swap1(odd ? r[0] : r[1]), n23 = swap1(odd ? r[2] : r[3]);
                        const uint32_t w01 = odd ? pack_bf16x2(n01, r[1]) : pack_bf16x2(r[0], n01);
                        const uint32_t w23 = odd ? pack_bf16x2(n23, r[3]) : pack_bf16x2(r[2], n23);
                        // lanes 0/1 of the quad keep rows 0/1, lanes 2/3 rows 2/3; the other pair of columns comes over
                        const uint32_t other = swap2(hi2 ? w01 : w23);
                        uint2 out;
                        out.x = hi2 ? other : w01;
                        out.y = hi2 ? w23 : other;
                        const int col0 = ti.n0 + wn * (WTN / 2 * 32) + jj * 32;   // (a 32-column block is valid or not as a whole)
                        if (row < M && (!kPartialN || col0 < ncols)) *(uint2*)((bf16*)C + (int64_t)row * N + col0 + (l32 & ~3)) = out;
                        // (keeps the compiler from fetching all accumulators first: that spills, and a reload from
                        // scratch waits for every load in flight, the next tile's first K tiles included)
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        } else {
#pragma unroll
        for (int i = 0; i < WTM; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int row = ti.m0 + wm * (WTM * 32) + i * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3);
                if (row < M) {
                    if (GLU) {
#pragma unroll
                        for (int jj = 0; jj < WTN / 2; ++jj) {
                            const int col0 = ti.n0 + wn * (WTN / 2 * 32) + jj * 32;
                            if (kPartialN && col0 >= ncols) continue;
                            int col = col0 + l32;
                            const float g = acc[i][jj][v], u = acc[i][jj + WTN / 2][v];
                            // (hardware reciprocal, 1 ulp: the result is rounded to bf16 anyway, and an IEEE division
                            // per element costs the tile epilogue several microseconds)
                            store_out<OUT>(C, (int64_t)row * N + col, g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u);
                        }
                    } else {
#pragma unroll
                        for (int jj = 0; jj < WTN; ++jj) {
                            const int col0 = ti.n0 + wn * (WTN * 32) + jj * 32;
                            if (kPartialN && col0 >= ncols) continue;
                            int col = col0 + l32;
                            store_out<OUT>(C, (OUT == OUT_SPLIT_F32 ? (int64_t)ti.split * split_stride : (int64_t)0) + (int64_t)row * N + col,
                                           acc[i][jj][v]);
                        }
                    }
                }
            }
        }
        }
#pragma unroll
        for (int i = 0; i < WTM; ++i)
#pragma unroll
            for (int jj = 0; jj < WTN; ++jj)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][jj][v] = 0.f;
    }
#undef TLT_READ1
#undef TLT_MFMA
#undef TLT_SLICE
#undef TLT_DMA_A
#undef TLT_DMA_B
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // drain the redundant tail fetches before the LDS is released
}

template <typename T, int OUT>
__device__ __forceinline__ void store_out_t(void* C, int64_t idx, float v) {
    if (OUT == OUT_T)
        ((T*)C)[idx] = from_float<T>(v);
    else if (OUT == OUT_F32)
        ((float*)C)[idx] = v;
    else
        ((float*)C)[idx] += v;
}

template <typename T, int OUT>
__global__ __launch_bounds__(256) void gemm_generic_k(int M, int N, int K, const T* __restrict__ A,
                                                      const T* __restrict__ W, void* __restrict__ C) {
    __shared__ float As[16][65], Ws[16][65];
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int idx = tid + i * 256, row = idx >> 4, k = idx & 15;
            int gm = m0 + row, gn = n0 + row, gk = k0 + k;
            As[k][row] = (gm < M && gk < K) ? to_float(A[(int64_t)gm * K + gk]) : 0.f;
            Ws[k][row] = (gn < N && gk < K) ? to_float(W[(int64_t)gn * K + gk]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = As[k][ty * 4 + i];
                w[i] = Ws[k][tx * 4 + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int row = m0 + ty * 4 + i;
        if (row >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int col = n0 + tx * 4 + j;
            if (col < N) store_out_t<T, OUT>(C, (int64_t)row * N + col, acc[i][j]);
        }
    }
}

template <int WGM, int WGN, int WTM, int WTN, int SA, int SB, bool GLU = false, bool NTW = false>
static hipError_t launch_pipe(hipStream_t s, int out_mode, int M, int N, int K, const void* A, const void* W, void* C,
                              const void* W2 = nullptr, int ksplit = 1, int ldc = 0, int kskew = 0) {
    // N counts the output columns this launch covers; ldc (default N) is the row stride of C
    constexpr int BM = 32 * WTM * WGM, BN = 32 * WTN * WGN;
    if (ldc == 0) ldc = N;
    constexpr int BNO = GLU ? BN / 2 : BN;
    // (only tile widths that do not divide 64 handle a partial last column tile; N % 32 == 0 either way)
    if ((BNO % 64 == 0 && N % BNO != 0) || N % 32 != 0) return hipErrorInvalidValue;
    const int nbm = (M + BM - 1) / BM, nbn = (N + BNO - 1) / BNO;
    const int total = nbm * nbn * ksplit;
    const int per_xcd = (total + 7) / 8;
    const size_t lds = ((size_t)SA * BM + (size_t)SB * BN) * 64 * sizeof(uint16_t);
    // persistent workgroups: as many as the chip holds at once (32 CUs per XCD, LDS-limited occupancy)
    const int occupancy = lds <= 80 * 1024 ? 2 : 1;
    // (a workgroup that walks several tiles needs at least SA K tiles in each)
    const bool persistent = (K / 64) / ksplit >= SA;
    const int wg_per_xcd = (!persistent || per_xcd < 32 * occupancy) ? per_xcd : 32 * occupancy;
    dim3 grid(wg_per_xcd * 8), block(64 * WGM * WGN);
#define LAUNCH(OUT)                                                                                                   \
    {                                                                                                                 \
        auto kern = gemm_bf16_pipe_k<WGM, WGN, WTM, WTN, SA, SB, OUT, GLU, NTW && (OUT == OUT_T || OUT == OUT_F32 || OUT == OUT_SPLIT_F32)>; \
        static bool attr_set = false;                                                                                 \
        if (!attr_set) {                                                                                              \
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
            if (e != hipSuccess) return e;                                                                            \
            attr_set = true;                                                                                          \
        }                                                                                                             \
        hipLaunchKernelGGL(kern, grid, block, lds, s, M, ldc, K, (const uint16_t*)A, (const uint16_t*)W,              \
                           (const uint16_t*)W2, C, nbm, total, per_xcd, ksplit, wg_per_xcd, (int32_t*)nullptr, kskew,              \
                           (int64_t)M * ldc, N);                                                                     \
    }
    if (GLU || out_mode == OUT_T) LAUNCH(OUT_T)
    else if (out_mode == OUT_F32) LAUNCH(OUT_F32)
    else if (out_mode == OUT_SPLIT_F32) LAUNCH(OUT_SPLIT_F32)
    else if (ksplit == 1) LAUNCH(OUT_ADD_F32)
    else LAUNCH(OUT_ATOMIC_ADD_F32)
#undef LAUNCH
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_generic(hipStream_t s, int out_mode, int M, int N, int K, const void* A, const void* W, void* C) {
    dim3 grid((N + 63) / 64, (M + 63) / 64), block(256);
    if (out_mode == OUT_T)
        hipLaunchKernelGGL((gemm_generic_k<T, OUT_T>), grid, block, 0, s, M, N, K, (const T*)A, (const T*)W, C);
    else if (out_mode == OUT_F32)
        hipLaunchKernelGGL((gemm_generic_k<T, OUT_F32>), grid, block, 0, s, M, N, K, (const T*)A, (const T*)W, C);
    else
        hipLaunchKernelGGL((gemm_generic_k<T, OUT_ADD_F32>), grid, block, 0, s, M, N, K, (const T*)A, (const T*)W, C);
    return hipGetLastError();
}

// 256x256 tiles over the columns that fill whole rounds of the chip's 256 CUs, 128x128 tiles (two
// workgroups per CU) over the rest: a last round that would leave most CUs idle is replaced by a
// shorter one.  glu: W/W2 are the gate/up matrices and N counts gate columns (a 256-row weight tile
// then yields 128 output columns, a 128-row one 64).
static hipError_t launch_tiled(hipStream_t s, int out_mode, int M, int N, int K, const void* A, const void* W,
                               const void* W2, void* C, bool glu) {
    const int bno256 = glu ? 128 : 256, bno128 = glu ? 64 : 128;
    const int nbm256 = (M + 255) / 256, nbm128 = (M + 127) / 128;
    const int nbn256 = N / bno256;   // whole 256-wide column tiles
    const size_t c_elt = (glu || out_mode == OUT_T) ? 2 : 4;
    auto small = [&](int n_cols, int col0) -> hipError_t {
        const int tiles = nbm128 * (n_cols / bno128);
        const void* w = (const uint16_t*)W + (int64_t)col0 * K;
        const void* w2 = W2 ? (const uint16_t*)W2 + (int64_t)col0 * K : nullptr;
        void* c = (char*)C + (size_t)col0 * c_elt;
        // (a single row of tiles: every weight row is read once, by one workgroup: non-temporal loads, see NTW)
        if (glu && nbm128 == 1) {
            if (tiles > 256) return launch_pipe<2, 2, 2, 2, 3, 2, true, true>(s, OUT_T, M, n_cols, K, A, w, c, w2, 1, N);
            return launch_pipe<2, 2, 2, 2, 3, 3, true, true>(s, OUT_T, M, n_cols, K, A, w, c, w2, 1, N);
        }
        if (glu) {
            if (tiles > 256) return launch_pipe<2, 2, 2, 2, 3, 2, true>(s, OUT_T, M, n_cols, K, A, w, c, w2, 1, N);
            return launch_pipe<2, 2, 2, 2, 3, 3, true>(s, OUT_T, M, n_cols, K, A, w, c, w2, 1, N);
        }
        if (nbm128 == 1) {
            if (tiles > 256) return launch_pipe<2, 2, 2, 2, 3, 2, false, true>(s, out_mode, M, n_cols, K, A, w, c, nullptr, 1, N);
            return launch_pipe<2, 2, 2, 2, 3, 3, false, true>(s, out_mode, M, n_cols, K, A, w, c, nullptr, 1, N);
        }
        // more 128-row tiles than CUs (some CUs would hold two workgroups and take twice as long as the others), but
        // 192- or 256-row tiles fit the chip once: one workgroup per CU with the CU to itself, whichever of the two
        // fills more of the CUs (o projection at M = 1536: 336 tiles -> 224 of 192 rows, 49.9 -> 43.0 us; qkv at
        // M = 1536: 432 -> 216 of 256 rows, 59.8 -> 54.2 us; o at M = 2048: 448 -> 224 of 256 rows, 62.4 -> 51.0 us;
        // best of four interleaved runs on cold weights)
        if (tiles > 256) {
            const int t192 = ((M + 191) / 192) * (n_cols / bno128), t256 = nbm256 * (n_cols / bno128);
            const bool fit192 = t192 <= 256, fit256 = t256 <= 256 && t256 >= 200;
            if (fit256 && (!fit192 || t256 >= t192))
                return launch_pipe<2, 2, 4, 2, 3, 4>(s, out_mode, M, n_cols, K, A, w, c, nullptr, 1, N);
            if (fit192) return launch_pipe<2, 2, 3, 2, 3, 4>(s, out_mode, M, n_cols, K, A, w, c, nullptr, 1, N);
        }
        if (tiles > 256) return launch_pipe<2, 2, 2, 2, 3, 2>(s, out_mode, M, n_cols, K, A, w, c, nullptr, 1, N);
        return launch_pipe<2, 2, 2, 2, 3, 3>(s, out_mode, M, n_cols, K, A, w, c, nullptr, 1, N);
    };
    auto big = [&](int n_cols) -> hipError_t {
        if (nbm256 == 1) {
            if (glu) return launch_pipe<2, 2, 4, 4, 3, 2, true, true>(s, OUT_T, M, n_cols, K, A, W, C, W2, 1, N);
            return launch_pipe<2, 2, 4, 4, 3, 2, false, true>(s, out_mode, M, n_cols, K, A, W, C, nullptr, 1, N);
        }
        if (glu) return launch_pipe<2, 2, 4, 4, 3, 2, true>(s, OUT_T, M, n_cols, K, A, W, C, W2, 1, N);
        return launch_pipe<2, 2, 4, 4, 3, 2>(s, out_mode, M, n_cols, K, A, W, C, nullptr, 1, N);
    };
    const int tiles256 = nbm256 * nbn256;
    // (with M <= 64 three quarters of a 256-row tile would be padding: the 128x128 tiles stream the
    // weights faster)
    // one row of big tiles, a hundred or more of them, streams cold weights faster than twice as
    // many TA-bound small ones
    if (nbm256 == 1 && M > 128 && tiles256 >= 100 && N % bno256 == 0) {
        // more than a round of them (the LM head: 594 tiles): the whole rounds, then what is left in 256x128 tiles,
        // so that the last, partly filled round is half as long (best of four interleaved runs, M = 160 .. 256:
        // 287-312 us in one launch, 267-296 this way, 267-311 with a rest of 128x128 tiles; 32B shape 401-436 /
        // 372-410 / 369-435)
        const int main_tiles = tiles256 / 256 * 256;
        if (!glu && main_tiles > 0 && main_tiles < tiles256) {
            hipError_t e = big(main_tiles * 256);
            if (e != hipSuccess) return e;
            const void* w = (const uint16_t*)W + (int64_t)main_tiles * 256 * K;
            void* c = (char*)C + (size_t)main_tiles * 256 * c_elt;
            return launch_pipe<2, 2, 4, 2, 3, 4, false, true>(s, out_mode, M, N - main_tiles * 256, K, A, w, c, nullptr, 1, N);
        }
        // gate/up with well under a round of big tiles: 256 rows x 96 output columns per workgroup (four waves of
        // 64 rows x 3 + 3 column blocks, the last tile partial) puts the weights on 4/3 as many CUs.  A CU pulls cold
        // weights at ~35 GB/s at most, however many loads it keeps in flight, and the activation rows that every
        // workgroup re-reads from L2 go through the same path, so the gain is less than the 4/3: best of four
        // interleaved runs on cold weights, M = 144 .. 256: 7B shape (148 -> 198 tiles) 84-86 -> 80-82 us, N = 13824,
        // K = 5120 (108 -> 144) 111 -> 102-104; with 192 -> 256 tiles (N = 24576) 102-105 -> 102-110, so not there
        if (glu && tiles256 <= 160 && (N + 95) / 96 <= 256)
            return launch_pipe<4, 1, 2, 6, 3, 2, true, true>(s, OUT_T, M, N, K, A, W, C, W2, 1, N);
        return big(N);
    }
    // up to 128 rows: half of a 256-row tile would be padding, and the LDS it frees holds a third weight slot
    // (gate/up at M = 128: 85 -> 70 us, LM head: 261 -> 251; at the 32B shape 406 -> 343)
    if (M > 64 && M <= 128 && tiles256 >= 100 && N % bno256 == 0) {
        if (glu) return launch_pipe<2, 2, 2, 4, 3, 3, true, true>(s, OUT_T, M, N, K, A, W, C, W2, 1, N);
        // (more than a round: whole rounds, the rest in 128x128 tiles: LM head 227-250 -> 219-241 us, 32B shape 313-343 -> 297-325)
        const int main_tiles = tiles256 / 256 * 256;
        if (main_tiles > 0 && main_tiles < tiles256) {
            hipError_t e = launch_pipe<2, 2, 2, 4, 3, 3, false, true>(s, out_mode, M, main_tiles * 256, K, A, W, C, nullptr, 1, N);
            if (e != hipSuccess) return e;
            const void* w = (const uint16_t*)W + (int64_t)main_tiles * 256 * K;
            void* c = (char*)C + (size_t)main_tiles * 256 * c_elt;
            return launch_pipe<2, 2, 2, 2, 3, 3, false, true>(s, out_mode, M, N - main_tiles * 256, K, A, w, c, nullptr, 1, N);
        }
        return launch_pipe<2, 2, 2, 4, 3, 3, false, true>(s, out_mode, M, N, K, A, W, C, nullptr, 1, N);
    }
    if (M <= 64 || tiles256 < 256) return small(N, 0);
    const int full_rounds = tiles256 / 256;
    const int main_nbn = full_rounds * 256 / nbm256;          // column tiles that make up the whole rounds
    const int rest_cols = N - main_nbn * bno256;
    const int rest_tiles256 = tiles256 - main_nbn * nbm256 + (N % bno256 ? nbm256 : 0);
    if (main_nbn == 0) return N % bno256 == 0 ? big(N) : small(N, 0);
    if (rest_cols == 0) return big(N);
    if (rest_tiles256 >= 140 && N % bno256 == 0) return big(N);   // the last round is well filled as it is
    hipError_t e = big(main_nbn * bno256);
    if (e != hipSuccess) return e;
    // the rest in 256x128 tiles, one per CU (gate/up, best of four interleaved runs: M = 1536, a rest of 120 big
    // tiles: 331 us with 128x128 tiles, 323 this way, 347 in one launch of big tiles; M = 1024, rest 80: 249 /
    // 232 / 255; M = 2048, rest 160: 468 / 454 / 435)
    if (rest_cols % bno256 == 0) {
        const int col0 = main_nbn * bno256;
        const void* w = (const uint16_t*)W + (int64_t)col0 * K;
        const void* w2 = W2 ? (const uint16_t*)W2 + (int64_t)col0 * K : nullptr;
        void* c = (char*)C + (size_t)col0 * c_elt;
        if (glu) return launch_pipe<2, 2, 4, 2, 3, 4, true>(s, OUT_T, M, rest_cols, K, A, w, c, w2, 1, N);
        return launch_pipe<2, 2, 4, 2, 3, 4>(s, out_mode, M, rest_cols, K, A, w, c, nullptr, 1, N);
    }
    return small(rest_cols, main_nbn * bno256);
}

// How a product whose fp32 result is summed by its consumer is cut along K (bf16 MFMA path).  kind 0: not at all;
// 1: 256x128 tiles; 2: 256x256 tiles; 3: 128x128 tiles.
//
// The plan is the minimum of a small cost model over (tile shape, number of cuts).  A launch takes a ramp plus, for
// every round of workgroups the chip has to run (one per CU; 128x128 tiles past 256 workgroups share CUs in pairs and
// run slower), the K steps of a cut at the tile shape's clocks per step plus its epilogue; every cut after the first
// adds M*N*4 bytes that the consumer (the norm or rotary kernel that sums the slices) reads at ~4 TB/s.  The
// constants were fitted to a sweep on the chip (nine projection shapes of the 7B / 32B / 70B models, M = 96 .. 1536,
// kinds 1-3, 1-12 cuts, cold weights, best of three interleaved runs, even cuts): the model's pick is within 0.9 %
// of the best measured plan on average (worst case 11 %), where the rules it replaces were 7.8 % off on average and
// up to 49 % (M = 384 .. 1024).  Uneven cuts, which paid when the cuts accumulated with atomics, lost 3-5 % to even
// ones in the same sweep, so the cuts are even.
struct SplitPlan {
    int kind = 0, ks = 1, skew = 0;
};
static SplitPlan plan_split(int M, int N, int K, int max_ks = 12, double uncut_credit_us = 0.0) {
    SplitPlan sp;
    if (N % 128 != 0 || M < 1) return sp;
    const int nk = K / kBK;
    const int nbm256 = (M + 255) / 256, nbm128 = (M + 127) / 128;
    auto cost_us = [&](int kind, int ks) -> double {
        int tiles;
        double step_clk, epilogue_clk;
        if (kind == 1) tiles = nbm256 * (N / 128), step_clk = 1396, epilogue_clk = 9827;
        else if (kind == 2) tiles = nbm256 * (N / 256), step_clk = 2266, epilogue_clk = 18240;
        else tiles = nbm128 * (N / 128), step_clk = 988, epilogue_clk = 5754;
        const int wgs = tiles * ks;
        const double steps = (double)nk / ks;
        double clk;
        if (kind == 3 && wgs > 256) clk = (double)((wgs + 511) / 512) * (steps * 2390 + epilogue_clk);
        else clk = (double)((wgs + 255) / 256) * (steps * step_clk + epilogue_clk);
        return 1.6 + clk / 1800.0 + (ks - 1) * (double)M * N * 4.0 / 4.0e6;
    };
    // (not cut at all, the product takes the tiled launcher's own pick of a tile shape: the best of the three here
    // and of the 192x128 tiles that launcher has besides, 1259 clocks per step and 4000 of epilogue)
    double best = cost_us(1, 1);
    if (cost_us(3, 1) < best) best = cost_us(3, 1);
    if (N % 256 == 0 && cost_us(2, 1) < best) best = cost_us(2, 1);
    {
        const int t192 = ((M + 191) / 192) * (N / 128);
        const double c192 = 1.6 + (double)((t192 + 255) / 256) * (nk * 1259.0 + 4000.0) / 1800.0;
        if (c192 < best) best = c192;
    }
    best -= uncut_credit_us;   // (what the uncut product saves its caller besides, e.g. an output in the model dtype)
    if (max_ks > 12) max_ks = 12;
    for (int kind = 1; kind <= 3; ++kind) {
        if (kind == 2 && N % 256 != 0) continue;
        for (int ks = 2; ks <= max_ks && nk / ks >= 6; ++ks) {
            const double c = cost_us(kind, ks);
            if (c < best) {
                best = c;
                sp.kind = kind, sp.ks = ks, sp.skew = 0;
            }
        }
    }
    return sp;
}

static bool pipe_ok(int N, int K, const void* A, const void* W) {
    const bool aligned = (((uintptr_t)A | (uintptr_t)W) & 15) == 0;
    // per-lane DMA offsets are 32-bit byte offsets inside a 256-row panel
    return aligned && K % kBK == 0 && N % 128 == 0 && (int64_t)258 * K * 2 < ((int64_t)1 << 31);
}

hipError_t gemm(hipStream_t s, int dtype, int out_mode, int M, int N, int K, const void* A, const void* W, void* C) {
    if (M <= 0 || N <= 0 || K <= 0) return hipSuccess;
    if (dtype == F32) return launch_generic<float>(s, out_mode, M, N, K, A, W, C);
    if (pipe_ok(N, K, A, W)) {
        // (accumulating into C: the K splits add their partial sums with fp32 atomics, in any order, so the
        // last bit of the result is not fixed.  The step itself uses gemm_parts, which is reproducible.)
        if (out_mode == OUT_ADD_F32) {
            const SplitPlan sp = plan_split(M, N, K);
            if (sp.kind == 1) return launch_pipe<2, 2, 4, 2, 3, 4>(s, out_mode, M, N, K, A, W, C, nullptr, sp.ks, 0, sp.skew);
            if (sp.kind == 2) return launch_pipe<2, 2, 4, 4, 3, 2>(s, out_mode, M, N, K, A, W, C, nullptr, sp.ks, 0, sp.skew);
            if (sp.kind == 3) return launch_pipe<2, 2, 2, 2, 3, 3>(s, out_mode, M, N, K, A, W, C, nullptr, sp.ks, 0, sp.skew);
        }
        return launch_tiled(s, out_mode, M, N, K, A, W, nullptr, C, false);
    }
    return launch_generic<bf16>(s, out_mode, M, N, K, A, W, C);
}

// room for the slices of the few-row products (at 256 rows 8 cuts of a 4608-wide product take 38 MB); a plan that
// does not fit the caller's buffer is cut less
// Whether the product as K-cut fp32 slices (gemm_parts) is expected to beat the same product stored once in the
// model dtype, counting the bytes the slices cost their reader and the writer over a bf16 result.
bool gemm_parts_pays(int dtype, int M, int N, int K) {
    if (dtype != BF16 || M < 1 || N % 128 != 0 || K % kBK != 0) return false;
    return plan_split(M, N, K, 12, (double)M * N * 4.0 / 4.0e6).kind != 0;
}

size_t gemm_parts_max_bytes() { return (size_t)256 * 65536 * 4 + 4096; }

hipError_t gemm_parts(hipStream_t s, int dtype, int M, int N, int K, const void* A, const void* W, float* parts,
                      size_t parts_bytes, int* n_parts) {
    *n_parts = 1;
    if (M <= 0 || N <= 0 || K <= 0) return hipSuccess;
    if ((size_t)M * N * 4 > parts_bytes) return hipErrorInvalidValue;
    if (dtype == BF16 && pipe_ok(N, K, A, W)) {
        const size_t room = parts_bytes / ((size_t)M * N * 4);
        const SplitPlan sp = plan_split(M, N, K, room > 12 ? 12 : (int)room);
        if (sp.kind != 0 && (size_t)sp.ks * M * N * 4 <= parts_bytes) {
            *n_parts = sp.ks;
            if (sp.kind == 1) return launch_pipe<2, 2, 4, 2, 3, 4>(s, OUT_SPLIT_F32, M, N, K, A, W, parts, nullptr, sp.ks, 0, sp.skew);
            if (sp.kind == 3 && M <= 128)
                return launch_pipe<2, 2, 2, 2, 3, 3, false, true>(s, OUT_SPLIT_F32, M, N, K, A, W, parts, nullptr, sp.ks, 0, sp.skew);
            if (sp.kind == 3) return launch_pipe<2, 2, 2, 2, 3, 3>(s, OUT_SPLIT_F32, M, N, K, A, W, parts, nullptr, sp.ks, 0, sp.skew);
            return launch_pipe<2, 2, 4, 4, 3, 2>(s, OUT_SPLIT_F32, M, N, K, A, W, parts, nullptr, sp.ks, 0, sp.skew);
        }
    }
    return gemm(s, dtype, OUT_F32, M, N, K, A, W, parts);
}

// ---- fused row argmax (big tiles only: every 256-row weight tile yields two 128-column blocks)
__global__ __launch_bounds__(256) void argmax_blocks_k(int M, int P, const float* __restrict__ pv,
                                                       const int32_t* __restrict__ pi, int32_t* __restrict__ out) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= M) return;
    float v = -INFINITY;
    int i = 0x7fffffff;
    for (int p = lane; p < P; p += 64) {
        const float ov = pv[(int64_t)row * P + p];
        const int oi = pi[(int64_t)row * P + p];
        if (ov > v || (ov == v && oi < i)) {
            v = ov;
            i = oi;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(v, o, 64);
        const int oi = __shfl_xor(i, o, 64);
        if (ov > v || (ov == v && oi < i)) {
            v = ov;
            i = oi;
        }
    }
    if (lane == 0) out[row] = i;
}

bool gemm_argmax_supported(int dtype, int M, int N, int K, const void* A, const void* W) {
    const bool aligned = (((uintptr_t)A | (uintptr_t)W) & 15) == 0;
    return dtype == BF16 && M > 64 && aligned && K % kBK == 0 && K / kBK >= 3 && N % 256 == 0 &&
           (int64_t)258 * K * 2 < ((int64_t)1 << 31);
}

size_t gemm_argmax_workspace_bytes(int M, int N) { return (size_t)M * (N / 128) * 8; }

hipError_t gemm_argmax(hipStream_t s, int M, int N, int K, const void* A, const void* W, void* ws, int32_t* out) {
    constexpr int SA = 3, SB = 2;
    const int P = N / 128;
    float* pv = (float*)ws;
    int32_t* pi = (int32_t*)(pv + (size_t)M * P);
    const int nbm = (M + 255) / 256, nbn = N / 256, total = nbm * nbn, per_xcd = (total + 7) / 8;
    const size_t lds = ((size_t)SA * 256 + (size_t)SB * 256) * 64 * sizeof(uint16_t);
    const int wg_per_xcd = per_xcd < 32 ? per_xcd : 32;
    auto kern = gemm_bf16_pipe_k<2, 2, 4, 4, SA, SB, OUT_ROWMAX, false>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(wg_per_xcd * 8), dim3(256), lds, s, M, P, K, (const uint16_t*)A, (const uint16_t*)W,
                       (const uint16_t*)nullptr, (void*)pv, nbm, total, per_xcd, 1, wg_per_xcd, pi, 0, (int64_t)0, nbn * 256);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(argmax_blocks_k, dim3((M + 3) / 4), dim3(256), 0, s, M, P, pv, pi, out);
    return hipGetLastError();
}

bool gemm_glu_supported(int dtype, int M, int N, int K, const void* A, const void* Wg, const void* Wu) {
    const bool aligned = (((uintptr_t)A | (uintptr_t)Wg | (uintptr_t)Wu) & 15) == 0;
    return dtype == BF16 && M > 0 && aligned && K % kBK == 0 && N % 128 == 0 && (int64_t)258 * K * 2 < ((int64_t)1 << 31);
}

// act[M][N] = silu(A Wg^T) * (A Wu^T), bf16 in and out; call only when gemm_glu_supported().
hipError_t gemm_glu(hipStream_t s, int M, int N, int K, const void* A, const void* Wg, const void* Wu, void* act) {
    return launch_tiled(s, OUT_T, M, N, K, A, Wg, Wu, act, true);
}

// ---- measurement aid: what the matrix pipes sustain with nothing else running ----
// Every wave (one per SIMD of every CU) loops over the 16 x 4 MFMAs of a 128x128 wave tile and a 64-wide K tile,
// in the GEMM kernel's issue order, on register operands that never change: no LDS, no memory, no waits.  On
// random data the chip holds about 1.8 GHz under its power limit here, so the rate this loop reaches, not the
// 2.4 GHz figure, is what a GEMM kernel's share of the peak is to be read against.
__global__ __launch_bounds__(256) void mfma_stream_k(const u32x4_t* __restrict__ frags, float* __restrict__ out, int iters) {
    const int lane = threadIdx.x & 63;
    bf16x8_t fa[4][4], fb[4][4];   // [K slice of 16][fragment]
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[s][i] = __builtin_bit_cast(bf16x8_t, frags[(s * 8 + i) * 64 + lane]);
            fb[s][i] = __builtin_bit_cast(bf16x8_t, frags[(s * 8 + 4 + i) * 64 + lane]);
        }
    f32x16_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int jj = (i & 1) ? 3 - j : j;
                    acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s][i], fb[s][jj], acc[i][jj], 0, 0, 0);
                }
        __builtin_amdgcn_sched_barrier(0);
    }
    float sum = 0.f;   // in a fixed order: i, then j, then the lane's 16 elements
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) sum += acc[i][j][v];
    out[blockIdx.x * 256 + threadIdx.x] = sum;
}

hipError_t mfma_stream(hipStream_t s, const void* frags, float* out, int iters) {
    hipLaunchKernelGGL(mfma_stream_k, dim3(kMfmaStreamBlocks), dim3(256), 0, s, (const u32x4_t*)frags, out, iters);
    return hipGetLastError();
}

}  // namespace tlt
