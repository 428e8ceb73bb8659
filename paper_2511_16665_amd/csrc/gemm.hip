// C[M][N] (op)= A[M][K] . W[N][K]^T  -- every projection of the decoder block, the LM head and the
// drafter's input projection.  Both operands are K-contiguous, which is what the MFMA operand
// layout wants: a lane feeds 8 consecutive k values of one row.
//
// bf16 path (gfx950): v_mfma_f32_32x32x16_bf16, fp32 accumulation.  A workgroup of 4 waves (2x2)
// owns a (64*WTM) x (64*WTN) tile; each wave owns WTM x WTN MFMA tiles of 32x32.  K is walked in
// steps of 64 through two LDS stages filled by direct global->LDS loads (no staging registers, no
// ds_write).  Workgroup ids are remapped so that each XCD (ids are dealt round-robin over the 8
// XCDs) walks a contiguous range of tiles, M fastest: neighbours on one XCD share the same weight
// tile in that XCD's L2 and every weight byte is fetched from HBM once.
// Measured ceilings on MI355X that shape this kernel: a register-only MFMA loop reaches 2.0-2.4
// PFLOP/s; adding the 64 KB per K-step of global->LDS traffic of a 256x256 tile caps a CU at
// ~1.35 PFLOP/s-equivalent even when every load hits L2 (the per-CU vector-memory path sustains
// about 24 B/clk), and at ~1.0 when half the loads come over the fabric.
//
// Generic path (fp32 mode, odd shapes): 64x64 LDS-tiled FMA kernel with full bounds checks.
#include "dev_common.h"
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
    else if (OUT == OUT_F32)
        ((float*)C)[idx] = v;
    else
        ((float*)C)[idx] += v;
}

// ------------------------------------------------------------------------------------------------
// The tiles go from global memory straight into LDS (global_load_lds_dwordx4,
// 1 KB = 8 tile rows per wave instruction), so no registers are spent on staging, nothing is
// re-written with ds_write, and the only wait is the vmcnt wait for the stage loaded S-1 steps ago.
// Tile rows are stored unpadded (128 B = 8 chunks of 16 B) with chunk c of row r at position
// c ^ (r & 7): the DMA lays lanes out contiguously, so the swizzle is applied by choosing which
// global chunk each lane fetches, and the fragment reads of 8 consecutive rows hit 8 distinct
// 16-byte columns.
constexpr uint32_t vmcnt_imm(int n) { return 0x0F70u | (uint32_t)(n & 15) | ((uint32_t)(n >> 4) << 14); }

template <int WGM, int WGN, int WTM, int WTN, int STAGES, int OUT>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_dtl_k(int M, int N, int K, const uint16_t* __restrict__ A,
                                                       const uint16_t* __restrict__ W, void* __restrict__ C, int nbm,
                                                       int total_tiles, int per_xcd) {
    constexpr int NW = WGM * WGN;                    // waves per workgroup, WGM x WGN grid of wave tiles
    constexpr int BM = 32 * WTM * WGM, BN = 32 * WTN * WGN;
    constexpr int STAGE = (BM + BN) * kBK;          // elements per stage
    constexpr int LA = BM / 8 / NW, LB = BN / 8 / NW;  // DMA instructions per wave per stage for A and W
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile rows must split evenly over the waves");
    extern __shared__ __align__(16) uint16_t lds[];

    const int pid = blockIdx.x;
    const int logical = (pid & 7) * per_xcd + (pid >> 3);
    if (logical >= total_tiles) return;
    const int tile_m = logical % nbm, tile_n = logical / nbm;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: LDS DMA bases live in SGPRs
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, lhi = lane >> 5;

    // DMA addressing: instruction i of this wave covers tile rows (wave + NW i) * 8 .. + 8
    const int r8 = lane >> 3, lc = (lane & 7) ^ r8;  // row in the block, logical chunk this lane fetches
    uint32_t offA[LA];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        int row = m0 + (wave + NW * i) * 8 + r8;
        row = row < M ? row : M - 1;
        offA[i] = (uint32_t)(row - m0) * (uint32_t)K + lc * 8;
    }
    const uint32_t offB0 = (uint32_t)(wave * 8 + r8) * (uint32_t)K + lc * 8;
    const uint32_t strideB = (uint32_t)(8 * NW) * (uint32_t)K;
    const uint16_t* gA = A + (int64_t)m0 * K;
    const uint16_t* gB = W + (int64_t)n0 * K;

#define TLT_DMA(stage, k0)                                                                                       \
    {                                                                                                            \
        uint16_t* sb = lds + (stage) * STAGE;                                                                    \
        _Pragma("unroll") for (int i = 0; i < LA; ++i) __builtin_amdgcn_global_load_lds(                          \
            (const __attribute__((address_space(1))) void*)(gA + (k0) + offA[i]),                                \
            (__attribute__((address_space(3))) void*)(sb + (wave + NW * i) * 512), 16, 0, 0);                     \
        _Pragma("unroll") for (int i = 0; i < LB; ++i) __builtin_amdgcn_global_load_lds(                          \
            (const __attribute__((address_space(1))) void*)(gB + (k0) + offB0 + i * strideB),                    \
            (__attribute__((address_space(3))) void*)(sb + BM * kBK + (wave + NW * i) * 512), 16, 0, 0);          \
    }

    f32x16_t acc[WTM][WTN];
#pragma unroll
    for (int i = 0; i < WTM; ++i)
#pragma unroll
        for (int j = 0; j < WTN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nk = K / kBK;
#pragma unroll
    for (int st = 0; st < STAGES - 1; ++st) {
        const int kt = st < nk ? st : nk - 1;
        TLT_DMA(st, kt * kBK)
    }
    // fragment addressing: row l32 of each 32-row MFMA tile, chunk (2 kk + lhi) ^ (row & 7)
    const int fragA = (wm * (WTM * 32) + l32) * kBK;
    const int fragB = BM * kBK + (wn * (WTN * 32) + l32) * kBK;
    const int sw = l32 & 7;
    for (int kt = 0; kt < nk; ++kt) {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((LA + LB) * (STAGES - 2)));  // this stage's DMA has landed
        __builtin_amdgcn_s_barrier();  // ... for every wave, and the stage about to be refilled is no longer read
        {
            const int nxt = kt + STAGES - 1;
            const int ktl = nxt < nk ? nxt : nk - 1;  // past the end: harmless re-fetch of the last tile
            TLT_DMA(nxt % STAGES, ktl * kBK)
        }
        const uint16_t* sb = lds + (kt % STAGES) * STAGE;
#pragma unroll
        for (int kk = 0; kk < kBK / 16; ++kk) {
            const int ch = ((2 * kk + lhi) ^ sw) * 8;
            bf16x8_t fa[WTM], fb[WTN];
#pragma unroll
            for (int i = 0; i < WTM; ++i)
                fa[i] = __builtin_bit_cast(bf16x8_t, *(const u32x4_t*)(sb + fragA + i * 32 * kBK + ch));
#pragma unroll
            for (int j = 0; j < WTN; ++j)
                fb[j] = __builtin_bit_cast(bf16x8_t, *(const u32x4_t*)(sb + fragB + j * 32 * kBK + ch));
#pragma unroll
            for (int i = 0; i < WTM; ++i)
#pragma unroll
                for (int j = 0; j < WTN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }
#undef TLT_DMA
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // drain the redundant tail fetches before the LDS is released

#pragma unroll
    for (int i = 0; i < WTM; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int row = m0 + wm * (WTM * 32) + i * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3);
            if (row < M) {
#pragma unroll
                for (int j = 0; j < WTN; ++j) {
                    int col = n0 + wn * (WTN * 32) + j * 32 + l32;
                    store_out<OUT>(C, (int64_t)row * N + col, acc[i][j][v]);
                }
            }
        }
    }
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

template <int WGM, int WGN, int WTM, int WTN, int STAGES>
static hipError_t launch_dtl(hipStream_t s, int out_mode, int M, int N, int K, const void* A, const void* W, void* C) {
    constexpr int BM = 32 * WTM * WGM, BN = 32 * WTN * WGN;
    const int nbm = (M + BM - 1) / BM, nbn = N / BN;
    const int total = nbm * nbn;
    const int per_xcd = (total + 7) / 8;
    const size_t lds = (size_t)STAGES * (BM + BN) * kBK * sizeof(uint16_t);
    dim3 grid(per_xcd * 8), block(64 * WGM * WGN);
#define LAUNCH(OUT)                                                                                                   \
    {                                                                                                                 \
        auto kern = gemm_bf16_dtl_k<WGM, WGN, WTM, WTN, STAGES, OUT>;                                                 \
        static bool attr_set = false;                                                                                 \
        if (!attr_set) {                                                                                              \
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
            if (e != hipSuccess) return e;                                                                            \
            attr_set = true;                                                                                          \
        }                                                                                                             \
        hipLaunchKernelGGL(kern, grid, block, lds, s, M, N, K, (const uint16_t*)A, (const uint16_t*)W, C, nbm, total,  \
                           per_xcd);                                                                                  \
    }
    if (out_mode == OUT_T) LAUNCH(OUT_T)
    else if (out_mode == OUT_F32) LAUNCH(OUT_F32)
    else LAUNCH(OUT_ADD_F32)
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

hipError_t gemm(hipStream_t s, int dtype, int out_mode, int M, int N, int K, const void* A, const void* W, void* C) {
    if (M <= 0 || N <= 0 || K <= 0) return hipSuccess;
    if (dtype == F32) return launch_generic<float>(s, out_mode, M, N, K, A, W, C);
    const bool aligned = (((uintptr_t)A | (uintptr_t)W) & 15) == 0;
    // per-lane DMA offsets are 32-bit element offsets inside a 256-row panel
    if (aligned && K % kBK == 0 && N % 128 == 0 && (int64_t)256 * K < ((int64_t)1 << 31)) {
        const int tiles256 = ((M + 255) / 256) * (N / 256);
        if (N % 256 == 0 && tiles256 >= 256) return launch_dtl<2, 2, 4, 4, 2>(s, out_mode, M, N, K, A, W, C);
        return launch_dtl<2, 2, 2, 2, 2>(s, out_mode, M, N, K, A, W, C);
    }
    return launch_generic<bf16>(s, out_mode, M, N, K, A, W, C);
}

}  // namespace tlt
