// C[M][N] (op)= A[M][K] . W[N][K]^T  -- every projection of the decoder block, the LM head and the
// drafter's input projection.  Both operands are K-contiguous, which is what the MFMA operand
// layout wants: a lane feeds 8 consecutive k values of one row.
//
// bf16 path (gfx950): v_mfma_f32_32x32x16_bf16, fp32 accumulation.  A workgroup of 4 waves (2x2)
// owns a (64*WTM) x (64*WTN) tile; each wave owns WTM x WTN MFMA tiles of 32x32.  K is walked in
// steps of 64 through two LDS buffers (rows padded to 72 elements so the 16-byte fragment reads of 16
// consecutive rows fall in distinct bank groups); the next K step's global loads are issued before
// the current step's MFMAs.  Workgroup ids are remapped so that each XCD (ids are dealt round-robin
// over the 8 XCDs) walks a contiguous range of tiles, M fastest: neighbours on one XCD share the
// same weight tile in that XCD's L2 and every weight byte is fetched from HBM once.
//
// Generic path (fp32 mode, odd shapes): 64x64 LDS-tiled FMA kernel with full bounds checks.
#include "dev_common.h"
#include "kernels.h"

namespace tlt {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;  // 16-byte register vector (HIP's uint4 struct defeats SROA)

constexpr int kBK = 64;
constexpr int kLdsStride = 72;  // elements per LDS row (64 + 8 pad)

template <int OUT>
__device__ __forceinline__ void store_out(void* C, int64_t idx, float v) {
    if (OUT == OUT_T)
        ((bf16*)C)[idx] = from_float<bf16>(v);
    else if (OUT == OUT_F32)
        ((float*)C)[idx] = v;
    else
        ((float*)C)[idx] += v;
}

template <int WTM, int WTN, int OUT>
__global__ __launch_bounds__(256) void gemm_bf16_mfma_k(int M, int N, int K, const uint16_t* __restrict__ A,
                                                        const uint16_t* __restrict__ W, void* __restrict__ C, int nbm,
                                                        int total_tiles, int per_xcd) {
    constexpr int BM = 64 * WTM, BN = 64 * WTN;
    constexpr int A_CHUNKS = BM / 32, B_CHUNKS = BN / 32;  // 16-byte chunks per thread per K step
    extern __shared__ __align__(16) uint16_t lds[];
    uint16_t* ldsA = lds;                                // [2][BM][72]
    uint16_t* ldsB = lds + 2 * BM * kLdsStride;          // [2][BN][72]

    const int pid = blockIdx.x;
    const int logical = (pid & 7) * per_xcd + (pid >> 3);
    if (logical >= total_tiles) return;
    const int tile_m = logical % nbm, tile_n = logical / nbm;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lhi = lane >> 5;

    // global -> register -> LDS staging: thread t moves 16-byte chunk c = t + 256*i of each tile,
    // i.e. row c/8, k-chunk c%8 (8 consecutive threads read one 128-byte row segment).
    u32x4_t ra[A_CHUNKS], rb[B_CHUNKS];
    const int ld_row = tid >> 3, ld_kc = (tid & 7) * 8;
    int64_t offA[A_CHUNKS];
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
        int gr = m0 + ld_row + i * 32;
        gr = gr < M ? gr : M - 1;
        offA[i] = (int64_t)gr * K + ld_kc;
    }
    const uint16_t* gB = W + (int64_t)(n0 + ld_row) * K + ld_kc;
    const int64_t strideB = (int64_t)32 * K;
    const int lds_st = ld_row * kLdsStride + ld_kc;
#define TLT_LOAD_GLOBAL(k0)                                                                   \
    {                                                                                         \
        _Pragma("unroll") for (int i = 0; i < A_CHUNKS; ++i) ra[i] = *(const u32x4_t*)(A + offA[i] + (k0)); \
        _Pragma("unroll") for (int i = 0; i < B_CHUNKS; ++i) rb[i] = *(const u32x4_t*)(gB + i * strideB + (k0)); \
    }
#define TLT_STORE_LDS(buf)                                                                                        \
    {                                                                                                             \
        _Pragma("unroll") for (int i = 0; i < A_CHUNKS; ++i)                                                      \
            *(u32x4_t*)(ldsA + ((buf) * BM + i * 32) * kLdsStride + lds_st) = ra[i];                                \
        _Pragma("unroll") for (int i = 0; i < B_CHUNKS; ++i)                                                      \
            *(u32x4_t*)(ldsB + ((buf) * BN + i * 32) * kLdsStride + lds_st) = rb[i];                                \
    }

    f32x16_t acc[WTM][WTN];
#pragma unroll
    for (int i = 0; i < WTM; ++i)
#pragma unroll
        for (int j = 0; j < WTN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nk = K / kBK;
    TLT_LOAD_GLOBAL(0)
    TLT_STORE_LDS(0)
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) TLT_LOAD_GLOBAL((kt + 1) * kBK)
        const uint16_t* pa = ldsA + (buf * BM + wm * (WTM * 32) + l32) * kLdsStride + lhi * 8;
        const uint16_t* pb = ldsB + (buf * BN + wn * (WTN * 32) + l32) * kLdsStride + lhi * 8;
#pragma unroll
        for (int kk = 0; kk < kBK / 16; ++kk) {
            bf16x8_t fa[WTM], fb[WTN];
#pragma unroll
            for (int i = 0; i < WTM; ++i)
                fa[i] = __builtin_bit_cast(bf16x8_t, *(const u32x4_t*)(pa + i * 32 * kLdsStride + kk * 16));
#pragma unroll
            for (int j = 0; j < WTN; ++j)
                fb[j] = __builtin_bit_cast(bf16x8_t, *(const u32x4_t*)(pb + j * 32 * kLdsStride + kk * 16));
#pragma unroll
            for (int i = 0; i < WTM; ++i)
#pragma unroll
                for (int j = 0; j < WTN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) TLT_STORE_LDS(buf ^ 1)
        __syncthreads();
    }

#undef TLT_LOAD_GLOBAL
#undef TLT_STORE_LDS
    // epilogue: accumulator register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32
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

template <int WTM, int WTN>
static hipError_t launch_mfma(hipStream_t s, int out_mode, int M, int N, int K, const void* A, const void* W, void* C) {
    constexpr int BM = 64 * WTM, BN = 64 * WTN;
    const int nbm = (M + BM - 1) / BM, nbn = N / BN;
    const int total = nbm * nbn;
    const int per_xcd = (total + 7) / 8;
    const size_t lds = (size_t)2 * (BM + BN) * kLdsStride * sizeof(uint16_t);
    dim3 grid(per_xcd * 8), block(256);
#define LAUNCH(OUT)                                                                                                   \
    {                                                                                                                 \
        auto kern = gemm_bf16_mfma_k<WTM, WTN, OUT>;                                                                  \
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
    if (aligned && K % kBK == 0 && N % 128 == 0) {
        if (N % 256 == 0) {
            const int tiles256 = ((M + 255) / 256) * (N / 256);
            if (tiles256 >= 256) return launch_mfma<4, 4>(s, out_mode, M, N, K, A, W, C);
        }
        return launch_mfma<2, 2>(s, out_mode, M, N, K, A, W, C);
    }
    return launch_generic<bf16>(s, out_mode, M, N, K, A, W, C);
}

}  // namespace tlt
