// Device-side helpers shared by the HIP kernels of libtlt (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tlt {

constexpr int kWave = 64;

// bf16 is carried as its 16 raw bits; conversions are explicit.
struct bf16 {
    uint16_t bits;
};

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16 x) { return __uint_as_float(((uint32_t)x.bits) << 16); }

template <typename T>
__device__ __forceinline__ T from_float(float x);
template <>
__device__ __forceinline__ float from_float<float>(float x) {
    return x;
}
template <>
__device__ __forceinline__ bf16 from_float<bf16>(float x) {  // round to nearest, ties to even
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return bf16{(uint16_t)((u >> 16) | 0x40)};  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return bf16{(uint16_t)(u >> 16)};
}

// Two floats -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// 16 bytes per lane from global memory straight into LDS at lds_byte_offset + lane * 16 (the offset
// must be wave-uniform).  Issued through inline assembly on purpose: the compiler then does not
// treat it as an LDS write it has to order against every later LDS read (which it does with a full
// vmcnt(0) wait, i.e. by draining the whole prefetch queue); the kernels that use this wait
// explicitly with s_waitcnt vmcnt(n) for exactly the stage they are about to read.
__device__ __forceinline__ void dma_global_to_lds_16(const void* gptr, uint32_t lds_byte_offset) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gptr), "s"(lds_byte_offset)
                 : "memory", "m0");
}

// (value, index) ordering used everywhere a "largest" element is picked:
// larger value first, lower index on equal values.
__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

// Physical row of cache slot `slot` of sequence b, or -1 when the block table cannot serve it.
// Row index is in units of [page_size] rows of one kv head: caller multiplies out the layout.
struct PageRef {
    int64_t page;
    int row;
};
__device__ __forceinline__ bool locate(const int32_t* block_table, int max_pages, int64_t n_pages, int page_size, int b,
                                       int slot, PageRef& out) {
    if (slot < 0) return false;
    int lp = slot / page_size;
    if (lp >= max_pages) return false;
    int pg = block_table[(int64_t)b * max_pages + lp];
    if (pg < 0 || pg >= n_pages) return false;
    out.page = pg;
    out.row = slot - lp * page_size;
    return true;
}

}  // namespace tlt
