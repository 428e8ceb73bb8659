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

// The wave's best (value, index) pair in the (value desc, index asc) order, left in every lane.  The order is total,
// so the result does not depend on how the lanes are paired; the pairing here avoids the LDS crossbar that a
// shuffle goes through (a dozen dependent ds_bpermute of ~100 clocks each per reduction): the two half-waves and the
// odd and even 16-lane rows trade through v_permlane32_swap / v_permlane16_swap (swapping a register with a copy of
// itself leaves the own and the partner's value side by side), the lanes of a row through DPP rotations by 8 and 4
// and the two quad permutations.
__device__ __forceinline__ void wave_best(float& v, int& i) {
    {
        const auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        const auto b = __builtin_amdgcn_permlane32_swap((uint32_t)i, (uint32_t)i, false, false);
        const float v0 = __uint_as_float(a[0]), v1 = __uint_as_float(a[1]);
        const int i0 = (int)b[0], i1 = (int)b[1];
        const bool first = better(v0, i0, v1, i1);
        v = first ? v0 : v1;
        i = first ? i0 : i1;
    }
    {
        const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        const auto b = __builtin_amdgcn_permlane16_swap((uint32_t)i, (uint32_t)i, false, false);
        const float v0 = __uint_as_float(a[0]), v1 = __uint_as_float(a[1]);
        const int i0 = (int)b[0], i1 = (int)b[1];
        const bool first = better(v0, i0, v1, i1);
        v = first ? v0 : v1;
        i = first ? i0 : i1;
    }
#define TLT_BEST_DPP(ctrl)                                                                                   \
    {                                                                                                        \
        const float ov = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, 0xF, 0xF, false)); \
        const int oi = __builtin_amdgcn_update_dpp(0, i, ctrl, 0xF, 0xF, false);                             \
        if (better(ov, oi, v, i)) {                                                                          \
            v = ov;                                                                                          \
            i = oi;                                                                                          \
        }                                                                                                    \
    }
    TLT_BEST_DPP(0x128)   // row_ror:8
    TLT_BEST_DPP(0x124)   // row_ror:4
    TLT_BEST_DPP(0x4E)    // quad_perm:[2,3,0,1]
    TLT_BEST_DPP(0xB1)    // quad_perm:[1,0,3,2]
#undef TLT_BEST_DPP
}

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
