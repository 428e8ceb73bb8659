// Row-wise kernels of the decoder block: embedding gather, RMSNorm, rotary embedding fused with the
// write of new keys/values into the paged cache, SiLU gating, the drafter's input rows.
// All are HBM-bound streaming kernels: one workgroup per row, 16-byte accesses where the layout allows.
#include "dev_common.h"
#include "kernels.h"

namespace tlt {

template <typename T>
__global__ void embed_rows_k(int M, int h, int V, const int32_t* __restrict__ tokens, const T* __restrict__ embed,
                             float* __restrict__ x) {
    int r = blockIdx.x;
    int t = tokens[r];
    bool ok = t >= 0 && t < V;
    const T* e = embed + (int64_t)(ok ? t : 0) * h;
    for (int c = threadIdx.x; c < h; c += blockDim.x) x[(int64_t)r * h + c] = ok ? to_float(e[c]) : 0.f;
}

// `add` (optional, [rows][h] in TA = T or float, no row_map then): the residual stream takes x[r] += add[r]
// first -- the output projection leaves its product there instead of read-modify-writing x itself.
template <typename T, typename TA>
__global__ __launch_bounds__(256) void rmsnorm_k(int h, float* __restrict__ x, const T* __restrict__ gamma,
                                                 float eps, T* __restrict__ out, const int32_t* __restrict__ row_map,
                                                 const TA* __restrict__ add, float* __restrict__ zero, int zero_n, int n_add,
                                                 int64_t add_stride, int assign) {
    __shared__ float red[4];
    int r = blockIdx.x;
    if (zero)
        for (int c = threadIdx.x; c < zero_n; c += 256) zero[(int64_t)r * zero_n + c] = 0.f;
    int64_t src = row_map ? row_map[r] : r;
    T* o = out + (int64_t)r * h;
    if (src < 0) {
        for (int c = threadIdx.x; c < h; c += 256) o[c] = from_float<T>(0.f);
        return;
    }
    float* xr = x + src * h;
    float ss = 0.f;
    for (int c = threadIdx.x; c < h; c += 256) {
        float v = (add && assign) ? 0.f : xr[c];
        if (add) {   // (each element is read, updated and later re-read by the same thread)
            for (int k = 0; k < n_add; ++k) v += to_float(add[k * add_stride + src * h + c]);
            xr[c] = v;
        }
        ss += v * v;
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = red[0] + red[1] + red[2] + red[3];
    float inv = 1.0f / sqrtf(tot / (float)h + eps);
    for (int c = threadIdx.x; c < h; c += 256) o[c] = from_float<T>(xr[c] * inv * to_float(gamma[c]));
}

// Same, for h % 4 == 0 and h <= 1024 * NK: the row is read once with 16-byte loads and stays in
// registers (NK float4 per thread) between the reduction and the scaling.
template <typename T, int NK, typename TA, int NB = 4, int NTHR = 256>   // NB: slices of `add` whose loads are issued together
__global__ __launch_bounds__(NTHR) void rmsnorm_vec_k(int h, float* __restrict__ x, const T* __restrict__ gamma,
                                                     float eps, T* __restrict__ out, const int32_t* __restrict__ row_map,
                                                     const TA* __restrict__ add, float* __restrict__ zero, int zero_n, int n_add,
                                                     int64_t add_stride, int assign) {
    __shared__ float red[NTHR / 64];
    const int r = blockIdx.x, h4 = h >> 2;
    if (zero)   // row r of a second buffer cleared on the way (zero_n % 4 == 0, 16-byte aligned: the launcher checks)
        for (int c = threadIdx.x; c < (zero_n >> 2); c += NTHR)
            ((float4*)(zero + (int64_t)r * zero_n))[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    const int64_t src = row_map ? row_map[r] : r;
    T* o = out + (int64_t)r * h;
    float4 v[NK];
    float ss = 0.f;
    if (src >= 0) {
        float4* xr = (float4*)(x + src * h);
#pragma unroll
        for (int k = 0; k < NK; ++k) {
            const int c = threadIdx.x + k * NTHR;
            v[k] = (c < h4 && !(add && assign)) ? xr[c] : make_float4(0.f, 0.f, 0.f, 0.f);
            if (add && c < h4) {
                const TA* a = add + src * h + 4 * c;
                if constexpr (sizeof(TA) == 2) {
                    const uint2 pk = *(const uint2*)a;
                    v[k].x += __uint_as_float(pk.x << 16);
                    v[k].y += __uint_as_float(pk.x & 0xffff0000u);
                    v[k].z += __uint_as_float(pk.y << 16);
                    v[k].w += __uint_as_float(pk.y & 0xffff0000u);
                } else {
                    // partial products, summed in their fixed order; the loads of up to four slices are issued
                    // together (one after the other they would each expose a memory latency)
                    for (int j0 = 0; j0 < n_add; j0 += NB) {
                        float4 av[NB];
#pragma unroll
                        for (int u = 0; u < NB; ++u)
                            av[u] = j0 + u < n_add ? *(const float4*)(a + (j0 + u) * add_stride) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                        for (int u = 0; u < NB; ++u) {
                            v[k].x += av[u].x; v[k].y += av[u].y; v[k].z += av[u].z; v[k].w += av[u].w;
                        }
                    }
                }
                xr[c] = v[k];
            }
            ss += v[k].x * v[k].x + v[k].y * v[k].y + v[k].z * v[k].z + v[k].w * v[k].w;
        }
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < NTHR / 64; ++w) tot += red[w];
    const float inv = src >= 0 ? 1.0f / sqrtf(tot / (float)h + eps) : 0.f;
#pragma unroll
    for (int k = 0; k < NK; ++k) {
        const int c = threadIdx.x + k * NTHR;
        if (c >= h4) continue;
        const T* g = gamma + 4 * c;
        float y[4] = {v[k].x * inv * to_float(g[0]), v[k].y * inv * to_float(g[1]), v[k].z * inv * to_float(g[2]),
                      v[k].w * inv * to_float(g[3])};
        if (src < 0) y[0] = y[1] = y[2] = y[3] = 0.f;
        if constexpr (sizeof(T) == 2) {
            *(uint2*)(o + 4 * c) = make_uint2(pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]));
        } else {
            *(float4*)(o + 4 * c) = make_float4(y[0], y[1], y[2], y[3]);
        }
    }
}

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
template <typename T>
union Piece {   // 16 bytes of T
    u32x4_t v;
    T e[16 / sizeof(T)];
    __device__ Piece() {}
};

// One workgroup per row.  Angles are formed in double (positions reach 32K, where an fp32 product
// pos * inv_freq already carries ~1e-3 rad of rounding), once per (row, pair index), then reused by
// every head.  q is rotated in place; k is rotated and stored with v at the row's cache slot.  An
// optional projection bias is added first (to q, k and v).
template <typename T, bool SRC32>   // SRC32: the projection arrives as fp32 partial products (its own instance: it needs many more registers)
__global__ __launch_bounds__(256) void rope_kv_write_k(Rows rows, KVLayer kv, T* __restrict__ qkv, int n_q_heads,
                                                       float theta, const T* __restrict__ bias,
                                                       const float* __restrict__ src32, int n_src, int64_t src_stride) {
    extern __shared__ float cs[];  // [d/2] cos, [d/2] sin
    const int d = kv.d, half = d >> 1;
    int r = blockIdx.x;
    int b = r / rows.n, i = r - b * rows.n;
    if (rows.n_valid && i >= rows.n_valid[b]) return;
    int ctx = kv.seq_len[b];
    int pos = ctx + rows.pos_base + (rows.pos_off ? rows.pos_off[r] : rows.pos_stride * i);
    int slot = ctx + rows.slot_base + i;
    const int qkv_dim = (n_q_heads + 2 * kv.n_kv) * d;
    T* row = qkv + (int64_t)r * qkv_dim;
    // src32 (optional): the projection's product still in fp32 (a split-K GEMM accumulated it there);
    // q then goes to `qkv` in T for the attention kernel, exactly as when it is rotated in place
    const float* row32 = SRC32 ? src32 + (int64_t)r * qkv_dim : nullptr;
    auto load_piece = [&](int elem, Piece<T>& out) {   // VEC consecutive elements of the row, as T
        if constexpr (SRC32) {
#pragma unroll
            for (int k = 0; k < 16 / (int)sizeof(T); k += 4) {
                float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
                for (int j0 = 0; j0 < n_src; j0 += 8) {   // partial products of a split projection, in their fixed order
                    float4 g[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        g[u] = j0 + u < n_src ? *(const float4*)(row32 + (j0 + u) * src_stride + elem + k) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        f.x += g[u].x; f.y += g[u].y; f.z += g[u].z; f.w += g[u].w;
                    }
                }
                out.e[k] = from_float<T>(f.x);
                out.e[k + 1] = from_float<T>(f.y);
                out.e[k + 2] = from_float<T>(f.z);
                out.e[k + 3] = from_float<T>(f.w);
            }
        } else {
            out.v = *(const u32x4_t*)(row + elem);
        }
    };
    // both halves of a rotation pair at once: with partial products every slice's loads for the two
    // pieces are issued together (one memory latency instead of one per piece and slice batch)
    auto load_pair = [&](int elem_lo, int elem_hi, Piece<T>& lo, Piece<T>& hi) {
        if constexpr (!SRC32) {
            lo.v = *(const u32x4_t*)(row + elem_lo);
            hi.v = *(const u32x4_t*)(row + elem_hi);
            return;
        }
        constexpr int NQ = 16 / (int)sizeof(T) / 4;   // float4 per piece
        float4 f[2][NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q) f[0][q] = f[1][q] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int j0 = 0; j0 < n_src; j0 += 8) {   // partial products of a split projection, in their fixed order
            float4 g[2][NQ][8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const bool on = j0 + u < n_src;
                    g[0][q][u] = on ? *(const float4*)(row32 + (j0 + u) * src_stride + elem_lo + 4 * q) : make_float4(0.f, 0.f, 0.f, 0.f);
                    g[1][q][u] = on ? *(const float4*)(row32 + (j0 + u) * src_stride + elem_hi + 4 * q) : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int q = 0; q < NQ; ++q)
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        f[hh][q].x += g[hh][q][u].x; f[hh][q].y += g[hh][q][u].y;
                        f[hh][q].z += g[hh][q][u].z; f[hh][q].w += g[hh][q][u].w;
                    }
        }
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            lo.e[4 * q] = from_float<T>(f[0][q].x); lo.e[4 * q + 1] = from_float<T>(f[0][q].y);
            lo.e[4 * q + 2] = from_float<T>(f[0][q].z); lo.e[4 * q + 3] = from_float<T>(f[0][q].w);
            hi.e[4 * q] = from_float<T>(f[1][q].x); hi.e[4 * q + 1] = from_float<T>(f[1][q].y);
            hi.e[4 * q + 2] = from_float<T>(f[1][q].z); hi.e[4 * q + 3] = from_float<T>(f[1][q].w);
        }
    };
    PageRef pr;
    bool have = locate(kv.block_table, kv.max_pages, kv.n_pages, kv.page_size, b, slot, pr);
    T* kc = (T*)kv.k;
    T* vc = (T*)kv.v;
    // 16-byte pieces: VEC consecutive pair indices j of one head per thread, both halves of each pair
    constexpr int VEC = 16 / sizeof(T);
    const int cph = half / VEC;   // pieces per half head
    const int n_piece = (n_q_heads + kv.n_kv) * cph;
    // the first piece's loads fly while the angles are computed
    Piece<T> lo0, hi0;
    lo0.v = u32x4_t{0u, 0u, 0u, 0u};
    hi0.v = lo0.v;
    if ((int)threadIdx.x < n_piece) {
        const int hd = threadIdx.x / cph, j0 = (threadIdx.x - hd * cph) * VEC;
        load_pair(hd * d + j0, hd * d + half + j0, lo0, hi0);
    }
    for (int j = threadIdx.x; j < half; j += 256) {
        double inv_freq = pow((double)theta, -2.0 * (double)j / (double)d);
        double sn, c;
        sincos((double)pos * inv_freq, &sn, &c);
        cs[j] = (float)c;
        cs[half + j] = (float)sn;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < n_piece; e += 256) {
        const int hd = e / cph, j0 = (e - hd * cph) * VEC;
        T* p = row + (int64_t)hd * d;
        Piece<T> lo, hi, blo, bhi;
        lo.v = lo0.v;
        hi.v = hi0.v;
        if (e != (int)threadIdx.x) load_pair(hd * d + j0, hd * d + half + j0, lo, hi);
        if (bias) {
            blo.v = *(const u32x4_t*)(bias + hd * d + j0);
            bhi.v = *(const u32x4_t*)(bias + hd * d + half + j0);
        }
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            float x1 = to_float(lo.e[k]), x2 = to_float(hi.e[k]);
            if (bias) {
                x1 += to_float(blo.e[k]);
                x2 += to_float(bhi.e[k]);
            }
            const float c = cs[j0 + k], sn = cs[half + j0 + k];
            lo.e[k] = from_float<T>(x1 * c - x2 * sn);
            hi.e[k] = from_float<T>(x2 * c + x1 * sn);
        }
        if (hd < n_q_heads) {
            *(u32x4_t*)(p + j0) = lo.v;
            *(u32x4_t*)(p + half + j0) = hi.v;
        } else if (have) {
            const int kh = hd - n_q_heads;
            const int64_t o = ((pr.page * kv.n_kv + kh) * kv.page_size + pr.row) * d;
            *(u32x4_t*)(kc + o + j0) = lo.v;
            *(u32x4_t*)(kc + o + half + j0) = hi.v;
        }
    }
    if (have) {
        const int v0 = (n_q_heads + kv.n_kv) * d;
        const T* vbias = bias ? bias + (int64_t)(n_q_heads + kv.n_kv) * d : nullptr;
        for (int e = threadIdx.x; e < kv.n_kv * d / VEC; e += 256) {
            const int kh = e * VEC / d, j0 = e * VEC - kh * d;
            Piece<T> x, bb;
            load_piece(v0 + e * VEC, x);
            if (vbias) {
                bb.v = *(const u32x4_t*)(vbias + e * VEC);
#pragma unroll
                for (int k = 0; k < VEC; ++k) x.e[k] = from_float<T>(to_float(x.e[k]) + to_float(bb.e[k]));
            }
            *(u32x4_t*)(vc + ((pr.page * kv.n_kv + kh) * kv.page_size + pr.row) * d + j0) = x.v;
        }
    }
}

template <typename T>
__global__ void swiglu_k(int64_t count, const T* __restrict__ g, const T* __restrict__ u, T* __restrict__ out) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) {
        float a = to_float(g[i]);
        out[i] = from_float<T>(a / (1.0f + expf(-a)) * to_float(u[i]));
    }
}

template <typename T>
__global__ void draft_input_k(int n, int h, int V, const int32_t* __restrict__ tok, const int32_t* __restrict__ src,
                              const int32_t* __restrict__ n_valid, int src_seq_stride, int64_t hidden_rows,
                              const float* __restrict__ hidden, const T* __restrict__ embed, T* __restrict__ xin) {
    int r = blockIdx.x;
    int b = r / n, i = r - b * n;
    int t = tok[r];
    int64_t sr = src[r];
    bool ok = t >= 0 && t < V && sr >= 0 && (!n_valid || i < n_valid[b]);
    if (ok && src_seq_stride > 0) {
        ok = sr < src_seq_stride;
        sr += (int64_t)b * src_seq_stride;
    }
    ok = ok && sr < hidden_rows;
    T* o = xin + (int64_t)r * 2 * h;
    for (int c = threadIdx.x; c < h; c += blockDim.x) {
        o[c] = ok ? embed[(int64_t)t * h + c] : from_float<T>(0.f);
        o[h + c] = ok ? from_float<T>(hidden[sr * h + c]) : from_float<T>(0.f);
    }
}

__global__ void add_i32_k(int n, int32_t* dst, const int32_t* a, int add_const) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] += (a ? a[i] : 0) + add_const;
}

__global__ void zero_f32_k(int64_t count, float4* __restrict__ dst) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) dst[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

__global__ void copy_f32_k(int64_t count, const float4* __restrict__ src, float4* __restrict__ dst) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) dst[i] = src[i];
}

// dst row (r / n) * dst_seq_stride + dst_base + r % n  <-  src row r   (h floats, h % 4 == 0)
__global__ void scatter_rows_k(int n, int h4, const float4* __restrict__ src, float4* __restrict__ dst, int dst_seq_stride,
                               int dst_base) {
    int r = blockIdx.x;
    int64_t d = (int64_t)(r / n) * dst_seq_stride + dst_base + (r % n);
    for (int c = threadIdx.x; c < h4; c += blockDim.x) dst[d * h4 + c] = src[(int64_t)r * h4 + c];
}

// Per sequence: last active row of x [B][n][h] -> dst row b * dst_seq_stride; nothing when n_valid[b] <= 0.
__global__ void gather_last_rows_k(int n, int h4, const int32_t* __restrict__ n_valid, const float4* __restrict__ src,
                                   float4* __restrict__ dst, int dst_seq_stride) {
    int b = blockIdx.x;
    int nv = n_valid ? n_valid[b] : n;
    if (nv > n) nv = n;
    if (nv <= 0) return;
    int64_t sr = (int64_t)b * n + nv - 1, d = (int64_t)b * dst_seq_stride;
    for (int c = threadIdx.x; c < h4; c += blockDim.x) dst[d * h4 + c] = src[sr * h4 + c];
}

__global__ void iota_scaled_k(int n, int32_t* out, int scale) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = i * scale;
}

#define DISPATCH_T(dtype, ...)              \
    if ((dtype) == F32) {                   \
        using T = float;                    \
        __VA_ARGS__;                        \
    } else {                                \
        using T = bf16;                     \
        __VA_ARGS__;                        \
    }

hipError_t embed_rows(hipStream_t s, int dtype, int M, int h, int V, const int32_t* tokens, const void* embed, float* x) {
    if (M <= 0) return hipSuccess;
    DISPATCH_T(dtype, hipLaunchKernelGGL(embed_rows_k<T>, dim3(M), dim3(256), 0, s, M, h, V, tokens, (const T*)embed, x));
    return hipGetLastError();
}

template <typename T, typename TA>
static void rmsnorm_launch_t(hipStream_t s, int M, int h, float* x, const void* gamma, float eps, void* out,
                             const int32_t* row_map, const void* add, float* zero, int zero_n, int n_add, bool assign) {
    const int64_t add_stride = (int64_t)M * h;
    const bool vec_ok = h % 4 == 0 && (((uintptr_t)x | (uintptr_t)add | (uintptr_t)zero) & 15) == 0 && zero_n % 4 == 0;
    if (vec_ok && h <= 4096 && add && n_add > 4 && sizeof(TA) == 4)
        // many slices (few rows, so few workgroups): one 16-byte position per thread and all its slices' loads in
        // flight at once
        hipLaunchKernelGGL((rmsnorm_vec_k<T, 1, TA, 12, 1024>), dim3(M), dim3(1024), 0, s, h, x, (const T*)gamma, eps, (T*)out,
                           row_map, (const TA*)add, zero, zero_n, n_add, add_stride, (int)assign);
    else if (vec_ok && h <= 4096)
        hipLaunchKernelGGL((rmsnorm_vec_k<T, 4, TA>), dim3(M), dim3(256), 0, s, h, x, (const T*)gamma, eps, (T*)out, row_map,
                           (const TA*)add, zero, zero_n, n_add, add_stride, (int)assign);
    else if (vec_ok && h <= 8192)   // (the 32B and 70B widths)
        hipLaunchKernelGGL((rmsnorm_vec_k<T, 8, TA>), dim3(M), dim3(256), 0, s, h, x, (const T*)gamma, eps, (T*)out, row_map,
                           (const TA*)add, zero, zero_n, n_add, add_stride, (int)assign);
    else
        hipLaunchKernelGGL((rmsnorm_k<T, TA>), dim3(M), dim3(256), 0, s, h, x, (const T*)gamma, eps, (T*)out, row_map,
                           (const TA*)add, zero, zero_n, n_add, add_stride, (int)assign);
}

static hipError_t rmsnorm_launch(hipStream_t s, int dtype, int M, int h, float* x, const void* gamma, float eps, void* out,
                                 const int32_t* row_map, const void* add, bool add_f32 = false, float* zero = nullptr,
                                 int zero_n = 0, int n_add = 1, bool assign = false) {
    if (M <= 0) return hipSuccess;
    if (add && !add_f32 && dtype != F32 && n_add != 1) return hipErrorInvalidValue;   // several addends: fp32 partial products only
    if (dtype == F32) rmsnorm_launch_t<float, float>(s, M, h, x, gamma, eps, out, row_map, add, zero, zero_n, n_add, assign);
    else if (add_f32) rmsnorm_launch_t<bf16, float>(s, M, h, x, gamma, eps, out, row_map, add, zero, zero_n, n_add, assign);
    else rmsnorm_launch_t<bf16, bf16>(s, M, h, x, gamma, eps, out, row_map, add, zero, zero_n, n_add, assign);
    return hipGetLastError();
}

hipError_t rmsnorm(hipStream_t s, int dtype, int M, int h, const float* x, const void* gamma, float eps, void* out,
                   const int32_t* row_map, float* zero, int zero_n) {
    return rmsnorm_launch(s, dtype, M, h, const_cast<float*>(x), gamma, eps, out, row_map, nullptr, false, zero, zero_n);   // x is only read
}

hipError_t rmsnorm_add(hipStream_t s, int dtype, int M, int h, float* x, const void* add, bool add_f32, const void* gamma,
                       float eps, void* out, int n_add, bool assign) {
    return rmsnorm_launch(s, dtype, M, h, x, gamma, eps, out, nullptr, add, add_f32, nullptr, 0, n_add, assign);
}

__global__ void add_parts_k(int64_t count4, float4* __restrict__ x, const float4* __restrict__ parts, int n_parts, int assign) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < count4; i += stride) {
        float4 v = assign ? make_float4(0.f, 0.f, 0.f, 0.f) : x[i];
        for (int k0 = 0; k0 < n_parts; k0 += 4) {
            float4 p[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) p[u] = k0 + u < n_parts ? parts[(k0 + u) * count4 + i] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                v.x += p[u].x; v.y += p[u].y; v.z += p[u].z; v.w += p[u].w;
            }
        }
        x[i] = v;
    }
}

hipError_t add_parts(hipStream_t s, int64_t count, float* x, const float* parts, int n_parts, bool assign) {
    if (count <= 0 || n_parts <= 0) return hipSuccess;
    const int64_t c4 = count / 4;
    int blocks = (int)((c4 + 255) / 256);
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(add_parts_k, dim3(blocks), dim3(256), 0, s, c4, (float4*)x, (const float4*)parts, n_parts, (int)assign);
    return hipGetLastError();
}

hipError_t rope_kv_write(hipStream_t s, int dtype, const Rows& rows, const KVLayer& kv, void* qkv, int n_q_heads,
                         float theta, const void* bias, const float* src32, int n_src) {
    int M = rows.B * rows.n;
    if (M <= 0) return hipSuccess;
    // the kernel moves 16-byte pieces: rows of qkv and of the cache are multiples of 16 bytes by the
    // configuration check, the bases must be aligned as well
    if ((((uintptr_t)qkv | (uintptr_t)bias | (uintptr_t)kv.k | (uintptr_t)kv.v | (uintptr_t)src32) & 15) != 0)
        return hipErrorInvalidValue;
    size_t lds = sizeof(float) * kv.d;
    const int64_t src_stride = (int64_t)M * (n_q_heads + 2 * kv.n_kv) * kv.d;
    if (src32) {
        DISPATCH_T(dtype, hipLaunchKernelGGL((rope_kv_write_k<T, true>), dim3(M), dim3(256), lds, s, rows, kv, (T*)qkv, n_q_heads,
                                             theta, (const T*)bias, src32, n_src, src_stride));
    } else {
        DISPATCH_T(dtype, hipLaunchKernelGGL((rope_kv_write_k<T, false>), dim3(M), dim3(256), lds, s, rows, kv, (T*)qkv, n_q_heads,
                                             theta, (const T*)bias, src32, n_src, src_stride));
    }
    return hipGetLastError();
}

hipError_t swiglu(hipStream_t s, int dtype, int64_t count, const void* g, const void* u, void* out) {
    if (count <= 0) return hipSuccess;
    int blocks = (int)((count + 255) / 256);
    if (blocks > 16384) blocks = 16384;
    DISPATCH_T(dtype, hipLaunchKernelGGL(swiglu_k<T>, dim3(blocks), dim3(256), 0, s, count, (const T*)g, (const T*)u, (T*)out));
    return hipGetLastError();
}

hipError_t draft_input(hipStream_t s, int dtype, int B, int n, int h, int V, const int32_t* tok, const int32_t* src,
                       const int32_t* n_valid, int src_seq_stride, int64_t hidden_rows, const float* hidden,
                       const void* embed, void* xin) {
    if (B * n <= 0) return hipSuccess;
    DISPATCH_T(dtype, hipLaunchKernelGGL(draft_input_k<T>, dim3(B * n), dim3(256), 0, s, n, h, V, tok, src, n_valid,
                                         src_seq_stride, hidden_rows, hidden, (const T*)embed, (T*)xin));
    return hipGetLastError();
}

hipError_t add_i32(hipStream_t s, int n, int32_t* dst, const int32_t* a, int add_const) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(add_i32_k, dim3((n + 255) / 256), dim3(256), 0, s, n, dst, a, add_const);
    return hipGetLastError();
}

hipError_t copy_f32(hipStream_t s, int64_t count, const float* src, float* dst) {
    if (count <= 0) return hipSuccess;
    int64_t c4 = count / 4;  // callers pass multiples of 4 floats (hidden sizes are)
    int blocks = (int)((c4 + 255) / 256);
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(copy_f32_k, dim3(blocks), dim3(256), 0, s, c4, (const float4*)src, (float4*)dst);
    return hipGetLastError();
}

hipError_t zero_f32(hipStream_t s, int64_t count, float* dst) {
    if (count <= 0) return hipSuccess;
    int64_t c4 = count / 4;  // callers pass multiples of 4 floats
    int blocks = (int)((c4 + 255) / 256);
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(zero_f32_k, dim3(blocks), dim3(256), 0, s, c4, (float4*)dst);
    return hipGetLastError();
}

hipError_t scatter_rows(hipStream_t s, int R, int n, int h, const float* src, float* dst, int dst_seq_stride, int dst_base) {
    if (R <= 0) return hipSuccess;
    hipLaunchKernelGGL(scatter_rows_k, dim3(R), dim3(256), 0, s, n, h / 4, (const float4*)src, (float4*)dst, dst_seq_stride,
                       dst_base);
    return hipGetLastError();
}

hipError_t gather_last_rows(hipStream_t s, int B, int n, int h, const int32_t* n_valid, const float* src, float* dst,
                            int dst_seq_stride) {
    if (B <= 0) return hipSuccess;
    hipLaunchKernelGGL(gather_last_rows_k, dim3(B), dim3(256), 0, s, n, h / 4, n_valid, (const float4*)src, (float4*)dst,
                       dst_seq_stride);
    return hipGetLastError();
}

hipError_t iota_scaled(hipStream_t s, int n, int32_t* out, int scale) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(iota_scaled_k, dim3((n + 255) / 256), dim3(256), 0, s, n, out, scale);
    return hipGetLastError();
}

}  // namespace tlt
