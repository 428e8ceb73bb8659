// Tree-masked grouped-query attention over the paged KV cache.
//
// Every active row (b, i) of every query head attends to the seq_len[b] committed cache rows and to
// the provisional rows seq_len[b] + j whose bit j is set in the row's mask (ancestors-or-self of a
// tree node; a causal prefix for chains).
//
// impl 0 ("wave-per-row"): one wavefront per (row, query head); lanes own keys for the score pass
//   and head dimensions for the value pass; online softmax across 64-key tiles.  Any dtype, any
//   head_dim that is a multiple of 64 up to 256.  Used for fp32 mode and as a cross-check.
#include "dev_common.h"
#include "kernels.h"

namespace tlt {

__device__ __forceinline__ bool region_visible(const Rows& rows, int r, int i, int j) {
    if (j >= rows.n_region) return false;
    if (!rows.mask) return j <= i;
    uint64_t w = rows.mask[(int64_t)r * rows.mask_words + (j >> 6)];
    return (w >> (j & 63)) & 1ull;
}

template <typename T>
__global__ __launch_bounds__(64) void attn_wave_per_row_k(Rows rows, KVLayer kv, const T* __restrict__ qkv,
                                                          T* __restrict__ out, int n_q_heads, float scale) {
    __shared__ float q_s[256];
    __shared__ float p_s[64];
    __shared__ int64_t base_s[64];
    const int lane = threadIdx.x;
    const int i = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
    const int r = b * rows.n + i;
    const int d = kv.d;
    const int G = n_q_heads / kv.n_kv, kh = hq / G;
    const int qkv_dim = (n_q_heads + 2 * kv.n_kv) * d;
    T* o = out + ((int64_t)r * n_q_heads + hq) * d;
    if (rows.n_valid && i >= rows.n_valid[b]) {
        for (int c = lane; c < d; c += 64) o[c] = from_float<T>(0.f);
        return;
    }
    const int ctx = kv.seq_len[b];
    const int total = ctx + rows.n_region;
    for (int c = lane; c < d; c += 64) q_s[c] = to_float(qkv[(int64_t)r * qkv_dim + hq * d + c]) * scale;
    __syncthreads();
    const T* kc = (const T*)kv.k;
    const T* vc = (const T*)kv.v;
    float m = -INFINITY, l = 0.f;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int t0 = 0; t0 < total; t0 += 64) {
        const int key = t0 + lane;
        bool vis = key < total && (key < ctx || region_visible(rows, r, i, key - ctx));
        PageRef pr;
        int64_t base = -1;
        if (vis && locate(kv.block_table, kv.max_pages, kv.n_pages, kv.page_size, b, key, pr))
            base = ((pr.page * kv.n_kv + kh) * kv.page_size + pr.row) * d;
        vis = base >= 0;
        float s = -INFINITY;
        if (vis) {
            s = 0.f;
            for (int c = 0; c < d; ++c) s = fmaf(q_s[c], to_float(kc[base + c]), s);
        }
        float tm = wave_max(s);
        float m_new = fmaxf(m, tm);
        if (m_new == -INFINITY) continue;  // nothing visible so far (uniform across the wave)
        float corr = expf(m - m_new);      // exp(-inf) = 0 on the first visible tile
        float p = vis ? expf(s - m_new) : 0.f;
        l = l * corr + wave_sum(p);
        m = m_new;
        __syncthreads();
        p_s[lane] = p;
        base_s[lane] = base;
        __syncthreads();
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[t] *= corr;
        const int nk = min(64, total - t0);
        for (int k = 0; k < nk; ++k) {
            float pk = p_s[k];
            if (pk == 0.f) continue;
            int64_t bk = base_s[k];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                int c = lane + 64 * t;
                if (c < d) acc[t] = fmaf(pk, to_float(vc[bk + c]), acc[t]);
            }
        }
    }
    float inv = l > 0.f ? 1.0f / l : 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        int c = lane + 64 * t;
        if (c < d) o[c] = from_float<T>(acc[t] * inv);
    }
}

size_t attention_workspace_bytes(int B, int n, int n_q_heads, int n_kv_heads, int d, int max_ctx) {
    (void)B; (void)n; (void)n_q_heads; (void)n_kv_heads; (void)d; (void)max_ctx;
    return 256;
}

hipError_t attention(hipStream_t s, int dtype, const Rows& rows, const KVLayer& kv, const void* qkv, void* out,
                     int n_q_heads, void* ws, size_t ws_bytes, int impl) {
    (void)ws; (void)ws_bytes; (void)impl;
    if (rows.B * rows.n <= 0) return hipSuccess;
    if (kv.d % 64 != 0 || kv.d > 256) return hipErrorInvalidValue;
    float scale = 1.0f / sqrtf((float)kv.d);
    dim3 grid(rows.n, n_q_heads, rows.B), block(64);
    if (dtype == F32)
        hipLaunchKernelGGL(attn_wave_per_row_k<float>, grid, block, 0, s, rows, kv, (const float*)qkv, (float*)out,
                           n_q_heads, scale);
    else
        hipLaunchKernelGGL(attn_wave_per_row_k<bf16>, grid, block, 0, s, rows, kv, (const bf16*)qkv, (bf16*)out,
                           n_q_heads, scale);
    return hipGetLastError();
}

}  // namespace tlt
