// Vocabulary-row reductions (argmax, log-softmax + top-k), the drafter's tree bookkeeping
// (candidate pool, frontier selection, pruning), the acceptance rules and the KV-cache commit.
//
// Ordering rule used wherever a "best" element is picked: larger value first, lower index on ties.
#include "dev_common.h"
#include "kernels.h"

namespace tlt {

// ------------------------------------------------------------------------------------------------
// block-wide helpers (256 threads = 4 waves)
__device__ __forceinline__ void block_best(float& v, int& i, float* sv, int* si) {
    wave_best(v, i);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
        sv[threadIdx.x >> 6] = v;
        si[threadIdx.x >> 6] = i;
    }
    __syncthreads();
    v = sv[0];
    i = si[0];
#pragma unroll
    for (int w = 1; w < 4; ++w)
        if (better(sv[w], si[w], v, i)) {
            v = sv[w];
            i = si[w];
        }
}

// (NW waves per workgroup; the partial results are combined in wave order, so a float sum is
// reproducible from run to run)
template <int NW = 4>
__device__ __forceinline__ float block_sum_f(float v, float* sv) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sv[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = sv[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) r += sv[w];
    return r;
}

template <int NW = 4>
__device__ __forceinline__ float block_max_f(float v, float* sv) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sv[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = sv[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) r = fmaxf(r, sv[w]);
    return r;
}

template <int NW = 4>
__device__ __forceinline__ unsigned long long block_sum_u64(unsigned long long v, unsigned long long* sv) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sv[threadIdx.x >> 6] = v;
    __syncthreads();
    unsigned long long r = sv[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) r += sv[w];
    return r;
}

template <int NW = 4>
__device__ __forceinline__ double block_max_d(double v, double* sv) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sv[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = sv[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) r = fmax(r, sv[w]);
    return r;
}

// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void row_argmax_k(int V, const float* __restrict__ logits, int32_t* __restrict__ out) {
    __shared__ float sv[4];
    __shared__ int si[4];
    const float* row = logits + (int64_t)blockIdx.x * V;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    int j = threadIdx.x;
    if (V % 4 == 0 && ((uintptr_t)logits & 15) == 0) {   // 16 bytes per lane; a lane's indices still increase
        for (int q = threadIdx.x * 4; q < V; q += 1024) {
            const float4 x = *(const float4*)(row + q);
            if (x.x > bv || bi == 0x7fffffff) bv = x.x, bi = q;
            if (x.y > bv) bv = x.y, bi = q + 1;
            if (x.z > bv) bv = x.z, bi = q + 2;
            if (x.w > bv) bv = x.w, bi = q + 3;
        }
        j = V;
    }
    for (; j < V; j += 256) {
        float v = row[j];
        if (better(v, j, bv, bi)) {
            bv = v;
            bi = j;
        }
    }
    block_best(bv, bi, sv, si);
    if (threadIdx.x == 0) out[blockIdx.x] = bi == 0x7fffffff ? 0 : bi;
}

// The same over one segment of a row (grid: segments x rows), for when there are too few rows to fill the chip with
// one workgroup each: (value, index) of the segment's best entry, index 0x7fffffff for an empty segment; and the
// merge of a row's segments, one wave per row (lowest index on ties, as in the single pass).
__global__ __launch_bounds__(256) void row_argmax_seg_k(int V, int seg, int S, const float* __restrict__ logits,
                                                        float* __restrict__ pv, int32_t* __restrict__ pi) {
    __shared__ float sv[4];
    __shared__ int si[4];
    const int sg = blockIdx.x, r = blockIdx.y;
    const float* row = logits + (int64_t)r * V;
    const int lo = sg * seg, hi = min(V, lo + seg);   // seg % 4 == 0
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    int j = lo + threadIdx.x;
    if (V % 4 == 0 && ((uintptr_t)logits & 15) == 0) {
        for (int q = lo + threadIdx.x * 4; q < hi; q += 1024) {
            const float4 x = *(const float4*)(row + q);
            if (x.x > bv || bi == 0x7fffffff) bv = x.x, bi = q;
            if (x.y > bv) bv = x.y, bi = q + 1;
            if (x.z > bv) bv = x.z, bi = q + 2;
            if (x.w > bv) bv = x.w, bi = q + 3;
        }
        j = hi;
    }
    for (; j < hi; j += 256) {
        const float v = row[j];
        if (better(v, j, bv, bi)) {
            bv = v;
            bi = j;
        }
    }
    block_best(bv, bi, sv, si);
    if (threadIdx.x == 0) {
        pv[(int64_t)r * S + sg] = bv;
        pi[(int64_t)r * S + sg] = bi;
    }
}

__global__ __launch_bounds__(64) void row_argmax_merge_k(int S, const float* __restrict__ pv, const int32_t* __restrict__ pi,
                                                         int32_t* __restrict__ out) {
    const int r = blockIdx.x, lane = threadIdx.x;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int k = lane; k < S; k += 64) {
        const float v = pv[(int64_t)r * S + k];
        const int i = pi[(int64_t)r * S + k];
        if (i != 0x7fffffff && (bi == 0x7fffffff || better(v, i, bv, bi))) bv = v, bi = i;
    }
    wave_best(bv, bi);
    if (lane == 0) out[r] = bi == 0x7fffffff ? 0 : bi;
}

// (max, log-sum-exp) of every logits row: out[2r] = max_j l_j, out[2r+1] = max + log(sum_j exp(l_j - max)).
__global__ __launch_bounds__(256) void row_lse_k(int V, const float* __restrict__ logits, float* __restrict__ out) {
    __shared__ float sf[4];
    const float* row = logits + (int64_t)blockIdx.x * V;
    float m = -INFINITY;
    for (int j = threadIdx.x; j < V; j += 256) m = fmaxf(m, row[j]);
    m = block_max_f<4>(m, sf);
    float se = 0.f;
    for (int j = threadIdx.x; j < V; j += 256) se += expf(row[j] - m);
    se = block_sum_f<4>(se, sf);
    if (threadIdx.x == 0) {
        out[2 * (int64_t)blockIdx.x] = m;
        out[2 * (int64_t)blockIdx.x + 1] = m + logf(se);
    }
}

// Log-softmax statistics and the K best tokens of every logits row, in two kernels.
// (1) One wave per (row, segment of kTopkSeg logits): the segment is read once into registers, then
//     its max, its sum of exponentials and its K best entries in the (value desc, index asc) order
//     are written out.
// (2) One wave per row merges the segments: the K best of the union of the per-segment lists are
//     the K best of the row because the order is total.
constexpr int kTopkSeg = 2048;     // logits per wave: 32 per lane, held in registers
constexpr int kTopkPerLane = kTopkSeg / 64;

// One WAVE per segment, no LDS and no barriers.  A lane owns 32 logits (eight 16-byte pieces, so
// the wave's loads are fully coalesced) and keeps its two best in the (value desc, index asc) order.
// Each of the K rounds takes the best lane candidate of the wave (xor-shuffle reduction) and the
// winning lane moves on to its second candidate; only a lane that wins a third time has to rescan
// its registers, which on real logits almost never happens, and the wave skips that code unless
// some lane needs it.
template <bool VEC4>
__global__ __launch_bounds__(256) void row_topk_seg_k(int V, int K, int n_seg, const float* __restrict__ logits,
                                                      float* __restrict__ seg_stat, float* __restrict__ seg_val,
                                                      int32_t* __restrict__ seg_idx) {
    const int lane = threadIdx.x & 63;
    const int seg = blockIdx.x * 4 + (threadIdx.x >> 6), row = blockIdx.y;
    if (seg >= n_seg) return;  // wave-uniform
    const int j0 = seg * kTopkSeg;
    const float* src = logits + (int64_t)row * V;
    float v[kTopkPerLane];
    // element e of this lane has index j0 + (e / 4) * 256 + lane * 4 + (e % 4): increasing in e
#pragma unroll
    for (int c = 0; c < kTopkPerLane / 4; ++c) {
        const int j = j0 + c * 256 + lane * 4;
        if (VEC4) {
            float4 x = j + 3 < V ? *(const float4*)(src + j) : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            if (j + 3 >= V && j < V) {   // ragged end of the row
                x.x = src[j];
                x.y = j + 1 < V ? src[j + 1] : -INFINITY;
                x.z = j + 2 < V ? src[j + 2] : -INFINITY;
            }
            v[4 * c] = x.x, v[4 * c + 1] = x.y, v[4 * c + 2] = x.z, v[4 * c + 3] = x.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[4 * c + e] = j + e < V ? src[j + e] : -INFINITY;
        }
    }
    auto index_of = [&](int e) { return j0 + (e >> 2) * 256 + lane * 4 + (e & 3); };
    // local best two; indices of a lane increase with e, so strict '>' keeps the lower index on ties
    float b1 = -INFINITY, b2 = -INFINITY;
    int e1 = -1, e2 = -1;
#pragma unroll
    for (int e = 0; e < kTopkPerLane; ++e) {
        const float x = index_of(e) < V ? v[e] : -INFINITY;
        const bool valid = index_of(e) < V;
        if (valid && (e1 < 0 || x > b1)) {
            b2 = b1, e2 = e1;
            b1 = x, e1 = e;
        } else if (valid && (e2 < 0 || x > b2)) {
            b2 = x, e2 = e;
        }
    }
    // softmax statistics of the segment
    const float mx = wave_max(b1);
    float se = 0.f;
#pragma unroll
    for (int e = 0; e < kTopkPerLane; ++e) se += index_of(e) < V ? expf(v[e] - mx) : 0.f;
    se = wave_sum(se);
    const int64_t o = (int64_t)row * n_seg + seg;
    if (lane == 0) {
        seg_stat[2 * o] = mx;
        seg_stat[2 * o + 1] = se;
    }
    // K rounds
    float cv = b1;                                  // this lane's current candidate
    int ci = e1 >= 0 ? index_of(e1) : 0x7fffffff;
    int wins = 0;
    uint32_t taken = 0;                             // elements of this lane already emitted
    for (int k = 0; k < K; ++k) {
        float wv = cv;
        int wi = ci;
        wave_best(wv, wi);
        if (lane == 0) {
            const bool have = wi != 0x7fffffff;
            seg_val[o * K + k] = have ? wv : -INFINITY;
            seg_idx[o * K + k] = have ? wi : 0x7fffffff;
        }
        const bool won = wi != 0x7fffffff && wi == ci;
        if (won) {
            ++wins;
            const int e = ((ci - j0) >> 8) * 4 + ((ci - j0) & 3);
            taken |= 1u << e;
            if (wins == 1) {
                cv = b2;
                ci = e2 >= 0 ? index_of(e2) : 0x7fffffff;
            }
        }
        if (__any(won && wins >= 2)) {   // rare: rescan the registers for the best element not yet emitted
            if (won && wins >= 2) {
                float nv = -INFINITY;
                int ne = -1;
#pragma unroll
                for (int e = 0; e < kTopkPerLane; ++e) {
                    const bool ok = index_of(e) < V && !((taken >> e) & 1u);
                    if (ok && (ne < 0 || v[e] > nv)) {
                        nv = v[e];
                        ne = e;
                    }
                }
                cv = nv;
                ci = ne >= 0 ? index_of(ne) : 0x7fffffff;
            }
        }
    }
}

__global__ __launch_bounds__(64) void row_topk_merge_k(int K, int n_seg, const float* __restrict__ seg_stat,
                                                       const float* __restrict__ seg_val,
                                                       const int32_t* __restrict__ seg_idx, int32_t* __restrict__ tok,
                                                       float* __restrict__ logp) {
    const int row = blockIdx.x, lane = threadIdx.x;
    const int64_t o = (int64_t)row * n_seg;
    float mx = -INFINITY;
    for (int sgm = lane; sgm < n_seg; sgm += 64) mx = fmaxf(mx, seg_stat[2 * (o + sgm)]);
    mx = wave_max(mx);
    float se = 0.f;
    for (int sgm = lane; sgm < n_seg; sgm += 64) se += seg_stat[2 * (o + sgm) + 1] * expf(seg_stat[2 * (o + sgm)] - mx);
    se = wave_sum(se);
    const float lse = mx + logf(se);
    const int n_cand = n_seg * K;
    // the candidates are read once: a lane keeps up to kMergeRegs of them in registers (75 segments x 8 at the
    // 152064-token vocabulary: 10 per lane); longer lists are scanned from memory in every round
    constexpr int kMergeRegs = 20;
    const bool in_regs = n_cand <= 64 * kMergeRegs;
    float rv[kMergeRegs];
    int rj[kMergeRegs];
#pragma unroll
    for (int r = 0; r < kMergeRegs; ++r) {
        const int c = lane + 64 * r;
        const bool on = in_regs && c < n_cand;
        rv[r] = on ? seg_val[o * K + c] : -INFINITY;
        rj[r] = on ? seg_idx[o * K + c] : 0x7fffffff;
    }
    float pv = INFINITY;
    int pi = -1;
    for (int k = 0; k < K; ++k) {
        float cv = -INFINITY;
        int ci = 0x7fffffff;
        if (in_regs) {
#pragma unroll
            for (int r = 0; r < kMergeRegs; ++r) {
                const float v = rv[r];
                const int j = rj[r];
                const bool after = v < pv || (v == pv && j > pi);
                if (j != 0x7fffffff && after && better(v, j, cv, ci)) {
                    cv = v;
                    ci = j;
                }
            }
        } else {
            for (int c = lane; c < n_cand; c += 64) {
                float v = seg_val[o * K + c];
                int j = seg_idx[o * K + c];
                bool after = v < pv || (v == pv && j > pi);
                if (j != 0x7fffffff && after && better(v, j, cv, ci)) {
                    cv = v;
                    ci = j;
                }
            }
        }
        wave_best(cv, ci);
        pv = cv;
        pi = ci;
        if (lane == 0) {
            bool have = ci != 0x7fffffff;
            tok[(int64_t)row * K + k] = have ? ci : -1;
            logp[(int64_t)row * K + k] = have ? cv - lse : -INFINITY;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Drafter tree bookkeeping.  Feature-buffer rows per sequence: 0 = output of the entry holding the
// root token; 1 + (level-1)*K + r = output of frontier node r of `level`.  Provisional drafter
// cache row of that node = (level-1)*K + r past the committed length; masks are over those rows.
__global__ void draft_level0_k(int B, int K, const int32_t* __restrict__ top_tok, const float* __restrict__ top_logp,
                               DraftState st) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= B * K) return;
    int b = idx / K, r = idx - b * K;
    int64_t p = (int64_t)b * st.P + r;
    st.pool_token[p] = top_tok[idx];
    st.pool_score[p] = top_logp[idx];
    st.pool_parent[p] = -1;
    st.pool_depth[p] = 1;
    uint64_t m0 = r < 64 ? (1ull << r) : 0ull, m1 = r >= 64 ? (1ull << (r - 64)) : 0ull;
    st.pool_mask[2 * p] = m0;
    st.pool_mask[2 * p + 1] = m1;
    st.fr_token[idx] = top_tok[idx];
    st.fr_src[idx] = 0;
    st.fr_pool[idx] = r;
    st.fr_mask[2 * idx] = m0;
    st.fr_mask[2 * idx + 1] = m1;
}

__global__ __launch_bounds__(256) void draft_level_select_k(int K, int level, const int32_t* __restrict__ top_tok,
                                                            const float* __restrict__ top_logp, DraftState st) {
    __shared__ float sc[256];
    __shared__ int par_pool[16];
    __shared__ uint64_t par_mask[16][2];
    const int b = blockIdx.x, c = threadIdx.x, KK = K * K;
    if (c < K) {
        int pp = st.fr_pool[b * K + c];
        par_pool[c] = pp;
        par_mask[c][0] = st.pool_mask[2 * ((int64_t)b * st.P + pp)];
        par_mask[c][1] = st.pool_mask[2 * ((int64_t)b * st.P + pp) + 1];
    }
    __syncthreads();
    float score = -INFINITY;
    int token = -1, fr = 0;
    if (c < KK) {
        fr = c / K;
        int64_t src = ((int64_t)b * K + fr) * K + (c - fr * K);
        token = top_tok[src];
        score = st.pool_score[(int64_t)b * st.P + par_pool[fr]] + top_logp[src];
        int64_t p = (int64_t)b * st.P + K + (int64_t)(level - 1) * KK + c;
        st.pool_token[p] = token;
        st.pool_score[p] = score;
        st.pool_parent[p] = par_pool[fr];
        st.pool_depth[p] = level + 1;
    }
    sc[c] = score;
    __syncthreads();
    if (c < KK) {
        int rank = 0;
        for (int j = 0; j < KK; ++j) rank += better(sc[j], j, score, c) ? 1 : 0;
        if (rank < K) {
            int slot = level * K + rank;  // provisional row of this node when it runs at level+1
            uint64_t m0 = par_mask[fr][0] | (slot < 64 ? (1ull << slot) : 0ull);
            uint64_t m1 = par_mask[fr][1] | (slot >= 64 ? (1ull << (slot - 64)) : 0ull);
            int pool_idx = K + (level - 1) * KK + c;
            int64_t p = (int64_t)b * st.P + pool_idx;
            st.pool_mask[2 * p] = m0;
            st.pool_mask[2 * p + 1] = m1;
            int o = b * K + rank;
            st.fr_token[o] = token;
            st.fr_src[o] = 1 + (level - 1) * K + fr;
            st.fr_pool[o] = pool_idx;
            st.fr_mask[2 * o] = m0;
            st.fr_mask[2 * o + 1] = m1;
        }
    }
}

// One workgroup per sequence.  LDS: score[P], node_of[P] (node index or -1).
__global__ __launch_bounds__(256) void draft_prune_k(int pool_n, int n_tree, const int32_t* __restrict__ root_tokens,
                                                     const int32_t* __restrict__ new_tokens,
                                                     const int32_t* __restrict__ n_new, int new_stride, DraftState st, int32_t* __restrict__ token,
                                                     int32_t* __restrict__ parent, int32_t* __restrict__ depth,
                                                     uint64_t* __restrict__ anc_mask, float* __restrict__ score) {
    extern __shared__ float lds_f[];
    float* sc = lds_f;
    int* node_of = (int*)(lds_f + pool_n);
    int* tpar = node_of + pool_n;  // [n_tree] parent node of each tree node
    const int b = blockIdx.x;
    const int64_t pb = (int64_t)b * st.P;
    for (int i = threadIdx.x; i < pool_n; i += 256) sc[i] = st.pool_score[pb + i];
    __syncthreads();
    const int keep = n_tree - 1;
    for (int i = threadIdx.x; i < pool_n; i += 256) {
        float s = sc[i];
        int rank = 0;
        for (int j = 0; j < pool_n; ++j) rank += better(sc[j], j, s, i) ? 1 : 0;
        node_of[i] = rank < keep ? 0 : -1;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < pool_n; i += 256) {
        if (node_of[i] < 0) continue;
        int before = 0;
        for (int j = 0; j < i; ++j) before += node_of[j] >= 0 ? 1 : 0;  // flags are still 0 / -1 here
        sc[i] = __int_as_float(before + 1);                             // stash; scores are re-read from global
    }
    __syncthreads();
    for (int i = threadIdx.x; i < pool_n; i += 256)
        if (node_of[i] >= 0) node_of[i] = __float_as_int(sc[i]);
    __syncthreads();
    const int64_t tb = (int64_t)b * n_tree;
    if (threadIdx.x == 0) {
        int root = -1;  // explicit root, else the last token handed to the drafter's catch-up
        if (root_tokens) {
            root = root_tokens[b];
        } else if (new_tokens && n_new) {
            int nv = n_new[b] < new_stride ? n_new[b] : new_stride;
            if (nv >= 1) root = new_tokens[(int64_t)b * new_stride + nv - 1];
        }
        token[tb] = root;
        parent[tb] = -1;
        depth[tb] = 0;
        score[tb] = 0.f;
        tpar[0] = -1;
    }
    for (int i = threadIdx.x; i < pool_n; i += 256) {
        int nd = node_of[i];
        if (nd < 0) continue;
        int pp = st.pool_parent[pb + i];
        int pn = pp < 0 ? 0 : node_of[pp];
        token[tb + nd] = st.pool_token[pb + i];
        parent[tb + nd] = pn;
        depth[tb + nd] = st.pool_depth[pb + i];
        score[tb + nd] = st.pool_score[pb + i];
        tpar[nd] = pn;
    }
    __syncthreads();
    for (int nd = threadIdx.x; nd < n_tree; nd += 256) {
        uint64_t m = 0;
        int a = nd, guard = 0;
        while (a >= 0 && guard++ < 64) {
            m |= 1ull << a;
            a = tpar[a];
        }
        anc_mask[tb + nd] = m;
    }
}

__global__ void tree_finalize_k(int B, int n, const int32_t* __restrict__ parent, int32_t* __restrict__ depth,
                                uint64_t* __restrict__ anc_mask) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= B * n) return;
    int b = idx / n, i = idx - b * n;
    const int32_t* par = parent + (int64_t)b * n;
    uint64_t m = 0;
    int a = i, dep = -1, guard = 0;
    while (a >= 0 && a < n && guard++ < 64) {
        m |= 1ull << a;
        ++dep;
        int p = par[a];
        a = p < a ? p : -1;  // parents precede children; anything else ends the walk
    }
    depth[idx] = dep;
    anc_mask[idx] = m;
}

// ------------------------------------------------------------------------------------------------
// Sampled drafting on a static template: a node's children are consecutive draws without
// replacement from q = softmax(logits / temperature) at that node.  The draw is the integer rule
// of the sampling acceptance (which presupposes exactly this process): weights floor(q_j * 2^32)
// from the fp32 q that is handed to the caller, pick the first index whose running sum exceeds
// (U * sum) >> 32, then zero the picked weight.  Given q, every pick is exact integer arithmetic.
__global__ void tmpl_tree_init_k(int B, int n, TmplParents tp, const int32_t* __restrict__ root_tokens,
                                 const int32_t* __restrict__ new_tokens, const int32_t* __restrict__ n_new, int new_stride,
                                 int32_t* __restrict__ token, int32_t* __restrict__ parent, float* __restrict__ score) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= B * n) return;
    int b = idx / n, i = idx - b * n;
    parent[idx] = tp.parent[i];
    score[idx] = 0.f;
    if (i == 0) {
        int t = -1;
        if (root_tokens) {
            t = root_tokens[b];
        } else {
            int k = n_new[b];
            if (k >= 1 && k <= new_stride) t = new_tokens[(int64_t)b * new_stride + k - 1];
        }
        token[idx] = t;
    }
}

__global__ void tmpl_level_rows_k(int B, int n, TmplRows rows, const int32_t* __restrict__ token,
                                  int32_t* __restrict__ fr_token, int32_t* __restrict__ fr_src,
                                  uint64_t* __restrict__ fr_mask) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= B * rows.R) return;
    int b = idx / rows.R, r = idx - b * rows.R;
    fr_token[idx] = token[(int64_t)b * n + rows.node[r]];
    fr_src[idx] = rows.src[r];
    fr_mask[idx] = rows.mask[r];
}

__device__ __forceinline__ unsigned long long q_weight(float q) {
    return (unsigned long long)floor((double)q * 4294967296.0);
}

// One workgroup of 16 waves per (sequence, node).  Wave w owns the contiguous index range
// [w*Vw, (w+1)*Vw), Vw a multiple of 256, and walks it 256 elements at a time (four consecutive
// elements per lane: 16-byte accesses when the row allows), so a wave's weight total is the total of
// a contiguous range and the threshold search goes wave -> 256-element step -> lane -> element.
constexpr int kDrawThreads = 1024, kDrawWaves = kDrawThreads / 64;
constexpr int kDrawMaxSteps = 64;   // step totals kept per wave: covers vocabularies up to 16 * 64 * 256 = 262144

template <bool VEC4>
__device__ __forceinline__ void load4(const float* __restrict__ p, int idx, int V, float (&x)[4], float fill) {
    if (VEC4) {   // V % 4 == 0 and idx % 4 == 0: all four in range or none
        if (idx < V) {
            const float4 v = *(const float4*)(p + idx);
            x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
        } else {
            x[0] = x[1] = x[2] = x[3] = fill;
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = idx + e < V ? p[idx + e] : fill;
    }
}

// With few rows one workgroup per row leaves most of the chip idle, and a CU pulls a 600 KB row three times at the
// rate of its own load path (81 us per level at 40 rows).  Then the row is cut into G segments: softmax_part_k takes
// each segment's maximum and sum of exponentials, softmax_q_k combines them (in segment order), writes its segment
// of q and the integer weight total of each of its 256-element steps, and softmax_draw_k<.., PRE = true> starts from
// those totals and only draws.  Given q the draw is the same exact integer search either way.
template <bool VEC4>
__global__ __launch_bounds__(kDrawThreads) void softmax_part_k(int V, int G, int seg, float inv_temperature,
                                                               const float* __restrict__ logits, float* __restrict__ part) {
    __shared__ float sf[kDrawWaves];
    const int tid = threadIdx.x;
    const int row = blockIdx.x / G, g = blockIdx.x - row * G;
    const float* l = logits + (int64_t)row * V;
    const int lo = g * seg, hi = min(V, lo + seg);   // lo % 4 == 0; hi % 4 == 0 when VEC4
    float x[4];
    float m = -INFINITY;
    for (int i = lo + tid * 4; i < hi; i += kDrawThreads * 4) {
        load4<VEC4>(l, i, hi, x, -INFINITY);
        m = fmaxf(fmaxf(m, fmaxf(x[0], x[1])), fmaxf(x[2], x[3]));
    }
    m = block_max_f<kDrawWaves>(m, sf);
    float sum = 0.f;
    for (int i = lo + tid * 4; i < hi; i += kDrawThreads * 4) {
        load4<VEC4>(l, i, hi, x, -INFINITY);
#pragma unroll
        for (int e = 0; e < 4; ++e) sum += expf((x[e] - m) * inv_temperature);   // exp(-inf) = 0 past the end
    }
    sum = block_sum_f<kDrawWaves>(sum, sf);
    if (tid == 0) {
        part[2 * (int64_t)blockIdx.x] = m;
        part[2 * (int64_t)blockIdx.x + 1] = sum;
    }
}

template <bool VEC4>
__global__ __launch_bounds__(kDrawThreads) void softmax_q_k(int n, int V, int G, int seg, int n_steps_all, float inv_temperature,
                                                            TmplRows rows, const float* __restrict__ logits,
                                                            const float* __restrict__ part, float* __restrict__ q_out,
                                                            unsigned long long* __restrict__ step_tot) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = blockIdx.x / G, g = blockIdx.x - row * G;
    const int b = row / rows.R, r = row - b * rows.R;
    const float* l = logits + (int64_t)row * V;
    float* q = q_out + ((int64_t)b * n + rows.node[r]) * V;
    const float* pr = part + 2 * (int64_t)row * G;
    float m = -INFINITY;
    for (int k = 0; k < G; ++k) m = fmaxf(m, pr[2 * k]);
    float z = 0.f;
    for (int k = 0; k < G; ++k) z += pr[2 * k + 1] * expf((pr[2 * k] - m) * inv_temperature);
    const float inv = 1.0f / z;
    const int lo = g * seg, hi = min(V, lo + seg);
    float x[4];
    for (int i0 = lo + wave * 256; i0 < hi; i0 += kDrawWaves * 256) {
        const int i = i0 + lane * 4;
        load4<VEC4>(l, i, V, x, -INFINITY);
        float qv[4];
        unsigned long long mine = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            qv[e] = expf((x[e] - m) * inv_temperature) * inv;
            if (i + e < V) mine += q_weight(qv[e]);
        }
        if (VEC4) {
            if (i < V) *(float4*)(q + i) = make_float4(qv[0], qv[1], qv[2], qv[3]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (i + e < V) q[i + e] = qv[e];
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o, 64);
        if (lane == 0) step_tot[(int64_t)row * n_steps_all + (i0 >> 8)] = mine;
    }
}

template <bool VEC4, bool PRE = false>
__global__ __launch_bounds__(kDrawThreads) void softmax_draw_k(int n, int V, float inv_temperature, TmplRows rows,
                                                               const float* __restrict__ logits,
                                                               const uint32_t* __restrict__ u_draw,
                                                               int32_t* __restrict__ token, float* __restrict__ q_out,
                                                               const unsigned long long* __restrict__ step_tot,
                                                               int n_steps_all) {
    __shared__ float sf[kDrawWaves];
    __shared__ unsigned long long wsum[kDrawWaves];
    __shared__ unsigned long long step_sum[kDrawWaves][kDrawMaxSteps];   // totals of each wave's 256-element steps
    __shared__ int pick_s;
    __shared__ int removed[16];   // a node has at most 16 children (the largest topK)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.x / rows.R, r = blockIdx.x - b * rows.R;
    const int node = rows.node[r], first = rows.first_child[r], n_child = rows.n_child[r];
    const float* l = logits + (int64_t)blockIdx.x * V;
    float* q = q_out + ((int64_t)b * n + node) * V;
    float x[4];

    float m = -INFINITY, inv = 0.f;
    if constexpr (!PRE) {
    for (int i = tid * 4; i < V; i += kDrawThreads * 4) {
        load4<VEC4>(l, i, V, x, -INFINITY);
        m = fmaxf(fmaxf(m, fmaxf(x[0], x[1])), fmaxf(x[2], x[3]));
    }
    m = block_max_f<kDrawWaves>(m, sf);
    float part = 0.f;
    for (int i = tid * 4; i < V; i += kDrawThreads * 4) {
        load4<VEC4>(l, i, V, x, -INFINITY);
#pragma unroll
        for (int e = 0; e < 4; ++e) part += expf((x[e] - m) * inv_temperature);   // exp(-inf) = 0 past the end
    }
    inv = 1.0f / block_sum_f<kDrawWaves>(part, sf);
    }

    // q, each wave's integer weight total over its own range, and the totals of its 256-element steps
    const int Vw = (V + kDrawWaves * 256 - 1) / (kDrawWaves * 256) * 256;
    const int w0 = wave * Vw, w1 = min(V, w0 + Vw);
    const int n_steps = Vw / 256;
    const bool fast = PRE || n_steps <= kDrawMaxSteps;   // (else the search walks a wave's range step by step; PRE: the launcher checks)
    unsigned long long acc = 0;
    if constexpr (PRE) {
        // the step totals of this wave's range, as softmax_q_k left them (one per lane: n_steps <= 64)
        const int k = lane;
        const unsigned long long mine = (k < n_steps && w0 + k * 256 < w1) ? step_tot[(int64_t)blockIdx.x * n_steps_all + (w0 >> 8) + k] : 0ull;
        if (k < kDrawMaxSteps) step_sum[wave][k] = mine;
        acc = mine;
    }
    for (int i0 = w0, k = 0; !PRE && i0 < w1; i0 += 256, ++k) {
        const int i = i0 + lane * 4;
        load4<VEC4>(l, i, V, x, -INFINITY);
        float qv[4];
        unsigned long long mine = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            qv[e] = expf((x[e] - m) * inv_temperature) * inv;
            if (i + e < V) mine += q_weight(qv[e]);
        }
        if (VEC4) {
            if (i < V) *(float4*)(q + i) = make_float4(qv[0], qv[1], qv[2], qv[3]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (i + e < V) q[i + e] = qv[e];
        }
        acc += mine;
        if (fast) {
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o, 64);
            if (lane == 0) step_sum[wave][k] = mine;
        }
    }
    if (fast && !PRE)
        for (int k = (w1 > w0 ? (w1 - w0 + 255) / 256 : 0) + lane; k < kDrawMaxSteps; k += 64) step_sum[wave][k] = 0;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (lane == 0) wsum[wave] = acc;
    __syncthreads();   // totals published; the row is complete before any of it is read back

    // weights of the 4 elements a lane holds in the step starting at i0 (tokens already drawn count zero)
    auto step_weights = [&](int i0, int c, unsigned long long (&wt)[4]) {
        const int i = i0 + lane * 4;
        load4<VEC4>(q, i, V, x, 0.f);
        unsigned long long mine = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            bool gone = i + e >= V;
            for (int k = 0; k < c; ++k) gone |= removed[k] == i + e;
            wt[e] = gone ? 0ull : q_weight(x[e]);
            mine += wt[e];
        }
        return mine;
    };
    auto wave_incl_scan = [&](unsigned long long v) {
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const unsigned long long up = __shfl_up(v, o, 64);
            if (lane >= o) v += up;
        }
        return v;
    };

    for (int c = 0; c < n_child; ++c) {
        unsigned long long S = 0;
#pragma unroll
        for (int w = 0; w < kDrawWaves; ++w) S += wsum[w];
        const unsigned long long thr =
            (unsigned long long)(((unsigned __int128)u_draw[(int64_t)b * n + first + c] * (unsigned __int128)S) >> 32);
        // the wave whose range holds the threshold (none when every weight is zero)
        int hit = -1;
        unsigned long long base = 0;
#pragma unroll
        for (int w = 0; w < kDrawWaves; ++w) {
            if (hit < 0) {
                if (base + wsum[w] > thr) hit = w;
                else base += wsum[w];
            }
        }
        if (tid == 0) pick_s = V - 1;
        __syncthreads();
        if (wave == hit) {
            int i0 = w0;
            if (fast) {   // the step: one step total per lane, scanned
                const unsigned long long mine = lane < kDrawMaxSteps ? step_sum[wave][lane] : 0ull;
                const unsigned long long incl = wave_incl_scan(mine);
                const unsigned long long over = __builtin_amdgcn_ballot_w64(base + incl > thr);
                const int k = over ? __builtin_ctzll(over) : 0;
                base += __shfl(incl - mine, k, 64);
                i0 = w0 + k * 256;
            }
            for (; i0 < w1; i0 += 256) {
                unsigned long long wt[4];
                const unsigned long long mine = step_weights(i0, c, wt);
                const unsigned long long incl = wave_incl_scan(mine);
                const unsigned long long step_total = __shfl(incl, 63, 64);
                if (base + step_total > thr) {   // uniform over the wave: the pick is in this step
                    unsigned long long run = base + incl - mine;
                    if (mine > 0 && run <= thr && thr < run + mine) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            run += wt[e];
                            if (run > thr) {
                                pick_s = i0 + lane * 4 + e;
                                break;
                            }
                        }
                    }
                    break;
                }
                base += step_total;
            }
        }
        __syncthreads();
        if (tid == 0) {
            const int pick = pick_s;
            bool gone = false;
            for (int k = 0; k < c; ++k) gone |= removed[k] == pick;
            if (!gone) {
                const unsigned long long w = q_weight(q[pick]);
                const int owner = pick / Vw;
                wsum[owner] -= w;
                if (fast) step_sum[owner][(pick - owner * Vw) / 256] -= w;
            }
            token[(int64_t)b * n + first + c] = pick;
            removed[c] = pick;
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------------
// Acceptance.
__global__ void accept_greedy_k(int B, int n, int stride, const int32_t* __restrict__ token,
                                const int32_t* __restrict__ parent, const int32_t* __restrict__ argmax,
                                int32_t* __restrict__ accept_len, int32_t* __restrict__ path_idx,
                                int32_t* __restrict__ out_tokens, int32_t* __restrict__ n_out) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int32_t* tok = token + (int64_t)b * n;
    const int32_t* par = parent + (int64_t)b * n;
    const int32_t* best = argmax + (int64_t)b * n;
    int32_t* path = path_idx + (int64_t)b * stride;
    int32_t* out = out_tokens + (int64_t)b * stride;
    for (int j = 0; j < stride; ++j) {
        path[j] = -1;
        out[j] = -1;
    }
    int cur = 0, a = 0;
    path[0] = 0;
    for (;;) {
        int t = best[cur];
        out[a] = t;
        int next = -1;
        for (int c = cur + 1; c < n; ++c)
            if (par[c] == cur && tok[c] == t) {
                next = c;
                break;
            }
        if (next < 0 || a + 1 >= stride) break;
        cur = next;
        path[++a] = cur;
    }
    accept_len[b] = a;
    n_out[b] = a + 1;
}

// Recursive rejection sampling.  Integer weights W (target), Qw (draft) and the residual R live in
// the scratch buffer ([B][3][V] u64, followed by the synchronisation area below).  Every sum over the
// vocabulary is an exact integer sum and every other operation a single IEEE double operation, so the
// decisions do not depend on how the vocabulary is split or in which order partial sums arrive.
//
// A sequence is worked on by G workgroups, each owning a contiguous slice of the vocabulary (its
// slices of W, Qw and R are written and read by it alone).  The walk down the tree is sequential --
// each decision needs vocabulary-wide totals -- so it proceeds in phases: in a phase every workgroup
// passes over its slice, adds its partial sums to the phase's slots with 64-bit atomics, and the G
// workgroups meet at the phase's counter; afterwards all of them read the same totals and take the
// same decision redundantly (no leader, nothing is broadcast).  The owner of the token the NEXT
// acceptance test is about adds that token's weights to further slots of the same phase, so no
// workgroup ever reads another one's slice.  Every phase has slots and a counter of its own in a
// zeroed area, so nothing is reset while others may still read it.
// The meeting is a bounded wait: the G * B workgroups of a launch (at most 256, 256 threads each)
// are co-resident on an idle chip; if that ever fails to hold long enough (another stream's kernels
// occupying the chip), a workgroup gives up after kAcceptSpinLimit polls, raises the status word and
// every workgroup of the launch leaves at its next poll.
__device__ __forceinline__ double u64_to_d(unsigned long long x) { return (double)x; }

constexpr int kAcceptThreads = 256;       // multi-workgroup sampling acceptance
constexpr int kAcceptMaxGroups = 64;      // workgroups per sequence
constexpr int kAcceptPhases = 2 * TLT_ACCEPT_MAX_NODES + 4;   // node passes (<= stride <= nodes + 1) + rejections (< nodes) + final
constexpr int kAcceptSlots = 5;           // per phase: S or residual total, SQ, next token's W, its R, its Qw
constexpr unsigned kAcceptSpinLimit = 1u << 24;

struct AcceptSync {   // one per sequence, zeroed before the launch
    unsigned long long sum[kAcceptPhases][kAcceptSlots];
    unsigned long long slice_total[kAcceptMaxGroups];
    unsigned int arrived[kAcceptPhases];
    float row_max[TLT_ACCEPT_MAX_NODES];   // largest logit of every tree node's row (written by accept_row_max_k)
};

__device__ __forceinline__ unsigned long long sync_load(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// All G workgroups of the sequence have finished phase `ph` (and their atomic adds are visible) when
// this returns true; false = gave up (status raised) or another workgroup did.
__device__ __forceinline__ bool accept_meet(AcceptSync* sy, int ph, int G, unsigned int* status, int* ok_s) {
    __syncthreads();
    if (threadIdx.x == 0) {
        __hip_atomic_fetch_add(&sy->arrived[ph], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        unsigned spins = 0;
        int ok = 1;
        while (__hip_atomic_load(&sy->arrived[ph], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < (unsigned)G) {
            __builtin_amdgcn_s_sleep(2);
            if (++spins > kAcceptSpinLimit || (__hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & 2u) != 0u) {
                __hip_atomic_fetch_or(status, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = 0;
                break;
            }
        }
        *ok_s = ok;
    }
    __syncthreads();
    return *ok_s != 0;
}

__global__ __launch_bounds__(kAcceptThreads) void accept_sync_clear_k(unsigned long long* p, int64_t count) {
    for (int64_t i = (int64_t)blockIdx.x * kAcceptThreads + threadIdx.x; i < count; i += (int64_t)gridDim.x * kAcceptThreads) p[i] = 0ull;
}

// Largest logit of every (sequence, node) row, one workgroup per row: every node pass of the walk needs its
// row's maximum first, and one parallel pass over all rows is cheaper than every workgroup of a sequence
// scanning the whole row again at every node.
__global__ __launch_bounds__(kAcceptThreads) void accept_row_max_k(int n, int V, const float* __restrict__ logits,
                                                                   AcceptSync* __restrict__ sync) {
    __shared__ float sf[kAcceptThreads / 64];
    const int b = blockIdx.x / n, i = blockIdx.x - b * n, tid = threadIdx.x;
    const float* l = logits + (int64_t)blockIdx.x * V;
    float m = -INFINITY;
    if (V % 4 == 0 && ((uintptr_t)l & 15) == 0) {
        for (int j = tid * 4; j < V; j += kAcceptThreads * 4) {
            const float4 x = *(const float4*)(l + j);
            m = fmaxf(fmaxf(m, fmaxf(x.x, x.y)), fmaxf(x.z, x.w));
        }
    } else {
        for (int j = tid; j < V; j += kAcceptThreads) m = fmaxf(m, l[j]);
    }
    m = block_max_f<kAcceptThreads / 64>(m, sf);
    if (tid == 0) sync[b].row_max[i] = m;
}

__global__ __launch_bounds__(kAcceptThreads) void accept_sample_k(int n, int V, int stride, int G, int slice, float temperature,
                                                       const int32_t* __restrict__ token,
                                                       const int32_t* __restrict__ parent,
                                                       const float* __restrict__ logits,
                                                       const float* __restrict__ draft_q,
                                                       const uint32_t* __restrict__ u_accept,
                                                       const uint32_t* __restrict__ u_final,
                                                       int32_t* __restrict__ accept_len, int32_t* __restrict__ path_idx,
                                                       int32_t* __restrict__ out_tokens, int32_t* __restrict__ n_out,
                                                       unsigned long long* __restrict__ ws, AcceptSync* __restrict__ sync,
                                                       unsigned int* __restrict__ status) {
    constexpr int NW = kAcceptThreads / 64;
    __shared__ unsigned long long su[NW];
    __shared__ int ok_s, pick_s;
    const int b = blockIdx.x / G, g = blockIdx.x - b * G, tid = threadIdx.x;
    const int32_t* tok = token + (int64_t)b * n;
    const int32_t* par = parent + (int64_t)b * n;
    int32_t* path = path_idx + (int64_t)b * stride;
    int32_t* out = out_tokens + (int64_t)b * stride;
    unsigned long long* W = ws + (int64_t)b * 3 * V;
    unsigned long long* Qw = W + V;
    unsigned long long* R = Qw + V;   // the residual is built here and swapped with W when it has mass
    AcceptSync* sy = sync + b;
    const int v0 = min(V, g * slice), v1 = min(V, v0 + slice);
    const bool writer = g == 0;       // the workgroup that writes what all of them know
    const double tau = (double)temperature;
    if (writer)
        for (int j = tid; j < stride; j += kAcceptThreads) {
            path[j] = -1;
            out[j] = -1;
        }
    __syncthreads();
    int cur = 0, a = 0, ph = 0;
    if (writer && tid == 0) path[0] = 0;
    unsigned long long S = 0, SQ = 0;
    auto owns = [&](int t) { return t >= v0 && t < v1; };
    auto next_child = [&](int after) {   // next child of `cur` with a token inside the vocabulary, or -1
        for (int c = after + 1; c < n; ++c)
            if (par[c] == cur && tok[c] >= 0 && tok[c] < V) return c;
        return -1;
    };
    for (;;) {
        const float* l = logits + ((int64_t)b * n + cur) * V;
        const float* q = draft_q + ((int64_t)b * n + cur) * V;
        // max_j (l_j / tau) = (max_j l_j) / tau: a correctly rounded division by a positive number keeps
        // the order, so the maximum is taken on the floats (by accept_row_max_k, before this kernel) and
        // divided once.
        const double m = (double)sy->row_max[cur] / tau;
        int c = a + 1 < stride ? next_child(cur) : -1;
        unsigned long long s = 0, sq = 0;
        for (int j = v0 + tid; j < v1; j += kAcceptThreads) {
            const unsigned long long w = (unsigned long long)floor(exp((double)l[j] / tau - m) * 4294967296.0);
            const unsigned long long qw = (unsigned long long)floor((double)q[j] * 4294967296.0);
            W[j] = w;
            Qw[j] = qw;
            s += w;
            sq += qw;
        }
        s = block_sum_u64<NW>(s, su);
        sq = block_sum_u64<NW>(sq, su);   // (block_sum's barriers also make this workgroup's W/Qw writes visible to it)
        if (ph >= kAcceptPhases) return;  // cannot happen for n <= TLT_ACCEPT_MAX_NODES (uniform)
        if (tid == 0) {
            atomicAdd(&sy->sum[ph][0], s);
            atomicAdd(&sy->sum[ph][1], sq);
            if (c >= 0 && owns(tok[c])) {
                atomicAdd(&sy->sum[ph][2], W[tok[c]]);
                atomicAdd(&sy->sum[ph][4], Qw[tok[c]]);
            }
        }
        if (!accept_meet(sy, ph, G, status, &ok_s)) return;
        S = sync_load(&sy->sum[ph][0]);
        SQ = sync_load(&sy->sum[ph][1]);
        unsigned long long wt = sync_load(&sy->sum[ph][2]), qt = sync_load(&sy->sum[ph][4]);
        ++ph;
        int next = -1;
        while (c >= 0) {
            const int t = tok[c];
            const double p = u64_to_d(wt) / u64_to_d(S);
            const double qq = SQ > 0 ? u64_to_d(qt) / u64_to_d(SQ) : 0.0;
            const double u = ((double)u_accept[(int64_t)b * n + c] + 0.5) / 4294967296.0;
            if (u * qq < p) {
                next = c;
                break;
            }
            // rejected: residual over the slice; the token of the child tested next is looked up on the way
            const int cn = next_child(c);
            unsigned long long s2 = 0;
            for (int j = v0 + tid; j < v1; j += kAcceptThreads) {
                const double pj = u64_to_d(W[j]) / u64_to_d(S);
                const double qj = SQ > 0 ? u64_to_d(Qw[j]) / u64_to_d(SQ) : 0.0;
                double r = pj - qj;
                if (r < 0.0) r = 0.0;
                const unsigned long long rw = (unsigned long long)floor(r * 4294967296.0);
                R[j] = rw;
                s2 += rw;
            }
            s2 = block_sum_u64<NW>(s2, su);
            if (ph >= kAcceptPhases) return;
            if (tid == 0) {
                atomicAdd(&sy->sum[ph][0], s2);
                if (cn >= 0 && owns(tok[cn])) {
                    const int tn = tok[cn];
                    atomicAdd(&sy->sum[ph][2], W[tn]);
                    atomicAdd(&sy->sum[ph][3], R[tn]);
                    atomicAdd(&sy->sum[ph][4], tn == t ? 0ull : Qw[tn]);   // the rejected token leaves the draft
                }
                if (owns(t)) Qw[t] = 0;
            }
            if (!accept_meet(sy, ph, G, status, &ok_s)) return;
            s2 = sync_load(&sy->sum[ph][0]);
            const bool swap = s2 > 0;   // the residual replaces the target weights when it has mass (uniform)
            wt = sync_load(&sy->sum[ph][swap ? 3 : 2]);
            SQ -= qt;                   // exact integer update of the draft's total
            qt = sync_load(&sy->sum[ph][4]);
            ++ph;
            if (swap) {
                unsigned long long* tmp = W;
                W = R;
                R = tmp;
                S = s2;
            }
            c = cn;
        }
        if (next < 0) break;
        if (writer && tid == 0) out[a] = tok[next];
        cur = next;
        ++a;
        if (writer && tid == 0) path[a] = cur;
    }
    // final draw: first index whose running sum exceeds (u_final * S) >> 32.  Slice totals first, then the
    // workgroup whose slice holds the threshold searches it.
    unsigned long long local = 0;
    const int chunk = (v1 - v0 + kAcceptThreads - 1) / kAcceptThreads;
    const int j0 = min(v1, v0 + tid * chunk), j1 = min(v1, j0 + chunk);
    for (int j = j0; j < j1; ++j) local += W[j];
    const unsigned long long mine = block_sum_u64<NW>(local, su);
    if (ph >= kAcceptPhases) return;
    if (tid == 0) __hip_atomic_store(&sy->slice_total[g], mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (!accept_meet(sy, ph, G, status, &ok_s)) return;
    const unsigned long long thr =
        (unsigned long long)(((unsigned __int128)u_final[b] * (unsigned __int128)S) >> 32);
    unsigned long long before = 0;
    int owner = -1;
    for (int k = 0; k < G; ++k) {   // uniform
        const unsigned long long tk = sync_load(&sy->slice_total[k]);
        if (owner < 0 && before + tk > thr) owner = k;
        if (owner < 0) before += tk;
    }
    if (owner < 0) {   // no mass anywhere: the oracle's fallback
        if (writer && tid == 0) {
            out[a] = V - 1;
            accept_len[b] = a;
            n_out[b] = a + 1;
        }
        return;
    }
    if (writer && tid == 0) {
        accept_len[b] = a;
        n_out[b] = a + 1;
    }
    if (g != owner) return;
    // exclusive scan of the threads' chunk totals (wave scan, then the waves' totals)
    unsigned long long incl = local;
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned long long up = __shfl_up(incl, o, 64);
        if (lane >= o) incl += up;
    }
    if (lane == 63) su[wave] = incl;
    if (tid == 0) pick_s = v1 - 1;
    __syncthreads();
    unsigned long long wbase = before;
    for (int w = 0; w < wave; ++w) wbase += su[w];
    const unsigned long long excl = wbase + incl - local;
    if (local > 0 && excl <= thr && thr < excl + local) {
        unsigned long long run = excl;
        for (int j = j0; j < j1; ++j) {
            run += W[j];
            if (run > thr) {
                pick_s = j;
                break;
            }
        }
    }
    __syncthreads();
    if (tid == 0) out[a] = pick_s;
}

// Target-only rule (for trees whose shape depends on the drafter's values): child c is accepted
// iff (U * S) >> 32 < W[token(c)] with the node's current integer target weights, a rejected child's
// weight leaves S; no child left -> the same final draw from what remains.  Weights are recomputed
// from the logits where needed (W_j = floor(exp(l_j/tau - max) * 2^32), exp in double), the tokens
// removed at the current node are kept in a short list; no workspace.
constexpr int kTargetOnlyThreads = 1024;   // one workgroup per sequence: as wide as a workgroup gets
__global__ __launch_bounds__(kTargetOnlyThreads) void accept_target_only_k(int n, int V, int stride, float temperature,
                                                                      const int32_t* __restrict__ token,
                                                                      const int32_t* __restrict__ parent,
                                                                      const float* __restrict__ logits,
                                                                      const uint32_t* __restrict__ u_accept,
                                                                      const uint32_t* __restrict__ u_final,
                                                                      int32_t* __restrict__ accept_len,
                                                                      int32_t* __restrict__ path_idx,
                                                                      int32_t* __restrict__ out_tokens,
                                                                      int32_t* __restrict__ n_out) {
    __shared__ unsigned long long su[kTargetOnlyThreads / 64];
    __shared__ double sd[kTargetOnlyThreads / 64];
    __shared__ unsigned long long scan[kTargetOnlyThreads];
    __shared__ int pick_s;
    __shared__ int removed[64];   // a node has fewer than 64 children
    const int b = blockIdx.x, tid = threadIdx.x;
    const int32_t* tok = token + (int64_t)b * n;
    const int32_t* par = parent + (int64_t)b * n;
    int32_t* path = path_idx + (int64_t)b * stride;
    int32_t* out = out_tokens + (int64_t)b * stride;
    const double tau = (double)temperature;
    for (int j = tid; j < stride; j += kTargetOnlyThreads) {
        path[j] = -1;
        out[j] = -1;
    }
    __syncthreads();
    int cur = 0, a = 0, n_removed = 0;
    if (tid == 0) path[0] = 0;
    unsigned long long S = 0;
    double m = 0.0;
    const float* l = logits;
    auto weight = [&](int j) { return (unsigned long long)floor(exp((double)l[j] / tau - m) * 4294967296.0); };
    auto is_removed = [&](int j) {
        bool gone = false;
        for (int k = 0; k < n_removed; ++k) gone |= removed[k] == j;
        return gone;
    };
    for (;;) {
        l = logits + ((int64_t)b * n + cur) * V;
        m = -INFINITY;
        for (int j = tid; j < V; j += kTargetOnlyThreads) m = fmax(m, (double)l[j] / tau);
        m = block_max_d<kTargetOnlyThreads / 64>(m, sd);
        unsigned long long s = 0;
        for (int j = tid; j < V; j += kTargetOnlyThreads) s += weight(j);
        S = block_sum_u64<kTargetOnlyThreads / 64>(s, su);
        n_removed = 0;
        int next = -1;
        for (int c = cur + 1; c < n && a + 1 < stride; ++c) {
            if (par[c] != cur) continue;   // uniform: every thread reads the same tree
            const int t = tok[c];
            __syncthreads();               // the removed list as left by the previous child
            const unsigned long long wt = (t >= 0 && t < V && !is_removed(t)) ? weight(t) : 0ull;
            const unsigned long long thr =
                (unsigned long long)(((unsigned __int128)u_accept[(int64_t)b * n + c] * (unsigned __int128)S) >> 32);
            if (thr < wt) {
                next = c;
                break;
            }
            S -= wt;
            __syncthreads();
            if (tid == 0 && wt > 0) removed[n_removed] = t;
            if (wt > 0) ++n_removed;
        }
        if (next < 0) break;
        if (tid == 0) out[a] = tok[next];
        cur = next;
        ++a;
        if (tid == 0) path[a] = cur;
        __syncthreads();
    }
    // final draw from what remains at the last node
    __syncthreads();
    const unsigned long long thr =
        (unsigned long long)(((unsigned __int128)u_final[b] * (unsigned __int128)S) >> 32);
    const int chunk = (V + kTargetOnlyThreads - 1) / kTargetOnlyThreads;
    const int j0 = min(V, tid * chunk), j1 = min(V, j0 + chunk);
    unsigned long long local = 0;
    for (int j = j0; j < j1; ++j) local += is_removed(j) ? 0ull : weight(j);
    scan[tid] = local;
    if (tid == 0) pick_s = V - 1;
    __syncthreads();
    if (tid == 0) {
        unsigned long long run = 0;
        for (int t = 0; t < kTargetOnlyThreads; ++t) {
            unsigned long long v = scan[t];
            scan[t] = run;
            run += v;
        }
    }
    __syncthreads();
    const unsigned long long excl = scan[tid];
    if (local > 0 && excl <= thr && thr < excl + local) {
        unsigned long long run = excl;
        for (int j = j0; j < j1; ++j) {
            run += is_removed(j) ? 0ull : weight(j);
            if (run > thr) {
                pick_s = j;
                break;
            }
        }
    }
    __syncthreads();
    if (tid == 0) {
        out[a] = pick_s;
        accept_len[b] = a;
        n_out[b] = a + 1;
    }
}

// ------------------------------------------------------------------------------------------------
// KV commit: row seq_len+path[j] -> row seq_len+j, j = 1..accept_len, for one (sequence, layer,
// kv head) per workgroup.  A thread owns one 16-byte column chunk of K or V for all j and walks j
// upward in batches of 8 (8 loads in flight, then 8 stores).  This order is hazard-free: a
// destination row j can only be the source of an earlier j' (path[j'] >= j'), which has already been
// read either in a previous batch or earlier in this batch's load phase.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

__global__ __launch_bounds__(64) void kv_commit_k(int n_layers, char* __restrict__ k_pool, char* __restrict__ v_pool,
                                                  int64_t n_pages, const int32_t* __restrict__ block_table,
                                                  const int32_t* __restrict__ seq_len, int max_pages, int page_size,
                                                  int n_kv, int row_bytes, const int32_t* __restrict__ accept_len,
                                                  const int32_t* __restrict__ path_idx, int stride) {
    const int kh = blockIdx.x % n_kv, layer = blockIdx.x / n_kv, b = blockIdx.y;
    int a = accept_len[b];
    if (a > stride - 1) a = stride - 1;
    if (a <= 0) return;
    const int chunks = row_bytes / 16;
    const int ctx = seq_len[b];
    const int32_t* path = path_idx + (int64_t)b * stride;
    const int64_t layer_off = (int64_t)layer * n_pages * n_kv * page_size * row_bytes;
    for (int t = threadIdx.x; t < 2 * chunks; t += 64) {
        char* pool = (t < chunks ? k_pool : v_pool) + layer_off;
        const int col = (t < chunks ? t : t - chunks) * 16;
        for (int j0 = 1; j0 <= a; j0 += 8) {
            u32x4_t tmp[8];
            bool ok[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                int j = j0 + e;
                ok[e] = false;
                if (j <= a) {
                    int p = path[j];
                    PageRef pr;
                    if (p > j && locate(block_table, max_pages, n_pages, page_size, b, ctx + p, pr)) {
                        tmp[e] = *(const u32x4_t*)(pool + ((pr.page * n_kv + kh) * page_size + pr.row) * row_bytes + col);
                        ok[e] = true;
                    }
                }
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                int j = j0 + e;
                PageRef pr;
                if (ok[e] && locate(block_table, max_pages, n_pages, page_size, b, ctx + j, pr))
                    *(u32x4_t*)(pool + ((pr.page * n_kv + kh) * page_size + pr.row) * row_bytes + col) = tmp[e];
            }
        }
    }
}

__global__ void seq_len_advance_k(int B, int32_t* seq_len, const int32_t* accept_len, int stride) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int a = accept_len[b];
    if (a > stride - 1) a = stride - 1;
    if (a < 0) a = 0;
    seq_len[b] += a + 1;
}

// ------------------------------------------------------------------------------------------------
hipError_t row_argmax(hipStream_t s, int M, int V, const float* logits, int32_t* out, void* scratch, size_t scratch_bytes) {
    if (M <= 0) return hipSuccess;
    // few rows: a row's scan over several workgroups (a single one pulls the 600 KB row through one CU's load path: 45 us)
    int S = M < 128 ? 256 / M : 1;
    S = S > 32 ? 32 : S;
    if (S >= 2 && scratch && ((uintptr_t)scratch & 7) == 0 && (size_t)M * S * 8 <= scratch_bytes) {
        const int seg = ((V + S - 1) / S + 3) / 4 * 4;
        float* pv = (float*)scratch;
        int32_t* pi = (int32_t*)(pv + (size_t)M * S);
        hipLaunchKernelGGL(row_argmax_seg_k, dim3(S, M), dim3(256), 0, s, V, seg, S, logits, pv, pi);
        hipLaunchKernelGGL(row_argmax_merge_k, dim3(M), dim3(64), 0, s, S, pv, pi, out);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(row_argmax_k, dim3(M), dim3(256), 0, s, V, logits, out);
    return hipGetLastError();
}

hipError_t row_lse(hipStream_t s, int M, int V, const float* logits, float* out) {
    if (M <= 0) return hipSuccess;
    hipLaunchKernelGGL(row_lse_k, dim3(M), dim3(256), 0, s, V, logits, out);
    return hipGetLastError();
}

size_t row_topk_workspace_bytes(int M, int V, int K) {
    const size_t n_seg = (size_t)(V + kTopkSeg - 1) / kTopkSeg;
    return (size_t)M * n_seg * (2 + 2 * (size_t)K) * 4 + 256;
}

hipError_t row_topk_logp(hipStream_t s, int M, int V, int K, const float* logits, int32_t* tok, float* logp, void* ws) {
    if (M <= 0) return hipSuccess;
    const int n_seg = (V + kTopkSeg - 1) / kTopkSeg;
    float* seg_stat = (float*)ws;
    float* seg_val = seg_stat + (size_t)M * n_seg * 2;
    int32_t* seg_idx = (int32_t*)(seg_val + (size_t)M * n_seg * K);
    const dim3 grid((n_seg + 3) / 4, M);
    if (V % 4 == 0 && ((uintptr_t)logits & 15) == 0)
        hipLaunchKernelGGL(row_topk_seg_k<true>, grid, dim3(256), 0, s, V, K, n_seg, logits, seg_stat, seg_val, seg_idx);
    else
        hipLaunchKernelGGL(row_topk_seg_k<false>, grid, dim3(256), 0, s, V, K, n_seg, logits, seg_stat, seg_val, seg_idx);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(row_topk_merge_k, dim3(M), dim3(64), 0, s, K, n_seg, seg_stat, seg_val, seg_idx, tok, logp);
    return hipGetLastError();
}

hipError_t draft_level0(hipStream_t s, int B, int K, const int32_t* top_tok, const float* top_logp, DraftState st,
                        int feat_rows_per_seq) {
    (void)feat_rows_per_seq;
    hipLaunchKernelGGL(draft_level0_k, dim3((B * K + 255) / 256), dim3(256), 0, s, B, K, top_tok, top_logp, st);
    return hipGetLastError();
}

hipError_t draft_level_select(hipStream_t s, int B, int K, int level, const int32_t* top_tok, const float* top_logp,
                              DraftState st, int feat_rows_per_seq) {
    (void)feat_rows_per_seq;
    hipLaunchKernelGGL(draft_level_select_k, dim3(B), dim3(256), 0, s, K, level, top_tok, top_logp, st);
    return hipGetLastError();
}

hipError_t draft_prune(hipStream_t s, int B, int pool_n, int n_tree, const int32_t* root_tokens,
                       const int32_t* new_tokens, const int32_t* n_new, int new_stride, DraftState st, int32_t* token, int32_t* parent, int32_t* depth, uint64_t* anc_mask, float* score) {
    size_t lds = sizeof(float) * (size_t)pool_n * 2 + sizeof(int) * (size_t)n_tree;
    hipLaunchKernelGGL(draft_prune_k, dim3(B), dim3(256), lds, s, pool_n, n_tree, root_tokens, new_tokens, n_new,
                       new_stride, st, token, parent, depth, anc_mask, score);
    return hipGetLastError();
}

hipError_t tree_finalize(hipStream_t s, int B, int n, const int32_t* parent, int32_t* depth, uint64_t* anc_mask) {
    hipLaunchKernelGGL(tree_finalize_k, dim3((B * n + 255) / 256), dim3(256), 0, s, B, n, parent, depth, anc_mask);
    return hipGetLastError();
}

hipError_t tmpl_tree_init(hipStream_t s, int B, int n, TmplParents tp, const int32_t* root_tokens, const int32_t* new_tokens,
                          const int32_t* n_new, int new_stride, int32_t* token, int32_t* parent, float* score) {
    hipLaunchKernelGGL(tmpl_tree_init_k, dim3((B * n + 255) / 256), dim3(256), 0, s, B, n, tp, root_tokens, new_tokens, n_new,
                       new_stride, token, parent, score);
    return hipGetLastError();
}

hipError_t tmpl_level_rows(hipStream_t s, int B, int n, TmplRows rows, const int32_t* token, int32_t* fr_token, int32_t* fr_src,
                           uint64_t* fr_mask) {
    hipLaunchKernelGGL(tmpl_level_rows_k, dim3((B * rows.R + 255) / 256), dim3(256), 0, s, B, n, rows, token, fr_token, fr_src,
                       fr_mask);
    return hipGetLastError();
}

hipError_t softmax_draw(hipStream_t s, int B, int n, int V, float temperature, TmplRows rows, const float* logits,
                        const uint32_t* u_draw, int32_t* token, float* q, void* scratch, size_t scratch_bytes) {
    // 16-byte accesses need every row of the logits and of q to start on a 16-byte boundary
    const bool vec4 = V % 4 == 0 && (((uintptr_t)logits | (uintptr_t)q) & 15) == 0;
    const int M = B * rows.R;
    // few rows: each row's softmax over several workgroups (see softmax_part_k), as many as fill most of the chip
    const int n_steps_all = (V + 255) / 256;
    const int Vw = (V + kDrawWaves * 256 - 1) / (kDrawWaves * 256) * 256;
    int G = M >= 96 ? 1 : 192 / M;
    G = G > 16 ? 16 : G;
    const int seg = G > 1 ? ((V + G - 1) / G + 1023) / 1024 * 1024 : V;
    if (G > 1) G = (V + seg - 1) / seg;   // (no empty segment)
    const size_t part_bytes = ((size_t)M * G * 2 * sizeof(float) + 255) / 256 * 256;
    const size_t need = part_bytes + (size_t)M * n_steps_all * sizeof(unsigned long long);
    if (G > 1 && scratch && need <= scratch_bytes && Vw / 256 <= kDrawMaxSteps && ((uintptr_t)scratch & 7) == 0) {
        float* part = (float*)scratch;
        unsigned long long* step_tot = (unsigned long long*)((char*)scratch + part_bytes);
        if (vec4) {
            hipLaunchKernelGGL(softmax_part_k<true>, dim3(M * G), dim3(kDrawThreads), 0, s, V, G, seg, 1.0f / temperature, logits, part);
            hipLaunchKernelGGL(softmax_q_k<true>, dim3(M * G), dim3(kDrawThreads), 0, s, n, V, G, seg, n_steps_all, 1.0f / temperature,
                               rows, logits, part, q, step_tot);
            hipLaunchKernelGGL((softmax_draw_k<true, true>), dim3(M), dim3(kDrawThreads), 0, s, n, V, 1.0f / temperature, rows,
                               logits, u_draw, token, q, step_tot, n_steps_all);
        } else {
            hipLaunchKernelGGL(softmax_part_k<false>, dim3(M * G), dim3(kDrawThreads), 0, s, V, G, seg, 1.0f / temperature, logits, part);
            hipLaunchKernelGGL(softmax_q_k<false>, dim3(M * G), dim3(kDrawThreads), 0, s, n, V, G, seg, n_steps_all, 1.0f / temperature,
                               rows, logits, part, q, step_tot);
            hipLaunchKernelGGL((softmax_draw_k<false, true>), dim3(M), dim3(kDrawThreads), 0, s, n, V, 1.0f / temperature, rows,
                               logits, u_draw, token, q, step_tot, n_steps_all);
        }
        return hipGetLastError();
    }
    if (vec4)
        hipLaunchKernelGGL((softmax_draw_k<true, false>), dim3(M), dim3(kDrawThreads), 0, s, n, V, 1.0f / temperature, rows,
                           logits, u_draw, token, q, (const unsigned long long*)nullptr, 0);
    else
        hipLaunchKernelGGL((softmax_draw_k<false, false>), dim3(M), dim3(kDrawThreads), 0, s, n, V, 1.0f / temperature, rows,
                           logits, u_draw, token, q, (const unsigned long long*)nullptr, 0);
    return hipGetLastError();
}

hipError_t accept_greedy(hipStream_t s, int B, int n, int V, int stride, const int32_t* token, const int32_t* parent,
                         const float* logits, const int32_t* argmax, int32_t* accept_len, int32_t* path_idx,
                         int32_t* out_tokens, int32_t* n_out) {
    (void)V; (void)logits;
    hipLaunchKernelGGL(accept_greedy_k, dim3((B + 63) / 64), dim3(64), 0, s, B, n, stride, token, parent, argmax,
                       accept_len, path_idx, out_tokens, n_out);
    return hipGetLastError();
}

static int accept_groups(int B) {
    int G = 256 / (B > 0 ? B : 1);
    return G < 1 ? 1 : (G > kAcceptMaxGroups ? kAcceptMaxGroups : G);
}

size_t accept_sample_workspace_bytes(int B, int V) {
    return ((size_t)B * 3 * (size_t)V * sizeof(unsigned long long) + 255) / 256 * 256 + (size_t)B * sizeof(AcceptSync);
}

hipError_t accept_sample(hipStream_t s, int B, int n, int V, int stride, float temperature, const int32_t* token,
                         const int32_t* parent, const float* logits, const float* draft_q, const uint32_t* u_accept,
                         const uint32_t* u_final, int32_t* accept_len, int32_t* path_idx, int32_t* out_tokens,
                         int32_t* n_out, void* ws, unsigned int* status) {
    if (n > TLT_ACCEPT_MAX_NODES) return hipErrorInvalidValue;
    const int G = accept_groups(B);
    const int slice = ((V + G - 1) / G + 3) & ~3;
    AcceptSync* sync = (AcceptSync*)((char*)ws + ((size_t)B * 3 * (size_t)V * sizeof(unsigned long long) + 255) / 256 * 256);
    const int64_t words = (int64_t)B * (int64_t)(sizeof(AcceptSync) / 8);
    hipLaunchKernelGGL(accept_sync_clear_k, dim3((unsigned)((words + kAcceptThreads - 1) / kAcceptThreads)), dim3(kAcceptThreads),
                       0, s, (unsigned long long*)sync, words);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(accept_row_max_k, dim3(B * n), dim3(kAcceptThreads), 0, s, n, V, logits, sync);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(accept_sample_k, dim3(B * G), dim3(kAcceptThreads), 0, s, n, V, stride, G, slice, temperature, token,
                       parent, logits, draft_q, u_accept, u_final, accept_len, path_idx, out_tokens, n_out,
                       (unsigned long long*)ws, sync, status);
    return hipGetLastError();
}

hipError_t accept_target_only(hipStream_t s, int B, int n, int V, int stride, float temperature, const int32_t* token,
                              const int32_t* parent, const float* logits, const uint32_t* u_accept, const uint32_t* u_final,
                              int32_t* accept_len, int32_t* path_idx, int32_t* out_tokens, int32_t* n_out) {
    hipLaunchKernelGGL(accept_target_only_k, dim3(B), dim3(kTargetOnlyThreads), 0, s, n, V, stride, temperature, token, parent,
                       logits, u_accept, u_final, accept_len, path_idx, out_tokens, n_out);
    return hipGetLastError();
}

hipError_t kv_commit(hipStream_t s, int dtype, int B, int n_layers, void* k_pool, void* v_pool, int64_t n_pages,
                     const int32_t* block_table, int32_t* seq_len, int max_pages, int page_size, int n_kv, int d,
                     const int32_t* accept_len, const int32_t* path_idx, int stride) {
    if (B <= 0) return hipSuccess;
    const int row_bytes = d * (dtype == F32 ? 4 : 2);
    hipLaunchKernelGGL(kv_commit_k, dim3(n_layers * n_kv, B), dim3(64), 0, s, n_layers, (char*)k_pool, (char*)v_pool,
                       n_pages, block_table, seq_len, max_pages, page_size, n_kv, row_bytes, accept_len, path_idx, stride);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(seq_len_advance_k, dim3((B + 63) / 64), dim3(64), 0, s, B, seq_len, accept_len, stride);
    return hipGetLastError();
}

}  // namespace tlt
