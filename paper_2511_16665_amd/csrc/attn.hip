// Tree-masked grouped-query attention over the paged KV cache.
//
// Every active row (b, i) of every query head attends to the seq_len[b] committed cache rows and to
// the provisional rows seq_len[b] + j whose bit j is set in the row's mask (ancestors-or-self of a
// tree node; a causal prefix for chains).
//
// impl 0 ("wave-per-row"): one wavefront per (row, query head); lanes own keys for the score pass
//   and head dimensions for the value pass; online softmax across 64-key tiles.  Any dtype, any
//   head_dim that is a multiple of 64 up to 256.  Used for fp32 mode and as a cross-check.
// impl 1 ("MFMA split-KV"): the bf16 / head_dim 128 production kernel, described further down.
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

// ------------------------------------------------------------------------------------------------
// impl 1 ("MFMA split-KV"), bf16, head_dim 128.
//
// One workgroup (8 waves, two per SIMD) owns (sequence b, kv head, chunk of CK keys, group of
// query-row tiles).  All G query heads of the kv head and all tree rows form the row set R = n*G,
// row r = i*G + g, cut into tiles of 16 rows dealt round-robin to the waves; a wave keeps its tiles'
// Q fragments and fp32 output accumulators in registers and the whole workgroup streams the chunk's
// K/V pages once through a 4-stage LDS ring in tiles of 64 keys, filled by direct global->LDS loads
// issued two tiles ahead.  A wave runs the instance of the program for the number of row tiles it owns
// (waves of one workgroup share the barriers and the fetches, not the code).
//
// Both products run on v_mfma_f32_16x16x32_bf16 in the transposed orientation:
//   S^T[key][row] = sum_d K[key][d] Q[row][d]      A = K rows from LDS, B = Q fragment
//   O^T[d][row]  += sum_key V^T[d][key] P^T[key][row]   A = V^T read with the LDS transpose load,
//                                                       B = P packed from S^T
// In that orientation a lane's S^T results (4 consecutive keys of its own row l%16) are already the
// k-slots the second product's B operand wants, so P never leaves registers, and the k-slot order
// (slot 4*sub + v of lane group g = key 16*sub + 4*g + v) is matched on the V side by which keys each
// transpose load addresses.  A lane's 32 accumulators all belong to one row, so the online-softmax
// rescale is a per-lane scalar.
// Each workgroup writes unnormalised partial outputs with their running max and sum (fp32); a
// second kernel merges the chunks.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

// max over the four 16-lane groups of a wave (lanes l, l^16, l^32, l^48) without going through the LDS
// crossbar: v_permlane32_swap / v_permlane16_swap exchange half-waves / odd and even 16-lane rows of
// two registers, so swapping a value with a copy of itself puts the partner's value beside it.
__device__ __forceinline__ float group_max4(float x) {
    const uint32_t u = __float_as_uint(x);
    const auto a = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const float m = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const uint32_t v = __float_as_uint(m);
    const auto b = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

constexpr int kD = 128;       // head_dim of this kernel
constexpr int kKT = 64;       // keys per LDS tile
constexpr int kStages = 4;                  // LDS ring depth
constexpr int kAhead = 2;                   // tiles of K/V in flight; one more stage stays readable for the late waves (below)
constexpr int kStageElems = 2 * kKT * kD;   // one stage: K tile then V tile, 16 KB each
constexpr float kNegBig = -1e30f;
constexpr int kMaxRows = 128;    // rows per sequence whose visibility bits are kept in LDS
constexpr int kMaxChunk = 4096;  // keys per chunk: bounds the page-id table kept in LDS

// Work decomposition.  A work item is (sequence, key range); each item is run by n_kv * row_groups
// workgroups.  The key ranges are cut ON THE DEVICE from the actual sequence lengths (the host only
// knows an upper bound): a one-workgroup planning kernel picks the item length so that the chip
// gets about two items per CU (8 .. 64 tiles of 64 keys), gives every sequence equally long chunks,
// and lists the items longest first.  Workgroups are dispatched in list order, so the long items
// start first and the short ones fill the tail (longest-processing-time-first list scheduling).
struct AttnItem {
    int b, k_begin, k_end, slot;   // slot: index of this item's partial result (slots of a sequence are contiguous)
};
struct AttnWork {        // lives in the workspace, written by attn_plan_k
    int n_items;
    int pad[3];
    // int slot0[B]; int n_chunks[B]; AttnItem items[max_items];
};

struct AttnPlan {
    int row_tiles;   // ceil(R / 16)
    int row_groups;  // row tiles are cut into groups of at most 8 * tpw = 24
    int tpw;         // row tiles per wave (template instance)
    int r_pad;       // row_tiles * 16
    int heads;       // workgroups per item: n_kv * row_groups
    int max_items;   // upper bound of the item count, from the host-side length bound
};

static AttnPlan plan_attention(int B, int n, int G, int n_kv, int bound_total) {
    AttnPlan p;
    p.row_tiles = (n * G + 15) / 16;
    p.r_pad = p.row_tiles * 16;
    p.row_groups = (p.row_tiles + 23) / 24;
    const int per_group = (p.row_tiles + p.row_groups - 1) / p.row_groups;
    const int per_wave = (per_group + 7) / 8;
    p.tpw = per_wave <= 1 ? 1 : (per_wave <= 2 ? 2 : 3);
    p.heads = n_kv * p.row_groups;
    // items <= sum_b ceil(tiles_b / T) <= total_tiles / T + B, and the planner picks T so that they fill
    // whole rounds of 256 workgroups with T <= 64: items * heads <= 256 * ceil((total_tiles / 64 + B) * heads / 256)
    const int64_t tiles_bound = (int64_t)B * ((bound_total + kKT - 1) / kKT);
    const int64_t a = (256 + p.heads - 1) / p.heads, c = (tiles_bound + 63) / 64;
    p.max_items = 2 * B + (int)(a + c);
    return p;
}

static size_t attn_work_bytes(int B, int max_items) {
    return (sizeof(AttnWork) + (size_t)2 * B * sizeof(int) + (size_t)max_items * sizeof(AttnItem) + 255) / 256 * 256;
}

__global__ __launch_bounds__(256) void attn_plan_k(const int32_t* __restrict__ seq_len, int B, int n_region, int heads,
                                                   int max_items, AttnWork* __restrict__ work, int len_bound,
                                                   unsigned int* __restrict__ status) {
    __shared__ int s_T, s_total, s_hist[66], s_pos[66];
    int* slot0 = (int*)(work + 1);
    int* nch = slot0 + B;
    AttnItem* items = (AttnItem*)(nch + B);
    const int tid = threadIdx.x;
    if (tid < 66) s_hist[tid] = 0;
    // the grid and the item list were sized from the caller's length bound: a longer sequence would lose
    // part of its context, which only the device can see
    if (status)
        for (int b = tid; b < B; b += 256)
            if (seq_len[b] > len_bound) atomicOr(status, 1u);
    // A workgroup takes a whole CU (248 VGPRs per wave, 128 KB of LDS), so the work items run in rounds of
    // 256.  Measured at the 7B benchmark shape (attention ms per step): one round of 256 items 4.02, two
    // rounds 4.33, four 4.20, and 4.6-4.8 when the count falls between whole rounds (384, 768 items): the
    // fewest whole rounds that the 64-tile cap on a chunk allows are the target.
    __shared__ int s_count[65];   // items for every chunk size T = 8 .. 64 (one candidate per thread)
    if (tid >= 8 && tid <= 64) {
        int64_t items = 0;
        for (int b = 0; b < B; ++b) items += ((max(seq_len[b], 0) + n_region + kKT - 1) / kKT + tid - 1) / tid;
        s_count[tid] = (int)(items < 0x7fffffff / 64 ? items : 0x7fffffff / 64);
    }
    __syncthreads();
    if (tid == 0) {
        // fewest rounds first; within a round count the smallest chunk size that fits (items closest to
        // filling the rounds).  Ends at the latest when T = 64 fits, which some round count always allows.
        int64_t total = 0;
        for (int b = 0; b < B; ++b) total += (max(seq_len[b], 0) + n_region + kKT - 1) / kKT;
        int64_t r = (total * heads + 256 * 64 - 1) / (256 * 64);
        int T = 64;
        for (r = r < 1 ? 1 : r;; ++r) {
            bool found = false;
            for (int t = 8; t <= 64 && !found; ++t)
                if ((int64_t)s_count[t] * heads <= 256 * r) {
                    T = t;
                    found = true;
                }
            if (found) break;
        }
        s_T = T;
    }
    __syncthreads();
    if (tid == 0) {
        int acc = 0;
        for (int b = 0; b < B; ++b) {
            const int tiles = (max(seq_len[b], 0) + n_region + kKT - 1) / kKT;
            const int k = (tiles + s_T - 1) / s_T;
            slot0[b] = acc;
            nch[b] = k;
            acc += k;
        }
        s_total = acc < max_items ? acc : max_items;   // cannot exceed the bound when seq_len respects the host's
        work->n_items = s_total;
    }
    __syncthreads();
    // counting sort by tile count, longest first
    for (int b = tid; b < B; b += 256) {
        const int total_b = max(seq_len[b], 0) + n_region;
        const int tiles = (total_b + kKT - 1) / kKT, k = nch[b];
        const int per = k > 0 ? (tiles + k - 1) / k : 0;
        for (int j = 0; j < k; ++j) {
            const int kb = j * per * kKT, ke = min(total_b, kb + per * kKT);
            if (slot0[b] + j < max_items) atomicAdd(&s_hist[ke > kb ? (ke - kb + kKT - 1) / kKT : 0], 1);
        }
    }
    __syncthreads();
    if (tid == 0) {
        int acc = 0;
        for (int t = 65; t >= 0; --t) {
            s_pos[t] = acc;
            acc += s_hist[t];
        }
    }
    __syncthreads();
    for (int b = tid; b < B; b += 256) {
        const int total_b = max(seq_len[b], 0) + n_region;
        const int tiles = (total_b + kKT - 1) / kKT, k = nch[b];
        const int per = k > 0 ? (tiles + k - 1) / k : 0;
        for (int j = 0; j < k; ++j) {
            const int kb = j * per * kKT, ke = min(total_b, kb + per * kKT);
            if (slot0[b] + j >= max_items) continue;
            const int pos = atomicAdd(&s_pos[ke > kb ? (ke - kb + kKT - 1) / kKT : 0], 1);
            items[pos] = AttnItem{b, kb, ke, slot0[b] + j};
        }
    }
}

// (non-temporal: a key or value row is read by one workgroup, or by the row groups of one work item at the same
// time, and not again before the next step; marked so, the stream leaves more of the caches to the activations and
// partial results around it: drafter attention 0.59 -> 0.48 ms per step, the step 0.3-0.5 % shorter, same box,
// alternating libraries)
__device__ __forceinline__ void dma_buf_16(u32x4_t rsrc, uint32_t voff_bytes, uint32_t soff_bytes,
                                           uint32_t lds_bytes) {
    asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, %2 offen nt lds"
                 :
                 : "v"(voff_bytes), "s"(rsrc), "s"(soff_bytes), "s"(lds_bytes)
                 : "memory", "m0");
}
// The workgroup's program, for a wave that owns NT row tiles (tiles wave, wave + 8, ...).  Waves of one
// workgroup may run different instances (a wave whose share of the row tiles is smaller skips the
// matrix and softmax work it has no rows for; NT = 0: it only fetches its part of the K/V tiles and
// keeps the barriers): every instance passes the same barriers in the same order.
// Workgroup id -> (work item, kv head, row group).  Ids are dealt round-robin over the 8 XCDs, and the row groups of
// one (item, kv head) read the same keys and values: they get ids 8 apart, so that they run on one XCD at the same
// time and the second finds the rows in that XCD's L2.  (With one row group this is item = id / n_kv, head = id % n_kv.)
__device__ __forceinline__ void attn_decode(int id, int heads, int n_kv, int& rank, int& kh, int& rg) {
    const int per = 8 * (heads / n_kv);
    const int g = id / per, within = id - g * per;
    rg = within >> 3;
    const int q = g * 8 + (within & 7);
    rank = q / n_kv;
    kh = q - rank * n_kv;
}

template <int NT>
__device__ __forceinline__ void attn_body(const Rows& rows, const KVLayer& kv, const uint16_t* __restrict__ qkv,
                                          float* __restrict__ part_o, float* __restrict__ part_ml,
                                          const AttnWork* __restrict__ work, int heads, int n_q_heads, int row_tiles,
                                          int tiles_per_group, int r_pad, float scale_log2, float lazy_raw) {
    constexpr int TPW = NT > 0 ? NT : 1;   // array extents (nothing is computed in them when NT = 0)
    extern __shared__ __align__(16) uint16_t lds[];
    int rank, kh, rg;
    attn_decode(blockIdx.x, heads, kv.n_kv, rank, kh, rg);
    if (rank >= work->n_items) return;  // uniform
    const AttnItem item = ((const AttnItem*)((const int*)(work + 1) + 2 * rows.B))[rank];
    const int b = item.b;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g4 = lane >> 4;
    const int G = n_q_heads / kv.n_kv;
    const int n = rows.n;
    const int R = n * G;
    const int k_begin = item.k_begin, k_end = item.k_end;
    if (k_begin >= k_end) return;  // uniform (an empty sequence)
    const int ctx = kv.seq_len[b];
    const int qkv_dim = (n_q_heads + 2 * kv.n_kv) * kD;
    const int nv = rows.n_valid ? min(rows.n_valid[b], n) : n;

    // ---- this wave's row tiles: Q fragments, masks, accumulators
    u32x4_t qf[TPW][4];
    int row_i[TPW];
    bool tile_on[TPW];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int tile = rg * tiles_per_group + wave + 8 * t;
        tile_on[t] = (wave + 8 * t) < tiles_per_group && tile < row_tiles;
        const int r = tile * 16 + l16;
        const int i = r / G, gq = r - i * G;
        const bool valid = tile_on[t] && r < R && i < nv;
        row_i[t] = valid ? i : -1;
        const uint16_t* qp = qkv + (int64_t)(b * n + (valid ? i : 0)) * qkv_dim + (kh * G + gq) * kD + g4 * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            u32x4_t z = {0u, 0u, 0u, 0u};
            qf[t][ks] = valid ? *(const u32x4_t*)(qp + ks * 32) : z;
        }
    }
    f32x4_t acc[TPW][8];
    float m_run[TPW];
    f32x4_t acc_l[TPW];   // running softmax denominator, accumulated by the matrix pipe (PV product against a row of ones)
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        m_run[t] = kNegBig;
        acc_l[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) acc[t][dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }

    // ---- K/V tiles: a ring of kStages LDS stages, each [64 keys][128] for K then the same for V,
    // filled by direct global->LDS loads.  One DMA instruction moves 4 keys (1 KB): lane -> key
    // lane/16 of the block, 16-byte slot lane%16, and it fetches logical chunk slot ^ swizzle(key), so a
    // row's chunks are XOR-swizzled by its key index: by key & 15 for K (the 16-byte fragment reads of 16
    // consecutive keys hit 16 distinct chunks) and by 2*key & 15 for V (a transposing read touches two
    // neighbouring chunks of each of 8 keys; with key & 15 those collided pairwise: a third of the LDS
    // cycles were bank conflicts).
    const uint16_t* kpool = (const uint16_t*)kv.k;
    const uint16_t* vpool = (const uint16_t*)kv.v;
    int32_t* page_ids = (int32_t*)(lds + kStages * kStageElems);
    uint64_t* mask_lds = (uint64_t*)(page_ids + kMaxChunk / 16 + 2);  // [n][2] visibility bits of this sequence's rows
    {
        for (int i = tid; i < n; i += 512) {
            uint64_t m0 = 0, m1 = 0;
            if (i < nv) {
                if (rows.mask) {
                    const uint64_t* mp = rows.mask + (int64_t)(b * n + i) * rows.mask_words;
                    m0 = mp[0];
                    m1 = rows.mask_words > 1 ? mp[1] : 0ull;
                } else {  // causal within the new rows
                    m0 = i >= 63 ? ~0ull : ((2ull << i) - 1ull);
                    m1 = i < 64 ? 0ull : (i >= 127 ? ~0ull : ((2ull << (i - 64)) - 1ull));
                }
            }
            mask_lds[2 * i] = m0;
            mask_lds[2 * i + 1] = m1;
        }
        // page ids of this chunk, range-checked once (-1 = not backed by the block table)
        const int first_page = k_begin / kv.page_size;
        const int n_pg = (k_end - 1) / kv.page_size - first_page + 1;
        int unbacked = 0;
        for (int pi = tid; pi < n_pg; pi += 512) {
            const int lp = first_page + pi;
            int pg = lp < kv.max_pages ? kv.block_table[(int64_t)b * kv.max_pages + lp] : -1;
            pg = (pg >= 0 && pg < kv.n_pages) ? pg : -1;
            page_ids[pi] = pg;
            unbacked |= pg < 0;
        }
        // slots whose DMA is skipped (unbacked pages: a caller error) must still hold finite values:
        // only then is the ring zeroed first
        if (__syncthreads_or(unbacked)) {
            u32x4_t z = {0u, 0u, 0u, 0u};
            for (int e = tid; e < kStages * kStageElems / 8; e += 512) *(u32x4_t*)(lds + e * 8) = z;
        }
    }
    __syncthreads();
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int n_tiles = (k_end - k_begin + kKT - 1) / kKT;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t*)lds;
    // Every DMA instruction of a wave covers 4 consecutive keys of one page, so the page, the source
    // address and the range check are wave-uniform: they live in scalar registers (a raw buffer
    // descriptor per instruction: base = the block's first key, size = the block, or 0 for a page the
    // block table does not back, which makes every lane out of range: nothing is fetched), and a lane
    // contributes only its constant offset inside the block.
    uint32_t ck[2], cv[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int key_t = (wave_u + 8 * e) * 4 + (lane >> 4);   // key slot inside the tile
        // logical 16-byte chunk this lane fetches: K rows are swizzled by the key slot (the 16 keys of
        // a QK^T fragment read then hit 16 distinct chunks), V rows by twice the key slot (a
        // transposing V read takes two neighbouring chunks of each of 8 keys: they stay distinct)
        ck[e] = (uint32_t)(((lane & 15) ^ (key_t & 15)) * 16);
        cv[e] = (uint32_t)(((lane & 15) ^ ((2 * key_t) & 15)) * 16);
    }
    const uint32_t kq = (uint32_t)lane >> 4;
    auto desc = [&](const uint16_t* base, uint32_t bytes) {
        const uint64_t p = (uint64_t)(uintptr_t)base;
        u32x4_t d;
        d[0] = __builtin_amdgcn_readfirstlane((uint32_t)p);
        d[1] = __builtin_amdgcn_readfirstlane((uint32_t)(p >> 32) & 0xffffu);
        d[2] = __builtin_amdgcn_readfirstlane(bytes);
        d[3] = 0x00020000u;
        return d;
    };
    auto issue_dma = [&](int tile, int stage) {
        const int t0 = k_begin + tile * kKT;
        const int last = k_end - 1;
        int kb[2], pgv[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            int k0 = t0 + (wave_u + 8 * e) * 4;             // first key of the 4-key block
            k0 = k0 <= last ? k0 : (last & ~3);             // blocks past the end re-read the last key's block
            kb[e] = k0;
            pgv[e] = page_ids[(k0 - k_begin) >> 4];         // page_size is 16 for this kernel
        }
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int blk = wave_u + 8 * e;
            const int pg = __builtin_amdgcn_readfirstlane(pgv[e]);
            const int lim = min(3, last - kb[e]);           // keys past the end re-read the last key (masked later)
            const int64_t off = (((int64_t)(pg < 0 ? 0 : pg) * kv.n_kv + kh) * 16 + (kb[e] & 15)) * kD;
            const uint32_t size = pg >= 0 ? 1024u : 0u;
            const uint32_t row = min(kq, (uint32_t)lim) << 8;
            const uint32_t dst = lds_base + (uint32_t)(stage * kStageElems + blk * 512) * 2u;
            dma_buf_16(desc(kpool + off, size), row | ck[e], 0u, dst);
            dma_buf_16(desc(vpool + off, size), row | cv[e], 0u, dst + kKT * kD * 2u);
        }
    };
#pragma unroll
    for (int st = 0; st < kAhead; ++st) issue_dma(st < n_tiles ? st : n_tiles - 1, st);

    // Drain every load issued so far (Q fragments, table reads, the first DMAs) once, here, so that the
    // compiler's own wait bookkeeping enters the loop clean and adds no vmcnt(0) of its own inside it,
    // which would also drain the DMA queue on every tile.
    __builtin_amdgcn_s_waitcnt(0x0F70u);
    // P of the tile whose PV product is still owed (packed bf16, the second product's B operand)
    u32x4_t pb[TPW][2];
#pragma unroll
    for (int t = 0; t < NT; ++t) pb[t][0] = pb[t][1] = u32x4_t{0u, 0u, 0u, 0u};
    auto pv_step = [&](const uint16_t* vt) {
        if constexpr (NT == 0) return;
        // ---- O^T += V^T P^T.  V stays row-major in LDS; ds_read_b64_tr_b16 hands lane (l16, g4) the
        // four keys 4*g4 .. 4*g4+3 of a 16-key sub-tile for head dimension 16*dt + l16: the 16 lanes of
        // a group address a 4-key x 16-dim block (lane s -> key s/4, dims 4*(s%4) ..) and the
        // instruction transposes it.  Two such reads (sub-tiles 2*half, 2*half+1) form the 8 k-slots.
        // Four batches (key half, dimension half) of 8 reads + 4*TPW MFMAs; a batch's reads are issued
        // before the MFMAs of the batch in front of it.
        typedef __attribute__((ext_vector_type(4))) short s16x4_t;
        typedef __attribute__((ext_vector_type(8))) short s16x8_t;
        s16x4_t vv[2][4][2];
        auto read_v = [&](int half, int dq, s16x4_t (*v)[2]) {
#pragma unroll
            for (int d4 = 0; d4 < 4; ++d4)
#pragma unroll
                for (int sub = 0; sub < 2; ++sub) {
                    const int dt = dq * 4 + d4;
                    const int key_t = half * 32 + sub * 16 + 4 * g4 + (l16 >> 2);
                    const int lcv = 2 * dt + ((l16 & 3) >> 1);
                    const uint16_t* vp = vt + key_t * kD + ((lcv ^ ((2 * key_t) & 15)) * 8) + (l16 & 1) * 4;
                    v[d4][sub] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)vp);
                }
        };
        auto mul_v = [&](int half, int dq, s16x4_t (*v)[2]) {
            if (dq == 0) {   // denominator: the same product against a V^T row of ones (bf16 1.0 = 0x3f80)
                const s16x8_t one8 = {0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80};
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc_l[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, one8),
                                                                      __builtin_bit_cast(bf16x8_t, pb[t][half]),
                                                                      acc_l[t], 0, 0, 0);
            }
#pragma unroll
            for (int d4 = 0; d4 < 4; ++d4) {
                const int dt = dq * 4 + d4;
                s16x8_t v8 = {v[d4][0][0], v[d4][0][1], v[d4][0][2], v[d4][0][3],
                              v[d4][1][0], v[d4][1][1], v[d4][1][2], v[d4][1][3]};
                bf16x8_t a = __builtin_bit_cast(bf16x8_t, v8);
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8_t, pb[t][half]),
                                                                        acc[t][dt], 0, 0, 0);
            }
        };
        read_v(0, 0, vv[0]);
        read_v(0, 1, vv[1]);
        mul_v(0, 0, vv[0]);
        read_v(1, 0, vv[0]);
        mul_v(0, 1, vv[1]);
        read_v(1, 1, vv[1]);
        mul_v(1, 0, vv[0]);
        mul_v(1, 1, vv[1]);
        __builtin_amdgcn_sched_group_barrier(0x100, 16, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 5 * NT, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 4 * NT, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 9 * NT, 0);
    };
    // The two waves that share a SIMD (w and w + 4) run the loop half a period apart, so that one's
    // softmax (VALU) runs under the other's two matrix products instead of both doing the same thing
    // at the same time.  Per tile a wave does [PV of the previous tile, S = QK^T] (matrix pipe) and then
    // [softmax] (VALU), two halves of about equal length.  The early waves 0..3 meet the tile barrier at
    // the top of the iteration, before the matrix half; the late waves 4..7 meet the same barrier
    // between their two halves, after QK^T of the tile before.  After each release the early wave of a
    // SIMD therefore multiplies while the late one exponentiates, and the other way round in the second
    // half of the period (measured with cycle stamps: with the late waves' barrier at the top as well,
    // one phase apart only, both multiplied at once and the late wave's softmax ran while the early
    // one sat at the barrier, 5700 against 5200 clocks per tile).  A wave raises its issue priority for
    // its matrix half: a late MFMA costs the pipe, a late exp only the wave that waits for it.
    // Barrier number it guarantees tile it has landed (every wave waited for its own DMAs first) and
    // that nobody reads stage (it - 2) % kStages any more, which is where the fetch issued after it
    // (tile it + 2) lands: the early waves read V of tile it-2 before barrier it, the late ones in the
    // iteration that ended with it.  Both kinds pass exactly n_tiles barriers.
    const bool late = wave_u >= 4;
    auto tile_wait = [&](int it) {
        __builtin_amdgcn_s_waitcnt(0x0F70u | (4 * (kAhead - 1)));  // vmcnt: this tile's 4 DMAs per wave have landed
        __builtin_amdgcn_s_barrier();
    };
    auto tile_fetch = [&](int it) {
        const int nxt = it + kAhead;
        issue_dma(nxt < n_tiles ? nxt : n_tiles - 1, nxt % kStages);
    };
    if (late) tile_wait(0);
    for (int it = 0; it < n_tiles; ++it) {
        if (!late) tile_wait(it);
        tile_fetch(it);
        __builtin_amdgcn_s_setprio(2);
        if (it > 0) pv_step(lds + ((it - 1) % kStages) * kStageElems + kKT * kD);
        const int t0 = k_begin + it * kKT;
        const uint16_t* kt = lds + (it % kStages) * kStageElems;
        // 1 for the tile(s) touching the tree region or the chunk's tail, else 0.  Used as the trip count
        // of the masking loop below: a loop with a uniform run-time bound stays a real branch, whereas an
        // `if` around this much select-able code gets flattened and would run on every tile.
        const int mask_reps = t0 + kKT > ctx ? 1 : 0;

        // ---- S^T = K Q^T: each K fragment is read once and feeds the TPW independent row tiles.  The
        // LDS reads are issued in batches of 4 fragments ahead of the 4*TPW MFMAs that consume them, so
        // one LDS latency is exposed per batch instead of one per fragment.
        f32x4_t scs[TPW][4];
        bf16x8_t kf[2][4];
        auto read_k = [&](int st, bf16x8_t* f) {
            const uint16_t* kp = kt + (st * 16 + l16) * kD;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                f[ks] = __builtin_bit_cast(bf16x8_t, *(const u32x4_t*)(kp + (((4 * ks + g4) ^ l16) * 8)));
        };
        auto mul_k = [&](int st, const bf16x8_t* f) {
#pragma unroll
            for (int t = 0; t < NT; ++t) scs[t][st] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    scs[t][st] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[ks], __builtin_bit_cast(bf16x8_t, qf[t][ks]),
                                                                         scs[t][st], 0, 0, 0);
        };
        // the next 16 keys' fragments fly under each batch's MFMAs: order = 8 reads, then
        // (12 MFMAs, 4 reads) twice, then the last two batches of MFMAs
        if constexpr (NT > 0) {
            read_k(0, kf[0]);
            read_k(1, kf[1]);
            mul_k(0, kf[0]);
            read_k(2, kf[0]);
            mul_k(1, kf[1]);
            read_k(3, kf[1]);
            mul_k(2, kf[0]);
            mul_k(3, kf[1]);
            __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 4 * NT, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 4 * NT, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 8 * NT, 0);
        }
        __builtin_amdgcn_s_setprio(0);
        if (late && it + 1 < n_tiles) tile_wait(it + 1);
        // ---- per row tile: online softmax, P packed straight into the second product's B operand
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            f32x4_t sc[4];
#pragma unroll
            for (int st = 0; st < 4; ++st) sc[st] = scs[t][st];
            float tmax = kNegBig;
            for (int rep = 0; rep < mask_reps; ++rep) {  // region / tail tile only (see mask_reps)
                uint64_t m0 = 0, m1 = 0;
                const int i = row_i[t];
                if (i >= 0) {  // from the LDS copy: no global load (and so no vmcnt wait) inside the loop
                    m0 = mask_lds[2 * i];
                    m1 = mask_lds[2 * i + 1];
                }
#pragma unroll
                for (int st = 0; st < 4; ++st)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int key = t0 + st * 16 + g4 * 4 + v;
                        const int jj = key - ctx;  // index into the masked region when >= 0
                        const uint64_t w = jj < 64 ? m0 : m1;
                        const bool bit = (w >> (jj & 63)) & 1ull;
                        const bool vis = (i >= 0) & (key < k_end) & ((jj < 0) | (bit & (jj < 128)));
                        sc[st][v] = vis ? sc[st][v] : kNegBig;
                    }
            }
#pragma unroll
            for (int st = 0; st < 4; ++st)
#pragma unroll
                for (int v = 0; v < 4; ++v) tmax = fmaxf(tmax, sc[st][v]);
            // Lazy running maximum: softmax is invariant to the reference value, which only has to keep
            // exp2 in range.  As long as no score of this tile exceeds the reference in use by more than
            // 2^8 in the exponent (P <= 256: harmless in bf16 and in the fp32 sums), it stays, and the
            // rescaling of the accumulators (33 multiplies per row tile), the exp of the correction and the
            // cross-lane maximum are all skipped; the decision is taken per wave.
            if (__builtin_amdgcn_ballot_w64(tmax > m_run[t] + lazy_raw) != 0) {
                tmax = group_max4(tmax);
                const float m_new = fmaxf(m_run[t], tmax);
                const float alpha = __builtin_amdgcn_exp2f((m_run[t] - m_new) * scale_log2);
                m_run[t] = m_new;
                acc_l[t] *= alpha;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) acc[t][dt] *= alpha;
            }
            // the clamp keeps exp2(x*c - mc) = 0 for masked scores (-1e30) while no key has been visible yet
            const float mc = fmaxf(m_run[t], -1e29f) * scale_log2;
            uint32_t pk[4][2];
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                float pv[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float x = sc[st][v];
                    float e = __builtin_amdgcn_exp2f(fmaf(x, scale_log2, -mc));
                    pv[v] = e;
                }
                pk[st][0] = pack_bf16x2(pv[0], pv[1]);
                pk[st][1] = pack_bf16x2(pv[2], pv[3]);
            }
            pb[t][0] = u32x4_t{pk[0][0], pk[0][1], pk[1][0], pk[1][1]};
            pb[t][1] = u32x4_t{pk[2][0], pk[2][1], pk[3][0], pk[3][1]};
        }
    }
    pv_step(lds + ((n_tiles - 1) % kStages) * kStageElems + kKT * kD);
    __builtin_amdgcn_s_waitcnt(0x0F70u);  // drain the redundant tail DMAs before the LDS is released

    // ---- partial results: part_o [slot][n_kv][r_pad][128], part_ml [..][r_pad][2]
    const int64_t pbase = ((int64_t)item.slot * kv.n_kv + kh) * r_pad;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        if (!tile_on[t]) continue;
        const int tile = rg * tiles_per_group + wave + 8 * t;
        const int r = tile * 16 + l16;
        const float l = acc_l[t][0];   // every lane of the row holds the full sum
        float* po = part_o + (pbase + r) * kD;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) *(f32x4_t*)(po + dt * 16 + g4 * 4) = acc[t][dt];
        if (g4 == 0) {
            part_ml[(pbase + r) * 2] = m_run[t];
            part_ml[(pbase + r) * 2 + 1] = l;
        }
    }
}

template <int TPW>
__global__ __launch_bounds__(512) void attn_mfma_k(Rows rows, KVLayer kv, const uint16_t* __restrict__ qkv,
                                                   float* __restrict__ part_o, float* __restrict__ part_ml,
                                                   const AttnWork* __restrict__ work, int heads, int n_q_heads,
                                                   int row_tiles, int tiles_per_group, int r_pad, float scale_log2,
                                                   float lazy_raw) {
    // row tiles of this wave that exist (tile indices rise with t, so they are the first n_on)
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    int rank_, kh_, rg;
    attn_decode(blockIdx.x, heads, kv.n_kv, rank_, kh_, rg);
    int n_on = 0;
#pragma unroll
    for (int t = 0; t < TPW; ++t)
        n_on += ((wave + 8 * t) < tiles_per_group && rg * tiles_per_group + wave + 8 * t < row_tiles) ? 1 : 0;
#define TLT_BODY(N) attn_body<N>(rows, kv, qkv, part_o, part_ml, work, heads, n_q_heads, row_tiles, tiles_per_group, r_pad, scale_log2, lazy_raw)
    if (n_on >= TPW) TLT_BODY(TPW);
    else if (TPW >= 2 && n_on == TPW - 1) TLT_BODY((TPW >= 2 ? TPW - 1 : 0));
    else if (TPW >= 3 && n_on == TPW - 2) TLT_BODY((TPW >= 3 ? TPW - 2 : 0));
    else TLT_BODY(0);
#undef TLT_BODY
}

// One wave per (b, kv head, row), four rows per workgroup: merges the chunks' partial outputs
// (running max in raw score units).
// BATCH: the loads of four chunks are issued before any of them is used.  With few rows in all (plain decoding, small
// batches) a wave's chunks, one load latency each, are the whole kernel (12 -> 5 us at batch 1, 16 chunks); with the
// chip full of waves the plain loop is the faster one (14 against 16 us at the benchmark shape).  The sums run in
// chunk order either way.
template <bool BATCH>
__global__ __launch_bounds__(256) void attn_combine_k(Rows rows, KVLayer kv, const float* __restrict__ part_o,
                                                     const float* __restrict__ part_ml, uint16_t* __restrict__ out,
                                                     const AttnWork* __restrict__ work, int n_q_heads, int max_items,
                                                     int r_pad, float scale_log2) {
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6), kh = blockIdx.y, b = blockIdx.z, lane = threadIdx.x & 63;
    const int G = n_q_heads / kv.n_kv;
    const int n = rows.n;
    if (r >= n * G) return;  // wave-uniform
    const int i = r / G, gq = r - i * G;
    const int nv = rows.n_valid ? min(rows.n_valid[b], n) : n;
    uint32_t* o = (uint32_t*)(out + ((int64_t)(b * n + i) * n_q_heads + kh * G + gq) * kD);
    const int* slot0 = (const int*)(work + 1);
    const int first = slot0[b];
    int used = slot0[rows.B + b];
    if (first + used > max_items) used = max(max_items - first, 0);
    if (i >= nv || used <= 0) {
        o[lane] = 0u;
        return;
    }
    const int64_t pbase = ((int64_t)first * kv.n_kv + kh) * r_pad + r;
    const int64_t pstride = (int64_t)kv.n_kv * r_pad;
    float M = kNegBig;
    float a0 = 0.f, a1 = 0.f, L = 0.f;
    if constexpr (BATCH) {
        for (int c0 = 0; c0 < used; c0 += 4) {
            float m4[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) m4[u] = c0 + u < used ? part_ml[(pbase + (c0 + u) * pstride) * 2] : kNegBig;
#pragma unroll
            for (int u = 0; u < 4; ++u) M = fmaxf(M, m4[u]);
        }
        for (int c0 = 0; c0 < used; c0 += 4) {
            float2 ml4[4], v4[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t pr = pbase + (c0 + u) * pstride;
                const bool on = c0 + u < used;
                ml4[u] = on ? *(const float2*)(part_ml + pr * 2) : make_float2(kNegBig, 0.f);
                v4[u] = on ? *(const float2*)(part_o + pr * kD + lane * 2) : make_float2(0.f, 0.f);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (c0 + u < used) {   // wave-uniform
                    const float w = exp2f((ml4[u].x - M) * scale_log2);
                    L += ml4[u].y * w;
                    a0 += v4[u].x * w;
                    a1 += v4[u].y * w;
                }
            }
        }
    } else {
    for (int c = 0; c < used; ++c) M = fmaxf(M, part_ml[(pbase + c * pstride) * 2]);
    for (int c = 0; c < used; ++c) {
        const int64_t pr = pbase + c * pstride;
        const float w = exp2f((part_ml[pr * 2] - M) * scale_log2);
        L += part_ml[pr * 2 + 1] * w;
        const float2 v = *(const float2*)(part_o + pr * kD + lane * 2);
        a0 += v.x * w;
        a1 += v.y * w;
    }
    }
    const float inv = L > 0.f ? 1.0f / L : 0.f;
    o[lane] = pack_bf16x2(a0 * inv, a1 * inv);
}

static size_t attn_need_bytes(int B, const AttnPlan& p, int n_kv) {
    return attn_work_bytes(B, p.max_items) + (size_t)p.max_items * n_kv * p.r_pad * (kD + 2) * sizeof(float);
}

size_t attention_workspace_bytes(int B, int n, int n_q_heads, int n_kv_heads, int d, int max_ctx) {
    if (d != kD) return 256;
    const int G = n_q_heads / n_kv_heads;
    size_t need = 0;   // any row count up to n may be asked for later
    for (int m = 1; m <= n; ++m) {
        const AttnPlan p = plan_attention(B, m, G, n_kv_heads, max_ctx + 128);
        const size_t x = attn_need_bytes(B, p, n_kv_heads);
        need = x > need ? x : need;
    }
    return need + 256;
}

template <int TPW>
static hipError_t launch_attn_mfma(hipStream_t s, const Rows& rows, const KVLayer& kv, const void* qkv, void* out,
                                   int n_q_heads, const AttnPlan& p, AttnWork* work, float* part_o, float* part_ml,
                                   bool reuse_plan, unsigned int* status) {
    const size_t lds = (size_t)kStages * kStageElems * sizeof(uint16_t) + (kMaxChunk / 16 + 2) * sizeof(int32_t) +
                       (size_t)kMaxRows * 2 * sizeof(uint64_t);
    if (rows.n > kMaxRows) return hipErrorInvalidValue;
    auto kern = attn_mfma_k<TPW>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_per_group = (p.row_tiles + p.row_groups - 1) / p.row_groups;
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)kD);
    if (!reuse_plan)
        hipLaunchKernelGGL(attn_plan_k, dim3(1), dim3(256), 0, s, kv.seq_len, rows.B, rows.n_region, p.heads, p.max_items, work,
                           kv.seq_len_bound, status);
    // (ids come in groups of 8 (item, kv head) pairs x row groups: see attn_decode)
    const int id_groups = (p.max_items * kv.n_kv + 7) / 8;
    hipLaunchKernelGGL(kern, dim3(id_groups * 8 * p.row_groups), dim3(512), lds, s, rows, kv, (const uint16_t*)qkv, part_o,
                       part_ml, work, p.heads, n_q_heads, p.row_tiles, tiles_per_group, p.r_pad, scale_log2,
                       8.0f / scale_log2);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int R = rows.n * (n_q_heads / kv.n_kv);
    if ((int64_t)R * kv.n_kv * rows.B <= 4096)   // (waves: half of what the chip holds at once)
        hipLaunchKernelGGL(attn_combine_k<true>, dim3((R + 3) / 4, kv.n_kv, rows.B), dim3(256), 0, s, rows, kv, part_o, part_ml,
                           (uint16_t*)out, work, n_q_heads, p.max_items, p.r_pad, scale_log2);
    else
        hipLaunchKernelGGL(attn_combine_k<false>, dim3((R + 3) / 4, kv.n_kv, rows.B), dim3(256), 0, s, rows, kv, part_o, part_ml,
                           (uint16_t*)out, work, n_q_heads, p.max_items, p.r_pad, scale_log2);
    return hipGetLastError();
}

hipError_t attention(hipStream_t s, int dtype, const Rows& rows, const KVLayer& kv, const void* qkv, void* out,
                     int n_q_heads, void* ws, size_t ws_bytes, int impl, bool reuse_plan, unsigned int* status) {
    if (rows.B * rows.n <= 0) return hipSuccess;
    if (kv.d % 64 != 0 || kv.d > 256) return hipErrorInvalidValue;
    const int G = n_q_heads / kv.n_kv;
    const bool mfma_ok = dtype == BF16 && kv.d == kD && rows.n_region <= 128 && kv.page_size == 16;
    if (mfma_ok && impl != 0) {
        const AttnPlan p = plan_attention(rows.B, rows.n, G, kv.n_kv, kv.seq_len_bound + rows.n_region);
        if (attn_need_bytes(rows.B, p, kv.n_kv) <= ws_bytes) {
            AttnWork* work = (AttnWork*)ws;
            float* part_o = (float*)((char*)ws + attn_work_bytes(rows.B, p.max_items));
            float* part_ml = part_o + (size_t)p.max_items * kv.n_kv * p.r_pad * kD;
            switch (p.tpw) {
                case 1: return launch_attn_mfma<1>(s, rows, kv, qkv, out, n_q_heads, p, work, part_o, part_ml, reuse_plan, status);
                case 2: return launch_attn_mfma<2>(s, rows, kv, qkv, out, n_q_heads, p, work, part_o, part_ml, reuse_plan, status);
                default: return launch_attn_mfma<3>(s, rows, kv, qkv, out, n_q_heads, p, work, part_o, part_ml, reuse_plan, status);
            }
        }
        if (impl == 1) return hipErrorInvalidValue;  // explicitly requested but the workspace cannot hold it
    }
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
