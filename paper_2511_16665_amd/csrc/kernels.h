// Host-side launchers of the HIP kernels behind libtlt's C ABI.  Internal header.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace tlt {

enum { F32 = 0, BF16 = 1 };
enum {
    OUT_T = 0,
    OUT_F32 = 1,
    OUT_ADD_F32 = 2,
    OUT_ATOMIC_ADD_F32 = 3, /* internal: split-K partial sums */
    OUT_ROWMAX = 4,         /* internal: per-row (max, argmax) of every 128-column block instead of C */
    OUT_SPLIT_F32 = 5       /* internal: every K split stores its fp32 partial product to a slice of its own */
};

// Rows of a layer forward, laid out [B][n].  Row (b, i) is active when i < n_valid[b] (all rows
// when n_valid is null).  Its rotary position is seq_len[b] + pos_base + (pos_off ? pos_off[b*n+i]
// : pos_stride*i); its key/value go to cache slot seq_len[b] + slot_base + i.  It attends to every
// slot < seq_len[b] and to region slot seq_len[b] + j (j < n_region) when bit j of its mask is set;
// a null mask means causal within the rows (bit j set for j <= i, with slot_base = 0).
struct Rows {
    int B = 0, n = 0;
    const int32_t* n_valid = nullptr;
    const int32_t* pos_off = nullptr;
    int pos_base = 0, pos_stride = 0;
    int slot_base = 0;
    const uint64_t* mask = nullptr;
    int mask_words = 1;
    int n_region = 0;
};

struct KVLayer {
    void* k = nullptr;  // this layer's [n_pages][n_kv][page][d]
    void* v = nullptr;
    int64_t n_pages = 0;
    const int32_t* block_table = nullptr;
    const int32_t* seq_len = nullptr;
    int max_pages = 0, page_size = 16, n_kv = 0, d = 0;
    int seq_len_bound = 0;
};

// ---- gemm.hip
hipError_t gemm(hipStream_t s, int dtype, int out_mode, int M, int N, int K, const void* A, const void* W, void* C);
// The product as a sum of partial products: parts [n][M][N] fp32 with sum_k parts[k] = A W^T, n >= 1 returned in
// *n_parts.  Products with too few tiles for the chip and a long K are cut along K over several workgroups
// per tile, each storing its partial product to a slice of its own (plain stores, every element of every
// slice is written: nothing has to be cleared, and the sum the consumer forms is the same on every run);
// all others are one plain fp32 product (n = 1).  parts_bytes bounds n * M * N * 4.
hipError_t gemm_parts(hipStream_t s, int dtype, int M, int N, int K, const void* A, const void* W, float* parts,
                      size_t parts_bytes, int* n_parts);
// upper bound of n * M * N * 4 over every shape (see gemm.hip)
size_t gemm_parts_max_bytes();
bool gemm_parts_pays(int dtype, int M, int N, int K);   // slices expected to beat one result in the model dtype
// fused gate/up projection of the SwiGLU MLP (bf16 MFMA path only): act = silu(A Wg^T) * (A Wu^T)
bool gemm_glu_supported(int dtype, int M, int N, int K, const void* A, const void* Wg, const void* Wu);
hipError_t gemm_glu(hipStream_t s, int M, int N, int K, const void* A, const void* Wg, const void* Wu, void* act);

// argmax over each row of A W^T without writing the product (the LM head when only the most likely
// token is wanted): the GEMM's epilogue leaves the best (value, column) of every 128-column block,
// a second kernel picks the best block; lowest column on ties, as row_argmax on the stored product.
// Call only when gemm_argmax_supported(); ws holds gemm_argmax_workspace_bytes(M, N) bytes.
bool gemm_argmax_supported(int dtype, int M, int N, int K, const void* A, const void* W);
size_t gemm_argmax_workspace_bytes(int M, int N);
hipError_t gemm_argmax(hipStream_t s, int M, int N, int K, const void* A, const void* W, void* ws, int32_t* out);
// Measurement aid: kMfmaStreamBlocks workgroups of 4 waves, each wave `iters` times the 64 MFMAs (32x32x16 bf16) of a
// 128x128x64 wave tile on the 32 fragments x 64 lanes x 16 bytes at `frags`; out[kMfmaStreamBlocks * 256] = every
// lane's sum of its accumulators.
constexpr int kMfmaStreamBlocks = 256;
hipError_t mfma_stream(hipStream_t s, const void* frags, float* out, int iters);

// ---- elementwise.hip
hipError_t embed_rows(hipStream_t s, int dtype, int M, int h, int V, const int32_t* tokens, const void* embed, float* x);
// out[r] = rmsnorm(x[row_map ? row_map[r] : r]) * gamma, stored in dtype.  Rows with row_map < 0 give zeros.
// zero (optional): a second fp32 buffer [M][zero_n] cleared row by row in the same launch.
hipError_t rmsnorm(hipStream_t s, int dtype, int M, int h, const float* x, const void* gamma, float eps, void* out,
                   const int32_t* row_map, float* zero = nullptr, int zero_n = 0);
// x[r] += sum_k add[k][r] (add [n_add][M][h] in fp32 when add_f32, else one [M][h] in dtype; assign: x[r] = that sum
// instead), then out[r] = rmsnorm(x[r]) * gamma.  The sum runs in the order k = 0, 1, ...: reproducible.
hipError_t rmsnorm_add(hipStream_t s, int dtype, int M, int h, float* x, const void* add, bool add_f32, const void* gamma,
                       float eps, void* out, int n_add = 1, bool assign = false);
// x += sum_k parts[k] (or x = with assign), count floats each (a multiple of 4)
hipError_t add_parts(hipStream_t s, int64_t count, float* x, const float* parts, int n_parts, bool assign);
// (bias: optional [(Hq+2Hkv)*d] in dtype, added to q, k and v before the rotation; src32: optional
// fp32 copy of the projection to read instead of qkv, which then only receives the rotated q)
// (src32 may hold n_src partial products [n_src][M][qkv_dim], which are summed in order)
hipError_t rope_kv_write(hipStream_t s, int dtype, const Rows& rows, const KVLayer& kv, void* qkv, int n_q_heads,
                         float theta, const void* bias, const float* src32 = nullptr, int n_src = 1);
hipError_t swiglu(hipStream_t s, int dtype, int64_t count, const void* g, const void* u, void* out);
// Rows [B][n]: xin[r] = [embed[tok[r]] ; hidden[src row]] in dtype (2h wide).  The hidden row is
// b*src_seq_stride + src[r] when src_seq_stride > 0, else src[r].  Rows with tok < 0, src < 0,
// i >= n_valid[b] or an out-of-range source give zeros.
hipError_t draft_input(hipStream_t s, int dtype, int B, int n, int h, int V, const int32_t* tok, const int32_t* src,
                       const int32_t* n_valid, int src_seq_stride, int64_t hidden_rows, const float* hidden,
                       const void* embed, void* xin);
hipError_t add_i32(hipStream_t s, int n, int32_t* dst, const int32_t* a, int add_const);
hipError_t copy_f32(hipStream_t s, int64_t count, const float* src, float* dst);
hipError_t zero_f32(hipStream_t s, int64_t count, float* dst);   // a kernel, not a memset: safe to capture in a graph
hipError_t scatter_rows(hipStream_t s, int R, int n, int h, const float* src, float* dst, int dst_seq_stride, int dst_base);
hipError_t gather_last_rows(hipStream_t s, int B, int n, int h, const int32_t* n_valid, const float* src, float* dst,
                            int dst_seq_stride);
hipError_t iota_scaled(hipStream_t s, int n, int32_t* out, int scale);

// ---- attn.hip
size_t attention_workspace_bytes(int B, int n, int n_q_heads, int n_kv_heads, int d, int max_ctx);
// status (optional): device word whose bit 0 is raised when some seq_len[b] exceeds kv.seq_len_bound (the MFMA
// kernel's work list is sized from that bound, so such a sequence would lose context rows).
hipError_t attention(hipStream_t s, int dtype, const Rows& rows, const KVLayer& kv, const void* qkv, void* out,
                     int n_q_heads, void* ws, size_t ws_bytes, int impl, bool reuse_plan = false,
                     unsigned int* status = nullptr);

// ---- sample.hip
// (scratch, may be null: 8-byte aligned device memory the call may use, M * 256 bytes at most, to spread few rows over the chip)
hipError_t row_argmax(hipStream_t s, int M, int V, const float* logits, int32_t* out, void* scratch = nullptr,
                      size_t scratch_bytes = 0);
// out [M][2]: (max, log-sum-exp) of every row
hipError_t row_lse(hipStream_t s, int M, int V, const float* logits, float* out);
// per row: log-softmax statistics and the K best (token, log-prob) pairs, best first.
size_t row_topk_workspace_bytes(int M, int V, int K);
hipError_t row_topk_logp(hipStream_t s, int M, int V, int K, const float* logits, int32_t* tok, float* logp, void* ws);

struct DraftState {  // device arrays owned by the workspace; P = pool capacity per sequence
    int P = 0;
    int32_t* pool_token = nullptr;   // [B][P]
    float* pool_score = nullptr;     // [B][P]
    int32_t* pool_parent = nullptr;  // [B][P] pool index or -1
    int32_t* pool_depth = nullptr;   // [B][P]
    int32_t* fr_token = nullptr;     // [B][K] frontier of the level about to run
    int32_t* fr_src = nullptr;       // [B][K] row of the feature buffer holding the parent's output
    int32_t* fr_pool = nullptr;      // [B][K] pool index of each frontier node
    uint64_t* fr_mask = nullptr;     // [B][K][2] visibility over provisional drafter rows
    uint64_t* pool_mask = nullptr;   // [B][P][2] mask of expanded candidates (valid for frontier members)
};
// level 0: root candidates -> pool[0..K) and first frontier (all of them, in rank order).
hipError_t draft_level0(hipStream_t s, int B, int K, const int32_t* top_tok, const float* top_logp, DraftState st,
                        int feat_rows_per_seq);
// level >= 1: K*K children of the frontier -> pool, next frontier = K best by path score.
hipError_t draft_level_select(hipStream_t s, int B, int K, int level, const int32_t* top_tok, const float* top_logp,
                              DraftState st, int feat_rows_per_seq);
hipError_t draft_prune(hipStream_t s, int B, int pool_n, int n_tree, const int32_t* root_tokens,
                       const int32_t* new_tokens, const int32_t* n_new, int new_stride, DraftState st, int32_t* token, int32_t* parent, int32_t* depth, uint64_t* anc_mask, float* score);
hipError_t tree_finalize(hipStream_t s, int B, int n, const int32_t* parent, int32_t* depth, uint64_t* anc_mask);

// ---- sampled drafting on a static template (the same for every sequence; passed by value)
struct TmplRows {   // the R template nodes one drafter pass / one sampling pass works on, per sequence
    int R = 0;
    uint8_t node[64];          // tree node index
    uint8_t first_child[64];   // its children are nodes first_child .. first_child + n_child - 1, in rank order
    uint8_t n_child[64];
    uint8_t src[64];           // feature-buffer row holding its parent's drafter output
    uint64_t mask[64];         // its visibility over the provisional drafter rows (itself and its ancestors)
};
struct TmplParents {
    int8_t parent[64];
};
// token[b][0] = root (root_tokens, or the last new token), parent[b][i] = template parent, score = 0.
hipError_t tmpl_tree_init(hipStream_t s, int B, int n, TmplParents tp, const int32_t* root_tokens, const int32_t* new_tokens,
                          const int32_t* n_new, int new_stride, int32_t* token, int32_t* parent, float* score);
// drafter input rows of one level: token of each node, feature row of its parent, visibility mask.
hipError_t tmpl_level_rows(hipStream_t s, int B, int n, TmplRows rows, const int32_t* token, int32_t* fr_token, int32_t* fr_src,
                           uint64_t* fr_mask);
// per row (b, r): q[b][node] = softmax(logits[b*R + r] / temperature); then the node's children are
// drawn from it one after the other without replacement with the uniforms u_draw[b][child].
// scratch (may be null): device memory the call may use, 8-byte aligned; with few rows and enough of it
// (B*R * (V/256 + 32) * 8 bytes) a row's softmax is spread over several workgroups.
hipError_t softmax_draw(hipStream_t s, int B, int n, int V, float temperature, TmplRows rows, const float* logits,
                        const uint32_t* u_draw, int32_t* token, float* q, void* scratch, size_t scratch_bytes);

hipError_t accept_greedy(hipStream_t s, int B, int n, int V, int stride, const int32_t* token, const int32_t* parent,
                         const float* logits, const int32_t* argmax, int32_t* accept_len, int32_t* path_idx,
                         int32_t* out_tokens, int32_t* n_out);
// ws: accept_sample_workspace_bytes(B, V) bytes of scratch (16-byte aligned; contents need not be preserved or
// cleared between calls).  status: device word; bit 1 is raised if the workgroups of a sequence could not meet
// (see the kernel) and the sequence's outputs are then undefined.  n <= TLT_ACCEPT_MAX_NODES.
#define TLT_ACCEPT_MAX_NODES 64
size_t accept_sample_workspace_bytes(int B, int V);
hipError_t accept_sample(hipStream_t s, int B, int n, int V, int stride, float temperature, const int32_t* token,
                         const int32_t* parent, const float* logits, const float* draft_q, const uint32_t* u_accept,
                         const uint32_t* u_final, int32_t* accept_len, int32_t* path_idx, int32_t* out_tokens,
                         int32_t* n_out, void* ws, unsigned int* status);
hipError_t accept_target_only(hipStream_t s, int B, int n, int V, int stride, float temperature, const int32_t* token,
                              const int32_t* parent, const float* logits, const uint32_t* u_accept, const uint32_t* u_final,
                              int32_t* accept_len, int32_t* path_idx, int32_t* out_tokens, int32_t* n_out);
hipError_t kv_commit(hipStream_t s, int dtype, int B, int n_layers, void* k_pool, void* v_pool, int64_t n_pages,
                     const int32_t* block_table, int32_t* seq_len, int max_pages, int page_size, int n_kv, int d,
                     const int32_t* accept_len, const int32_t* path_idx, int stride);

}  // namespace tlt
