/* libtlt: the speculative-decoding step of a long-tail rollout on one MI355X (gfx950).
 *
 * One step = drafter tree expansion -> target verification forward -> lossless acceptance ->
 * commit of the accepted path into the paged KV cache (the rollout workflow steps 1-4 of the
 * paper's system overview, Section 3 "Architecture & Workflow"; the mechanism is stated in
 * Section 2.2 "Mechanism of Speculative Decoding").
 *
 * Conventions
 *  - Plain C ABI.  Every pointer is either HOST or DEVICE memory as marked.  The caller owns all
 *    device memory (weights, KV pools, block tables, workspace, inputs, outputs); the context
 *    owns only host-side descriptors.  No entry point allocates or frees device memory.
 *  - Every entry point enqueues its kernels on the caller's stream (`hipStream_t` passed as
 *    void*) and returns without waiting; outputs are valid once that stream has been synchronised.
 *  - Return value: TLT_OK or a negative error code; nothing has been enqueued when an error code
 *    other than TLT_EHIP is returned.  Host-side arguments are validated; device contents
 *    (page ids, lengths) are additionally range-checked inside the kernels, which skip a row
 *    rather than touch memory outside the pools.
 *  - Matrices are row-major [out_features][in_features].  `dtype` selects the storage type of
 *    weights, KV cache and intermediate activations (fp32 or bf16); accumulation, the residual
 *    stream, softmax, logits and hidden-state outputs are always fp32.
 *  - Shapes: B sequences, n tree nodes per sequence (node 0 = root = last emitted token, not yet
 *    in the cache; parents precede children), h = hidden, V = vocab.
 */
#ifndef TLT_H
#define TLT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    TLT_OK = 0,
    TLT_EINVAL = -1,   /* NULL / out-of-range argument */
    TLT_ESHAPE = -2,   /* size exceeds what tlt_create was told, or workspace too small */
    TLT_ENOPAGES = -3, /* block table cannot hold seq_len_bound + new rows */
    TLT_EHIP = -4,     /* a HIP call failed (see tlt_last_hip_error) */
    TLT_ENOTIMPL = -5,
    TLT_ESYNC = -6     /* reported by tlt_device_status: workgroups of a kernel could not meet on the device */
};

enum { TLT_F32 = 0, TLT_BF16 = 1 };
enum { TLT_MAX_TREE = 64, TLT_MAX_TOPK = 16, TLT_MAX_DEPTH = 16 };

typedef struct tlt_model_cfg {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, mlp, vocab;
    float rms_eps, rope_theta;
    int32_t dtype;     /* TLT_F32 or TLT_BF16 */
    int32_t page_size; /* tokens per KV page (16) */
} tlt_model_cfg;

/* DEVICE pointers to one decoder block's parameters, all of the model dtype.
 * wqkv [(Hq+2Hkv)*d][h] stacks q heads, k heads, v heads; wo [h][Hq*d]; wg, wu [F][h]; wd [h][F].
 * bqkv [(Hq+2Hkv)*d] is the bias of the query/key/value projections (the Qwen2.5 targets of
 * Section 6.1 have one), added before the rotary embedding; NULL = no bias. */
typedef struct tlt_layer_weights {
    const void *attn_norm, *wqkv, *wo, *mlp_norm, *wg, *wu, *wd;
    const void *bqkv;
} tlt_layer_weights;

/* embed, lm_head [V][h], final_norm [h]: DEVICE.  layers: HOST array of n_layers entries (copied by
 * tlt_create).  fc [h][2h] (DEVICE) is the drafter's input projection (columns 0..h-1 act on the
 * token embedding, h..2h-1 on the hidden state) and is NULL for the target.  The drafter reuses
 * the target's embed / lm_head / final_norm (Section 4.1 "Model Architecture"). */
typedef struct tlt_weights {
    const void *embed, *lm_head, *final_norm;
    const tlt_layer_weights *layers;
    const void *fc;
} tlt_weights;

/* Paged KV cache of one model.  k_pool, v_pool: DEVICE [n_layers][n_pages][n_kv_heads][page_size][d]
 * in the model dtype.  block_table: DEVICE [B][max_pages] page ids; slot s of sequence b lives in
 * page block_table[b][s / page_size] at row s % page_size.  seq_len: DEVICE [B] committed tokens.
 * seq_len_bound: HOST-known upper bound of max_b seq_len[b] (sizes the attention grid and is
 * checked against the block table).  A bound below some seq_len[b] is a caller error that only the
 * device can see: the call's outputs are wrong and tlt_device_status reports TLT_ESHAPE. */
typedef struct tlt_kv {
    void *k_pool, *v_pool;
    int64_t n_pages;
    const int32_t *block_table;
    int32_t *seq_len;
    int32_t max_pages;
    int32_t seq_len_bound;
} tlt_kv;

/* Token tree, DEVICE arrays [B][n] each.  anc_mask bit j of node i = node j is i or an ancestor of
 * i.  score = sum of draft log-probabilities from the root (0 for the root). */
typedef struct tlt_tree {
    int32_t *token, *parent, *depth;
    uint64_t *anc_mask;
    float *score;
    int32_t n;
} tlt_tree;

typedef struct tlt_ctx tlt_ctx;

const char *tlt_strerror(int code);
/* hipError_t value of the last failing HIP call seen by this context (0 if none). */
int tlt_last_hip_error(const tlt_ctx *ctx);

/* Bytes of DEVICE workspace needed for the given limits (max_ctx = largest seq_len_bound + n). */
size_t tlt_workspace_bytes(const tlt_model_cfg *cfg, int max_batch, int max_n, int max_depth, int max_topk,
                           int max_ctx);

/* Creates a context.  `draft` may be NULL (then tlt_draft_expand returns TLT_EINVAL).  The
 * workspace must stay allocated until tlt_destroy; calls on one context must not overlap. */
int tlt_create(tlt_ctx **out, const tlt_model_cfg *cfg, const tlt_weights *target, const tlt_weights *draft,
               int max_batch, int max_n, int max_depth, int max_topk, int max_ctx, void *workspace,
               size_t workspace_bytes);
int tlt_destroy(tlt_ctx *ctx);

/* Drafter: catch up on newly committed positions, then expand and prune the token tree
 * (Section 4.1 "Model Architecture": single decoder block fed with the target's hidden state and
 * the token embedding through a linear layer; Section 5.1 "Tree-based Drafting": topK options per
 * step for Draft_Depth steps, keep the Tokens_to_Verify most confident nodes).
 *
 * Extend: for sequence b and j < n_new[b], drafter cache entry draft_kv.seq_len[b]+j is built from
 * token new_tokens[b][j] and hidden-state row hidden[b][new_src[b][j]]; draft_kv.seq_len[b] +=
 * n_new[b].  After a step, new_tokens = tlt_accept's out_tokens, new_src = its path_idx, n_new =
 * its n_out, hidden = tlt_verify_forward's out_hidden.  0 <= n_new[b] <= new_stride <= 64; at
 * least one call with n_new[b] >= 1 must precede the first expansion of sequence b.
 * Expand (skipped when depth == 0 or out_tree == NULL): level 0 takes the topk most likely tokens
 * after the root; each further level runs the topk frontier nodes through the drafter, takes
 * each one's topk children and keeps the topk best of the topk^2 by path score as next frontier;
 * finally the n_verify-1 candidates of highest path score plus the root form the tree, in creation
 * order.  The root's token is root_tokens[b], or, when root_tokens is NULL, the last new token of
 * sequence b (new_tokens[b][n_new[b]-1]: the bonus token of the previous step).  Ties prefer the candidate created first / the lower token.
 * out_tree->n must equal min(n_verify, 1 + topk + (depth-1)*topk^2).
 * Provisional drafter entries use rows seq_len .. seq_len + (depth-1)*topk - 1 of draft_kv; there may
 * be at most 128 of them: (depth-1)*topk > 128 returns TLT_ESHAPE.
 * All pointers DEVICE except the structs themselves.  mode must be 0 (deterministic top-k); sampled
 * drafting has its own entry point, tlt_draft_sample. */
int tlt_draft_expand(tlt_ctx *ctx, void *stream, int B, int depth, int topk, int n_verify, int mode,
                     const int32_t *new_tokens, const int32_t *new_src, const int32_t *n_new, int new_stride,
                     const float *hidden, int hidden_n, const int32_t *root_tokens, tlt_kv *draft_kv,
                     tlt_tree *out_tree);

/* Read-out of the candidate pool the last tlt_draft_expand(B, depth, topk, ...) of this context left
 * in the workspace (Section 5.1: every level's topk * topk candidates stay candidates for the final
 * selection): DEVICE arrays [B][topk + (depth-1)*topk^2] in creation order (level, then the parent's
 * rank in its frontier, then the child's rank): token, parent (pool index, -1 = child of the root),
 * score (path log-probability).  For tests and inspection; enqueues device-to-device copies. */
int tlt_draft_pool(tlt_ctx *ctx, void *stream, int B, int depth, int topk, int32_t *token, int32_t *parent,
                   float *score);

/* Static tree template of sampled drafting, HOST arrays of n_verify entries each (no GPU work).
 * The paper samples its rollouts (temperature 0.9, Section 6.1) and requires the output
 * distribution to stay the target's (Section 1, Section 3 principle (a)); that only holds when the
 * shape of the tree does not depend on the drawn tokens, so the shape is fixed by the three
 * parameters of Section 5.1: of the full topk-ary tree of `depth` levels keep the n_verify-1 nodes of
 * highest prior weight prod_j 0.6 * 0.4^(r_j) (r_j = child ranks on the way down), plus the root.
 * Equal weights: the shallower node, then the smaller rank sequence.  Nodes are numbered by depth,
 * then parent number, then rank, so parents precede children and siblings are consecutive.
 * Outputs: parent (-1 for the root), rank among its siblings (-1 for the root), node_depth, and
 * *n_nodes = min(n_verify, size of the full tree + 1).  TLT_EINVAL on bad arguments. */
int tlt_template_build(int topk, int depth, int n_verify, int32_t *parent, int32_t *rank, int32_t *node_depth,
                       int32_t *n_nodes);

/* Sampled drafting on that template (the drafting half of the sampling mode; same drafter and same
 * extend step as tlt_draft_expand, whose argument meanings carry over).  For every node i that has
 * children, out_draft_q[b][i][:] = softmax(drafter logits at node i / temperature) in fp32, and
 * its children's tokens are drawn from it one after the other without replacement: with weights
 * floor(q_j * 2^32), the child with uniform U = u_draw[b][child] is the first token whose running
 * weight sum exceeds (U * total) >> 32, and its weight is then zeroed.  This is the process
 * tlt_accept's mode 1 presupposes (pass out_draft_q as its draft_q).  Rows of out_draft_q for nodes
 * without children are not written.  out_tree->n must equal the template's node count; parent,
 * depth and anc_mask are filled from the template, score with zeros.  depth >= 1.
 * Provisional drafter entries use rows seq_len .. seq_len + (nodes with children, root excluded) - 1
 * of draft_kv.  u_draw [B][n] uint32 and out_draft_q [B][n][V] fp32 are DEVICE pointers. */
int tlt_draft_sample(tlt_ctx *ctx, void *stream, int B, int depth, int topk, int n_verify, float temperature,
                     const int32_t *new_tokens, const int32_t *new_src, const int32_t *n_new, int new_stride,
                     const float *hidden, int hidden_n, const int32_t *root_tokens, tlt_kv *draft_kv,
                     const uint32_t *u_draw, tlt_tree *out_tree, float *out_draft_q);

/* Fills depth and anc_mask of a caller-made tree from token/parent (parents must precede
 * children; parent[0] = -1). */
int tlt_tree_finalize(tlt_ctx *ctx, void *stream, int B, tlt_tree *tree);

/* Target verification of all tree nodes in one forward pass (Section 2.2): node i attends to the
 * seq_len[b] committed tokens and to its ancestors-or-self, with rotary position seq_len[b] +
 * depth[i]; its key/value are written to provisional slot seq_len[b] + i.  seq_len is unchanged.
 * Outputs (DEVICE, any may be NULL): out_logits [B][n][V] fp32; out_argmax [B][n] (lowest index on
 * ties); out_lse [B][n][2] fp32 = (largest logit, log-sum-exp of the row), from which the target's
 * log-probability of any token follows as logit - out_lse[..][1]; out_hidden [B][n][h] fp32 = last
 * block's output before the final norm.  When only out_argmax is asked for, the logits are never
 * written (the LM head's epilogue reduces them); out_lse without out_logits materialises them in the
 * workspace. */
int tlt_verify_forward(tlt_ctx *ctx, void *stream, int B, const tlt_tree *tree, tlt_kv *kv, float *out_logits,
                       int32_t *out_argmax, float *out_lse, float *out_hidden);

/* Lossless acceptance (Section 2.2: keep the drafted prefix up to the first disagreement plus the
 * target's own token; Section 1 / Section 3 principle (a): output distributed exactly as the
 * target's).
 * mode 0, greedy: from the root follow the child whose token equals the target's argmax at the
 *   current node (target_argmax if non-NULL, else argmax of target_logits).
 * mode 1, sampling at `temperature`: recursive rejection sampling; draft_q [B][n][V] row i is the
 *   distribution node i's children were drawn from without replacement, u_accept [B][n] and
 *   u_final [B] are caller-supplied 32-bit uniforms.  Integer/double arithmetic as documented in
 *   the design notes makes every decision reproducible bit for bit.
 * mode 2, sampling at `temperature` on trees whose shape depends on the drafter's values (the
 *   deterministic top-k trees of tlt_draft_expand), where the draft distribution may not enter the
 *   rule: with the node's integer target weights W (sum S), a child with token t and uniform U =
 *   u_accept[b][child] is accepted iff (U * S) >> 32 < W[t], i.e. with the probability that a draw
 *   from the target would have been t; a rejected child's weight leaves W and S; when no child is
 *   left the token is drawn from what remains with u_final.  Lossless for any tree; draft_q unused.
 * Outputs (DEVICE): accept_len [B] (drafted tokens kept, without the bonus token); path_idx
 * [B][stride] node indices root..last accepted; out_tokens [B][stride] accepted tokens then the
 * bonus token; n_out [B] = accept_len+1; unused entries = -1.  stride >= 1 caps accept_len+1. */
int tlt_accept(tlt_ctx *ctx, void *stream, int B, int mode, float temperature, const tlt_tree *tree,
               const float *target_logits, const int32_t *target_argmax, const float *draft_q,
               const uint32_t *u_accept, const uint32_t *u_final, int stride, int32_t *accept_len,
               int32_t *path_idx, int32_t *out_tokens, int32_t *n_out);

/* tlt_accept's mode 1 for callers that cannot allocate device memory or provide a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): no context; the integer
 * weights and the rendezvous area live in a 16 MiB static device array inside the library (each GPU
 * the library runs on holds it until the process ends).  Same arguments, outputs and arithmetic as
 * tlt_accept(mode 1), plus `vocab` (no context to take it from).  Limit: B * vocab * 24 bytes plus
 * 7 KB per sequence must fit in 16 MiB less 256 bytes (B = 4 at a vocabulary of 152064), else
 * TLT_ESHAPE; tree->n <= 64.  status (DEVICE, may be NULL): word the caller has zeroed; bit 1
 * (TLT_STATUS_NO_RENDEZVOUS) is raised as described at tlt_device_status.  Calls on one GPU share
 * the array: calls that overlap in time (different streams) race; calls on one stream are ordered.
 * Allocates nothing and calls no allocating routine. */
int tlt_accept_sample_static(void *stream, int B, int vocab, float temperature, const tlt_tree *tree,
                             const float *target_logits, const float *draft_q, const uint32_t *u_accept,
                             const uint32_t *u_final, int stride, int32_t *accept_len, int32_t *path_idx,
                             int32_t *out_tokens, int32_t *n_out, uint32_t *status);

/* Keeps the accepted path: in every layer and kv head, row seq_len[b]+path_idx[b][j] moves to row
 * seq_len[b]+j for j <= accept_len[b]; then seq_len[b] += accept_len[b]+1 (the bonus token is not
 * cached: it is the next root).  kv->seq_len_bound is NOT updated (host field: the caller adds
 * its own bound, e.g. stride). */
int tlt_kv_commit(tlt_ctx *ctx, void *stream, int B, tlt_kv *kv, const int32_t *accept_len,
                  const int32_t *path_idx, int stride);

/* ---- HIP-graph pool (Section 5.1 "Memory-Efficient CUDAGraph Capture": graphs captured per batch-size
 * bucket instead of per batch size, the drafter's graph apart from the target's, one graph shared by every
 * strategy with the same key).  tlt_graph_pool_step runs one greedy step -- tlt_draft_expand (mode 0, root =
 * last new token), tlt_verify_forward (argmax and hidden state only), tlt_accept (mode 0), tlt_kv_commit, with
 * exactly the arguments below -- for the first `bucket` slots of the caller's buffers, bucket = the smallest
 * pool bucket >= B (slots B .. bucket-1 must hold valid sequences), by launching two instantiated graphs on
 * `stream`.  A graph is captured on first use of its key: the drafter's by (bucket, depth, topk, n_verify, its
 * pointer arguments), the target's by (bucket, tree, its pointer arguments); capturing synchronises `stream`,
 * runs the calls once for real on a stream of the pool, puts back what that run changed, and captures them.
 * Every graph is captured with the sequence-length bound given at creation (the grids of a graph are frozen):
 * every sequence must stay below seq_len_bound, and seq_len_bound + tree->n within what the block tables hold.
 * All buffers are the caller's and shared by all graphs (a graph owns kernel nodes and their arguments only);
 * the same pointers must be passed to replay a graph.  No host synchronisation happens in a replay.  Profiling
 * (tlt_profile_begin) records nothing inside graphs. */
typedef struct tlt_graph_pool tlt_graph_pool;
typedef struct tlt_step_args {
    /* as tlt_draft_expand: the tokens committed by the step before, the rows of `hidden` they came from */
    const int32_t *new_tokens, *new_src, *n_new;
    int32_t new_stride;
    const float *hidden;   /* [bucket][hidden_n][h]: out_hidden of the step before */
    int32_t hidden_n;
    tlt_kv *draft_kv;
    tlt_tree *tree;        /* drafter's output, target's input */
    tlt_kv *kv;
    int32_t *argmax;       /* [bucket][tree->n] */
    float *hidden_out;     /* [bucket][tree->n][h]; may be `hidden` itself */
    int32_t stride;
    int32_t *accept_len, *path_idx, *out_tokens, *n_out;   /* as tlt_accept */
} tlt_step_args;
/* buckets: HOST, strictly increasing batch sizes, each <= the context's max_batch.  The pool refers to the
 * context: destroy the pool first.  Errors: TLT_EINVAL (arguments), TLT_ESHAPE (B above the largest bucket),
 * TLT_EHIP (capture, instantiation or launch failed: tlt_last_hip_error), or whatever the captured calls return. */
int tlt_graph_pool_create(tlt_ctx *ctx, const int32_t *buckets, int n_buckets, int seq_len_bound, tlt_graph_pool **out);
int tlt_graph_pool_destroy(tlt_graph_pool *pool);
int tlt_graph_pool_step(tlt_graph_pool *pool, void *stream, int B, int depth, int topk, int n_verify,
                        const tlt_step_args *args);
int tlt_graph_pool_count(const tlt_graph_pool *pool, int32_t *n_draft, int32_t *n_target);

/* ---- auxiliary entry points (unit tests, per-kernel measurement) ---- */

/* C[M][N] (op)= A[M][K] . W[N][K]^T on DEVICE buffers of dtype (TLT_F32/TLT_BF16).
 * out_mode 0: C stored in dtype; 1: C stored as fp32; 2: fp32 C += product (products cut along K add their
 * partial sums with atomics here, so the last bit can differ from run to run; the step itself keeps the
 * partial products apart and sums them in a fixed order). */
int tlt_gemm(void *stream, int dtype, int out_mode, int M, int N, int K, const void *A, const void *W, void *C);

/* act[M][N] = silu(A Wg^T) * (A Wu^T), bf16 DEVICE operands and result: the fused gate/up projection of
 * the decoder block's MLP (the two products never reach memory).  TLT_ENOTIMPL when the shape is not
 * covered (N % 128, K % 64, operands not 16-byte aligned, act not 8-byte aligned). */
int tlt_gemm_glu(void *stream, int M, int N, int K, const void *A, const void *Wg, const void *Wu, void *act);

/* Measurement aid (no step of the decoding path): the rate the matrix pipes sustain with nothing else running.
 * 256 workgroups of four waves; every wave repeats, `iters` times, the 64 matrix instructions (32x32x16, bf16 in,
 * fp32 accumulation) that a 128x128 wave tile of the GEMM kernels issues per 64-wide K tile, in those kernels'
 * order, on operands it holds in registers: 4 K slices x (4 activation + 4 weight fragments), fragment f of slice s
 * for lane l being the 8 bf16 values at frags[((s * 8 + f) * 64 + l) * 8 ..] (f < 4: rows l % 32 of activation
 * block f, f >= 4: rows l % 32 of weight block f - 4; k = 8 * (l / 32) .. + 7 of the slice).  frags: DEVICE, 32768
 * bytes, 16-byte aligned.  out: DEVICE, 65536 floats; out[workgroup * 256 + thread] = the sum of the 256
 * accumulator elements the thread's lane holds (every wave computes the same 128x128 product, `iters` times
 * over).  Flops per call: 1024 waves x iters x 64 instructions x 32768.  Timed by the caller (events around the
 * call).  TLT_EINVAL: null or misaligned pointers, iters outside 1 .. 2^20 (a call then runs for about a second at most). */
int tlt_mfma_stream(void *stream, const void *frags, float *out, int iters);

/* out[m] = argmax_n (A W^T)[m][n] (lowest n on ties) for bf16 DEVICE operands, without storing the
 * product: what tlt_verify_forward runs as its LM head when only out_argmax is asked for.  ws: DEVICE
 * scratch of at least M * (N/128) * 8 bytes.  TLT_ENOTIMPL when the shape is not covered (N % 256,
 * K % 64, M <= 64, misaligned operands): callers then take tlt_gemm + their own argmax. */
int tlt_gemm_argmax(void *stream, int M, int N, int K, const void *A, const void *W, void *ws, size_t ws_bytes,
                    int32_t *out);

/* The tree attention of one decoder block on its own (Section 2.2: every tree node attends to the
 * committed context and to its ancestors-or-self).  qkv [B][n][(Hq+2Hkv)*d] in dtype holds the rotated
 * queries (the key/value part is not read: the tree's keys and values must already sit in the cache at
 * slots seq_len[b] + i); kv describes ONE layer's pools [n_pages][Hkv][page_size][d]; anc_mask [B][n];
 * out [B][n][Hq*d] in dtype.  ws: DEVICE scratch of tlt_attention_workspace_bytes(...) bytes for the
 * bound max_ctx >= kv->seq_len_bound + n.  impl as in tlt_set_attention_impl.  TLT_ESHAPE when the
 * explicitly requested kernel does not cover the shape or the scratch is too small. */
size_t tlt_attention_workspace_bytes(int B, int n, int n_q_heads, int n_kv_heads, int head_dim, int max_ctx);
int tlt_attention(void *stream, int dtype, int B, int n, int n_q_heads, int n_kv_heads, int head_dim, int page_size,
                  const void *qkv, const uint64_t *anc_mask, const tlt_kv *kv, void *out, void *ws, size_t ws_bytes,
                  int impl);

/* Attention kernel choice for cross-checks: -1 automatic (default), 0 wave-per-row kernel,
 * 1 MFMA split-KV kernel (bf16, head_dim 128 only; other shapes fall back to 0). */
int tlt_set_attention_impl(tlt_ctx *ctx, int impl);

/* Conditions that only the device can see are recorded in a status word in the workspace and reported
 * here: synchronises `stream`, writes the bits to *flags (HOST, may be NULL), clears them, and returns
 * TLT_ESHAPE when a kernel found seq_len[b] above the caller's seq_len_bound (the attention then covered
 * only part of that sequence's context: the outputs of that call are wrong), TLT_ESYNC when the
 * workgroups of a sampling acceptance could not meet because the chip was busy with other streams'
 * work (that call's outputs are undefined: repeat it), else TLT_OK. */
enum { TLT_STATUS_CONTEXT_TRUNCATED = 1, TLT_STATUS_NO_RENDEZVOUS = 2 };
int tlt_device_status(tlt_ctx *ctx, void *stream, uint32_t *flags);

/* Measurement switch: 1 = with more than 256 rows the attention output projection's product is rounded
 * to the model dtype before it joins the fp32 residual stream (2 bytes per element less to write
 * and read back per block); 0 (default) = it stays fp32, as the conventions at the top state. */
int tlt_set_oproj_rounding(tlt_ctx *ctx, int round_to_model_dtype);

/* Per-kernel-class timing with HIP events on the launch stream.  Classes: 0 GEMMs of the target's
 * verification forward, 1 its tree attention, 2 KV commit, 3 everything else, 4 the drafter's GEMMs,
 * 5 the drafter's attention.  tlt_profile_read synchronises the recorded events and returns, per
 * class, summed milliseconds, launches, algorithmic flops and algorithmic bytes since the last
 * tlt_profile_begin(ctx, 1).  enable: 1 = start afresh, 2 = resume (records kept), 0 = pause (records kept
 * until the next read or fresh start).  Arrays are HOST, TLT_PROFILE_CLASSES entries each. */
enum { TLT_PROFILE_CLASSES = 6 };
int tlt_profile_begin(tlt_ctx *ctx, int enable);
int tlt_profile_read(tlt_ctx *ctx, double *ms, int64_t *launches, double *flops, double *bytes);

/* ---- strategy selection (host only: no GPU work, no stream) ---------------------------------
 * The Bucketed-Epsilon-Greedy selector of Algorithm 1 (Section 5.2) with the elastic activation
 * rule of Section 5.1.  A strategy is (Draft_Depth, topK, Tokens_to_Verify).  Strategies are grouped
 * by Tokens_to_Verify in descending order and group i serves the batch-size bucket
 * [thresholds[i], thresholds[i+1] - 1] (the last bucket is open-ended; batch sizes below
 * thresholds[0] use the first bucket), so n_thresholds must equal the number of distinct
 * Tokens_to_Verify values and thresholds must increase strictly.  Every strategy keeps the rewards
 * and mean emitted lengths of its last `window` recorded steps.
 *
 * tlt_mab_select: writes the chosen strategy's index (position in the `strategies` array given at
 * creation) or -1 when batch_size >= sd_threshold (speculation off, decode normally).  A bucket with
 * one strategy returns it.  Otherwise u = (u1 + 0.5) / 2^32 < epsilon explores: candidate number
 * floor(u2 * |V| / 2^32) in creation order; else the candidate with the largest median reward over
 * its window wins (an empty window counts as +infinity, so untried strategies go first; an even
 * count takes the mean of the middle pair; ties go to the earlier candidate).  u1, u2 are the
 * caller's uniform 32-bit random numbers.
 *
 * tlt_mab_record: for the step just run with `strategy`: a = sum(accept_lens) / batch_size + 1,
 * reward = a * batch_size / elapsed_time (emitted tokens per unit time); both are appended to the
 * strategy's windows and returned through a_bar / reward when those are not NULL.  accept_lens is
 * a HOST array of batch_size entries (accepted draft tokens per sequence, bonus token excluded).
 *
 * All arrays are HOST memory and are copied; errors: TLT_EINVAL. */
typedef struct tlt_strategy {
    int32_t draft_depth, topk, tokens_to_verify;
} tlt_strategy;
typedef struct tlt_mab tlt_mab;
int tlt_mab_create(const tlt_strategy *strategies, int n_strategies, const int32_t *thresholds, int n_thresholds,
                   double epsilon, int window, int sd_threshold, tlt_mab **out);
void tlt_mab_destroy(tlt_mab *mab);
int tlt_mab_select(tlt_mab *mab, int batch_size, uint32_t u1, uint32_t u2, int32_t *strategy);
int tlt_mab_record(tlt_mab *mab, int strategy, double elapsed_time, const int32_t *accept_lens, int batch_size,
                   double *a_bar, double *reward);
/* Median reward over the strategy's window (+infinity when empty) and the number of entries held. */
int tlt_mab_median_reward(const tlt_mab *mab, int strategy, double *median, int32_t *count);

/* ---- model-free drafter (host only) ----------------------------------------------------------
 * The n-gram retrieval drafter of Section 5.3: a database per prompt, filled from that prompt's
 * rollout responses, that proposes a candidate tree from the tokens preceding the position to predict.
 * It is a second producer of tlt_tree: the arrays it writes are HOST memory; copy them to the device
 * and call tlt_tree_finalize, then tlt_verify_forward / tlt_accept / tlt_kv_commit as with the
 * learned drafter's trees.
 *
 * order n: tlt_ngram_insert adds, for every window of k+1 consecutive tokens (k = 1 .. n-1) of the
 * response, one count to (first k tokens) -> (last token), under prompt_id.
 * tlt_ngram_propose: context = the last context_len tokens of the sequence, ending with the root
 * token (the one emitted last).  A continuation list is that of the longest seen suffix (at most
 * n-1 tokens) of a context, ranked by count, equal counts by lower token id, with confidence
 * log(count / total).  Node 0 = root; level 1 = the topk best continuations of the context; for
 * each further level up to `depth` every frontier node proposes its topk best continuations and
 * the topk best new candidates by path score (ties: created earlier) form the next frontier; the
 * n_nodes-1 best candidates by path score are kept in creation order.  If fewer exist, the tree is
 * padded with children of the root carrying the smallest token ids it has no child for yet
 * (score -infinity): exactly n_nodes nodes are always written.  token/parent hold n_nodes int32,
 * score (may be NULL) n_nodes floats.  Errors: TLT_EINVAL. */
typedef struct tlt_ngram tlt_ngram;
int tlt_ngram_create(int order, tlt_ngram **out);
void tlt_ngram_destroy(tlt_ngram *db);
int tlt_ngram_insert(tlt_ngram *db, int64_t prompt_id, const int32_t *tokens, int len);
int tlt_ngram_propose(const tlt_ngram *db, int64_t prompt_id, const int32_t *context, int context_len, int depth,
                      int topk, int n_nodes, int32_t *token, int32_t *parent, float *score);

#ifdef __cplusplus
}
#endif
#endif
