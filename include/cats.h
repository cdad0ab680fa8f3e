/*
 * cats.h - C ABI of the MI355X (gfx950) draft-tree verification library.
 *
 * The library runs the target verification pass of cascaded tree speculation
 * (paper Sec. 3.2 "Cascaded verification design", paragraph "Target
 * verification pass"; Algorithm 1, Stage 3 and the walk / bonus / commit steps
 * after it; tree mask of Fig. 4, right): all T nodes of a draft tree go through
 * a range of decoder layers in one batched pass, every layer's weights being
 * read from HBM once; each node attends to the committed context and to its own
 * ancestors; the longest root-descending chain whose tokens match the target's
 * greedy choices is accepted, one bonus token is produced, and the KV cache is
 * rolled back to the accepted path.
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer unless its comment says HOST.
 *  - bf16 = the upper 16 bits of an IEEE float32.  Matrices are row-major
 *    [out][in] (y = x W^T).  The layer is pre-norm RMSNorm + multi-head
 *    attention with rotary embedding (half-split pairing, dimension j pairs with
 *    j + head_dim/2) + SwiGLU feed-forward, no biases.
 *  - The caller owns all weights, caches, inputs and outputs; the library only
 *    borrows them until the enqueued work has run.  A cats_ctx owns scratch
 *    memory sized at creation; no call allocates after cats_create.
 *  - Work is enqueued on the given HIP stream (a hipStream_t passed as void*,
 *    NULL = default stream) and the call returns without waiting, except where
 *    a HOST output pointer is given (then the call synchronises the stream).
 *  - Every function returns CATS_OK (0) or a negative cats_status.  Arguments are
 *    validated on the host before anything is enqueued: a call that returns
 *    CATS_EINVAL, CATS_ECAPACITY or CATS_ESTATE has enqueued nothing.  CATS_EHIP
 *    reports a HIP runtime failure, which may surface after part of the call's
 *    work was enqueued; the outputs of such a call are undefined.
 *  - Calls that use one cats_ctx must not overlap in time (they share scratch).
 */
#ifndef CATS_H
#define CATS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CATS_MAX_TREE 128  /* largest tree (nodes incl. root)                  */
#define CATS_MAX_DEPTH 16  /* deepest node; an accepted path has <= 17 entries */
#define CATS_MAX_LAYERS 128

typedef enum {
    CATS_OK = 0,
    CATS_EINVAL = -1,    /* null pointer, bad shape, malformed tree, token out of range */
    CATS_ECAPACITY = -2, /* ctx_len + T exceeds max_ctx, or a tree exceeds its arrays       */
    CATS_ESTATE = -3,    /* no tree has been set                                         */
    CATS_EHIP = -4       /* a HIP runtime call failed                                    */
} cats_status;

typedef struct cats_ctx cats_ctx;

/* Model shape.  Requirements: hidden == n_heads*head_dim, head_dim == 64 or 128,
 * hidden % 64 == 0, ffn % 16 == 0, max_ctx % 64 == 0, 1 <= max_tree <= CATS_MAX_TREE. */
typedef struct {
    int32_t n_layers, hidden, n_heads, head_dim, ffn, vocab;
    int32_t max_ctx;  /* rows each KV cache holds                         */
    int32_t max_tree; /* largest T this context will be asked to verify   */
    float rms_eps, rope_base;
    int32_t packed_weights; /* 0: matrices are row-major [out][in]; 1: every matrix (the seven
                             * of each layer and w_lm) was re-tiled by cats_pack_matrix        */
} cats_model_desc;

/* One decoder layer, bf16.  wq/wk/wv/wo: [hidden][hidden]; w_gate/w_up:
 * [ffn][hidden]; w_down: [hidden][ffn]; g_attn/g_ffn: RMSNorm gains [hidden].
 * With packed_weights the seven matrices are cats_pack_matrix outputs instead.
 * An attention-only block (the draft and shallow-verifier adapters of Sec. 3.3: normalisation,
 * one attention layer, residual; the second normalisation is the g_final of the LM-head call)
 * has w_gate = w_up = w_down = g_ffn = NULL: x += attention(rmsnorm(x, g_attn)) and nothing
 * else.  Either all four are NULL or none (CATS_EINVAL otherwise); the host-streamed entry
 * point takes full layers only. */
typedef struct {
    const void *wq, *wk, *wv, *wo, *w_gate, *w_up, *w_down, *g_attn, *g_ffn;
} cats_layer_weights;

/* One layer's KV cache, bf16.  k: [n_heads][max_ctx][head_dim], keys stored after
 * rotation.  v: [n_heads][head_dim][max_ctx], i.e. values stored TRANSPOSED so
 * that the row (context) index is the contiguous one.  Rows [0, ctx_len) are the
 * committed context; a verify call writes rows ctx_len .. ctx_len+T-1.  The cache is what is
 * kept between calls and its precision is bf16; within one call the rows that the call itself
 * appends also take part in attention with their rounding remainders (kept in the context's
 * scratch), i.e. at about 16 mantissa bits. */
typedef struct {
    void *k, *v;
} cats_kv_layer;

/* A draft tree in topological order: HOST arrays of n entries, copied during
 * cats_set_tree.  parent[0] = -1, 0 <= parent[i] < i, depth[0] = 0,
 * depth[i] = depth[parent[i]] + 1 <= CATS_MAX_DEPTH, 0 <= token[i] < vocab.
 * Node 0 is the last committed token (its K/V is not in the cache yet); every
 * other node carries a candidate token judged by the target's prediction at
 * its parent. */
typedef struct {
    const int32_t *token, *parent, *depth;
    int32_t n;
} cats_tree;

/* Outcome of greedy acceptance (Algorithm 1: walk, bonus token, commit). */
typedef struct {
    int32_t n_accepted;                 /* accepted candidates = depth of the last accepted node */
    int32_t path[CATS_MAX_DEPTH + 1];   /* node indices, root first; n_accepted+1 valid, rest -1  */
    int32_t tokens[CATS_MAX_DEPTH + 1]; /* token ids of those nodes                               */
    int32_t bonus_token;                /* target's argmax at the last accepted node              */
    int32_t new_ctx_len;                /* ctx_len + n_accepted + 1                               */
} cats_accept_result;

/* Create / destroy a context (allocates all scratch for the given shape on the
 * current device).  HOST pointers. */
int cats_create(const cats_model_desc *desc, cats_ctx **out);
int cats_destroy(cats_ctx *ctx);

/* One-time re-tiling of a weight matrix into the order in which the weight-streaming
 * kernel consumes it, so that every wave load is one contiguous kilobyte (the layer-weight
 * stream of the "Target verification pass" then reads HBM purely sequentially).
 * Layout: rows are padded to a multiple of 32 and columns to a multiple of 128 with zeros;
 * the 1 KB fragment of row block rb (32 rows), column chunk c (128 columns) and step j
 * (16 columns, j < 8) starts at byte ((rb * ceil(cols/128) + c) * 8 + j) * 1024 and holds,
 * for lane l < 64, the 8 values W[32 rb + l % 32][128 c + 16 j + 8 (l / 32) .. +7].
 * src: bf16 [rows][cols] row-major (DEVICE), cols % 16 == 0; dst: DEVICE buffer of
 * cats_packed_matrix_bytes(rows, cols) bytes, must not overlap src. */
size_t cats_packed_matrix_bytes(int32_t rows, int32_t cols);
int cats_pack_matrix(const void *src, void *dst, int32_t rows, int32_t cols, void *stream);

/* Validate a tree and upload it (tree ingest; the ancestor sets that form the
 * tree attention mask of Fig. 4 are derived from parent[] on the device).
 * Synchronous with respect to the host arrays: they may be freed on return. */
int cats_set_tree(cats_ctx *ctx, const cats_tree *tree, void *stream);

/* One decoder layer over all T tree nodes (Algorithm 1, Stage 3, one layer of
 * M_{L_SV+1 : L_total}): hidden <- hidden + Attn(RMSNorm(hidden)) then
 * hidden <- hidden + FFN(RMSNorm(hidden)).  hidden: float32 [T][hidden], in/out
 * (the residual stream is kept in float32).  Node i is rotated at position
 * ctx_len + depth[i]; its key/value go to cache row ctx_len + i. */
int cats_verify_layer(cats_ctx *ctx, const cats_layer_weights *w, float *hidden,
                      const cats_kv_layer *kv, int32_t ctx_len, void *stream);

/* Tree-masked attention alone (Fig. 4 right-lower; the tree attention mask of the
 * target verification pass).  q: bf16 [T][hidden], already rotated; kv rows
 * ctx_len .. ctx_len+T-1 must already hold the tree nodes' keys/values.
 * out: bf16 [T][hidden].  Node i sees rows [0, ctx_len) and rows ctx_len + a
 * for a in ancestors(i) + {i}. */
int cats_tree_attention(cats_ctx *ctx, const void *q, const cats_kv_layer *kv, int32_t ctx_len,
                        void *out, void *stream);

/* Greedy acceptance and KV roll-back (Algorithm 1: the walk over the tree for the longest
 * accepted prefix, the bonus token, and the roll-back of the KV cache along the accepted path).  node_argmax: int32 [T], the target's greedy token at every node.
 * kv: HOST array indexed by layer; layers [layer_begin, layer_end) are
 * compacted: row ctx_len + path[k] moves to row ctx_len + k.  Rows from
 * new_ctx_len on are left undefined.  out_dev: device result (required);
 * out_host: optional HOST copy (the call then waits for the stream). */
int cats_accept_and_compact(cats_ctx *ctx, const int32_t *node_argmax, const cats_kv_layer *kv,
                            int32_t layer_begin, int32_t layer_end, int32_t ctx_len,
                            cats_accept_result *out_dev, cats_accept_result *out_host,
                            void *stream);

/* A whole verify step: input rows (embedding lookup of the tree tokens when
 * `embed` [vocab][hidden] bf16 is given, else `hidden_in` float32 [T][hidden],
 * the hidden states of the tree that Alg. 1 hands to stage 3), layers [layer_begin, layer_end) of `layers`
 * (HOST array indexed by layer), final RMSNorm (g_final) + LM head (w_lm
 * [vocab][hidden]) + per-node argmax, then acceptance and compaction as above.
 * Optional device outputs: hidden_out float32 [T][hidden] (residual stream after
 * the last layer), logits_out float32 [T][vocab], argmax_out int32 [T],
 * margin_out float32 [T] (gap between the two largest logits of each node). */
int cats_verify_tree(cats_ctx *ctx, const cats_layer_weights *layers, int32_t layer_begin,
                     int32_t layer_end, const void *embed, const float *hidden_in,
                     const void *g_final, const void *w_lm, const cats_kv_layer *kv,
                     int32_t ctx_len, float *hidden_out, float *logits_out, int32_t *argmax_out,
                     float *margin_out, cats_accept_result *out_dev, cats_accept_result *out_host,
                     void *stream);

/* Acceptance criterion Acc of the walk in cats_verify_tree / cats_verify_tree_streamed (Alg. 1:
 * Acc may be greedy or typical; Sec. 3.2 names typical acceptance by citation only, so the inequality is
 * the cited work's: a candidate token x judged at its parent's distribution
 * p = softmax(logits / temperature) passes when p(x) > min(epsilon, delta * exp(-H(p))), H the
 * entropy of p).  mode 0 = greedy (the default: the token must equal the parent's argmax), mode
 * 1 = typical with epsilon >= 0, delta >= 0, temperature > 0.  Everything else of the walk is
 * unchanged: deepest accepted node, lowest index among equals, bonus token = argmax at that
 * node.  cats_accept_and_compact always walks greedily from the argmax array it is given.
 * HOST call, takes effect for later enqueues.  CATS_EINVAL for a bad mode or parameters. */
int cats_set_acceptance(cats_ctx *ctx, int32_t mode, float epsilon, float delta, float temperature);

/* Diagnostics of the last typical-mode cats_verify_tree on this context (copies enqueued on
 * `stream`, which must be the stream of that call or ordered after it).  All optional, DEVICE
 * float32 [T]: lse_out, entropy_out = log-sum-exp and entropy of softmax(logits / temperature)
 * per node; prob_out, threshold_out = probability of each node's token under its parent's
 * distribution and the threshold it was compared with (node 0: 1 and 0). */
int cats_typical_stats(cats_ctx *ctx, float *lse_out, float *entropy_out, float *prob_out,
                       float *threshold_out, void *stream);

/* KV roll-back alone along an accept result that already exists on the device (Alg. 1, the
 * roll-back line at the end of a cycle): rows ctx_len + path[k] -> ctx_len + k, k = 0..n_accepted,
 * in layers [layer_begin, layer_end) of kv (HOST array indexed by layer).  For caches that the
 * call which produced result_dev did not cover: the shallow layers of a staged cycle, adapter
 * caches. */
int cats_compact_along(cats_ctx *ctx, const cats_accept_result *result_dev, const cats_kv_layer *kv,
                       int32_t layer_begin, int32_t layer_end, int32_t ctx_len, void *stream);

/* Shallow-verification stage, correction re-forward (Sec. 3.2, shallow verification stage; Alg. 1,
 * stage 2: the correction tokens are forwarded again through the resident layers under the tree
 * mask while the main draft chain is not).  Forwards only nodes [node_begin, T) of the tree set
 * by cats_set_tree through layers [layer_begin, layer_end): their queries see the KV context and
 * their ancestors; their K/V rows are written at cache rows ctx_len + node.  The K/V rows of the
 * ancestors among nodes [0, node_begin) must already be in those layers' caches at rows
 * ctx_len + node (left there by an earlier cats_verify_tree / cats_verify_nodes call on a tree
 * whose first node_begin nodes were the same, without compaction in between).
 * Input rows: embedding lookup of the nodes' tokens when `embed` is given, else hidden_in
 * float32 [T - node_begin][hidden] (DEVICE).  hidden_out: DEVICE float32 [T - node_begin][hidden],
 * the residual stream of those nodes after layer layer_end - 1 (required).  No LM head, no
 * acceptance: stage 3 (cats_verify_tree over the remaining layers with hidden_in) does that.
 * CATS_EINVAL for node_begin outside [0, T). */
int cats_verify_nodes(cats_ctx *ctx, const cats_layer_weights *layers, int32_t layer_begin,
                      int32_t layer_end, const void *embed, const float *hidden_in,
                      const cats_kv_layer *kv, int32_t ctx_len, int32_t node_begin,
                      float *hidden_out, void *stream);

/* Drafting stage on the device (Sec. 3.2, draft stage; Alg. 1, stage 1: gamma sequential passes
 * through the draft layers, the draft adapter and the shared LM head, y = argmax H(o)).  The chain
 * root, d_1 .. d_gamma becomes the context's tree; step k forwards node k alone through layers
 * [layer_begin, layer_end) of `layers` (its K/V at cache row ctx_len + k of kv), then through the
 * attention-only block `adapter` (cache kv_adapter, one layer), applies RMSNorm with g_adapter_out
 * and the LM head w_lm, and writes the argmax as the token of node k + 1 ON THE DEVICE, where
 * step k + 1 reads it for its embedding row: no host round trip between the tokens.
 * layers, kv: HOST arrays indexed by layer (kv_adapter: HOST pointer to one cats_kv_layer);
 * embed, g_adapter_out, w_lm: DEVICE.  Outputs (DEVICE): tokens_out int32 [gamma + 1] = root and
 * the gamma drafted tokens; hidden_out float32 [gamma + 1][hidden], optional: every chain node's
 * residual stream after layer layer_end - 1 (what the shallow-verification stage continues from;
 * when given, the last draft takes one more pass through the draft layers, without the adapter).
 * Afterwards the context's tree is that chain (cats_verify_nodes can continue on it).
 * CATS_EINVAL: gamma outside [1, CATS_MAX_DEPTH] or gamma + 1 > max_tree, empty layer range,
 * adapter with feed-forward matrices, root token out of range; CATS_ECAPACITY: ctx_len + gamma + 1
 * > max_ctx. */
int cats_draft_chain(cats_ctx *ctx, const cats_layer_weights *layers, int32_t layer_begin,
                     int32_t layer_end, const cats_layer_weights *adapter, const void *g_adapter_out,
                     const void *w_lm, const void *embed, const cats_kv_layer *kv,
                     const cats_kv_layer *kv_adapter, int32_t ctx_len, int32_t root_token,
                     int32_t gamma, int32_t *tokens_out, float *hidden_out, void *stream);

/* Verification tree of one cascaded cycle (Alg. 1, stage 2: ChainTree / BuildTree; Fig. 4 right
 * upper).  HOST arrays only, nothing is enqueued.  Node 0 carries root_token (the last committed
 * token); draft position i (token main_tokens[i], i < gamma) is node i + 1, child of node i; every
 * position whose corrections[i] is >= 0 and differs from main_tokens[i] adds one leaf carrying
 * corrections[i] as a sibling of draft position i (child of node i), numbered after the chain in
 * position order.  corrections may be NULL (plain chain).  Outputs token/parent/depth[capacity],
 * *n_out = 1 + gamma + number of corrections, corr_node[gamma] (optional: node of the correction
 * at each position, -1 where there is none).  Because the chain comes first, the corrections are
 * exactly nodes [gamma + 1, n): the range cats_verify_nodes re-forwards.
 * CATS_EINVAL: gamma outside [0, CATS_MAX_DEPTH] or a NULL output; CATS_ECAPACITY: more nodes
 * than capacity or CATS_MAX_TREE. */
int cats_build_tree(int32_t root_token, const int32_t *main_tokens, int32_t gamma,
                    const int32_t *corrections, int32_t capacity, int32_t *token, int32_t *parent,
                    int32_t *depth, int32_t *n_out, int32_t *corr_node);

/* Reduced KL loss for adapter training (Sec. 3.3, Eq. 2; Appendix B steps 1-3) and its gradient.
 * target_logits, draft_logits: DEVICE float32 [n_pos][vocab], row-major, 16-byte aligned;
 * p_target and q_draft are their softmaxes.  Per position t with mask[t] != 0 (mask: DEVICE
 * uint8 [n_pos], NULL = every position counts): T_K(t) = the top_k tokens of highest target
 * probability (equal values: lower index first), p~ = p_target renormalised over T_K(t),
 * loss_t = -sum_{v in T_K(t)} p~(v) log q_draft(v).
 * Outputs (DEVICE): loss_out float32 [1] = mean of loss_t over the unmasked positions (0 if there
 * is none); per_pos_out float32 [n_pos] = loss_t (0 where masked; required, it is also the
 * workspace of the mean); topk_idx_out int32 [n_pos][top_k], optional: T_K(t) most probable
 * first (-1 where masked); grad_out float32 [n_pos][vocab], optional, 16-byte aligned:
 * d loss / d draft_logits = (q_draft - p~) / |M| (zero rows where masked).
 * Logits must be finite.  Enqueues on `stream` and returns; nothing is allocated.
 * CATS_EINVAL: NULL required pointer, misaligned pointer, n_pos < 1, vocab not a positive
 * multiple of 4, top_k outside [1, min(CATS_LOSS_MAX_K, vocab)]; CATS_ECAPACITY: vocab above
 * CATS_LOSS_MAX_VOCAB (a whole row is held in one workgroup's registers). */
#define CATS_LOSS_MAX_K 64
#define CATS_LOSS_MAX_VOCAB 36864
int cats_reduced_kl_loss(const float *target_logits, const float *draft_logits, const uint8_t *mask,
                         int32_t n_pos, int32_t vocab, int32_t top_k, float *loss_out,
                         float *per_pos_out, int32_t *topk_idx_out, float *grad_out, void *stream);

/* Offload regime (Sec. 3.2: the target layers arrive from slower memory one chunk after the
 * other while the previous chunk computes; Fig. 4 left): the same verify step with the layer weights held
 * in pinned HOST memory.  host_layers: HOST array indexed by layer whose nine pointers are
 * pinned HOST addresses (packed matrices if the context was created with packed_weights).
 * staging[0..1]: two DEVICE buffers of cats_layer_weight_bytes() each; layer l is copied into staging[l & 1] on the context's own copy stream while layer
 * l-1 computes on `stream` (events order the two streams; the copy of layer l+2 waits until
 * layer l has been consumed).  Everything else is as in cats_verify_tree (embed, g_final and
 * w_lm are DEVICE pointers).  The call returns after enqueueing unless out_host is given. */
size_t cats_layer_weight_bytes(const cats_model_desc *desc);
int cats_verify_tree_streamed(cats_ctx *ctx, const cats_layer_weights *host_layers,
                              int32_t layer_begin, int32_t layer_end, void *const staging[2],
                              const void *embed, const float *hidden_in, const void *g_final,
                              const void *w_lm, const cats_kv_layer *kv, int32_t ctx_len,
                              float *hidden_out, float *logits_out, int32_t *argmax_out,
                              float *margin_out, cats_accept_result *out_dev,
                              cats_accept_result *out_host, void *stream);

/* Final RMSNorm + LM head + argmax alone (Algorithm 1: p_tgt = softmax(H(H_tgt)) for the
 * target, y = argmax H(o) behind the draft and shallow-verifier adapters, whose second
 * normalisation gain is passed as g_final: the LM head is shared; greedy decisions need only the
 * argmax).  hidden: DEVICE float32 [n_rows][hidden], 1 <= n_rows <= max_tree (any rows: the
 * tree set in the context plays no part).  Outputs (DEVICE): argmax_out int32 [n_rows]; optional
 * logits_out float32 [n_rows][vocab] and margin_out float32 [n_rows]. */
int cats_lm_head_argmax(cats_ctx *ctx, const float *hidden, int32_t n_rows, const void *g_final,
                        const void *w_lm, float *logits_out, int32_t *argmax_out, float *margin_out,
                        void *stream);

/* cats_tree_attention for callers that cannot allocate device memory or hold a cats_ctx: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same result as
 * cats_set_tree + cats_tree_attention, same kernels.  Calls no hipMalloc / hipFree and no
 * allocating library routine: the tree masks and the per-chunk partial results live in a fixed
 * array inside the library's code object (CATS_NOALLOC_SCRATCH_BYTES, one copy per GPU, held
 * until the process ends).  q, kv, out: DEVICE, as for cats_tree_attention; parent: HOST int32
 * [n_nodes] in topological order (parent[0] = -1, 0 <= parent[i] < i, depth <= CATS_MAX_DEPTH),
 * copied during the call.  The cache layout is given by n_heads, head_dim (64 or 128) and
 * max_ctx (multiple of 64).  Only kernel launches are enqueued on `stream`.
 * CATS_EINVAL: NULL pointer, malformed tree, bad shape.  CATS_ECAPACITY: n_nodes >
 * CATS_MAX_TREE, ctx_len + n_nodes > max_ctx, or a shape whose partial results do not fit the
 * fixed array (8 MiB hold every shape with n_heads * head_dim <= 8192 on a 256-CU device).
 * All calls on one GPU share that GPU's array, which keeps the last call's contents: calls that
 * overlap in time on one GPU (different streams, different threads) race; order them. */
#define CATS_NOALLOC_SCRATCH_BYTES (8u << 20)
int cats_tree_attention_noalloc(const void *q, const cats_kv_layer *kv, const int32_t *parent,
                                int32_t n_nodes, int32_t n_heads, int32_t head_dim, int32_t max_ctx,
                                int32_t ctx_len, void *out, void *stream);

/* Measurement aid for the weight-streaming GEMM (the layer-weight pass of the
 * "Target verification pass"): while enabled, every GEMM launch made through
 * this context carries a pair of HIP events attached to its dispatch on its own
 * stream (kernel begin / end; at most 1024 launches between two reads).  cats_profile_gemm_read waits for them and
 * returns the summed kernel time in milliseconds and the launch count (HOST
 * outputs), then starts a new collection. */
int cats_profile_gemm(cats_ctx *ctx, int enable);
int cats_profile_gemm_read(cats_ctx *ctx, float *total_ms, int32_t *launches);

/* Name of the dominant (weight-streaming) kernel as it appears in profiler
 * output, and the text of a status code.  HOST strings, never freed. */
const char *cats_gemm_kernel_name(void);
const char *cats_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* CATS_H */
