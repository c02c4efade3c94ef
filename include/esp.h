/*
 * esp.h -- C ABI of the ESP (Embedding-Space Probing) speculate-and-verify decode step
 * for MI355X (gfx950).  Plain pointers and sizes only; no C++ or framework types.
 *
 * One decode step (paper Sec. 3.3, Fig. 1 right) is four calls on one stream:
 *
 *   esp_tree_forward      forward of [last accepted token | draft-tree tokens | mask tokens]
 *                         against the KV cache under the tree attention mask, LM head and
 *                         argmax at the tree rows                       (Sec. 2, Sec. 3.3, App. C/E)
 *   esp_verify_accept     lossless longest-accepted-path check, bonus token, KV commit
 *                                                                       (Sec. 2 Eq. 3, Sec. 3.3, Sec. 4)
 *   esp_mask_topk         LM head + vocabulary softmax + Top-K' at the mask rows aligned to the
 *                         accepted position                             (Sec. 2 Eq. 2, Sec. 3.3)
 *   esp_build_prune_tree  pruning rule and dynamic tree construction -> next block
 *                                                                       (Sec. 3.4 Alg. 1, Sec. 3.5, App. C)
 *
 * Conventions
 *  - "device" = pointer into GPU memory owned by the caller; "host" = ordinary host memory.
 *    The library never allocates or frees device memory and never keeps a caller pointer
 *    beyond the call, except the weight pointers handed to esp_create (kept until esp_destroy)
 *    and the workspace.
 *  - Every call enqueues its kernels on the ctx stream and returns without synchronising,
 *    except where stated.  The return value reports what the host can check (null pointers,
 *    shapes, capacities known on the host).  Conditions only the device can see (a sequence
 *    whose length exceeds the host's bound or its capacity, a malformed tree) set a sticky
 *    device status word, read with esp_last_device_status(); the offending work is skipped,
 *    never executed out of bounds.
 *  - No entry point throws or aborts.
 *  - Matrices are row-major [out_features, in_features] in the model dtype.
 *  - Rows: a block holds `batch` sequences, sequence b owning rows
 *    [b*rows_per_seq, b*rows_per_seq + n_rows[b]).  Within a sequence rows 0..n_nodes-1 are
 *    tree nodes in (depth, creation) order, row 0 the last accepted token; mask rows follow
 *    (Fig. 3).  ESP_LAYOUT_PER_NODE: node a owns mask rows n_nodes + a*k + (j-1), j = 1..k,
 *    so n_rows = (k+1) n_nodes (block complexity, Sec. 3.3).  ESP_LAYOUT_ROOT_CHAIN: only the
 *    root owns a chain, n_rows = n_nodes + k.
 */
#ifndef ESP_H_
#define ESP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct esp_ctx esp_ctx; /* opaque; host object, owns nothing on the device */

typedef enum {
  ESP_OK = 0,
  ESP_EINVAL = 1,    /* null pointer or value out of range */
  ESP_ESHAPE = 2,    /* shape the kernels do not support */
  ESP_ECAPACITY = 3, /* rows / batch / length beyond what ctx or workspace was created for */
  ESP_EDTYPE = 4,
  ESP_EDEVICE = 5,   /* a HIP call failed */
  ESP_ESTATE = 6
} esp_status;

typedef enum { ESP_F32 = 0, ESP_BF16 = 1 } esp_dtype;

enum { ESP_LAYOUT_PER_NODE = 0, ESP_LAYOUT_ROOT_CHAIN = 1 };

enum {
  ESP_MAX_MASKS = 8,         /* k */
  ESP_MAX_ROWS_PER_SEQ = 1024,
  ESP_MAX_TOPK = 32,         /* K' */
  ESP_MAX_TREE_NODES = 256,  /* B */
  ESP_KV_BLOCK = 64          /* V-cache slot blocking, see esp_kv */
};

/* bits of the device status word */
enum {
  ESP_DEV_LEN_OVER_BOUND = 1,  /* kv.len[b] + n_rows[b] exceeds kv.len_bound or seq capacity */
  ESP_DEV_BAD_TREE = 2,        /* parent not before child, n_nodes/n_rows out of range      */
  ESP_DEV_BAD_TOKEN = 4        /* token id outside the vocabulary                            */
};

typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ff, vocab;
  float rope_theta; /* rotary base; pairs (i, i + head_dim/2) turn by pos * theta^(-2i/head_dim) */
  float rms_eps;
  int32_t qk_norm;  /* 1: per-head RMSNorm over head_dim on q and k before the rotation */
  int32_t dtype;    /* esp_dtype of weights, KV cache, mask embeddings and hidden_out */
} esp_model_desc;

/* Weights: the arrays of per-layer pointers are HOST arrays of n_layers DEVICE pointers. */
typedef struct {
  const void *embed;             /* [vocab, d_model]                                   */
  const void *lm_head;           /* [vocab, d_model] (untied)                          */
                                 /* bf16 models: every matrix below and lm_head in the */
                                 /* layout of esp_pack_weight; embed stays row-major   */
  const void *final_norm;        /* [d_model]                                          */
  const void *const *wqkv;       /* [(n_q + 2 n_kv) * head_dim, d_model]: q, k, v rows */
  const void *const *wo;         /* [d_model, n_q * head_dim]                          */
  const void *const *w_gate_up;  /* [2 d_ff, d_model].  ESP_F32: all gate rows, then all up rows.
                                  * ESP_BF16: blocks of 32 rows alternate (gate rows 0..31, up rows
                                  * 0..31, gate rows 32..63, ...) before esp_pack_weight, so that the
                                  * projection can apply the SwiGLU in its epilogue */
  const void *const *w_down;     /* [d_model, d_ff]                                    */
  const void *const *norm_attn;  /* [d_model]                                          */
  const void *const *norm_mlp;   /* [d_model]                                          */
  const void *const *q_norm;     /* [head_dim], NULL unless qk_norm                    */
  const void *const *k_norm;     /* [head_dim], NULL unless qk_norm                    */
} esp_weights;

/* KV cache pool (device, model dtype), shared by the sequences of a batch.  k and v each hold
 * [n_layers][n_kv_heads] planes of capacity * head_dim elements.  A plane is a sequence of blocks
 * of 32 slots; inside a block the elements sit in the order the matrix cores consume them
 * (64 lanes x 8 elements per fragment), head_dim a multiple of 32:
 *   k block: [head_dim/16][64][8]     element (slot, d) at ((d/16)*64 + ((d/8)%2)*32 + slot%32)*8 + d%8
 *   v block: [head_dim/32][2][64][8]  element (slot, d), key = slot%32, at
 *            (((d/32)*2 + key/16)*64 + ((key/4)%2)*32 + d%32)*8 + 4*((key/8)%2) + key%4
 * Callers never index the pool themselves: esp_kv_store / esp_kv_load convert from and to plain
 * [slots][head_dim] rows.
 * Sequence b owns slots [base[b], base[b] + seq_cap[b]); base[b] is a multiple of 64.
 * Slots [0, len[b]) of a sequence hold committed tokens; a forward writes the block's rows at
 * len[b] + row (scratch until committed). */
typedef struct {
  void *k, *v;             /* device */
  int32_t *len;            /* device [batch]; advanced by esp_verify_accept                   */
  const int32_t *base;     /* device [batch]                                                  */
  const int32_t *seq_cap;  /* device [batch]                                                  */
  int64_t capacity;        /* host: slots per (layer, kv head) in the pool, multiple of 64    */
  int32_t len_bound;       /* host: upper bound of len[b] over the batch for this call; sizes */
                           /* the attention launch (the kernels read the true len on device)  */
} esp_kv;

/* One forward block.  Scalars are host values; arrays are device memory sized for
 * batch * rows_per_seq rows, written by esp_build_prune_tree / esp_block_from_tree. */
typedef struct {
  int32_t batch;
  int32_t rows_per_seq; /* row stride of a sequence, <= ESP_MAX_ROWS_PER_SEQ               */
  int32_t k_masks;      /* k, 0..ESP_MAX_MASKS                                              */
  int32_t layout;
  int32_t anc_words;    /* 64-bit words per ancestor bitset = ceil(rows_per_seq / 64)       */
  int32_t *n_rows;      /* [batch]                                                          */
  int32_t *n_nodes;     /* [batch]                                                          */
  int32_t *tok;         /* [rows] token id of node rows, -1 on mask rows                    */
  int32_t *parent;      /* [rows] tree parent row (in-sequence index), -1 for the root;     */
                        /*        mask rows: the row before them in their chain             */
  int32_t *depth;       /* [rows] position of a row = len[b] + depth (App. E)               */
  int32_t *mask_j;      /* [rows] 0 for node rows, 1..k for mask rows                       */
  int32_t *attach;      /* [rows] node row a mask row hangs on (node rows: themselves)      */
  uint64_t *anc;        /* [rows][anc_words] bit c set: row may attend to block row c       */
} esp_block;

/* Parameters of the tree builder (Alg. 1; Sec. 3.5). */
typedef struct {
  int32_t B;            /* node budget including the root, <= ESP_MAX_TREE_NODES             */
  int32_t k;            /* mask tokens = maximum depth                                       */
  int32_t K;            /* cap on children per expanded node (children = min(K, B - i))      */
  int32_t expand_width; /* nodes expanded per depth: 1 = Top-1 expansion (App. C), <=0 = all */
  int32_t prune_parent; /* drop a candidate equal to its parent's token (Sec. 3.5)           */
  int32_t prune_last;   /* also drop the last generated token at depths >= 2                 */
  int32_t layout;       /* layout of the block to write                                      */
  int32_t static_widths[ESP_MAX_MASKS]; /* [K_1..K_k] fixed tree, no selection; all 0 = dynamic */
} esp_tree_params;

const char *esp_status_str(esp_status s);

/* Workspace (device scratch for activations, split-K partials, attention partials, logits of
 * the mask rows).  max_rows_per_seq and max_batch bound every later block; max_kv_len bounds
 * kv.len_bound + rows_per_seq. */
size_t esp_workspace_bytes(const esp_model_desc *m, int32_t max_batch, int32_t max_rows_per_seq,
                           int64_t max_kv_len);

/* Creates the host context.  `workspace` is device memory of at least esp_workspace_bytes(),
 * 256-byte aligned, owned by the caller and used by every call until esp_destroy.  `stream` is a
 * hipStream_t (NULL = the default stream).  Calls on one ctx must not overlap.
 * Errors: EINVAL (null / non-positive sizes), ESHAPE (head_dim not in {64,128} for bf16 models,
 * d_model or d_ff not a multiple of 64 for bf16, n_q_heads not a multiple of n_kv_heads, ...),
 * ECAPACITY (workspace too small), EDTYPE. */
esp_status esp_create(const esp_model_desc *m, const esp_weights *w, int32_t max_batch,
                      int32_t max_rows_per_seq, int64_t max_kv_len, void *workspace,
                      size_t workspace_bytes, void *stream, esp_ctx **out);
esp_status esp_destroy(esp_ctx *ctx);

/* Synchronises the stream and returns (and clears) the sticky device status bits. */
esp_status esp_last_device_status(esp_ctx *ctx, int32_t *host_out);

/* ---- the four calls of a step ------------------------------------------------------------ */

/* Sample matching (the paper's temperature-1 mode, Sec. 4 / appendix on sampling): when enabled,
 * node_argmax[r] of esp_tree_forward is not the arg-max but a temperature-1 draw of the token that
 * follows row r, taken as arg-max over the vocabulary of logit + Gumbel noise.  The noise is a
 * counter-based function of (seed, absolute position of the drawn token, token id), so the draw at a
 * position is the same whether that position is reached by one-token-at-a-time decoding or inside a
 * tree, and esp_verify_accept (exact match against the draws) stays lossless with respect to
 * sampling with the same seed.  Disabled (greedy) after esp_create.  Host state only; applies to
 * later esp_tree_forward calls on this context. */
esp_status esp_set_sampling(esp_ctx *ctx, int32_t enabled, uint32_t seed);

/* Forward of all rows of `blk` (Sec. 3.3): h0 = embed[tok] on node rows, mask_embed[j-1] on mask
 * rows (Sec. 3.1); per layer RMSNorm, QKV, optional QK-norm, rotary at position len[b]+depth,
 * K/V of the rows written to cache slots len[b]+row, tree-masked grouped-query attention over
 * cache slots [0,len[b]) plus the block rows in the row's ancestor bitset (App. C), output
 * projection, SwiGLU MLP; final RMSNorm.
 *   mask_embed  device [k_masks, d_model], model dtype ([batch, k_masks, d_model] after esp_set_mask_batch)
 *   hidden_out  device [batch*rows_per_seq, d_model], model dtype: final-norm hidden states
 *   node_argmax device [batch*rows_per_seq] int32: argmax over the vocabulary of the LM head at
 *               node rows (lowest id on ties); entries of mask rows are left untouched
 *   logits_dbg  NULL, or device [batch*rows_per_seq, vocab] fp32 receiving the LM-head logits of
 *               every row (parity tests)
 * Errors: EINVAL, ECAPACITY (batch/rows beyond ctx, len_bound + rows_per_seq > max_kv_len). */
esp_status esp_tree_forward(esp_ctx *ctx, const esp_block *blk, const void *mask_embed,
                            const esp_kv *kv, void *hidden_out, int32_t *node_argmax,
                            float *logits_dbg);

/* Greedy verification (Sec. 2 Eq. 3): starting at the root, a child is accepted iff its token
 * equals node_argmax of its parent; the walk ends at the first miss at node n*; node_argmax[n*]
 * is the bonus token (Sec. 4: tau counts accepted + bonus).  Then the K/V of the accepted rows are
 * moved to slots len+1.. in path order (the root already sits at len) and len[b] += n_emit[b].
 * Outputs (device): n_emit [batch]; emit_tok, accepted_row [batch][ESP_MAX_MASKS+1]
 * (accepted_row[b][0] = 0, the root, then the accepted rows); star_row [batch] = n*. */
esp_status esp_verify_accept(esp_ctx *ctx, const esp_block *blk, const int32_t *node_argmax,
                             const esp_kv *kv, int32_t *n_emit, int32_t *emit_tok,
                             int32_t *accepted_row, int32_t *star_row);

/* Proposal (Sec. 2 Eq. 2; Sec. 3.3): LM head on the mask rows aligned to the accepted position,
 * softmax over the full vocabulary in fp32, the Kp most probable tokens per row ordered by
 * (probability descending, id ascending).  PER_NODE: rows mask(n*, i), i = 1..k.  ROOT_CHAIN:
 * rows mask(root, a+i), i = 1..k-a, with a = n_emit-1 accepted tokens.
 *   hidden   device: hidden_out of esp_tree_forward, unchanged since that call.  For blocks of at
 *            most 128 rows (bf16) the forward has already taken all rows through the LM head and
 *            left the logits in the workspace; this call then reads its rows there instead of
 *            streaming the LM-head matrix a second time (recognised by the same `hidden` pointer
 *            and row count; any other esp_tree_forward in between invalidates it)
 *   topk_id  device [batch][k_masks][Kp] int32;  topk_p same shape fp32
 *   n_lists  device [batch] int32: number of valid lists (depths the next tree may have)
 *   logits_out NULL or device [batch][k_masks][vocab] fp32 (parity tests)
 * Errors: EINVAL (Kp < 1 or > ESP_MAX_TOPK or > vocab). */
esp_status esp_mask_topk(esp_ctx *ctx, const esp_block *blk, const int32_t *star_row,
                         const int32_t *n_emit, const void *hidden, int32_t Kp, int32_t *topk_id,
                         float *topk_p, int32_t *n_lists, float *logits_out);

/* Pruning + dynamic tree (Alg. 1, Sec. 3.5): root = last emitted token with P = 1; for depth
 * i = 1..n_lists the expanded nodes of depth i-1 (all of the current node set, or its
 * expand_width most probable) take their first min(K, B-i) candidates of list i that survive the
 * pruning rule, P(child) = P(parent) * p as one fp32 product; between depths the node set is the
 * B-i most probable not-yet-used candidates; the tree is the root plus the B-1 most probable of
 * all candidates (ties: earlier created first).  Writes every array of `next` for each sequence.
 * Fixed trees (static_widths set; Sec. 4.3): root, K_1 children, K_i children under the first node
 * of depth i-1.  Their rows do not depend on the lists, so they are built once per block: the
 * context remembers which blocks (by the address of `tok`) hold the rows of which fixed tree, and a
 * later call with the same parameters writes only the tokens (per sequence the kernel still checks
 * that the block holds a tree of that size and that no list runs out, and builds in full if not).
 * A caller that writes the structure arrays of such a block itself must pass the block through
 * esp_block_from_tree before the next esp_build_prune_tree.
 * Errors: EINVAL (B, k, K, Kp out of range; k != next->k_masks), ECAPACITY (rows of the tree
 * exceed next->rows_per_seq). */
esp_status esp_build_prune_tree(esp_ctx *ctx, const esp_tree_params *p, const int32_t *topk_id,
                                const float *topk_p, int32_t Kp, const int32_t *n_lists,
                                const int32_t *n_emit, const int32_t *emit_tok, esp_block *next);

/* ---- stage-level and auxiliary entry points ----------------------------------------------- */

/* Fills depth, mask rows, attach, mask_j, parent of mask rows, n_rows and the ancestor bitsets
 * from blk->tok / blk->parent / blk->n_nodes of the node rows (already on the device). */
esp_status esp_block_from_tree(esp_ctx *ctx, esp_block *blk);

/* Mask vectors (Sec. 3.1): Eq. 4, m_i = mean of embed[prompt tokens] (fp32 accumulation), and
 * Eq. 5, m <- m + lambda (embed[last emitted token of sequence 0] - m).  mask_embed: device
 * [k, d_model] model dtype.  tokens: device int32. */
esp_status esp_mask_mean(esp_ctx *ctx, const int32_t *tokens, int32_t n_tokens, int32_t k,
                         void *mask_embed);
esp_status esp_mask_ema(esp_ctx *ctx, const int32_t *n_emit, const int32_t *emit_tok, float lambda,
                        int32_t k, void *mask_embed);

/* Mask vectors per sequence (Eq. 4 and Eq. 5 are stated per generation).  esp_set_mask_batch with
 * per_sequence != 0 makes esp_tree_forward read the mask rows of sequence b from
 * mask_embed + b * k_masks * d_model, i.e. mask_embed is device [batch, k_masks, d_model]; 0 (the state a
 * new context is in) is the shared [k_masks, d_model] form.  Host-side state only: takes effect for the calls
 * enqueued after it.  esp_mask_ema_batch is Eq. 5 for that form: the vectors of sequence b move towards
 * the embedding of b's own last emitted token (n_emit[b], emit_tok[b][.]); sequences that emitted nothing
 * keep theirs.  The initialisers above write one [k, d_model] slice per call: pass mask_embed + b * k * d_model. */
esp_status esp_set_mask_batch(esp_ctx *ctx, int32_t per_sequence);
esp_status esp_mask_ema_batch(esp_ctx *ctx, int32_t batch, const int32_t *n_emit, const int32_t *emit_tok,
                              float lambda, int32_t k, void *mask_embed);

/* The two other initialisations of the mask-design ablation (Sec. 4) and the out-of-distribution
 * rows of the appendix table on mask initialisation.
 * esp_mask_last_k: hard initialisation, mask i (0-based) = embed[tokens[n_tokens - k + i]], the last
 *   k prompt tokens in prompt order (the index printed in the paper would skip exactly those
 *   tokens; its words are followed).  EINVAL if n_tokens < k.
 * esp_mask_gaussian: m_i = mu + (shift + z_i) sigma with the Gaussian fit of the embedding table:
 *   mu[d_model] the mean over the vocabulary per dimension, sigma one scalar, the root mean square
 *   deviation of all entries from their dimension's mean (two passes over the table, fp32 slab
 *   sums added in fp64).  z: device fp32 [k, d_model], the caller's standard normal draws (the
 *   library draws nothing), or NULL for z = 0; shift 0 gives the paper's "Sample" variant, z NULL
 *   with shift 5 or 10 its mu + 5 sigma and mu + 10 sigma rows.  Uses the context's logits buffer
 *   as scratch (logits kept for esp_mask_topk by the last esp_tree_forward are dropped).
 * mask_embed: device [k, d_model] model dtype. */
esp_status esp_mask_last_k(esp_ctx *ctx, const int32_t *tokens, int32_t n_tokens, int32_t k,
                           void *mask_embed);
esp_status esp_mask_gaussian(esp_ctx *ctx, const float *z, float shift, int32_t k, void *mask_embed);

/* Copies plain K/V rows [n_slots][n_kv_heads][head_dim] (model dtype, device) of one layer into /
 * out of the cache layout at slots base + first_slot .. */
esp_status esp_kv_store(esp_ctx *ctx, const esp_kv *kv, int32_t layer, int32_t seq_base,
                        int32_t first_slot, int32_t n_slots, const void *k_rows, const void *v_rows);
esp_status esp_kv_load(esp_ctx *ctx, const esp_kv *kv, int32_t layer, int32_t seq_base,
                       int32_t first_slot, int32_t n_slots, void *k_rows, void *v_rows);

/* Rewrites a row-major bf16 matrix W[N,K] (device) into the streaming layout the bf16 GEMMs read:
 * tiles of 32 output rows x 64 inputs, each 4 KB contiguous in MFMA operand order, tiles ordered
 * [K/64][N/32].  dst: device, N*K bf16, must not alias src.  Needs N % 32 == 0, K % 64 == 0.
 * Every bf16 matrix handed to esp_create (wqkv, wo, w_gate_up, w_down, lm_head) must be in this
 * layout; embed and the norm gains stay plain.  fp32 models use plain row-major matrices. */
esp_status esp_pack_weight(void *stream, const void *src, void *dst, int32_t N, int32_t K);

/* C[M,N] (fp32, device) = A[M,K] * W[N,K]^T, A and W in `dtype` (device), on `stream`.
 * bf16 needs N % 32 == 0 and K % 64 == 0; w_packed != 0: W is in the streaming layout.
 * `partials` is device scratch of esp_gemm_scratch_bytes(M,N,K) bytes (split-K partial sums;
 * reduced in a fixed order). */
size_t esp_gemm_scratch_bytes(int32_t M, int32_t N, int32_t K);
esp_status esp_gemm(void *stream, int32_t dtype, const void *A, const void *W, int32_t w_packed,
                    float *C, int32_t M, int32_t N, int32_t K, void *partials, size_t partial_bytes);

/* LM head with the greedy choice of Sec. 2 Eq. 3 taken in the GEMM's epilogue (the path
 * esp_tree_forward uses at the tree rows): argmax[m] = arg-max over n of A[m,:] . W[n,:], lowest n on
 * ties, for bf16 A[M,K] and W[N,K] in the streaming layout (both device).  The [M,N] logits are never
 * written.  `scratch`: device, esp_gemm_argmax_scratch_bytes(M,N) bytes (per-tile (value, index)
 * pairs).  ESP_ESHAPE if N % 32 or K % 64. */
size_t esp_gemm_argmax_scratch_bytes(int32_t M, int32_t N);
esp_status esp_gemm_argmax(void *stream, const void *A, const void *W, int32_t M, int32_t N, int32_t K,
                           void *scratch, size_t scratch_bytes, int32_t *argmax);

/* Tree-masked grouped-query attention of one layer (the kernel esp_tree_forward uses):
 * q device [batch*rows_per_seq, n_q_heads, head_dim] model dtype, already rotated; K/V of the
 * block rows already in the cache at len[b]+row; out same shape as q. */
esp_status esp_attn_tree(esp_ctx *ctx, const esp_block *blk, const esp_kv *kv, int32_t layer,
                         const void *q, void *out);

/* Fused softmax + Top-K over `rows` fp32 logit rows of `vocab` entries (device): ids/probs
 * [rows][Kp], ordered by (probability descending, id ascending).  `scratch`: device memory of
 * esp_softmax_topk_scratch_bytes() bytes (per-chunk statistics and candidates). */
size_t esp_softmax_topk_scratch_bytes(int32_t rows, int32_t vocab, int32_t Kp);
esp_status esp_softmax_topk(void *stream, const float *logits, int32_t rows, int32_t vocab,
                            int32_t Kp, int32_t *ids, float *probs, void *scratch,
                            size_t scratch_bytes);

/* esp_softmax_topk for callers that cannot allocate or bring a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the per-segment records live in a
 * device array that is part of the library image (2.06 MiB per GPU, held until the process ends)
 * instead of `scratch`.  Same kernels, same results as esp_softmax_topk.  The call allocates
 * nothing and synchronises nothing; the device that is current at the call must be the stream's.
 * Limit: rows * min(64, ceil(vocab / 2048)) * (2 + 2 Kp) <= 128 * 64 * 66 floats, i.e. up to 128
 * rows at any vocabulary and Kp (more rows for smaller vocabularies or Kp); beyond that
 * ESP_ECAPACITY and nothing is launched.  All calls on one GPU share the one array: calls that
 * overlap in time on the same GPU (different streams or threads) race; successive calls on one
 * stream do not (every record a call reads it has written itself).
 * Errors: EINVAL as esp_softmax_topk, ECAPACITY, EDEVICE (symbol lookup or launch failed). */
esp_status esp_softmax_topk_static(void *stream, const float *logits, int32_t rows, int32_t vocab,
                                   int32_t Kp, int32_t *ids, float *probs);

/* Optional timing of launch sites with HIP events recorded on the ctx stream (benchmarks).
 * esp_profile_enable: bit s of site_mask turns site s on (0 = off, the default; events are host
 * objects, no device memory is allocated).  esp_profile_read: synchronises the stream, adds the
 * finished spans to per-site totals and returns, then clears, the totals of `site`. */
enum {
  ESP_SITE_GEMM_LAYER = 0, /* QKV, O, gate/up and down projections          */
  ESP_SITE_ATTN = 1,       /* tree attention main kernel                    */
  ESP_SITE_ATTN_MERGE = 2,
  ESP_SITE_LM_HEAD = 3,    /* LM-head GEMMs (tree rows and mask rows)       */
  ESP_SITE_TOPK = 4,       /* softmax + Top-K (both passes)                 */
  ESP_SITE_TREE = 5,       /* verify/commit, row lists, tree build          */
  ESP_SITE_GLUE = 6,       /* embed, norms, rotary/KV append, SwiGLU, argmax */
  ESP_SITE_COUNT = 7
};
esp_status esp_profile_enable(esp_ctx *ctx, uint32_t site_mask);
esp_status esp_profile_read(esp_ctx *ctx, int32_t site, int64_t *launches, double *total_ms);

#ifdef __cplusplus
}
#endif
#endif /* ESP_H_ */
