/*
 * libspecvla_verify - the per-step tree-verification pass of Spec-VLA on one MI355X (gfx950).
 *
 * What the pass computes (paper: Alg. 1, the step "compute the reference token set in
 * parallel"; Sec. 4.1: the draft tokens form a tree whose paths are verified in parallel;
 * Sec. 4.3 / Eq. 5: relaxed acceptance): a Llama-shaped verifier scores all T nodes of a draft
 * token tree in one forward pass over a prefix KV cache, takes the greedy argmax over the
 * action tokens at every node (Eq. 1), accepts a draft token when the distance between its
 * bin and the verifier's bin is at most r, and returns the longest accepted root-to-node path
 * plus the verifier's own token that follows it.
 *
 * Conventions
 *   - Plain C ABI.  Every pointer is tagged [host] or [device] below.  The caller owns every
 *     buffer; the library allocates no device memory and frees nothing.  Between calls it keeps
 *     nothing but read-only facts about the device (how many XCDs it has) and, for the one call
 *     that takes no workspace (sv_action_head_argmax_noalloc), the address of its built-in
 *     scratch.  `stream` is a hipStream_t passed as void*; all device work of a call is enqueued
 *     on it and the call returns without waiting for it.
 *   - Every call returns an int status: SV_OK (0) or a negative SV_ERR_* code.  Arguments are
 *     checked on the host before anything is launched; on error nothing was launched.
 *     Faults inside kernels surface at the caller's next synchronisation, as with any launch.
 *   - Calls that share no buffers may run concurrently from several threads.
 *   - Rows of matrices are contiguous ("[rows, cols]" = row-major).  Weights are stored
 *     [out_features, in_features] as in Llama checkpoints.
 *   - T counts the root: node 0 of every tree is the last committed token, nodes 1..T-1 are
 *     draft tokens.  parent[0] = -1 and 0 <= parent[i] < i.  depth(root) = 0.
 *   - The residual stream x is always float32, whatever the storage type of weights and
 *     cache: activations are a negligible share of the bytes moved and keeping them wide
 *     keeps near-tie argmax flips rare.
 */
#ifndef SPECVLA_VERIFY_H
#define SPECVLA_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SV_OK 0
#define SV_ERR_NULL (-1)      /* a required pointer is NULL */
#define SV_ERR_SHAPE (-2)     /* a size is unsupported (see each call) */
#define SV_ERR_TREE (-3)      /* parent array is not a tree in the stated form, or too deep */
#define SV_ERR_TOKEN (-4)     /* action range / threshold arguments are inconsistent */
#define SV_ERR_WORKSPACE (-5) /* workspace or packed buffer too small or misaligned */
#define SV_ERR_DTYPE (-6)     /* cfg->dtype is none of SV_F32, SV_BF16, SV_BF16_W8, SV_BF16_W4 (or the wrong one for the call) */
#define SV_ERR_LAUNCH (-7)    /* the HIP runtime reported an error at launch */

#define SV_F32 0
#define SV_BF16 1
/* A bf16 model (gains, KV cache, LM head and activations as with SV_BF16) whose seven matrices
 * per layer are stored in 8 bits - E4M3 codes of the OCP 8-bit floating point specification -
 * with one float32 scale per output row: W[n][k] = value(code[n][k]) * scale[n].  The paper's
 * App. C runs the verifier on weights held in fewer bits; on a path bound by the bytes of the
 * weights this halves them.  Packed with sv_pack_layer_w8; every other call is the same. */
#define SV_BF16_W8 2
/* The same with 4-bit integer codes (App. C, Tables 5 and 6: int4 weights): a code c in 0 .. 15
 * stands for the integer c - 8, W[n][k] = (code[n][k] - 8) * scale[n] with one float32 scale per
 * output row; a raw matrix holds two codes per byte, the code of the even k in the low four
 * bits.  Packed with sv_pack_layer_w4 (K of every matrix must be a multiple of 256, as for
 * SV_BF16); every other call is the same. */
#define SV_BF16_W4 3

#define SV_MAX_TREE_NODES 128 /* T <= 128: the ancestor mask has at most two 64-bit words */
#define SV_MAX_DEPTH 31       /* depth of a node, in edges */

/* Shape of the verifier (Sec. 4.1, 5.1: OpenVLA = Llama-2 backbone). */
typedef struct sv_model_cfg {
  int32_t dtype;      /* SV_F32, SV_BF16, SV_BF16_W8 or SV_BF16_W4: storage type of weights and KV cache */
  int32_t hidden;     /* H */
  int32_t n_heads;    /* nh (multi-head attention, n_kv_heads = n_heads) */
  int32_t head_dim;   /* d; nh * d is the attention width (need not equal H) */
  int32_t mlp_dim;    /* F, SwiGLU inner width */
  int32_t vocab;      /* V, rows of the LM head */
  float rms_eps;      /* RMSNorm epsilon */
  float rope_theta;   /* RoPE base */
} sv_model_cfg;

/* One decoder layer as the caller holds it: [device] pointers, cfg->dtype elements.
 * g1, g2: [H]; wq, wk, wv: [nh*d, H]; wo: [H, nh*d]; wg, wu: [F, H]; wd: [H, F]. */
typedef struct sv_layer_weights {
  const void *g1, *wq, *wk, *wv, *wo, *g2, *wg, *wu, *wd;
} sv_layer_weights;

/* KV cache of ONE layer for B episodes.  k and v: [device], layout
 * [B][n_heads][capacity][head_dim], cfg->dtype.  Rows 0 .. prefix_len[b]-1 of episode b
 * hold the prefix (vision patches + instruction tokens; keys already rotated) and are only
 * read.  sv_verify_layer WRITES the tree's own rotated keys and values to rows
 * prefix_len[b] .. prefix_len[b]+T-1, so capacity >= prefix_len_max + T is required.
 * prefix_len: [device] int32[B].  prefix_len_max: [host value] an upper bound of all
 * prefix_len[b], used for checking and launch planning; kernels clamp prefix_len[b] to it. */
typedef struct sv_kv_view {
  void *k;
  void *v;
  const int32_t *prefix_len;
  int32_t prefix_len_max;
  int32_t capacity;
} sv_kv_view;

/* Draft trees of B episodes, T nodes each, as produced by sv_tree_build_masks and copied
 * to the device by the caller.  All [device]: parent int32[B*T], depth int32[B*T],
 * anc_mask uint64[B*T*n_words] with n_words = ceil(T/64); bit j of node i's mask (word j/64)
 * is set iff node j lies on the path root..i, i itself included. */
typedef struct sv_tree {
  const int32_t *parent;
  const int32_t *depth;
  const uint64_t *anc_mask;
  int32_t n_nodes; /* T, 1..SV_MAX_TREE_NODES */
  int32_t n_words; /* ceil(T/64) */
} sv_tree;

const char *sv_version(void);
const char *sv_strerror(int status);

/* Host-only.  Checks B parent arrays ([host] int32[B*T]: parent[b*T] = -1, 0 <= parent < own
 * index otherwise) and derives depth ([host] int32[B*T]) and ancestor-or-self masks ([host]
 * uint64[B*T*ceil(T/64)]).  These encode which keys a tree node may attend to and its
 * position P + depth (Sec. 4.1: every path of the tree is verified as if decoded alone).
 * SV_ERR_TREE if an array is not such a tree or a depth exceeds d_cap (d_cap <= SV_MAX_DEPTH);
 * SV_ERR_SHAPE if T is outside 1..SV_MAX_TREE_NODES or B < 1. */
int sv_tree_build_masks(const int32_t *parent, int B, int T, int d_cap, int32_t *depth,
                        uint64_t *anc_mask);

/* Host-only.  Bytes of the packed form of one layer (sv_pack_layer) -> *bytes. */
int sv_packed_layer_bytes(const sv_model_cfg *cfg, size_t *bytes);

/* One-time, load-time re-tiling of a layer's nine tensors into the order the kernels stream
 * them (q/k/v fused, gate/up fused, matrices cut into matrix-core fragments, gains widened to
 * float32).  raw: [host] struct of [device] pointers; packed: [device], 256-byte aligned,
 * packed_bytes >= sv_packed_layer_bytes.  The packed layout is private to the library and
 * may change between versions; raw tensors are not needed afterwards.
 * SV_BF16 needs d = 128 and H, nh*d, F multiples of 256; SV_F32 takes any sizes with d even
 * and d <= 128. */
int sv_pack_layer(const sv_model_cfg *cfg, const sv_layer_weights *raw, void *packed,
                  size_t packed_bytes, void *stream);

/* The row scales of a layer's matrices for SV_BF16_W8 and SV_BF16_W4: [device] float32, sq, sk, sv: [nh*d];
 * so, sd: [H]; sg, su: [F]. */
typedef struct sv_layer_scales {
  const float *sq, *sk, *sv, *so, *sg, *su, *sd;
} sv_layer_scales;

/* sv_pack_layer for cfg->dtype = SV_BF16_W8 (App. C: weights in fewer bits): raw->g1, g2 are
 * bf16 gains, raw->wq .. wd uint8 E4M3 codes in the shapes of sv_layer_weights, scales their
 * row scales.  Same size rules as SV_BF16; packed_bytes >= sv_packed_layer_bytes(cfg).
 * SV_ERR_DTYPE for any other dtype (and sv_pack_layer returns it for SV_BF16_W8). */
int sv_pack_layer_w8(const sv_model_cfg *cfg, const sv_layer_weights *raw,
                     const sv_layer_scales *scales, void *packed, size_t packed_bytes,
                     void *stream);

/* sv_pack_layer for cfg->dtype = SV_BF16_W4 (App. C: int4 weights): raw->g1, g2 are bf16 gains,
 * raw->wq .. wd the int4 codes, [device] uint8 [out][in / 2] (two codes per byte, even k in the
 * low four bits), scales their row scales as for sv_pack_layer_w8.  Same size rules as SV_BF16;
 * packed_bytes >= sv_packed_layer_bytes(cfg).  SV_ERR_DTYPE for any other dtype (and
 * sv_pack_layer returns it for SV_BF16_W4). */
int sv_pack_layer_w4(const sv_model_cfg *cfg, const sv_layer_weights *raw,
                     const sv_layer_scales *scales, void *packed, size_t packed_bytes,
                     void *stream);

/* Host-only.  Bytes of device scratch that sv_verify_layer / sv_action_head_argmax need for
 * B episodes of T nodes and up to n_scored scored vocabulary rows -> *bytes. */
int sv_workspace_bytes(const sv_model_cfg *cfg, int B, int T, int n_scored, size_t *bytes);

/* Prepares a freshly allocated (or otherwise dirty) workspace: zeroes the inter-workgroup
 * arrival counters at its start with a small kernel on `stream`.  Call once after allocating
 * the workspace and before its first use; every later call of the library leaves the counters
 * zero again.  workspace: [device], 256-byte aligned, ws_bytes >= sv_workspace_bytes(...). */
int sv_workspace_init(const sv_model_cfg *cfg, int B, int T, int n_scored, void *workspace,
                      size_t ws_bytes, void *stream);

/* The draft tree of every episode, built on the device from the recorded top-K predictions of
 * the draft model (Sec. 4.1: those predictions form a tree with several paths; Sec. 5.1: top 8,
 * at most 50 nodes).  Candidate c of an episode has a parent (an earlier candidate, or -1 =
 * the root), a token and the log-probability the drafter gave it; its score is the joint
 * log-probability of its path, accumulated in float32 from the root down.  The T - 1 best
 * candidates are kept (lower candidate index wins ties), numbered breadth first behind the
 * root (by depth, then candidate index).  The outputs are what sv_tree / sv_relaxed_accept
 * take.
 *   cand_parent, cand_token: [device] int32 [B, n_cand];  cand_logp: [device] float32 [B, n_cand]
 *   root_token: [device] int32 [B] (becomes draft_token of node 0)
 *   parent, depth, draft_token: [device, out] int32 [B, T];  anc_mask: [device, out] uint64
 *   [B, T, ceil(T/64)];  status: [device, out] int32 [B]: 0 = ok, bit 0 = some cand_parent is
 *   not an earlier candidate, bit 1 = a kept candidate is deeper than d_cap, bit 2 = a kept
 *   candidate's parent was not kept (log-probabilities above zero); a flagged episode gets a
 *   valid placeholder tree (all nodes children of the root).
 * SV_ERR_SHAPE unless 1 <= T <= SV_MAX_TREE_NODES, T - 1 <= n_cand <= 1024, B >= 1,
 * 0 <= d_cap <= SV_MAX_DEPTH.  Nothing is read on the host. */
int sv_tree_build_device(const int32_t *cand_parent, const float *cand_logp,
                         const int32_t *cand_token, int n_cand, const int32_t *root_token, int B,
                         int T, int d_cap, int32_t *parent, int32_t *depth, uint64_t *anc_mask,
                         int32_t *draft_token, int32_t *status, void *stream);

/* One decoder layer over all B*T tree nodes (Alg. 1's parallel verification, one layer of
 * M_V): RMSNorm, q/k/v projections, RoPE at position prefix_len[b] + depth, append of the
 * tree's keys/values to the cache, attention of node i over {prefix keys} + {tree nodes on
 * the path root..i}, output projection + residual, RMSNorm, SwiGLU MLP + residual.
 *   packed:    [device] from sv_pack_layer (same cfg)
 *   x:         [device] float32 [B*T, H], residual stream, updated in place
 *   kv, tree:  [host] structs of [device] pointers, see above; tree->n_nodes = T
 *   workspace: [device], 256-byte aligned, ws_bytes >= sv_workspace_bytes(cfg, B, T, *),
 *              prepared once with sv_workspace_init; calls sharing a workspace must not overlap
 * bf16 models (also with 8-bit or 4-bit weights): up to 64 rows, and any number of rows with
 * 8-bit or 4-bit weights, the projections are split along K and their partial sums travel
 * in 16 bits with one scale per 64-row x 32-column tile (error <= 2^-14 of the tile's largest
 * partial sum, each row first brought to a common size); with more than 64 rows and bf16
 * weights the projections run on kernels bound by the matrix cores whose partial sums, where K
 * is split at all, are float32.  A partial sum that is not finite
 * travels as a code of its own and comes back as NaN: a NaN or infinity reaches exactly the
 * outputs it reaches by the layer's own arithmetic, one exception aside - inside the tree
 * attention a NaN in the value row of a tree node also reaches the other nodes of that episode
 * and head, whether or not they attend to it (a probability of zero times NaN); other episodes
 * are never touched.  The workgroups of such a projection wait for each other (bounded) and
 * check where they ran; a wait that runs out or an unexpected placement leaves the outputs of
 * the call undefined and raises the status word (sv_workspace_region, SV_WS_STATUS), which
 * callers that cannot rule out a GPU shared with other work should read before they trust or
 * commit the results.
 * (long long) B * n_heads * capacity must stay below 2^31.
 * SV_ERR_SHAPE if B < 1, T outside 1..SV_MAX_TREE_NODES, capacity < prefix_len_max + T, or
 * cfg sizes are unsupported for the dtype (see sv_pack_layer). */
int sv_verify_layer(const sv_model_cfg *cfg, const void *packed, float *x,
                    const sv_kv_view *kv, const sv_tree *tree, int B, void *workspace,
                    size_t ws_bytes, void *stream);

/* The whole verifier stack (Sec. 4.1: M_V scores every draft position in one forward pass):
 * exactly sv_verify_layer for layer 0 .. n_layers-1 in turn on the same x, issued from one call.
 *   packed: [host] array of n_layers [device] pointers, each from sv_pack_layer
 *   kv:     [host] array of n_layers views (one cache per layer)
 *   others: as sv_verify_layer
 * SV_ERR_SHAPE if n_layers < 1; otherwise the errors of sv_verify_layer. */
int sv_verify_stack(const sv_model_cfg *cfg, int n_layers, const void *const *packed, float *x,
                    const sv_kv_view *kv, const sv_tree *tree, int B, void *workspace,
                    size_t ws_bytes, void *stream);

/* Final RMSNorm, LM-head logits of vocabulary rows [vocab_lo, vocab_hi) and the greedy
 * choice among them (Eq. 1), the lowest id winning exact ties.  vocab_lo = V - 256,
 * vocab_hi = V scores the action tokens only (Sec. 4.3: 256 bins <-> 256 tokens).
 *   g_final: [device] [H] cfg->dtype;  w_lm: [device] [V, H] cfg->dtype (plain row-major)
 *   x: [device] float32 [n_rows, H];  out_token: [device] int32[n_rows]
 *   out_logits: [device] float32 [n_rows, vocab_hi - vocab_lo], or NULL
 * SV_ERR_SHAPE unless 0 <= vocab_lo < vocab_hi <= V and n_rows >= 1. */
int sv_action_head_argmax(const sv_model_cfg *cfg, const void *g_final, const void *w_lm,
                          const float *x, int n_rows, int vocab_lo, int vocab_hi,
                          int32_t *out_token, float *out_logits, void *workspace,
                          size_t ws_bytes, void *stream);

/* sv_action_head_argmax for callers that cannot allocate device memory and have no workspace to
 * hand over: code recorded into a HIP graph, tight serving loops, harnesses that forbid
 * hipMalloc.  Same kernels, same results; the scratch (normalised rows, logit planes: 3 MiB) is
 * a fixed array inside the library image, one copy per GPU for the life of the process.  The
 * call allocates nothing and frees nothing.  Limits: n_rows <= 64, vocab_hi - vocab_lo <= 256,
 * hidden <= 8192; beyond them SV_ERR_WORKSPACE and nothing is launched.  All calls on one GPU
 * share that GPU's array: calls that overlap in time on one GPU (different streams or threads)
 * race; calls on one stream are ordered and fine.  Every byte a call reads from the array it
 * has written itself first, so nothing needs clearing between calls. */
int sv_action_head_argmax_noalloc(const sv_model_cfg *cfg, const void *g_final, const void *w_lm,
                                  const float *x, int n_rows, int vocab_lo, int vocab_hi,
                                  int32_t *out_token, float *out_logits, void *stream);

/* The same head for bf16 models (SV_BF16, SV_BF16_W8) on the streaming matrix-core kernel of
 * the layers: the head rows [vocab_lo, vocab_hi) are re-tiled once at load time, and every
 * call then reads them once at streaming speed (final RMSNorm, Eq. 1; Sec. 4.3 for the
 * action rows).  vocab_hi - vocab_lo must be a multiple of 32 and H a multiple of 256.
 *   sv_packed_head_bytes: host-only, bytes of the packed form -> *bytes
 *   sv_pack_head: g_final [device] [H] bf16, w_lm [device] [V, H] bf16 row-major;
 *                 packed [device], 256-byte aligned, packed_bytes >= sv_packed_head_bytes
 *   sv_action_head_argmax_packed: packed_head from sv_pack_head with the same cfg and range;
 *                 x, out_token, out_logits as in sv_action_head_argmax; workspace sized and
 *                 initialised with n_scored = vocab_hi - vocab_lo
 * SV_ERR_DTYPE for SV_F32, SV_ERR_SHAPE for ranges or sizes outside the rules above. */
int sv_packed_head_bytes(const sv_model_cfg *cfg, int vocab_lo, int vocab_hi, size_t *bytes);
int sv_pack_head(const sv_model_cfg *cfg, const void *g_final, const void *w_lm, int vocab_lo,
                 int vocab_hi, void *packed, size_t packed_bytes, void *stream);
int sv_action_head_argmax_packed(const sv_model_cfg *cfg, const void *packed_head, const float *x,
                                 int n_rows, int vocab_lo, int vocab_hi, int32_t *out_token,
                                 float *out_logits, void *workspace, size_t ws_bytes,
                                 void *stream);

/* Relaxed acceptance (Eq. 5, Alg. 1) over B trees and the longest accepted path.  Integer
 * only.  bin(t) = t - action_lo.  Node c >= 1 passes when draft_token[c] and
 * target_token[parent[c]] are both action tokens and |bin difference| <= r; r = 0 is strict
 * matching (Eq. 3).  A node is accepted when it and every node above it pass (tokens after
 * the first rejection on a path are dropped).  best = deepest accepted node, lowest index
 * among equals.
 *   draft_token, target_token: [device] int32[B*T] (entry 0 of each tree's draft is unused)
 *   accept_mask:  [device] uint8[B*T], 1 = accepted (root always 1)
 *   accepted_len: [device] int32[B] = depth(best);  best_node: [device] int32[B]
 *   path:         [device] int32[B, d_cap+1]: root..best, then -1
 *   out_tokens:   [device] int32[B, d_cap+1]: the accepted draft tokens, then the verifier's
 *                 token target_token[best] (Alg. 1: accepted positions keep the draft token;
 *                 the verifier's token fills the first rejected position or is the extra
 *                 token), then -1.  A step thus emits accepted_len + 1 tokens.
 * Nodes deeper than d_cap are treated as rejected.  SV_ERR_TOKEN if n_bins < 1, r < 0 or
 * action_lo < 0; SV_ERR_SHAPE for B < 1, bad T or d_cap outside 0..SV_MAX_DEPTH. */
int sv_relaxed_accept(const sv_tree *tree, const int32_t *draft_token,
                      const int32_t *target_token, int action_lo, int n_bins, int r, int B,
                      int d_cap, uint8_t *accept_mask, int32_t *accepted_len,
                      int32_t *best_node, int32_t *path, int32_t *out_tokens, void *stream);

/* Between two verification passes (the outer loop of Alg. 1): makes the accepted path part of
 * the prefix of ONE layer's cache.  The K/V rows of path[b][1..accepted_len[b]] (appended by
 * sv_verify_layer at rows prefix_len[b] + node) move to rows prefix_len[b] + 1 .. + len; the
 * root already sits at row prefix_len[b].  Call once per layer with that layer's kv view and
 * the path / accepted_len that sv_relaxed_accept wrote ([device] int32 [B, d_cap+1] / [B]); then
 * call sv_advance_prefix once.  The verifier's bonus token out_tokens[b][len] is the root of the
 * next tree.  kv->prefix_len is only read here. */
int sv_commit_path(const sv_model_cfg *cfg, const sv_kv_view *kv, int T, const int32_t *path,
                   const int32_t *accepted_len, int B, int d_cap, void *stream);

/* prefix_len[b] += accepted_len[b] + 1 on the device ([device] int32[B] each).  The caller
 * raises its host-side bound kv.prefix_len_max by d_cap + 1 (or by what it reads back) and must
 * stop, or move to a larger cache, before prefix_len_max + T would exceed the capacity: the next
 * sv_verify_layer refuses such a view (SV_ERR_SHAPE), and kernels clamp prefix_len[b] to
 * prefix_len_max. */
int sv_advance_prefix(int32_t *prefix_len, const int32_t *accepted_len, int B, int d_cap,
                      void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SPECVLA_VERIFY_H */
