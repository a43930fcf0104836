/*
 * cerberus.h — C ABI of the MI355X (gfx950) Cerberus verify-step library.
 *
 * The library runs one decoding step of the Cerberus method (Algorithm 1 of the paper) for a
 * batch of independent sequences on one GPU:
 *   - the base decoder over a static candidate tree with tree-masked attention against the KV
 *     cache (tree verification, Algorithm 1 line 13; tree settings of Section 5.1),
 *   - greedy longest-prefix acceptance and KV-cache compaction,
 *   - the entropy gate on the last hidden state of the last accepted token (Section 4.2),
 *   - the Cerberus heads, all heads per Resblock stage in one launch, and their per-head top-k
 *     (Section 4.1), which give the next step's candidates.
 *
 * Conventions
 *   - Every function returns a cerberus_status (0 = OK, negative = error); nothing throws or
 *     aborts.  Argument errors are detected on the host before any kernel is launched.
 *   - Pointers marked DEVICE are device memory owned by the caller and only borrowed; pointers
 *     marked HOST are ordinary host memory, read during the call only.  The library allocates and
 *     frees no device memory: everything it needs lives in the caller's workspace.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream)
 *     and is asynchronous; only cerberus_init synchronises.  Calls on one context must not
 *     overlap (they share the workspace).
 *   - Matrices are row-major [out][in].  `dtype` selects storage and GEMM-input precision:
 *     CERBERUS_F32 = float everywhere (reference mode for small models),
 *     CERBERUS_BF16 = bf16 weights / KV cache / GEMM inputs, fp32 accumulation, fp32 residual
 *     stream, norms, softmax, entropy and logits.
 *   - Capacity (kv_len + tree size <= kv_capacity) lives on the device and cannot be checked on
 *     the host without a sync; kernels skip out-of-capacity writes and OR a bit into
 *     cerberus_state.status, a sticky device word the caller reads with the other outputs.
 */
#ifndef CERBERUS_H
#define CERBERUS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cerberus_ctx cerberus_ctx; /* opaque, host side */

typedef enum {
  CERBERUS_OK = 0,
  CERBERUS_ERR_ARG = -1,      /* null pointer, negative size, batch out of range            */
  CERBERUS_ERR_SHAPE = -2,    /* config / tree shape the kernels do not support             */
  CERBERUS_ERR_CAPACITY = -3, /* workspace too small                                        */
  CERBERUS_ERR_HIP = -4,      /* a HIP runtime call failed; see cerberus_last_error()       */
  CERBERUS_ERR_UNIMPL = -5
} cerberus_status;

enum { CERBERUS_F32 = 0, CERBERUS_BF16 = 1 };

/* bits of cerberus_state.status (device word) */
enum { CERBERUS_DEV_KV_OVERFLOW = 1, CERBERUS_DEV_BAD_TOKEN = 2, CERBERUS_DEV_LOG_FULL = 4 };

enum { CERBERUS_MAX_TREE = 192, CERBERUS_MAX_HEADS = 8, CERBERUS_MAX_TOPK = 16, CERBERUS_MAX_BATCH = 16 };

/* Model and method parameters (Algorithm 1 "Require": N layers, threshold T; Section 5.1
 * "Training": 4 heads of 4 Resblocks + 1 FC).                                                 */
typedef struct {
  int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
  int32_t n_cerb_heads;    /* Hc, 1..CERBERUS_MAX_HEADS                                      */
  int32_t n_resblocks;     /* R, Resblocks per head                                          */
  int32_t special_block;   /* index of the Resblock that takes Concat(h_i, h_{i-1}) in heads
                              i >= 1 (Section 4.1); from it on those heads are 2*d_model wide.
                              -1 = no link: independent heads, all d_model wide               */
  int32_t dtype;           /* CERBERUS_F32 or CERBERUS_BF16                                  */
  int32_t max_batch;       /* 1..CERBERUS_MAX_BATCH                                          */
  int32_t kv_capacity;     /* rows per sequence in the KV slab                               */
  int32_t topk;            /* candidates kept per head, > max rank used by the tree          */
  float rms_eps, rope_theta;
  float entropy_threshold; /* T of Algorithm 1: entropy > T -> auto-regressive step; may be +inf */
} cerberus_config;

/* Weights, all DEVICE, element type per `dtype`, row-major [out][in].  The pointer arrays
 * themselves are HOST arrays.  In bf16 mode cerberus_init repacks the matrices into the
 * workspace and copies gains and biases, so after it returns only `embed` must stay alive; in
 * fp32 mode the matrices are read in place and must all stay alive.                           */
typedef struct {
  const void *embed;            /* [vocab][d]                                                */
  const void *final_norm;       /* [d]                                                       */
  const void *lm_head;          /* [vocab][d]  (LH of Algorithm 1)                           */
  const void *const *attn_norm; /* [n_layers] -> [d]                                         */
  const void *const *wqkv;      /* [n_layers] -> [3d][d], rows Q then K then V               */
  const void *const *wo;        /* [n_layers] -> [d][d]                                      */
  const void *const *ffn_norm;  /* [n_layers] -> [d]                                         */
  const void *const *w_gate_up; /* [n_layers] -> [2F][d], rows gate then up                  */
  const void *const *w_down;    /* [n_layers] -> [d][F]                                      */
  const void *const *res_w;     /* [Hc*R], entry i*R+s -> [w][w], w = block width (d or 2d)  */
  const void *const *res_b;     /* [Hc*R], entry i*R+s -> [w]                                */
  const void *const *head_fc;   /* [Hc] -> [vocab][w_last], no bias                          */
} cerberus_weights;

/* Static candidate tree (Section 5.1 "Tree Settings"), HOST arrays copied at init.  Node 0 is
 * the root (carries the pending LM-head token); a node at depth delta >= 1 carries candidate
 * `rank[n]` of head delta-1.                                                                 */
typedef struct {
  int32_t n_nodes;       /* T, 1..CERBERUS_MAX_TREE, root included                          */
  const int32_t *parent; /* [T], parent[0] = -1, 0 <= parent[n] < n                         */
  const int32_t *rank;   /* [T], 0 <= rank[n] < topk; depth(n) <= Hc                        */
} cerberus_tree;

/* Per-sequence state, DEVICE arrays indexed by sequence b < batch.  A first step after prefill
 * is seeded by the caller: filled KV rows 0..kv_len-1, root_token, cand, gate_flag.          */
typedef struct {
  void *kv;                 /* [n_layers][2 (K,V)][max_batch][n_heads][kv_capacity][head_dim] */
  int32_t *kv_len;          /* committed rows L_b; advanced by the accepted length            */
  int32_t *root_token;      /* pending token: chosen by the base model, not yet in the cache  */
  int32_t *cand;            /* [batch][Hc][topk] candidates of the heads, best first          */
  int32_t *gate_flag;       /* 1 = next step auto-regressive (entropy > T), 0 = parallel      */
  float *entropy;           /* entropy in bits of the gate's input, last step                 */
  int32_t *accept_len;      /* tokens committed by the last step, 1..Hc+1                     */
  int32_t *accepted_tokens; /* [batch][Hc+1] committed tokens, first accept_len valid         */
  int32_t *accepted_nodes;  /* [batch][Hc+1] their tree nodes                                 */
  int32_t *status;          /* one sticky word, OR of CERBERUS_DEV_* bits                     */
} cerberus_state;

/* Optional taps for tests and benchmarks (one struct standing for both a "set overrides" and a "debug
 * outputs" call), all DEVICE, any may be NULL.  Outputs are written by
 * the next steps; `forced_*` replace computed values.  Row index of node n of sequence b is
 * b*T + n.                                                                                   */
typedef struct {
  float *logits;       /* out [batch*T][vocab] LM-head logits of every tree node             */
  float *h_last;       /* out [batch*T][d] final-norm output of every tree node              */
  float *head_logits;  /* out [batch][Hc][vocab] logits of the decoding heads                */
  int32_t *node_token; /* out [batch*T] token carried by every node                          */
  int32_t *node_argmax;/* out [batch*T] base model's next token at every node                */
  const int32_t *forced_node_argmax; /* in [batch*T]: replaces node_argmax before acceptance */
  const float *forced_gate_hidden;   /* in [batch][d]: replaces the gate's input vector      */
} cerberus_taps;

/* Bytes of DEVICE workspace cerberus_init needs for this config and tree (0 on bad input).    */
size_t cerberus_workspace_bytes(const cerberus_config *cfg, const cerberus_tree *tree);

/* Validates everything, copies the tree tables, repacks the weight matrices into `workspace`
 * (DEVICE, 256-byte aligned, kept by the context until cerberus_destroy) and returns a context.
 * Synchronous.  The device current at the call is the context's device.                       */
int cerberus_init(cerberus_ctx **out, const cerberus_config *cfg, const cerberus_weights *w,
                  const cerberus_tree *tree, void *workspace, size_t workspace_bytes);

/* One decoding step of Algorithm 1 for `batch` sequences.  Sequence b runs the whole tree if
 * gate_flag[b] == 0 and a tree of size 1 (plain auto-regressive step, Algorithm 1 line 9)
 * otherwise; then acceptance, KV compaction, the gate on the last accepted node's h_last and,
 * where the gate says parallel, the heads and their top-k.  Updates every field of `st`.      */
int cerberus_verify_step(cerberus_ctx *ctx, const cerberus_state *st, int32_t batch, void *stream);

/* Same with a tree of size 1 for every sequence, whatever gate_flag says.                      */
int cerberus_ar_step(cerberus_ctx *ctx, const cerberus_state *st, int32_t batch, void *stream);

/* Prompt phase of Algorithm 1 (lines 1-5) for sequence `seq` of the batch: a causal forward of
 * `n_tokens` prompt tokens (DEVICE int32) appended at cache rows kv_len.., in passes of up to
 * CERBERUS_MAX_TREE rows (the result does not depend on the pass size up to the rounding of the cache: rows
 * of earlier passes are read back from the cache in its storage type), then on the last position the LM head (-> root_token), the
 * gate (-> gate_flag, entropy) and, where the gate says parallel, the heads (-> cand): the state a
 * first decoding step starts from.  kv_len[seq] advances by n_tokens; accept_len[seq] is set to 0;
 * the other sequences of the batch are not touched.  Tokens outside the vocabulary count as token 0
 * and set CERBERUS_DEV_BAD_TOKEN; a prompt that does not fit the cache sets CERBERUS_DEV_KV_OVERFLOW
 * and stops at the first pass that no longer fits.                                             */
int cerberus_prefill(cerberus_ctx *ctx, const cerberus_state *st, int32_t batch, int32_t seq,
                     const int32_t *tokens, int32_t n_tokens, void *stream);

/* `n_steps` steps of cerberus_verify_step enqueued back to back (Algorithm 1's loop, lines 6-18):
 * the gate flag a step leaves on the device selects the shape of the next one, nothing crosses to
 * the host in between.  After every step the tokens it committed are appended to the log:
 * out_tokens is DEVICE [batch][out_capacity], out_count DEVICE [batch] (read, then advanced by the
 * step's accept_len).  A sequence whose log is full keeps decoding, logs nothing more and sets
 * CERBERUS_DEV_LOG_FULL; a sequence out of cache capacity sits the remaining steps out
 * (CERBERUS_DEV_KV_OVERFLOW), as in a single step.                                             */
int cerberus_decode(cerberus_ctx *ctx, const cerberus_state *st, int32_t batch, int32_t n_steps,
                    int32_t *out_tokens, int32_t out_capacity, int32_t *out_count, void *stream);

/* The gate alone (Section 4.2): for each of `rows` vectors hidden[r][0..d) (DEVICE, fp32),
 * P = softmax(hidden[r]), entropy_out[r] = -sum P log2 P, flag_out[r] = entropy > T.          */
int cerberus_gate(cerberus_ctx *ctx, const float *hidden, int32_t rows, float *entropy_out,
                  int32_t *flag_out, void *stream);

/* Acceptance and compaction alone (Section 3.1 names tree verification but gives no rule; this is the
 * greedy longest-prefix reading: walk from the root while a child carries the base model's own next
 * token).  node_argmax / node_token are DEVICE [batch*T]; every
 * sequence is taken to have run the whole tree, its K/V in cache rows kv_len..kv_len+T-1.
 * Writes accept_len, accepted_*, root_token, moves cache rows and advances kv_len.            */
int cerberus_accept(cerberus_ctx *ctx, const int32_t *node_argmax, const int32_t *node_token,
                    const cerberus_state *st, int32_t batch, void *stream);

/* cerberus_accept for callers that cannot allocate device memory or hand over a workspace for it
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same inputs,
 * outputs and result, but the kernels' scratch (row map, accepted path, last-row list) lives in a
 * static device array of the library, 32 KB per GPU, held until the process ends.  Limits: up to
 * CERBERUS_MAX_BATCH sequences and 1024 tree rows in all (batch * n_nodes); larger calls return
 * CERBERUS_ERR_CAPACITY.  It calls no allocating routine.  All calls on one GPU share that GPU's
 * array: calls that overlap on one GPU (two streams, two contexts) race; calls in stream order do not.
 * The array's address is resolved by cerberus_init on the context's device.                    */
int cerberus_accept_noalloc(cerberus_ctx *ctx, const int32_t *node_argmax, const int32_t *node_token,
                            const cerberus_state *st, int32_t batch, void *stream);

/* Installs (or, with NULL, clears) the taps; the struct is copied.                             */
int cerberus_set_taps(cerberus_ctx *ctx, const cerberus_taps *taps);

/* Tuning knobs, by name; returns CERBERUS_ERR_ARG for an unknown name or a bad value.  None of
 * them changes what is computed, only how the launches are shaped:
 *   "gemm_target_wgs" (1..65536, default 768)  workgroups a GEMM launch aims for when choosing split-K
 *   "gemm_max_split"  (1..16, default 8)       upper bound of the split-K factor
 *   "gemm_wg_slots"   (0..65536, default 512)  workgroups resident at once (2 per CU x 256 CUs): a split that
 *                                              fills >= 90 % of them in one round is preferred; 0 = off
 *   "gemm_uneven_split" (0 or 1, default 0)    1: take the split the target gives even if it does not divide K
 *   "gemm_nsub"       (2 or 4, default 2)      16-column slabs per wave (64*nsub columns per workgroup)
 *   "gemm_nsub_rows"  (0, 2 or 4, default 0)   the same for launches of more than 64 rows (several row blocks);
 *                                              4 runs one workgroup per CU with the whole register file; 0 picks
 *                                              4 for the down projection and the LM head past 256 rows, else 2
 *   "gemm_team"       (0..3, default 3)        bf16 launches of more than 128 rows run, on the kernel that deals
 *                                              (column block, k) ranges to teams of one workgroup per 128-row
 *                                              block: 1 the gate/up projection, 2 also QKV and 3 also the LM head
 *                                              (these two only past 256 rows);
 *                                              0: everything on the 64-row blocks of the split-K kernel
 *   "act_split"       (0 or 1, default 1)      1: GEMM inputs as hi + lo bf16 planes; 0: hi plane only
 *                                              (bf16-rounded GEMM inputs: faster, less accurate)
 *   "attn_chunk"      (128 or 256, default 128) committed cache rows per round of an attention workgroup
 *   "attn_target_wgs" (1..65536, default 1024) workgroups the attention work list aims at (over all heads): the
 *                                              longer the sequences, the more rounds a workgroup walks
 *   "attn_mfma"       (0 or 1, default 1)      0: plain attention kernel instead of the MFMA one
 *   "gemm_fused"      (0 or 1, default 1)      1: bf16 launches of up to 64 rows run QKV + RoPE + KV write and
 *                                              gate/up + SwiGLU as one whole-K launch each (where the shapes
 *                                              allow: at most 6 slabs of 16 columns per compute unit); 0: split-K
 *                                              GEMM plus a separate RoPE / SwiGLU launch, as for larger launches */
int cerberus_set_param(cerberus_ctx *ctx, const char *name, int32_t value);

/* Benchmark hook: enqueues back to back, for every layer (or head stage), the GEMM launches of
 * one kind exactly as a step launches them for `rows` rows, reading whatever the activation
 * buffers hold; results land in scratch.  kind: 0 QKV, 1 attention output, 2 FFN gate/up,
 * 3 FFN down, 4 LM head, 5 head Resblocks (all stages), 6 head FC.  Where a step of `rows` rows runs the
 * QKV or gate/up projection as a whole-K fused launch, so does the hook (over the rows of the last
 * step's row map, which must have had that many; without the cache write).  Writes to *bytes (HOST, may
 * be NULL) the weight + activation bytes the launches read once each.  kind + 100 launches nothing
 * and writes 1.0 if a step of `rows` rows runs that kind as a whole-K fused launch, else 0.0.  */
int cerberus_bench_gemm(cerberus_ctx *ctx, int32_t kind, int32_t rows, void *stream, double *bytes);

/* Text of the last error raised on this thread (never NULL).                                   */
const char *cerberus_last_error(void);

void cerberus_destroy(cerberus_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* CERBERUS_H */
