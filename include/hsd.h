/*
 * hsd.h -- C ABI of the HSD verification hot path for AMD MI355X (gfx950).
 *
 * The library runs the target decoder's *verification pass* of Hierarchical Speculative Decoding:
 * one forward pass of the decoder over every sequence's block [pending token, d_1 .. d_k] on top of
 * the sequence's accepted context held in a paged KV cache (paper Section 3.2, Eq. 8), the model's own
 * top-1 token at every row (Eq. 10), greedy acceptance of the longest draft prefix that matches it
 * (Eq. 9 and Eq. 11; by default at tau -> 1, i.e. exact match, in the linear-draft case in which the
 * prefix tree is a chain and the tree-ancestry mask is the causal mask; hsd_batch.log_tau selects the
 * relaxed test and hsd_batch.tree_end a packed prefix tree per sequence), and the bonus token of Eq. 12.
 * Stage 1 (many short region drafts verified together, Eq. 2) and Stage 2 (one long page draft, Eq. 4)
 * are the same operator on different shapes, hence two entry points with one semantic definition.
 *
 * Conventions
 *  - "dev" pointers are device (HBM) pointers owned by the caller; the library never allocates or
 *    frees device memory and keeps no device state besides what the caller hands in.
 *  - Every call that takes a stream only enqueues work on it and returns; it never synchronises.
 *  - Return value: HSD_OK (0) or a negative hsd_status.  Argument errors are found on the host
 *    before anything is launched.  Conditions that only the device can see (KV pool exhausted,
 *    block table too short) set bits in hsd_batch.status and leave the affected sequence's outputs
 *    unspecified -- but never touch memory outside the caller's buffers.
 *  - Linear weights are row-major [out_features, in_features] (y = x W^T), in the model dtype
 *    (bf16 or fp32).  RMSNorm gains are always fp32.
 *  - All integer arrays are int32.
 */
#ifndef HSD_H_
#define HSD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum hsd_status {
  HSD_OK = 0,
  HSD_EINVAL = -1,  /* null pointer, non-positive size, unsupported dimension or dtype            */
  HSD_ENOSPC = -2,  /* workspace too small                                                       */
  HSD_ERANGE = -3,  /* a size exceeds a documented maximum                                       */
  HSD_EARCH = -4,   /* current device is not gfx950                                              */
  HSD_ENODEV = -5,  /* no usable HIP device                                                      */
  HSD_EHIP = -6     /* a HIP runtime call (launch, attribute query) failed                       */
} hsd_status;

enum { HSD_FP32 = 0, HSD_BF16 = 1 };

/* bits of hsd_batch.status (device-side conditions) */
enum {
  HSD_STATUS_POOL_EXHAUSTED = 1, /* not enough free KV blocks for the speculative append */
  HSD_STATUS_TABLE_OVERFLOW = 2, /* seq_len + q_len exceeds max_blocks_per_seq * 16       */
  HSD_STATUS_BAD_SLOT = 4,       /* a seq_slot entry lies outside [0, n_slots)           */
  HSD_STATUS_BAD_TREE = 8        /* a tree_end / tree_depth entry was not a valid packed tree */
};

enum { HSD_KV_BLOCK_TOKENS = 16, HSD_HEAD_DIM = 64, HSD_MAX_SEQ = 4096 };

/* Decoder dimensions (Llama family: pre-norm RMSNorm, rotate-half RoPE, GQA, SwiGLU, untied head).
 * Requirements: head_dim == 64, kv_block_tokens == 16, n_q_heads % n_kv_heads == 0,
 * d_model, d_ffn and vocab multiples of 128. */
typedef struct hsd_model_desc {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int32_t dtype; /* HSD_BF16 or HSD_FP32: storage type of weights, KV cache and GEMM operands */
  int32_t kv_block_tokens;
  float rms_eps, rope_theta;
  /* Attention key split (bf16 models; a deployment choice, not part of the architecture).  0: every query tile
   * walks all of its keys in one workgroup.  c > 0 (a multiple of 128): the keys of a sequence are cut at the
   * absolute positions c, 2c, ... (at most 8 chunks; the last is open ended), each chunk is scored by a workgroup
   * of its own and the chunks of a row are folded in ascending order.  Gives short, wide batches (region-level
   * drafts over ~1k cached tokens: c = 512) and single long drafts (c = 1024) the parallelism to fill the chip;
   * costs 264 bytes of workspace traffic per (row, head, chunk), so leave it 0 for many long sequences.  The cut
   * points depend on positions only: results stay independent of the batch; against c = 0 they differ in
   * rounding (the grouping of the fp32 sums).  When set, hsd_workspace_bytes grows by 8 * n_q_heads * 264 bytes
   * per row. */
  int32_t attn_key_chunk;
} hsd_model_desc;

/* Weights.  The per-layer members are HOST arrays of n_layers device pointers (copied by hsd_create). */
typedef struct hsd_weights {
  const void *tok_embed;         /* dev [vocab, d_model]                                   */
  const float *final_norm;       /* dev [d_model] fp32                                     */
  const void *lm_head;           /* dev [vocab, d_model]                                   */
  const float *const *attn_norm; /* [n_layers] -> dev [d_model] fp32                       */
  const void *const *wqkv;       /* -> dev [(n_q+2 n_kv) * 64, d_model]; rows q | k | v     */
  const void *const *wo;         /* -> dev [d_model, n_q * 64]                             */
  const float *const *ffn_norm;  /* -> dev [d_model] fp32                                  */
  const void *const *w_gate_up;  /* -> dev [2 * d_ffn, d_model]; rows gate | up             */
  const void *const *w_down;     /* -> dev [d_model, d_ffn]                                */
} hsd_weights;

/* Paged KV cache.  k_pool and v_pool: dev [n_layers][n_blocks][n_kv_heads][1024] in the model dtype.  A K page
 * is [16 tokens][64 dims]; a V page is stored transposed, [64 dims][16 token slots], token t in slot
 * 8*((t>>2)&1) + 4*(t>>3) + (t&3) (the order the attention kernel's matrix-core operands want).  The contents
 * are written and read only by the library.
 * free_list is a stack of free block ids, free_count its height; both live on the device and are
 * maintained by the library (hsd_kv_pool_init, verify, commit). */
typedef struct hsd_kv_pool {
  void *k_pool, *v_pool;
  int32_t n_blocks;
  int32_t *free_list;  /* dev [n_blocks] */
  int32_t *free_count; /* dev [1]        */
} hsd_kv_pool;

/* One verification round over a packed, ragged batch of sequences (regions or pages).
 * Sequence s owns rows cu_q[s] .. cu_q[s+1]-1 of the packed arrays; its block is
 * [pending token, d_1 .. d_k], q_len = k+1 >= 1, at absolute positions L .. L+k with L = seq_len[slot(s)].
 * The per-sequence state (seq_len, block_table) persists across rounds in rows addressed by seq_slot, so a
 * round may verify any subset of the live sequences; the per-round outputs are indexed by s. */
typedef struct hsd_batch {
  int32_t n_seq;              /* 1 .. HSD_MAX_SEQ                                                     */
  int32_t total_q;            /* cu_q[n_seq]; number of packed rows                                   */
  int32_t max_blocks_per_seq; /* row length of block_table                                            */
  int32_t n_slots;            /* rows of the persistent per-sequence state (seq_len, block_table)     */
  const int32_t *cu_q;        /* dev [n_seq+1], increasing, cu_q[0] = 0                               */
  const int32_t *seq_slot;    /* dev [n_seq]: state row used by batch sequence s (distinct entries),  */
                              /*   or NULL for the identity (then n_slots >= n_seq)                   */
  const int32_t *tokens;      /* dev [total_q]; a negative id means: take row r of `embeds` instead   */
  const float *embeds;        /* dev [total_q, d_model] fp32 input rows, or NULL if no id is negative */
  int32_t *seq_len;           /* dev [n_slots] committed KV length; read by verify, updated by commit */
  int32_t *block_table;       /* dev [n_slots][max_blocks_per_seq]; -1 = entry owns no block          */
  int32_t *argmax;            /* dev out [total_q] model top-1 per row (lowest id among equal maxima); */
                              /*   NULL => skip LM head and acceptance (prefill)                      */
  float *top2_margin;         /* dev out [total_q] top-1 minus top-2 logit, or NULL                   */
  int32_t *accept_len;        /* dev out [n_seq] alpha in [0, k]; input of commit                     */
  int32_t *bonus;             /* dev out [n_seq] argmax[cu_q[s] + alpha]; input of commit             */
  int32_t *status;            /* dev [1] in/out: HSD_STATUS_* bits are OR-ed in; caller clears        */
  float *logits_dump;         /* dev out [n_dump, vocab] fp32 logits of selected rows (debug) or NULL */
  const int32_t *dump_rows;   /* dev [n_dump] packed row indices                                      */
  int32_t n_dump;
  /* Relaxed acceptance (paper Section 3.2, Eq. 11): the draft token d_{i+1} is accepted at row i iff          */
  /* log p(d_{i+1}) - log p(u_hat) >= log_tau, i.e. iff its logit is within -log_tau of the row's largest.      */
  /* log_tau = 0 (tau = 1) selects the exact-match rule (d_{i+1} == arg-max, lowest id among equal maxima).     */
  float log_tau;              /* <= 0, finite                                                         */
  float *draft_gap;           /* dev out [total_q] or NULL: logit of the row's OWN token under its parent row    */
                              /*   (the previous row of a chain) minus that row's max logit (<= 0; -inf on the  */
                              /*   first row of a sequence); required if log_tau < 0                            */
  /* Prefix-tree batching (paper Section 3.2, Eq. 7 and the tree-ancestry mask).  NULL tree_end = every block    */
  /* is a chain.  Otherwise each sequence's block is a prefix tree packed in depth-first pre-order: local row 0   */
  /* is the root (it carries the pending token), and the subtree of local row i is local rows                    */
  /* i .. tree_end[cu_q[s]+i]-1.  A row sits at position seq_len + tree_depth (its place on its own root-to-node */
  /* path), sees the accepted context plus its ancestors and itself, and its K/V go to cache slot seq_len + i.   */
  /* Acceptance walks the tree from the root (Eq. 9-12); commit moves the accepted path's K/V to the contiguous  */
  /* slots seq_len+1 .. seq_len+alpha and rolls the rest back.  Malformed entries are clamped to a valid tree    */
  /* and reported as HSD_STATUS_BAD_TREE.                                                                        */
  const int32_t *tree_end;    /* dev [total_q] or NULL                                                */
  const int32_t *tree_depth;  /* dev [total_q]; required with tree_end; root = 0, child = parent + 1  */
  int32_t *stop_row;          /* dev out [n_seq]: local row of the stop node; required with tree_end  */
                              /*   when argmax is given; input of commit                              */
} hsd_batch;

typedef struct hsd_ctx hsd_ctx; /* opaque; host memory only (descriptor + copied pointer tables) */

const char *hsd_status_string(int status);

/* Pure host check of a descriptor / batch / pool / workspace size; what the verify calls run first.
 * Never dereferences a device pointer.  `pool` may be NULL to check the batch alone. */
int hsd_validate_model(const hsd_model_desc *desc);
int hsd_validate_batch(const hsd_model_desc *desc, const hsd_kv_pool *pool, const hsd_batch *batch,
                       size_t ws_bytes);

/* Creates a context for the current HIP device (must be gfx950).  Copies desc and the pointer tables;
 * the weight buffers themselves stay owned by the caller and must outlive the context. */
int hsd_create(const hsd_model_desc *desc, const hsd_weights *weights, hsd_ctx **out);
void hsd_destroy(hsd_ctx *ctx);

/* Device workspace needed by a verify/prefill call with total_q <= max_total_q, n_seq <= max_n_seq
 * (from the descriptor alone, so it can be called before hsd_create). */
size_t hsd_workspace_bytes(const hsd_model_desc *desc, int32_t max_total_q, int32_t max_n_seq);

/* Marks every block free (free_list = all ids, free_count = n_blocks). */
int hsd_kv_pool_init(void *stream, const hsd_kv_pool *pool);

/* Region-level verification (paper Section 3.1 Stage 1, Eq. 2): many short ragged draft blocks.
 * For every sequence: takes KV blocks from the pool for positions seq_len .. seq_len+q_len-1
 * (writing their ids into block_table), appends the keys/values of ALL q_len rows there
 * (speculatively), computes argmax for every row, then alpha = number of leading draft tokens with
 * tokens[base+i] == argmax[base+i-1], and bonus = argmax[base+alpha] (Eq. 9-12, exact match).
 * With batch.log_tau < 0 a draft token is accepted iff its logit is within -log_tau of its parent row's
 * largest (Eq. 11); with batch.tree_end the block is a packed prefix tree, rows see their ancestors only,
 * and the walk descends from the root through the admissible child (see hsd_batch).
 * seq_len is not modified: call hsd_kv_commit_rollback afterwards. */
int hsd_verify_region_batch(hsd_ctx *ctx, void *stream, const hsd_kv_pool *pool, const hsd_batch *batch,
                            void *workspace, size_t ws_bytes);

/* hsd_verify_region_batch for callers that cannot allocate or hand over a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs, kernels and bits as
 * hsd_verify_region_batch; the workspace is a fixed device array inside the library (hsd_noalloc_scratch_bytes(),
 * 16 MiB, held by every GPU the library runs on until the process ends).  Calls no allocating routine.
 * Returns HSD_ERANGE when hsd_workspace_bytes(desc, batch->total_q, batch->n_seq) exceeds that size (for the
 * 24-layer d1024 model: up to about 670 rows per call).  All calls on one GPU share the array (whatever context they
 * use): calls that overlap in time on one GPU race; calls on one stream, or ordered by events, are safe.  Nothing in
 * the array needs to start at zero and nothing is kept between calls. */
int hsd_verify_region_batch_noalloc(hsd_ctx *ctx, void *stream, const hsd_kv_pool *pool, const hsd_batch *batch);
size_t hsd_noalloc_scratch_bytes(void);

/* Page-level verification (Section 3.1 Stage 2, Eq. 4): few long draft blocks.  Same semantics and
 * outputs as hsd_verify_region_batch, and the same bits for every row (a row's arithmetic does not depend on the
 * entry point).  The attention workgroups are twice as large here (64 query rows of four query heads share each
 * 128-key K/V stage in LDS instead of 32), which halves the K/V traffic per query of a long block; batches of
 * many short blocks are better served by the smaller workgroups of hsd_verify_region_batch. */
int hsd_verify_page(hsd_ctx *ctx, void *stream, const hsd_kv_pool *pool, const hsd_batch *batch,
                    void *workspace, size_t ws_bytes);

/* KV maintenance after a verify: the cache upkeep and the rollback of rejected rows that Section 4.2 counts
 * into the decoding time.  For each sequence with accept_len[s] = alpha >= 0:
 * seq_len += 1 + alpha (the pending token and the accepted draft tokens become committed context);
 * pending_out[s] = bonus[s].  With alpha < 0: pure rollback, seq_len and pending_out[s] unchanged.
 * In both cases blocks lying wholly beyond the new length go back to the pool and their
 * block_table slots become -1; rejected rows inside the last kept block are simply overwritten by
 * the next round.  For a packed prefix tree (batch.tree_end) the accepted path's keys/values are first
 * moved from their pre-order slots to the contiguous slots seq_len+1 .. seq_len+alpha (needs
 * batch.stop_row as written by the verify call).  pending_out: dev [n_seq] or NULL. */
int hsd_kv_commit_rollback(hsd_ctx *ctx, void *stream, const hsd_kv_pool *pool, const hsd_batch *batch,
                           int32_t *pending_out);

/* Set-up helper (not part of the timed loop): forward pass without LM head over the given rows
 * (batch.argmax and the acceptance outputs are ignored), then commits every row:
 * seq_len += q_len.  Used to build the visual/prompt prefix. */
int hsd_prefill(hsd_ctx *ctx, void *stream, const hsd_kv_pool *pool, const hsd_batch *batch,
                void *workspace, size_t ws_bytes);

/* Measurement aid (for callers that report a per-kernel roofline; not a step of the method).
 * After hsd_profile_enable(ctx, which, max_launches) every launch of the kernel class `which` made by a
 * verify call is bracketed by a pair of HIP events recorded on the caller's stream (at most max_launches
 * pairs; later launches are not timed).  hsd_profile_read waits for the recorded events, returns the number
 * of timed launches and the sum of their durations in milliseconds, and clears the record.
 * hsd_profile_enable(ctx, HSD_PROF_NONE, 0) switches timing off and releases the events. */
enum {
  HSD_PROF_NONE = 0,
  HSD_PROF_GEMM_QKV = 1,
  HSD_PROF_ATTENTION = 2,
  HSD_PROF_GEMM_O = 3,
  HSD_PROF_GEMM_GATE_UP = 4,
  HSD_PROF_GEMM_DOWN = 5,
  HSD_PROF_GEMM_LM_HEAD = 6,
  HSD_PROF_RMSNORM = 7
};
int hsd_profile_enable(hsd_ctx *ctx, int which, int32_t max_launches);
int hsd_profile_read(hsd_ctx *ctx, int32_t *n_launches, float *total_ms);

/* Debug and experiment controls (not a step of the method; production callers never need them).  They change how
 * the work is launched, never what a row's result is, except HSD_DEBUG_FORCE_SIMPLE (other kernels, other rounding).
 *   HSD_DEBUG_SYNC_LAYERS   value != 0: the verify/prefill calls WAIT for the stream after every layer (an
 *                           exception to "never synchronises"; bounds the launches in flight for counter tools)
 *   HSD_DEBUG_FORCE_SIMPLE  value != 0: bf16 models run the plain fp32-FMA kernels (cross-check of the MFMA path)
 *   HSD_DEBUG_GEMM_CFG_*    tile configuration (0..13) of one GEMM call site, used for every row count
 * Returns HSD_EINVAL for an unknown knob or a value out of range. */
enum {
  HSD_DEBUG_SYNC_LAYERS = 1,
  HSD_DEBUG_FORCE_SIMPLE = 2,
  HSD_DEBUG_GEMM_CFG_QKV = 6,
  HSD_DEBUG_GEMM_CFG_O = 7,
  HSD_DEBUG_GEMM_CFG_GATE_UP = 8,
  HSD_DEBUG_GEMM_CFG_DOWN = 9,
  HSD_DEBUG_GEMM_CFG_LM_HEAD = 10
};
int hsd_debug_set(hsd_ctx *ctx, int knob, int64_t value);

/* Hardware probes (measurement helpers, not a step of the method): launch one of four small kernels that exercise a
 * single resource of the chip, so that a caller can time it and state what the chip sustains -- the yardsticks the
 * GEMM and attention rooflines are read against.  The call only enqueues on `stream` (device pointer/handle as for
 * the verify calls) and never waits; the caller brackets it with events.
 *   HSD_PROBE_MFMA      `n_workgroups` x 4 waves issue 16 bf16 32x32x16 MFMAs per wave and iteration, no memory
 *                       traffic: 16 * 32768 flop per wave and iteration
 *   HSD_PROBE_LOAD_REG  `n_workgroups` x 256 threads stream an L2-resident region with 16-byte loads into registers:
 *                       32768 bytes per workgroup and iteration
 *   HSD_PROBE_LOAD_LDS  the same with loads that write LDS directly
 *   HSD_PROBE_LDS_READ  `n_workgroups` x `arg` waves (1..16) read LDS with conflict-free 128-bit reads: 8192 bytes
 *                       per wave and iteration
 * `scratch` (device, `scratch_bytes`): at least 4 bytes; the two load probes read it as eight regions of
 * scratch_bytes / 8 bytes (one per XCD), each a multiple of 32 KiB, at least 32 KiB and below 2 GiB; contents are
 * irrelevant and unchanged except for its first 4 bytes, which a probe may overwrite.
 * Returns HSD_EINVAL for an unknown kind, n_workgroups or iters < 1, or a scratch buffer that does not fit the kind. */
enum { HSD_PROBE_MFMA = 0, HSD_PROBE_LOAD_REG = 1, HSD_PROBE_LOAD_LDS = 2, HSD_PROBE_LDS_READ = 3 };
int hsd_probe_launch(void *stream, int kind, int n_workgroups, int iters, int arg, void *scratch, size_t scratch_bytes);

#ifdef __cplusplus
}
#endif
#endif /* HSD_H_ */
