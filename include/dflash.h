/*
 * dflash.h -- C ABI of the DFlash speculative-decoding step for one MI355X (gfx950).
 *
 * One step of the method (arxiv 2602.06036, Section 3.1 and Section 4.1) is four calls, always in
 * this order, all enqueued on the caller's HIP stream without host synchronisation:
 *
 *     dflash_draft_block -> dflash_verify -> dflash_accept -> dflash_kv_commit
 *
 * Conventions
 *   - Every pointer is marked (host) or (device).  Device memory is owned by the caller (weights,
 *     packed blobs, KV pools, workspace, inputs, outputs) and must stay valid until the enqueued
 *     work has finished.  The library allocates no device memory.
 *   - Return value: DFLASH_OK or a negative DFLASH_E* code.  Errors that the host can see
 *     (null pointers, sizes, unsupported shapes) are reported before anything is enqueued;
 *     dflash_last_error() then gives a message.  Conditions only the device can see (a sequence
 *     that outgrew its pages or the host's max_seq_len hint, a page id outside the pool) raise a sticky
 *     device flag that dflash_device_status() reads; the offending rows are skipped or incomplete, never
 *     accessed out of bounds.
 *   - Linear maps are given as [out_features, in_features] row-major (y = W x, the paper's
 *     notation), in the model's dtype; norm gains are fp32.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Block layout (Section 4.2): slot 0 of every block is the clean anchor token (the previous
 *     step's bonus token) at position seq_lens[s]; slots 1..B-1 are the drafted tokens.
 */
#ifndef DFLASH_H
#define DFLASH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DFLASH_PAGE_SIZE 16      /* tokens per KV page (fixed: one page is one 16-wide MFMA tile) */
#define DFLASH_MAX_BLOCK 16      /* largest block size B */
#define DFLASH_MAX_TAPS 8

enum { DFLASH_F32 = 0, DFLASH_BF16 = 1 };
enum {
  DFLASH_OK = 0,
  DFLASH_EINVAL = -1,      /* bad argument or unsupported shape */
  DFLASH_ECAPACITY = -2,   /* sequence length + block exceeds the pages of the block table */
  DFLASH_EWORKSPACE = -3,  /* workspace / pool / blob buffer too small */
  DFLASH_EHIP = -4         /* a HIP call failed */
};
enum { DFLASH_POOL_TARGET = 0, DFLASH_POOL_DRAFT = 1 };

/* Shape of one model (target decoder or draft model); Section 5 "Implementation". */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rope_theta, rms_eps;
  int32_t qk_norm; /* 1: per-head RMSNorm on q and k before RoPE */
  int32_t dtype;   /* DFLASH_F32 | DFLASH_BF16: storage type of weights, activations fed to GEMMs, KV */
  /* Routed-expert FFN (the mixture-of-experts target of Section 5, Qwen3-Coder-30B-A3B; the paper names the model and
   * leaves the rule to it): n_experts > 0 replaces every layer's dense FFN by n_experts SwiGLU experts of width
   * d_expert; a token goes to the top_k experts by router logit (ties -> lowest index), weighted by the softmax over
   * the chosen logits.  d_ffn is then unused.  Target only, bf16 only; n_experts a multiple of 16 up to 256,
   * top_k <= 16, d_expert a multiple of 64, d_model a multiple of 128, and n_experts * ceil(max_seqs * block_size / 32)
   * <= 8192 (checked by dflash_workspace_bytes / dflash_create).  All three 0 = dense model. */
  int32_t n_experts, top_k, d_expert;
} dflash_dims;

/* One Transformer layer's weights (device), canonical layout. */
typedef struct {
  const void *wq, *wk, *wv, *wo; /* [Hq*hd, D], [Hkv*hd, D], [Hkv*hd, D], [D, Hq*hd] */
  const void *wg, *wu, *wd;      /* [F, D], [F, D], [D, F]; routed experts: stacked [E, Fe, D], [E, Fe, D], [E, D, Fe] */
  const float *g1, *g2;          /* [D] pre-attention / pre-FFN RMSNorm gains */
  const float *qn, *kn;          /* [hd] per-head q / k norm gains (ignored unless qk_norm) */
  const void *wr;                /* [E, D] router (ignored unless n_experts) */
} dflash_layer_weights;

/* Runtime geometry and caller-owned buffers. */
typedef struct {
  int32_t block_size;        /* B, 2..DFLASH_MAX_BLOCK; B * (n_q_heads / n_kv_heads) <= 64 for both models, or, for bf16 models
                                with head_dim 64 or 128, a larger value whose repeated halving stays whole down to 64
                                (8 query heads per kv head at B = 16: two attention workgroups per kv head) */
  int32_t max_seqs;          /* largest n_seqs of any call */
  int32_t max_pages_per_seq; /* row length of the block table */
  int32_t n_pages;           /* pages in each pool; page ids are 0..n_pages-1 in both pools */
  int32_t n_taps;            /* tapped target layers (Section 5: 5) */
  int32_t tap_layers[DFLASH_MAX_TAPS]; /* 0-based, ascending; the layer's output is tapped */
  int32_t mask_token_id;     /* id whose embedding fills the masked slots */
  void *target_kv_pool;      /* (device) dflash_kv_pool_bytes(target, n_pages) bytes */
  void *draft_kv_pool;       /* (device) dflash_kv_pool_bytes(draft, n_pages) bytes */
  void *workspace;           /* (device) dflash_workspace_bytes() bytes, 256-byte aligned */
  size_t workspace_bytes;
} dflash_runtime;

/* Per-call batch description. */
typedef struct {
  int32_t n_seqs;             /* S in [0, max_seqs]; with S = 0 the four step calls return DFLASH_OK and enqueue nothing
                                 (the pointers below are then not looked at) */
  int32_t max_seq_len;        /* (host) upper bound on seq_lens[s] over the batch; sizes launch grids only.  A sequence that is
                                 longer than this on the device may have its last cached rows left out of attention: the call
                                 then raises the sticky device status (dflash_device_status returns DFLASH_ECAPACITY) */
  int32_t *seq_lens;          /* (device) [S] committed length n_s; updated by dflash_kv_commit */
  const int32_t *block_table; /* (device) [S, max_pages_per_seq] page ids; pages covering n_s + B tokens must be valid */
  int32_t *anchor;            /* (device) [S] clean token at position n_s; updated by dflash_kv_commit */
  int32_t block_size;         /* rows per sequence of this call: 0 = the context's block_size, else 2..that value.  Section 5.5
                                 discusses smaller blocks where verification is compute-bound (large batches): a caller may
                                 choose the block per step.  The four calls of one step must use the same value; every [S,B]
                                 array of a call has this many columns. */
} dflash_batch;

typedef struct dflash_ctx dflash_ctx;

/* ---- sizes ------------------------------------------------------------------------------- */
size_t dflash_target_blob_bytes(const dflash_dims *target);
size_t dflash_draft_blob_bytes(const dflash_dims *draft, int32_t n_taps, int32_t d_target);
size_t dflash_kv_pool_bytes(const dflash_dims *model, int32_t n_pages);
size_t dflash_workspace_bytes(const dflash_dims *target, const dflash_dims *draft, const dflash_runtime *rt);

/* ---- one-time weight packing (device -> device, enqueued on stream) ---------------------------
 * Rewrites canonical weights into the library's streaming layout inside a caller-owned blob:
 * Q/K/V rows concatenated, gate/up rows interleaved in groups of 16 so SwiGLU fuses into the GEMM
 * epilogue, and for bf16 every matrix cut into 16x32 tiles stored in MFMA operand order.  The
 * canonical copies may be freed once the stream has finished.  Shared embedding and LM head
 * (Section 4.2) live in the target blob and are used by the draft as well. */
int dflash_pack_target_head(const dflash_dims *target, const void *embed /*(device) [V,D]*/,
                            const void *lm_head /*(device) [V,D]*/, const float *final_gain /*(device) [D]*/,
                            void *blob, void *stream);
int dflash_pack_target_layer(const dflash_dims *target, int32_t layer, const dflash_layer_weights *w /*(host struct)*/,
                             void *blob, void *stream);
/* W_c is [D, n_taps*D_target] (Appendix A.3), g_c its RMSNorm gain, final_gain the draft's final norm. */
int dflash_pack_draft_head(const dflash_dims *draft, int32_t n_taps, int32_t d_target, const void *w_c,
                           const float *g_c, const float *final_gain, void *blob, void *stream);
int dflash_pack_draft_layer(const dflash_dims *draft, int32_t n_taps, int32_t d_target, int32_t layer,
                            const dflash_layer_weights *w, void *blob, void *stream);

/* ---- context ----------------------------------------------------------------------------- */
/* Validates shapes and buffer sizes and records pointers; touches no device memory except
 * clearing the device status word (one synchronous 4-byte copy). */
int dflash_create(const dflash_dims *target, const void *target_blob, const dflash_dims *draft,
                  const void *draft_blob, const dflash_runtime *rt, dflash_ctx **out);
int dflash_destroy(dflash_ctx *ctx);
const char *dflash_last_error(const dflash_ctx *ctx); /* ctx may be NULL: message of the last failed create/pack/size call */
/* Synchronises `stream`, returns and clears the sticky device status (0, or DFLASH_ECAPACITY). */
int dflash_device_status(dflash_ctx *ctx, void *stream);

/* ---- the step ------------------------------------------------------------------------------ */
/* Draft (Section 4.1 "Parallel diffusion drafting", Appendix A.3): one forward pass of the draft
 * model over the block [anchor, mask x (B-1)] at positions n_s .. n_s+B-1.  Block rows attend without
 * mask to the n_s cached context-feature K/V rows of each draft layer and to all B block rows.
 * temperature == 0: draft_tokens[s,j] = argmax of slot j's logits (ties -> lowest id);
 * temperature  > 0: a draw from softmax(logits/temperature) by Gumbel-max with the counter-based
 * generator keyed by *rng_key.  draft_tokens (device) [S,B] out, slot 0 = anchor.
 * logits_out (device, nullable) [S,B,V] fp32 receives the draft logits (row j = slot j).
 * The token choice is fused into the LM-head GEMM (per-workgroup row maxima, combined by a small
 * second kernel); the [S,B,V] logits are materialised only if logits_out is given or temperature > 0
 * (dflash_accept then needs the proposal distribution). */
int dflash_draft_block(dflash_ctx *ctx, const dflash_batch *batch, float temperature,
                       const uint64_t *rng_key /*(device) [1], nullable when temperature == 0*/,
                       int32_t *draft_tokens, float *logits_out, void *stream);

/* Verify (Section 3.1): one causal forward of the target over tokens[s,0..B-1] at positions
 * n_s .. n_s+B-1 against the paged KV cache; row j sees cache rows 0..n_s-1 and block rows <= j.
 * Writes the B new K/V rows of every layer into the target pool (speculatively: they become
 * visible only when dflash_kv_commit advances seq_lens) and the tapped hidden states into the
 * workspace.  tgt_argmax (device, nullable) [S,B]: greedy token after row j.  logits_out (device, nullable)
 * [S,B,V] fp32.  With both null the LM head is skipped: the call then only writes K/V rows and taps (a prefill
 * chunk that ends no prompt).  The logits are materialised only if logits_out is given or the last
 * dflash_draft_block call on this context sampled (temperature > 0), i.e. dflash_accept will need them. */
int dflash_verify(dflash_ctx *ctx, const dflash_batch *batch, const int32_t *tokens /*(device) [S,B]*/,
                  int32_t *tgt_argmax, float *logits_out, void *stream);

/* Accept (Section 3.1: tau = accept_len + 1 in [1, B], bonus token included).
 * temperature == 0: accept_len[s] = largest a with draft_tokens[s,j] == tgt_argmax[s,j-1] for all
 * 1 <= j <= a; out_tokens[s] = d_1..d_a, tgt_argmax[s,a], then -1 padding.
 * temperature  > 0: speculative sampling on the logits the preceding dflash_draft_block and
 * dflash_verify calls left in the workspace: slot j accepted iff u[s,j] * q_j(d_j) < p_{j-1}(d_j);
 * first rejected slot is replaced by a draw from normalise(max(p - q, 0)); all accepted -> bonus
 * draw from the last row.  uniforms (device) [S,B] fp32 in [0,1).  DFLASH_EINVAL if this step's
 * dflash_draft_block did not run with temperature > 0 (the workspace then holds no logits). */
int dflash_accept(dflash_ctx *ctx, const dflash_batch *batch, const int32_t *draft_tokens,
                  const int32_t *tgt_argmax, float temperature, const float *uniforms /*nullable when greedy*/,
                  const uint64_t *rng_key /*(device) [1], nullable when greedy*/,
                  int32_t *accept_len /*(device) [S] out*/, int32_t *out_tokens /*(device) [S,B] out*/, void *stream);

/* For callers that cannot allocate device memory or hand over a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the temperature > 0 branch of dflash_accept on logits the caller holds itself
 * (e.g. the logits_out of dflash_draft_block and dflash_verify), with the rows' softmax statistics kept in an array that
 * is built into the library (64 KB of device memory per GPU, held until the process ends) instead of a workspace.
 * target_logits, draft_logits (device) [S,B,V] fp32; draft_tokens (device) [S,B]; uniforms (device) [S,B]; rng_key
 * (device) [1]; outputs as dflash_accept.  Needs no context, allocates nothing, calls no allocating routine.
 * At most 4096 rows (n_seqs * block_size): DFLASH_ECAPACITY beyond that; DFLASH_EINVAL for temperature <= 0 (greedy
 * acceptance needs no scratch at all: use dflash_accept).  All calls on one GPU share the one array: calls that overlap
 * on the same GPU (different streams, different threads) race on it and must be serialised by the caller.  Nothing in
 * the array has to start at zero: every call overwrites the entries it reads. */
int dflash_accept_sampled_noalloc(const float *target_logits, const float *draft_logits, const int32_t *draft_tokens,
                                  const float *uniforms, const uint64_t *rng_key, float temperature, int32_t n_seqs,
                                  int32_t block_size, int32_t vocab, int32_t *accept_len, int32_t *out_tokens, void *stream);

/* Commit / rollback (Section 4.1, Appendix A.3): fuses the tapped hidden states of the block rows,
 * H_t = RMSNorm(W_c [taps]), projects them with every draft layer's W_K, W_V (k-norm, RoPE at the
 * row's position) into the draft pool at positions n_s .. n_s+B-1, then advances
 * seq_lens[s] += accept_len[s] + 1 and sets anchor[s] = out_tokens[s, accept_len[s]].
 * Rows beyond the accepted prefix stay in the pools but are invisible (rolled back) and are
 * overwritten by the next step.  accept_len[s] = -1 commits nothing for sequence s (length and anchor
 * unchanged): an idle slot of the batch, or a prompt that ended in an earlier prefill chunk.  kv_slots_out (device, nullable) [S,B] int64: page*16+offset of
 * each committed row, -1 for rolled-back rows.
 * The call belongs to the preceding dflash_verify on this context with the same batch (same rows, same seq_lens):
 * it reads that call's tapped hidden states and rotary angles from the workspace. */
int dflash_kv_commit(dflash_ctx *ctx, const dflash_batch *batch, const int32_t *accept_len,
                     const int32_t *out_tokens, int64_t *kv_slots_out, void *stream);

/* Prefill (Section 4.1: "Given a prompt, the target model first performs a standard prefill pass to generate the first
 * token"; the hidden features of the tapped layers are taken for every prompt token and become the draft's context).
 * prompt_lens (host) [S]: new tokens of each sequence (0 = none); tokens (device): those tokens of all sequences
 * concatenated in sequence order.  batch->seq_lens[s] tokens are already cached (0 for a fresh prompt; more for a prompt
 * that arrives in pieces or shares a cached prefix).  The new tokens run through the target causally, as passes of up to
 * max_seqs * B rows (every block of B tokens of every prompt is one row block of a verification-shaped pass): their K/V
 * rows go into the target pool, the tapped hidden states of ALL rows are fused and projected into the draft pool
 * (as dflash_kv_commit does for a block), the LM head runs on each prompt's last row only.  Afterwards
 * seq_lens[s] += prompt_lens[s] and, for every sequence with new tokens, anchor[s] = first_tokens[s] (device, nullable)
 * = the greedy token after its last prompt token -- the state the first dflash_draft_block call starts from.
 * The block table must cover seq_lens[s] + prompt_lens[s] rounded up to whole blocks (the padding rows of a prompt's last
 * block are written too, invisibly); DFLASH_ECAPACITY otherwise.  prompt_lens is read before the call returns. */
int dflash_prefill(dflash_ctx *ctx, const dflash_batch *batch, const int32_t *tokens, const int32_t *prompt_lens,
                   int32_t *first_tokens, void *stream);

/* ---- per-launch timing (benchmarks) -------------------------------------------------------------
 * While enabled, every GEMM and attention launch is bracketed by a pair of HIP events on the caller's
 * stream (this slows the step down: time whole steps with profiling off).  dflash_profile_read
 * synchronises the stream, sums elapsed milliseconds, launch counts and algorithmic bytes (GEMM: the
 * weight matrix once; attention: the K and V rows within the host's max_seq_len hint once) per class
 * into arrays of DFLASH_PROF_CLASSES entries (host) and forgets the recorded launches. */
#define DFLASH_PROF_CLASSES 8
enum {
  DFLASH_PROF_GEMM_STORE = 0,  /* QKV, W_c and context-K/V projections */
  DFLASH_PROF_GEMM_RESID = 1,  /* O and down projections (+ residual) */
  DFLASH_PROF_GEMM_SWIGLU = 2, /* gate/up projection (+ SwiGLU) */
  DFLASH_PROF_ATTN = 3,        /* split-KV block attention */
  DFLASH_PROF_ATTN_MERGE = 4,
  DFLASH_PROF_GEMM_LMHEAD = 5,
  DFLASH_PROF_MOE_GATEUP = 6,  /* routed experts: grouped gate/up (+ SwiGLU) launch; bytes = an upper bound, every expert */
  DFLASH_PROF_MOE_DOWN = 7     /*   that the rows can reach; grouped down projection */
};
int dflash_profile_enable(dflash_ctx *ctx, int32_t enable);
int dflash_profile_read(dflash_ctx *ctx, void *stream, float *ms, int32_t *count, double *bytes);

/* Routed-expert targets: totals since the last read (or create) of routing launches (one per target layer and
 * dflash_verify call), experts reached by at least one row, 16-row bands of the expert-sorted row list and work items
 * of the grouped launches, into out[0..3] (host); out[4] = the bands per work item (1, 2, 4, or 8 = grouped launches of the
 * LDS-staged GEMM) of the last routing launch.  experts / launches * bytes of one expert's matrices = what a layer's expert
 * GEMMs had to read.  Synchronises the stream and clears all five. */
int dflash_moe_stats(dflash_ctx *ctx, void *stream, int64_t *out);

/* State export for tests and tuning: GEMM launches per kernel family since the last call (or create) into
 * out[0..DFLASH_GEMM_KINDS-1] (host), cleared by the call.  Says which kernel a shape, a row count or a tuning
 * variable actually selected.  Host counters: no synchronisation, no device access. */
#define DFLASH_GEMM_KINDS 6
enum {
  DFLASH_GEMM_STREAMING = 0, /* weight-streaming kernel, up to 64 rows (K split across workgroups and wavefronts) */
  DFLASH_GEMM_TILED4 = 1,    /* LDS-staged tiles, four wavefronts */
  DFLASH_GEMM_TILED8 = 2,    /* LDS-staged tiles, eight wavefronts (384 or 256 weight rows) */
  DFLASH_GEMM_FEW_ROWS = 3,  /* unsplit projection with the residual update in its epilogue (one band of rows) */
  DFLASH_GEMM_GROUPED = 4,   /* routed experts: grouped launches */
  DFLASH_GEMM_F32 = 5        /* fp32 models */
};
int dflash_gemm_counts(dflash_ctx *ctx, int64_t *out);

/* Routed-expert targets, state export for tests and debugging: while `choices` (device, [n_layers, max_seqs * block_size,
 * top_k] int32, caller-owned) is set, every routed target layer leaves the experts it chose for row m (by decreasing
 * router logit) at choices[(layer * max_seqs * block_size + m) * top_k ..]; NULL switches the trace off again.  Rows
 * beyond the call's S * B rows are not written.  The routing itself is unchanged (the kernels keep their choices there
 * instead of in the workspace). */
int dflash_moe_trace(dflash_ctx *ctx, int32_t *choices);

/* ---- machine probes (benchmarks; not part of the method) -----------------------------------------
 * What one launch can reach on this GPU, to put the kernels' figures beside: neither needs a context.
 * dflash_probe_hbm_read: `launches` back-to-back kernels (256 workgroups of 256 threads, 8 non-temporal 1 KB
 * loads in flight per wavefront), launch i reading bytes_per_launch bytes at buf + i * bytes_per_launch
 * (device memory, at least launches * bytes_per_launch bytes, a multiple of 1024; use more than the 256 MB
 * memory-side cache in total so that every launch reads HBM).  *ms_total (host) = time of all launches.
 * dflash_probe_mfma: one kernel of `workgroups` x 4 wavefronts, each issuing iters rounds of independent bf16
 * MFMAs on register operands: shape 0 = 16 x v_mfma_f32_16x16x32_bf16 per round, shape 1 = 4 x
 * v_mfma_f32_32x32x16_bf16 per round.  *ms (host) = its time, *flops (host) = 2*m*n*k per MFMA.
 * Both synchronise the stream.  DFLASH_EINVAL on bad arguments, DFLASH_EHIP if the device reports an error. */
int dflash_probe_hbm_read(const void *buf, size_t bytes_per_launch, int32_t launches, float *ms_total, void *stream);
int dflash_probe_mfma(int32_t shape, int32_t workgroups, int32_t iters, float *ms, double *flops, void *stream);

/* ---- cache import / export (state migration, tests) ------------------------------------------ */
/* Copies rows [start, start+count) of sequence `seq` of one layer between the paged pool and
 * canonical fp32 buffers k, v (device) [count, Hkv, hd].  K rows are stored post-RoPE.
 * count = 0 is valid (nothing is copied; k and v may then be null). */
int dflash_kv_read(dflash_ctx *ctx, const dflash_batch *batch, int32_t pool, int32_t layer, int32_t seq,
                   int32_t start, int32_t count, float *k, float *v, void *stream);
int dflash_kv_write(dflash_ctx *ctx, const dflash_batch *batch, int32_t pool, int32_t layer, int32_t seq,
                    int32_t start, int32_t count, const float *k, const float *v, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DFLASH_H */
