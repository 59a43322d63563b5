// C ABI of the DFlash speculative-decoding step (see include/dflash.h) and the host-side
// orchestration that enqueues the gfx950 kernels.  No device memory is allocated here.
#include "../../include/dflash.h"

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <type_traits>
#include <vector>

#include "attn.h"
#include "attn_mfma.h"
#include "common.h"
#include "gemm.h"
#include "gemm_resid.h"
#include "gemm_tiled.h"
#include "misc.h"
#include "moe.h"

// Scratch of dflash_accept_sampled_noalloc (the entry point for callers that cannot allocate): the rows' softmax
// statistics, (max, log-sum-exp) of the target rows followed by those of the draft rows.  Every GPU the library runs
// on holds its own copy of this array until the process ends; host code reaches it through the address that
// hipGetSymbolAddress returns for the current device, never through this name.
#define DFLASH_NOALLOC_MAX_ROWS 4096
static __device__ __align__(256) unsigned char scratch[2 * DFLASH_NOALLOC_MAX_ROWS * sizeof(float2)];

namespace {

thread_local char g_err[512] = "";

int fail(char* dst, int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  if (dst) memcpy(dst, g_err, sizeof g_err);
  return code;
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
inline size_t esize(int dtype) { return dtype == DFLASH_BF16 ? 2 : 4; }
inline int round_rows(int dtype, int M) { return dtype == DFLASH_BF16 ? (M + 15) & ~15 : M; }

inline int env_int(const char* name, int dflt) {
  const char* e = getenv(name);
  const int v = e ? atoi(e) : 0;
  return v > 0 ? v : dflt;
}

// Tuning and testing knobs, read from the environment whenever a context is created (or a workspace is sized): a
// context keeps the values it was created with, so a test that sets one before dflash_create gets exactly that path
// whatever ran earlier in the process.  Defaults are what the measurements in the documentation use.
struct Knobs {
  int gemm_wide;            // DFLASH_GEMM_WIDE: 1 = eight-wavefront tiles where they fill one round of the CUs (default), 2 = wherever one fits (tests), any other value = never
  int attn_target_wgs;      // DFLASH_ATTN_TARGET_WGS: workgroups an attention launch aims at
  int attn_wide_min_chunk;  // DFLASH_ATTN_WIDE_MIN_CHUNK: keys per workgroup from which the key-split attention kernel is used
  int gemm_target_wgs;      // DFLASH_GEMM_TARGET_WGS: workgroups a K-split streaming GEMM aims at
  int gemm_u;               // DFLASH_GEMM_U: k tiles per prefetch stage (one band of rows)
  int gemm_nt8;             // DFLASH_GEMM_NT8: matrices with at least 8 * this row bands use 8 weight tiles per activation fragment
  int gemm_fill;            // DFLASH_GEMM_FILL: 1 = weight tiles per wavefront (8 or 6) and K split chosen to fill whole rounds of the CUs
  int gemm_fill4;           // DFLASH_GEMM_FILL4: the same for 17-64 rows
  int gemm_u4;              // DFLASH_GEMM_U4: k tiles per prefetch stage for 17-64 rows
  int gemm_solo_pct;        // DFLASH_GEMM_SOLO_PCT: tiled GEMM picker, time penalty (percent) of a ring tile alone on its CU
  int gemm_pd;              // DFLASH_GEMM_PD: tiled GEMM, k tiles in flight from global memory (192/128-row tiles)
  int gemm_ring;            // DFLASH_GEMM_RING: 1 = direct-to-LDS ring for the small tiles, other = register staging
  int gemm_tile, gemm_wm, gemm_ks;   // DFLASH_GEMM_TILE / _WM / _KS: force the tiled GEMM's shape / rows per tile / K split (0 = by estimated time)
  int lm_stats;             // DFLASH_LM_STATS: 1 = softmax statistics from the LM-head epilogue, other = from the stored logits
  int moe_mt;               // DFLASH_MOE_MT: 1, 2, 4 or 8 forces the bands per routed-expert work item (0 = by rows per expert)
  int moe_gather_min_rows;  // DFLASH_MOE_GATHER_MIN_ROWS: rows from which the routed-expert GEMMs get their rows copied into list order
  int moe_phases;           // DFLASH_MOE_PHASES: 2 = two-half sum form of the 4-band down projection
  int moe_down_u;           // DFLASH_MOE_DOWN_U: k tiles per stage of the one-band down projection
  int fuse;                 // DFLASH_FUSE: few-row path, see dflash_ctx::fuse
  int resid_nw, resid_u;    // DFLASH_RESID_NW / _U: wavefronts per workgroup and k tiles per stage of the unsplit projection kernel
};
Knobs read_knobs() {
  Knobs k;
  k.gemm_wide = env_int("DFLASH_GEMM_WIDE", 1);
  k.attn_target_wgs = env_int("DFLASH_ATTN_TARGET_WGS", 256);
  k.attn_wide_min_chunk = env_int("DFLASH_ATTN_WIDE_MIN_CHUNK", 512);
  k.gemm_target_wgs = env_int("DFLASH_GEMM_TARGET_WGS", 256);
  k.gemm_u = env_int("DFLASH_GEMM_U", 2);
  k.gemm_nt8 = env_int("DFLASH_GEMM_NT8", 1);
  k.gemm_fill = env_int("DFLASH_GEMM_FILL", 1);
  k.gemm_fill4 = env_int("DFLASH_GEMM_FILL4", 1);
  k.gemm_u4 = env_int("DFLASH_GEMM_U4", 1);
  k.gemm_solo_pct = env_int("DFLASH_GEMM_SOLO_PCT", 120);
  k.gemm_pd = env_int("DFLASH_GEMM_PD", 2);
  k.gemm_ring = env_int("DFLASH_GEMM_RING", 1);
  k.gemm_tile = env_int("DFLASH_GEMM_TILE", 0);
  k.gemm_wm = env_int("DFLASH_GEMM_WM", 0);
  k.gemm_ks = env_int("DFLASH_GEMM_KS", 0);
  k.lm_stats = env_int("DFLASH_LM_STATS", 1);
  k.moe_mt = env_int("DFLASH_MOE_MT", 0);
  k.moe_gather_min_rows = env_int("DFLASH_MOE_GATHER_MIN_ROWS", 64);
  k.moe_phases = env_int("DFLASH_MOE_PHASES", 2);
  k.moe_down_u = env_int("DFLASH_MOE_DOWN_U", 1);
  k.fuse = env_int("DFLASH_FUSE", 1);
  if (k.fuse != 1 && k.fuse != 2) k.fuse = 0;
  k.resid_nw = env_int("DFLASH_RESID_NW", 4);
  k.resid_u = env_int("DFLASH_RESID_U", 8);
  return k;
}

struct LayerOff {
  size_t wqkv, wo, wgu, wd, wr, g1, g2, qn, kn, end;
};

// routed-expert layers: rows of the expert-sorted token list (every used expert's share padded to whole 16-row bands)
// and work items of the grouped GEMMs, both as upper bounds for M token rows
inline int moe_positions(const dflash_dims& d, int M) {
  const int mk = M * d.top_k, used = std::min(d.n_experts, mk);
  return (mk + 15 * used + 15) & ~15;
}
inline int moe_items(const dflash_dims& d, int M, int MT) { return std::min(d.n_experts, M * d.top_k) + moe_positions(d, M) / 16 / MT + 1; }

LayerOff layer_layout(const dflash_dims& d) {
  const size_t es = esize(d.dtype);
  const size_t qd = (size_t)d.n_q_heads * d.head_dim, kd = (size_t)d.n_kv_heads * d.head_dim;
  LayerOff o;
  size_t off = 0;
  o.wqkv = off; off += align256((qd + 2 * kd) * d.d_model * es);
  o.wo = off;   off += align256((size_t)d.d_model * qd * es);
  // routed experts: the experts' packed gate/up and down matrices one after the other, and the router
  const size_t ffn = d.n_experts ? (size_t)d.n_experts * d.d_expert : (size_t)d.d_ffn;
  o.wgu = off;  off += align256(2 * ffn * d.d_model * es);
  o.wd = off;   off += align256((size_t)d.d_model * ffn * es);
  o.wr = off;   off += align256((size_t)d.n_experts * d.d_model * es);
  o.g1 = off;   off += align256((size_t)d.d_model * 4);
  o.g2 = off;   off += align256((size_t)d.d_model * 4);
  o.qn = off;   off += align256((size_t)d.head_dim * 4);
  o.kn = off;   off += align256((size_t)d.head_dim * 4);
  o.end = off;
  return o;
}

struct TargetLayout {
  size_t embed, lm, gf, layer0, total;
  LayerOff lo;
};
TargetLayout target_layout(const dflash_dims& d) {
  const size_t es = esize(d.dtype);
  TargetLayout t;
  size_t off = 0;
  t.embed = off; off += align256((size_t)d.vocab * d.d_model * es);
  t.lm = off;    off += align256((size_t)d.vocab * d.d_model * es);
  t.gf = off;    off += align256((size_t)d.d_model * 4);
  t.layer0 = off;
  t.lo = layer_layout(d);
  t.total = off + t.lo.end * d.n_layers;
  return t;
}

struct DraftLayout {
  size_t wc, gc, gf, wkv_all, layer0, total;
  LayerOff lo;
};
DraftLayout draft_layout(const dflash_dims& d, int n_taps, int d_target) {
  const size_t es = esize(d.dtype);
  const size_t kd = (size_t)d.n_kv_heads * d.head_dim;
  DraftLayout t;
  size_t off = 0;
  t.wc = off;      off += align256((size_t)d.d_model * n_taps * d_target * es);
  t.gc = off;      off += align256((size_t)d.d_model * 4);
  t.gf = off;      off += align256((size_t)d.d_model * 4);
  t.wkv_all = off; off += align256((size_t)d.n_layers * 2 * kd * d.d_model * es);
  t.layer0 = off;
  t.lo = layer_layout(d);
  t.total = off + t.lo.end * d.n_layers;
  return t;
}

int check_dims(const dflash_dims* d, const char* who) {
  if (!d) return fail(nullptr, DFLASH_EINVAL, "%s dims: null", who);
  if (d->dtype != DFLASH_F32 && d->dtype != DFLASH_BF16) return fail(nullptr, DFLASH_EINVAL, "%s: dtype must be DFLASH_F32 or DFLASH_BF16", who);
  const bool routed = d->n_experts != 0;   // d_ffn is unused (and unchecked) when every layer's FFN is routed experts
  if (d->n_layers < 1 || d->d_model < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || (!routed && d->d_ffn < 1) || d->vocab < 1)
    return fail(nullptr, DFLASH_EINVAL, "%s: non-positive dimension", who);
  if (d->n_q_heads % d->n_kv_heads) return fail(nullptr, DFLASH_EINVAL, "%s: n_q_heads must be a multiple of n_kv_heads", who);
  if (d->head_dim > 128 || d->head_dim < 16 || d->head_dim % 16) return fail(nullptr, DFLASH_EINVAL, "%s: head_dim must be a multiple of 16 in [16,128]", who);
  const int qd = d->n_q_heads * d->head_dim;
  if (d->dtype == DFLASH_BF16) {
    if (d->d_model % 32 || (!routed && d->d_ffn % 32) || qd % 32 || d->vocab % 16)
      return fail(nullptr, DFLASH_EINVAL, "%s: bf16 needs d_model, d_ffn, Hq*hd multiples of 32 and vocab a multiple of 16", who);
  } else {
    if (d->d_model % 8 || (!routed && d->d_ffn % 16) || qd % 8) return fail(nullptr, DFLASH_EINVAL, "%s: fp32 needs d_model, Hq*hd multiples of 8 and d_ffn a multiple of 16", who);
  }
  if (!(d->rope_theta > 1.f) || !(d->rms_eps >= 0.f)) return fail(nullptr, DFLASH_EINVAL, "%s: bad rope_theta / rms_eps", who);
  if (d->n_experts) {
    if (d->dtype != DFLASH_BF16) return fail(nullptr, DFLASH_EINVAL, "%s: routed experts need the bf16 dtype", who);
    if (d->n_experts < 0 || d->n_experts > MOE_MAX_EXPERTS || d->n_experts % 16)
      return fail(nullptr, DFLASH_EINVAL, "%s: n_experts must be a multiple of 16 in [16,%d]", who, MOE_MAX_EXPERTS);
    if (d->top_k < 1 || d->top_k > MOE_MAX_TOPK || d->top_k > d->n_experts) return fail(nullptr, DFLASH_EINVAL, "%s: top_k must be in [1,min(%d,n_experts)]", who, MOE_MAX_TOPK);
    if (d->d_expert < 64 || d->d_expert % 64 || d->d_model % 128) return fail(nullptr, DFLASH_EINVAL, "%s: routed experts need d_expert a multiple of 64 and d_model a multiple of 128", who);
  } else if (d->top_k || d->d_expert) {
    return fail(nullptr, DFLASH_EINVAL, "%s: top_k / d_expert set without n_experts", who);
  }
  return DFLASH_OK;
}

// ---- attention split policy -----------------------------------------------------------------------
// log2 of the workgroups that share one kv head's query heads in the MFMA attention kernels (64 query rows each at
// most); -1: this shape does not fit them
inline int attn_q_shift(const dflash_dims& m, int block_size) {
  const int group = m.n_q_heads / m.n_kv_heads;
  int sh = 0;
  while (((block_size * group) >> sh) > 64) ++sh;
  if (sh == 0) return 0;
  return (m.dtype == DFLASH_BF16 && (m.head_dim == 128 || m.head_dim == 64) && group % (1 << sh) == 0) ? sh : -1;
}

struct SplitPlan {
  int n_splits, chunk;
  int bound;  // >= n_splits for this and every smaller max_tokens (sizes the partial buffers)
};
SplitPlan plan_splits(int S, int n_kv_heads, int max_tokens, int target_wgs) {
  // the attention kernel runs one workgroup per CU (its accumulators fill the register file), so aim at
  // one round of workgroups on the 256 CUs (target_wgs: Knobs::attn_target_wgs)
  const int max_splits = 64;
  int splits = (target_wgs + S * n_kv_heads - 1) / (S * n_kv_heads);
  const int by_len = (max_tokens + 63) / 64;
  splits = std::max(1, std::min(splits, std::min(by_len, max_splits)));
  int chunk = (max_tokens + splits - 1) / splits;
  chunk = (chunk + 63) & ~63;
  SplitPlan p;
  p.bound = splits;
  p.chunk = chunk;
  p.n_splits = (max_tokens + chunk - 1) / chunk;
  return p;
}

// ---- workspace ------------------------------------------------------------------------------------
// rows of partial results the split-K arena holds for a context of at most max_rows activation rows
inline int arena_rows(int max_rows) { return std::max(1024, 4 * max_rows); }

constexpr int ARGMAX_CHUNKS = 32;   // workgroups that share one vocabulary row in the argmax

struct Workspace {
  size_t status, arena, h, a, q, o, act, taps, fuse, ht, logits_d, logits_t, part_o, part_ml, stats_p, stats_q, amax, lsep, rope_t, rope_d, ssq, pf_lens, pf_plens, pf_table, pf_tokens, pf_end_row, pf_end_seq, pf_first, pf_anchor, total;
  size_t moe_sel_e, moe_sel_w, moe_sel_pos, moe_row_of, moe_items, moe_a, moe_act, moe_y;   // routed-expert target only
};
Workspace workspace_layout(const dflash_dims& t, const dflash_dims& d, const dflash_runtime& rt, const Knobs& kn) {
  const size_t es = esize(t.dtype);
  const int M = rt.max_seqs * rt.block_size;
  const size_t Mr = round_rows(t.dtype, M);
  const size_t planes = t.dtype == DFLASH_BF16 ? 2 : 1;   // bf16 GEMM inputs are hi+lo pairs
  const size_t qd = (size_t)std::max(t.n_q_heads * t.head_dim, d.n_q_heads * d.head_dim);
  const size_t nqkv = std::max((size_t)(t.n_q_heads + 2 * t.n_kv_heads) * t.head_dim, (size_t)(d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim);
  const size_t F = std::max(t.d_ffn, d.d_ffn);
  const size_t D = t.d_model;
  Workspace w;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t r = off; off += align256(bytes); return r; };
  w.status = take(256);
  w.h = take((size_t)M * D * 4);
  w.a = take(Mr * D * es * planes);
  w.q = take((size_t)M * qd * es);
  w.o = take(Mr * qd * es * planes);
  w.act = take(Mr * F * es * planes);
  w.taps = take(Mr * (size_t)rt.n_taps * D * es * planes);
  w.fuse = take((size_t)M * D * 4);
  w.ht = take(Mr * D * es * planes);
  // arena: K-range partial results of the QKV / O / down / W_c / context-K/V GEMMs (consumed by the next kernel)
  const size_t n_max = std::max(std::max(nqkv, D), (size_t)d.n_layers * 2 * d.n_kv_heads * d.head_dim);
  w.arena = take((size_t)arena_rows(M) * n_max * 4);
  w.logits_d = take((size_t)M * t.vocab * 4);
  w.logits_t = take((size_t)M * t.vocab * 4);
  // attention partials: worst case over batch sizes and both models
  size_t part_rows = 0;
  const int max_tokens = rt.max_pages_per_seq * DFLASH_PAGE_SIZE;
  for (int S = 1; S <= rt.max_seqs; ++S) {
    for (const dflash_dims* m : {&t, &d}) {
      for (int blk = 2; blk <= rt.block_size; ++blk) {   // a call may use a smaller block than the context's (dflash_batch::block_size)
        const int sh = attn_q_shift(*m, blk);
        if (sh < 0) continue;
        const SplitPlan p = plan_splits(S, m->n_kv_heads << sh, max_tokens, kn.attn_target_wgs);
        part_rows = std::max(part_rows, (size_t)S * blk * m->n_q_heads * p.bound);
      }
    }
  }
  const size_t hd = std::max(t.head_dim, d.head_dim);
  w.part_o = take(part_rows * hd * 4);
  w.part_ml = take(part_rows * 8);
  w.stats_p = take((size_t)M * 8);
  w.stats_q = take((size_t)M * 8);
  w.amax = take((size_t)M * std::max(ARGMAX_CHUNKS, t.vocab / 16 + 1) * 8);   // one partial per weight row band at most
  w.lsep = take((size_t)M * (t.vocab / 16 + 1) * 8);    // per-workgroup softmax statistics of an LM-head launch
  w.rope_t = take((size_t)M * (t.head_dim / 2) * 8);   // rotary tables of the call's rows (target, draft)
  w.rope_d = take((size_t)M * (d.head_dim / 2) * 8);
  w.ssq = take((size_t)M * (D / 16 + 1) * 4);          // pieces of the rows' sums of squares (deferred RMSNorm, few-row path)
  // dflash_prefill: the prompts' lengths and the pseudo-sequence batch of a pass (see prefill_plan_kernel)
  w.pf_lens = take((size_t)rt.max_seqs * 4);
  w.pf_plens = take((size_t)rt.max_seqs * 4);
  w.pf_table = take((size_t)rt.max_seqs * rt.max_pages_per_seq * 4);
  w.pf_tokens = take((size_t)M * 4);
  w.pf_end_row = take((size_t)rt.max_seqs * 4);
  w.pf_end_seq = take((size_t)rt.max_seqs * 4);
  w.pf_first = take((size_t)rt.max_seqs * 4);
  w.pf_anchor = take((size_t)rt.max_seqs * 4);
  w.moe_sel_e = w.moe_sel_w = w.moe_sel_pos = w.moe_row_of = w.moe_items = w.moe_a = w.moe_act = w.moe_y = 0;
  if (t.n_experts) {
    const size_t mk = (size_t)M * t.top_k, np = moe_positions(t, M);
    w.moe_sel_e = take(mk * 4);
    w.moe_sel_w = take(mk * 4);
    w.moe_sel_pos = take(mk * 4);
    w.moe_row_of = take(np * 4);
    w.moe_items = take((size_t)moe_items(t, M, 1) * 16);
    w.moe_a = take(np * D * es * planes);              // the normalised rows in list order, GEMM operand layout
    w.moe_act = take(np * t.d_expert * es * planes);   // SwiGLU products of the sorted list, GEMM operand layout
    w.moe_y = take(np * D * 4);                        // the experts' outputs, one row per list position
  }
  w.total = off;
  return w;
}

int check_runtime(const dflash_dims* t, const dflash_dims* d, const dflash_runtime* rt) {
  if (!rt) return fail(nullptr, DFLASH_EINVAL, "runtime: null");
  if (rt->block_size < 2 || rt->block_size > DFLASH_MAX_BLOCK) return fail(nullptr, DFLASH_EINVAL, "block_size must be in [2,%d]", DFLASH_MAX_BLOCK);
  if (rt->max_seqs < 1 || rt->max_pages_per_seq < 1 || rt->n_pages < 1) return fail(nullptr, DFLASH_EINVAL, "max_seqs, max_pages_per_seq, n_pages must be positive");
  if (rt->n_taps < 1 || rt->n_taps > DFLASH_MAX_TAPS) return fail(nullptr, DFLASH_EINVAL, "n_taps must be in [1,%d]", DFLASH_MAX_TAPS);
  for (int i = 0; i < rt->n_taps; ++i) {
    if (rt->tap_layers[i] < 0 || rt->tap_layers[i] >= t->n_layers || (i && rt->tap_layers[i] <= rt->tap_layers[i - 1]))
      return fail(nullptr, DFLASH_EINVAL, "tap_layers must be ascending layer indices of the target");
  }
  if (rt->mask_token_id < 0 || rt->mask_token_id >= t->vocab) return fail(nullptr, DFLASH_EINVAL, "mask_token_id outside the vocabulary");
  if (t->dtype != d->dtype) return fail(nullptr, DFLASH_EINVAL, "target and draft must share the dtype");
  if (t->d_model != d->d_model || t->vocab != d->vocab) return fail(nullptr, DFLASH_EINVAL, "draft shares embedding and LM head: d_model and vocab must match the target");
  if (d->n_experts) return fail(nullptr, DFLASH_EINVAL, "the draft model is dense: n_experts must be 0");
  if (t->n_experts && (int64_t)t->n_experts * ((rt->max_seqs * rt->block_size + 31) / 32) > MOE_MASK_WORDS)
    return fail(nullptr, DFLASH_EINVAL, "routed experts: n_experts * ceil(max_seqs * block_size / 32) must not exceed %d", MOE_MASK_WORDS);
  if (t->dtype == DFLASH_BF16 && ((size_t)rt->n_taps * t->d_model) % 32) return fail(nullptr, DFLASH_EINVAL, "n_taps*d_model must be a multiple of 32");
  for (const dflash_dims* m : {t, d})
    if (attn_q_shift(*m, rt->block_size) < 0)
      return fail(nullptr, DFLASH_EINVAL, "block_size * (n_q_heads/n_kv_heads) above 64 needs bf16, head_dim 64 or 128 and a group size that halves evenly");
  return DFLASH_OK;
}

}  // namespace

struct dflash_ctx {
  dflash_dims t, d;
  dflash_runtime rt;
  TargetLayout tl;
  DraftLayout dl;
  Workspace ws;
  const char* tblob;
  const char* dblob;
  char* wsp;
  char err[512];
  Knobs k;                                             // tuning / testing knobs as they stood when the context was created
  int64_t gemm_counts[DFLASH_GEMM_KINDS] = {};         // dflash_gemm_counts: GEMM launches per kernel family since the last read
  int32_t* moe_trace = nullptr;                        // dflash_moe_trace: where the routed layers also leave their expert choices
  bool have_logits_d = false, have_logits_t = false;   // the workspace holds this step's draft / target logits
  float draft_temperature = 0.f;                       // of the last dflash_draft_block call
  float stats_q_T = 0.f, stats_p_T = 0.f;              // > 0: ws.stats_q / ws.stats_p hold this step's (max, log-sum-exp) rows at that temperature
  // k.fuse, few-row path (one band of rows, dense bf16 model): 1 = the O projection runs unsplit with the residual update in
  // its epilogue and the RMSNorm that follows deferred into the gate/up GEMM; 2 = the down projection as well (then no
  // separate normalisation launch is left in a layer); 0 = separate kernels throughout
  // optional per-launch timing (dflash_profile_*): event pairs around the GEMM and attention launches
  bool prof_on = false;
  std::vector<hipEvent_t> ev;
  std::vector<int> ev_cls;
  std::vector<double> ev_bytes;
};

namespace {

#define CTX_FAIL(ctx, code, ...) fail((ctx)->err, code, __VA_ARGS__)

constexpr size_t kMaxProfLaunches = 16384;

struct ProfScope {
  dflash_ctx* c;
  hipStream_t st;
  hipEvent_t stop = nullptr;
  ProfScope(dflash_ctx* c_, hipStream_t st_, int cls, double bytes) : c(c_), st(st_) {
    if (!c->prof_on || c->ev_cls.size() >= kMaxProfLaunches) return;
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return;
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return; }
    c->ev.push_back(a);
    c->ev.push_back(b);
    c->ev_cls.push_back(cls);
    c->ev_bytes.push_back(bytes);
    (void)hipEventRecord(a, st);
    stop = b;
  }
  ~ProfScope() {
    if (stop) (void)hipEventRecord(stop, st);
  }
};

template <typename T>
struct Engine {
  dflash_ctx* c;
  hipStream_t st;
  int hip_err = 0;

  void check() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess && !hip_err) {
      hip_err = 1;
      fail(c->err, DFLASH_EHIP, "HIP launch failed: %s", hipGetErrorString(e));
    }
  }
  template <typename P> P* ws(size_t off) { return reinterpret_cast<P*>(c->wsp + off); }
  int32_t* status() { return ws<int32_t>(c->ws.status); }

  // rows per sequence of this call: the batch's own block size if it gives one, else the context's
  int blk(const dflash_batch* b) const { return b->block_size > 0 ? b->block_size : c->rt.block_size; }
  SeqGeom geom(const dflash_batch* b) {
    SeqGeom g;
    g.seq_lens = b->seq_lens;
    g.block_table = b->block_table;
    g.max_pages_per_seq = c->rt.max_pages_per_seq;
    g.n_pages = c->rt.n_pages;
    g.block_size = blk(b);
    g.status = status();
    return g;
  }

  // Result of a GEMM that still has to be summed over its K ranges by the consumer.
  struct Slab {
    const float* p = nullptr;
    int ks = 0;
    size_t stride = 0;
    RowMix mix;   // routed experts: p holds the experts' outputs per list position, to be mixed per row (see rmsnorm_kernel)
  };
  Slab pending;          // partial sums that the next RMSNorm adds into the residual stream ws.h
  int amax_parts = 0;    // > 0: the last LM-head GEMM left that many per-row argmax partials in ws.amax (fused epilogue)
  int lse_parts = 0;     // > 0: ... and that many per-row softmax-statistics partials in ws.lsep
  bool lm_skip_store = false;   // the LM-head GEMM may drop its logits when its argmax is fused (nobody will read them)
  int pending_tap = -1;  // tap index to be taken from the completed residual stream by the next RMSNorm

  // Few-row path: ws.a holds x * gain with the division by the row's rms deferred to the GEMM that reads it; the
  // pieces of the rows' sums of squares are in ws.ssq (see gemm_resid.h)
  int cur_layer = 0;     // layer index of the layer() call in progress (routed experts: row of the choice trace)
  int defer_parts = 0;
  bool few_rows(const dflash_dims& m, int M, int level = 2) const {
    return std::is_same<T, bf16_t>::value && c->k.fuse >= level && !m.n_experts && M <= 16 && m.d_model % 16 == 0;
  }
  EpiArgs deferred(EpiArgs ep, const dflash_dims& m) {
    ep.ssq = ws<float>(c->ws.ssq);
    ep.ssq_parts = defer_parts;
    ep.ssq_inv_D = 1.0f / (float)m.d_model;
    ep.ssq_eps = m.rms_eps;
    return ep;
  }
  // h += A W^T, ws.a = h * gain_next, sums of squares -> ws.ssq, optional tap (gemm_bf16_resid_kernel)
  void resid(const T* W, const T* A, int M, int N, int K, const float* gain_next, int tap);
  void layer_few_rows(const dflash_dims& m, const char* lbase, const LayerOff& lo, T* pool, int l, const dflash_batch* b, bool causal,
                      const float* gain_next, int tap) {
    const int S = b->n_seqs, B = blk(b), M = S * B, D = m.d_model;
    const int qd = m.n_q_heads * m.head_dim, kd = m.n_kv_heads * m.head_dim, nqkv = qd + 2 * kd;
    float* arena = ws<float>(c->ws.arena);
    T* a = ws<T>(c->ws.a);
    const Slab qs = gemm(reinterpret_cast<const T*>(lbase + lo.wqkv), a, M, nqkv, D, EPI_STORE, deferred(EpiArgs{arena, nqkv, 0, nullptr, 0}, m));
    qkv_post(m, lbase, lo, pool, l, b, qs);
    attention(m, pool, l, b, causal);
    resid(reinterpret_cast<const T*>(lbase + lo.wo), ws<T>(c->ws.o), M, D, qd, reinterpret_cast<const float*>(lbase + lo.g2), -1);
    gemm(reinterpret_cast<const T*>(lbase + lo.wgu), a, M, 2 * m.d_ffn, D, EPI_SWIGLU, deferred(EpiArgs{nullptr, 0, 0, ws<T>(c->ws.act), m.d_ffn}, m));
    resid(reinterpret_cast<const T*>(lbase + lo.wd), ws<T>(c->ws.act), M, D, m.d_ffn, gain_next, tap);
  }
  void qkv_post(const dflash_dims& m, const char* lbase, const LayerOff& lo, T* pool, int l, const dflash_batch* b, const Slab& qs) {
    const int M = b->n_seqs * blk(b);
    const int qd = m.n_q_heads * m.head_dim, kd = m.n_kv_heads * m.head_dim, nqkv = qd + 2 * kd;
    RopeArgs ra;
    ra.n_q_heads = m.n_q_heads; ra.n_kv_heads = m.n_kv_heads; ra.head_dim = m.head_dim;
    ra.q_off = 0; ra.k_off = qd; ra.v_off = qd + kd;
    ra.qk_norm = m.qk_norm; ra.eps = m.rms_eps; ra.layer = l;
    ra.rope = ws<float2>(&m == &c->t ? c->ws.rope_t : c->ws.rope_d);
    hipLaunchKernelGGL(qkv_post_kernel<T>, dim3(M, (m.n_q_heads + 2 * m.n_kv_heads + 3) / 4), dim3(256), 0, st, qs.p, nqkv,
                       reinterpret_cast<const float*>(lbase + lo.qn), reinterpret_cast<const float*>(lbase + lo.kn), ws<T>(c->ws.q), pool,
                       geom(b), ra, qs.ks, qs.stride);
    check();
  }

  // ---- GEMM dispatch ------------------------------------------------------------------------------
  // STORE: partial slabs into ep.out (room for max_ks(M) * M * ld floats).  RESID: y is to be added to
  // ws.h: the bf16 path writes partial slabs into the arena and returns them as pending, the fp32 path
  // adds in place and returns nothing.  SWIGLU: complete activations, never split.
  Slab gemm(const T* W, const T* A, int M, int N, int K, int epi, EpiArgs ep, bool allow_split = true);

  void norm(const float* base, Slab delta, float* h_out, const float* gain, T* out, int M, int D, float eps, int tap = -1) {
    T* taps = tap >= 0 ? ws<T>(c->ws.taps) : (T*)nullptr;
    const int tap_K = c->rt.n_taps * c->t.d_model;
    if (delta.mix.pos)
      hipLaunchKernelGGL((rmsnorm_kernel<T, 256, true>), dim3(M), dim3(256), 0, st, base, delta.p, delta.ks, delta.stride, h_out, gain, out, D,
                         eps, taps, tap, tap_K, delta.mix);
    else if (D >= 4096)   // one 16-byte chunk per thread: the row's loads are all in flight at once
      hipLaunchKernelGGL((rmsnorm_kernel<T, 1024>), dim3(M), dim3(1024), 0, st, base, delta.p, delta.ks, delta.stride, h_out, gain, out, D,
                         eps, taps, tap, tap_K, RowMix{});
    else
      hipLaunchKernelGGL((rmsnorm_kernel<T, 256>), dim3(M), dim3(256), 0, st, base, delta.p, delta.ks, delta.stride, h_out, gain, out, D,
                         eps, taps, tap, tap_K, RowMix{});
    check();
  }
  // row-wise argmax (or Gumbel-perturbed argmax) in two launches: per-chunk winners, then one wavefront per row
  void argmax(const float* logits, int V, int M, int B, int32_t* out, int skip_slot0, int mode, float inv_T, const uint64_t* key) {
    float2* part = ws<float2>(c->ws.amax);
    int parts = amax_parts;
    if (parts == 0) {   // not fused into the LM head (fp32 models): partials from the stored logits
      parts = ARGMAX_CHUNKS;
      hipLaunchKernelGGL(argmax_rows_kernel, dim3(ARGMAX_CHUNKS, M), dim3(256), 0, st, logits, V, B, part, mode, inv_T, key);
      check();
    }
    hipLaunchKernelGGL(argmax_finish_kernel, dim3(M), dim3(64), 0, st, part, parts, B, out, skip_slot0);
    check();
    amax_parts = 0;
  }
  // RMSNorm of the residual stream, folding in whatever the previous GEMM left pending
  void norm_h(const float* gain, int M, int D, float eps) {
    float* h = ws<float>(c->ws.h);
    norm(h, pending, h, gain, ws<T>(c->ws.a), M, D, eps, pending_tap);
    pending = Slab{};
    pending_tap = -1;
  }

  void attention(const dflash_dims& m, const T* pool, int layer, const dflash_batch* b, bool causal);

  // one Transformer layer on the M block rows held in ws.h
  void layer(const dflash_dims& m, const char* lbase, const LayerOff& lo, T* pool, int l, const dflash_batch* b, bool causal) {
    const int S = b->n_seqs, B = blk(b), M = S * B, D = m.d_model;
    const int qd = m.n_q_heads * m.head_dim, kd = m.n_kv_heads * m.head_dim, nqkv = qd + 2 * kd;
    float* h = ws<float>(c->ws.h);
    float* arena = ws<float>(c->ws.arena);
    T* a = ws<T>(c->ws.a);
    T* o = ws<T>(c->ws.o);
    T* act = ws<T>(c->ws.act);
    norm_h(reinterpret_cast<const float*>(lbase + lo.g1), M, D, m.rms_eps);
    const Slab qs = gemm(reinterpret_cast<const T*>(lbase + lo.wqkv), a, M, nqkv, D, EPI_STORE, EpiArgs{arena, nqkv, 0, nullptr, 0});
    qkv_post(m, lbase, lo, pool, l, b, qs);
    attention(m, pool, l, b, causal);
    if (few_rows(m, M, 1)) {
      // one band of rows: unsplit O projection with the residual update in its epilogue, the second RMSNorm deferred
      // into the gate/up GEMM (gemm_resid.h); the down projection keeps its K split and the normalisation kernel
      resid(reinterpret_cast<const T*>(lbase + lo.wo), o, M, D, qd, reinterpret_cast<const float*>(lbase + lo.g2), -1);
      gemm(reinterpret_cast<const T*>(lbase + lo.wgu), a, M, 2 * m.d_ffn, D, EPI_SWIGLU, deferred(EpiArgs{nullptr, 0, 0, act, m.d_ffn}, m));
      pending = gemm(reinterpret_cast<const T*>(lbase + lo.wd), act, M, D, m.d_ffn, EPI_RESID, EpiArgs{h, D, 0, nullptr, 0});
      return;
    }
    pending = gemm(reinterpret_cast<const T*>(lbase + lo.wo), o, M, D, qd, EPI_RESID, EpiArgs{h, D, 0, nullptr, 0});
    norm_h(reinterpret_cast<const float*>(lbase + lo.g2), M, D, m.rms_eps);
    if (m.n_experts) {
      cur_layer = l;
      pending = moe_ffn(m, lbase, lo, M);
      return;
    }
    gemm(reinterpret_cast<const T*>(lbase + lo.wgu), a, M, 2 * m.d_ffn, D, EPI_SWIGLU, EpiArgs{nullptr, 0, 0, act, m.d_ffn});
    pending = gemm(reinterpret_cast<const T*>(lbase + lo.wd), act, M, D, m.d_ffn, EPI_RESID, EpiArgs{h, D, 0, nullptr, 0});
  }

  // Routed-expert FFN on the normalised rows in ws.a: router GEMM -> top-k routing into an expert-sorted row list ->
  // gate/up (+ SwiGLU) and down projections as grouped launches, every workgroup streaming the matrix of the expert
  // its bands belong to -> weighted sum per token, left as a slab that the next RMSNorm adds to the residual stream.
  Slab moe_ffn(const dflash_dims& m, const char* lbase, const LayerOff& lo, int M);

  // final norm + LM head with the row argmax fused into the GEMM epilogue where the kernel supports it (then
  // amax_parts > 0 and, unless want_logits, the [M, V] logits are never written); argmax() finishes the job
  // stats_T > 0: the epilogue also leaves the softmax statistics of logits / stats_T, combined into stats_out; returns
  // whether that happened (kernels without the fused epilogue leave it to row_lse_kernel)
  // few: the final norm is already deferred into ws.a / ws.ssq by the last layer's down projection
  bool lm_head(const float* final_gain, float eps, int M, float* logits, bool want_logits, int B, int mode, float inv_T,
               const uint64_t* key, float stats_T = 0.f, float2* stats_out = nullptr, bool few = false) {
    const dflash_dims& t = c->t;
    EpiArgs ep{logits, t.vocab, 0, nullptr, 0};
    if (few) {
      ep = deferred(ep, t);
      ep.ssq_eps = eps;
    } else {
      norm_h(final_gain, M, t.d_model, eps);
    }
    ep.amax = ws<float2>(c->ws.amax);
    ep.amax_mode = mode;
    ep.amax_inv_T = inv_T;
    ep.amax_key = key;
    ep.amax_B = B;
    if (stats_T > 0.f && c->k.lm_stats == 1) {
      ep.lse = ws<float2>(c->ws.lsep);
      ep.lse_inv_T = 1.0f / stats_T;
    }
    lm_skip_store = !want_logits;
    amax_parts = 0;
    lse_parts = 0;
    gemm(reinterpret_cast<const T*>(c->tblob + c->tl.lm), ws<T>(c->ws.a), M, t.vocab, t.d_model, EPI_STORE, ep, false);
    lm_skip_store = false;
    if (lse_parts == 0) return false;
    hipLaunchKernelGGL(lse_finish_kernel, dim3(M), dim3(64), 0, st, ws<float2>(c->ws.lsep), lse_parts, stats_out);
    check();
    lse_parts = 0;
    return true;
  }

  int draft_block(const dflash_batch* b, float temperature, const uint64_t* rng_key, int32_t* draft_tokens, float* logits_out) {
    const int S = b->n_seqs, B = blk(b), M = S * B;
    const dflash_dims& d = c->d;
    hipLaunchKernelGGL(build_block_kernel, dim3((M + 255) / 256), dim3(256), 0, st, b->anchor, draft_tokens, S, B, c->rt.mask_token_id);
    check();
    const bool few = few_rows(d, M);
    const char* l0 = c->dblob + c->dl.layer0;
    EmbedFuse ef;
    if (few) {
      ef.gain = reinterpret_cast<const float*>(l0 + c->dl.lo.g1);
      ef.a_out = ws<T>(c->ws.a);
      ef.ssq = ws<float>(c->ws.ssq);
      defer_parts = 1;
    }
    hipLaunchKernelGGL(embed_kernel<T>, dim3(M), dim3(256), 0, st, reinterpret_cast<const T*>(c->tblob + c->tl.embed), draft_tokens,
                       ws<float>(c->ws.h), d.d_model, d.vocab, status(), b->seq_lens, B, b->max_seq_len,
                       RopeTab{ws<float2>(c->ws.rope_d), log((double)d.rope_theta), d.head_dim}, RopeTab{nullptr, 0.0, 0}, ef);
    check();
    for (int i = 0; i < d.n_layers; ++i) {
      const char* lb = l0 + c->dl.lo.end * i;
      if (few) {
        const float* gn = i + 1 < d.n_layers ? reinterpret_cast<const float*>(lb + c->dl.lo.end + c->dl.lo.g1)
                                             : reinterpret_cast<const float*>(c->dblob + c->dl.gf);
        layer_few_rows(d, lb, c->dl.lo, reinterpret_cast<T*>(c->rt.draft_kv_pool), i, b, false, gn, -1);
      } else {
        layer(d, lb, c->dl.lo, reinterpret_cast<T*>(c->rt.draft_kv_pool), i, b, false);
      }
    }
    float* logits = ws<float>(c->ws.logits_d);
    const int mode = temperature > 0.f ? 1 : 0;
    const float inv_T = mode ? 1.0f / temperature : 1.0f;
    const bool want_logits = logits_out || mode;        // sampling: dflash_accept needs the proposal distribution
    const bool st_q = lm_head(reinterpret_cast<const float*>(c->dblob + c->dl.gf), d.rms_eps, M, logits, want_logits, B, mode, inv_T, rng_key,
                              mode ? temperature : 0.f, ws<float2>(c->ws.stats_q), few);
    c->stats_q_T = st_q ? temperature : 0.f;
    c->have_logits_d = want_logits || amax_parts == 0;
    c->draft_temperature = temperature;
    argmax(logits, d.vocab, M, B, draft_tokens, 1, mode, inv_T, rng_key);
    if (logits_out) {
      if (hipMemcpyAsync(logits_out, logits, (size_t)M * d.vocab * 4, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return CTX_FAIL(c, DFLASH_EHIP, "logits copy failed");
    }
    return hip_err ? DFLASH_EHIP : DFLASH_OK;
  }

  int verify(const dflash_batch* b, const int32_t* tokens, int32_t* tgt_argmax, float* logits_out) {
    const int S = b->n_seqs, B = blk(b), M = S * B;
    const dflash_dims& t = c->t;
    // the draft's table is for the context K/V rows that the commit of this verification will project
    const bool few = few_rows(t, M);
    const char* l0 = c->tblob + c->tl.layer0;
    EmbedFuse ef;
    if (few) {
      ef.gain = reinterpret_cast<const float*>(l0 + c->tl.lo.g1);
      ef.a_out = ws<T>(c->ws.a);
      ef.ssq = ws<float>(c->ws.ssq);
      defer_parts = 1;
    }
    hipLaunchKernelGGL(embed_kernel<T>, dim3(M), dim3(256), 0, st, reinterpret_cast<const T*>(c->tblob + c->tl.embed), tokens,
                       ws<float>(c->ws.h), t.d_model, t.vocab, status(), b->seq_lens, B, b->max_seq_len,
                       RopeTab{ws<float2>(c->ws.rope_t), log((double)t.rope_theta), t.head_dim},
                       RopeTab{ws<float2>(c->ws.rope_d), log((double)c->d.rope_theta), c->d.head_dim}, ef);
    check();
    int tap = 0;
    for (int l = 0; l < t.n_layers; ++l) {
      const char* lb = l0 + c->tl.lo.end * l;
      const bool tapped = tap < c->rt.n_taps && c->rt.tap_layers[tap] == l;
      if (few) {
        const float* gn = l + 1 < t.n_layers ? reinterpret_cast<const float*>(lb + c->tl.lo.end + c->tl.lo.g1)
                                             : reinterpret_cast<const float*>(c->tblob + c->tl.gf);
        layer_few_rows(t, lb, c->tl.lo, reinterpret_cast<T*>(c->rt.target_kv_pool), l, b, true, gn, tapped ? tap : -1);
      } else {
        layer(t, lb, c->tl.lo, reinterpret_cast<T*>(c->rt.target_kv_pool), l, b, true);
        if (tapped) pending_tap = tap;   // taken by the next RMSNorm
      }
      if (tapped) ++tap;
    }
    float* logits = ws<float>(c->ws.logits_t);
    if (!tgt_argmax && !logits_out) {
      // nobody wants the tokens after these rows (a prefill chunk that ends no prompt): K/V rows and taps are all the
      // call is for, so the final norm runs only if the last layer's output is itself tapped, and the LM head not at all
      if (pending_tap >= 0) norm_h(reinterpret_cast<const float*>(c->tblob + c->tl.gf), M, t.d_model, t.rms_eps);
      pending = Slab{};
      c->have_logits_t = false;
      c->stats_p_T = 0.f;
      return hip_err ? DFLASH_EHIP : DFLASH_OK;
    }
    const bool want_logits = logits_out || c->draft_temperature > 0.f;   // sampling: dflash_accept needs the target distribution
    const float sT = c->draft_temperature > 0.f ? c->draft_temperature : 0.f;
    const bool st_p = lm_head(reinterpret_cast<const float*>(c->tblob + c->tl.gf), t.rms_eps, M, logits, want_logits, B, 0, 1.0f, nullptr, sT,
                              ws<float2>(c->ws.stats_p), few);
    c->stats_p_T = st_p ? sT : 0.f;
    c->have_logits_t = want_logits || amax_parts == 0;
    if (tgt_argmax) argmax(logits, t.vocab, M, B, tgt_argmax, 0, 0, 1.0f, (const uint64_t*)nullptr);
    else amax_parts = 0;
    if (logits_out) {
      if (hipMemcpyAsync(logits_out, logits, (size_t)M * t.vocab * 4, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return CTX_FAIL(c, DFLASH_EHIP, "logits copy failed");
    }
    return hip_err ? DFLASH_EHIP : DFLASH_OK;
  }

  int accept(const dflash_batch* b, const int32_t* draft_tokens, const int32_t* tgt_argmax, float temperature, const float* uniforms,
             const uint64_t* rng_key, int32_t* accept_len, int32_t* out_tokens) {
    const int S = b->n_seqs, B = blk(b), M = S * B, V = c->t.vocab;
    if (temperature <= 0.f) {
      hipLaunchKernelGGL(accept_greedy_kernel, dim3((S + 63) / 64), dim3(64), 0, st, draft_tokens, tgt_argmax, S, B, accept_len, out_tokens);
      check();
    } else {
      const float inv_T = 1.0f / temperature;
      // the (max, log-sum-exp) rows normally come out of the LM-head epilogues; another temperature than the one
      // the draft was sampled at, or a kernel without that epilogue, takes them from the stored logits
      if (c->stats_p_T != temperature) {
        hipLaunchKernelGGL(row_lse_kernel, dim3(M), dim3(1024), 0, st, ws<float>(c->ws.logits_t), V, inv_T, ws<float2>(c->ws.stats_p));
        check();
      }
      if (c->stats_q_T != temperature) {
        hipLaunchKernelGGL(row_lse_kernel, dim3(M), dim3(1024), 0, st, ws<float>(c->ws.logits_d), V, inv_T, ws<float2>(c->ws.stats_q));
        check();
      }
      hipLaunchKernelGGL(accept_sampling_kernel, dim3(S), dim3(1024), 0, st, ws<float>(c->ws.logits_t), ws<float>(c->ws.logits_d),
                         ws<float2>(c->ws.stats_p), ws<float2>(c->ws.stats_q), draft_tokens, uniforms, rng_key, V, B, inv_T,
                         accept_len, out_tokens);
      check();
    }
    return hip_err ? DFLASH_EHIP : DFLASH_OK;
  }

  int commit(const dflash_batch* b, const int32_t* accept_len, const int32_t* out_tokens, int64_t* kv_slots) {
    const int S = b->n_seqs;
    commit_project(b);
    hipLaunchKernelGGL(commit_update_kernel, dim3((S + 63) / 64), dim3(64), 0, st, geom(b), b->seq_lens, b->anchor, accept_len,
                       out_tokens, S, kv_slots);
    check();
    return hip_err ? DFLASH_EHIP : DFLASH_OK;
  }

  // H_t = RMSNorm(W_c [taps]) of the rows of the preceding verification pass, projected with every draft layer's W_K, W_V
  // into the draft pool at the rows' positions (Appendix A.3)
  void commit_project(const dflash_batch* b) {
    const int S = b->n_seqs, B = blk(b), M = S * B;
    const dflash_dims& d = c->d;
    const int D = d.d_model, kd = d.n_kv_heads * d.head_dim, nkv = d.n_layers * 2 * kd;
    float* arena = ws<float>(c->ws.arena);
    T* ht = ws<T>(c->ws.ht);
    const Slab fs = gemm(reinterpret_cast<const T*>(c->dblob + c->dl.wc), ws<T>(c->ws.taps), M, D, c->rt.n_taps * c->t.d_model, EPI_STORE,
                         EpiArgs{arena, D, 0, nullptr, 0});
    norm(nullptr, fs, ws<float>(c->ws.fuse), reinterpret_cast<const float*>(c->dblob + c->dl.gc), ht, M, D, d.rms_eps);
    const Slab kvs = gemm(reinterpret_cast<const T*>(c->dblob + c->dl.wkv_all), ht, M, nkv, D, EPI_STORE, EpiArgs{arena, nkv, 0, nullptr, 0});
    {   // k-norm, RoPE and page write of all draft layers' context K/V in one launch (grid.z = layer)
      RopeArgs ra;
      ra.n_q_heads = 0; ra.n_kv_heads = d.n_kv_heads; ra.head_dim = d.head_dim;
      ra.q_off = 0; ra.k_off = 0; ra.v_off = kd;
      ra.qk_norm = d.qk_norm; ra.eps = d.rms_eps; ra.layer = 0;
      ra.rope = ws<float2>(c->ws.rope_d);   // written by the verify call whose taps are being committed
      ra.col_stride = 2 * kd;
      ra.kn_stride = c->dl.lo.end / sizeof(float);     // layer records are 256-byte aligned
      const char* lbase = c->dblob + c->dl.layer0;
      hipLaunchKernelGGL(qkv_post_kernel<T>, dim3(M, (2 * d.n_kv_heads + 3) / 4, d.n_layers), dim3(256), 0, st, kvs.p, nkv, (const float*)nullptr,
                         reinterpret_cast<const float*>(lbase + c->dl.lo.kn), (T*)nullptr, reinterpret_cast<T*>(c->rt.draft_kv_pool),
                         geom(b), ra, kvs.ks, kvs.stride);
      check();
    }
  }

  // Prefill of the prompts' new tokens as many-row passes of at most max_seqs pseudo-sequences (prefill_plan_kernel): the
  // target's layers over all rows (K/V rows into the target pool, taps), the LM head on the last row of every prompt
  // only, the taps of all rows fused and projected into the draft's context cache.  lens_host: new tokens per prompt.
  int prefill(const dflash_batch* b, const int32_t* tokens, const int32_t* lens_host, int32_t* first_out) {
    const int S = b->n_seqs, B = blk(b);
    const dflash_dims& t = c->t;
    int total_chunks = 0, max_len = 0;
    for (int s = 0; s < S; ++s) {
      total_chunks += (lens_host[s] + B - 1) / B;
      max_len = std::max(max_len, lens_host[s]);
    }
    if (total_chunks == 0) return DFLASH_OK;
    int32_t* d_lens = ws<int32_t>(c->ws.pf_lens);
    if (hipMemcpyAsync(d_lens, lens_host, (size_t)S * 4, hipMemcpyHostToDevice, st) != hipSuccess) return CTX_FAIL(c, DFLASH_EHIP, "prefill: length upload failed");
    for (int chunk0 = 0; chunk0 < total_chunks; chunk0 += c->rt.max_seqs) {
      const int n = std::min(c->rt.max_seqs, total_chunks - chunk0), M = n * B;
      // prompts whose last chunk lies in this pass (the host counts them from the same lengths as the kernel)
      int n_end = 0, first = 0;
      for (int s = 0; s < S; ++s) {
        const int nc = (lens_host[s] + B - 1) / B;
        if (nc > 0 && first + nc - 1 >= chunk0 && first + nc - 1 < chunk0 + n) ++n_end;
        first += nc;
      }
      PrefillPlan pp;
      pp.lens = d_lens; pp.seq_lens = b->seq_lens; pp.block_table = b->block_table; pp.tokens = tokens;
      pp.S = S; pp.B = B; pp.mpps = c->rt.max_pages_per_seq; pp.chunk0 = chunk0; pp.n_chunks = n;
      pp.p_lens = ws<int32_t>(c->ws.pf_plens); pp.p_table = ws<int32_t>(c->ws.pf_table); pp.p_tokens = ws<int32_t>(c->ws.pf_tokens);
      pp.end_row = ws<int32_t>(c->ws.pf_end_row); pp.end_seq = ws<int32_t>(c->ws.pf_end_seq);
      hipLaunchKernelGGL(prefill_plan_kernel, dim3(n), dim3(256), 0, st, pp);
      check();
      dflash_batch pb;
      pb.n_seqs = n;
      pb.max_seq_len = std::min(b->max_seq_len + max_len, c->rt.max_pages_per_seq * DFLASH_PAGE_SIZE - B);
      pb.seq_lens = pp.p_lens; pb.block_table = pp.p_table; pb.anchor = ws<int32_t>(c->ws.pf_anchor);
      pb.block_size = B;
      hipLaunchKernelGGL(embed_kernel<T>, dim3(M), dim3(256), 0, st, reinterpret_cast<const T*>(c->tblob + c->tl.embed), pp.p_tokens,
                         ws<float>(c->ws.h), t.d_model, t.vocab, status(), pb.seq_lens, B, pb.max_seq_len,
                         RopeTab{ws<float2>(c->ws.rope_t), log((double)t.rope_theta), t.head_dim},
                         RopeTab{ws<float2>(c->ws.rope_d), log((double)c->d.rope_theta), c->d.head_dim}, EmbedFuse{});
      check();
      int tap = 0;
      for (int l = 0; l < t.n_layers; ++l) {
        layer(t, c->tblob + c->tl.layer0 + c->tl.lo.end * l, c->tl.lo, reinterpret_cast<T*>(c->rt.target_kv_pool), l, &pb, true);
        if (tap < c->rt.n_taps && c->rt.tap_layers[tap] == l) pending_tap = tap++;
      }
      if (n_end > 0 || pending_tap >= 0) norm_h(reinterpret_cast<const float*>(c->tblob + c->tl.gf), M, t.d_model, t.rms_eps);
      pending = Slab{};
      if (n_end > 0) {   // the first generated token of every prompt that ends here: LM head on those rows only
        T* rows_a = ws<T>(c->ws.ht);   // free until the projection below
        hipLaunchKernelGGL(gather_operand_rows_kernel<T>, dim3(n_end), dim3(256), 0, st, ws<T>(c->ws.a), pp.end_row, rows_a, t.d_model);
        check();
        float* logits = ws<float>(c->ws.logits_t);
        EpiArgs ep{logits, t.vocab, 0, nullptr, 0};
        ep.amax = ws<float2>(c->ws.amax);
        ep.amax_B = 1;
        lm_skip_store = true;
        amax_parts = 0;
        gemm(reinterpret_cast<const T*>(c->tblob + c->tl.lm), rows_a, n_end, t.vocab, t.d_model, EPI_STORE, ep, false);
        lm_skip_store = false;
        argmax(logits, t.vocab, n_end, 1, ws<int32_t>(c->ws.pf_first), 0, 0, 1.0f, (const uint64_t*)nullptr);
        hipLaunchKernelGGL(prefill_first_kernel, dim3((n_end + 63) / 64), dim3(64), 0, st, ws<int32_t>(c->ws.pf_first), pp.end_seq, n_end, b->anchor,
                           first_out);
        check();
      }
      commit_project(&pb);
    }
    hipLaunchKernelGGL(prefill_advance_kernel, dim3((S + 63) / 64), dim3(64), 0, st, b->seq_lens, d_lens, S);
    check();
    c->have_logits_t = c->have_logits_d = false;
    c->stats_p_T = c->stats_q_T = 0.f;
    return hip_err ? DFLASH_EHIP : DFLASH_OK;
  }
};

// ---- GEMM dispatch ----------------------------------------------------------------------------------
constexpr int kMaxKSplit = 16;

thread_local int g_launch_parts = 0;   // column blocks of the last bf16 GEMM launch (= fused-argmax partials per row)
thread_local int g_launch_kind = 0;    // kernel family of that launch (DFLASH_GEMM_* of dflash_gemm_counts)

template <int NT, int MT, int U>
void launch_bf16(hipStream_t st, const bf16_t* W, const bf16_t* A, int M, int N, int K, int epi, EpiArgs ep, int ks) {
  const dim3 grid((N / 16) / NT, ((M + 15) / 16 + MT - 1) / MT, ks), block(256);
  g_launch_parts = (int)grid.x;
  g_launch_kind = DFLASH_GEMM_STREAMING;
  if (epi == EPI_SWIGLU) {
    if constexpr (NT >= 2) hipLaunchKernelGGL((gemm_bf16_kernel<NT, MT, U, EPI_SWIGLU>), grid, block, 0, st, W, A, M, N, K, ep);
  } else {
    hipLaunchKernelGGL((gemm_bf16_kernel<NT, MT, U, EPI_STORE>), grid, block, 0, st, W, A, M, N, K, ep);
  }
}

template <int WN, int WM, int PD, int NS = 2, int WY = 2>
void launch_tiled(hipStream_t st, const bf16_t* W, const bf16_t* A, int M, int N, int K, int epi, EpiArgs ep, int ks) {
  const int n_blocks = (N / 16 + WY * WN - 1) / (WY * WN), m_blocks = ((M + 15) / 16 + 2 * WM - 1) / (2 * WM);
  const dim3 grid(((n_blocks + 7) / 8) * 8 * m_blocks, ks), block(128 * WY);
  g_launch_parts = n_blocks;
  g_launch_kind = WY == 4 ? DFLASH_GEMM_TILED8 : DFLASH_GEMM_TILED4;
  if (epi == EPI_SWIGLU)
    hipLaunchKernelGGL((gemm_bf16_tiled_kernel<WN, WM, PD, EPI_SWIGLU, NS, false, WY>), grid, block, 0, st, W, A, M, N, K, n_blocks, m_blocks, ep);
  else
    hipLaunchKernelGGL((gemm_bf16_tiled_kernel<WN, WM, PD, EPI_STORE, NS, false, WY>), grid, block, 0, st, W, A, M, N, K, n_blocks, m_blocks, ep);
}

inline int gemm_class(int epi, int N, int vocab) { return (epi == EPI_STORE && N == vocab) ? DFLASH_PROF_GEMM_LMHEAD : epi; }

// K split across workgroups: aim at enough workgroups that every CU keeps several wavefronts streaming,
// keep at least 2 k-tiles per wavefront, and stay inside the arena.
inline int pick_ksplit(int n_blocks, int KT, int M, int arena, int target) {
  int ks = 1;
  while (ks < kMaxKSplit && n_blocks * ks * 2 <= target && KT / (ks * 2 * 4) >= 2 && ks * 2 * M <= arena) ks *= 2;
  return ks;
}

template <>
Engine<bf16_t>::Slab Engine<bf16_t>::gemm(const bf16_t* W, const bf16_t* A, int M, int N, int K, int epi, EpiArgs ep, bool allow_split) {
  ProfScope prof(c, st, gemm_class(epi, N, c->t.vocab), (double)N * K * 2);
  const int U = c->k.gemm_u;   // k-tiles per prefetch stage
  const int nt = N / 16, KT = K / 32;
  int kepi = epi;
  if (epi == EPI_RESID) {   // partial slabs into the arena; the next RMSNorm adds them to the residual stream
    ep.out = ws<float>(c->ws.arena);
    kepi = EPI_STORE;
  }
  const bool split = allow_split && epi != EPI_SWIGLU;
  const int arena = arena_rows(c->rt.max_seqs * c->rt.block_size);
  int ks = 1;
  if (ep.amax && (split || epi != EPI_STORE)) ep.amax = nullptr;   // the fused argmax needs complete sums
  if (ep.lse && (split || epi != EPI_STORE)) ep.lse = nullptr;      // so do the fused softmax statistics
  if (ep.amax && lm_skip_store) ep.out = nullptr;
  if (M <= 16) {
    const int NT8 = c->k.gemm_nt8, FILL = c->k.gemm_fill;
    if (FILL == 1 && NT8 && nt >= 8 * NT8 && (nt % 8 == 0 || nt % 6 == 0)) {
      // a launch of 192 workgroups leaves a quarter of the CUs idle: among 8 or 6 weight tiles per wavefront and
      // any K split (not only powers of two) take the fullest last round; ties go to 8 tiles, then to fewer K ranges
      int best_nt = 0, best_ks = 1;
      double best_fill = -1.0;
      for (int cand : {8, 6}) {
        if (nt % cand) continue;
        const int nb = nt / cand;
        for (int k = 1; k <= (split ? kMaxKSplit : 1); ++k) {
          if (k > 1 && (KT / (k * 4) < 2 || k * M > arena)) break;
          const int wgs = nb * k, rounds = (wgs + 255) / 256;
          const double fill = (double)wgs / (rounds * 256.0) - 0.02 * (rounds - 1);   // a single round beats several
          if (fill > best_fill + 1e-9) { best_fill = fill; best_nt = cand; best_ks = k; }
        }
      }
      ks = best_ks;
      ep.slab = (size_t)M * ep.ld;
      if (best_nt == 8) launch_bf16<8, 1, 2>(st, W, A, M, N, K, kepi, ep, ks);
      else launch_bf16<6, 1, 2>(st, W, A, M, N, K, kepi, ep, ks);
    } else if (NT8 && nt % 8 == 0 && nt >= 8 * NT8) {
      if (split) ks = pick_ksplit(nt / 8, KT, M, arena, c->k.gemm_target_wgs);
      ep.slab = (size_t)M * ep.ld;
      if (U >= 2) launch_bf16<8, 1, 2>(st, W, A, M, N, K, kepi, ep, ks);
      else launch_bf16<8, 1, 1>(st, W, A, M, N, K, kepi, ep, ks);
    } else if (nt % 4 == 0) {
      if (split) ks = pick_ksplit(nt / 4, KT, M, arena, c->k.gemm_target_wgs);
      ep.slab = (size_t)M * ep.ld;
      if (U >= 4) launch_bf16<4, 1, 4>(st, W, A, M, N, K, kepi, ep, ks);
      else if (U >= 2) launch_bf16<4, 1, 2>(st, W, A, M, N, K, kepi, ep, ks);
      else launch_bf16<4, 1, 1>(st, W, A, M, N, K, kepi, ep, ks);
    } else if (nt % 2 == 0) {
      if (split) ks = pick_ksplit(nt / 2, KT, M, arena, c->k.gemm_target_wgs);
      ep.slab = (size_t)M * ep.ld;
      launch_bf16<2, 1, 4>(st, W, A, M, N, K, kepi, ep, ks);
    } else {
      if (split) ks = pick_ksplit(nt, KT, M, arena, c->k.gemm_target_wgs);
      ep.slab = (size_t)M * ep.ld;
      launch_bf16<1, 1, 4>(st, W, A, M, N, K, kepi, ep, ks);
    }
  } else if (M <= 64 && nt % 8 == 0) {
    // still bandwidth-bound: the same streaming kernel with two or four activation bands per weight tile.  As for a
    // single band, 8 or 6 weight tiles per wavefront and the K split are chosen for the fullest rounds of the 256 CUs
    // (gate/up of the 8B shape: 192 workgroups with 8 tiles, 256 with 6)
    const int FILL4 = c->k.gemm_fill4;   // any value but 1: 8 tiles and power-of-two K splits only
    int best_nt = 8;
    if (FILL4 == 1) {
      double best_fill = -1.0;
      for (int cand : {8, 6}) {
        if (nt % cand) continue;
        const int nb = nt / cand;
        for (int k = 1; k <= (split ? kMaxKSplit : 1); ++k) {
          if (k > 1 && (KT / (k * 4) < 2 || k * M > arena)) break;
          const int wgs = nb * k, rounds = (wgs + 255) / 256;
          const double fill = (double)wgs / (rounds * 256.0) - 0.02 * (rounds - 1);
          if (fill > best_fill + 1e-9) { best_fill = fill; best_nt = cand; ks = k; }
        }
      }
    } else if (split) {
      ks = pick_ksplit(nt / 8, KT, M, arena, c->k.gemm_target_wgs);
    }
    ep.slab = (size_t)M * ep.ld;
    const int U4 = c->k.gemm_u4;   // k-tiles per prefetch stage for 16 < M <= 64 (2 measured slower)
    if (M <= 32) {
      if (best_nt == 6) launch_bf16<6, 2, 1>(st, W, A, M, N, K, kepi, ep, ks);
      else if (U4 >= 2) launch_bf16<8, 2, 2>(st, W, A, M, N, K, kepi, ep, ks);
      else launch_bf16<8, 2, 1>(st, W, A, M, N, K, kepi, ep, ks);
    } else {
      // (the single-buffered two-workgroups-per-CU form of this kernel that the routed experts use was measured here
      // too: 58.7 us against 48.2 for gate/up at 64 rows -- a dense launch has fewer workgroups than CUs)
      if (best_nt == 6) launch_bf16<6, 4, 1>(st, W, A, M, N, K, kepi, ep, ks);
      else if (U4 >= 2) launch_bf16<8, 4, 2>(st, W, A, M, N, K, kepi, ep, ks);
      else launch_bf16<8, 4, 1>(st, W, A, M, N, K, kepi, ep, ks);
    }
  } else if (M > 64 && nt % 2 == 0) {
    // compute-bound: LDS-staged tiles of 256, 192 or 128 weight rows x 128 activation rows.  Pick the shape and
    // K split with the least estimated time: workgroups on the busiest CU x MFMA time of one workgroup (larger
    // tiles move fewer operand bytes per flop, hence the efficiency factors; a workgroup alone on its CU has
    // nobody to hide its barriers and LDS latency behind), plus the traffic of the partial slabs.
    struct Cand { int wn, wm; double eff; };
    static const Cand cands[6] = {{8, 4, 1.0}, {6, 4, 0.95}, {4, 4, 0.85}, {8, 2, 0.8}, {6, 2, 0.75}, {4, 2, 0.65}};
    int best_wn = 4, best_wm = 4;
    bool best_solo = false;
    double best = 1e30;
    for (const Cand& cd : cands) {
      if (c->k.gemm_tile && cd.wn != c->k.gemm_tile) continue;
      if (c->k.gemm_wm && cd.wm != c->k.gemm_wm) continue;
      const int mb = ((M + 15) / 16 + 2 * cd.wm - 1) / (2 * cd.wm);
      const int wgs = ((nt + 2 * cd.wn - 1) / (2 * cd.wn)) * mb;
      for (int k = 1; k <= kMaxKSplit; k *= 2) {
        if (k > 1 && (!split || KT / k < 8 || k * M > arena)) break;
        if (c->k.gemm_ks && split && k != c->k.gemm_ks && c->k.gemm_ks * M <= arena && KT / c->k.gemm_ks >= 8) continue;
        const int per_cu = (wgs * k + 255) / 256;
        const double mfma_us = 32.0 * cd.wn * cd.wm * ((KT + k - 1) / k) / 2400.0;   // MFMA issue time of one workgroup
        const double slab_us = k > 1 ? (double)k * M * N * 8 / 4e6 : 0.0;
        // a workgroup alone on its CU has nobody to hide its barriers behind; the 128-row tiles then run as a
        // three-slot direct-to-LDS ring (they have the LDS to themselves), which loses less
        const bool solo = per_cu == 1, solo_ring = solo && !split && cd.wm == 4 && cd.wn >= 6;   // measured: only pays where K is not split
        const double solo_pen = c->k.gemm_solo_pct / 100.0;   // measured 120 against 140 and 100
        const bool small_ring = cd.wm == 2 || cd.wn == 4;   // tiles that run as a direct-to-LDS ring anyway
        const double t = per_cu * mfma_us / cd.eff * (solo ? (solo_ring ? 1.15 : (small_ring ? solo_pen : 1.4)) : 1.0) + slab_us;
        if (t < best) { best = t; best_wn = cd.wn; best_wm = cd.wm; ks = k; best_solo = solo_ring; }
      }
    }
    ep.slab = (size_t)M * ep.ld;
    // Eight-wavefront tiles (four wavefronts along N: 384 or 256 weight rows x 128 or 64 activation rows, one workgroup
    // per CU): two of the four-wavefront workgroups fused along N, so the activation stage is fetched once for twice
    // the weight rows.  Taken when such a tiling with some K split gives exactly one round that fills the CUs (225-256
    // workgroups).  Isolated launches at 512 rows over random operands, against the best four-wavefront choice: gate/up
    // 166 against 197 us, QKV 46 against 51.  Whole step: 25.2 against 25.8 ms at 512 rows, 12.24 against 12.42 at 256.
    // Over several rounds they lose (gate/up of a 1024-row prefill pass, two rounds: 49.8 against 48.8 ms per prefill; the LM
    // head at 512 rows, five to seven rounds: 1157-1230 against 1090 us).
    const bool forced = c->k.gemm_tile || c->k.gemm_wm || c->k.gemm_ks;   // a forced four-wavefront shape stays forced
    if (c->k.gemm_wide == 2 || (c->k.gemm_wide == 1 && !forced)) {
      const bool any_fill = c->k.gemm_wide == 2;   // 2: the first fitting eight-wavefront tile whatever the number of workgroups
      static const int wide[4][2] = {{6, 4}, {4, 4}, {6, 2}, {4, 2}};
      for (const auto& wd : wide) {
        if (nt % (4 * wd[0])) continue;
        if (any_fill && ((c->k.gemm_tile && c->k.gemm_tile != wd[0]) || (c->k.gemm_wm && c->k.gemm_wm != wd[1]))) continue;
        const int mb = ((M + 15) / 16 + 2 * wd[1] - 1) / (2 * wd[1]);
        const int wgs = nt / (4 * wd[0]) * mb;
        for (int k = 1; k <= kMaxKSplit; k *= 2) {
          if (k > 1 && (!split || KT / k < 8 || k * M > arena)) break;
          if (any_fill ? (c->k.gemm_ks && split && k != c->k.gemm_ks && c->k.gemm_ks * M <= arena && KT / c->k.gemm_ks >= 8)
                       : (wgs * k < 225 || wgs * k > 256))
            continue;
          ks = k;
          if (wd[0] == 6 && wd[1] == 4) launch_tiled<6, 4, 1, 3, 4>(st, W, A, M, N, K, kepi, ep, ks);
          else if (wd[0] == 4 && wd[1] == 4) launch_tiled<4, 4, 1, 3, 4>(st, W, A, M, N, K, kepi, ep, ks);
          else if (wd[0] == 6) launch_tiled<6, 2, 1, 3, 4>(st, W, A, M, N, K, kepi, ep, ks);
          else launch_tiled<4, 2, 1, 4, 4>(st, W, A, M, N, K, kepi, ep, ks);
          check();
          ++c->gemm_counts[g_launch_kind];
          if (ep.amax) amax_parts = g_launch_parts;
          if (ep.lse) lse_parts = g_launch_parts;
          if (epi == EPI_SWIGLU) return Slab{};
          return Slab{ep.out, ks, ep.slab};
        }
      }
    }
    const int PD = c->k.gemm_pd;              // k tiles in flight from global memory (192/128-row tiles)
    const bool RING = c->k.gemm_ring == 1;    // any other value: register-staged variant for the small tiles
    if (best_wm == 2 && RING) {
      if (best_wn == 8) launch_tiled<8, 2, 1, 3>(st, W, A, M, N, K, kepi, ep, ks);
      else if (best_wn == 6) launch_tiled<6, 2, 1, 3>(st, W, A, M, N, K, kepi, ep, ks);
      else launch_tiled<4, 2, 1, 4>(st, W, A, M, N, K, kepi, ep, ks);
    } else if (best_wm == 2) {
      if (best_wn == 8) launch_tiled<8, 2, 2>(st, W, A, M, N, K, kepi, ep, ks);
      else if (best_wn == 6) launch_tiled<6, 2, 2>(st, W, A, M, N, K, kepi, ep, ks);
      else launch_tiled<4, 2, 2>(st, W, A, M, N, K, kepi, ep, ks);
    } else if (best_wn == 4 && RING) launch_tiled<4, 4, 1, 3>(st, W, A, M, N, K, kepi, ep, ks);
    else if (best_wn == 6 && best_solo && RING) launch_tiled<6, 4, 1, 3>(st, W, A, M, N, K, kepi, ep, ks);
    else if (best_wn == 8 && best_solo && RING) launch_tiled<8, 4, 1, 3>(st, W, A, M, N, K, kepi, ep, ks);
    else if (best_wn == 8) launch_tiled<8, 4, 1>(st, W, A, M, N, K, kepi, ep, ks);   // no registers left for a second set
    else if (best_wn == 6 && PD == 2) launch_tiled<6, 4, 2>(st, W, A, M, N, K, kepi, ep, ks);
    else if (best_wn == 6) launch_tiled<6, 4, 1>(st, W, A, M, N, K, kepi, ep, ks);
    else if (PD == 2) launch_tiled<4, 4, 2>(st, W, A, M, N, K, kepi, ep, ks);
    else launch_tiled<4, 4, 1>(st, W, A, M, N, K, kepi, ep, ks);
  } else {
    const int my = ((M + 15) / 16 + 3) / 4;
    if (nt % 2 == 0) {
      if (split && my == 1) ks = pick_ksplit(nt / 2, KT, M, arena, c->k.gemm_target_wgs);
      ep.slab = (size_t)M * ep.ld;
      launch_bf16<2, 4, 2>(st, W, A, M, N, K, kepi, ep, ks);
    } else {
      if (split && my == 1) ks = pick_ksplit(nt, KT, M, arena, c->k.gemm_target_wgs);
      ep.slab = (size_t)M * ep.ld;
      launch_bf16<1, 4, 2>(st, W, A, M, N, K, kepi, ep, ks);
    }
  }
  check();
  ++c->gemm_counts[g_launch_kind];
  if (ep.amax) amax_parts = g_launch_parts;
  if (ep.lse) lse_parts = g_launch_parts;
  if (epi == EPI_SWIGLU) return Slab{};
  return Slab{ep.out, ks, ep.slab};
}

// (four weight tiles per wavefront instead of eight were measured at 512 rows: 192 us against 174 for gate/up)
template <int MT, int U, int EPI, int PH = 1>
void launch_grouped(hipStream_t st, const bf16_t* W, const bf16_t* A, int rows, int N, int K, EpiArgs ep, int n_items) {
  const dim3 grid(((n_items + 7) / 8) * 8 * ((N / 16) / 8), 1, 1), block(256);
  ep.grp_n_items = n_items;
  hipLaunchKernelGGL((gemm_bf16_kernel<8, MT, U, EPI, true, PH>), grid, block, 0, st, W, A, rows, N, K, ep);
}

// grouped launch of the LDS-staged kernel: items of up to 8 bands (one 128-row activation block each)
template <int WN, int PD, int EPI, int NS>
void launch_grouped_tiled(hipStream_t st, const bf16_t* W, const bf16_t* A, int rows, int N, int K, EpiArgs ep, int n_items) {
  const int n_blocks = (N / 16 + 2 * WN - 1) / (2 * WN);
  const dim3 grid(((n_items + 7) / 8) * 8 * n_blocks, 1), block(256);
  hipLaunchKernelGGL((gemm_bf16_tiled_kernel<WN, 4, PD, EPI, NS, true>), grid, block, 0, st, W, A, rows, N, K, n_blocks, n_items, ep);
}

template <>
Engine<bf16_t>::Slab Engine<bf16_t>::moe_ffn(const dflash_dims& m, const char* lbase, const LayerOff& lo, int M) {
  const int D = m.d_model, E = m.n_experts, Fe = m.d_expert, k = m.top_k;
  float* arena = ws<float>(c->ws.arena);
  const bf16_t* a = ws<bf16_t>(c->ws.a);
  const Slab rs = gemm(reinterpret_cast<const bf16_t*>(lbase + lo.wr), a, M, E, D, EPI_STORE, EpiArgs{arena, E, 0, nullptr, 0});
  // bands per work item: enough for the rows an expert gets on average plus two standard deviations of an even spread,
  // so that nearly every expert's matrix is streamed by one row of workgroups only
  const double avg = (double)M * k / E, want = avg + 2.0 * sqrt(avg);
  const int mt_force = c->k.moe_mt;   // 1, 2, 4 or 8 forces the bands per work item
  // from 64 rows per expert on (a many-row prefill pass) the items are 128-row blocks of the LDS-staged kernel: the
  // streaming kernel would need two or more 64-row items for many experts, each streaming the expert's matrices.
  // Measured on one-pass prefills of the 30B-A3B shape, whose rows crowd on about a quarter of the experts: 1024 rows
  // 23.9 ms against 28.6, 2048 rows 40.5 against 51.9, 512 rows 14.9 against 16.9; the decode step of 32 sequences (32
  // rows on every expert) loses, 26.8 against 24.5 ms, so batches below 64 rows per expert keep the 64-row items
  const int MT = (mt_force == 1 || mt_force == 2 || mt_force == 4 || mt_force == 8) ? mt_force
                 : (want <= 16.0 ? 1 : (want <= 32.0 ? 2 : (avg < 64.0 ? 4 : 8)));
  const int n_items = moe_items(m, M, MT), n_pos = moe_positions(m, M);
  MoeRoute r;
  r.logits = rs.p; r.ks = rs.ks; r.stride = rs.stride;
  r.M = M; r.E = E; r.k = k; r.MT = MT;
  // with a trace buffer the choices of this layer are kept there (the kernels write and re-read them in place)
  r.sel_e = c->moe_trace ? c->moe_trace + (size_t)cur_layer * c->rt.max_seqs * c->rt.block_size * k : ws<int32_t>(c->ws.moe_sel_e);
  r.sel_w = ws<float>(c->ws.moe_sel_w); r.sel_pos = ws<int32_t>(c->ws.moe_sel_pos);
  r.row_of = ws<int32_t>(c->ws.moe_row_of);
  r.items = ws<int4>(c->ws.moe_items); r.max_items = n_items;
  r.counters = reinterpret_cast<unsigned long long*>(c->wsp + c->ws.status + 64);
  r.n_bands_out = reinterpret_cast<int32_t*>(c->wsp + c->ws.status + 128);
  if (M <= MOE_FUSED_ROWS) {
    hipLaunchKernelGGL(moe_route_kernel<true>, dim3(1), dim3(1024), 0, st, r);
  } else {
    hipLaunchKernelGGL(moe_topk_kernel, dim3((M + 3) / 4), dim3(256), 0, st, r);
    check();
    hipLaunchKernelGGL(moe_route_kernel<false>, dim3(1), dim3(1024), 0, st, r);
  }
  check();
  bf16_t* act = ws<bf16_t>(c->ws.moe_act);
  float* y = ws<float>(c->ws.moe_y);
  // tuning knob: from this many rows on the listed rows are first copied into list order (the GEMM then reads whole
  // fragments); below, the GEMM reads them through the list
  const int gather_min = c->k.moe_gather_min_rows;
  const bool gathered = M >= gather_min || MT == 8;   // the LDS-staged kernel copies whole fragments: list order only
  if (gathered) {
    hipLaunchKernelGGL(moe_gather_kernel, dim3((D / 32 + 3) / 4, n_pos / 16), dim3(256), 0, st, reinterpret_cast<const u32x4*>(a), r.row_of,
                       r.n_bands_out, D / 32, ws<u32x4>(c->ws.moe_a));
    check();
    a = ws<bf16_t>(c->ws.moe_a);
  }
  const double used = (double)std::min(E, M * k);   // experts whose matrices are streamed, at most
  // tuning knob: the 4-band grouped down projection runs single-buffered with the cross-wavefront sum in two halves (200
  // registers, 64 KB of LDS: two workgroups per CU cover each other's waits); 1 = the double-buffered form, one
  // workgroup per CU.  Measured at 512 rows: 91-95 us against 104-106.  The gate/up launch gains nothing from it (165-181
  // us from run to run against 167-176) and stays double-buffered.
  const int ph4 = c->k.moe_phases;
  {
    ProfScope prof(c, st, DFLASH_PROF_MOE_GATEUP, used * 2 * Fe * D * 2);
    EpiArgs ep{nullptr, 0, 0, act, Fe};
    ep.grp_items = r.items; ep.grp_w_stride = (size_t)2 * Fe * D; ep.grp_rows = r.row_of;
    if (gathered) ep.grp_rows = nullptr;
    const bf16_t* W = reinterpret_cast<const bf16_t*>(lbase + lo.wgu);
    if (MT == 8) {
      ep.slab = 0;
      if ((2 * Fe / 16) % 12 == 0) launch_grouped_tiled<6, 1, EPI_SWIGLU, 3>(st, W, a, n_pos, 2 * Fe, D, ep, n_items);
      else launch_grouped_tiled<4, 1, EPI_SWIGLU, 3>(st, W, a, n_pos, 2 * Fe, D, ep, n_items);
    } else if (MT == 1) launch_grouped<1, 2, EPI_SWIGLU>(st, W, a, n_pos, 2 * Fe, D, ep, n_items);   // one k tile per stage: no faster (78.9 us)
    else if (MT == 2) launch_grouped<2, 1, EPI_SWIGLU>(st, W, a, n_pos, 2 * Fe, D, ep, n_items);
    else launch_grouped<4, 1, EPI_SWIGLU>(st, W, a, n_pos, 2 * Fe, D, ep, n_items);
    check();
    ++c->gemm_counts[DFLASH_GEMM_GROUPED];
  }
  {
    ProfScope prof(c, st, DFLASH_PROF_MOE_DOWN, used * Fe * D * 2);
    EpiArgs ep{y, D, 0, nullptr, 0};
    ep.grp_items = r.items; ep.grp_w_stride = (size_t)D * Fe;
    const bf16_t* W = reinterpret_cast<const bf16_t*>(lbase + lo.wd);
    // tuning knob: k tiles per prefetch stage of the one-band down projection.  Its K is short (6 k tiles per wavefront
    // at the 30B-A3B shape): one tile per stage leaves registers for four workgroups per CU, whose prologues and
    // epilogues overlap (measured 48 us against 54 with two tiles per stage and 60 with four)
    const int down_u = c->k.moe_down_u;
    if (MT == 8) launch_grouped_tiled<4, 1, EPI_STORE, 3>(st, W, act, n_pos, D, Fe, ep, n_items);
    else if (MT == 1 && down_u == 1) launch_grouped<1, 1, EPI_STORE>(st, W, act, n_pos, D, Fe, ep, n_items);
    else if (MT == 1) launch_grouped<1, 2, EPI_STORE>(st, W, act, n_pos, D, Fe, ep, n_items);
    else if (MT == 2) launch_grouped<2, 1, EPI_STORE>(st, W, act, n_pos, D, Fe, ep, n_items);
    else if (ph4 == 2) launch_grouped<4, 1, EPI_STORE, 2>(st, W, act, n_pos, D, Fe, ep, n_items);
    else launch_grouped<4, 1, EPI_STORE>(st, W, act, n_pos, D, Fe, ep, n_items);
    check();
    ++c->gemm_counts[DFLASH_GEMM_GROUPED];
  }
  // the weighted sum of a row's experts' outputs is taken by the next RMSNorm, which adds it to the residual stream
  Slab out{y, 1, 0};
  out.mix.pos = r.sel_pos; out.mix.w = r.sel_w; out.mix.k = k;
  return out;
}
template <>
Engine<float>::Slab Engine<float>::moe_ffn(const dflash_dims&, const char*, const LayerOff&, int) { return Slab{}; }   // rejected at create: bf16 only

template <>
Engine<float>::Slab Engine<float>::gemm(const float* W, const float* A, int M, int N, int K, int epi, EpiArgs ep, bool) {
  ProfScope prof(c, st, gemm_class(epi, N, c->t.vocab), (double)N * K * 4);
  const int cols = epi == EPI_SWIGLU ? N / 2 : N;
  const dim3 grid((cols + 3) / 4), block(256);
  switch (epi) {
    case EPI_STORE: hipLaunchKernelGGL(gemm_f32_kernel<EPI_STORE>, grid, block, 0, st, W, A, M, N, K, ep); break;
    case EPI_RESID: hipLaunchKernelGGL(gemm_f32_kernel<EPI_RESID>, grid, block, 0, st, W, A, M, N, K, ep); break;
    default: hipLaunchKernelGGL(gemm_f32_kernel<EPI_SWIGLU>, grid, block, 0, st, W, A, M, N, K, ep); break;
  }
  check();
  ++c->gemm_counts[DFLASH_GEMM_F32];
  if (epi == EPI_STORE) return Slab{ep.out, 1, (size_t)M * ep.ld};
  return Slab{};
}

template <int U, int NW>
void launch_resid(hipStream_t st, const bf16_t* W, const bf16_t* A, int M, int N, int K, ResidArgs ra) {
  hipLaunchKernelGGL((gemm_bf16_resid_kernel<U, NW>), dim3(N / 16), dim3(64 * NW), 0, st, W, A, M, N, K, ra);
}

template <>
void Engine<bf16_t>::resid(const bf16_t* W, const bf16_t* A, int M, int N, int K, const float* gain_next, int tap) {
  ProfScope prof(c, st, DFLASH_PROF_GEMM_RESID, (double)N * K * 2);
  ResidArgs ra;
  ra.h = ws<float>(c->ws.h);
  ra.gain_next = gain_next;
  ra.a_out = ws<bf16_t>(c->ws.a);
  ra.ssq = ws<float>(c->ws.ssq);
  ra.taps = tap >= 0 ? ws<bf16_t>(c->ws.taps) : nullptr;
  ra.tap_idx = tap;
  ra.tap_K = c->rt.n_taps * c->t.d_model;
  const int nw = c->k.resid_nw, u = c->k.resid_u;
  if (nw == 16) launch_resid<4, 16>(st, W, A, M, N, K, ra);
  else if (nw == 8 && u <= 4) launch_resid<4, 8>(st, W, A, M, N, K, ra);
  else if (nw == 8) launch_resid<8, 8>(st, W, A, M, N, K, ra);
  else launch_resid<8, 4>(st, W, A, M, N, K, ra);
  check();
  ++c->gemm_counts[DFLASH_GEMM_FEW_ROWS];
  defer_parts = N / 16;
}
template <>
void Engine<float>::resid(const float*, const float*, int, int, int, const float*, int) {}   // bf16 only (few_rows() is false for fp32)

template <typename T>
void Engine<T>::attention(const dflash_dims& m, const T* pool, int layer, const dflash_batch* b, bool causal) {
  const int S = b->n_seqs, B = blk(b), M = S * B;
  const int max_tokens = std::min(b->max_seq_len + B, c->rt.max_pages_per_seq * DFLASH_PAGE_SIZE);
  const int q_shift = attn_q_shift(m, B);
  const SplitPlan p = plan_splits(S, m.n_kv_heads << q_shift, max_tokens, c->k.attn_target_wgs);
  AttnArgs aa;
  aa.n_q_heads = m.n_q_heads; aa.n_kv_heads = m.n_kv_heads; aa.head_dim = m.head_dim; aa.layer = layer;
  aa.causal = causal ? 1 : 0; aa.chunk = p.chunk; aa.n_splits = p.n_splits; aa.scale = 1.0f / sqrtf((float)m.head_dim);
  aa.q_shift = q_shift;
  float* part_o = ws<float>(c->ws.part_o);
  float2* part_ml = ws<float2>(c->ws.part_ml);
  {
    // algorithmic bytes: every cached K and V row of this layer once (upper bound from the host hint)
    ProfScope prof(c, st, DFLASH_PROF_ATTN, (double)S * max_tokens * 2 * m.n_kv_heads * m.head_dim * sizeof(T));
    if (!attn_mfma_launch<T>(st, ws<T>(c->ws.q), pool, geom(b), aa, S, part_o, part_ml, c->k.attn_wide_min_chunk))
      hipLaunchKernelGGL(attn_partial_simple_kernel<T>, dim3(p.n_splits, m.n_kv_heads, S), dim3(256), 0, st, ws<T>(c->ws.q), pool,
                         geom(b), aa, part_o, part_ml);
    check();
  }
  {
    ProfScope prof(c, st, DFLASH_PROF_ATTN_MERGE, 0.0);
    if (M < 128)   // measured: 9.0 us against 6.5 us at 64 rows, 8.4 against 10 at 256
      hipLaunchKernelGGL(attn_merge_rows_kernel<T>, dim3(M * m.n_q_heads), dim3(128), 0, st, part_o, part_ml, ws<T>(c->ws.o), m.n_q_heads,
                         m.head_dim, p.n_splits);
    else
      hipLaunchKernelGGL(attn_merge_kernel<T>, dim3((M + 15) / 16, m.n_q_heads), dim3(16 * (m.head_dim / 4)), 0, st, part_o, part_ml,
                         ws<T>(c->ws.o), m.n_q_heads, m.head_dim, p.n_splits, M);
    check();
  }
}

// ---- packing helpers -----------------------------------------------------------------------------------
template <typename T>
int pack_rows(hipStream_t st, PackSrc ps, int K, int total_rows, void* dst, int dst_row0, int dst_rows) {
  const size_t chunks = (size_t)total_rows * (K / 8);
  hipLaunchKernelGGL(pack_kernel<T>, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st, ps, K, total_rows, reinterpret_cast<T*>(dst),
                     dst_row0, dst_rows);
  return hipGetLastError() == hipSuccess ? DFLASH_OK : fail(nullptr, DFLASH_EHIP, "pack launch failed");
}
// packs `rows` rows into rows dst_row0.. of the dst_rows-row matrix at dst (dst_rows < 0: the matrix is just these rows)
int pack_any(int dtype, hipStream_t st, PackSrc ps, int K, int rows, void* dst, int dst_row0 = 0, int dst_rows = -1) {
  if (dst_rows < 0) dst_rows = rows;
  return dtype == DFLASH_BF16 ? pack_rows<bf16_t>(st, ps, K, rows, dst, dst_row0, dst_rows)
                              : pack_rows<float>(st, ps, K, rows, dst, dst_row0, dst_rows);
}
PackSrc one(const void* p, int rows) {
  PackSrc s{};
  s.src[0] = p; s.rows[0] = rows; s.n_src = 1; s.mode = 0;
  return s;
}
int copy_f32(hipStream_t st, void* dst, const float* src, size_t n) {
  return hipMemcpyAsync(dst, src, n * 4, hipMemcpyDeviceToDevice, st) == hipSuccess ? DFLASH_OK : fail(nullptr, DFLASH_EHIP, "gain copy failed");
}

int pack_layer_common(const dflash_dims& d, const LayerOff& lo, char* lbase, const dflash_layer_weights* w, hipStream_t st) {
  if (!w || !w->wq || !w->wk || !w->wv || !w->wo || !w->wg || !w->wu || !w->wd || !w->g1 || !w->g2)
    return fail(nullptr, DFLASH_EINVAL, "layer weights: null pointer");
  if (d.n_experts && !w->wr) return fail(nullptr, DFLASH_EINVAL, "layer weights: n_experts set but the router wr is null");
  if (d.qk_norm && (!w->qn || !w->kn)) return fail(nullptr, DFLASH_EINVAL, "layer weights: qk_norm set but qn/kn null");
  const int qd = d.n_q_heads * d.head_dim, kd = d.n_kv_heads * d.head_dim;
  int rc;
  PackSrc qkv{};
  qkv.src[0] = w->wq; qkv.src[1] = w->wk; qkv.src[2] = w->wv;
  qkv.rows[0] = qd; qkv.rows[1] = kd; qkv.rows[2] = kd; qkv.n_src = 3; qkv.mode = 0;
  if ((rc = pack_any(d.dtype, st, qkv, d.d_model, qd + 2 * kd, lbase + lo.wqkv))) return rc;
  if ((rc = pack_any(d.dtype, st, one(w->wo, d.d_model), qd, d.d_model, lbase + lo.wo))) return rc;
  if (d.n_experts) {   // every expert is packed as a matrix of its own, the blobs one after the other
    const size_t es = esize(d.dtype), fd = (size_t)d.d_expert * d.d_model;
    for (int e = 0; e < d.n_experts; ++e) {
      PackSrc gu{};
      gu.src[0] = (const char*)w->wg + e * fd * es; gu.src[1] = (const char*)w->wu + e * fd * es;
      gu.rows[0] = gu.rows[1] = d.d_expert; gu.n_src = 2; gu.mode = 1;
      if ((rc = pack_any(d.dtype, st, gu, d.d_model, 2 * d.d_expert, lbase + lo.wgu + e * 2 * fd * es))) return rc;
      if ((rc = pack_any(d.dtype, st, one((const char*)w->wd + e * fd * es, d.d_model), d.d_expert, d.d_model, lbase + lo.wd + e * fd * es))) return rc;
    }
    if ((rc = pack_any(d.dtype, st, one(w->wr, d.n_experts), d.d_model, d.n_experts, lbase + lo.wr))) return rc;
  } else {
    PackSrc gu{};
    gu.src[0] = w->wg; gu.src[1] = w->wu; gu.rows[0] = gu.rows[1] = d.d_ffn; gu.n_src = 2; gu.mode = 1;
    if ((rc = pack_any(d.dtype, st, gu, d.d_model, 2 * d.d_ffn, lbase + lo.wgu))) return rc;
    if ((rc = pack_any(d.dtype, st, one(w->wd, d.d_model), d.d_ffn, d.d_model, lbase + lo.wd))) return rc;
  }
  if ((rc = copy_f32(st, lbase + lo.g1, w->g1, d.d_model))) return rc;
  if ((rc = copy_f32(st, lbase + lo.g2, w->g2, d.d_model))) return rc;
  if (d.qk_norm) {
    if ((rc = copy_f32(st, lbase + lo.qn, w->qn, d.head_dim))) return rc;
    if ((rc = copy_f32(st, lbase + lo.kn, w->kn, d.head_dim))) return rc;
  }
  return DFLASH_OK;
}

template <typename T>
int run_kv_copy(dflash_ctx* ctx, const dflash_batch* b, int pool, int layer, int seq, int start, int count, float* k, float* v, int dir,
                hipStream_t st) {
  const dflash_dims& m = pool == DFLASH_POOL_TARGET ? ctx->t : ctx->d;
  Engine<T> e{ctx, st};
  T* p = reinterpret_cast<T*>(pool == DFLASH_POOL_TARGET ? ctx->rt.target_kv_pool : ctx->rt.draft_kv_pool);
  hipLaunchKernelGGL(kv_copy_kernel<T>, dim3(count, m.n_kv_heads), dim3(128), 0, st, p, e.geom(b), layer, m.n_kv_heads, m.head_dim, seq,
                     start, k, v, dir);
  e.check();
  return e.hip_err ? DFLASH_EHIP : DFLASH_OK;
}

int check_batch(dflash_ctx* ctx, const dflash_batch* b) {
  if (!ctx) return fail(nullptr, DFLASH_EINVAL, "ctx: null");
  if (!b) return CTX_FAIL(ctx, DFLASH_EINVAL, "batch: null pointer");
  if (b->n_seqs == 0) return DFLASH_OK;   // an empty batch is valid: the step calls enqueue nothing
  if (!b->seq_lens || !b->block_table || !b->anchor) return CTX_FAIL(ctx, DFLASH_EINVAL, "batch: null pointer");
  if (b->n_seqs < 0 || b->n_seqs > ctx->rt.max_seqs) return CTX_FAIL(ctx, DFLASH_EINVAL, "batch: n_seqs %d outside [0,%d]", b->n_seqs, ctx->rt.max_seqs);
  if (b->max_seq_len < 0) return CTX_FAIL(ctx, DFLASH_EINVAL, "batch: negative max_seq_len");
  if (b->block_size != 0 && (b->block_size < 2 || b->block_size > ctx->rt.block_size))
    return CTX_FAIL(ctx, DFLASH_EINVAL, "batch: block_size %d outside [2,%d] (0 = the context's)", b->block_size, ctx->rt.block_size);
  const int blk = b->block_size > 0 ? b->block_size : ctx->rt.block_size;
  if ((int64_t)b->max_seq_len + blk > (int64_t)ctx->rt.max_pages_per_seq * DFLASH_PAGE_SIZE)
    return CTX_FAIL(ctx, DFLASH_ECAPACITY, "batch: max_seq_len %d + block %d exceeds the %d tokens a block-table row covers", b->max_seq_len,
                    blk, ctx->rt.max_pages_per_seq * DFLASH_PAGE_SIZE);
  return DFLASH_OK;
}

}  // namespace

namespace {
// times `enqueue` on `st` with a pair of events; synchronises
template <typename F>
int timed(hipStream_t st, float* ms, F&& enqueue) {
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess) return fail(nullptr, DFLASH_EHIP, "probe: event creation failed");
  if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return fail(nullptr, DFLASH_EHIP, "probe: event creation failed"); }
  int rc = DFLASH_OK;
  if (hipEventRecord(a, st) != hipSuccess) rc = DFLASH_EHIP;
  enqueue();
  if (hipEventRecord(b, st) != hipSuccess || hipEventSynchronize(b) != hipSuccess || hipEventElapsedTime(ms, a, b) != hipSuccess ||
      hipGetLastError() != hipSuccess)
    rc = DFLASH_EHIP;
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  return rc == DFLASH_OK ? rc : fail(nullptr, DFLASH_EHIP, "probe: the device reported an error");
}
}  // namespace

// =====================================================================================================
extern "C" {

size_t dflash_target_blob_bytes(const dflash_dims* target) {
  if (check_dims(target, "target")) return 0;
  return target_layout(*target).total;
}
size_t dflash_draft_blob_bytes(const dflash_dims* draft, int32_t n_taps, int32_t d_target) {
  if (check_dims(draft, "draft") || n_taps < 1 || d_target < 1) return 0;
  return draft_layout(*draft, n_taps, d_target).total;
}
size_t dflash_kv_pool_bytes(const dflash_dims* m, int32_t n_pages) {
  if (check_dims(m, "model") || n_pages < 1) return 0;
  return (size_t)m->n_layers * n_pages * m->n_kv_heads * 2 * DFLASH_PAGE_SIZE * m->head_dim * esize(m->dtype);
}
size_t dflash_workspace_bytes(const dflash_dims* target, const dflash_dims* draft, const dflash_runtime* rt) {
  if (check_dims(target, "target") || check_dims(draft, "draft") || check_runtime(target, draft, rt)) return 0;
  return workspace_layout(*target, *draft, *rt, read_knobs()).total;
}

int dflash_pack_target_head(const dflash_dims* target, const void* embed, const void* lm_head, const float* final_gain, void* blob,
                            void* stream) {
  int rc;
  if ((rc = check_dims(target, "target"))) return rc;
  if (!embed || !lm_head || !final_gain || !blob) return fail(nullptr, DFLASH_EINVAL, "pack_target_head: null pointer");
  const TargetLayout tl = target_layout(*target);
  hipStream_t st = (hipStream_t)stream;
  char* base = (char*)blob;
  if (hipMemcpyAsync(base + tl.embed, embed, (size_t)target->vocab * target->d_model * esize(target->dtype), hipMemcpyDeviceToDevice, st) != hipSuccess)
    return fail(nullptr, DFLASH_EHIP, "embedding copy failed");
  if ((rc = pack_any(target->dtype, st, one(lm_head, target->vocab), target->d_model, target->vocab, base + tl.lm))) return rc;
  return copy_f32(st, base + tl.gf, final_gain, target->d_model);
}

int dflash_pack_target_layer(const dflash_dims* target, int32_t layer, const dflash_layer_weights* w, void* blob, void* stream) {
  int rc;
  if ((rc = check_dims(target, "target"))) return rc;
  if (!blob || layer < 0 || layer >= target->n_layers) return fail(nullptr, DFLASH_EINVAL, "pack_target_layer: bad layer or blob");
  const TargetLayout tl = target_layout(*target);
  return pack_layer_common(*target, tl.lo, (char*)blob + tl.layer0 + tl.lo.end * layer, w, (hipStream_t)stream);
}

int dflash_pack_draft_head(const dflash_dims* draft, int32_t n_taps, int32_t d_target, const void* w_c, const float* g_c,
                           const float* final_gain, void* blob, void* stream) {
  int rc;
  if ((rc = check_dims(draft, "draft"))) return rc;
  if (!w_c || !g_c || !final_gain || !blob || n_taps < 1 || d_target < 1) return fail(nullptr, DFLASH_EINVAL, "pack_draft_head: bad argument");
  if (draft->dtype == DFLASH_BF16 && ((size_t)n_taps * d_target) % 32) return fail(nullptr, DFLASH_EINVAL, "n_taps*d_target must be a multiple of 32");
  const DraftLayout dl = draft_layout(*draft, n_taps, d_target);
  hipStream_t st = (hipStream_t)stream;
  char* base = (char*)blob;
  if ((rc = pack_any(draft->dtype, st, one(w_c, draft->d_model), n_taps * d_target, draft->d_model, base + dl.wc))) return rc;
  if ((rc = copy_f32(st, base + dl.gc, g_c, draft->d_model))) return rc;
  return copy_f32(st, base + dl.gf, final_gain, draft->d_model);
}

int dflash_pack_draft_layer(const dflash_dims* draft, int32_t n_taps, int32_t d_target, int32_t layer, const dflash_layer_weights* w,
                            void* blob, void* stream) {
  int rc;
  if ((rc = check_dims(draft, "draft"))) return rc;
  if (!blob || layer < 0 || layer >= draft->n_layers || n_taps < 1 || d_target < 1) return fail(nullptr, DFLASH_EINVAL, "pack_draft_layer: bad argument");
  const DraftLayout dl = draft_layout(*draft, n_taps, d_target);
  hipStream_t st = (hipStream_t)stream;
  char* base = (char*)blob;
  if ((rc = pack_layer_common(*draft, dl.lo, base + dl.layer0 + dl.lo.end * layer, w, st))) return rc;
  // second copy of this layer's W_K, W_V rows inside the all-layers matrix used at commit
  const int kd = draft->n_kv_heads * draft->head_dim;
  PackSrc kv{};
  kv.src[0] = w->wk; kv.src[1] = w->wv; kv.rows[0] = kv.rows[1] = kd; kv.n_src = 2; kv.mode = 0;
  return pack_any(draft->dtype, st, kv, draft->d_model, 2 * kd, base + dl.wkv_all, layer * 2 * kd, draft->n_layers * 2 * kd);
}

int dflash_create(const dflash_dims* target, const void* target_blob, const dflash_dims* draft, const void* draft_blob,
                  const dflash_runtime* rt, dflash_ctx** out) {
  int rc;
  if (!out) return fail(nullptr, DFLASH_EINVAL, "create: out is null");
  *out = nullptr;
  if ((rc = check_dims(target, "target")) || (rc = check_dims(draft, "draft")) || (rc = check_runtime(target, draft, rt))) return rc;
  if (!target_blob || !draft_blob) return fail(nullptr, DFLASH_EINVAL, "create: null blob");
  if (!rt->target_kv_pool || !rt->draft_kv_pool || !rt->workspace) return fail(nullptr, DFLASH_EINVAL, "create: null pool or workspace");
  if (((uintptr_t)rt->workspace & 255) || ((uintptr_t)rt->target_kv_pool & 255) || ((uintptr_t)rt->draft_kv_pool & 255) ||
      ((uintptr_t)target_blob & 255) || ((uintptr_t)draft_blob & 255))
    return fail(nullptr, DFLASH_EINVAL, "create: buffers must be 256-byte aligned");
  if ((draft->n_layers * 2 * draft->n_kv_heads * draft->head_dim) % 16) return fail(nullptr, DFLASH_EINVAL, "draft K/V width must be a multiple of 16");
  const Knobs knobs = read_knobs();
  const Workspace ws = workspace_layout(*target, *draft, *rt, knobs);
  if (rt->workspace_bytes < ws.total) return fail(nullptr, DFLASH_EWORKSPACE, "create: workspace has %zu bytes, %zu needed", rt->workspace_bytes, ws.total);
  dflash_ctx* c = new (std::nothrow) dflash_ctx;
  if (!c) return fail(nullptr, DFLASH_EINVAL, "create: out of host memory");
  c->t = *target; c->d = *draft; c->rt = *rt;
  c->tl = target_layout(*target);
  c->dl = draft_layout(*draft, rt->n_taps, target->d_model);
  c->ws = ws;
  c->tblob = (const char*)target_blob; c->dblob = (const char*)draft_blob; c->wsp = (char*)rt->workspace;
  c->err[0] = 0;
  c->k = knobs;
  if (hipMemset(c->wsp + ws.status, 0, 256) != hipSuccess) {
    delete c;
    return fail(nullptr, DFLASH_EHIP, "create: cannot clear the device status word");
  }
  *out = c;
  return DFLASH_OK;
}

int dflash_destroy(dflash_ctx* ctx) {
  if (ctx)
    for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
  delete ctx;
  return DFLASH_OK;
}

int dflash_profile_enable(dflash_ctx* ctx, int32_t enable) {
  if (!ctx) return fail(nullptr, DFLASH_EINVAL, "ctx: null");
  ctx->prof_on = enable != 0;
  return DFLASH_OK;
}

int dflash_profile_read(dflash_ctx* ctx, void* stream, float* ms, int32_t* count, double* bytes) {
  if (!ctx) return fail(nullptr, DFLASH_EINVAL, "ctx: null");
  if (!ms || !count || !bytes) return CTX_FAIL(ctx, DFLASH_EINVAL, "profile_read: null output");
  if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return CTX_FAIL(ctx, DFLASH_EHIP, "stream synchronise failed");
  for (int i = 0; i < DFLASH_PROF_CLASSES; ++i) { ms[i] = 0.f; count[i] = 0; bytes[i] = 0.0; }
  for (size_t i = 0; i < ctx->ev_cls.size(); ++i) {
    float t = 0.f;
    if (hipEventElapsedTime(&t, ctx->ev[2 * i], ctx->ev[2 * i + 1]) == hipSuccess) {
      const int k = ctx->ev_cls[i];
      ms[k] += t; count[k] += 1; bytes[k] += ctx->ev_bytes[i];
    }
  }
  for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
  ctx->ev.clear(); ctx->ev_cls.clear(); ctx->ev_bytes.clear();
  return DFLASH_OK;
}

int dflash_probe_hbm_read(const void* buf, size_t bytes_per_launch, int32_t launches, float* ms_total, void* stream) {
  if (!buf || !ms_total || launches < 1 || bytes_per_launch < 1024 || bytes_per_launch % 1024)
    return fail(nullptr, DFLASH_EINVAL, "probe_hbm_read: need a buffer, launches >= 1 and a multiple of 1024 bytes per launch");
  hipStream_t st = (hipStream_t)stream;
  return timed(st, ms_total, [&] {
    for (int i = 0; i < launches; ++i)
      hipLaunchKernelGGL(probe_read_kernel, dim3(256), dim3(256), 0, st,
                         reinterpret_cast<const u32x4*>(static_cast<const char*>(buf) + (size_t)i * bytes_per_launch), bytes_per_launch / 1024);
  });
}

int dflash_probe_mfma(int32_t shape, int32_t workgroups, int32_t iters, float* ms, double* flops, void* stream) {
  if (!ms || !flops || workgroups < 1 || workgroups > 65536 || iters < 1 || shape < 0 || shape > 1)
    return fail(nullptr, DFLASH_EINVAL, "probe_mfma: need outputs, shape 0 or 1, 1..65536 workgroups and iters >= 1");
  hipStream_t st = (hipStream_t)stream;
  const int rc = timed(st, ms, [&] {
    if (shape == 0) hipLaunchKernelGGL(probe_mfma_kernel, dim3(workgroups), dim3(256), 0, st, iters);
    else hipLaunchKernelGGL(probe_mfma32_kernel, dim3(workgroups), dim3(256), 0, st, iters);
  });
  *flops = (double)workgroups * 4 * iters * (shape == 0 ? 16 * (2.0 * 16 * 16 * 32) : 4 * (2.0 * 32 * 32 * 16));
  return rc;
}

const char* dflash_last_error(const dflash_ctx* ctx) { return ctx ? ctx->err : g_err; }

int dflash_device_status(dflash_ctx* ctx, void* stream) {
  if (!ctx) return fail(nullptr, DFLASH_EINVAL, "ctx: null");
  int32_t v = 0;
  if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return CTX_FAIL(ctx, DFLASH_EHIP, "stream synchronise failed");
  if (hipMemcpy(&v, ctx->wsp + ctx->ws.status, 4, hipMemcpyDeviceToHost) != hipSuccess) return CTX_FAIL(ctx, DFLASH_EHIP, "status read failed");
  if (v) {
    if (hipMemset(ctx->wsp + ctx->ws.status, 0, 4) != hipSuccess) return CTX_FAIL(ctx, DFLASH_EHIP, "status clear failed");
    return CTX_FAIL(ctx, DFLASH_ECAPACITY, "device: a row addressed a page outside the block table / pool, a token id was outside the vocabulary, or a sequence was longer than the batch's max_seq_len");
  }
  return DFLASH_OK;
}

int dflash_moe_stats(dflash_ctx* ctx, void* stream, int64_t* out) {
  if (!ctx || !out) return fail(ctx ? ctx->err : nullptr, DFLASH_EINVAL, "moe_stats: null argument");
  if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return CTX_FAIL(ctx, DFLASH_EHIP, "stream synchronise failed");
  if (hipMemcpy(out, ctx->wsp + ctx->ws.status + 64, 40, hipMemcpyDeviceToHost) != hipSuccess) return CTX_FAIL(ctx, DFLASH_EHIP, "statistics read failed");
  if (hipMemset(ctx->wsp + ctx->ws.status + 64, 0, 40) != hipSuccess) return CTX_FAIL(ctx, DFLASH_EHIP, "statistics clear failed");
  return DFLASH_OK;
}

int dflash_gemm_counts(dflash_ctx* ctx, int64_t* out) {
  if (!ctx || !out) return fail(ctx ? ctx->err : nullptr, DFLASH_EINVAL, "gemm_counts: null argument");
  for (int i = 0; i < DFLASH_GEMM_KINDS; ++i) {
    out[i] = ctx->gemm_counts[i];
    ctx->gemm_counts[i] = 0;
  }
  return DFLASH_OK;
}

int dflash_moe_trace(dflash_ctx* ctx, int32_t* choices) {
  if (!ctx) return fail(nullptr, DFLASH_EINVAL, "ctx: null");
  if (choices && !ctx->t.n_experts) return CTX_FAIL(ctx, DFLASH_EINVAL, "moe_trace: the target has no routed experts");
  ctx->moe_trace = choices;
  return DFLASH_OK;
}

#define DISPATCH(ctx, call)                                                        \
  ((ctx)->t.dtype == DFLASH_BF16 ? Engine<bf16_t>{(ctx), (hipStream_t)stream}.call \
                                 : Engine<float>{(ctx), (hipStream_t)stream}.call)

int dflash_draft_block(dflash_ctx* ctx, const dflash_batch* batch, float temperature, const uint64_t* rng_key, int32_t* draft_tokens,
                       float* logits_out, void* stream) {
  int rc;
  if ((rc = check_batch(ctx, batch))) return rc;
  if (batch->n_seqs == 0) return DFLASH_OK;
  if (!draft_tokens) return CTX_FAIL(ctx, DFLASH_EINVAL, "draft_block: draft_tokens is null");
  if (!(temperature >= 0.f)) return CTX_FAIL(ctx, DFLASH_EINVAL, "draft_block: negative temperature");
  if (temperature > 0.f && !rng_key) return CTX_FAIL(ctx, DFLASH_EINVAL, "draft_block: sampling needs rng_key");
  return DISPATCH(ctx, draft_block(batch, temperature, rng_key, draft_tokens, logits_out));
}

int dflash_verify(dflash_ctx* ctx, const dflash_batch* batch, const int32_t* tokens, int32_t* tgt_argmax, float* logits_out, void* stream) {
  int rc;
  if ((rc = check_batch(ctx, batch))) return rc;
  if (batch->n_seqs == 0) return DFLASH_OK;
  if (!tokens) return CTX_FAIL(ctx, DFLASH_EINVAL, "verify: null tokens");
  return DISPATCH(ctx, verify(batch, tokens, tgt_argmax, logits_out));
}

int dflash_accept(dflash_ctx* ctx, const dflash_batch* batch, const int32_t* draft_tokens, const int32_t* tgt_argmax, float temperature,
                  const float* uniforms, const uint64_t* rng_key, int32_t* accept_len, int32_t* out_tokens, void* stream) {
  int rc;
  if ((rc = check_batch(ctx, batch))) return rc;
  if (batch->n_seqs == 0) return DFLASH_OK;
  if (!draft_tokens || !tgt_argmax || !accept_len || !out_tokens) return CTX_FAIL(ctx, DFLASH_EINVAL, "accept: null pointer");
  if (!(temperature >= 0.f)) return CTX_FAIL(ctx, DFLASH_EINVAL, "accept: negative temperature");
  if (temperature > 0.f && (!uniforms || !rng_key)) return CTX_FAIL(ctx, DFLASH_EINVAL, "accept: sampling needs uniforms and rng_key");
  if (temperature > 0.f && !(ctx->have_logits_d && ctx->have_logits_t))
    return CTX_FAIL(ctx, DFLASH_EINVAL, "accept: sampling needs the logits of this step: run dflash_draft_block with temperature > 0 and then dflash_verify first");
  return DISPATCH(ctx, accept(batch, draft_tokens, tgt_argmax, temperature, uniforms, rng_key, accept_len, out_tokens));
}

int dflash_kv_commit(dflash_ctx* ctx, const dflash_batch* batch, const int32_t* accept_len, const int32_t* out_tokens, int64_t* kv_slots_out,
                     void* stream) {
  int rc;
  if ((rc = check_batch(ctx, batch))) return rc;
  if (batch->n_seqs == 0) return DFLASH_OK;
  if (!accept_len || !out_tokens) return CTX_FAIL(ctx, DFLASH_EINVAL, "kv_commit: null pointer");
  return DISPATCH(ctx, commit(batch, accept_len, out_tokens, kv_slots_out));
}

int dflash_prefill(dflash_ctx* ctx, const dflash_batch* batch, const int32_t* tokens, const int32_t* prompt_lens, int32_t* first_tokens,
                   void* stream) {
  int rc;
  if ((rc = check_batch(ctx, batch))) return rc;
  if (batch->n_seqs == 0) return DFLASH_OK;
  if (!prompt_lens) return CTX_FAIL(ctx, DFLASH_EINVAL, "prefill: null prompt_lens");
  const int B = batch->block_size > 0 ? batch->block_size : ctx->rt.block_size;
  int longest = 0;
  for (int s = 0; s < batch->n_seqs; ++s) {
    if (prompt_lens[s] < 0) return CTX_FAIL(ctx, DFLASH_EINVAL, "prefill: negative prompt length");
    longest = std::max(longest, prompt_lens[s]);
  }
  if (longest == 0) return DFLASH_OK;   // no sequence has new tokens
  if (!tokens) return CTX_FAIL(ctx, DFLASH_EINVAL, "prefill: null tokens");
  // the last chunk of a prompt is padded to a whole block of rows, whose K/V rows are written too (invisible)
  if ((int64_t)batch->max_seq_len + (longest + B - 1) / B * B > (int64_t)ctx->rt.max_pages_per_seq * DFLASH_PAGE_SIZE)
    return CTX_FAIL(ctx, DFLASH_ECAPACITY, "prefill: max_seq_len %d + the longest prompt (%d, padded to whole blocks of %d) exceeds the %d tokens a block-table row covers",
                    batch->max_seq_len, longest, B, ctx->rt.max_pages_per_seq * DFLASH_PAGE_SIZE);
  return DISPATCH(ctx, prefill(batch, tokens, prompt_lens, first_tokens));
}

// address of `scratch` on the current device, looked up once per device
static int noalloc_scratch(void** out) {
  static std::mutex mu;
  static void* ptrs[64] = {nullptr};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return fail(nullptr, DFLASH_EHIP, "accept_sampled_noalloc: cannot tell the current device");
  std::lock_guard<std::mutex> lock(mu);
  if (!ptrs[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(nullptr, DFLASH_EHIP, "accept_sampled_noalloc: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
    ptrs[dev] = p;
  }
  *out = ptrs[dev];
  return DFLASH_OK;
}

int dflash_accept_sampled_noalloc(const float* target_logits, const float* draft_logits, const int32_t* draft_tokens, const float* uniforms,
                                  const uint64_t* rng_key, float temperature, int32_t n_seqs, int32_t block_size, int32_t vocab,
                                  int32_t* accept_len, int32_t* out_tokens, void* stream) {
  if (n_seqs == 0) return DFLASH_OK;
  if (!target_logits || !draft_logits || !draft_tokens || !uniforms || !rng_key || !accept_len || !out_tokens)
    return fail(nullptr, DFLASH_EINVAL, "accept_sampled_noalloc: null pointer");
  if (!(temperature > 0.f)) return fail(nullptr, DFLASH_EINVAL, "accept_sampled_noalloc: temperature must be positive (greedy acceptance needs no scratch: dflash_accept)");
  if (n_seqs < 0 || block_size < 2 || block_size > DFLASH_MAX_BLOCK || vocab < 1)
    return fail(nullptr, DFLASH_EINVAL, "accept_sampled_noalloc: need n_seqs >= 0, block_size in [2,%d], vocab >= 1", DFLASH_MAX_BLOCK);
  if ((int64_t)n_seqs * block_size > DFLASH_NOALLOC_MAX_ROWS)
    return fail(nullptr, DFLASH_ECAPACITY, "accept_sampled_noalloc: %lld rows exceed the %d rows of the built-in scratch array",
                (long long)n_seqs * block_size, DFLASH_NOALLOC_MAX_ROWS);
  void* base = nullptr;
  int rc;
  if ((rc = noalloc_scratch(&base))) return rc;
  float2* stats_p = reinterpret_cast<float2*>(base);
  float2* stats_q = stats_p + DFLASH_NOALLOC_MAX_ROWS;
  hipStream_t st = (hipStream_t)stream;
  const int M = n_seqs * block_size;
  const float inv_T = 1.0f / temperature;
  hipLaunchKernelGGL(row_lse_kernel, dim3(M), dim3(1024), 0, st, target_logits, vocab, inv_T, stats_p);
  hipLaunchKernelGGL(row_lse_kernel, dim3(M), dim3(1024), 0, st, draft_logits, vocab, inv_T, stats_q);
  hipLaunchKernelGGL(accept_sampling_kernel, dim3(n_seqs), dim3(1024), 0, st, target_logits, draft_logits, stats_p, stats_q, draft_tokens, uniforms,
                     rng_key, vocab, block_size, inv_T, accept_len, out_tokens);
  if (hipGetLastError() != hipSuccess) return fail(nullptr, DFLASH_EHIP, "accept_sampled_noalloc: launch failed");
  return DFLASH_OK;
}

static int kv_copy_checked(dflash_ctx* ctx, const dflash_batch* batch, int32_t pool, int32_t layer, int32_t seq, int32_t start, int32_t count,
                           float* k, float* v, int dir, void* stream) {
  int rc;
  if ((rc = check_batch(ctx, batch))) return rc;
  if (pool != DFLASH_POOL_TARGET && pool != DFLASH_POOL_DRAFT) return CTX_FAIL(ctx, DFLASH_EINVAL, "kv copy: bad pool");
  const dflash_dims& m = pool == DFLASH_POOL_TARGET ? ctx->t : ctx->d;
  if (layer < 0 || layer >= m.n_layers || seq < 0 || seq >= batch->n_seqs || start < 0 || count < 0 || (count > 0 && (!k || !v)))
    return CTX_FAIL(ctx, DFLASH_EINVAL, "kv copy: bad layer, seq, range or pointer");
  if ((int64_t)start + count > (int64_t)ctx->rt.max_pages_per_seq * DFLASH_PAGE_SIZE) return CTX_FAIL(ctx, DFLASH_ECAPACITY, "kv copy: range beyond the block table");
  if (count == 0) return DFLASH_OK;
  return ctx->t.dtype == DFLASH_BF16 ? run_kv_copy<bf16_t>(ctx, batch, pool, layer, seq, start, count, k, v, dir, (hipStream_t)stream)
                                     : run_kv_copy<float>(ctx, batch, pool, layer, seq, start, count, k, v, dir, (hipStream_t)stream);
}

int dflash_kv_read(dflash_ctx* ctx, const dflash_batch* batch, int32_t pool, int32_t layer, int32_t seq, int32_t start, int32_t count,
                   float* k, float* v, void* stream) {
  return kv_copy_checked(ctx, batch, pool, layer, seq, start, count, k, v, 0, stream);
}
int dflash_kv_write(dflash_ctx* ctx, const dflash_batch* batch, int32_t pool, int32_t layer, int32_t seq, int32_t start, int32_t count,
                    const float* k, const float* v, void* stream) {
  return kv_copy_checked(ctx, batch, pool, layer, seq, start, count, const_cast<float*>(k), const_cast<float*>(v), 1, stream);
}

}  // extern "C"
