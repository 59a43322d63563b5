"""TEST INFRASTRUCTURE ONLY -- plain CPU oracle (numpy, float64) for one DFlash speculative
decoding step: block-diffusion draft forward, causal verification by the target, acceptance,
KV commit / rollback.  It shares no code with the HIP path and the product never imports it.

What each function follows (arxiv 2602.06036):
  * speculative cycle, tau in [1, gamma+1] with the bonus token ........ Section 3.1, Eq. 1
  * one parallel pass drafts the whole block ............................. Section 3.2, Eq. 3; Section 4.1
  * block = clean anchor (previous bonus token) + block_size-1 masks ..... Section 4.2 ("Random sampling of masked blocks")
  * bidirectional attention inside the block and to the context features . Section 4.2 (sparse-mask paragraph), Fig. 2
  * tap layers, fusion H_t = RMSNorm(W_c [H^(l1);...]) .................... Section 5 ("Implementation"), Appendix A.3
  * K_i = [W_K H_t ; W_K H_d], V_i likewise, Q_i = W_Q H_d ................ Appendix A.3
  * shared (frozen) embedding and LM head ................................ Section 4.2
  * losslessness of the verified output .................................. Abstract, Section 1
The target is a standard pre-norm decoder (RMSNorm, RoPE, GQA, SwiGLU) of the Qwen3 / LLaMA
family the paper evaluates (Section 5).  The Qwen3-Coder-30B-A3B target named there is a
mixture-of-experts model; the paper gives no routing rule, so `_ffn` follows that public model
family's: top-k router logits, weights = softmax over the chosen logits, weighted sum of the
chosen SwiGLU experts.  The temperature-1 rule is the standard speculative
sampling rule of the cited Leviathan et al. work, which the paper uses without restating.

Precision: float64 throughout.  `rnd` is the storage-rounding hook (class Rounding): the identity
for an fp32 model.  A bf16 model keeps its weights, its K/V cache rows and the query rows in bf16
(`rnd.kv`, 8 significand bits) and hands every GEMM input -- normalised activations, attention
output, SwiGLU product, taps, H_t -- to the matrix units as a pair of bf16 numbers hi + lo
(`rnd(x)`, about 16 significand bits).  Residual stream, accumulators, softmax and logits stay wide.
The pair format is this build's choice, not the paper's: with single-bf16 GEMM inputs two correct
bf16 evaluations of the same model (differing only in summation order) end up 2-3 % of the logit
standard deviation apart, because one flipped rounding perturbs all later roundings; that is
above the 2e-2 logit bound at the 8B shape.  tests/test_oracle_model.py measures both variants.

Loop order.  `target_forward_tokens` walks layer by layer and, inside a layer, token by token
with a growing KV list (token j attends the list as it stands after its own K/V were appended).
That is the token-by-token decoder with the two loops interchanged, which changes no operand of
any operation; tests check it against one-token-at-a-time calls and against the masked matrix form.

Pins (tests/test_oracle_*.py): RoPE vs complex rotation and shift invariance; RMSNorm scale
invariance; layer with empty cache vs torch CPU scaled_dot_product_attention; sequence (matrix)
form vs token loop; draft with no context vs non-causal SDPA; joint softmax vs log-sum-exp merge;
context-permutation invariance; W_c only reaches K/V; losslessness of greedy speculative decoding
vs plain greedy decoding; routed experts vs the dense FFN (identical experts), the full softmax
mixture (top_k = all), expert relabelling and a hand-routed case; greedy acceptance vs brute force; speculative sampling vs exact
enumeration and chi-square; Appendix A.3 memory figures.
Parity unpinned: draft tokens / accept lengths produced by a random-weight drafter have no
independent definition beyond these steps; they are pinned only through the component pins above.
"""
from __future__ import annotations

import math
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np



# --------------------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------------------
def _same(x: np.ndarray) -> np.ndarray:
    return x


class Rounding:
    """rnd(x): rounding of a GEMM input; rnd.kv(x): rounding of stored q / k / v rows.
    rnd.at(site) is the rounding of the GEMM input at one of the sites "norm" (output of any RMSNorm of the
    residual stream), "attn_out" (attention output, input of W_o), "ffn_act" (SwiGLU product, input of W_d),
    "taps" and "fused" (inputs of W_c and of the context W_K / W_V): `sites` overrides `act` per site, which is
    how the tests measure what each site's precision is worth; the models used for parity override nothing."""

    def __init__(self, act: Callable[[np.ndarray], np.ndarray], kv: Callable[[np.ndarray], np.ndarray],
                 sites: Optional[Dict[str, Callable[[np.ndarray], np.ndarray]]] = None):
        self.act, self.kv, self.sites = act, kv, dict(sites or {})

    def __call__(self, x: np.ndarray) -> np.ndarray:
        return self.act(x)

    def at(self, site: str) -> Callable[[np.ndarray], np.ndarray]:
        return self.sites.get(site, self.act)


identity = Rounding(_same, _same)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest-even rounding of an fp32 value to 8 significand bits, returned as float64."""
    f = np.ascontiguousarray(np.asarray(x, dtype=np.float64).astype(np.float32))
    u = f.view(np.uint32)
    u = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return u.view(np.float32).astype(np.float64)


def round_bf16_pair(x: np.ndarray) -> np.ndarray:
    """hi + lo with hi = bf16(x), lo = bf16(x - hi), the subtraction done in single precision."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    hi = round_bf16(f).astype(np.float32)
    lo = round_bf16((f - hi).astype(np.float32))
    return hi.astype(np.float64) + lo


BF16_MODEL = Rounding(round_bf16_pair, round_bf16)
BF16_SINGLE = Rounding(round_bf16, round_bf16)     # single-bf16 GEMM inputs; used only to measure the noise


def rounding_for(dtype: str) -> Rounding:
    return BF16_MODEL if dtype == "bf16" else identity


# --------------------------------------------------------------------------------------
# elementary operations
# --------------------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """x * g / sqrt(mean(x^2) + eps) over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing: dims (i, i+hd/2) rotate by pos * theta^(-2i/hd).
    x: [T, H, hd]; pos: [T]."""
    hd = x.shape[-1]
    half = hd // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]       # [T, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def softmax(s: np.ndarray) -> np.ndarray:
    e = np.exp(s - np.max(s, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


class KVList:
    """Per-layer growing K/V lists of one sequence: K[l][:n] is [n, Hkv, hd]."""

    def __init__(self, n_layers: int, n_kv_heads: int, head_dim: int, capacity: int,
                 dtype=np.float64):
        self.k = [np.zeros((capacity, n_kv_heads, head_dim), dtype) for _ in range(n_layers)]
        self.v = [np.zeros((capacity, n_kv_heads, head_dim), dtype) for _ in range(n_layers)]
        self.n = 0                      # rows valid in every layer

    def truncate(self, n: int) -> None:
        self.n = n


def _heads(x: np.ndarray, n_heads: int, hd: int) -> np.ndarray:
    return x.reshape(x.shape[0], n_heads, hd)


def _qkv(W, m, pre: str, a: np.ndarray, pos: np.ndarray, rnd: "Rounding"):
    """Projections of normalised rows a [T, D] -> q [T,Hq,hd], k, v [T,Hkv,hd]; optional per-head
    RMSNorm on q and k, then RoPE at `pos`; each stored with the q/k/v rounding."""
    q = _heads(a @ W(pre + "wq").T, m.n_q_heads, m.head_dim)
    k = _heads(a @ W(pre + "wk").T, m.n_kv_heads, m.head_dim)
    v = _heads(a @ W(pre + "wv").T, m.n_kv_heads, m.head_dim)
    if m.qk_norm:
        q = rmsnorm(q, W(pre + "qn"), m.rms_eps)
        k = rmsnorm(k, W(pre + "kn"), m.rms_eps)
    q = rope(q, pos, m.rope_theta)
    k = rope(k, pos, m.rope_theta)
    return rnd.kv(q), rnd.kv(k), rnd.kv(v)


def _attend(m, q: np.ndarray, K: np.ndarray, V: np.ndarray) -> np.ndarray:
    """One query row set q [Hq, hd] over keys K, values V [n, Hkv, hd] (all visible);
    query head i reads kv head i // (Hq/Hkv)."""
    group = m.n_q_heads // m.n_kv_heads
    scale = 1.0 / math.sqrt(m.head_dim)
    out = np.empty((m.n_q_heads, m.head_dim))
    for h in range(m.n_q_heads):
        kv = h // group
        p = softmax((K[:, kv, :] @ q[h]) * scale)
        out[h] = p @ V[:, kv, :]
    return out


ROUTE_MARGINS: Optional[List[float]] = None   # a test may set this to a list: every routing decision then appends
                                              # the gap between the last chosen and the best rejected router logit
ROUTE_CHOICES: Optional[List[List[int]]] = None   # likewise: the chosen experts of every routing decision, ascending


def moe_route(logits: np.ndarray, top_k: int):
    """Routing of one token (the public Qwen3-MoE rule; the paper names the model, Section 5, but not the rule): the
    top_k experts by router logit (ties -> lowest index), weighted by the softmax over those top_k logits (the
    softmax over all experts renormalised over the chosen ones is the same thing).  Returns (indices in order of
    decreasing logit, weights)."""
    idx = np.argsort(-logits, kind="stable")[:top_k]
    return idx, softmax(logits[idx])


def _ffn(W, m, pre: str, h: np.ndarray, rnd: "Rounding") -> np.ndarray:
    a = rnd.at("norm")(rmsnorm(h, W(pre + "g2"), m.rms_eps))
    if getattr(m, "n_experts", 0):
        # routed experts: y_t = sum over the token's top_k experts e of w_e * W_d^e (silu(W_g^e a_t) * (W_u^e a_t))
        Wr, Wg, Wu, Wd = W(pre + "wr"), W(pre + "wg"), W(pre + "wu"), W(pre + "wd")
        router = a @ Wr.T
        out = np.zeros_like(h)
        for t in range(h.shape[0]):
            idx, wts = moe_route(router[t], m.top_k)
            if ROUTE_MARGINS is not None and m.top_k < m.n_experts:
                ROUTE_MARGINS.append(float(router[t, idx[-1]] - np.delete(router[t], idx).max()))
            if ROUTE_CHOICES is not None:
                ROUTE_CHOICES.append(sorted(int(e) for e in idx))
            for e, wt in zip(idx, wts):
                act = rnd.at("ffn_act")(silu(Wg[e] @ a[t]) * (Wu[e] @ a[t]))
                out[t] += wt * (Wd[e] @ act)
        return h + out
    act = rnd.at("ffn_act")(silu(a @ W(pre + "wg").T) * (a @ W(pre + "wu").T))
    return h + act @ W(pre + "wd").T


# --------------------------------------------------------------------------------------
# target model
# --------------------------------------------------------------------------------------
def target_forward_tokens(W, m, tokens: Sequence[int], start_pos: int, kv: KVList,
                          tap_layers: Sequence[int], rnd: "Rounding" = identity,
                          want_logits: bool = True):
    """Run `tokens` (positions start_pos ..) through the target against the cached rows
    kv[:start_pos]; appends their K/V (kv.n becomes start_pos+T).  Token j sees cache rows
    0..start_pos+j.  Returns (logits [T, V] or None, taps [T, n_tap, D])."""
    T = len(tokens)
    assert kv.n == start_pos
    pos = np.arange(start_pos, start_pos + T)
    h = W("E")[np.asarray(tokens, dtype=np.int64)].copy()                        # [T, D]
    taps = np.zeros((T, len(tap_layers), m.d_model))
    for l in range(m.n_layers):
        pre = f"L{l}."
        a = rnd.at("norm")(rmsnorm(h, W(pre + "g1"), m.rms_eps))
        q, k, v = _qkv(W, m, pre, a, pos, rnd)
        o = np.empty((T, m.n_q_heads, m.head_dim))
        for j in range(T):                       # token by token, list grows
            kv.k[l][start_pos + j] = k[j]
            kv.v[l][start_pos + j] = v[j]
            n_vis = start_pos + j + 1
            o[j] = _attend(m, q[j], kv.k[l][:n_vis].astype(np.float64, copy=False),
                           kv.v[l][:n_vis].astype(np.float64, copy=False))
        h = h + rnd.at("attn_out")(o.reshape(T, -1)) @ W(pre + "wo").T
        h = _ffn(W, m, pre, h, rnd)
        for t, tl in enumerate(tap_layers):
            if tl == l:
                taps[:, t, :] = h
    kv.n = start_pos + T
    logits = None
    if want_logits:
        logits = rnd.at("norm")(rmsnorm(h, W("gf"), m.rms_eps)) @ W("lm").T
    return logits, taps


def target_forward_sequence(W, m, tokens: Sequence[int], kv: KVList, tap_layers: Sequence[int],
                            rnd: "Rounding" = identity, logit_rows: Optional[Sequence[int]] = None):
    """Whole-sequence causal forward from an empty cache in matrix form (masked T x T scores):
    the textbook definition of the decoder over a sequence.  Fills kv[0:T].  Returns
    (logits for `logit_rows` (default: all rows), taps [T, n_tap, D])."""
    T = len(tokens)
    assert kv.n == 0
    pos = np.arange(T)
    group = m.n_q_heads // m.n_kv_heads
    scale = 1.0 / math.sqrt(m.head_dim)
    mask = np.triu(np.full((T, T), -np.inf), k=1)
    h = W("E")[np.asarray(tokens, dtype=np.int64)].copy()
    taps = np.zeros((T, len(tap_layers), m.d_model))
    for l in range(m.n_layers):
        pre = f"L{l}."
        a = rnd.at("norm")(rmsnorm(h, W(pre + "g1"), m.rms_eps))
        q, k, v = _qkv(W, m, pre, a, pos, rnd)
        kv.k[l][:T] = k
        kv.v[l][:T] = v
        o = np.empty((T, m.n_q_heads, m.head_dim))
        for hq in range(m.n_q_heads):
            g = hq // group
            p = softmax(q[:, hq, :] @ k[:, g, :].T * scale + mask)
            o[:, hq, :] = p @ v[:, g, :]
        h = h + rnd.at("attn_out")(o.reshape(T, -1)) @ W(pre + "wo").T
        h = _ffn(W, m, pre, h, rnd)
        for t, tl in enumerate(tap_layers):
            if tl == l:
                taps[:, t, :] = h
    kv.n = T
    rows = np.arange(T) if logit_rows is None else np.asarray(logit_rows)
    logits = rnd.at("norm")(rmsnorm(h[rows], W("gf"), m.rms_eps)) @ W("lm").T
    return logits, taps


# --------------------------------------------------------------------------------------
# draft model (Appendix A.3)
# --------------------------------------------------------------------------------------
def fuse_taps(Wd, md, taps: np.ndarray, rnd: "Rounding" = identity) -> np.ndarray:
    """H_t = RMSNorm(W_c [H^(l1); ...; H^(lk)]) per token; taps [T, n_tap, D_target] are
    concatenated in ascending layer order.  Returns [T, D_draft]."""
    x = rnd.at("taps")(taps).reshape(taps.shape[0], -1)
    return rnd.at("fused")(rmsnorm(x @ Wd("wc").T, Wd("gc"), md.rms_eps))


def draft_context_kv(Wd, md, H_t: np.ndarray, pos: np.ndarray, rnd: "Rounding" = identity):
    """Per draft layer i: K = W_K^i H_t (per-head k-norm if enabled, RoPE at the token's own
    position), V = W_V^i H_t.  The features get no per-layer input norm and never pass through
    Q / O / FFN.  Returns [(K [T,Hkv,hd], V [T,Hkv,hd])] per layer."""
    out = []
    for i in range(md.n_layers):
        pre = f"L{i}."
        k = _heads(H_t @ Wd(pre + "wk").T, md.n_kv_heads, md.head_dim)
        v = _heads(H_t @ Wd(pre + "wv").T, md.n_kv_heads, md.head_dim)
        if md.qk_norm:
            k = rmsnorm(k, Wd(pre + "kn"), md.rms_eps)
        k = rope(k, pos, md.rope_theta)
        out.append((rnd.kv(k), rnd.kv(v)))
    return out


def draft_block_forward(Wd, md, anchor: int, n: int, ctx: KVList, block_size: int, mask_id: int,
                        rnd: "Rounding" = identity) -> np.ndarray:
    """One pass over the block [anchor, mask, ..., mask] placed at positions n .. n+B-1.
    Every block row attends, without any mask, to all n cached context rows of its layer and to
    all B block rows.  Returns logits [B, V]; row j is the prediction for the token of slot j
    (row 0, the anchor's, is not used by the step)."""
    B = block_size
    assert ctx.n == n
    tokens = np.array([anchor] + [mask_id] * (B - 1), dtype=np.int64)
    pos = np.arange(n, n + B)
    h = Wd("E")[tokens].copy()
    for i in range(md.n_layers):
        pre = f"L{i}."
        a = rnd.at("norm")(rmsnorm(h, Wd(pre + "g1"), md.rms_eps))
        q, k, v = _qkv(Wd, md, pre, a, pos, rnd)
        K = np.concatenate([ctx.k[i][:n].astype(np.float64, copy=False), k], axis=0)
        V = np.concatenate([ctx.v[i][:n].astype(np.float64, copy=False), v], axis=0)
        o = np.stack([_attend(md, q[j], K, V) for j in range(B)])
        h = h + rnd.at("attn_out")(o.reshape(B, -1)) @ Wd(pre + "wo").T
        h = _ffn(Wd, md, pre, h, rnd)
    return rnd.at("norm")(rmsnorm(h, Wd("gf"), md.rms_eps)) @ Wd("lm").T


# --------------------------------------------------------------------------------------
# acceptance
# --------------------------------------------------------------------------------------
def greedy_accept(block: Sequence[int], tgt_argmax: Sequence[int]) -> int:
    """block = [anchor, d_1 .. d_{B-1}]; tgt_argmax[j] = target's greedy token after block[j].
    Returns a = number of leading drafts with d_j == tgt_argmax[j-1]."""
    a = 0
    while a + 1 < len(block) and block[a + 1] == tgt_argmax[a]:
        a += 1
    return a


def sampling_accept(p_rows: np.ndarray, q_rows: np.ndarray, block: Sequence[int],
                    u: Sequence[float], draw: Callable[[np.ndarray, int, int], int]):
    """Speculative-sampling acceptance for one sequence.
    p_rows[j] = target distribution after block[j] (j = 0..B-1); q_rows[j] = draft distribution
    slot j was drawn from (j = 1..B-1; row 0 unused); u[j] = uniform for slot j.
    Slot j is accepted iff u[j] * q_j(d_j) < p_{j-1}(d_j).  At the first rejected slot j the
    replacement is drawn from normalise(max(p_{j-1} - q_j, 0)); if none is rejected the bonus token
    is drawn from p_{B-1}.  draw(weights, slot, purpose) returns an index (purpose 1 = residual,
    2 = bonus).  Returns (a, final_token)."""
    B = len(block)
    for j in range(1, B):
        d = block[j]
        if not (u[j] * q_rows[j][d] < p_rows[j - 1][d]):
            resid = np.maximum(p_rows[j - 1] - q_rows[j], 0.0)
            return j - 1, draw(resid, j, 1)
    return B - 1, draw(p_rows[B - 1], B, 2)


# --------------------------------------------------------------------------------------
# counter-based random numbers (specified in prose; the HIP kernels implement it separately)
# --------------------------------------------------------------------------------------
_M64 = (1 << 64) - 1
PURPOSE_DRAFT, PURPOSE_RESIDUAL, PURPOSE_BONUS = 0, 1, 2


def _mix64(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def counter_uniform(key: int, seq: int, slot: int, purpose: int, idx: np.ndarray) -> np.ndarray:
    """u in (0,1) with 23 random bits: counter c = (((seq*64 + slot)*4 + purpose) << 32) | idx,
    z = mix64(key + 0x9E3779B97F4A7C15 * (c + 1)) (mod 2^64), u = ((z >> 41) + 0.5) / 2^23
    (23 bits keep x + 0.5 exact in single precision as well)."""
    with np.errstate(over="ignore"):
        hi = np.uint64((((seq * 64 + slot) * 4 + purpose) << 32) & _M64)
        c = hi | np.asarray(idx, dtype=np.uint64)
        z = _mix64(np.uint64(key & _M64) + np.uint64(0x9E3779B97F4A7C15) * (c + np.uint64(1)))
    return ((z >> np.uint64(41)).astype(np.float64) + 0.5) * 2.0 ** -23


def gumbel_scores(logw: np.ndarray, key: int, seq: int, slot: int, purpose: int) -> np.ndarray:
    """log-weight + Gumbel noise; argmax of this is a draw from normalise(exp(logw))."""
    u = counter_uniform(key, seq, slot, purpose, np.arange(logw.shape[-1]))
    return logw - np.log(-np.log(u))


def top2_margin(scores: np.ndarray) -> float:
    if scores.shape[-1] < 2:
        return math.inf
    part = np.partition(scores[np.isfinite(scores)], -2)
    return float(part[-1] - part[-2]) if part.size >= 2 else math.inf


# --------------------------------------------------------------------------------------
# one sequence's decoding state and the speculative step
# --------------------------------------------------------------------------------------
class SeqState:
    def __init__(self, mt, md, capacity: int, cache_dtype=np.float64):
        self.kv = KVList(mt.n_layers, mt.n_kv_heads, mt.head_dim, capacity, cache_dtype)
        self.ctx = KVList(md.n_layers, md.n_kv_heads, md.head_dim, capacity, cache_dtype)
        self.n = 0
        self.anchor = -1


def _append_context(Wd, md, st: SeqState, taps: np.ndarray, start: int, rnd: "Rounding") -> None:
    H_t = fuse_taps(Wd, md, taps, rnd)
    pos = np.arange(start, start + taps.shape[0])
    for i, (k, v) in enumerate(draft_context_kv(Wd, md, H_t, pos, rnd)):
        st.ctx.k[i][start:start + len(pos)] = k
        st.ctx.v[i][start:start + len(pos)] = v
    st.ctx.n = start + taps.shape[0]


def prefill_with_logits(Wt, Wd, mt, md, tap_layers, prompt: Sequence[int], st: SeqState,
                        rnd: "Rounding" = identity) -> Tuple[int, np.ndarray]:
    """Standard prefill (Section 4.1): target over the prompt, taps of every prompt token fused
    and projected into the draft's context K/V; the first generated token becomes the anchor.
    Returns (that token, the logits row it is the argmax of)."""
    T = len(prompt)
    logits, taps = target_forward_sequence(Wt, mt, prompt, st.kv, tap_layers, rnd, logit_rows=[T - 1])
    _append_context(Wd, md, st, taps, 0, rnd)
    st.n = T
    st.anchor = int(np.argmax(logits[0]))
    return st.anchor, logits[0]


def prefill(Wt, Wd, mt, md, tap_layers, prompt: Sequence[int], st: SeqState,
            rnd: "Rounding" = identity) -> int:
    """prefill_with_logits without the logits."""
    return prefill_with_logits(Wt, Wd, mt, md, tap_layers, prompt, st, rnd)[0]


def spec_step(Wt, Wd, mt, md, tap_layers, st: SeqState, block_size: int, mask_id: int,
              rnd: "Rounding" = identity, temperature: float = 0.0,
              uniforms: Optional[Sequence[float]] = None, key: int = 0, seq_id: int = 0,
              proposal: Optional[Sequence[int]] = None) -> Dict:
    """One draft -> verify -> accept -> commit cycle for one sequence.
    `proposal` (tests only) replaces the drafted tokens d_1..d_{B-1}."""
    B, n = block_size, st.n
    greedy = temperature == 0.0
    draft_logits = draft_block_forward(Wd, md, st.anchor, n, st.ctx, B, mask_id, rnd)
    draft_scores = None
    if greedy:
        d = [int(np.argmax(draft_logits[j])) for j in range(1, B)]
        draft_scores = draft_logits
    else:
        draft_scores = np.stack([gumbel_scores(draft_logits[j] / temperature, key, seq_id, j,
                                               PURPOSE_DRAFT) for j in range(B)])
        d = [int(np.argmax(draft_scores[j])) for j in range(1, B)]
    if proposal is not None:
        d = [int(x) for x in proposal]
    block = [int(st.anchor)] + d
    # verification: B single-token forwards in sequence (speculative KV rows appended)
    logits, taps = target_forward_tokens(Wt, mt, block, n, st.kv, tap_layers, rnd)
    tgt_argmax = [int(np.argmax(logits[j])) for j in range(B)]
    final_scores = None
    if greedy:
        a = greedy_accept(block, tgt_argmax)
        final = tgt_argmax[a]
    else:
        p = softmax(logits / temperature)
        q = softmax(draft_logits / temperature)
        rec = {}

        def draw(wts, slot, purpose):
            with np.errstate(divide="ignore"):
                s = gumbel_scores(np.log(wts), key, seq_id, slot, purpose)
            rec["scores"] = s
            return int(np.argmax(s))

        a, final = sampling_accept(p, q, block, uniforms, draw)
        final_scores = rec["scores"]
    emitted = d[:a] + [final]
    # commit: rows n..n+a keep their target KV, the rest is rolled back
    st.kv.truncate(n + a + 1)
    _append_context(Wd, md, st, taps[: a + 1], n, rnd)
    st.n = n + a + 1
    st.anchor = final
    return dict(block=block, draft_logits=draft_logits, draft_scores=draft_scores, logits=logits,
                tgt_argmax=tgt_argmax, accept_len=a, emitted=emitted, final_scores=final_scores,
                taps=taps)


def plain_greedy_decode(Wt, mt, prompt: Sequence[int], n_new: int, rnd: "Rounding" = identity,
                        capacity: Optional[int] = None) -> List[int]:
    """Token-by-token greedy decoding of the target alone: the definition the speculative
    output must reproduce."""
    cap = capacity or (len(prompt) + n_new + 1)
    kv = KVList(mt.n_layers, mt.n_kv_heads, mt.head_dim, cap)
    logits = None
    for i, t in enumerate(prompt):
        logits, _ = target_forward_tokens(Wt, mt, [int(t)], i, kv, (), rnd,
                                          want_logits=(i == len(prompt) - 1))
    out = []
    for i in range(n_new):
        tok = int(np.argmax(logits[0]))
        out.append(tok)
        if i + 1 < n_new:
            logits, _ = target_forward_tokens(Wt, mt, [tok], len(prompt) + i, kv, (), rnd)
    return out


def fusion_memory_bytes(d_model: int, n_taps: int, seq_len: int, block_size: int,
                        bytes_per_el: int = 2) -> Dict[str, int]:
    """Sizes quoted in Appendix A.3: W_c, projection input/output for a prefill of seq_len
    tokens, and the temporary activation (input + output) while decoding one block."""
    return dict(
        w_c=n_taps * d_model * d_model * bytes_per_el,
        proj_in=seq_len * n_taps * d_model * bytes_per_el,
        proj_out=seq_len * d_model * bytes_per_el,
        decode_tmp=block_size * (n_taps + 1) * d_model * bytes_per_el,
    )
