"""Pins for the oracle's target and draft forwards: library routines (torch CPU float64),
special cases, and invariances that the method's definition implies."""
from dataclasses import replace

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import dflash_oracle as O
from synth import inputs as si
from tests.helpers import W64, tiny_workload


# ---- an independent reference built from torch library routines -------------------------
def _t(x):
    return torch.from_numpy(np.asarray(x, dtype=np.float64))


def _rope_complex(x, pos, theta):
    # x [T, H, hd] -> complex rotation of (x_i, x_{i+hd/2})
    hd = x.shape[-1]
    z = torch.complex(x[..., : hd // 2], x[..., hd // 2:])
    freq = theta ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    rot = torch.polar(torch.ones(len(pos), hd // 2, dtype=torch.float64), _t(pos)[:, None] * freq[None])
    z = z * rot[:, None, :]
    return torch.cat([z.real, z.imag], -1)


def torch_layer(W, m, pre, h, pos, causal, extra_kv=None):
    """One decoder layer on rows h [T, D] that attend to each other (causal or not) and,
    when given, to extra K/V rows (all visible), using SDPA."""
    T = h.shape[0]
    a = F.rms_norm(h, (m.d_model,), _t(W(pre + "g1")), m.rms_eps)
    q = F.linear(a, _t(W(pre + "wq"))).view(T, m.n_q_heads, m.head_dim)
    k = F.linear(a, _t(W(pre + "wk"))).view(T, m.n_kv_heads, m.head_dim)
    v = F.linear(a, _t(W(pre + "wv"))).view(T, m.n_kv_heads, m.head_dim)
    if m.qk_norm:
        q = F.rms_norm(q, (m.head_dim,), _t(W(pre + "qn")), m.rms_eps)
        k = F.rms_norm(k, (m.head_dim,), _t(W(pre + "kn")), m.rms_eps)
    q, k = _rope_complex(q, pos, m.rope_theta), _rope_complex(k, pos, m.rope_theta)
    mask = None
    if extra_kv is not None:
        ek, ev = extra_kv
        n = ek.shape[0]
        k = torch.cat([_t(ek), k], 0)
        v = torch.cat([_t(ev), v], 0)
        mask = torch.ones(T, n + T, dtype=torch.bool)
        if causal:
            mask[:, n:] = torch.tril(torch.ones(T, T, dtype=torch.bool))
        o = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], k.permute(1, 0, 2)[None],
                                           v.permute(1, 0, 2)[None], attn_mask=mask, enable_gqa=True)
    else:
        o = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], k.permute(1, 0, 2)[None],
                                           v.permute(1, 0, 2)[None], is_causal=causal, enable_gqa=True)
    o = o[0].permute(1, 0, 2).reshape(T, -1)
    h = h + F.linear(o, _t(W(pre + "wo")))
    a2 = F.rms_norm(h, (m.d_model,), _t(W(pre + "g2")), m.rms_eps)
    h = h + F.linear(F.silu(F.linear(a2, _t(W(pre + "wg")))) * F.linear(a2, _t(W(pre + "wu"))),
                     _t(W(pre + "wd")))
    return h


def torch_target(W, m, tokens):
    h = _t(W("E"))[torch.as_tensor(np.asarray(tokens, dtype=np.int64))]
    pos = np.arange(len(tokens))
    hs = []
    for l in range(m.n_layers):
        h = torch_layer(W, m, f"L{l}.", h, pos, causal=True)
        hs.append(h)
    logits = F.linear(F.rms_norm(h, (m.d_model,), _t(W("gf")), m.rms_eps), _t(W("lm")))
    return logits.numpy(), [x.numpy() for x in hs]


CASES = [dict(qk_norm=False, kv_heads=4), dict(qk_norm=True, kv_heads=2)]


@pytest.mark.parametrize("case", CASES)
def test_target_sequence_form_matches_torch_library(case):
    w = tiny_workload(seed=3, n_layers=3, vocab=200, taps=(0, 2), **case)
    wt, _ = si.make_weights(w, 1)
    W = W64(wt)
    toks = si.make_prompts(replace(w, ctx_min=23, ctx_max=23))[0]
    kv = O.KVList(3, w.target.n_kv_heads, 64, 64)
    logits, taps = O.target_forward_sequence(W, w.target, toks, kv, w.tap_layers)
    ref_logits, ref_h = torch_target(W, w.target, toks)
    assert np.allclose(logits, ref_logits, atol=1e-10)
    assert np.allclose(taps[:, 0], ref_h[0], atol=1e-10)        # tap = residual stream after the layer
    assert np.allclose(taps[:, 1], ref_h[2], atol=1e-10)


@pytest.mark.parametrize("case", CASES)
def test_token_loop_equals_sequence_form_and_single_token_calls(case):
    w = tiny_workload(seed=4, n_layers=2, vocab=300, taps=(1,), **case)
    wt, _ = si.make_weights(w, 1)
    W = W64(wt)
    toks = si.make_prompts(replace(w, ctx_min=19, ctx_max=19))[0]
    m = w.target
    kv_a = O.KVList(2, m.n_kv_heads, 64, 32)
    la, ta = O.target_forward_sequence(W, m, toks, kv_a, w.tap_layers)
    # (i) prefix through the cache, then a block of 8 tokens in one call
    kv_b = O.KVList(2, m.n_kv_heads, 64, 32)
    lb0, tb0 = O.target_forward_tokens(W, m, toks[:11], 0, kv_b, w.tap_layers)
    lb1, tb1 = O.target_forward_tokens(W, m, toks[11:], 11, kv_b, w.tap_layers)
    assert np.allclose(np.concatenate([lb0, lb1]), la, atol=1e-11)
    assert np.allclose(np.concatenate([tb0, tb1]), ta, atol=1e-11)
    for l in range(2):
        assert np.allclose(kv_a.k[l][:19], kv_b.k[l][:19], atol=1e-12)
        assert np.allclose(kv_a.v[l][:19], kv_b.v[l][:19], atol=1e-12)
    # (ii) strictly one token per call: the plain autoregressive decoder
    kv_c = O.KVList(2, m.n_kv_heads, 64, 32)
    rows = [O.target_forward_tokens(W, m, [int(t)], i, kv_c, w.tap_layers)[0][0] for i, t in enumerate(toks)]
    assert np.allclose(np.stack(rows), la, atol=1e-11)
    assert np.allclose(np.stack(rows[11:]), lb1, atol=1e-12)


def _draft_setup(seed, n_ctx, case, draft_layers=2, B=6):
    w = tiny_workload(seed=seed, n_layers=3, draft_layers=draft_layers, vocab=256, block=B,
                      taps=(0, 1), **case)
    wt, wd = si.make_weights(w, 1)
    Wt, Wd = W64(wt), W64(wd)
    st = O.SeqState(w.target, w.draft, 64)
    toks = si.make_prompts(replace(w, ctx_min=max(n_ctx, 1), ctx_max=max(n_ctx, 1)))[0]
    if n_ctx > 0:
        O.prefill(Wt, Wd, w.target, w.draft, w.tap_layers, toks, st)
    else:
        st.anchor = int(toks[0])
    return w, Wt, Wd, st


@pytest.mark.parametrize("case", CASES)
def test_draft_without_context_is_a_plain_bidirectional_transformer(case):
    w, Wt, Wd, st = _draft_setup(5, 0, case)
    md, B = w.draft, w.block_size
    got = O.draft_block_forward(Wd, md, st.anchor, 0, st.ctx, B, w.mask_token_id)
    toks = np.array([st.anchor] + [w.mask_token_id] * (B - 1))
    h = _t(Wd("E"))[torch.as_tensor(toks)]
    for i in range(md.n_layers):
        h = torch_layer(Wd, md, f"L{i}.", h, np.arange(B), causal=False)
    ref = F.linear(F.rms_norm(h, (md.d_model,), _t(Wd("gf")), md.rms_eps), _t(Wd("lm"))).numpy()
    assert np.allclose(got, ref, atol=1e-10)


@pytest.mark.parametrize("case", CASES)
def test_draft_with_context_matches_library_attention_over_concatenated_kv(case):
    """K = [W_K H_t ; W_K H_d] (Appendix A.3): the context rows enter as extra, fully visible
    K/V rows of every layer; the fused feature itself is checked against F.linear + rms_norm."""
    w, Wt, Wd, st = _draft_setup(6, 13, case)
    md, mt, B, n = w.draft, w.target, w.block_size, st.n
    got = O.draft_block_forward(Wd, md, st.anchor, n, st.ctx, B, w.mask_token_id)
    # rebuild the context K/V independently from the torch target's hidden states
    toks = si.make_prompts(replace(w, ctx_min=13, ctx_max=13))[0]
    _, hs = torch_target(Wt, mt, toks)
    cat = torch.cat([_t(hs[l]) for l in w.tap_layers], -1)              # ascending layer order
    H_t = F.rms_norm(F.linear(cat, _t(Wd("wc"))), (md.d_model,), _t(Wd("gc")), md.rms_eps)
    btoks = np.array([st.anchor] + [w.mask_token_id] * (B - 1))
    h = _t(Wd("E"))[torch.as_tensor(btoks)]
    for i in range(md.n_layers):
        pre = f"L{i}."
        ek = F.linear(H_t, _t(Wd(pre + "wk"))).view(n, md.n_kv_heads, md.head_dim)
        ev = F.linear(H_t, _t(Wd(pre + "wv"))).view(n, md.n_kv_heads, md.head_dim)
        if md.qk_norm:
            ek = F.rms_norm(ek, (md.head_dim,), _t(Wd(pre + "kn")), md.rms_eps)
        ek = _rope_complex(ek, np.arange(n), md.rope_theta)
        assert np.allclose(st.ctx.k[i][:n], ek.numpy(), atol=1e-10)
        assert np.allclose(st.ctx.v[i][:n], ev.numpy(), atol=1e-10)
        h = torch_layer(Wd, md, pre, h, np.arange(n, n + B), causal=False,
                        extra_kv=(ek.numpy(), ev.numpy()))
    ref = F.linear(F.rms_norm(h, (md.d_model,), _t(Wd("gf")), md.rms_eps), _t(Wd("lm"))).numpy()
    assert np.allclose(got, ref, atol=1e-10)


def test_joint_softmax_equals_lse_merge_of_context_and_block_parts():
    rng = np.random.default_rng(8)

    class M:
        n_q_heads, n_kv_heads, head_dim = 4, 2, 32
    n, B = 21, 5
    q = rng.standard_normal((4, 32))
    K = rng.standard_normal((n + B, 2, 32))
    V = rng.standard_normal((n + B, 2, 32))
    joint = O._attend(M, q, K, V)
    for h in range(4):
        g = h // 2
        s = torch.from_numpy(K[:, g] @ q[h] / np.sqrt(32))
        parts = []
        for sl in (slice(0, n), slice(n, n + B)):
            lse = torch.logsumexp(s[sl], 0)
            o = torch.softmax(s[sl], 0) @ torch.from_numpy(V[sl, g])
            parts.append((lse, o))
        tot = torch.logsumexp(torch.stack([parts[0][0], parts[1][0]]), 0)
        merged = sum(torch.exp(l - tot) * o for l, o in parts)
        assert np.allclose(joint[h], merged.numpy(), atol=1e-12)


def test_draft_invariant_to_context_slot_order_and_wc_scale():
    case = CASES[1]
    w, Wt, Wd, st = _draft_setup(9, 17, case)
    md, B, n = w.draft, w.block_size, st.n
    base = O.draft_block_forward(Wd, md, st.anchor, n, st.ctx, B, w.mask_token_id)
    # (a) context rows carry their position inside K (RoPE applied before caching): storing them
    # in another order changes nothing
    perm = np.random.default_rng(0).permutation(n)
    ctx2 = O.KVList(md.n_layers, md.n_kv_heads, md.head_dim, 64)
    for i in range(md.n_layers):
        ctx2.k[i][:n] = st.ctx.k[i][:n][perm]
        ctx2.v[i][:n] = st.ctx.v[i][:n][perm]
    ctx2.n = n
    assert np.allclose(O.draft_block_forward(Wd, md, st.anchor, n, ctx2, B, w.mask_token_id), base, atol=1e-11)
    # (b) the fused feature is normalised: scaling W_c leaves H_t, hence the draft, unchanged
    taps = np.random.default_rng(1).standard_normal((4, 2, w.target.d_model))
    h1 = O.fuse_taps(Wd, md, taps)
    Wd2 = lambda name: (3.0 * Wd(name) if name == "wc" else Wd(name))
    md0 = replace(md, rms_eps=0.0)
    assert np.allclose(O.fuse_taps(Wd2, md0, taps), O.fuse_taps(Wd, md0, taps), atol=1e-12)
    assert h1.shape == (4, md.d_model)
    # (c) the context only ever enters through K/V: dropping every context row of V and K
    # (n = 0) must equal the plain bidirectional block
    ctx0 = O.KVList(md.n_layers, md.n_kv_heads, md.head_dim, 8)
    d0 = O.draft_block_forward(Wd, md, st.anchor, 0, ctx0, B, w.mask_token_id)
    assert not np.allclose(d0, base, atol=1e-6)


def test_block_rows_see_each_other_bidirectionally():
    """Changing the LAST slot's input must change the FIRST mask slot's output (no causal mask
    in the draft), whereas in the target an earlier row never sees a later one."""
    w, Wt, Wd, st = _draft_setup(10, 9, CASES[0], draft_layers=1)
    md, B, n = w.draft, w.block_size, st.n
    base = O.draft_block_forward(Wd, md, st.anchor, n, st.ctx, B, w.mask_token_id)

    def Wd_alt(name):               # perturb only the mask embedding -> rows 1..B-1 change input
        a = Wd(name)
        if name == "E":
            a = a.copy()
            a[w.mask_token_id] += 0.05
        return a
    alt = O.draft_block_forward(Wd_alt, md, st.anchor, n, st.ctx, B, w.mask_token_id)
    assert np.abs(alt[0] - base[0]).max() > 1e-6        # anchor row sees the masks after it
    kv1 = O.KVList(3, w.target.n_kv_heads, 64, 64)
    kv2 = O.KVList(3, w.target.n_kv_heads, 64, 64)
    a1, _ = O.target_forward_tokens(Wt, w.target, [5, 6, 7, 8], 0, kv1, ())
    a2, _ = O.target_forward_tokens(Wt, w.target, [5, 6, 7, 9], 0, kv2, ())
    assert np.array_equal(a1[:3], a2[:3]) and not np.allclose(a1[3], a2[3])


# ---- routed-expert target (the mixture-of-experts target named in Section 5) -----------------------------------
def _moe_case(seed, E, k, T=9, d=64, fe=48):
    m = si.ModelDims(1, d, 2, 2, 32, 4 * d, 50, 1e4, 1e-6, False, E, k, fe)
    r = np.random.default_rng(seed)
    t = {"L0.g2": 1.0 + 0.1 * r.uniform(-1, 1, d), "L0.wr": r.standard_normal((E, d)),
         "L0.wg": r.standard_normal((E, fe, d)) / 8, "L0.wu": r.standard_normal((E, fe, d)) / 8,
         "L0.wd": r.standard_normal((E, d, fe)) / 8}
    return m, t, r.standard_normal((T, d))


def _dense_ffn_torch(h, g2, wg, wu, wd, eps):
    a = F.rms_norm(_t(h), (h.shape[-1],), _t(g2), eps)
    return (_t(h) + F.linear(F.silu(F.linear(a, _t(wg))) * F.linear(a, _t(wu)), _t(wd))).numpy()


def test_route_weights_closed_form_and_tie_rule():
    idx, wts = O.moe_route(np.array([1.0, 3.0, 2.0, 0.0]), 2)
    assert list(idx) == [1, 2]
    assert np.allclose(wts, [1 / (1 + np.exp(-1.0)), 1 / (1 + np.exp(1.0))], atol=1e-15)
    idx, wts = O.moe_route(np.array([0.5, 2.0, 2.0, 2.0]), 2)          # ties go to the lower index
    assert list(idx) == [1, 2] and np.allclose(wts, [0.5, 0.5])
    # the full softmax renormalised over the chosen experts is the same weighting
    lg = np.random.default_rng(0).standard_normal(11)
    idx, wts = O.moe_route(lg, 4)
    p = np.exp(lg) / np.exp(lg).sum()
    assert np.allclose(wts, p[idx] / p[idx].sum(), atol=1e-15) and set(idx) == set(np.argsort(-lg)[:4])


@pytest.mark.parametrize("k", [1, 2, 5])
def test_identical_experts_reduce_to_the_dense_ffn(k):
    m, t, h = _moe_case(1, 5, k)
    for key in ("wg", "wu", "wd"):
        t["L0." + key][:] = t["L0." + key][0]
    got = O._ffn(lambda n: t[n], m, "L0.", h, O.identity)
    ref = _dense_ffn_torch(h, t["L0.g2"], t["L0.wg"][0], t["L0.wu"][0], t["L0.wd"][0], m.rms_eps)
    assert np.allclose(got, ref, atol=1e-11)


def test_all_experts_chosen_is_the_full_softmax_mixture():
    m, t, h = _moe_case(2, 6, 6)
    got = O._ffn(lambda n: t[n], m, "L0.", h, O.identity)
    a = F.rms_norm(_t(h), (h.shape[-1],), _t(t["L0.g2"]), m.rms_eps)
    p = torch.softmax(F.linear(a, _t(t["L0.wr"])), -1)                                   # [T, E]
    act = F.silu(torch.einsum("efd,td->tef", _t(t["L0.wg"]), a)) * torch.einsum("efd,td->tef", _t(t["L0.wu"]), a)
    ref = _t(h) + torch.einsum("te,edf,tef->td", p, _t(t["L0.wd"]), act)
    assert np.allclose(got, ref.numpy(), atol=1e-11)


def test_hand_routed_tokens_get_exactly_their_expert():
    """Router rows are scaled unit vectors and token t is (a multiple of) router row t mod E before the norm gain is
    undone, so with top_k = 1 token t must come out of expert t mod E alone, with weight 1."""
    m, t, h = _moe_case(3, 4, 1, T=8)
    t["L0.g2"][:] = 1.0
    q, _ = np.linalg.qr(np.random.default_rng(5).standard_normal((m.d_model, m.d_model)))
    t["L0.wr"] = 3.0 * q[:4]
    h = np.stack([(1.0 + 0.3 * i) * q[i % 4] for i in range(8)])
    got = O._ffn(lambda n: t[n], m, "L0.", h, O.identity)
    for i in range(8):
        e = i % 4
        ref = _dense_ffn_torch(h[i:i + 1], t["L0.g2"], t["L0.wg"][e], t["L0.wu"][e], t["L0.wd"][e], m.rms_eps)
        assert np.allclose(got[i], ref[0], atol=1e-11)


def test_relabelling_the_experts_changes_nothing_and_margins_are_reported():
    m, t, h = _moe_case(4, 7, 3)
    O.ROUTE_MARGINS = []
    try:
        a = O._ffn(lambda n: t[n], m, "L0.", h, O.identity)
        margins = list(O.ROUTE_MARGINS)
    finally:
        O.ROUTE_MARGINS = None
    assert len(margins) == h.shape[0] and min(margins) > 0
    perm = np.random.default_rng(9).permutation(7)
    t2 = {k: (v[perm] if k != "L0.g2" else v) for k, v in t.items()}
    assert np.allclose(O._ffn(lambda n: t2[n], m, "L0.", h, O.identity), a, atol=1e-12)
    # dropping the chosen experts' weighting (plain sum) or the renormalisation is visible
    t3 = dict(t)
    t3["L0.wr"] = t["L0.wr"] * 0.0                                       # flat router: first k experts, weights 1/k
    flat = O._ffn(lambda n: t3[n], m, "L0.", h, O.identity)
    mean3 = np.mean([_dense_ffn_torch(h, t["L0.g2"], t["L0.wg"][e], t["L0.wu"][e], t["L0.wd"][e], m.rms_eps) - h
                     for e in range(3)], axis=0)
    assert np.allclose(flat - h, mean3, atol=1e-11)


def test_moe_target_sequence_form_equals_token_loop():
    w = si.small_moe_workload(n_experts=6, top_k=2, d_expert=64)
    w = replace(w, dtype="f32", target=replace(w.target, n_layers=2, d_model=128, n_q_heads=2, n_kv_heads=1, head_dim=64,
                                               vocab=300), mask_token_id=299)
    w = replace(w, draft=replace(w.draft, d_model=128, n_q_heads=2, n_kv_heads=1, head_dim=64, vocab=300, d_ffn=256))
    wt, _ = si.make_weights(w, 1)
    W = W64(wt)
    toks = si.make_prompts(replace(w, ctx_min=13, ctx_max=13))[0]
    m = w.target
    kv_a, kv_b = O.KVList(2, 1, 64, 16), O.KVList(2, 1, 64, 16)
    la, ta = O.target_forward_sequence(W, m, toks, kv_a, w.tap_layers)
    lb0, _ = O.target_forward_tokens(W, m, toks[:5], 0, kv_b, w.tap_layers)
    lb1, _ = O.target_forward_tokens(W, m, toks[5:], 5, kv_b, w.tap_layers)
    assert np.allclose(np.concatenate([lb0, lb1]), la, atol=1e-11)


def test_routed_stack_is_discontinuous_at_router_ties_and_a_dense_stack_is_not():
    """Why routed-expert parity tests look at router gaps: perturb every embedding row by a relative 1e-4 (the size of
    the bf16 storage noise between two correct evaluations).  A dense 24-layer stack answers with a uniformly small
    change of the logits.  The routed stack of the same size answers the same way on every row -- except the one whose
    smallest router gap (1.5e-5) is below the perturbation of its router logits: that row takes another expert and
    ends up an order of magnitude further away.  The oracle's ROUTE_MARGINS find that row in advance."""
    T, n_layers, eps = 48, 24, 1e-4

    def logits_pair(t):
        w = si.Workload("deep", "f32", t, replace(t, n_layers=1, n_experts=0, top_k=0, d_expert=0), (0,), 511, 16, 1, T, T, 0.0, 0)
        wt, _ = si.make_weights(w, 4)
        W = W64(wt)
        toks = si.make_prompts(w)[0]
        O.ROUTE_MARGINS = []
        try:
            la, _ = O.target_forward_sequence(W, t, toks, O.KVList(n_layers, 1, 64, T), ())
            gaps = np.array(O.ROUTE_MARGINS).reshape(n_layers, T).min(0) if t.n_experts else None
        finally:
            O.ROUTE_MARGINS = None
        E0 = W("E")
        E1 = E0 * (1.0 + eps * np.random.default_rng(1).standard_normal(E0.shape))
        lb, _ = O.target_forward_sequence(lambda n: E1 if n == "E" else W(n), t, toks, O.KVList(n_layers, 1, 64, T), ())
        return np.abs(la - lb).max(1) / la.std(), gaps

    dense, _ = logits_pair(si.ModelDims(n_layers, 128, 2, 1, 64, 256, 512, 1e4, 1e-6, True))
    assert dense.max() < 2 * np.median(dense) < 40 * eps
    moe, gaps = logits_pair(si.ModelDims(n_layers, 128, 2, 1, 64, 256, 512, 1e4, 1e-6, True, 32, 4, 64))
    worst = int(np.argmax(moe))
    assert worst == int(np.argmin(gaps)) and gaps[worst] < eps
    assert moe[worst] > 10 * np.median(moe)
    assert moe[gaps > 2e-3].max() < 4 * np.median(moe) < 40 * eps


def test_tap_layers_follow_the_paper():
    assert si.tap_layers_for(36, 5) == (1, 9, 17, 25, 33)      # second layer .. third-to-last
    assert si.workload(1).tap_layers == (0,)


def test_bf16_pair_inputs_keep_two_evaluations_within_the_logit_bound():
    """Why GEMM inputs are bf16 pairs: evaluate the same bf16 model twice, the second time with the
    embedding scaled by (1 + 1e-5) (far below bf16 resolution, standing in for a different summation
    order).  With single-bf16 GEMM inputs the two logit sets differ by percents of the logit standard
    deviation; with hi+lo pairs by hundredths of a percent (what is left comes from the bf16 q/k/v rows)."""
    t = si.ModelDims(6, 256, 4, 1, 64, 768, 2048, 1e6, 1e-6, True)
    w = si.Workload("noise", "bf16", t, replace(t, n_layers=1), (1,), t.vocab - 1, 16, 1, 48, 48, 0.0, 7)
    wt, _ = si.make_weights(w, 4)
    W = W64(wt)
    toks = si.make_prompts(w)[0]

    def run(rnd, scale):
        Wp = lambda name: (W(name) * scale if name == "E" else W(name))
        kv = O.KVList(t.n_layers, t.n_kv_heads, t.head_dim, 64)
        return O.target_forward_sequence(Wp, t, toks, kv, (), rnd)[0]
    exact = run(O.identity, 1.0)
    sigma = exact.std()
    single = np.abs(run(O.BF16_SINGLE, 1.0) - run(O.BF16_SINGLE, 1.0 + 1e-5)).max() / sigma
    pair = np.abs(run(O.BF16_MODEL, 1.0) - run(O.BF16_MODEL, 1.0 + 1e-5)).max() / sigma
    assert single > 0.008          # > 1e-2 in logit units at the 8B shape's sigma of 1.28
    assert pair < 0.004


def test_every_gemm_input_site_is_worth_its_lo_plane():
    """Per-site measurement behind keeping hi+lo pairs at EVERY GEMM input (oracle only).  A 36-layer model (the depth of
    the 8B shape) is evaluated twice per rounding model, the second time with the embedding scaled by (1 + 1e-5), which
    stands in for another summation order; the rms distance of the two logit sets, in percent of the logit spread, is the
    noise floor any other correct evaluation (the GPU's) lands at.  With pairs everywhere that floor comes from the bf16
    q/k/v rows alone; one bf16 number at the attention output (input of W_o) or at the SwiGLU product (input of W_d)
    alone triples it, at the normalised activations it grows sevenfold.  In logit units at the 8B spread of 1.28 the
    maxima over a few thousand logits are then 1.2e-2 to 3e-2 against the 2e-2 bound, so no site can give up its lo plane."""
    t = si.ModelDims(36, 256, 4, 1, 64, 768, 2048, 1e6, 1e-6, True)
    w = si.Workload("noise", "bf16", t, replace(t, n_layers=1), (1,), t.vocab - 1, 16, 1, 48, 48, 0.0, 7)
    wt, _ = si.make_weights(w, 4)
    W = W64(wt)
    toks = si.make_prompts(w)[0]

    def run(rnd, scale):
        Wp = lambda name: (W(name) * scale if name == "E" else W(name))
        kv = O.KVList(t.n_layers, t.n_kv_heads, t.head_dim, 64)
        return O.target_forward_sequence(Wp, t, toks, kv, (), rnd)[0]
    sigma = run(O.identity, 1.0).std()
    one, pair = O.round_bf16, O.round_bf16_pair

    def noise(sites):
        rnd = O.Rounding(pair, one, sites)
        d = run(rnd, 1.0) - run(rnd, 1.0 + 1e-5)
        return 100 * np.sqrt((d ** 2).mean()) / sigma, 100 * np.abs(d).max() / sigma
    base_rms, base_max = noise({})
    rows = {"attn_out": noise({"attn_out": one}), "ffn_act": noise({"ffn_act": one}), "norm": noise({"norm": one}),
            "attn_out+ffn_act": noise({"attn_out": one, "ffn_act": one})}
    print(f"two evaluations, rms / max in % of the logit spread: pairs everywhere {base_rms:.3f} / {base_max:.3f}; "
          + "; ".join(f"one bf16 number at {k} {v[0]:.3f} / {v[1]:.3f}" for k, v in rows.items()))
    assert base_max < 0.7
    for k, (rms, mx) in rows.items():
        assert rms > 2.0 * base_rms, k
    assert rows["attn_out+ffn_act"][1] * 1.28 / 100 > 1.2e-2      # in logit units at the 8B spread: no margin left under 2e-2
