"""Pins for the oracle's speculative step: losslessness against plain greedy decoding
(Abstract / Section 1), the range of tau (Section 3.1), greedy acceptance against brute force,
and the temperature-1 rule against exact enumeration and a chi-square test."""
import itertools
import os
from dataclasses import replace

import numpy as np
import pytest
from scipy import stats

from oracle import dflash_oracle as O
from synth import inputs as si
from tests.helpers import W64, tiny_workload


def _run_spec(w, Wt, Wd, prompt, n_steps, rnd=O.identity, proposals=None):
    st = O.SeqState(w.target, w.draft, len(prompt) + (n_steps + 1) * w.block_size + 1)
    first = O.prefill(Wt, Wd, w.target, w.draft, w.tap_layers, prompt, st, rnd)
    out, accepts = [first], []
    for s in range(n_steps):
        prop = proposals(s, st) if proposals else None
        r = O.spec_step(Wt, Wd, w.target, w.draft, w.tap_layers, st, w.block_size, w.mask_token_id,
                        rnd, proposal=prop)
        assert 1 <= r["accept_len"] + 1 <= w.block_size           # tau in [1, gamma+1]
        assert len(r["emitted"]) == r["accept_len"] + 1
        assert st.n == len(prompt) + len(out) - 1 + len(r["emitted"])
        assert st.kv.n == st.n and st.ctx.n == st.n
        out += r["emitted"]
        accepts.append(r["accept_len"])
    return out, accepts, st


def test_config1_greedy_speculation_is_lossless():
    """Config 1 (fp32 tiny model, prompt 128, B=8, 20 steps): the speculative output equals
    token-by-token greedy decoding of the target, whatever the (random) drafter proposes."""
    w = si.workload(1)
    wt, wd = si.make_weights(w, 4)
    Wt, Wd = W64(wt), W64(wd)
    prompt = si.make_prompts(w)[0]
    out, accepts, _ = _run_spec(w, Wt, Wd, prompt, w.n_steps)
    ref = O.plain_greedy_decode(Wt, w.target, prompt, len(out))
    assert out == ref
    assert len(out) >= 1 + w.n_steps


@pytest.mark.parametrize("dtype,qk_norm,kv_heads", [("f32", False, 4), ("bf16", True, 2)])
def test_lossless_with_long_accepts_and_rollback(dtype, qk_norm, kv_heads):
    """Proposals built from the true continuation (k correct tokens, then a wrong one) force every
    accept length 0..B-1, so commit and rollback of KV rows and context features are exercised;
    the emitted sequence must still be the plain greedy one and the state must equal a fresh
    prefill of the emitted text."""
    w = tiny_workload(seed=21, n_layers=2, draft_layers=1, vocab=512, block=6, qk_norm=qk_norm,
                      kv_heads=kv_heads, dtype=dtype, taps=(0, 1), d=128, heads=4, hd=32, ffn=256)
    wt, wd = si.make_weights(w, 1)
    Wt, Wd = W64(wt), W64(wd)
    rnd = O.rounding_for(dtype)
    prompt = si.make_prompts(replace(w, ctx_min=12, ctx_max=12))[0]
    ref = O.plain_greedy_decode(Wt, w.target, prompt, 80, rnd)
    plan = [0, 5, 3, 1, 5, 2, 4, 0, 5]
    emitted_so_far = [1]

    def proposals(s, st):
        k = plan[s]
        done = st.n - len(prompt) + 1                 # tokens of ref already emitted (incl. anchor)
        good = ref[done: done + w.block_size - 1]
        prop = list(good)
        if k < w.block_size - 1:
            prop[k] = (prop[k] + 1) % (w.target.vocab - 1)
        return prop
    out, accepts, st = _run_spec(w, Wt, Wd, prompt, len(plan), rnd, proposals)
    assert accepts == plan
    assert out == ref[: len(out)]
    # state after the steps == state of a fresh prefill over prompt + emitted (minus the anchor)
    text = list(prompt) + out[:-1]
    fresh = O.SeqState(w.target, w.draft, len(text) + 1)
    O.prefill(Wt, Wd, w.target, w.draft, w.tap_layers, text, fresh, rnd)
    assert fresh.n == st.n and fresh.anchor == st.anchor
    tol = 1e-9 if dtype == "f32" else 2e-2      # bf16: one-ulp flips of stored rows are allowed
    for l in range(w.target.n_layers):
        assert np.allclose(fresh.kv.k[l][: st.n], st.kv.k[l][: st.n], atol=tol)
        assert np.allclose(fresh.kv.v[l][: st.n], st.kv.v[l][: st.n], atol=tol)
    for l in range(w.draft.n_layers):
        assert np.allclose(fresh.ctx.k[l][: st.n], st.ctx.k[l][: st.n], atol=tol)
        assert np.allclose(fresh.ctx.v[l][: st.n], st.ctx.v[l][: st.n], atol=tol)


def test_greedy_accept_brute_force():
    """Every (draft string, target-argmax string) pair over a 3-letter vocabulary, B <= 5, against
    the definition 'length of the common prefix of d_1.. and t_0..' written with a library routine."""
    for B in range(1, 6):
        for d in itertools.product(range(3), repeat=B - 1):
            for t in itertools.product(range(3), repeat=B):
                a = O.greedy_accept([9] + list(d), list(t))
                common = os.path.commonprefix([list(d), list(t[: B - 1])])
                assert a == len(common)
                assert 0 <= a <= B - 1


def _exact_first_token_distribution(p0, q1, grid=4096):
    """Distribution of the first emitted token when slot 1 is drafted from q1 and verified
    against p0, obtained by running the oracle's acceptance on a fine grid of uniforms and
    capturing the residual weights it asks to draw from."""
    V = len(p0)
    out = np.zeros(V)
    us = (np.arange(grid) + 0.5) / grid
    for d in range(V):
        if q1[d] == 0:
            continue
        for u in us:
            rec = {}

            def draw(wts, slot, purpose):
                rec["w"], rec["purpose"] = np.array(wts, dtype=float), purpose
                return -1
            a, tok = O.sampling_accept(np.stack([p0, p0]), np.stack([q1, q1]), [7, d], [0.0, u], draw)
            if a == 1:
                out[d] += q1[d] / grid
            else:
                assert rec["purpose"] == 1
                out += q1[d] / grid * rec["w"] / rec["w"].sum()
    return out


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_speculative_sampling_reproduces_target_distribution_exactly(seed):
    rng = np.random.default_rng(seed)
    V = 5
    p = rng.dirichlet(np.ones(V))
    q = rng.dirichlet(np.ones(V))
    if seed == 2:
        q[1] = 0.0
        q /= q.sum()                     # a token the drafter can never propose
    got = _exact_first_token_distribution(p, q)
    assert np.allclose(got, p, atol=2.0 / 4096)


def test_sampling_accept_all_accepted_draws_bonus_from_last_row():
    p = np.array([[0.5, 0.5], [0.25, 0.75], [0.9, 0.1]])
    q = np.array([[0.5, 0.5], [0.5, 0.5], [0.5, 0.5]])
    seen = {}

    def draw(wts, slot, purpose):
        seen.update(w=np.array(wts), slot=slot, purpose=purpose)
        return 1
    a, tok = O.sampling_accept(p, q, [0, 0, 1], [0.0, 0.99, 0.99], draw)   # p/q = 1, 1.5 -> accept
    assert (a, tok) == (2, 1) and seen["purpose"] == 2 and seen["slot"] == 3
    assert np.array_equal(seen["w"], p[2])
    a, tok = O.sampling_accept(p, q, [0, 1, 0], [0.0, 0.2, 0.6], draw)     # slot2: p1(0)/q = 0.5 < 0.6
    assert a == 1 and seen["purpose"] == 1 and seen["slot"] == 2
    assert np.allclose(seen["w"], [0.0, 0.25])


def test_temperature1_step_matches_plain_target_sampling_chi_square():
    """Tiny-vocabulary model: the first two tokens emitted by speculative sampling steps are
    distributed as two tokens sampled from the target alone (exact joint by enumeration)."""
    V, B = 8, 4
    w = tiny_workload(seed=33, n_layers=1, draft_layers=1, vocab=V + 1, block=B, d=32, heads=2,
                      kv_heads=2, hd=16, ffn=64, taps=(0,))
    wt, wd = si.make_weights(w, 1)
    # larger logits so the distributions are far from uniform
    wt.t["lm"] = wt.t["lm"] * 40.0
    wd.t["lm"] = wt.t["lm"]
    Wt, Wd = W64(wt), W64(wd)
    prompt = np.array([1, 5, 2, 7, 3], dtype=np.int32)
    st0 = O.SeqState(w.target, w.draft, 32)
    O.prefill(Wt, Wd, w.target, w.draft, w.tap_layers, prompt, st0)
    anchor = st0.anchor

    def clone(st):
        c = O.SeqState(w.target, w.draft, 32)
        for a, b in ((c.kv, st.kv), (c.ctx, st.ctx)):
            for l in range(len(a.k)):
                a.k[l][:] = b.k[l]
                a.v[l][:] = b.v[l]
            a.n = b.n
        c.n, c.anchor = st.n, st.anchor
        return c

    # exact joint of (x1, x2) under the target alone
    def next_dist(prefix):
        kv = O.KVList(1, 2, 16, 32)
        lg, _ = O.target_forward_tokens(Wt, w.target, list(prompt) + prefix, 0, kv, ())
        return O.softmax(lg[-1])
    p1 = next_dist([anchor])
    joint = np.stack([p1[x] * next_dist([anchor, x]) for x in range(V + 1)])
    N = 6000
    rng = np.random.default_rng(0)
    c1 = np.zeros(V + 1)
    c2 = np.zeros((V + 1, V + 1))
    n_pairs = 0
    for it in range(N):
        st = clone(st0)
        toks = []
        for step in range(2):
            u = rng.random(B)
            r = O.spec_step(Wt, Wd, w.target, w.draft, w.tap_layers, st, B, w.mask_token_id,
                            temperature=1.0, uniforms=u, key=10_000 * it + step, seq_id=0)
            toks += r["emitted"]
            if len(toks) >= 2:
                break
        c1[toks[0]] += 1
        c2[toks[0], toks[1]] += 1
    keep = p1 * N >= 5
    assert stats.chisquare(np.append(c1[keep], c1[~keep].sum() + 1e-9),
                           np.append(p1[keep] * N, p1[~keep].sum() * N + 1e-9)).pvalue > 1e-3
    e2 = (joint * N).ravel()
    k2 = e2 >= 5
    assert stats.chisquare(np.append(c2.ravel()[k2], c2.ravel()[~k2].sum() + 1e-9),
                           np.append(e2[k2], e2[~k2].sum() + 1e-9)).pvalue > 1e-3
