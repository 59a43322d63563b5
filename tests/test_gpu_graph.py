"""The whole speculative step (draft -> verify -> accept -> commit) captured once into a HIP graph and replayed:
every call only enqueues kernels and device-to-device copies on the caller's stream, reads nothing back and
allocates nothing, and the per-sequence state (lengths, anchors, caches) lives on the device, so one captured
step replayed N times is N decoding steps.  Each replay is checked bit for bit against the same step run
eagerly from the same state, with eager work and synchronisations between the replays."""
from dataclasses import replace

import numpy as np
import pytest

from synth import inputs as si
from tests.helpers import tiny_workload

pytestmark = pytest.mark.gpu

N_STEPS = 5


def _snapshot(g):
    return dict(target=g.e.target_pool.clone(), draft=g.e.draft_pool.clone(), lens=g.seq_lens.clone(), anchor=g.anchor.clone(),
                host_lens=g.host_lens.copy())


def _restore(g, snap):
    g.e.target_pool.copy_(snap["target"])
    g.e.draft_pool.copy_(snap["draft"])
    g.seq_lens.copy_(snap["lens"])
    g.anchor.copy_(snap["anchor"])
    g.host_lens = snap["host_lens"].copy()


def _outputs(g):
    import torch
    torch.cuda.synchronize(g.dev)
    return dict(draft=g.draft_tokens.cpu().numpy().copy(), tgt=g.tgt_argmax.cpu().numpy().copy(),
                accept=g.accept_len.cpu().numpy().copy(), out=g.out_tokens.cpu().numpy().copy(),
                slots=g.kv_slots.cpu().numpy().copy(), lens=g.seq_lens.cpu().numpy().copy(),
                anchor=g.anchor.cpu().numpy().copy(), logits=g.logits_t.cpu().numpy().copy())


def _enqueue_step(g, batch, temperature, rng, uniforms):
    import paper_2602_06036_amd as dfl
    dfl.dflash_draft_block(g.e, batch, g.draft_tokens, temperature, rng, g.logits_d)
    dfl.dflash_verify(g.e, batch, g.draft_tokens, g.tgt_argmax, g.logits_t)
    dfl.dflash_accept(g.e, batch, g.draft_tokens, g.tgt_argmax, g.accept_len, g.out_tokens, temperature, uniforms, rng)
    dfl.dflash_kv_commit(g.e, batch, g.accept_len, g.out_tokens, g.kv_slots)


def _run(w, prompts, temperature):
    import torch
    from tests.gpu_harness import GpuModel
    wt, wd = si.make_weights(w, 8)
    Bk = w.block_size
    max_len = max(len(p) for p in prompts) + (N_STEPS + 1) * Bk
    g = GpuModel(w, wt, wd, max_len, n_seqs=len(prompts))
    g.prefill(prompts)
    snap = _snapshot(g)
    rng = torch.tensor([77], dtype=torch.int64, device=g.dev) if temperature > 0 else None
    uniforms = torch.from_numpy(si.make_uniforms(replace(w, n_seqs=len(prompts)), 0).astype(np.float32)).to(g.dev) \
        if temperature > 0 else None
    # the launch shapes (attention splits) are planned on the host from an upper bound of the lengths: give the
    # bound that holds for every replayed step
    bound = int(g.host_lens.max()) + N_STEPS * Bk
    batch = g.e.batch(g.seq_lens, g.block_table, g.anchor, bound)

    eager = []
    for _ in range(N_STEPS):
        _enqueue_step(g, batch, temperature, rng, uniforms)
        eager.append(_outputs(g))
    g.e.device_status()

    _restore(g, snap)
    torch.cuda.synchronize(g.dev)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        _enqueue_step(g, batch, temperature, rng, uniforms)      # warm-up on the capture stream, then undo it
    torch.cuda.synchronize(g.dev)
    _restore(g, snap)
    torch.cuda.synchronize(g.dev)
    with torch.cuda.graph(graph, stream=side):
        _enqueue_step(g, batch, temperature, rng, uniforms)
    torch.cuda.synchronize(g.dev)
    _restore(g, snap)                                            # capture does not execute, but be explicit
    for i in range(N_STEPS):
        graph.replay()
        got = _outputs(g)
        for k, v in eager[i].items():
            assert np.array_equal(got[k], v), f"replay {i}: {k} differs from the eager step"
        # eager work between replays: a read through the library and a synchronisation
        g.host_lens = got["lens"].astype(np.int64)
        g.read_kv(0, 0, 0, 0, int(got["lens"][0]))
    g.e.device_status()
    assert (eager[-1]["lens"] > snap["lens"].cpu().numpy()).all()
    g.e.close()


def test_graph_replay_tiny_fp32_greedy():
    w = tiny_workload(seed=5, n_layers=2, draft_layers=1, vocab=512, block=8, n_seqs=2, taps=(0,))
    prompts = [p[:n] for p, n in zip(si.make_prompts(replace(w, ctx_min=40, ctx_max=40)), (40, 27))]
    _run(w, prompts, 0.0)


def test_graph_replay_small_bf16_greedy_and_sampling():
    w = si.small_bf16_workload(n_seqs=3, ctx_min=20, ctx_max=90, seed=13)
    prompts = si.make_prompts(w)
    _run(w, prompts, 0.0)
    _run(replace(w, temperature=1.0), prompts, 1.0)


@pytest.mark.parametrize("fuse", ["1", "2"])
def test_graph_replay_single_band_of_rows(fuse, monkeypatch):
    """Batch 1 at B = 16 (one band of rows: the unsplit projections with the residual update and the deferred RMSNorm) replays
    like every other shape, greedy and sampled."""
    monkeypatch.setenv("DFLASH_FUSE", fuse)
    w = si.small_bf16_workload(n_seqs=1, ctx_min=40, ctx_max=90, seed=17)
    prompts = si.make_prompts(w)
    _run(w, prompts, 0.0)
    _run(replace(w, temperature=1.0), prompts, 1.0)


@pytest.mark.parametrize("n_seqs", [3, 10])
def test_graph_replay_routed_expert_target(n_seqs):
    """The routed-expert step is graph-capturable too: routing, the expert-sorted row list and the work items live on the
    device and are rebuilt by every replay (48 rows: fused routing, rows read through the list; 160 rows: separate
    expert choice, rows copied into list order)."""
    w = si.small_moe_workload(n_seqs=n_seqs, ctx_min=12, ctx_max=40, seed=72, n_experts=16, top_k=4)
    _run(w, si.make_prompts(w), 0.0)


def test_step_without_materialised_logits_gives_the_same_tokens():
    """Greedy steps that ask for no logits (the LM-head GEMMs then only leave their fused per-row argmax partials
    and never write the [S, B, V] logits) choose exactly the tokens of steps that do; a sampling accept after a
    greedy draft is refused because the workspace holds no distributions."""
    import torch
    import paper_2602_06036_amd as dfl
    from paper_2602_06036_amd import binding as B
    from tests.gpu_harness import GpuModel
    for w in (si.small_bf16_workload(n_seqs=3, ctx_min=20, ctx_max=90, seed=19),
              si.small_bf16_workload(n_seqs=9, ctx_min=17, ctx_max=40, seed=29)):     # 48 and 144 rows per step
        prompts = si.make_prompts(w)
        wt, wd = si.make_weights(w, 8)
        g = GpuModel(w, wt, wd, max(len(p) for p in prompts) + 4 * w.block_size, n_seqs=len(prompts))
        g.prefill(prompts)
        snap = _snapshot(g)
        ref = [g.step(want_logits=True) for _ in range(2)]
        _restore(g, snap)
        for r in ref:
            out = g.step(want_logits=False)
            for k in ("drafted", "tgt_argmax", "accept_len", "out_tokens", "kv_slots", "anchor"):
                assert np.array_equal(out[k], r[k]), k
        u = torch.rand((g.S, g.Bk), device=g.dev)
        key = torch.tensor([5], dtype=torch.int64, device=g.dev)
        with pytest.raises(B.DFlashError) as ei:
            dfl.dflash_accept(g.e, g.batch(), g.draft_tokens, g.tgt_argmax, g.accept_len, g.out_tokens, 1.0, u, key)
        assert ei.value.code == B.DFLASH_EINVAL
        g.e.close()


def test_machine_probes_report_plausible_rates():
    """The probe entry points (read-only HBM streaming, register-resident MFMA loop) run and land between a loose
    lower bound and the published peaks of the part."""
    import torch
    from paper_2602_06036_amd import binding as B
    buf = torch.zeros(2 << 30, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    n = 10
    B.dflash_probe_hbm_read(buf, 201326592, n)
    ms = B.dflash_probe_hbm_read(buf, 201326592, n)
    gbps = 201326592 * n / ms / 1e6
    assert 1000 < gbps < 8000, gbps
    for shape in (0, 1):
        B.dflash_probe_mfma(shape, 512, 2000)
        ms, fl = B.dflash_probe_mfma(shape, 512, 20000)
        assert 300 < fl / ms / 1e9 < 2500, (shape, fl / ms / 1e9)
    with pytest.raises(B.DFlashError):
        B.dflash_probe_hbm_read(buf, 1000, 1)
    with pytest.raises(B.DFlashError):
        B.dflash_probe_mfma(2, 512, 10)


@pytest.mark.parametrize("kind", ["small_bf16", "fp32"])
def test_several_steps_in_one_graph_against_the_oracle(kind):
    """The resident decode loop: THREE consecutive speculative steps captured into one HIP graph (lengths, anchors and
    caches stay on the device between them; the proposals that force accept lengths through the range are copied in by
    device-to-device copies inside the graph), replayed once, and every step compared with the CPU oracle's step --
    draft and target logits, drafted tokens, target tokens, accept lengths, emitted tokens, slot ids -- not with an
    eager run of the same kernels.  The oracle runs first: given equal states the two sides evolve identically, so its
    proposals are the ones the captured steps verify."""
    import torch
    import paper_2602_06036_amd as dfl
    from oracle import dflash_oracle as O
    from tests.test_gpu_parity import Lockstep, MARGIN, TOL
    n_steps = 3
    if kind == "fp32":
        w = tiny_workload(seed=25, n_layers=2, draft_layers=1, vocab=512, block=8, n_seqs=2, taps=(0,))
        prompts = [p[:n] for p, n in zip(si.make_prompts(replace(w, ctx_min=40, ctx_max=40)), (40, 27))]
        plans = [[7, 0], [2, 5], [0, 7]]
    else:
        w = si.small_bf16_workload(n_seqs=3, ctx_min=20, ctx_max=90, seed=37)
        prompts = si.make_prompts(w)
        plans = [[15, 0, 9], [3, 15, 1], [0, 6, 15]]
    Bk, S, V = w.block_size, len(prompts), w.target.vocab
    ls = Lockstep(w, prompts, max_len=max(len(p) for p in prompts) + (n_steps + 2) * Bk)
    first, got, mism = ls.prefill()
    assert not mism
    g = ls.g
    dev = g.dev
    # the oracle's three steps (on copies of its states, which the comparison below steps again): proposals per step
    import copy
    states = copy.deepcopy(ls.states)
    proposals = []
    for k in range(n_steps):
        prop = np.stack([ls._true_continuation(st, plans[k][s]) for s, st in enumerate(states)])
        proposals.append(prop)
        for s, st in enumerate(states):
            O.spec_step(ls.Wt, ls.Wd, w.target, w.draft, w.tap_layers, st, Bk, w.mask_token_id, ls.rnd, proposal=prop[s])
    prop_dev = [torch.from_numpy(p.astype(np.int32)).to(dev) for p in proposals]
    outs = [dict(draft=torch.zeros((S, Bk), dtype=torch.int32, device=dev), block=torch.zeros((S, Bk), dtype=torch.int32, device=dev),
                 tgt=torch.zeros((S, Bk), dtype=torch.int32, device=dev), acc=torch.zeros(S, dtype=torch.int32, device=dev),
                 out=torch.zeros((S, Bk), dtype=torch.int32, device=dev), slots=torch.zeros((S, Bk), dtype=torch.int64, device=dev),
                 ld=torch.zeros((S, Bk, V), dtype=torch.float32, device=dev), lt=torch.zeros((S, Bk, V), dtype=torch.float32, device=dev))
            for _ in range(n_steps)]
    bound = int(g.host_lens.max()) + n_steps * Bk
    batch = g.e.batch(g.seq_lens, g.block_table, g.anchor, bound)

    def enqueue():
        for k in range(n_steps):
            o = outs[k]
            dfl.dflash_draft_block(g.e, batch, o["block"], 0.0, None, o["ld"])
            o["draft"].copy_(o["block"])
            o["block"][:, 1:].copy_(prop_dev[k])
            dfl.dflash_verify(g.e, batch, o["block"], o["tgt"], o["lt"])
            dfl.dflash_accept(g.e, batch, o["block"], o["tgt"], o["acc"], o["out"])
            dfl.dflash_kv_commit(g.e, batch, o["acc"], o["out"], o["slots"])

    snap = _snapshot(g)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue()                                               # warm-up on the capture stream, then undo it
    torch.cuda.synchronize(dev)
    _restore(g, snap)
    torch.cuda.synchronize(dev)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        enqueue()
    torch.cuda.synchronize(dev)
    _restore(g, snap)
    for o in outs:
        for t in o.values():
            t.zero_()
    torch.cuda.synchronize(dev)
    graph.replay()
    torch.cuda.synchronize(dev)
    g.e.device_status()
    tol = TOL[w.dtype]
    lens = g.host_lens.copy()
    for k in range(n_steps):
        o = {n: t.cpu().numpy() for n, t in outs[k].items()}
        assert np.array_equal(o["block"][:, 1:], proposals[k])
        for s, st in enumerate(ls.states):
            r = O.spec_step(ls.Wt, ls.Wd, w.target, w.draft, w.tap_layers, st, Bk, w.mask_token_id, ls.rnd, proposal=proposals[k][s])
            assert o["block"][s, 0] == r["block"][0], f"step {k} seq {s}: anchor"
            assert np.abs(o["ld"][s, 1:] - r["draft_logits"][1:]).max() <= tol, f"step {k} seq {s}: draft logits"
            assert np.abs(o["lt"][s] - r["logits"]).max() <= tol, f"step {k} seq {s}: target logits"
            for j in range(1, Bk):
                assert o["draft"][s, j] == int(np.argmax(r["draft_scores"][j])) or O.top2_margin(r["draft_scores"][j]) < MARGIN
            flips = [j for j in range(Bk) if o["tgt"][s, j] != r["tgt_argmax"][j]]
            for j in flips:
                assert O.top2_margin(r["logits"][j]) < MARGIN, f"step {k} seq {s}: target token row {j}"
            a = r["accept_len"]
            if flips:
                pytest.skip("a near-tie of the target's two best logits makes the later captured steps differ from the oracle's (legitimately)")
            assert o["acc"][s] == a == plans[k][s] and list(o["out"][s, : a + 1]) == r["emitted"] and (o["out"][s, a + 1:] == -1).all()
        assert np.array_equal(o["slots"], g.expected_slots(lens, o["acc"]))
        lens = lens + o["acc"] + 1
    assert np.array_equal(g.seq_lens.cpu().numpy(), lens)
    g.host_lens = lens
    ls.check_cache([0, w.target.n_layers - 1], [0])
    g.e.close()
