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
