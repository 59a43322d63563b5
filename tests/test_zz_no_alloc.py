"""The entry point for callers that cannot allocate (dflash_accept_sampled_noalloc: softmax statistics in an array
built into the library) against dflash_accept on the same logits: two calls in a row, the second with a smaller
input.  Runs last in the suite (file name), alone or after the other tests."""
import numpy as np
import pytest

from synth import inputs as si

pytestmark = pytest.mark.gpu


def test_accept_without_allocation_matches_dflash_accept(monkeypatch):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2602_06036_amd as dfl
    from paper_2602_06036_amd import binding as B
    from tests.gpu_harness import GpuModel
    # the reference takes its softmax statistics from the stored logits, as the new entry point does (the LM-head epilogue
    # sums the same exponentials in another order)
    monkeypatch.setenv("DFLASH_LM_STATS", "2")
    T, key = 0.7, 4242
    for n_seqs, block in ((5, 16), (2, 8)):          # the second call is the smaller one
        w = si.small_bf16_workload(n_seqs=n_seqs, ctx_min=20, ctx_max=90, seed=23 + n_seqs, block_size=block, temperature=T)
        wt, wd = si.make_weights(w, 8)
        g = GpuModel(w, wt, wd, 90 + 4 * block)
        g.prefill(si.make_prompts(w))
        dev = g.dev
        rng = torch.tensor([key], dtype=torch.int64, device=dev)
        for step in range(2):
            u = torch.from_numpy(si.make_uniforms(w, step)).to(dev)
            b = g.batch()
            dfl.dflash_draft_block(g.e, b, g.draft_tokens, T, rng, g.logits_d)
            dfl.dflash_verify(g.e, b, g.draft_tokens, g.tgt_argmax, g.logits_t)
            dfl.dflash_accept(g.e, b, g.draft_tokens, g.tgt_argmax, g.accept_len, g.out_tokens, T, u, rng)
            acc = torch.full_like(g.accept_len, -7)
            out = torch.full_like(g.out_tokens, -7)
            B.dflash_accept_sampled_noalloc(g.logits_t, g.logits_d, g.draft_tokens, u, rng, T, acc, out)
            torch.cuda.synchronize(dev)
            assert np.array_equal(acc.cpu().numpy(), g.accept_len.cpu().numpy()), (n_seqs, block, step)
            assert np.array_equal(out.cpu().numpy(), g.out_tokens.cpu().numpy()), (n_seqs, block, step)
            assert ((acc >= 0) & (acc < block)).all()
            dfl.dflash_kv_commit(g.e, b, g.accept_len, g.out_tokens)
            g.host_lens += g.accept_len.cpu().numpy() + 1
        g.e.close()
    # limits: too many rows, greedy temperature
    big = torch.zeros((257, 16, 8), dtype=torch.float32, device=dev)
    toks = torch.zeros((257, 16), dtype=torch.int32, device=dev)
    uu = torch.zeros((257, 16), dtype=torch.float32, device=dev)
    al = torch.zeros(257, dtype=torch.int32, device=dev)
    with pytest.raises(B.DFlashError) as ei:
        B.dflash_accept_sampled_noalloc(big, big, toks, uu, rng, 1.0, al, toks.clone())
    assert ei.value.code == B.DFLASH_ECAPACITY
    with pytest.raises(B.DFlashError) as ei:
        B.dflash_accept_sampled_noalloc(big[:4], big[:4], toks[:4], uu[:4], rng, 0.0, al[:4], toks[:4].clone())
    assert ei.value.code == B.DFLASH_EINVAL
