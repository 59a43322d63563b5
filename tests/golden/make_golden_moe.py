#!/usr/bin/env python3
"""Writes tests/golden/golden_moe_30b.json: the CPU oracle's result of ONE speculative step at the full shape of the
mixture-of-experts target of the paper's Section 5 (Qwen3-Coder-30B-A3B: 48 layers, 128 experts, 8 per token) with its
8-layer drafter, for a sampled sequence of the batch-1 and of the batch-32 bench workloads, from a seeded synthetic
cache state.

Calls only oracle/ and synth/ (never the HIP path).  The model's 57 GB of weights never exist at once: every tensor has
a random stream of its own (synth.inputs.make_tensor), so the oracle's layer-by-layer walk generates a layer's tensors
when it gets there and drops them afterwards.  About a quarter of an hour and 12 GB of RAM per sampled sequence.

The verified block is the oracle's own draft (no constructed continuation: every extra target pass costs the whole
model again).  Stored per sampled sequence: the same fields as golden_8b.json, plus the smallest gaps between a chosen
and the best rejected router logit of the step (a GPU token on such a near-tie may go to another expert).
"""
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import dflash_oracle as O  # noqa: E402
from synth import inputs as si  # noqa: E402

CASES = {"moe_b1": dict(n_seqs=1, seqs=[0]), "moe_b32": dict(n_seqs=32, seqs=[17])}
CTX = 2048
N_COLS = 64


class LazyWeights:
    """name -> float64 tensor, generated on demand; only the tensors of the layer last asked for are kept (plus the
    head tensors).  The embedding table answers row lookups without being upcast as a whole."""

    def __init__(self, w, prefix, shared=None):
        self.w, self.prefix, self.specs = w, prefix, si.tensor_specs(w)
        self.layer, self.layer_cache, self.head_cache = None, {}, {}
        self.shared = {} if shared is None else shared        # embedding and LM head: one copy for target and draft

    def _f64(self, prefix, key):
        a = si.make_tensor(self.w, prefix, key, self.specs)
        return si.bf16_bits_to_f32(a).astype(np.float64).reshape(a.shape) if a.dtype == np.uint16 else a.astype(np.float64)

    def __call__(self, name):
        if name in ("E", "lm"):                               # shared by target and draft: the target's tensors
            if name not in self.shared:
                self.shared[name] = self._f64("t", name)
            return self.shared[name]
        if not name.startswith("L"):
            if name not in self.head_cache:
                self.head_cache[name] = self._f64(self.prefix, name)
            return self.head_cache[name]
        layer = name.split(".")[0]
        if layer != self.layer:
            self.layer, self.layer_cache = layer, {}
        if name not in self.layer_cache:
            self.layer_cache[name] = self._f64(self.prefix, name)
        return self.layer_cache[name]


def load_state(w, seq, n):
    st = O.SeqState(w.target, w.draft, n + w.block_size + 1, cache_dtype=np.float32)
    for pool, lists, m in (("target", st.kv, w.target), ("draft", st.ctx, w.draft)):
        for l in range(m.n_layers):
            k, v = si.make_state_rows(w, seq, pool, l, n)
            lists.k[l][:n] = k
            lists.v[l][:n] = v
        lists.n = n
    st.n = n
    st.anchor = si.make_anchor(w, seq)
    return st


def main():
    out_path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden_moe_30b.json")
    only = [a for a in sys.argv[1:] if a in CASES] or sorted(CASES)
    results = json.load(open(out_path)) if os.path.exists(out_path) else {}
    t0 = time.time()
    for cfg in only:
        w = si.qwen3_30b_a3b_workload(CASES[cfg]["n_seqs"], CTX)
        Wt = LazyWeights(w, "t")
        Wd = LazyWeights(w, "d", Wt.shared)
        rnd = O.rounding_for(w.dtype)
        cols = np.sort(np.random.default_rng(w.seed).choice(w.target.vocab, N_COLS, replace=False)).astype(int)
        Bk = w.block_size
        for seq in CASES[cfg]["seqs"]:
            name = f"{cfg}_seq{seq}"
            if name in results and "--redo" not in sys.argv:
                continue
            n = CTX
            print(f"[{time.time()-t0:7.1f}s] {name}: state", flush=True)
            st = load_state(w, seq, n)
            rec = dict(config=cfg, seq=seq, n=n, anchor=int(st.anchor), cols=[int(c) for c in cols])
            O.ROUTE_MARGINS = []
            try:
                r = O.spec_step(Wt, Wd, w.target, w.draft, w.tap_layers, st, Bk, w.mask_token_id, rnd,
                                temperature=0.0, uniforms=None, key=0, seq_id=seq, proposal=None)
                gaps = np.sort(np.array(O.ROUTE_MARGINS))
            finally:
                O.ROUTE_MARGINS = None
            ds = r["draft_scores"]
            a = r["accept_len"]
            rec.update(
                block=[int(x) for x in r["block"]],
                oracle_draft=[int(np.argmax(ds[j])) for j in range(1, Bk)],
                draft_margin=[O.top2_margin(ds[j]) for j in range(1, Bk)],
                tgt_argmax=[int(x) for x in r["tgt_argmax"]],
                tgt_margin=[O.top2_margin(r["logits"][j]) for j in range(Bk)],
                accept_len=int(a), emitted=[int(x) for x in r["emitted"]],
                draft_logits_cols=[[float(x) for x in r["draft_logits"][j][cols]] for j in range(Bk)],
                tgt_logits_cols=[[float(x) for x in r["logits"][j][cols]] for j in range(Bk)],
                logit_std=float(r["logits"].std()),
                routing_decisions=int(gaps.size), smallest_router_gaps=[float(x) for x in gaps[:8]],
                ctx_k_new=[[float(x) for x in st.ctx.k[l][n + j, 0, :8]] for l in (0, w.draft.n_layers - 1) for j in range(a + 1)],
                ctx_v_new=[[float(x) for x in st.ctx.v[l][n + j, 0, :8]] for l in (0, w.draft.n_layers - 1) for j in range(a + 1)],
            )
            results[name] = rec
            json.dump(results, open(out_path, "w"), indent=0)
            print(f"[{time.time()-t0:7.1f}s]   accept_len {rec['accept_len']} emitted {rec['emitted']} min margins draft "
                  f"{min(rec['draft_margin']):.4f} target {min(rec['tgt_margin']):.4f} router gaps {gaps[:3]}", flush=True)
    print(f"[{time.time()-t0:7.1f}s] wrote {out_path}", flush=True)


if __name__ == "__main__":
    main()
