#!/usr/bin/env python3
"""Writes tests/golden/golden_8b.json: the CPU oracle's result of ONE speculative step at the full
8B shape (configurations 2-5) from a seeded synthetic cache state -- every sequence of configurations 2, 3
and 4, two sampled sequences of configuration 5 -- and, for configuration 2, a true prefill of its 2048
random prompt tokens (Section 4.1) followed by plain greedy decoding of six tokens and one speculative step
(record "cfg2_prefill_seq0": first token, sampled cache rows, the plain continuation, the step).

Calls only oracle/ and synth/ (never the HIP path).  Takes tens of minutes and ~35 GB of RAM on 8 cores;
the GPU tests (tests/test_gpu_full_size.py) regenerate the same weights and states from the same seeds
and compare what the kernels produce against these stored values.

Stored per sampled sequence: length, anchor, the oracle's drafted tokens and their top-2 margins, the
block that was verified (constructed: k true-continuation tokens, then a wrong one), the target's
greedy tokens and margins, accept length, emitted tokens, and draft / target logits at 64 seeded
vocabulary columns of every row.
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

# configuration -> sampled sequences and, for greedy configurations, how many proposals are made correct
CASES = {
    2: dict(seqs=[0], k=[3]),
    3: dict(seqs=list(range(16)), k=[0, 1, 3, 0, 4, 2, 1, 0, 5, 2, 0, 6, 1, 3, 0, 9]),
    4: dict(seqs=[0, 1, 2, 3], k=[0, 1, 2, 3]),
    5: dict(seqs=[0, 3, 8, 12, 17, 21, 26, 31], k=None),
}
N_COLS = 64
RNG_KEY = 20260206


class RowLookup:
    """Embedding table that upcasts only the rows asked for."""

    def __init__(self, weights, name):
        self.w, self.name = weights, name

    def __getitem__(self, idx):
        a = self.w.raw(self.name)[idx]
        return si.bf16_bits_to_f32(a).astype(np.float64).reshape(a.shape) if a.dtype == np.uint16 else a.astype(np.float64)


def getter(weights):
    emb = RowLookup(weights, "E")

    def W(name):
        return emb if name == "E" else weights.f64(name)
    return W


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


def sample_cols(w):
    return np.sort(np.random.default_rng(w.seed).choice(w.target.vocab, N_COLS, replace=False)).astype(int)


def store_step(rec, r, st, w, n, cols, greedy, uniforms):
    """What a speculative step of the oracle leaves in a record: tokens, margins, logits at the sampled columns, and the
    committed context-feature rows of the first and last draft layer (first 8 dims of head 0)."""
    Bk = w.block_size
    ds = r["draft_scores"]
    rec.update(
        block=[int(x) for x in r["block"]],
        oracle_draft=[int(np.argmax(ds[j])) for j in range(1, Bk)],
        draft_margin=[O.top2_margin(ds[j]) for j in range(1, Bk)],
        tgt_argmax=[int(x) for x in r["tgt_argmax"]],
        tgt_margin=[O.top2_margin(r["logits"][j]) for j in range(Bk)],
        accept_len=int(r["accept_len"]), emitted=[int(x) for x in r["emitted"]],
        draft_logits_cols=[[float(x) for x in r["draft_logits"][j][cols]] for j in range(Bk)],
        tgt_logits_cols=[[float(x) for x in r["logits"][j][cols]] for j in range(Bk)],
        logit_std=float(r["logits"].std()),
    )
    if not greedy:
        rec["key"] = RNG_KEY
        rec["uniforms"] = [float(x) for x in uniforms]
        rec["final_margin"] = O.top2_margin(r["final_scores"])
        # how close each acceptance test was: |u q(d) - p(d)| / p(d) for the tested slots
        p = O.softmax(r["logits"] / w.temperature)
        q = O.softmax(r["draft_logits"] / w.temperature)
        rec["accept_test_margin"] = [
            float(abs(uniforms[j] * q[j][r["block"][j]] - p[j - 1][r["block"][j]]) / p[j - 1][r["block"][j]])
            for j in range(1, min(Bk, r["accept_len"] + 2))]
    a = r["accept_len"]
    rec["ctx_k_new"] = [[float(x) for x in st.ctx.k[l][n + j, 0, :8]] for l in (0, w.draft.n_layers - 1) for j in range(a + 1)]
    rec["ctx_v_new"] = [[float(x) for x in st.ctx.v[l][n + j, 0, :8]] for l in (0, w.draft.n_layers - 1) for j in range(a + 1)]


def prefill_case(w, Wt, Wd, wt, rnd, cols, t0):
    """Configuration 2 from a true prefill: prompt of 2048 random tokens through the oracle's sequence form, the
    first generated token, a few cache rows of several layers, six tokens of plain greedy decoding (the sequence
    that speculative steps must reproduce), and one speculative step whose first two proposals are that
    continuation and the third a wrong token."""
    Bk = w.block_size
    prompt = [int(t) for t in si.make_prompts(w)[0]]
    n = len(prompt)
    st = O.SeqState(w.target, w.draft, n + 4 * Bk, cache_dtype=np.float32)
    print(f"[{time.time()-t0:7.1f}s] cfg 2 prefill of {n} tokens", flush=True)
    logits, taps = O.target_forward_sequence(Wt, w.target, prompt, st.kv, w.tap_layers, rnd, logit_rows=[n - 1])
    H_t = O.fuse_taps(Wd, w.draft, taps, rnd)
    for i, (k, v) in enumerate(O.draft_context_kv(Wd, w.draft, H_t, np.arange(n), rnd)):
        st.ctx.k[i][:n] = k
        st.ctx.v[i][:n] = v
    st.ctx.n = st.n = n
    st.anchor = int(np.argmax(logits[0]))
    del taps, H_t
    rec = dict(config="2p", seq=0, n=n, anchor=int(st.anchor), first_margin=O.top2_margin(logits[0]), cols=[int(c) for c in cols],
               first_logits_cols=[float(x) for x in logits[0][cols]])
    rows = [0, 1, 17, 1000, 2046, 2047]
    rec["kv_rows"] = rows
    rec["kv_layers"] = [0, 1, 17, 35]
    rec["tgt_k"] = [[[float(x) for x in st.kv.k[l][r, 3, :8]] for r in rows] for l in rec["kv_layers"]]
    rec["tgt_v"] = [[[float(x) for x in st.kv.v[l][r, 3, :8]] for r in rows] for l in rec["kv_layers"]]
    rec["ctx_layers"] = [0, w.draft.n_layers - 1]
    rec["ctx_k"] = [[[float(x) for x in st.ctx.k[l][r, 5, :8]] for r in rows] for l in rec["ctx_layers"]]
    rec["ctx_v"] = [[[float(x) for x in st.ctx.v[l][r, 5, :8]] for r in rows] for l in rec["ctx_layers"]]
    print(f"[{time.time()-t0:7.1f}s]   first token {st.anchor} (margin {rec['first_margin']:.4f}); plain greedy decoding", flush=True)
    tok, cont, margins = st.anchor, [], []
    for j in range(6):
        lg, _ = O.target_forward_tokens(Wt, w.target, [tok], n + j, st.kv, (), rnd)
        tok = int(np.argmax(lg[0]))
        cont.append(tok)
        margins.append(O.top2_margin(lg[0]))
    st.kv.truncate(n)
    rec["plain_greedy"] = cont
    rec["plain_greedy_margin"] = margins
    print(f"[{time.time()-t0:7.1f}s]   continuation {cont}", flush=True)
    k = 2
    dl = O.draft_block_forward(Wd, w.draft, st.anchor, n, st.ctx, Bk, w.mask_token_id, rnd)
    drafted = [int(np.argmax(dl[j])) for j in range(1, Bk)]
    wrong = drafted[k] if drafted[k] != cont[k] else (cont[k] + 1) % (w.target.vocab - 1)
    proposal = cont[:k] + [wrong] + drafted[k + 1:]
    rec["k_correct"] = k
    return st, rec, proposal


def main():
    out_path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden_8b.json")
    only = [int(x) for x in sys.argv[1:] if x.isdigit()] or sorted(CASES)
    results = {}
    if os.path.exists(out_path):
        results = json.load(open(out_path))
    t0 = time.time()
    wt = wd = None
    for cfg in only:
        w = si.workload(cfg)
        if wt is None:
            print(f"[{time.time()-t0:7.1f}s] generating weights (seed {w.wseed})", flush=True)
            wt, wd = si.make_weights(w, 8)
        Wt, Wd = getter(wt), getter(wd)
        rnd = O.rounding_for(w.dtype)
        lens = si.make_context_lengths(w)
        cols = sample_cols(w)
        Bk = w.block_size
        if cfg == 2 and ("cfg2_prefill_seq0" not in results or "--redo" in sys.argv):
            st, rec, proposal = prefill_case(w, Wt, Wd, wt, rnd, cols, t0)
            n = st.n
            r = O.spec_step(Wt, Wd, w.target, w.draft, w.tap_layers, st, Bk, w.mask_token_id, rnd, proposal=proposal)
            store_step(rec, r, st, w, n, cols, True, None)
            results["cfg2_prefill_seq0"] = rec
            json.dump(results, open(out_path, "w"), indent=0)
            print(f"[{time.time()-t0:7.1f}s]   accept_len {rec['accept_len']} emitted {rec['emitted']}", flush=True)
            del st
        for i, seq in enumerate(CASES[cfg]["seqs"]):
            n = int(lens[seq])
            if f"cfg{cfg}_seq{seq}" in results and "--redo" not in sys.argv:
                continue                                   # resumable: keep what an earlier run stored
            print(f"[{time.time()-t0:7.1f}s] cfg {cfg} seq {seq} n={n}: state", flush=True)
            st = load_state(w, seq, n)
            rec = dict(config=cfg, seq=seq, n=n, anchor=int(st.anchor), cols=[int(c) for c in cols])
            greedy = w.temperature == 0.0
            proposal = None
            if greedy:
                # the oracle's own draft, then k true-continuation tokens and a wrong one in front of it
                k = CASES[cfg]["k"][i]
                dl = O.draft_block_forward(Wd, w.draft, st.anchor, n, st.ctx, Bk, w.mask_token_id, rnd)
                drafted = [int(np.argmax(dl[j])) for j in range(1, Bk)]
                tok, cont = st.anchor, []
                for j in range(k):
                    lg, _ = O.target_forward_tokens(Wt, w.target, [tok], n + j, st.kv, (), rnd)
                    tok = int(np.argmax(lg[0]))
                    cont.append(tok)
                lg, _ = O.target_forward_tokens(Wt, w.target, [tok], n + k, st.kv, (), rnd)
                true_next = int(np.argmax(lg[0]))
                st.kv.truncate(n)
                wrong = drafted[k] if drafted[k] != true_next else (true_next + 1) % (w.target.vocab - 1)
                proposal = cont + [wrong] + drafted[k + 1:]
                rec["k_correct"] = k
                print(f"[{time.time()-t0:7.1f}s]   continuation of {k} tokens done", flush=True)
            uniforms = si.make_uniforms(w, 0)[seq].astype(np.float64) if not greedy else None
            r = O.spec_step(Wt, Wd, w.target, w.draft, w.tap_layers, st, Bk, w.mask_token_id, rnd,
                            temperature=w.temperature, uniforms=uniforms, key=RNG_KEY, seq_id=seq, proposal=proposal)
            store_step(rec, r, st, w, n, cols, greedy, uniforms)
            results[f"cfg{cfg}_seq{seq}"] = rec
            json.dump(results, open(out_path, "w"), indent=0)
            print(f"[{time.time()-t0:7.1f}s]   accept_len {rec['accept_len']} emitted {rec['emitted']} "
                  f"min margins draft {min(rec['draft_margin']):.4f} target {min(rec['tgt_margin']):.4f}", flush=True)
    if "--exact" in sys.argv and "cfg2_seq0" in results and ("tgt_logits_cols_exact" not in results["cfg2_seq0"] or "--redo" in sys.argv):
        # configuration 2 once more in exact arithmetic (no storage rounding anywhere) on the same cached rows and the
        # same block: what the GPU's distance from the unrounded model is measured against
        w = si.workload(2)
        if wt is None:
            print(f"[{time.time()-t0:7.1f}s] generating weights (seed {w.wseed})", flush=True)
            wt, wd = si.make_weights(w, 8)
        rec = results["cfg2_seq0"]
        st = load_state(w, 0, rec["n"])
        print(f"[{time.time()-t0:7.1f}s] cfg 2 seq 0 in exact arithmetic", flush=True)
        r = O.spec_step(getter(wt), getter(wd), w.target, w.draft, w.tap_layers, st, w.block_size, w.mask_token_id, O.identity,
                        proposal=rec["block"][1:])
        cols = np.array(rec["cols"])
        rec["tgt_logits_cols_exact"] = [[float(x) for x in r["logits"][j][cols]] for j in range(w.block_size)]
        rec["draft_logits_cols_exact"] = [[float(x) for x in r["draft_logits"][j][cols]] for j in range(w.block_size)]
        json.dump(results, open(out_path, "w"), indent=0)
    print(f"[{time.time()-t0:7.1f}s] wrote {out_path}", flush=True)


if __name__ == "__main__":
    main()
