"""Test-side driver of the HIP path: uploads seeded weights, packs them, prefills by chunked
verification with forced commits, runs speculative steps through the C ABI, and moves cache state
between the oracle's per-sequence lists and the paged pools."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

import paper_2602_06036_amd as dfl
from paper_2602_06036_amd import binding as B
from synth import inputs as si


def to_dev(arr: np.ndarray, dev) -> torch.Tensor:
    if arr.dtype == np.uint16:                                   # bf16 bit patterns
        return torch.from_numpy(arr.view(np.int16)).to(dev).view(torch.bfloat16)
    return torch.from_numpy(arr).to(dev)


class GpuModel:
    def __init__(self, w: si.Workload, wt: si.Weights, wd: si.Weights, max_len: int, n_seqs: Optional[int] = None,
                 shuffle_pages: bool = True, device: str = "cuda:0", max_seqs: Optional[int] = None, blobs=None):
        self.w = w
        self.dev = torch.device(device)
        self.S = n_seqs or w.n_seqs
        self.Bk = w.block_size
        table, n_pages = si.make_block_table(w if self.S == w.n_seqs else _with_seqs(w, self.S), max_len, shuffle_pages)
        self.table_host = table
        self.e = dfl.Engine(w.target, w.draft, w.dtype, w.block_size, max_seqs or self.S, table.shape[1], n_pages,
                            w.tap_layers, w.mask_token_id, device, blobs=blobs)
        e = self.e
        if blobs is None:
            self._pack(w, wt, wd)
        e.create()
        self._alloc_io(w, table)

    def _pack(self, w, wt, wd):
        e = self.e
        e.pack_target_head(to_dev(wt.raw("E"), self.dev), to_dev(wt.raw("lm"), self.dev), to_dev(wt.raw("gf"), self.dev))
        for l in range(w.target.n_layers):
            e.pack_target_layer(l, {k: to_dev(wt.raw(f"L{l}.{k}"), self.dev) for k in si.layer_shapes(w.target)})
            torch.cuda.synchronize(self.dev)
        e.pack_draft_head(to_dev(wd.raw("wc"), self.dev), to_dev(wd.raw("gc"), self.dev), to_dev(wd.raw("gf"), self.dev))
        for l in range(w.draft.n_layers):
            e.pack_draft_layer(l, {k: to_dev(wd.raw(f"L{l}.{k}"), self.dev) for k in si.LAYER_MATS + si.LAYER_GAINS})
            torch.cuda.synchronize(self.dev)
        torch.cuda.synchronize(self.dev)

    def blobs(self):
        return (self.e.target_blob, self.e.draft_blob)

    def _alloc_io(self, w, table):
        self.block_table = torch.from_numpy(table).to(self.dev)
        self.seq_lens = torch.zeros(self.S, dtype=torch.int32, device=self.dev)
        self.anchor = torch.zeros(self.S, dtype=torch.int32, device=self.dev)
        self.host_lens = np.zeros(self.S, dtype=np.int64)
        V = w.target.vocab
        self.draft_tokens = torch.zeros((self.S, self.Bk), dtype=torch.int32, device=self.dev)
        self.tgt_argmax = torch.zeros_like(self.draft_tokens)
        self.accept_len = torch.zeros(self.S, dtype=torch.int32, device=self.dev)
        self.out_tokens = torch.zeros_like(self.draft_tokens)
        self.kv_slots = torch.zeros((self.S, self.Bk), dtype=torch.int64, device=self.dev)
        self.logits_d = torch.zeros((self.S, self.Bk, V), dtype=torch.float32, device=self.dev)
        self.logits_t = torch.zeros_like(self.logits_d)

    def batch(self, block: int = 0):
        return self.e.batch(self.seq_lens, self.block_table, self.anchor, int(self.host_lens.max()), block)

    # ---- prefill by chunked verification with forced commits ---------------------------------------
    def prefill(self, prompts: Sequence[np.ndarray]) -> np.ndarray:
        S, Bk = self.S, self.Bk
        lens = np.array([len(p) for p in prompts])
        n_chunks = int((lens.max() + Bk - 1) // Bk)
        for c in range(n_chunks):
            toks = np.zeros((S, Bk), dtype=np.int32)
            r = np.clip(lens - c * Bk, 0, Bk)
            for s in range(S):
                toks[s, : r[s]] = prompts[s][c * Bk: c * Bk + r[s]]
            tokens = torch.from_numpy(toks).to(self.dev)
            b = self.batch()
            # a chunk that ends no prompt needs no token out of the target: the LM head is skipped
            ends_one = bool(((lens > c * Bk) & (lens <= (c + 1) * Bk)).any())
            dfl.dflash_verify(self.e, b, tokens, self.tgt_argmax if ends_one else None)
            acc = torch.from_numpy((r - 1).astype(np.int32)).to(self.dev)
            dfl.dflash_kv_commit(self.e, b, acc, self.tgt_argmax)
            self.host_lens += r
        torch.cuda.synchronize(self.dev)
        self.e.device_status()
        assert np.array_equal(self.seq_lens.cpu().numpy(), self.host_lens)
        return self.anchor.cpu().numpy().copy()

    def prefill_one_pass(self, prompts: Sequence[np.ndarray]) -> np.ndarray:
        """The same prefill as ONE verify + commit with many rows: every B-token chunk of every prompt becomes a
        pseudo-sequence whose committed length is the chunk's offset and whose block-table row is its prompt's.
        Inside a layer all K/V rows are written to the pages before attention runs, so chunk i sees chunks
        0..i-1 of its prompt exactly as a causal prefill does; the forced commit then projects the taps of all
        prompt rows into the draft's context cache.  Needs a context created with max_seqs >= number of chunks."""
        S, Bk = self.S, self.Bk
        lens = np.array([len(p) for p in prompts])
        owner, offset, rows = [], [], []
        for s in range(S):
            for c in range(int((lens[s] + Bk - 1) // Bk)):
                owner.append(s); offset.append(c * Bk); rows.append(min(Bk, lens[s] - c * Bk))
        n = len(owner)
        toks = np.zeros((n, Bk), dtype=np.int32)
        for i in range(n):
            toks[i, : rows[i]] = prompts[owner[i]][offset[i]: offset[i] + rows[i]]
        dev = self.dev
        p_lens = torch.from_numpy(np.array(offset, dtype=np.int32)).to(dev)
        p_table = self.block_table[torch.from_numpy(np.array(owner, dtype=np.int64)).to(dev)].contiguous()
        p_anchor = torch.zeros(n, dtype=torch.int32, device=dev)
        tokens = torch.from_numpy(toks).to(dev)
        argmax = torch.zeros((n, Bk), dtype=torch.int32, device=dev)
        acc = torch.from_numpy(np.array(rows, dtype=np.int32) - 1).to(dev)
        b = self.e.batch(p_lens, p_table, p_anchor, int(max(offset)))
        dfl.dflash_verify(self.e, b, tokens, argmax)
        dfl.dflash_kv_commit(self.e, b, acc, argmax)
        torch.cuda.synchronize(dev)
        self.e.device_status()
        last = [max(i for i in range(n) if owner[i] == s) for s in range(S)]
        first_tokens = p_anchor.cpu().numpy()[last].astype(np.int32)
        assert np.array_equal(p_lens.cpu().numpy()[last], lens)
        self.host_lens = lens.astype(np.int64)
        self.seq_lens.copy_(torch.from_numpy(lens.astype(np.int32)).to(dev))
        self.anchor.copy_(torch.from_numpy(first_tokens).to(dev))
        return first_tokens.copy()

    def prefill_entry(self, prompts: Sequence[np.ndarray], pieces: int = 1) -> np.ndarray:
        """Prefill through the library's own entry point (dflash_prefill): all prompts in one call, or, with pieces > 1,
        every prompt cut into that many consecutive parts handed over in as many calls (a prompt that arrives in
        pieces: the later calls find the earlier parts cached)."""
        lens = np.array([len(p) for p in prompts])
        first = torch.full((self.S,), -1, dtype=torch.int32, device=self.dev)
        cuts = [np.linspace(0, n, pieces + 1).astype(int) for n in lens]
        for k in range(pieces):
            part = [np.asarray(p[c[k]: c[k + 1]], dtype=np.int32) for p, c in zip(prompts, cuts)]
            toks = torch.from_numpy(np.concatenate(part) if sum(len(x) for x in part) else np.zeros(0, np.int32)).to(self.dev)
            dfl.dflash_prefill(self.e, self.batch(), toks, [len(x) for x in part], first)
            self.host_lens += np.array([len(x) for x in part])
        torch.cuda.synchronize(self.dev)
        self.e.device_status()
        assert np.array_equal(self.seq_lens.cpu().numpy(), self.host_lens)
        got = self.anchor.cpu().numpy().copy()
        assert np.array_equal(got[lens > 0], first.cpu().numpy()[lens > 0])
        return got

    # ---- one speculative step --------------------------------------------------------------------------
    def step(self, proposals: Optional[np.ndarray] = None, temperature: float = 0.0, uniforms: Optional[np.ndarray] = None,
             key: int = 0, want_logits: bool = True, block: int = 0) -> Dict[str, np.ndarray]:
        """block: rows per sequence of this step when it is to differ from the context's block size (dflash_batch::block_size);
        the step's [S, block] arrays are then separate tensors of that shape."""
        b = self.batch(block)
        if block and block != self.Bk:
            V = self.w.target.vocab
            draft_tokens = torch.zeros((self.S, block), dtype=torch.int32, device=self.dev)
            tgt_argmax, out_tokens = torch.zeros_like(draft_tokens), torch.zeros_like(draft_tokens)
            kv_slots = torch.zeros((self.S, block), dtype=torch.int64, device=self.dev)
            logits_d = torch.zeros((self.S, block, V), dtype=torch.float32, device=self.dev) if want_logits else None
            logits_t = torch.zeros_like(logits_d) if want_logits else None
        else:
            draft_tokens, tgt_argmax, out_tokens, kv_slots = self.draft_tokens, self.tgt_argmax, self.out_tokens, self.kv_slots
            logits_d, logits_t = (self.logits_d, self.logits_t) if want_logits else (None, None)
        rng = torch.tensor([key], dtype=torch.int64, device=self.dev) if temperature > 0 else None
        dfl.dflash_draft_block(self.e, b, draft_tokens, temperature, rng, logits_d)
        drafted = draft_tokens.cpu().numpy().copy()
        if proposals is not None:                 # entries < 0 keep the GPU's own draft for that slot
            blk = drafted.copy()
            blk[:, 1:] = np.where(proposals >= 0, proposals, drafted[:, 1:])
            draft_tokens.copy_(torch.from_numpy(blk).to(self.dev))
        dfl.dflash_verify(self.e, b, draft_tokens, tgt_argmax, logits_t)
        u = torch.from_numpy(np.ascontiguousarray(uniforms, dtype=np.float32)).to(self.dev) if uniforms is not None else None
        dfl.dflash_accept(self.e, b, draft_tokens, tgt_argmax, self.accept_len, out_tokens, temperature, u, rng)
        lens_before = self.host_lens.copy()
        dfl.dflash_kv_commit(self.e, b, self.accept_len, out_tokens, kv_slots)
        torch.cuda.synchronize(self.dev)
        self.e.device_status()
        a = self.accept_len.cpu().numpy().copy()
        self.host_lens = lens_before + a + 1
        assert np.array_equal(self.seq_lens.cpu().numpy(), self.host_lens)
        out = dict(drafted=drafted, block=draft_tokens.cpu().numpy().copy(), tgt_argmax=tgt_argmax.cpu().numpy().copy(),
                   accept_len=a, out_tokens=out_tokens.cpu().numpy().copy(), kv_slots=kv_slots.cpu().numpy().copy(),
                   lens_before=lens_before, anchor=self.anchor.cpu().numpy().copy())
        if want_logits:
            out["logits_d"] = logits_d.cpu().numpy().copy()
            out["logits_t"] = logits_t.cpu().numpy().copy()
        return out

    # ---- cache state in canonical form -----------------------------------------------------------------------
    def read_kv(self, pool: int, layer: int, seq: int, start: int, count: int):
        k, v = dfl.dflash_kv_read(self.e, self.batch(), pool, layer, seq, start, count)
        torch.cuda.synchronize(self.dev)
        return k.cpu().numpy(), v.cpu().numpy()

    def write_kv(self, pool: int, layer: int, seq: int, start: int, k: np.ndarray, v: np.ndarray):
        dfl.dflash_kv_write(self.e, self.batch(), pool, layer, seq, start,
                            torch.from_numpy(np.ascontiguousarray(k, dtype=np.float32)).to(self.dev),
                            torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to(self.dev))

    def load_state(self, states) -> None:
        """Teacher forcing / synthetic state: copy each oracle SeqState (lists of K/V rows, length,
        anchor) into the paged pools."""
        lens = np.array([st.n for st in states], dtype=np.int32)
        self.host_lens = lens.astype(np.int64)
        self.seq_lens.copy_(torch.from_numpy(lens).to(self.dev))
        self.anchor.copy_(torch.from_numpy(np.array([st.anchor for st in states], dtype=np.int32)).to(self.dev))
        for s, st in enumerate(states):
            for l in range(self.w.target.n_layers):
                self.write_kv(B.DFLASH_POOL_TARGET, l, s, 0, st.kv.k[l][: st.n], st.kv.v[l][: st.n])
            for l in range(self.w.draft.n_layers):
                self.write_kv(B.DFLASH_POOL_DRAFT, l, s, 0, st.ctx.k[l][: st.n], st.ctx.v[l][: st.n])
        torch.cuda.synchronize(self.dev)

    def load_synthetic(self, sampled: Sequence[int]) -> None:
        """Synthetic cache state (unit normals, bf16-rounded) for every sequence: sequences in `sampled` get the
        seeded rows of synth.make_state_rows (the oracle's goldens use the same), the others device-generated
        rows of the same distribution."""
        w = self.w
        lens = si.make_context_lengths(w)[: self.S]
        self.host_lens = lens.astype(np.int64)
        self.seq_lens.copy_(torch.from_numpy(lens.astype(np.int32)).to(self.dev))
        self.anchor.copy_(torch.from_numpy(np.array([si.make_anchor(w, s) for s in range(self.S)], dtype=np.int32)).to(self.dev))
        gen = torch.Generator(device=self.dev)
        gen.manual_seed(w.seed)
        for s in range(self.S):
            n = int(lens[s])
            for pool, pid, m in (("target", B.DFLASH_POOL_TARGET, w.target), ("draft", B.DFLASH_POOL_DRAFT, w.draft)):
                for l in range(m.n_layers):
                    if s in sampled:
                        k, v = si.make_state_rows(w, s, pool, l, n)
                        self.write_kv(pid, l, s, 0, k, v)
                    else:
                        kv = torch.randn((2, n, m.n_kv_heads, m.head_dim), generator=gen, device=self.dev, dtype=torch.float32)
                        if w.dtype == "bf16":
                            kv = kv.to(torch.bfloat16).to(torch.float32)
                        dfl.dflash_kv_write(self.e, self.batch(), pid, l, s, 0, kv[0].contiguous(), kv[1].contiguous())
            torch.cuda.synchronize(self.dev)

    def expected_slots(self, lens_before: np.ndarray, accept_len: np.ndarray, block: int = 0) -> np.ndarray:
        """page*16 + offset from the page table (the definition of a KV slot id), -1 past the accepted prefix."""
        out = -np.ones((self.S, block or self.Bk), dtype=np.int64)
        for s in range(self.S):
            for j in range(int(accept_len[s]) + 1):
                pos = int(lens_before[s]) + j
                out[s, j] = int(self.table_host[s, pos // 16]) * 16 + pos % 16
        return out


def _with_seqs(w: si.Workload, n: int) -> si.Workload:
    from dataclasses import replace
    return replace(w, n_seqs=n)
