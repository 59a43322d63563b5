"""Small test-side helpers: cached float64 weight getters and tiny workloads."""
from dataclasses import replace

import numpy as np

from synth import inputs as si


class W64:
    """Callable name -> float64 array with a cache (tiny models only)."""

    def __init__(self, weights, cache=True):
        self.w = weights
        self.cache = {} if cache else None

    def __call__(self, name):
        if self.cache is None:
            return self.w.f64(name)
        if name not in self.cache:
            self.cache[name] = self.w.f64(name)
        return self.cache[name]


def tiny_workload(seed=0, n_layers=2, draft_layers=1, vocab=1024, block=8, qk_norm=False,
                  kv_heads=4, dtype="f32", n_seqs=1, ctx=(128, 128), taps=None, d=256, heads=4,
                  hd=64, ffn=1024):
    t = si.tiny_dims(n_layers, vocab=vocab, d=d, heads=heads, kv_heads=kv_heads, hd=hd, ffn=ffn,
                     qk_norm=qk_norm)
    dd = replace(t, n_layers=draft_layers)
    taps = taps if taps is not None else (0,)
    return si.Workload("tiny", dtype, t, dd, tuple(taps), vocab - 1, block, n_seqs, ctx[0], ctx[1],
                       0.0, seed)
