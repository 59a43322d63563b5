"""Seeded synthetic workloads for the speculative-decoding step.

Everything the oracle tests and the HIP-path tests feed to their respective implementations
comes from here: model shapes, random-initialised weights, random prompts, page tables and
acceptance uniforms.  The paper evaluates on trained Qwen3 / LLaMA checkpoints and public
benchmark suites (Section 5); none of those is available, so these inputs reproduce only the
shapes, lengths and batch structure.  No model arithmetic is implemented in this module.
"""
from __future__ import annotations

import zlib
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Dict, Iterable, List, Optional, Tuple

import numpy as np

PAGE_SIZE = 16


# --------------------------------------------------------------------------------------
# bf16 storage helpers (data format only: round-to-nearest-even of an fp32 bit pattern)
# --------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------------------
# shapes
# --------------------------------------------------------------------------------------
@dataclass(frozen=True)
class ModelDims:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_theta: float
    rms_eps: float
    qk_norm: bool
    # routed-expert FFN (the Qwen3-Coder-30B-A3B target of Section 5 is a mixture-of-experts model): n_experts > 0
    # replaces the dense FFN by n_experts SwiGLU experts of width d_expert, top_k of them per token
    n_experts: int = 0
    top_k: int = 0
    d_expert: int = 0

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                      # "f32" | "bf16"
    target: ModelDims
    draft: ModelDims
    tap_layers: Tuple[int, ...]     # 0-based target layers whose output is tapped
    mask_token_id: int
    block_size: int
    n_seqs: int
    ctx_min: int
    ctx_max: int                    # per-sequence context drawn uniformly in [ctx_min, ctx_max]
    temperature: float
    seed: int
    n_steps: int = 1
    weight_seed: Optional[int] = None   # None: weights use `seed`; the 8B configurations share one set

    @property
    def wseed(self) -> int:
        return self.seed if self.weight_seed is None else self.weight_seed


def tap_layers_for(n_layers: int, n_taps: int) -> Tuple[int, ...]:
    """n_taps layer indices spread evenly from the second layer to the third-to-last one
    (0-based 1 .. n_layers-3), as Section 5 'Implementation' describes."""
    if n_taps == 1:
        return (0,)
    lo, hi = 1, n_layers - 3
    return tuple(int(round(lo + t * (hi - lo) / (n_taps - 1))) for t in range(n_taps))


def tiny_dims(n_layers: int, vocab: int = 1024, d: int = 256, heads: int = 4, kv_heads: int = 4,
              hd: int = 64, ffn: int = 1024, theta: float = 1e4, qk_norm: bool = False) -> ModelDims:
    return ModelDims(n_layers, d, heads, kv_heads, hd, ffn, vocab, theta, 1e-6, qk_norm)


def dims_8b(n_layers: int) -> ModelDims:
    return ModelDims(n_layers, 4096, 32, 8, 128, 12288, 151936, 1e6, 1e-6, True)


def workload(idx: int) -> Workload:
    """The five configurations of the benchmark definition (1-based)."""
    if idx == 1:
        t = tiny_dims(2)
        return Workload("cfg1_tiny_f32", "f32", t, replace(t, n_layers=1), (0,), t.vocab - 1,
                        8, 1, 128, 128, 0.0, 0, n_steps=20)
    t = dims_8b(36)
    d = dims_8b(5)
    taps = tap_layers_for(36, 5)
    mask = t.vocab - 1
    if idx == 2:
        return Workload("cfg2_8b_b1_ctx2048", "bf16", t, d, taps, mask, 16, 1, 2048, 2048, 0.0, 2)
    if idx == 3:
        return Workload("cfg3_8b_b16_ctx1k-4k", "bf16", t, d, taps, mask, 16, 16, 1024, 4096, 0.0, 3, weight_seed=2)
    if idx == 4:
        return Workload("cfg4_8b_b4_ctx16k", "bf16", t, d, taps, mask, 16, 4, 16384, 16384, 0.0, 4, weight_seed=2)
    if idx == 5:
        return Workload("cfg5_8b_b32_ctx8k_T1", "bf16", t, d, taps, mask, 16, 32, 8192, 8192, 1.0, 5, weight_seed=2)
    raise ValueError(idx)


def llama31_8b_workload(n_seqs: int = 1, ctx: int = 2048) -> Workload:
    """The second target shape of Section 5 ('Implementation', Table 5): LLaMA-3.1-8B (32 layers, FFN 14336,
    vocabulary 128256, rope base 5e5, no q/k norm) with a 5-layer drafter and block size 10."""
    t = ModelDims(32, 4096, 32, 8, 128, 14336, 128256, 5e5, 1e-5, False)
    d = replace(t, n_layers=5)
    return Workload("llama31_8b_b10", "bf16", t, d, tap_layers_for(32, 5), t.vocab - 1, 10, n_seqs, ctx, ctx, 0.0, 6)


def qwen3_30b_a3b_workload(n_seqs: int = 1, ctx: int = 2048) -> Workload:
    """The shape of the mixture-of-experts target of Section 5 (Qwen3-Coder-30B-A3B: 48 layers, d_model 2048, 32 query /
    4 KV heads of 128, 128 experts of width 768 with 8 per token, QK-norm) with the paper's drafter for it (8 dense
    layers, Section 5 "Implementation"; dense FFN width: this build's choice of 6144) and block size 16."""
    t = ModelDims(48, 2048, 32, 4, 128, 6144, 151936, 1e7, 1e-6, True, 128, 8, 768)
    d = ModelDims(8, 2048, 32, 4, 128, 6144, 151936, 1e7, 1e-6, True)
    return Workload("qwen3_30b_a3b", "bf16", t, d, tap_layers_for(48, 5), t.vocab - 1, 16, n_seqs, ctx, ctx, 0.0, 7)


def wide_moe_workload(n_seqs: int, ctx_min: int = 12, ctx_max: int = 40, seed: int = 91) -> Workload:
    """Two target layers at the full width of the Section 5 mixture-of-experts target (d_model 2048, 32 query / 4 KV
    heads, 128 experts of width 768, 8 per token) with a small vocabulary and a one-layer dense drafter: the expert
    GEMMs, routing and attention run in the launch shapes of the full model at a size the oracle handles."""
    t = ModelDims(2, 2048, 32, 4, 128, 1024, 4096, 1e7, 1e-6, True, 128, 8, 768)
    d = ModelDims(1, 2048, 32, 4, 128, 1024, 4096, 1e7, 1e-6, True)
    return Workload("wide_moe", "bf16", t, d, (0, 1), t.vocab - 1, 16, n_seqs, ctx_min, ctx_max, 0.0, seed)


def small_moe_workload(n_seqs: int = 3, ctx_min: int = 20, ctx_max: int = 100, seed: int = 61, n_experts: int = 16,
                       top_k: int = 2, d_expert: int = 256) -> Workload:
    """The small bf16 model with a routed-expert target (structure of the Qwen3-Coder-30B-A3B target of Section 5:
    every target layer's FFN is n_experts SwiGLU experts, top_k per token) and the usual dense 2-layer drafter."""
    t = ModelDims(4, 512, 8, 2, 128, 1536, 4096, 1e6, 1e-6, True, n_experts, top_k, d_expert)
    d = ModelDims(2, 512, 8, 2, 128, 1536, 4096, 1e6, 1e-6, True)
    return Workload("small_moe", "bf16", t, d, (0, 1), t.vocab - 1, 16, n_seqs, ctx_min, ctx_max, 0.0, seed)


def small_bf16_workload(n_seqs: int = 3, ctx_min: int = 20, ctx_max: int = 150, seed: int = 11,
                        block_size: int = 16, temperature: float = 0.0, draft_layers: int = 2,
                        n_taps: int = 5) -> Workload:
    """A scaled-down bf16 model with the 8B model's structure (GQA 4:1, head_dim 128, QK-norm,
    five taps) that the oracle can prefill and step in seconds.  draft_layers / n_taps give the drafter depth
    and the number of tapped target layers of the ablations in Section 5.5 (3, 5, 8 layers; 3 or 5 features)."""
    t = ModelDims(8, 512, 8, 2, 128, 1536, 4096, 1e6, 1e-6, True)
    d = replace(t, n_layers=draft_layers)
    return Workload("small_bf16", "bf16", t, d, tap_layers_for(8, n_taps), t.vocab - 1, block_size,
                    n_seqs, ctx_min, ctx_max, temperature, seed)


# --------------------------------------------------------------------------------------
# weights
# --------------------------------------------------------------------------------------
LAYER_MATS = ("wq", "wk", "wv", "wo", "wg", "wu", "wd")
LAYER_GAINS = ("g1", "g2", "qn", "kn")


def layer_shapes(m: ModelDims) -> Dict[str, Tuple[int, ...]]:
    """Every linear map is stored [out_features, in_features] (y = W x, the paper's notation).  A routed-expert
    layer has the router "wr" [E, D] and the experts' matrices stacked along a leading expert axis."""
    if m.n_experts:
        return {
            "g1": (m.d_model,), "g2": (m.d_model,), "qn": (m.head_dim,), "kn": (m.head_dim,),
            "wq": (m.q_dim, m.d_model), "wk": (m.kv_dim, m.d_model), "wv": (m.kv_dim, m.d_model),
            "wo": (m.d_model, m.q_dim), "wr": (m.n_experts, m.d_model),
            "wg": (m.n_experts, m.d_expert, m.d_model), "wu": (m.n_experts, m.d_expert, m.d_model),
            "wd": (m.n_experts, m.d_model, m.d_expert),
        }
    return {
        "g1": (m.d_model,), "g2": (m.d_model,), "qn": (m.head_dim,), "kn": (m.head_dim,),
        "wq": (m.q_dim, m.d_model), "wk": (m.kv_dim, m.d_model), "wv": (m.kv_dim, m.d_model),
        "wo": (m.d_model, m.q_dim),
        "wg": (m.d_ffn, m.d_model), "wu": (m.d_ffn, m.d_model), "wd": (m.d_model, m.d_ffn),
    }


class Weights:
    """name -> array.  Matrices are fp32 ("f32") or bf16 bit patterns in uint16 ("bf16");
    norm gains are always fp32.  `f64(name)` gives the exact stored value upcast to float64."""

    def __init__(self, dtype: str):
        self.dtype = dtype
        self.t: Dict[str, np.ndarray] = {}

    def raw(self, name: str) -> np.ndarray:
        return self.t[name]

    def f64(self, name: str) -> np.ndarray:
        a = self.t[name]
        if a.dtype == np.uint16:
            return bf16_bits_to_f32(a).astype(np.float64)
        return a.astype(np.float64)

    def f32(self, name: str) -> np.ndarray:
        a = self.t[name]
        if a.dtype == np.uint16:
            return bf16_bits_to_f32(a)
        return a

    def names(self) -> Iterable[str]:
        return self.t.keys()


def _rng(seed: int, name: str) -> np.random.Generator:
    return np.random.default_rng([seed, zlib.crc32(name.encode())])


def _matrix(seed: int, name: str, shape, dtype: str, std: float = 0.02) -> np.ndarray:
    x = _rng(seed, name).standard_normal(shape, dtype=np.float32)
    x *= np.float32(std)
    return f32_to_bf16_bits(x) if dtype == "bf16" else x


def _gain(seed: int, name: str, n: int) -> np.ndarray:
    # near 1 but not exactly 1, so that a mixed-up or dropped gain vector is visible
    return (1.0 + 0.1 * _rng(seed, name).uniform(-1.0, 1.0, n)).astype(np.float32)


def tensor_specs(w: Workload) -> Dict[Tuple[str, str], Tuple[tuple, bool]]:
    """(model prefix "t" | "d", tensor name) -> (shape, is a norm gain) for every tensor of the workload, in the order
    make_weights creates them.  The shared embedding "E" and LM head "lm" are listed once, under the target."""
    t, d = w.target, w.draft
    specs: Dict[Tuple[str, str], Tuple[tuple, bool]] = {}
    specs[("t", "E")] = ((t.vocab, t.d_model), False)
    specs[("t", "lm")] = ((t.vocab, t.d_model), False)
    specs[("t", "gf")] = ((t.d_model,), True)
    for l in range(t.n_layers):
        for k, shp in layer_shapes(t).items():
            specs[("t", f"L{l}.{k}")] = (tuple(shp), k in LAYER_GAINS)
    specs[("d", "wc")] = ((d.d_model, len(w.tap_layers) * t.d_model), False)
    specs[("d", "gc")] = ((d.d_model,), True)
    specs[("d", "gf")] = ((d.d_model,), True)
    for l in range(d.n_layers):
        for k, shp in layer_shapes(d).items():
            specs[("d", f"L{l}.{k}")] = (tuple(shp), k in LAYER_GAINS)
    return specs


def make_tensor(w: Workload, prefix: str, key: str, specs=None) -> np.ndarray:
    """One tensor of the workload, exactly as make_weights would hold it (every tensor has a random stream of its
    own, keyed by seed and name): lets a model too large for the host be walked layer by layer."""
    shape, gain = (specs or tensor_specs(w))[(prefix, key)]
    full = f"{prefix}.{key}"
    return _gain(w.wseed, full, shape[0]) if gain else _matrix(w.wseed, full, shape, w.dtype)


def make_weights(w: Workload, n_threads: int = 8) -> Tuple[Weights, Weights]:
    """(target, draft) weights.  The draft shares the target's embedding and LM head (by
    reference), has its own layers, final-norm gain, fusion matrix W_c and fusion-norm gain."""
    tgt, drf = Weights(w.dtype), Weights(w.dtype)
    specs = tensor_specs(w)

    def run(job):
        prefix, key = job
        (tgt if prefix == "t" else drf).t[key] = make_tensor(w, prefix, key, specs)

    if n_threads > 1:
        with ThreadPoolExecutor(n_threads) as ex:
            list(ex.map(run, list(specs)))
    else:
        for j in specs:
            run(j)
    drf.t["E"] = tgt.t["E"]
    drf.t["lm"] = tgt.t["lm"]
    return tgt, drf


# --------------------------------------------------------------------------------------
# prompts, page tables, uniforms
# --------------------------------------------------------------------------------------
def make_prompts(w: Workload) -> List[np.ndarray]:
    """One int32 token array per sequence; ids uniform in [0, vocab-1) so that the mask id
    (vocab-1) never occurs as data."""
    r = _rng(w.seed, "prompts")
    lens = r.integers(w.ctx_min, w.ctx_max + 1, size=w.n_seqs)
    return [r.integers(0, w.target.vocab - 1, size=int(n)).astype(np.int32) for n in lens]


def make_block_table(w: Workload, max_len: int, shuffle: bool = True,
                     extra_pages: int = 3) -> Tuple[np.ndarray, int]:
    """Page table [n_seqs, pages_per_seq] (int32) covering max_len tokens per sequence, pages
    handed out in a seeded shuffled order so that sequences are not contiguous in the pool.
    Returns (table, n_pages_in_pool)."""
    pps = (max_len + PAGE_SIZE - 1) // PAGE_SIZE
    n_pages = w.n_seqs * pps + extra_pages
    ids = np.arange(n_pages, dtype=np.int32)
    if shuffle:
        _rng(w.seed, "pages").shuffle(ids)
    return ids[: w.n_seqs * pps].reshape(w.n_seqs, pps).copy(), n_pages


def make_uniforms(w: Workload, step: int) -> np.ndarray:
    """Acceptance uniforms u[s, j] in [0, 1) as fp32, one draw per sequence and block slot."""
    return _rng(w.seed, f"uniforms{step}").random((w.n_seqs, w.block_size), dtype=np.float32)


def make_accept_plan(w: Workload, step: int = 0) -> np.ndarray:
    """Per-sequence number of correct proposals k_s in [0, block_size-1] for tests that feed
    verification with constructed proposals (true continuation for k_s slots, then a wrong one)."""
    return _rng(w.seed, f"plan{step}").integers(0, w.block_size, size=w.n_seqs).astype(np.int32)


# --------------------------------------------------------------------------------------
# synthetic cache state (stands in for a prefill at sizes the CPU oracle cannot prefill)
# --------------------------------------------------------------------------------------
def make_context_lengths(w: Workload) -> np.ndarray:
    """Committed length n_s of every sequence (the same draw as make_prompts uses)."""
    r = _rng(w.seed, "prompts")
    return r.integers(w.ctx_min, w.ctx_max + 1, size=w.n_seqs).astype(np.int64)


def make_state_rows(w: Workload, seq: int, pool: str, layer: int, n: int) -> Tuple[np.ndarray, np.ndarray]:
    """K and V rows [n, Hkv, hd] (fp32 holding bf16-representable values for a bf16 workload) of one layer
    of one sequence's cache: unit-variance normals, the scale real K rows have after k-norm and RoPE.
    pool: "target" | "draft"."""
    m = w.target if pool == "target" else w.draft
    r = _rng(w.seed, f"state.{w.name}.{seq}.{pool}.{layer}")
    out = []
    for _ in range(2):
        x = r.standard_normal((n, m.n_kv_heads, m.head_dim), dtype=np.float32)
        if w.dtype == "bf16":
            x = bf16_bits_to_f32(f32_to_bf16_bits(x)).reshape(x.shape)
        out.append(x)
    return out[0], out[1]


def make_anchor(w: Workload, seq: int) -> int:
    return int(_rng(w.seed, f"anchor.{w.name}.{seq}").integers(0, w.target.vocab - 1))
