"""Thin ctypes binding of the C ABI in include/dflash.h.

Argument marshalling only: every step of the speculative-decoding path runs inside the HIP
library.  PyTorch is used for device allocations and the current HIP stream, nothing else.
The binding fails loudly when the library has not been built (python -m paper_2602_06036_amd.build).
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdflash.so")

DFLASH_F32, DFLASH_BF16 = 0, 1
DFLASH_OK, DFLASH_EINVAL, DFLASH_ECAPACITY, DFLASH_EWORKSPACE, DFLASH_EHIP = 0, -1, -2, -3, -4
DFLASH_POOL_TARGET, DFLASH_POOL_DRAFT = 0, 1
PAGE_SIZE, MAX_TAPS = 16, 8

EXPORTS = [
    "dflash_target_blob_bytes", "dflash_draft_blob_bytes", "dflash_kv_pool_bytes", "dflash_workspace_bytes",
    "dflash_pack_target_head", "dflash_pack_target_layer", "dflash_pack_draft_head", "dflash_pack_draft_layer",
    "dflash_create", "dflash_destroy", "dflash_last_error", "dflash_device_status",
    "dflash_draft_block", "dflash_verify", "dflash_accept", "dflash_kv_commit",
    "dflash_prefill", "dflash_accept_sampled_noalloc", "dflash_kv_read", "dflash_kv_write", "dflash_profile_enable", "dflash_profile_read", "dflash_moe_stats", "dflash_moe_trace", "dflash_gemm_counts",
    "dflash_probe_hbm_read", "dflash_probe_mfma",
]


class Dims(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float), ("qk_norm", C.c_int32), ("dtype", C.c_int32)] + \
               [(n, C.c_int32) for n in ("n_experts", "top_k", "d_expert")]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2", "qn", "kn", "wr")]


class Runtime(C.Structure):
    _fields_ = [("block_size", C.c_int32), ("max_seqs", C.c_int32), ("max_pages_per_seq", C.c_int32), ("n_pages", C.c_int32),
                ("n_taps", C.c_int32), ("tap_layers", C.c_int32 * MAX_TAPS), ("mask_token_id", C.c_int32),
                ("target_kv_pool", C.c_void_p), ("draft_kv_pool", C.c_void_p), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_size_t)]


class Batch(C.Structure):
    _fields_ = [("n_seqs", C.c_int32), ("max_seq_len", C.c_int32), ("seq_lens", C.c_void_p), ("block_table", C.c_void_p),
                ("anchor", C.c_void_p), ("block_size", C.c_int32)]


class DFlashError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"dflash error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2602_06036_amd.build` "
                              "(there is no CPU fallback)")
        l = C.CDLL(LIB_PATH)
        P, I, F = C.c_void_p, C.c_int32, C.c_float
        l.dflash_target_blob_bytes.restype = C.c_size_t
        l.dflash_target_blob_bytes.argtypes = [C.POINTER(Dims)]
        l.dflash_draft_blob_bytes.restype = C.c_size_t
        l.dflash_draft_blob_bytes.argtypes = [C.POINTER(Dims), I, I]
        l.dflash_kv_pool_bytes.restype = C.c_size_t
        l.dflash_kv_pool_bytes.argtypes = [C.POINTER(Dims), I]
        l.dflash_workspace_bytes.restype = C.c_size_t
        l.dflash_workspace_bytes.argtypes = [C.POINTER(Dims), C.POINTER(Dims), C.POINTER(Runtime)]
        l.dflash_pack_target_head.argtypes = [C.POINTER(Dims), P, P, P, P, P]
        l.dflash_pack_target_layer.argtypes = [C.POINTER(Dims), I, C.POINTER(LayerWeights), P, P]
        l.dflash_pack_draft_head.argtypes = [C.POINTER(Dims), I, I, P, P, P, P, P]
        l.dflash_pack_draft_layer.argtypes = [C.POINTER(Dims), I, I, I, C.POINTER(LayerWeights), P, P]
        l.dflash_create.argtypes = [C.POINTER(Dims), P, C.POINTER(Dims), P, C.POINTER(Runtime), C.POINTER(P)]
        l.dflash_destroy.argtypes = [P]
        l.dflash_last_error.restype = C.c_char_p
        l.dflash_last_error.argtypes = [P]
        l.dflash_device_status.argtypes = [P, P]
        l.dflash_draft_block.argtypes = [P, C.POINTER(Batch), F, P, P, P, P]
        l.dflash_verify.argtypes = [P, C.POINTER(Batch), P, P, P, P]
        l.dflash_accept.argtypes = [P, C.POINTER(Batch), P, P, F, P, P, P, P, P]
        l.dflash_kv_commit.argtypes = [P, C.POINTER(Batch), P, P, P, P]
        l.dflash_prefill.argtypes = [P, C.POINTER(Batch), P, C.POINTER(C.c_int32), P, P]
        l.dflash_accept_sampled_noalloc.argtypes = [P, P, P, P, P, F, I, I, I, P, P, P]
        l.dflash_kv_read.argtypes = [P, C.POINTER(Batch), I, I, I, I, I, P, P, P]
        l.dflash_kv_write.argtypes = [P, C.POINTER(Batch), I, I, I, I, I, P, P, P]
        l.dflash_profile_enable.argtypes = [P, I]
        l.dflash_profile_read.argtypes = [P, P, C.POINTER(C.c_float), C.POINTER(C.c_int32), C.POINTER(C.c_double)]
        l.dflash_moe_stats.argtypes = [P, P, C.POINTER(C.c_int64)]
        l.dflash_moe_trace.argtypes = [P, P]
        l.dflash_gemm_counts.argtypes = [P, P]
        for name in EXPORTS:
            if name not in ("dflash_target_blob_bytes", "dflash_draft_blob_bytes", "dflash_kv_pool_bytes",
                            "dflash_workspace_bytes", "dflash_last_error"):
                getattr(l, name).restype = C.c_int
        _lib = l
    return _lib


def make_dims(m, dtype: str) -> Dims:
    """m: any object with the ModelDims attributes."""
    return Dims(m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.d_ffn, m.vocab,
                float(m.rope_theta), float(m.rms_eps), int(bool(m.qk_norm)),
                DFLASH_BF16 if dtype == "bf16" else DFLASH_F32,
                int(getattr(m, "n_experts", 0)), int(getattr(m, "top_k", 0)), int(getattr(m, "d_expert", 0)))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous()
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(rc: int, ctx=None):
    if rc != DFLASH_OK:
        raise DFlashError(rc, lib().dflash_last_error(ctx).decode())


def _layer_struct(w: Dict[str, torch.Tensor]) -> LayerWeights:
    return LayerWeights(*[_ptr(w.get(k)) for k in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2", "qn", "kn", "wr")])


class Engine:
    """Owns the device buffers (torch tensors) that the C library works on, and the context."""

    def __init__(self, target, draft, dtype: str, block_size: int, max_seqs: int, max_pages_per_seq: int,
                 n_pages: int, tap_layers: Sequence[int], mask_token_id: int, device: str = "cuda:0", blobs=None):
        self.l = lib()
        self.device = torch.device(device)
        self.dtype = dtype
        self.target, self.draft = target, draft
        self.td, self.dd = make_dims(target, dtype), make_dims(draft, dtype)
        self.B, self.max_seqs, self.max_pages_per_seq, self.n_pages = block_size, max_seqs, max_pages_per_seq, n_pages
        self.n_taps = len(tap_layers)
        rt = Runtime()
        rt.block_size, rt.max_seqs, rt.max_pages_per_seq, rt.n_pages = block_size, max_seqs, max_pages_per_seq, n_pages
        rt.n_taps = self.n_taps
        for i, t in enumerate(tap_layers):
            rt.tap_layers[i] = int(t)
        rt.mask_token_id = mask_token_id
        self.rt = rt
        tb = self.l.dflash_target_blob_bytes(C.byref(self.td))
        db = self.l.dflash_draft_blob_bytes(C.byref(self.dd), self.n_taps, target.d_model)
        if tb == 0 or db == 0:
            _check(DFLASH_EINVAL)
        if blobs is not None:                      # already-packed weights of the same models (shared between engines)
            self.target_blob, self.draft_blob = blobs
            assert self.target_blob.numel() == tb and self.draft_blob.numel() == db
        else:
            self.target_blob = torch.empty(tb, dtype=torch.uint8, device=self.device)
            self.draft_blob = torch.empty(db, dtype=torch.uint8, device=self.device)
        self.ctx = None

    # ---- weights -------------------------------------------------------------------------------
    def pack_target_head(self, embed, lm_head, final_gain):
        _check(self.l.dflash_pack_target_head(C.byref(self.td), _ptr(embed), _ptr(lm_head), _ptr(final_gain),
                                              _ptr(self.target_blob), _stream()))

    def pack_target_layer(self, layer: int, w: Dict[str, torch.Tensor]):
        s = _layer_struct(w)
        _check(self.l.dflash_pack_target_layer(C.byref(self.td), layer, C.byref(s), _ptr(self.target_blob), _stream()))

    def pack_draft_head(self, w_c, g_c, final_gain):
        _check(self.l.dflash_pack_draft_head(C.byref(self.dd), self.n_taps, self.target.d_model, _ptr(w_c), _ptr(g_c),
                                             _ptr(final_gain), _ptr(self.draft_blob), _stream()))

    def pack_draft_layer(self, layer: int, w: Dict[str, torch.Tensor]):
        s = _layer_struct(w)
        _check(self.l.dflash_pack_draft_layer(C.byref(self.dd), self.n_taps, self.target.d_model, layer, C.byref(s),
                                              _ptr(self.draft_blob), _stream()))

    # ---- context -------------------------------------------------------------------------------
    def create(self):
        tp = self.l.dflash_kv_pool_bytes(C.byref(self.td), self.n_pages)
        dp = self.l.dflash_kv_pool_bytes(C.byref(self.dd), self.n_pages)
        ws = self.l.dflash_workspace_bytes(C.byref(self.td), C.byref(self.dd), C.byref(self.rt))
        if tp == 0 or dp == 0 or ws == 0:
            _check(DFLASH_EINVAL)
        self.target_pool = torch.zeros(tp, dtype=torch.uint8, device=self.device)
        self.draft_pool = torch.zeros(dp, dtype=torch.uint8, device=self.device)
        self.workspace = torch.zeros(ws, dtype=torch.uint8, device=self.device)
        self.rt.target_kv_pool, self.rt.draft_kv_pool = _ptr(self.target_pool), _ptr(self.draft_pool)
        self.rt.workspace, self.rt.workspace_bytes = _ptr(self.workspace), ws
        torch.cuda.synchronize(self.device)
        h = C.c_void_p()
        _check(self.l.dflash_create(C.byref(self.td), _ptr(self.target_blob), C.byref(self.dd), _ptr(self.draft_blob),
                                    C.byref(self.rt), C.byref(h)))
        self.ctx = h
        return self

    def close(self):
        if self.ctx is not None:
            self.l.dflash_destroy(self.ctx)
            self.ctx = None

    def batch(self, seq_lens: torch.Tensor, block_table: torch.Tensor, anchor: torch.Tensor, max_seq_len: int,
              block_size: int = 0) -> Batch:
        """block_size: rows per sequence of the calls made with this batch (0 = the context's block size)."""
        assert seq_lens.dtype == torch.int32 and block_table.dtype == torch.int32 and anchor.dtype == torch.int32
        assert block_table.shape == (seq_lens.shape[0], self.max_pages_per_seq)
        return Batch(int(seq_lens.shape[0]), int(max_seq_len), _ptr(seq_lens), _ptr(block_table), _ptr(anchor), int(block_size))

    def profile_enable(self, on: bool):
        _check(self.l.dflash_profile_enable(self.ctx, int(on)), self.ctx)

    def profile_read(self):
        """{class index: (ms, launches, algorithmic bytes)} since the last read."""
        n = 8
        ms, cnt, by = (C.c_float * n)(), (C.c_int32 * n)(), (C.c_double * n)()
        _check(self.l.dflash_profile_read(self.ctx, _stream(), ms, cnt, by), self.ctx)
        return {i: (float(ms[i]), int(cnt[i]), float(by[i])) for i in range(n) if cnt[i]}

    def moe_stats(self):
        """(routing launches, experts reached, 16-row bands, work items) since the last read, and the bands per work
        item of the last routing launch; routed-expert targets only."""
        out = (C.c_int64 * 5)()
        _check(self.l.dflash_moe_stats(self.ctx, _stream(), out), self.ctx)
        return int(out[0]), int(out[1]), int(out[2]), int(out[3]), int(out[4])

    def gemm_counts(self):
        """GEMM launches per kernel family since the last call: (streaming, tiled4, tiled8, few_rows, grouped, f32)."""
        out = (C.c_int64 * 6)()
        _check(self.l.dflash_gemm_counts(self.ctx, out), self.ctx)
        return tuple(int(v) for v in out)

    def moe_trace(self, on: bool = True):
        """Routed-expert targets: a [n_layers, max_seqs * B, top_k] int32 tensor that every following verify / prefill pass
        fills with the experts chosen per layer and row (None and off with on=False)."""
        if not on:
            _check(self.l.dflash_moe_trace(self.ctx, None), self.ctx)
            self._moe_trace = None
            return None
        self._moe_trace = torch.full((self.target.n_layers, self.max_seqs * self.B, self.target.top_k), -1, dtype=torch.int32, device=self.device)
        _check(self.l.dflash_moe_trace(self.ctx, _ptr(self._moe_trace)), self.ctx)
        return self._moe_trace

    def device_status(self):
        _check(self.l.dflash_device_status(self.ctx, _stream()), self.ctx)


# ---- the four calls of the step (same names as the C ABI) ------------------------------------------
def dflash_draft_block(e: Engine, batch: Batch, draft_tokens: torch.Tensor, temperature: float = 0.0,
                       rng_key: Optional[torch.Tensor] = None, logits_out: Optional[torch.Tensor] = None):
    _check(e.l.dflash_draft_block(e.ctx, C.byref(batch), float(temperature), _ptr(rng_key), _ptr(draft_tokens),
                                  _ptr(logits_out), _stream()), e.ctx)


def dflash_verify(e: Engine, batch: Batch, tokens: torch.Tensor, tgt_argmax: Optional[torch.Tensor],
                  logits_out: Optional[torch.Tensor] = None):
    _check(e.l.dflash_verify(e.ctx, C.byref(batch), _ptr(tokens), _ptr(tgt_argmax), _ptr(logits_out), _stream()), e.ctx)


def dflash_accept(e: Engine, batch: Batch, draft_tokens: torch.Tensor, tgt_argmax: torch.Tensor, accept_len: torch.Tensor,
                  out_tokens: torch.Tensor, temperature: float = 0.0, uniforms: Optional[torch.Tensor] = None,
                  rng_key: Optional[torch.Tensor] = None):
    _check(e.l.dflash_accept(e.ctx, C.byref(batch), _ptr(draft_tokens), _ptr(tgt_argmax), float(temperature), _ptr(uniforms),
                             _ptr(rng_key), _ptr(accept_len), _ptr(out_tokens), _stream()), e.ctx)


def dflash_accept_sampled_noalloc(target_logits: torch.Tensor, draft_logits: torch.Tensor, draft_tokens: torch.Tensor, uniforms: torch.Tensor,
                                  rng_key: torch.Tensor, temperature: float, accept_len: torch.Tensor, out_tokens: torch.Tensor):
    """Speculative-sampling acceptance on logits the caller holds, [S, B, V] fp32 each; no context, no workspace."""
    S, Bk, V = target_logits.shape
    assert draft_logits.shape == target_logits.shape and target_logits.dtype == torch.float32 and draft_logits.dtype == torch.float32
    _check(lib().dflash_accept_sampled_noalloc(_ptr(target_logits), _ptr(draft_logits), _ptr(draft_tokens), _ptr(uniforms), _ptr(rng_key),
                                               float(temperature), int(S), int(Bk), int(V), _ptr(accept_len), _ptr(out_tokens), _stream()))


def dflash_kv_commit(e: Engine, batch: Batch, accept_len: torch.Tensor, out_tokens: torch.Tensor,
                     kv_slots_out: Optional[torch.Tensor] = None):
    _check(e.l.dflash_kv_commit(e.ctx, C.byref(batch), _ptr(accept_len), _ptr(out_tokens), _ptr(kv_slots_out), _stream()), e.ctx)


def dflash_prefill(e: Engine, batch: Batch, tokens: torch.Tensor, prompt_lens, first_tokens: Optional[torch.Tensor] = None):
    """tokens: int32 device tensor, the new tokens of all sequences concatenated; prompt_lens: host ints, one per sequence."""
    assert tokens.dtype == torch.int32 and tokens.is_contiguous() and int(tokens.numel()) == int(sum(prompt_lens))
    lens = (C.c_int32 * len(prompt_lens))(*[int(x) for x in prompt_lens])
    _check(e.l.dflash_prefill(e.ctx, C.byref(batch), _ptr(tokens), lens, _ptr(first_tokens), _stream()), e.ctx)


def dflash_kv_read(e: Engine, batch: Batch, pool: int, layer: int, seq: int, start: int, count: int):
    m = e.target if pool == DFLASH_POOL_TARGET else e.draft
    k = torch.empty((count, m.n_kv_heads, m.head_dim), dtype=torch.float32, device=e.device)
    v = torch.empty_like(k)
    _check(e.l.dflash_kv_read(e.ctx, C.byref(batch), pool, layer, seq, start, count, _ptr(k), _ptr(v), _stream()), e.ctx)
    return k, v


def dflash_kv_write(e: Engine, batch: Batch, pool: int, layer: int, seq: int, start: int, k: torch.Tensor, v: torch.Tensor):
    assert k.dtype == torch.float32 and v.dtype == torch.float32 and k.shape == v.shape
    _check(e.l.dflash_kv_write(e.ctx, C.byref(batch), pool, layer, seq, start, int(k.shape[0]), _ptr(k), _ptr(v), _stream()), e.ctx)


# ---- machine probes (same names as the C ABI) -----------------------------------------------------------
def dflash_probe_hbm_read(buf: torch.Tensor, bytes_per_launch: int, launches: int) -> float:
    """Milliseconds for `launches` read-only streaming kernels over consecutive pieces of `buf`."""
    assert buf.is_cuda and buf.is_contiguous() and buf.numel() * buf.element_size() >= bytes_per_launch * launches
    ms = C.c_float()
    _check(lib().dflash_probe_hbm_read(C.c_void_p(buf.data_ptr()), C.c_size_t(bytes_per_launch), launches, C.byref(ms), _stream()))
    return float(ms.value)


def dflash_probe_mfma(shape: int, workgroups: int, iters: int):
    """(milliseconds, flops) of one kernel of register-resident bf16 MFMAs (shape 0: 16x16x32, 1: 32x32x16)."""
    ms, fl = C.c_float(), C.c_double()
    _check(lib().dflash_probe_mfma(shape, workgroups, iters, C.byref(ms), C.byref(fl), _stream()))
    return float(ms.value), float(fl.value)
