"""CPU-side checks of the C ABI: the library loads, exports every symbol the header declares,
and its size / argument-validation entry points (which launch nothing) behave."""
import ctypes as C
import os
import re

import pytest

from synth import inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2602_06036_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2602_06036_amd import build
        build.build(verbose=False)
    return binding


def test_every_declared_symbol_is_exported(B):
    hdr = open(os.path.join(ROOT, "include", "dflash.h")).read()
    declared = sorted(set(re.findall(r"\b(dflash_[a-z_]+)\s*\(", hdr)))
    assert set(declared) == set(B.EXPORTS)
    l = B.lib()
    for name in declared:
        assert hasattr(l, name), name


def test_struct_sizes_match_the_header(B):
    assert C.sizeof(B.Dims) == 14 * 4
    assert C.sizeof(B.LayerWeights) == 12 * 8
    assert C.sizeof(B.Batch) == 8 + 3 * 8 + 8          # block_size and the padding behind it
    assert C.sizeof(B.Runtime) == 4 * 4 + 4 + 8 * 4 + 4 + 4 * 8   # incl. no padding surprises
    

def test_sizes_for_the_8b_shape(B):
    w = si.workload(2)
    l = B.lib()
    td, dd = B.make_dims(w.target, "bf16"), B.make_dims(w.draft, "bf16")
    per_layer = (6144 * 4096 + 4096 * 4096 + 2 * 12288 * 4096 + 4096 * 12288) * 2
    tb = l.dflash_target_blob_bytes(C.byref(td))
    assert 36 * per_layer + 2 * 151936 * 4096 * 2 <= tb <= 36 * per_layer + 2 * 151936 * 4096 * 2 + 36 * 40000 + 20000
    # 147456 bytes of target KV per token (36 layers x 2 x 8 heads x 128 x 2 bytes)
    assert l.dflash_kv_pool_bytes(C.byref(td), 10) == 10 * 16 * 147456
    assert l.dflash_kv_pool_bytes(C.byref(dd), 10) == 10 * 16 * 20480
    db = l.dflash_draft_blob_bytes(C.byref(dd), 5, 4096)
    assert db >= 5 * per_layer + 4096 * 20480 * 2 + 5 * 2 * 1024 * 4096 * 2


def test_routed_expert_sizes_and_shape_checks(B):
    """Blob and workspace sizes of the 30B-A3B-shaped mixture-of-experts target (48 layers, 128 experts of width 768,
    8 per token), and the shapes the routed-expert path refuses."""
    from dataclasses import replace
    w = si.qwen3_30b_a3b_workload(1, 2048)
    l = B.lib()
    td, dd = B.make_dims(w.target, "bf16"), B.make_dims(w.draft, "bf16")
    m = w.target
    experts = 128 * 3 * 768 * 2048 * 2
    attn = ((32 + 2 * 4) * 128 * 2048 + 2048 * 32 * 128) * 2
    tb = l.dflash_target_blob_bytes(C.byref(td))
    lo = 48 * (experts + attn + 128 * 2048 * 2) + 2 * m.vocab * 2048 * 2
    assert lo <= tb <= lo + 48 * 40000 + 20000
    rt = B.Runtime()
    rt.block_size, rt.max_seqs, rt.max_pages_per_seq, rt.n_pages, rt.n_taps, rt.mask_token_id = 16, 32, 130, 32 * 130, 5, 7
    for i, t in enumerate(w.tap_layers):
        rt.tap_layers[i] = t
    ws_moe = l.dflash_workspace_bytes(C.byref(td), C.byref(dd), C.byref(rt))
    dense = B.make_dims(replace(m, n_experts=0, top_k=0, d_expert=0), "bf16")
    ws_dense = l.dflash_workspace_bytes(C.byref(dense), C.byref(dd), C.byref(rt))
    n_pos = 512 * 8 + 15 * 128        # every expert's share of the 4096 (row, expert) pairs padded to 16 rows, at most
    # list-ordered copy of the rows, their SwiGLU products (hi+lo bf16 pairs), the experts' fp32 outputs
    assert ws_moe - ws_dense >= n_pos * (2048 * 4 + 768 * 4 + 2048 * 4)
    assert ws_moe - ws_dense <= n_pos * (2048 * 4 + 768 * 4 + 2048 * 4) + 3 * 4096 * 4 + n_pos * 4 + 600 * 16 + 16 * 256
    for bad in (replace(m, n_experts=24), replace(m, top_k=0), replace(m, top_k=17), replace(m, d_expert=96),
                replace(m, n_experts=512), replace(m, n_experts=0)):
        assert l.dflash_target_blob_bytes(C.byref(B.make_dims(bad, "bf16"))) == 0
        assert l.dflash_last_error(None)
    assert l.dflash_target_blob_bytes(C.byref(B.make_dims(m, "f32"))) == 0            # bf16 only
    assert l.dflash_workspace_bytes(C.byref(td), C.byref(td), C.byref(rt)) == 0       # the drafter is dense


def test_bad_shapes_are_rejected_with_a_message(B):
    from dataclasses import replace
    w = si.workload(2)
    l = B.lib()
    bad = B.make_dims(replace(w.target, d_model=4100), "bf16")
    assert l.dflash_target_blob_bytes(C.byref(bad)) == 0
    assert b"multiples of 32" in l.dflash_last_error(None)
    bad = B.make_dims(replace(w.target, n_q_heads=30), "bf16")
    assert l.dflash_target_blob_bytes(C.byref(bad)) == 0
    td, dd = B.make_dims(w.target, "bf16"), B.make_dims(w.draft, "bf16")
    rt = B.Runtime()
    rt.block_size, rt.max_seqs, rt.max_pages_per_seq, rt.n_pages, rt.n_taps = 17, 1, 8, 8, 5
    assert l.dflash_workspace_bytes(C.byref(td), C.byref(dd), C.byref(rt)) == 0
    assert b"block_size" in l.dflash_last_error(None)
    rt.block_size = 16
    for i, t in enumerate((1, 9, 9, 25, 33)):
        rt.tap_layers[i] = t
    rt.mask_token_id = 151935
    assert l.dflash_workspace_bytes(C.byref(td), C.byref(dd), C.byref(rt)) == 0   # taps not ascending
    for i, t in enumerate((1, 9, 17, 25, 33)):
        rt.tap_layers[i] = t
    ws = l.dflash_workspace_bytes(C.byref(td), C.byref(dd), C.byref(rt))
    # decode-time temporaries stay small: two [16, V] fp32 logit buffers dominate
    assert 2 * 16 * 151936 * 4 < ws < 96 << 20
    out = C.c_void_p()
    assert l.dflash_create(C.byref(td), None, C.byref(dd), None, C.byref(rt), C.byref(out)) == B.DFLASH_EINVAL
    assert out.value is None


def _runtime(B, max_seqs, pages_per_seq, block=16):
    rt = B.Runtime()
    rt.block_size, rt.max_seqs, rt.max_pages_per_seq, rt.n_pages, rt.n_taps = block, max_seqs, pages_per_seq, max_seqs * pages_per_seq, 5
    for i, t in enumerate((1, 9, 17, 25, 33)):
        rt.tap_layers[i] = t
    rt.mask_token_id = 151935
    return rt


def test_workspace_grows_monotonically_with_batch_and_context(B):
    """Host-side sizing: a context created for more sequences or longer block tables never needs less
    workspace (callers size once for their largest batch), and configuration 5 stays far below the HBM size."""
    w = si.workload(2)
    l = B.lib()
    td, dd = B.make_dims(w.target, "bf16"), B.make_dims(w.draft, "bf16")
    prev = 0
    for s in (1, 2, 3, 4, 7, 8, 16, 31, 32, 33, 64):
        ws = l.dflash_workspace_bytes(C.byref(td), C.byref(dd), C.byref(_runtime(B, s, 160)))
        assert ws >= prev > -1, (s, ws, prev)
        prev = ws
    prev = 0
    for pages in (1, 2, 8, 64, 129, 512, 1030, 4096, 8192):
        ws = l.dflash_workspace_bytes(C.byref(td), C.byref(dd), C.byref(_runtime(B, 4, pages)))
        assert ws >= prev, (pages, ws, prev)
        prev = ws
    ws5 = l.dflash_workspace_bytes(C.byref(td), C.byref(dd), C.byref(_runtime(B, 32, 8192 // 16 + 2)))
    assert 2 * 512 * 151936 * 4 < ws5 < 3 << 30


def test_step_calls_reject_null_handles_before_touching_the_device(B):
    l = B.lib()
    batch = B.Batch(1, 0, None, None, None)
    assert l.dflash_draft_block(None, C.byref(batch), C.c_float(0.0), None, None, None, None) == B.DFLASH_EINVAL
    assert l.dflash_verify(None, C.byref(batch), None, None, None, None) == B.DFLASH_EINVAL
    assert l.dflash_accept(None, C.byref(batch), None, None, C.c_float(0.0), None, None, None, None, None) == B.DFLASH_EINVAL
    assert l.dflash_kv_commit(None, C.byref(batch), None, None, None, None) == B.DFLASH_EINVAL
    assert b"ctx" in l.dflash_last_error(None)
    counts = (C.c_int64 * 6)()
    assert l.dflash_gemm_counts(None, counts) == B.DFLASH_EINVAL
    assert l.dflash_moe_trace(None, None) == B.DFLASH_EINVAL
    assert l.dflash_destroy(None) in (B.DFLASH_OK, B.DFLASH_EINVAL)
