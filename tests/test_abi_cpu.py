"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and validates
arguments before any launch (no kernel runs in this file)."""
import ctypes as C
import os
import re

import pytest

from paper_2601_13155_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return binding.load()


def test_exports_every_declared_symbol(lib):
    text = open(os.path.join(ROOT, "include", "spts.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(spts_[a-z_0-9]+)\s*\(", text))
    assert {"spts_probe_attn", "spts_probe_ffn", "spts_select_topk", "spts_layer_prefill", "spts_msdp_compact",
            "spts_decode_layer", "spts_greedy_token", "spts_channel_importance", "spts_select_topk_segmented", "spts_select_topk_batched", "spts_layer_prefill_batched", "spts_msdp_compact_batched", "spts_decode_layer_batched", "spts_greedy_token_batched"} <= declared
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(binding.EXPORTS)


def test_strerror(lib):
    assert lib.spts_strerror(0) == b"ok"
    for code in range(-6, 0):
        assert lib.spts_strerror(code) not in (b"ok", b"unknown status")
    assert lib.spts_strerror(-99) == b"unknown status"


def test_workspace_and_create_validation(lib):
    m = binding.model_desc(synth.TINY)
    nb = binding.spts_workspace_bytes(m, 512, 32, 16, 688)
    assert nb > 0 and nb % 256 == 0
    assert binding.spts_workspace_bytes(m, 1024, 32, 16, 688) > nb
    assert binding.spts_workspace_bytes(m, 0, 32, 16, 688) == 0
    bad = binding.model_desc(synth.TINY); bad.Hkv = 3
    assert binding.spts_workspace_bytes(bad, 512, 32, 16, 688) == 0
    h = C.c_void_p()
    fake_ws = C.c_void_p(1 << 20)   # never dereferenced: create only records it
    assert lib.spts_create(C.byref(h), C.byref(bad), None, fake_ws, nb, 512, 32, 16, 688) == binding.SPTS_ESHAPE
    bad2 = binding.model_desc(synth.TINY); bad2.dtype = 7
    assert lib.spts_create(C.byref(h), C.byref(bad2), None, fake_ws, nb, 512, 32, 16, 688) == binding.SPTS_EDTYPE
    assert lib.spts_create(C.byref(h), C.byref(m), None, fake_ws, nb - 1, 512, 32, 16, 688) == binding.SPTS_EWORKSPACE
    assert lib.spts_create(C.byref(h), C.byref(m), None, C.c_void_p((1 << 20) + 4), nb, 512, 32, 16, 688) == binding.SPTS_EALIGN
    assert lib.spts_create(C.byref(h), C.byref(m), None, None, nb, 512, 32, 16, 688) == binding.SPTS_EINVAL
    assert lib.spts_create(C.byref(h), C.byref(m), None, fake_ws, nb, 512, 32, 16, 688) == binding.SPTS_OK
    try:
        # argument errors are reported before anything is launched
        A = 1 << 21
        assert lib.spts_select_topk(h, A, 100, 101, 0, A) == binding.SPTS_EINVAL          # k > N
        assert lib.spts_select_topk(h, A, 100, -1, 0, A) == binding.SPTS_EINVAL
        assert lib.spts_select_topk(h, A, 100, 0, 0, None) == binding.SPTS_OK             # k == 0 writes nothing
        assert lib.spts_select_topk(h, A, 0, 0, 0, A) == binding.SPTS_OK                  # empty input
        assert lib.spts_select_topk(h, A + 4, 100, 10, 0, A) == binding.SPTS_EALIGN
        assert lib.spts_select_topk(h, None, 100, 10, 0, A) == binding.SPTS_EINVAL
        assert lib.spts_select_topk(h, A, 513, 10, 0, A) == binding.SPTS_EWORKSPACE       # N > max_tokens
        assert lib.spts_select_topk_batched(h, A, 100, 10, 0, -1, A) == binding.SPTS_EINVAL
        assert lib.spts_select_topk_batched(h, A, 100, 101, 0, 2, A) == binding.SPTS_EINVAL
        assert lib.spts_select_topk_batched(h, A, 100, 10, 0, 0, None) == binding.SPTS_OK  # empty batch
        w = binding.spts_layer_weights()
        assert lib.spts_probe_attn(h, A, A, 100, C.byref(w), 8, A, A) == binding.SPTS_EINVAL      # null weights
        w.Wq = w.Wk = w.gamma1 = A
        assert lib.spts_probe_attn(h, A, A, 100, C.byref(w), 0, A, A) == binding.SPTS_EINVAL      # P < 1
        assert lib.spts_probe_attn(h, A, A, 100, C.byref(w), 101, A, A) == binding.SPTS_EINVAL    # P > N
        assert lib.spts_probe_attn(h, A, A, 100, C.byref(w), 64, A, A) == binding.SPTS_EWORKSPACE  # P > max_probe
        assert lib.spts_probe_attn(h, A, A, 0, C.byref(w), 8, A, A) == binding.SPTS_OK            # N == 0
        cfg = binding.spts_layer_cfg(1, 8, -1, 10, 1, 0)
        assert lib.spts_layer_prefill(h, A, A, 100, C.byref(w), C.byref(cfg), None, None, None, None) == binding.SPTS_EINVAL
        so = (C.c_int64 * 3)(0, 60, 100); bud = (C.c_int64 * 2)(10, 10)
        bat = lambda offs, b, P, m1=bud: lib.spts_layer_prefill_batched(h, A, A, offs, b, C.byref(w), 1, P, m1, bud, 1, None, None, None, None)
        assert bat(so, -1, 8) == binding.SPTS_EINVAL
        assert bat(so, 0, 8) == binding.SPTS_OK                                            # empty batch
        assert bat(None, 2, 8) == binding.SPTS_EINVAL
        assert bat((C.c_int64 * 3)(4, 60, 100), 2, 8) == binding.SPTS_EINVAL               # offsets must start at 0
        assert bat((C.c_int64 * 3)(0, 60, 600), 2, 8) == binding.SPTS_EWORKSPACE           # more rows than max_tokens
        assert bat(so, 2, 8) == binding.SPTS_EINVAL                                        # incomplete weights
        assert lib.spts_msdp_compact_batched(h, A, A, A, so, 2, (C.c_int64 * 2)(10, -1), 1, A, A, A, None) == binding.SPTS_EINVAL
        assert lib.spts_msdp_compact_batched(h, A, A, A, so, 2, (C.c_int64 * 2)(0, 0), 1, None, None, None, None) == binding.SPTS_OK
        assert lib.spts_msdp_compact_batched(h, A, A, A, so, 2, bud, 1, A, A, A, None) == binding.SPTS_EINVAL  # x_out overlaps x_in
        assert lib.spts_msdp_compact(h, A, A, A, 100, -5, 1, A, A, A, None) == binding.SPTS_EINVAL
        assert lib.spts_msdp_compact(h, A, A, A, 100, 50, 1, A, A, A, None) == binding.SPTS_EINVAL  # x_out overlaps x_in
        assert lib.spts_last_hip_error(h) == 0
        assert lib.spts_uses_mfma(h) == 0                                                 # fp32 model: generic kernels
    finally:
        lib.spts_destroy(h)


def test_binding_fails_loudly_without_library(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libspts.so")
    with pytest.raises(RuntimeError):
        binding.load()


def test_host_slab_packing_layout():
    """runtime.pack_slab32 (the layout spts_pack_slab32 documents): element (s * rows + r) * 32 + j = a[r, 32 s + j]."""
    import numpy as np
    from paper_2601_13155_amd import runtime
    rows, K = 5, 96
    a = np.arange(rows * K, dtype=np.float32).reshape(rows, K)
    p = runtime.pack_slab32(a)
    assert p.shape == a.shape
    flat = p.reshape(-1)
    for r in range(rows):
        for k in range(K):
            assert flat[((k // 32) * rows + r) * 32 + k % 32] == a[r, k]
