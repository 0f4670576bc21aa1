"""ctypes binding of libspts (include/spts.h): argument marshalling only.

Every function has the name and argument order of its C entry point and takes
torch tensors that live on the GPU (PyTorch is used for device memory and
streams only).  No step of the method is computed here, and there is no CPU
fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspts.so")

SPTS_OK = 0
SPTS_EINVAL, SPTS_ESHAPE, SPTS_EALIGN, SPTS_EWORKSPACE, SPTS_EDTYPE, SPTS_EHIP = -1, -2, -3, -4, -5, -6
SPTS_F32, SPTS_BF16 = 0, 1

EXPORTS = (
    "spts_workspace_bytes", "spts_create", "spts_destroy", "spts_strerror", "spts_last_hip_error", "spts_uses_mfma",
    "spts_probe_attn", "spts_probe_ffn", "spts_select_topk", "spts_select_topk_static", "spts_select_topk_batched", "spts_select_topk_segmented", "spts_layer_prefill", "spts_layer_prefill_batched", "spts_msdp_compact", "spts_msdp_compact_batched",
    "spts_decode_layer", "spts_decode_layer_batched", "spts_greedy_token", "spts_greedy_token_batched", "spts_channel_importance",
    "spts_pack_slab32",
    "spts_profile_begin", "spts_profile_end", "spts_profile_count", "spts_profile_get",
)


class spts_model_desc(C.Structure):
    _fields_ = [("D", C.c_int32), ("H", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32), ("Dff", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float), ("dtype", C.c_int32)]


class spts_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("Wq", "Wk", "Wv", "Wo", "gamma1", "Wgate", "Wup", "Wdown", "gamma2",
                                           "Ug", "Vg", "Uu", "Vu", "Ud", "Vd")] + [("r", C.c_int32), ("Dlow", C.c_int32)] + \
               [(n, C.c_void_p) for n in ("Wq_s", "Wk_s", "Wv_s", "Wo_s", "Wgate_s", "Wup_s", "Wdown_s", "Vg_s", "Vu_s", "Vd_s", "Ug_s", "Uu_s")] + \
               [("Ud_orthonormal", C.c_int32)]


class spts_layer_cfg(C.Structure):
    _fields_ = [("skip", C.c_int32), ("probe_len", C.c_int32), ("m_attn", C.c_int64), ("m_ffn", C.c_int64),
                ("protect_last", C.c_int32), ("kv_mode", C.c_int32)]


class spts_kv_out(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("pos", C.c_void_p), ("capacity", C.c_int64), ("count", C.c_int64)]


_lib = None


def load() -> C.CDLL:
    """Loads libspts.so built in-tree; raises if it is missing (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` first")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.spts_workspace_bytes.restype = C.c_size_t
    lib.spts_workspace_bytes.argtypes = [C.POINTER(spts_model_desc), i64, i32, i32, i32]
    lib.spts_create.restype = C.c_int
    lib.spts_create.argtypes = [C.POINTER(vp), C.POINTER(spts_model_desc), vp, vp, C.c_size_t, i64, i32, i32, i32]
    lib.spts_destroy.restype = None
    lib.spts_destroy.argtypes = [vp]
    lib.spts_strerror.restype = C.c_char_p
    lib.spts_strerror.argtypes = [C.c_int]
    lib.spts_last_hip_error.restype = C.c_int
    lib.spts_last_hip_error.argtypes = [vp]
    lib.spts_uses_mfma.restype = C.c_int
    lib.spts_uses_mfma.argtypes = [vp]
    lib.spts_probe_attn.restype = C.c_int
    lib.spts_probe_attn.argtypes = [vp, vp, vp, i64, C.POINTER(spts_layer_weights), i32, vp, vp]
    lib.spts_probe_ffn.restype = C.c_int
    lib.spts_probe_ffn.argtypes = [vp, vp, i64, C.POINTER(spts_layer_weights), vp, vp, vp]
    lib.spts_select_topk.restype = C.c_int
    lib.spts_select_topk.argtypes = [vp, vp, i64, i64, i32, vp]
    lib.spts_select_topk_static.restype = C.c_int
    lib.spts_select_topk_static.argtypes = [vp, vp, i64, i64, i32, vp]
    lib.spts_select_topk_batched.restype = C.c_int
    lib.spts_select_topk_batched.argtypes = [vp, vp, i64, i64, i32, i32, vp]
    lib.spts_select_topk_segmented.restype = C.c_int
    lib.spts_select_topk_segmented.argtypes = [vp, vp, vp, vp, vp, i32, i64, i32, vp]
    lib.spts_layer_prefill.restype = C.c_int
    lib.spts_layer_prefill.argtypes = [vp, vp, vp, i64, C.POINTER(spts_layer_weights), C.POINTER(spts_layer_cfg),
                                       C.POINTER(spts_kv_out), vp, vp, vp]
    lib.spts_layer_prefill_batched.restype = C.c_int
    lib.spts_layer_prefill_batched.argtypes = [vp, vp, vp, C.POINTER(C.c_int64), i32, C.POINTER(spts_layer_weights), i32, i32,
                                               C.POINTER(C.c_int64), C.POINTER(C.c_int64), i32, C.POINTER(spts_kv_out),
                                               vp, vp, vp]
    lib.spts_msdp_compact.restype = C.c_int
    lib.spts_msdp_compact.argtypes = [vp, vp, vp, vp, i64, i64, i32, vp, vp, vp, vp]
    lib.spts_msdp_compact_batched.restype = C.c_int
    lib.spts_msdp_compact_batched.argtypes = [vp, vp, vp, vp, C.POINTER(C.c_int64), i32, C.POINTER(C.c_int64), i32, vp, vp, vp, vp]
    lib.spts_decode_layer.restype = C.c_int
    lib.spts_decode_layer.argtypes = [vp, vp, i32, C.POINTER(spts_layer_weights), C.POINTER(spts_kv_out)]
    lib.spts_decode_layer_batched.restype = C.c_int
    lib.spts_decode_layer_batched.argtypes = [vp, vp, C.POINTER(C.c_int32), i32, C.POINTER(spts_layer_weights), C.POINTER(spts_kv_out)]
    lib.spts_greedy_token_batched.restype = C.c_int
    lib.spts_greedy_token_batched.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp]
    lib.spts_greedy_token.restype = C.c_int
    lib.spts_greedy_token.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp]
    lib.spts_channel_importance.restype = C.c_int
    lib.spts_channel_importance.argtypes = [vp, vp, i64, C.POINTER(spts_layer_weights), i64, vp]
    lib.spts_pack_slab32.restype = C.c_int
    lib.spts_pack_slab32.argtypes = [vp, vp, i64, i64, vp]
    lib.spts_profile_begin.restype = C.c_int
    lib.spts_profile_begin.argtypes = [vp]
    lib.spts_profile_end.restype = C.c_int
    lib.spts_profile_end.argtypes = [vp]
    lib.spts_profile_count.restype = C.c_int
    lib.spts_profile_count.argtypes = [vp]
    lib.spts_profile_get.restype = C.c_int
    lib.spts_profile_get.argtypes = [vp, C.c_int, C.POINTER(C.c_char_p), C.POINTER(C.c_double), C.POINTER(i64)]
    _lib = lib
    return lib


class SptsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {load().spts_strerror(status).decode()} ({status})")


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _check(status: int, where: str):
    if status != SPTS_OK:
        raise SptsError(status, where)


def model_desc(shape) -> spts_model_desc:
    """shape: any object with D, H, Hkv, d, Dff, rms_eps, rope_base, dtype ('f32' | 'bf16')."""
    return spts_model_desc(shape.D, shape.H, shape.Hkv, shape.d, shape.Dff, shape.rms_eps, shape.rope_base,
                           SPTS_BF16 if shape.dtype == "bf16" else SPTS_F32)


def layer_weights(tensors: dict, r: int = 0, Dlow: int = 0, ud_orthonormal: bool = False) -> spts_layer_weights:
    """tensors: name -> device tensor in the ABI layout ([d_out, d_in]); missing names become NULL.
    ud_orthonormal: the caller's statement that Ud has orthonormal columns (see spts_layer_weights in spts.h)."""
    w = spts_layer_weights()
    for name, typ in spts_layer_weights._fields_:
        if typ is C.c_void_p:
            setattr(w, name, _ptr(tensors.get(name)))
    w.r, w.Dlow = int(r), int(Dlow)
    w.Ud_orthonormal = 1 if ud_orthonormal else 0
    w._keepalive = tensors  # keep the device tensors referenced as long as the struct lives
    return w


def spts_workspace_bytes(model: spts_model_desc, max_tokens: int, max_probe: int, max_r: int, max_dlow: int) -> int:
    return int(load().spts_workspace_bytes(C.byref(model), max_tokens, max_probe, max_r, max_dlow))


SPTS_TOPK_STATIC_MAX_N = 1048576


def spts_select_topk_static(stream, scores, N: int, k: int, protect_last: int, idx_out):
    """Context-free TopK on the library's own static scratch; stream: a torch stream, a raw hipStream_t or None."""
    h = getattr(stream, "cuda_stream", stream)
    _check(load().spts_select_topk_static(h, _ptr(scores), N, k, protect_last, _ptr(idx_out)), "spts_select_topk_static")


class Context:
    """Owns an spts_ctx and its workspace tensor (allocated through torch on the current device)."""

    def __init__(self, shape, max_tokens: int, max_probe: int, max_r: int, max_dlow: int, stream=None):
        import torch
        lib = load()
        if not torch.cuda.is_available():
            raise RuntimeError("libspts needs a GPU: no device is visible (there is no CPU fallback)")
        self.shape = shape
        self.model = model_desc(shape)
        nbytes = spts_workspace_bytes(self.model, max_tokens, max_probe, max_r, max_dlow)
        if nbytes == 0:
            raise SptsError(SPTS_EINVAL, "spts_workspace_bytes")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        h = C.c_void_p()
        _check(lib.spts_create(C.byref(h), C.byref(self.model), self.stream.cuda_stream, self.workspace.data_ptr(),
                               nbytes, max_tokens, max_probe, max_r, max_dlow), "spts_create")
        self.handle = h

    def close(self):
        if getattr(self, "handle", None):
            load().spts_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def uses_mfma(self) -> bool:
        return bool(load().spts_uses_mfma(self.handle))

    # ---- the five calls; each returns the status raised as SptsError when non-zero -------------
    def spts_probe_attn(self, x, pos, N, w: spts_layer_weights, probe_len, k_out, s_mha):
        _check(load().spts_probe_attn(self.handle, _ptr(x), _ptr(pos), N, C.byref(w), probe_len, _ptr(k_out), _ptr(s_mha)),
               "spts_probe_attn")

    def spts_probe_ffn(self, x, N, w: spts_layer_weights, s_mha, c_ffn, s_ffn):
        _check(load().spts_probe_ffn(self.handle, _ptr(x), N, C.byref(w), _ptr(s_mha), _ptr(c_ffn), _ptr(s_ffn)),
               "spts_probe_ffn")

    def spts_select_topk(self, scores, N, k, protect_last, idx_out):
        _check(load().spts_select_topk(self.handle, _ptr(scores), N, k, protect_last, _ptr(idx_out)), "spts_select_topk")

    def spts_select_topk_batched(self, scores, N, k, protect_last, batch, idx_out):
        _check(load().spts_select_topk_batched(self.handle, _ptr(scores), N, k, protect_last, batch, _ptr(idx_out)),
               "spts_select_topk_batched")

    def spts_select_topk_segmented(self, scores, seg_offsets, seg_k, out_offsets, batch, max_len, protect_last, idx_out):
        _check(load().spts_select_topk_segmented(self.handle, _ptr(scores), _ptr(seg_offsets), _ptr(seg_k), _ptr(out_offsets),
                                                 batch, max_len, protect_last, _ptr(idx_out)), "spts_select_topk_segmented")

    def spts_layer_prefill(self, x, pos, N, w: spts_layer_weights, cfg: spts_layer_cfg, kv: Optional[spts_kv_out] = None,
                           s_mha=None, idx_attn=None, idx_ffn=None):
        _check(load().spts_layer_prefill(self.handle, _ptr(x), _ptr(pos), N, C.byref(w), C.byref(cfg),
                                         C.byref(kv) if kv is not None else None, _ptr(s_mha), _ptr(idx_attn),
                                         _ptr(idx_ffn)), "spts_layer_prefill")

    def spts_layer_prefill_batched(self, x, pos, seq_offsets, w: spts_layer_weights, probe_len: int, m_attn, m_ffn,
                                   protect_last: int = 1, kv=None, s_mha=None, idx_attn=None, idx_ffn=None, skip: int = 1):
        """seq_offsets [batch+1], m_attn / m_ffn [batch]: host integer sequences; kv: list of spts_kv_out or None
        (their count fields are updated in place)."""
        batch = len(seq_offsets) - 1
        so = (C.c_int64 * (batch + 1))(*[int(v) for v in seq_offsets])
        ma = (C.c_int64 * max(batch, 1))(*[int(v) for v in m_attn])
        mf = (C.c_int64 * max(batch, 1))(*[int(v) for v in m_ffn])
        kva = None
        if kv is not None:
            kva = (spts_kv_out * batch)(*kv)
        _check(load().spts_layer_prefill_batched(self.handle, _ptr(x), _ptr(pos), so, batch, C.byref(w), skip, probe_len, ma, mf,
                                                 protect_last, kva, _ptr(s_mha), _ptr(idx_attn), _ptr(idx_ffn)),
               "spts_layer_prefill_batched")
        if kv is not None:
            for dst, src in zip(kv, kva):
                dst.count = src.count

    def spts_msdp_compact_batched(self, x_in, pos_in, s_mha, seq_offsets, n_next, protect_last, x_out, pos_out, map_new2old,
                                  map_old2new=None):
        """seq_offsets [batch+1], n_next [batch]: host integer sequences.  Returns the new offsets (host list)."""
        batch = len(seq_offsets) - 1
        so = (C.c_int64 * (batch + 1))(*[int(v) for v in seq_offsets])
        nn = (C.c_int64 * max(batch, 1))(*[int(v) for v in n_next])
        _check(load().spts_msdp_compact_batched(self.handle, _ptr(x_in), _ptr(pos_in), _ptr(s_mha), so, batch, nn, protect_last,
                                                _ptr(x_out), _ptr(pos_out), _ptr(map_new2old), _ptr(map_old2new)),
               "spts_msdp_compact_batched")
        new = [0]
        for b in range(batch):
            new.append(new[-1] + min(int(seq_offsets[b + 1]) - int(seq_offsets[b]), int(n_next[b])))
        return new

    def spts_decode_layer(self, x, pos: int, w: spts_layer_weights, cache: spts_kv_out):
        _check(load().spts_decode_layer(self.handle, _ptr(x), pos, C.byref(w), C.byref(cache)), "spts_decode_layer")

    def spts_decode_layer_batched(self, x, pos, w: spts_layer_weights, caches):
        """x [batch, D] device tensor; pos: host integers; caches: list of spts_kv_out (count fields updated in place)."""
        batch = len(caches)
        pa = (C.c_int32 * max(batch, 1))(*[int(v) for v in pos])
        ka = (spts_kv_out * max(batch, 1))(*caches)
        _check(load().spts_decode_layer_batched(self.handle, _ptr(x), pa, batch, C.byref(w), ka), "spts_decode_layer_batched")
        for dst, src in zip(caches, ka):
            dst.count = src.count

    def spts_greedy_token_batched(self, x, gamma_f, table, V: int, batch: int, token_out, logits_out=None, x_next=None):
        _check(load().spts_greedy_token_batched(self.handle, _ptr(x), _ptr(gamma_f), _ptr(table), V, batch, _ptr(token_out),
                                                _ptr(logits_out), _ptr(x_next)), "spts_greedy_token_batched")

    def spts_greedy_token(self, x, gamma_f, table, V: int, token_out, logits_out=None, x_next=None):
        _check(load().spts_greedy_token(self.handle, _ptr(x), _ptr(gamma_f), _ptr(table), V, _ptr(token_out),
                                        _ptr(logits_out), _ptr(x_next)), "spts_greedy_token")

    def spts_channel_importance(self, x_cal, T: int, w: spts_layer_weights, k: int, importance_out):
        _check(load().spts_channel_importance(self.handle, _ptr(x_cal), T, C.byref(w), k, _ptr(importance_out)),
               "spts_channel_importance")

    def spts_pack_slab32(self, W, rows: int, K: int, out):
        _check(load().spts_pack_slab32(self.handle, _ptr(W), rows, K, _ptr(out)), "spts_pack_slab32")

    def spts_msdp_compact(self, x_in, pos_in, s_mha, N, N_next, protect_last, x_out, pos_out, map_new2old,
                          map_old2new=None):
        _check(load().spts_msdp_compact(self.handle, _ptr(x_in), _ptr(pos_in), _ptr(s_mha), N, N_next, protect_last,
                                        _ptr(x_out), _ptr(pos_out), _ptr(map_new2old), _ptr(map_old2new)),
               "spts_msdp_compact")

    def spts_profile_begin(self):
        _check(load().spts_profile_begin(self.handle), "spts_profile_begin")

    def spts_profile_end(self) -> dict:
        """Ends profiling; returns {phase: (total_ms, launches)} for the phases that ran."""
        lib = load()
        _check(lib.spts_profile_end(self.handle), "spts_profile_end")
        out = {}
        for i in range(lib.spts_profile_count(self.handle)):
            name, ms, n = C.c_char_p(), C.c_double(), C.c_int64()
            _check(lib.spts_profile_get(self.handle, i, C.byref(name), C.byref(ms), C.byref(n)), "spts_profile_get")
            if n.value:
                out[name.value.decode()] = (ms.value, n.value)
        return out

    # raw status (for error-path tests)
    def raw(self, name, *args):
        return getattr(load(), name)(self.handle, *args)
