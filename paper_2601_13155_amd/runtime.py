"""Host-side conveniences around the C-ABI binding: uploads, context creation, layer/stack drivers.

Marshalling and sequencing only: every arithmetic step of the path runs inside libspts kernels.
"""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np

from . import binding, synth


def _torch():
    import torch
    return torch


def to_device(a: np.ndarray, dtype: str):
    """fp32 numpy array (already rounded to the storage dtype) -> device tensor of that dtype."""
    torch = _torch()
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda")
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def to_host(t) -> np.ndarray:
    torch = _torch()
    if t.dtype == torch.bfloat16:
        return t.to(torch.float32).cpu().numpy()
    return t.cpu().numpy()


def make_context(shape, max_tokens: int, max_probe: int, max_r: int, max_dlow: int) -> binding.Context:
    return binding.Context(shape, max_tokens, max_probe, max_r, max_dlow)


SLAB_PACKED = ("Wq", "Wk", "Wv", "Wo", "Wgate", "Wup", "Wdown", "Vg", "Vu", "Vd", "Ug", "Uu")


def pack_slab32(a: np.ndarray) -> np.ndarray:
    """Host-side slab-major copy of a row-major [rows, K] matrix (K % 32 == 0): element (s * rows + r) * 32 + j of the
    result is a[r, 32 * s + j]; same shape and dtype, the layout spts_pack_slab32 writes on the device."""
    rows, K = a.shape
    return np.ascontiguousarray(a.reshape(rows, K // 32, 32).transpose(1, 0, 2)).reshape(rows, K)


def ud_columns_orthonormal(Ud: np.ndarray, Vd: np.ndarray, tol: float = 1e-2) -> bool:
    """True when U_down [D, r] has orthonormal columns up to `tol` (what a truncated SVD with Sigma folded into V gives,
    also after rounding to bf16), all-zero columns of a zero-padded rank allowed if the matching rows of Vd are zero."""
    U = np.asarray(Ud, dtype=np.float64)
    G = U.T @ U
    d = np.diag(G).copy()
    zero = d == 0.0
    if np.any(np.abs(d[~zero] - 1.0) > tol) or np.max(np.abs(G - np.diag(d)), initial=0.0) > tol:
        return False
    return not zero.any() or not np.any(np.asarray(Vd)[zero])


def upload_layer(w: Dict[str, np.ndarray], shape, r: int, pack: bool = True,
                 ud_orthonormal: Optional[bool] = None) -> binding.spts_layer_weights:
    """Weights in the paper's orientation (synth.make_layer) -> device struct in the ABI layout.  pack (bf16 only): the
    projection and FFN matrices also get the slab-major copies that the prefill GEMMs prefer.  ud_orthonormal: whether to
    tell the library that U_down has orthonormal columns (it then takes the proxy's output norm from z alone); None =
    check the matrix here."""
    if ud_orthonormal is None:
        ud_orthonormal = "Ud" in w and "Vd" in w and ud_columns_orthonormal(w["Ud"], w["Vd"])
    abi = synth.to_abi_layout(w)
    dev = {k: to_device(v, shape.dtype) for k, v in abi.items()}
    if pack and shape.dtype == "bf16":
        for name in SLAB_PACKED:
            if name in abi and abi[name].shape[1] % 32 == 0:
                dev[name + "_s"] = to_device(pack_slab32(np.asarray(abi[name])), shape.dtype)
    dlow = int(abi["Vd"].shape[1]) if "Vd" in abi else 0
    return binding.layer_weights(dev, r=r if "Ug" in abi else 0, Dlow=dlow, ud_orthonormal=bool(ud_orthonormal))


def run_layer(ctx: binding.Context, x: np.ndarray, pos: np.ndarray, dw: binding.spts_layer_weights, shape, *, skip: int,
              probe_len: int, m_attn: int, m_ffn: int, protect_last: int = 1, kv_mode: int = 0, want_kv: bool = False):
    """One spts_layer_prefill call on host arrays; returns host arrays (tests and smoke use this)."""
    torch = _torch()
    N = int(x.shape[0])
    xd = to_device(x, shape.dtype)
    posd = torch.from_numpy(np.ascontiguousarray(pos, dtype=np.int32)).cuda()
    Ma = min(N, m_attn) if skip else N
    Mf = min(N, m_ffn) if skip else N
    s = torch.zeros(max(N, 1), dtype=torch.float32, device="cuda")
    ia = torch.full((max(Ma, 1),), -1, dtype=torch.int32, device="cuda")
    iff = torch.full((max(Mf, 1),), -1, dtype=torch.int32, device="cuda")
    cfg = binding.spts_layer_cfg(skip, probe_len, m_attn, m_ffn, protect_last, kv_mode)
    kv = None
    if want_kv:
        cap = N if (not skip or kv_mode == 1) else Ma
        tdt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        kk = torch.zeros((max(cap, 1), shape.Hkv, shape.d), dtype=tdt, device="cuda")
        vv = torch.zeros_like(kk)
        pp = torch.zeros(max(cap, 1), dtype=torch.int32, device="cuda")
        kv = binding.spts_kv_out(kk.data_ptr(), vv.data_ptr(), pp.data_ptr(), cap, 0)
    ctx.spts_layer_prefill(xd, posd, N, dw, cfg, kv, s, ia, iff)
    torch.cuda.synchronize()
    out = dict(x=to_host(xd).astype(np.float64), s_mha=s[:N].cpu().numpy(), idx_attn=ia[:Ma].cpu().numpy(),
               idx_ffn=iff[:Mf].cpu().numpy())
    if want_kv:
        cnt = int(kv.count)
        out.update(kv_count=cnt, k_cache=to_host(kk[:cnt]).astype(np.float64), v_cache=to_host(vv[:cnt]).astype(np.float64),
                   pos_cache=pp[:cnt].cpu().numpy())
    return out


def select_proxy_channels(ctx: binding.Context, dw: binding.spts_layer_weights, shape, x_cal: np.ndarray, k: int, dlow: int):
    """The data-driven part of the offline proxy construction (Sec. 3.3) on the GPU: channel scores of Eq.
    (channel_importance) over the calibration rows x_cal [T, D], then C = TopK(I, dlow).  Returns (channel ids
    ascending [dlow] int32, scores [Dff] fp32) as host arrays; the SVD of the sliced matrices stays in the harness
    (synth.proxy_factors).  Sequencing of two library calls only."""
    torch = _torch()
    T = int(x_cal.shape[0])
    imp = torch.zeros(shape.Dff, dtype=torch.float32, device="cuda")
    ctx.spts_channel_importance(to_device(x_cal, shape.dtype), T, dw, int(k), imp)
    sel = torch.empty(dlow, dtype=torch.int32, device="cuda")
    ctx.spts_select_topk(imp, shape.Dff, dlow, 0, sel)
    torch.cuda.synchronize()
    return sel.cpu().numpy(), imp.cpu().numpy()


class KVCache:
    """Device buffers of one layer's cache: k, v [capacity, Hkv, d], pos [capacity]; count lives on the host."""

    def __init__(self, shape, capacity: int):
        torch = _torch()
        tdt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        self.k = torch.zeros((max(capacity, 1), shape.Hkv, shape.d), dtype=tdt, device="cuda")
        self.v = torch.zeros_like(self.k)
        self.pos = torch.zeros(max(capacity, 1), dtype=torch.int32, device="cuda")
        self.struct = binding.spts_kv_out(self.k.data_ptr(), self.v.data_ptr(), self.pos.data_ptr(), capacity, 0)

    @property
    def count(self) -> int:
        return int(self.struct.count)

    def host(self):
        """(k, v, pos) of the filled rows as host arrays (fp64 / int32)."""
        n = self.count
        return to_host(self.k[:n]).astype(np.float64), to_host(self.v[:n]).astype(np.float64), self.pos[:n].cpu().numpy()


class DecodeRunner:
    """Decode phase on the GPU: per token one spts_decode_layer per layer over that layer's cache, then
    (optionally) spts_greedy_token.  Only enqueues work; token ids stay on the device."""

    def __init__(self, ctx: binding.Context, shape, layers: List[binding.spts_layer_weights], caches: List[KVCache],
                 gamma_f=None, table=None):
        torch = _torch()
        self.ctx, self.shape, self.layers, self.caches = ctx, shape, layers, caches
        self.gamma_f, self.table = gamma_f, table
        tdt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        self.x = torch.zeros(shape.D, dtype=tdt, device="cuda")
        self.x_next = torch.zeros(shape.D, dtype=tdt, device="cuda")
        self.token = torch.zeros(4, dtype=torch.int32, device="cuda")
        self.logits = torch.zeros(table.shape[0], dtype=torch.float32, device="cuda") if table is not None else None

    def step(self, pos: int):
        """Runs self.x (in place) through every layer as the token at absolute position pos."""
        for w, c in zip(self.layers, self.caches):
            self.ctx.spts_decode_layer(self.x, pos, w, c.struct)

    def greedy(self):
        """token = argmax over the table of the final-normed self.x; self.x_next = table[token]."""
        self.ctx.spts_greedy_token(self.x, self.gamma_f, self.table, int(self.table.shape[0]), self.token, self.logits,
                                   self.x_next)

    def generate(self, pos0: int, steps: int, tokens_out=None):
        """steps greedy decode steps starting from self.x at position pos0; tokens_out [steps] int32 device."""
        for t in range(steps):
            self.step(pos0 + t)
            self.greedy()
            if tokens_out is not None:
                tokens_out[t:t + 1].copy_(self.token[:1])
            self.x.copy_(self.x_next)


class BatchedDecodeRunner:
    """Decode phase for a batch of sequences: per step one spts_decode_layer_batched per layer over the sequences'
    caches of that layer (caches[b][l]), then spts_greedy_token_batched.  Only enqueues work."""

    def __init__(self, ctx: binding.Context, shape, layers: List[binding.spts_layer_weights], caches: List[List[KVCache]],
                 gamma_f, table):
        torch = _torch()
        self.ctx, self.shape, self.layers, self.caches = ctx, shape, layers, caches
        self.gamma_f, self.table = gamma_f, table
        self.batch = len(caches)
        tdt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        self.x = torch.zeros((self.batch, shape.D), dtype=tdt, device="cuda")
        self.x_next = torch.zeros_like(self.x)
        self.tokens = torch.zeros(max(self.batch, 4), dtype=torch.int32, device="cuda")
        self.logits = torch.zeros((self.batch, table.shape[0]), dtype=torch.float32, device="cuda")

    def step(self, pos: List[int]):
        for l, w in enumerate(self.layers):
            self.ctx.spts_decode_layer_batched(self.x, pos, w, [seq[l].struct for seq in self.caches])

    def generate(self, pos0: List[int], steps: int):
        for t in range(steps):
            self.step([p + t for p in pos0])
            self.ctx.spts_greedy_token_batched(self.x, self.gamma_f, self.table, int(self.table.shape[0]), self.batch,
                                               self.tokens, self.logits, self.x_next)
            self.x.copy_(self.x_next)


class StackRunner:
    """Runs Alg. 1's outer loop on the GPU: per layer one spts_layer_prefill, at stage ends one
    spts_msdp_compact.  Buffers are allocated once; run() only enqueues work (no host sync)."""

    def __init__(self, ctx: binding.Context, shape, layers: List[binding.spts_layer_weights], plan: List[dict],
                 probe_len: int, protect_last: int = 1, skip: int = 1, keep_trace: bool = False,
                 caches: Optional[List["KVCache"]] = None):
        torch = _torch()
        self.ctx, self.shape, self.layers, self.plan = ctx, shape, layers, plan
        self.caches = caches   # per-layer KV caches filled by the prefill (None = not kept)
        self.probe_len, self.protect_last, self.skip = probe_len, protect_last, skip
        N0 = plan[0]["N"]
        tdt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        self.xa = torch.empty((N0, shape.D), dtype=tdt, device="cuda")
        self.xb = torch.empty((N0, shape.D), dtype=tdt, device="cuda")
        self.posa = torch.empty(N0, dtype=torch.int32, device="cuda")
        self.posb = torch.empty(N0, dtype=torch.int32, device="cuda")
        self.s = torch.empty(N0, dtype=torch.float32, device="cuda")
        self.new2old = torch.empty(N0, dtype=torch.int32, device="cuda")
        self.keep_trace = keep_trace
        self.trace = []
        self.cfgs = []
        for item in plan:
            skip_l = 1 if (skip and item.get("skip", 1)) else 0   # a plan item may mark its layer dense
            self.cfgs.append(binding.spts_layer_cfg(skip_l, probe_len, item["m_attn"], item["m_ffn"], protect_last, 0))

    def run(self, x0, pos0):
        """x0 [N0, D] device tensor (copied, not modified), pos0 [N0] int32 device tensor.
        Returns (x, pos, N_final) as views into the runner's buffers."""
        torch = _torch()
        xa, xb, pa, pb = self.xa, self.xb, self.posa, self.posb
        N = self.plan[0]["N"]
        xa[:N].copy_(x0)
        pa[:N].copy_(pos0)
        self.trace = []
        for li, (w, item, cfg) in enumerate(zip(self.layers, self.plan, self.cfgs)):
            tr = None
            if self.keep_trace:
                tr = dict(N=N, x_in=xa[:N].clone(), pos_in=pa[:N].clone(),
                          idx_attn=torch.empty(max(min(N, item["m_attn"]), 1), dtype=torch.int32, device="cuda"),
                          idx_ffn=torch.empty(max(min(N, item["m_ffn"]), 1), dtype=torch.int32, device="cuda"))
            self.ctx.spts_layer_prefill(xa, pa, N, w, cfg, self.caches[li].struct if self.caches else None, self.s,
                                        tr["idx_attn"] if tr else None, tr["idx_ffn"] if tr else None)
            if tr is not None:
                tr["x_out"] = xa[:N].clone()
                tr["s_mha"] = self.s[:N].clone()
            if cfg.skip and item.get("N_next") is not None:
                n_next = min(N, item["N_next"])
                self.ctx.spts_msdp_compact(xa, pa, self.s, N, n_next, self.protect_last, xb, pb, self.new2old, None)
                if tr is not None:
                    tr["map_new2old"] = self.new2old[:n_next].clone()
                xa, xb = xb, xa
                pa, pb = pb, pa
                N = n_next
            if tr is not None:
                self.trace.append(tr)
        return xa[:N], pa[:N], N


class BatchedStackRunner:
    """Alg. 1's outer loop over a batch of sequences laid back to back: per layer one spts_layer_prefill_batched,
    at stage ends one spts_msdp_compact_batched.  `plans` holds one layer plan (Workload.layer_plan()) per sequence;
    all plans have the same layers, stage ends and skip flags."""

    def __init__(self, ctx: binding.Context, shape, layers: List[binding.spts_layer_weights], plans: List[List[dict]],
                 probe_len: int, protect_last: int = 1):
        torch = _torch()
        self.ctx, self.shape, self.layers, self.plans = ctx, shape, layers, plans
        self.probe_len, self.protect_last = probe_len, protect_last
        n0 = sum(p[0]["N"] for p in plans)
        tdt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        self.xa = torch.empty((n0, shape.D), dtype=tdt, device="cuda")
        self.xb = torch.empty((n0, shape.D), dtype=tdt, device="cuda")
        self.posa = torch.empty(n0, dtype=torch.int32, device="cuda")
        self.posb = torch.empty(n0, dtype=torch.int32, device="cuda")
        self.s = torch.empty(n0, dtype=torch.float32, device="cuda")
        self.new2old = torch.empty(n0, dtype=torch.int32, device="cuda")

    def run(self, x0, pos0):
        """x0 [sum N0_b, D], pos0 [sum N0_b]: the sequences back to back.  Returns (x, pos, offsets)."""
        xa, xb, pa, pb = self.xa, self.xb, self.posa, self.posb
        offs = [0]
        for p in self.plans:
            offs.append(offs[-1] + p[0]["N"])
        xa[:offs[-1]].copy_(x0)
        pa[:offs[-1]].copy_(pos0)
        for li, w in enumerate(self.layers):
            items = [p[li] for p in self.plans]
            skip_l = int(items[0].get("skip", 1))
            assert all(int(it.get("skip", 1)) == skip_l for it in items), "a layer is dense or skipped for the whole batch"
            self.ctx.spts_layer_prefill_batched(xa, pa, offs, w, self.probe_len, [it["m_attn"] for it in items],
                                                [it["m_ffn"] for it in items], self.protect_last, None, self.s, skip=skip_l)
            if skip_l and items[0].get("N_next") is not None:
                offs = self.ctx.spts_msdp_compact_batched(xa, pa, self.s, offs, [it["N_next"] for it in items],
                                                          self.protect_last, xb, pb, self.new2old)
                xa, xb = xb, xa
                pa, pb = pb, pa
        return xa[:offs[-1]], pa[:offs[-1]], offs

