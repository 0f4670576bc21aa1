"""Seeded synthetic inputs for the SPTS token-skipped prefill path.

This module only *makes inputs*: hidden states, layer weights, low-rank proxy
factors, position ids and the integer budgets of the five workload
configurations.  It holds none of the method's arithmetic (no norm, RoPE,
attention, scoring, selection or FFN) and is the only code that the CPU
oracle's tests and the HIP path's tests/bench both use.

Everything is generated with numpy's counter-based Philox generator keyed by
``(seed, tensor id)`` so any tensor can be regenerated anywhere without files.

Recipe (stands in for the paper's long-context benchmark inputs and trained
checkpoints, which are not available):

* weights: i.i.d. ``N(0, 1/d_in)`` per matrix, norm gains ``gamma = 1``;
* hidden states: i.i.d. ``N(0, 1)``; row 0 scaled x20 (attention-sink
  stand-in); a seeded random 2 % of rows scaled x8 ("heavy" tokens);
* proxy factors: truncated SVD of each FFN matrix, ``W ~= U V`` with
  ``U in R^{D x r}`` holding orthonormal columns and ``V = Sigma_r V_r^T``
  (Sec. 3.3, "Low-rank Proxy FFN"); no channel selection, i.e. ``Dlow = Dff``.

Matrices are returned in the paper's orientation (``X @ W``; ``W_down`` is
``D x Dff`` and is applied transposed, Eq. (ffn_function)).  ``to_abi_layout``
re-lays them out the way the C-ABI wants them (every matrix ``[d_out, d_in]``
row-major, i.e. ``y = x @ W_abi^T``).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

# tensor ids for the Philox key
_TID_HIDDEN = 1
_TID_HEAVY = 2
_TID_WEIGHT0 = 16  # + 16 * layer + matrix index


@dataclass(frozen=True)
class ModelShape:
    """Dimensions of one decoder layer (paper notation: D, H, d, Dff)."""
    D: int
    H: int
    Hkv: int
    d: int
    Dff: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    dtype: str = "bf16"  # "f32" or "bf16" (storage type; accumulation is fp32 on the GPU)


@dataclass(frozen=True)
class Workload:
    """One of the benchmark configurations: shapes, length and integer budgets."""
    name: str
    shape: ModelShape
    N: int
    layers: int
    probe_len: int
    attn_keep: float
    ffn_keep: float
    r: int
    seed: int
    # cumulative keep ratios of the candidate set per stage, and the 1-based
    # layers after which a compaction runs (empty = no MSDP)
    stage_end_layers: Tuple[int, ...] = ()
    stage_cum_keep: Tuple[float, ...] = (1.0,)
    protect_last: int = 1
    # The paper's own schedule (Sec. 4.1, implementation details) instead of ratios: the first
    # `dense_layers` layers run dense; stage s then uses the absolute budget stage_budgets[s] for both
    # branches, and every stage end removes `stage_prune` candidates.  Empty stage_budgets = ratios.
    dense_layers: int = 0
    stage_budgets: Tuple[int, ...] = ()
    stage_prune: int = 0
    # proxy: Dlow channels of the FFN (0 = all Dff), rank r zero-padded to r_pad columns (0 = no padding)
    dlow: int = 0
    r_pad: int = 0
    # Which modules are switched on (the rows of Table ablation_main_speed): "full" = PAP + LTP + MSDP;
    # "pap+ltp" = the same budgets but the candidate set is never pruned; "pap" = additionally every
    # candidate takes the FFN (no proxy, no FFN selection).
    components: str = "full"

    def stage_sizes(self) -> List[int]:
        """Candidate counts per stage: floor(cum_keep_s * N_0), or N_0 - s * stage_prune."""
        if self.components != "full":
            return [self.N] * (len(self.stage_end_layers) + 1)
        if self.stage_budgets:
            return [max(0, self.N - s * self.stage_prune) for s in range(len(self.stage_end_layers) + 1)]
        return [int(math.floor(c * self.N + 1e-9)) for c in self.stage_cum_keep]

    def layer_plan(self) -> List[dict]:
        """Per layer: skip flag, candidate count, budgets and the compaction target (or None)."""
        sizes = self.stage_sizes()
        plan = []
        s = 0
        for l in range(1, self.layers + 1):
            n = sizes[s]
            if l <= self.dense_layers:
                item = dict(layer=l, N=n, m_attn=n, m_ffn=n, N_next=None, skip=0)
            elif self.stage_budgets:
                b = min(n, self.stage_budgets[s])
                item = dict(layer=l, N=n, m_attn=b, m_ffn=b, N_next=None, skip=1)
            else:
                item = dict(layer=l, N=n,
                            m_attn=int(math.floor(self.attn_keep * n + 1e-9)),
                            m_ffn=int(math.floor(self.ffn_keep * n + 1e-9)),
                            N_next=None, skip=1)
            if self.components == "pap" and item["skip"]:
                item["m_ffn"] = n
            if s < len(self.stage_end_layers) and l == self.stage_end_layers[s]:
                if self.components == "full":
                    item["N_next"] = sizes[s + 1]
                s += 1
            plan.append(item)
        return plan

    @property
    def proxy_r(self) -> int:
        """Rank of the stored proxy factors (the true rank r, or its zero-padded size)."""
        return self.r_pad if self.r_pad else self.r

    @property
    def proxy_dlow(self) -> int:
        return self.dlow if self.dlow else self.shape.Dff


LLAMA8B = ModelShape(D=4096, H=32, Hkv=8, d=128, Dff=14336, rms_eps=1e-5, rope_base=500000.0, dtype="bf16")
QWEN7B = ModelShape(D=3584, H=28, Hkv=4, d=128, Dff=18944, rms_eps=1e-6, rope_base=1000000.0, dtype="bf16")
TINY = ModelShape(D=256, H=4, Hkv=2, d=64, Dff=688, rms_eps=1e-5, rope_base=10000.0, dtype="f32")

WORKLOADS: Dict[str, Workload] = {
    "c0": Workload("c0", TINY, N=512, layers=1, probe_len=32, attn_keep=0.5, ffn_keep=0.5, r=16, seed=0),
    "c1": Workload("c1", LLAMA8B, N=8192, layers=1, probe_len=64, attn_keep=0.4, ffn_keep=0.4, r=256, seed=1),
    "c2": Workload("c2", LLAMA8B, N=32768, layers=32, probe_len=64, attn_keep=0.4, ffn_keep=0.4, r=256, seed=2,
                   stage_end_layers=(8, 16, 24), stage_cum_keep=(1.0, 0.7, 0.5, 0.35)),
    "c3": Workload("c3", LLAMA8B, N=131072, layers=4, probe_len=128, attn_keep=0.25, ffn_keep=0.3, r=256, seed=3),
    "c4": Workload("c4", QWEN7B, N=32768, layers=28, probe_len=64, attn_keep=0.4, ffn_keep=0.4, r=256, seed=4,
                   stage_end_layers=(7, 14, 21), stage_cum_keep=(1.0, 0.7, 0.5, 0.35)),
    # The paper's LLaMA schedule at 32K (Sec. 4.1): layers 1-10 dense, then (4, 5, 5, 5, 3) layers with active
    # budgets (9, 7, 4, 2, 1)K, 1K candidates pruned at each of the four stage ends, single-row probe,
    # (Dlow, r) = (512, 192).  The fifth budget is the one the KV-cache table of Sec. 4.3 implies.  The rank-192
    # factors are stored zero-padded to 256 columns (identical result; 256 is what the matrix-core tiles divide).
    "p32": Workload("p32", LLAMA8B, N=32768, layers=32, probe_len=1, attn_keep=0.0, ffn_keep=0.0, r=192, seed=5,
                    stage_end_layers=(14, 19, 24, 29), dense_layers=10,
                    stage_budgets=(9216, 7168, 4096, 2048, 1024), stage_prune=1024, dlow=512, r_pad=256),
    # The paper's Qwen schedule at 32K (Sec. 4.1): 28 layers, layers 1-9 dense, then (4, 4, 4, 4, 3) layers with
    # budgets (13, 10, 7, 4, 1)K, 2K candidates pruned at each stage end, (Dlow, r) = (1024, 256).  The paper
    # prints four budgets; the fifth continues their step of 3K, as the LLaMA schedule's fifth continues its own.
    "q32": Workload("q32", QWEN7B, N=32768, layers=28, probe_len=1, attn_keep=0.0, ffn_keep=0.0, r=256, seed=6,
                    stage_end_layers=(13, 17, 21, 25), dense_layers=9,
                    stage_budgets=(13312, 10240, 7168, 4096, 1024), stage_prune=2048, dlow=1024),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (tests shrink N / layers)."""
    return replace(w, **kw)


def _gen(seed: int, tid: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(tid)]))


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array -> nearest-even bfloat16 value, returned as fp32 (data formatting only)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)   # finite inputs: no wrap-around
    r += u
    r &= np.uint32(0xFFFF0000)
    return r.view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array holding bf16-representable values -> uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def storage_round(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round an fp32 array to the values the storage dtype can hold."""
    return round_to_bf16(a) if dtype == "bf16" else np.ascontiguousarray(a, dtype=np.float32)


def hidden_states(seed: int, N: int, D: int, dtype: str = "f32") -> np.ndarray:
    """[N, D] fp32: N(0,1); row 0 x20; a seeded random 2 % of the rows x8."""
    x = _gen(seed, _TID_HIDDEN).standard_normal((N, D), dtype=np.float32)
    n_heavy = int(round(0.02 * N))
    if n_heavy > 0 and N > 1:
        heavy = _gen(seed, _TID_HEAVY).choice(np.arange(1, N), size=min(n_heavy, N - 1), replace=False)
        x[heavy] *= 8.0
    if N > 0:
        x[0] *= 20.0
    return storage_round(x, dtype)


def positions(N: int) -> np.ndarray:
    return np.arange(N, dtype=np.int32)


_MATS = ("Wq", "Wk", "Wv", "Wo", "Wgate", "Wup", "Wdown")


def layer_weights(seed: int, layer: int, shape: ModelShape) -> Dict[str, np.ndarray]:
    """fp32 weights of one layer in the paper's orientation, N(0, 1/d_in)."""
    D, H, Hkv, d, Dff = shape.D, shape.H, shape.Hkv, shape.d, shape.Dff
    dims = {
        "Wq": (D, H * d), "Wk": (D, Hkv * d), "Wv": (D, Hkv * d), "Wo": (H * d, D),
        "Wgate": (D, Dff), "Wup": (D, Dff),
        "Wdown": (D, Dff),  # applied transposed: d_in = Dff
    }
    def one(item):
        i, name = item
        rows, cols = dims[name]
        d_in = cols if name == "Wdown" else rows
        g = _gen(seed, _TID_WEIGHT0 + 16 * layer + i)
        w = g.standard_normal((rows, cols), dtype=np.float32)
        w *= np.float32(1.0 / math.sqrt(d_in))
        return name, storage_round(w, shape.dtype)

    # every matrix has its own generator key, so the threads below do not change any value
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=4) as ex:
        out: Dict[str, np.ndarray] = dict(ex.map(one, enumerate(_MATS)))
    out["gamma1"] = np.ones(D, dtype=np.float32)
    out["gamma2"] = np.ones(D, dtype=np.float32)
    return out


def truncated_svd(W: np.ndarray, r: int) -> Tuple[np.ndarray, np.ndarray]:
    """Rank-r factors of W [D, C]: U [D, r] (orthonormal columns), V = Sigma_r V_r^T [r, C].

    Uses LAPACK's SVD when the matrix is small and the eigen-decomposition of
    the Gram matrix W W^T (same factors, far cheaper) when it is large.  This is
    set-up, not part of the timed path.
    """
    W64 = np.asarray(W, dtype=np.float64)
    Dm, C = W64.shape
    r = int(r)
    if Dm * C <= 1 << 21:
        U, s, Vt = np.linalg.svd(W64, full_matrices=False)
        return U[:, :r].copy(), (s[:r, None] * Vt[:r]).copy()
    import scipy.linalg as sl
    G = W64 @ W64.T
    lo = max(Dm - r, 0)
    _, vec = sl.eigh(G, subset_by_index=[lo, Dm - 1])
    U = vec[:, ::-1].copy()  # descending singular value order
    return U, U.T @ W64


def proxy_channels(seed: int, layer: int, Dff: int, dlow: int) -> np.ndarray:
    """The Dlow FFN channels the proxy keeps, ascending.  A seeded random subset: it stands in for the
    calibration-based channel selection of Eq. (channel_importance), which needs text activations."""
    if not dlow or dlow >= Dff:
        return np.arange(Dff)
    return np.sort(_gen(seed, 7000 + layer).choice(Dff, size=dlow, replace=False))


def proxy_factors(weights: Dict[str, np.ndarray], r: int, dtype: str, channels: Optional[np.ndarray] = None,
                  r_pad: int = 0) -> Dict[str, np.ndarray]:
    """Ug,Vg,Uu,Vu,Ud,Vd with W_gate[:, ch] ~= Ug Vg, W_up[:, ch] ~= Uu Vu, W_down[:, ch] ~= Ud Vd
    (ch = all channels unless given).  r_pad > r appends zero columns / rows (same products)."""
    out: Dict[str, np.ndarray] = {}
    for tag, name in (("g", "Wgate"), ("u", "Wup"), ("d", "Wdown")):
        W = weights[name] if channels is None else np.ascontiguousarray(weights[name][:, channels])
        U, V = truncated_svd(W, r)
        if r_pad and r_pad > r:
            U = np.concatenate([U, np.zeros((U.shape[0], r_pad - r), U.dtype)], axis=1)
            V = np.concatenate([V, np.zeros((r_pad - r, V.shape[1]), V.dtype)], axis=0)
        out["U" + tag] = storage_round(U.astype(np.float32), dtype)
        out["V" + tag] = storage_round(V.astype(np.float32), dtype)
    return out


def make_layer(seed: int, layer: int, shape: ModelShape, r: int, dlow: int = 0, r_pad: int = 0,
               channels: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """Weights + proxy factors of one layer.  The proxy keeps all Dff channels (dlow = 0), a seeded random subset of
    dlow channels, or exactly `channels` (ascending ids, e.g. the set the offline construction of Sec. 3.3 chose)."""
    w = layer_weights(seed, layer, shape)
    if channels is not None:
        ch = np.asarray(channels, dtype=np.int64)
    else:
        ch = proxy_channels(seed, layer, shape.Dff, dlow) if dlow else None
    w.update(proxy_factors(w, r, shape.dtype, ch, r_pad))
    return w


def calibration_states(seed: int, T: int, D: int, dtype: str) -> np.ndarray:
    """Synthetic calibration token set for the offline proxy construction: [T, D] i.i.d. N(0, 1) rows
    (unit RMS in expectation, like states after an RMSNorm with gamma = 1).  Stands in for the FFN
    inputs collected on calibration text, which this build does not have."""
    return storage_round(_gen(seed, 9002).standard_normal((T, D), dtype=np.float32), dtype)


def vocab_table(seed: int, V: int, D: int, dtype: str) -> np.ndarray:
    """Synthetic vocabulary table [V, D], i.i.d. N(0, 1): serves as LM head and as embedding in the
    decode harness (the method defines neither)."""
    t = _gen(seed, 9001).standard_normal((V, D), dtype=np.float32)
    return storage_round(t, dtype)


def to_abi_layout(w: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    """Paper orientation -> the C-ABI's ``[d_out, d_in]`` row-major matrices."""
    out = {}
    for k, v in w.items():
        if k in ("Wq", "Wk", "Wv", "Wo", "Wgate", "Wup", "Ug", "Vg", "Uu", "Vu"):
            out[k] = np.ascontiguousarray(v.T)
        else:  # Wdown [D,Dff], Ud [D,r], Vd [r,Dlow] are applied transposed by the method
            out[k] = np.ascontiguousarray(v)
    return out
