"""Algorithmic work of the SPTS prefill path: flops and HBM bytes per step.

Host-side bookkeeping only; used for the roofline figures of ``bench.py``.
Counts what the method itself must do (Alg. 1), never the dense work avoided.
A multiply-accumulate counts as 2 flops.  ``b`` is bytes per stored element.
"""
from __future__ import annotations

from typing import Dict, Iterable, Optional, Sequence


def proxy_macs_per_token_per_projection(D: int, Dff: int, Dlow: Optional[int], r: Optional[int]) -> int:
    """Multiply-accumulates of one proxy projection for one token (Appendix C, proxy-scale table).

    A factorised projection ``x U V`` costs ``r * (D + Dlow)``; without the
    factorisation (r is None) it costs ``D * Dlow``; without channel reduction
    (Dlow is None) ``Dlow = Dff``.
    """
    dl = Dff if Dlow is None else Dlow
    if r is None:
        return D * dl
    return r * (D + dl)


def kv_cached_tokens(N: int, dense_layers: int, stage_layers: Sequence[int], budgets: Sequence[int],
                     prune_per_stage: int = 0) -> int:
    """Total (token, layer) pairs held in the KV cache after a prefill of N tokens.

    Dense layers cache all N tokens; a skip layer of stage s caches
    ``min(N_s, M_fixed_s)`` tokens (Sec. 3.2 last paragraph, Sec. 3.4), where
    the candidate count shrinks by ``prune_per_stage`` after every stage.
    """
    total = dense_layers * N
    cand = N
    for n_layers, m in zip(stage_layers, budgets):
        total += n_layers * min(cand, m)
        cand = max(cand - prune_per_stage, 0)
    return total


def layer_flops(D: int, H: int, Hkv: int, d: int, Dff: int, N: int, P: int, Ma: int, Mf: int,
                r: int, Dlow: int, skip: bool = True) -> Dict[str, float]:
    """Flops of one layer, by step (2 per MAC; causal attention counts the lower triangle)."""
    if not skip:
        return {
            "qkv_proj": 2.0 * N * D * (H + 2 * Hkv) * d,
            "attention": 4.0 * H * d * N * N / 2.0,
            "o_proj": 2.0 * N * H * d * D,
            "ffn": 2.0 * N * 3 * D * Dff,
        }
    return {
        "k_proj": 2.0 * N * D * Hkv * d,
        "probe_q": 2.0 * P * D * H * d,
        "probe_attn": 2.0 * H * P * N * d,
        "qv_proj": 2.0 * Ma * D * (H + Hkv) * d,
        "attention": 4.0 * H * d * Ma * Ma / 2.0,
        "o_proj": 2.0 * Ma * H * d * D,
        "proxy": 2.0 * N * 3 * proxy_macs_per_token_per_projection(D, Dff, Dlow, r),
        "ffn": 2.0 * Mf * 3 * D * Dff,
    }


def layer_bytes(D: int, Hkv: int, d: int, N: int, Ma: int, Mf: int, b: int) -> Dict[str, float]:
    """Algorithmic HBM bytes of the memory-bound steps of one skip layer."""
    return {
        "rmsnorm": 2.0 * N * D * b,              # each of the two norms
        "probe_attn": N * Hkv * d * b + 4.0 * N,  # K once + scores
        "topk_attn": 4.0 * N + 4.0 * Ma,
        "topk_ffn": 4.0 * N + 4.0 * Mf,
        "gather_attn": 2.0 * Ma * D * b,
        "gather_ffn": 2.0 * Mf * D * b,
        "scatter_attn": 3.0 * Ma * D * b,
        "scatter_ffn": 3.0 * Mf * D * b,
    }


def compact_bytes(D: int, N: int, N_next: int, b: int) -> float:
    return 2.0 * N_next * D * b + 4.0 * N + 8.0 * N_next


def stack_flops(shape, plan: Iterable[dict], P: int, r: int, Dlow: int, skip: bool = True) -> float:
    tot = 0.0
    for item in plan:
        n = item["N"] if skip else plan_first_n(plan)
        f = layer_flops(shape.D, shape.H, shape.Hkv, shape.d, shape.Dff, n, P,
                        min(n, item["m_attn"]), min(n, item["m_ffn"]), r, Dlow, skip)
        tot += sum(f.values())
    return tot


def plan_first_n(plan) -> int:
    for item in plan:
        return item["N"]
    return 0
