"""Pins of the oracle's LTP decision inside a layer (Alg. 1, LTP block; Eq. (ffn_importance), (ffn_selection)):
the FFN's active set is TopK of C^FFN * S^MHA, with S^MHA the probe score of the same layer taken BEFORE the
attention update and C^FFN the proxy's output norm on the state AFTER it.

The independent sides: a torch composition of the attention half and of the probe, scalar Python loops for the
proxy (Eq. (proxy_ffn), (ffn_transformation)) and a Python sort for TopK.  Each test also shows that the
plausible mistakes (ranking by C alone, by S alone, or by a score recomputed after the attention update) would
select a different set on its input, so it could not pass with them.  Runs without a GPU.
"""
import math

import numpy as np
import torch

from oracle import spts_oracle as orc
from paper_2601_13155_amd import synth
from tests.helpers import oracle_model, small_shape


def _brute_topk(scores, k, protect_last=1):
    n = len(scores)
    key = [float(s) + 0.0 for s in scores]
    if protect_last and k >= 1:
        key[n - 1] = float("inf")
    order = sorted(range(n), key=lambda i: (-key[i], i))
    return sorted(order[:k])


def _loop_proxy_norm(xn2_row, w):
    """C = || ((silu(x Ug Vg) * (x Uu Vu)) Vd^T) Ud^T ||_2 for one row, scalar loops only."""
    D, r = w["Ug"].shape
    dlow = w["Vg"].shape[1]
    f = lambda name: np.asarray(w[name], dtype=np.float64)
    Ug, Vg, Uu, Vu, Ud, Vd = f("Ug"), f("Vg"), f("Uu"), f("Vu"), f("Ud"), f("Vd")
    v = [float(t) for t in xn2_row]
    tg = [sum(v[i] * Ug[i, a] for i in range(D)) for a in range(r)]
    tu = [sum(v[i] * Uu[i, a] for i in range(D)) for a in range(r)]
    hp = []
    for c in range(dlow):
        g = sum(tg[a] * Vg[a, c] for a in range(r))
        u = sum(tu[a] * Vu[a, c] for a in range(r))
        hp.append(g / (1.0 + math.exp(-g)) * u)
    z = [sum(hp[c] * Vd[a, c] for c in range(dlow)) for a in range(r)]
    o = [sum(z[a] * Ud[i, a] for a in range(r)) for i in range(D)]
    return math.sqrt(sum(t * t for t in o))


def _loop_rmsnorm(row, gamma, eps):
    ms = sum(float(t) * float(t) for t in row) / len(row)
    return [float(t) / math.sqrt(ms + eps) * float(g) for t, g in zip(row, gamma)]


def _torch_attention_half(x, pos, w, shape, P):
    """(S^MHA of the last P rows, state after a dense attention update) from torch library routines."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    X = t(x)
    N = X.shape[0]
    H, Hkv, d = shape.H, shape.Hkv, shape.d
    xn = X * torch.rsqrt(X.pow(2).mean(-1, keepdim=True) + shape.rms_eps) * t(w["gamma1"])

    def rot(v, heads):
        v = v.reshape(N, heads, d)
        z = torch.complex(v[..., : d // 2], v[..., d // 2:])
        inv = torch.pow(torch.tensor(shape.rope_base, dtype=torch.float64), -torch.arange(0, d, 2, dtype=torch.float64) / d)
        ang = t(pos).to(torch.float64)[:, None] * inv[None, :]
        z = z * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    q = rot(xn @ t(w["Wq"]), H).permute(1, 0, 2)                                        # [H, N, d]
    k = rot(xn @ t(w["Wk"]), Hkv).permute(1, 0, 2).repeat_interleave(H // Hkv, dim=0)
    v = (xn @ t(w["Wv"])).reshape(N, Hkv, d).permute(1, 0, 2).repeat_interleave(H // Hkv, dim=0)
    causal = torch.tril(torch.ones(N, N, dtype=torch.bool))
    prob = torch.softmax((q @ k.transpose(1, 2) / math.sqrt(d)).masked_fill(~causal, float("-inf")), dim=-1)  # [H, N, N]
    S = prob[:, N - P:, :].mean(dim=(0, 1))
    att = (prob @ v).permute(1, 0, 2).reshape(N, H * d)
    return S.numpy(), (X + att @ t(w["Wo"])).numpy()


def _layer(seed, N, r=8):
    shape = small_shape()
    w = synth.make_layer(seed, 0, shape, r)
    return shape, oracle_model(shape), w, synth.hidden_states(seed, N, shape.D), synth.positions(N) * 2 + 1


def test_ltp_set_is_topk_of_proxy_norm_times_pre_attention_score():
    shape, mdl, w, x, pos = _layer(seed=21, N=36)
    N, P, Mf = 36, 4, 13
    w = dict(w); w["Wo"] = w["Wo"] * 6.0          # the attention update reshapes the state, so pre != post scores
    out = orc.layer_prefill(x, pos, w, mdl, orc.LayerCfg(skip=1, probe_len=P, m_attn=N, m_ffn=Mf, protect_last=1))
    S_pre, x_mid = _torch_attention_half(x, pos, w, shape, P)
    C = np.array([_loop_proxy_norm(_loop_rmsnorm(x_mid[n], w["gamma2"], mdl.rms_eps), w) for n in range(N)])
    want = _brute_topk(C * S_pre, Mf)
    assert out.idx_ffn.tolist() == want
    assert np.allclose(out.c_ffn, C, rtol=1e-10) and np.allclose(out.s_ffn, C * S_pre, rtol=1e-10)
    assert np.allclose(out.s_mha, S_pre, rtol=1e-10)
    # the mistakes this input tells apart
    S_post, _ = _torch_attention_half(x_mid, pos, w, shape, P)
    assert _brute_topk(C, Mf) != want                      # C^FFN alone
    assert _brute_topk(S_pre, Mf) != want                  # S^MHA alone
    assert _brute_topk(C * S_post, Mf) != want             # score recomputed after the attention update
    C_pre = np.array([_loop_proxy_norm(_loop_rmsnorm(x[n], w["gamma2"], mdl.rms_eps), w) for n in range(N)])
    assert _brute_topk(C_pre * S_pre, Mf) != want          # proxy applied to the state before the attention update


def test_constant_proxy_norm_leaves_the_mha_ranking():
    """Identical rows and a zero output projection: every row reaches the FFN in the same state, so C^FFN is
    one constant and the LTP set must be TopK of S^MHA (which still varies through the rotary positions)."""
    shape, mdl, w, x, pos = _layer(seed=22, N=40)
    N, P, Mf = 40, 1, 14
    w = dict(w); w["Wo"] = np.zeros_like(w["Wo"])
    x = np.repeat(x[3:4], N, axis=0)
    out = orc.layer_prefill(x, pos, w, mdl, orc.LayerCfg(skip=1, probe_len=P, m_attn=17, m_ffn=Mf, protect_last=1))
    assert np.ptp(out.c_ffn) <= 1e-12 * out.c_ffn.max()
    S_pre, _ = _torch_attention_half(x, pos, w, shape, P)
    gaps = np.diff(np.sort(S_pre))
    assert gaps.min() > 1e-9 * S_pre.max()                 # no near ties that the constant's rounding could flip
    want = _brute_topk(S_pre, Mf)
    assert out.idx_ffn.tolist() == want
    assert _brute_topk(np.ones(N), Mf) != want             # ranking by C alone would take the lowest indices


def test_flat_mha_score_leaves_the_proxy_ranking():
    """Zero key projection and a single probe row: every logit is 0, S^MHA = 1/N for every candidate, and the
    LTP set must be TopK of C^FFN on the post-attention state (proxy from scalar loops)."""
    shape, mdl, w, x, pos = _layer(seed=23, N=34)
    N, Ma, Mf = 34, 12, 11
    w = dict(w); w["Wk"] = np.zeros_like(w["Wk"]); w["Wo"] = w["Wo"] * 4.0
    cfg = orc.LayerCfg(skip=1, probe_len=1, m_attn=Ma, m_ffn=Mf, protect_last=1)
    out = orc.layer_prefill(x, pos, w, mdl, cfg)
    assert np.allclose(out.s_mha, 1.0 / N, rtol=1e-12)
    assert out.idx_attn.tolist() == list(range(Ma - 1)) + [N - 1]       # ties go to the lowest index, last row protected
    # state after the attention update of the active rows (attention over the active set is pinned in
    # test_oracle_pins.py); the FFN budget 0 leaves it as the layer's output
    x_mid = orc.layer_prefill(x, pos, w, mdl, orc.LayerCfg(skip=1, probe_len=1, m_attn=Ma, m_ffn=0, protect_last=1)).x
    assert np.any(x_mid[out.idx_attn] != x[out.idx_attn])
    C = np.array([_loop_proxy_norm(_loop_rmsnorm(x_mid[n], w["gamma2"], mdl.rms_eps), w) for n in range(N)])
    want = _brute_topk(C, Mf)
    assert out.idx_ffn.tolist() == want
    C_pre = np.array([_loop_proxy_norm(_loop_rmsnorm(x[n], w["gamma2"], mdl.rms_eps), w) for n in range(N)])
    assert _brute_topk(C_pre, Mf) != want                  # proxy on the pre-attention state
    assert _brute_topk(np.full(N, 1.0 / N), Mf) != want    # S^MHA alone
