"""Pins of the CPU oracle against things other than itself (runs without a GPU).

Each test names the definition or identity of the paper it pins.  The
independent sides are: torch CPU fp64 library routines (scaled dot product
attention, complex rotation, linear), brute-force Python sorting, closed
forms and invariants.
"""
import math

import numpy as np
import pytest
import torch

from oracle import spts_oracle as orc
from paper_2601_13155_amd import synth
from tests.helpers import oracle_model, small_shape


def _layer(seed=3, N=48, r=8, **kw):
    shape = small_shape(**kw)
    w = synth.make_layer(seed, 0, shape, r)
    x = synth.hidden_states(seed, N, shape.D)
    return shape, oracle_model(shape), w, x, synth.positions(N)


# ---------------------------------------------------------------- dense block (P1)
def _torch_dense_block(x, pos, w, shape):
    """Pre-norm LLaMA block from torch library routines, independent of the oracle's code."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    X = t(x)
    N = X.shape[0]
    H, Hkv, d = shape.H, shape.Hkv, shape.d

    def norm(v, g):
        return v * torch.rsqrt(v.pow(2).mean(-1, keepdim=True) + shape.rms_eps) * t(g)

    def rot(v, heads):  # complex-multiplication form of the rotary embedding
        v = v.reshape(N, heads, d)
        z = torch.complex(v[..., : d // 2], v[..., d // 2:])
        inv = torch.pow(torch.tensor(shape.rope_base, dtype=torch.float64),
                        -torch.arange(0, d, 2, dtype=torch.float64) / d)
        ang = t(pos).to(torch.float64)[:, None] * inv[None, :]
        z = z * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    xn = norm(X, w["gamma1"])
    q = rot(xn @ t(w["Wq"]), H).permute(1, 0, 2)
    k = rot(xn @ t(w["Wk"]), Hkv).permute(1, 0, 2).repeat_interleave(H // Hkv, dim=0)
    v = (xn @ t(w["Wv"])).reshape(N, Hkv, d).permute(1, 0, 2).repeat_interleave(H // Hkv, dim=0)
    att = torch.nn.functional.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
    X = X + att.permute(1, 0, 2).reshape(N, H * d) @ t(w["Wo"])
    xn2 = norm(X, w["gamma2"])
    hdn = torch.nn.functional.silu(xn2 @ t(w["Wgate"])) * (xn2 @ t(w["Wup"]))
    X = X + torch.nn.functional.linear(hdn, t(w["Wdown"]))   # h @ Wdown^T
    return X.numpy()


def test_dense_layer_matches_torch_composition():
    shape, mdl, w, x, pos = _layer(N=40)
    out = orc.layer_prefill(x, pos, w, mdl, orc.LayerCfg(skip=0))
    ref = _torch_dense_block(x, pos, w, shape)
    assert np.max(np.abs(out.x - ref)) < 1e-10 * np.max(np.abs(ref))


def test_dense_layer_matches_torch_on_config0_shape():
    wl = synth.scaled(synth.WORKLOADS["c0"], N=96)
    w = synth.make_layer(wl.seed, 0, wl.shape, wl.r)
    x = synth.hidden_states(wl.seed, wl.N, wl.shape.D)
    pos = synth.positions(wl.N) * 3 + 5          # non-trivial absolute positions
    out = orc.layer_prefill(x, pos, w, oracle_model(wl.shape), orc.LayerCfg(skip=0))
    ref = _torch_dense_block(x, pos, w, wl.shape)
    assert np.max(np.abs(out.x - ref)) < 1e-10 * np.max(np.abs(ref))


def test_keep_all_reproduces_dense_layer():
    shape, mdl, w, x, pos = _layer()
    N = x.shape[0]
    dense = orc.layer_prefill(x, pos, w, mdl, orc.LayerCfg(skip=0))
    full = orc.layer_prefill(x, pos, w, mdl, orc.LayerCfg(skip=1, probe_len=4, m_attn=N, m_ffn=N))
    assert np.array_equal(full.idx_attn, np.arange(N))
    assert np.max(np.abs(dense.x - full.x)) < 1e-12 * np.max(np.abs(dense.x))
    # budgets above N are clipped to N (M = min(|T|, M_fixed), Sec. 3.4)
    over = orc.layer_prefill(x, pos, w, mdl, orc.LayerCfg(skip=1, probe_len=4, m_attn=10 * N, m_ffn=10 * N))
    assert np.array_equal(over.x, full.x)


# ---------------------------------------------------------------- skip rule (P2, P3)
def test_keep_zero_is_identity():
    shape, mdl, w, x, pos = _layer()
    out = orc.layer_prefill(x, pos, w, mdl, orc.LayerCfg(skip=1, probe_len=4, m_attn=0, m_ffn=0, protect_last=1))
    assert np.array_equal(out.x, x.astype(np.float64))
    assert out.idx_attn.size == 0 and out.idx_ffn.size == 0


def test_inactive_rows_untouched_and_count_kept():
    shape, mdl, w, x, pos = _layer(N=64)
    out = orc.layer_prefill(x, pos, w, mdl, orc.LayerCfg(skip=1, probe_len=8, m_attn=20, m_ffn=24))
    assert out.x.shape == x.shape
    touched = np.zeros(64, bool)
    touched[out.idx_attn] = True
    touched[out.idx_ffn] = True
    assert np.array_equal(out.x[~touched], x.astype(np.float64)[~touched])
    changed = np.any(out.x != x, axis=1)
    assert np.array_equal(changed, touched)
    assert out.idx_attn.size == 20 and out.idx_ffn.size == 24
    assert out.k_cache.shape == (20, shape.Hkv, shape.d) and out.v_cache.shape == (20, shape.Hkv, shape.d)
    assert np.array_equal(out.pos_cache, pos[out.idx_attn])


# ---------------------------------------------------------------- probe (P4)
def test_probe_scores_sum_to_one_and_nonnegative():
    shape, mdl, w, x, pos = _layer(N=70)
    for P in (1, 5, 16):
        _, S = orc.probe_attn(x, pos, w, mdl, P)
        assert S.min() >= 0.0
        assert abs(S.sum() - 1.0) < 1e-12


def test_probe_p1_is_head_mean_of_last_attention_row():
    """Eq. (mha_importance): brute force over the full causal probability matrix (torch softmax)."""
    shape, mdl, w, x, pos = _layer(N=33)
    K, S = orc.probe_attn(x, pos, w, mdl, 1)
    xn = orc.rmsnorm(x, w["gamma1"], mdl.rms_eps)
    Q = orc.project_queries(xn, pos, w["Wq"], mdl)
    N = 33
    acc = np.zeros(N)
    mask = torch.tril(torch.ones(N, N, dtype=torch.bool))
    for h in range(shape.H):
        g = h // (shape.H // shape.Hkv)
        logits = torch.from_numpy(Q[:, h] @ K[:, g].T / math.sqrt(shape.d))
        prob = torch.softmax(logits.masked_fill(~mask, float("-inf")), dim=-1)
        acc += prob[-1].numpy()
    assert np.max(np.abs(acc / shape.H - S)) < 1e-14


def test_probe_window_rows_are_causal_inside_window():
    """R2: probe row p sees candidates up to N-P+p only; with P = N it is the column mean of the full matrix."""
    shape, mdl, w, x, pos = _layer(N=12)
    N = 12
    K, S = orc.probe_attn(x, pos, w, mdl, N)
    xn = orc.rmsnorm(x, w["gamma1"], mdl.rms_eps)
    Q = orc.project_queries(xn, pos, w["Wq"], mdl)
    acc = np.zeros(N)
    for h in range(shape.H):
        g = h // (shape.H // shape.Hkv)
        for i in range(N):
            l = np.array([Q[i, h] @ K[j, g] / math.sqrt(shape.d) for j in range(i + 1)])
            p = np.exp(l - l.max())
            acc[: i + 1] += p / p.sum()
    assert np.max(np.abs(acc / (shape.H * N) - S)) < 1e-14


def test_rope_is_a_rotation_and_relative():
    mdl = oracle_model(small_shape())
    rng = np.random.default_rng(0)
    a = rng.standard_normal((5, 2, 16))
    b = rng.standard_normal((5, 2, 16))
    pos = np.array([0, 3, 10, 500, 100000])
    ra, rb = orc.rope(a, pos, 10000.0), orc.rope(b, pos, 10000.0)
    assert np.allclose(np.linalg.norm(ra, axis=-1), np.linalg.norm(a, axis=-1), rtol=1e-13)
    assert np.array_equal(ra[0], a[0])                         # position 0 is the identity
    # <rope(a,p), rope(b,p+s)> depends on s only
    r1 = np.sum(orc.rope(a[:1], [7], 10000.0) * orc.rope(b[:1], [19], 10000.0))
    r2 = np.sum(orc.rope(a[:1], [1007], 10000.0) * orc.rope(b[:1], [1019], 10000.0))
    assert abs(r1 - r2) < 1e-11
    # pair (j, j+d/2), theta_0 = 1: first pair rotates by exactly pos radians
    e = np.zeros((1, 1, 16)); e[0, 0, 0] = 1.0
    out = orc.rope(e, [2], 10000.0)[0, 0]
    assert abs(out[0] - math.cos(2.0)) < 1e-15 and abs(out[8] - math.sin(2.0)) < 1e-15
    # last pair uses theta = base^(-(d-2)/d)
    e = np.zeros((1, 1, 16)); e[0, 0, 7] = 1.0
    out = orc.rope(e, [1000], 10000.0)[0, 0]
    ang = 1000 * 10000.0 ** (-14.0 / 16.0)
    assert abs(out[7] - math.cos(ang)) < 1e-13 and abs(out[15] - math.sin(ang)) < 1e-13


# ---------------------------------------------------------------- LTP (P5, P6, P10)
def test_full_rank_proxy_reproduces_exact_ffn_ranking():
    shape, mdl, w, x, pos = _layer(N=40)
    full = synth.proxy_factors(w, min(shape.D, shape.Dff), "f32")
    w2 = dict(w); w2.update({k: v.astype(np.float64) for k, v in full.items()})
    # use fp64 factors from an fp64 SVD for an exact statement
    for tag, name in (("g", "Wgate"), ("u", "Wup"), ("d", "Wdown")):
        U, V = synth.truncated_svd(w[name], min(shape.D, shape.Dff))
        w2["U" + tag], w2["V" + tag] = U, V
    xn2 = orc.rmsnorm(x, w["gamma2"], mdl.rms_eps)
    C = orc.transformation_scores(xn2, w2)
    exact = np.linalg.norm(orc.ffn(xn2, w["Wgate"], w["Wup"], w["Wdown"]), axis=-1)
    assert np.max(np.abs(C - exact)) < 1e-10 * exact.max()
    assert np.array_equal(np.argsort(-C, kind="stable"), np.argsort(-exact, kind="stable"))
    c, s = orc.probe_ffn(x, w2, mdl, None)
    assert np.array_equal(c, s)
    s_mha = np.linspace(1.0, 2.0, 40)
    c2, s2 = orc.probe_ffn(x, w2, mdl, s_mha)
    assert np.allclose(s2, c2 * s_mha, rtol=0, atol=0)


def test_truncated_svd_meets_eckart_young():
    rng = np.random.default_rng(5)
    for shape_, big in (((24, 60), False), ((1100, 2000), True)):   # second case takes the Gram/eigh branch
        W = rng.standard_normal(shape_)
        sv = np.linalg.svd(W, compute_uv=False)
        for r in (1, 7, shape_[0]):
            U, V = synth.truncated_svd(W, r)
            assert U.shape == (shape_[0], r) and V.shape == (r, shape_[1])
            err = np.linalg.norm(W - U @ V) ** 2
            assert abs(err - np.sum(sv[r:] ** 2)) < 1e-8 * np.sum(sv ** 2)
            assert np.allclose(U.T @ U, np.eye(r), atol=1e-8)          # Sigma lives in V (R13)
            assert np.allclose(np.linalg.norm(V, axis=1), sv[:r], rtol=1e-7)


def test_ffn_is_token_independent():
    shape, mdl, w, x, pos = _layer(N=30)
    xn2 = orc.rmsnorm(x, w["gamma2"], mdl.rms_eps)
    allrows = orc.ffn(xn2, w["Wgate"], w["Wup"], w["Wdown"])
    rows = np.array([2, 3, 17, 29])
    assert np.allclose(orc.ffn(xn2[rows], w["Wgate"], w["Wup"], w["Wdown"]), allrows[rows], rtol=1e-13, atol=1e-13)
    # one-row FFN from scalar loops (definition of Eq. (ffn_function))
    v = xn2[5]
    g = np.array([sum(v[i] * float(w["Wgate"][i, j]) for i in range(shape.D)) for j in range(shape.Dff)])
    u = np.array([sum(v[i] * float(w["Wup"][i, j]) for i in range(shape.D)) for j in range(shape.Dff)])
    hcol = g / (1 + np.exp(-g)) * u
    y = np.array([sum(hcol[j] * float(w["Wdown"][i, j]) for j in range(shape.Dff)) for i in range(shape.D)])
    assert np.allclose(y, allrows[5], rtol=1e-11, atol=1e-12)


# ---------------------------------------------------------------- TopK / compaction (P7)
def _brute_topk(scores, k, protect_last):
    n = len(scores)
    key = [float(s) + 0.0 for s in scores]
    if protect_last and k >= 1:
        key[n - 1] = float("inf")
    order = sorted(range(n), key=lambda i: (-key[i], i))
    return sorted(order[:k])


@pytest.mark.parametrize("protect", [0, 1])
def test_topk_matches_bruteforce_sort(protect):
    rng = np.random.default_rng(11)
    cases = []
    for n in (1, 2, 63, 64, 65, 257, 1000):
        cases.append(rng.random(n).astype(np.float32))
        cases.append(np.full(n, 0.25, dtype=np.float32))                       # all equal
        z = rng.random(n).astype(np.float32); z[rng.random(n) < 0.6] = 0.0    # many zeros
        cases.append(z)
        cases.append(rng.integers(0, 4, n).astype(np.float32))                 # heavy duplicates
        m = rng.random(n).astype(np.float32); m[::3] = -0.0                    # signed zeros
        cases.append(m)
    for s in cases:
        n = len(s)
        for k in sorted({0, 1, n // 3, n // 2, n - 1, n}):
            if k < 0:
                continue
            got = orc.topk_select(s, k, protect)
            assert got.dtype == np.int32
            assert list(got) == _brute_topk(list(s), k, protect), (n, k)


def test_topk_nested_and_protect_last():
    rng = np.random.default_rng(2)
    s = rng.random(300).astype(np.float32)
    s[-1] = 0.0
    prev = set()
    for k in range(0, 301, 7):
        cur = set(orc.topk_select(s, k, 0).tolist())
        assert prev <= cur
        prev = cur
    assert 299 not in orc.topk_select(s, 10, 0)
    assert 299 in orc.topk_select(s, 1, 1)
    assert orc.topk_select(s, 0, 1).size == 0


def test_msdp_compact_maps():
    rng = np.random.default_rng(4)
    N, D = 50, 6
    x = rng.standard_normal((N, D))
    pos = np.arange(N) * 2 + 1
    s = rng.random(N).astype(np.float32)
    for n_next in (0, 1, 17, 50, 80):
        xo, po, new2old, old2new = orc.msdp_compact(x, pos, s, n_next, 1)
        m = min(N, n_next)
        assert xo.shape == (m, D) and new2old.shape == (m,)
        assert np.all(np.diff(new2old) > 0)
        assert np.array_equal(xo, x[new2old]) and np.array_equal(po, pos[new2old])
        assert np.array_equal(old2new[new2old], np.arange(m))
        assert np.count_nonzero(old2new >= 0) == m
        if m >= 1:
            assert new2old[-1] == N - 1
        if m == N:
            assert np.array_equal(new2old, np.arange(N))
        assert set(new2old.tolist()) == set(_brute_topk(list(s), m, 1))


# ---------------------------------------------------------------- positions (P11)
def test_relabelled_candidates_with_positions_attached():
    """R4: results depend on positions, not on the order candidates are stored in.

    The probe window (last P rows) keeps its place; the earlier rows are shuffled.
    """
    shape, mdl, w, x, pos = _layer(N=40)
    N, P = 40, 4
    pos = pos * 2 + 3
    cfg = orc.LayerCfg(skip=1, probe_len=P, m_attn=15, m_ffn=18, protect_last=1)
    base = orc.layer_prefill(x, pos, w, mdl, cfg)
    rng = np.random.default_rng(8)
    perm = np.concatenate([rng.permutation(N - P), np.arange(N - P, N)])
    out = orc.layer_prefill(x[perm], pos[perm], w, mdl, cfg)
    assert set(perm[out.idx_attn].tolist()) == set(base.idx_attn.tolist())
    assert set(perm[out.idx_ffn].tolist()) == set(base.idx_ffn.tolist())
    unperm = np.empty_like(out.x)
    unperm[perm] = out.x
    assert np.max(np.abs(unperm - base.x)) < 1e-11 * np.max(np.abs(base.x))


def test_reduced_attention_is_attention_over_active_set_only():
    """R5 / Alg. 1: with kv_mode 0 an active row never sees an inactive key."""
    shape, mdl, w, x, pos = _layer(N=32)
    cfg = orc.LayerCfg(skip=1, probe_len=2, m_attn=10, m_ffn=0, protect_last=1)
    out = orc.layer_prefill(x, pos, w, mdl, cfg)
    Ta = out.idx_attn
    # perturbing an inactive row must not change any active row's attention update
    inactive = np.setdiff1d(np.arange(32), Ta)
    x2 = x.copy(); x2[inactive[0]] += 1.0
    out2 = orc.layer_prefill(x2, pos, w, mdl, cfg, force_idx_attn=Ta)
    assert np.array_equal(out.x[Ta], out2.x[Ta])
    # whereas kv_mode 1 does see it (for rows after it)
    cfg1 = orc.LayerCfg(skip=1, probe_len=2, m_attn=10, m_ffn=0, protect_last=1, kv_mode=1)
    a = orc.layer_prefill(x, pos, w, mdl, cfg1, force_idx_attn=Ta)
    b = orc.layer_prefill(x2, pos, w, mdl, cfg1, force_idx_attn=Ta)
    later = Ta[Ta > inactive[0]]
    assert later.size > 0 and np.any(a.x[later] != b.x[later])
    # kv_mode 1 with every row active equals the dense layer
    full1 = orc.layer_prefill(x, pos, w, mdl, orc.LayerCfg(skip=1, probe_len=2, m_attn=32, m_ffn=32, kv_mode=1))
    dense = orc.layer_prefill(x, pos, w, mdl, orc.LayerCfg(skip=0))
    assert np.max(np.abs(full1.x - dense.x)) < 1e-12 * np.max(np.abs(dense.x))


# ---------------------------------------------------------------- stack (Alg. 1 outer loop)
def test_stack_stage_sizes_and_nesting():
    wl = synth.scaled(synth.WORKLOADS["c2"], N=200, layers=4, stage_end_layers=(1, 2, 3), probe_len=4, r=4,
                      shape=small_shape())
    plan = wl.layer_plan()
    assert [p["N"] for p in plan] == [200, 140, 100, 70]
    assert [p["N_next"] for p in plan] == [140, 100, 70, None]
    layers = [synth.make_layer(wl.seed, l, wl.shape, wl.r) for l in range(4)]
    x = synth.hidden_states(wl.seed, wl.N, wl.shape.D)
    xo, po, trace = orc.stack_prefill(x, synth.positions(wl.N), layers, oracle_model(wl.shape), plan, wl.probe_len)
    assert xo.shape == (70, wl.shape.D) and po.shape == (70,)
    assert np.all(np.diff(po) > 0) and po[-1] == 199         # last token survives every stage (R7)
    # N_{s+1} >= M_a  =>  the pruned candidate set contains that layer's active MHA set (TopK nestedness)
    for lo, item in zip(trace[:3], plan[:3]):
        assert set(lo.idx_attn.tolist()) <= set(lo.map_new2old.tolist())


def test_real_workload_budgets():
    p2 = synth.WORKLOADS["c2"].layer_plan()
    assert [p2[i]["N"] for i in (0, 8, 16, 24)] == [32768, 22937, 16384, 11468]
    assert [p2[i]["m_attn"] for i in (0, 8, 16, 24)] == [13107, 9174, 6553, 4587]
    assert [i + 1 for i, p in enumerate(p2) if p["N_next"]] == [8, 16, 24]
    p3 = synth.WORKLOADS["c3"].layer_plan()
    assert p3[0]["m_attn"] == 32768 and p3[0]["m_ffn"] == 39321
    p4 = synth.WORKLOADS["c4"].layer_plan()
    assert [i + 1 for i, p in enumerate(p4) if p["N_next"]] == [7, 14, 21]
    p1 = synth.WORKLOADS["c1"].layer_plan()
    assert p1[0]["m_attn"] == 3276


def test_bf16_round_hook_matches_torch_bfloat16():
    rng = np.random.default_rng(1)
    a = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-6, 6, 5000), [0.0, -0.0, 1.0, 65280.0]])
    ref = torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(orc.bf16_round(a), ref)
    assert np.array_equal(synth.round_to_bf16(a.astype(np.float32)).astype(np.float64), ref)
    bits = synth.bf16_bits(synth.round_to_bf16(a.astype(np.float32)))
    assert np.array_equal(synth.bf16_bits_to_f32(bits).astype(np.float64), ref)


def test_prefill_query_hook_moves_one_rounding_point_only():
    """bf16_prefill: the prefill's queries are rounded after the factor log2(e)/sqrt(d) is folded in (torch bfloat16
    as the independent rounding), the decode's queries and every other tensor as with bf16_round, and the plain
    algorithm (identity) does not know the factor at all."""
    shape = small_shape()
    mdl = oracle_model(shape)
    w = synth.make_layer(5, 0, shape, 8)
    xn = synth.hidden_states(5, 9, shape.D)
    pos = synth.positions(9) * 3 + 2
    q = orc.project_queries(xn, pos, w["Wq"], mdl)                      # fp64, no rounding
    c = np.float32(np.float32(1.4426950408889634) / np.sqrt(np.float32(mdl.d)))
    want = torch.from_numpy((q * float(c)).astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy() / float(c)
    got = orc.project_queries(xn, pos, w["Wq"], mdl, orc.bf16_prefill, prefill=True)
    assert np.array_equal(got, want)
    plain = torch.from_numpy(q.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert not np.array_equal(got, plain)                               # the point really moved
    assert np.array_equal(orc.project_queries(xn, pos, w["Wq"], mdl, orc.bf16_prefill), plain)            # decode call
    assert np.array_equal(orc.project_queries(xn, pos, w["Wq"], mdl, orc.bf16_round, prefill=True), plain)
    assert np.array_equal(orc.project_queries(xn, pos, w["Wq"], mdl, orc.identity, prefill=True), q)
    assert np.array_equal(orc.bf16_prefill(q), orc.bf16_round(q))
    # relative to the exact queries both roundings are within half a bf16 ulp (2^-9)
    assert np.max(np.abs(got - q) / np.maximum(np.abs(q), 1e-300)) <= 2.0 ** -8


def test_output_norm_of_an_orthonormal_projection_is_the_norm_of_z():
    """Eq. (ffn_transformation) with U_down from a truncated SVD (orthonormal columns, Sigma in V): ||z U_d^T|| = ||z||,
    also for a rank zero-padded with zero columns of U_d and zero rows of V_d; not for a U_d with mixed columns.  The
    check a caller runs before stating orthonormality (runtime.ud_columns_orthonormal) agrees on all three."""
    from paper_2601_13155_amd import runtime
    shape = small_shape()
    mdl = oracle_model(shape)
    xn2 = synth.hidden_states(12, 23, shape.D)
    for r, r_pad in ((8, 0), (6, 8)):
        w = synth.make_layer(12, 0, shape, r, r_pad=r_pad)
        f = lambda k: np.asarray(w[k], dtype=np.float64)
        z = (orc.silu(xn2 @ f("Ug") @ f("Vg")) * (xn2 @ f("Uu") @ f("Vu"))) @ f("Vd").T
        assert np.allclose(orc.transformation_scores(xn2, w), np.linalg.norm(z, axis=1), rtol=1e-6)
        assert runtime.ud_columns_orthonormal(w["Ud"], w["Vd"])
    w2 = dict(w)
    w2["Ud"] = f("Ud") @ (np.eye(f("Ud").shape[1]) + 0.3 * np.random.default_rng(0).standard_normal((f("Ud").shape[1],) * 2))
    assert not runtime.ud_columns_orthonormal(w2["Ud"], w2["Vd"])
    assert not np.allclose(orc.transformation_scores(xn2, w2), np.linalg.norm(z, axis=1), rtol=1e-2)
    w3 = dict(w)   # zero-padded columns whose Vd rows are NOT zero: z has components the projection drops
    w3["Vd"] = f("Vd") + 0.1
    assert not runtime.ud_columns_orthonormal(w3["Ud"], w3["Vd"])
