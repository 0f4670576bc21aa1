"""Pins of the oracle's decode phase against things other than itself (runs without a GPU).

Independent sides: the prefill path on one more token (a different code path: full causal
attention matrix instead of one query over a cache), a loop-by-loop softmax over the cache, an
invariance, and numpy's argmax.
"""
import math

import numpy as np

from oracle import spts_oracle as orc
from paper_2601_13155_amd import synth
from tests.helpers import oracle_model, small_shape


def _stack(seed=11, N=40, layers=3, r=8):
    shape = small_shape()
    ws = [synth.make_layer(seed, l, shape, r) for l in range(layers)]
    x = synth.hidden_states(seed, N + 1, shape.D)
    return shape, oracle_model(shape), ws, x, synth.positions(N + 1)


def test_dense_prefill_plus_one_decode_step_equals_prefill_of_one_more_token():
    """Alg. 1 with skip false everywhere: causality makes the last row of an (N+1)-token prefill a
    function of the first N tokens' keys/values only, which is what the decode step consumes."""
    shape, mdl, ws, x, pos = _stack()
    N = x.shape[0] - 1
    plan = [dict(m_attn=N + 1, m_ffn=N + 1, N_next=None)] * len(ws)
    full_x, _, full_tr = orc.stack_prefill(x, pos, ws, mdl, plan, probe_len=4, skip=0)
    plan_n = [dict(m_attn=N, m_ffn=N, N_next=None)] * len(ws)
    _, _, tr = orc.stack_prefill(x[:N], pos[:N], ws, mdl, plan_n, probe_len=4, skip=0)
    caches = [orc.LayerCache(t.k_cache, t.v_cache, t.pos_cache) for t in tr]
    h, caches2 = orc.decode_step(x[N], int(pos[N]), ws, mdl, caches)
    assert np.allclose(h, full_x[N], rtol=1e-10, atol=1e-12)
    for c, t in zip(caches2, full_tr):
        assert c.k.shape[0] == N + 1
        assert np.allclose(c.k, t.k_cache, rtol=1e-10, atol=1e-12)
        assert np.allclose(c.v, t.v_cache, rtol=1e-10, atol=1e-12)
        assert np.array_equal(c.pos, t.pos_cache)


def test_two_decode_steps_equal_prefill_of_two_more_tokens():
    shape, mdl, ws, x, pos = _stack(seed=12, N=30)
    x = np.concatenate([x, synth.hidden_states(99, 1, shape.D)], axis=0)
    pos = synth.positions(x.shape[0])
    N = x.shape[0] - 2
    dense = lambda n: [dict(m_attn=n, m_ffn=n, N_next=None)] * len(ws)
    full_x, _, _ = orc.stack_prefill(x, pos, ws, mdl, dense(N + 2), probe_len=4, skip=0)
    _, _, tr = orc.stack_prefill(x[:N], pos[:N], ws, mdl, dense(N), probe_len=4, skip=0)
    caches = [orc.LayerCache(t.k_cache, t.v_cache, t.pos_cache) for t in tr]
    h1, caches = orc.decode_step(x[N], int(pos[N]), ws, mdl, caches)
    h2, caches = orc.decode_step(x[N + 1], int(pos[N + 1]), ws, mdl, caches)
    assert np.allclose(h1, full_x[N], rtol=1e-10, atol=1e-12)
    assert np.allclose(h2, full_x[N + 1], rtol=1e-10, atol=1e-12)


def test_decode_attention_against_loops_over_a_compressed_cache():
    """The cache left by a skip layer holds the active pairs only (Sec. 3.2 last paragraph); the new
    token's attention is a softmax over exactly those pairs plus its own, per query head with the
    grouped KV head (written out with Python loops)."""
    shape = small_shape()
    mdl = oracle_model(shape)
    w = synth.make_layer(5, 0, shape, 8)
    N = 24
    x = synth.hidden_states(5, N, shape.D)
    pos = synth.positions(N)
    lo = orc.layer_prefill(x, pos, w, mdl, orc.LayerCfg(1, 4, 9, 9, 1, 0))
    assert lo.k_cache.shape[0] == 9 and np.array_equal(lo.pos_cache, pos[lo.idx_attn])
    cache = orc.LayerCache(lo.k_cache, lo.v_cache, lo.pos_cache)
    xt = synth.hidden_states(77, 1, shape.D)[0].astype(np.float64)
    out, c2 = orc.decode_layer(xt, N, w, mdl, cache)
    assert c2.k.shape[0] == 10 and c2.pos[-1] == N

    # by hand
    f = lambda a: np.asarray(a, dtype=np.float64)
    xn = xt / math.sqrt(np.mean(xt * xt) + shape.rms_eps) * f(w["gamma1"])
    H, Hkv, d = shape.H, shape.Hkv, shape.d

    def rot(vec, p):
        o = vec.copy()
        for j in range(d // 2):
            th = p * shape.rope_base ** (-2.0 * j / d)
            a, b = vec[j], vec[j + d // 2]
            o[j] = a * math.cos(th) - b * math.sin(th)
            o[j + d // 2] = b * math.cos(th) + a * math.sin(th)
        return o

    q = (xn @ f(w["Wq"])).reshape(H, d)
    kn = (xn @ f(w["Wk"])).reshape(Hkv, d)
    vn = (xn @ f(w["Wv"])).reshape(Hkv, d)
    att = np.zeros((H, d))
    for h in range(H):
        g = h // (H // Hkv)
        qh = rot(q[h], N)
        keys = [cache.k[m, g] for m in range(9)] + [rot(kn[g], N)]
        vals = [cache.v[m, g] for m in range(9)] + [vn[g]]
        logit = [float(np.dot(qh, kk)) / math.sqrt(d) for kk in keys]
        mx = max(logit)
        e = [math.exp(l - mx) for l in logit]
        for m in range(10):
            att[h] += e[m] / sum(e) * vals[m]
    x1 = xt + att.reshape(-1) @ f(w["Wo"])
    xn2 = x1 / math.sqrt(np.mean(x1 * x1) + shape.rms_eps) * f(w["gamma2"])
    g_ = xn2 @ f(w["Wgate"]); u_ = xn2 @ f(w["Wup"])
    x2 = x1 + ((g_ / (1 + np.exp(-g_))) * u_) @ f(w["Wdown"]).T
    assert np.allclose(out, x2, rtol=1e-10, atol=1e-12)
    assert np.allclose(c2.k[-1], np.stack([rot(kn[g], N) for g in range(Hkv)]), rtol=1e-12, atol=1e-14)
    assert np.allclose(c2.v[-1], vn, rtol=1e-12, atol=1e-14)


def test_decode_is_invariant_under_a_permutation_of_the_cache_rows():
    shape = small_shape()
    mdl = oracle_model(shape)
    w = synth.make_layer(6, 0, shape, 8)
    N = 20
    lo = orc.layer_prefill(synth.hidden_states(6, N, shape.D), synth.positions(N), w, mdl, orc.LayerCfg(0, 1, N, N, 1, 0))
    xt = synth.hidden_states(78, 1, shape.D)[0]
    a, _ = orc.decode_layer(xt, N + 3, w, mdl, orc.LayerCache(lo.k_cache, lo.v_cache, lo.pos_cache))
    perm = np.random.default_rng(0).permutation(N)
    b, _ = orc.decode_layer(xt, N + 3, w, mdl, orc.LayerCache(lo.k_cache[perm], lo.v_cache[perm], lo.pos_cache[perm]))
    assert np.allclose(a, b, rtol=1e-11, atol=1e-13)
    # and it does depend on the cache: dropping a pair changes the result
    c, _ = orc.decode_layer(xt, N + 3, w, mdl, orc.LayerCache(lo.k_cache[1:], lo.v_cache[1:], lo.pos_cache[1:]))
    assert not np.allclose(a, c, rtol=1e-6, atol=1e-9)


def test_greedy_token_is_argmax_of_normed_projection_with_lowest_index_ties():
    shape = small_shape()
    mdl = oracle_model(shape)
    rng = np.random.default_rng(3)
    table = rng.standard_normal((50, shape.D))
    table[37] = table[12]                      # identical rows -> identical logits
    h = rng.standard_normal(shape.D)
    gamma = 1.0 + 0.1 * rng.standard_normal(shape.D)
    tok, logits = orc.greedy_token(h, gamma, table, mdl)
    hn = h / math.sqrt(np.mean(h * h) + shape.rms_eps) * gamma
    ref = table @ hn
    assert np.allclose(logits, ref, rtol=1e-12, atol=1e-12)
    assert tok == int(np.argmax(ref))
    # force the tie to be the maximum: the lower id wins
    h2 = table[12] / gamma * 10.0
    tok2, lg2 = orc.greedy_token(h2, gamma, table, mdl)
    assert lg2[12] == lg2[37] and tok2 == 12
