"""GPU parity of the decode phase (one new token over the per-layer caches left by the prefill)
against the oracle, lock-step: at every step the oracle starts from the GPU's own input state and
the GPU's own cache contents, so differences do not accumulate across steps or layers."""
import numpy as np
import pytest

from oracle import spts_oracle as orc
from paper_2601_13155_amd import binding, runtime, synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

_CTX = {}


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available()
    return torch


def ctx_for(shape, max_tokens):
    key = (shape, max_tokens)
    if key not in _CTX:
        _CTX[key] = runtime.make_context(shape, max_tokens, 128, 256, shape.Dff)
    return _CTX[key]


def _shape(dtype):
    return synth.TINY if dtype == "f32" else synth.ModelShape(D=256, H=4, Hkv=2, d=64, Dff=688, dtype="bf16")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("skip", [1, 0])
def test_decode_layer_lockstep(torch, dtype, skip):
    """Prefill one layer on the GPU (token-skipped: the cache holds the active pairs only; or dense),
    then push three new tokens through spts_decode_layer."""
    shape = _shape(dtype)
    mdl = H.oracle_model(shape)
    rnd = H.rnd_for(dtype)
    tol = H.TOL[dtype]["hidden"]
    N, P, r = 300, 8, 16
    w = synth.make_layer(21, 0, shape, r)
    dw = runtime.upload_layer(w, shape, r)
    ctx = ctx_for(shape, 2048)
    x = synth.hidden_states(21, N, shape.D, dtype)
    pos = synth.positions(N)
    m = int(0.4 * N)
    cache = runtime.KVCache(shape, (m if skip else N) + 3)
    cfg = binding.spts_layer_cfg(skip, P, m, m, 1, 0)
    xd = runtime.to_device(x, dtype)
    ctx.spts_layer_prefill(xd, torch.from_numpy(pos).cuda(), N, dw, cfg, cache.struct, None, None, None)
    torch.cuda.synchronize()
    assert cache.count == (m if skip else N)
    new = synth.hidden_states(22, 3, shape.D, dtype)
    for t in range(3):
        kh, vh, ph = cache.host()
        xt = runtime.to_device(new[t:t + 1].copy(), dtype).reshape(-1)
        x_in = runtime.to_host(xt).astype(np.float64)
        ctx.spts_decode_layer(xt, N + t, dw, cache.struct)
        torch.cuda.synchronize()
        ref_x, ref_c = orc.decode_layer(x_in, N + t, w, mdl, orc.LayerCache(kh, vh, ph), rnd)
        got = runtime.to_host(xt).astype(np.float64)
        assert H.row_rel_err(got[None, :], ref_x[None, :]) <= tol, (t, H.row_rel_err(got[None, :], ref_x[None, :]))
        k2, v2, p2 = cache.host()
        assert k2.shape[0] == kh.shape[0] + 1 and p2[-1] == N + t
        assert np.array_equal(k2[:-1], kh) and np.array_equal(v2[:-1], vh) and np.array_equal(p2[:-1], ph)
        assert H.row_rel_err(k2[-1].reshape(1, -1), ref_c.k[-1].reshape(1, -1)) <= tol
        assert H.row_rel_err(v2[-1].reshape(1, -1), ref_c.v[-1].reshape(1, -1)) <= tol


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("nseq", [2, 3, 8, 16])
def test_decode_layer_batched_lockstep(torch, dtype, nseq):
    """A batch of sequences with caches of different lengths (one batched token-skipped prefill fills them), then two
    batched decode steps: every sequence's state and appended pair against the oracle's single-sequence decode from
    the GPU's own input state and cache contents; then the batched greedy head against the oracle per sequence."""
    shape = _shape(dtype)
    mdl = H.oracle_model(shape)
    rnd = H.rnd_for(dtype)
    tol = H.TOL[dtype]["hidden"]
    lens = [300, 45, 170, 64, 511, 33, 96, 257, 40, 129, 77, 18, 200, 31, 64, 99][:nseq]
    P, r = 8, 16
    w = synth.make_layer(23, 0, shape, r)
    dw = runtime.upload_layer(w, shape, r)
    ctx = ctx_for(shape, 4096)
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    xs = np.concatenate([synth.hidden_states(300 + b, n, shape.D, dtype) for b, n in enumerate(lens)])
    ps = np.concatenate([synth.positions(n) for n in lens])
    ma = [int(0.4 * n) for n in lens]
    caches = [runtime.KVCache(shape, m + 2) for m in ma]
    kvs = [c.struct for c in caches]
    ctx.spts_layer_prefill_batched(runtime.to_device(xs, dtype), torch.from_numpy(ps).cuda(), offs, dw, P, ma, ma, 1, kvs)
    torch.cuda.synchronize()
    assert [k.count for k in kvs] == ma
    new = synth.hidden_states(24, 2 * nseq, shape.D, dtype).reshape(2, nseq, shape.D)
    for t in range(2):
        before = [c.host() for c in caches]
        xt = runtime.to_device(new[t].copy(), dtype)
        x_in = runtime.to_host(xt).astype(np.float64)
        pos_t = [n + t for n in lens]
        ctx.spts_decode_layer_batched(xt, pos_t, dw, kvs)
        torch.cuda.synchronize()
        got = runtime.to_host(xt).astype(np.float64)
        for b in range(nseq):
            kh, vh, ph = before[b]
            ref_x, ref_c = orc.decode_layer(x_in[b], pos_t[b], w, mdl, orc.LayerCache(kh, vh, ph), rnd)
            assert H.row_rel_err(got[b][None, :], ref_x[None, :]) <= tol, (t, b)
            k2, v2, p2 = caches[b].host()
            assert k2.shape[0] == kh.shape[0] + 1 and p2[-1] == pos_t[b]
            assert np.array_equal(k2[:-1], kh) and np.array_equal(v2[:-1], vh) and np.array_equal(p2[:-1], ph)
            assert H.row_rel_err(k2[-1].reshape(1, -1), ref_c.k[-1].reshape(1, -1)) <= tol
            assert H.row_rel_err(v2[-1].reshape(1, -1), ref_c.v[-1].reshape(1, -1)) <= tol
    # greedy head over the batch
    V = 1000
    table = synth.vocab_table(7, V, shape.D, dtype)
    gamma_f = np.ones(shape.D, dtype=np.float32)
    td, gd = runtime.to_device(table, dtype), runtime.to_device(gamma_f, dtype)
    toks = torch.zeros(nseq, dtype=torch.int32, device="cuda")
    logits = torch.zeros((nseq, V), dtype=torch.float32, device="cuda")
    xnext = torch.zeros_like(xt)
    ctx.spts_greedy_token_batched(xt, gd, td, V, nseq, toks, logits, xnext)
    torch.cuda.synchronize()
    lg, tk = logits.cpu().numpy(), toks.cpu().numpy()
    for b in range(nseq):
        ref_tok, ref_logits = orc.greedy_token(got[b], gamma_f, table, mdl, rnd)
        assert np.max(np.abs(lg[b] - ref_logits)) <= tol * np.max(np.abs(ref_logits))
        assert tk[b] == int(np.flatnonzero(lg[b] == lg[b].max())[0])        # argmax of the GPU's logits, lowest id
        assert torch.equal(xnext[b], td[int(tk[b])])


def _fill_cache(torch, cache, shape, n, seed):
    """n cached pairs written directly, positions 0..n-1: seeded normal keys scaled by 4 (peaked attention) and values
    scaled by 8, so that the attention output dominates the layer's output and a misplaced key, value column or
    dropped tile shows in it (on the oracle alone: two swapped value columns move the output by 3-6 %, permuted keys
    by 30-40 %, a missing half of the values by 8-20 %, against the 2 % bar)."""
    rng = np.random.default_rng(seed)
    k = (4.0 * rng.standard_normal((n, shape.Hkv, shape.d))).astype(np.float32)
    v = (8.0 * rng.standard_normal((n, shape.Hkv, shape.d))).astype(np.float32)
    cache.k[:n].copy_(runtime.to_device(k, shape.dtype))
    cache.v[:n].copy_(runtime.to_device(v, shape.dtype))
    cache.pos[:n].copy_(torch.arange(n, dtype=torch.int32))
    cache.struct.count = n


_SHARP_SHAPES = {
    "bf16-d128-g1": synth.ModelShape(D=512, H=4, Hkv=4, d=128, Dff=1024, dtype="bf16"),
    "bf16-d128-g2": synth.ModelShape(D=512, H=4, Hkv=2, d=128, Dff=1024, dtype="bf16"),
    "bf16-d128-g4": synth.ModelShape(D=512, H=8, Hkv=2, d=128, Dff=1024, dtype="bf16"),
    "bf16-d128-g8": synth.ModelShape(D=512, H=8, Hkv=1, d=128, Dff=1024, dtype="bf16"),
    "bf16-d64": synth.ModelShape(D=256, H=4, Hkv=2, d=64, Dff=688, dtype="bf16"),
    "f32-tiny": synth.TINY,
}


@pytest.mark.parametrize("name", list(_SHARP_SHAPES))
def test_decode_attention_sharp_single_and_batched(torch, name):
    """Decode over caches whose attention output dominates the layer (see _fill_cache), with cache lengths on and
    around the kernel's step and split edges (0 cached pairs, 31 / 32 / 33 and 63 / 64 / 65 keys with the new pair, one
    split, many splits): bf16 with head dimension 128 and 1 / 2 / 4 / 8 query heads per KV head, bf16 with head
    dimension 64, fp32.  One sequence at a time, then the same caches as one batch."""
    shape = _SHARP_SHAPES[name]
    dt = shape.dtype
    mdl = H.oracle_model(shape)
    rnd = H.rnd_for(dt)
    tol = H.TOL[dt]["hidden"]
    w = synth.make_layer(41, 0, shape, 16)
    dw = runtime.upload_layer(w, shape, 16)
    ctx = ctx_for(shape, 4096)
    lens = [0, 30, 31, 32, 63, 64, 65, 700, 2049, 3000]
    caches = [runtime.KVCache(shape, n + 3) for n in lens]
    for b, (c, n) in enumerate(zip(caches, lens)):
        _fill_cache(torch, c, shape, n, 500 + b)
    new = synth.hidden_states(42, 2 * len(lens), shape.D, dt).reshape(2, len(lens), shape.D)

    def check(b, x_in, got, before, pos):
        kh, vh, ph = before
        ref_x, ref_c = orc.decode_layer(x_in, pos, w, mdl, orc.LayerCache(kh, vh, ph), rnd)
        assert H.row_rel_err(got[None, :], ref_x[None, :]) <= tol, (name, lens[b], H.row_rel_err(got[None, :], ref_x[None, :]))
        k2, v2, p2 = caches[b].host()
        assert k2.shape[0] == kh.shape[0] + 1 and p2[-1] == pos
        assert np.array_equal(k2[:-1], kh) and np.array_equal(v2[:-1], vh)
        assert H.row_rel_err(k2[-1].reshape(1, -1), ref_c.k[-1].reshape(1, -1)) <= tol

    for b, n in enumerate(lens):
        before = caches[b].host()
        xt = runtime.to_device(new[0, b:b + 1].copy(), dt).reshape(-1)
        x_in = runtime.to_host(xt).astype(np.float64)
        ctx.spts_decode_layer(xt, n, dw, caches[b].struct)
        torch.cuda.synchronize()
        check(b, x_in, runtime.to_host(xt).astype(np.float64), before, n)
    before = [c.host() for c in caches]
    xt = runtime.to_device(new[1].copy(), dt)
    x_in = runtime.to_host(xt).astype(np.float64)
    pos_t = [n + 1 for n in lens]
    ctx.spts_decode_layer_batched(xt, pos_t, dw, [c.struct for c in caches])
    torch.cuda.synchronize()
    got = runtime.to_host(xt).astype(np.float64)
    for b in range(len(lens)):
        check(b, x_in[b], got[b], before[b], pos_t[b])


def test_decode_rejects_a_full_cache(torch):
    shape = _shape("f32")
    w = synth.make_layer(21, 0, shape, 16)
    dw = runtime.upload_layer(w, shape, 16)
    ctx = ctx_for(shape, 2048)
    cache = runtime.KVCache(shape, 4)
    cache.struct.count = 4
    xt = torch.zeros(shape.D, dtype=torch.float32, device="cuda")
    with pytest.raises(binding.SptsError):
        ctx.spts_decode_layer(xt, 4, dw, cache.struct)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_stack_prefill_then_greedy_decode_lockstep(torch, dtype):
    """Token-skipped prefill of a 3-layer stack with stage-end pruning fills the per-layer caches (ragged:
    different lengths per layer); then 4 greedy decode steps.  Per step: every layer against the oracle
    from the GPU's own state, logits against the oracle, and the token is the oracle's argmax of the
    GPU's own logits (ties to the lowest id)."""
    shape = _shape(dtype)
    mdl = H.oracle_model(shape)
    rnd = H.rnd_for(dtype)
    tol = H.TOL[dtype]["hidden"]
    wl = synth.scaled(synth.WORKLOADS["c2"], shape=shape, N=400, layers=3, stage_end_layers=(1, 2), probe_len=16, r=16,
                      stage_cum_keep=(1.0, 0.7, 0.5))
    plan = wl.layer_plan()
    ws = [synth.make_layer(wl.seed, l, shape, wl.r) for l in range(wl.layers)]
    dws = [runtime.upload_layer(w, shape, wl.r) for w in ws]
    ctx = ctx_for(shape, 2048)
    steps = 4
    caches = [runtime.KVCache(shape, min(it["N"], it["m_attn"]) + steps) for it in plan]
    runner = runtime.StackRunner(ctx, shape, dws, plan, wl.probe_len, caches=caches)
    x0 = synth.hidden_states(wl.seed, wl.N, shape.D, dtype)
    runner.run(runtime.to_device(x0, dtype), torch.from_numpy(synth.positions(wl.N)).cuda())
    torch.cuda.synchronize()
    assert [c.count for c in caches] == [min(it["N"], it["m_attn"]) for it in plan] == [160, 112, 80]

    V = 1000
    table = synth.vocab_table(wl.seed, V, shape.D, dtype)
    gamma_f = np.ones(shape.D, dtype=np.float32)
    td, gd = runtime.to_device(table, dtype), runtime.to_device(gamma_f, dtype)
    dec = runtime.DecodeRunner(ctx, shape, dws, caches, gd, td)
    dec.x.copy_(td[17])          # first decode input: the table row of an arbitrary prompt-final token
    tokens = []
    for t in range(steps):
        # lock-step per layer
        for li, (w, dw, c) in enumerate(zip(ws, dws, caches)):
            kh, vh, ph = c.host()
            x_in = runtime.to_host(dec.x).astype(np.float64)
            ctx.spts_decode_layer(dec.x, wl.N + t, dw, c.struct)
            torch.cuda.synchronize()
            ref_x, _ = orc.decode_layer(x_in, wl.N + t, w, mdl, orc.LayerCache(kh, vh, ph), rnd)
            got = runtime.to_host(dec.x).astype(np.float64)
            assert H.row_rel_err(got[None, :], ref_x[None, :]) <= tol, (t, li)
        h = runtime.to_host(dec.x).astype(np.float64)
        dec.greedy()
        torch.cuda.synchronize()
        tok = int(dec.token[0])
        lg = dec.logits.cpu().numpy()
        ref_tok, ref_lg = orc.greedy_token(h, gamma_f, table, mdl, rnd, orc.f32_round)
        assert np.max(np.abs(lg - ref_lg)) <= tol * np.max(np.abs(ref_lg))
        assert tok == int(np.flatnonzero(lg == lg.max())[0])          # the decision, on the GPU's own logits
        if tok != ref_tok:                                             # only a near-tie may differ
            assert abs(ref_lg[tok] - ref_lg[ref_tok]) <= 2 * tol * np.max(np.abs(ref_lg))
        assert np.array_equal(runtime.to_host(dec.x_next), table[tok].astype(runtime.to_host(dec.x_next).dtype))
        tokens.append(tok)
        dec.x.copy_(dec.x_next)
    assert [c.count for c in caches] == [160 + steps, 112 + steps, 80 + steps]
    assert all(int(c.pos[c.count - 1]) == wl.N + steps - 1 for c in caches)
    assert len(set(tokens)) >= 1


def test_decode_is_deterministic_and_consistent_with_dense_prefill(torch):
    """Two identical decode calls give bitwise identical states (all merges run in a fixed order), and a dense
    GPU prefill of N tokens + one decode step lands within tolerance of the last row of a dense GPU prefill of
    N+1 tokens (the oracle pins the same identity for itself)."""
    dtype = "bf16"
    shape = _shape(dtype)
    N, r = 257, 16
    w = synth.make_layer(23, 0, shape, r)
    dw = runtime.upload_layer(w, shape, r)
    ctx = ctx_for(shape, 2048)
    x = synth.hidden_states(23, N + 1, shape.D, dtype)
    pos = torch.from_numpy(synth.positions(N + 1)).cuda()
    cfg = binding.spts_layer_cfg(0, 1, N + 1, N + 1, 1, 0)
    outs = []
    for rep in range(2):
        cache = runtime.KVCache(shape, N + 1)
        xd = runtime.to_device(x[:N].copy(), dtype)
        ctx.spts_layer_prefill(xd, pos[:N].contiguous(), N, dw, cfg, cache.struct, None, None, None)
        xt = runtime.to_device(x[N:N + 1].copy(), dtype).reshape(-1)
        ctx.spts_decode_layer(xt, N, dw, cache.struct)
        torch.cuda.synchronize()
        outs.append((xt.clone(), cache.k.clone(), cache.v.clone()))
    assert all(torch.equal(a, b) for a, b in zip(outs[0], outs[1]))
    full = runtime.to_device(x.copy(), dtype)
    ctx.spts_layer_prefill(full, pos, N + 1, dw, cfg, None, None, None, None)
    torch.cuda.synchronize()
    a = runtime.to_host(outs[0][0]).astype(np.float64)[None, :]
    b = runtime.to_host(full[N]).astype(np.float64)[None, :]
    assert H.row_rel_err(a, b) <= H.TOL[dtype]["hidden"]
