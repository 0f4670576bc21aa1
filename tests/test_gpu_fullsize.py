"""GPU parity at the full sizes of the benchmark configurations (synth.WORKLOADS), in the launch configuration that
bench.py times (matrix-core kernels, 8B-shaped bf16 layer).

* c1 (N = 8192): the whole layer against the oracle, lock-step.
* c2 (N = 32768): the whole 32-layer stack; the first layer of every stage and the last layer on sampled
  rows the oracle computes one by one from the GPU's own layer input, plus, on every layer, properties
  that hold at any size (selection = oracle TopK of the GPU's scores, untouched rows, all three
  compaction maps, score sum).
* c3 (N = 131072): properties of the probe / TopK / skip rule at long length.
"""

import numpy as np
import pytest

from oracle import spts_oracle as orc
from paper_2601_13155_amd import runtime, synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

_CACHE = {}


def llama_layer():
    if "w" not in _CACHE:
        wl = synth.WORKLOADS["c1"]
        _CACHE["w"] = synth.make_layer(wl.seed, 0, wl.shape, wl.r)
        _CACHE["dw"] = runtime.upload_layer(_CACHE["w"], wl.shape, wl.r)
    return _CACHE["w"], _CACHE["dw"]


def ctx_for(max_tokens):
    key = ("ctx", max_tokens)
    if key not in _CACHE:
        shape = synth.LLAMA8B
        _CACHE[key] = runtime.make_context(shape, max_tokens, 128, 256, shape.Dff)
    return _CACHE[key]


def test_c1_full_layer_lockstep():
    import torch
    wl = synth.WORKLOADS["c1"]
    shape = wl.shape
    w, dw = llama_layer()
    ctx = ctx_for(32768)
    assert ctx.uses_mfma()
    x = synth.hidden_states(wl.seed, wl.N, shape.D, shape.dtype)
    pos = synth.positions(wl.N)
    item = wl.layer_plan()[0]
    gpu = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=wl.probe_len, m_attn=item["m_attn"],
                            m_ffn=item["m_ffn"], protect_last=1)
    cfg = orc.LayerCfg(1, wl.probe_len, item["m_attn"], item["m_ffn"], 1, 0)
    res = H.lockstep_layer(gpu, x, pos, w, H.oracle_model(shape), cfg, shape.dtype)
    print(f"c1: swaps attn={res['swaps_attn']} ffn={res['swaps_ffn']} hidden err={res['err']:.3e}")
    assert res["swaps_attn"] <= item["m_attn"] // 50 and res["swaps_ffn"] <= item["m_ffn"] // 50
    assert np.array_equal(gpu["idx_attn"], orc.topk_select(gpu["s_mha"], item["m_attn"], 1))
    torch.cuda.empty_cache()


def _sampled_layer_check(x_in, pos, w, shape, cfg, gpu, n_samples, seed):
    """Oracle on sampled rows of one skip layer (kv_mode 0), from the GPU's own layer input.
    Checks S^MHA everywhere, the selections (swap-counted), and the output hidden state of sampled
    rows (active in attention and/or FFN) one by one."""
    mdl = H.oracle_model(shape)
    rnd = orc.bf16_round
    tol = H.TOL["bf16"]
    N = x_in.shape[0]
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    xn = rnd(orc.rmsnorm(x_in, w["gamma1"], mdl.rms_eps))
    K = orc.project_keys(xn, pos, w["Wk"], mdl, rnd)
    P = cfg.probe_len
    qp = orc.project_queries(xn[N - P:], pos[N - P:], w["Wq"], mdl, rnd)
    S = orc.f32_round(orc.probe_scores(qp, K, mdl))
    assert H.score_rel_err(gpu["s_mha"], S) <= tol["score"]
    Ma = min(N, cfg.m_attn)
    swaps_a = H.count_swaps(gpu["idx_attn"], orc.topk_select(S, Ma, 1), S, tol["score"], 1)
    Ta = gpu["idx_attn"]
    rng = np.random.default_rng(seed)
    # sampled active rows (always include the first, the last and a few early ones)
    pick = np.unique(np.concatenate([[0, 1, Ma - 1], rng.choice(Ma, size=n_samples, replace=False)]))
    Vh = rnd((xn[Ta] @ f64(w["Wv"])).reshape(Ma, mdl.Hkv, mdl.d))
    Kh = K[Ta]
    x_new = {}
    for i in pick:
        row = int(Ta[i])
        q = orc.project_queries(xn[row:row + 1], pos[row:row + 1], w["Wq"], mdl, rnd)
        att = rnd(orc.causal_attention(q, Kh[: i + 1], Vh[: i + 1], pos[row:row + 1], pos[Ta[: i + 1]], mdl))
        o = att.reshape(1, -1) @ f64(w["Wo"])
        x_new[row] = rnd(f64(x_in[row]) + o[0])
    # FFN half on sampled rows: rows whose post-attention state is known = sampled active rows, and
    # inactive rows (unchanged by attention)
    inactive = np.setdiff1d(np.arange(N), Ta)
    extra = rng.choice(inactive, size=min(n_samples, inactive.size), replace=False)
    rows = np.concatenate([np.array(sorted(x_new.keys()), dtype=np.int64), extra])
    x_mid = np.stack([x_new[r] if r in x_new else f64(x_in[r]) for r in rows])
    xn2 = rnd(orc.rmsnorm(x_mid, w["gamma2"], mdl.rms_eps))
    in_f = np.isin(rows, gpu["idx_ffn"])
    upd = orc.ffn(xn2[in_f], w["Wgate"], w["Wup"], w["Wdown"], rnd)
    x_out = x_mid.copy()
    x_out[in_f] = rnd(x_mid[in_f] + upd)
    err = H.row_rel_err(gpu["x"][rows], x_out)
    assert err <= tol["hidden"], f"sampled rows: {err}"
    assert in_f.any() and (~in_f).any()
    return swaps_a, err, len(rows)


def test_c2_whole_stack_properties_and_sampled_layers():
    import torch
    wl = synth.WORKLOADS["c2"]
    shape = wl.shape
    w, dw = llama_layer()
    ctx = ctx_for(32768)
    plan = wl.layer_plan()
    x0 = synth.hidden_states(wl.seed, wl.N, shape.D, shape.dtype)
    pos0 = synth.positions(wl.N)
    # the whole 32-layer stack (three stage ends) with the bench's runner
    n_layers = wl.layers
    runner = runtime.StackRunner(ctx, shape, [dw] * n_layers, plan[:n_layers], wl.probe_len, keep_trace=True)
    xo, po, n_final = runner.run(runtime.to_device(x0, shape.dtype), torch.from_numpy(pos0).cuda())
    torch.cuda.synchronize()
    assert n_final == 11468
    for li, (tr, item) in enumerate(zip(runner.trace, plan[:n_layers])):
        N = tr["N"]
        s = tr["s_mha"].cpu().numpy()
        ia = tr["idx_attn"][: item["m_attn"]].cpu().numpy()
        iff = tr["idx_ffn"][: item["m_ffn"]].cpu().numpy()
        assert abs(float(s.astype(np.float64).sum()) - 1.0) < 2e-3 and s.min() >= 0.0
        # level A: the selection is the oracle's TopK of the scores the GPU stored
        assert np.array_equal(ia, orc.topk_select(s, item["m_attn"], 1)), li
        assert np.all(np.diff(iff) > 0) and iff[-1] == N - 1 and iff.size == item["m_ffn"]
        # Eq. (skip): rows outside both active sets are bitwise untouched
        touched = torch.zeros(N, dtype=torch.bool, device="cuda")
        touched[tr["idx_attn"][: item["m_attn"]].long()] = True
        touched[tr["idx_ffn"][: item["m_ffn"]].long()] = True
        assert torch.equal(tr["x_in"][~touched], tr["x_out"][~touched]), li
        changed = (tr["x_in"][touched] != tr["x_out"][touched]).any(dim=1).float().mean().item()
        assert changed > 0.99, (li, changed)
        if item["N_next"] is not None:
            n2o = tr["map_new2old"].cpu().numpy()
            assert np.array_equal(n2o, orc.topk_select(s, item["N_next"], 1))
            nxt = runner.trace[li + 1]
            assert torch.equal(nxt["x_in"], tr["x_out"][tr["map_new2old"].long()])          # bitwise row copies
            assert torch.equal(nxt["pos_in"], tr["pos_in"][tr["map_new2old"].long()])
    assert bool(torch.isfinite(xo.float()).all())
    # first layer of every stage and the last layer: sampled rows against the oracle, from the GPU's own layer input
    for li in (0, 8, 16, 24, n_layers - 1):
        tr = runner.trace[li]
        item = plan[li]
        gpu = dict(x=runtime.to_host(tr["x_out"]).astype(np.float64), s_mha=tr["s_mha"].cpu().numpy(),
                   idx_attn=tr["idx_attn"][: item["m_attn"]].cpu().numpy(), idx_ffn=tr["idx_ffn"][: item["m_ffn"]].cpu().numpy())
        cfg = orc.LayerCfg(1, wl.probe_len, item["m_attn"], item["m_ffn"], 1, 0)
        x_in = runtime.to_host(tr["x_in"]).astype(np.float64)
        swaps, err, n_rows = _sampled_layer_check(x_in, tr["pos_in"].cpu().numpy(), w, shape, cfg, gpu,
                                                  n_samples=24 if li == 0 else 10, seed=7 + li)
        print(f"c2 layer {li + 1} (N={tr['N']}): attention-set swaps={swaps} sampled rows={n_rows} err={err:.3e}", flush=True)
        assert swaps <= item["m_attn"] // 50
    del runner
    torch.cuda.empty_cache()


def test_c4_qwen_shaped_layer_lockstep():
    """Config c4's layer shape (D = 3584, 28 query / 4 KV heads: 7 query heads per KV head, Dff = 18944) at
    N = 4096: the whole layer against the oracle, lock-step, plus a stage-end compaction and two decode steps
    over the layer's compressed cache."""
    import torch
    wl = synth.WORKLOADS["c4"]
    shape = wl.shape
    N = 4096
    w = synth.make_layer(wl.seed, 0, shape, wl.r)
    dw = runtime.upload_layer(w, shape, wl.r)
    ctx = runtime.make_context(shape, N, wl.probe_len, wl.r, shape.Dff)
    assert ctx.uses_mfma()
    x = synth.hidden_states(wl.seed, N, shape.D, shape.dtype)
    pos = synth.positions(N)
    m_attn, m_ffn = int(wl.attn_keep * N), int(wl.ffn_keep * N)
    gpu = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=wl.probe_len, m_attn=m_attn, m_ffn=m_ffn,
                            protect_last=1)
    cfg = orc.LayerCfg(1, wl.probe_len, m_attn, m_ffn, 1, 0)
    res = H.lockstep_layer(gpu, x, pos, w, H.oracle_model(shape), cfg, shape.dtype)
    print(f"c4 layer: swaps attn={res['swaps_attn']} ffn={res['swaps_ffn']} hidden err={res['err']:.3e}")
    assert res["swaps_attn"] <= m_attn // 50 and res["swaps_ffn"] <= m_ffn // 50
    # stage-end pruning to 0.7 N with the layer's scores
    n_next = int(0.7 * N)
    xd = runtime.to_device(gpu["x"].astype(np.float32), shape.dtype)
    sd = torch.from_numpy(gpu["s_mha"]).cuda()
    pd = torch.from_numpy(pos).cuda()
    xo = torch.empty((n_next, shape.D), dtype=xd.dtype, device="cuda")
    po = torch.empty(n_next, dtype=torch.int32, device="cuda")
    n2o = torch.empty(n_next, dtype=torch.int32, device="cuda")
    o2n = torch.empty(N, dtype=torch.int32, device="cuda")
    ctx.spts_msdp_compact(xd, pd, sd, N, n_next, 1, xo, po, n2o, o2n)
    rx, rp, rn2o, ro2n = orc.msdp_compact(gpu["x"], pos, gpu["s_mha"], n_next, 1)
    assert np.array_equal(n2o.cpu().numpy(), rn2o) and np.array_equal(o2n.cpu().numpy(), ro2n)
    assert np.array_equal(po.cpu().numpy(), rp)
    assert torch.equal(xo, xd[n2o.long()])
    # decode over this layer's compressed cache (7 query heads per KV head; D and Dff of the Qwen shape)
    from paper_2601_13155_amd import binding
    cache = runtime.KVCache(shape, m_attn + 2)
    xd2 = runtime.to_device(x, shape.dtype)
    ctx.spts_layer_prefill(xd2, pd, N, dw, binding.spts_layer_cfg(1, wl.probe_len, m_attn, m_ffn, 1, 0), cache.struct,
                           None, None, None)
    torch.cuda.synchronize()
    assert cache.count == m_attn
    mdl = H.oracle_model(shape)
    new = synth.hidden_states(91, 3, shape.D, shape.dtype)[1:]
    for t in range(2):
        kh, vh, ph = cache.host()
        xt = runtime.to_device(new[t:t + 1].copy(), shape.dtype).reshape(-1)
        x_in = runtime.to_host(xt).astype(np.float64)
        ctx.spts_decode_layer(xt, N + t, dw, cache.struct)
        torch.cuda.synchronize()
        ref_x, ref_c = orc.decode_layer(x_in, N + t, w, mdl, orc.LayerCache(kh, vh, ph), orc.bf16_round)
        got = runtime.to_host(xt).astype(np.float64)
        err = H.row_rel_err(got[None, :], ref_x[None, :])
        print(f"c4 decode step {t}: hidden err {err:.3e}")
        assert err <= H.TOL["bf16"]["hidden"]
        k2, v2, p2 = cache.host()
        assert H.row_rel_err(k2[-1].reshape(1, -1), ref_c.k[-1].reshape(1, -1)) <= H.TOL["bf16"]["hidden"]
        assert H.row_rel_err(v2[-1].reshape(1, -1), ref_c.v[-1].reshape(1, -1)) <= H.TOL["bf16"]["hidden"]
    del ctx, dw
    torch.cuda.empty_cache()


def test_c3_long_sequence_properties():
    import torch
    wl = synth.WORKLOADS["c3"]
    shape = wl.shape
    w, dw = llama_layer()
    ctx = ctx_for(131072)
    item = wl.layer_plan()[0]
    N = wl.N
    x = synth.hidden_states(wl.seed, N, shape.D, shape.dtype)
    pos = synth.positions(N)
    gpu = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=wl.probe_len, m_attn=item["m_attn"],
                            m_ffn=item["m_ffn"], protect_last=1, want_kv=True)
    s = gpu["s_mha"]
    assert abs(float(s.astype(np.float64).sum()) - 1.0) < 2e-3 and s.min() >= 0.0
    assert np.array_equal(gpu["idx_attn"], orc.topk_select(s, item["m_attn"], 1))
    assert gpu["idx_ffn"].size == item["m_ffn"] and np.all(np.diff(gpu["idx_ffn"]) > 0) and gpu["idx_ffn"][-1] == N - 1
    touched = np.zeros(N, bool); touched[gpu["idx_attn"]] = True; touched[gpu["idx_ffn"]] = True
    assert np.array_equal(gpu["x"][~touched], x[~touched].astype(np.float64))
    assert np.all(np.isfinite(gpu["x"]))
    # cached keys of sampled active rows against the oracle (rotary at positions up to 131071)
    mdl = H.oracle_model(shape)
    rng = np.random.default_rng(3)
    sel = np.unique(np.concatenate([[0, item["m_attn"] - 1], rng.choice(item["m_attn"], 64, replace=False)]))
    rows = gpu["idx_attn"][sel]
    xn = orc.bf16_round(orc.rmsnorm(x[rows], w["gamma1"], mdl.rms_eps))
    k_ref = orc.project_keys(xn, pos[rows], w["Wk"], mdl, orc.bf16_round)
    assert H.row_rel_err(gpu["k_cache"][sel].reshape(len(sel), -1), k_ref.reshape(len(sel), -1)) <= H.TOL["bf16"]["hidden"]
    assert np.array_equal(gpu["pos_cache"], pos[gpu["idx_attn"]]) and gpu["kv_count"] == item["m_attn"]
    torch.cuda.empty_cache()


def test_paper_schedule_layer_lockstep():
    """An 8B-shaped skip layer with the paper's own settings (Sec. 4.1): single-row probe, absolute budget,
    proxy on Dlow = 512 channels with rank 192 stored zero-padded to 256; N = 8192, matrix-core kernels."""
    import torch
    wl = synth.WORKLOADS["p32"]
    shape = wl.shape
    w = synth.make_layer(wl.seed, 11, shape, wl.r, wl.dlow, wl.r_pad)
    assert w["Vg"].shape == (256, 512) and w["Vd"].shape == (256, 512)
    dw = runtime.upload_layer(w, shape, wl.proxy_r)
    ctx = ctx_for(32768)
    N, budget = 8192, 2304
    x = synth.hidden_states(wl.seed, N, shape.D, shape.dtype)
    pos = synth.positions(N)
    gpu = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=1, m_attn=budget, m_ffn=budget, protect_last=1)
    cfg = orc.LayerCfg(1, 1, budget, budget, 1, 0)
    res = H.lockstep_layer(gpu, x, pos, w, H.oracle_model(shape), cfg, shape.dtype)
    print(f"p32 layer: swaps attn={res['swaps_attn']} ffn={res['swaps_ffn']} hidden err={res['err']:.3e}")
    assert res["swaps_attn"] <= budget // 50 and res["swaps_ffn"] <= budget // 50
    assert np.array_equal(gpu["idx_attn"], orc.topk_select(gpu["s_mha"], budget, 1))
    del dw
    torch.cuda.empty_cache()


def test_qwen_paper_schedule_layer_lockstep():
    """A Qwen-shaped skip layer with the paper's settings for that model (Sec. 4.1): single-row probe,
    (Dlow, r) = (1024, 256), first-stage budget 13K of 32K scaled to N = 4096 (1664 active tokens)."""
    import torch
    wl = synth.WORKLOADS["q32"]
    shape = wl.shape
    N, budget = 4096, 1664
    w = synth.make_layer(wl.seed, 10, shape, wl.r, wl.dlow, wl.r_pad)
    assert w["Vg"].shape == (256, 1024) and w["Ug"].shape == (shape.D, 256)
    dw = runtime.upload_layer(w, shape, wl.proxy_r)
    ctx = runtime.make_context(shape, N, 1, wl.proxy_r, wl.proxy_dlow)
    assert ctx.uses_mfma()
    x = synth.hidden_states(wl.seed, N, shape.D, shape.dtype)
    pos = synth.positions(N)
    gpu = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=1, m_attn=budget, m_ffn=budget, protect_last=1)
    cfg = orc.LayerCfg(1, 1, budget, budget, 1, 0)
    res = H.lockstep_layer(gpu, x, pos, w, H.oracle_model(shape), cfg, shape.dtype)
    print(f"q32 layer: swaps attn={res['swaps_attn']} ffn={res['swaps_ffn']} hidden err={res['err']:.3e}")
    assert res["swaps_attn"] <= budget // 50 and res["swaps_ffn"] <= budget // 50
    assert np.array_equal(gpu["idx_attn"], orc.topk_select(gpu["s_mha"], budget, 1))
    del dw, ctx
    torch.cuda.empty_cache()


def test_decode_batched_8b_shaped_layer():
    """8B-shaped bf16 layer, five sequences: a batched token-skipped prefill fills the caches, then two batched decode
    steps on the matrix-core GEMV (K = 4096 and 14336: unrolled and tail k-steps); every sequence against the oracle."""
    import torch
    wl = synth.WORKLOADS["c1"]
    shape = wl.shape
    w, dw = llama_layer()
    ctx = ctx_for(32768)
    lens = [1500, 700, 64, 2048, 333]
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    xs = np.concatenate([synth.hidden_states(400 + b, n, shape.D, shape.dtype) for b, n in enumerate(lens)])
    ps = np.concatenate([synth.positions(n) for n in lens])
    ma = [int(0.4 * n) for n in lens]
    caches = [runtime.KVCache(shape, m + 2) for m in ma]
    kvs = [c.struct for c in caches]
    ctx.spts_layer_prefill_batched(runtime.to_device(xs, shape.dtype), torch.from_numpy(ps).cuda(), offs, dw, 64, ma, ma, 1, kvs)
    torch.cuda.synchronize()
    assert [k.count for k in kvs] == ma
    mdl = H.oracle_model(shape)
    new = synth.hidden_states(78, 2 * len(lens), shape.D, shape.dtype).reshape(2, len(lens), shape.D)
    for t in range(2):
        before = [c.host() for c in caches]
        xt = runtime.to_device(new[t].copy(), shape.dtype)
        x_in = runtime.to_host(xt).astype(np.float64)
        pos_t = [n + t for n in lens]
        ctx.spts_decode_layer_batched(xt, pos_t, dw, kvs)
        torch.cuda.synchronize()
        got = runtime.to_host(xt).astype(np.float64)
        for b in range(len(lens)):
            kh, vh, ph = before[b]
            ref_x, ref_c = orc.decode_layer(x_in[b], pos_t[b], w, mdl, orc.LayerCache(kh, vh, ph), orc.bf16_round)
            err = H.row_rel_err(got[b][None, :], ref_x[None, :])
            assert err <= H.TOL["bf16"]["hidden"], (t, b, err)
            k2, v2, p2 = caches[b].host()
            assert p2[-1] == pos_t[b] and k2.shape[0] == kh.shape[0] + 1
            assert H.row_rel_err(k2[-1].reshape(1, -1), ref_c.k[-1].reshape(1, -1)) <= H.TOL["bf16"]["hidden"]


def test_decode_8b_shaped_layer_after_skipped_prefill():
    """8B-shaped bf16 layer: token-skipped prefill of 8192 tokens fills the cache with the 3276 active pairs;
    two new tokens then go through spts_decode_layer, each checked against the oracle from the GPU's own
    input state and cache contents."""
    import torch
    from paper_2601_13155_amd import binding
    wl = synth.WORKLOADS["c1"]
    shape = wl.shape
    w, dw = llama_layer()
    ctx = ctx_for(32768)
    item = wl.layer_plan()[0]
    N = wl.N
    cache = runtime.KVCache(shape, item["m_attn"] + 2)
    cfg = binding.spts_layer_cfg(1, wl.probe_len, item["m_attn"], item["m_ffn"], 1, 0)
    xd = runtime.to_device(synth.hidden_states(wl.seed, N, shape.D, shape.dtype), shape.dtype)
    ctx.spts_layer_prefill(xd, torch.from_numpy(synth.positions(N)).cuda(), N, dw, cfg, cache.struct, None, None, None)
    torch.cuda.synchronize()
    assert cache.count == item["m_attn"] == 3276
    mdl = H.oracle_model(shape)
    new = synth.hidden_states(77, 3, shape.D, shape.dtype)[1:]
    for t in range(2):
        kh, vh, ph = cache.host()
        xt = runtime.to_device(new[t:t + 1].copy(), shape.dtype).reshape(-1)
        x_in = runtime.to_host(xt).astype(np.float64)
        ctx.spts_decode_layer(xt, N + t, dw, cache.struct)
        torch.cuda.synchronize()
        ref_x, ref_c = orc.decode_layer(x_in, N + t, w, mdl, orc.LayerCache(kh, vh, ph), orc.bf16_round)
        got = runtime.to_host(xt).astype(np.float64)
        err = H.row_rel_err(got[None, :], ref_x[None, :])
        print(f"decode step {t}: hidden err {err:.3e}")
        assert err <= H.TOL["bf16"]["hidden"]
        k2, v2, p2 = cache.host()
        assert p2[-1] == N + t and k2.shape[0] == kh.shape[0] + 1
        assert H.row_rel_err(k2[-1].reshape(1, -1), ref_c.k[-1].reshape(1, -1)) <= H.TOL["bf16"]["hidden"]
        assert H.row_rel_err(v2[-1].reshape(1, -1), ref_c.v[-1].reshape(1, -1)) <= H.TOL["bf16"]["hidden"]
    torch.cuda.empty_cache()


def test_channel_importance_8b_shaped():
    """Offline channel scores (Eq. (channel_importance)) for an 8B-shaped FFN on 1024 synthetic calibration
    tokens with rho = 0.2 (matrix-core saliency GEMM, channel-major), then the paper's Dlow = 512 selection."""
    import torch
    shape = synth.LLAMA8B
    w, dw = llama_layer()
    ctx = ctx_for(32768)
    T, k, dlow = 1024, 204, 512
    xc = synth.calibration_states(3, T, shape.D, shape.dtype)
    imp = torch.zeros(shape.Dff, dtype=torch.float32, device="cuda")
    ctx.spts_channel_importance(runtime.to_device(xc, shape.dtype), T, dw, k, imp)
    got = imp.cpu().numpy()
    ref = orc.channel_importance(xc, w["Wgate"], w["Wup"], k, orc.bf16_round)
    tol = H.TOL["bf16"]["score"]
    err = np.max(np.abs(got - ref)) / np.max(np.abs(ref))
    sel = torch.empty(dlow, dtype=torch.int32, device="cuda")
    ctx.spts_select_topk(imp, shape.Dff, dlow, 0, sel)
    sel = sel.cpu().numpy()
    assert np.array_equal(sel, orc.select_channels(got, dlow))
    swaps = H.count_swaps(sel, orc.select_channels(ref, dlow), ref, tol, 0)
    print(f"channel importance: max rel err {err:.3e}, selection swaps {swaps} of {dlow}")
    assert err <= tol
