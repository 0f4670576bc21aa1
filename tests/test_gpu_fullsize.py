"""GPU parity at the full sizes of the benchmark configurations (synth.WORKLOADS), in the launch configuration that
bench.py times (matrix-core kernels, bf16 layers of the 8B and the Qwen shape).

* c1 (N = 8192): the whole layer against the oracle, lock-step, with the bf16-faithful oracle and with the plain
  fp64 algorithm (no intermediate rounding).
* c2 (N = 32768, 32 layers) and c4 (Qwen shape, 28 layers): the whole stack.  On every layer properties that hold at
  any size (attention selection = oracle TopK of the GPU's scores, untouched rows, compaction maps, score sum); on
  the first layer of every stage and the last layer S^MHA element-wise, the attention set swap-counted and sampled
  rows (attention over the active keys, FFN) the oracle computes one by one from the GPU's own layer input; on two
  layers the FFN selection against the oracle's TopK(C^FFN * S^MHA) over all candidates.  c4 then decodes 8 greedy
  tokens over its 28 ragged caches, every layer of every token against the oracle.
* c3 (N = 131072, P = 128): S^MHA element-wise, both selections swap-counted, sampled rows with attention over the
  32768 active keys.
"""

from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

from oracle import spts_oracle as orc
from paper_2601_13155_amd import binding, runtime, synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

_CACHE = {}


def _f64(w):
    """fp64 copies of a layer's matrices, made once: the oracle's own conversion is then free."""
    return {k: np.asarray(v, dtype=np.float64) for k, v in w.items()}


def llama_layer():
    if "w" not in _CACHE:
        wl = synth.WORKLOADS["c1"]
        _CACHE["w"] = _f64(synth.make_layer(wl.seed, 0, wl.shape, wl.r))
        _CACHE["dw"] = runtime.upload_layer(_CACHE["w"], wl.shape, wl.r)
    return _CACHE["w"], _CACHE["dw"]


def ctx_for(max_tokens):
    key = ("ctx", max_tokens)
    if key not in _CACHE:
        shape = synth.LLAMA8B
        _CACHE[key] = runtime.make_context(shape, max_tokens, 128, 256, shape.Dff)
    return _CACHE[key]


def _rows_parallel(fn, n_rows, chunk=4096, workers=8):
    """fn(lo, hi) over row chunks on a few host threads (numpy releases the GIL); results concatenated in row order.
    Only used for row-independent steps of the oracle, so chunking changes no value."""
    spans = [(lo, min(lo + chunk, n_rows)) for lo in range(0, n_rows, chunk)]
    with ThreadPoolExecutor(max_workers=workers) as ex:
        parts = list(ex.map(lambda s: fn(*s), spans))
    return np.concatenate(parts, axis=0)


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
    print(f"c1: swaps attn={res['swaps_attn']} ffn={res['swaps_ffn']} score err={res['s_err']:.3e} hidden err={res['err']:.3e}")
    assert res["swaps_attn"] <= item["m_attn"] // 50 and res["swaps_ffn"] <= item["m_ffn"] // 50
    # the same GPU result against the plain fp64 algorithm: no rounding anywhere inside the oracle
    res = H.lockstep_layer(gpu, x, pos, w, H.oracle_model(shape), cfg, shape.dtype, rnd=orc.identity)
    print(f"c1 vs plain fp64 oracle: swaps attn={res['swaps_attn']} ffn={res['swaps_ffn']} score err={res['s_err']:.3e} "
          f"hidden err={res['err']:.3e}")
    torch.cuda.empty_cache()


def _sampled_layer_check(x_in, pos, w, shape, cfg, gpu, n_samples, seed):
    """Oracle on sampled rows of one skip layer (kv_mode 0), from the GPU's own layer input.
    Checks S^MHA everywhere, the attention selection (swap-counted), and the output hidden state of sampled
    rows (active in attention and/or FFN) one by one.  Returns (swaps, score error, hidden error, rows, S)."""
    mdl = H.oracle_model(shape)
    rnd = orc.bf16_prefill
    tol = H.TOL["bf16"]
    N = x_in.shape[0]
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    xn = _rows_parallel(lambda lo, hi: rnd(orc.rmsnorm(x_in[lo:hi], w["gamma1"], mdl.rms_eps)), N)
    K = _rows_parallel(lambda lo, hi: orc.project_keys(xn[lo:hi], pos[lo:hi], w["Wk"], mdl, rnd), N)
    P = cfg.probe_len
    qp = orc.project_queries(xn[N - P:], pos[N - P:], w["Wq"], mdl, rnd, prefill=True)
    S = orc.f32_round(orc.probe_scores(qp, K, mdl))
    s_err = H.score_rel_err(gpu["s_mha"], S)
    assert s_err <= tol["score"], f"S^MHA: {s_err}"
    Ma = min(N, cfg.m_attn)
    band = min(tol["score"], 2.0 * s_err / (1.0 - s_err) * (1.0 + 1e-6) + 1e-12)
    swaps_a = H.count_swaps(gpu["idx_attn"], orc.topk_select(S, Ma, 1), S, band, 1)
    assert swaps_a <= H.swap_bound(Ma, "bf16")
    Ta = gpu["idx_attn"]
    rng = np.random.default_rng(seed)
    # sampled active rows (always include the first, the last and a few early ones)
    pick = np.unique(np.concatenate([[0, 1, Ma - 1], rng.choice(Ma, size=n_samples, replace=False)]))
    xa = xn[Ta]
    Vh = _rows_parallel(lambda lo, hi: rnd((xa[lo:hi] @ f64(w["Wv"])).reshape(hi - lo, mdl.Hkv, mdl.d)), Ma)
    Kh = K[Ta]
    x_new = {}
    for i in pick:
        row = int(Ta[i])
        q = orc.project_queries(xn[row:row + 1], pos[row:row + 1], w["Wq"], mdl, rnd, prefill=True)
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
    return swaps_a, s_err, err, len(rows), S


def _ffn_selection_check(ctx, dw, w, shape, x_in_dev, pos_dev, cfg, idx_attn, idx_ffn, S_oracle):
    """Eq. (ffn_importance) / (ffn_selection) over ALL candidates of a layer at full size.  The GPU hands over its
    own post-attention state (the same layer call with an FFN budget of 0 stops after the attention update) and its
    own C^FFN / S^FFN on it (spts_probe_ffn); the oracle computes C^FFN from that state and multiplies by ITS
    S^MHA of the layer input.  Checks: the attention half is reproducible, the GPU's FFN set is the TopK of the
    GPU's S^FFN (bit-exact), C^FFN and S^FFN element-wise within tolerance, and the set against the oracle's TopK
    with near-tie swaps counted in the band the measured score error implies.  Returns (swaps, c_err, sf_err)."""
    import torch
    mdl = H.oracle_model(shape)
    rnd = orc.bf16_prefill
    tol = H.TOL["bf16"]["score"]
    N = int(x_in_dev.shape[0])
    Ma, Mf = min(N, cfg.m_attn), min(N, cfg.m_ffn)
    xm = x_in_dev.clone()
    s_dev = torch.zeros(N, dtype=torch.float32, device="cuda")
    ia = torch.zeros(Ma, dtype=torch.int32, device="cuda")
    ctx.spts_layer_prefill(xm, pos_dev, N, dw, binding.spts_layer_cfg(1, cfg.probe_len, cfg.m_attn, 0, 1, 0), None, s_dev, ia, None)
    assert np.array_equal(ia.cpu().numpy(), idx_attn), "the attention half is not reproducible"
    c_dev = torch.zeros(N, dtype=torch.float32, device="cuda")
    sf_dev = torch.zeros(N, dtype=torch.float32, device="cuda")
    ctx.spts_probe_ffn(xm, N, dw, s_dev, c_dev, sf_dev)
    torch.cuda.synchronize()
    sf_gpu = sf_dev.cpu().numpy()
    assert np.array_equal(idx_ffn, orc.topk_select(sf_gpu, Mf, 1)), "FFN set is not the TopK of the GPU's own S^FFN"
    x_mid = runtime.to_host(xm).astype(np.float64)
    C = _rows_parallel(lambda lo, hi: orc.transformation_scores(rnd(orc.rmsnorm(x_mid[lo:hi], w["gamma2"], mdl.rms_eps)), w, rnd), N)
    C = orc.f32_round(C)
    SF = orc.f32_round(C * S_oracle)
    c_err = H.score_rel_err(c_dev.cpu().numpy(), C)
    sf_err = H.score_rel_err(sf_gpu, SF)
    assert c_err <= tol and sf_err <= tol, (c_err, sf_err)
    band = min(tol, 2.0 * sf_err / (1.0 - sf_err) * (1.0 + 1e-6) + 1e-12)
    swaps = H.count_swaps(idx_ffn, orc.topk_select(SF, Mf, 1), SF, band, 1)
    assert swaps <= H.swap_bound(Mf, "bf16"), swaps
    return swaps, c_err, sf_err


def _stack_checks(tag, wl, w, dw, ctx, sampled, ffn_checked, caches=None):
    """The whole stack of workload `wl` on the GPU with the bench's runner, then the per-layer properties, the
    sampled-row oracle checks on the layers `sampled` and the FFN selection checks on `ffn_checked` (0-based)."""
    import torch
    shape = wl.shape
    plan = wl.layer_plan()
    n_layers = wl.layers
    x0 = synth.hidden_states(wl.seed, wl.N, shape.D, shape.dtype)
    pos0 = synth.positions(wl.N)
    runner = runtime.StackRunner(ctx, shape, [dw] * n_layers, plan[:n_layers], wl.probe_len, keep_trace=True, caches=caches)
    xo, po, n_final = runner.run(runtime.to_device(x0, shape.dtype), torch.from_numpy(pos0).cuda())
    torch.cuda.synchronize()
    assert n_final == wl.stage_sizes()[-1]
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
        if caches is not None:
            assert caches[li].count == item["m_attn"]
            assert torch.equal(caches[li].pos[: item["m_attn"]], tr["pos_in"][tr["idx_attn"][: item["m_attn"]].long()])
        if item["N_next"] is not None:
            n2o = tr["map_new2old"].cpu().numpy()
            assert np.array_equal(n2o, orc.topk_select(s, item["N_next"], 1))
            nxt = runner.trace[li + 1]
            assert torch.equal(nxt["x_in"], tr["x_out"][tr["map_new2old"].long()])          # bitwise row copies
            assert torch.equal(nxt["pos_in"], tr["pos_in"][tr["map_new2old"].long()])
    assert bool(torch.isfinite(xo.float()).all())
    for li in sampled:
        tr = runner.trace[li]
        item = plan[li]
        gpu = dict(x=runtime.to_host(tr["x_out"]).astype(np.float64), s_mha=tr["s_mha"].cpu().numpy(),
                   idx_attn=tr["idx_attn"][: item["m_attn"]].cpu().numpy(), idx_ffn=tr["idx_ffn"][: item["m_ffn"]].cpu().numpy())
        cfg = orc.LayerCfg(1, wl.probe_len, item["m_attn"], item["m_ffn"], 1, 0)
        x_in = runtime.to_host(tr["x_in"]).astype(np.float64)
        swaps, s_err, err, n_rows, S = _sampled_layer_check(x_in, tr["pos_in"].cpu().numpy(), w, shape, cfg, gpu,
                                                            n_samples=24 if li == 0 else 10, seed=7 + li)
        msg = f"{tag} layer {li + 1} (N={tr['N']}): S^MHA err={s_err:.2e} attention-set swaps={swaps}/{item['m_attn']} sampled rows={n_rows} err={err:.3e}"
        if li in ffn_checked:
            sw_f, c_err, sf_err = _ffn_selection_check(ctx, dw, w, shape, tr["x_in"], tr["pos_in"], cfg, gpu["idx_attn"],
                                                       gpu["idx_ffn"], S)
            msg += f"; FFN-set swaps={sw_f}/{item['m_ffn']} C^FFN err={c_err:.2e} S^FFN err={sf_err:.2e}"
        print(msg, flush=True)
    del runner
    torch.cuda.empty_cache()


def test_c2_whole_stack_properties_and_sampled_layers():
    wl = synth.WORKLOADS["c2"]
    w, dw = llama_layer()
    _stack_checks("c2", wl, w, dw, ctx_for(32768), sampled=(0, 8, 16, 24, wl.layers - 1), ffn_checked=(0, 24))


def test_c4_qwen_stack_then_greedy_decode_lockstep():
    """Config c4 at size: the 28-layer Qwen-shaped stack (7 query heads per KV head, D = 3584, Dff = 18944) at
    N = 32768 with its three stage ends, filling 28 ragged caches; then 8 greedy decode steps over those caches,
    every layer of every token against the oracle from the GPU's own input state and cache contents (Alg. 1 with
    Is_prefill_phase false), and the token decision on the GPU's own logits."""
    import torch
    wl = synth.WORKLOADS["c4"]
    shape = wl.shape
    mdl = H.oracle_model(shape)
    w = _f64(synth.make_layer(wl.seed, 0, shape, wl.r))
    dw = runtime.upload_layer(w, shape, wl.r)
    ctx = runtime.make_context(shape, wl.N, wl.probe_len, wl.r, shape.Dff)
    assert ctx.uses_mfma()
    steps = 8
    plan = wl.layer_plan()
    caches = [runtime.KVCache(shape, it["m_attn"] + steps) for it in plan]
    _stack_checks("c4", wl, w, dw, ctx, sampled=(0, 7, 14, 21, wl.layers - 1), ffn_checked=(0, 21), caches=caches)
    assert [c.count for c in caches[::7]] == [13107, 9174, 6553, 4587]

    V = 8192
    table = synth.vocab_table(wl.seed, V, shape.D, shape.dtype)
    table64 = table.astype(np.float64)
    gamma_f = np.ones(shape.D, dtype=np.float32)
    td, gd = runtime.to_device(table, shape.dtype), runtime.to_device(gamma_f, shape.dtype)
    dec = runtime.DecodeRunner(ctx, shape, [dw] * wl.layers, caches, gd, td)
    dec.x.copy_(td[17])
    tol = H.TOL["bf16"]["hidden"]
    worst = 0.0
    for t in range(steps):
        pos_t = wl.N + t
        snaps = []
        for c in caches:
            kh, vh, ph = c.host()
            x_in = runtime.to_host(dec.x).astype(np.float64)
            ctx.spts_decode_layer(dec.x, pos_t, dw, c.struct)
            torch.cuda.synchronize()
            k2 = runtime.to_host(c.k[c.count - 1]).astype(np.float64)
            v2 = runtime.to_host(c.v[c.count - 1]).astype(np.float64)
            snaps.append((x_in, kh, vh, ph, runtime.to_host(dec.x).astype(np.float64), k2, v2, int(c.pos[c.count - 1])))

        def check(sn):
            x_in, kh, vh, ph, got, k2, v2, p2 = sn
            ref_x, ref_c = orc.decode_layer(x_in, pos_t, w, mdl, orc.LayerCache(kh, vh, ph), orc.bf16_round)
            assert p2 == pos_t
            return max(H.row_rel_err(got[None, :], ref_x[None, :]),
                       H.row_rel_err(k2.reshape(1, -1), ref_c.k[-1].reshape(1, -1)),
                       H.row_rel_err(v2.reshape(1, -1), ref_c.v[-1].reshape(1, -1)))

        with ThreadPoolExecutor(max_workers=8) as ex:
            errs = list(ex.map(check, snaps))
        assert max(errs) <= tol, (t, int(np.argmax(errs)), max(errs))
        worst = max(worst, max(errs))
        h = runtime.to_host(dec.x).astype(np.float64)
        dec.greedy()
        torch.cuda.synchronize()
        tok = int(dec.token[0])
        lg = dec.logits.cpu().numpy()
        ref_tok, ref_lg = orc.greedy_token(h, gamma_f, table64, mdl, orc.bf16_round, orc.f32_round)
        assert np.max(np.abs(lg - ref_lg)) <= tol * np.max(np.abs(ref_lg))
        assert tok == int(np.flatnonzero(lg == lg.max())[0])
        if tok != ref_tok:
            assert abs(ref_lg[tok] - ref_lg[ref_tok]) <= 2 * tol * np.max(np.abs(ref_lg))
        dec.x.copy_(dec.x_next)
        print(f"c4 decode step {t}: token {tok}, worst layer error {max(errs):.3e}", flush=True)
    assert [c.count for c in caches[::7]] == [13107 + steps, 9174 + steps, 6553 + steps, 4587 + steps]
    del ctx, dw, dec, caches
    torch.cuda.empty_cache()


def test_c4_qwen_shaped_layer_lockstep():
    """Config c4's layer shape (D = 3584, 28 query / 4 KV heads: 7 query heads per KV head, Dff = 18944) at
    N = 4096: the whole layer against the oracle, lock-step, plus a stage-end compaction."""
    import torch
    wl = synth.WORKLOADS["c4"]
    shape = wl.shape
    N = 4096
    w = _f64(synth.make_layer(wl.seed, 0, shape, wl.r))
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
    del ctx, dw
    torch.cuda.empty_cache()


def test_c3_long_sequence_against_the_oracle():
    """Config c3's first layer at N = 131072 with a 128-row probe window: S^MHA of all candidates element-wise
    against the oracle, the attention set (32768 of 131072) and the FFN set (39321) swap-counted, sampled rows
    with the reduced attention over up to 32768 active keys and the FFN, untouched rows, cached keys."""
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
    cfg = orc.LayerCfg(1, wl.probe_len, item["m_attn"], item["m_ffn"], 1, 0)
    swaps, s_err, err, n_rows, S = _sampled_layer_check(x.astype(np.float64), pos, w, shape, cfg, gpu, n_samples=16, seed=5)
    xd = runtime.to_device(x, shape.dtype)
    sw_f, c_err, sf_err = _ffn_selection_check(ctx, dw, w, shape, xd, torch.from_numpy(pos).cuda(), cfg, gpu["idx_attn"],
                                               gpu["idx_ffn"], S)
    print(f"c3 layer 1 (N={N}, P={wl.probe_len}): S^MHA err={s_err:.2e} attention-set swaps={swaps}/{item['m_attn']} "
          f"sampled rows={n_rows} err={err:.3e}; FFN-set swaps={sw_f}/{item['m_ffn']} C^FFN err={c_err:.2e} S^FFN err={sf_err:.2e}",
          flush=True)
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


def test_paper_proxy_built_on_the_gpu_then_layer_lockstep():
    """Sec. 3.3 end to end at the 8B shape with the paper's settings: channel scores over 2048 synthetic calibration
    rows with rho = 0.2, C = TopK(I, 512) on the GPU, rank-192 SVD of W[:, C] (stored zero-padded to 256) in the
    harness, then a single-row-probe skip layer at N = 8192 with that proxy, lock-step against the oracle, which
    selects its own channels (sets compared, near ties counted) and continues from the GPU's set."""
    import torch
    wl = synth.WORKLOADS["p32"]
    shape = wl.shape
    ctx = ctx_for(32768)
    base = synth.layer_weights(wl.seed, 12, shape)
    dw0 = runtime.upload_layer(base, shape, 0)
    T, dlow = 2048, wl.dlow
    k = int(0.2 * T)
    xc = synth.calibration_states(wl.seed, T, shape.D, shape.dtype)
    sel, imp = runtime.select_proxy_channels(ctx, dw0, shape, xc, k, dlow)
    ref_imp = orc.channel_importance(xc, base["Wgate"], base["Wup"], k, orc.bf16_round)
    tol = H.TOL["bf16"]["score"]
    assert np.max(np.abs(imp - ref_imp)) <= tol * np.max(np.abs(ref_imp))
    assert np.array_equal(sel, orc.select_channels(imp, dlow))
    swaps = H.count_swaps(sel, orc.select_channels(ref_imp, dlow), ref_imp, tol, 0)
    assert swaps <= H.swap_bound(dlow, "bf16")
    del dw0
    w = _f64(synth.make_layer(wl.seed, 12, shape, wl.r, r_pad=wl.r_pad, channels=sel))
    assert w["Vg"].shape == (256, 512)
    dw = runtime.upload_layer(w, shape, wl.proxy_r)
    N, budget = 8192, 2304
    x = synth.hidden_states(wl.seed, N, shape.D, shape.dtype)
    pos = synth.positions(N)
    gpu = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=1, m_attn=budget, m_ffn=budget, protect_last=1)
    res = H.lockstep_layer(gpu, x, pos, w, H.oracle_model(shape), orc.LayerCfg(1, 1, budget, budget, 1, 0), shape.dtype)
    print(f"built proxy: channel swaps {swaps}/{dlow}; layer swaps attn={res['swaps_attn']} ffn={res['swaps_ffn']} hidden err={res['err']:.3e}")
    del dw
    torch.cuda.empty_cache()

