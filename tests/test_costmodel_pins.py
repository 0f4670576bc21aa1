"""Pins of the host-side cost model against the two closed-form tables the paper prints."""
import os


from paper_2601_13155_amd import costmodel as cm

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                yield line.split()


def test_proxy_flops_table():
    D, Dff = 4096, 14336
    n_ok = 0
    for dlow, r, printed, consistent in _rows("proxy_flops_table.txt"):
        dl = None if dlow == "/" else int(dlow)
        rr = None if r == "/" else int(r)
        macs = cm.proxy_macs_per_token_per_projection(D, Dff, dl, rr)
        if consistent == "1":
            assert round(macs / 1000.0) == int(printed), (dlow, r, macs)
            n_ok += 1
        else:
            assert round(macs / 1000.0) != int(printed)
    assert n_ok == 5
    assert cm.proxy_macs_per_token_per_projection(D, Dff, 512, 192) == 884736


def test_kv_cache_memory_table():
    K = 1024
    for ctx, full, with_pap, saving in _rows("kv_cache_memory_table.txt"):
        N = int(ctx) * K
        # 10 dense layers, then stages of 4/5/5/5 layers with budgets 9/7/4/2 K; the three layers after
        # the last stage end run at the inferred next budget of 1 K.
        cached = cm.kv_cached_tokens(N, dense_layers=10, stage_layers=(4, 5, 5, 5, 3),
                                     budgets=(9 * K, 7 * K, 4 * K, 2 * K, 1 * K), prune_per_stage=K)
        ratio = cached / (32.0 * N)
        assert abs(ratio * float(full) - float(with_pap)) < 0.006, (ctx, ratio * float(full))
        assert abs((1.0 - ratio) * 100.0 - float(saving)) < 0.06


def test_paper_schedule_plan_reproduces_the_cache_table():
    """The layer plan of the paper-schedule workload (the object the stack driver executes) caches the
    same number of tokens as the closed form behind the KV-cache table, at every length of the table."""
    from paper_2601_13155_amd import synth
    K = 1024
    for ctx in (4, 8, 12, 16):
        wl = synth.scaled(synth.WORKLOADS["p32"], N=ctx * K)
        plan = wl.layer_plan()
        assert len(plan) == 32 and sum(1 - it["skip"] for it in plan) == 10
        cached = sum(min(it["N"], it["m_attn"]) for it in plan)
        assert cached == cm.kv_cached_tokens(ctx * K, dense_layers=10, stage_layers=(4, 5, 5, 5, 3),
                                             budgets=(9 * K, 7 * K, 4 * K, 2 * K, 1 * K), prune_per_stage=K)
    # 32K (beyond the table): 6.625 of 16 parts cached
    plan = synth.WORKLOADS["p32"].layer_plan()
    assert sum(min(it["N"], it["m_attn"]) for it in plan) / (32.0 * 32768) == 6.625 / 16


def test_layer_flops_matches_hand_count():
    # 8B-shaped layer at N = 8192, keep 0.4, P = 64, r = 256, Dlow = Dff
    f = cm.layer_flops(4096, 32, 8, 128, 14336, 8192, 64, 3276, 3276, 256, 14336)
    assert f["k_proj"] == 2.0 * 8192 * 4096 * 1024
    assert f["ffn"] == 2.0 * 3276 * 3 * 4096 * 14336
    assert abs(sum(f.values()) / 1e12 - 1.80) < 0.02
    dense = cm.layer_flops(4096, 32, 8, 128, 14336, 8192, 64, 8192, 8192, 256, 14336, skip=False)
    assert abs(sum(dense.values()) / 1e12 - 4.12) < 0.02


def test_component_toggles_and_qwen_schedule_plans():
    """Plans behind the component ablation (Table ablation_main_speed: PAP, +LTP, +MSDP) and the Qwen
    schedule of Sec. 4.1, checked against numbers written out by hand from the text."""
    from paper_2601_13155_amd import synth
    K = 1024
    q = synth.WORKLOADS["q32"].layer_plan()
    assert len(q) == 28 and [it["skip"] for it in q] == [0] * 9 + [1] * 19
    # stage ends after the 13th, 17th, 21st and 25th layer; 2K candidates go at each
    assert [it["layer"] for it in q if it["N_next"] is not None] == [13, 17, 21, 25]
    assert [it["N"] for it in q][9:] == [32 * K] * 4 + [30 * K] * 4 + [28 * K] * 4 + [26 * K] * 4 + [24 * K] * 3
    assert [it["m_attn"] for it in q][9:] == [13 * K] * 4 + [10 * K] * 4 + [7 * K] * 4 + [4 * K] * 4 + [1 * K] * 3
    assert all(it["m_attn"] == it["m_ffn"] for it in q)
    # at 8K the first LLaMA budget (9K) exceeds the sequence: min(N, M_fixed) keeps every token
    p8 = synth.scaled(synth.WORKLOADS["p32"], N=8 * K).layer_plan()
    assert [min(it["N"], it["m_attn"]) for it in p8][10:14] == [8 * K] * 4 and p8[14]["N"] == 7 * K
    for name in ("p32", "q32"):
        full = synth.WORKLOADS[name].layer_plan()
        nl = synth.scaled(synth.WORKLOADS[name], components="pap+ltp").layer_plan()
        pap = synth.scaled(synth.WORKLOADS[name], components="pap").layer_plan()
        for f, a, b in zip(full, nl, pap):
            assert a["N"] == b["N"] == 32 * K and a["N_next"] is None and b["N_next"] is None
            assert a["skip"] == b["skip"] == f["skip"]
            assert a["m_attn"] == b["m_attn"] == (f["m_attn"] if f["skip"] else 32 * K)   # same budgets, set never pruned
            assert a["m_ffn"] == a["m_attn"] and b["m_ffn"] == 32 * K                      # PAP alone: FFN for every token

