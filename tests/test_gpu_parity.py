"""GPU parity tests: every call goes through the C ABI and is compared with the CPU oracle.

Bar: index sets / compaction maps bit-exact (on identical fp32 scores); scores and hidden states
within the tolerance of tests/helpers.TOL (fp32 1e-4, bf16 2e-2, relative).
"""
import numpy as np
import pytest

from oracle import spts_oracle as orc
from paper_2601_13155_amd import binding, runtime, synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available()
    return torch


_CTX = {}


def ctx_for(shape, max_tokens, max_probe=128, max_r=256, max_dlow=None):
    key = (shape, max_tokens, max_probe, max_r, max_dlow or shape.Dff)
    if key not in _CTX:
        _CTX[key] = runtime.make_context(shape, max_tokens, max_probe, max_r, max_dlow or shape.Dff)
    return _CTX[key]


# ------------------------------------------------------------------------------------------ TopK
def _topk_cases(rng):
    # sizes straddle the register-resident variants of the kernel (8, 16, 32 keys per lane x 1024 lanes)
    for n in (1, 2, 63, 64, 65, 1000, 1024, 1025, 5000, 8192, 8193, 16384, 16385, 22937, 32768, 32769, 40000, 131072):
        yield "uniform", rng.random(n).astype(np.float32)
        yield "all_equal", np.full(n, 0.5, dtype=np.float32)
        z = rng.random(n).astype(np.float32); z[rng.random(n) < 0.7] = 0.0
        yield "many_zeros", z
        yield "duplicates", rng.integers(0, 5, n).astype(np.float32)
        e = np.exp(-rng.random(n) * 100).astype(np.float32); e[::7] = -0.0
        yield "softmax_like_signed_zero", e
        yield "tiny_denormal", (rng.random(n) * 1e-44).astype(np.float32)
        # probabilities of similar magnitude (what a probe produces): nearly all keys share their top bits
        yield "probability_like", ((1.0 + 0.3 * rng.standard_normal(n)).clip(0.05, None) / n).astype(np.float32)


def test_select_topk_bit_exact(torch):
    rng = np.random.default_rng(0)
    ctx = ctx_for(synth.TINY, 131072)
    for name, s in _topk_cases(rng):
        n = len(s)
        sd = torch.from_numpy(s).cuda()
        ks = sorted({0, 1, 2, n // 3, int(0.4 * n), n - 1, n})
        for k in ks:
            if k < 0 or k > n:
                continue
            for protect in (0, 1):
                out = torch.full((max(k, 1),), -7, dtype=torch.int32, device="cuda")
                ctx.spts_select_topk(sd, n, k, protect, out)
                got = out[:k].cpu().numpy()
                ref = orc.topk_select(s, k, protect)
                assert np.array_equal(got, ref), (name, n, k, protect)
                if k == 0:
                    assert int(out[0]) == -7

def test_select_topk_chip_wide_bit_exact(torch):
    """Rows longer than one workgroup's registers take the chip-wide radix select (a launch per pass over up to 128
    workgroups): lengths around its slice sizes (1, 2, 4 and 8 keys per lane) up to its maximum of 2^20 scores, back
    to back on one context (the scratch tables are reused from call to call), same adversarial value patterns."""
    rng = np.random.default_rng(1)
    shape = synth.ModelShape(D=32, H=1, Hkv=1, d=16, Dff=32, dtype="f32")
    ctx = runtime.make_context(shape, 1 << 20, 4, 4, 32)
    for n in (20000, 20001, 32769, 131071, 131073, 262144, 262145, 300001, 524288, 524289, (1 << 20) - 5, 1 << 20):
        cases = {
            "uniform": rng.random(n).astype(np.float32),
            "all_equal": np.full(n, 0.25, dtype=np.float32),
            "duplicates": rng.integers(0, 3, n).astype(np.float32),
            "probability_like": ((1.0 + 0.3 * rng.standard_normal(n)).clip(0.05, None) / n).astype(np.float32),
        }
        z = rng.random(n).astype(np.float32); z[rng.random(n) < 0.9] = 0.0; z[::5] = -0.0
        cases["many_signed_zeros"] = z
        for name, s in cases.items():
            sd = torch.from_numpy(s).cuda()
            for k in sorted({1, n // 4, int(0.3 * n), n - 1, n}):
                for protect in (0, 1):
                    out = torch.full((k,), -7, dtype=torch.int32, device="cuda")
                    ctx.spts_select_topk(sd, n, k, protect, out)
                    assert np.array_equal(out.cpu().numpy(), orc.topk_select(s, k, protect)), (name, n, k, protect)
    del ctx
    torch.cuda.empty_cache()



def test_select_topk_deterministic_and_nested(torch):
    rng = np.random.default_rng(1)
    ctx = ctx_for(synth.TINY, 131072)
    s = rng.random(100000).astype(np.float32)
    sd = torch.from_numpy(s).cuda()
    prev = None
    for k in (10, 1000, 40000, 99999):
        a = torch.empty(k, dtype=torch.int32, device="cuda")
        b = torch.empty(k, dtype=torch.int32, device="cuda")
        ctx.spts_select_topk(sd, len(s), k, 1, a)
        ctx.spts_select_topk(sd, len(s), k, 1, b)
        assert torch.equal(a, b)
        cur = set(a.cpu().numpy().tolist())
        if prev is not None:
            assert prev <= cur
        prev = cur


def test_select_topk_batched_rows_match_oracle(torch):
    rng = np.random.default_rng(2)
    ctx = ctx_for(synth.TINY, 131072)
    # 40000, 65540 and 131072 take the streaming long-row kernel (16-byte loads), 40001 the scalar one
    for n, batch in ((1000, 7), (8193, 5), (40000, 3), (40001, 2), (65540, 3), (131072, 2)):
        s = ((1.0 + 0.3 * rng.standard_normal((batch, n))).clip(0.05, None) / n).astype(np.float32)
        s[1, ::3] = s[1, 0]   # a row with many ties (long rows: more than a wavefront's LDS region holds -> the sweep fallback)
        s[0] = (np.exp(2.0 * rng.standard_normal(n)) / n).astype(np.float32)   # scores over many octaves (sparse histogram bins)
        if batch > 2:
            s[2, : n // 2] = s[2, 0]   # two values only: both routes of the long-row kernel meet ties at the threshold
            s[2, n // 2:] = s[2, n - 1]
        sd = torch.from_numpy(s).cuda()
        for k in (1, int(0.4 * n), n):
            out = torch.full((batch, k), -7, dtype=torch.int32, device="cuda")
            ctx.spts_select_topk_batched(sd, n, k, 1, batch, out)
            got = out.cpu().numpy()
            for b in range(batch):
                assert np.array_equal(got[b], orc.topk_select(s[b], k, 1)), (n, k, b)


def test_select_topk_segmented_matches_oracle_per_sequence(torch):
    rng = np.random.default_rng(4)
    ctx = ctx_for(synth.TINY, 131072)
    for lens in ((5, 1, 900, 64, 1025), (9000, 100, 8192), (20000, 3)):
        lens = np.array(lens, dtype=np.int64)
        offs = np.concatenate([[0], np.cumsum(lens)])
        ks = np.array([max(0, int(0.4 * n)) if i % 2 == 0 else n + 3 for i, n in enumerate(lens)], dtype=np.int64)  # some budgets exceed the length
        kept = np.minimum(ks, lens)
        ooffs = np.concatenate([[0], np.cumsum(kept)])[:-1]
        s = ((1.0 + 0.3 * rng.standard_normal(int(offs[-1]))).clip(0.05, None) / 1000.0).astype(np.float32)
        s[int(offs[1]):int(offs[1]) + 3] = s[int(offs[1])]      # ties at the start of the second sequence
        sd = torch.from_numpy(s).cuda()
        out = torch.full((int(kept.sum()) + 1,), -7, dtype=torch.int32, device="cuda")
        ctx.spts_select_topk_segmented(sd, torch.from_numpy(offs).cuda(), torch.from_numpy(ks).cuda(),
                                       torch.from_numpy(ooffs).cuda(), len(lens), int(lens.max()), 1, out)
        got = out.cpu().numpy()
        for b in range(len(lens)):
            seg = s[offs[b]:offs[b + 1]]
            ref = orc.topk_select(seg, int(kept[b]), 1)
            assert np.array_equal(got[ooffs[b]:ooffs[b] + kept[b]], ref), (lens, b)
        assert got[-1] == -7


# ------------------------------------------------------------------------------------------ MSDP
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_msdp_compact_bit_exact(torch, dtype):
    shape = H.small_shape(dtype=dtype, D=72)   # row bytes 144 (bf16): exercises the non-16-byte-multiple? no: 144 = 9*16
    ctx = ctx_for(shape, 4096)
    rng = np.random.default_rng(3)
    for N in (1, 7, 300, 4096):
        x = synth.storage_round(rng.standard_normal((N, shape.D)).astype(np.float32), dtype)
        pos = (np.arange(N) * 3 + 2).astype(np.int32)
        s = rng.random(N).astype(np.float32)
        s[rng.random(N) < 0.3] = 0.0
        xd = runtime.to_device(x, dtype)
        pd, sd = torch.from_numpy(pos).cuda(), torch.from_numpy(s).cuda()
        for n_next in sorted({0, 1, N // 2, int(0.7 * N), N, N + 5}):
            keep = min(N, n_next)
            xo = torch.zeros((max(keep, 1), shape.D), dtype=xd.dtype, device="cuda")
            po = torch.zeros(max(keep, 1), dtype=torch.int32, device="cuda")
            n2o = torch.zeros(max(keep, 1), dtype=torch.int32, device="cuda")
            o2n = torch.zeros(N, dtype=torch.int32, device="cuda")
            ctx.spts_msdp_compact(xd, pd, sd, N, n_next, 1, xo, po, n2o, o2n)
            rx, rp, rn2o, ro2n = orc.msdp_compact(x, pos, s, n_next, 1)
            assert np.array_equal(n2o[:keep].cpu().numpy(), rn2o)
            assert np.array_equal(o2n.cpu().numpy(), ro2n)
            assert np.array_equal(po[:keep].cpu().numpy(), rp)
            assert np.array_equal(runtime.to_host(xo[:keep]), rx.astype(np.float32))   # bitwise row copies


# ------------------------------------------------------------------------------------------ probes
def _mk(shape, N, r, seed):
    w = synth.make_layer(seed, 0, shape, r)
    x = synth.hidden_states(seed, N, shape.D, shape.dtype)
    pos = (synth.positions(N) * 2 + 1).astype(np.int32)
    return w, x, pos


PROBE_CASES = [
    ("c0", synth.TINY, 512, 32, 16),
    ("c0_ragged", synth.TINY, 333, 7, 16),
    ("c0_p1", synth.TINY, 200, 1, 16),
    # single probe row (the paper's default): the scan kernel, several 1024-key chunks, ragged tails
    ("c0_p1_chunks", synth.TINY, 2500, 1, 16),
    ("p1_n1", synth.TINY, 1, 1, 16),
    ("p1_small_bf16_d16", H.small_shape(dtype="bf16"), 1300, 1, 8),
    ("p1_bf16_d128", synth.ModelShape(D=512, H=8, Hkv=2, d=128, Dff=1024, dtype="bf16", rope_base=500000.0), 3001, 1, 64),
    ("p1_bf16_d64_grp7", synth.ModelShape(D=448, H=7, Hkv=1, d=64, Dff=1024, dtype="bf16"), 1025, 1, 64),
    ("small_bf16", H.small_shape(dtype="bf16"), 150, 5, 8),
    ("bf16_d128", synth.ModelShape(D=512, H=8, Hkv=2, d=128, Dff=1024, dtype="bf16", rope_base=500000.0), 700, 64, 64),
    ("bf16_d128_ragged", synth.ModelShape(D=512, H=8, Hkv=2, d=128, Dff=1024, dtype="bf16", rope_base=500000.0), 1111, 33, 64),
    ("bf16_all_mfma", synth.ModelShape(D=1024, H=8, Hkv=2, d=128, Dff=2048, dtype="bf16", rope_base=500000.0), 1500, 64, 256),
    ("bf16_d64_mfma", synth.ModelShape(D=512, H=8, Hkv=4, d=64, Dff=1024, dtype="bf16"), 1100, 16, 256),
    # 512 probe rows per kv head (8 wavefronts x 64 rows), d = 128 and d = 64
    ("bf16_rows512", synth.ModelShape(D=1024, H=8, Hkv=2, d=128, Dff=2048, dtype="bf16", rope_base=500000.0), 1500, 128, 256),
    ("bf16_rows512_d64", synth.ModelShape(D=512, H=8, Hkv=2, d=64, Dff=1024, dtype="bf16"), 1237, 128, 256),
]


@pytest.mark.parametrize("name,shape,N,P,r", PROBE_CASES, ids=[c[0] for c in PROBE_CASES])
def test_probe_attn_and_ffn(torch, name, shape, N, P, r):
    ctx = ctx_for(shape, 4096)
    w, x, pos = _mk(shape, N, r, seed=5)
    dw = runtime.upload_layer(w, shape, r)
    mdl = H.oracle_model(shape)
    rnd = H.rnd_for(shape.dtype)
    tol = H.TOL[shape.dtype]
    xd = runtime.to_device(x, shape.dtype)
    pd = torch.from_numpy(pos).cuda()
    kd = torch.zeros((N, shape.Hkv, shape.d), dtype=xd.dtype, device="cuda")
    sd = torch.zeros(N, dtype=torch.float32, device="cuda")
    ctx.spts_probe_attn(xd, pd, N, dw, P, kd, sd)
    K, S = orc.probe_attn(x, pos, w, mdl, P, rnd)
    assert H.row_rel_err(runtime.to_host(kd).reshape(N, -1), K.reshape(N, -1)) <= tol["hidden"]
    s_gpu = sd.cpu().numpy()
    assert H.score_rel_err(s_gpu, S) <= tol["score"]
    assert abs(float(s_gpu.astype(np.float64).sum()) - 1.0) < 1e-3
    # LTP probe on the same x, conditioned on the GPU's own S (identical inputs on both sides)
    cd = torch.zeros(N, dtype=torch.float32, device="cuda")
    fd = torch.zeros(N, dtype=torch.float32, device="cuda")
    ctx.spts_probe_ffn(xd, N, dw, sd, cd, fd)
    c_ref, sf_ref = orc.probe_ffn(x, w, mdl, s_gpu, rnd)
    assert H.score_rel_err(cd.cpu().numpy(), c_ref) <= tol["score"]
    assert H.score_rel_err(fd.cpu().numpy(), sf_ref) <= tol["score"]
    # s_mha = NULL -> s_ffn = c_ffn ; c_ffn = NULL allowed
    f2 = torch.zeros(N, dtype=torch.float32, device="cuda")
    ctx.spts_probe_ffn(xd, N, dw, None, None, f2)
    assert torch.equal(f2, cd)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_probe_ffn_output_norm_with_and_without_the_orthonormality_statement(torch, dtype):
    """C^FFN = ||z Ud^T|| as written, and as ||z|| when the caller states that Ud has orthonormal columns (SVD-built
    factors; upload_layer checks the matrix and makes the statement by default): both against the oracle, which always
    evaluates the output projection, and against each other.  Then a Ud that is NOT orthonormal (columns rescaled and
    mixed): the upload must not make the statement, and the general path must match the oracle; forcing the statement
    on it gives the scores of a different proxy (the test shows the difference is large, i.e. the check matters)."""
    shape = synth.ModelShape(D=512, H=8, Hkv=2, d=64, Dff=1024, dtype=dtype)
    N, r = 777, 64
    ctx = ctx_for(shape, 2048, max_r=r)
    w = dict(synth.make_layer(31, 0, shape, r))
    x = synth.hidden_states(31, N, shape.D, shape.dtype)
    mdl = H.oracle_model(shape)
    tol = H.TOL[dtype]["score"]
    xd = runtime.to_device(x, shape.dtype)

    def scores(dw):
        cd = torch.full((N,), -1.0, dtype=torch.float32, device="cuda")
        fd = torch.full((N,), -1.0, dtype=torch.float32, device="cuda")
        ctx.spts_probe_ffn(xd, N, dw, None, cd, fd)
        torch.cuda.synchronize()
        assert torch.equal(cd, fd)          # no S^MHA given: S^FFN = C^FFN
        return cd.cpu().numpy().astype(np.float64)

    assert runtime.ud_columns_orthonormal(w["Ud"], w["Vd"])
    auto = runtime.upload_layer(w, shape, r)
    assert auto.Ud_orthonormal == 1
    c_ref, _ = orc.probe_ffn(x, w, mdl, None, H.rnd_for(dtype))
    c_fast = scores(auto)
    c_full = scores(runtime.upload_layer(w, shape, r, ud_orthonormal=False))
    assert H.score_rel_err(c_fast, c_ref) <= tol and H.score_rel_err(c_full, c_ref) <= tol
    assert H.score_rel_err(c_fast, c_full) <= (3e-3 if dtype == "bf16" else 1e-5)
    # a proxy whose Ud is not orthonormal
    rng = np.random.default_rng(3)
    mix = np.eye(r) + 0.3 * rng.standard_normal((r, r))
    w2 = dict(w)
    w2["Ud"] = synth.storage_round((np.asarray(w["Ud"], dtype=np.float64) @ mix).astype(np.float32), dtype)
    assert not runtime.ud_columns_orthonormal(w2["Ud"], w2["Vd"])
    dw2 = runtime.upload_layer(w2, shape, r)
    assert dw2.Ud_orthonormal == 0
    c_ref2, _ = orc.probe_ffn(x, w2, mdl, None, H.rnd_for(dtype))
    assert H.score_rel_err(scores(dw2), c_ref2) <= tol
    forced = scores(runtime.upload_layer(w2, shape, r, ud_orthonormal=True))
    assert H.score_rel_err(forced, c_ref2) > 0.1


@pytest.mark.parametrize("N,dlow", [(1, 0), (31, 0), (257, 0), (1237, 0), (2048, 0), (900, 256), (1500, 512), (3000, 1024)],
                         ids=lambda v: str(v))
def test_probe_ffn_hidden_layer_kernel_shapes(torch, N, dlow):
    """LTP probe with the rank-256 proxy, whose hidden layer runs in the register-stationary kernel: row counts around its
    32-row wavefronts and 256-row workgroups, channel counts of 8 to 64 tiles (all of Dff, or Dlow < Dff channels), against
    the oracle; and against the same call with row-major factors only (no slab-major copies: the hidden layer then takes the
    dual-product GEMM), which must give the same scores to the last bit but for K-split groupings of the projection."""
    shape = synth.ModelShape(D=1024, H=8, Hkv=2, d=128, Dff=2048, dtype="bf16", rope_base=500000.0)
    ctx = ctx_for(shape, 4096)
    w = synth.make_layer(15, 0, shape, 256, dlow=dlow)
    x = synth.hidden_states(15, N, shape.D, shape.dtype)
    mdl = H.oracle_model(shape)
    tol = H.TOL["bf16"]["score"]
    s_mha = np.random.default_rng(N).random(N).astype(np.float32)
    xd = runtime.to_device(x, shape.dtype)
    sd = torch.from_numpy(s_mha).cuda()
    outs = []
    for pack in (True, False):
        dw = runtime.upload_layer(w, shape, 256, pack=pack)
        assert dw.Dlow == (dlow or shape.Dff) and bool(dw.Vg_s) == pack
        cd = torch.full((N,), -1.0, dtype=torch.float32, device="cuda")
        fd = torch.full((N,), -1.0, dtype=torch.float32, device="cuda")
        ctx.spts_probe_ffn(xd, N, dw, sd, cd, fd)
        torch.cuda.synchronize()
        outs.append((cd.cpu().numpy(), fd.cpu().numpy()))
    c_ref, f_ref = orc.probe_ffn(x, w, mdl, s_mha, orc.bf16_round)
    for c_got, f_got in outs:
        assert H.score_rel_err(c_got, c_ref) <= tol, H.score_rel_err(c_got, c_ref)
        assert H.score_rel_err(f_got, f_ref) <= tol
    assert H.score_rel_err(outs[0][0], outs[1][0]) <= 1e-2


# ------------------------------------------------------------------------------------------ layer
LAYER_CASES = [
    # name, shape, N, P, r, keep_attn, keep_ffn
    ("c0", synth.TINY, 512, 32, 16, 0.5, 0.5),
    ("c0_ragged", synth.TINY, 301, 32, 16, 0.37, 0.61),
    ("small_bf16", H.small_shape(dtype="bf16"), 130, 4, 8, 0.4, 0.4),
    ("bf16_d128", synth.ModelShape(D=512, H=8, Hkv=2, d=128, Dff=1024, dtype="bf16", rope_base=500000.0), 900, 64, 64, 0.4, 0.4),
    ("bf16_d128_ragged", synth.ModelShape(D=512, H=8, Hkv=2, d=128, Dff=1024, dtype="bf16", rope_base=500000.0), 1237, 64, 64, 0.4, 0.3),
    ("bf16_all_mfma", synth.ModelShape(D=1024, H=8, Hkv=2, d=128, Dff=2048, dtype="bf16", rope_base=500000.0), 1500, 64, 256, 0.4, 0.4),
    ("bf16_d64_mfma", synth.ModelShape(D=512, H=8, Hkv=4, d=64, Dff=1024, dtype="bf16"), 1100, 16, 256, 0.3, 0.5),
]


@pytest.mark.parametrize("name,shape,N,P,r,ka,kf", LAYER_CASES, ids=[c[0] for c in LAYER_CASES])
def test_layer_prefill_lockstep(torch, name, shape, N, P, r, ka, kf):
    ctx = ctx_for(shape, 2048)
    w, x, pos = _mk(shape, N, r, seed=0 if name.startswith("c0") else 6)
    dw = runtime.upload_layer(w, shape, r)
    mdl = H.oracle_model(shape)
    m_attn, m_ffn = int(ka * N), int(kf * N)
    if name.endswith("mfma"):
        assert ctx.uses_mfma()
    gpu = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=P, m_attn=m_attn, m_ffn=m_ffn, protect_last=1,
                            want_kv=True)
    cfg = orc.LayerCfg(1, P, m_attn, m_ffn, 1, 0)
    res = H.lockstep_layer(gpu, x, pos, w, mdl, cfg, shape.dtype)
    if shape.dtype == "f32":
        assert res["swaps_attn"] == 0 and res["swaps_ffn"] == 0
    # Level A: the GPU's TopK on the GPU's own scores is the oracle's TopK on those scores
    assert np.array_equal(gpu["idx_attn"], orc.topk_select(gpu["s_mha"], m_attn, 1))
    # rows outside both active sets are bitwise untouched (Eq. (skip))
    touched = np.zeros(N, bool); touched[gpu["idx_attn"]] = True; touched[gpu["idx_ffn"]] = True
    assert np.array_equal(gpu["x"][~touched], x[~touched].astype(np.float64))
    # KV cache holds the active pairs
    ref = res["ref"]
    assert gpu["kv_count"] == m_attn
    assert np.array_equal(gpu["pos_cache"], pos[gpu["idx_attn"]])
    tol = H.TOL[shape.dtype]["hidden"]
    assert H.row_rel_err(gpu["k_cache"].reshape(m_attn, -1), ref.k_cache.reshape(m_attn, -1)) <= tol
    assert H.row_rel_err(gpu["v_cache"].reshape(m_attn, -1), ref.v_cache.reshape(m_attn, -1)) <= tol


@pytest.mark.parametrize("name,shape,N,P,r", [
    ("d128", synth.ModelShape(D=1024, H=8, Hkv=2, d=128, Dff=2048, dtype="bf16", rope_base=500000.0), 1500, 64, 256),
    ("d64", synth.ModelShape(D=512, H=8, Hkv=4, d=64, Dff=1024, dtype="bf16"), 1100, 16, 256),
    ("generic", H.small_shape(dtype="bf16"), 130, 4, 8),
], ids=["d128", "d64", "generic"])
def test_bf16_layer_against_the_plain_fp64_algorithm(torch, name, shape, N, P, r):
    """The bf16 layer against the layer exactly as the paper defines it: the oracle in plain fp64 with NO rounding at
    any intermediate (rnd = identity); only the inputs are bf16 values.  Same bars as the bf16-faithful runs: scores
    and hidden states within 2e-2, selections up to counted near-tie swaps; skip branch and dense branch."""
    ctx = ctx_for(shape, 2048)
    w, x, pos = _mk(shape, N, r, seed=12)
    dw = runtime.upload_layer(w, shape, r)
    mdl = H.oracle_model(shape)
    ma, mf = int(0.4 * N), int(0.4 * N)
    skip = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=P, m_attn=ma, m_ffn=mf, want_kv=True)
    res = H.lockstep_layer(skip, x, pos, w, mdl, orc.LayerCfg(1, P, ma, mf, 1, 0), shape.dtype, rnd=orc.identity)
    print(f"{name} vs plain fp64: swaps attn={res['swaps_attn']} ffn={res['swaps_ffn']} score err={res['s_err']:.2e} hidden err={res['err']:.2e}")
    tol = H.TOL["bf16"]["hidden"]
    assert H.row_rel_err(skip["k_cache"].reshape(ma, -1), res["ref"].k_cache.reshape(ma, -1)) <= tol
    assert H.row_rel_err(skip["v_cache"].reshape(ma, -1), res["ref"].v_cache.reshape(ma, -1)) <= tol
    dense = runtime.run_layer(ctx, x, pos, dw, shape, skip=0, probe_len=P, m_attn=0, m_ffn=0)
    H.lockstep_layer(dense, x, pos, w, mdl, orc.LayerCfg(0, P, N, N, 1, 0), shape.dtype, rnd=orc.identity)


@pytest.mark.parametrize("name,shape,N,P,r", [
    ("d128", synth.ModelShape(D=1024, H=8, Hkv=2, d=128, Dff=2048, dtype="bf16", rope_base=500000.0), 1500, 64, 256),
    ("d64", synth.ModelShape(D=512, H=8, Hkv=4, d=64, Dff=1024, dtype="bf16"), 1100, 16, 256),
], ids=["d128", "d64"])
def test_layer_modes_on_matrix_core_kernels(torch, name, shape, N, P, r):
    """The matrix-core attention with separate query / key sets (kv_mode = 1: active queries against the keys
    and values of all candidates, visible prefix found by search), the dense branch and the literal TopK
    (protect_last = 0) at tile-sized shapes."""
    ctx = ctx_for(shape, 2048)
    assert ctx.uses_mfma()
    w, x, pos = _mk(shape, N, r, seed=8)
    dw = runtime.upload_layer(w, shape, r)
    mdl = H.oracle_model(shape)
    ma, mf = int(0.3 * N), int(0.45 * N)
    kv1 = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=P, m_attn=ma, m_ffn=mf, kv_mode=1, want_kv=True)
    H.lockstep_layer(kv1, x, pos, w, mdl, orc.LayerCfg(1, P, ma, mf, 1, 1), shape.dtype)
    assert kv1["kv_count"] == N and np.array_equal(kv1["pos_cache"], pos)
    lit = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=P, m_attn=ma, m_ffn=mf, protect_last=0)
    H.lockstep_layer(lit, x, pos, w, mdl, orc.LayerCfg(1, P, ma, mf, 0, 0), shape.dtype)
    dense = runtime.run_layer(ctx, x, pos, dw, shape, skip=0, probe_len=P, m_attn=0, m_ffn=0, want_kv=True)
    H.lockstep_layer(dense, x, pos, w, mdl, orc.LayerCfg(0, P, N, N, 1, 0), shape.dtype)
    assert dense["kv_count"] == N


@pytest.mark.parametrize("name,shape,N,P,r", [
    ("d128", synth.ModelShape(D=1024, H=8, Hkv=2, d=128, Dff=2048, dtype="bf16", rope_base=500000.0), 1500, 64, 256),
    ("d64", synth.ModelShape(D=512, H=8, Hkv=4, d=64, Dff=1024, dtype="bf16"), 1100, 16, 256),
    ("tiny_f32", synth.TINY, 301, 32, 16),
], ids=["d128", "d64", "tiny_f32"])
def test_layer_with_peaked_dominant_attention(torch, name, shape, N, P, r):
    """The same layer calls with Wk scaled by 4 and Wv by 8: the softmax concentrates on a few keys and the attention
    output dominates the residual stream, so a misplaced key, value column, mask edge or rounding point in the
    attention path moves the layer output by percents instead of averaging out over hundreds of keys (the probe scores
    sharpen in the same way).  Dense branch, skip branch, and active queries against all keys (kv_mode = 1)."""
    ctx = ctx_for(shape, 2048)
    w = dict(synth.make_layer(8, 0, shape, r))
    w["Wk"] = (4.0 * np.asarray(w["Wk"], dtype=np.float32)).astype(np.float32)
    w["Wv"] = (8.0 * np.asarray(w["Wv"], dtype=np.float32)).astype(np.float32)
    x = synth.hidden_states(8, N, shape.D, shape.dtype)
    pos = (synth.positions(N) * 2 + 1).astype(np.int32)
    dw = runtime.upload_layer(w, shape, r)
    mdl = H.oracle_model(shape)
    ma, mf = int(0.3 * N), int(0.45 * N)
    dense = runtime.run_layer(ctx, x, pos, dw, shape, skip=0, probe_len=P, m_attn=0, m_ffn=0)
    H.lockstep_layer(dense, x, pos, w, mdl, orc.LayerCfg(0, P, N, N, 1, 0), shape.dtype)
    skip = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=P, m_attn=ma, m_ffn=mf)
    H.lockstep_layer(skip, x, pos, w, mdl, orc.LayerCfg(1, P, ma, mf, 1, 0), shape.dtype)
    kv1 = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=P, m_attn=ma, m_ffn=mf, kv_mode=1)
    H.lockstep_layer(kv1, x, pos, w, mdl, orc.LayerCfg(1, P, ma, mf, 1, 1), shape.dtype)


@pytest.mark.parametrize("name,shape", [
    ("d128_g4", synth.ModelShape(D=512, H=8, Hkv=2, d=128, Dff=1024, dtype="bf16", rope_base=500000.0)),
    ("d64_g2", synth.ModelShape(D=512, H=8, Hkv=4, d=64, Dff=1024, dtype="bf16")),
    ("d128_g1", synth.ModelShape(D=512, H=4, Hkv=4, d=128, Dff=1024, dtype="bf16")),
], ids=["d128_g4", "d64_g2", "d128_g1"])
def test_matrix_core_layer_at_edge_sizes(torch, name, shape):
    """Sequence lengths and attention budgets around the matrix-core kernels' blocks: one token, one 32-key block and
    one key more, one 64-key tile and one more, the 64 / 128 / 256 queries a workgroup takes per head (4, 2 or 1 heads
    of a kv-head group share a workgroup) and one more.  Dense branch and a skip layer with a tiny and a ragged
    attention budget, each lock-step against the oracle."""
    r = 64
    ctx = ctx_for(shape, 1024, max_probe=64, max_r=r)
    assert ctx.uses_mfma()
    mdl = H.oracle_model(shape)
    w = synth.make_layer(44, 0, shape, r)
    dw = runtime.upload_layer(w, shape, r)
    for N in (1, 2, 33, 64, 65, 129, 257, 300):
        x = synth.hidden_states(44 + N, N, shape.D, shape.dtype)
        pos = (synth.positions(N) * 3 + 5).astype(np.int32)
        P = min(8, N)
        dense = runtime.run_layer(ctx, x, pos, dw, shape, skip=0, probe_len=P, m_attn=0, m_ffn=0)
        H.lockstep_layer(dense, x, pos, w, mdl, orc.LayerCfg(0, P, N, N, 1, 0), shape.dtype)
        for ma in sorted({1, min(N, 33), max(1, (2 * N) // 3)}):
            mf = max(1, N // 2)
            skip = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=P, m_attn=ma, m_ffn=mf)
            H.lockstep_layer(skip, x, pos, w, mdl, orc.LayerCfg(1, P, ma, mf, 1, 0), shape.dtype)


def test_attention_under_steep_logits(torch):
    """Wk scaled by 16 and by 160: logits spread over tens to hundreds of log2 units, so a query's reference maximum
    in the matrix-core attention moves many times along the keys (and at 160 an exponential taken against a stale
    reference overflows before the move is noticed).  A move that forgets to rescale the accumulator, the row sum or
    the next block's logits is an error of order one, or a NaN.  bf16 rounding of q and k perturbs a logit in
    proportion to its size, so the bar is wider than the usual 2e-2: 8e-2 at 16 (measured 3.5e-2), and at 160, where
    the softmax is one-hot on keys that bf16 can no longer rank, only finiteness and a bounded output."""
    shape = synth.ModelShape(D=1024, H=8, Hkv=2, d=128, Dff=2048, dtype="bf16", rope_base=500000.0)
    N, P, r = 1500, 64, 256
    ctx = ctx_for(shape, 2048)
    x = synth.hidden_states(8, N, shape.D, shape.dtype)
    pos = (synth.positions(N) * 2 + 1).astype(np.int32)
    mdl = H.oracle_model(shape)
    for f in (16.0, 160.0):
        w = dict(synth.make_layer(8, 0, shape, r))
        w["Wk"] = (f * np.asarray(w["Wk"], dtype=np.float32)).astype(np.float32)
        w["Wv"] = (8.0 * np.asarray(w["Wv"], dtype=np.float32)).astype(np.float32)
        dw = runtime.upload_layer(w, shape, r)
        dense = runtime.run_layer(ctx, x, pos, dw, shape, skip=0, probe_len=P, m_attn=0, m_ffn=0)
        got = np.asarray(dense["x"], dtype=np.float64)
        assert np.isfinite(got).all()
        if f == 16.0:
            H.lockstep_layer(dense, x, pos, w, mdl, orc.LayerCfg(0, P, N, N, 1, 0), shape.dtype, hidden_tol=8e-2)
        else:
            ref = orc.layer_prefill(x, pos, w, mdl, orc.LayerCfg(0, P, N, N, 1, 0), rnd=H.rnd_for(shape.dtype)).x
            assert H.row_rel_err(got, ref) <= 0.5


def test_pack_slab32_matches_the_host_layout(torch):
    """spts_pack_slab32 on the device against the same permutation written with numpy (bit-exact), and its error codes."""
    ctx = ctx_for(synth.ModelShape(D=512, H=8, Hkv=2, d=128, Dff=1024, dtype="bf16", rope_base=500000.0), 2048)
    rng = np.random.default_rng(3)
    for rows, K in ((48, 96), (1, 32), (333, 4096), (1024, 512)):
        a = rng.standard_normal((rows, K)).astype(np.float32)
        ad = runtime.to_device(a, "bf16")
        out = torch.zeros_like(ad)
        ctx.spts_pack_slab32(ad, rows, K, out)
        torch.cuda.synchronize()
        want = runtime.pack_slab32(runtime.to_host(ad))
        assert np.array_equal(runtime.to_host(out), want), (rows, K)
        # the layout itself, element by element on a sample
        flat = runtime.to_host(out).reshape(-1)
        src = runtime.to_host(ad)
        for r_, k_ in ((0, 0), (rows - 1, K - 1), (rows // 2, 33 % K), (rows - 1, 31)):
            assert flat[((k_ // 32) * rows + r_) * 32 + k_ % 32] == src[r_, k_]
    ad = runtime.to_device(rng.standard_normal((8, 48)).astype(np.float32), "bf16")
    with pytest.raises(binding.SptsError):
        ctx.spts_pack_slab32(ad, 8, 48, torch.zeros_like(ad))          # K % 32 != 0
    with pytest.raises(binding.SptsError):
        ctx.spts_pack_slab32(ad, 0, 32, torch.zeros_like(ad))


@pytest.mark.parametrize("name,shape,N,P,r", [
    ("d128", synth.ModelShape(D=1024, H=8, Hkv=2, d=128, Dff=2048, dtype="bf16", rope_base=500000.0), 1500, 64, 256),
    ("d64", synth.ModelShape(D=512, H=8, Hkv=4, d=64, Dff=1024, dtype="bf16"), 1100, 16, 256),
], ids=["d128", "d64"])
def test_layer_with_row_major_weights_only(torch, name, shape, N, P, r):
    """The other tests upload the slab-major weight copies as well (runtime.upload_layer packs by default), so the
    prefill GEMMs read the weights through them; here the struct carries the row-major matrices alone.  Both paths
    against the oracle, skip and dense, and against each other (same products in the same k order; only the K shares
    of split tiles may group differently)."""
    ctx = ctx_for(shape, 2048)
    w, x, pos = _mk(shape, N, r, seed=9)
    mdl = H.oracle_model(shape)
    ma, mf = int(0.35 * N), int(0.4 * N)
    outs = {}
    for pack in (False, True):
        dw = runtime.upload_layer(w, shape, r, pack=pack)
        assert bool(dw.Wgate_s) == pack and bool(dw.Wq_s) == pack
        skip = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=P, m_attn=ma, m_ffn=mf, want_kv=True)
        H.lockstep_layer(skip, x, pos, w, mdl, orc.LayerCfg(1, P, ma, mf, 1, 0), shape.dtype)
        dense = runtime.run_layer(ctx, x, pos, dw, shape, skip=0, probe_len=P, m_attn=0, m_ffn=0)
        H.lockstep_layer(dense, x, pos, w, mdl, orc.LayerCfg(0, P, N, N, 1, 0), shape.dtype)
        outs[pack] = (skip, dense)
    for a, b in zip(outs[False], outs[True]):
        assert H.row_rel_err(a["x"], b["x"]) <= H.TOL["bf16"]["hidden"]
    assert np.array_equal(outs[False][0]["idx_attn"], outs[True][0]["idx_attn"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_layer_dense_keepall_keepzero_and_modes(torch, dtype):
    shape = synth.TINY if dtype == "f32" else synth.ModelShape(D=256, H=4, Hkv=2, d=64, Dff=688, dtype="bf16")
    N, P, r = 200, 8, 16
    ctx = ctx_for(shape, 2048)
    w, x, pos = _mk(shape, N, r, seed=9)
    dw = runtime.upload_layer(w, shape, r)
    mdl = H.oracle_model(shape)
    # dense branch of Alg. 1
    dense = runtime.run_layer(ctx, x, pos, dw, shape, skip=0, probe_len=P, m_attn=0, m_ffn=0, want_kv=True)
    H.lockstep_layer(dense, x, pos, w, mdl, orc.LayerCfg(skip=0), dtype)
    assert dense["kv_count"] == N
    # keep everything == dense (same kernels, same rows: bitwise)
    full = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=P, m_attn=N, m_ffn=10 * N)
    assert np.array_equal(full["idx_attn"], np.arange(N)) and np.array_equal(full["idx_ffn"], np.arange(N))
    assert np.array_equal(full["x"], dense["x"])
    # keep nothing == identity, bitwise
    none = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=P, m_attn=0, m_ffn=0)
    assert np.array_equal(none["x"], x.astype(np.float64))
    # literal mode (protect_last = 0) and kv_mode = 1
    lit = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=P, m_attn=60, m_ffn=70, protect_last=0)
    H.lockstep_layer(lit, x, pos, w, mdl, orc.LayerCfg(1, P, 60, 70, 0, 0), dtype)
    kv1 = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=P, m_attn=60, m_ffn=70, kv_mode=1, want_kv=True)
    H.lockstep_layer(kv1, x, pos, w, mdl, orc.LayerCfg(1, P, 60, 70, 1, 1), dtype)
    assert kv1["kv_count"] == N
    # tiny inputs: N = 1 and N = P
    for n_small in (1, P):
        ws, xs, ps = w, x[:n_small], pos[:n_small]
        g = runtime.run_layer(ctx, xs, ps, dw, shape, skip=1, probe_len=min(P, n_small), m_attn=max(n_small // 2, 1),
                              m_ffn=max(n_small // 2, 1))
        H.lockstep_layer(g, xs, ps, ws, mdl, orc.LayerCfg(1, min(P, n_small), max(n_small // 2, 1), max(n_small // 2, 1), 1, 0), dtype)


def test_layer_prefill_is_deterministic(torch):
    shape = synth.ModelShape(D=512, H=8, Hkv=2, d=128, Dff=1024, dtype="bf16")
    ctx = ctx_for(shape, 2048)
    w, x, pos = _mk(shape, 777, 64, seed=2)
    dw = runtime.upload_layer(w, shape, 64)
    a = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=64, m_attn=300, m_ffn=300)
    b = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=64, m_attn=300, m_ffn=300)
    for k in ("x", "s_mha", "idx_attn", "idx_ffn"):
        assert np.array_equal(a[k], b[k]), k


# ------------------------------------------------------------------------------------------ stack
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_stack_with_msdp_lockstep(torch, dtype):
    """Alg. 1 outer loop with stage-end pruning: every layer is re-computed by the oracle from the
    GPU's own layer input (lock-step), every compaction map is compared bit-exactly."""
    shape = synth.TINY if dtype == "f32" else synth.ModelShape(D=256, H=4, Hkv=2, d=64, Dff=688, dtype="bf16")
    wl = synth.scaled(synth.WORKLOADS["c2"], shape=shape, N=400, layers=4, stage_end_layers=(1, 2, 3), probe_len=16, r=16)
    plan = wl.layer_plan()
    ws = [synth.make_layer(wl.seed, l, shape, wl.r) for l in range(wl.layers)]
    dws = [runtime.upload_layer(w, shape, wl.r) for w in ws]
    ctx = ctx_for(shape, 2048)
    runner = runtime.StackRunner(ctx, shape, dws, plan, wl.probe_len, keep_trace=True)
    x0 = synth.hidden_states(wl.seed, wl.N, shape.D, dtype)
    pos0 = synth.positions(wl.N)
    xo, po, n_final = runner.run(runtime.to_device(x0, dtype), torch.from_numpy(pos0).cuda())
    torch.cuda.synchronize()
    assert n_final == plan[-1]["N"] == 140
    mdl = H.oracle_model(shape)
    for tr, item, w in zip(runner.trace, plan, ws):
        N = tr["N"]
        x_in = runtime.to_host(tr["x_in"]); pos_in = tr["pos_in"].cpu().numpy()
        gpu = dict(x=runtime.to_host(tr["x_out"]).astype(np.float64), s_mha=tr["s_mha"].cpu().numpy(),
                   idx_attn=tr["idx_attn"][:min(N, item["m_attn"])].cpu().numpy(),
                   idx_ffn=tr["idx_ffn"][:min(N, item["m_ffn"])].cpu().numpy())
        H.lockstep_layer(gpu, x_in, pos_in, w, mdl, orc.LayerCfg(1, wl.probe_len, item["m_attn"], item["m_ffn"], 1, 0), dtype)
        if item["N_next"] is not None:
            _, rp, rn2o, _ = orc.msdp_compact(gpu["x"], pos_in, gpu["s_mha"], item["N_next"], 1)
            assert np.array_equal(tr["map_new2old"].cpu().numpy(), rn2o)
    assert po[-1].item() == wl.N - 1


@pytest.mark.parametrize("components", ["full", "pap+ltp", "pap"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_stack_paper_schedule_lockstep(torch, dtype, components):
    """The paper's own schedule in miniature (Sec. 4.1): dense first layers, absolute budgets per stage,
    a fixed number of candidates pruned at every stage end, single-row probe, proxy on a channel subset
    (Dlow < Dff) with a zero-padded rank; and the two reduced variants of Table ablation_main_speed (no
    stage pruning; attention skipping only, where the FFN budget covers every candidate)."""
    shape = synth.TINY if dtype == "f32" else synth.ModelShape(D=256, H=4, Hkv=2, d=64, Dff=688, dtype="bf16")
    wl = synth.scaled(synth.WORKLOADS["p32"], shape=shape, N=500, layers=6, dense_layers=2, stage_end_layers=(3, 4, 5),
                      stage_budgets=(200, 150, 100, 50), stage_prune=30, r=12, r_pad=16, dlow=256, components=components)
    plan = wl.layer_plan()
    n_expect = [500, 500, 500, 470, 440, 410] if components == "full" else [500] * 6
    assert [it["skip"] for it in plan] == [0, 0, 1, 1, 1, 1] and [it["N"] for it in plan] == n_expect
    assert [it["m_ffn"] for it in plan][2:] == ([500] * 4 if components == "pap" else [200, 150, 100, 50])
    ws = [synth.make_layer(wl.seed, l, shape, wl.r, wl.dlow, wl.r_pad) for l in range(wl.layers)]
    assert ws[0]["Vg"].shape == (16, 256) and not ws[0]["Ug"][:, 12:].any()
    dws = [runtime.upload_layer(w, shape, wl.proxy_r) for w in ws]
    ctx = ctx_for(shape, 2048)
    runner = runtime.StackRunner(ctx, shape, dws, plan, wl.probe_len, keep_trace=True)
    x0 = synth.hidden_states(wl.seed, wl.N, shape.D, dtype)
    pos0 = synth.positions(wl.N)
    xo, po, n_final = runner.run(runtime.to_device(x0, dtype), torch.from_numpy(pos0).cuda())
    torch.cuda.synchronize()
    assert n_final == n_expect[-1]
    mdl = H.oracle_model(shape)
    for tr, item, w in zip(runner.trace, plan, ws):
        N = tr["N"]
        x_in = runtime.to_host(tr["x_in"]); pos_in = tr["pos_in"].cpu().numpy()
        gpu = dict(x=runtime.to_host(tr["x_out"]).astype(np.float64), s_mha=tr["s_mha"].cpu().numpy(),
                   idx_attn=tr["idx_attn"][:min(N, item["m_attn"])].cpu().numpy(),
                   idx_ffn=tr["idx_ffn"][:min(N, item["m_ffn"])].cpu().numpy())
        cfg = orc.LayerCfg(item["skip"], wl.probe_len, item["m_attn"], item["m_ffn"], 1, 0)
        H.lockstep_layer(gpu, x_in, pos_in, w, mdl, cfg, dtype)
        if item["N_next"] is not None:
            _, rp, rn2o, _ = orc.msdp_compact(gpu["x"], pos_in, gpu["s_mha"], item["N_next"], 1)
            assert np.array_equal(tr["map_new2old"].cpu().numpy(), rn2o)
    assert po[-1].item() == wl.N - 1


# ------------------------------------------------------------------------------------------ batch of sequences
@pytest.mark.parametrize("name,shape,lens,P,r", [
    ("f32", synth.TINY, (301, 37, 512), 4, 16),
    ("bf16_mfma", synth.ModelShape(D=1024, H=8, Hkv=2, d=128, Dff=2048, dtype="bf16", rope_base=500000.0), (700, 260, 1333), 64, 256),
    ("bf16_p1", synth.ModelShape(D=512, H=8, Hkv=4, d=64, Dff=1024, dtype="bf16"), (64, 1, 900, 129), 1, 64),
], ids=lambda v: v if isinstance(v, str) else None)
def test_layer_prefill_batched_lockstep_per_sequence(torch, name, shape, lens, P, r):
    """spts_layer_prefill_batched on sequences of different lengths laid back to back: every sequence must come
    out as the oracle's single-sequence layer gives it (probe, selections and attention stay inside the sequence),
    lock-step as for the single-sequence call; the per-sequence caches hold each sequence's active pairs."""
    dtype = shape.dtype
    w = synth.make_layer(41, 0, shape, r)
    dw = runtime.upload_layer(w, shape, r)
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    Ntot = int(offs[-1])
    ctx = ctx_for(shape, 4096)
    xs = [synth.hidden_states(100 + b, n, shape.D, dtype) for b, n in enumerate(lens)]
    # positions with gaps, restarting in every sequence
    rng = np.random.default_rng(7)
    ps = [np.sort(rng.choice(3 * n + 5, size=n, replace=False)).astype(np.int32) for n in lens]
    ma = [int(0.4 * n) for n in lens]
    mf = [max(1, int(0.55 * n)) for n in lens]
    ma[1] = lens[1] + 10                      # budget above the length: the whole sequence is active
    xd = runtime.to_device(np.concatenate(xs), dtype)
    posd = torch.from_numpy(np.concatenate(ps)).cuda()
    MaT = sum(min(n, m) for n, m in zip(lens, ma)); MfT = sum(min(n, m) for n, m in zip(lens, mf))
    s = torch.zeros(Ntot, dtype=torch.float32, device="cuda")
    ia = torch.full((max(MaT, 1),), -1, dtype=torch.int32, device="cuda")
    iff = torch.full((max(MfT, 1),), -1, dtype=torch.int32, device="cuda")
    caches = [runtime.KVCache(shape, min(n, m)) for n, m in zip(lens, ma)]
    kvs = [c.struct for c in caches]
    ctx.spts_layer_prefill_batched(xd, posd, offs, dw, P, ma, mf, 1, kvs, s, ia, iff)
    torch.cuda.synchronize()
    x_out = runtime.to_host(xd).astype(np.float64)
    s_out, ia, iff = s.cpu().numpy(), ia.cpu().numpy(), iff.cpu().numpy()
    mdl = H.oracle_model(shape)
    oa = of = 0
    for b, n in enumerate(lens):
        r0 = int(offs[b]); a_b, f_b = min(n, ma[b]), min(n, mf[b])
        gpu = dict(x=x_out[r0:r0 + n], s_mha=s_out[r0:r0 + n], idx_attn=ia[oa:oa + a_b] - r0, idx_ffn=iff[of:of + f_b] - r0)
        assert gpu["idx_attn"].min(initial=0) >= 0 and gpu["idx_attn"].max(initial=0) < n
        res = H.lockstep_layer(gpu, xs[b], ps[b], w, mdl, orc.LayerCfg(1, P, ma[b], mf[b], 1, 0), dtype)
        assert res["swaps_attn"] <= max(1, a_b // 50) and res["swaps_ffn"] <= max(1, f_b // 50), (b, res["swaps_attn"], res["swaps_ffn"])
        assert kvs[b].count == a_b
        kh, vh, ph = caches[b].k[:a_b], caches[b].v[:a_b], caches[b].pos[:a_b].cpu().numpy()
        assert np.array_equal(ph, ps[b][gpu["idx_attn"]])
        ref = res["ref"]
        tol = H.TOL[dtype]["hidden"]
        assert H.row_rel_err(runtime.to_host(kh).reshape(a_b, -1).astype(np.float64), ref.k_cache.reshape(a_b, -1)) <= tol
        assert H.row_rel_err(runtime.to_host(vh).reshape(a_b, -1).astype(np.float64), ref.v_cache.reshape(a_b, -1)) <= tol
        oa += a_b; of += f_b


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_layer_prefill_batched_dense_branch(torch, dtype):
    """skip = 0 on a batch: every sequence goes through the dense branches of Alg. 1 on its own (attention inside
    the sequence, all rows in the FFN), and its cache receives all of its pairs."""
    shape = synth.TINY if dtype == "f32" else synth.ModelShape(D=512, H=8, Hkv=2, d=128, Dff=1024, dtype="bf16", rope_base=500000.0)
    lens = (130, 1, 517)
    w = synth.make_layer(43, 0, shape, 16)
    dw = runtime.upload_layer(w, shape, 16)
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    ctx = ctx_for(shape, 4096)
    xs = [synth.hidden_states(200 + b, n, shape.D, dtype) for b, n in enumerate(lens)]
    ps = [synth.positions(n) for n in lens]
    xd = runtime.to_device(np.concatenate(xs), dtype)
    posd = torch.from_numpy(np.concatenate(ps)).cuda()
    caches = [runtime.KVCache(shape, n) for n in lens]
    kvs = [c.struct for c in caches]
    ctx.spts_layer_prefill_batched(xd, posd, offs, dw, 0, [0] * 3, [0] * 3, 1, kvs, None, None, None, skip=0)
    torch.cuda.synchronize()
    x_out = runtime.to_host(xd).astype(np.float64)
    mdl = H.oracle_model(shape)
    tol = H.TOL[dtype]["hidden"]
    for b, n in enumerate(lens):
        r0 = int(offs[b])
        ref = orc.layer_prefill(xs[b], ps[b], w, mdl, orc.LayerCfg(0, 1, n, n, 1, 0), rnd=H.rnd_for(dtype))
        assert H.row_rel_err(x_out[r0:r0 + n], ref.x) <= tol, b
        assert kvs[b].count == n
        assert np.array_equal(caches[b].pos[:n].cpu().numpy(), ps[b])
        assert H.row_rel_err(runtime.to_host(caches[b].k[:n]).reshape(n, -1).astype(np.float64), ref.k_cache.reshape(n, -1)) <= tol
        assert H.row_rel_err(runtime.to_host(caches[b].v[:n]).reshape(n, -1).astype(np.float64), ref.v_cache.reshape(n, -1)) <= tol


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_msdp_compact_batched_bit_exact(torch, dtype):
    """Stage-end pruning of a batch: per sequence the maps the oracle's compaction gives on the same fp32 scores
    (as rows of the batch), rows and positions copied bit for bit; ties inside a sequence, an empty target and a
    target above the length included."""
    shape = H.small_shape(dtype=dtype)
    lens = (257, 3, 1000, 64, 1)
    nnext = (100, 5, 999, 0, 1)
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    Ntot = int(offs[-1])
    rng = np.random.default_rng(11)
    sc = rng.random(Ntot).astype(np.float32)
    sc[300:700] = np.float32(0.25)                       # a run of ties inside the third sequence
    x = synth.hidden_states(5, Ntot, shape.D, dtype)
    pos = np.concatenate([np.sort(rng.choice(4 * n + 3, size=n, replace=False)) for n in lens]).astype(np.int32)
    ctx = ctx_for(shape, 2048)
    xd = runtime.to_device(x, dtype); pd = torch.from_numpy(pos).cuda(); sd = torch.from_numpy(sc).cuda()
    keep = [min(n, k) for n, k in zip(lens, nnext)]
    KT = sum(keep)
    xo = torch.zeros((KT, shape.D), dtype=xd.dtype, device="cuda")
    po = torch.zeros(KT, dtype=torch.int32, device="cuda")
    n2o = torch.zeros(KT, dtype=torch.int32, device="cuda")
    o2n = torch.zeros(Ntot, dtype=torch.int32, device="cuda")
    new_offs = ctx.spts_msdp_compact_batched(xd, pd, sd, offs, nnext, 1, xo, po, n2o, o2n)
    torch.cuda.synchronize()
    assert new_offs == list(np.concatenate([[0], np.cumsum(keep)]))
    n2o_h, o2n_h = n2o.cpu().numpy(), o2n.cpu().numpy()
    ref_o2n = np.full(Ntot, -1, dtype=np.int32)
    for b, n in enumerate(lens):
        r0, o0 = int(offs[b]), new_offs[b]
        _, rp, rn2o, _ = orc.msdp_compact(x[r0:r0 + n], pos[r0:r0 + n], sc[r0:r0 + n], nnext[b], 1)
        assert np.array_equal(n2o_h[o0:o0 + keep[b]], rn2o + r0), b
        assert np.array_equal(po[o0:o0 + keep[b]].cpu().numpy(), rp)
        ref_o2n[rn2o + r0] = np.arange(o0, o0 + keep[b])
    assert np.array_equal(o2n_h, ref_o2n)
    assert torch.equal(xo, xd[n2o.long()])


def test_batched_stack_equals_the_sequences_run_alone(torch):
    """A three-layer stack (one dense layer, two skip layers, a stage end) over a batch of three sequences (bf16, matrix-core shape) gives every
    sequence the candidates, positions and hidden states that the single-sequence stack gives it.  (Each step of the
    single-sequence stack is checked against the oracle elsewhere; this checks the batch plumbing end to end.)"""
    shape = synth.ModelShape(D=512, H=8, Hkv=2, d=128, Dff=1024, dtype="bf16", rope_base=500000.0)
    lens = (900, 300, 1500)
    wls = [synth.Workload("b", shape, N=n, layers=3, probe_len=16, attn_keep=0.4, ffn_keep=0.5, r=64, seed=9,
                          stage_end_layers=(2,), stage_cum_keep=(1.0, 0.6), dense_layers=1) for n in lens]
    plans = [wl.layer_plan() for wl in wls]
    ws = [synth.make_layer(9, l, shape, 64) for l in range(3)]
    dws = [runtime.upload_layer(w, shape, 64) for w in ws]
    ctx = ctx_for(shape, 4096)
    xs = [runtime.to_device(synth.hidden_states(50 + b, n, shape.D, "bf16"), "bf16") for b, n in enumerate(lens)]
    ps = [torch.from_numpy(synth.positions(n)).cuda() for n in lens]
    bx, bp, boffs = runtime.BatchedStackRunner(ctx, shape, dws, plans, 16).run(torch.cat(xs), torch.cat(ps))
    bx, bp = bx.float().cpu().numpy(), bp.cpu().numpy()
    for b, n in enumerate(lens):
        sx, sp, sn = runtime.StackRunner(ctx, shape, dws, plans[b], 16).run(xs[b], ps[b])
        torch.cuda.synchronize()
        assert boffs[b + 1] - boffs[b] == sn == plans[b][-1]["N"]
        got_p, got_x = bp[boffs[b]:boffs[b + 1]], bx[boffs[b]:boffs[b + 1]]
        ref_p, ref_x = sp.cpu().numpy(), sx.float().cpu().numpy()
        # a near-tie at a stage end may keep a different candidate in the two runs (the GEMMs split K differently for
        # different row counts): compare the candidates both kept, and require almost all to be common
        common, ig, ir = np.intersect1d(got_p, ref_p, return_indices=True)
        assert len(common) >= sn - max(2, sn // 100), (b, len(common), sn)
        assert H.row_rel_err(got_x[ig], ref_x[ir]) <= H.TOL["bf16"]["hidden"]


# ------------------------------------------------------------------------------------------ proxy builder
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_channel_importance_and_selection(torch, dtype):
    """Eq. (channel_importance) on a synthetic calibration set; the channel choice is the library's TopK
    of the scores (bit-exact against the oracle's TopK of the same scores, swap-counted against the
    oracle's own scores)."""
    shape = synth.TINY if dtype == "f32" else synth.ModelShape(D=256, H=4, Hkv=2, d=64, Dff=688, dtype="bf16")
    w = synth.make_layer(31, 0, shape, 16)
    dw = runtime.upload_layer(w, shape, 16)
    ctx = ctx_for(shape, 2048)
    tol = H.TOL[dtype]["score"]
    for T, k in ((300, 60), (1, 1), (257, 257), (1024, 5)):
        xc = synth.calibration_states(31, T, shape.D, dtype)
        imp = torch.full((shape.Dff,), -1.0, dtype=torch.float32, device="cuda")
        ctx.spts_channel_importance(runtime.to_device(xc, dtype), T, dw, k, imp)
        got = imp.cpu().numpy()
        ref = orc.channel_importance(xc, w["Wgate"], w["Wup"], k, H.rnd_for(dtype))
        assert np.max(np.abs(got - ref)) <= tol * np.max(np.abs(ref)), (T, k, np.max(np.abs(got - ref)) / np.max(np.abs(ref)))
        dlow = 256
        sel = torch.empty(dlow, dtype=torch.int32, device="cuda")
        ctx.spts_select_topk(imp, shape.Dff, dlow, 0, sel)
        sel = sel.cpu().numpy()
        assert np.array_equal(sel, orc.select_channels(got, dlow))
        H.count_swaps(sel, orc.select_channels(ref, dlow), ref, tol, 0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_proxy_built_from_selected_channels_runs_the_layer(torch, dtype):
    """The offline construction of Sec. 3.3 end to end: channel scores on a calibration set and C = TopK(I, Dlow) on
    the GPU (spts_channel_importance, spts_select_topk), the rank-r SVD of W[:, C] in the harness, then a token-skipped
    layer with that Dlow < Dff proxy.  The oracle does the same through select_channels: the channel sets must agree
    up to counted near ties, the oracle then builds its factors from the GPU's set and the layer runs lock-step."""
    if dtype == "f32":
        shape, N, P, r, dlow, T = synth.TINY, 301, 8, 16, 128, 200
    else:
        shape, N, P, r, dlow, T = synth.ModelShape(D=1024, H=8, Hkv=2, d=128, Dff=2048, dtype="bf16", rope_base=500000.0), 1500, 1, 64, 512, 700
    base = synth.layer_weights(41, 0, shape)
    ctx = ctx_for(shape, 2048)
    dw0 = runtime.upload_layer(base, shape, 0)                      # FFN matrices only: the scores need no proxy
    xc = synth.calibration_states(41, T, shape.D, dtype)
    k = max(1, int(0.2 * T))                                        # rho = 0.2
    sel, imp = runtime.select_proxy_channels(ctx, dw0, shape, xc, k, dlow)
    ref_imp = orc.channel_importance(xc, base["Wgate"], base["Wup"], k, H.rnd_for(dtype))
    tol = H.TOL[dtype]["score"]
    assert np.max(np.abs(imp - ref_imp)) <= tol * np.max(np.abs(ref_imp))
    assert np.array_equal(sel, orc.select_channels(imp, dlow))
    swaps = H.count_swaps(sel, orc.select_channels(ref_imp, dlow), ref_imp, tol, 0)
    assert swaps <= H.swap_bound(dlow, dtype)
    w = synth.make_layer(41, 0, shape, r, channels=sel)
    assert w["Vg"].shape == (r, dlow) and w["Vd"].shape == (r, dlow)
    dw = runtime.upload_layer(w, shape, r)
    assert dw.Dlow == dlow
    x = synth.hidden_states(41, N, shape.D, dtype)
    pos = synth.positions(N)
    ma, mf = int(0.4 * N), int(0.3 * N)
    gpu = runtime.run_layer(ctx, x, pos, dw, shape, skip=1, probe_len=P, m_attn=ma, m_ffn=mf)
    res = H.lockstep_layer(gpu, x, pos, w, H.oracle_model(shape), orc.LayerCfg(1, P, ma, mf, 1, 0), dtype)
    print(f"{dtype}: channel swaps {swaps}/{dlow}, layer swaps attn={res['swaps_attn']} ffn={res['swaps_ffn']} err={res['err']:.2e}")

