"""CPU oracle for the SPTS token-skipped decoder-layer prefill (TEST INFRASTRUCTURE).

A plain, slow numpy/fp64 statement of what the path computes, written from the
paper (Sec. 3.1-3.4, Eq. (skip), (mha_importance), (ffn_function), (proxy_ffn),
(ffn_transformation), (ffn_importance), (ffn_selection), (stage_prune) and
Alg. 1).  SPTS is a heuristic (the exact selection problem of Sec. 3.2 is
NP-hard), so the oracle is the algorithm's steps in the paper's order, not a
closed form.  Library primitives used as steps: matmul, exp, sort.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this file.  It shares no code with the HIP path and
imports nothing from the product package.

All matrices are in the paper's orientation: ``K = X W_K``; ``W_gate``,
``W_up``, ``W_down`` are ``D x Dff`` and the FFN is
``(silu(X W_gate) * (X W_up)) W_down^T``; proxy factors ``U in R^{D x r}``,
``V in R^{r x Dlow}``.

Readings taken where the paper is silent (each shared with the HIP path):

 R1  Pre-norm block: RMSNorm before MHA and before FFN; rotary embedding with
     rotate-half pairing (j, j + d/2) and theta_j = base^(-2j/d) on q and k;
     cached keys are post-rotary.  (Alg. 1 omits norm and positions.)
 R2  Probe window P > 1 (Appendix C, "query length"): the last P candidates,
     causal inside the window, each row a full softmax, plain mean over the
     P*H rows.  P = 1 is Eq. (mha_importance) as printed.
 R3  Grouped-query attention: the mean runs over the H query heads; query head
     h reads KV head h // (H / Hkv).
 R4  Every candidate keeps its original absolute position through selection
     and pruning; rotary angles and the causal mask use those positions.
 R5  Reduced attention is over the active set only (K-hat, V-hat of Alg. 1);
     ``kv_mode = 1`` (keys/values of all candidates) is an extra.
 R6  TopK is the k largest under (score descending, index ascending), returned
     in ascending index order; -0.0 == +0.0.
 R7  ``protect_last``: when set and k >= 1 the last candidate always belongs
     to the selected set (its score is treated as +inf).
 R10 LTP and MSDP use the probe score of the same layer, computed before the
     attention update (Alg. 1 reuses S^MHA).
 R13 Sigma of the SVD goes into V.

``rnd`` hooks: ``identity`` gives the plain fp64 algorithm; ``bf16_round``
rounds at the points where a bf16 implementation stores a tensor (the
"bf16-faithful" mode used to tighten parity bands); ``bf16_prefill`` is the same
for a prefill that stores its queries with the softmax factor folded in.
Accumulation is fp64 in all modes.

Pins (tests/test_oracle_pins.py): dense block against an independent
composition of torch CPU fp64 routines; keep=1 == dense; keep=0 == identity;
sum(S) == 1 and the P=1 score against the last row of a brute-force attention
matrix; full-rank proxy == exact FFN norm; TopK against a stable sort;
permutation invariance with positions attached; FFN token independence.
Pins (tests/test_oracle_ltp_pins.py): the layer's LTP decision, TopK of C^FFN * S^MHA with the
pre-attention score and the post-attention proxy norm, against a torch composition of the attention
half, a scalar-loop proxy and a Python sort; a constant-C layer (set = TopK of S^MHA) and a flat-S
layer (set = TopK of C^FFN).
Numerical values of scores/selected sets on real text are not printed anywhere
in the paper: parity unpinned for those (only the properties above pin them).

Decode phase (Alg. 1 with ``skip`` false because ``Is_prefill_phase`` is false;
Sec. 3.2 last paragraph and Appendix "KV Cache flexibility" for what the cache
holds): ``decode_layer`` / ``decode_step`` run one new token through the dense
branches over each layer's cache of active key/value pairs and append the
token's own pair; ``greedy_token`` is a final norm, a vocabulary projection and
an argmax (a synthetic head: the vocabulary table is not part of the method).
Offline proxy construction (Sec. 3.3, activation saliency and Eq. (channel_importance)):
``channel_saliency`` / ``channel_importance`` / ``select_channels`` give the per-channel score
(mean of the top-rho fraction of saliencies over a calibration token set) and the Dlow channels
the proxy keeps.  Reading R20: the calibration set holds the FFN's inputs, i.e. the states after
the pre-FFN RMSNorm.  Pins (tests/test_oracle_builder_pins.py): loops on tiny inputs, rho = 1
(plain column mean), k = 1 (column maximum), invariance under a permutation of the tokens,
a planted dominant channel.

Pins (tests/test_oracle_decode_pins.py): dense prefill of N+1 tokens == dense
prefill of N tokens + one decode step (last row and caches); attention over the
cache against a loop-by-loop softmax; invariance under a permutation of the
cache rows; argmax tie rule.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Callable, Dict, Optional, Tuple

import numpy as np

Array = np.ndarray


def identity(a: Array) -> Array:
    return a


def bf16_round(a: Array) -> Array:
    """Round fp64/fp32 values to the nearest-even bfloat16 value (returned as fp64)."""
    f = np.asarray(a, dtype=np.float64).astype(np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).astype(np.float64).reshape(f.shape)


def f32_round(a: Array) -> Array:
    return np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)


def bf16_prefill(a: Array) -> Array:
    """``bf16_round`` for a bf16 prefill that stores its queries (probe window and active rows) already multiplied
    by the softmax factor log2(e)/sqrt(d): the mark below makes ``project_queries`` round q * factor instead of q for
    the prefill calls, which moves a bf16 rounding point and nothing else (with ``identity`` nothing changes)."""
    return bf16_round(a)


bf16_prefill.prefill_queries_scaled = True


@dataclass
class Model:
    D: int
    H: int
    Hkv: int
    d: int
    Dff: int
    rms_eps: float
    rope_base: float


# --------------------------------------------------------------------------
# building blocks
# --------------------------------------------------------------------------
def rmsnorm(x: Array, gamma: Array, eps: float) -> Array:
    """x / sqrt(mean_j x_j^2 + eps) * gamma, row-wise (R1)."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gamma, dtype=np.float64)


def rope(t: Array, pos: Array, base: float) -> Array:
    """Rotary embedding on t [n, heads, d] at absolute positions pos [n] (R1, R4).

    Pair (j, j + d/2) is rotated by the angle pos * base^(-2j/d).
    """
    t = np.asarray(t, dtype=np.float64)
    n, _, d = t.shape
    half = d // 2
    j = np.arange(half, dtype=np.float64)
    theta = base ** (-2.0 * j / d)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * theta[None, :]  # [n, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    a = t[..., :half]
    b = t[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(z: Array) -> Array:
    return z / (1.0 + np.exp(-z))


def softmax_rows(logits: Array) -> Array:
    """Row softmax with max subtraction; -inf entries get probability 0."""
    m = np.max(logits, axis=-1, keepdims=True)
    e = np.exp(logits - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def project_keys(xn: Array, pos: Array, Wk: Array, mdl: Model, rnd=identity) -> Array:
    """K = rope(Xn W_K) for all candidates -> [N, Hkv, d] (Sec. 3.2; Alg. 1 PAP block)."""
    N = xn.shape[0]
    k = (xn @ np.asarray(Wk, dtype=np.float64)).reshape(N, mdl.Hkv, mdl.d)
    return rnd(rope(k, pos, mdl.rope_base))


def project_queries(xn_rows: Array, pos_rows: Array, Wq: Array, mdl: Model, rnd=identity, prefill: bool = False) -> Array:
    """Q = rope(Xn W_Q) for the given rows -> [n, H, d].  ``prefill`` with a hook marked ``prefill_queries_scaled``:
    the value that is rounded is q * log2(e)/sqrt(d) (the factor as an fp32 number); the queries returned are still q."""
    n = xn_rows.shape[0]
    q = rope((xn_rows @ np.asarray(Wq, dtype=np.float64)).reshape(n, mdl.H, mdl.d), pos_rows, mdl.rope_base)
    if prefill and getattr(rnd, "prefill_queries_scaled", False):
        c = float(np.float32(np.float32(1.4426950408889634) / np.sqrt(np.float32(mdl.d))))
        return rnd(q * c) / c
    return rnd(q)


def probe_scores(qp: Array, k: Array, mdl: Model) -> Array:
    """S^MHA, Eq. (mha_importance), with the window/GQA readings R2, R3.

    qp [P, H, d]: rotary queries of the last P candidates (probe row p is
    candidate N-P+p); k [N, Hkv, d].  Row (p, h) is a softmax over the
    candidates n <= N-P+p of q.k/sqrt(d); S is the mean of the P*H rows.
    """
    P, H, d = qp.shape
    N = k.shape[0]
    grp = H // mdl.Hkv
    S = np.zeros(N, dtype=np.float64)
    n_idx = np.arange(N)
    row_last = (N - P) + np.arange(P)                       # candidate index of each probe row
    visible = n_idx[None, :] <= row_last[:, None]           # [P, N]
    for h in range(H):
        g = h // grp
        logits = (qp[:, h, :] @ k[:, g, :].T) / math.sqrt(d)  # [P, N]
        logits = np.where(visible, logits, -np.inf)
        S += softmax_rows(logits).sum(axis=0)
    return S / (H * P)


def topk_select(scores: Array, k: int, protect_last: int = 0) -> Array:
    """Indices of the k largest scores, ties to the lower index, ascending (R6, R7).

    Written as the definition: a stable sort of all indices by descending score.
    """
    s = np.asarray(scores).astype(np.float64) + 0.0   # +0.0 folds -0.0 into +0.0
    N = s.shape[0]
    k = int(min(max(k, 0), N))
    if k == 0:
        return np.zeros(0, dtype=np.int32)
    if protect_last:
        s = s.copy()
        s[N - 1] = np.inf
    order = np.argsort(-s, kind="stable")              # stable: equal scores keep index order
    return np.sort(order[:k]).astype(np.int32)


def causal_attention(q: Array, k: Array, v: Array, qpos: Array, kpos: Array, mdl: Model) -> Array:
    """softmax(q k^T / sqrt(d) + mask) v with mask kpos[j] <= qpos[i], GQA (R3, R4).

    q [Mq, H, d], k/v [Mk, Hkv, d] -> [Mq, H, d].
    """
    Mq, H, d = q.shape
    grp = H // mdl.Hkv
    allowed = np.asarray(kpos)[None, :] <= np.asarray(qpos)[:, None]   # [Mq, Mk]
    out = np.zeros((Mq, H, d), dtype=np.float64)
    for h in range(H):
        g = h // grp
        logits = (q[:, h, :] @ k[:, g, :].T) / math.sqrt(d)
        logits = np.where(allowed, logits, -np.inf)
        out[:, h, :] = softmax_rows(logits) @ v[:, g, :]
    return out


def ffn(xn_rows: Array, Wgate: Array, Wup: Array, Wdown: Array, rnd=identity) -> Array:
    """Eq. (ffn_function): (silu(X W_gate) * (X W_up)) W_down^T, W_* in R^{D x Dff}."""
    g = xn_rows @ np.asarray(Wgate, dtype=np.float64)
    u = xn_rows @ np.asarray(Wup, dtype=np.float64)
    h = rnd(silu(g) * u)
    return h @ np.asarray(Wdown, dtype=np.float64).T


def proxy_ffn(xn: Array, w: Dict[str, Array], rnd=identity) -> Array:
    """Eq. (proxy_ffn): f(X) = (silu(X Ug Vg) * (X Uu Vu)) Vd^T Ud^T."""
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    tg = rnd(xn @ f64(w["Ug"]))
    tu = rnd(xn @ f64(w["Uu"]))
    gate = silu(tg @ f64(w["Vg"]))
    up = tu @ f64(w["Vu"])
    hp = rnd(gate * up)
    z = rnd(hp @ f64(w["Vd"]).T)
    return z @ f64(w["Ud"]).T


def transformation_scores(xn2: Array, w: Dict[str, Array], rnd=identity) -> Array:
    """C_n = ||f(X_n)||_2, Eq. (ffn_transformation)."""
    o = proxy_ffn(xn2, w, rnd)
    return np.sqrt(np.sum(o * o, axis=-1))


# --------------------------------------------------------------------------
# the five boundary calls
# --------------------------------------------------------------------------
def probe_attn(x: Array, pos: Array, w: Dict[str, Array], mdl: Model, probe_len: int,
               rnd=identity) -> Tuple[Array, Array]:
    """PAP probe: returns (K [N,Hkv,d] post-rotary, S^MHA [N])."""
    x = np.asarray(x, dtype=np.float64)
    N = x.shape[0]
    P = int(probe_len)
    xn = rnd(rmsnorm(x, w["gamma1"], mdl.rms_eps))
    k = project_keys(xn, pos, w["Wk"], mdl, rnd)
    qp = project_queries(xn[N - P:], np.asarray(pos)[N - P:], w["Wq"], mdl, rnd, prefill=True)
    return k, probe_scores(qp, k, mdl)


def probe_ffn(x: Array, w: Dict[str, Array], mdl: Model, s_mha: Optional[Array],
              rnd=identity) -> Tuple[Array, Array]:
    """LTP probe on the post-attention residual x: returns (C^FFN, S^FFN = C * S^MHA)."""
    xn2 = rnd(rmsnorm(np.asarray(x, dtype=np.float64), w["gamma2"], mdl.rms_eps))
    c = transformation_scores(xn2, w, rnd)
    s = c if s_mha is None else c * np.asarray(s_mha, dtype=np.float64)
    return c, s


@dataclass
class LayerCfg:
    skip: int = 1
    probe_len: int = 1
    m_attn: int = 0
    m_ffn: int = 0
    protect_last: int = 1
    kv_mode: int = 0


@dataclass
class LayerOut:
    x: Array
    s_mha: Optional[Array] = None
    idx_attn: Optional[Array] = None
    idx_ffn: Optional[Array] = None
    c_ffn: Optional[Array] = None
    s_ffn: Optional[Array] = None
    k_cache: Optional[Array] = None
    v_cache: Optional[Array] = None
    pos_cache: Optional[Array] = None


def layer_prefill(x: Array, pos: Array, w: Dict[str, Array], mdl: Model, cfg: LayerCfg,
                  rnd=identity,
                  score_cast: Callable[[Array], Array] = identity,
                  force_idx_attn: Optional[Array] = None,
                  force_idx_ffn: Optional[Array] = None) -> LayerOut:
    """One decoder layer of Alg. 1 (PAP block, LTP block), in place semantics on a copy of x.

    ``score_cast`` is applied to scores before a TopK takes its decision, so
    that the decision is taken in the precision the scores are stored in.
    ``force_idx_*`` replace the oracle's own selected sets (used by lock-step
    parity after near-tie swaps have been counted): either an index array, or a
    callable ``f(scores, own_idx) -> idx`` that sees the oracle's scores and its
    own selection and returns the set to continue with.
    """
    x = rnd(np.array(x, dtype=np.float64, copy=True))
    pos = np.asarray(pos)
    N = x.shape[0]
    out = LayerOut(x=x)
    if N == 0:
        return out
    f64 = lambda a: np.asarray(a, dtype=np.float64)

    # ---------------- MHA ----------------
    xn = rnd(rmsnorm(x, w["gamma1"], mdl.rms_eps))
    k_all = project_keys(xn, pos, w["Wk"], mdl, rnd)
    if cfg.skip:
        P = int(cfg.probe_len)
        qp = project_queries(xn[N - P:], pos[N - P:], w["Wq"], mdl, rnd, prefill=True)
        S = score_cast(probe_scores(qp, k_all, mdl))
        out.s_mha = S
        Ma = min(N, int(cfg.m_attn))
        Ta = topk_select(S, Ma, cfg.protect_last)
        if callable(force_idx_attn):
            Ta = np.asarray(force_idx_attn(S, Ta), dtype=np.int32)
        elif force_idx_attn is not None:
            Ta = np.asarray(force_idx_attn, dtype=np.int32)
    else:
        S = None
        Ta = np.arange(N, dtype=np.int32)
    out.idx_attn = Ta
    if Ta.size > 0:
        xa = xn[Ta]
        q = project_queries(xa, pos[Ta], w["Wq"], mdl, rnd, prefill=True)
        if cfg.skip and cfg.kv_mode == 1:
            kk = k_all
            vv = rnd((xn @ f64(w["Wv"])).reshape(N, mdl.Hkv, mdl.d))
            kpos = pos
        else:
            kk = k_all[Ta]
            vv = rnd((xa @ f64(w["Wv"])).reshape(Ta.size, mdl.Hkv, mdl.d))
            kpos = pos[Ta]
        out.k_cache, out.v_cache, out.pos_cache = kk, vv, kpos
        att = rnd(causal_attention(q, kk, vv, pos[Ta], kpos, mdl)).reshape(Ta.size, mdl.H * mdl.d)
        o = att @ f64(w["Wo"])
        x[Ta] = rnd(x[Ta] + o)

    # ---------------- FFN ----------------
    xn2 = rnd(rmsnorm(x, w["gamma2"], mdl.rms_eps))
    if cfg.skip:
        c = transformation_scores(xn2, w, rnd)
        out.c_ffn = score_cast(c)
        SF = score_cast(out.c_ffn * S)
        out.s_ffn = SF
        Mf = min(N, int(cfg.m_ffn))
        Tf = topk_select(SF, Mf, cfg.protect_last)
        if callable(force_idx_ffn):
            Tf = np.asarray(force_idx_ffn(SF, Tf), dtype=np.int32)
        elif force_idx_ffn is not None:
            Tf = np.asarray(force_idx_ffn, dtype=np.int32)
    else:
        Tf = np.arange(N, dtype=np.int32)
    out.idx_ffn = Tf
    if Tf.size > 0:
        x[Tf] = rnd(x[Tf] + ffn(xn2[Tf], w["Wgate"], w["Wup"], w["Wdown"], rnd))
    out.x = x
    return out


def msdp_compact(x: Array, pos: Array, s_mha: Array, N_next: int, protect_last: int = 1):
    """Stage-end pruning, Eq. (stage_prune): keep TopK(S^MHA, min(N, N_next)) candidates.

    Returns (x_out, pos_out, map_new2old, map_old2new) with -1 for dropped rows.
    """
    N = x.shape[0]
    keep = topk_select(s_mha, min(N, int(N_next)), protect_last)
    old2new = np.full(N, -1, dtype=np.int32)
    old2new[keep] = np.arange(keep.size, dtype=np.int32)
    return x[keep].copy(), np.asarray(pos)[keep].copy(), keep, old2new


def stack_prefill(x: Array, pos: Array, layers, mdl: Model, plan, probe_len: int,
                  protect_last: int = 1, skip: int = 1, rnd=identity, score_cast=identity):
    """Alg. 1 outer loop: ``layers[l]`` weights, ``plan[l]`` = dict(m_attn, m_ffn, N_next|None[, skip])."""
    x = np.array(x, dtype=np.float64, copy=True)
    pos = np.array(pos, copy=True)
    trace = []
    for w, item in zip(layers, plan):
        # a plan item may mark its layer dense (the paper's schedule keeps the first layers dense)
        skip_l = 1 if (skip and item.get("skip", 1)) else 0
        cfg = LayerCfg(skip=skip_l, probe_len=probe_len, m_attn=item["m_attn"], m_ffn=item["m_ffn"],
                       protect_last=protect_last)
        lo = layer_prefill(x, pos, w, mdl, cfg, rnd, score_cast)
        x = lo.x
        if skip_l and item.get("N_next") is not None:
            x, pos, new2old, _ = msdp_compact(x, pos, lo.s_mha, item["N_next"], protect_last)
            lo.map_new2old = new2old
        trace.append(lo)
    return x, pos, trace


# ------------------------------------------------------------------------------------------------
# Decode phase over the per-layer caches left by the prefill
# ------------------------------------------------------------------------------------------------
@dataclass
class LayerCache:
    """Key/value pairs one layer holds: k, v [M, Hkv, d] (keys post-rotary), pos [M] absolute."""
    k: Array
    v: Array
    pos: Array


def decode_layer(x_t: Array, pos_t: int, w: Dict[str, Array], mdl: Model, cache: LayerCache, rnd=identity):
    """One decoder layer for one new token in the decode phase (Alg. 1 else-branches: standard MHA
    with residual, the cache is updated; standard FFN).  x_t [D]; returns (x_out [D], new cache).

    The token's rotary key and its value join the cache first; its query then attends to every
    cached pair (all cached positions are <= pos_t, so the causal mask hides nothing).
    """
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    x = rnd(np.array(x_t, dtype=np.float64, copy=True)).reshape(1, -1)
    p = np.array([pos_t])
    xn = rnd(rmsnorm(x, w["gamma1"], mdl.rms_eps))
    k_new = project_keys(xn, p, w["Wk"], mdl, rnd)
    v_new = rnd((xn @ f64(w["Wv"])).reshape(1, mdl.Hkv, mdl.d))
    q = project_queries(xn, p, w["Wq"], mdl, rnd)
    kk = np.concatenate([f64(cache.k), k_new], axis=0)
    vv = np.concatenate([f64(cache.v), v_new], axis=0)
    kpos = np.concatenate([np.asarray(cache.pos), p])
    att = rnd(causal_attention(q, kk, vv, p, kpos, mdl)).reshape(1, mdl.H * mdl.d)
    x = rnd(x + att @ f64(w["Wo"]))
    xn2 = rnd(rmsnorm(x, w["gamma2"], mdl.rms_eps))
    x = rnd(x + ffn(xn2, w["Wgate"], w["Wup"], w["Wdown"], rnd))
    return x[0], LayerCache(kk, vv, kpos)


def decode_step(x_t: Array, pos_t: int, layers, mdl: Model, caches, rnd=identity):
    """All layers for one new token: returns (final hidden state [D], list of updated caches)."""
    x = np.asarray(x_t, dtype=np.float64)
    out = []
    for w, c in zip(layers, caches):
        x, c2 = decode_layer(x, pos_t, w, mdl, c, rnd)
        out.append(c2)
    return x, out


def greedy_token(h: Array, gamma_f: Array, table: Array, mdl: Model, rnd=identity, logit_cast=identity):
    """Final RMSNorm, logits against the vocabulary table [V, D], argmax with ties to the lowest
    token id.  Returns (token, logits [V]); ``logit_cast`` is applied before the decision."""
    hn = rnd(rmsnorm(np.asarray(h, dtype=np.float64).reshape(1, -1), gamma_f, mdl.rms_eps))
    logits = logit_cast((hn @ np.asarray(table, dtype=np.float64).T)[0])
    best = np.flatnonzero(logits == np.max(logits))
    return int(best[0]), logits


# ------------------------------------------------------------------------------------------------
# Offline proxy construction: data-driven choice of the Dlow channels (Sec. 3.3)
# ------------------------------------------------------------------------------------------------
def channel_saliency(x_cal: Array, Wgate: Array, Wup: Array, rnd=identity) -> Array:
    """z(x) = |silu(x W_gate) * (x W_up)| for every calibration token: [T, Dff] (Sec. 3.3)."""
    x = np.asarray(x_cal, dtype=np.float64)
    g = x @ np.asarray(Wgate, dtype=np.float64)
    u = x @ np.asarray(Wup, dtype=np.float64)
    return np.abs(rnd(silu(g) * u))


def channel_importance(x_cal: Array, Wgate: Array, Wup: Array, k: int, rnd=identity) -> Array:
    """Eq. (channel_importance): I_j = mean of the k = rho*|G| largest saliencies of channel j."""
    z = channel_saliency(x_cal, Wgate, Wup, rnd)
    T = z.shape[0]
    k = int(min(max(k, 1), T))
    top = -np.sort(-z, axis=0)[:k]          # k largest per column
    return top.sum(axis=0) / float(k)


def select_channels(importance: Array, dlow: int) -> Array:
    """C = TopK(I, Dlow), ascending channel ids; ties to the lower id (the TopK rule of R6)."""
    return topk_select(importance, dlow, 0)
