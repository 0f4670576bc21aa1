"""Pins of the oracle's offline channel selection (Sec. 3.3, Eq. (channel_importance)) against things
other than itself: Python loops, closed-form special cases, invariances (runs without a GPU)."""
import math

import numpy as np

from oracle import spts_oracle as orc


def _case(T=37, D=12, Dff=20, seed=0):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((T, D)), rng.standard_normal((D, Dff)) / math.sqrt(D), rng.standard_normal((D, Dff)) / math.sqrt(D)


def test_importance_against_loops():
    x, Wg, Wu = _case()
    T, Dff, k = x.shape[0], Wg.shape[1], 7
    I = orc.channel_importance(x, Wg, Wu, k)
    for j in range(Dff):
        vals = []
        for t in range(T):
            g = float(np.dot(x[t], Wg[:, j])); u = float(np.dot(x[t], Wu[:, j]))
            vals.append(abs(g / (1.0 + math.exp(-g)) * u))
        vals.sort(reverse=True)
        assert abs(I[j] - sum(vals[:k]) / k) < 1e-12


def test_special_cases_mean_and_max():
    x, Wg, Wu = _case(seed=1)
    z = orc.channel_saliency(x, Wg, Wu)
    assert np.all(z >= 0)
    assert np.allclose(orc.channel_importance(x, Wg, Wu, x.shape[0]), z.mean(axis=0), rtol=1e-13)   # rho = 1
    assert np.allclose(orc.channel_importance(x, Wg, Wu, 1), z.max(axis=0), rtol=0, atol=0)         # one value
    # monotone in k: averaging in smaller values can only lower the score
    a, b = orc.channel_importance(x, Wg, Wu, 3), orc.channel_importance(x, Wg, Wu, 9)
    assert np.all(a >= b - 1e-15)


def test_token_permutation_invariance_and_planted_channel():
    x, Wg, Wu = _case(seed=2)
    perm = np.random.default_rng(5).permutation(x.shape[0])
    assert np.allclose(orc.channel_importance(x, Wg, Wu, 5), orc.channel_importance(x[perm], Wg, Wu, 5), rtol=1e-13)
    # a channel whose gate and up columns are scaled up dominates and must be selected first
    Wg2, Wu2 = Wg.copy(), Wu.copy()
    Wg2[:, 4] *= 50.0; Wu2[:, 4] *= 50.0
    I = orc.channel_importance(x, Wg2, Wu2, 5)
    assert int(np.argmax(I)) == 4
    C = orc.select_channels(I, 6)
    assert 4 in C and np.all(np.diff(C) > 0) and C.size == 6
    # the selection is the Dlow largest scores
    assert set(C.tolist()) == set(np.argsort(-I, kind="stable")[:6].tolist())
