"""Pins for the oracle's log-probability of given tokens under the current policy
(Section 4, "Cross-stage Importance Sampling Correction": L^(theta) of Eq. 8)."""
import math

import numpy as np
import pytest
from scipy.special import log_softmax

from oracle import copris_oracle as O
from paper_2511_05589_amd import workloads as W


def _case(seed=0, M=7, H=32, V=50, std=0.5):
    rng = np.random.default_rng(seed)
    h = rng.normal(size=(M, H))
    w = rng.normal(scale=std, size=(V, H))
    tok = rng.integers(0, V, size=M)
    return h, w, tok


def test_brute_force_scalar_loops():
    h, w, tok = _case(1, M=4, H=9, V=13)
    res = O.lmhead_token_logprob(h, w, tok, 0.7)
    for m in range(4):
        z = [sum(h[m, k] * w[v, k] for k in range(9)) / 0.7 for v in range(13)]
        zm = max(z)
        lse = zm + math.log(sum(math.exp(x - zm) for x in z))
        assert res["lse"][m] == pytest.approx(lse, rel=1e-13)
        assert res["logprob"][m] == pytest.approx(z[tok[m]] - lse, rel=1e-12, abs=1e-13)


def test_against_library_log_softmax():
    h, w, tok = _case(2, M=11, H=64, V=301)
    for T in (1.0, 0.6):
        res = O.lmhead_token_logprob(h, w, tok, T)
        ref = log_softmax((h @ w.T) / T, axis=1)
        np.testing.assert_allclose(res["logprob"], ref[np.arange(11), tok], rtol=1e-12, atol=1e-12)


def test_probabilities_of_all_tokens_of_a_position_sum_to_one():
    h, w, _ = _case(3, M=1, H=16, V=40)
    hh = np.repeat(h, 40, axis=0)
    res = O.lmhead_token_logprob(hh, w, np.arange(40), 1.0)
    assert np.exp(res["logprob"]).sum() == pytest.approx(1.0, rel=1e-13)
    assert np.ptp(res["lse"]) == 0.0


def test_zero_weights_give_the_uniform_distribution():
    h, w, tok = _case(4, M=5, H=8, V=1000)
    res = O.lmhead_token_logprob(h, np.zeros_like(w), tok, 1.0)
    np.testing.assert_allclose(res["logprob"], -math.log(1000), rtol=1e-14)


def test_weight_orientation_and_row_independence():
    h, w, tok = _case(5, M=6, H=12, V=12)     # square on purpose: a transposed W would still run
    res = O.lmhead_token_logprob(h, w, tok, 1.0)
    bad = O.lmhead_token_logprob(h, w.T.copy(), tok, 1.0)
    assert np.abs(res["logprob"] - bad["logprob"]).max() > 1e-3
    perm = np.random.default_rng(0).permutation(6)
    res_p = O.lmhead_token_logprob(h[perm], w, tok[perm], 1.0)
    np.testing.assert_array_equal(res_p["logprob"], res["logprob"][perm])


def test_dominating_logit():
    # one vocabulary row aligned with the hidden state, the rest orthogonal: p -> 1 for it
    H, V = 8, 20
    h = np.zeros((2, H)); h[:, 0] = 30.0
    w = np.zeros((V, H)); w[7, 0] = 1.0
    res = O.lmhead_token_logprob(h, w, np.array([7, 3]), 1.0)
    assert res["logprob"][0] == pytest.approx(-(V - 1) * math.exp(-30.0), rel=1e-6)
    assert res["logprob"][1] == pytest.approx(-30.0 - (V - 1) * math.exp(-30.0), rel=1e-12)


def test_agrees_with_the_sampling_path_on_its_own_token():
    # the log-prob stored at rollout time and the one recomputed under the same weights
    # are the same number: the ratio of Eq. 8 is exactly 1 on-policy
    case = W.make_small_lmhead_case(6, 5, 32, 200, W.F32)
    s = O.lmhead_logprob(case["hidden"], case["weight"], case["seq_id"], case["step"], case["seed"], 1.0)
    t = O.lmhead_token_logprob(case["hidden"], case["weight"], s["token"], 1.0)
    np.testing.assert_array_equal(t["logprob"], s["logprob"])
    np.testing.assert_array_equal(t["lse"], s["lse"])
