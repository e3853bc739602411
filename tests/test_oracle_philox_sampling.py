"""Pins for the oracle's Philox stream, uniform mapping and Gumbel-max sampler.

Nothing here calls the HIP path.  The pins are: the generator's published
known-answer vectors, an independently written pure-Python-int Philox, moments of
the uniform / Gumbel variates, and a chi-square test of sampled token
frequencies against softmax(z) (Table 4 of the paper fixes top-p 1, top-k -1,
T 1: the sampler's law is the untruncated softmax).
"""
import math
import os

import numpy as np
import pytest
from scipy import stats
from scipy.special import softmax

from oracle import copris_oracle as O


def _philox_pyint(ctr, key):
    """Second implementation: plain Python integers, one block at a time."""
    c = [int(x) & 0xFFFFFFFF for x in ctr]
    k = [int(x) & 0xFFFFFFFF for x in key]
    for r in range(10):
        prod_a = 0xD2511F53 * c[0]
        prod_b = 0xCD9E8D57 * c[2]
        c = [((prod_b >> 32) ^ c[1] ^ k[0]) & 0xFFFFFFFF, prod_b & 0xFFFFFFFF,
             ((prod_a >> 32) ^ c[3] ^ k[1]) & 0xFFFFFFFF, prod_a & 0xFFFFFFFF]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def test_philox_known_answers(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.split("#")[0].replace("->", " ").split()
            if line:
                rows.append([int(w, 16) for w in line])
    assert len(rows) == 3
    for r in rows:
        got = O.philox4x32_10(r[0:4], r[4:6])
        assert [int(x) for x in got] == r[6:10]
        assert _philox_pyint(r[0:4], r[4:6]) == r[6:10]


def test_philox_vectorised_matches_python_ints():
    rng = np.random.default_rng(1)
    ctr = rng.integers(0, 2**32, size=(4, 200), dtype=np.uint64)
    key = rng.integers(0, 2**32, size=(2, 200), dtype=np.uint64)
    got = np.stack(O.philox4x32_10(tuple(ctr), tuple(key)), axis=1)
    for j in range(200):
        assert list(map(int, got[j])) == _philox_pyint(ctr[:, j], key[:, j])


def test_uniform_layout_word_and_counter():
    # vocabulary entry v uses word v&3 of block v>>2; counter = (blk, step, id lo, id hi)
    seed, sid, step, V = 0x0123456789ABCDEF, (5 << 32) | 77, 4242, 37
    u = O.sampling_uniforms(seed, sid, step, V)
    for v in (0, 1, 2, 3, 4, 5, 35, 36):
        words = _philox_pyint((v >> 2, step, 77, 5), (0x89ABCDEF, 0x01234567))
        expect = ((words[v & 3] >> 9) + 0.5) / 2**23
        assert u[v] == expect
    # independent of V (prefix property) and of anything but (seed, id, step)
    assert np.array_equal(O.sampling_uniforms(seed, sid, step, 9), u[:9])
    assert not np.array_equal(O.sampling_uniforms(seed, sid, step + 1, V), u)
    assert not np.array_equal(O.sampling_uniforms(seed, sid + 1, step, V), u)
    assert not np.array_equal(O.sampling_uniforms(seed + 1, sid, step, V), u)
    assert not np.array_equal(O.sampling_uniforms(seed, sid + (1 << 32), step, V), u)
    assert not np.array_equal(O.sampling_uniforms(seed + (1 << 32), sid, step, V), u)


def test_uniforms_open_interval_fp32_exact_and_moments():
    u = O.sampling_uniforms(7, 11, 13, 1 << 18)
    assert u.min() > 0.0 and u.max() < 1.0
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)   # exact in fp32
    n = u.size
    assert abs(u.mean() - 0.5) < 5 / math.sqrt(12 * n)
    assert abs(u.var() - 1 / 12) < 1e-3
    # uniformity over 64 cells
    chi = stats.chisquare(np.bincount((u * 64).astype(int), minlength=64))
    assert chi.pvalue > 1e-4


def test_gumbel_moments_and_range():
    g = O.gumbel_noise(3, 5, 9, 1 << 18)
    n = g.size
    euler_gamma = 0.5772156649015329
    assert abs(g.mean() - euler_gamma) < 5 * math.sqrt(math.pi**2 / 6 / n)
    assert abs(g.var() - math.pi**2 / 6) < 0.03
    # range implied by the 2^-24-midpoint mapping
    assert g.min() >= -math.log(-math.log(2.0**-24)) - 1e-12
    assert g.max() <= -math.log(-math.log(1 - 2.0**-24)) + 1e-12
    # distribution: exp(-exp(-g)) is uniform
    ks = stats.kstest(np.exp(-np.exp(-g)), "uniform")
    assert ks.pvalue > 1e-4


def test_zero_weights_token_is_argmax_of_noise_and_logprob_is_minus_log_V():
    C, H, V = 5, 8, 203
    hidden = np.random.default_rng(0).standard_normal((C, H))
    weight = np.zeros((V, H))
    seq_id = np.array([10, 11, 2**40 + 3, 13, 14], dtype=np.int64)
    step = np.array([0, 1, 2, 3, 70000], dtype=np.int32)
    res = O.lmhead_logprob(hidden, weight, seq_id, step, seed=99, temperature=1.0)
    for c in range(C):
        g = O.gumbel_noise(99, int(seq_id[c]), int(step[c]), V)
        assert res["token"][c] == int(np.argmax(g))
    np.testing.assert_allclose(res["logprob"], -math.log(V), rtol=0, atol=1e-13)


def test_sampler_frequencies_follow_softmax():
    # one fixed logit vector, many (trajectory, step) streams
    V, H, n = 12, 6, 30000
    rng = np.random.default_rng(5)
    weight = rng.standard_normal((V, H))
    h = rng.standard_normal(H)
    z = weight @ h
    hidden = np.tile(h, (n, 1))
    seq_id = np.arange(n, dtype=np.int64) // 100 + 1000
    step = (np.arange(n) % 100).astype(np.int32)
    res = O.lmhead_logprob(hidden, weight, seq_id, step, seed=2024, temperature=1.0)
    counts = np.bincount(res["token"], minlength=V)
    p = softmax(z)
    chi = stats.chisquare(counts, p * n)
    assert chi.pvalue > 1e-3, (counts, p * n)
    # the kept log-prob is the model's log-softmax at the drawn token
    np.testing.assert_allclose(res["logprob"], np.log(p)[res["token"]], atol=1e-12)


def test_sampler_temperature_scales_logits_for_sampling_and_logprob():
    V, H, n = 8, 4, 20000
    rng = np.random.default_rng(8)
    weight = rng.standard_normal((V, H))
    h = rng.standard_normal(H)
    T = 0.6                                  # the paper's evaluation temperature (Table 4)
    p = softmax((weight @ h) / T)
    res = O.lmhead_logprob(np.tile(h, (n, 1)), weight, np.arange(n, dtype=np.int64),
                           np.zeros(n, dtype=np.int32), seed=1, temperature=T)
    chi = stats.chisquare(np.bincount(res["token"], minlength=V), p * n)
    assert chi.pvalue > 1e-3
    np.testing.assert_allclose(res["logprob"], np.log(p)[res["token"]], atol=1e-12)
