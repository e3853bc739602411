"""Pins for the oracle's re-prefill attention (causal, packed variable-length sequences) and
KV page fill (Section 4, "Prioritized Resumption": buffered partial trajectories are
continued in the next stage, which needs their KV under the new weights)."""
import math

import numpy as np
import pytest
from scipy.special import softmax

from oracle import copris_oracle as O


def _case(seed, lens, Hq=4, Hkv=2, D=8):
    rng = np.random.default_rng(seed)
    T = int(sum(lens))
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    return (rng.normal(size=(T, Hq, D)), rng.normal(size=(T, Hkv, D)), rng.normal(size=(T, Hkv, D)), cu)


def test_brute_force_scalar_loops():
    q, k, v, cu = _case(1, [3, 1, 5], Hq=2, Hkv=1, D=4)
    out, lse = O.prefill_attn(q, k, v, cu, 0.5)
    for b in range(3):
        for t in range(cu[b], cu[b + 1]):
            for h in range(2):
                sc = [0.5 * sum(q[t, h, d] * k[u, 0, d] for d in range(4)) for u in range(cu[b], t + 1)]
                mx = max(sc)
                w = [math.exp(x - mx) for x in sc]
                for d in range(4):
                    want = sum(wi * v[cu[b] + i, 0, d] for i, wi in enumerate(w)) / sum(w)
                    assert out[t, h, d] == pytest.approx(want, rel=1e-12, abs=1e-14)
                assert lse[t, h] == pytest.approx(mx + math.log(sum(w)), rel=1e-12)


def test_against_library_softmax_with_an_explicit_mask():
    q, k, v, cu = _case(2, [7, 12], Hq=4, Hkv=2, D=8)
    out, _ = O.prefill_attn(q, k, v, cu, 0.3)
    for b in range(2):
        s0, s1 = cu[b], cu[b + 1]
        n = s1 - s0
        for h in range(4):
            S = 0.3 * q[s0:s1, h] @ k[s0:s1, h // 2].T
            S = np.where(np.tril(np.ones((n, n), bool)), S, -np.inf)
            np.testing.assert_allclose(out[s0:s1, h], softmax(S, axis=1) @ v[s0:s1, h // 2], rtol=1e-12, atol=1e-14)


def test_causality_and_sequence_isolation():
    q, k, v, cu = _case(3, [6, 9])
    out, lse = O.prefill_attn(q, k, v, cu, 1.0)
    k2, v2 = k.copy(), v.copy()
    k2[4:6] += 10.0; v2[4:6] -= 3.0           # the last two tokens of sequence 0
    out2, _ = O.prefill_attn(q, k2, v2, cu, 1.0)
    np.testing.assert_array_equal(out2[:4], out[:4])      # earlier tokens do not see them
    np.testing.assert_array_equal(out2[6:], out[6:])      # the other sequence does not either
    assert np.abs(out2[4:6] - out[4:6]).max() > 1e-3


def test_first_token_returns_its_own_value_and_zero_queries_give_running_means():
    q, k, v, cu = _case(4, [5], Hq=2, Hkv=2)
    out, lse = O.prefill_attn(q, k, v, cu, 1.0)
    np.testing.assert_allclose(out[0], v[0], rtol=1e-15)
    out0, lse0 = O.prefill_attn(np.zeros_like(q), k, v, cu, 1.0)
    for t in range(5):
        np.testing.assert_allclose(out0[t], v[:t + 1].mean(axis=0), rtol=1e-13)
        np.testing.assert_allclose(lse0[t], math.log(t + 1), rtol=1e-13)


def test_last_token_equals_decode_attention_over_the_filled_pages():
    # ties the prefill to the decode oracle: after the page fill, decoding with the last
    # token's query over the whole context gives the prefill's last row
    lens = [19, 1, 33]
    q, k, v, cu = _case(5, lens, Hq=6, Hkv=2, D=16)
    P, num_pages = 16, 9
    rng = np.random.default_rng(0)
    bt = np.full((3, 3), -1, dtype=np.int32)
    perm = rng.permutation(num_pages)
    used = 0
    for b, n in enumerate(lens):
        npg = (n + P - 1) // P
        bt[b, :npg] = perm[used:used + npg]; used += npg
    kc = np.full((num_pages, 2, P, 16), np.nan); vc = np.full((num_pages, 2, P, 16), np.nan)
    O.kv_page_fill(k, v, cu, bt, kc, vc)
    out, lse = O.prefill_attn(q, k, v, cu, 0.25)
    last = cu[1:] - 1
    dout, dlse = O.decode_attn(q[last], kc, vc, bt, np.array(lens), 0.25)
    np.testing.assert_allclose(dout, out[last], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(dlse, lse[last], rtol=1e-13)
    # the fill touched exactly the slots that hold a token
    filled = ~np.isnan(kc[:, 0, :, 0])
    assert filled.sum() == sum(lens)
    t = 20                                  # token 20 of sequence 2: page 1, slot 4
    np.testing.assert_array_equal(kc[bt[2, 1], :, 4], k[cu[2] + t])
    np.testing.assert_array_equal(vc[bt[2, 1], :, 4], v[cu[2] + t])


def test_head_mapping_and_scale():
    q, k, v, cu = _case(6, [8], Hq=4, Hkv=2)
    out, _ = O.prefill_attn(q, k, v, cu, 0.7)
    # GQA equals MHA with the kv heads repeated
    out_rep, _ = O.prefill_attn(q, np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1), cu, 0.7)
    np.testing.assert_allclose(out, out_rep, rtol=1e-14)
    # swapping the two kv heads changes the result (head h reads kv head h // g)
    out_sw, _ = O.prefill_attn(q, k[:, ::-1], v[:, ::-1], cu, 0.7)
    assert np.abs(out - out_sw).max() > 1e-3
    out_sc, _ = O.prefill_attn(q, k, v, cu, 0.35)
    assert np.abs(out - out_sc).max() > 1e-3
    out_q, _ = O.prefill_attn(0.5 * q, k, v, cu, 0.7)      # scaling q = scaling the scores
    np.testing.assert_allclose(out_q, out_sc, rtol=1e-13)
