"""Pins for the oracle's paged grouped-query decode attention.

The paper names no formula (generation runs inside an inference engine,
Appendix A.2): the definition is textbook softmax attention of one query over
the sequence's cached keys/values.  Pins: a brute-force scalar-loop twin, the
library softmax on densely gathered K/V, closed forms, and invariants.
"""
import math

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import copris_oracle as O
from paper_2511_05589_amd import workloads as W


def _f(case, key):
    return W.to_f32(case[key], case["dtype"]).astype(np.float64)


def _brute(case):
    """Scalar loops; walks tokens one by one through the block table."""
    q, K, V = _f(case, "q"), _f(case, "k_cache"), _f(case, "v_cache")
    bt, ctx, P = case["block_table"], case["ctx_len"], case["page_size"]
    C, Hq, D = q.shape
    g = Hq // case["Hkv"]
    out = np.zeros((C, Hq, D))
    lse = np.full((C, Hq), -np.inf)
    for i in range(C):
        for h in range(Hq):
            kvh = h // g
            scores = []
            for t in range(int(ctx[i])):
                page, slot = int(bt[i, t // P]), t % P
                s = 0.0
                for d in range(D):
                    s += q[i, h, d] * K[page, kvh, slot, d]
                scores.append(s * case["scale"])
            if not scores:
                continue
            m = max(scores)
            wts = [math.exp(s - m) for s in scores]
            tot = sum(wts)
            for t, w in enumerate(wts):
                page, slot = int(bt[i, t // P]), t % P
                for d in range(D):
                    out[i, h, d] += (w / tot) * V[page, kvh, slot, d]
            lse[i, h] = m + math.log(tot)
    return out, lse


def _run(case):
    return O.decode_attn(_f(case, "q"), _f(case, "k_cache"), _f(case, "v_cache"),
                         case["block_table"], case["ctx_len"], case["scale"])


@pytest.mark.parametrize("seed,C,Hq,Hkv,D,P,ctx", [
    (1, 3, 4, 2, 8, 4, [1, 5, 9]),
    (2, 2, 6, 1, 4, 16, [16, 33]),
    (3, 4, 7, 7, 16, 2, [3, 2, 1, 7]),
    (4, 2, 14, 2, 8, 8, [8, 17]),
])
def test_matches_brute_force(seed, C, Hq, Hkv, D, P, ctx):
    case = W.make_small_decode_case(seed, C, Hq, Hkv, D, W.F32, P, ctx)
    out, lse = _run(case)
    bout, blse = _brute(case)
    np.testing.assert_allclose(out, bout, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, blse, rtol=0, atol=1e-12)


def test_matches_library_softmax_on_dense_gather_tiny_config():
    cfg = W.DECODE_CONFIGS[0]
    inp = W.make_decode_inputs(cfg, with_lmhead=False)
    q = W.to_f32(inp["q"], cfg.dtype).astype(np.float64)
    K = W.to_f32(inp["k_cache"], cfg.dtype).astype(np.float64)
    V = W.to_f32(inp["v_cache"], cfg.dtype).astype(np.float64)
    out, lse = O.decode_attn(q, K, V, inp["block_table"], inp["ctx_len"], inp["scale"])
    assert np.isfinite(out).all()
    for i in range(cfg.C):
        n = int(inp["ctx_len"][i])
        tok = np.arange(n)
        pages = inp["block_table"][i, tok // cfg.page_size]
        for h in range(cfg.Hq):
            Kd = K[pages, h // cfg.g, tok % cfg.page_size]          # [n, D] dense
            Vd = V[pages, h // cfg.g, tok % cfg.page_size]
            s = inp["scale"] * Kd @ q[i, h]
            np.testing.assert_allclose(out[i, h], softmax(s) @ Vd, atol=1e-12)
            np.testing.assert_allclose(lse[i, h], logsumexp(s), atol=1e-12)


def test_closed_forms():
    case = W.make_small_decode_case(7, 4, 4, 2, 8, W.F32, 4, [1, 6, 8, 11])
    K, V, q = _f(case, "k_cache"), _f(case, "v_cache"), _f(case, "q")
    bt, ctx = case["block_table"], case["ctx_len"]
    out, lse = O.decode_attn(q, K, V, bt, ctx, case["scale"])
    # one token of context: the output is that token's value row
    np.testing.assert_array_equal(out[0, 0], V[bt[0, 0], 0, 0])
    np.testing.assert_array_equal(out[0, 3], V[bt[0, 0], 1, 0])
    # zero query: uniform weights -> mean of the values, lse = ln n
    out0, lse0 = O.decode_attn(np.zeros_like(q), K, V, bt, ctx, case["scale"])
    for i in range(4):
        n = int(ctx[i])
        tok = np.arange(n)
        for kvh in range(2):
            mean = V[bt[i, tok // 4], kvh, tok % 4].mean(axis=0)
            np.testing.assert_allclose(out0[i, 2 * kvh], mean, atol=1e-13)
        np.testing.assert_allclose(lse0[i], math.log(n), atol=1e-13)
    # constant values -> that constant, whatever the weights
    Vc = np.where(np.isnan(V), np.nan, 3.25)
    outc, _ = O.decode_attn(q, K, Vc, bt, ctx, case["scale"])
    np.testing.assert_allclose(outc, 3.25, atol=1e-13)
    # two query heads of one group with the same query give the same output
    q2 = q.copy()
    q2[:, 1] = q2[:, 0]
    out2, _ = O.decode_attn(q2, K, V, bt, ctx, case["scale"])
    np.testing.assert_array_equal(out2[:, 0], out2[:, 1])
    assert not np.allclose(out2[:, 0], out2[:, 2])


def test_gqa_equals_mha_with_repeated_kv_heads():
    case = W.make_small_decode_case(9, 3, 6, 2, 8, W.F32, 4, [5, 9, 12])
    K, V, q = _f(case, "k_cache"), _f(case, "v_cache"), _f(case, "q")
    out, lse = O.decode_attn(q, K, V, case["block_table"], case["ctx_len"], case["scale"])
    Kr, Vr = np.repeat(K, 3, axis=1), np.repeat(V, 3, axis=1)       # head h -> kv head h//3
    outr, lser = O.decode_attn(q, Kr, Vr, case["block_table"], case["ctx_len"], case["scale"])
    np.testing.assert_array_equal(out, outr)
    np.testing.assert_array_equal(lse, lser)


def test_physical_page_permutation_leaves_output_unchanged_bitwise():
    case = W.make_small_decode_case(11, 4, 4, 2, 16, W.F32, 8, [3, 40, 17, 64])
    K, V, q = _f(case, "k_cache"), _f(case, "v_cache"), _f(case, "q")
    bt, ctx = case["block_table"], case["ctx_len"]
    out, lse = O.decode_attn(q, K, V, bt, ctx, case["scale"])
    perm = np.random.default_rng(0).permutation(K.shape[0])      # new id of old page p is perm[p]
    K2, V2 = np.empty_like(K), np.empty_like(V)
    K2[perm], V2[perm] = K, V
    bt2 = np.where(bt >= 0, perm[np.maximum(bt, 0)], -1).astype(np.int32)
    out2, lse2 = O.decode_attn(q, K2, V2, bt2, ctx, case["scale"])
    np.testing.assert_array_equal(out, out2)
    np.testing.assert_array_equal(lse, lse2)


def test_poisoned_unused_slots_never_leak_and_poison_is_there():
    case = W.make_small_decode_case(13, 3, 2, 1, 8, W.F32, 8, [5, 8, 13], poison=True)
    assert np.isnan(_f(case, "k_cache")).any() and np.isnan(_f(case, "v_cache")).any()
    out, lse = _run(case)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    clean = W.make_small_decode_case(13, 3, 2, 1, 8, W.F32, 8, [5, 8, 13], poison=False)
    outc, lsec = _run(clean)
    np.testing.assert_array_equal(out, outc)


def test_large_scores_do_not_overflow_and_pick_the_max_key():
    case = W.make_small_decode_case(15, 1, 1, 1, 4, W.F32, 4, [6], poison=False)
    K, V = _f(case, "k_cache"), _f(case, "v_cache")
    q = np.full((1, 1, 4), 500.0)
    bt = case["block_table"]
    K[:] = 0.0
    K[bt[0, 1], 0, 1] = 1.0                       # token 5 has score 2000*scale, others 0
    out, lse = O.decode_attn(q, K, V, bt, case["ctx_len"], 1.0)
    np.testing.assert_allclose(out[0, 0], V[bt[0, 1], 0, 1], atol=1e-300)
    assert np.isfinite(lse).all() and abs(lse[0, 0] - 2000.0) < 1e-9


def test_zero_length_sequence():
    case = W.make_small_decode_case(17, 2, 2, 1, 4, W.F32, 4, [0, 3])
    out, lse = _run(case)
    assert (out[0] == 0).all() and np.isneginf(lse[0]).all() and np.isfinite(out[1]).all()


def test_scale_and_head_mapping_are_not_symmetric():
    # a wrong kv-head mapping (h % Hkv instead of h // g) or a dropped scale changes the answer
    case = W.make_small_decode_case(19, 1, 4, 2, 8, W.F32, 4, [9], poison=False)
    K, V, q = _f(case, "k_cache"), _f(case, "v_cache"), _f(case, "q")
    out, _ = O.decode_attn(q, K, V, case["block_table"], case["ctx_len"], case["scale"])
    # head 1 belongs to kv head 0: changing kv head 1 must not move it, changing kv head 0 must
    K1 = K.copy(); K1[:, 1] *= -2.0
    o1, _ = O.decode_attn(q, K1, V, case["block_table"], case["ctx_len"], case["scale"])
    np.testing.assert_array_equal(out[0, :2], o1[0, :2])
    assert not np.allclose(out[0, 2:], o1[0, 2:])
    o2, _ = O.decode_attn(q, K, V, case["block_table"], case["ctx_len"], 1.0)
    assert not np.allclose(out, o2)
