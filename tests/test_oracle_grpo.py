"""Pins for the oracle's GRPO clipped surrogate on the cross-stage ratio.

Eq. 3: L = min(r A, clip(r, 1-eps, 1+eps) A) per token, r from Eq. 8, A the
group-normalised advantage of Eq. 4 (one per trajectory); Eq. 2 averages per
sequence and then over sequences, Table 4 lists "token mean" aggregation and
clip ratio low 0.2 / high 0.28.
"""
import math

import numpy as np
import pytest

from oracle import copris_oracle as O
from paper_2511_05589_amd import workloads as W


def _run(b, **over):
    a = dict(b); a.update(over)
    return O.grpo_surrogate(a["logp_cur"], a["logp_buf"], a["logp_roll"], a["cu_seqlens"], a["split"],
                            a["mask"], a["adv"], a["eps_low"], a["eps_high"])


def _small(seed=0, B=6, lo=1, hi=40, sigma=0.3, mask_zero_frac=0.2, **kw):
    cfg = W.ISConfig(99, "t", B=B, layout="packed", len_lo=lo, len_hi=hi, sigma=sigma,
                     mask_zero_frac=mask_zero_frac, **kw)
    return W.make_is_inputs(cfg, rng=np.random.default_rng(seed))


def _one_token(delta, adv, eps_low=0.2, eps_high=0.28):
    """A batch of one sequence of one token with cur - old = delta."""
    f = lambda x: np.array([x], dtype=np.float64)
    return O.grpo_surrogate(f(-1.0 + delta), f(-1.0), f(np.nan), np.array([0, 1]), np.array([1]), None,
                            f(adv), eps_low, eps_high)


def test_brute_force_token_loop():
    b = _small(seed=3, eps_high=0.28)
    res = _run(b)
    cu = b["cu_seqlens"]
    tot_all, cnt_all, seq_terms = 0.0, 0, []
    for s in range(b["B"]):
        A = float(b["adv"][s])
        tot, cnt = 0.0, 0
        for j in range(cu[s], cu[s + 1]):
            if b["mask"][j] == 0:
                assert res["surr"][j] == 0.0 and res["grad"][j] == 0.0
                continue
            old = b["logp_buf"][j] if j - cu[s] < b["split"][s] else b["logp_roll"][j]
            r = math.exp(float(b["logp_cur"][j]) - float(old))
            rc = min(max(r, 1 - b["eps_low"]), 1 + b["eps_high"])
            want = min(r * A, rc * A)
            assert res["surr"][j] == pytest.approx(want, rel=1e-14, abs=0.0)
            if r * A <= rc * A:
                assert res["grad"][j] == pytest.approx(r * A, rel=1e-14, abs=0.0)
            else:
                assert res["grad"][j] == 0.0
            tot += want; cnt += 1
        assert res["seq_surr"][s] == pytest.approx(tot, rel=1e-12, abs=1e-300)
        assert res["seq_cnt"][s] == cnt
        tot_all += tot; cnt_all += cnt
        seq_terms.append(tot / cnt if cnt else 0.0)
    assert res["obj_token_mean"] == pytest.approx(tot_all / cnt_all, rel=1e-12)
    assert res["obj_seq_mean"] == pytest.approx(sum(seq_terms) / b["B"], rel=1e-12)


@pytest.mark.parametrize("delta,adv,want_surr,want_grad", [
    # inside the clip range: the plain policy-gradient term
    (math.log(1.1), 2.0, 1.1 * 2.0, 1.1 * 2.0),
    (math.log(0.9), -3.0, 0.9 * -3.0, 0.9 * -3.0),
    # positive advantage: gains above 1+eps_high are cut off (no gradient) ...
    (math.log(1.5), 2.0, 1.28 * 2.0, 0.0),
    # ... but a ratio below 1-eps_low is NOT clipped (the min keeps the smaller, unclipped term)
    (math.log(0.5), 2.0, 0.5 * 2.0, 0.5 * 2.0),
    # negative advantage: mirrored
    (math.log(0.5), -1.0, 0.8 * -1.0, 0.0),
    (math.log(1.5), -1.0, 1.5 * -1.0, 1.5 * -1.0),
    # a trajectory from a group with equal rewards contributes nothing
    (math.log(1.5), 0.0, 0.0, 0.0),
])
def test_branches_of_the_clipped_min_with_table_4_bounds(delta, adv, want_surr, want_grad):
    res = _one_token(delta, adv)
    assert res["surr"][0] == pytest.approx(want_surr, rel=1e-14, abs=0.0)
    assert res["grad"][0] == pytest.approx(want_grad, rel=1e-14, abs=0.0)
    assert res["obj_token_mean"] == pytest.approx(want_surr, rel=1e-14, abs=0.0)
    assert res["obj_seq_mean"] == pytest.approx(want_surr, rel=1e-14, abs=0.0)


def test_on_policy_tokens_give_the_advantage_exactly():
    b = _small(seed=4)
    old = np.where(np.isnan(b["logp_buf"]), b["logp_roll"], b["logp_buf"])
    res = _run(b, logp_cur=old, mask=None)
    A_tok = np.repeat(b["adv"].astype(np.float64), np.diff(b["cu_seqlens"]))
    np.testing.assert_array_equal(res["surr"], A_tok)
    np.testing.assert_array_equal(res["grad"], A_tok)


def test_consistent_with_the_ratio_function():
    b = _small(seed=5, eps_high=0.28)
    res = _run(b)
    ir = O.is_ratio(b["logp_cur"], b["logp_buf"], b["logp_roll"], b["cu_seqlens"], b["split"], b["mask"],
                    b["eps_low"], b["eps_high"])
    A_tok = np.repeat(b["adv"].astype(np.float64), np.diff(b["cu_seqlens"]))
    np.testing.assert_array_equal(res["surr"], np.minimum(ir["ratio"] * A_tok, ir["ratio_clipped"] * A_tok))
    np.testing.assert_array_equal(res["seq_cnt"], ir["seq_cnt"])
    # the surrogate is a lower bound of both terms
    assert (res["surr"] <= ir["ratio"] * A_tok).all() and (res["surr"] <= ir["ratio_clipped"] * A_tok).all()


def test_gradient_matches_central_differences_of_the_token_mean_objective():
    b = _small(seed=6, B=4, hi=12, sigma=0.4, eps_high=0.28)
    b["adv"] = np.array([1.3, -0.7, 0.0, 2.1], dtype=np.float32)[: b["B"]]
    cur = b["logp_cur"].astype(np.float64)
    res = _run(b, logp_cur=cur)
    total = int(res["seq_cnt"].sum())
    old = np.where(np.isnan(b["logp_buf"]), b["logp_roll"], b["logp_buf"]).astype(np.float64)
    r = np.exp(cur - old)
    h = 1e-6
    checked = 0
    for j in np.flatnonzero(b["mask"] != 0):
        if min(abs(r[j] - 0.8), abs(r[j] - 1.28)) < 1e-3:
            continue      # at a kink the one-sided derivatives differ
        up, dn = cur.copy(), cur.copy()
        up[j] += h; dn[j] -= h
        fd = (_run(b, logp_cur=up)["obj_token_mean"] - _run(b, logp_cur=dn)["obj_token_mean"]) / (2 * h)
        assert fd == pytest.approx(res["grad"][j] / total, rel=1e-6, abs=1e-9)
        checked += 1
    assert checked > 10
    # masked tokens have no influence at all
    for j in np.flatnonzero(b["mask"] == 0)[:3]:
        up = cur.copy(); up[j] = 5.0
        assert _run(b, logp_cur=up)["obj_token_mean"] == res["obj_token_mean"]


def test_positive_homogeneity_in_the_advantage():
    b = _small(seed=7, eps_high=0.28)
    res1 = _run(b)
    res4 = _run(b, adv=b["adv"] * np.float32(4.0))
    np.testing.assert_allclose(res4["surr"], 4.0 * res1["surr"], rtol=1e-15)
    np.testing.assert_allclose(res4["grad"], 4.0 * res1["grad"], rtol=1e-15)
    assert res4["obj_seq_mean"] == pytest.approx(4.0 * res1["obj_seq_mean"], rel=1e-13)


def test_the_two_aggregations():
    # two sequences, lengths 1 and 3, everything on-policy: surr = adv per token
    f = lambda *x: np.array(x, dtype=np.float64)
    res = O.grpo_surrogate(f(-1, -2, -3, -4), f(-1, -2, -3, -4), f(0, 0, 0, 0), np.array([0, 1, 4]),
                           np.array([1, 3]), None, f(6.0, -2.0), 0.2, 0.28)
    assert res["obj_token_mean"] == pytest.approx((6.0 - 2.0 * 3) / 4)     # Table 4: token mean
    assert res["obj_seq_mean"] == pytest.approx((6.0 + -2.0) / 2)          # Eq. 2: mean of sequence means
    # equal lengths: the two agree
    b = _small(seed=8, B=5, lo=9, hi=9, mask_zero_frac=0.0)
    r = _run(b)
    assert r["obj_token_mean"] == pytest.approx(r["obj_seq_mean"], rel=1e-13)
    # an empty sequence adds nothing to the sums but counts in Eq. 2's 1/G
    res2 = O.grpo_surrogate(f(-1, -2, -3, -4), f(-1, -2, -3, -4), f(0, 0, 0, 0), np.array([0, 1, 1, 4]),
                            np.array([1, 0, 3]), None, f(6.0, 9.0, -2.0), 0.2, 0.28)
    assert res2["obj_token_mean"] == pytest.approx(res["obj_token_mean"])
    assert res2["obj_seq_mean"] == pytest.approx((6.0 + 0.0 - 2.0) / 3)


def test_stage_resegmentation_and_unread_sides():
    # Eq. 6: only the number of buffered tokens matters, and the unselected side is never read
    b = _small(seed=9, eps_high=0.28)
    res = _run(b)
    old = np.where(np.isnan(b["logp_buf"]), b["logp_roll"], b["logp_buf"])
    lens = np.diff(b["cu_seqlens"])
    res_all_buf = _run(b, logp_buf=old, logp_roll=np.full_like(old, np.nan), split=lens.astype(np.int32))
    res_all_roll = _run(b, logp_roll=old, logp_buf=np.full_like(old, np.nan), split=np.zeros_like(b["split"]))
    for k in ("surr", "grad", "seq_surr"):
        np.testing.assert_array_equal(res[k], res_all_buf[k])
        np.testing.assert_array_equal(res[k], res_all_roll[k])
    assert np.isfinite(res["surr"]).all() and np.isfinite(res["grad"]).all()


def test_overflowing_ratio():
    # r = +inf: a positive advantage is capped at (1+eps_high) A, a negative one is unbounded below
    assert _one_token(1000.0, 2.0)["surr"][0] == pytest.approx(1.28 * 2.0)
    assert _one_token(1000.0, 2.0)["grad"][0] == 0.0
    assert _one_token(1000.0, -2.0)["surr"][0] == -np.inf
