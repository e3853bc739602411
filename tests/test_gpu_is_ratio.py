"""GPU parity: copris_is_ratio through the C ABI vs the fp64 oracle."""
import numpy as np
import pytest

from paper_2511_05589_amd import workloads as W
from tests import parity as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def R():
    from paper_2511_05589_amd import runner
    runner.require_gpu()
    return runner


def _cfg(B, lo, hi, sigma=0.05, layout="packed", pad_to=0, zf=0.1, eps_high=0.2):
    return W.ISConfig(77, "t", B=B, layout=layout, len_lo=lo, len_hi=hi, pad_to=pad_to, sigma=sigma,
                      mask_zero_frac=zf, eps_high=eps_high)


def test_tiny_padded_config(R):
    b = W.make_is_inputs(W.IS_CONFIGS[0])
    P.check_is(R.run_is_ratio(b), P.oracle_is(b), b, what="cfg0")


def test_cross_stage_batch_full_size(R):
    b = W.make_is_inputs(W.IS_CONFIGS[4])
    got = R.run_is_ratio(b)
    P.check_is(got, P.oracle_is(b), b, what="cfg4")
    assert got["seq_nclip"].sum() > 50          # the clip branch did fire at sigma = 0.05


@pytest.mark.parametrize("seed", range(6))
def test_ragged_small_batches(R, seed):
    rng = np.random.default_rng(seed)
    # lengths around the vector width and the workgroup stride, odd offsets, heavy clipping
    cfg = _cfg(B=int(rng.integers(1, 40)), lo=1, hi=int(rng.choice([7, 130, 4100, 9000])), sigma=0.3)
    b = W.make_is_inputs(cfg, rng=rng)
    P.check_is(R.run_is_ratio(b), P.oracle_is(b), b, what=f"seed{seed}")


def test_no_mask_and_asymmetric_clip(R):
    b = W.make_is_inputs(_cfg(B=9, lo=1, hi=3000, sigma=0.3, zf=0.0, eps_high=0.28),
                         rng=np.random.default_rng(11))
    got = R.run_is_ratio(b, use_mask=False)
    P.check_is(got, P.oracle_is(b, use_mask=False), b, use_mask=False, what="nomask")
    assert np.isclose(got["ratio_clipped"].max(), 1.28) and np.isclose(got["ratio_clipped"].min(), 0.8)


def test_equal_logprobs_give_exactly_one(R):
    b = W.make_is_inputs(_cfg(B=5, lo=1, hi=700, zf=0.0), rng=np.random.default_rng(3), poison=False)
    b["logp_buf"] = b["logp_roll"] = b["logp_cur"]
    got = R.run_is_ratio(b)
    assert (got["ratio"] == 1.0).all() and (got["ratio_clipped"] == 1.0).all()
    assert (got["seq_nclip"] == 0).all()
    np.testing.assert_array_equal(got["seq_sum"], got["seq_cnt"].astype(np.float32))


def test_split_extremes_empty_sequences_and_overflow(R):
    n = 37
    rng = np.random.default_rng(5)
    base = -rng.exponential(1.0, 3 * n).astype(np.float32)
    cur = (base + rng.normal(0, 0.3, 3 * n)).astype(np.float32)
    cur[5], base[5] = 0.0, -800.0          # exp overflows to +inf, clipped to 1+eps
    nan = np.float32(np.nan)
    lens = np.array([n, 0, n, 0, n])
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    split = np.array([0, 0, n, 0, 11], dtype=np.int32)     # fresh, empty, all buffered, empty, mixed
    local = np.arange(3 * n) - np.repeat(cu[:-1], lens)
    is_buf = local < np.repeat(split, lens)
    b = {"B": 5, "N": 3 * n, "cu_seqlens": cu, "split": split, "mask": None, "logp_cur": cur,
         "logp_buf": np.where(is_buf, base, nan), "logp_roll": np.where(is_buf, nan, base),
         "eps_low": 0.2, "eps_high": 0.2}
    got = R.run_is_ratio(b, use_mask=False)
    P.check_is(got, P.oracle_is(b, use_mask=False), b, use_mask=False, what="extremes")
    assert np.isinf(got["ratio"][5]) and np.isclose(got["ratio_clipped"][5], 1.2)
    assert list(got["seq_cnt"]) == [n, 0, n, 0, n] and got["seq_sum"][1] == 0.0


def test_bitwise_reproducible(R):
    b = W.make_is_inputs(_cfg(B=33, lo=1, hi=6000, sigma=0.3), rng=np.random.default_rng(9))
    a, c = R.run_is_ratio(b), R.run_is_ratio(b)
    for k in a:
        np.testing.assert_array_equal(a[k], c[k])
