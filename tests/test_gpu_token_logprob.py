"""GPU parity: copris_lmhead_token_logprob through the C ABI vs the fp64 oracle."""
import math

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


def _case(seed, M, H, V, dtype, w_std=0.05):
    c = W.make_small_lmhead_case(seed, M, H, V, dtype, w_std=w_std)
    rng = np.random.default_rng(seed + 1)
    tok = rng.integers(0, V, size=M).astype(np.int32)
    # the ends of the vocabulary and of the tiles
    for i, t in enumerate([0, V - 1, min(V - 1, 127), min(V - 1, 128), (V - 1) // 128 * 128, V // 2]):
        if i < M:
            tok[i] = t
    return c["hidden"], c["weight"], tok


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
@pytest.mark.parametrize("M,H,V", [(1, 64, 50), (17, 512, 4099), (256, 128, 2500), (300, 512, 3001),
                                   (1000, 256, 9000),     # four row blocks share the persistent grid
                                   (1300, 256, 9001),     # the 256 x 256 kernel: six row blocks, ragged tails
                                   (2049, 128, 700),      # ... fewer tiles than workgroups, one-row last block
                                   (129, 192, 70000),     # more tiles than workgroups per row block
                                   (40, 3584, 777), (5, 72, 260)])
def test_small_shapes(R, dtype, M, H, V):
    h, w, tok = _case(M * 3 + V, M, H, V, dtype)
    lp, lse = R.run_token_logprob(h, w, tok, 1.0, dtype)
    P.check_token_logprob(lp, lse, P.oracle_token_logprob(h, w, tok, 1.0, dtype), f"{dtype} {M}x{H}x{V}")


def test_temperature(R):
    h, w, tok = _case(5, 48, 256, 3000, W.BF16, w_std=0.1)
    lp, lse = R.run_token_logprob(h, w, tok, 0.6, W.BF16)
    P.check_token_logprob(lp, lse, P.oracle_token_logprob(h, w, tok, 0.6, W.BF16), "T=0.6")


def test_zero_weights_and_tokens_outside_the_vocabulary(R):
    M, H, V = 12, 64, 5000
    h, w, tok = _case(6, M, H, V, W.BF16)
    tok[7], tok[8] = -1, V
    lp, lse = R.run_token_logprob(h, np.zeros_like(w), tok, 1.0, W.BF16)
    ok = np.ones(M, bool); ok[[7, 8]] = False
    np.testing.assert_allclose(lp[ok], -math.log(V), atol=1e-5)
    np.testing.assert_allclose(lse, math.log(V), atol=1e-5)
    assert np.isnan(lp[7]) and np.isnan(lp[8])


def test_on_policy_recompute_matches_the_rollout_log_prob(R):
    # the log-prob stored at rollout time and the one recomputed under the same weights for
    # the sampled token agree far below the ratio tolerance: r of Eq. 8 is 1 on-policy
    inp = W.make_small_lmhead_case(8, 200, 512, 20000, W.BF16, w_std=0.05)
    tok, lp, lse = R.run_lmhead_logprob(inp, W.BF16)
    lp2, lse2 = R.run_token_logprob(inp["hidden"], inp["weight"], tok, 1.0, W.BF16)
    np.testing.assert_allclose(lp2, lp, atol=2e-5)
    np.testing.assert_allclose(lse2, lse, atol=2e-5)


def test_micro_batch_at_the_7b_shape_on_sampled_rows(R):
    cfg = W.DECODE_CONFIGS[2]
    b = W.make_token_logprob_inputs(cfg, 8192)
    lp, lse = R.run_token_logprob(b["hidden"], b["weight"], b["tokens"], 1.0, cfg.dtype)
    assert np.isfinite(lp).all() and np.isfinite(lse).all()
    rows = np.random.default_rng(1).choice(8192, size=24, replace=False)
    rows[:4] = [0, 255, 256, 8191]
    ref = P.oracle_token_logprob(b["hidden"], b["weight"], b["tokens"], 1.0, cfg.dtype, rows=rows)
    P.check_token_logprob(lp[rows], lse[rows], ref, "7B-shaped micro-batch")
    # every row: lse is near ln V + var/2 for these weights, log-probs are negative
    assert (lp < 0).all() and np.abs(lse - lse.mean()).max() < 1.0
