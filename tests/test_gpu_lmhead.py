"""GPU parity: copris_lmhead_logprob through the C ABI vs the fp64 oracle."""
import math

import numpy as np
import pytest

from oracle import copris_oracle as O
from paper_2511_05589_amd import workloads as W
from tests import parity as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def R():
    from paper_2511_05589_amd import runner
    runner.require_gpu()
    return runner


def test_tiny_config_fp32(R):
    cfg = W.DECODE_CONFIGS[0]
    inp = W.make_decode_inputs(cfg, with_attn=False)
    tok, lp, lse = R.run_lmhead_logprob(inp, cfg.dtype)
    P.check_lmhead(tok, lp, lse, P.oracle_lmhead(inp, cfg.dtype), "cfg0")


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
@pytest.mark.parametrize("C,H,V", [(1, 64, 50), (3, 256, 1000), (17, 512, 4099), (64, 1536, 9000),
                                   (256, 128, 2500), (33, 3584, 777),
                                   (300, 512, 3001),      # two batch blocks, ragged vocabulary tail
                                   (129, 192, 70000),     # more tiles than persistent workgroups
                                   (5, 72, 260)])         # hidden size the matrix-core kernel does not take
def test_small_shapes(R, dtype, C, H, V):
    inp = W.make_small_lmhead_case(C * 7 + V, C, H, V, dtype, w_std=0.05)
    tok, lp, lse = R.run_lmhead_logprob(inp, dtype)
    n_exempt = P.check_lmhead(tok, lp, lse, P.oracle_lmhead(inp, dtype), f"{dtype} {C}x{H}x{V}")
    assert n_exempt <= 2          # expected near-ties: about C / 1000


def test_zero_weights_token_is_argmax_of_the_noise(R):
    # isolates the Philox counter layout and the uniform -> Gumbel mapping
    C, H, V = 16, 64, 5000
    inp = W.make_small_lmhead_case(1, C, H, V, W.F32)
    inp["weight"] = np.zeros_like(inp["weight"])
    inp["seq_id"][3] = (7 << 32) | 5             # exercise the high counter word
    inp["step"][4] = 70000
    tok, lp, lse = R.run_lmhead_logprob(inp, W.F32)
    for c in range(C):
        g = O.gumbel_noise(inp["seed"], int(inp["seq_id"][c]), int(inp["step"][c]), V)
        order = np.argsort(-g)
        assert tok[c] == order[0] or (g[order[0]] - g[order[1]] < P.NEAR_TIE and tok[c] == order[1])
    np.testing.assert_allclose(lp, -math.log(V), atol=1e-5)


def test_temperature_and_row_permutation(R):
    inp = W.make_small_lmhead_case(9, 24, 256, 3000, W.BF16, w_std=0.1)
    inp["temperature"] = 0.6
    tok, lp, lse = R.run_lmhead_logprob(inp, W.BF16)
    P.check_lmhead(tok, lp, lse, P.oracle_lmhead(inp, W.BF16), "T=0.6")
    perm = np.random.default_rng(0).permutation(24)
    inp2 = dict(inp)
    for k in ("hidden", "seq_id", "step"):
        inp2[k] = inp[k][perm]
    tok2, lp2, lse2 = R.run_lmhead_logprob(inp2, W.BF16)
    np.testing.assert_array_equal(tok[perm], tok2)
    np.testing.assert_array_equal(lp[perm], lp2)


def test_bitwise_reproducible(R):
    inp = W.make_small_lmhead_case(10, 40, 512, 7000, W.BF16)
    a, b = R.run_lmhead_logprob(inp, W.BF16), R.run_lmhead_logprob(inp, W.BF16)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)


@pytest.mark.parametrize("k", [1, 2])
def test_full_size_configs_every_row(R, k):
    # the 1.5B- and 7B-shaped LM heads (vocabulary 151936): every one of the C rows
    cfg = W.DECODE_CONFIGS[k]
    inp = W.make_decode_inputs(cfg, with_attn=False)
    tok, lp, lse = R.run_lmhead_logprob(inp, cfg.dtype)
    assert ((0 <= tok) & (tok < cfg.V)).all() and np.isfinite(lp).all() and (lp <= 0).all()
    exempt = 0
    for r0 in range(0, cfg.C, 64):            # 64 rows of full log-softmax at a time (78 MB in fp64)
        rows = np.arange(r0, min(r0 + 64, cfg.C))
        ref = P.oracle_lmhead(inp, cfg.dtype, rows=rows)
        exempt += P.check_lmhead(tok[rows], lp[rows], lse[rows], ref, f"cfg{k} rows {r0}..")
    assert exempt <= 2
