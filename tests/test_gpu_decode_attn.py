"""GPU parity: copris_decode_attn through the C ABI vs the fp64 oracle."""
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


def _run_case(R, case, dtype, what):
    out, lse = R.run_decode_attn(case, dtype)
    ref_out, ref_lse = P.oracle_attn(case, dtype)
    return P.check_attn(out, lse, ref_out, ref_lse, dtype, what)


def test_tiny_config_fp32(R):
    cfg = W.DECODE_CONFIGS[0]
    inp = W.make_decode_inputs(cfg, with_lmhead=False)
    _run_case(R, inp, cfg.dtype, "cfg0")


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
@pytest.mark.parametrize("Hq,Hkv,D", [(4, 2, 64), (7, 1, 128), (12, 2, 128), (28, 4, 128), (8, 8, 128), (16, 1, 128)])
def test_small_shapes_ragged_lengths(R, dtype, Hq, Hkv, D):
    # one token, page multiple -1/0/+1, a chunk boundary -1/0/+1, several chunks with a ragged tail
    ctx = [1, 15, 16, 17, 33, 511, 512, 513, 1024, 1500, 2049, 100]
    case = W.make_small_decode_case(100 + Hq + D, len(ctx), Hq, Hkv, D, dtype, 16, ctx)
    _run_case(R, case, dtype, f"{dtype} {Hq}/{Hkv}/{D}")


def test_zero_length_and_wide_block_table(R):
    ctx = [0, 40, 0, 700]
    case = W.make_small_decode_case(5, 4, 12, 2, 128, W.BF16, 16, ctx, max_pages=64)
    out, lse = R.run_decode_attn(case, W.BF16)
    ref_out, ref_lse = P.oracle_attn(case, W.BF16)
    P.check_attn(out, lse, ref_out, ref_lse, W.BF16, "zero-length")
    assert (out[0] == 0).all() and (out[2] == 0).all()


def test_generic_path_other_page_size(R):
    ctx = [3, 64, 65, 700]
    case = W.make_small_decode_case(6, 4, 6, 2, 64, W.BF16, 8, ctx)
    _run_case(R, case, W.BF16, "page8")


def test_page_permutation_is_bitwise_invariant_and_runs_are_reproducible(R):
    ctx = [1000, 37, 1536, 513]
    case = W.make_small_decode_case(7, 4, 28, 4, 128, W.BF16, 16, ctx)
    out1, lse1 = R.run_decode_attn(case, W.BF16)
    out1b, lse1b = R.run_decode_attn(case, W.BF16)
    np.testing.assert_array_equal(out1, out1b)
    np.testing.assert_array_equal(lse1, lse1b)
    perm = np.random.default_rng(1).permutation(case["num_pages"])
    c2 = dict(case)
    for k in ("k_cache", "v_cache"):
        moved = np.empty_like(case[k])
        moved[perm] = case[k]
        c2[k] = moved
    bt = case["block_table"]
    c2["block_table"] = np.where(bt >= 0, perm[np.maximum(bt, 0)], -1).astype(np.int32)
    out2, lse2 = R.run_decode_attn(c2, W.BF16)
    np.testing.assert_array_equal(out1, out2)
    np.testing.assert_array_equal(lse1, lse2)


def test_batch_order_equivariance_and_chunking_independence(R):
    # permuting the batch rows permutes the outputs; the split along the context depends on
    # the position in the batch, so equality is to rounding, not bitwise
    ctx = [1000, 37, 1536, 513, 16, 2500, 800, 64]
    case = W.make_small_decode_case(21, len(ctx), 28, 4, 128, W.BF16, 16, ctx)
    out1, lse1 = R.run_decode_attn(case, W.BF16)
    perm = np.random.default_rng(2).permutation(len(ctx))
    c2 = dict(case)
    for k in ("q", "block_table", "ctx_len"):
        c2[k] = case[k][perm]
    out2, lse2 = R.run_decode_attn(c2, W.BF16)
    assert np.abs(out1[perm] - out2).max() <= 2 ** -6          # one bf16 ulp at |x| < 4
    np.testing.assert_allclose(lse1[perm], lse2, atol=1e-5)


def test_single_head_group_and_many_short_sequences(R):
    # g = 1 (no grouping) and more sequences than pages per share
    rng = np.random.default_rng(3)
    ctx = rng.integers(1, 40, size=300).tolist()
    case = W.make_small_decode_case(22, len(ctx), 4, 4, 128, W.BF16, 16, ctx)
    _run_case(R, case, W.BF16, "g=1 short")


def test_thousands_of_sequences(R):
    # more sequences than a wavefront derives its own cursor for: a scan kernel prepares them;
    # with contexts of a page or two nearly every segment lies inside one share, and some shares
    # hold dozens of whole segments
    rng = np.random.default_rng(4)
    ctx = rng.integers(0, 34, size=4500).tolist()
    case = W.make_small_decode_case(23, len(ctx), 6, 2, 128, W.BF16, 16, ctx)
    _run_case(R, case, W.BF16, "4500 sequences")


def test_large_scores_do_not_overflow(R):
    case = W.make_small_decode_case(8, 2, 7, 1, 128, W.BF16, 16, [600, 31], poison=True)
    q = W.to_f32(case["q"], W.BF16) * 40.0           # scores of magnitude ~ 10^2..10^3 * scale
    case["q"] = W.to_storage(q, W.BF16)
    _run_case(R, case, W.BF16, "large scores")


def _sampled_subproblem(inp, cfg, seqs):
    """The same sequences with their pages gathered into a compact pool (so that the
    oracle does not widen the whole multi-GB cache)."""
    P_ = cfg.page_size
    npg = (inp["ctx_len"][seqs].astype(np.int64) + P_ - 1) // P_
    pages = np.concatenate([inp["block_table"][s, :n] for s, n in zip(seqs, npg)])
    bt = np.full((len(seqs), int(npg.max())), -1, dtype=np.int32)
    off = 0
    for i, n in enumerate(npg):
        bt[i, :n] = np.arange(off, off + n)
        off += n
    return {"q": inp["q"][seqs], "k_cache": inp["k_cache"][pages], "v_cache": inp["v_cache"][pages],
            "block_table": bt, "ctx_len": inp["ctx_len"][seqs], "scale": inp["scale"]}


def _check_sequences(inp, cfg, out, lse, seqs, what, chunk=32):
    """Oracle comparison of the given sequences, a chunk at a time (bounds the fp64 copies)."""
    worst = 0.0
    for i in range(0, len(seqs), chunk):
        part = np.asarray(seqs[i:i + chunk])
        sub = _sampled_subproblem(inp, cfg, part)
        ref_out, ref_lse = P.oracle_attn(sub, cfg.dtype)
        worst = max(worst, P.check_attn(out[part], lse[part], ref_out, ref_lse, cfg.dtype, f"{what} seqs {i}.."))
    return worst


@pytest.mark.parametrize("k", [1, 2])
def test_full_size_configs_every_sequence(R, k):
    # the 1.5B- and 7B-shaped steps, in the launch configuration the benchmark times:
    # every one of the C sequences against the oracle
    cfg = W.DECODE_CONFIGS[k]
    inp = W.make_decode_inputs(cfg, with_lmhead=False)
    out, lse = R.run_decode_attn(inp, cfg.dtype)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    _check_sequences(inp, cfg, out, lse, np.arange(cfg.C), f"cfg{k}")


def test_long_tail_config_every_resumed_trajectory(R):
    # C = 512: all ten 32768-token sequences, the shortest, and sixteen others
    cfg = W.DECODE_CONFIGS[3]
    inp = W.make_decode_inputs(cfg, with_lmhead=False)
    out, lse = R.run_decode_attn(inp, cfg.dtype)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    ctx = inp["ctx_len"]
    longest = np.flatnonzero(ctx == ctx.max())
    assert len(longest) == 10 and ctx.max() == 32768
    rest = np.setdiff1d(np.arange(cfg.C), longest)
    others = np.random.default_rng(3).choice(rest, 16, replace=False)
    seqs = np.unique(np.concatenate([longest, np.argsort(ctx)[:2], others]))
    _check_sequences(inp, cfg, out, lse, seqs, "cfg3", chunk=8)
