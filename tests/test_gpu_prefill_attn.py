"""GPU parity: copris_prefill_attn through the C ABI vs the fp64 oracle."""
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


def _check_all(R, b, what):
    out, lse, kc, vc = R.run_prefill_attn(b, W.BF16)
    ref_out, ref_lse, ref_kc, ref_vc = P.oracle_prefill(b, W.BF16)
    P.check_attn(out, lse, ref_out, ref_lse, W.BF16, what)
    # the page fill is data movement: bit-exact, and slots without a token stay untouched
    np.testing.assert_array_equal(kc, ref_kc)
    np.testing.assert_array_equal(vc, ref_vc)


@pytest.mark.parametrize("Hq,Hkv", [(28, 4), (12, 2), (4, 4), (8, 4), (16, 4), (8, 1), (6, 2), (5, 1)])
def test_ragged_lengths_every_group_size(R, Hq, Hkv):
    # lengths around the page, the query-block and the tile boundaries
    lens = [1, 15, 16, 17, 31, 32, 33, 47, 48, 49, 64, 100, 257]
    b = W.make_prefill_case(Hq * 10 + Hkv, lens, Hq, Hkv, 128, W.BF16)
    _check_all(R, b, f"{Hq}/{Hkv}")


@pytest.mark.parametrize("Hq,Hkv", [(28, 4), (12, 4), (8, 4)])
def test_empty_sequences_among_others_and_a_loose_length_bound(R, Hq, Hkv):
    # sequences of length 0 own no tile and no page; max_seqlen may exceed every length (the
    # grid is then larger than needed and the surplus workgroups leave at once)
    lens = [0, 33, 0, 0, 130, 1, 0]
    b = W.make_prefill_case(Hq + 3, lens, Hq, Hkv, 128, W.BF16)
    d = R.stage_prefill_attn(b, W.BF16)
    d.max_seqlen = int(d.block_table.shape[1]) * 16          # the loosest bound the call accepts
    d.run()
    import torch
    torch.cuda.synchronize()
    out = R.out_to_f32(d.out)
    ref_out, ref_lse, ref_kc, ref_vc = P.oracle_prefill(b, W.BF16)
    P.check_attn(out, d.lse.cpu().numpy(), ref_out, ref_lse, W.BF16, f"{Hq}/{Hkv} with empties")
    np.testing.assert_array_equal(R.out_to_f32(d.k_cache), ref_kc)
    np.testing.assert_array_equal(R.out_to_f32(d.v_cache), ref_vc)


def test_seeded_random_group_sizes_and_lengths(R):
    # every supported group size against lengths around the page, block, tile and super-tile
    # boundaries, a few sequences per case (the workgroup <-> (head, tile) mapping differs with
    # the group size)
    rng = np.random.default_rng(2024)
    combos = [(28, 4), (12, 2), (4, 4), (8, 4), (16, 4), (8, 1), (6, 2), (5, 1), (3, 1), (7, 1), (14, 2), (2, 2),
              (1, 1), (32, 4), (24, 8)]
    pick = [0, 1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 95, 96, 97, 127, 128, 129, 200, 255, 256, 257, 300, 511]
    for it, (Hq, Hkv) in enumerate(combos):
        lens = [int(x) for x in rng.choice(pick, size=int(rng.integers(1, 7)))]
        if sum(lens) == 0:
            lens[0] = 5
        b = W.make_prefill_case(1000 + it, lens, Hq, Hkv, 128, W.BF16)
        _check_all(R, b, f"{Hq}/{Hkv} lens {lens}")


@pytest.mark.parametrize("gain", [6.0, 20.0])
def test_large_scores_move_the_softmax_reference_often(R, gain):
    # queries scaled up: scores spread over tens of log2 units, so the kernel's softmax
    # reference (kept until a score outgrows it by 2^6) moves on many steps, weights reach
    # their upper bound, and nearly-one-hot rows appear; the oracle knows none of this
    lens = [40, 333, 1030]
    b = dict(W.make_prefill_case(21, lens, 28, 4, 128, W.BF16))
    q = W.bf16_bits_to_f32(b["q"]) * gain
    # an ascending ramp on one query head: every step brings a new maximum
    ramp = np.linspace(0.0, 3.0, q.shape[0], dtype=np.float32)[:, None]
    q[:, 3, :] = ramp * np.sign(W.bf16_bits_to_f32(b["k"])[:, 0, :]).astype(np.float32)
    b["q"] = W.f32_to_bf16_bits(q)
    # nearly one-hot rows return single V rows; with |v| up to 5 half a bf16 ulp of the stored
    # output alone would be 1.6e-2, so the values are scaled to |v| < 1.3 (half an ulp 3.9e-3)
    # and the same absolute bar as everywhere else applies
    b["v"] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(b["v"]) * 0.25)
    out, lse, kc, vc = R.run_prefill_attn(b, W.BF16)
    ref_out, ref_lse, ref_kc, ref_vc = P.oracle_prefill(b, W.BF16)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    err = np.abs(out.astype(np.float64) - ref_out).max()
    assert err <= P.ATTN_TOL[W.BF16], f"gain {gain}: worst {err:.3e}"
    # scores reach several hundred here: fp32 accumulation of a 128-term dot product of that
    # size carries ~1e-7 of it, so the log-sum-exp bound has a relative part
    lerr = np.abs(lse.astype(np.float64) - ref_lse)
    assert (lerr <= P.ATTN_LSE_TOL[W.BF16] + 1e-4 * np.abs(ref_lse)).all(), f"gain {gain}: lse worst {lerr.max():.3e}"
    np.testing.assert_array_equal(kc, ref_kc)
    np.testing.assert_array_equal(vc, ref_vc)


def test_one_longer_sequence_and_many_short(R):
    rng = np.random.default_rng(4)
    lens = [700] + rng.integers(1, 40, size=30).tolist()
    b = W.make_prefill_case(9, lens, 14, 2, 128, W.BF16)
    _check_all(R, b, "700 + short")


def test_causality_on_the_device(R):
    b = W.make_prefill_case(11, [90, 50], 28, 4, 128, W.BF16)
    out1, lse1, _, _ = R.run_prefill_attn(b, W.BF16)
    b2 = dict(b)
    k2, v2 = b["k"].copy(), b["v"].copy()
    k2[60:90] = W.f32_to_bf16_bits(np.full((30, 4, 128), 3.0, np.float32))     # the tail of sequence 0
    v2[60:90] = W.f32_to_bf16_bits(np.full((30, 4, 128), -5.0, np.float32))
    b2["k"], b2["v"] = k2, v2
    out2, lse2, _, _ = R.run_prefill_attn(b2, W.BF16)
    np.testing.assert_array_equal(out2[:60], out1[:60])     # earlier tokens: bitwise unchanged
    np.testing.assert_array_equal(out2[90:], out1[90:])     # the other sequence too
    assert np.abs(out2[60:90] - out1[60:90]).max() > 0.1


def test_decode_continues_from_the_refilled_pages(R):
    # after the re-prefill the decode kernel, given the last token's query and ctx_len = len,
    # reproduces the prefill's last row (same pages, same arithmetic up to the split order)
    import torch
    from paper_2511_05589_amd import binding
    lens = [333, 16, 1, 1200]
    b = W.make_prefill_case(12, lens, 28, 4, 128, W.BF16)
    d = R.stage_prefill_attn(b, W.BF16)
    d.run()
    last = torch.from_numpy((np.asarray(b["cu_seqlens"][1:]) - 1).astype(np.int64)).to(d.q.device)
    qd = d.q[last].contiguous()
    ctx = torch.from_numpy(np.asarray(lens, dtype=np.int32)).to(d.q.device)
    outd = torch.full_like(qd, float("nan"))
    lsed = torch.full((len(lens), 28), float("nan"), dtype=torch.float32, device=d.q.device)
    ws = R.workspace(binding.decode_attn_workspace_bytes(len(lens), 28, 4, 128, 16, d.block_table.shape[1]))
    binding.decode_attn(qd, d.k_cache, d.v_cache, d.block_table, ctx, outd, lsed, ws, scale=d.scale,
                        dtype=d.dtype)
    torch.cuda.synchronize()
    np.testing.assert_allclose(outd.float().cpu().numpy(), d.out[last].float().cpu().numpy(), atol=2 ** -6)
    np.testing.assert_allclose(lsed.cpu().numpy(), d.lse[last].cpu().numpy(), atol=2e-3)


def test_resumed_trajectories_at_the_7b_shape_on_sampled_tokens(R):
    # 12 buffered trajectories with the length recipe of the 7B-shaped config
    cfg = W.DECODE_CONFIGS[2]
    lens = W.make_ctx_len(cfg, np.random.default_rng(5))[:12]
    lens[0] = 16384                                # one at the cap
    b = W.make_prefill_case(13, lens, cfg.Hq, cfg.Hkv, cfg.D, W.BF16)
    out, lse, kc, vc = R.run_prefill_attn(b, W.BF16)
    ref_kc, ref_vc = P.oracle_page_fill(b, W.BF16)
    np.testing.assert_array_equal(kc, ref_kc)
    np.testing.assert_array_equal(vc, ref_vc)
    rng = np.random.default_rng(6)
    seq_tok = [(0, 16383), (0, 0), (0, 8191)]
    for s, n in enumerate(lens):
        seq_tok += [(s, int(t)) for t in rng.integers(0, n, size=3)] + [(s, int(n) - 1)]
    rows, ref_out, ref_lse = P.oracle_prefill_rows(b, W.BF16, seq_tok, ref_kc, ref_vc)
    P.check_attn(out[rows], lse[rows], ref_out, ref_lse, W.BF16, "7B-shaped re-prefill")
    assert np.isfinite(out).all()


def test_unsupported_shapes_are_refused(R):
    from paper_2511_05589_amd import binding
    b = W.make_prefill_case(14, [20], 18, 2, 128, W.BF16)       # group of 9: not compiled
    with pytest.raises(binding.CoprisError) as e:
        R.run_prefill_attn(b, W.BF16)
    assert e.value.code == binding.COPRIS_EUNSUPPORTED
