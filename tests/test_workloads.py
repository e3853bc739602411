"""The seeded input generators: determinism, shapes, length distributions and the
storage-dtype rounding (pinned against torch's bfloat16 cast)."""
import numpy as np
import torch

from paper_2511_05589_amd import workloads as W


def test_bf16_rounding_is_nearest_even_like_the_library_cast():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40],
                                 dtype=np.float32)])
    bits = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, ref)
    back = W.bf16_bits_to_f32(bits)
    np.testing.assert_array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_generators_are_deterministic():
    a = W.make_decode_inputs(W.DECODE_CONFIGS[0])
    b = W.make_decode_inputs(W.DECODE_CONFIGS[0])
    for k in ("ctx_len", "block_table", "q", "k_cache", "v_cache", "hidden", "weight", "seq_id", "step"):
        np.testing.assert_array_equal(a[k], b[k])
    x, y = W.make_is_inputs(W.IS_CONFIGS[0]), W.make_is_inputs(W.IS_CONFIGS[0])
    for k in ("cu_seqlens", "split", "mask", "logp_cur", "logp_buf", "logp_roll"):
        np.testing.assert_array_equal(x[k], y[k])


def test_context_length_recipes():
    for k, (lo, hi, mean_lo, mean_hi) in {0: (33, 544, 120, 400), 1: (257, 8448, 1300, 2800),
                                           2: (513, 16896, 3000, 4300)}.items():
        cfg = W.DECODE_CONFIGS[k]
        ctx = W.make_ctx_len(cfg)
        assert ctx.shape == (cfg.C,) and ctx.min() >= lo and ctx.max() <= hi
        assert mean_lo < ctx.mean() < mean_hi, (k, ctx.mean())
    ctx = W.make_ctx_len(W.DECODE_CONFIGS[3])
    assert ctx.shape == (512,)
    assert (ctx == 32768).sum() == 10
    assert ((ctx >= 2048) & (ctx <= 16384)).sum() >= 41
    assert (ctx <= 2048).sum() >= 461 - 1 and ctx.min() >= 256
    # shuffled over slots: the long ones are not all at the end
    assert np.flatnonzero(ctx == 32768).min() < 400


def test_page_tables_are_a_partial_permutation_and_poison_covers_unused_slots():
    cfg = W.DECODE_CONFIGS[0]
    inp = W.make_decode_inputs(cfg)
    bt, ctx, P = inp["block_table"], inp["ctx_len"], cfg.page_size
    used = bt[bt >= 0]
    assert used.size == ((ctx + P - 1) // P).sum() == np.unique(used).size
    assert used.max() < inp["num_pages"]
    K = W.to_f32(inp["k_cache"], cfg.dtype)
    ref = np.zeros(inp["num_pages"], dtype=bool); ref[used] = True
    assert np.isnan(K[~ref]).all()
    for i in range(cfg.C):
        n = int(ctx[i]); npg = (n + P - 1) // P
        assert np.isfinite(K[bt[i, :npg - 1]]).all()
        last = K[bt[i, npg - 1]]
        tail = n - (npg - 1) * P
        assert np.isfinite(last[:, :tail]).all() and np.isnan(last[:, tail:]).all()
    # physical pages of a sequence are not contiguous (shuffled)
    assert (np.diff(bt[0, :(ctx[0] + P - 1) // P]) != 1).any()


def test_lmhead_inputs_scale():
    cfg = W.DECODE_CONFIGS[0]
    inp = W.make_decode_inputs(cfg, with_attn=False)
    w = W.to_f32(inp["weight"], cfg.dtype)
    assert w.shape == (cfg.V, cfg.H) and abs(w.std() - 0.02) < 1e-3
    assert np.unique(inp["seq_id"]).size == cfg.C
    assert (inp["step"] == inp["ctx_len"] - cfg.prompt).all()
