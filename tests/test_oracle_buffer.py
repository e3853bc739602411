"""Pins for the oracle's buffer of partial trajectories (Section 4, "Buffering of Partial
Trajectories", Eq. 6), the per-step KV append and the pool-state commands."""
import numpy as np

from oracle import copris_oracle as O


def test_concatenation_of_a_hand_worked_buffer():
    # trajectory 3: two tokens in stage 0, one in stage 2; trajectory 5: one token in stage 2
    buf = {}
    O.buffer_append(buf, 3, 0, 11, -0.5)
    O.buffer_append(buf, 3, 0, 12, -1.5)
    O.buffer_append(buf, 5, 2, 21, -0.25)
    O.buffer_append(buf, 3, 2, 13, -2.5)
    assert buf[3] == [(0, [11, 12], [-0.5, -1.5]), (2, [13], [-2.5])]
    b = O.buffer_concat(buf, [5, 3], stage=2)
    assert b["cu_seqlens"].tolist() == [0, 1, 4] and b["tokens"].tolist() == [21, 11, 12, 13]
    assert b["split"].tolist() == [0, 2]
    np.testing.assert_array_equal(b["logp_buf"], [np.nan, -0.5, -1.5, np.nan])
    np.testing.assert_array_equal(b["logp_roll"], [-0.25, np.nan, np.nan, -2.5])
    # consumed one stage later: everything is an earlier piece
    b3 = O.buffer_concat(buf, [3], stage=3)
    assert b3["split"].tolist() == [3] and np.isnan(b3["logp_roll"]).all()
    np.testing.assert_array_equal(b3["logp_buf"], [-0.5, -1.5, -2.5])
    # a trajectory the buffer does not know is empty
    assert O.buffer_concat(buf, [9], stage=1)["cu_seqlens"].tolist() == [0, 0]


def test_concatenation_is_the_flat_vector_whatever_the_number_of_stages():
    # Eq. 6: L_i is one vector along the token axis; cutting the same tokens into more or
    # fewer stages changes only where the split falls
    rng = np.random.default_rng(0)
    lp = -rng.exponential(size=40)
    tok = rng.integers(0, 1000, size=40)
    for cuts in ([40], [7, 33], [7, 1, 20, 12], [1] * 40):
        buf, t = {}, 0
        for st, n in enumerate(cuts):
            for _ in range(n):
                O.buffer_append(buf, 0, st, tok[t], lp[t])
                t += 1
        last = len(cuts) - 1
        b = O.buffer_concat(buf, [0], stage=last)
        flat = np.where(np.isnan(b["logp_buf"]), b["logp_roll"], b["logp_buf"])
        np.testing.assert_array_equal(flat, lp)
        np.testing.assert_array_equal(b["tokens"], tok)
        assert b["split"][0] == 40 - cuts[-1]
        # exactly one side is populated at every token, the earlier pieces are a prefix
        assert (np.isnan(b["logp_buf"]) != np.isnan(b["logp_roll"])).all()
        assert not np.isnan(b["logp_buf"][:b["split"][0]]).any()
        # and the ratio of Eq. 8 does not see the segmentation
        cur = lp + rng.normal(0, 0.05, size=40)
        r = O.is_ratio(cur, b["logp_buf"], b["logp_roll"], b["cu_seqlens"], b["split"], None, 0.2, 0.28)
        np.testing.assert_allclose(r["ratio"], np.exp(cur - lp), rtol=1e-15)


def test_appending_token_by_token_is_the_page_fill():
    # growing every request one position at a time leaves the caches exactly as filling the
    # pages from the packed sequences does (kv_page_fill is pinned on its own)
    rng = np.random.default_rng(1)
    lens = [1, 16, 17, 40]
    P, Hkv, D = 16, 2, 8
    cu = np.concatenate([[0], np.cumsum(lens)])
    k, v = rng.normal(size=(cu[-1], Hkv, D)), rng.normal(size=(cu[-1], Hkv, D))
    n_pages = sum((n + P - 1) // P for n in lens) + 3
    perm = rng.permutation(n_pages)
    bt = np.full((len(lens), 3), -1)
    nxt = 0
    for b, n in enumerate(lens):
        for j in range((n + P - 1) // P):
            bt[b, j] = perm[nxt]
            nxt += 1
    ref_k, ref_v = np.full((n_pages, Hkv, P, D), np.nan), np.full((n_pages, Hkv, P, D), np.nan)
    O.kv_page_fill(k, v, cu, bt, ref_k, ref_v)
    got_k, got_v = np.full_like(ref_k, np.nan), np.full_like(ref_v, np.nan)
    for t in range(max(lens)):
        ctx = np.asarray([t + 1 if t < n else 0 for n in lens])      # finished requests hold nothing
        rows = np.asarray([cu[b] + min(t, n - 1) for b, n in enumerate(lens)])
        O.kv_append(k[rows], v[rows], bt, ctx, got_k, got_v)
    np.testing.assert_array_equal(got_k, ref_k)
    np.testing.assert_array_equal(got_v, ref_v)


def test_pool_commands():
    seq_id, ctx, step = np.full(3, -1), np.zeros(3, int), np.zeros(3, int)
    bt = np.zeros((3, 2), int)
    cmds = [2, 7, 33, 4, 0, -1, 0, 0] + [2, 0, 9, 2, 1, 5]
    O.pool_commands_apply(cmds, 2, 2, seq_id, ctx, step, bt)
    assert seq_id.tolist() == [-1, -1, 7] and ctx.tolist() == [0, 0, 33] and step.tolist() == [0, 0, 4]
    assert bt.tolist() == [[0, 0], [0, 0], [9, 5]]
