"""GPU parity, bit for bit: the device side of the rollout loop (pool-state commands, KV
append, buffer append, Eq. 6's concatenation of the buffered pieces) against the oracle."""
import numpy as np
import pytest

from oracle import copris_oracle as O
from paper_2511_05589_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2511_05589_amd import binding, runner
    dev = runner.require_gpu()
    return torch, binding, runner, dev


def test_pool_commands(gpu):
    torch, binding, runner, dev = gpu
    rng = np.random.default_rng(0)
    pool, max_pages = 300, 9
    seq_id, ctx, step = rng.integers(-1, 50, pool), rng.integers(0, 99, pool).astype(np.int32), rng.integers(0, 9, pool).astype(np.int32)
    table = rng.integers(0, 1000, (pool, max_pages)).astype(np.int32)
    slots = rng.permutation(pool)[:270]
    slot_cmds = np.stack([slots, rng.integers(-1, 1 << 20, 270), rng.integers(0, 5000, 270), rng.integers(0, 4000, 270)], 1)
    cells = rng.permutation(pool * max_pages)[:700]
    page_cmds = np.stack([cells // max_pages, cells % max_pages, rng.integers(0, 1 << 20, 700)], 1)
    cmds = np.concatenate([slot_cmds.reshape(-1), page_cmds.reshape(-1)]).astype(np.int32)
    d = [runner.to_device(x, device=dev) for x in (seq_id.astype(np.int64), ctx, step, table)]
    binding.rollout_apply(runner.to_device(cmds, device=dev), 270, 700, *d)
    binding.rollout_apply(runner.to_device(cmds, device=dev), 0, 0, *d)      # nothing to do
    torch.cuda.synchronize()
    O.pool_commands_apply(cmds, 270, 700, seq_id, ctx, step, table)
    for got, ref in zip(d, (seq_id, ctx, step, table)):
        np.testing.assert_array_equal(got.cpu().numpy(), ref)


def test_commands_that_name_no_slot_are_skipped(gpu):
    # a fixed-size command buffer padded with slot -1 (and entries outside the pool or the block
    # table's row) changes what its valid commands say and nothing else
    torch, binding, runner, dev = gpu
    rng = np.random.default_rng(3)
    pool, max_pages = 64, 5
    seq_id, ctx, step = rng.integers(-1, 50, pool), rng.integers(0, 99, pool).astype(np.int32), rng.integers(0, 9, pool).astype(np.int32)
    table = rng.integers(0, 1000, (pool, max_pages)).astype(np.int32)
    slot_cmds = np.full((pool, 4), -1, dtype=np.int64)
    valid_s = rng.permutation(pool)[:20]
    slot_cmds[:20] = np.stack([valid_s, rng.integers(-1, 1 << 20, 20), rng.integers(0, 5000, 20), rng.integers(0, 4000, 20)], 1)
    slot_cmds[20] = [pool, 7, 7, 7]                      # past the pool
    page_cmds = np.full((pool, 3), -1, dtype=np.int64)
    cells = rng.permutation(pool * max_pages)[:30]
    page_cmds[:30] = np.stack([cells // max_pages, cells % max_pages, rng.integers(0, 1 << 20, 30)], 1)
    page_cmds[30] = [3, max_pages, 9]                    # past the row
    page_cmds[31] = [pool + 2, 0, 9]
    cmds = np.concatenate([slot_cmds.reshape(-1), page_cmds.reshape(-1)]).astype(np.int32)
    d = [runner.to_device(x, device=dev) for x in (seq_id.astype(np.int64), ctx, step, table)]
    binding.rollout_apply(runner.to_device(cmds, device=dev), pool, pool, *d)
    torch.cuda.synchronize()
    only_valid = np.concatenate([slot_cmds[:20].reshape(-1), page_cmds[:30].reshape(-1)]).astype(np.int32)
    O.pool_commands_apply(only_valid, 20, 30, seq_id, ctx, step, table)
    for got, ref in zip(d, (seq_id, ctx, step, table)):
        np.testing.assert_array_equal(got.cpu().numpy(), ref)


@pytest.mark.parametrize("dtype,D,Hkv", [(W.BF16, 128, 4), (W.F32, 64, 2), (W.BF16, 64, 1)])
def test_kv_append(gpu, dtype, D, Hkv):
    torch, binding, runner, dev = gpu
    rng = np.random.default_rng(1)
    C, P, max_pages = 37, 16, 6
    num_pages = C * max_pages
    ctx = rng.integers(0, max_pages * P + 1, C).astype(np.int32)
    ctx[:6] = [0, 1, 16, 17, max_pages * P, 0]
    table = rng.permutation(num_pages).reshape(C, max_pages).astype(np.int32)
    k_new, v_new = (W.to_storage(rng.normal(size=(C, Hkv, D)).astype(np.float32), dtype) for _ in range(2))
    kc, vc = (W.to_storage(rng.normal(size=(num_pages, Hkv, P, D)).astype(np.float32), dtype) for _ in range(2))
    dk, dv = runner.to_device(kc, device=dev), runner.to_device(vc, device=dev)
    binding.kv_append(runner.to_device(k_new, device=dev), runner.to_device(v_new, device=dev),
                      runner.to_device(table, device=dev), runner.to_device(ctx, device=dev), dk, dv,
                      dtype=runner.dtype_code(dtype))
    torch.cuda.synchronize()
    O.kv_append(k_new, v_new, table, ctx, kc, vc)
    view = (lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)) if dtype == W.BF16 else (lambda t: t.cpu().numpy())
    np.testing.assert_array_equal(view(dk), kc)
    np.testing.assert_array_equal(view(dv), vc)


def test_buffer_append_and_concatenation(gpu):
    torch, binding, runner, dev = gpu
    rng = np.random.default_rng(2)
    n_traj, max_resp, pool = 23, 40, 9
    up = lambda a: runner.to_device(a, device=dev)
    buf_token = torch.full((n_traj, max_resp), -1, dtype=torch.int32, device=dev)
    buf_logp = torch.full((n_traj, max_resp), float("nan"), dtype=torch.float32, device=dev)
    buf_tag = torch.full((n_traj, max_resp), -1, dtype=torch.int32, device=dev)
    ora, gen = {}, np.zeros(n_traj, int)
    for stage in range(4):
        for _ in range(8):
            trs = rng.permutation(n_traj)[:pool]
            trs = np.where(gen[trs] < max_resp, trs, -1)
            trs[rng.integers(0, pool)] = -1                          # an idle slot
            step = np.where(trs >= 0, gen[np.maximum(trs, 0)], 0).astype(np.int32)
            ctx = (step + 5).astype(np.int32) * (trs >= 0)
            tok = rng.integers(0, 150000, pool).astype(np.int32)
            lp = (-rng.exponential(size=pool)).astype(np.float32)
            d_step, d_ctx = up(step), up(ctx)
            binding.traj_append(up(tok), up(lp), up(trs.astype(np.int64)), d_step, d_ctx, stage, buf_token, buf_logp, buf_tag)
            act = trs >= 0
            np.testing.assert_array_equal(d_step.cpu().numpy(), step + act)      # the slot advances
            np.testing.assert_array_equal(d_ctx.cpu().numpy(), ctx + act)
            for c in np.flatnonzero(act):
                O.buffer_append(ora, trs[c], stage, tok[c], lp[c])
                gen[trs[c]] += 1
        # a batch formed in this stage, some trajectories never generated anything
        batch = rng.permutation(n_traj)[:11]
        cat = O.buffer_concat(ora, batch, stage)
        B, N = len(batch), int(cat["cu_seqlens"][-1])
        tokens = torch.full((N,), -7, dtype=torch.int32, device=dev)
        lb, lr = torch.zeros(N, device=dev), torch.zeros(N, device=dev)
        split = torch.full((B,), -7, dtype=torch.int32, device=dev)
        binding.traj_gather(buf_token, buf_logp, buf_tag, up(batch.astype(np.int32)), up(cat["cu_seqlens"].astype(np.int32)),
                            stage, tokens, lb, lr, split)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(tokens.cpu().numpy(), cat["tokens"])
        np.testing.assert_array_equal(split.cpu().numpy(), cat["split"])
        np.testing.assert_array_equal(lb.cpu().numpy(), cat["logp_buf"].astype(np.float32))    # NaN == NaN here
        np.testing.assert_array_equal(lr.cpu().numpy(), cat["logp_roll"].astype(np.float32))
    # rows past what was appended were never written
    tags = buf_tag.cpu().numpy()
    assert ((tags >= 0).sum(axis=1) == gen).all()


def test_empty_calls_enqueue_nothing(gpu):
    torch, binding, runner, dev = gpu
    lib = binding.load_library()
    assert lib.copris_kv_append(None, None, None, None, None, None, 0, 2, 128, 16, 4, 10, 1, None) == 0
    assert lib.copris_traj_append(None, None, None, None, None, 0, None, None, None, 0, 5, 8, None) == 0
    assert lib.copris_traj_gather(None, None, None, None, None, 0, None, None, None, None, 0, 5, 8, None) == 0
    assert lib.copris_kv_append(None, None, None, None, None, None, 3, 2, 128, 16, 4, 10, 1, None) == binding.COPRIS_EINVAL
    assert lib.copris_kv_append(None, None, None, None, None, None, 3, 2, 4, 16, 4, 10, 1, None) == binding.COPRIS_EUNSUPPORTED
