"""GPU: copris_lmhead_logprob_noalloc (partials in the library's static device array) gives bit
for bit what copris_lmhead_logprob gives with a caller workspace - on two calls in a row, the
second on a smaller input - and refuses shapes the array cannot hold."""
import numpy as np
import pytest

from paper_2511_05589_amd import workloads as W

pytestmark = pytest.mark.gpu


def _both(R, binding, torch, inp, dtype):
    d = R.stage_lmhead(inp, dtype)
    d.run()
    torch.cuda.synchronize()
    ref = [d.token.cpu().numpy().copy(), d.logprob.cpu().numpy().copy(), d.lse.cpu().numpy().copy()]
    d.token.fill_(-1)
    d.logprob.fill_(float("nan"))
    d.lse.fill_(float("nan"))
    binding.lmhead_logprob_noalloc(d.hidden, d.weight, d.seq_id, d.step, d.token, d.logprob, d.lse,
                                   seed=d.seed, temperature=d.temperature, dtype=d.dtype)
    torch.cuda.synchronize()
    got = [d.token.cpu().numpy(), d.logprob.cpu().numpy(), d.lse.cpu().numpy()]
    return got, ref


def test_no_alloc_entry_point_matches_the_workspace_one():
    import torch
    from paper_2511_05589_amd import binding, runner as R
    R.require_gpu()
    assert binding.load_library().copris_lmhead_logprob_noalloc_max_bytes() == 4 << 20
    # first call: two batch blocks on the matrix-core path, more tiles than workgroups;
    # second call, right after it: fewer rows, fewer parts (stale partials of the first call
    # stay in the array past what the second one writes and reads);
    # third: the vector-ALU path (fp32), which lays the partials out per 64-entry tile
    cases = [(W.BF16, (300, 512, 70000)), (W.BF16, (40, 256, 3000)), (W.F32, (9, 72, 2600)),
             (W.BF16, (256, 1536, 20000))]
    for dtype, shape in cases:
        inp = W.make_small_lmhead_case(sum(shape), *shape, dtype)
        got, ref = _both(R, binding, torch, inp, dtype)
        for g, r in zip(got, ref):
            np.testing.assert_array_equal(g, r)
    # a shape whose partials do not fit is refused with a clear error and enqueues nothing
    inp = W.make_small_lmhead_case(1, 100, 72, 151936, W.F32)       # 100 * 2374 * 20 bytes > 4 MiB
    d = R.stage_lmhead(inp, W.F32)
    d.token.fill_(-5)
    with pytest.raises(binding.CoprisError) as e:
        binding.lmhead_logprob_noalloc(d.hidden, d.weight, d.seq_id, d.step, d.token, d.logprob, d.lse,
                                       seed=d.seed, temperature=1.0, dtype=d.dtype)
    assert e.value.code == binding.COPRIS_EWORKSPACE and "static" in str(e.value)
    torch.cuda.synchronize()
    assert (d.token.cpu().numpy() == -5).all()
