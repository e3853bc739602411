"""GPU: one decode step (attention, LM head with sampling through the entry point that
allocates nothing, ratio kernel) captured in a HIP graph.  The library enqueues kernels only -
no memset, no copy, no allocation, no wait - so a captured step must replay bit for bit like
the eager one, also after the inputs changed in place between replays."""
import numpy as np
import pytest

from paper_2511_05589_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2511_05589_amd import binding, runner
    runner.require_gpu()
    return torch, binding, runner


def _bits(t):
    import torch
    return (t.view(torch.int16) if t.dtype == torch.bfloat16 else t).cpu().numpy().copy()


def test_a_captured_decode_step_replays_like_the_eager_one(gpu):
    torch, binding, R = gpu
    case = W.make_small_decode_case(77, 12, 28, 4, 128, W.BF16, 16, [900, 16, 1, 0, 1025, 33, 257, 64, 5000, 2, 700, 48])
    attn = R.stage_attn(case, W.BF16)
    lm = R.stage_lmhead(W.make_small_lmhead_case(78, 12, 512, 9000, W.BF16), W.BF16)
    isb = R.stage_is_ratio(W.make_is_inputs(W.IS_CONFIGS[0]))

    def step(stream):
        attn.run(stream)
        binding.lmhead_logprob_noalloc(lm.hidden, lm.weight, lm.seq_id, lm.step, lm.token, lm.logprob, lm.lse,
                                       seed=lm.seed, temperature=lm.temperature, dtype=lm.dtype, stream=stream)
        isb.run(stream)

    def outputs():
        torch.cuda.synchronize()
        return [_bits(x) for x in (attn.out, attn.lse, lm.token, lm.logprob, lm.lse, isb.ratio, isb.ratio_clipped,
                                   isb.seq_sum, isb.seq_cnt, isb.seq_nclip)]

    def poison():
        for x in (attn.out, attn.lse, lm.logprob, lm.lse, isb.ratio, isb.ratio_clipped, isb.seq_sum):
            x.fill_(float("nan"))
        for x in (lm.token, isb.seq_cnt, isb.seq_nclip):
            x.fill_(-9)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step(side)                       # (first use of the static array: its address is looked up here, not under capture)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(torch.cuda.current_stream())
    torch.cuda.synchronize()

    for replay in range(4):
        # the program's own eager work between the replays: new inputs, in place
        attn.q.mul_(-0.5 if replay % 2 else 1.25)
        lm.step.add_(1 + replay)
        isb.logp_cur.add_(0.01 * (replay + 1))
        torch.cuda.synchronize()
        poison()
        step(None)
        eager = outputs()
        poison()
        graph.replay()
        replayed = outputs()
        for a, b in zip(eager, replayed):
            np.testing.assert_array_equal(a, b)
    assert (eager[2] >= 0).all() and (eager[2] < 9000).all()
