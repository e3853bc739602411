"""GPU: what the header promises about optional outputs and streams.  `lse = NULL` leaves the
other outputs bit for bit as they are with it; calls on side streams with disjoint workspaces
and outputs run side by side and give bit for bit what the same calls give on the default
stream."""
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
    return (t.view(torch.int16) if t.dtype == torch.bfloat16 else t).cpu().numpy()


def test_null_lse_changes_nothing_else(gpu):
    torch, binding, R = gpu
    # decode attention: the matrix-core path and the generic one
    for dtype, D in ((W.BF16, 128), (W.F32, 64)):
        case = W.make_small_decode_case(31, 5, 12, 2, D, dtype, 16, [700, 16, 1, 0, 1025])
        d = R.stage_attn(case, dtype)
        d.run()
        torch.cuda.synchronize()
        ref = _bits(d.out).copy()
        d.out.fill_(float("nan"))
        d.lse = None
        d.run()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(_bits(d.out), ref)
    # LM head with sampling: matrix-core path, generic path
    for dtype, shape in ((W.BF16, (40, 512, 7000)), (W.F32, (9, 72, 260))):
        inp = W.make_small_lmhead_case(12, *shape, dtype)
        d = R.stage_lmhead(inp, dtype)
        d.run()
        torch.cuda.synchronize()
        tok, lp = d.token.cpu().numpy().copy(), d.logprob.cpu().numpy().copy()
        d.token.fill_(-1)
        d.logprob.fill_(float("nan"))
        d.lse = None
        d.run()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(d.token.cpu().numpy(), tok)
        np.testing.assert_array_equal(d.logprob.cpu().numpy(), lp)
    # given-token log-probs: the 128-row kernel and the 256 x 256 one
    for M in (50, 600):
        inp = W.make_small_lmhead_case(13, M, 256, 3000, W.BF16)
        tokens = np.random.default_rng(M).integers(0, 3000, M)
        d = R.stage_token_logprob(inp["hidden"], inp["weight"], tokens, 1.0, W.BF16)
        d.run()
        torch.cuda.synchronize()
        lp = d.logprob.cpu().numpy().copy()
        d.logprob.fill_(float("nan"))
        d.lse = None
        d.run()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(d.logprob.cpu().numpy(), lp)
    # re-prefill attention
    b = W.make_prefill_case(14, [40, 333, 17], 28, 4, 128, W.BF16)
    d = R.stage_prefill_attn(b, W.BF16)
    d.run()
    torch.cuda.synchronize()
    ref = _bits(d.out).copy()
    d.out.fill_(float("nan"))
    d.lse = None
    d.run()
    torch.cuda.synchronize()
    np.testing.assert_array_equal(_bits(d.out), ref)


def test_side_streams_with_disjoint_workspaces(gpu):
    torch, binding, R = gpu
    ctx = [1000, 37, 1536, 513, 16, 2500, 800, 64] * 6
    case = W.make_small_decode_case(41, len(ctx), 28, 4, 128, W.BF16, 16, ctx)
    lmc = W.make_small_lmhead_case(42, 64, 1536, 30000, W.BF16)
    isb = W.make_is_inputs(W.IS_CONFIGS[0])
    # two independent sets of (inputs, outputs, workspace) per call
    attn = [R.stage_attn(case, W.BF16) for _ in range(2)]
    lm = [R.stage_lmhead(lmc, W.BF16) for _ in range(2)]
    isd = [R.stage_is_ratio(isb) for _ in range(2)]
    assert attn[0].ws.data_ptr() != attn[1].ws.data_ptr() and lm[0].ws.data_ptr() != lm[1].ws.data_ptr()
    # reference: the default stream, one call after the other
    attn[0].run(); lm[0].run(); isd[0].run()
    torch.cuda.synchronize()
    outs = lambda a, l, i: [_bits(a.out).copy(), a.lse.cpu().numpy().copy(), l.token.cpu().numpy().copy(),
                            l.logprob.cpu().numpy().copy(), l.lse.cpu().numpy().copy(), i.ratio.cpu().numpy().copy(),
                            i.ratio_clipped.cpu().numpy().copy(), i.seq_sum.cpu().numpy().copy(),
                            i.seq_cnt.cpu().numpy().copy(), i.seq_nclip.cpu().numpy().copy()]
    ref = outs(attn[0], lm[0], isd[0])
    for a, l, i in zip(attn, lm, isd):
        a.out.fill_(float("nan")); a.lse.fill_(float("nan")); l.token.fill_(-1); l.logprob.fill_(float("nan"))
        l.lse.fill_(float("nan")); i.ratio.fill_(float("nan")); i.ratio_clipped.fill_(float("nan"))
        i.seq_sum.fill_(float("nan")); i.seq_cnt.fill_(-7); i.seq_nclip.fill_(-7)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(6)]        # default priority
    for rep in range(3):                                     # the six calls overlap on the device
        attn[0].run(streams[0]); attn[1].run(streams[1])
        lm[0].run(streams[2]); lm[1].run(streams[3])
        isd[0].run(streams[4]); isd[1].run(streams[5])
    for s in streams:
        s.synchronize()
    torch.cuda.synchronize()
    for j in range(2):
        for got, want in zip(outs(attn[j], lm[j], isd[j]), ref):
            np.testing.assert_array_equal(got, want)
