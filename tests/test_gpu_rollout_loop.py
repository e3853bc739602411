"""GPU: the fixed-concurrency rollout loop end to end (Section 4) against the oracle.

The loop (product code) drives prefill, KV pages, decode attention, sampling, the log-prob
buffer with its stage tags (Eq. 6), early termination, resumption under a new policy version,
and Eq. 8 / Eq. 2-4 on every training batch.  The test replays the loop's recorded plan with
the oracle's functions on the same seeded stand-in inputs, and checks the stage statistics
against the library's scheduler and the oracle's token-by-token simulation.
"""
import numpy as np
import pytest

from oracle import copris_oracle as O
from paper_2511_05589_amd import workloads as W
from tests import parity as P

pytestmark = pytest.mark.gpu

PROMPT = [5, 18, 3, 33, 9, 12]
RESP = [[4, 21], [30, 2], [17, 6], [3, 35], [9, 9], [14, 5]]
POOL, BATCH = 4, 2
DIMS = dict(Hq=8, Hkv=2, D=128, H=256, V=2048)
SEED, SAMPLE_SEED = 5, 7


@pytest.fixture(scope="module")
def run():
    from paper_2511_05589_amd import runner
    from paper_2511_05589_amd.rollout_loop import RolloutLoop
    runner.require_gpu()
    policy = W.StandInPolicy(SEED, PROMPT, RESP, dtype=W.BF16, **DIMS)
    loop = RolloutLoop(policy, POOL, BATCH, sample_seed=SAMPLE_SEED)
    stages = loop.run(max_stages=3)
    return policy, loop, stages


STAT_KEYS = ("steps", "generated", "slot_steps_idle", "batch_tokens", "batch_offpolicy", "batch_traj_offpolicy",
             "max_staleness", "resumed", "reprefill_tokens", "paused", "buffered_complete", "peak_pages")


def test_the_schedule_is_the_schedulers(run):
    from paper_2511_05589_amd import binding
    _, _, stages = run
    lib = binding.rollout_schedule(PROMPT, RESP, POOL, BATCH, max_stages=3)
    ora = O.rollout_schedule(PROMPT, RESP, POOL, BATCH, max_stages=3)
    assert len(stages) == len(lib) == len(ora) == 3
    for k, st in enumerate(stages):
        for key in STAT_KEYS:
            assert st["stats"][key] == lib[k][key] == ora[k][key], (k, key)
        assert st["stats"]["batch_inputs"] == lib[k]["batch_inputs"][:BATCH] == ora[k]["batch_inputs"]
    # the case is built so that the concurrency mechanics all occur
    assert sum(st["stats"]["resumed"] for st in stages) > 0
    assert sum(st["stats"]["batch_offpolicy"] for st in stages) > 0


def test_every_page_comes_back(run):
    _, loop, _ = run
    # inputs that never left keep no pages either: pages belong to running requests only
    assert not loop.pages_of
    assert sorted(loop.free_pages) == list(range(loop.num_pages))


def _dense_attn(policy, tr, p, ver):
    """Oracle decode attention of position p of trajectory tr over its own rows 0..p."""
    t = policy.tables(tr, ver)
    f = lambda x: W.to_f32(x, policy.dtype).astype(np.float64)
    n = p + 1
    npg = (n + 15) // 16
    kc = np.zeros((npg, policy.Hkv, 16, policy.D))
    vc = np.zeros_like(kc)
    k, v = f(t["k"][:n]), f(t["v"][:n])
    for j in range(n):
        kc[j // 16, :, j % 16] = k[j]
        vc[j // 16, :, j % 16] = v[j]
    return O.decode_attn(f(t["q"][p:p + 1]), kc, vc, np.arange(npg, dtype=np.int32)[None], np.asarray([n]),
                         policy.scale)


def test_replay_with_the_oracle(run):
    policy, loop, stages = run
    gen = [0] * len(loop.traj)
    exempt = 0
    for k, st in enumerate(stages):
        ver = st["version"]
        w = W.to_f32(policy.weight(ver), policy.dtype)
        for step in st["plan"]:
            for tr, n in zip(step["entered"], step["prefill_len"]):
                assert n == PROMPT[tr // 2] + gen[tr]          # prompt + what the buffer holds
            for tr in step["active"]:
                g = gen[tr]
                p = PROMPT[tr // 2] + g
                t = loop.traj[tr]
                assert t.tag[g] == k
                # attention over pages that prefill and the appends built (a wrong page or a
                # stale version would show here)
                ref_out, ref_lse = _dense_attn(policy, tr, p, ver)
                P.check_attn(t.attn_out[g][None], t.attn_lse[g][None], ref_out, ref_lse, policy.dtype,
                             f"stage {k} traj {tr} pos {p}")
                h = W.to_f32(policy.tables(tr, ver)["hidden"][p:p + 1], policy.dtype)
                ref = O.lmhead_logprob(h, w, np.asarray([tr]), np.asarray([g]), SAMPLE_SEED, 1.0, return_full=True)
                tok = int(t.tokens[g])
                if tok != int(ref["token"][0]):
                    assert ref["best"][0] - ref["runner_up"][0] < P.NEAR_TIE and tok == int(ref["second_token"][0])
                    exempt += 1
                assert abs(t.logp[g] - ref["logp"][0, tok]) <= P.LOGPROB_TOL
                gen[tr] += 1
    assert exempt <= 2
    # every trajectory that started stopped at its length or was left paused; tags never decrease
    for tr, t in enumerate(loop.traj):
        assert len(t.tokens) == gen[tr] <= RESP[tr // 2][tr % 2]
        assert all(a <= b for a, b in zip(t.tag, t.tag[1:]))


def test_training_batches(run):
    policy, loop, stages = run
    saw_offpolicy = False
    for k, st in enumerate(stages):
        tr = st["train"]
        w = W.to_f32(policy.weight(st["version"]), policy.dtype)
        ref = O.lmhead_token_logprob(W.to_f32(tr["hidden"], policy.dtype), w, tr["tokens"], 1.0)
        assert np.abs(tr["logp_cur"] - ref["logprob"]).max() <= P.LOGPROB_TOL
        b = {"N": int(tr["cu_seqlens"][-1]), "B": len(tr["trajectories"]), "mask": None,
             "cu_seqlens": tr["cu_seqlens"], "split": tr["split"], "logp_cur": tr["logp_cur"],
             "logp_buf": tr["logp_buf"], "logp_roll": tr["logp_roll"], "adv": tr["adv"],
             "eps_low": 0.2, "eps_high": 0.28}
        P.check_is(tr, P.oracle_is(b, use_mask=False), b, use_mask=False, what=f"stage {k}")
        P.check_grpo(tr, P.oracle_grpo(b, use_mask=False), b, use_mask=False, what=f"stage {k}")
        # tokens of the current stage: the sampling kernel's log-prob and the given-token
        # kernel's agree, so their ratio is 1 up to the kernels' rounding; tokens of earlier
        # stages were generated under another version and are not
        on = tr["tags"] == k
        assert np.abs(tr["ratio"][on] - 1.0).max(initial=0.0) <= 2e-3
        if (~on).any():
            saw_offpolicy = True
            assert np.abs(tr["ratio"][~on] - 1.0).max() > 1e-2
        # the split is the count of earlier-stage tokens, which Eq. 6 makes a prefix
        for s, trj in enumerate(tr["trajectories"]):
            tags = np.asarray(loop.traj[trj].tag)
            assert (tags[:tr["split"][s]] < k).all() and (tags[tr["split"][s]:] == k).all()
    assert saw_offpolicy
