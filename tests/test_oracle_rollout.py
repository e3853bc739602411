"""Pins for the oracle's rollout manager (Section 4: Concurrency-Controlled Generation, Early
Termination, Buffering of Partial Trajectories, Prioritized Resumption)."""
import numpy as np
import pytest

from oracle import copris_oracle as O


def test_hand_worked_schedule():
    # 3 inputs x 2 samples, pool 3, a training step needs 1 input.  Lengths:
    #   input 0: (2, 5)   input 1: (3, 1)   input 2: (4, 2)        prompts 10, 20, 30
    # stage 0: slots run (0,0) (0,1) (1,0).
    #   step 1: gen 1,1,1        step 2: (0,0) finishes -> slot gets (1,1)
    #   step 3: (0,1)=3, (1,0)=3 finishes, (1,1)=1 finishes -> input 1 complete -> stop.
    #   batch = [1], 4 tokens, all on-policy; paused: (0,1) with 3 tokens; buffered complete: (0,0).
    # stage 1: resume (0,1) [re-prefill 10 + 3], then fresh (2,0), (2,1).
    #   step 1: (0,1)=4  (2,0)=1  (2,1)=1      step 2: (0,1)=5 finishes -> input 0 complete -> stop.
    #   batch = [0]: tokens 2 + 5 = 7, off-policy = 2 (from (0,0)) + 3 (from (0,1)) = 5, both
    #   trajectories off-policy, staleness 1; paused: (2,0)=2, (2,1)=2 -> but (2,1) has length 2:
    #   it finished at step 2 -> paused 1, buffered complete 1.
    # stage 2: resume (2,0) [30 + 2]: steps 3, 4 -> finishes at step 2 of the stage -> input 2.
    st = O.rollout_schedule([10, 20, 30], [[2, 5], [3, 1], [4, 2]], pool=3, batch_inputs=1)
    assert len(st) == 3
    s0, s1, s2 = st
    assert (s0["steps"], s0["generated"], s0["batch_inputs"], s0["batch_tokens"], s0["batch_offpolicy"]) == (3, 9, [1], 4, 0)
    assert (s0["paused"], s0["buffered_complete"], s0["resumed"], s0["reprefill_tokens"]) == (1, 1, 0, 0)
    assert s0["slot_steps_idle"] == 0
    assert (s1["steps"], s1["generated"], s1["batch_inputs"], s1["batch_tokens"], s1["batch_offpolicy"]) == (2, 6, [0], 7, 5)
    assert (s1["batch_traj_offpolicy"], s1["max_staleness"], s1["resumed"], s1["reprefill_tokens"]) == (2, 1, 1, 13)
    assert (s1["paused"], s1["buffered_complete"]) == (1, 1)
    assert (s2["steps"], s2["generated"], s2["batch_inputs"], s2["batch_tokens"], s2["batch_offpolicy"]) == (2, 2, [2], 6, 4)
    assert (s2["resumed"], s2["reprefill_tokens"], s2["paused"], s2["slot_steps_idle"]) == (1, 32, 0, 4)
    # pages: stage 0 step 3 holds (0,1): ceil(13/16)=1, (1,0): ceil(23/16)=2, (1,1): ceil(21/16)=2
    assert s0["peak_pages"] == 5


def _random_case(seed, I=12, N=4, lo=1, hi=60):
    rng = np.random.default_rng(seed)
    return rng.integers(5, 40, size=I), rng.integers(lo, hi, size=(I, N))


def test_synchronous_limit_is_on_policy():
    # pool >= all trajectories and B = all inputs: one stage, nothing paused, nothing stale,
    # and the stage lasts as long as the longest trajectory (the long-tail problem, Section 3.2)
    p, r = _random_case(1)
    st = O.rollout_schedule(p, r, pool=r.size, batch_inputs=len(p))
    assert len(st) == 1
    s = st[0]
    assert s["steps"] == r.max() and s["generated"] == r.sum() == s["batch_tokens"]
    assert s["batch_offpolicy"] == 0 and s["paused"] == 0 and s["resumed"] == 0
    assert s["slot_steps_idle"] == r.size * r.max() - r.sum()


@pytest.mark.parametrize("seed", range(5))
def test_conservation_and_bounds(seed):
    p, r = _random_case(10 + seed, I=16, N=4)
    pool, B = 7, 3
    st = O.rollout_schedule(p, r, pool=pool, batch_inputs=B)
    consumed = [i for s in st for i in s["batch_inputs"]]
    assert len(consumed) == len(set(consumed)) and all(len(s["batch_inputs"]) == B for s in st)
    assert len(st) == len(p) // B                       # every stage that can complete does
    # every token of a consumed trajectory was generated exactly once
    assert sum(s["batch_tokens"] for s in st) == r[consumed].sum()
    assert sum(s["generated"] for s in st) >= r[consumed].sum()
    for k, s in enumerate(st):
        # "N' - 1 partially generated trajectories remain": the request that completed the
        # batch has just finished, so at most pool - 1 are paused
        assert s["paused"] <= pool - 1
        assert s["generated"] + s["slot_steps_idle"] == pool * s["steps"]
        assert s["batch_offpolicy"] <= s["batch_tokens"] and s["max_staleness"] <= k
        if k == 0:
            assert s["batch_offpolicy"] == 0 and s["resumed"] == 0
        else:
            # everything paused is resumed first (a stage that finds enough complete inputs
            # in the buffer runs no step and resumes nothing)
            assert s["resumed"] == (st[k - 1]["paused"] if s["steps"] > 0 else 0)
    # more concurrency -> more paused / off-policy work (Section 5.4, concurrency ablation)
    st_big = O.rollout_schedule(p, r, pool=14, batch_inputs=B)
    assert sum(s["batch_offpolicy"] for s in st_big) >= sum(s["batch_offpolicy"] for s in st)


def test_resumption_has_priority_and_keeps_tags():
    # one long trajectory is paused over several stages: it is always dispatched first, its
    # re-prefill grows by what it generated, and its tokens' staleness grows by one per stage
    p = [8, 8, 8, 8]
    r = [[50, 1], [2, 2], [2, 2], [2, 2]]
    st = O.rollout_schedule(p, r, pool=2, batch_inputs=1)
    # stage 0: (0,0) and (0,1) run; (0,1) finishes at step 1 -> (1,0) starts, finishes at step 3
    #          -> (1,1) runs steps 4, 5 -> input 1 complete at step 5: (0,0) has 5 tokens
    assert st[0]["batch_inputs"] == [1] and st[0]["steps"] == 5 and st[0]["paused"] == 1
    assert st[1]["resumed"] == 1 and st[1]["reprefill_tokens"] == 8 + 5
    assert st[1]["batch_inputs"] == [2] and st[1]["steps"] == 4
    assert st[2]["reprefill_tokens"] == 8 + 9 and st[2]["batch_inputs"] == [3]
    # input 0 can only complete alone: the last stage consumes it with tags 0, 1, 2, 3
    assert st[3]["batch_inputs"] == [0] and st[3]["max_staleness"] == 3
    assert st[3]["batch_tokens"] == 51 and st[3]["batch_offpolicy"] == 1 + 5 + 4 + 4
