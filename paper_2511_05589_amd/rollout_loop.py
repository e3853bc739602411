"""A fixed-concurrency rollout loop that drives the library's kernels end to end
(Section 4: Concurrency-Controlled Generation, Early Termination, Buffering of Partial
Trajectories with Eq. 6, Prioritized Resumption; Eq. 8 and Eq. 2-4 on the training batch).

The transformer is replaced by a stand-in (`workloads.StandInPolicy`): the query, key, value
and final hidden state of a trajectory position are seeded noise per policy version, and a
trajectory stops at a given length.  Everything around it is the real path:

  * a pool of `pool` requests, refilled whenever one finishes, paused trajectories first;
  * a KV page allocator (free list); pages are released when a request finishes or is
    paused, because a new policy version invalidates them;
  * (re-)prefill of every request that enters the pool: `copris_prefill_attn` rebuilds the
    pages of prompt + generated tokens under the current version;
  * one decode step per iteration: the new position's key / value are appended to its page
    (a copy, the one step a decoder layer would do that this library does not), then
    `copris_decode_attn` over the active set and `copris_lmhead_logprob` sample a token and
    its log-prob, which goes to the trajectory's buffer tagged with the stage;
  * a stage stops as soon as `batch_inputs` inputs have all their samples; on that batch
    `copris_lmhead_token_logprob` gives the current policy's log-probs of the buffered tokens,
    `copris_is_ratio` the cross-stage ratios and `copris_grpo_surrogate` the clipped surrogate.

The schedule follows the same rules as `copris_rollout_schedule` (which a test checks stage
by stage); this module is a driver and a test vehicle, sized for small cases: it steps token
by token from Python.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

from . import binding
from .runner import dtype_code, require_gpu, to_device, workspace
from .workloads import BF16, StandInPolicy


@dataclass
class Trajectory:
    tokens: list = field(default_factory=list)     # sampled token per generated position
    logp: list = field(default_factory=list)       # its log-prob under the generating policy
    tag: list = field(default_factory=list)        # stage that generated it (Eq. 6: pieces in stage order)
    attn_out: list = field(default_factory=list)   # decode attention output [Hq, D] (fp32) per position
    attn_lse: list = field(default_factory=list)   # and its log-sum-exp [Hq]
    started: bool = False


class RolloutLoop:
    def __init__(self, policy: StandInPolicy, pool: int, batch_inputs: int, *, sample_seed: int = 7,
                 temperature: float = 1.0, eps_low: float = 0.2, eps_high: float = 0.28,
                 page_size: int = 16, page_seed: int = 11):
        self.m = policy
        self.pool, self.batch_inputs = int(pool), int(batch_inputs)
        self.sample_seed, self.temperature = int(sample_seed), float(temperature)
        self.eps_low, self.eps_high = float(eps_low), float(eps_high)
        self.page_size = int(page_size)
        self.dev = require_gpu()
        self.dt = dtype_code(policy.dtype)
        self.I = int(policy.prompt_len.size)
        self.N = policy.samples
        max_len = int((policy.prompt_len[:, None] + policy.resp_len).max())
        self.max_pages = (max_len + page_size - 1) // page_size
        self.num_pages = self.pool * self.max_pages + 3
        # physical pages are handed out in a shuffled order, so block tables are scattered
        order = np.random.default_rng(page_seed).permutation(self.num_pages)
        self.free_pages = [int(x) for x in order]
        tdt = torch.bfloat16 if policy.dtype == BF16 else torch.float32
        shape = (self.num_pages, policy.Hkv, page_size, policy.D)
        self.k_cache = torch.full(shape, float("nan"), dtype=tdt, device=self.dev)
        self.v_cache = torch.full(shape, float("nan"), dtype=tdt, device=self.dev)
        self.traj = [Trajectory() for _ in range(self.I * self.N)]
        self.pages_of = {}                      # running trajectory -> list of physical pages
        self.consumed = [False] * self.I
        self.stages = []                        # per-stage dicts: stats, plan, training batch
        self.attn_ws = workspace(binding.decode_attn_workspace_bytes(
            self.pool, policy.Hq, policy.Hkv, policy.D, page_size, self.max_pages), self.dev)
        self.lm_ws = workspace(binding.lmhead_logprob_workspace_bytes(self.pool, policy.H, policy.V), self.dev)

    # ---- helpers -------------------------------------------------------------------------
    def _gen(self, tr):
        return len(self.traj[tr].tokens)

    def _target(self, tr):
        i, s = divmod(tr, self.N)
        return int(self.m.resp_len[i, s])

    def _prompt(self, tr):
        return int(self.m.prompt_len[tr // self.N])

    def _ensure_pages(self, tr, n_tokens):
        need = (n_tokens + self.page_size - 1) // self.page_size
        pages = self.pages_of.setdefault(tr, [])
        while len(pages) < need:
            pages.append(self.free_pages.pop(0))

    def _release(self, tr):
        self.free_pages.extend(self.pages_of.pop(tr, []))

    def _table(self, trs):
        bt = np.zeros((len(trs), self.max_pages), dtype=np.int32)
        for r, tr in enumerate(trs):
            p = self.pages_of[tr]
            bt[r, :len(p)] = p
        return to_device(bt, device=self.dev)

    def _complete_inputs(self):
        return [i for i in range(self.I) if not self.consumed[i] and all(
            self.traj[i * self.N + s].started and self._gen(i * self.N + s) >= self._target(i * self.N + s)
            for s in range(self.N))]

    # ---- kernels ---------------------------------------------------------------------------
    def _prefill(self, trs, ver):
        """Rebuild the pages of prompt + generated tokens of the requests entering the pool."""
        lens = [self._prompt(tr) + self._gen(tr) for tr in trs]
        for tr, n in zip(trs, lens):
            self._ensure_pages(tr, n)
        q = np.concatenate([self.m.tables(tr, ver)["q"][:n] for tr, n in zip(trs, lens)])
        k = np.concatenate([self.m.tables(tr, ver)["k"][:n] for tr, n in zip(trs, lens)])
        v = np.concatenate([self.m.tables(tr, ver)["v"][:n] for tr, n in zip(trs, lens)])
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        qd, kd, vd = (to_device(x, device=self.dev) for x in (q, k, v))
        out = torch.empty_like(qd)
        lse = torch.empty((qd.shape[0], self.m.Hq), dtype=torch.float32, device=self.dev)
        binding.prefill_attn(qd, kd, vd, to_device(cu, device=self.dev), self._table(trs), self.k_cache,
                             self.v_cache, out, lse, max_seqlen=int(max(lens)), scale=self.m.scale, dtype=self.dt)
        return lens, lse.cpu().numpy()

    def _decode_step(self, active, ver, stage):
        pos = [self._prompt(tr) + self._gen(tr) for tr in active]
        for tr, p in zip(active, pos):
            self._ensure_pages(tr, p + 1)
        # KV append of the new position (plain copies into the pages)
        page = torch.tensor([self.pages_of[tr][p // self.page_size] for tr, p in zip(active, pos)], device=self.dev)
        off = torch.tensor([p % self.page_size for p in pos], device=self.dev)
        k_new = to_device(np.stack([self.m.tables(tr, ver)["k"][p] for tr, p in zip(active, pos)]), device=self.dev)
        v_new = to_device(np.stack([self.m.tables(tr, ver)["v"][p] for tr, p in zip(active, pos)]), device=self.dev)
        self.k_cache[page, :, off, :] = k_new
        self.v_cache[page, :, off, :] = v_new
        C = len(active)
        q = to_device(np.stack([self.m.tables(tr, ver)["q"][p] for tr, p in zip(active, pos)]), device=self.dev)
        ctx = to_device(np.asarray([p + 1 for p in pos], dtype=np.int32), device=self.dev)
        out = torch.empty_like(q)
        lse = torch.empty((C, self.m.Hq), dtype=torch.float32, device=self.dev)
        binding.decode_attn(q, self.k_cache, self.v_cache, self._table(active), ctx, out, lse, self.attn_ws,
                            scale=self.m.scale, dtype=self.dt)
        hidden = to_device(np.stack([self.m.tables(tr, ver)["hidden"][p] for tr, p in zip(active, pos)]),
                           device=self.dev)
        seq_id = to_device(np.asarray(active, dtype=np.int64), device=self.dev)
        step = to_device(np.asarray([self._gen(tr) for tr in active], dtype=np.int32), device=self.dev)
        token = torch.empty(C, dtype=torch.int32, device=self.dev)
        logp = torch.empty(C, dtype=torch.float32, device=self.dev)
        llse = torch.empty(C, dtype=torch.float32, device=self.dev)
        binding.lmhead_logprob(hidden, self.weight_dev, seq_id, step, token, logp, llse, self.lm_ws,
                               seed=self.sample_seed, temperature=self.temperature, dtype=self.dt)
        torch.cuda.synchronize()
        tok, lp = token.cpu().numpy(), logp.cpu().numpy()
        o, l = out.float().cpu().numpy(), lse.cpu().numpy()
        for r, tr in enumerate(active):
            t = self.traj[tr]
            t.tokens.append(int(tok[r]))
            t.logp.append(float(lp[r]))
            t.tag.append(stage)
            t.attn_out.append(o[r])
            t.attn_lse.append(l[r])

    def _train_batch(self, batch, ver, stage):
        """Eq. 8 and Eq. 2-4 on the inputs that leave: current-policy log-probs of the buffered
        tokens, ratios against the buffered log-probs, clipped surrogate."""
        trs = [i * self.N + s for i in batch for s in range(self.N)]
        lens = [self._gen(tr) for tr in trs]
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        M = int(cu[-1])
        hidden = np.concatenate([self.m.tables(tr, ver)["hidden"][self._prompt(tr):self._prompt(tr) + n]
                                 for tr, n in zip(trs, lens)])
        tokens = np.concatenate([np.asarray(self.traj[tr].tokens, dtype=np.int32) for tr in trs])
        tags = np.concatenate([np.asarray(self.traj[tr].tag, dtype=np.int64) for tr in trs])
        old = np.concatenate([np.asarray(self.traj[tr].logp, dtype=np.float32) for tr in trs])
        split = np.asarray([int((np.asarray(self.traj[tr].tag) < stage).sum()) for tr in trs], dtype=np.int32)
        # Eq. 6: a trajectory's buffer is its per-stage pieces in token order, so the tokens of
        # earlier stages are a prefix; the side of the split that is not selected holds NaN
        logp_buf = np.where(tags < stage, old, np.float32("nan")).astype(np.float32)
        logp_roll = np.where(tags < stage, np.float32("nan"), old).astype(np.float32)
        adv = np.random.default_rng([self.m.seed, 0xAD, stage]).normal(size=len(trs)).astype(np.float32)
        dev = self.dev
        hd, tk = to_device(hidden, device=dev), to_device(tokens, device=dev)
        logp_cur = torch.empty(M, dtype=torch.float32, device=dev)
        lse = torch.empty(M, dtype=torch.float32, device=dev)
        ws = workspace(binding.lmhead_token_logprob_workspace_bytes(M, self.m.H, self.m.V, self.dt), dev)
        binding.lmhead_token_logprob(hd, self.weight_dev, tk, logp_cur, lse, ws, temperature=self.temperature,
                                     dtype=self.dt)
        cud, spd = to_device(cu, device=dev), to_device(split, device=dev)
        bufd, rolld, advd = (to_device(x, device=dev) for x in (logp_buf, logp_roll, adv))
        f = lambda n, t=torch.float32: torch.empty(n, dtype=t, device=dev)
        ratio, clipped, seq_sum = f(M), f(M), f(len(trs))
        seq_cnt, seq_nclip = f(len(trs), torch.int32), f(len(trs), torch.int32)
        binding.is_ratio(logp_cur, bufd, rolld, cud, spd, None, ratio, clipped, seq_sum, seq_cnt, seq_nclip,
                         eps_low=self.eps_low, eps_high=self.eps_high)
        surr, grad, seq_surr, seq_cnt2, obj = f(M), f(M), f(len(trs)), f(len(trs), torch.int32), f(2)
        binding.grpo_surrogate(logp_cur, bufd, rolld, cud, spd, None, advd, surr, grad, seq_surr, seq_cnt2, obj,
                               eps_low=self.eps_low, eps_high=self.eps_high)
        torch.cuda.synchronize()
        g = lambda t: t.cpu().numpy()
        return {"trajectories": trs, "cu_seqlens": cu, "split": split, "tokens": tokens, "tags": tags,
                "hidden": hidden, "logp_buf": logp_buf, "logp_roll": logp_roll, "adv": adv,
                "logp_cur": g(logp_cur), "ratio": g(ratio), "ratio_clipped": g(clipped), "seq_sum": g(seq_sum),
                "seq_cnt": g(seq_cnt), "seq_nclip": g(seq_nclip), "surr": g(surr), "grad": g(grad),
                "seq_surr": g(seq_surr), "obj_token_mean": float(g(obj)[0]), "obj_seq_mean": float(g(obj)[1])}

    # ---- the loop --------------------------------------------------------------------------
    def run(self, max_stages: int):
        for stage in range(max_stages):
            ver = stage                              # one policy version per rollout stage
            self.weight_dev = to_device(self.m.weight(ver), device=self.dev)
            T = len(self.traj)
            resume_q = [tr for tr in range(T) if not self.consumed[tr // self.N] and self.traj[tr].started
                        and self._gen(tr) < self._target(tr)]
            fresh_q = [tr for tr in range(T) if not self.traj[tr].started]
            queue, n_resume, qpos = resume_q + fresh_q, len(resume_q), 0
            st = {"steps": 0, "generated": 0, "slot_steps_idle": 0, "resumed": 0, "reprefill_tokens": 0,
                  "peak_pages": 0}
            plan = []                                # per decode step: (entered, their prefill lengths, active)
            active = []
            done = self._complete_inputs() if len(self._complete_inputs()) >= self.batch_inputs else None
            while done is None:
                entered = []
                while len(active) < self.pool and qpos < len(queue):
                    tr = queue[qpos]
                    if qpos < n_resume:
                        st["resumed"] += 1
                        st["reprefill_tokens"] += self._prompt(tr) + self._gen(tr)
                    qpos += 1
                    self.traj[tr].started = True
                    active.append(tr)
                    entered.append(tr)
                if not active:
                    break
                lens = self._prefill(entered, ver)[0] if entered else []
                self._decode_step(active, ver, stage)
                plan.append({"entered": list(entered), "prefill_len": list(lens), "active": list(active)})
                st["steps"] += 1
                st["slot_steps_idle"] += self.pool - len(active)
                st["generated"] += len(active)
                st["peak_pages"] = max(st["peak_pages"], sum(len(self.pages_of[tr]) for tr in active))
                for tr in active:
                    if self._gen(tr) >= self._target(tr):
                        self._release(tr)
                active = [tr for tr in active if self._gen(tr) < self._target(tr)]
                ci = self._complete_inputs()
                if len(ci) >= self.batch_inputs:
                    done = ci
            if done is None:
                break
            for tr in active:                        # paused: their pages die with the policy version
                self._release(tr)
            batch = done[:self.batch_inputs]
            train = self._train_batch(batch, ver, stage)
            tags = train["tags"]
            st["batch_inputs"] = batch
            st["batch_tokens"] = int(tags.size)
            st["batch_offpolicy"] = int((tags < stage).sum())
            st["batch_traj_offpolicy"] = int((train["split"] > 0).sum())
            st["max_staleness"] = int((stage - tags).max()) if tags.size else 0
            for i in batch:
                self.consumed[i] = True
            live = [tr for tr in range(T) if not self.consumed[tr // self.N] and self.traj[tr].started]
            st["paused"] = sum(1 for tr in live if self._gen(tr) < self._target(tr))
            st["buffered_complete"] = sum(1 for tr in live if self._gen(tr) >= self._target(tr))
            self.stages.append({"stats": st, "plan": plan, "train": train, "version": ver})
        return self.stages
