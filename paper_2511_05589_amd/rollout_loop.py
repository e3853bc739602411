"""Rollout stages under the library's rollout manager, with the pool state and the buffer of
partial trajectories resident on the device (Section 4: Concurrency-Controlled Generation,
Early Termination, Buffering of Partial Trajectories with Eq. 6, Prioritized Resumption;
Eq. 8 and Eq. 2-4 on the training batch).

Who does what:

  * `copris_rollout_*` (host C++) takes every scheduling decision: the trajectory in every
    pool slot, what enters and is (re-)prefilled, the KV pages of every request, when the
    stage stops, which inputs leave as the batch and how many of each trajectory's tokens
    come from earlier stages.  This module asks it before every step and decides nothing.
  * The device keeps, between steps, the per-slot state (`seq_id`, `ctx_len`, `step`, block
    table) and the buffer rows of every trajectory (token, log-prob, stage tag).  Per step it
    runs `copris_rollout_apply` (the manager's commands), `copris_prefill_attn` for entering
    requests, `copris_kv_append`, `copris_decode_attn`, `copris_lmhead_logprob` and
    `copris_traj_append`; per batch `copris_traj_gather`, `copris_lmhead_token_logprob`,
    `copris_is_ratio` and `copris_grpo_surrogate`.  Nothing is read back inside a stage; the
    host waits for the device once per stage, when it collects the batch's results.
  * The transformer is a stand-in (`workloads.StandInPolicy`): query, key, value and final
    hidden state of a trajectory position are seeded noise per policy version, held in
    device tables here and looked up by row; a trajectory ends at a given length, which is
    what lets the manager plan a stage without waiting for tokens.

With `graph=True` the steps of a stage in which no request enters - all but a few - are one
HIP graph, captured once per stage and replayed: the manager's commands of such a step fit a
fixed-size buffer (at most one slot command and one new page per slot; unused entries name
slot -1, which `copris_rollout_apply` skips), so the host's work per step is `next_step`, one
small copy and the replay.

Sized for small cases (the stand-in tables of every trajectory are resident).
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding
from .runner import dtype_code, require_gpu, to_device, workspace
from .workloads import BF16, StandInPolicy


def _upload(a: np.ndarray, dev) -> torch.Tensor:
    """Host array -> device through pinned memory, without waiting for the stream."""
    return torch.from_numpy(np.ascontiguousarray(a)).pin_memory().to(dev, non_blocking=True)


class _DeviceTables:
    """The stand-in model of one policy version on the device: the rows of all trajectories
    back to back, `row0[tr]` being the first row of trajectory tr."""

    def __init__(self, policy: StandInPolicy, ver: int, dev):
        n_traj = policy.resp_len.size
        lens = [policy.length(tr) for tr in range(n_traj)]
        self.row0_host = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        cat = lambda key: to_device(np.concatenate([policy.tables(tr, ver)[key] for tr in range(n_traj)]), device=dev)
        self.q, self.k, self.v, self.hidden = cat("q"), cat("k"), cat("v"), cat("hidden")
        self.row0 = to_device(self.row0_host[:-1], device=dev)
        self.weight = to_device(policy.weight(ver), device=dev)


class RolloutLoop:
    def __init__(self, policy: StandInPolicy, pool: int, batch_inputs: int, *, sample_seed: int = 7,
                 temperature: float = 1.0, eps_low: float = 0.2, eps_high: float = 0.28,
                 page_size: int = 16, page_seed: int = 11, record: bool = True, graph: bool = False):
        self.m = policy
        self.pool, self.batch_inputs = int(pool), int(batch_inputs)
        self.sample_seed, self.temperature = int(sample_seed), float(temperature)
        self.eps_low, self.eps_high = float(eps_low), float(eps_high)
        self.page_size = int(page_size)
        self.record = bool(record)
        self.graph = bool(graph)
        if self.graph and self.record:
            raise ValueError("graph=True replays captured steps: per-step outputs cannot be recorded")
        self.dev = dev = require_gpu()
        self.dt = dtype_code(policy.dtype)
        self.N = policy.samples
        self.n_traj = int(policy.resp_len.size)
        self.max_resp = int(policy.resp_len.max())
        longest = int((policy.prompt_len[:, None] + policy.resp_len).max())
        self.num_pages = self.pool * ((longest + page_size - 1) // page_size) + 3
        # physical pages are handed out in a shuffled order, so block tables are scattered
        order = np.random.default_rng(page_seed).permutation(self.num_pages)
        self.manager = binding.RolloutManager(policy.prompt_len, policy.resp_len, self.pool, self.batch_inputs,
                                              page_size, num_pages=self.num_pages, page_order=order)
        self.max_pages = self.manager.max_pages
        tdt = torch.bfloat16 if policy.dtype == BF16 else torch.float32
        shape = (self.num_pages, policy.Hkv, page_size, policy.D)
        self.k_cache = torch.full(shape, float("nan"), dtype=tdt, device=dev)
        self.v_cache = torch.full(shape, float("nan"), dtype=tdt, device=dev)
        # pool state
        self.seq_id = torch.full((self.pool,), -1, dtype=torch.int64, device=dev)
        self.ctx_len = torch.zeros(self.pool, dtype=torch.int32, device=dev)
        self.step = torch.zeros(self.pool, dtype=torch.int32, device=dev)
        self.block_table = torch.zeros((self.pool, self.max_pages), dtype=torch.int32, device=dev)
        # the buffer: one row per trajectory
        self.buf_token = torch.full((self.n_traj, self.max_resp), -1, dtype=torch.int32, device=dev)
        self.buf_logp = torch.full((self.n_traj, self.max_resp), float("nan"), dtype=torch.float32, device=dev)
        self.buf_tag = torch.full((self.n_traj, self.max_resp), -1, dtype=torch.int32, device=dev)
        # per-step outputs
        self.attn_out = torch.empty((self.pool, policy.Hq, policy.D), dtype=tdt, device=dev)
        self.attn_lse = torch.empty((self.pool, policy.Hq), dtype=torch.float32, device=dev)
        self.token = torch.empty(self.pool, dtype=torch.int32, device=dev)
        self.logprob = torch.empty(self.pool, dtype=torch.float32, device=dev)
        self.attn_ws = workspace(binding.decode_attn_workspace_bytes(
            self.pool, policy.Hq, policy.Hkv, policy.D, page_size, self.max_pages), dev)
        self.lm_ws = workspace(binding.lmhead_logprob_workspace_bytes(self.pool, policy.H, policy.V), dev)
        self.stages = []
        self.host_syncs = 0                  # times the host waited for the device
        # graph mode: the fixed-size command buffer of a captured step (pool slot commands of 4
        # ints, then pool page commands of 3), and a ring of pinned host copies of it
        self.cmd_words = 7 * self.pool
        self.cmd_dev = torch.full((self.cmd_words,), -1, dtype=torch.int32, device=dev) if self.graph else None
        self.cmd_ring = torch.full((256, self.cmd_words), -1, dtype=torch.int32).pin_memory() if self.graph else None
        self.cmd_ring_np = self.cmd_ring.numpy() if self.graph else None
        self.cmd_events = [None] * 256
        self.cmd_next = 0
        self.graph_steps = 0                 # steps that ran as a graph replay

    # ---- one decode step, all on the stream, nothing read back ---------------------------
    def _prefill(self, plan, tab):
        ent = plan["entered"][plan["entered"][:, 2] > 0]
        if ent.shape[0] == 0:
            return
        lens = ent[:, 2].astype(np.int64)
        rows = np.concatenate([tab.row0_host[t] + np.arange(n) for t, n in zip(ent[:, 1], lens)])
        idx = _upload(rows, self.dev)
        cu = _upload(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32), self.dev)
        table = self.block_table.index_select(0, _upload(ent[:, 0].astype(np.int64), self.dev))
        q, k, v = tab.q.index_select(0, idx), tab.k.index_select(0, idx), tab.v.index_select(0, idx)
        binding.prefill_attn(q, k, v, cu, table, self.k_cache, self.v_cache, torch.empty_like(q), None,
                             max_seqlen=int(lens.max()), scale=self.m.scale, dtype=self.dt)

    def _decode_step(self, plan, tab, stage, log):
        binding.rollout_apply(_upload(plan["cmds"], self.dev), plan["n_slot_cmds"], plan["n_page_cmds"],
                              self.seq_id, self.ctx_len, self.step, self.block_table)
        self._prefill(plan, tab)
        self._forward_and_sample(tab, stage, log)

    def _forward_and_sample(self, tab, stage, log):
        # the stand-in's forward pass for the position being decoded: a row look-up
        row = tab.row0.index_select(0, self.seq_id.clamp(min=0)) + (self.ctx_len - 1).clamp(min=0)
        q, hidden = tab.q.index_select(0, row), tab.hidden.index_select(0, row)
        binding.kv_append(tab.k.index_select(0, row), tab.v.index_select(0, row), self.block_table, self.ctx_len,
                          self.k_cache, self.v_cache, dtype=self.dt)
        binding.decode_attn(q, self.k_cache, self.v_cache, self.block_table, self.ctx_len, self.attn_out,
                            self.attn_lse, self.attn_ws, scale=self.m.scale, dtype=self.dt)
        binding.lmhead_logprob(hidden, tab.weight, self.seq_id, self.step, self.token, self.logprob, None,
                               self.lm_ws, seed=self.sample_seed, temperature=self.temperature, dtype=self.dt)
        if self.record:
            log.append((self.attn_out.float(), self.attn_lse.clone()))
        binding.traj_append(self.token, self.logprob, self.seq_id, self.step, self.ctx_len, stage,
                            self.buf_token, self.buf_logp, self.buf_tag)

    # ---- graph mode: a step without entering requests ----------------------------------------
    def _fits_graph(self, plan) -> bool:
        return (plan["entered"].shape[0] == 0 and plan["n_slot_cmds"] <= self.pool
                and plan["n_page_cmds"] <= self.pool)

    def _stage_commands(self, plan):
        """The plan's commands, padded to the captured step's fixed layout, in the next pinned
        ring entry; returns that entry (a pinned host tensor)."""
        i = self.cmd_next
        self.cmd_next = (i + 1) % len(self.cmd_events)
        if self.cmd_events[i] is not None:
            self.cmd_events[i].synchronize()     # (the copy that last read this entry; long done)
        row = self.cmd_ring_np[i]
        row.fill(-1)
        ns, npg = plan["n_slot_cmds"], plan["n_page_cmds"]
        cmds = plan["cmds"]
        row[:4 * ns] = cmds[:4 * ns]
        row[4 * self.pool:4 * self.pool + 3 * npg] = cmds[4 * ns:4 * ns + 3 * npg]
        return i

    def _graph_step(self, plan, tab, stage, state):
        i = self._stage_commands(plan)
        self.cmd_dev.copy_(self.cmd_ring[i], non_blocking=True)
        ev = torch.cuda.Event()
        ev.record()
        self.cmd_events[i] = ev
        if state.get("graph") is None:
            # capture this stage's step: commands -> pool state, forward pass, append, attention,
            # sampling, buffer append (the stage tag and the policy's tables are fixed for a stage)
            g = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.graph(g, stream=side):
                binding.rollout_apply(self.cmd_dev, self.pool, self.pool, self.seq_id, self.ctx_len, self.step,
                                      self.block_table)
                self._forward_and_sample(tab, stage, None)
            torch.cuda.current_stream().wait_stream(side)
            state["graph"] = g
        state["graph"].replay()
        self.graph_steps += 1

    # ---- Eq. 8 and Eq. 2-4 on the batch that leaves ------------------------------------------
    def _train_batch(self, st, tab, stage):
        bt = st["batch_traj"]
        trs, lens = bt[:, 0], bt[:, 1].astype(np.int64)
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        M, B, dev = int(cu[-1]), len(trs), self.dev
        f = lambda n, t=torch.float32: torch.empty(n, dtype=t, device=dev)
        cud, trd = _upload(cu, dev), _upload(trs.astype(np.int32), dev)
        tokens, logp_buf, logp_roll, split = f(M, torch.int32), f(M), f(M), f(B, torch.int32)
        binding.traj_gather(self.buf_token, self.buf_logp, self.buf_tag, trd, cud, stage, tokens, logp_buf,
                            logp_roll, split)
        prompt = self.m.prompt_len[trs // self.N]
        rows = np.concatenate([tab.row0_host[t] + p + np.arange(n) for t, p, n in zip(trs, prompt, lens)])
        hidden = tab.hidden.index_select(0, _upload(rows, dev))
        adv_host = np.random.default_rng([self.m.seed, 0xAD, stage]).normal(size=B).astype(np.float32)
        adv = _upload(adv_host, dev)
        logp_cur, lse = f(M), f(M)
        ws = workspace(binding.lmhead_token_logprob_workspace_bytes(M, self.m.H, self.m.V, self.dt), dev)
        binding.lmhead_token_logprob(hidden, tab.weight, tokens, logp_cur, lse, ws, temperature=self.temperature,
                                     dtype=self.dt)
        ratio, clipped, seq_sum = f(M), f(M), f(B)
        seq_cnt, seq_nclip = f(B, torch.int32), f(B, torch.int32)
        binding.is_ratio(logp_cur, logp_buf, logp_roll, cud, split, None, ratio, clipped, seq_sum, seq_cnt,
                         seq_nclip, eps_low=self.eps_low, eps_high=self.eps_high)
        surr, grad, seq_surr, seq_cnt2, obj = f(M), f(M), f(B), f(B, torch.int32), f(2)
        binding.grpo_surrogate(logp_cur, logp_buf, logp_roll, cud, split, None, adv, surr, grad, seq_surr,
                               seq_cnt2, obj, eps_low=self.eps_low, eps_high=self.eps_high)
        torch.cuda.synchronize()             # the one wait of the stage
        self.host_syncs += 1
        g = lambda t: t.cpu().numpy()
        out = {"trajectories": trs.tolist(), "cu_seqlens": cu, "split": g(split), "manager_split": bt[:, 2].copy(),
               "tokens": g(tokens), "logp_buf": g(logp_buf), "logp_roll": g(logp_roll), "adv": adv_host,
               "logp_cur": g(logp_cur), "ratio": g(ratio), "ratio_clipped": g(clipped), "seq_sum": g(seq_sum),
               "seq_cnt": g(seq_cnt), "seq_nclip": g(seq_nclip), "surr": g(surr), "grad": g(grad),
               "seq_surr": g(seq_surr), "obj_token_mean": float(g(obj)[0]), "obj_seq_mean": float(g(obj)[1])}
        if self.record:
            tag_rows = g(self.buf_tag)
            out["tags"] = np.concatenate([tag_rows[t, :n] for t, n in zip(trs, lens)]) if B else np.zeros(0, np.int32)
            out["hidden"] = np.concatenate([self.m.tables(t, stage)["hidden"][p:p + n]
                                            for t, p, n in zip(trs, prompt, lens)])
        return out

    # ---- stages ------------------------------------------------------------------------------
    def run(self, max_stages: int):
        for _ in range(max_stages):
            stage = self.manager.begin_stage()
            tab = _DeviceTables(self.m, stage, self.dev)        # one policy version per stage
            plans, log, state = [], [], {}
            while True:
                # (graph mode keeps no per-step record, so the plan may alias the manager's arrays)
                code, plan = self.manager.next_step(copy=not self.graph)
                if code != binding.ROLLOUT_STEP:
                    break
                if self.graph and self._fits_graph(plan):
                    self._graph_step(plan, tab, stage, state)
                else:
                    self._decode_step(plan, tab, stage, log)
                if not self.graph:
                    plans.append(plan)
            state.clear()                        # (the stage's graph goes with its tables)
            if code == binding.ROLLOUT_EXHAUSTED:
                break
            st = self.manager.end_stage()
            train = self._train_batch(st, tab, stage)
            steps = [{"slot_traj": p["slot_traj"], "entered": p["entered"], "finishing": p["finishing"]}
                     for p in plans]
            if self.record:
                for s, (o, l) in zip(steps, log):
                    s["attn_out"], s["attn_lse"] = o.cpu().numpy(), l.cpu().numpy()
            self.stages.append({"stats": {k: v for k, v in st.items() if k != "batch_traj"}, "steps": steps,
                                "train": train, "version": stage})
        return self.stages

    def buffers(self):
        """The buffer rows as host arrays: (tokens, log-probs, stage tags), [n_traj, max_resp]."""
        return self.buf_token.cpu().numpy(), self.buf_logp.cpu().numpy(), self.buf_tag.cpu().numpy()
