"""Device staging for the binding: numpy workload arrays -> HBM tensors -> one call
through the C ABI -> numpy results.  Plumbing only (allocation, copies, dtype
views); all arithmetic happens inside libcopris.so.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

from . import binding
from .workloads import BF16, F32


def require_gpu() -> torch.device:
    if not torch.cuda.is_available():
        raise RuntimeError("libcopris needs an MI355X (no CPU fallback exists)")
    return torch.device("cuda:0")


def dtype_code(dtype: str) -> int:
    return {F32: binding.COPRIS_F32, BF16: binding.COPRIS_BF16}[dtype]


def to_device(a: np.ndarray, dtype: Optional[str] = None, device=None) -> torch.Tensor:
    """Upload a storage array; bf16 bit patterns (uint16) become torch.bfloat16."""
    device = device or require_gpu()
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def out_to_f32(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy()


def workspace(nbytes: int, device=None) -> torch.Tensor:
    device = device or require_gpu()
    # torch's caching allocator hands out blocks aligned to at least 512 bytes
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


@dataclass
class AttnDevice:
    q: torch.Tensor
    k_cache: torch.Tensor
    v_cache: torch.Tensor
    block_table: torch.Tensor
    ctx_len: torch.Tensor
    out: torch.Tensor
    lse: torch.Tensor
    ws: torch.Tensor
    scale: float
    dtype: int

    def run(self, stream=None):
        binding.decode_attn(self.q, self.k_cache, self.v_cache, self.block_table, self.ctx_len,
                            self.out, self.lse, self.ws, scale=self.scale, dtype=self.dtype,
                            stream=stream)


def stage_attn(inp: dict, dtype: str, device=None) -> AttnDevice:
    device = device or require_gpu()
    q = to_device(inp["q"], device=device)
    k = to_device(inp["k_cache"], device=device)
    v = to_device(inp["v_cache"], device=device)
    bt = to_device(inp["block_table"].astype(np.int32), device=device)
    ctx = to_device(inp["ctx_len"].astype(np.int32), device=device)
    C, Hq, D = q.shape
    _, Hkv, P, _ = k.shape
    out = torch.full_like(q, float("nan"))
    lse = torch.full((C, Hq), float("nan"), dtype=torch.float32, device=device)
    ws = workspace(binding.decode_attn_workspace_bytes(C, Hq, Hkv, D, P, bt.shape[1]), device)
    return AttnDevice(q, k, v, bt, ctx, out, lse, ws, float(inp["scale"]), dtype_code(dtype))


def run_decode_attn(inp: dict, dtype: str):
    """One copris_decode_attn call; returns (out fp32 ndarray, lse ndarray)."""
    d = stage_attn(inp, dtype)
    d.run()
    torch.cuda.synchronize()
    return out_to_f32(d.out), d.lse.cpu().numpy()


@dataclass
class LmDevice:
    hidden: torch.Tensor
    weight: torch.Tensor
    seq_id: torch.Tensor
    step: torch.Tensor
    token: torch.Tensor
    logprob: torch.Tensor
    lse: torch.Tensor
    ws: torch.Tensor
    seed: int
    temperature: float
    dtype: int

    def run(self, stream=None):
        binding.lmhead_logprob(self.hidden, self.weight, self.seq_id, self.step, self.token,
                               self.logprob, self.lse, self.ws, seed=self.seed,
                               temperature=self.temperature, dtype=self.dtype, stream=stream)


def stage_lmhead(inp: dict, dtype: str, device=None) -> LmDevice:
    device = device or require_gpu()
    hidden = to_device(inp["hidden"], device=device)
    weight = to_device(inp["weight"], device=device)
    seq_id = to_device(np.asarray(inp["seq_id"], dtype=np.int64), device=device)
    step = to_device(np.asarray(inp["step"], dtype=np.int32), device=device)
    C, H = hidden.shape
    V = weight.shape[0]
    token = torch.full((C,), -1, dtype=torch.int32, device=device)
    logprob = torch.full((C,), float("nan"), dtype=torch.float32, device=device)
    lse = torch.full((C,), float("nan"), dtype=torch.float32, device=device)
    ws = workspace(binding.lmhead_logprob_workspace_bytes(C, H, V), device)
    return LmDevice(hidden, weight, seq_id, step, token, logprob, lse, ws, int(inp["seed"]),
                    float(inp["temperature"]), dtype_code(dtype))


def run_lmhead_logprob(inp: dict, dtype: str):
    d = stage_lmhead(inp, dtype)
    d.run()
    torch.cuda.synchronize()
    return d.token.cpu().numpy(), d.logprob.cpu().numpy(), d.lse.cpu().numpy()


@dataclass
class IsDevice:
    logp_cur: torch.Tensor
    logp_buf: torch.Tensor
    logp_roll: torch.Tensor
    cu_seqlens: torch.Tensor
    split: torch.Tensor
    mask: Optional[torch.Tensor]
    ratio: torch.Tensor
    ratio_clipped: torch.Tensor
    seq_sum: torch.Tensor
    seq_cnt: torch.Tensor
    seq_nclip: torch.Tensor
    eps_low: float
    eps_high: float

    def run(self, stream=None):
        binding.is_ratio(self.logp_cur, self.logp_buf, self.logp_roll, self.cu_seqlens, self.split,
                         self.mask, self.ratio, self.ratio_clipped, self.seq_sum, self.seq_cnt,
                         self.seq_nclip, eps_low=self.eps_low, eps_high=self.eps_high, stream=stream)


def stage_is_ratio(b: dict, device=None, use_mask: bool = True) -> IsDevice:
    device = device or require_gpu()
    N, B = int(b["N"]), int(b["B"])
    f = lambda k: to_device(np.asarray(b[k], dtype=np.float32), device=device)
    mask = to_device(np.asarray(b["mask"], dtype=np.uint8), device=device) if (
        use_mask and b.get("mask") is not None) else None
    nanf = lambda n: torch.full((max(n, 1),), float("nan"), dtype=torch.float32, device=device)
    return IsDevice(f("logp_cur"), f("logp_buf"), f("logp_roll"),
                    to_device(np.asarray(b["cu_seqlens"], dtype=np.int32), device=device),
                    to_device(np.asarray(b["split"], dtype=np.int32), device=device), mask,
                    nanf(N), nanf(N), nanf(B),
                    torch.full((max(B, 1),), -7, dtype=torch.int32, device=device),
                    torch.full((max(B, 1),), -7, dtype=torch.int32, device=device),
                    float(b["eps_low"]), float(b["eps_high"]))


def run_is_ratio(b: dict, use_mask: bool = True) -> dict:
    d = stage_is_ratio(b, use_mask=use_mask)
    d.run()
    torch.cuda.synchronize()
    N, B = int(b["N"]), int(b["B"])
    return {"ratio": d.ratio.cpu().numpy()[:N], "ratio_clipped": d.ratio_clipped.cpu().numpy()[:N],
            "seq_sum": d.seq_sum.cpu().numpy()[:B], "seq_cnt": d.seq_cnt.cpu().numpy()[:B],
            "seq_nclip": d.seq_nclip.cpu().numpy()[:B]}


@dataclass
class GrpoDevice:
    logp_cur: torch.Tensor
    logp_buf: torch.Tensor
    logp_roll: torch.Tensor
    cu_seqlens: torch.Tensor
    split: torch.Tensor
    mask: Optional[torch.Tensor]
    adv: torch.Tensor
    surr: torch.Tensor
    grad: torch.Tensor
    seq_surr: torch.Tensor
    seq_cnt: torch.Tensor
    objective: torch.Tensor
    eps_low: float
    eps_high: float

    def run(self, stream=None):
        binding.grpo_surrogate(self.logp_cur, self.logp_buf, self.logp_roll, self.cu_seqlens,
                               self.split, self.mask, self.adv, self.surr, self.grad, self.seq_surr,
                               self.seq_cnt, self.objective, eps_low=self.eps_low,
                               eps_high=self.eps_high, stream=stream)


def stage_grpo_surrogate(b: dict, device=None, use_mask: bool = True) -> GrpoDevice:
    device = device or require_gpu()
    N, B = int(b["N"]), int(b["B"])
    f = lambda k: to_device(np.asarray(b[k], dtype=np.float32), device=device)
    mask = to_device(np.asarray(b["mask"], dtype=np.uint8), device=device) if (
        use_mask and b.get("mask") is not None) else None
    nanf = lambda n: torch.full((max(n, 1),), float("nan"), dtype=torch.float32, device=device)
    return GrpoDevice(f("logp_cur"), f("logp_buf"), f("logp_roll"),
                      to_device(np.asarray(b["cu_seqlens"], dtype=np.int32), device=device),
                      to_device(np.asarray(b["split"], dtype=np.int32), device=device), mask,
                      f("adv") if B > 0 else nanf(1), nanf(N), nanf(N), nanf(B),
                      torch.full((max(B, 1),), -7, dtype=torch.int32, device=device), nanf(2),
                      float(b["eps_low"]), float(b["eps_high"]))


def run_grpo_surrogate(b: dict, use_mask: bool = True) -> dict:
    d = stage_grpo_surrogate(b, use_mask=use_mask)
    d.run()
    torch.cuda.synchronize()
    N, B = int(b["N"]), int(b["B"])
    obj = d.objective.cpu().numpy()
    return {"surr": d.surr.cpu().numpy()[:N], "grad": d.grad.cpu().numpy()[:N],
            "seq_surr": d.seq_surr.cpu().numpy()[:B], "seq_cnt": d.seq_cnt.cpu().numpy()[:B],
            "obj_token_mean": float(obj[0]), "obj_seq_mean": float(obj[1])}


@dataclass
class TokenLogprobDevice:
    hidden: torch.Tensor
    weight: torch.Tensor
    tokens: torch.Tensor
    logprob: torch.Tensor
    lse: torch.Tensor
    ws: torch.Tensor
    temperature: float
    dtype: int

    def run(self, stream=None):
        binding.lmhead_token_logprob(self.hidden, self.weight, self.tokens, self.logprob, self.lse,
                                     self.ws, temperature=self.temperature, dtype=self.dtype,
                                     stream=stream)


def stage_token_logprob(hidden, weight, tokens, temperature: float, dtype: str, device=None,
                        weight_dev: Optional[torch.Tensor] = None) -> TokenLogprobDevice:
    """hidden / weight are storage arrays (bf16 as uint16 bit patterns); weight_dev lets a
    caller reuse a weight tensor that is already on the device."""
    device = device or require_gpu()
    h = to_device(hidden, device=device)
    w = weight_dev if weight_dev is not None else to_device(weight, device=device)
    t = to_device(np.asarray(tokens, dtype=np.int32), device=device)
    M, H = h.shape
    V = w.shape[0]
    code = dtype_code(dtype)
    logprob = torch.full((M,), float("nan"), dtype=torch.float32, device=device)
    lse = torch.full((M,), float("nan"), dtype=torch.float32, device=device)
    ws = workspace(binding.lmhead_token_logprob_workspace_bytes(M, H, V, code), device)
    return TokenLogprobDevice(h, w, t, logprob, lse, ws, float(temperature), code)


def run_token_logprob(hidden, weight, tokens, temperature: float, dtype: str):
    d = stage_token_logprob(hidden, weight, tokens, temperature, dtype)
    d.run()
    torch.cuda.synchronize()
    return d.logprob.cpu().numpy(), d.lse.cpu().numpy()


@dataclass
class PrefillDevice:
    q: torch.Tensor
    k: torch.Tensor
    v: torch.Tensor
    cu_seqlens: torch.Tensor
    block_table: torch.Tensor
    k_cache: torch.Tensor
    v_cache: torch.Tensor
    out: torch.Tensor
    lse: torch.Tensor
    max_seqlen: int
    scale: float
    dtype: int

    def run(self, stream=None):
        binding.prefill_attn(self.q, self.k, self.v, self.cu_seqlens, self.block_table, self.k_cache,
                             self.v_cache, self.out, self.lse, max_seqlen=self.max_seqlen,
                             scale=self.scale, dtype=self.dtype, stream=stream)


def stage_prefill_attn(b: dict, dtype: str, device=None) -> PrefillDevice:
    """b: q [T,Hq,D], k, v [T,Hkv,D] (storage arrays), cu_seqlens, block_table, num_pages,
    page_size, scale.  The caches start as NaN so that untouched slots stay recognisable."""
    device = device or require_gpu()
    q, k, v = (to_device(b[x], device=device) for x in ("q", "k", "v"))
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    shape = (int(b["num_pages"]), Hkv, int(b["page_size"]), D)
    kc = torch.full(shape, float("nan"), dtype=q.dtype, device=device)
    vc = torch.full(shape, float("nan"), dtype=q.dtype, device=device)
    out = torch.full_like(q, float("nan"))
    lse = torch.full((max(T, 1), Hq), float("nan"), dtype=torch.float32, device=device)
    lens = np.diff(np.asarray(b["cu_seqlens"], dtype=np.int64))
    return PrefillDevice(q, k, v, to_device(np.asarray(b["cu_seqlens"], dtype=np.int32), device=device),
                         to_device(np.asarray(b["block_table"], dtype=np.int32), device=device), kc, vc,
                         out, lse, int(max(lens.max(initial=1), 1)), float(b["scale"]), dtype_code(dtype))


def run_prefill_attn(b: dict, dtype: str):
    """Returns (out fp32 [T,Hq,D], lse [T,Hq], k_cache, v_cache as float32 arrays)."""
    d = stage_prefill_attn(b, dtype)
    d.run()
    torch.cuda.synchronize()
    return (out_to_f32(d.out), d.lse.cpu().numpy(), out_to_f32(d.k_cache), out_to_f32(d.v_cache))
