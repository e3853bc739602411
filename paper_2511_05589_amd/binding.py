"""Thin ctypes binding of libcopris.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels.  PyTorch is used for
device memory and stream handles, nothing else.  There is no CPU fallback: if
the shared library is missing the import of a symbol fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_char_p, c_float, c_int, c_int64, c_size_t, c_uint64, c_void_p
from typing import Optional

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libcopris.so")

COPRIS_OK = 0
COPRIS_EINVAL = -1
COPRIS_EWORKSPACE = -2
COPRIS_EUNSUPPORTED = -3
COPRIS_ELAUNCH = -4
COPRIS_F32 = 0
COPRIS_BF16 = 1

# name -> (restype, argtypes), mirroring include/copris.h
SIGNATURES = {
    "copris_strerror": (c_char_p, [c_int]),
    "copris_version": (c_char_p, []),
    "copris_last_error_detail": (c_char_p, []),
    "copris_set_launch_hook": (None, [c_void_p, c_void_p]),
    "copris_decode_attn_workspace_bytes": (c_size_t, [c_int] * 6),
    "copris_decode_attn": (c_int, [c_void_p] * 8 + [c_size_t] + [c_int] * 6 + [c_int64, c_float, c_int, c_void_p]),
    "copris_prefill_attn": (c_int, [c_void_p] * 9 + [c_int, c_int64] + [c_int] * 5 + [c_int64, c_int, c_float,
                                                                                     c_int, c_void_p]),
    "copris_lmhead_logprob_workspace_bytes": (c_size_t, [c_int] * 3),
    "copris_lmhead_logprob": (c_int, [c_void_p] * 4 + [c_uint64, c_float] + [c_void_p] * 4
                              + [c_size_t] + [c_int] * 4 + [c_void_p]),
    "copris_lmhead_token_logprob_workspace_bytes": (c_size_t, [c_int] * 4),
    "copris_lmhead_token_logprob": (c_int, [c_void_p] * 3 + [c_float] + [c_void_p] * 3 + [c_size_t]
                                    + [c_int] * 4 + [c_void_p]),
    "copris_is_ratio": (c_int, [c_void_p] * 6 + [c_float, c_float] + [c_void_p] * 5
                        + [c_int, c_int64, c_void_p]),
    "copris_grpo_surrogate": (c_int, [c_void_p] * 7 + [c_float, c_float] + [c_void_p] * 5
                              + [c_int, c_int64, c_void_p]),
}



class StageStats(ctypes.Structure):
    """copris_stage_stats of include/copris.h."""
    _fields_ = [(n, c_int64) for n in (
        "steps", "generated", "slot_steps_idle", "batch_tokens", "batch_offpolicy",
        "batch_traj_offpolicy", "max_staleness", "resumed", "reprefill_tokens", "paused",
        "buffered_complete", "peak_pages")]


SIGNATURES["copris_rollout_schedule"] = (c_int, [c_void_p, c_void_p] + [c_int] * 6 + [c_void_p] * 3)

_lib = None


class CoprisError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        detail = load_library().copris_last_error_detail().decode() if code == COPRIS_ELAUNCH else ""
        super().__init__(f"{where}: {strerror(code)} (code {code}) {detail}".rstrip())


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load libcopris.so (built in-tree by paper_2511_05589_amd.build) and type its symbols."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} not found: build it with `python -m paper_2511_05589_amd.build` "
            "(there is no fallback path)")
    # PyTorch ships its own HIP runtime (same soname as the system one).  Import it
    # first so that the loader binds libcopris to that already-loaded copy: two HIP
    # runtimes in one process cannot share streams or device memory.
    import torch  # noqa: F401
    lib = ctypes.CDLL(path)
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)          # AttributeError if the symbol is not exported
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load_library().copris_strerror(int(code)).decode()


def version() -> str:
    return load_library().copris_version().decode()


LAUNCH_HOOK = ctypes.CFUNCTYPE(None, c_char_p, c_int, c_void_p, c_void_p)
_hook_ref = None


def set_launch_hook(fn) -> None:
    """fn(kernel: bytes, phase: int, stream: int|None, user) or None to remove the hook."""
    global _hook_ref
    lib = load_library()
    if fn is None:
        lib.copris_set_launch_hook(None, None)
        _hook_ref = None
        return
    _hook_ref = LAUNCH_HOOK(fn)           # keep the trampoline alive
    lib.copris_set_launch_hook(ctypes.cast(_hook_ref, c_void_p), None)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    h = stream.cuda_stream
    return h if h else None


def _check(code: int, where: str) -> None:
    if code != COPRIS_OK:
        raise CoprisError(code, where)


def decode_attn_workspace_bytes(C, Hq, Hkv, D, page_size, max_pages) -> int:
    return int(load_library().copris_decode_attn_workspace_bytes(C, Hq, Hkv, D, page_size, max_pages))


def decode_attn(q, k_cache, v_cache, block_table, ctx_len, out, lse, workspace, *, scale: float,
                dtype: int, stream=None) -> None:
    """copris_decode_attn on device tensors (shapes as in include/copris.h)."""
    C, Hq, D = q.shape
    num_pages, Hkv, page_size, _ = k_cache.shape
    max_pages = block_table.shape[1]
    code = load_library().copris_decode_attn(
        _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_table), _ptr(ctx_len), _ptr(out),
        _ptr(lse), _ptr(workspace), workspace.numel() * workspace.element_size(),
        C, Hq, Hkv, D, page_size, max_pages, num_pages, float(scale), int(dtype), _stream(stream))
    _check(code, "copris_decode_attn")


def lmhead_logprob_workspace_bytes(C, H, V) -> int:
    return int(load_library().copris_lmhead_logprob_workspace_bytes(C, H, V))


def lmhead_logprob(hidden, weight, seq_id, step, token, logprob, lse, workspace, *, seed: int,
                   temperature: float, dtype: int, stream=None) -> None:
    """copris_lmhead_logprob on device tensors."""
    C, H = hidden.shape
    V = weight.shape[0]
    code = load_library().copris_lmhead_logprob(
        _ptr(hidden), _ptr(weight), _ptr(seq_id), _ptr(step), int(seed) & 0xFFFFFFFFFFFFFFFF,
        float(temperature), _ptr(token), _ptr(logprob), _ptr(lse), _ptr(workspace),
        workspace.numel() * workspace.element_size(), C, H, V, int(dtype), _stream(stream))
    _check(code, "copris_lmhead_logprob")


def is_ratio(logp_cur, logp_buf, logp_roll, cu_seqlens, split, mask, ratio, ratio_clipped,
             seq_sum, seq_cnt, seq_nclip, *, eps_low: float, eps_high: float, stream=None) -> None:
    """copris_is_ratio on device tensors."""
    B = cu_seqlens.numel() - 1
    N = logp_cur.numel()
    code = load_library().copris_is_ratio(
        _ptr(logp_cur), _ptr(logp_buf), _ptr(logp_roll), _ptr(cu_seqlens), _ptr(split), _ptr(mask),
        float(eps_low), float(eps_high), _ptr(ratio), _ptr(ratio_clipped), _ptr(seq_sum),
        _ptr(seq_cnt), _ptr(seq_nclip), B, N, _stream(stream))
    _check(code, "copris_is_ratio")


def grpo_surrogate(logp_cur, logp_buf, logp_roll, cu_seqlens, split, mask, adv, surr, grad, seq_surr,
                   seq_cnt, objective, *, eps_low: float, eps_high: float, stream=None) -> None:
    """copris_grpo_surrogate on device tensors."""
    B = cu_seqlens.numel() - 1
    N = logp_cur.numel()
    code = load_library().copris_grpo_surrogate(
        _ptr(logp_cur), _ptr(logp_buf), _ptr(logp_roll), _ptr(cu_seqlens), _ptr(split), _ptr(mask),
        _ptr(adv), float(eps_low), float(eps_high), _ptr(surr), _ptr(grad), _ptr(seq_surr),
        _ptr(seq_cnt), _ptr(objective), B, N, _stream(stream))
    _check(code, "copris_grpo_surrogate")


def lmhead_token_logprob_workspace_bytes(M, H, V, dtype) -> int:
    return int(load_library().copris_lmhead_token_logprob_workspace_bytes(M, H, V, int(dtype)))


def lmhead_token_logprob(hidden, weight, tokens, logprob, lse, workspace, *, temperature: float,
                         dtype: int, stream=None) -> None:
    """copris_lmhead_token_logprob on device tensors."""
    M, H = hidden.shape
    V = weight.shape[0]
    code = load_library().copris_lmhead_token_logprob(
        _ptr(hidden), _ptr(weight), _ptr(tokens), float(temperature), _ptr(logprob), _ptr(lse),
        _ptr(workspace), workspace.numel() * workspace.element_size(), M, H, V, int(dtype),
        _stream(stream))
    _check(code, "copris_lmhead_token_logprob")


def prefill_attn(q, k, v, cu_seqlens, block_table, k_cache, v_cache, out, lse, *, max_seqlen: int,
                 scale: float, dtype: int, stream=None) -> None:
    """copris_prefill_attn on device tensors (shapes as in include/copris.h)."""
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    num_pages, _, page_size, _ = k_cache.shape
    B = cu_seqlens.numel() - 1
    code = load_library().copris_prefill_attn(
        _ptr(q), _ptr(k), _ptr(v), _ptr(cu_seqlens), _ptr(block_table), _ptr(k_cache), _ptr(v_cache),
        _ptr(out), _ptr(lse), B, T, Hq, Hkv, D, page_size, block_table.shape[1], num_pages,
        int(max_seqlen), float(scale), int(dtype), _stream(stream))
    _check(code, "copris_prefill_attn")


def rollout_schedule(prompt_len, resp_len, pool: int, batch_inputs: int, page_size: int = 16,
                     max_stages: Optional[int] = None) -> list:
    """copris_rollout_schedule on host arrays (numpy); returns a list of per-stage dicts."""
    import numpy as np
    p = np.ascontiguousarray(prompt_len, dtype=np.int32)
    r = np.ascontiguousarray(resp_len, dtype=np.int32)
    n_inputs = int(p.size)
    samples = int(r.shape[1]) if r.ndim == 2 and n_inputs else 1
    if max_stages is None:
        max_stages = n_inputs // max(int(batch_inputs), 1) + 1
    stats = (StageStats * max(max_stages, 1))()
    batch = np.zeros((max(max_stages, 1), max(int(batch_inputs), 1)), dtype=np.int32)
    n = c_int(0)
    code = load_library().copris_rollout_schedule(
        p.ctypes.data, r.ctypes.data, n_inputs, samples, int(pool), int(batch_inputs), int(page_size),
        int(max_stages), ctypes.addressof(stats), batch.ctypes.data, ctypes.addressof(n))
    _check(code, "copris_rollout_schedule")
    out = []
    for k in range(n.value):
        d = {name: int(getattr(stats[k], name)) for name, _ in StageStats._fields_}
        d["batch_inputs"] = batch[k].tolist()
        out.append(d)
    return out
