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
# COPRIS_LIB selects another build of the library (e.g. one with host sanitizers)
LIB_PATH = os.environ.get("COPRIS_LIB") or os.path.join(_PKG_DIR, "libcopris.so")

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
    "copris_lmhead_logprob_noalloc_max_bytes": (c_size_t, []),
    "copris_lmhead_logprob_noalloc": (c_int, [c_void_p] * 4 + [c_uint64, c_float] + [c_void_p] * 3
                                      + [c_int] * 4 + [c_void_p]),
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


class RolloutPlan(ctypes.Structure):
    """copris_rollout_plan of include/copris.h."""
    _fields_ = [(n, ctypes.c_int32) for n in ("stage", "n_active", "n_entered", "n_finishing", "n_slot_cmds",
                                              "n_page_cmds")] + [
        (n, ctypes.POINTER(ctypes.c_int32)) for n in ("slot_traj", "entered", "finishing", "cmds", "block_table")]


ROLLOUT_STEP, ROLLOUT_STAGE_END, ROLLOUT_EXHAUSTED = 0, 1, 2
SIGNATURES.update({
    "copris_rollout_create": (c_int, [c_void_p, c_void_p] + [c_int] * 5 + [c_int64, c_void_p, c_void_p]),
    "copris_rollout_destroy": (None, [c_void_p]),
    "copris_rollout_max_pages": (c_int, [c_void_p]),
    "copris_rollout_free_pages": (c_int64, [c_void_p]),
    "copris_rollout_begin_stage": (c_int, [c_void_p]),
    "copris_rollout_next_step": (c_int, [c_void_p, c_void_p]),
    "copris_rollout_stop": (c_int, [c_void_p, c_void_p, c_int]),
    "copris_rollout_end_stage": (c_int, [c_void_p] * 4),
    "copris_rollout_apply": (c_int, [c_void_p, c_int, c_int] + [c_void_p] * 4 + [c_int, c_int, c_void_p]),
    "copris_kv_append": (c_int, [c_void_p] * 6 + [c_int] * 5 + [c_int64, c_int, c_void_p]),
    "copris_traj_append": (c_int, [c_void_p] * 5 + [c_int] + [c_void_p] * 3 + [c_int, c_int64, c_int, c_void_p]),
    "copris_traj_gather": (c_int, [c_void_p] * 5 + [c_int] + [c_void_p] * 4 + [c_int, c_int64, c_int, c_void_p]),
})

_lib = None


class CoprisError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        detail = load_library().copris_last_error_detail().decode() if code in (COPRIS_ELAUNCH, COPRIS_EWORKSPACE) else ""
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


def _expect(t, dtype: Optional[str], name: str, optional: bool = False) -> None:
    """Host-side check of a tensor argument before its address crosses the C ABI: on the GPU,
    contiguous, of the expected torch dtype (a name such as "int32"; None = any)."""
    if t is None:
        if optional:
            return
        raise TypeError(f"{name}: a device tensor is required")
    if not t.is_cuda:
        raise TypeError(f"{name}: must be a GPU tensor, got device {t.device}")
    if not t.is_contiguous():
        raise TypeError(f"{name}: must be contiguous")
    if dtype is not None and str(t.dtype) != "torch." + dtype:
        raise TypeError(f"{name}: expected torch.{dtype}, got {t.dtype}")


def _elem(dtype_code: int) -> str:
    return {COPRIS_F32: "float32", COPRIS_BF16: "bfloat16"}.get(int(dtype_code))


def _stream(stream, ref=None) -> Optional[int]:
    """The raw stream handle (None = the null stream); `ref` is a tensor argument of the call,
    which must live on the stream's device."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream(ref.device if ref is not None else None)
    if ref is not None and stream.device != ref.device:
        raise TypeError(f"stream on {stream.device} but tensors on {ref.device}")
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
    e = _elem(dtype)
    _expect(q, e, "q"); _expect(k_cache, e, "k_cache"); _expect(v_cache, e, "v_cache"); _expect(out, e, "out")
    _expect(block_table, "int32", "block_table"); _expect(ctx_len, "int32", "ctx_len")
    _expect(lse, "float32", "lse", optional=True); _expect(workspace, "uint8", "workspace")
    C, Hq, D = q.shape
    num_pages, Hkv, page_size, _ = k_cache.shape
    max_pages = block_table.shape[1]
    code = load_library().copris_decode_attn(
        _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_table), _ptr(ctx_len), _ptr(out),
        _ptr(lse), _ptr(workspace), workspace.numel() * workspace.element_size(),
        C, Hq, Hkv, D, page_size, max_pages, num_pages, float(scale), int(dtype), _stream(stream, q))
    _check(code, "copris_decode_attn")


def lmhead_logprob_workspace_bytes(C, H, V) -> int:
    return int(load_library().copris_lmhead_logprob_workspace_bytes(C, H, V))


def lmhead_logprob(hidden, weight, seq_id, step, token, logprob, lse, workspace, *, seed: int,
                   temperature: float, dtype: int, stream=None) -> None:
    """copris_lmhead_logprob on device tensors."""
    e = _elem(dtype)
    _expect(hidden, e, "hidden"); _expect(weight, e, "weight"); _expect(seq_id, "int64", "seq_id")
    _expect(step, "int32", "step"); _expect(token, "int32", "token"); _expect(logprob, "float32", "logprob")
    _expect(lse, "float32", "lse", optional=True); _expect(workspace, "uint8", "workspace")
    C, H = hidden.shape
    V = weight.shape[0]
    code = load_library().copris_lmhead_logprob(
        _ptr(hidden), _ptr(weight), _ptr(seq_id), _ptr(step), int(seed) & 0xFFFFFFFFFFFFFFFF,
        float(temperature), _ptr(token), _ptr(logprob), _ptr(lse), _ptr(workspace),
        workspace.numel() * workspace.element_size(), C, H, V, int(dtype), _stream(stream, hidden))
    _check(code, "copris_lmhead_logprob")


def lmhead_logprob_noalloc(hidden, weight, seq_id, step, token, logprob, lse, *, seed: int,
                           temperature: float, dtype: int, stream=None) -> None:
    """copris_lmhead_logprob_noalloc on device tensors (partials in the library's static array)."""
    e = _elem(dtype)
    _expect(hidden, e, "hidden"); _expect(weight, e, "weight"); _expect(seq_id, "int64", "seq_id")
    _expect(step, "int32", "step"); _expect(token, "int32", "token"); _expect(logprob, "float32", "logprob")
    _expect(lse, "float32", "lse", optional=True)
    C, H = hidden.shape
    V = weight.shape[0]
    code = load_library().copris_lmhead_logprob_noalloc(
        _ptr(hidden), _ptr(weight), _ptr(seq_id), _ptr(step), int(seed) & 0xFFFFFFFFFFFFFFFF,
        float(temperature), _ptr(token), _ptr(logprob), _ptr(lse), C, H, V, int(dtype),
        _stream(stream, hidden))
    _check(code, "copris_lmhead_logprob_noalloc")


def is_ratio(logp_cur, logp_buf, logp_roll, cu_seqlens, split, mask, ratio, ratio_clipped,
             seq_sum, seq_cnt, seq_nclip, *, eps_low: float, eps_high: float, stream=None) -> None:
    """copris_is_ratio on device tensors."""
    for t, n in ((logp_cur, "logp_cur"), (logp_buf, "logp_buf"), (logp_roll, "logp_roll"), (ratio, "ratio"),
                 (ratio_clipped, "ratio_clipped"), (seq_sum, "seq_sum")):
        _expect(t, "float32", n)
    for t, n in ((cu_seqlens, "cu_seqlens"), (split, "split"), (seq_cnt, "seq_cnt"), (seq_nclip, "seq_nclip")):
        _expect(t, "int32", n)
    _expect(mask, "uint8", "mask", optional=True)
    B = cu_seqlens.numel() - 1
    N = logp_cur.numel()
    code = load_library().copris_is_ratio(
        _ptr(logp_cur), _ptr(logp_buf), _ptr(logp_roll), _ptr(cu_seqlens), _ptr(split), _ptr(mask),
        float(eps_low), float(eps_high), _ptr(ratio), _ptr(ratio_clipped), _ptr(seq_sum),
        _ptr(seq_cnt), _ptr(seq_nclip), B, N, _stream(stream, cu_seqlens))
    _check(code, "copris_is_ratio")


def grpo_surrogate(logp_cur, logp_buf, logp_roll, cu_seqlens, split, mask, adv, surr, grad, seq_surr,
                   seq_cnt, objective, *, eps_low: float, eps_high: float, stream=None) -> None:
    """copris_grpo_surrogate on device tensors."""
    for t, n in ((logp_cur, "logp_cur"), (logp_buf, "logp_buf"), (logp_roll, "logp_roll"), (adv, "adv"),
                 (surr, "surr"), (grad, "grad"), (seq_surr, "seq_surr"), (objective, "objective")):
        _expect(t, "float32", n)
    for t, n in ((cu_seqlens, "cu_seqlens"), (split, "split"), (seq_cnt, "seq_cnt")):
        _expect(t, "int32", n)
    _expect(mask, "uint8", "mask", optional=True)
    B = cu_seqlens.numel() - 1
    N = logp_cur.numel()
    code = load_library().copris_grpo_surrogate(
        _ptr(logp_cur), _ptr(logp_buf), _ptr(logp_roll), _ptr(cu_seqlens), _ptr(split), _ptr(mask),
        _ptr(adv), float(eps_low), float(eps_high), _ptr(surr), _ptr(grad), _ptr(seq_surr),
        _ptr(seq_cnt), _ptr(objective), B, N, _stream(stream, objective))
    _check(code, "copris_grpo_surrogate")


def lmhead_token_logprob_workspace_bytes(M, H, V, dtype) -> int:
    return int(load_library().copris_lmhead_token_logprob_workspace_bytes(M, H, V, int(dtype)))


def lmhead_token_logprob(hidden, weight, tokens, logprob, lse, workspace, *, temperature: float,
                         dtype: int, stream=None) -> None:
    """copris_lmhead_token_logprob on device tensors."""
    e = _elem(dtype)
    _expect(hidden, e, "hidden"); _expect(weight, e, "weight"); _expect(tokens, "int32", "tokens")
    _expect(logprob, "float32", "logprob"); _expect(lse, "float32", "lse", optional=True)
    _expect(workspace, "uint8", "workspace")
    M, H = hidden.shape
    V = weight.shape[0]
    code = load_library().copris_lmhead_token_logprob(
        _ptr(hidden), _ptr(weight), _ptr(tokens), float(temperature), _ptr(logprob), _ptr(lse),
        _ptr(workspace), workspace.numel() * workspace.element_size(), M, H, V, int(dtype),
        _stream(stream, hidden))
    _check(code, "copris_lmhead_token_logprob")


def prefill_attn(q, k, v, cu_seqlens, block_table, k_cache, v_cache, out, lse, *, max_seqlen: int,
                 scale: float, dtype: int, stream=None) -> None:
    """copris_prefill_attn on device tensors (shapes as in include/copris.h)."""
    e = _elem(dtype)
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (k_cache, "k_cache"), (v_cache, "v_cache"), (out, "out")):
        _expect(t, e, n)
    _expect(cu_seqlens, "int32", "cu_seqlens"); _expect(block_table, "int32", "block_table")
    _expect(lse, "float32", "lse", optional=True)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    num_pages, _, page_size, _ = k_cache.shape
    B = cu_seqlens.numel() - 1
    code = load_library().copris_prefill_attn(
        _ptr(q), _ptr(k), _ptr(v), _ptr(cu_seqlens), _ptr(block_table), _ptr(k_cache), _ptr(v_cache),
        _ptr(out), _ptr(lse), B, T, Hq, Hkv, D, page_size, block_table.shape[1], num_pages,
        int(max_seqlen), float(scale), int(dtype), _stream(stream, q))
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


class RolloutManager:
    """The stepwise rollout manager (copris_rollout_* of include/copris.h) on host arrays."""

    def __init__(self, prompt_len, resp_len, pool: int, batch_inputs: int, page_size: int = 16,
                 num_pages: Optional[int] = None, page_order=None):
        import numpy as np
        p = np.ascontiguousarray(prompt_len, dtype=np.int32)
        r = np.ascontiguousarray(resp_len, dtype=np.int32)
        self.n_inputs, self.samples = int(r.shape[0]), int(r.shape[1])
        self.pool, self.batch_inputs, self.page_size = int(pool), int(batch_inputs), int(page_size)
        longest = int((p[:, None].astype(np.int64) + r).max()) if r.size else 1
        if num_pages is None:
            num_pages = self.pool * ((longest + self.page_size - 1) // self.page_size)
        order = None if page_order is None else np.ascontiguousarray(page_order, dtype=np.int32)
        h = c_void_p()
        code = load_library().copris_rollout_create(
            p.ctypes.data, r.ctypes.data, self.n_inputs, self.samples, self.pool, self.batch_inputs,
            self.page_size, int(num_pages), None if order is None else order.ctypes.data, ctypes.addressof(h))
        _check(code, "copris_rollout_create")
        self._h = h
        self.num_pages = int(num_pages)
        self.max_pages = int(load_library().copris_rollout_max_pages(h))

    def close(self) -> None:
        if self._h is not None:
            load_library().copris_rollout_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def free_pages(self) -> int:
        return int(load_library().copris_rollout_free_pages(self._h))

    def begin_stage(self) -> int:
        k = load_library().copris_rollout_begin_stage(self._h)
        if k < 0:
            raise CoprisError(k, "copris_rollout_begin_stage")
        return k

    def next_step(self, copy: bool = True):
        """Returns (code, plan): code is ROLLOUT_STEP / ROLLOUT_STAGE_END / ROLLOUT_EXHAUSTED; plan is a
        dict of the manager's arrays (None unless code is ROLLOUT_STEP): numpy copies, or with
        copy=False views of the manager's own memory that are valid until the next call."""
        import numpy as np
        plan = RolloutPlan()
        code = load_library().copris_rollout_next_step(self._h, ctypes.addressof(plan))
        if code < 0:
            raise CoprisError(code, "copris_rollout_next_step")
        if code != ROLLOUT_STEP:
            return code, None

        def arr(ptr, n):
            if not n:
                return np.zeros(0, np.int32)
            a = np.ctypeslib.as_array(ptr, shape=(n,))
            return a.copy() if copy else a
        return code, {
            "stage": plan.stage, "n_active": plan.n_active,
            "slot_traj": arr(plan.slot_traj, self.pool),
            "entered": arr(plan.entered, 4 * plan.n_entered).reshape(-1, 4),
            "finishing": arr(plan.finishing, plan.n_finishing),
            "n_slot_cmds": plan.n_slot_cmds, "n_page_cmds": plan.n_page_cmds,
            "cmds": arr(plan.cmds, 4 * plan.n_slot_cmds + 3 * plan.n_page_cmds),
            "block_table": arr(plan.block_table, self.pool * self.max_pages).reshape(self.pool, self.max_pages),
        }

    def stop(self, slots) -> None:
        import numpy as np
        s = np.ascontiguousarray(slots, dtype=np.int32)
        _check(load_library().copris_rollout_stop(self._h, s.ctypes.data, int(s.size)), "copris_rollout_stop")

    def end_stage(self) -> dict:
        """Stage statistics (the fields of copris_stage_stats), `batch_inputs` and `batch_traj`
        [B * samples, 3] = (trajectory, response tokens, tokens of earlier stages)."""
        import numpy as np
        stats = StageStats()
        binp = np.zeros(self.batch_inputs, dtype=np.int32)
        btr = np.zeros((self.batch_inputs * self.samples, 3), dtype=np.int32)
        code = load_library().copris_rollout_end_stage(self._h, ctypes.addressof(stats), binp.ctypes.data,
                                                       btr.ctypes.data)
        _check(code, "copris_rollout_end_stage")
        d = {name: int(getattr(stats, name)) for name, _ in StageStats._fields_}
        d["batch_inputs"] = binp.tolist()
        d["batch_traj"] = btr
        return d


def rollout_apply(cmds, n_slot_cmds: int, n_page_cmds: int, seq_id, ctx_len, step, block_table, *,
                  stream=None) -> None:
    """copris_rollout_apply on device tensors (cmds: the plan's commands, already on the device)."""
    _expect(cmds, "int32", "cmds"); _expect(seq_id, "int64", "seq_id")
    _expect(ctx_len, "int32", "ctx_len"); _expect(step, "int32", "step"); _expect(block_table, "int32", "block_table")
    pool, max_pages = block_table.shape
    code = load_library().copris_rollout_apply(_ptr(cmds), int(n_slot_cmds), int(n_page_cmds), _ptr(seq_id),
                                               _ptr(ctx_len), _ptr(step), _ptr(block_table), pool, max_pages,
                                               _stream(stream, block_table))
    _check(code, "copris_rollout_apply")


def kv_append(k_new, v_new, block_table, ctx_len, k_cache, v_cache, *, dtype: int, stream=None) -> None:
    """copris_kv_append on device tensors."""
    for t, n in ((k_new, "k_new"), (v_new, "v_new"), (k_cache, "k_cache"), (v_cache, "v_cache")):
        _expect(t, None, n)
    _expect(block_table, "int32", "block_table"); _expect(ctx_len, "int32", "ctx_len")
    C, Hkv, D = k_new.shape
    num_pages, _, page_size, _ = k_cache.shape
    code = load_library().copris_kv_append(_ptr(k_new), _ptr(v_new), _ptr(block_table), _ptr(ctx_len),
                                           _ptr(k_cache), _ptr(v_cache), C, Hkv, D, page_size,
                                           block_table.shape[1], num_pages, int(dtype), _stream(stream, k_cache))
    _check(code, "copris_kv_append")


def traj_append(token, logprob, seq_id, step, ctx_len, stage: int, buf_token, buf_logp, buf_tag, *,
                stream=None) -> None:
    """copris_traj_append on device tensors (buffers [n_traj, max_resp])."""
    _expect(token, "int32", "token"); _expect(logprob, "float32", "logprob"); _expect(seq_id, "int64", "seq_id")
    _expect(step, "int32", "step"); _expect(ctx_len, "int32", "ctx_len")
    _expect(buf_token, "int32", "buf_token"); _expect(buf_logp, "float32", "buf_logp"); _expect(buf_tag, "int32", "buf_tag")
    n_traj, max_resp = buf_token.shape
    code = load_library().copris_traj_append(_ptr(token), _ptr(logprob), _ptr(seq_id), _ptr(step), _ptr(ctx_len),
                                             int(stage), _ptr(buf_token), _ptr(buf_logp), _ptr(buf_tag),
                                             token.numel(), n_traj, max_resp, _stream(stream, buf_token))
    _check(code, "copris_traj_append")


def traj_gather(buf_token, buf_logp, buf_tag, traj, cu_seqlens, stage: int, tokens_out, logp_buf_out,
                logp_roll_out, split_out, *, stream=None) -> None:
    """copris_traj_gather on device tensors."""
    _expect(buf_token, "int32", "buf_token"); _expect(buf_logp, "float32", "buf_logp"); _expect(buf_tag, "int32", "buf_tag")
    _expect(traj, "int32", "traj"); _expect(cu_seqlens, "int32", "cu_seqlens"); _expect(tokens_out, "int32", "tokens_out")
    _expect(logp_buf_out, "float32", "logp_buf_out"); _expect(logp_roll_out, "float32", "logp_roll_out")
    _expect(split_out, "int32", "split_out")
    n_traj, max_resp = buf_token.shape
    code = load_library().copris_traj_gather(_ptr(buf_token), _ptr(buf_logp), _ptr(buf_tag), _ptr(traj),
                                             _ptr(cu_seqlens), int(stage), _ptr(tokens_out), _ptr(logp_buf_out),
                                             _ptr(logp_roll_out), _ptr(split_out), traj.numel(), n_traj, max_resp,
                                             _stream(stream, buf_token))
    _check(code, "copris_traj_gather")
