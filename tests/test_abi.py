"""The C-ABI shared library loads and exports every symbol include/copris.h declares.
Host-only entry points (error text, workspace sizes, argument rejection) are called;
nothing here launches a kernel."""
import ctypes
import os
import re

import pytest

from paper_2511_05589_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2511_05589_amd.build import build
        build()
    return binding.load_library()


def _declared():
    text = open(os.path.join(ROOT, "include", "copris.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(copris_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(lib):
    names = _declared()
    assert {"copris_decode_attn", "copris_lmhead_logprob", "copris_is_ratio",
            "copris_decode_attn_workspace_bytes", "copris_lmhead_logprob_workspace_bytes",
            "copris_strerror"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
        assert n in binding.SIGNATURES, f"{n} has no binding signature"
    assert sorted(binding.SIGNATURES) == names


def test_error_text_and_version(lib):
    assert binding.strerror(0) == "ok"
    for code in (-1, -2, -3, -4):
        assert binding.strerror(code) not in ("ok", "unknown error code")
    assert binding.strerror(-99) == "unknown error code"
    assert re.fullmatch(r"\d+\.\d+\.\d+", binding.version())


def test_workspace_queries_are_host_only_and_monotone(lib):
    a = binding.decode_attn_workspace_bytes(256, 28, 4, 128, 16, 1056)
    b = binding.decode_attn_workspace_bytes(256, 28, 4, 128, 16, 2112)
    assert 0 < a < b and a % 256 == 0
    assert binding.decode_attn_workspace_bytes(0, 28, 4, 128, 16, 10) == 0
    assert binding.decode_attn_workspace_bytes(8, 28, 5, 128, 16, 10) == 0      # Hq % Hkv != 0
    x = binding.lmhead_logprob_workspace_bytes(256, 3584, 151936)
    assert x > 0 and x % 256 == 0
    assert binding.lmhead_logprob_workspace_bytes(256, 3584, 0) == 0


def test_bad_arguments_are_rejected_before_any_launch(lib):
    # null pointers / bad scalars return COPRIS_EINVAL without touching a device
    r = lib.copris_decode_attn(None, None, None, None, None, None, None, None, 0,
                               8, 4, 2, 64, 16, 4, 10, 0.125, 0, None)
    assert r == binding.COPRIS_EINVAL
    r = lib.copris_lmhead_logprob(None, None, None, None, 1, 1.0, None, None, None, None, 0,
                                  8, 256, 1024, 0, None)
    assert r == binding.COPRIS_EINVAL
    r = lib.copris_is_ratio(None, None, None, None, None, None, 1.5, 0.2, None, None, None, None,
                            None, 4, 100, None)
    assert r == binding.COPRIS_EINVAL
    # B == 0, N == 0 is a valid empty batch
    assert lib.copris_is_ratio(None, None, None, None, None, None, 0.2, 0.2, None, None, None,
                               None, None, 0, 0, None) == binding.COPRIS_OK


def test_bad_arguments_of_the_later_entry_points(lib):
    fake = 256          # a non-null, aligned "pointer": every call below is refused before it is used
    # grpo surrogate: objective is required, eps_low must be below 1
    assert lib.copris_grpo_surrogate(None, None, None, None, None, None, None, 0.2, 0.28, None, None, None,
                                     None, None, 0, 0, None) == binding.COPRIS_EINVAL
    assert lib.copris_grpo_surrogate(fake, fake, fake, fake, fake, None, fake, 1.0, 0.28, fake, fake, fake,
                                     fake, fake, 2, 10, None) == binding.COPRIS_EINVAL
    # given-token log-probs: temperature, dtype, H alignment, workspace
    args = lambda **k: [k.get("hidden", fake), fake, fake, k.get("T", 1.0), fake, None, k.get("ws", fake),
                        k.get("wsb", 1 << 40), 8, k.get("H", 256), 1024, k.get("dtype", 1), None]
    assert lib.copris_lmhead_token_logprob(*args(T=0.0)) == binding.COPRIS_EINVAL
    assert lib.copris_lmhead_token_logprob(*args(dtype=7)) == binding.COPRIS_EUNSUPPORTED
    assert lib.copris_lmhead_token_logprob(*args(H=250)) == binding.COPRIS_EINVAL
    assert lib.copris_lmhead_token_logprob(*args(hidden=None)) == binding.COPRIS_EINVAL
    assert lib.copris_lmhead_token_logprob(*args(wsb=16)) == binding.COPRIS_EWORKSPACE
    assert lib.copris_lmhead_token_logprob(*args(ws=264)) == binding.COPRIS_EWORKSPACE   # not 256-aligned
    assert binding.lmhead_token_logprob_workspace_bytes(8192, 3584, 151936, 1) > 0
    assert binding.lmhead_token_logprob_workspace_bytes(8192, 3584, 151936, 5) == 0
    # re-prefill attention: shapes the kernel is not compiled for, bad bounds, empty batches
    pf = lambda **k: [fake] * 8 + [None, k.get("B", 2), k.get("T", 100), k.get("Hq", 28), 4, k.get("D", 128),
                                   k.get("P", 16), 8, 64, k.get("maxlen", 100), 0.088, k.get("dtype", 1), None]
    assert lib.copris_prefill_attn(*pf(D=64)) == binding.COPRIS_EUNSUPPORTED
    assert lib.copris_prefill_attn(*pf(dtype=0)) == binding.COPRIS_EUNSUPPORTED
    assert lib.copris_prefill_attn(*pf(Hq=40)) == binding.COPRIS_EUNSUPPORTED      # group of 10
    assert lib.copris_prefill_attn(*pf(Hq=30)) == binding.COPRIS_EINVAL            # not a multiple of Hkv
    assert lib.copris_prefill_attn(*pf(maxlen=129)) == binding.COPRIS_EINVAL       # beyond max_pages * P
    assert lib.copris_prefill_attn(*pf(B=0, T=0)) == binding.COPRIS_OK
    assert lib.copris_prefill_attn(*pf(B=0, T=5)) == binding.COPRIS_EINVAL
    # rollout manager (host function)
    import ctypes
    n = ctypes.c_int(-1)
    assert lib.copris_rollout_schedule(None, None, 0, 1, 4, 1, 16, 0, None, None, ctypes.addressof(n)) == binding.COPRIS_OK
    assert n.value == 0
    assert lib.copris_rollout_schedule(None, None, 3, 1, 4, 1, 16, 0, None, None, ctypes.addressof(n)) == binding.COPRIS_EINVAL
    assert lib.copris_rollout_schedule(None, None, 0, 1, 4, 1, 16, 0, None, None, None) == binding.COPRIS_EINVAL


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(FileNotFoundError):
        binding.load_library(str(tmp_path / "libcopris.so"))
