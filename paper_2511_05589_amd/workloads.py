"""Seeded synthetic inputs for the CoPRIS rollout-decode hot path.

This module only *draws* inputs: context lengths, paged KV pools, hidden states,
LM-head weights and importance-sampling batches.  It contains none of the
method's arithmetic (no attention, no softmax, no sampling, no ratios), so both
the CPU oracle's tests and the HIP path's tests may take their inputs from it.

The shapes follow the workload the paper describes: a fixed concurrency pool of
requests (Section 4, "Concurrency-Controlled Generation") whose response lengths
are long-tailed (Section 3.2, Figure 1a), prompts up to 1024 tokens and
responses up to 15360 / 31744 tokens (Table 4), some of the requests being
partial trajectories resumed from the buffer (Section 4, "Prioritized
Resumption"), and training batches whose trajectories are split between a
buffered old-policy stage and the current stage (Eq. 6, Eq. 8).

All randomness is `numpy.random.default_rng(seed)` (PCG64), split with `spawn`
into sub-streams in the fixed order
[ctx lengths, page permutation, q, K, V, hidden, W, IS].
Tensors are drawn in fp32 and rounded (nearest-even) to the storage dtype.
bf16 tensors are held as uint16 bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

BASE_SEED = 20251105

F32 = "f32"
BF16 = "bf16"


# --------------------------------------------------------------------------
# storage-dtype helpers (bit manipulation only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    out = np.empty(u.shape, dtype=np.uint16)
    # in slabs, to bound the temporary memory for GB-sized pools
    flat_u = u.reshape(-1)
    flat_o = out.reshape(-1)
    step = 1 << 26
    for s in range(0, flat_u.size, step):
        w = flat_u[s:s + step]
        nan = (w & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
        r = (w + (((w >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF))) >> np.uint32(16)
        r = r.astype(np.uint16)
        r[nan] = np.uint16(0x7FC0)
        flat_o[s:s + step] = r
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen uint16 bf16 bit patterns to the exact fp32 values they denote."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == F32:
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == BF16:
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def to_f32(x: np.ndarray, dtype: str) -> np.ndarray:
    """Exact fp32 values of a storage array."""
    if dtype == F32:
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == BF16:
        return bf16_bits_to_f32(x)
    raise ValueError(dtype)


def nan_storage(dtype: str):
    return np.float32(np.nan) if dtype == F32 else np.uint16(0x7FC0)


# --------------------------------------------------------------------------
# configurations
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class DecodeConfig:
    """One decode-step workload (attention and, where H>0, the LM head)."""
    index: int
    name: str
    C: int                # concurrency: sequences in flight
    Hq: int
    Hkv: int
    D: int
    dtype: str
    page_size: int
    # context-length recipe
    ctx_recipe: str       # "lognormal" | "longtail"
    prompt: int = 0
    mu: float = 0.0
    sigma: float = 0.0
    cap: int = 0
    # LM head (H == 0: the config names no LM head)
    H: int = 0
    V: int = 0
    temperature: float = 1.0
    spare_frac: float = 0.25

    @property
    def seed(self) -> int:
        return BASE_SEED + 1000 * self.index

    @property
    def g(self) -> int:
        return self.Hq // self.Hkv

    @property
    def max_ctx(self) -> int:
        return self.prompt + self.cap if self.ctx_recipe == "lognormal" else 32768

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == F32 else 2


@dataclass(frozen=True)
class ISConfig:
    """One cross-stage importance-sampling batch."""
    index: int
    name: str
    B: int
    layout: str           # "padded" | "packed"
    len_lo: int
    len_hi: int
    pad_to: int = 0
    sigma: float = 0.05
    eps_low: float = 0.2
    eps_high: float = 0.2
    mask_zero_frac: float = 0.0

    @property
    def seed(self) -> int:
        return BASE_SEED + 1000 * self.index


DECODE_CONFIGS = {
    0: DecodeConfig(0, "tiny", C=8, Hq=4, Hkv=2, D=64, dtype=F32, page_size=16,
                    ctx_recipe="lognormal", prompt=32, mu=5.0, sigma=1.0, cap=512,
                    H=256, V=1024),
    1: DecodeConfig(1, "1.5B-shaped", C=64, Hq=12, Hkv=2, D=128, dtype=BF16, page_size=16,
                    ctx_recipe="lognormal", prompt=256, mu=7.0, sigma=1.0, cap=8192,
                    H=1536, V=151936),
    2: DecodeConfig(2, "7B-shaped", C=256, Hq=28, Hkv=4, D=128, dtype=BF16, page_size=16,
                    ctx_recipe="lognormal", prompt=512, mu=7.5, sigma=1.1, cap=16384,
                    H=3584, V=151936),
    3: DecodeConfig(3, "long-tail-stress", C=512, Hq=28, Hkv=4, D=128, dtype=BF16, page_size=16,
                    ctx_recipe="longtail", spare_frac=0.02),
}

IS_CONFIGS = {
    0: ISConfig(0, "tiny-is", B=8, layout="padded", len_lo=1, len_hi=512, pad_to=512),
    4: ISConfig(4, "cross-stage-is", B=256, layout="packed", len_lo=1024, len_hi=16384,
                mask_zero_frac=0.01),
}


def substreams(seed: int):
    """The eight sub-streams of one config, in their fixed order."""
    names = ["ctx", "perm", "q", "k", "v", "hidden", "w", "is"]
    return dict(zip(names, np.random.default_rng(seed).spawn(len(names))))


# --------------------------------------------------------------------------
# context lengths
# --------------------------------------------------------------------------
def make_ctx_len(cfg: DecodeConfig, rng: Optional[np.random.Generator] = None) -> np.ndarray:
    """Context length of every sequence in the pool, int32 [C].

    lognormal: ctx = prompt + min(max(rint(LogNormal(mu, sigma)), 1), cap);
    longtail:  90 % uniform in [256, 2048], 8 % in [2048, 16384], the rest at
               exactly 32768 (resumed partial trajectories), shuffled over slots.
    """
    rng = rng if rng is not None else substreams(cfg.seed)["ctx"]
    if cfg.ctx_recipe == "lognormal":
        x = rng.lognormal(cfg.mu, cfg.sigma, size=cfg.C)
        resp = np.minimum(np.maximum(np.rint(x), 1), cfg.cap)
        return (cfg.prompt + resp).astype(np.int32)
    if cfg.ctx_recipe == "longtail":
        n_long = int(round(0.02 * cfg.C))
        n_mid = int(round(0.08 * cfg.C))
        n_short = cfg.C - n_long - n_mid
        short = rng.integers(256, 2048, size=n_short, endpoint=True)
        mid = rng.integers(2048, 16384, size=n_mid, endpoint=True)
        long_ = np.full(n_long, 32768)
        ctx = np.concatenate([short, mid, long_])
        rng.shuffle(ctx)
        return ctx.astype(np.int32)
    raise ValueError(cfg.ctx_recipe)


# --------------------------------------------------------------------------
# paged KV pool + queries
# --------------------------------------------------------------------------
def make_block_table(ctx_len: np.ndarray, page_size: int, spare_frac: float,
                     rng: np.random.Generator, max_pages: Optional[int] = None):
    """Hand out physical pages in a seeded random order.

    Returns (block_table int32 [C, max_pages], num_pages).  Entries past a
    sequence's last page hold -1 (never dereferenced by a correct reader).
    """
    ctx_len = np.asarray(ctx_len, dtype=np.int64)
    n_pages = (ctx_len + page_size - 1) // page_size
    used = int(n_pages.sum())
    num_pages = used + int(np.ceil(spare_frac * used)) + 1
    phys = rng.permutation(num_pages)[:used].astype(np.int32)
    width = int(n_pages.max()) if n_pages.size and n_pages.max() > 0 else 1
    if max_pages is not None:
        if max_pages < width:
            raise ValueError("max_pages too small")
        width = max_pages
    bt = np.full((ctx_len.size, width), -1, dtype=np.int32)
    off = 0
    for i, n in enumerate(n_pages):
        bt[i, :n] = phys[off:off + n]
        off += n
    return bt, num_pages


def _normal_storage(rng: np.random.Generator, shape, dtype: str, std: float = 1.0) -> np.ndarray:
    """N(0, std) drawn in fp32, rounded to the storage dtype, slab by slab."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32 if dtype == F32 else np.uint16)
    step = 1 << 26
    for s in range(0, n, step):
        m = min(step, n - s)
        x = rng.standard_normal(m, dtype=np.float32)
        if std != 1.0:
            x *= np.float32(std)
        out[s:s + m] = to_storage(x, dtype)
    return out.reshape(shape)


def poison_unused_slots(cache: np.ndarray, block_table: np.ndarray, ctx_len: np.ndarray,
                        page_size: int, dtype: str) -> None:
    """NaN-fill every slot no sequence owns: unreferenced pages and the slots
    of a last page at or beyond the sequence's length.  In place."""
    num_pages = cache.shape[0]
    nan = nan_storage(dtype)
    referenced = np.zeros(num_pages, dtype=bool)
    for i, n in enumerate(np.asarray(ctx_len, dtype=np.int64)):
        npg = (n + page_size - 1) // page_size
        pages = block_table[i, :npg]
        referenced[pages] = True
        tail = int(n % page_size)
        if npg > 0 and tail != 0:
            cache[pages[-1], :, tail:, :] = nan
    cache[~referenced] = nan


def make_decode_inputs(cfg: DecodeConfig, *, ctx_len: Optional[np.ndarray] = None,
                       poison: bool = True, with_lmhead: bool = True,
                       with_attn: bool = True) -> dict:
    """All inputs of one decode step for `cfg`.

    Keys: ctx_len, block_table, num_pages, q, k_cache, v_cache (storage dtype,
    layout [num_pages, Hkv, page_size, D]), scale; and where the config names an
    LM head: hidden [C, H], weight [V, H], seq_id int64 [C], step int32 [C],
    seed, temperature.
    """
    st = substreams(cfg.seed)
    out: dict = {"cfg": cfg}
    if ctx_len is None:
        ctx_len = make_ctx_len(cfg, st["ctx"])
    ctx_len = np.asarray(ctx_len, dtype=np.int32)
    out["ctx_len"] = ctx_len
    if with_attn:
        bt, num_pages = make_block_table(ctx_len, cfg.page_size, cfg.spare_frac, st["perm"])
        out["block_table"] = bt
        out["num_pages"] = num_pages
        out["q"] = _normal_storage(st["q"], (cfg.C, cfg.Hq, cfg.D), cfg.dtype)
        shape = (num_pages, cfg.Hkv, cfg.page_size, cfg.D)
        out["k_cache"] = _normal_storage(st["k"], shape, cfg.dtype)
        out["v_cache"] = _normal_storage(st["v"], shape, cfg.dtype)
        if poison:
            poison_unused_slots(out["k_cache"], bt, ctx_len, cfg.page_size, cfg.dtype)
            poison_unused_slots(out["v_cache"], bt, ctx_len, cfg.page_size, cfg.dtype)
        out["scale"] = float(1.0 / np.sqrt(cfg.D))
    if with_lmhead and cfg.H > 0:
        out["hidden"] = _normal_storage(st["hidden"], (cfg.C, cfg.H), cfg.dtype)
        out["weight"] = _normal_storage(st["w"], (cfg.V, cfg.H), cfg.dtype, std=0.02)
        # stable trajectory ids (not slot indices) and the index of the token
        # being generated within its response
        out["seq_id"] = (np.int64(cfg.seed) * np.int64(1_000_003)
                         + np.arange(cfg.C, dtype=np.int64) * np.int64(7919))
        out["step"] = np.maximum(ctx_len.astype(np.int64) - cfg.prompt, 0).astype(np.int32)
        out["seed"] = int(0x5EED0000_00000000 + cfg.seed)
        out["temperature"] = float(cfg.temperature)
    return out


def make_token_logprob_inputs(cfg: DecodeConfig, M: int) -> dict:
    """One micro-batch of M positions for the log-prob recompute under the current policy:
    the LM head of `cfg` (the same weight stream as make_decode_inputs), hidden states
    N(0,1) and given tokens uniform over the vocabulary, both from a stream of their own."""
    st = substreams(cfg.seed)
    rng_h, rng_t = np.random.default_rng(cfg.seed + 77).spawn(2)
    return {"cfg": cfg, "M": int(M),
            "hidden": _normal_storage(rng_h, (M, cfg.H), cfg.dtype),
            "weight": _normal_storage(st["w"], (cfg.V, cfg.H), cfg.dtype, std=0.02),
            "tokens": rng_t.integers(0, cfg.V, size=M, dtype=np.int64).astype(np.int32),
            "temperature": float(cfg.temperature)}


def make_prefill_case(seed: int, lens, Hq: int, Hkv: int, D: int, dtype: str, page_size: int = 16,
                      spare_frac: float = 0.25) -> dict:
    """Resumed partial trajectories to re-prefill: packed q / k / v ~ N(0,1) for sequences of
    the given lengths, and a block table over seeded, randomly interleaved physical pages."""
    rng_perm, rng_q, rng_k, rng_v = np.random.default_rng(seed).spawn(4)
    lens = np.asarray(lens, dtype=np.int32)
    T = int(lens.sum())
    cu = np.zeros(lens.size + 1, dtype=np.int32)
    np.cumsum(lens, out=cu[1:])
    bt, num_pages = make_block_table(lens, page_size, spare_frac, rng_perm)
    return {"q": _normal_storage(rng_q, (T, Hq, D), dtype), "k": _normal_storage(rng_k, (T, Hkv, D), dtype),
            "v": _normal_storage(rng_v, (T, Hkv, D), dtype), "cu_seqlens": cu, "lens": lens,
            "block_table": bt, "num_pages": num_pages, "page_size": page_size,
            "scale": float(1.0 / np.sqrt(D)), "Hq": Hq, "Hkv": Hkv, "D": D, "dtype": dtype}


def make_small_decode_case(seed: int, C: int, Hq: int, Hkv: int, D: int, dtype: str,
                           page_size: int, ctx_len, *, spare_frac: float = 0.25,
                           max_pages: Optional[int] = None, poison: bool = True) -> dict:
    """A free-form attention case (for randomized small-shape tests)."""
    rng_perm, rng_q, rng_k, rng_v = np.random.default_rng(seed).spawn(4)
    ctx_len = np.asarray(ctx_len, dtype=np.int32)
    assert ctx_len.shape == (C,)
    bt, num_pages = make_block_table(ctx_len, page_size, spare_frac, rng_perm, max_pages)
    q = _normal_storage(rng_q, (C, Hq, D), dtype)
    shape = (num_pages, Hkv, page_size, D)
    k = _normal_storage(rng_k, shape, dtype)
    v = _normal_storage(rng_v, shape, dtype)
    if poison:
        poison_unused_slots(k, bt, ctx_len, page_size, dtype)
        poison_unused_slots(v, bt, ctx_len, page_size, dtype)
    return {"ctx_len": ctx_len, "block_table": bt, "num_pages": num_pages, "q": q,
            "k_cache": k, "v_cache": v, "scale": float(1.0 / np.sqrt(D)),
            "C": C, "Hq": Hq, "Hkv": Hkv, "D": D, "dtype": dtype, "page_size": page_size}


def make_small_lmhead_case(seed: int, C: int, H: int, V: int, dtype: str,
                           w_std: float = 0.02) -> dict:
    rng_h, rng_w, rng_i = np.random.default_rng(seed).spawn(3)
    return {"hidden": _normal_storage(rng_h, (C, H), dtype),
            "weight": _normal_storage(rng_w, (V, H), dtype, std=w_std),
            "seq_id": rng_i.integers(0, 2**62, size=C, dtype=np.int64),
            "step": rng_i.integers(0, 32768, size=C, dtype=np.int64).astype(np.int32),
            "seed": int(rng_i.integers(0, 2**63, dtype=np.int64)),
            "temperature": 1.0, "C": C, "H": H, "V": V, "dtype": dtype}


# --------------------------------------------------------------------------
# cross-stage importance-sampling batches
# --------------------------------------------------------------------------
def make_is_inputs(cfg: ISConfig, *, rng: Optional[np.random.Generator] = None,
                   sigma: Optional[float] = None, poison: bool = True) -> dict:
    """One batch for the token-level cross-stage ratio.

    Every trajectory is split at a random stage boundary `split_b` (uniform in
    0..len_b) into a buffered old-policy prefix and a suffix generated in the
    current rollout stage.  base ~ -Exp(1) is the old-policy log-prob of every
    token; `logp_buf` holds it on the prefix, `logp_roll` on the suffix (the
    other side of each is NaN-poisoned: it must never be read), and
    `logp_cur = fp32(base + N(0, sigma))` on all tokens.

    padded layout: B rows of `pad_to` slots, cu_seqlens = pad_to*b, the mask
    marks the first len_b slots of each row (the rest is padding);
    packed layout: cu_seqlens are the running sums of len_b, the mask is all
    ones except a seeded fraction of zeros.
    """
    rng = rng if rng is not None else substreams(cfg.seed)["is"]
    sigma = cfg.sigma if sigma is None else sigma
    lens = rng.integers(cfg.len_lo, cfg.len_hi, size=cfg.B, endpoint=True).astype(np.int64)
    split = np.array([rng.integers(0, n, endpoint=True) for n in lens], dtype=np.int32)
    if cfg.layout == "padded":
        seg = np.full(cfg.B, cfg.pad_to, dtype=np.int64)
    else:
        seg = lens
    cu = np.zeros(cfg.B + 1, dtype=np.int64)
    np.cumsum(seg, out=cu[1:])
    N = int(cu[-1])
    base = (-rng.exponential(1.0, size=N)).astype(np.float32)
    noise = rng.normal(0.0, sigma, size=N)
    logp_cur = (base.astype(np.float64) + noise).astype(np.float32)
    local = np.arange(N, dtype=np.int64) - np.repeat(cu[:-1], seg)
    is_buf = local < np.repeat(split.astype(np.int64), seg)
    nan = np.float32(np.nan) if poison else np.float32(0.0)
    logp_buf = np.where(is_buf, base, nan).astype(np.float32)
    logp_roll = np.where(is_buf, nan, base).astype(np.float32)
    if cfg.layout == "padded":
        mask = (local < np.repeat(lens, seg)).astype(np.uint8)
    else:
        mask = (rng.random(N) >= cfg.mask_zero_frac).astype(np.uint8)
    if poison:
        # masked-out inputs must not leak either
        logp_cur = np.where(mask == 1, logp_cur, np.float32(np.nan)).astype(np.float32)
    # One advantage per trajectory, drawn last so that the arrays above do not depend on
    # it: standard normal (group-normalised advantages have zero mean and unit
    # variance), every eighth exactly 0 (a group whose samples all earned the same reward).
    adv = rng.normal(0.0, 1.0, size=cfg.B).astype(np.float32)
    adv[rng.random(cfg.B) < 0.125] = 0.0
    return {"cfg": cfg, "B": cfg.B, "N": N, "lens": lens.astype(np.int32),
            "cu_seqlens": cu.astype(np.int32), "split": split, "mask": mask,
            "logp_cur": logp_cur, "logp_buf": logp_buf, "logp_roll": logp_roll,
            "adv": adv, "eps_low": cfg.eps_low, "eps_high": cfg.eps_high}


# --------------------------------------------------------------------------
# Stand-in for the transformer under the rollout loop: per-position tensors are seeded noise
# --------------------------------------------------------------------------
class StandInPolicy:
    """Seeded stand-in for a decoder under successive policy versions (no arithmetic of the
    method here: the rollout loop and the tests both draw their inputs from it).

    Trajectory tr = input * samples + sample has positions 0 .. prompt_len + resp_len - 1.
    Under policy version `ver`, position p of trajectory tr has a query [Hq, D], a key and a
    value [Hkv, D] and a final hidden state [H]: normal noise keyed by (seed, tr, ver), in
    the storage dtype.  The LM-head matrix of version ver is W0 + drift * ver * W1 (rounded to
    the storage dtype), so that successive policies differ a little, as after a training step.
    """

    def __init__(self, seed: int, prompt_len, resp_len, Hq: int, Hkv: int, D: int, H: int, V: int,
                 dtype: str = BF16, drift: float = 0.05):
        self.seed = int(seed)
        self.prompt_len = np.asarray(prompt_len, dtype=np.int64)
        self.resp_len = np.asarray(resp_len, dtype=np.int64)
        self.samples = int(self.resp_len.shape[1])
        self.Hq, self.Hkv, self.D, self.H, self.V = Hq, Hkv, D, H, V
        self.dtype = dtype
        self.drift = float(drift)
        self.scale = 1.0 / float(np.sqrt(D))
        self._tables = {}
        self._weights = {}
        rng = np.random.default_rng([self.seed, 0x57])
        self._w0 = rng.normal(0.0, 0.05, size=(V, H)).astype(np.float32)
        self._w1 = rng.normal(0.0, 0.05, size=(V, H)).astype(np.float32)

    def length(self, tr: int) -> int:
        i, s = divmod(int(tr), self.samples)
        return int(self.prompt_len[i] + self.resp_len[i, s])

    def tables(self, tr: int, ver: int) -> dict:
        key = (int(tr), int(ver))
        if key not in self._tables:
            rng = np.random.default_rng([self.seed, 1 + int(tr), int(ver)])
            L = self.length(tr)
            self._tables[key] = {
                "q": _normal_storage(rng, (L, self.Hq, self.D), self.dtype),
                "k": _normal_storage(rng, (L, self.Hkv, self.D), self.dtype),
                "v": _normal_storage(rng, (L, self.Hkv, self.D), self.dtype),
                "hidden": _normal_storage(rng, (L, self.H), self.dtype),
            }
        return self._tables[key]

    def weight(self, ver: int) -> np.ndarray:
        ver = int(ver)
        if ver not in self._weights:
            self._weights[ver] = to_storage(self._w0 + self.drift * ver * self._w1, self.dtype)
        return self._weights[ver]
