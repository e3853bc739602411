"""Shared comparison helpers for the GPU-vs-oracle parity tests.

Tolerances (stated by the benchmark spec; the fp32 ones follow from the
arithmetic: fp32 accumulation with hardware exp2/log2 of ~1 ulp over at most a few
thousand terms):
  attention output  max-abs <= 2e-2 for bf16 inputs, <= 1e-4 for fp32 inputs
  attention lse     <= 2e-3 (bf16) / 1e-4 (fp32) absolute
  log-probs, lse    <= 1e-3 absolute
  IS ratios         <= 1e-5 relative
  sampled tokens    bit-exact, except where the oracle's two largest perturbed
                    scores differ by < 1e-3: then either of the two is accepted and
                    the log-prob is checked against the oracle's log-prob of the
                    token the GPU chose
"""
import numpy as np

from oracle import copris_oracle as O
from paper_2511_05589_amd import workloads as W

ATTN_TOL = {W.BF16: 2e-2, W.F32: 1e-4}
ATTN_LSE_TOL = {W.BF16: 2e-3, W.F32: 1e-4}
LOGPROB_TOL = 1e-3
RATIO_RTOL = 1e-5
NEAR_TIE = 1e-3


def oracle_attn(inp, dtype):
    f = lambda k: W.to_f32(inp[k], dtype).astype(np.float64)
    return O.decode_attn(f("q"), f("k_cache"), f("v_cache"), inp["block_table"], inp["ctx_len"],
                         inp["scale"])


def check_attn(out, lse, ref_out, ref_lse, dtype, what=""):
    assert np.isfinite(out).all(), f"{what}: non-finite attention output"
    err = np.abs(out.astype(np.float64) - ref_out).max()
    assert err <= ATTN_TOL[dtype], f"{what}: attention max-abs error {err:.3e}"
    fin = np.isfinite(ref_lse)
    lerr = np.abs(lse.astype(np.float64)[fin] - ref_lse[fin]).max() if fin.any() else 0.0
    assert lerr <= ATTN_LSE_TOL[dtype], f"{what}: lse error {lerr:.3e}"
    assert (np.isneginf(lse[~fin])).all()
    return err


def oracle_lmhead(inp, dtype, rows=None):
    h = W.to_f32(inp["hidden"], dtype)
    sid, st = np.asarray(inp["seq_id"]), np.asarray(inp["step"])
    if rows is not None:
        h, sid, st = h[rows], sid[rows], st[rows]
    return O.lmhead_logprob(h, W.to_f32(inp["weight"], dtype), sid, st, inp["seed"],
                            inp["temperature"], return_full=True)


def check_lmhead(token, logprob, lse, ref, what=""):
    """ref: oracle dict with `logp`.  Returns the number of near-tie exemptions used."""
    C = token.shape[0]
    exempt = 0
    for c in range(C):
        t = int(token[c])
        if t != int(ref["token"][c]):
            gap = ref["best"][c] - ref["runner_up"][c]
            assert gap < NEAR_TIE and t == int(ref["second_token"][c]), (
                f"{what}: row {c} token {t} != oracle {int(ref['token'][c])} (gap {gap:.3e})")
            exempt += 1
        err = abs(float(logprob[c]) - ref["logp"][c, t])
        assert err <= LOGPROB_TOL, f"{what}: row {c} logprob error {err:.3e}"
    lerr = np.abs(lse.astype(np.float64) - ref["lse"]).max()
    assert lerr <= LOGPROB_TOL, f"{what}: lse error {lerr:.3e}"
    return exempt


def oracle_is(b, use_mask=True):
    return O.is_ratio(b["logp_cur"], b["logp_buf"], b["logp_roll"], b["cu_seqlens"], b["split"],
                      b["mask"] if use_mask else None, b["eps_low"], b["eps_high"])


def check_is(got, ref, b, use_mask=True, what=""):
    N, B = int(b["N"]), int(b["B"])
    counted = (np.asarray(b["mask"]) != 0) if (use_mask and b.get("mask") is not None) else np.ones(N, bool)
    cu = np.asarray(b["cu_seqlens"], dtype=np.int64)
    in_seq = np.zeros(N, dtype=bool)
    for s in range(B):
        in_seq[cu[s]:cu[s + 1]] = True
    counted = counted & in_seq
    for key in ("ratio", "ratio_clipped"):
        g, r = got[key].astype(np.float64), ref[key]
        assert (g[in_seq & ~counted] == 0.0).all(), f"{what}: {key} not 0 at masked tokens"
        gi, ri = g[counted], r[counted]
        both_inf = np.isinf(gi) & np.isinf(ri)
        # the reference may overflow fp32 where fp64 does not: accept inf vs > fp32 max
        big = ri > 3.4e38
        ok = both_inf | (big & np.isinf(gi))
        rel = np.abs(gi[~ok] - ri[~ok]) / np.maximum(np.abs(ri[~ok]), 1e-300)
        assert rel.size == 0 or rel.max() <= RATIO_RTOL, f"{what}: {key} rel error {rel.max():.3e}"
    np.testing.assert_array_equal(got["seq_cnt"], ref["seq_cnt"])
    lo, hi = 1.0 - b["eps_low"], 1.0 + b["eps_high"]
    r = ref["ratio"]
    border = counted & ((np.abs(r - lo) <= 1e-6 * lo) | (np.abs(r - hi) <= 1e-6 * hi))
    slack = np.add.reduceat(border.astype(np.int64), cu[:-1]) if N > 0 else np.zeros(B, np.int64)
    slack = np.where(cu[1:] > cu[:-1], slack, 0)
    assert (np.abs(got["seq_nclip"].astype(np.int64) - ref["seq_nclip"]) <= slack).all(), what
    srel = np.abs(got["seq_sum"].astype(np.float64) - ref["seq_sum"]) / np.maximum(ref["seq_sum"], 1.0)
    assert srel.max(initial=0.0) <= RATIO_RTOL, f"{what}: seq_sum rel error {srel.max():.3e}"


# ---- GRPO clipped surrogate -------------------------------------------------
SURR_RTOL = 1e-5      # same bar as the ratios the terms are built from


def oracle_grpo(b, use_mask=True):
    return O.grpo_surrogate(b["logp_cur"], b["logp_buf"], b["logp_roll"], b["cu_seqlens"], b["split"],
                            b["mask"] if use_mask else None, b["adv"], b["eps_low"], b["eps_high"])


def check_grpo(got, ref, b, use_mask=True, what=""):
    """Per-token terms to SURR_RTOL relative; the branch of the min is a decision that fp32
    and fp64 may take differently only where the ratio sits on a clip bound (then either
    branch's gradient is accepted); counts exact; sums relative to the sum of magnitudes."""
    N, B = int(b["N"]), int(b["B"])
    counted = (np.asarray(b["mask"]) != 0) if (use_mask and b.get("mask") is not None) else np.ones(N, bool)
    cu = np.asarray(b["cu_seqlens"], dtype=np.int64)
    lens = np.diff(cu)
    in_seq = np.zeros(N, dtype=bool)
    for s in range(B):
        in_seq[cu[s]:cu[s + 1]] = True
    counted = counted & in_seq
    A_tok = np.zeros(N)
    A_tok[in_seq] = np.repeat(np.asarray(b["adv"], dtype=np.float64), lens)
    ir = O.is_ratio(b["logp_cur"], b["logp_buf"], b["logp_roll"], b["cu_seqlens"], b["split"],
                    b["mask"] if use_mask else None, b["eps_low"], b["eps_high"])
    r = ir["ratio"]
    lo, hi = 1.0 - b["eps_low"], 1.0 + b["eps_high"]
    border = counted & ((np.abs(r - lo) <= 1e-6 * lo) | (np.abs(r - hi) <= 1e-6 * hi))
    for key in ("surr", "grad"):
        g = got[key].astype(np.float64)
        assert (g[in_seq & ~counted] == 0.0).all(), f"{what}: {key} not 0 at masked tokens"
    gs, rs = got["surr"].astype(np.float64)[counted], ref["surr"][counted]
    fin = np.isfinite(rs)
    assert (gs[~fin] == rs[~fin]).all() or np.isnan(rs[~fin]).all(), f"{what}: non-finite surr differs"
    err = np.abs(gs[fin] - rs[fin])
    assert (err <= SURR_RTOL * np.abs(rs[fin]) + 1e-30).all(), f"{what}: surr rel error {(err / np.maximum(np.abs(rs[fin]), 1e-300)).max():.3e}"
    gg, rg = got["grad"].astype(np.float64), ref["grad"]
    t1 = r * A_tok
    ok = np.abs(gg - rg) <= SURR_RTOL * np.abs(rg) + 1e-30
    either = border & ((gg == 0.0) | (np.abs(gg - t1) <= SURR_RTOL * np.abs(t1) + 1e-30))
    bad = counted & np.isfinite(rg) & ~(ok | either)
    assert not bad.any(), f"{what}: grad differs at {np.flatnonzero(bad)[:5]}"
    np.testing.assert_array_equal(got["seq_cnt"], ref["seq_cnt"])
    mag = np.add.reduceat(np.where(counted, np.abs(ref["surr"]), 0.0), cu[:-1]) if N > 0 else np.zeros(B)
    mag = np.where(lens > 0, mag, 0.0)
    finite_seq = np.isfinite(ref["seq_surr"])
    serr = np.abs(got["seq_surr"].astype(np.float64) - ref["seq_surr"])[finite_seq]
    assert (serr <= SURR_RTOL * np.maximum(mag[finite_seq], 1e-30)).all(), f"{what}: seq_surr error {serr.max():.3e}"
    if finite_seq.all():
        total = max(int(ref["seq_cnt"].sum()), 1)
        assert abs(got["obj_token_mean"] - ref["obj_token_mean"]) <= SURR_RTOL * mag.sum() / total + 1e-30, what
        per_seq_mag = np.where(ref["seq_cnt"] > 0, mag / np.maximum(ref["seq_cnt"], 1), 0.0)
        assert abs(got["obj_seq_mean"] - ref["obj_seq_mean"]) <= SURR_RTOL * per_seq_mag.sum() / max(B, 1) + 1e-30, what


# ---- log-prob of given tokens ------------------------------------------------
def oracle_token_logprob(hidden, weight, tokens, temperature, dtype, rows=None):
    h = W.to_f32(hidden, dtype)
    t = np.asarray(tokens)
    if rows is not None:
        h, t = h[rows], t[rows]
    return O.lmhead_token_logprob(h, W.to_f32(weight, dtype), t, temperature)


def check_token_logprob(logprob, lse, ref, what=""):
    err = np.abs(logprob.astype(np.float64) - ref["logprob"]).max()
    assert err <= LOGPROB_TOL, f"{what}: logprob error {err:.3e}"
    lerr = np.abs(lse.astype(np.float64) - ref["lse"]).max()
    assert lerr <= LOGPROB_TOL, f"{what}: lse error {lerr:.3e}"
    return err


# ---- re-prefill attention ------------------------------------------------------
def oracle_prefill(b, dtype):
    """Oracle outputs for every token, plus the oracle-filled caches (fp32 views of the
    storage values, NaN where no token maps)."""
    q, k, v = (W.to_f32(b[x], dtype) for x in ("q", "k", "v"))
    out, lse = O.prefill_attn(q, k, v, b["cu_seqlens"], b["scale"])
    kc, vc = oracle_page_fill(b, dtype)
    return out, lse, kc, vc


def oracle_page_fill(b, dtype):
    k, v = W.to_f32(b["k"], dtype), W.to_f32(b["v"], dtype)
    shape = (int(b["num_pages"]), k.shape[1], int(b["page_size"]), k.shape[2])
    kc = np.full(shape, np.nan, dtype=np.float32)
    vc = np.full(shape, np.nan, dtype=np.float32)
    O.kv_page_fill(k, v, b["cu_seqlens"], b["block_table"], kc, vc)
    return kc, vc


def oracle_prefill_rows(b, dtype, seq_tok, kc, vc):
    """Oracle rows for sampled (sequence, token) pairs through the decode oracle over the
    oracle-filled pages (the two oracles are pinned to each other on the CPU)."""
    q = W.to_f32(b["q"], dtype)
    cu = np.asarray(b["cu_seqlens"], dtype=np.int64)
    seqs = np.array([s for s, _ in seq_tok])
    toks = np.array([t for _, t in seq_tok])
    rows = cu[seqs] + toks
    out, lse = O.decode_attn(q[rows], kc, vc, np.asarray(b["block_table"])[seqs], toks + 1, b["scale"])
    return rows, out, lse
