"""CPU oracle for the CoPRIS rollout-decode hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what one decode step and the cross-stage
importance-sampling ratio compute.  It exists to check the HIP kernels; it is
not a fallback.  Only tests, the smoke check and the benchmark's `cpu_baseline`
leg may import it.  It shares no code with the HIP path and imports nothing
from the product package.

Every function is pinned by CPU-only tests against something other than itself
(brute-force loops on tiny inputs, library softmax / logsumexp, closed forms,
invariants, published Philox known-answer vectors); none is "parity unpinned".

What the paper fixes and what it leaves open:

* The paper runs generation inside a third-party inference engine (Appendix
  A.2) and gives no formula for attention, the LM head or the sampler.  Those
  are therefore the textbook definitions: scaled dot-product softmax attention
  of the one new query against the sequence's cached keys and values,
  log-softmax of the LM-head logits, and an exact draw from softmax(z / T).
* Table 4 fixes the sampler: temperature 1.0, top-p 1.0, top-k -1, i.e. the
  untruncated softmax.  Gumbel-max (argmax_v z_v + G_v with G_v iid standard
  Gumbel) is an exact sampler of that distribution.
* Section 4 ("Buffering of Partial Trajectories", Eq. 6) keeps, for each
  generated token, its log-probability under the policy that generated it.
* Section 4 ("Cross-stage Importance Sampling Correction", Eq. 8) defines the
  token ratio r = exp(L_cur - L_buffered); Eq. 3 clips it to [1-eps, 1+eps]
  (Table 4 lists separate low / high clip ratios, hence two epsilons).
"""
from __future__ import annotations

import numpy as np

# --------------------------------------------------------------------------
# Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
# as 1, 2, 3", SC'11).  Counter-based generator: 128-bit counter, 64-bit key,
# ten rounds.  Written with numpy uint64 lanes so whole vocab rows go at once.
# --------------------------------------------------------------------------
_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = np.uint64(0x9E3779B9)
_PHILOX_W1 = np.uint64(0xBB67AE85)
_MASK32 = np.uint64(0xFFFFFFFF)
_SH32 = np.uint64(32)


def philox4x32_10(counter, key):
    """counter: 4 arrays (or scalars) of 32-bit words c0..c3; key: 2 words k0,k1.
    Returns 4 uint32 arrays x0..x3 (broadcast shape of the inputs)."""
    c0, c1, c2, c3 = [np.asarray(c, dtype=np.uint64) & _MASK32 for c in counter]
    k0, k1 = [np.asarray(k, dtype=np.uint64) & _MASK32 for k in key]
    c0, c1, c2, c3, k0, k1 = np.broadcast_arrays(c0, c1, c2, c3, k0, k1)
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + _PHILOX_W0) & _MASK32
            k1 = (k1 + _PHILOX_W1) & _MASK32
        p0 = _PHILOX_M0 * c0          # 32x32 -> 64 bit, no overflow in uint64
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> _SH32, p0 & _MASK32
        hi1, lo1 = p1 >> _SH32, p1 & _MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def sampling_uniforms(seed: int, seq_id: int, step: int, V: int) -> np.ndarray:
    """The V uniforms of the stream Philox(seed, seq, step), fp64 in (0, 1).

    Vocabulary entry v takes word (v & 3) of the block whose counter is
    (v >> 2, step, seq_id low word, seq_id high word) under the key
    (seed low word, seed high word).  A word x maps to the midpoint of one of
    2^23 equal cells: u = ((x >> 9) + 0.5) / 2^23, which is exact in fp32 and
    never 0 or 1.  The stream depends on the trajectory and its token index
    only, never on the batch slot, so a resumed trajectory continues it.
    """
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    sid = int(seq_id) & 0xFFFFFFFFFFFFFFFF
    nblk = (V + 3) // 4
    blk = np.arange(nblk, dtype=np.uint64)
    x = philox4x32_10((blk, int(step) & 0xFFFFFFFF, sid & 0xFFFFFFFF, sid >> 32),
                      (seed & 0xFFFFFFFF, seed >> 32))
    words = np.stack(x, axis=1).reshape(-1)[:V]          # v -> word v&3 of block v>>2
    return ((words >> np.uint32(9)).astype(np.float64) + 0.5) * (2.0 ** -23)


def gumbel_noise(seed: int, seq_id: int, step: int, V: int) -> np.ndarray:
    """Standard Gumbel variates G_v = -ln(-ln u_v) for one (trajectory, token)."""
    u = sampling_uniforms(seed, seq_id, step, V)
    return -np.log(-np.log(u))


# --------------------------------------------------------------------------
# O1: paged-KV grouped-query decode attention
# --------------------------------------------------------------------------
def decode_attn(q, k_cache, v_cache, block_table, ctx_len, scale, page_size=None):
    """Softmax attention of each sequence's single new query over its context.

    q           [C, Hq, D]
    k_cache     [num_pages, Hkv, P, D]   (v_cache alike)
    block_table [C, max_pages] int       logical page j of seq i -> physical page
    ctx_len     [C] int                  tokens whose K/V are cached (includes
                                          the current token); entries of the
                                          block table past ceil(ctx/P) are ignored
    Query head h reads KV head h // (Hq // Hkv).
    Token t of a sequence lives in page block_table[i, t // P], slot t % P.
    Returns (out [C, Hq, D] fp64, lse [C, Hq] fp64); a sequence of length 0
    gives out = 0 and lse = -inf.
    """
    q = np.asarray(q, dtype=np.float64)
    C, Hq, D = q.shape
    _, Hkv, P, Dk = k_cache.shape
    assert Dk == D and Hq % Hkv == 0
    if page_size is not None:
        assert page_size == P
    g = Hq // Hkv
    out = np.zeros((C, Hq, D), dtype=np.float64)
    lse = np.full((C, Hq), -np.inf, dtype=np.float64)
    for i in range(C):
        n = int(ctx_len[i])
        if n == 0:
            continue
        npg = (n + P - 1) // P
        pages = np.asarray(block_table[i, :npg], dtype=np.int64)
        for kvh in range(Hkv):
            K = np.asarray(k_cache[pages, kvh], dtype=np.float64).reshape(npg * P, D)[:n]
            Vv = np.asarray(v_cache[pages, kvh], dtype=np.float64).reshape(npg * P, D)[:n]
            for h in range(kvh * g, (kvh + 1) * g):
                s = scale * (K @ q[i, h])
                m = s.max()
                p = np.exp(s - m)
                denom = p.sum()
                out[i, h] = (p @ Vv) / denom
                lse[i, h] = m + np.log(denom)
    return out, lse


# --------------------------------------------------------------------------
# Re-prefill of resumed partial trajectories (Section 4, "Prioritized Resumption";
# Section 5.3 names the re-prefilling of off-policy trajectories as a cost): the
# buffered prefix of a trajectory is run through the model again under the new
# weights, which refills its KV pages.  The attention part of that: causal
# self-attention over packed variable-length sequences, and the page fill.
# --------------------------------------------------------------------------
def prefill_attn(q, k, v, cu_seqlens, scale):
    """Causal softmax attention over a packed batch of sequences.

    q [T, Hq, D], k, v [T, Hkv, D]; sequence b owns rows cu_seqlens[b] ..
    cu_seqlens[b+1]-1 in token order.  Query head h reads KV head h // (Hq // Hkv).
    Token t of a sequence attends to tokens 0..t of the same sequence:
    out[t] = softmax_{u<=t}(scale * q[t].k[u]) . v[u].
    Returns (out [T, Hq, D] fp64, lse [T, Hq] fp64).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    assert Hq % Hkv == 0
    g = Hq // Hkv
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    out = np.zeros((T, Hq, D))
    lse = np.full((T, Hq), -np.inf)
    for b in range(cu.size - 1):
        s0, s1 = int(cu[b]), int(cu[b + 1])
        for t in range(s0, s1):
            for h in range(Hq):
                K = k[s0:t + 1, h // g]
                V = v[s0:t + 1, h // g]
                s = scale * (K @ q[t, h])
                m = s.max()
                p = np.exp(s - m)
                denom = p.sum()
                out[t, h] = (p @ V) / denom
                lse[t, h] = m + np.log(denom)
    return out, lse


def kv_page_fill(k, v, cu_seqlens, block_table, k_cache, v_cache):
    """Writes every sequence's K and V rows into its pages (in place): token t of
    sequence b goes to page block_table[b, t // P], slot t % P.  Slots that no token
    maps to are left as they were.  Pure data movement, in the caches' own dtype."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    P = k_cache.shape[2]
    for b in range(cu.size - 1):
        s0, s1 = int(cu[b]), int(cu[b + 1])
        for t in range(s1 - s0):
            page = int(block_table[b, t // P])
            k_cache[page, :, t % P, :] = k[s0 + t]
            v_cache[page, :, t % P, :] = v[s0 + t]


def pool_commands_apply(cmds, n_slot_cmds, n_page_cmds, seq_id, ctx_len, step, block_table):
    """The rollout manager's per-step commands applied to the pool state (in place):
    n_slot_cmds x (slot, trajectory or -1, ctx_len, step), then n_page_cmds x (slot, page index,
    physical page)."""
    cmds = [int(x) for x in cmds]
    for i in range(n_slot_cmds):
        slot, tr, n, g = cmds[4 * i:4 * i + 4]
        seq_id[slot], ctx_len[slot], step[slot] = tr, n, g
    base = 4 * n_slot_cmds
    for i in range(n_page_cmds):
        slot, idx, page = cmds[base + 3 * i:base + 3 * i + 3]
        block_table[slot, idx] = page


def kv_append(k_new, v_new, block_table, ctx_len, k_cache, v_cache):
    """One decode step's cache update (in place): row c of k_new / v_new [C, Hkv, D] is the key /
    value of the position being decoded by request c, token index ctx_len[c] - 1 of its context,
    i.e. page block_table[c, t // P], slot t % P.  Requests with ctx_len <= 0 hold nothing."""
    P = k_cache.shape[2]
    for c in range(len(ctx_len)):
        t = int(ctx_len[c]) - 1
        if t < 0:
            continue
        page = int(block_table[c, t // P])
        k_cache[page, :, t % P, :] = k_new[c]
        v_cache[page, :, t % P, :] = v_new[c]


# --------------------------------------------------------------------------
# The buffer of Section 4 ("Buffering of Partial Trajectories").  Per trajectory i the
# buffer holds the generated tokens and L_i, the log-prob of every token under the policy
# of the stage that generated it; Eq. 6: L_i is the concatenation, along the token axis,
# of the pieces L_i^(1), ..., L_i^(K) of the K stages the trajectory was generated over.
# Here the buffer is a dict trajectory -> list of pieces, one piece per stage that
# generated tokens of it: (stage, [tokens], [log-probs]).
# --------------------------------------------------------------------------
def buffer_append(buffer, traj, stage, token, logprob):
    """The token a request just sampled joins the piece of the current stage (a new piece is
    opened when the trajectory has none for this stage yet)."""
    pieces = buffer.setdefault(int(traj), [])
    if not pieces or pieces[-1][0] != int(stage):
        pieces.append((int(stage), [], []))
    pieces[-1][1].append(int(token))
    pieces[-1][2].append(float(logprob))


def buffer_concat(buffer, trajs, stage):
    """Eq. 6 for the trajectories of a training batch formed in `stage`.  For each, the pieces
    are concatenated in stage order.  Returns the packed batch the ratio of Eq. 8 is formed on:
      cu_seqlens [B+1], tokens [N]
      logp_buf  [N]  L_i restricted to the pieces of EARLIER stages (NaN on this stage's piece)
      logp_roll [N]  this stage's piece (NaN on the earlier ones)
      split [B]      tokens of trajectory b that come from earlier stages
    The earlier pieces form a prefix because stages follow each other in time."""
    cu, toks, lbuf, lroll, split = [0], [], [], [], []
    for tr in trajs:
        pieces = sorted(buffer.get(int(tr), []), key=lambda pc: pc[0])
        n_old = 0
        for st, tk, lp in pieces:
            toks.extend(tk)
            if st < stage:
                lbuf.extend(lp)
                lroll.extend([np.nan] * len(lp))
                n_old += len(lp)
            else:
                lbuf.extend([np.nan] * len(lp))
                lroll.extend(lp)
        split.append(n_old)
        cu.append(len(toks))
    return {"cu_seqlens": np.asarray(cu, dtype=np.int64), "tokens": np.asarray(toks, dtype=np.int64),
            "logp_buf": np.asarray(lbuf, dtype=np.float64), "logp_roll": np.asarray(lroll, dtype=np.float64),
            "split": np.asarray(split, dtype=np.int64)}


# --------------------------------------------------------------------------
# O2: LM head + log-softmax + Gumbel-max sample + chosen-token log-prob
# --------------------------------------------------------------------------
def lmhead_logprob(hidden, weight, seq_id, step, seed, temperature, return_full=False):
    """For every row c: z = (hidden[c] . weight[v]) / T over the vocabulary,
    lse = logsumexp(z), token = argmax_v (z_v + G_v) with the Gumbel variates of
    Philox(seed, seq_id[c], step[c]) (lowest index on an exact tie), and
    logprob = z[token] - lse: the log-probability, under the generating policy,
    that the buffer keeps for the token (Section 4, Eq. 6).

    Returns a dict: token int32 [C], logprob [C], lse [C], best [C] and
    runner_up [C] (the two largest perturbed scores), second_token int32 [C],
    and with return_full the full log-softmax matrix `logp` [C, V].
    """
    h = np.asarray(hidden, dtype=np.float64)
    w = np.asarray(weight, dtype=np.float64)
    C = h.shape[0]
    V = w.shape[0]
    z = (h @ w.T) / float(temperature)
    zmax = z.max(axis=1, keepdims=True)
    lse = (zmax + np.log(np.exp(z - zmax).sum(axis=1, keepdims=True)))[:, 0]
    token = np.empty(C, dtype=np.int32)
    second = np.empty(C, dtype=np.int32)
    best = np.empty(C)
    runner = np.empty(C)
    for c in range(C):
        score = z[c] + gumbel_noise(seed, int(seq_id[c]), int(step[c]), V)
        t = int(np.argmax(score))            # first index of the maximum
        token[c] = t
        best[c] = score[t]
        if V > 1:
            score[t] = -np.inf
            t2 = int(np.argmax(score))
            second[c] = t2
            runner[c] = score[t2]
        else:
            second[c] = t
            runner[c] = -np.inf
    res = {"token": token, "logprob": z[np.arange(C), token] - lse, "lse": lse,
           "best": best, "runner_up": runner, "second_token": second}
    if return_full:
        res["logp"] = z - lse[:, None]
    return res


# --------------------------------------------------------------------------
# Log-probability of GIVEN tokens under the current policy (Section 4, "Cross-stage
# Importance Sampling Correction": the buffered trajectories' log-probs are
# recomputed under pi_theta; they are L^(theta) in Eq. 8).
# --------------------------------------------------------------------------
def lmhead_token_logprob(hidden, weight, tokens, temperature):
    """For every row m: z = (hidden[m] . weight[v]) / T over the vocabulary,
    lse = logsumexp(z), logprob = z[tokens[m]] - lse.  No sampling: the token of
    each position is given (teacher forcing).  The same temperature-scaled
    log-softmax as `lmhead_logprob`, so that the ratio of Eq. 8 compares like
    with like.

    Returns logprob [M], lse [M] (fp64).
    """
    h = np.asarray(hidden, dtype=np.float64)
    w = np.asarray(weight, dtype=np.float64)
    tok = np.asarray(tokens, dtype=np.int64)
    z = (h @ w.T) / float(temperature)
    zmax = z.max(axis=1, keepdims=True)
    lse = (zmax + np.log(np.exp(z - zmax).sum(axis=1, keepdims=True)))[:, 0]
    return {"logprob": z[np.arange(h.shape[0]), tok] - lse, "lse": lse}


# --------------------------------------------------------------------------
# O3: token-level cross-stage importance ratio, clip, masked per-sequence sums
# --------------------------------------------------------------------------
def is_ratio(logp_cur, logp_buf, logp_roll, cu_seqlens, split, mask, eps_low, eps_high):
    """Eq. 8 with the clip of Eq. 3, over a packed batch.

    Sequence b owns tokens cu_seqlens[b] .. cu_seqlens[b+1]-1.  Its first
    split[b] tokens were generated in earlier stages, so their old-policy
    log-probs are the buffered ones (logp_buf); the rest were generated in the
    current rollout stage (logp_roll).  By Eq. 6 the buffer of a trajectory that
    spans K stages is one flat vector in token order, so K never appears here.
    For a counted token: r = exp(cur - old), rc = min(max(r, 1-eps_low), 1+eps_high).
    A masked token (mask == 0) gives 0 in both outputs and is not counted; the
    side of the split that is not selected is never read.

    Returns ratio [N], ratio_clipped [N] (fp64), seq_sum [B] (sum of rc over
    counted tokens), seq_cnt [B], seq_nclip [B] (counted tokens with rc != r).
    """
    cur = np.asarray(logp_cur, dtype=np.float64)
    buf = np.asarray(logp_buf, dtype=np.float64)
    roll = np.asarray(logp_roll, dtype=np.float64)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    B = cu.size - 1
    N = cur.size
    ratio = np.zeros(N)
    clipped = np.zeros(N)
    seq_sum = np.zeros(B)
    seq_cnt = np.zeros(B, dtype=np.int64)
    seq_nclip = np.zeros(B, dtype=np.int64)
    lo = 1.0 - float(eps_low)
    hi = 1.0 + float(eps_high)
    for b in range(B):
        s, e = int(cu[b]), int(cu[b + 1])
        if e <= s:
            continue
        k = min(max(int(split[b]), 0), e - s)
        old = np.concatenate([buf[s:s + k], roll[s + k:e]])
        counted = np.ones(e - s, dtype=bool) if mask is None else (np.asarray(mask[s:e]) != 0)
        with np.errstate(over="ignore", invalid="ignore"):
            r = np.exp(cur[s:e] - old)
        rc = np.minimum(np.maximum(r, lo), hi)
        ratio[s:e] = np.where(counted, r, 0.0)
        clipped[s:e] = np.where(counted, rc, 0.0)
        seq_sum[b] = rc[counted].sum()
        seq_cnt[b] = int(counted.sum())
        seq_nclip[b] = int((rc[counted] != r[counted]).sum())
    return {"ratio": ratio, "ratio_clipped": clipped, "seq_sum": seq_sum,
            "seq_cnt": seq_cnt, "seq_nclip": seq_nclip}


# --------------------------------------------------------------------------
# GRPO clipped surrogate on the cross-stage ratio (Section 3.1, Eq. 2-4).
# --------------------------------------------------------------------------
def grpo_surrogate(logp_cur, logp_buf, logp_roll, cu_seqlens, split, mask, adv, eps_low, eps_high):
    """Eq. 3 per token, on the ratio of Eq. 8, and the two aggregations of Eq. 2 / Table 4.

    The old-policy log-prob of a token is selected exactly as in `is_ratio`
    (buffered prefix of split[b] tokens, then this stage's rollout).  adv[b] is
    the group-normalised advantage of Eq. 4: one number per trajectory, the same
    for all of its tokens.  For a counted token of sequence b

        r  = exp(cur - old)                          (Eq. 8)
        rc = min(max(r, 1-eps_low), 1+eps_high)      (clip of Eq. 3; Table 4: 0.2 / 0.28)
        t1 = r * adv[b],  t2 = rc * adv[b]
        surr = t1 if t1 <= t2 else t2                (Eq. 3: the smaller of the two terms)
        grad = t1 if t1 <= t2 else 0                 (d surr / d cur: dr/dcur = r, and the
                                                      clipped term is constant wherever it
                                                      differs from the unclipped one)

    A masked token gives 0 in both outputs and is not counted.  Aggregations:
    token mean (Table 4, "loss aggregation mode"): sum of surr over all counted
    tokens / number of counted tokens; sequence mean (Eq. 2): mean over the B
    sequences of (sum of surr over the sequence's counted tokens / their number),
    a sequence without counted tokens contributing 0.  Table 4 sets the KL
    coefficient to 0, so Eq. 2's KL term is absent.

    Returns surr [N], grad [N], seq_surr [B], seq_cnt [B], obj_token_mean, obj_seq_mean.
    """
    cur = np.asarray(logp_cur, dtype=np.float64)
    buf = np.asarray(logp_buf, dtype=np.float64)
    roll = np.asarray(logp_roll, dtype=np.float64)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    A = np.asarray(adv, dtype=np.float64)
    B = cu.size - 1
    N = cur.size
    surr = np.zeros(N)
    grad = np.zeros(N)
    seq_surr = np.zeros(B)
    seq_cnt = np.zeros(B, dtype=np.int64)
    lo = 1.0 - float(eps_low)
    hi = 1.0 + float(eps_high)
    for b in range(B):
        s, e = int(cu[b]), int(cu[b + 1])
        if e <= s:
            continue
        k = min(max(int(split[b]), 0), e - s)
        old = np.concatenate([buf[s:s + k], roll[s + k:e]])
        counted = np.ones(e - s, dtype=bool) if mask is None else (np.asarray(mask[s:e]) != 0)
        with np.errstate(over="ignore", invalid="ignore"):
            r = np.exp(cur[s:e] - old)
            rc = np.minimum(np.maximum(r, lo), hi)
            t1 = r * A[b]
            t2 = rc * A[b]
            unclipped = t1 <= t2
        tok = np.where(unclipped, t1, t2)
        surr[s:e] = np.where(counted, tok, 0.0)
        grad[s:e] = np.where(counted & unclipped, t1, 0.0)
        seq_surr[b] = tok[counted].sum()
        seq_cnt[b] = int(counted.sum())
    total = int(seq_cnt.sum())
    obj_token_mean = float(seq_surr.sum() / total) if total > 0 else 0.0
    per_seq = np.where(seq_cnt > 0, seq_surr / np.maximum(seq_cnt, 1), 0.0)
    obj_seq_mean = float(per_seq.sum() / B) if B > 0 else 0.0
    return {"surr": surr, "grad": grad, "seq_surr": seq_surr, "seq_cnt": seq_cnt,
            "obj_token_mean": obj_token_mean, "obj_seq_mean": obj_seq_mean}


# --------------------------------------------------------------------------
# Rollout management (Section 4): concurrency-controlled generation, early
# termination, buffering of partial trajectories, prioritized resumption.
# Host logic, integers only.  The model is replaced by given response lengths.
# --------------------------------------------------------------------------
def rollout_schedule(prompt_len, resp_len, pool, batch_inputs, page_size=16, max_stages=None):
    """Token-by-token simulation of the rollout manager of Section 4.

    prompt_len [I] and resp_len [I, N]: input i has N trajectories; trajectory (i, s)
    stops after resp_len[i, s] >= 1 generated tokens.  `pool` is the fixed number of
    concurrent requests N' ("Concurrency-Controlled Generation"), `batch_inputs` the
    number B of inputs a training step needs ("Early Termination").

    A rollout stage k = 0, 1, ... runs under one policy version:
      * dispatch order: buffered unfinished trajectories first ("Prioritized
        Resumption"), in (input, sample) order, then trajectories that have not
        started, in (input, sample) order;
      * the pool is filled to N' requests; each decode step every active request
        generates one token, tagged with the stage (Eq. 6: the buffered log-probs of a
        trajectory are the concatenation of its per-stage pieces, so a tag per token
        is all the bookkeeping the concatenation needs); a request that reaches its
        length finishes and its slot is refilled before the next step;
      * after a step, if at least B inputs have all N trajectories finished, the stage
        stops at once: the B complete inputs with the lowest indices form the training
        batch and leave; running requests are paused and stay in the buffer with what
        they have generated; finished trajectories of incomplete inputs stay too;
      * a resumed trajectory is re-prefilled: prompt + tokens generated so far.
    KV pages (page_size tokens each) are held by running requests only; they are
    released when a request finishes or is paused (a new policy invalidates them).

    The simulation ends when a stage cannot complete B inputs (inputs exhausted) or
    after max_stages.  Returns a list of per-stage dicts:
      steps              decode steps of the stage
      generated          tokens generated in the stage
      slot_steps_idle    pool slots x steps that had no request to run
      batch_inputs       indices of the inputs consumed by the training step
      batch_tokens       response tokens of the batch
      batch_offpolicy    of which generated in an earlier stage (tag < k)
      batch_traj_offpolicy  trajectories of the batch with at least one such token
      max_staleness      max over batch tokens of (k - tag)
      resumed            trajectories resumed at the start of the stage
      reprefill_tokens   prompt + generated tokens re-prefilled for them
      paused             unfinished trajectories left in the buffer at the end
      buffered_complete  finished trajectories of incomplete inputs left in the buffer
      peak_pages         most KV pages held at once during the stage
    """
    prompt_len = [int(x) for x in prompt_len]
    resp = [[int(x) for x in row] for row in resp_len]
    I = len(prompt_len)
    N = len(resp[0]) if I else 0
    gen = [[0] * N for _ in range(I)]            # tokens generated so far
    tags = [[[] for _ in range(N)] for _ in range(I)]   # stage tag of every generated token
    started = [[False] * N for _ in range(I)]
    consumed = [False] * I
    stages = []
    k = 0

    def pages(i, s):
        return (prompt_len[i] + gen[i][s] + page_size - 1) // page_size

    while max_stages is None or k < max_stages:
        # dispatch queue of this stage
        resume_q = [(i, s) for i in range(I) for s in range(N)
                    if not consumed[i] and started[i][s] and gen[i][s] < resp[i][s]]
        fresh_q = [(i, s) for i in range(I) for s in range(N) if not started[i][s]]
        queue = resume_q + fresh_q
        n_resume = len(resume_q)
        qpos = 0
        active = []
        st = {"steps": 0, "generated": 0, "slot_steps_idle": 0, "resumed": 0, "reprefill_tokens": 0,
              "peak_pages": 0}

        def complete_inputs():
            return [i for i in range(I) if not consumed[i]
                    and all(started[i][s] and gen[i][s] >= resp[i][s] for s in range(N))]

        done = None
        if len(complete_inputs()) >= batch_inputs:
            done = complete_inputs()          # enough inputs were already complete in the buffer
        while done is None:
            while len(active) < pool and qpos < len(queue):
                i, s = queue[qpos]
                if qpos < n_resume:
                    st["resumed"] += 1
                    st["reprefill_tokens"] += prompt_len[i] + gen[i][s]
                qpos += 1
                started[i][s] = True
                active.append((i, s))
            if not active:
                break                           # nothing left to run: the stage cannot complete
            # one decode step
            st["steps"] += 1
            st["slot_steps_idle"] += pool - len(active)
            for i, s in active:
                gen[i][s] += 1
                tags[i][s].append(k)
            st["generated"] += len(active)
            st["peak_pages"] = max(st["peak_pages"], sum(pages(i, s) for i, s in active))
            active = [(i, s) for i, s in active if gen[i][s] < resp[i][s]]
            ci = complete_inputs()
            if len(ci) >= batch_inputs:
                done = ci
        if done is None:
            break
        batch = done[:batch_inputs]
        toks = [t for i in batch for s in range(N) for t in tags[i][s]]
        st["batch_inputs"] = batch
        st["batch_tokens"] = len(toks)
        st["batch_offpolicy"] = sum(1 for t in toks if t < k)
        st["batch_traj_offpolicy"] = sum(1 for i in batch for s in range(N) if any(t < k for t in tags[i][s]))
        st["max_staleness"] = max((k - t for t in toks), default=0)
        for i in batch:
            consumed[i] = True
        st["paused"] = sum(1 for i in range(I) for s in range(N)
                           if not consumed[i] and started[i][s] and gen[i][s] < resp[i][s])
        st["buffered_complete"] = sum(1 for i in range(I) for s in range(N)
                                      if not consumed[i] and started[i][s] and gen[i][s] >= resp[i][s])
        stages.append(st)
        k += 1
    return stages
