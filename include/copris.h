/*
 * copris.h - C ABI of the CoPRIS rollout-decode hot path on MI355X (gfx950).
 *
 * One decode step of a fixed concurrency pool of C requests (Section 4,
 * "Concurrency-Controlled Generation": N' requests stay in flight) with ragged,
 * long-tailed context lengths (Section 3.2), some of them partial trajectories
 * resumed from the buffer (Section 4, "Prioritized Resumption"):
 *
 *   copris_decode_attn     paged-KV grouped-query decode attention
 *   copris_lmhead_logprob  LM-head projection fused with log-softmax, Gumbel-max
 *                          sampling and the chosen token's log-probability: the
 *                          per-token log-prob under the generating policy that the
 *                          buffer keeps (Section 4, "Buffering of Partial
 *                          Trajectories", Eq. 6)
 *   copris_is_ratio        token-level cross-stage importance ratio (Section 4,
 *                          "Cross-stage Importance Sampling Correction", Eq. 8)
 *                          with the clip of Eq. 3 and masked per-sequence sums
 *
 * and the steps around it:
 *
 *   copris_grpo_surrogate        the clipped surrogate of Eq. 3 on that ratio, its
 *                                derivative and the aggregations of Eq. 2 / Table 4
 *   copris_lmhead_token_logprob  log-probs of given tokens under the current policy
 *                                (the recomputed side of Eq. 8), micro-batch sized
 *   copris_prefill_attn          causal attention over resumed partial trajectories,
 *                                refilling their KV pages (re-prefill, Section 5.3)
 *   copris_rollout_schedule      the rollout manager of Section 4 for given response
 *                                lengths (host function)
 *
 * Conventions
 *   - Plain C.  Every pointer argument is a DEVICE pointer owned by the caller,
 *     unless stated otherwise.  The library allocates nothing, never
 *     synchronises and never copies to the host: every call only enqueues
 *     kernels on `stream` (a hipStream_t passed as void*; NULL = the null
 *     stream) and returns.
 *   - Outputs are fully overwritten; inputs are never modified.  The only global
 *     state is the profiling hook (process-wide) and the static array of
 *     copris_lmhead_logprob_noalloc: every other call is re-entrant across streams
 *     given disjoint workspaces and outputs.
 *   - Tensors are dense, row-major, last index fastest, and their base
 *     addresses must be 16-byte aligned.
 *   - dtype: COPRIS_F32 (0) or COPRIS_BF16 (1).  bf16 tensors accumulate in fp32.
 *   - Return value: COPRIS_OK (0) or a negative error code.  Arguments are
 *     checked on the host without touching device memory; a rejected call
 *     enqueues nothing.  The CONTENTS of device arrays (a block-table entry
 *     outside [0, num_pages), cu_seqlens that do not increase, ...) cannot be
 *     checked without a device round trip and are the caller's responsibility.
 */
#ifndef COPRIS_H
#define COPRIS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define COPRIS_OK            0
#define COPRIS_EINVAL       -1   /* null pointer, bad shape, misaligned base, bad scalar */
#define COPRIS_EWORKSPACE   -2   /* workspace smaller than the *_workspace_bytes query   */
#define COPRIS_EUNSUPPORTED -3   /* dtype / head_dim / page_size / group size not built  */
#define COPRIS_ELAUNCH      -4   /* the HIP runtime reported an error at launch          */

#define COPRIS_F32  0
#define COPRIS_BF16 1

/* Text for an error code (static storage, host pointer, never NULL). */
const char* copris_strerror(int code);

/* Library version, "major.minor.patch" (static storage, host pointer). */
const char* copris_version(void);

/* After a call on this thread returned COPRIS_ELAUNCH: which kernel failed to launch
 * and the HIP runtime's error text (thread-local storage, host pointer, "" if none). */
const char* copris_last_error_detail(void);

/* Profiling aid.  While a hook is set, every kernel launch of the library calls it on
 * the launching host thread, before (phase 0) and after (phase 1) the launch is
 * enqueued, with the kernel's name and the stream: a caller can record events there
 * to time individual kernels.  Process-wide, not thread-safe against concurrent
 * calls; pass NULL to remove it.  The hook must not call back into the library. */
typedef void (*copris_launch_hook_fn)(const char* kernel, int phase, void* stream, void* user);
void copris_set_launch_hook(copris_launch_hook_fn hook, void* user);

/* ------------------------------------------------------------------------
 * Paged-KV grouped-query decode attention.
 *
 * The paper runs generation inside an inference engine (Appendix A.2) and
 * states no formula; the operation is softmax attention of each request's one
 * new query over its own cached context:
 *
 *   for sequence i, query head h, kv head kvh = h / (Hq/Hkv), tokens t < ctx_len[i]:
 *     page = block_table[i][t / page_size],  slot = t % page_size
 *     s_t  = scale * sum_d q[i][h][d] * k_cache[page][kvh][slot][d]
 *     out[i][h][:] = sum_t softmax(s)_t * v_cache[page][kvh][slot][:]
 *     lse[i][h]    = log sum_t exp(s_t)
 *
 * Work is split along the context, so a few very long resumed trajectories do not
 * serialise the step: for bf16 / D = 128 / page 16 the (kv head, page) slabs of the
 * whole pool form one stream that is cut into equal shares, one per wavefront, and
 * the pieces of a sequence are combined in share order; other shapes split every
 * context into 512-token chunks, combined in chunk order.  Either way the partition
 * depends on ctx_len only: results are bitwise reproducible and do not depend on the
 * physical page order.
 *
 *   q           [C, Hq, D]                      dtype
 *   k_cache     [num_pages, Hkv, page_size, D]  dtype; RoPE already applied
 *   v_cache     [num_pages, Hkv, page_size, D]  dtype
 *   block_table [C, max_pages] int32; entries at or past ceil(ctx_len/page_size)
 *               are ignored (may hold anything)
 *   ctx_len     [C] int32, 0 <= ctx_len[i] <= max_pages*page_size; counts every
 *               token whose K/V is in the cache, the current one included
 *   out         [C, Hq, D] dtype (bf16: rounded to nearest even)
 *   lse         [C, Hq] fp32, or NULL
 *   workspace   device scratch of at least copris_decode_attn_workspace_bytes()
 *               bytes, 256-byte aligned; contents on entry and exit are arbitrary
 *   scale       usually 1/sqrt(D)
 *
 * Slots of a last page at or past ctx_len, and pages the block table does not
 * reference, are never allowed to influence the result (they may hold NaN).
 * ctx_len[i] == 0 gives out = 0, lse = -inf.
 * Every block_table entry that is used must lie in [0, num_pages) (not checked: that
 * would need a device round trip).
 * Supported: D in {64, 128}; page_size a divisor of 512; Hq/Hkv <= 16; C*Hkv < 2^20;
 * C * ceil(max_pages*page_size / 512) * Hkv < 2^31.
 * ------------------------------------------------------------------------ */
size_t copris_decode_attn_workspace_bytes(int C, int Hq, int Hkv, int D,
                                          int page_size, int max_pages);

int copris_decode_attn(const void* q, const void* k_cache, const void* v_cache,
                       const int32_t* block_table, const int32_t* ctx_len,
                       void* out, float* lse,
                       void* workspace, size_t workspace_bytes,
                       int C, int Hq, int Hkv, int D, int page_size, int max_pages,
                       int64_t num_pages, float scale, int dtype, void* stream);

/* ------------------------------------------------------------------------
 * Re-prefill attention of resumed partial trajectories.
 *
 * Section 4, "Prioritized Resumption": the buffered partial trajectories are continued
 * in the next rollout stage, under new weights, so their context has to be run through
 * the model again (Section 5.3 names this re-prefilling as a cost of high concurrency).
 * This is the attention of that pass and the refill of the KV pages: causal softmax
 * attention over a packed batch of variable-length sequences,
 *
 *   out[j, h, :] = softmax_{u <= t}( scale * q[j, h, :] . k[s+u, h / g, :] ) . v[s+u, h / g, :]
 *
 * for token t of sequence b (s = cu_seqlens[b], j = s + t, g = Hq / Hkv), and
 *
 *   k_cache[block_table[b, t / P], kvh, t % P, :] = k[j, kvh, :]      (v_cache alike)
 *
 * after which copris_decode_attn can continue the sequence with ctx_len = its length.
 * Cache slots that no token maps to are not written.
 *
 *   q    [T, Hq, D]  dtype        k, v [T, Hkv, D] dtype (packed, token-major)
 *   cu_seqlens  [B+1] int32, cu[0] = 0, cu[B] = T
 *   block_table [B, max_pages] int32, entries >= ceil(len_b / P) ignored
 *   k_cache, v_cache [num_pages, Hkv, P, D] dtype, written
 *   out  [T, Hq, D]  dtype        lse [T, Hq] fp32 or NULL
 *   max_seqlen  an upper bound of the sequence lengths (sizes the launch)
 *
 * No workspace.  Compiled for dtype = COPRIS_BF16, D = 128, page_size = 16 and
 * Hq / Hkv <= 8; anything else returns COPRIS_EUNSUPPORTED.
 * ------------------------------------------------------------------------ */
int copris_prefill_attn(const void* q, const void* k, const void* v,
                        const int32_t* cu_seqlens, const int32_t* block_table,
                        void* k_cache, void* v_cache, void* out, float* lse,
                        int B, int64_t T, int Hq, int Hkv, int D, int page_size,
                        int max_pages, int64_t num_pages, int max_seqlen,
                        float scale, int dtype, void* stream);

/* ------------------------------------------------------------------------
 * LM head fused with log-softmax, Gumbel-max sampling and log-prob gather.
 *
 * Table 4 fixes the rollout sampler (temperature 1.0, top-p 1.0, top-k -1): one
 * draw from the untruncated softmax.  Section 4 (Eq. 6) keeps the drawn token's
 * log-probability under the generating policy.  For every row c:
 *
 *   z_v     = (sum_k hidden[c][k] * weight[v][k]) / temperature      v = 0..V-1
 *   lse     = log sum_v exp(z_v)
 *   u_v     = uniform of Philox4x32-10 (Salmon et al., SC'11):
 *               key     = (seed & 0xffffffff, seed >> 32)
 *               counter = (v >> 2, step[c], seq_id[c] & 0xffffffff, seq_id[c] >> 32)
 *               x       = output word (v & 3);  u_v = ((x >> 9) + 0.5) * 2^-23
 *   token   = argmax_v (z_v - ln(-ln u_v))      (lowest v on an exact tie)
 *   logprob = z_token - lse
 *
 * The V logits are never written to memory; the weight matrix is streamed once.
 * The random stream depends on (seed, seq_id, step) only - not on the slot c,
 * the batch size or the launch shape - so a resumed trajectory continues it.
 *
 *   hidden  [C, H] dtype            weight [V, H] dtype (row v = vocabulary entry v)
 *   seq_id  [C] int64  stable trajectory id (not the slot index)
 *   step    [C] int32  index of the token being generated within its response
 *   token   [C] int32 out     logprob [C] fp32 out     lse [C] fp32 out or NULL
 *   workspace  at least copris_lmhead_logprob_workspace_bytes() bytes, 256-byte aligned
 *
 * Requires temperature > 0, H % 8 == 0 for bf16 (H % 4 == 0 for fp32), V < 2^31.
 * ------------------------------------------------------------------------ */
size_t copris_lmhead_logprob_workspace_bytes(int C, int H, int V);

int copris_lmhead_logprob(const void* hidden, const void* weight,
                          const int64_t* seq_id, const int32_t* step,
                          uint64_t seed, float temperature,
                          int32_t* token, float* logprob, float* lse,
                          void* workspace, size_t workspace_bytes,
                          int C, int H, int V, int dtype, void* stream);

/* ------------------------------------------------------------------------
 * copris_lmhead_logprob for callers that cannot allocate device memory or carry a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments and results as copris_lmhead_logprob, without the
 * workspace: the per-(row, part) partials go to a static device array of the library
 * (copris_lmhead_logprob_noalloc_max_bytes() bytes, 4 MiB; each GPU the library is
 * used on holds one until the process ends).  The call allocates nothing and frees
 * nothing.  The device that `stream` belongs to must be the current device.
 *
 * A shape that needs more partials than the array holds returns COPRIS_EWORKSPACE (the
 * text of copris_last_error_detail() gives the sizes) and enqueues nothing.  The need
 * is C x parts x 20 bytes: for bf16 with H % 64 == 0, parts = min(512 / ceil(C / 256),
 * ceil(V / 128)), at most 2.6 MB for any C up to 200 000; for other shapes parts =
 * ceil(V / 64), e.g. C <= 88 at V = 151 936.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 * (different streams, or threads) race.  Nothing in it needs clearing between calls:
 * every partial a call reads it has written first.
 * ------------------------------------------------------------------------ */
size_t copris_lmhead_logprob_noalloc_max_bytes(void);

int copris_lmhead_logprob_noalloc(const void* hidden, const void* weight,
                                  const int64_t* seq_id, const int32_t* step,
                                  uint64_t seed, float temperature,
                                  int32_t* token, float* logprob, float* lse,
                                  int C, int H, int V, int dtype, void* stream);

/* ------------------------------------------------------------------------
 * Log-probability of GIVEN tokens under the current policy (teacher forcing).
 *
 * Section 4, "Cross-stage Importance Sampling Correction": the log-probs of the
 * buffered trajectories' tokens are recomputed under the current policy; they are
 * L^(theta) in Eq. 8 (logp_cur of copris_is_ratio).  For every position m:
 *
 *   z[v]       = dot(hidden[m, :], weight[v, :]) / temperature
 *   lse[m]     = log sum_v exp(z[v])
 *   logprob[m] = z[tokens[m]] - lse[m]
 *
 * the same temperature-scaled log-softmax as copris_lmhead_logprob, without the
 * sampler.  The logits are not materialised.  A token outside [0, V) gives NaN.
 *
 *   hidden  [M, H] dtype       weight [V, H] dtype (row v = vocabulary entry v)
 *   tokens  [M] int32          logprob [M] fp32 out     lse [M] fp32 out or NULL
 *   workspace  at least copris_lmhead_token_logprob_workspace_bytes() bytes, 256-byte aligned
 *
 * Requires temperature > 0, H % 8 == 0 for bf16 (H % 4 == 0 for fp32), V < 2^31.
 * ------------------------------------------------------------------------ */
size_t copris_lmhead_token_logprob_workspace_bytes(int M, int H, int V, int dtype);

int copris_lmhead_token_logprob(const void* hidden, const void* weight, const int32_t* tokens,
                                float temperature, float* logprob, float* lse,
                                void* workspace, size_t workspace_bytes,
                                int M, int H, int V, int dtype, void* stream);

/* ------------------------------------------------------------------------
 * Token-level cross-stage importance ratio over a packed batch.
 *
 * Eq. 8: r = exp(L_cur - L_old); Eq. 3: clip(r, 1-eps_low, 1+eps_high) (Table 4
 * lists clip ratio low and high separately).  By Eq. 6 the buffered log-probs of
 * a trajectory that spans several stages are one vector in token order, so a
 * trajectory is described by one number: split[b], how many of its tokens were
 * generated in earlier stages.  For sequence b, local index t, j = cu_seqlens[b]+t:
 *
 *   old = t < split[b] ? logp_buf[j] : logp_roll[j]     (the other side is not read)
 *   if mask && !mask[j]:  ratio[j] = ratio_clipped[j] = 0, token not counted
 *   else r = exp(logp_cur[j] - old); rc = min(max(r, 1-eps_low), 1+eps_high)
 *        seq_sum[b] += rc; seq_cnt[b] += 1; seq_nclip[b] += (rc != r)
 *
 * Nothing is clamped before the exponential: an overflow to +inf is clipped to
 * 1+eps_high; NaN in a counted input propagates.  Sums are formed in a fixed
 * order (bitwise reproducible).
 *
 *   logp_cur, logp_buf, logp_roll [N] fp32      cu_seqlens [B+1] int32, cu[0]=0, cu[B]=N
 *   split [B] int32 in 0..len_b                 mask [N] uint8 or NULL (all counted)
 *   ratio, ratio_clipped [N] fp32 out           seq_sum [B] fp32, seq_cnt, seq_nclip [B] int32 out
 *
 * Requires 0 <= eps_low < 1, eps_high >= 0, B >= 0, 0 <= N < 2^31.
 * ------------------------------------------------------------------------ */
int copris_is_ratio(const float* logp_cur, const float* logp_buf, const float* logp_roll,
                    const int32_t* cu_seqlens, const int32_t* split, const uint8_t* mask,
                    float eps_low, float eps_high,
                    float* ratio, float* ratio_clipped,
                    float* seq_sum, int32_t* seq_cnt, int32_t* seq_nclip,
                    int B, int64_t N, void* stream);

/* ------------------------------------------------------------------------
 * GRPO clipped surrogate on the cross-stage ratio, over the same packed batch.
 *
 * Section 3.1, Eq. 3: L = min(r A, clip(r, 1-eps_low, 1+eps_high) A) per token,
 * with r the ratio of Eq. 8 (old-policy log-prob selected by split[b] exactly as
 * in copris_is_ratio) and A = adv[b] the group-normalised advantage of Eq. 4, one
 * number per trajectory.  For a counted token:
 *
 *   t1 = r * adv[b];  t2 = clip(r) * adv[b]
 *   surr[j] = t1 <= t2 ? t1 : t2
 *   grad[j] = t1 <= t2 ? t1 : 0        d surr[j] / d logp_cur[j]  (dr/dlogp_cur = r; the
 *                                      clipped term is constant where it differs from r)
 *   seq_surr[b] += surr[j]; seq_cnt[b] += 1
 *
 * A masked token gives surr = grad = 0 and is not counted.  Then
 *
 *   objective[0] = sum_b seq_surr[b] / sum_b seq_cnt[b]       token mean (Table 4,
 *                                                             "loss aggregation mode")
 *   objective[1] = (1/B) sum_b seq_surr[b] / seq_cnt[b]       Eq. 2: mean over the
 *                  sequences of the per-sequence mean; a sequence without counted
 *                  tokens contributes 0
 *
 * Both are to be maximised (the loss is their negative); Table 4 sets the KL
 * coefficient to 0, so Eq. 2's KL term is absent.  grad is not divided by any
 * count: the gradient of objective[0] with respect to logp_cur[j] is
 * grad[j] / sum_b seq_cnt[b].  No clamp before the exponential; comparisons with
 * NaN are false (a NaN ratio gives surr = t2 = NaN, grad = 0).  Sums are formed in
 * a fixed order (bitwise reproducible); the two objectives are accumulated in fp64.
 *
 *   logp_cur, logp_buf, logp_roll [N] fp32      cu_seqlens [B+1] int32, cu[0]=0, cu[B]=N
 *   split [B] int32 in 0..len_b                 mask [N] uint8 or NULL (all counted)
 *   adv [B] fp32                                surr, grad [N] fp32 out
 *   seq_surr [B] fp32, seq_cnt [B] int32 out    objective [2] fp32 out
 *
 * Requires 0 <= eps_low < 1, eps_high >= 0, B >= 0, 0 <= N < 2^31; the [N] arrays
 * and mask 16-byte aligned.  B == 0 writes objective = {0, 0}.
 * ------------------------------------------------------------------------ */
int copris_grpo_surrogate(const float* logp_cur, const float* logp_buf, const float* logp_roll,
                          const int32_t* cu_seqlens, const int32_t* split, const uint8_t* mask,
                          const float* adv, float eps_low, float eps_high,
                          float* surr, float* grad, float* seq_surr, int32_t* seq_cnt,
                          float* objective, int B, int64_t N, void* stream);

/* ------------------------------------------------------------------------
 * Rollout manager: the schedule of Section 4 for given response lengths.  HOST
 * function: every pointer is host memory, nothing touches the GPU.
 *
 * "Concurrency-Controlled Generation": a fixed pool of `pool` (N') requests is kept
 * in flight; a finished trajectory's slot is refilled at once.  "Early Termination": a
 * stage stops as soon as `batch_inputs` (B) inputs have all of their `samples` (N)
 * trajectories finished; the B complete inputs with the lowest indices leave as the
 * training batch.  "Buffering of Partial Trajectories": running requests are paused
 * and keep what they generated, with the stage each token was generated in (the
 * per-stage pieces of Eq. 6); finished trajectories of incomplete inputs stay too.
 * "Prioritized Resumption": the next stage dispatches the paused trajectories first,
 * in (input, sample) order, then trajectories that have not started, in the same
 * order; a resumed trajectory is re-prefilled (prompt + generated tokens).  One
 * decode step gives every running request one token.  KV pages of page_size tokens
 * are held by running requests only.
 *
 *   prompt_len [n_inputs] int32 >= 0      resp_len [n_inputs, samples] int32 >= 1
 *   stats      [max_stages] out           batch_out [max_stages, batch_inputs] int32 out
 *   n_stages   out: stages that completed a batch (the schedule ends when the inputs
 *              cannot complete another one, or after max_stages)
 * ------------------------------------------------------------------------ */
typedef struct copris_stage_stats {
  int64_t steps;                /* decode steps of the stage */
  int64_t generated;            /* tokens generated in the stage */
  int64_t slot_steps_idle;      /* pool slots x steps without a request to run */
  int64_t batch_tokens;         /* response tokens of the training batch */
  int64_t batch_offpolicy;      /* ... of which generated in an earlier stage */
  int64_t batch_traj_offpolicy; /* trajectories of the batch with such tokens */
  int64_t max_staleness;        /* max over batch tokens of (stage - stage generated in) */
  int64_t resumed;              /* trajectories resumed in the stage */
  int64_t reprefill_tokens;     /* prompt + generated tokens re-prefilled for them */
  int64_t paused;               /* unfinished trajectories in the buffer at the end */
  int64_t buffered_complete;    /* finished trajectories of incomplete inputs, likewise */
  int64_t peak_pages;           /* most KV pages held at once */
} copris_stage_stats;

int copris_rollout_schedule(const int32_t* prompt_len, const int32_t* resp_len,
                            int n_inputs, int samples, int pool, int batch_inputs,
                            int page_size, int max_stages, copris_stage_stats* stats,
                            int32_t* batch_out, int* n_stages);

/* ------------------------------------------------------------------------
 * Rollout manager, one decode step at a time: the same rules as
 * copris_rollout_schedule for a caller that runs the kernels between the calls.
 * HOST functions; every pointer is host memory.
 *
 * The manager takes every decision of Section 4.  "Concurrency-Controlled
 * Generation": which trajectory occupies which of the `pool` (N') slots; an emptied
 * slot is refilled before the next step.  "Prioritized Resumption": paused
 * trajectories enter first, in (input, sample) order, and are re-prefilled with
 * prompt + generated tokens.  "Early Termination": next_step answers
 * COPRIS_ROLLOUT_STAGE_END as soon as `batch_inputs` (B) inputs have all their
 * samples.  "Buffering of Partial Trajectories": end_stage pauses what still runs
 * and names the batch, with each trajectory's number of tokens from earlier stages
 * (the boundary between the buffered pieces of Eq. 6 and this stage's piece: `split`
 * of copris_is_ratio).  It also owns the KV page allocator: pages are taken from a
 * free list in `page_order` (NULL: ascending), held by running requests only, and
 * returned when a request finishes or is paused (the next policy invalidates them).
 *
 * A trajectory ends after resp_len[input][sample] tokens, or earlier when the caller
 * reports an end-of-sequence token with copris_rollout_stop.  With lengths known in
 * advance a whole stage can be enqueued without reading anything back from the device.
 *
 * Protocol:  create;  per stage:  begin_stage;  loop { next_step -> STEP: run the
 * plan, optionally copris_rollout_stop;  STAGE_END: leave the loop;  EXHAUSTED: no
 * batch can be completed any more };  end_stage;  ...  destroy.
 *
 * copris_rollout_create   num_pages >= pool * ceil(max(prompt + resp) / page_size), so
 *                         that no request is ever preempted; page_order [num_pages] a
 *                         permutation of 0..num_pages-1 or NULL; *out receives the
 *                         handle (owned by the caller until copris_rollout_destroy).
 * copris_rollout_begin_stage  returns the stage index (>= 0) or a negative error.
 * copris_rollout_next_step    fills *plan; the arrays it points to belong to the
 *                         manager and stay valid until the next call on the handle.
 *                         Returns COPRIS_ROLLOUT_STEP / _STAGE_END / _EXHAUSTED or a
 *                         negative error.  A returned STEP counts as run.
 * copris_rollout_stop     slots [n]: requests whose last generated token ended them.
 * copris_rollout_end_stage    only after STAGE_END.  stats [1]; batch_inputs_out
 *                         [batch_inputs]; batch_traj_out [batch_inputs * samples][3] =
 *                         {trajectory (input * samples + sample), response tokens,
 *                         tokens generated in earlier stages}.
 * Not thread-safe per handle.  Errors: COPRIS_EINVAL.
 * ------------------------------------------------------------------------ */
#define COPRIS_ROLLOUT_STEP      0
#define COPRIS_ROLLOUT_STAGE_END 1
#define COPRIS_ROLLOUT_EXHAUSTED 2

typedef struct copris_rollout copris_rollout;

typedef struct copris_rollout_plan {
  int32_t stage;          /* stage (policy version) the step belongs to */
  int32_t n_active;       /* requests that run in this step */
  int32_t n_entered;      /* requests that enter the pool before this step */
  int32_t n_finishing;    /* requests that generate their last token in this step */
  int32_t n_slot_cmds;    /* slot commands in cmds */
  int32_t n_page_cmds;    /* page commands in cmds */
  const int32_t* slot_traj;    /* [pool] trajectory in every slot during the step, -1 = idle */
  const int32_t* entered;      /* [n_entered][4] slot, trajectory, tokens to (re-)prefill
                                  (prompt + generated), 1 if resumed from the buffer */
  const int32_t* finishing;    /* [n_finishing] slots */
  const int32_t* cmds;         /* the input of copris_rollout_apply: n_slot_cmds x {slot,
                                  trajectory or -1, ctx_len, step}, then n_page_cmds x {slot,
                                  page index, physical page} */
  const int32_t* block_table;  /* [pool][max_pages] the manager's copy of the block table */
} copris_rollout_plan;

int copris_rollout_create(const int32_t* prompt_len, const int32_t* resp_len, int n_inputs,
                          int samples, int pool, int batch_inputs, int page_size, int64_t num_pages,
                          const int32_t* page_order, copris_rollout** out);
void copris_rollout_destroy(copris_rollout* h);
int copris_rollout_max_pages(const copris_rollout* h);       /* block-table row length */
int64_t copris_rollout_free_pages(const copris_rollout* h);  /* pages on the free list now */
int copris_rollout_begin_stage(copris_rollout* h);
int copris_rollout_next_step(copris_rollout* h, copris_rollout_plan* plan);
int copris_rollout_stop(copris_rollout* h, const int32_t* slots, int n);
int copris_rollout_end_stage(copris_rollout* h, copris_stage_stats* stats, int32_t* batch_inputs_out,
                             int32_t* batch_traj_out);

/* ------------------------------------------------------------------------
 * Device side of the rollout loop: the per-slot state of the pool and the buffer of
 * Section 4 ("Buffering of Partial Trajectories") live in device memory, so that a
 * stage runs without a read-back per token.  DEVICE pointers, enqueued on `stream`.
 *
 * Pool state, one entry per slot:  seq_id [pool] int64 (trajectory, -1 = idle; also the
 * Philox stream id of copris_lmhead_logprob), ctx_len [pool] int32 (cached tokens incl.
 * the position being decoded; 0 = idle), step [pool] int32 (index of the token being
 * generated), block_table [pool][max_pages] int32.
 * Buffer, one row per trajectory:  buf_token, buf_tag int32 and buf_logp fp32
 * [n_traj][max_resp]: the sampled token, the stage that generated it and its log-prob
 * under that stage's policy.  By Eq. 6 a trajectory's buffered log-probs are its
 * per-stage pieces concatenated in token order, which is how a row fills up.
 *
 * copris_rollout_apply   applies one plan's commands (copris_rollout_plan.cmds, copied
 *     to the device by the caller): sets seq_id / ctx_len / step of the slots whose
 *     occupant changed and the block-table entries of newly taken pages.  Layout:
 *     n_slot_cmds x {slot, trajectory, ctx_len, step}, then n_page_cmds x {slot, page
 *     index, physical page}.  A command whose slot lies outside [0, pool) (or whose
 *     page index lies outside [0, max_pages)) is skipped, so a caller may pad a
 *     buffer of fixed size with slot -1 and pass fixed counts (a step captured in a
 *     HIP graph).
 * copris_kv_append       k_new, v_new [C, Hkv, D] dtype: the new position's key / value
 *     of every slot goes to token position ctx_len[c] - 1 of its pages
 *     (k_cache[block_table[c][t / P]][kvh][t % P][:]); slots with ctx_len <= 0 are
 *     skipped.  Supported: D % 8 == 0 (bf16) or D % 4 == 0 (fp32).
 * copris_traj_append     after sampling: for every slot with seq_id >= 0 stores
 *     token[c], logprob[c] and `stage` at buf_*[seq_id[c]][step[c]] and advances the
 *     slot (step[c] += 1, ctx_len[c] += 1).  step[c] >= max_resp stores nothing.
 * copris_traj_gather     packs a training batch out of the buffer (Eq. 6): for
 *     trajectory traj[b], tokens j = cu_seqlens[b] + t, t < cu_seqlens[b+1] - cu_seqlens[b]:
 *       tokens_out[j] = buf_token[traj[b]][t]
 *       earlier = buf_tag[traj[b]][t] < stage
 *       logp_buf_out[j]  = earlier ? buf_logp[..][t] : NaN      (the buffered pieces)
 *       logp_roll_out[j] = earlier ? NaN : buf_logp[..][t]      (this stage's piece)
 *       split_out[b] = number of tokens with earlier == true
 *     which are the inputs of copris_lmhead_token_logprob, copris_is_ratio and
 *     copris_grpo_surrogate.
 * All four: COPRIS_EINVAL on null pointers / bad sizes, COPRIS_ELAUNCH on a launch
 * error; n == 0 / C == 0 / B == 0 enqueue nothing.
 * ------------------------------------------------------------------------ */
int copris_rollout_apply(const int32_t* cmds, int n_slot_cmds, int n_page_cmds, int64_t* seq_id,
                         int32_t* ctx_len, int32_t* step, int32_t* block_table, int pool,
                         int max_pages, void* stream);

int copris_kv_append(const void* k_new, const void* v_new, const int32_t* block_table,
                     const int32_t* ctx_len, void* k_cache, void* v_cache, int C, int Hkv, int D,
                     int page_size, int max_pages, int64_t num_pages, int dtype, void* stream);

int copris_traj_append(const int32_t* token, const float* logprob, const int64_t* seq_id,
                       int32_t* step, int32_t* ctx_len, int stage, int32_t* buf_token,
                       float* buf_logp, int32_t* buf_tag, int C, int64_t n_traj, int max_resp,
                       void* stream);

int copris_traj_gather(const int32_t* buf_token, const float* buf_logp, const int32_t* buf_tag,
                       const int32_t* traj, const int32_t* cu_seqlens, int stage,
                       int32_t* tokens_out, float* logp_buf_out, float* logp_roll_out,
                       int32_t* split_out, int B, int64_t n_traj, int max_resp, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* COPRIS_H */
