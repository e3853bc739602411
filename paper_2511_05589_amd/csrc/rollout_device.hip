// Device side of the rollout loop (Section 4): the pool's per-slot state and the buffer of
// partial trajectories stay in device memory between decode steps.
//   rollout_apply_kernel   the manager's per-step commands -> slot state and block table
//   kv_append_kernel       the new position's key / value -> its page
//   traj_append_kernel     sampled token, log-prob, stage tag -> the trajectory's buffer row;
//                          advances the slot
//   traj_gather_kernel     buffer rows -> the packed training batch (Eq. 6: the per-stage
//                          pieces of a trajectory, concatenated in token order)
// All of them move a few bytes per slot or per token: plain copies with bounds checks, no
// tuning beyond coalesced access.
#include "copris.h"
#include "copris_device.h"
#include "copris_internal.h"

namespace copris {

__global__ __launch_bounds__(256) void rollout_apply_kernel(
    const int32_t* __restrict__ cmds, int n_slot, int n_page, int64_t* __restrict__ seq_id,
    int32_t* __restrict__ ctx_len, int32_t* __restrict__ step, int32_t* __restrict__ block_table,
    int pool, int max_pages) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_slot) {
    const int32_t* c = cmds + 4 * i;
    const int slot = c[0];
    if (slot >= 0 && slot < pool) {
      seq_id[slot] = c[1];
      ctx_len[slot] = c[2];
      step[slot] = c[3];
    }
  } else if (i < n_slot + n_page) {
    const int32_t* c = cmds + 4 * n_slot + 3 * (i - n_slot);
    const int slot = c[0], idx = c[1];
    if (slot >= 0 && slot < pool && idx >= 0 && idx < max_pages)
      block_table[static_cast<size_t>(slot) * max_pages + idx] = c[2];
  }
}

// One workgroup per (slot, kv head); threads move 16-byte pieces of the two rows.
__global__ __launch_bounds__(64) void kv_append_kernel(
    const uint4* __restrict__ k_new, const uint4* __restrict__ v_new,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ ctx_len,
    uint4* __restrict__ k_cache, uint4* __restrict__ v_cache, int Hkv, int row_vec, int page_size,
    int max_pages, int64_t num_pages) {
  const int c = blockIdx.x, kvh = blockIdx.y;
  const int n = ctx_len[c];
  if (n <= 0 || n > max_pages * page_size) return;
  const int t = n - 1;
  const int64_t page = block_table[static_cast<size_t>(c) * max_pages + t / page_size];
  if (page < 0 || page >= num_pages) return;
  const size_t src = (static_cast<size_t>(c) * Hkv + kvh) * row_vec;
  const size_t dst = ((static_cast<size_t>(page) * Hkv + kvh) * page_size + t % page_size) * row_vec;
  for (int e = threadIdx.x; e < row_vec; e += 64) {
    k_cache[dst + e] = k_new[src + e];
    v_cache[dst + e] = v_new[src + e];
  }
}

__global__ __launch_bounds__(256) void traj_append_kernel(
    const int32_t* __restrict__ token, const float* __restrict__ logprob,
    const int64_t* __restrict__ seq_id, int32_t* __restrict__ step, int32_t* __restrict__ ctx_len,
    int stage, int32_t* __restrict__ buf_token, float* __restrict__ buf_logp,
    int32_t* __restrict__ buf_tag, int C, int64_t n_traj, int max_resp) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= C) return;
  const int64_t tr = seq_id[c];
  if (tr < 0 || tr >= n_traj) return;
  const int g = step[c];
  if (g >= 0 && g < max_resp) {
    const size_t at = static_cast<size_t>(tr) * max_resp + g;
    buf_token[at] = token[c];
    buf_logp[at] = logprob[c];
    buf_tag[at] = stage;
  }
  step[c] = g + 1;
  ctx_len[c] += 1;
}

// One workgroup per trajectory of the batch.
__global__ __launch_bounds__(256) void traj_gather_kernel(
    const int32_t* __restrict__ buf_token, const float* __restrict__ buf_logp,
    const int32_t* __restrict__ buf_tag, const int32_t* __restrict__ traj,
    const int32_t* __restrict__ cu_seqlens, int stage, int32_t* __restrict__ tokens_out,
    float* __restrict__ logp_buf_out, float* __restrict__ logp_roll_out,
    int32_t* __restrict__ split_out, int64_t n_traj, int max_resp) {
  __shared__ int s_cnt[256 / kWave];
  const int b = blockIdx.x;
  const int64_t tr = traj[b];
  const int64_t j0 = cu_seqlens[b];
  int64_t len = static_cast<int64_t>(cu_seqlens[b + 1]) - j0;
  len = len < 0 ? 0 : (len > max_resp ? max_resp : len);
  const bool ok = tr >= 0 && tr < n_traj;
  const float nan = __int_as_float(0x7fc00000);
  int earlier_cnt = 0;
  for (int64_t t = threadIdx.x; t < len; t += 256) {
    const size_t at = static_cast<size_t>(ok ? tr : 0) * max_resp + t;
    const bool earlier = ok && buf_tag[at] < stage;
    const float lp = ok ? buf_logp[at] : nan;
    tokens_out[j0 + t] = ok ? buf_token[at] : -1;
    logp_buf_out[j0 + t] = earlier ? lp : nan;
    logp_roll_out[j0 + t] = earlier ? nan : lp;
    earlier_cnt += earlier ? 1 : 0;
  }
  const int w = wave_sum_i(earlier_cnt);
  if ((threadIdx.x & (kWave - 1)) == 0) s_cnt[threadIdx.x / kWave] = w;
  __syncthreads();
  if (threadIdx.x == 0) {
    int tot = 0;
#pragma unroll
    for (int i = 0; i < 256 / kWave; ++i) tot += s_cnt[i];
    split_out[b] = tot;
  }
}

}  // namespace copris

namespace {
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
}

extern "C" {

int copris_rollout_apply(const int32_t* cmds, int n_slot_cmds, int n_page_cmds, int64_t* seq_id,
                         int32_t* ctx_len, int32_t* step, int32_t* block_table, int pool,
                         int max_pages, void* stream_) {
  if (n_slot_cmds < 0 || n_page_cmds < 0 || pool <= 0 || max_pages <= 0) return COPRIS_EINVAL;
  const int64_t n = static_cast<int64_t>(n_slot_cmds) + n_page_cmds;
  if (n == 0) return COPRIS_OK;
  if (n >= (1ll << 30) || !cmds || !seq_id || !ctx_len || !step || !block_table) return COPRIS_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  (void)hipGetLastError();
  COPRIS_PRE("rollout_apply_kernel");
  hipLaunchKernelGGL(copris::rollout_apply_kernel, dim3(static_cast<unsigned>((n + 255) / 256)),
                     dim3(256), 0, stream, cmds, n_slot_cmds, n_page_cmds, seq_id, ctx_len, step,
                     block_table, pool, max_pages);
  COPRIS_POST("rollout_apply_kernel");
  return COPRIS_OK;
}

int copris_kv_append(const void* k_new, const void* v_new, const int32_t* block_table,
                     const int32_t* ctx_len, void* k_cache, void* v_cache, int C, int Hkv, int D,
                     int page_size, int max_pages, int64_t num_pages, int dtype, void* stream_) {
  if (C < 0 || Hkv <= 0 || Hkv > 65535 || D <= 0 || page_size <= 0 || max_pages <= 0 || num_pages <= 0)
    return COPRIS_EINVAL;
  if (static_cast<int64_t>(max_pages) * page_size > (1ll << 30)) return COPRIS_EINVAL;
  if (dtype != COPRIS_F32 && dtype != COPRIS_BF16) return COPRIS_EUNSUPPORTED;
  const int row_bytes = D * (dtype == COPRIS_BF16 ? 2 : 4);
  if (row_bytes % 16 != 0) return COPRIS_EUNSUPPORTED;
  if (C == 0) return COPRIS_OK;
  if (!k_new || !v_new || !block_table || !ctx_len || !k_cache || !v_cache) return COPRIS_EINVAL;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache))
    return COPRIS_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  (void)hipGetLastError();
  COPRIS_PRE("kv_append_kernel");
  hipLaunchKernelGGL(copris::kv_append_kernel, dim3(C, Hkv), dim3(64), 0, stream,
                     static_cast<const uint4*>(k_new), static_cast<const uint4*>(v_new), block_table,
                     ctx_len, static_cast<uint4*>(k_cache), static_cast<uint4*>(v_cache), Hkv,
                     row_bytes / 16, page_size, max_pages, num_pages);
  COPRIS_POST("kv_append_kernel");
  return COPRIS_OK;
}

int copris_traj_append(const int32_t* token, const float* logprob, const int64_t* seq_id,
                       int32_t* step, int32_t* ctx_len, int stage, int32_t* buf_token,
                       float* buf_logp, int32_t* buf_tag, int C, int64_t n_traj, int max_resp,
                       void* stream_) {
  if (C < 0 || n_traj <= 0 || max_resp <= 0) return COPRIS_EINVAL;
  if (C == 0) return COPRIS_OK;
  if (!token || !logprob || !seq_id || !step || !ctx_len || !buf_token || !buf_logp || !buf_tag)
    return COPRIS_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  (void)hipGetLastError();
  COPRIS_PRE("traj_append_kernel");
  hipLaunchKernelGGL(copris::traj_append_kernel, dim3((C + 255) / 256), dim3(256), 0, stream, token,
                     logprob, seq_id, step, ctx_len, stage, buf_token, buf_logp, buf_tag, C, n_traj,
                     max_resp);
  COPRIS_POST("traj_append_kernel");
  return COPRIS_OK;
}

int copris_traj_gather(const int32_t* buf_token, const float* buf_logp, const int32_t* buf_tag,
                       const int32_t* traj, const int32_t* cu_seqlens, int stage,
                       int32_t* tokens_out, float* logp_buf_out, float* logp_roll_out,
                       int32_t* split_out, int B, int64_t n_traj, int max_resp, void* stream_) {
  if (B < 0 || n_traj <= 0 || max_resp <= 0) return COPRIS_EINVAL;
  if (B == 0) return COPRIS_OK;
  if (!buf_token || !buf_logp || !buf_tag || !traj || !cu_seqlens || !tokens_out || !logp_buf_out ||
      !logp_roll_out || !split_out)
    return COPRIS_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  (void)hipGetLastError();
  COPRIS_PRE("traj_gather_kernel");
  hipLaunchKernelGGL(copris::traj_gather_kernel, dim3(B), dim3(256), 0, stream, buf_token, buf_logp,
                     buf_tag, traj, cu_seqlens, stage, tokens_out, logp_buf_out, logp_roll_out,
                     split_out, n_traj, max_resp);
  COPRIS_POST("traj_gather_kernel");
  return COPRIS_OK;
}

}  // extern "C"
