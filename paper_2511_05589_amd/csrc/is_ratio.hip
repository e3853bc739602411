// Token-level cross-stage importance ratio (Section 4, Eq. 8) with the clip of
// Eq. 3, a token mask and per-sequence sums, over a packed batch; and the GRPO
// clipped surrogate (Eq. 2-4) on the same ratio.
//
// A plain bandwidth kernel: one workgroup streams one sequence in 16-byte
// vectors.  Only the old-policy array that `split` selects is fetched for a
// group of four tokens (17 algorithmic bytes per token: 4 cur + 4 old + 1 mask
// in, 8 out).  Per-sequence sums are reduced lane -> wave -> workgroup in a
// fixed order, so results are bitwise reproducible.
#include "copris_device.h"
#include "copris_internal.h"

namespace copris {

constexpr int kIsThreads = 1024;

// Every byte of the batch is touched once: non-temporal loads and stores keep the streams out
// of the L2.  (The builtins take native vector types.)
typedef float is_f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream4(const float* p) {
  const is_f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const is_f32x4*>(p));
  return make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void store_stream4(float* p, const float4& x) {
  const is_f32x4 v = {x.x, x.y, x.z, x.w};
  __builtin_nontemporal_store(v, reinterpret_cast<is_f32x4*>(p));
}

// Per-token operations.  Both produce two fp32 outputs per token and a per-sequence
// accumulator; a token that is not counted writes 0 to both (select, never multiply, so
// that NaNs at masked positions do not leak).

// Eq. 8 and the clip of Eq. 3: out0 = r, out1 = clip(r); sums clip(r), counts clipped tokens.
struct RatioOp {
  float lo, hi;
  struct Acc {
    float sum;
    int cnt;
    int aux;
  };
  __device__ __forceinline__ void token(float cur, float old, bool counted, float& out0,
                                        float& out1, Acc& acc) const {
    const float r = expf(cur - old);
    // comparisons are false for NaN, so a NaN ratio stays NaN after the clip
    const float rc = r < lo ? lo : (r > hi ? hi : r);
    out0 = counted ? r : 0.0f;
    out1 = counted ? rc : 0.0f;
    acc.sum += counted ? rc : 0.0f;
    acc.cnt += counted ? 1 : 0;
    acc.aux += (counted && !(rc == r)) ? 1 : 0;
  }
};

// Eq. 3 with the advantage of Eq. 4: out0 = min(r A, clip(r) A), out1 = its derivative
// with respect to the current log-prob (r A where the unclipped term is the smaller one
// or ties, else 0); sums out0.
struct GrpoOp {
  float lo, hi, adv;
  struct Acc {
    float sum;
    int cnt;
    int aux;
  };
  __device__ __forceinline__ void token(float cur, float old, bool counted, float& out0,
                                        float& out1, Acc& acc) const {
    const float r = expf(cur - old);
    const float rc = r < lo ? lo : (r > hi ? hi : r);
    const float t1 = r * adv, t2 = rc * adv;
    const bool unclipped = t1 <= t2;
    const float s = unclipped ? t1 : t2;
    out0 = counted ? s : 0.0f;
    out1 = (counted && unclipped) ? t1 : 0.0f;
    acc.sum += counted ? s : 0.0f;
    acc.cnt += counted ? 1 : 0;
  }
};

// One workgroup streams sequence b.  Tokens are taken in groups of four aligned on the
// global index, so that vector accesses are 16-byte aligned whatever cu_seqlens[b] is.
template <bool HAS_MASK, typename Op>
__device__ __forceinline__ typename Op::Acc stream_sequence(
    const Op& op, const float* __restrict__ logp_cur, const float* __restrict__ logp_buf,
    const float* __restrict__ logp_roll, const uint8_t* __restrict__ mask, int64_t j0, int64_t j1,
    int64_t jsplit, float* __restrict__ out0, float* __restrict__ out1) {
  typename Op::Acc acc{0.0f, 0, 0};
  const int64_t gbase = j0 & ~static_cast<int64_t>(3);
  for (int64_t gj = gbase + 4 * static_cast<int64_t>(threadIdx.x); gj < j1;
       gj += 4 * static_cast<int64_t>(kIsThreads)) {
    if (gj >= j0 && gj + 4 <= j1) {
      const float4 c = load_stream4(logp_cur + gj);
      float4 o;
      if (gj + 4 <= jsplit) {
        o = load_stream4(logp_buf + gj);
      } else if (gj >= jsplit) {
        o = load_stream4(logp_roll + gj);
      } else {  // the one group that straddles the stage boundary
        o.x = gj + 0 < jsplit ? logp_buf[gj + 0] : logp_roll[gj + 0];
        o.y = gj + 1 < jsplit ? logp_buf[gj + 1] : logp_roll[gj + 1];
        o.z = gj + 2 < jsplit ? logp_buf[gj + 2] : logp_roll[gj + 2];
        o.w = gj + 3 < jsplit ? logp_buf[gj + 3] : logp_roll[gj + 3];
      }
      uint32_t m4 = 0x01010101u;
      if (HAS_MASK) m4 = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(mask + gj));
      float4 r, rc;
      op.token(c.x, o.x, (m4 & 0x000000ffu) != 0, r.x, rc.x, acc);
      op.token(c.y, o.y, (m4 & 0x0000ff00u) != 0, r.y, rc.y, acc);
      op.token(c.z, o.z, (m4 & 0x00ff0000u) != 0, r.z, rc.z, acc);
      op.token(c.w, o.w, (m4 & 0xff000000u) != 0, r.w, rc.w, acc);
      store_stream4(out0 + gj, r);
      store_stream4(out1 + gj, rc);
    } else {  // ragged head or tail of the sequence
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int64_t j = gj + e;
        if (j >= j0 && j < j1) {
          const float old = j < jsplit ? logp_buf[j] : logp_roll[j];
          const bool counted = HAS_MASK ? (mask[j] != 0) : true;
          float r, rc;
          op.token(logp_cur[j], old, counted, r, rc, acc);
          out0[j] = r;
          out1[j] = rc;
        }
      }
    }
  }

  // lane -> wave -> workgroup, fixed order; thread 0 returns the totals
  __shared__ float s_sum[kIsThreads / kWave];
  __shared__ int s_cnt[kIsThreads / kWave];
  __shared__ int s_aux[kIsThreads / kWave];
  const float wsum = wave_sum(acc.sum);
  const int wcnt = wave_sum_i(acc.cnt);
  const int waux = wave_sum_i(acc.aux);
  const int wave = threadIdx.x / kWave;
  if ((threadIdx.x & (kWave - 1)) == 0) {
    s_sum[wave] = wsum;
    s_cnt[wave] = wcnt;
    s_aux[wave] = waux;
  }
  __syncthreads();
  typename Op::Acc tot{0.0f, 0, 0};
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 0; w < kIsThreads / kWave; ++w) {
      tot.sum += s_sum[w];
      tot.cnt += s_cnt[w];
      tot.aux += s_aux[w];
    }
  }
  return tot;
}

__device__ __forceinline__ void sequence_bounds(const int32_t* cu_seqlens, const int32_t* split, int b,
                                                int64_t& j0, int64_t& j1, int64_t& jsplit) {
  j0 = cu_seqlens[b];
  j1 = cu_seqlens[b + 1];
  const int64_t len = j1 > j0 ? j1 - j0 : 0;
  int64_t sp = split[b];
  sp = sp < 0 ? 0 : (sp > len ? len : sp);
  jsplit = j0 + sp;   // tokens j < jsplit are buffered (earlier stages)
}

template <bool HAS_MASK>
__global__ __launch_bounds__(kIsThreads) void is_ratio_kernel(
    const float* __restrict__ logp_cur, const float* __restrict__ logp_buf,
    const float* __restrict__ logp_roll, const int32_t* __restrict__ cu_seqlens,
    const int32_t* __restrict__ split, const uint8_t* __restrict__ mask, float lo, float hi,
    float* __restrict__ ratio, float* __restrict__ ratio_clipped, float* __restrict__ seq_sum,
    int32_t* __restrict__ seq_cnt, int32_t* __restrict__ seq_nclip) {
  const int b = blockIdx.x;
  int64_t j0, j1, jsplit;
  sequence_bounds(cu_seqlens, split, b, j0, j1, jsplit);
  const RatioOp op{lo, hi};
  const RatioOp::Acc tot = stream_sequence<HAS_MASK>(op, logp_cur, logp_buf, logp_roll, mask, j0, j1,
                                                     jsplit, ratio, ratio_clipped);
  if (threadIdx.x == 0) {
    seq_sum[b] = tot.sum;
    seq_cnt[b] = tot.cnt;
    seq_nclip[b] = tot.aux;
  }
}

template <bool HAS_MASK>
__global__ __launch_bounds__(kIsThreads) void grpo_surrogate_kernel(
    const float* __restrict__ logp_cur, const float* __restrict__ logp_buf,
    const float* __restrict__ logp_roll, const int32_t* __restrict__ cu_seqlens,
    const int32_t* __restrict__ split, const uint8_t* __restrict__ mask,
    const float* __restrict__ adv, float lo, float hi, float* __restrict__ surr,
    float* __restrict__ grad, float* __restrict__ seq_surr, int32_t* __restrict__ seq_cnt) {
  const int b = blockIdx.x;
  int64_t j0, j1, jsplit;
  sequence_bounds(cu_seqlens, split, b, j0, j1, jsplit);
  const GrpoOp op{lo, hi, adv[b]};
  const GrpoOp::Acc tot = stream_sequence<HAS_MASK>(op, logp_cur, logp_buf, logp_roll, mask, j0, j1,
                                                    jsplit, surr, grad);
  if (threadIdx.x == 0) {
    seq_surr[b] = tot.sum;
    seq_cnt[b] = tot.cnt;
  }
}

// objective[0] = token mean (Table 4), objective[1] = mean of the sequence means (Eq. 2).
// One workgroup; thread t takes sequences t, t+256, ... and the 256 partial sums are added
// in index order, in fp64: the result does not depend on anything but the inputs.
__global__ __launch_bounds__(256) void grpo_objective_kernel(const float* __restrict__ seq_surr,
                                                             const int32_t* __restrict__ seq_cnt,
                                                             int B, float* __restrict__ objective) {
  __shared__ double s_tot[256];
  __shared__ double s_mean[256];
  __shared__ long long s_cnt[256];
  double tot = 0.0, mean = 0.0;
  long long cnt = 0;
  for (int b = threadIdx.x; b < B; b += 256) {
    const int c = seq_cnt[b];
    const double s = static_cast<double>(seq_surr[b]);
    if (c > 0) {
      tot += s;
      mean += s / static_cast<double>(c);
      cnt += c;
    }
  }
  s_tot[threadIdx.x] = tot;
  s_mean[threadIdx.x] = mean;
  s_cnt[threadIdx.x] = cnt;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0, m = 0.0;
    long long c = 0;
    for (int i = 0; i < 256; ++i) {
      t += s_tot[i];
      m += s_mean[i];
      c += s_cnt[i];
    }
    objective[0] = c > 0 ? static_cast<float>(t / static_cast<double>(c)) : 0.0f;
    objective[1] = B > 0 ? static_cast<float>(m / static_cast<double>(B)) : 0.0f;
  }
}

int launch_is_ratio(const float* logp_cur, const float* logp_buf, const float* logp_roll,
                    const int32_t* cu_seqlens, const int32_t* split, const uint8_t* mask,
                    float eps_low, float eps_high, float* ratio, float* ratio_clipped,
                    float* seq_sum, int32_t* seq_cnt, int32_t* seq_nclip, int B,
                    hipStream_t stream) {
  if (B == 0) return 0;
  const float lo = 1.0f - eps_low, hi = 1.0f + eps_high;
  COPRIS_PRE("is_ratio_kernel");
  if (mask != nullptr) {
    hipLaunchKernelGGL(is_ratio_kernel<true>, dim3(B), dim3(kIsThreads), 0, stream, logp_cur,
                       logp_buf, logp_roll, cu_seqlens, split, mask, lo, hi, ratio, ratio_clipped,
                       seq_sum, seq_cnt, seq_nclip);
  } else {
    hipLaunchKernelGGL(is_ratio_kernel<false>, dim3(B), dim3(kIsThreads), 0, stream, logp_cur,
                       logp_buf, logp_roll, cu_seqlens, split, mask, lo, hi, ratio, ratio_clipped,
                       seq_sum, seq_cnt, seq_nclip);
  }
  COPRIS_POST("is_ratio_kernel");
  return 0;
}

int launch_grpo_surrogate(const float* logp_cur, const float* logp_buf, const float* logp_roll,
                          const int32_t* cu_seqlens, const int32_t* split, const uint8_t* mask,
                          const float* adv, float eps_low, float eps_high, float* surr, float* grad,
                          float* seq_surr, int32_t* seq_cnt, float* objective, int B,
                          hipStream_t stream) {
  const float lo = 1.0f - eps_low, hi = 1.0f + eps_high;
  if (B > 0) {
    COPRIS_PRE("grpo_surrogate_kernel");
    if (mask != nullptr) {
      hipLaunchKernelGGL(grpo_surrogate_kernel<true>, dim3(B), dim3(kIsThreads), 0, stream, logp_cur,
                         logp_buf, logp_roll, cu_seqlens, split, mask, adv, lo, hi, surr, grad,
                         seq_surr, seq_cnt);
    } else {
      hipLaunchKernelGGL(grpo_surrogate_kernel<false>, dim3(B), dim3(kIsThreads), 0, stream, logp_cur,
                         logp_buf, logp_roll, cu_seqlens, split, mask, adv, lo, hi, surr, grad,
                         seq_surr, seq_cnt);
    }
    COPRIS_POST("grpo_surrogate_kernel");
  }
  COPRIS_PRE("grpo_objective_kernel");
  hipLaunchKernelGGL(grpo_objective_kernel, dim3(1), dim3(256), 0, stream, seq_surr, seq_cnt, B,
                     objective);
  COPRIS_POST("grpo_objective_kernel");
  return 0;
}

}  // namespace copris
