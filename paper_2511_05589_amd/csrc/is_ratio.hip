// Token-level cross-stage importance ratio (Section 4, Eq. 8) with the clip of
// Eq. 3, a token mask and per-sequence sums, over a packed batch.
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

struct IsAcc {
  float sum;
  int cnt;
  int nclip;
};

__device__ __forceinline__ void is_token(float cur, float old, bool counted, float lo, float hi,
                                         float& r_out, float& rc_out, IsAcc& acc) {
  const float r = expf(cur - old);
  // comparisons are false for NaN, so a NaN ratio stays NaN after the clip
  const float rc = r < lo ? lo : (r > hi ? hi : r);
  r_out = counted ? r : 0.0f;          // select, never multiply: masked NaNs do not leak
  rc_out = counted ? rc : 0.0f;
  acc.sum += counted ? rc : 0.0f;
  acc.cnt += counted ? 1 : 0;
  acc.nclip += (counted && !(rc == r)) ? 1 : 0;
}

template <bool HAS_MASK>
__global__ __launch_bounds__(kIsThreads) void is_ratio_kernel(
    const float* __restrict__ logp_cur, const float* __restrict__ logp_buf,
    const float* __restrict__ logp_roll, const int32_t* __restrict__ cu_seqlens,
    const int32_t* __restrict__ split, const uint8_t* __restrict__ mask, float lo, float hi,
    float* __restrict__ ratio, float* __restrict__ ratio_clipped, float* __restrict__ seq_sum,
    int32_t* __restrict__ seq_cnt, int32_t* __restrict__ seq_nclip) {
  const int b = blockIdx.x;
  const int64_t j0 = cu_seqlens[b];
  const int64_t j1 = cu_seqlens[b + 1];
  const int64_t len = j1 > j0 ? j1 - j0 : 0;
  int64_t sp = split[b];
  sp = sp < 0 ? 0 : (sp > len ? len : sp);
  const int64_t jsplit = j0 + sp;   // tokens j < jsplit are buffered (earlier stages)

  IsAcc acc{0.0f, 0, 0};
  // groups of four tokens, aligned on the global index so that vector accesses
  // are 16-byte aligned whatever cu_seqlens[b] is
  const int64_t gbase = j0 & ~static_cast<int64_t>(3);
  for (int64_t gj = gbase + 4 * static_cast<int64_t>(threadIdx.x); gj < j1;
       gj += 4 * static_cast<int64_t>(kIsThreads)) {
    if (gj >= j0 && gj + 4 <= j1) {
      const float4 c = *reinterpret_cast<const float4*>(logp_cur + gj);
      float4 o;
      if (gj + 4 <= jsplit) {
        o = *reinterpret_cast<const float4*>(logp_buf + gj);
      } else if (gj >= jsplit) {
        o = *reinterpret_cast<const float4*>(logp_roll + gj);
      } else {  // the one group that straddles the stage boundary
        o.x = gj + 0 < jsplit ? logp_buf[gj + 0] : logp_roll[gj + 0];
        o.y = gj + 1 < jsplit ? logp_buf[gj + 1] : logp_roll[gj + 1];
        o.z = gj + 2 < jsplit ? logp_buf[gj + 2] : logp_roll[gj + 2];
        o.w = gj + 3 < jsplit ? logp_buf[gj + 3] : logp_roll[gj + 3];
      }
      uint32_t m4 = 0x01010101u;
      if (HAS_MASK) m4 = *reinterpret_cast<const uint32_t*>(mask + gj);
      float4 r, rc;
      is_token(c.x, o.x, (m4 & 0x000000ffu) != 0, lo, hi, r.x, rc.x, acc);
      is_token(c.y, o.y, (m4 & 0x0000ff00u) != 0, lo, hi, r.y, rc.y, acc);
      is_token(c.z, o.z, (m4 & 0x00ff0000u) != 0, lo, hi, r.z, rc.z, acc);
      is_token(c.w, o.w, (m4 & 0xff000000u) != 0, lo, hi, r.w, rc.w, acc);
      *reinterpret_cast<float4*>(ratio + gj) = r;
      *reinterpret_cast<float4*>(ratio_clipped + gj) = rc;
    } else {  // ragged head or tail of the sequence
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int64_t j = gj + e;
        if (j >= j0 && j < j1) {
          const float old = j < jsplit ? logp_buf[j] : logp_roll[j];
          const bool counted = HAS_MASK ? (mask[j] != 0) : true;
          float r, rc;
          is_token(logp_cur[j], old, counted, lo, hi, r, rc, acc);
          ratio[j] = r;
          ratio_clipped[j] = rc;
        }
      }
    }
  }

  // lane -> wave -> workgroup, fixed order
  __shared__ float s_sum[kIsThreads / kWave];
  __shared__ int s_cnt[kIsThreads / kWave];
  __shared__ int s_ncl[kIsThreads / kWave];
  const float wsum = wave_sum(acc.sum);
  const int wcnt = wave_sum_i(acc.cnt);
  const int wncl = wave_sum_i(acc.nclip);
  const int wave = threadIdx.x / kWave;
  if ((threadIdx.x & (kWave - 1)) == 0) {
    s_sum[wave] = wsum;
    s_cnt[wave] = wcnt;
    s_ncl[wave] = wncl;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float ts = 0.0f;
    int tc = 0, tn = 0;
#pragma unroll
    for (int w = 0; w < kIsThreads / kWave; ++w) {
      ts += s_sum[w];
      tc += s_cnt[w];
      tn += s_ncl[w];
    }
    seq_sum[b] = ts;
    seq_cnt[b] = tc;
    seq_nclip[b] = tn;
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

}  // namespace copris
