// LM-head projection fused with log-softmax, Gumbel-max sampling and the chosen
// token's log-probability (the per-token log-prob under the generating policy that
// the buffer keeps: Section 4, Eq. 6; sampler settings: Table 4).
//
// The V logits of a row are never written out.  Every (row, vocabulary tile) pair
// produces one small partial
//     m    = max_v z_v                s = sum_v exp(z_v - m)
//     best = max_v (z_v + G_v)        idx, z = its vocabulary index and raw logit
// and a merge kernel combines the partials of a row: lse = m + ln s,
// logprob = z_best - lse.  Ties on the perturbed score go to the lowest index, in
// the tiles and in the merge, so the result does not depend on the tiling.
#include "copris_device.h"
#include "copris_internal.h"

namespace copris {

struct LmPartial {
  float m, s, best, z;
  int32_t idx;
};

constexpr int kLmTileV = 64;      // vocabulary rows per tile (generic kernel)
constexpr int kLmTileC = 16;      // batch rows per workgroup (generic kernel)
constexpr int kLmBK = 256;        // hidden-dim slab staged in LDS

static inline size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

LmWorkspace lm_workspace_layout(int C, int H, int V) {
  (void)H;
  LmWorkspace w{};
  w.n_tiles = (V + kLmTileV - 1) / kLmTileV;
  w.part = 0;
  w.total = align256(static_cast<size_t>(C) * w.n_tiles * sizeof(LmPartial));
  return w;
}

// (score, idx) ordering: larger score first, then lower index.
__device__ __forceinline__ bool better(float sa, int ia, float sb, int ib) {
  return sa > sb || (sa == sb && ia < ib);
}

__device__ __forceinline__ void combine(LmPartial& a, const LmPartial& o) {
  const float m = fmaxf(a.m, o.m);
  // exp(-inf - m) = 0 handles empty partials (m = -inf, s = 0) as long as m is finite
  const float sa = a.m == -INFINITY ? 0.0f : a.s * __expf(a.m - m);
  const float sb = o.m == -INFINITY ? 0.0f : o.s * __expf(o.m - m);
  a.m = m;
  a.s = sa + sb;
  if (better(o.best, o.idx, a.best, a.idx)) {
    a.best = o.best;
    a.idx = o.idx;
    a.z = o.z;
  }
}

__device__ __forceinline__ LmPartial wave_combine(LmPartial p) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    LmPartial q;
    q.m = __shfl_xor(p.m, o, kWave);
    q.s = __shfl_xor(p.s, o, kWave);
    q.best = __shfl_xor(p.best, o, kWave);
    q.z = __shfl_xor(p.z, o, kWave);
    q.idx = __shfl_xor(p.idx, o, kWave);
    combine(p, q);
  }
  return p;
}

// One logit -> a single-element partial.
__device__ __forceinline__ LmPartial logit_partial(float z, int v, uint32_t word) {
  LmPartial p;
  p.m = z;
  p.s = 1.0f;
  p.best = z + gumbel_from_uniform(word_to_uniform(word));
  p.z = z;
  p.idx = v;
  return p;
}

__device__ __forceinline__ LmPartial empty_partial() {
  LmPartial p;
  p.m = -INFINITY;
  p.s = 0.0f;
  p.best = -INFINITY;
  p.z = 0.0f;
  p.idx = 0x7fffffff;
  return p;
}

// --------------------------------------------------------------------------
// generic kernel (fp32 or bf16, vector ALU): wave w of a workgroup owns batch rows
// 4w..4w+3 of the 16-row block, lane l owns vocabulary row tile*64 + l.
// --------------------------------------------------------------------------
template <typename T> struct WVec;
template <> struct WVec<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void load(const float* p, float (&x)[8]) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
  }
  static __device__ __forceinline__ float one(const float* p) { return *p; }
};
template <> struct WVec<uint16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void load(const uint16_t* p, float (&x)[8]) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    x[0] = bf16lo_to_f32(v.x); x[1] = bf16hi_to_f32(v.x);
    x[2] = bf16lo_to_f32(v.y); x[3] = bf16hi_to_f32(v.y);
    x[4] = bf16lo_to_f32(v.z); x[5] = bf16hi_to_f32(v.z);
    x[6] = bf16lo_to_f32(v.w); x[7] = bf16hi_to_f32(v.w);
  }
  static __device__ __forceinline__ float one(const uint16_t* p) { return bf16_to_f32(*p); }
};

template <typename T>
__global__ __launch_bounds__(256) void lmhead_generic_kernel(
    const T* __restrict__ hidden, const T* __restrict__ weight, const int64_t* __restrict__ seq_id,
    const int32_t* __restrict__ step, uint32_t key0, uint32_t key1, float inv_temperature,
    LmPartial* __restrict__ part, int C, int H, int V, int n_tiles) {
  constexpr int NV = WVec<T>::N;
  __shared__ float s_h[kLmTileC][kLmBK];
  const int tile = blockIdx.x, cb = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int v = tile * kLmTileV + lane;
  const bool v_ok = v < V;
  const T* wrow = weight + static_cast<size_t>(v_ok ? v : 0) * H;
  float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};

  for (int k0 = 0; k0 < H; k0 += kLmBK) {
    const int kn = min(kLmBK, H - k0);
    __syncthreads();
    for (int e = tid; e < kLmTileC * kn; e += 256) {
      const int r = e / kn, k = e - r * kn;
      const int c = cb * kLmTileC + r;
      s_h[r][k] = c < C ? WVec<T>::one(hidden + static_cast<size_t>(c) * H + k0 + k) : 0.0f;
    }
    __syncthreads();
    if (v_ok) {
      for (int k = 0; k < kn; k += NV) {
        float x[8];
        WVec<T>::load(wrow + k0 + k, x);
#pragma unroll
        for (int j = 0; j < NV; ++j) {
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[r] = fmaf(s_h[4 * wave + r][k + j], x[j], acc[r]);
        }
      }
    }
  }

#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int c = cb * kLmTileC + 4 * wave + r;
    if (c >= C) continue;   // uniform across the wave
    LmPartial p = empty_partial();
    if (v_ok) {
      const uint64_t sid = static_cast<uint64_t>(seq_id[c]);
      const Philox4 x = philox4x32_10(static_cast<uint32_t>(v) >> 2, static_cast<uint32_t>(step[c]),
                                      static_cast<uint32_t>(sid), static_cast<uint32_t>(sid >> 32),
                                      key0, key1);
      const int sel = v & 3;
      const uint32_t word = sel == 0 ? x.x : (sel == 1 ? x.y : (sel == 2 ? x.z : x.w));
      p = logit_partial(acc[r] * inv_temperature, v, word);
    }
    p = wave_combine(p);
    if (lane == 0) part[static_cast<size_t>(c) * n_tiles + tile] = p;
  }
}

// --------------------------------------------------------------------------
// merge: one workgroup per batch row over its n_tiles partials.
// --------------------------------------------------------------------------
__global__ __launch_bounds__(256) void lmhead_merge_kernel(const LmPartial* __restrict__ part,
                                                           int n_tiles, int32_t* __restrict__ token,
                                                           float* __restrict__ logprob,
                                                           float* __restrict__ lse) {
  __shared__ LmPartial s_part[256 / kWave];
  const int c = blockIdx.x, tid = threadIdx.x;
  LmPartial p = empty_partial();
  for (int t = tid; t < n_tiles; t += 256) combine(p, part[static_cast<size_t>(c) * n_tiles + t]);
  p = wave_combine(p);
  if ((tid & (kWave - 1)) == 0) s_part[tid / kWave] = p;
  __syncthreads();
  if (tid == 0) {
    LmPartial a = s_part[0];
#pragma unroll
    for (int w = 1; w < 256 / kWave; ++w) combine(a, s_part[w]);
    const float l = a.m + logf(a.s);
    token[c] = a.idx;
    logprob[c] = a.z - l;
    if (lse != nullptr) lse[c] = l;
  }
}

int launch_lmhead_logprob(const void* hidden, const void* weight, const int64_t* seq_id,
                          const int32_t* step, uint64_t seed, float temperature, int32_t* token,
                          float* logprob, float* lse, void* workspace, int C, int H, int V,
                          int dtype, hipStream_t stream) {
  const LmWorkspace w = lm_workspace_layout(C, H, V);
  LmPartial* part = reinterpret_cast<LmPartial*>(static_cast<char*>(workspace) + w.part);
  const uint32_t key0 = static_cast<uint32_t>(seed), key1 = static_cast<uint32_t>(seed >> 32);
  const float inv_t = 1.0f / temperature;
  const dim3 grid(w.n_tiles, (C + kLmTileC - 1) / kLmTileC);
  if (dtype == 0) {
    hipLaunchKernelGGL(lmhead_generic_kernel<float>, grid, dim3(256), 0, stream,
                       static_cast<const float*>(hidden), static_cast<const float*>(weight),
                       seq_id, step, key0, key1, inv_t, part, C, H, V, w.n_tiles);
  } else {
    hipLaunchKernelGGL(lmhead_generic_kernel<uint16_t>, grid, dim3(256), 0, stream,
                       static_cast<const uint16_t*>(hidden), static_cast<const uint16_t*>(weight),
                       seq_id, step, key0, key1, inv_t, part, C, H, V, w.n_tiles);
  }
  COPRIS_CHECK_LAUNCH("lmhead_generic_kernel");
  hipLaunchKernelGGL(lmhead_merge_kernel, dim3(C), dim3(256), 0, stream, part, w.n_tiles, token,
                     logprob, lse);
  COPRIS_CHECK_LAUNCH("lmhead_merge_kernel");
  return 0;
}

}  // namespace copris
