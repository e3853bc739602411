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
#include <type_traits>

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
// matrix-core kernel (bf16, H % 32 == 0).
//
// Z^T[v][c] = W[v][:] . hidden[c][:] with the VOCABULARY as the M side of
// mfma_f32_32x32x16_bf16 and the batch as the N side: a lane's 16 accumulators of a
// 32x32 block are then 4 runs of 4 consecutive vocabulary entries of ONE batch row,
// i.e. exactly one Philox block (4 words) per run, and the row's running
// log-sum-exp / arg-max state lives in that lane.
//
// A workgroup (4 waves, 2x2) owns a 128 (vocab) x 256 (batch) tile and walks the
// hidden dimension in slabs of 32: coalesced 16-byte loads, one slab ahead, into
// registers, parked in double-buffered LDS with an XOR swizzle, read back as MFMA
// operands.  Workgroups are persistent over vocabulary tiles and keep their
// per-row state across tiles, so W is streamed from HBM exactly once and only
// gridDim.x partials per row reach the merge.
//
// Sampling without a second logarithm: argmax_v (z_v - ln E_v), E_v = -ln u_v, is
// argmin_v E_v / exp(z_v - m); the exponential is the one the log-sum-exp needs
// anyway, and candidates are compared by cross-multiplication
// (E_v * p_best < E_best * p_v), rescaling p_best whenever the running max moves.
// --------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMfBM = 128;       // vocabulary rows per tile
constexpr int kMfBN = 256;       // batch rows per workgroup
constexpr int kMfBK = 32;        // hidden-dim slab
constexpr int kMfMaxGrid = 512;  // persistent workgroups along the vocabulary (2 per CU)
constexpr float kLn2f = 0.6931471805599453f;

struct LmLaneState {
  float m, s;        // running max and sum of exp(z - m)
  float e_best;      // -log2(u) of the current best candidate (inf: none yet)
  float p_best;      // exp(z_best - m)
  float z_best;
  int idx;
};

// 16-byte granule g (0..3) of row `row` of a [rows][32] bf16 slab
__device__ __forceinline__ int lm_swz(int row, int g) { return row * 4 + (g ^ ((row >> 2) & 3)); }

__device__ __forceinline__ void lm_epilogue_block(const f32x16& acc, LmLaneState& st, int vbase,
                                                  int V, bool tail, float inv_temperature, uint32_t step_c,
                                                  uint32_t sid_lo, uint32_t sid_hi, uint32_t key0,
                                                  uint32_t key1) {
  // accumulator r is vocabulary entry vbase + 8*(r/4) + r%4
  float z[16];
  float gm = -INFINITY;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    z[r] = acc[r] * inv_temperature;
    if (tail && vbase + 8 * (r >> 2) + (r & 3) >= V) z[r] = -INFINITY;
    gm = fmaxf(gm, z[r]);
  }
  const float m_new = fmaxf(st.m, gm);
  if (m_new == -INFINITY) return;            // nothing valid seen so far (vocabulary tail)
  const float alpha = __expf(st.m - m_new);  // 0 on the first block (m = -inf)
  st.s *= alpha;
  st.p_best *= alpha;
  st.m = m_new;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int vq = vbase + 8 * q;
    const Philox4 x = philox4x32_10(static_cast<uint32_t>(vq) >> 2, step_c, sid_lo, sid_hi, key0, key1);
    const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float zz = z[4 * q + j];
      const float p = __expf(zz - m_new);            // 0 for masked entries
      st.s += p;
      const float e = -__builtin_amdgcn_logf(word_to_uniform(w[j]));   // -log2(u) > 0
      // strictly better only: on an exact tie the earlier (lower) index stays
      if (e * st.p_best < st.e_best * p) {
        st.e_best = e;
        st.p_best = p;
        st.z_best = zz;
        st.idx = vq + j;
      }
    }
  }
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void lmhead_mfma_kernel(
    const uint16_t* __restrict__ hidden, const uint16_t* __restrict__ weight,
    const int64_t* __restrict__ seq_id, const int32_t* __restrict__ step, uint32_t key0,
    uint32_t key1, float inv_temperature, LmPartial* __restrict__ part, int C, int H, int V,
    int n_tiles, int n_parts) {
  __shared__ u32x4 lds_w[2][kMfBM * 4];
  __shared__ u32x4 lds_h[2][kMfBN * 4];
  __shared__ LmPartial s_part[2][kMfBN / 2];   // wave-row 1 hands its partials to wave-row 0
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;     // vocabulary half, batch half
  const int l32 = lane & 31, kb = lane >> 5;
  const int c0 = blockIdx.y * kMfBN;

  // this lane owns batch rows c0 + 128*wn + 32*nt + l32
  uint32_t step_c[4], sid_lo[4], sid_hi[4];
  bool c_ok[4];
  LmLaneState st[4];
#pragma unroll
  for (int nt = 0; nt < 4; ++nt) {
    const int c = c0 + 128 * wn + 32 * nt + l32;
    c_ok[nt] = c < C;
    const uint64_t sid = c_ok[nt] ? static_cast<uint64_t>(seq_id[c]) : 0;
    step_c[nt] = c_ok[nt] ? static_cast<uint32_t>(step[c]) : 0;
    sid_lo[nt] = static_cast<uint32_t>(sid);
    sid_hi[nt] = static_cast<uint32_t>(sid >> 32);
    st[nt] = LmLaneState{-INFINITY, 0.0f, INFINITY, 0.0f, 0.0f, 0x7fffffff};
  }

  // staging: thread t moves granules t + 256*j; granule G = (row G>>2, 16-byte chunk G&3)
  const int g_st = tid & 3;
  const int row_st = tid >> 2;                 // + 64*j
  const int nk = H / kMfBK;

  for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const int v0 = tile * kMfBM;
    f32x16 acc[2][4];
#pragma unroll
    for (int it = 0; it < 2; ++it)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[it][nt][r] = 0.0f;

    u32x4 rw[2], rh[4];
    auto load_regs = [&](const int ks) __attribute__((always_inline)) {
      const size_t koff = static_cast<size_t>(ks) * kMfBK + g_st * 8;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int v = v0 + row_st + 64 * j;
        rw[j] = u32x4{0u, 0u, 0u, 0u};
        if (v < V) rw[j] = *reinterpret_cast<const u32x4*>(weight + static_cast<size_t>(v) * H + koff);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = c0 + row_st + 64 * j;
        rh[j] = u32x4{0u, 0u, 0u, 0u};
        if (c < C) rh[j] = *reinterpret_cast<const u32x4*>(hidden + static_cast<size_t>(c) * H + koff);
      }
    };

    load_regs(0);
    for (int ks = 0; ks < nk; ++ks) {
      const int sb = ks & 1;
#pragma unroll
      for (int j = 0; j < 2; ++j) lds_w[sb][lm_swz(row_st + 64 * j, g_st)] = rw[j];
#pragma unroll
      for (int j = 0; j < 4; ++j) lds_h[sb][lm_swz(row_st + 64 * j, g_st)] = rh[j];
      if (ks + 1 < nk) load_regs(ks + 1);
      __syncthreads();
#pragma unroll
      for (int k16 = 0; k16 < 2; ++k16) {
        bf16x8 a[2], b[4];
#pragma unroll
        for (int it = 0; it < 2; ++it)
          a[it] = __builtin_bit_cast(bf16x8, lds_w[sb][lm_swz(64 * wm + 32 * it + l32, 2 * k16 + kb)]);
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
          b[nt] = __builtin_bit_cast(bf16x8, lds_h[sb][lm_swz(128 * wn + 32 * nt + l32, 2 * k16 + kb)]);
#pragma unroll
        for (int it = 0; it < 2; ++it)
#pragma unroll
          for (int nt = 0; nt < 4; ++nt)
            acc[it][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[it], b[nt], acc[it][nt], 0, 0, 0);
      }
    }
    __syncthreads();   // the next tile's first slab reuses an LDS buffer

    const bool tail = v0 + kMfBM > V;   // only the last tile can hold rows past V
    // written out per batch block: the unrolled body is too large for the unroll pragma
    auto epilogue = [&](auto ntc) __attribute__((always_inline)) {
      constexpr int nt = decltype(ntc)::value;
      if (c_ok[nt]) {
        lm_epilogue_block(acc[0][nt], st[nt], v0 + 64 * wm + 4 * kb, V, tail, inv_temperature,
                          step_c[nt], sid_lo[nt], sid_hi[nt], key0, key1);
        lm_epilogue_block(acc[1][nt], st[nt], v0 + 64 * wm + 32 + 4 * kb, V, tail, inv_temperature,
                          step_c[nt], sid_lo[nt], sid_hi[nt], key0, key1);
      }
    };
    epilogue(std::integral_constant<int, 0>{});
    epilogue(std::integral_constant<int, 1>{});
    epilogue(std::integral_constant<int, 2>{});
    epilogue(std::integral_constant<int, 3>{});
  }

  // lane state -> partial; combine the two k-halves of a wave, then the two wave-rows
#pragma unroll
  for (int nt = 0; nt < 4; ++nt) {
    LmPartial p;
    p.m = st[nt].m;
    p.s = st[nt].s;
    p.z = st[nt].z_best;
    p.idx = st[nt].idx;
    // perturbed score z + G with G = -ln(E), E = -ln u = e_best * ln 2
    p.best = st[nt].idx == 0x7fffffff ? -INFINITY : st[nt].z_best - logf(st[nt].e_best * kLn2f);
    LmPartial o;
    o.m = __shfl_xor(p.m, 32, kWave);
    o.s = __shfl_xor(p.s, 32, kWave);
    o.best = __shfl_xor(p.best, 32, kWave);
    o.z = __shfl_xor(p.z, 32, kWave);
    o.idx = __shfl_xor(p.idx, 32, kWave);
    combine(p, o);
    if (wm == 1 && kb == 0) s_part[wn][32 * nt + l32] = p;
    __syncthreads();
    if (wm == 0 && kb == 0) {
      combine(p, s_part[wn][32 * nt + l32]);
      const int c = c0 + 128 * wn + 32 * nt + l32;
      if (c < C) part[static_cast<size_t>(c) * n_parts + blockIdx.x] = p;
    }
    __syncthreads();
  }
}

// --------------------------------------------------------------------------
// merge: one workgroup per batch row over its partials.
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
  int n_parts = w.n_tiles;
  if (dtype == 1 && H % kMfBK == 0) {
    const int n_tiles = (V + kMfBM - 1) / kMfBM;
    n_parts = n_tiles < kMfMaxGrid ? n_tiles : kMfMaxGrid;   // <= w.n_tiles: fits the workspace
    const dim3 grid(n_parts, (C + kMfBN - 1) / kMfBN);
    COPRIS_PRE("lmhead_mfma_kernel");
    hipLaunchKernelGGL(lmhead_mfma_kernel, grid, dim3(256), 0, stream,
                       static_cast<const uint16_t*>(hidden), static_cast<const uint16_t*>(weight),
                       seq_id, step, key0, key1, inv_t, part, C, H, V, n_tiles, n_parts);
    COPRIS_POST("lmhead_mfma_kernel");
  } else {
    const dim3 grid(w.n_tiles, (C + kLmTileC - 1) / kLmTileC);
    COPRIS_PRE("lmhead_generic_kernel");
    if (dtype == 0) {
      hipLaunchKernelGGL(lmhead_generic_kernel<float>, grid, dim3(256), 0, stream,
                         static_cast<const float*>(hidden), static_cast<const float*>(weight),
                         seq_id, step, key0, key1, inv_t, part, C, H, V, w.n_tiles);
    } else {
      hipLaunchKernelGGL(lmhead_generic_kernel<uint16_t>, grid, dim3(256), 0, stream,
                         static_cast<const uint16_t*>(hidden), static_cast<const uint16_t*>(weight),
                         seq_id, step, key0, key1, inv_t, part, C, H, V, w.n_tiles);
    }
    COPRIS_POST("lmhead_generic_kernel");
  }
  COPRIS_PRE("lmhead_merge_kernel");
  hipLaunchKernelGGL(lmhead_merge_kernel, dim3(C), dim3(256), 0, stream, part, n_parts, token,
                     logprob, lse);
  COPRIS_POST("lmhead_merge_kernel");
  return 0;
}

}  // namespace copris
