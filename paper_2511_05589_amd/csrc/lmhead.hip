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
#include <mutex>
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

// GIVEN: no sampling; the partial that holds vocabulary entry target[c] carries its logit
// (best = +inf marks it, so the same combine picks it up).
template <typename T, bool GIVEN>
__global__ __launch_bounds__(256) void lmhead_generic_kernel(
    const T* __restrict__ hidden, const T* __restrict__ weight, const int64_t* __restrict__ seq_id,
    const int32_t* __restrict__ step, const int32_t* __restrict__ target, uint32_t key0,
    uint32_t key1, float inv_temperature, LmPartial* __restrict__ part, int C, int H, int V,
    int n_tiles) {
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
    if (v_ok && GIVEN) {
      const float z = acc[r] * inv_temperature;
      const bool hit = v == target[c];
      p.m = z;
      p.s = 1.0f;
      p.z = z;
      p.best = hit ? INFINITY : -INFINITY;
      p.idx = hit ? v : 0x7fffffff;
    } else if (v_ok) {
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
// A workgroup (4 waves) owns a 128 (vocab) x 256 (batch) tile and walks the hidden
// dimension in slabs of 64 (128-byte row segments: full cache lines).  Workgroups are
// persistent over vocabulary tiles and keep their per-row state across tiles, so W is
// streamed from HBM exactly once and only gridDim.x partials per row reach the merge.
// Two workgroups share a CU, so one's epilogue (vector ALU) overlaps the other's
// products (matrix cores) and loads.
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
constexpr int kMfBK = 64;        // hidden-dim slab (128 bytes of a row)
constexpr int kMfMaxGrid = 512;  // persistent workgroups along the vocabulary (2 per CU)
constexpr float kLn2f = 0.6931471805599453f;

struct LmLaneState {
  float m, s;        // running max and sum of exp(z - m)
  float e_best;      // -log2(u) of the current best candidate (inf: none yet)
  float p_best;      // exp(z_best - m)
  float z_best;
  int idx;
};

// LDS position (in 16-byte granules) of granule g (0..7) of row `row` of a [rows][64]
// bf16 slab.  Sixteen lanes that read one granule column of sixteen consecutive rows
// touch sixteen different 4-bank groups.
__device__ __forceinline__ int lm_swz(int row, int g) { return row * 8 + (g ^ ((row >> 1) & 7)); }

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

// Same block, no sampling: running log-sum-exp, and the logit of vocabulary entry `target`
// if this lane holds it.
__device__ __forceinline__ void lm_given_block(const f32x16& acc, LmLaneState& st, int vbase, int V,
                                               bool tail, float inv_temperature, int target) {
  float z[16];
  float gm = -INFINITY;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    z[r] = acc[r] * inv_temperature;
    if (tail && vbase + 8 * (r >> 2) + (r & 3) >= V) z[r] = -INFINITY;
    gm = fmaxf(gm, z[r]);
  }
  const float m_new = fmaxf(st.m, gm);
  if (m_new == -INFINITY) return;
  st.s *= __expf(st.m - m_new);
  st.m = m_new;
  float s = 0.0f;
#pragma unroll
  for (int r = 0; r < 16; ++r) s += __expf(z[r] - m_new);
  st.s += s;
  const int d = target - vbase;                  // entry vbase + 8q + j sits in accumulator 4q + j
  if (d >= 0 && d < 32 && (d & 4) == 0 && target < V) {
    const int sel = (d >> 3) * 4 + (d & 3);
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (r == sel) st.z_best = z[r];
    st.idx = target;
  }
}

// ---- memory pipeline of the matrix-core kernel --------------------------------
// Both operands reach LDS through LDS-direct loads (global_load_lds_dwordx4: each
// lane's 16 bytes land at base + 16*lane, no registers in between), so the data in
// flight lives in LDS rings:
//   W       [128 rows][64 k] slabs of 16 KB, ring of two, issued a slab and a half ahead (a
//           slab's slot is given away as soon as every wave has its operands in registers);
//   hidden  [128 rows][64 k] units of 16 KB - the two batch halves of a slab are
//           consumed one after the other against the same W slab - ring of three,
//           issued two units (one slab) ahead.
// Every wave issues a quarter of each slab and unit, one load at a time between the matrix
// products.  The outstanding-load counter of a wave retires in order, so the issue order is
// chosen such that what a wait needs is always older than what may stay in flight: per slab
// d hidden (d+1, half 0), then W(d+2), and after the middle barrier hidden (d+1, half 1).  The
// compiler cannot count LDS-direct loads per buffer (it would drain them all before any LDS
// read), so the operand reads are inline ds_read_b128 and every wait is explicit.  80 KB of LDS per workgroup: two workgroups fill a CU's 160 KB.
constexpr int kLmStreamOnce = 2;                    // cache policy of the W loads: non-temporal (every byte is read once)
constexpr int kNW = 2;                              // W ring slabs
constexpr int kNH = 3;                              // hidden ring units
constexpr int kSlab = 128 * kMfBK * 2;              // 16 KB: a W slab or a hidden unit
constexpr int kHRing = kNW * kSlab;                 // hidden ring starts here
constexpr int kMfLds = kHRing + kNH * kSlab;        // 80 KB

template <int OFF>
__device__ __forceinline__ u32x4 lds_read128(uint32_t addr) {
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}
// (Waits on these reads are inline "s_waitcnt lgkmcnt(N)" statements that tie the operands
// which must have arrived, so that no use can be scheduled above the wait.)

// Timing probes (never defined in the product build; `python -m paper_2511_05589_amd.build
// --define NAME --out other.so` builds one, bench.py --lib times it; the results of such a
// build are wrong by design, every access stays in bounds and every loop ends):
//   COPRIS_LM_PROBE_NO_MFMA      the matrix products become one scalar multiply-add each
//   COPRIS_LM_PROBE_NO_EPILOGUE  no log-sum-exp / sampling after a tile
//   COPRIS_LM_PROBE_NO_W_LOADS   the W stream is not requested (operands are whatever LDS holds)
//   COPRIS_LM_PROBE_NO_H_LOADS   the hidden stream is not requested
//   COPRIS_LM_PROBE_W_FROM_L2    every workgroup re-reads the first two vocabulary tiles
// They separate what bounds the kernel: the memory pipeline alone, the products alone, the
// lead of the W stream.
#if defined(COPRIS_LM_PROBE_NO_MFMA)
#define COPRIS_LM_MFMA(fa, fb, c) ((c)[0] += static_cast<float>((fa)[0]) * static_cast<float>((fb)[0]), (c))
#else
#define COPRIS_LM_MFMA(fa, fb, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, c, 0, 0, 0)
#endif

// HALVES = 2: 256 batch rows per workgroup (two halves of 128 against every W slab), W ring
// of two slabs, hidden ring of three units.  HALVES = 1 (C <= 128): only the first half
// exists, so there is no second half of products, loads and barrier; the hidden ring needs two
// units and the W ring gets three slabs (a slab is requested two slabs ahead).
template <bool GIVEN, int HALVES>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void lmhead_mfma_kernel(
    const uint16_t* __restrict__ hidden, const uint16_t* __restrict__ weight,
    const int64_t* __restrict__ seq_id, const int32_t* __restrict__ step,
    const int32_t* __restrict__ target, uint32_t key0, uint32_t key1, float inv_temperature,
    LmPartial* __restrict__ part, int C, int H, int V, int n_tiles, int n_parts) {
  __shared__ __attribute__((aligned(1024))) char smem[kMfLds];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wq = wave & 1;     // vocabulary half; 64-row block of a batch half
  const int l32 = lane & 31, kb = lane >> 5;
  const int c0 = blockIdx.y * kMfBN;
  const int nkd = H / kMfBK;                   // slabs per tile
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(smem));
  const uint32_t pitch = static_cast<uint32_t>(H) * 2u;
  constexpr int kRingW = HALVES == 2 ? kNW : 3;        // W ring slabs
  constexpr int kRingH = HALVES == 2 ? kNH : 2;        // hidden ring units
  constexpr int kHBase = kRingW * kSlab;               // hidden ring starts here
  static_assert(kHBase + kRingH * kSlab <= kMfLds, "rings exceed the workgroup's LDS");

  // operand read offsets inside a slab / unit (bytes); it / nt add 32 rows = 4096 bytes
  uint32_t a_off[4], b_off[4];
#pragma unroll
  for (int k16 = 0; k16 < 4; ++k16) {
    a_off[k16] = lm_swz(64 * wm + l32, 2 * k16 + kb) * 16;
    b_off[k16] = lm_swz(64 * wq + l32, 2 * k16 + kb) * 16;
  }

  // ---- loader cursors (wave-uniform) ----
  const int my_tiles = blockIdx.x < n_tiles ? (n_tiles - 1 - blockIdx.x) / gridDim.x + 1 : 0;
  const int total = my_tiles * nkd;            // W slabs this workgroup consumes (hidden units: 2x)
  // Every wave moves a quarter of every W slab and of every hidden unit: rows 32*wave ..
  // 32*wave+31, four instructions of 8 rows x 128 bytes.  LDS position 64*chunk + lane of a
  // slab holds (row 8*chunk + lane/8, stored granule lane%8); the lane fetches the global
  // granule that the swizzle maps there: (row>>1)&7 = lane>>4 for even chunks, +4 for odd
  // ones, i.e. bit 6 of the byte offset flips for odd j.
  const int ld_row = 32 * wave + (lane >> 3);                // + 8*j
  const uint32_t ld_g = ((lane & 7) ^ (lane >> 4)) * 16;
  int w_tile = blockIdx.x, w_kd = 0, w_ring = 0;             // W cursor (tile, slab) and ring slot
  int h_n = 0, h_kd = 0, h_ring = 0;                         // hidden units issued so far (half = h_n & 1), slab, slot
  const char* wbase = reinterpret_cast<const char*>(weight);
  const char* hbase = reinterpret_cast<const char*>(hidden);
  // Rows past V re-read the last vocabulary row (masked in the epilogue); rows past C
  // duplicate the last batch row (never used).
  // one of the four loads of this wave's quarter of the W slab / hidden unit at the cursor
  auto w_load = [&](int j) __attribute__((always_inline)) {
    char* dst = smem + w_ring * kSlab + (4 * wave + j) * 1024;
    const uint32_t koff = static_cast<uint32_t>(w_kd) * (kMfBK * 2) + ld_g;
#if defined(COPRIS_LM_PROBE_W_FROM_L2)
    const int v = min((w_tile & 1) * kMfBM + ld_row + 8 * j, V - 1);
#else
    const int v = min(w_tile * kMfBM + ld_row + 8 * j, V - 1);
#endif
#if !defined(COPRIS_LM_PROBE_NO_W_LOADS)
    __builtin_amdgcn_global_load_lds(wbase + (static_cast<uint32_t>(v) * pitch + (koff ^ ((j & 1) * 64))), dst,
                                     16, 0, kLmStreamOnce);
#else
    (void)v; (void)koff; (void)dst;
#endif
  };
  auto w_advance = [&]() __attribute__((always_inline)) {
    w_ring = w_ring + 1 == kRingW ? 0 : w_ring + 1;
    if (++w_kd == nkd) {
      w_kd = 0;
      w_tile += gridDim.x;
    }
  };
  auto h_load = [&](int j) __attribute__((always_inline)) {
    char* dst = smem + kHBase + h_ring * kSlab + (4 * wave + j) * 1024;
    const uint32_t koff = static_cast<uint32_t>(h_kd) * (kMfBK * 2) + ld_g;
    const int c = min(c0 + (HALVES == 2 ? 128 * (h_n & 1) : 0) + ld_row + 8 * j, C - 1);
#if !defined(COPRIS_LM_PROBE_NO_H_LOADS)
    __builtin_amdgcn_global_load_lds(hbase + (static_cast<uint32_t>(c) * pitch + (koff ^ ((j & 1) * 64))), dst,
                                     16, 0, 0);
#else
    (void)c; (void)koff; (void)dst;
#endif
  };
  auto h_advance = [&]() __attribute__((always_inline)) {
    h_ring = h_ring + 1 == kRingH ? 0 : h_ring + 1;
    if ((HALVES == 1 || (h_n & 1)) && ++h_kd == nkd) h_kd = 0;
    ++h_n;
  };
  auto issue_w = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < 4; ++j) w_load(j);
    w_advance();
  };
  auto issue_h = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < 4; ++j) h_load(j);
    h_advance();
  };

  // this lane owns batch rows c0 + 128*half + 64*wq + 32*nt + l32 (state index 2*half + nt);
  // their stream keys stay in registers (a global load inside the tile loop would drain
  // the prefetch queue)
  LmLaneState st[4];
  uint32_t step_c[4], sid_lo[4], sid_hi[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    st[i] = LmLaneState{-INFINITY, 0.0f, INFINITY, 0.0f, 0.0f, 0x7fffffff};
    const int c = c0 + 128 * (i >> 1) + 64 * wq + 32 * (i & 1) + l32;
    if (GIVEN) {   // step_c holds the row's given token
      step_c[i] = c < C ? static_cast<uint32_t>(target[c]) : 0xffffffffu;
      sid_lo[i] = sid_hi[i] = 0;
    } else {
      const uint64_t sid = c < C ? static_cast<uint64_t>(seq_id[c]) : 0;
      step_c[i] = c < C ? static_cast<uint32_t>(step[c]) : 0;
      sid_lo[i] = static_cast<uint32_t>(sid);
      sid_hi[i] = static_cast<uint32_t>(sid >> 32);
    }
  }

  // prologue = the loads of "slabs -2 and -1".  A wave's loads complete in issue order, and
  // that order is, per slab d: hidden (d+1, half 0), W(d+2) | hidden (d+1, half 1).  So at the
  // top of slab d the wave may leave its newest eight loads (W(d+1), hidden (d, 1)) in flight
  // and knows hidden (d, 0) has landed; at mid-slab it may leave the eight issued since the
  // top and knows W(d+1) and hidden (d, 1) have.
  // (HALVES = 1: per slab d hidden (d+1), W(d+3); at the top of slab d the newest four loads,
  // W(d+2), may stay in flight and hidden (d), W(d+1) have landed.)
  if (total > 0) {
    if (HALVES == 2) {
      issue_w();
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // W(0): the first slab reads it before any barrier of the loop
      issue_h();
      issue_w();
      issue_h();
    } else {
      issue_w();
      issue_w();
      issue_h();
      issue_w();
      asm volatile("s_waitcnt vmcnt(12)" ::: "memory");  // W(0)
    }
  }
  asm volatile("s_barrier" ::: "memory");

  int ring = 0, hring = 0;                     // W / hidden ring slots being consumed
  for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const int v0 = tile * kMfBM;
    f32x16 acc[2][2][2];                       // [batch half][it][nt]
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i >> 2][(i >> 1) & 1][i & 1][r] = 0.0f;

    if constexpr (HALVES == 1) {
      for (int kd = 0; kd < nkd; ++kd) {
        const uint32_t wb = lds0 + ring * kSlab;
        ring = ring + 1 == kRingW ? 0 : ring + 1;
        u32x4 a[4][2];
#pragma unroll
        for (int k16 = 0; k16 < 4; ++k16) {
          a[k16][0] = lds_read128<0>(wb + a_off[k16]);
          a[k16][1] = lds_read128<4096>(wb + a_off[k16]);
        }
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(a[0][0]), "+v"(a[0][1]), "+v"(a[1][0]), "+v"(a[1][1]), "+v"(a[2][0]),
                       "+v"(a[2][1]), "+v"(a[3][0]), "+v"(a[3][1])::"memory");
        // ---- top: hidden unit (d) and W(d+1) have landed; every wave holds W(d)'s operands ----
        asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        asm volatile("s_barrier" ::: "memory");
        const uint32_t hb = lds0 + kHBase + hring * kSlab;
        hring = hring + 1 == kRingH ? 0 : hring + 1;
        u32x4 b[4][2];
#pragma unroll
        for (int k16 = 0; k16 < 4; ++k16) {
          b[k16][0] = lds_read128<0>(hb + b_off[k16]);
          b[k16][1] = lds_read128<4096>(hb + b_off[k16]);
        }
#pragma unroll
        for (int grp = 0; grp < 2; ++grp) {
          if (grp == 0) {
            asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(b[0][0]), "+v"(b[0][1]), "+v"(b[1][0]), "+v"(b[1][1])::"memory");
          } else {
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(b[2][0]), "+v"(b[2][1]), "+v"(b[3][0]), "+v"(b[3][1])::"memory");
          }
#pragma unroll
          for (int m = 0; m < 8; ++m) {
            const int k16 = 2 * grp + (m >> 2), it = (m >> 1) & 1;
            const bf16x8 fa = __builtin_bit_cast(bf16x8, a[k16][it]);
            const bf16x8 fb = __builtin_bit_cast(bf16x8, b[k16][m & 1]);
            acc[0][it][m & 1] = COPRIS_LM_MFMA(fa, fb, acc[0][it][m & 1]);
            if (m & 1) {   // hidden (d+1) into the slot of (d-1), then W(d+3) into the slot of W(d)
              const int q = 4 * grp + (m >> 1);                                   // 0 .. 7
              __builtin_amdgcn_sched_barrier(0);
              if (q < 4) {
                h_load(q);
                if (q == 3) h_advance();
              } else {
                w_load(q - 4);
                if (q == 7) w_advance();
              }
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        }
      }
    } else
    for (int kd = 0; kd < nkd; ++kd) {
      // The W operands of the slab go to registers BEFORE the top barrier (the slab has been
      // in LDS, for every wave, since the middle barrier of the slab before), so that barrier
      // also says "every wave holds its operands": the slot of W(d) is free from there on and
      // W(d+2) is requested right away - a slab is on its way for a slab and a half although
      // the ring holds only two.
      const uint32_t wb = lds0 + ring * kSlab;
      ring ^= 1;
      u32x4 a[4][2];
#pragma unroll
      for (int k16 = 0; k16 < 4; ++k16) {
        a[k16][0] = lds_read128<0>(wb + a_off[k16]);
        a[k16][1] = lds_read128<4096>(wb + a_off[k16]);
      }
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(a[0][0]), "+v"(a[0][1]), "+v"(a[1][0]), "+v"(a[1][1]), "+v"(a[2][0]),
                     "+v"(a[2][1]), "+v"(a[3][0]), "+v"(a[3][1])::"memory");
      // ---- top: hidden unit (d, half 0) has landed ----
      asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
      asm volatile("s_barrier" ::: "memory");   // ... for every wave; all are done with slab d-1
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        if (half == 1) {
          // ---- middle: W(d+1) and hidden unit (d, half 1) have landed ----
          asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
          asm volatile("s_barrier" ::: "memory");             // all are done with unit (d, half 0)
        }
        const uint32_t hb = lds0 + kHBase + hring * kSlab;
        hring = hring + 1 == kRingH ? 0 : hring + 1;
        // all eight hidden operands of the half at once, then sixteen products in two groups
        // of eight: one wait per eight products instead of one per four
        u32x4 b[4][2];
#pragma unroll
        for (int k16 = 0; k16 < 4; ++k16) {
          b[k16][0] = lds_read128<0>(hb + b_off[k16]);
          b[k16][1] = lds_read128<4096>(hb + b_off[k16]);
        }
#pragma unroll
        for (int grp = 0; grp < 2; ++grp) {
          if (grp == 0) {
            asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(b[0][0]), "+v"(b[0][1]), "+v"(b[1][0]), "+v"(b[1][1])::"memory");
          } else {
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(b[2][0]), "+v"(b[2][1]), "+v"(b[3][0]), "+v"(b[3][1])::"memory");
          }
#pragma unroll
          for (int m = 0; m < 8; ++m) {
            const int k16 = 2 * grp + (m >> 2), it = (m >> 1) & 1;
            const bf16x8 fa = __builtin_bit_cast(bf16x8, a[k16][it]);
            const bf16x8 fb = __builtin_bit_cast(bf16x8, b[k16][m & 1]);
            acc[half][it][m & 1] = COPRIS_LM_MFMA(fa, fb, acc[half][it][m & 1]);
            // The twelve loads a wave issues per slab go out one at a time between the
            // products.  Issued in a bunch they keep every wave of the CU at the issue stage
            // while the address unit works through them, and the matrix pipes idle meanwhile;
            // spread out they cost the products nothing.  First half: hidden (d+1, half 0) (its
            // slot is free since the top barrier), then W(d+2) (likewise); second half: hidden
            // (d+1, half 1) (the middle barrier has freed the slot of (d, half 0)).  Past the
            // last slab the loads re-read clamped rows into ring slots nobody reads any more.
            if (half == 0 && (m & 1)) {
              const int q = 4 * grp + (m >> 1);                                   // 0 .. 7
              __builtin_amdgcn_sched_barrier(0);
              if (q < 4) {
                h_load(q);
                if (q == 3) h_advance();
              } else {
                w_load(q - 4);
                if (q == 7) w_advance();
              }
              __builtin_amdgcn_sched_barrier(0);
            } else if (half == 1 && (m == 1 || m == 5)) {
              const int q = 2 * grp + (m >> 2);                                   // 0 .. 3
              __builtin_amdgcn_sched_barrier(0);
              h_load(q);
              if (q == 3) h_advance();
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        }
      }
    }

    const bool tail = v0 + kMfBM > V;   // only the last tile can hold rows past V
    // written out per batch block: the unrolled body is too large for the unroll pragma
    auto epilogue = [&](auto ic) __attribute__((always_inline)) {
      constexpr int i = decltype(ic)::value;       // state index = 2*half + nt
      const int c = c0 + 128 * (i >> 1) + 64 * wq + 32 * (i & 1) + l32;
#if defined(COPRIS_LM_PROBE_NO_EPILOGUE)
      if (c < C) {   // keep the accumulators alive, nothing else
        st[i].s += acc[i >> 1][0][i & 1][0] + acc[i >> 1][1][i & 1][15];
        st[i].m = 0.0f;
        st[i].idx = v0;
      } else
#endif
      if (c < C && GIVEN) {
        lm_given_block(acc[i >> 1][0][i & 1], st[i], v0 + 64 * wm + 4 * kb, V, tail, inv_temperature,
                       static_cast<int>(step_c[i]));
        lm_given_block(acc[i >> 1][1][i & 1], st[i], v0 + 64 * wm + 32 + 4 * kb, V, tail,
                       inv_temperature, static_cast<int>(step_c[i]));
      } else if (c < C) {
        lm_epilogue_block(acc[i >> 1][0][i & 1], st[i], v0 + 64 * wm + 4 * kb, V, tail,
                          inv_temperature, step_c[i], sid_lo[i], sid_hi[i], key0, key1);
        lm_epilogue_block(acc[i >> 1][1][i & 1], st[i], v0 + 64 * wm + 32 + 4 * kb, V, tail,
                          inv_temperature, step_c[i], sid_lo[i], sid_hi[i], key0, key1);
      }
    };
    epilogue(std::integral_constant<int, 0>{});
    epilogue(std::integral_constant<int, 1>{});
    if (HALVES == 2) {
      epilogue(std::integral_constant<int, 2>{});
      epilogue(std::integral_constant<int, 3>{});
    }
  }

  // lane state -> partial; combine the two k-halves of a wave, then the two vocabulary
  // halves.  The exchange buffer reuses the ring memory: all slabs have been consumed.
  asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
  LmPartial(*s_part)[kMfBN / 2] = reinterpret_cast<LmPartial(*)[kMfBN / 2]>(smem);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    LmPartial p;
    p.m = st[i].m;
    p.s = st[i].s;
    p.z = st[i].z_best;
    p.idx = st[i].idx;
    // perturbed score z + G with G = -ln(E), E = -ln u = e_best * ln 2
    if (GIVEN) {
      p.best = st[i].idx == 0x7fffffff ? -INFINITY : INFINITY;
    } else {
      p.best = st[i].idx == 0x7fffffff ? -INFINITY : st[i].z_best - logf(st[i].e_best * kLn2f);
    }
    LmPartial o;
    o.m = __shfl_xor(p.m, 32, kWave);
    o.s = __shfl_xor(p.s, 32, kWave);
    o.best = __shfl_xor(p.best, 32, kWave);
    o.z = __shfl_xor(p.z, 32, kWave);
    o.idx = __shfl_xor(p.idx, 32, kWave);
    combine(p, o);
    if (wm == 1 && kb == 0) s_part[wq][32 * i + l32] = p;
    __syncthreads();
    if (wm == 0 && kb == 0) {
      combine(p, s_part[wq][32 * i + l32]);
      const int c = c0 + 128 * (i >> 1) + 64 * wq + 32 * (i & 1) + l32;
      if (c < C) part[static_cast<size_t>(c) * n_parts + blockIdx.x] = p;
    }
    __syncthreads();
  }
}

// --------------------------------------------------------------------------
// matrix-core kernel for micro-batches of given tokens (many row blocks).
//
// With hundreds of row blocks the work is a plain dense contraction and what counts is
// bytes moved into LDS per flop.  One 8-wave workgroup per CU owns a 256 (vocab) x 256
// (batch) tile - 64 KB of operands per 64-wide slab of the hidden dimension instead of
// the 96 KB that two 128 x 256 workgroups move for the same flops - and the whole 160 KB
// of LDS is one pipeline: W slabs [256][64] in a ring of three (issued three slabs ahead),
// hidden slabs [256][64] in a ring of two.  Every wave issues its eighth of both slabs,
// the hidden part first, so that its in-order load counter can wait for the hidden slab
// while the younger W slab stays in flight.  The one barrier per slab sits before the last
// eight products of the slab, after all of the slab's LDS reads: the refill and the first
// operand reads of the next slab are issued there and overlap those products.
// No sampler here: the epilogue is the running log-sum-exp and the given token's logit.
// --------------------------------------------------------------------------
constexpr int kGmBM = 256;                          // vocabulary rows per tile
constexpr int kGmBN = 256;                          // batch rows per workgroup
constexpr int kGmSlab = 256 * kMfBK * 2;            // 32 KB
constexpr int kGmNW = 3;                            // W ring slabs
constexpr int kGmHRing = kGmNW * kGmSlab;           // hidden ring (2 slabs) starts here
constexpr int kGmLds = kGmHRing + 2 * kGmSlab;      // 160 KB
constexpr int kGmMaxGrid = 256;                     // one workgroup per CU
constexpr int kGmMinRows = 384;                     // below this the 128-row kernel is used

template <int N>
__device__ __forceinline__ void lds_wait6(u32x4 (&a)[4], u32x4 (&b)[2]) {
  asm volatile("s_waitcnt lgkmcnt(%6)"
               : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1])
               : "n"(N)
               : "memory");
}

template <bool W_DEEP>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void lmhead_gemm_given_kernel(
    const uint16_t* __restrict__ hidden, const uint16_t* __restrict__ weight,
    const int32_t* __restrict__ target, float inv_temperature, LmPartial* __restrict__ part, int C,
    int H, int V, int n_tiles, int n_parts) {
  __shared__ __attribute__((aligned(1024))) char smem[kGmLds];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wq = wave & 3;     // 128-row vocabulary half; 64-row batch block
  const int l32 = lane & 31, kb = lane >> 5;
  // grid = (row blocks, tile lanes): consecutive workgroups (which the dispatcher deals out
  // to the XCDs in turn) differ in the row block, so one XCD's L2 sees few row blocks
  const int lane_id = blockIdx.y, n_lanes = gridDim.y;
  const int c0 = blockIdx.x * kGmBN;
  const int nkd = H / kMfBK;
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(smem));
  const uint32_t pitch = static_cast<uint32_t>(H) * 2u;
  // the deep stream (three slots, issued three slabs ahead) and the shallow one (two slots)
  constexpr int kWSlots = W_DEEP ? 3 : 2, kHSlots = W_DEEP ? 2 : 3;
  constexpr int kHBase = kWSlots * kGmSlab;

  // operand read offsets inside a slab (bytes); each further 32-row block adds 4096
  uint32_t a_off[4], b_off[4];
#pragma unroll
  for (int k16 = 0; k16 < 4; ++k16) {
    a_off[k16] = lm_swz(128 * wm + l32, 2 * k16 + kb) * 16;
    b_off[k16] = lm_swz(64 * wq + l32, 2 * k16 + kb) * 16;
  }

  // ---- loader cursors (wave-uniform).  Wave w moves rows 32w .. 32w+31 of every slab:
  // four instructions of 8 rows x 128 bytes; LDS position 64*chunk + lane holds (row
  // 8*chunk + lane/8, stored granule lane%8) and the lane fetches the global granule the
  // swizzle maps there ((row>>1)&7 = lane>>4 for even chunks, +4 for odd ones).
  const int my_tiles = (n_tiles - 1 - lane_id) / n_lanes + 1;
  const int total = my_tiles * nkd;            // slabs this workgroup consumes
  const int ld_row = 32 * wave + (lane >> 3);
  const uint32_t ld_g = ((lane & 7) ^ (lane >> 4)) * 16;
  int w_tile = lane_id, w_kd = 0, w_slot = 0;
  int h_kd = 0, h_slot = 0;
  const char* wbase = reinterpret_cast<const char*>(weight);
  const char* hbase = reinterpret_cast<const char*>(hidden);
  // one of the four loads of this wave's eighth of the W / hidden slab at the cursor
  auto w_load = [&](int j) __attribute__((always_inline)) {
    char* dst = smem + w_slot * kGmSlab + (4 * wave + j) * 1024;
    const uint32_t koff = static_cast<uint32_t>(w_kd) * (kMfBK * 2) + ld_g;
    const int v = min(w_tile * kGmBM + ld_row + 8 * j, V - 1);   // rows past V re-read the last row (masked later)
    __builtin_amdgcn_global_load_lds(wbase + (static_cast<uint32_t>(v) * pitch + (koff ^ ((j & 1) * 64))), dst,
                                     16, 0, 0);
  };
  auto w_advance = [&]() __attribute__((always_inline)) {
    w_slot = w_slot + 1 == kWSlots ? 0 : w_slot + 1;
    if (++w_kd == nkd) {
      w_kd = 0;
      w_tile += n_lanes;
    }
  };
  auto h_load = [&](int j) __attribute__((always_inline)) {
    char* dst = smem + kHBase + h_slot * kGmSlab + (4 * wave + j) * 1024;
    const uint32_t koff = static_cast<uint32_t>(h_kd) * (kMfBK * 2) + ld_g;
    const int c = min(c0 + ld_row + 8 * j, C - 1);               // rows past C duplicate the last row (unused)
    __builtin_amdgcn_global_load_lds(hbase + (static_cast<uint32_t>(c) * pitch + (koff ^ ((j & 1) * 64))), dst,
                                     16, 0, 0);
  };
  auto h_advance = [&]() __attribute__((always_inline)) {
    h_slot = h_slot + 1 == kHSlots ? 0 : h_slot + 1;
    if (++h_kd == nkd) h_kd = 0;
  };
  // Load k (0..7) of the set a barrier opens: the shallow stream's slab first, then the deep
  // one's.  Past the workgroup's last slab the loads re-read clamped rows into ring slots
  // nobody reads any more, so none of them needs a condition.
  auto load_one = [&](int k) __attribute__((always_inline)) {
    const bool is_h = W_DEEP ? k < 4 : k >= 4;
    if (is_h) {
      h_load(k & 3);
      if ((k & 3) == 3) h_advance();
    } else {
      w_load(k & 3);
      if ((k & 3) == 3) w_advance();
    }
  };

  // this lane owns batch rows c0 + 64*wq + 32*nt + l32; their given tokens are fetched
  // before the pipeline starts (the prologue's wait covers them)
  LmLaneState st[2];
  int tgt[2];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    st[nt] = LmLaneState{-INFINITY, 0.0f, INFINITY, 0.0f, 0.0f, 0x7fffffff};
    const int c = c0 + 64 * wq + 32 * nt + l32;
    tgt[nt] = c < C ? target[c] : -1;
  }

  // prologue: slab 0 of both streams and slab 1 of the deep one land; then the steady order
  // begins - after the barrier that ends slab d, the shallow stream's slab d+2 and the deep
  // one's slab d+3 go out, one load at a time between the matrix products of the next 32
  // (issued in a bunch they keep all eight waves at the issue stage while the address unit
  // works through them, and the matrix pipes idle).  The first two loads of the set that the
  // prologue's barrier opens go out here, the other six with the products of slab 0.
  for (int k = 0; k < 4; ++k) load_one(k);          // shallow slab 0
  for (int k = 4; k < 8; ++k) load_one(k);          // deep slab 0
  for (int k = 4; k < 8; ++k) load_one(k);          // deep slab 1
  asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
  load_one(0);
  load_one(1);

  u32x4 a[2][4], b[2][2];
  int wslot = 0, hslot = 0;                     // ring slots of the slab being consumed
  uint32_t wb = lds0, hb = lds0 + kHBase;
  auto read_operands = [&](auto bufc, auto k16c) __attribute__((always_inline)) {
    constexpr int buf = decltype(bufc)::value, k16 = decltype(k16c)::value;
    a[buf][0] = lds_read128<0>(wb + a_off[k16]);
    a[buf][1] = lds_read128<4096>(wb + a_off[k16]);
    a[buf][2] = lds_read128<8192>(wb + a_off[k16]);
    a[buf][3] = lds_read128<12288>(wb + a_off[k16]);
    b[buf][0] = lds_read128<0>(hb + b_off[k16]);
    b[buf][1] = lds_read128<4096>(hb + b_off[k16]);
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I3 = std::integral_constant<int, 3>;
  read_operands(I0{}, I0{});

  int d = 0;
  for (int tile = lane_id; tile < n_tiles; tile += n_lanes) {
    const int v0 = tile * kGmBM;
    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i >> 1][i & 1][r] = 0.0f;
    // eight products from operand buffer `buf`; if `issue`, loads FIRST and FIRST+1 of the
    // open set go out after the second and the sixth of them
    auto products = [&](auto bufc, auto firstc, const bool issue) __attribute__((always_inline)) {
      constexpr int buf = decltype(bufc)::value, kFirst = decltype(firstc)::value;
      const bf16x8 fb0 = __builtin_bit_cast(bf16x8, b[buf][0]);
      const bf16x8 fb1 = __builtin_bit_cast(bf16x8, b[buf][1]);
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {
        const bf16x8 fa = __builtin_bit_cast(bf16x8, a[buf][rb]);
        acc[rb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb0, acc[rb][0], 0, 0, 0);
        acc[rb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb1, acc[rb][1], 0, 0, 0);
        if (rb == 0 || rb == 2) {
          __builtin_amdgcn_sched_barrier(0);
          if (issue) load_one(kFirst + (rb >> 1));
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    };
    using L0 = std::integral_constant<int, 0>;
    using L2 = std::integral_constant<int, 2>;
    using L4 = std::integral_constant<int, 4>;
    using L6 = std::integral_constant<int, 6>;

    for (int kd = 0; kd < nkd; ++kd, ++d) {
      read_operands(I1{}, I1{});
      lds_wait6<6>(a[0], b[0]);
      products(I0{}, L2{}, true);
      read_operands(I0{}, I2{});
      lds_wait6<6>(a[1], b[1]);
      products(I1{}, L4{}, true);
      read_operands(I1{}, I3{});
      lds_wait6<6>(a[0], b[0]);
      products(I0{}, L6{}, true);
      // every LDS read of slab d is complete; the other operand buffer is tied as well so
      // that the products just issued from it stay above this wait
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(a[1][0]), "+v"(a[1][1]), "+v"(a[1][2]), "+v"(a[1][3]), "+v"(b[1][0]),
                     "+v"(b[1][1]), "+v"(a[0][0]), "+v"(a[0][1]), "+v"(a[0][2]), "+v"(a[0][3]),
                     "+v"(b[0][0]), "+v"(b[0][1])::"memory");
      const bool more = d + 1 < total;
      if (more) {
        // slab d+1 has landed (this wave's part: only the deep stream's slab d+2, the newest
        // four loads, is younger) ...
        asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        asm volatile("s_barrier" ::: "memory");   // ... for every wave, and all are done reading slab d
        wslot = wslot + 1 == kWSlots ? 0 : wslot + 1;
        hslot = hslot + 1 == kHSlots ? 0 : hslot + 1;
        wb = lds0 + wslot * kGmSlab;
        hb = lds0 + kHBase + hslot * kGmSlab;
        read_operands(I0{}, I0{});                // first operands of slab d+1, under the products below
      }
      products(I1{}, L0{}, more);                 // with the first two loads into the slots of slab d
    }

    const bool tail = v0 + kGmBM > V;   // only the last tile can hold rows past V
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const int c = c0 + 64 * wq + 32 * nt + l32;
      if (c < C) {
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
          lm_given_block(acc[rb][nt], st[nt], v0 + 128 * wm + 32 * rb + 4 * kb, V, tail, inv_temperature,
                         tgt[nt]);
      }
    }
  }

  // lane state -> partial; combine the two k-halves of a wave, then the two vocabulary
  // halves.  The exchange buffer reuses the ring memory: all slabs have been consumed.
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  LmPartial(*s_part)[64] = reinterpret_cast<LmPartial(*)[64]>(smem);
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    LmPartial p;
    p.m = st[nt].m;
    p.s = st[nt].s;
    p.z = st[nt].z_best;
    p.idx = st[nt].idx;
    p.best = st[nt].idx == 0x7fffffff ? -INFINITY : INFINITY;
    LmPartial o;
    o.m = __shfl_xor(p.m, 32, kWave);
    o.s = __shfl_xor(p.s, 32, kWave);
    o.best = __shfl_xor(p.best, 32, kWave);
    o.z = __shfl_xor(p.z, 32, kWave);
    o.idx = __shfl_xor(p.idx, 32, kWave);
    combine(p, o);
    if (wm == 1 && kb == 0) s_part[wq][32 * nt + l32] = p;
    __syncthreads();
    if (wm == 0 && kb == 0) {
      combine(p, s_part[wq][32 * nt + l32]);
      const int c = c0 + 64 * wq + 32 * nt + l32;
      if (c < C) part[static_cast<size_t>(c) * n_parts + lane_id] = p;
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
    if (token != nullptr) token[c] = a.idx;
    // no candidate at all (a given token outside [0, V)): not a number
    logprob[c] = a.idx == 0x7fffffff ? __int_as_float(0x7fc00000) : a.z - l;
    if (lse != nullptr) lse[c] = l;
  }
}

// True if the matrix-core kernels take the shape (they address both operands with 32-bit
// byte offsets).
static bool lm_use_mfma(int C, int H, int V, int dtype) {
  return dtype == 1 && H % kMfBK == 0 && static_cast<uint64_t>(V) * H * 2 < (1ull << 32) &&
         static_cast<uint64_t>(C) * H * 2 < (1ull << 32);
}
// Micro-batches of given tokens go to the 256 x 256 kernel.
static bool lm_use_gemm(int C, int H, int V, int dtype, bool given) {
  return given && C >= kGmMinRows && lm_use_mfma(C, H, V, dtype);
}

// Partials per row.  Matrix-core kernels: the grid is (parts, blocks of 256 rows) with
// parts * blocks <= the resident workgroups (512, or 256 for the 256 x 256 kernel) where
// possible, so that the workgroups that run at the same time walk the same vocabulary tiles
// (W comes from HBM once and is shared through the caches) and each keeps its rows' state
// across all of its tiles.
static int lm_parts(int C, int H, int V, int dtype, bool given) {
  if (!lm_use_mfma(C, H, V, dtype)) return (V + kLmTileV - 1) / kLmTileV;
  const bool gemm = lm_use_gemm(C, H, V, dtype, given);
  const int bm = gemm ? kGmBM : kMfBM;
  const int n_tiles = (V + bm - 1) / bm;
  const int blocks = (C + kMfBN - 1) / kMfBN;
  int parts = (gemm ? kGmMaxGrid : kMfMaxGrid) / blocks;
  parts = parts < 1 ? 1 : parts;
  return parts < n_tiles ? parts : n_tiles;
}

size_t lm_token_workspace_bytes(int M, int H, int V, int dtype) {
  return align256(static_cast<size_t>(M) * lm_parts(M, H, V, dtype, true) * sizeof(LmPartial));
}

// Both modes: target == nullptr samples (seq_id / step / seed), else scores the given tokens.
static int launch_lmhead(const void* hidden, const void* weight, const int64_t* seq_id,
                         const int32_t* step, const int32_t* target, uint64_t seed,
                         float temperature, int32_t* token, float* logprob, float* lse,
                         void* workspace, int C, int H, int V, int dtype, hipStream_t stream) {
  LmPartial* part = static_cast<LmPartial*>(workspace);
  const uint32_t key0 = static_cast<uint32_t>(seed), key1 = static_cast<uint32_t>(seed >> 32);
  const float inv_t = 1.0f / temperature;
  const bool given = target != nullptr;
  const int n_parts = lm_parts(C, H, V, dtype, given);
  if (lm_use_gemm(C, H, V, dtype, given)) {
    const int n_tiles = (V + kGmBM - 1) / kGmBM;
    const dim3 grid((C + kGmBN - 1) / kGmBN, n_parts);
    COPRIS_PRE("lmhead_gemm_given_kernel");
    hipLaunchKernelGGL(lmhead_gemm_given_kernel<true>, grid, dim3(512), 0, stream,
                       static_cast<const uint16_t*>(hidden), static_cast<const uint16_t*>(weight),
                       target, inv_t, part, C, H, V, n_tiles, n_parts);
    COPRIS_POST("lmhead_gemm_given_kernel");
  } else if (lm_use_mfma(C, H, V, dtype)) {
    const int n_tiles = (V + kMfBM - 1) / kMfBM;
    const dim3 grid(n_parts, (C + kMfBN - 1) / kMfBN);
    COPRIS_PRE("lmhead_mfma_kernel");
#define COPRIS_LM_MFMA_LAUNCH(G, HV)                                                                   \
  hipLaunchKernelGGL((lmhead_mfma_kernel<G, HV>), grid, dim3(256), 0, stream,                            \
                     static_cast<const uint16_t*>(hidden), static_cast<const uint16_t*>(weight), seq_id, \
                     step, target, key0, key1, inv_t, part, C, H, V, n_tiles, n_parts)
    const bool one_half = C <= kMfBN / 2;      // only the first 128 batch rows exist
    if (given && one_half) COPRIS_LM_MFMA_LAUNCH(true, 1);
    else if (given) COPRIS_LM_MFMA_LAUNCH(true, 2);
    else if (one_half) COPRIS_LM_MFMA_LAUNCH(false, 1);
    else COPRIS_LM_MFMA_LAUNCH(false, 2);
#undef COPRIS_LM_MFMA_LAUNCH
    COPRIS_POST("lmhead_mfma_kernel");
  } else {
    const dim3 grid(n_parts, (C + kLmTileC - 1) / kLmTileC);
#define COPRIS_LM_GENERIC(T, G)                                                                   \
  hipLaunchKernelGGL((lmhead_generic_kernel<T, G>), grid, dim3(256), 0, stream,                   \
                     static_cast<const T*>(hidden), static_cast<const T*>(weight), seq_id, step,  \
                     target, key0, key1, inv_t, part, C, H, V, n_parts)
    COPRIS_PRE("lmhead_generic_kernel");
    if (dtype == 0 && given) COPRIS_LM_GENERIC(float, true);
    else if (dtype == 0) COPRIS_LM_GENERIC(float, false);
    else if (given) COPRIS_LM_GENERIC(uint16_t, true);
    else COPRIS_LM_GENERIC(uint16_t, false);
#undef COPRIS_LM_GENERIC
    COPRIS_POST("lmhead_generic_kernel");
  }
  COPRIS_PRE("lmhead_merge_kernel");
  hipLaunchKernelGGL(lmhead_merge_kernel, dim3(C), dim3(256), 0, stream, part, n_parts, token,
                     logprob, lse);
  COPRIS_POST("lmhead_merge_kernel");
  return 0;
}

int launch_lmhead_logprob(const void* hidden, const void* weight, const int64_t* seq_id,
                          const int32_t* step, uint64_t seed, float temperature, int32_t* token,
                          float* logprob, float* lse, void* workspace, int C, int H, int V,
                          int dtype, hipStream_t stream) {
  return launch_lmhead(hidden, weight, seq_id, step, nullptr, seed, temperature, token, logprob, lse,
                       workspace, C, H, V, dtype, stream);
}

// --------------------------------------------------------------------------
// The sampling call for callers that cannot allocate: the per-(row, part) partials live in a
// file-scope device array instead of a caller workspace.  Every GPU the library runs on holds
// its own copy of the array at its own address; the address is looked up once per device.
// --------------------------------------------------------------------------
constexpr size_t kLmScratchBytes = 4u << 20;
static __device__ __align__(256) unsigned char scratch[kLmScratchBytes];

size_t lm_noalloc_scratch_limit() { return kLmScratchBytes; }

size_t lm_noalloc_scratch_needed(int C, int H, int V, int dtype) {
  return static_cast<size_t>(C) * lm_parts(C, H, V, dtype, false) * sizeof(LmPartial);
}

// Device address of this GPU's copy of `scratch` (nullptr + *err set on failure).
static void* lm_scratch_on_current_device(hipError_t* err) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptrs[kMaxDevices] = {};
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= kMaxDevices) {
    *err = hipErrorInvalidDevice;
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (ptrs[dev] == nullptr) {
    void* p = nullptr;
    *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (*err != hipSuccess) return nullptr;
    ptrs[dev] = p;
  }
  return ptrs[dev];
}

int launch_lmhead_logprob_noalloc(const void* hidden, const void* weight, const int64_t* seq_id,
                                  const int32_t* step, uint64_t seed, float temperature,
                                  int32_t* token, float* logprob, float* lse, int C, int H, int V,
                                  int dtype, hipStream_t stream) {
  hipError_t err = hipSuccess;
  void* ws = lm_scratch_on_current_device(&err);
  if (ws == nullptr) {
    set_error_detail("hipGetSymbolAddress(scratch)", err);
    return kErrLaunch;
  }
  return launch_lmhead(hidden, weight, seq_id, step, nullptr, seed, temperature, token, logprob, lse, ws,
                       C, H, V, dtype, stream);
}

int launch_lmhead_token_logprob(const void* hidden, const void* weight, const int32_t* tokens,
                                float temperature, float* logprob, float* lse, void* workspace,
                                int M, int H, int V, int dtype, hipStream_t stream) {
  return launch_lmhead(hidden, weight, nullptr, nullptr, tokens, 0, temperature, nullptr, logprob,
                       lse, workspace, M, H, V, dtype, stream);
}

}  // namespace copris
