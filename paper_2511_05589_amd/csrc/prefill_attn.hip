// Re-prefill of resumed partial trajectories: causal attention over packed
// variable-length sequences, filling the sequences' KV pages on the way
// (Section 4, "Prioritized Resumption": buffered partial trajectories are continued in the
// next rollout stage; Section 5.3 names their re-prefilling as a cost of high concurrency).
//
// bf16, head_dim 128, page 16.  The unit of work is (query head, tile of 32 query tokens): one
// wave, the tile as two blocks of 16 queries.  A workgroup is four waves = four consecutive
// units of one (sequence, kv head, super-tile of T tiles), the units numbered tile-major
// (unit u = tile u / g, head u % g of the kv head's g query heads) and T = 4 / gcd(g, 4) so that
// the units of a super-tile fill whole workgroups for every g: no wave is without a unit except
// at the end of a sequence.  A workgroup's units lie in at most two neighbouring tiles (g >= 4),
// so its waves need the same K/V rows: the workgroup walks the sequence's K/V once, up to
// the last of its tiles, and a wave whose own tile is over only keeps fetching.
// A step of one wave is a chain (scores -> weights -> value product) that no second wave of the
// same workgroup can overlap, because they all pass the same barrier, so the matrix pipes are
// kept busy by TWO independent workgroups per CU whose chains drift apart.
// The workgroup walks the K/V in 32-token steps (two pages); a wave's last step is its tile's
// own tokens; a step's K and V rows (2 x 8 KB) are fetched once by all
// waves together with LDS-direct loads, three steps ahead, into a ring of four LDS buffers
// (the XOR swizzle is applied by choosing which global granule a lane fetches) and read by
// every wave in operand layout.  Per block of 16 queries:
//     S^T[token][query] = K[token][:] . Q[query][:]           2 x 4 x mfma 16x16x32 (16 tokens each)
//     O^T[d][query]    += V^T[d][token] . P^T[token][query]   8 x mfma 16x16x32 (all 32 tokens)
// The value product runs over the step's 32 tokens at once (the 32-deep instruction has
// twice the rate of the 16-deep one): its k-slot (g, e) is token 4g+e of the first page for
// e < 4 and token 4g+e-4 of the second page for e >= 4, which is exactly how the two score
// tiles leave the weights in a lane and how the transposing LDS read delivers V - both
// operands are two register pairs put side by side, nothing moves between lanes.
// The K and V operands are read from LDS once per step and used for both query blocks,
// and max / sum / rescale of a query live in the lane that owns it.  Only the last step
// needs the causal mask.  The workgroup that holds a tile's unit of head 0 also copies
// that tile's K/V rows to the sequence's pages (each row is written by exactly one
// workgroup).  Super-tiles are taken from the end of the sequences first (the long ones).
//
// LDS reads are inline instructions with explicit waits: the compiler cannot tell which
// LDS-direct load fills which buffer and would wait for all of them before any LDS read.
#include <type_traits>

#include "copris_device.h"
#include "copris_internal.h"

namespace copris {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kD = 128;
constexpr int kP = 16;
constexpr int kTileQ = 32;                        // query tokens per workgroup
constexpr int kPageGranules = kP * kD * 2 / 16;   // 256 16-byte granules of K (and of V) per page
constexpr int kSubs = 2;                          // pages per step
constexpr int kStepTok = kSubs * kP;              // 32 tokens per step (= kTileQ: a tile's own tokens are one step)
constexpr int kStepGranules = kSubs * kPageGranules;   // 512 granules of K (and of V) per step
constexpr int kHalfBytes = kStepGranules * 16;    // 8 KB: a step's K rows (or V rows)
constexpr int kBufBytes = 2 * kHalfBytes;         // 16 KB: one ring buffer = K rows, then V rows
constexpr int kRing = 4;                          // ring buffers
constexpr int kAhead = kRing - 1;                 // a step is requested this many steps before its use
constexpr int kThreads = 256;                     // four waves = four units; all fetch
constexpr int kHeadsPerWg = kThreads / 64;
constexpr int kLoadsPerStep = 2 * kStepGranules / kThreads;   // LDS-direct loads a wave issues per step
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kSlack = 6.0f;   // scores may exceed the softmax reference by 2^kSlack
constexpr float kBig = 64.0f;    // = 2^kSlack
static_assert(kLoadsPerStep == 4, "the waits below count four loads per wave and step");

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  uint32_t r;
  asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(lo), "v"(hi));
  return r;
}

// LDS position (in 16-byte granules) of granule c of token row `row` of a page (conflict-free
// for the row-wise fills and for both operand read patterns).
__device__ __forceinline__ int swz_k(int row, int c) { return row * 16 + (c ^ (row & 15)); }
__device__ __forceinline__ int swz_v(int row, int c) { return row * 16 + (c ^ ((row & 7) << 1)); }

template <int OFF>
__device__ __forceinline__ u32x4 lds_read128(uint32_t addr) {
  u32x4 x;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(x) : "v"(addr), "n"(OFF) : "memory");
  return x;
}
// the transposing read: four 16-bit elements of four rows, delivered in MFMA operand order
template <int OFF>
__device__ __forceinline__ s16x4 lds_read_tr16(uint32_t addr) {
  s16x4 x;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(x) : "v"(addr), "n"(OFF) : "memory");
  return x;
}

// (two workgroups per CU: 256 registers per lane)
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void prefill_attn_kernel(
    const uint16_t* __restrict__ q, const u32x4* __restrict__ k, const u32x4* __restrict__ v,
    const int32_t* __restrict__ cu_seqlens, const int32_t* __restrict__ block_table,
    u32x4* __restrict__ k_cache, u32x4* __restrict__ v_cache, uint16_t* __restrict__ out,
    float* __restrict__ lse, int Hq, int Hkv, int super_tiles, int wgs_per_super, int max_pages,
    float scale_log2e) {
  __shared__ __attribute__((aligned(1024))) char smem[kRing * kBufBytes];

  const int b = blockIdx.z, kvh = blockIdx.y;
  const int g = Hq / Hkv;
  const int s0 = cu_seqlens[b];
  const int len = cu_seqlens[b + 1] - s0;
  const int n_tiles = (len + kTileQ - 1) / kTileQ;
  const int n_super = (n_tiles + super_tiles - 1) / super_tiles;
  const int sidx = static_cast<int>(blockIdx.x) / wgs_per_super, wg = static_cast<int>(blockIdx.x) % wgs_per_super;
  if (sidx >= n_super) return;
  const int tile0 = (n_super - 1 - sidx) * super_tiles;   // late (long) super-tiles first
  const int units = g * super_tiles;                       // units of a super-tile: u -> (tile0 + u / g, head u % g)
  if (tile0 + (kHeadsPerWg * wg) / g >= n_tiles) return;   // not even the first unit has a tile
  // the last step of the workgroup: the tile of its last unit that has one
  const int last_tile = min(tile0 + min(kHeadsPerWg * wg + kHeadsPerWg - 1, units - 1) / g, n_tiles - 1);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15;        // N index of both products: the query within a block
  const int bq = lane >> 4;       // k-group of the MFMA operand layouts
  const int unit = kHeadsPerWg * wg + wave;
  const int tile = __builtin_amdgcn_readfirstlane(tile0 + unit / g);   // this wave's tile ...
  const bool computes = unit < units && tile < n_tiles;                // ... if it has one (else the wave only moves data)
  const int head = kvh * g + unit % g;
  const int q0 = tile * kTileQ;                      // first query token of the tile
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(smem));

  // ---- a tile's own K/V rows go to the sequence's pages, by the workgroup that holds the
  // tile's unit of head 0 (slots past the end of the sequence are left alone) ----
  for (int i4 = 0; i4 < kHeadsPerWg; ++i4) {
    const int u = kHeadsPerWg * wg + i4;
    const int ut = tile0 + u / g;
    if (u >= units || u % g != 0 || ut >= n_tiles) continue;
    const int32_t* bt = block_table + static_cast<size_t>(b) * max_pages;
#pragma unroll
    for (int j = 0; j < 2 * kStepGranules / kThreads; ++j) {
      const int i = tid + j * kThreads;             // i < 512: K, else V; token (i & 511) >> 4, granule i & 15
      const int gi = i & (kStepGranules - 1);
      const int tok = ut * kTileQ + (gi >> 4);
      if (tok < len) {
        const size_t src = (static_cast<size_t>(s0 + tok) * Hkv + kvh) * (kD * 2 / 16) + (gi & 15);
        const size_t dst = (static_cast<size_t>(bt[tok / kP]) * Hkv + kvh) * kPageGranules + (gi & (kPageGranules - 1));
        if (i < kStepGranules) k_cache[dst] = k[src];
        else v_cache[dst] = v[src];
      }
    }
  }

  // Q^T operands: lane (n, bq) holds Q[query n of block nb][32*kk + 8*bq .. +8]; queries past
  // the end of the sequence are zero
  bf16x8 qf[2][4];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const int tq = q0 + 16 * nb + n;
    const u32x4* qrow =
        reinterpret_cast<const u32x4*>(q + (static_cast<size_t>(s0 + tq) * Hq + head) * kD);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      u32x4 x = {0u, 0u, 0u, 0u};
      if (computes && tq < len) x = qrow[kk * 4 + bq];
      qf[nb][kk] = __builtin_bit_cast(bf16x8, x);
    }
  }

  // ---- LDS-direct fetch of one step (32 tokens of K and of V) into a ring buffer ----
  // A wave moves rows 8*wave .. 8*wave+7 of K and of V: per operand two instructions of four
  // rows x 256 bytes.  LDS position lane%16 of row 8*wave + 4*j + lane/16 takes the global
  // granule that the swizzle maps there.  Rows past the end of the sequence re-read its last
  // row (they are masked below); steps past the last one do the same into buffers nobody reads.
  const int ld_row = 8 * wave + (lane >> 4);                       // + 4*j
  const size_t row_pitch = static_cast<size_t>(Hkv) * (kD * 2);
  const char* kbase = reinterpret_cast<const char*>(k) + (static_cast<size_t>(s0) * Hkv + kvh) * (kD * 2);
  const char* vbase = reinterpret_cast<const char*>(v) + (static_cast<size_t>(s0) * Hkv + kvh) * (kD * 2);
  uint32_t ld_gk[2], ld_gv[2];                                     // byte offset of the lane's granule in its row
  uint32_t ld_ok[2], ld_ov[2];                                     // ... and in a whole step, for steps that need no clamp
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int row = ld_row + 4 * j;
    ld_gk[j] = static_cast<uint32_t>((lane & 15) ^ (row & 15)) * 16;
    ld_gv[j] = static_cast<uint32_t>((lane & 15) ^ ((row & 7) << 1)) * 16;
    ld_ok[j] = static_cast<uint32_t>(row) * static_cast<uint32_t>(row_pitch) + ld_gk[j];
    ld_ov[j] = static_cast<uint32_t>(row) * static_cast<uint32_t>(row_pitch) + ld_gv[j];
  }
  auto fetch = [&](int step) __attribute__((always_inline)) {
    char* dst = smem + (step & (kRing - 1)) * kBufBytes + (8 * wave) * 256;
    if (step * kStepTok + kStepTok <= len) {
      // a whole step inside the sequence: one address for the wave plus the lane's fixed offset
      const size_t so = static_cast<size_t>(step) * kStepTok * row_pitch;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        __builtin_amdgcn_global_load_lds(kbase + so + ld_ok[j], dst + j * 1024, 16, 0, 0);
        __builtin_amdgcn_global_load_lds(vbase + so + ld_ov[j], dst + kHalfBytes + j * 1024, 16, 0, 0);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int tok = min(step * kStepTok + ld_row + 4 * j, len - 1);
        const size_t ro = static_cast<size_t>(tok) * row_pitch;
        __builtin_amdgcn_global_load_lds(kbase + (ro + ld_gk[j]), dst + j * 1024, 16, 0, 0);
        __builtin_amdgcn_global_load_lds(vbase + (ro + ld_gv[j]), dst + kHalfBytes + j * 1024, 16, 0, 0);
      }
    }
  };

  // operand read addresses inside a ring buffer (bytes)
  uint32_t k_off[4], v_off[8];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) k_off[kk] = lds0 + swz_k(n, 4 * kk + bq) * 16;
  {
    const int vrow = 4 * bq + (n >> 2);
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
      v_off[dt] = lds0 + kHalfBytes + swz_v(vrow, 2 * dt + ((n & 3) >> 1)) * 16 + (n & 1) * 8;
  }

  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.0f, 0.0f};
  f32x4 o[2][8];
#pragma unroll
  for (int i = 0; i < 16; ++i) o[i >> 3][i & 7] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

  // A wave's loads complete in issue order, four per step: once at most 4*(kAhead-1) are
  // outstanding, the step after the current one has landed.
#pragma unroll
  for (int st = 0; st < kAhead; ++st) fetch(st);
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(4 * (kAhead - 1)) : "memory");

  // one step.  diag = true: the tile's own tokens (causal mask, end of the sequence).
  // active = false: a step after the wave's own tile (another wave of the workgroup still
  // needs the rows), or a wave without a unit: it fetches and waits with the others.
  auto do_step = [&](const int step, const bool active, auto diag) __attribute__((always_inline)) {
    constexpr bool kDiag = decltype(diag)::value;
    const uint32_t boff = static_cast<uint32_t>(step & (kRing - 1)) * kBufBytes;
    fetch(step + kAhead);          // into the buffer of step-1, which every wave left at the last barrier

    if (active) {
      // Scores of the two pages: K rows as the A operand (token = lane & 15), read once for
      // both query blocks.  This lane: query n of each block, tokens 4*bq .. 4*bq+3 of each page.
      // A block whose queries all lie before a page's tokens is fully masked there: its
      // weights are exp2(-inf - m) = 0 (m is finite from step 0 on: token 0 is visible to
      // every query).
      float t[kSubs][2][4];
      u32x4 kf[kSubs][4];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) kf[0][kk] = lds_read128<0>(boff + k_off[kk]);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) kf[1][kk] = lds_read128<kPageGranules * 16>(boff + k_off[kk]);
#pragma unroll
      for (int sub = 0; sub < kSubs; ++sub) {
        if (sub == 0) {
          asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(kf[0][0]), "+v"(kf[0][1]), "+v"(kf[0][2]), "+v"(kf[0][3])::"memory");
        } else {
          asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(kf[1][0]), "+v"(kf[1][1]), "+v"(kf[1][2]), "+v"(kf[1][3])::"memory");
        }
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          f32x4 sc = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
          for (int kk = 0; kk < 4; ++kk)
            sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[sub][kk]), qf[nb][kk], sc, 0, 0, 0);
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) t[sub][nb][rr] = sc[rr];   // raw: the scale rides on the exponent's fma
        }
      }
      if (kDiag) {
#pragma unroll
        for (int sub = 0; sub < kSubs; ++sub)
#pragma unroll
          for (int nb = 0; nb < 2; ++nb) {
            const int tq = q0 + 16 * nb + n;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
              const int tk = step * kStepTok + sub * kP + 4 * bq + rr;
              t[sub][nb][rr] = (tk <= tq && tk < len) ? t[sub][nb][rr] : -INFINITY;
            }
          }
      }
      // V^T operands of the first four head-dim tiles are requested now and arrive during the
      // softmax: as the A operand through the transposing read (per page the lane gets rows
      // 4*bq + n/4 .. of columns 16*dt + 4*(n%4) .. +3), the two pages' halves side by side.
      s16x4 vf[8][2];
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        vf[dt][0] = lds_read_tr16<0>(boff + v_off[dt]);
        vf[dt][1] = lds_read_tr16<kPageGranules * 16>(boff + v_off[dt]);
      }
      // The running reference m of a query only has to keep the weights in range, so it is
      // left alone while no score of the step exceeds it by more than kSlack (in log2 units):
      // the step then needs no maximum, no exchange between lanes and no rescaling of the
      // state.  The weights are formed against the old reference first; if one of them is
      // above 2^kSlack (then so is the lane's sum of them - the test - and also while m is
      // still -inf), the references that have to move are moved and the weights formed again.
      float w[2][kSubs][4], add[2];
      auto weights = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
          for (int sub = 0; sub < kSubs; ++sub)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr)
              w[nb][sub][rr] = __builtin_amdgcn_exp2f(__builtin_fmaf(t[sub][nb][rr], scale_log2e, -m_run[nb]));
          add[nb] = ((w[nb][0][0] + w[nb][0][1]) + (w[nb][0][2] + w[nb][0][3])) +
                    ((w[nb][1][0] + w[nb][1][1]) + (w[nb][1][2] + w[nb][1][3]));
        }
      };
      weights();
      // (written so that a NaN sum - a masked score against m = -inf - also takes the branch)
      const bool grow = !(add[0] <= kBig && add[1] <= kBig);
      if (__builtin_amdgcn_ballot_w64(grow) != 0) {
        float alpha[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          float mx = fmaxf(fmaxf(t[0][nb][0], t[0][nb][1]), fmaxf(t[0][nb][2], t[0][nb][3]));
#pragma unroll
          for (int sub = 1; sub < kSubs; ++sub)
            mx = fmaxf(mx, fmaxf(fmaxf(t[sub][nb][0], t[sub][nb][1]), fmaxf(t[sub][nb][2], t[sub][nb][3])));
          mx *= scale_log2e;                         // (the scale is positive: max commutes with it)
          mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
          mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
          // only a query whose own scores outgrew its reference moves it, so a query's
          // arithmetic does not depend on the other queries of the wave
          const float m_new = (mx > m_run[nb] + kSlack) ? mx : m_run[nb];
          alpha[nb] = __builtin_amdgcn_exp2f(m_run[nb] - m_new);
          m_run[nb] = m_new;
          l_run[nb] *= alpha[nb];
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) o[i >> 3][i & 7] *= alpha[i >> 3];
        weights();
      }
      // weights of the step's 32 tokens as the B operand of the 32-deep value product:
      // the first page's four in k-slots 0..3, the second page's in 4..7
      bf16x8 pf[2];
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        l_run[nb] += add[nb];
        pf[nb] = __builtin_bit_cast(
            bf16x8, u32x4{pack_bf16x2(w[nb][0][0], w[nb][0][1]), pack_bf16x2(w[nb][0][2], w[nb][0][3]),
                          pack_bf16x2(w[nb][1][0], w[nb][1][1]), pack_bf16x2(w[nb][1][2], w[nb][1][3])});
      }
#pragma unroll
      for (int dt = 4; dt < 8; ++dt) {
        vf[dt][0] = lds_read_tr16<0>(boff + v_off[dt]);
        vf[dt][1] = lds_read_tr16<kPageGranules * 16>(boff + v_off[dt]);
      }
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        if (half == 0) {
          asm volatile("s_waitcnt lgkmcnt(8)"
                       : "+v"(vf[0][0]), "+v"(vf[0][1]), "+v"(vf[1][0]), "+v"(vf[1][1]), "+v"(vf[2][0]),
                         "+v"(vf[2][1]), "+v"(vf[3][0]), "+v"(vf[3][1])::"memory");
        } else {
          asm volatile("s_waitcnt lgkmcnt(0)"
                       : "+v"(vf[4][0]), "+v"(vf[4][1]), "+v"(vf[5][0]), "+v"(vf[5][1]), "+v"(vf[6][0]),
                         "+v"(vf[6][1]), "+v"(vf[7][0]), "+v"(vf[7][1])::"memory");
        }
#pragma unroll
        for (int dt = 4 * half; dt < 4 * half + 4; ++dt) {
          const s16x4 v0 = vf[dt][0], v1 = vf[dt][1];
          const s16x8 vv = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
          const bf16x8 va = __builtin_bit_cast(bf16x8, vv);
          o[0][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pf[0], o[0][dt], 0, 0, 0);
          o[1][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pf[1], o[1][dt], 0, 0, 0);
        }
      }
    }
    // the next step has landed, for every wave; all are done with this step's buffer
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(4 * (kAhead - 1)) : "memory");
  };
  const int my_last = computes ? tile : -1;
  int step = 0;
  for (; step < my_last; ++step) do_step(step, true, std::false_type{});
  if (computes) {
    do_step(tile, true, std::true_type{});
    step = tile + 1;
  }
  for (; step <= last_tile; ++step) do_step(step, false, std::false_type{});
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // (the loads past the last step land before the LDS is given back)

  // normalise and store: lane (n, bq) owns d = 16*dt + 4*bq + r of query n
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const int tq = q0 + 16 * nb + n;
    float l_all = l_run[nb];
    l_all += __shfl_xor(l_all, 16, kWave);
    l_all += __shfl_xor(l_all, 32, kWave);
    if (computes && tq < len) {
      const float inv = 1.0f / l_all;
      uint16_t* dst = out + (static_cast<size_t>(s0 + tq) * Hq + head) * kD + 4 * bq;
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) {
        const uint2 w = make_uint2(pack_bf16x2(o[nb][dt][0] * inv, o[nb][dt][1] * inv),
                                   pack_bf16x2(o[nb][dt][2] * inv, o[nb][dt][3] * inv));
        *reinterpret_cast<uint2*>(dst + 16 * dt) = w;
      }
      if (lse != nullptr && bq == 0)
        lse[static_cast<size_t>(s0 + tq) * Hq + head] = (m_run[nb] + __builtin_amdgcn_logf(l_all)) * kLn2;
    }
  }
}

}  // namespace

bool prefill_attn_supported(int Hq, int Hkv, int D, int page_size, int dtype) {
  if (dtype != 1 || D != kD || page_size != kP || Hq % Hkv != 0) return false;
  const int g = Hq / Hkv;
  return g >= 1 && g <= 8;
}

int launch_prefill_attn(const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                        const int32_t* block_table, void* k_cache, void* v_cache, void* out,
                        float* lse, int B, int Hq, int Hkv, int max_pages, int max_seqlen,
                        float scale, hipStream_t stream) {
  const int g = Hq / Hkv;
  // super-tile of T tiles: the smallest T for which g * T units fill whole workgroups
  const int gcd4 = (g % 4 == 0) ? 4 : (g % 2 == 0 ? 2 : 1);
  const int super_tiles = kHeadsPerWg / gcd4;
  const int wgs_per_super = g * super_tiles / kHeadsPerWg;
  const int n_tiles_max = (max_seqlen + kTileQ - 1) / kTileQ;
  const dim3 grid(((n_tiles_max + super_tiles - 1) / super_tiles) * wgs_per_super, Hkv, B);
  const float scale_log2e = scale * kLog2e;
  COPRIS_PRE("prefill_attn_kernel");
  hipLaunchKernelGGL(prefill_attn_kernel, grid, dim3(kThreads), 0, stream,
                     static_cast<const uint16_t*>(q), static_cast<const u32x4*>(k),
                     static_cast<const u32x4*>(v), cu_seqlens, block_table,
                     static_cast<u32x4*>(k_cache), static_cast<u32x4*>(v_cache),
                     static_cast<uint16_t*>(out), lse, Hq, Hkv, super_tiles, wgs_per_super, max_pages, scale_log2e);
  COPRIS_POST("prefill_attn_kernel");
  return 0;
}

}  // namespace copris
