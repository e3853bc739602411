// Re-prefill of resumed partial trajectories: causal attention over packed
// variable-length sequences, filling the sequences' KV pages on the way
// (Section 4, "Prioritized Resumption": buffered partial trajectories are continued in the
// next rollout stage; Section 5.3 names their re-prefilling as a cost of high concurrency).
//
// bf16, head_dim 128, page 16.  One workgroup owns (sequence, kv head, tile of 32 query
// tokens); wave h of it owns query head kvh*g + h for those 32 tokens, as two blocks of 16
// queries.  The workgroup walks the sequence's K/V in 32-token steps (two pages) up to the
// tile's own tokens, which are the last step; a step's K and V rows (2 x 8 KB) are fetched
// once by all waves together, register-staged two steps ahead, parked in a double-buffered
// LDS tile and read by every wave in operand layout.  Per block of 16 queries:
//     S^T[token][query] = K[token][:] . Q[query][:]           2 x 4 x mfma 16x16x32 (16 tokens each)
//     O^T[d][query]    += V^T[d][token] . P^T[token][query]   8 x mfma 16x16x32 (all 32 tokens)
// The value product runs over the step's 32 tokens at once (the 32-deep instruction has
// twice the rate of the 16-deep one): its k-slot (g, e) is token 4g+e of the first page for
// e < 4 and token 4g+e-4 of the second page for e >= 4, which is exactly how the two score
// tiles leave the weights in a lane and how the transposing LDS read delivers V - both
// operands are two register pairs put side by side, nothing moves between lanes.
// The K and V operands are read from LDS once per step and used for both query blocks,
// and max / sum / rescale of a query live in the lane that owns it.  Only the last step
// needs the causal mask.  The workgroup that owns a tile also writes
// that tile's K/V rows to the sequence's pages (each row is written by exactly one
// workgroup).  Tiles are taken from the end of the sequences first (the long ones).
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
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kSlack = 6.0f;   // scores may exceed the softmax reference by 2^kSlack
constexpr float kBig = 64.0f;    // = 2^kSlack

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  uint32_t r;
  asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(lo), "v"(hi));
  return r;
}

// LDS position (in 16-byte granules) of granule c of token row `row` (conflict-free for the
// row-wise writes and for both operand read patterns).
__device__ __forceinline__ int swz_k(int row, int c) { return row * 16 + (c ^ (row & 15)); }
__device__ __forceinline__ int swz_v(int row, int c) { return row * 16 + (c ^ ((row & 7) << 1)); }

// Threads of a workgroup: four or eight waves (they divide the 1024 granules of a step
// evenly and keep the staging registers few); the first G compute, all fetch.
template <int G> struct PrefillThreads {
  static constexpr int value = G <= 4 ? 256 : 512;
};

template <int G>
__global__ __launch_bounds__(PrefillThreads<G>::value) void prefill_attn_kernel(
    const uint16_t* __restrict__ q, const u32x4* __restrict__ k, const u32x4* __restrict__ v,
    const int32_t* __restrict__ cu_seqlens, const int32_t* __restrict__ block_table,
    u32x4* __restrict__ k_cache, u32x4* __restrict__ v_cache, uint16_t* __restrict__ out,
    float* __restrict__ lse, int Hq, int Hkv, int max_pages, float scale_log2e) {
  constexpr int kThreads = PrefillThreads<G>::value;
  constexpr int kStage = 2 * kStepGranules / kThreads;   // granules a thread moves per step
  static_assert(kStage * kThreads == 2 * kStepGranules, "a step's granules divide evenly over the threads");
  __shared__ u32x4 lds_k[2][kStepGranules];
  __shared__ u32x4 lds_v[2][kStepGranules];

  const int b = blockIdx.z, kvh = blockIdx.y;
  const int s0 = cu_seqlens[b];
  const int len = cu_seqlens[b + 1] - s0;
  const int n_tiles = (len + kTileQ - 1) / kTileQ;
  if (static_cast<int>(blockIdx.x) >= n_tiles) return;
  const int tile = n_tiles - 1 - blockIdx.x;        // late (long) tiles first
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15;        // N index of both products: the query within a block
  const int bq = lane >> 4;       // k-group of the MFMA operand layouts
  const bool computes = wave < G;                 // (the other waves only move data)
  const int head = kvh * G + min(wave, G - 1);
  const int q0 = tile * kTileQ;                      // first query token of the tile
  const int last_step = tile;                        // the tile's own tokens
  const int last_page = (len - 1) / kP;
  const int32_t* bt = block_table + static_cast<size_t>(b) * max_pages;

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

  // ---- cooperative, register-staged fetch of one step (32 tokens of K and of V) ----
  // granule i of a step: i < 512 is K, else V; token (i & 511) >> 4, column granule i & 15.
  // Rows past the end of the sequence re-read its last row (they are masked below).
  // two register stages: the fetch of step s+2 is in flight while step s+1 is parked
  u32x4 stage_a[kStage], stage_b[kStage];
  auto fetch = [&](u32x4 (&stage)[kStage], int step) __attribute__((always_inline)) {
    // steps past the last one re-read the last token's rows (never parked)
#pragma unroll
    for (int j = 0; j < kStage; ++j) {
      const int i = tid + j * kThreads;
      const int tok = min(step * kStepTok + ((i & (kStepGranules - 1)) >> 4), len - 1);
      const size_t g = (static_cast<size_t>(s0 + tok) * Hkv + kvh) * (kD * 2 / 16) + (i & 15);
      const u32x4* src = (i < kStepGranules) ? k : v;
      stage[j] = src[g];
    }
  };
  // park the staged step in LDS buffer `buf` (page-sized halves, each swizzled on its own);
  // the step of the tile's own tokens also goes to the sequence's pages (slots past the end
  // of the sequence are left alone)
  auto park = [&](u32x4 (&stage)[kStage], int step, int buf, auto may_own) __attribute__((always_inline)) {
    const bool own = decltype(may_own)::value && step == tile;
#pragma unroll
    for (int j = 0; j < kStage; ++j) {
      const int i = tid + j * kThreads;
      const int gi = i & (kStepGranules - 1), sub = gi >> 8, tok = (gi >> 4) & 15, c = gi & 15;
      const bool live = own && step * kStepTok + sub * kP + tok < len;
      // (the table entry of a page past the sequence's last one is never read)
      const size_t page =
          own ? (static_cast<size_t>(bt[min(kSubs * step + sub, last_page)]) * Hkv + kvh) * kPageGranules : 0;
      if (i < kStepGranules) {
        lds_k[buf][sub * kPageGranules + swz_k(tok, c)] = stage[j];
        if (live) k_cache[page + (gi & (kPageGranules - 1))] = stage[j];
      } else {
        lds_v[buf][sub * kPageGranules + swz_v(tok, c)] = stage[j];
        if (live) v_cache[page + (gi & (kPageGranules - 1))] = stage[j];
      }
    }
  };

  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.0f, 0.0f};
  f32x4 o[2][8];
#pragma unroll
  for (int i = 0; i < 16; ++i) o[i >> 3][i & 7] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

  fetch(stage_a, 0);
  fetch(stage_b, 1);
  park(stage_a, 0, 0, std::true_type{});
  __syncthreads();

  // one step; `cur` holds the rows of step+1 (fetched a step ago), `nxt` is free and takes
  // the fetch of step+2 (unconditional: a fetch past the end stays in bounds and is dropped)
  // diag = false: a step strictly before the tile's own tokens whose successor is not the
  // tile's own step either (no mask, no page write, and the step after it exists)
  auto do_step = [&](u32x4 (&cur)[kStage], u32x4 (&nxt)[kStage], const int step, auto diag) __attribute__((always_inline)) {
    constexpr bool kDiag = decltype(diag)::value;
    const int buf = step & 1;
    fetch(nxt, step + 2);

    if (computes) {
      const bool tail = kDiag && step * kStepTok + kStepTok > len;  // tokens past the end of the sequence
      // Scores of the two pages: K rows as the A operand (token = lane & 15), read once for
      // both query blocks.  This lane: query n of each block, tokens 4*bq .. 4*bq+3 of each page.
      // A block whose queries all lie before a page's tokens is fully masked there: its
      // weights are exp2(-inf - m) = 0 (m is finite from step 0 on: token 0 is visible to
      // every query).
      float t[kSubs][2][4];
#pragma unroll
      for (int sub = 0; sub < kSubs; ++sub) {
        if (sub > 0) __builtin_amdgcn_sched_barrier(0);   // (one page's K operands in registers at a time)
        bf16x8 kf[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
          kf[kk] = __builtin_bit_cast(bf16x8, lds_k[buf][sub * kPageGranules + swz_k(n, 4 * kk + bq)]);
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          f32x4 sc = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
          for (int kk = 0; kk < 4; ++kk)
            sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kk], qf[nb][kk], sc, 0, 0, 0);
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) t[sub][nb][rr] = sc[rr];   // raw: the scale rides on the exponent's fma
        }
      }
      if (kDiag && (step == tile || tail)) {           // the tile's own step, or one at the end
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
      // V^T as the A operand through the transposing read (per page the lane gets rows
      // 4*bq + n/4 .. of columns 16*dt + 4*(n%4) .. +3): the two pages' halves side by side.
      // (Read only now: held across the scores and the softmax the V operands would not fit
      // in the register file beside the two staging sets.)
      __builtin_amdgcn_sched_barrier(0);
      {
        const int vrow = 4 * bq + (n >> 2);
        const char* vbase = reinterpret_cast<const char*>(lds_v[buf]) + (n & 1) * 8;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
          const char* addr = vbase + swz_v(vrow, 2 * dt + ((n & 3) >> 1)) * 16;
          const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(addr));
          const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4*)(addr + kPageGranules * 16));
          const s16x8 vv = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
          const bf16x8 vf = __builtin_bit_cast(bf16x8, vv);
          o[0][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[0], o[0][dt], 0, 0, 0);
          o[1][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[1], o[1][dt], 0, 0, 0);
        }
      }
    }
    // park step+1; that LDS buffer was last read one step ago
    if (kDiag) {
      if (step < last_step) park(cur, step + 1, buf ^ 1, std::true_type{});
    } else {
      park(cur, step + 1, buf ^ 1, std::false_type{});
    }
    __syncthreads();
  };
  int step = 0;
  for (; step + 2 <= tile - 1; step += 2) {       // pairs of steps well before the tile's own
    do_step(stage_b, stage_a, step, std::false_type{});
    do_step(stage_a, stage_b, step + 1, std::false_type{});
  }
  for (; step <= last_step; ++step) {             // the last one to three steps, one code copy:
    do_step(stage_b, stage_a, step, std::true_type{});
#pragma unroll
    for (int j = 0; j < kStage; ++j) {            // the two staging sets trade places
      const u32x4 x = stage_a[j];
      stage_a[j] = stage_b[j];
      stage_b[j] = x;
    }
  }

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
  const dim3 grid((max_seqlen + kTileQ - 1) / kTileQ, Hkv, B);
  const float scale_log2e = scale * kLog2e;
#define COPRIS_PREFILL(G)                                                                        \
  hipLaunchKernelGGL(prefill_attn_kernel<G>, grid, dim3(PrefillThreads<G>::value), 0, stream,    \
                     static_cast<const uint16_t*>(q), static_cast<const u32x4*>(k),              \
                     static_cast<const u32x4*>(v), cu_seqlens, block_table,                      \
                     static_cast<u32x4*>(k_cache), static_cast<u32x4*>(v_cache),                 \
                     static_cast<uint16_t*>(out), lse, Hq, Hkv, max_pages, scale_log2e)
  COPRIS_PRE("prefill_attn_kernel");
  switch (g) {
    case 1: COPRIS_PREFILL(1); break;
    case 2: COPRIS_PREFILL(2); break;
    case 3: COPRIS_PREFILL(3); break;
    case 4: COPRIS_PREFILL(4); break;
    case 5: COPRIS_PREFILL(5); break;
    case 6: COPRIS_PREFILL(6); break;
    case 7: COPRIS_PREFILL(7); break;
    default: COPRIS_PREFILL(8); break;
  }
#undef COPRIS_PREFILL
  COPRIS_POST("prefill_attn_kernel");
  return 0;
}

}  // namespace copris
