// Paged-KV grouped-query decode attention for gfx950, split along the context.
//
// Tuned path (bf16, head_dim 128, page 16): the (kv head, page) slabs of the whole pool
// are laid out as ONE flat sequence of "slots" (sequence-major, then kv head, then page)
// and cut into equal contiguous shares, one per persistent wavefront ("stream-K"): the
// split is balanced to one page whatever the length distribution, a 32k-token resumed
// trajectory is simply spread over many wavefronts, and nothing is scheduled at run time.
//   split kernel   one wavefront per share.  It first derives its own start cursor
//                  (sequence, kv head, page) from ctx_len with one wave-level prefix sum
//                  (no separate pass over ctx_len, no extra launch), then walks its slots
//                  with a wave-uniform cursor (physical pages from the block table, one
//                  slot ahead) and a three-page-deep register prefetch.  Whenever the
//                  (sequence, kv head) segment changes: a segment that lies wholly inside
//                  the share is normalised and stored to `out` right there; one that a
//                  share boundary cuts leaves its online-softmax partial (running max,
//                  weight sum, weighted value sum of the g query heads of the kv head)
//   merge kernel   per (sequence, kv head) that a boundary cuts: log-sum-exp combination
//                  of the partials in share order, normalisation, store; it also writes
//                  the zeros of empty sequences
// (For more than 4096 sequences a one-workgroup scan kernel computes the cursors first.)
// The partition depends on ctx_len only, the merge order is fixed: results are bitwise
// reproducible and do not depend on the physical page order.
//
// The split kernel keeps the kernel HBM-bound by doing both contractions on the matrix
// cores with the TOKENS (scores) or the head dimension (values) as the 16-row M side and
// the 16-padded group of query heads as the N side:
//     S^T[token][head] = K_page[token][:] . Q[head][:]          4 x mfma 16x16x32
//     O^T[d][head]    += V_page^T[d][token] . P^T[token][head]  8 x mfma 16x16x16
// With that orientation the score tile leaves the first product already in the register
// layout the second one wants for P^T, and every per-head softmax quantity (max, sum,
// rescale factor) lives in the lane that owns the head.  A (page, kv head) slab is one
// contiguous 4 KB run: it is fetched with fully coalesced 16-byte loads, parked in LDS
// with an XOR swizzle, and read back in MFMA operand layout (V through the transposing
// LDS read).
//
// Generic path (fp32, other head_dim / page sizes): a list of (sequence, 512-token chunk)
// items, one workgroup per (item, kv head) on the vector ALU, same partial format.
#include <type_traits>

#include "copris_device.h"
#include "copris_internal.h"

namespace copris {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// --------------------------------------------------------------------------
// workspace
// --------------------------------------------------------------------------
static inline size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

AttnWorkspace attn_workspace_layout(int C, int Hq, int Hkv, int D, int page_size, int max_pages) {
  AttnWorkspace w{};
  const int g = Hq / Hkv;
  const int64_t max_tokens = static_cast<int64_t>(max_pages) * page_size;
  const int64_t chunks = (max_tokens + kAttnChunkTokens - 1) / kAttnChunkTokens;
  w.max_list = static_cast<int64_t>(C) * (chunks > 0 ? chunks : 1);
  // list: (seq, chunk) items of the generic path, or one int4 start cursor per wavefront of
  // the tuned path
  const int64_t list_len = w.max_list > 2 * kAttnWaves ? w.max_list : 2 * kAttnWaves;
  // partials: one per (item, kv head), or one per (wavefront, segment) overlap
  const int64_t part_a = w.max_list * Hkv;
  const int64_t part_b = static_cast<int64_t>(kAttnWaves) + static_cast<int64_t>(C) * Hkv;
  const int64_t parts = part_a > part_b ? part_a : part_b;
  size_t off = 0;
  w.hdr = off;      off = align256(off + 64 * sizeof(int32_t));
  w.seq_off = off;  off = align256(off + (static_cast<size_t>(C) + 1) * sizeof(int32_t));
  w.list = off;     off = align256(off + static_cast<size_t>(list_len) * sizeof(int2));
  w.ml = off;       off = align256(off + static_cast<size_t>(parts) * g * sizeof(float2));
  w.acc = off;      off = align256(off + static_cast<size_t>(parts) * g * D * sizeof(float));
  w.total = off;
  return w;
}

// --------------------------------------------------------------------------
// a1: work list.  One workgroup; sequences in blocks of 1024 with a carried offset.
// --------------------------------------------------------------------------
constexpr int kListThreads = 1024;

__global__ __launch_bounds__(kListThreads) void attn_worklist_kernel(
    const int32_t* __restrict__ ctx_len, int C, int max_tokens, int32_t* __restrict__ hdr,
    int32_t* __restrict__ seq_off, int2* __restrict__ list) {
  __shared__ int s_wave[kListThreads / kWave];
  __shared__ int s_carry;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  if (tid == 0) s_carry = 0;
  __syncthreads();
  for (int base = 0; base < C; base += kListThreads) {
    const int i = base + tid;
    int n = i < C ? ctx_len[i] : 0;
    n = n < 0 ? 0 : (n > max_tokens ? max_tokens : n);
    const int nch = (n + kAttnChunkTokens - 1) / kAttnChunkTokens;
    int incl = nch;   // inclusive scan inside the wave
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const int up = __shfl_up(incl, o, kWave);
      if (lane >= o) incl += up;
    }
    if (lane == kWave - 1) s_wave[wave] = incl;
    __syncthreads();
    int before = s_carry;
    for (int w = 0; w < wave; ++w) before += s_wave[w];
    const int excl = before + incl - nch;
    if (i < C) {
      seq_off[i] = excl;
      for (int c = 0; c < nch; ++c) list[excl + c] = make_int2(i, c);
    }
    __syncthreads();
    if (tid == kListThreads - 1) s_carry = before + incl;
    __syncthreads();
  }
  if (tid == 0) {
    seq_off[C] = s_carry;
    hdr[0] = s_carry;
    hdr[1] = 0;
  }
}

// --------------------------------------------------------------------------
// a2 (generic): fp32 or bf16, any head_dim in {64,128}, any page size.  One
// workgroup of 256 threads per (entry, kv head); tokens in tiles of 256.
// --------------------------------------------------------------------------
template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
};
template <> struct Elem<uint16_t> {
  static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_to_f32(*p); }
};

template <typename T, int D>
__global__ __launch_bounds__(256) void attn_split_generic_kernel(
    const T* __restrict__ q, const T* __restrict__ k_cache, const T* __restrict__ v_cache,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ ctx_len,
    const int32_t* __restrict__ hdr, const int2* __restrict__ list, float2* __restrict__ ws_ml,
    float* __restrict__ ws_acc, int Hq, int Hkv, int g, int page_size, int max_pages,
    int max_tokens, float scale_log2e) {
  constexpr int NT = 256;
  constexpr int NP = NT / D;                 // token-parallel parts in the value pass
  __shared__ float s_q[kAttnMaxGroup][D];
  __shared__ float s_p[kAttnMaxGroup * NT];  // weights of the tile; reused for the part sums
  __shared__ float s_red[kAttnMaxGroup][NT / kWave];
  const int item = blockIdx.x;
  if (item >= hdr[0] * Hkv) return;
  const int li = item / Hkv, kvh = item - li * Hkv;
  const int seq = list[li].x, chunk = list[li].y;
  int n = ctx_len[seq];
  n = n > max_tokens ? max_tokens : n;
  const int t0 = chunk * kAttnChunkTokens;
  const int t1 = min(n, t0 + kAttnChunkTokens);
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;

  for (int e = tid; e < g * D; e += NT)
    s_q[e / D][e % D] = Elem<T>::load(q + (static_cast<size_t>(seq) * Hq + kvh * g) * D + e);
  __syncthreads();

  float m_run[kAttnMaxGroup], l_run[kAttnMaxGroup], acc[kAttnMaxGroup];
#pragma unroll
  for (int h = 0; h < kAttnMaxGroup; ++h) { m_run[h] = -INFINITY; l_run[h] = 0.0f; acc[h] = 0.0f; }
  const int d_own = tid % D, part = tid / D;
  const int32_t* bt = block_table + static_cast<size_t>(seq) * max_pages;

  for (int ts = t0; ts < t1; ts += NT) {
    const int tt = ts + tid;
    const bool valid = tt < t1;
    float s[kAttnMaxGroup];
#pragma unroll
    for (int h = 0; h < kAttnMaxGroup; ++h) s[h] = 0.0f;
    if (valid) {
      const int page = bt[tt / page_size], slot = tt % page_size;
      const T* krow = k_cache + ((static_cast<size_t>(page) * Hkv + kvh) * page_size + slot) * D;
      for (int d = 0; d < D; ++d) {
        const float kv = Elem<T>::load(krow + d);
#pragma unroll
        for (int h = 0; h < kAttnMaxGroup; ++h)
          if (h < g) s[h] = fmaf(s_q[h][d], kv, s[h]);
      }
    }
#pragma unroll
    for (int h = 0; h < kAttnMaxGroup; ++h) {
      if (h < g) {
        s[h] = valid ? s[h] * scale_log2e : -INFINITY;
        const float wm = wave_max(s[h]);
        if (lane == 0) s_red[h][wave] = wm;
      }
    }
    __syncthreads();
    float alpha[kAttnMaxGroup];
#pragma unroll
    for (int h = 0; h < kAttnMaxGroup; ++h) {
      alpha[h] = 1.0f;
      if (h < g) {
        float mt = s_red[h][0];
#pragma unroll
        for (int w = 1; w < NT / kWave; ++w) mt = fmaxf(mt, s_red[h][w]);
        const float m_new = fmaxf(m_run[h], mt);
        alpha[h] = __builtin_amdgcn_exp2f(m_run[h] - m_new);
        m_run[h] = m_new;
        const float p = valid ? __builtin_amdgcn_exp2f(s[h] - m_new) : 0.0f;
        s_p[h * NT + tid] = p;
        s[h] = p;
      }
    }
    __syncthreads();   // s_red consumed, s_p complete
#pragma unroll
    for (int h = 0; h < kAttnMaxGroup; ++h) {
      if (h < g) {
        const float ws = wave_sum(s[h]);
        if (lane == 0) s_red[h][wave] = ws;
      }
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < kAttnMaxGroup; ++h) {
      if (h < g) {
        float lt = s_red[h][0];
#pragma unroll
        for (int w = 1; w < NT / kWave; ++w) lt += s_red[h][w];
        l_run[h] = l_run[h] * alpha[h] + lt;
        acc[h] *= alpha[h];
      }
    }
    const int ntile = min(NT, t1 - ts);
    for (int t2 = part; t2 < ntile; t2 += NP) {
      const int tok = ts + t2;
      const int page = bt[tok / page_size], slot = tok % page_size;
      const float vv = Elem<T>::load(
          v_cache + ((static_cast<size_t>(page) * Hkv + kvh) * page_size + slot) * D + d_own);
#pragma unroll
      for (int h = 0; h < kAttnMaxGroup; ++h)
        if (h < g) acc[h] = fmaf(s_p[h * NT + t2], vv, acc[h]);
    }
    __syncthreads();   // before the next tile overwrites s_p / s_red
  }

  // sum the token-parallel parts in a fixed order: s_p viewed as [NP][16][D]
#pragma unroll
  for (int h = 0; h < kAttnMaxGroup; ++h)
    if (h < g) s_p[(part * kAttnMaxGroup + h) * D + d_own] = acc[h];
  __syncthreads();
  if (part == 0) {
#pragma unroll
    for (int h = 0; h < kAttnMaxGroup; ++h) {
      if (h < g) {
        float a = 0.0f;
#pragma unroll
        for (int pp = 0; pp < NP; ++pp) a += s_p[(pp * kAttnMaxGroup + h) * D + d_own];
        ws_acc[(static_cast<size_t>(item) * g + h) * D + d_own] = a;
      }
    }
  }
  if (tid == 0) {
#pragma unroll
    for (int h = 0; h < kAttnMaxGroup; ++h)
      if (h < g) ws_ml[static_cast<size_t>(item) * g + h] = make_float2(m_run[h], l_run[h]);
  }
}

// --------------------------------------------------------------------------
// a1/a2 (tuned): bf16, head_dim 128, page 16, g <= 16, flat slot stream.
// --------------------------------------------------------------------------
constexpr int kD = 128;
constexpr int kP = 16;
constexpr int kPageGranules = kP * kD * 2 / 16;   // 256 16-byte granules per (page, kv head)

// The slot stream: for every sequence in batch order, for every kv head, the pages of the
// context in order; one slot = one (page, kv head) = 16 tokens x 128 dims of K and of V.
// Wavefront w of the split kernel takes the slots [w*share, (w+1)*share).
// This kernel (one workgroup) writes
//   seq_pg[i] = pages of the sequences before i (seq_pg[C] = all pages),
//   hdr[0] = slots in total, hdr[1] = share,
//   start[w] = {sequence, kv head, page index, pages of that sequence} of slot w*share
//              (sequence = -1: no slots for this wavefront).
__global__ __launch_bounds__(kListThreads) void attn_scan_kernel(
    const int32_t* __restrict__ ctx_len, int C, int max_tokens, int Hkv, int32_t* __restrict__ hdr,
    int32_t* __restrict__ seq_pg, int4* __restrict__ start) {
  __shared__ int s_wave[kListThreads / kWave];
  __shared__ int s_carry;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  if (tid == 0) s_carry = 0;
  __syncthreads();
  for (int base = 0; base < C; base += kListThreads) {
    const int i = base + tid;
    int n = i < C ? ctx_len[i] : 0;
    n = n < 0 ? 0 : (n > max_tokens ? max_tokens : n);
    const int npg = (n + kP - 1) / kP;
    int incl = npg;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const int up = __shfl_up(incl, o, kWave);
      if (lane >= o) incl += up;
    }
    if (lane == kWave - 1) s_wave[wave] = incl;
    __syncthreads();
    int before = s_carry;
    for (int w = 0; w < wave; ++w) before += s_wave[w];
    if (i < C) seq_pg[i] = before + incl - npg;
    __syncthreads();
    if (tid == kListThreads - 1) s_carry = before + incl;
    __syncthreads();
  }
  const int pages = s_carry;
  const int total = pages * Hkv;
  const int share = total > 0 ? (total + kAttnWaves - 1) / kAttnWaves : 1;
  if (tid == 0) {
    seq_pg[C] = pages;
    hdr[0] = total;
    hdr[1] = share;
  }
  __syncthreads();   // seq_pg[] (written above by this workgroup) is read below
  for (int w = tid; w < kAttnWaves; w += kListThreads) {
    const int64_t slot = static_cast<int64_t>(w) * share;
    int4 st = make_int4(-1, 0, 0, 0);
    if (slot < total) {
      // the last sequence whose first slot is <= slot (empty sequences share their
      // successor's first slot and are skipped by taking the last)
      int lo = 0, hi = C - 1;
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (static_cast<int64_t>(seq_pg[mid]) * Hkv <= slot) lo = mid; else hi = mid - 1;
      }
      const int pg0 = seq_pg[lo];
      const int npg = (lo + 1 < C ? seq_pg[lo + 1] : pages) - pg0;
      const int r = static_cast<int>(slot - static_cast<int64_t>(pg0) * Hkv);
      st = make_int4(lo, r / npg, r % npg, npg);
    }
    start[w] = st;
  }
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  uint32_t r;
  asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(lo), "v"(hi));
  return r;
}

struct PageRegs {
  u32x4 k[4];
  u32x4 v[4];
};

__device__ __forceinline__ void load_page(PageRegs& r, const u32x4* __restrict__ kc,
                                          const u32x4* __restrict__ vc, int page, int Hkv, int kvh,
                                          int lane) {
  const size_t base = (static_cast<size_t>(page) * Hkv + kvh) * kPageGranules + lane;
  // non-temporal: every K / V byte is read once per call, and keeping the stream out of the
  // L2 leaves it to the block table, the queries and the partials (measured: the split kernel
  // 0.336 -> 0.305 ms at the 7B-shaped step)
#pragma unroll
  for (int i = 0; i < 4; ++i) r.k[i] = __builtin_nontemporal_load(kc + base + i * 64);
#pragma unroll
  for (int i = 0; i < 4; ++i) r.v[i] = __builtin_nontemporal_load(vc + base + i * 64);
}

// LDS position (in 16-byte granules) of granule c of token row `row`.
__device__ __forceinline__ int swz_k(int row, int c) { return row * 16 + (c ^ (row & 15)); }
__device__ __forceinline__ int swz_v(int row, int c) { return row * 16 + (c ^ ((row & 7) << 1)); }

// s_waitcnt vmcnt(0) with the other counters left alone (gfx9 encoding)
#define COPRIS_WAIT_VM0() __builtin_amdgcn_s_waitcnt(0x0F70)

// Pages of sequence i as the kernels count them.
__device__ __forceinline__ int attn_pages_of(const int32_t* __restrict__ ctx_len, int i, int max_tokens) {
  const int n = min(max(ctx_len[i], 0), max_tokens);
  return (n + kP - 1) / kP;
}

// One wavefront: total pages of the pool and the start cursor of slot `w * share` of the
// slot stream, from ctx_len alone.  Lane l owns the sequences [l*chunk, (l+1)*chunk); an
// inclusive prefix sum over the lanes gives the pages before each lane's range; the one
// lane whose range holds the slot walks its (at most `chunk`) sequences.  Returns the
// cursor in every lane ({-1,..}: no slot for this wavefront) and total / share by reference.
__device__ __forceinline__ int4 attn_derive_cursor(const int32_t* __restrict__ ctx_len, int C,
                                                   int max_tokens, int Hkv, int w, int& total,
                                                   int& share) {
  const int lane = threadIdx.x & (kWave - 1);
  const int chunk = (C + kWave - 1) / kWave;
  const int i0 = min(lane * chunk, C), i1 = min(i0 + chunk, C);
  // up to 8 sequences per lane (C <= 512) stay in registers, so that the walk below costs
  // no second round trip to memory
  constexpr int kReg = 8;
  int reg[kReg];
  int mine = 0;
  if (chunk <= kReg) {
#pragma unroll
    for (int j = 0; j < kReg; ++j) {
      reg[j] = i0 + j < i1 ? attn_pages_of(ctx_len, i0 + j, max_tokens) : 0;
      mine += reg[j];
    }
  } else {
    for (int i = i0; i < i1; ++i) mine += attn_pages_of(ctx_len, i, max_tokens);
  }
  int incl = mine;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int up = __shfl_up(incl, o, kWave);
    if (lane >= o) incl += up;
  }
  const int pages = __shfl(incl, kWave - 1, kWave);
  total = pages * Hkv;
  share = total > 0 ? (total + kAttnWaves - 1) / kAttnWaves : 1;
  const int64_t slot = static_cast<int64_t>(w) * share;
  int4 st = make_int4(-1, 0, 0, 0);
  if (slot >= total) return st;
  const int64_t before = static_cast<int64_t>(incl - mine) * Hkv;     // slots before this lane's range
  const bool holds = before <= slot && slot < before + static_cast<int64_t>(mine) * Hkv;
  const uint64_t ball = __builtin_amdgcn_ballot_w64(holds);            // exactly one lane
  const int owner = __builtin_ctzll(ball);
  if (holds) {
    int64_t pg0 = incl - mine;
    if (chunk <= kReg) {
      bool found = false;
#pragma unroll
      for (int j = 0; j < kReg; ++j) {
        const int npg = reg[j];
        if (!found && slot < (pg0 + npg) * Hkv) {
          const int r = static_cast<int>(slot - pg0 * Hkv);
          st = make_int4(i0 + j, r / npg, r % npg, npg);
          found = true;
        }
        pg0 += found ? 0 : npg;
      }
    } else {
      for (int i = i0; i < i1; ++i) {
        const int npg = attn_pages_of(ctx_len, i, max_tokens);
        if (slot < (pg0 + npg) * Hkv) {
          const int r = static_cast<int>(slot - pg0 * Hkv);
          st = make_int4(i, r / npg, r % npg, npg);
          break;
        }
        pg0 += npg;
      }
    }
  }
  st.x = __shfl(st.x, owner, kWave);
  st.y = __shfl(st.y, owner, kWave);
  st.z = __shfl(st.z, owner, kWave);
  st.w = __shfl(st.w, owner, kWave);
  return st;
}

// entry word of a slot: tokens of the page inside the context - 1 (4 bits), first / last
// page of its (sequence, kv head) segment (1 + 1), kv head (8), sequence (17)
constexpr int kCodeFirst = 1 << 4, kCodeLast = 1 << 5, kCodeKvhShift = 6, kCodeSeqShift = 14;
constexpr int kAttnMaxSeqTuned = 1 << 17;
constexpr int kAttnMaxSeqInKernelCursor = 4096;

template <int NS, bool PRESCAN>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_split_flat_kernel(
    const uint16_t* __restrict__ q, const u32x4* __restrict__ k_cache,
    const u32x4* __restrict__ v_cache, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ ctx_len, const int32_t* __restrict__ hdr,
    const int4* __restrict__ start, float2* __restrict__ ws_ml, float* __restrict__ ws_acc,
    uint16_t* __restrict__ out, float* __restrict__ lse, int C, int Hq, int Hkv, int g,
    int max_pages, int max_tokens, float scale_log2e) {
  __shared__ u32x4 lds_k[kPageGranules];
  __shared__ u32x4 lds_v[kPageGranules];
  const int lane = threadIdx.x;
  const int head = lane & 15;     // N index of both products: the query head of the group
  const int b = lane >> 4;        // k-group of the MFMA operand layouts
  const int wv = blockIdx.x;
  int total, share;
  int4 st;
  if (PRESCAN) {
    total = hdr[0];
    share = hdr[1];
    st = start[wv];
  } else {
    st = attn_derive_cursor(ctx_len, C, max_tokens, Hkv, wv, total, share);
    st.x = __builtin_amdgcn_readfirstlane(st.x);
    st.y = __builtin_amdgcn_readfirstlane(st.y);
    st.z = __builtin_amdgcn_readfirstlane(st.z);
    st.w = __builtin_amdgcn_readfirstlane(st.w);
    total = __builtin_amdgcn_readfirstlane(total);
    share = __builtin_amdgcn_readfirstlane(share);
  }
  if (st.x < 0) return;
  const int64_t first = static_cast<int64_t>(wv) * share;
  const int n = static_cast<int>(min(static_cast<int64_t>(share), total - first));   // slots of this wavefront

  // Fetch cursor over the slot stream (all wave-uniform): the next slot to request is page
  // f_p of (sequence f_seq, kv head f_kvh); f_page is its physical page, read one slot ahead
  // so that the table look-up is off the refill's path.
  int f_seq = st.x, f_kvh = st.y, f_p = st.z, f_npg = st.w;
  int f_ctx = min(max(ctx_len[f_seq], 0), max_tokens);
  int f_page = block_table[static_cast<size_t>(f_seq) * max_pages + f_p];
  auto next_entry = [&](int& page, int& code) __attribute__((always_inline)) {
    page = f_page;
    code = (min(kP, f_ctx - f_p * kP) - 1) | (f_p == 0 ? kCodeFirst : 0) |
           (f_p + 1 == f_npg ? kCodeLast : 0) | (f_kvh << kCodeKvhShift) | (f_seq << kCodeSeqShift);
    if (++f_p == f_npg) {
      f_p = 0;
      if (++f_kvh == Hkv) {   // on to the next sequence that has a context
        f_kvh = 0;
        f_npg = 0;
        while (f_npg == 0 && ++f_seq < C) {
          f_ctx = min(max(ctx_len[f_seq], 0), max_tokens);
          f_npg = (f_ctx + kP - 1) / kP;
        }
      }
    }
    f_page = f_seq < C ? block_table[static_cast<size_t>(f_seq) * max_pages + f_p] : 0;
  };

  // state of the segment (sequence, kv head) being accumulated
  int cur_seg = -1;
  bf16x8 qf[4];
  float m_run = -INFINITY, l_run = 0.0f;
  f32x4 o[8];

  bool seg_whole = false;   // the segment began with its first page inside this share
  bool seg_ends = false;    // the slot just processed was the segment's last page
  auto flush = [&]() __attribute__((always_inline)) {   // result of (this wavefront, cur_seg)
    float l_all = l_run;
    l_all += __shfl_xor(l_all, 16, kWave);
    l_all += __shfl_xor(l_all, 32, kWave);
    if (seg_whole && seg_ends) {
      // no other wavefront saw this segment: normalise and store (lane (head, b) owns
      // d = 16dt + 4b + r); same arithmetic as the merge of a single partial
      if (head < g) {
        const int seq = cur_seg / Hkv, kvh = cur_seg - seq * Hkv;
        const size_t oh = static_cast<size_t>(seq) * Hq + kvh * g + head;
        uint16_t* dst = out + oh * kD + 4 * b;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
          ushort4 r;
          r.x = f32_to_bf16(o[dt][0] / l_all);
          r.y = f32_to_bf16(o[dt][1] / l_all);
          r.z = f32_to_bf16(o[dt][2] / l_all);
          r.w = f32_to_bf16(o[dt][3] / l_all);
          *reinterpret_cast<ushort4*>(dst + 16 * dt) = r;
        }
        if (lse != nullptr && b == 0) lse[oh] = (m_run + __builtin_amdgcn_logf(l_all)) * kLn2;
      }
      return;
    }
    if (head < g) {
      const size_t slot = (static_cast<size_t>(wv) + cur_seg) * g + head;
      float* dst = ws_acc + slot * kD + 4 * b;    // lane (head, b) owns d = 16dt + 4b + r
#pragma unroll
      for (int dt = 0; dt < 8; ++dt)
        *reinterpret_cast<float4*>(dst + 16 * dt) = make_float4(o[dt][0], o[dt][1], o[dt][2], o[dt][3]);
      if (b == 0) ws_ml[slot] = make_float2(m_run, l_all);
    }
  };
  auto begin_segment = [&](const int seq, const int kvh) __attribute__((always_inline)) {
    cur_seg = seq * Hkv + kvh;
    // Q^T operand: lane (head, b) holds Q[head][32*kk + 8*b .. +8]; padded heads are zero
    const u32x4* qrow =
        reinterpret_cast<const u32x4*>(q + (static_cast<size_t>(seq) * Hq + kvh * g + head) * kD);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      u32x4 x = {0u, 0u, 0u, 0u};
      if (head < g) x = qrow[kk * 4 + b];
      qf[kk] = __builtin_bit_cast(bf16x8, x);
    }
    // complete these loads here (rare path) so that the common path never has to wait
    // for anything younger than its own page prefetches
    COPRIS_WAIT_VM0();
    m_run = -INFINITY;
    l_run = 0.0f;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) o[dt] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  };

  // One slot: park its page in LDS, refill the registers with the page NS slots ahead,
  // then both products.  `code` is the slot's entry word (wave-uniform).
  // steady: the slot NS ahead exists, so the refill is unconditional (which lets the
  // compiler count outstanding loads exactly and keep the younger stages in flight).
  auto do_slot = [&](PageRegs& r, int& code, const int i, auto steady) __attribute__((always_inline)) {
    constexpr bool kSteady = decltype(steady)::value;
    const int valid = (code & 15) + 1;           // tokens of this page inside the context
    const int kvh = (code >> kCodeKvhShift) & 255, seq = code >> kCodeSeqShift;
    if (seq * Hkv + kvh != cur_seg) {
      if (cur_seg >= 0) flush();
      begin_segment(seq, kvh);
      seg_whole = (code & kCodeFirst) != 0;     // ... so far: it starts inside this share
    }
    seg_ends = (code & kCodeLast) != 0;
    // granule (j*64+lane) = token row 4j+b, column granule `head`
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      lds_k[swz_k(4 * j + b, head)] = r.k[j];
      lds_v[swz_v(4 * j + b, head)] = r.v[j];
    }
    if (kSteady || i + NS < n) {
      int page;
      next_entry(page, code);
      load_page(r, k_cache, v_cache, page, Hkv, (code >> kCodeKvhShift) & 255, lane);
    }
    __syncthreads();
#if defined(COPRIS_ATTN_PROBE_NO_COMPUTE)
    // timing probe: the page is fetched and parked, nothing is computed from it
    {
      const u32x4 kk0 = lds_k[lane];
      const u32x4 vv0 = lds_v[lane];
      l_run += __uint_as_float((kk0[0] ^ vv0[1]) & 0x3fffffffu);
      (void)valid;
      __syncthreads();
      return;
    }
#endif

    // S^T[token][head]: A = K rows (token = lane&15), B = Q^T
    f32x4 sc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const bf16x8 kf = __builtin_bit_cast(bf16x8, lds_k[swz_k(head, 4 * kk + b)]);
      sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[kk], sc, 0, 0, 0);
    }
    // this lane: head `head`, tokens 4b..4b+3 of the page
    float t[4];
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) t[rr] = sc[rr] * scale_log2e;
    if (valid < kP) {
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) t[rr] = (4 * b + rr < valid) ? t[rr] : -INFINITY;
    }
    float mx = fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3]));
    mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    float p[4];
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) p[rr] = __builtin_amdgcn_exp2f(t[rr] - m_new);
    l_run = l_run * alpha + ((p[0] + p[1]) + (p[2] + p[3]));
    const uint2 pk = make_uint2(pack_bf16x2(p[0], p[1]), pack_bf16x2(p[2], p[3]));
    const s16x4 pf = __builtin_bit_cast(s16x4, pk);
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) o[dt] *= alpha;
    }
    // O^T[d][head] += V^T[d][token] P^T[token][head]: A = V^T via the transposing
    // read (lane supplies row 4b + L/4, columns 16dt + 4(L%4)..+3, L = lane&15)
    const int vrow = 4 * b + (head >> 2);
    const char* vbase = reinterpret_cast<const char*>(lds_v) + (head & 1) * 8;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
      const char* addr = vbase + swz_v(vrow, 2 * dt + ((head & 3) >> 1)) * 16;
      s16x4 vf = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(addr));
      if (valid < kP) {   // rows past the context may hold anything (NaN): zero them
#pragma unroll
        for (int rr = 0; rr < 4; ++rr)
          vf[rr] = (4 * b + rr < valid) ? vf[rr] : static_cast<short>(0);
      }
      o[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vf, pf, o[dt], 0, 0, 0);
    }
    __syncthreads();   // the next page may overwrite the LDS tiles
  };

  static_assert(NS == 3, "the page pipeline below is written out for three stages");
  PageRegs st0, st1, st2;
  int c0 = 0, c1 = 0, c2 = 0;   // entry words of the slots held in st0..st2
  int i = 0;
  {
    int page;
    next_entry(page, c0);
    load_page(st0, k_cache, v_cache, page, Hkv, (c0 >> kCodeKvhShift) & 255, lane);
  }
  if (n >= 2 * NS) {
    {
      int page;
      next_entry(page, c1);
      load_page(st1, k_cache, v_cache, page, Hkv, (c1 >> kCodeKvhShift) & 255, lane);
    }
    {
      int page;
      next_entry(page, c2);
      load_page(st2, k_cache, v_cache, page, Hkv, (c2 >> kCodeKvhShift) & 255, lane);
    }
    do {   // steady state: every refill exists
      do_slot(st0, c0, i, std::true_type{});
      do_slot(st1, c1, i + 1, std::true_type{});
      do_slot(st2, c2, i + 2, std::true_type{});
      i += NS;
    } while (i + 2 * NS <= n);
  } else {
    if (1 < n) {
      int page;
      next_entry(page, c1);
      load_page(st1, k_cache, v_cache, page, Hkv, (c1 >> kCodeKvhShift) & 255, lane);
    }
    if (2 < n) {
      int page;
      next_entry(page, c2);
      load_page(st2, k_cache, v_cache, page, Hkv, (c2 >> kCodeKvhShift) & 255, lane);
    }
  }
  for (; i < n; i += NS) {   // the last 3..5 slots of the share (or a short share)
    do_slot(st0, c0, i, std::false_type{});
    if (i + 1 < n) do_slot(st1, c1, i + 1, std::false_type{});
    if (i + 2 < n) do_slot(st2, c2, i + 2, std::false_type{});
  }
  flush();
}

// --------------------------------------------------------------------------
// a3: merge.  One workgroup per (sequence, query head), one thread per head_dim index.
// --------------------------------------------------------------------------
template <typename T> __device__ __forceinline__ void store_out(T* p, float v);
template <> __device__ __forceinline__ void store_out<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_out<uint16_t>(uint16_t* p, float v) { *p = f32_to_bf16(v); }

template <typename T>
__global__ void attn_merge_kernel(const int32_t* __restrict__ seq_off,
                                  const float2* __restrict__ ws_ml,
                                  const float* __restrict__ ws_acc, T* __restrict__ out,
                                  float* __restrict__ lse, int Hq, int Hkv, int g, int D) {
  // one workgroup per (sequence, query head); thread d owns one head_dim index
  const int seq = blockIdx.x, hq = blockIdx.y, d = threadIdx.x;
  const int kvh = hq / g, h = hq - kvh * g;
  const int e0 = seq_off[seq], e1 = seq_off[seq + 1];
  const size_t stride = static_cast<size_t>(Hkv) * g;          // slots per list entry
  const size_t slot0 = (static_cast<size_t>(e0) * Hkv + kvh) * g + h;
  const int n = e1 - e0;
  float m_star = -INFINITY;
  for (int e = 0; e < n; ++e) m_star = fmaxf(m_star, ws_ml[slot0 + e * stride].x);
  float denom = 0.0f, num = 0.0f;
  int e = 0;
  for (; e + 4 <= n; e += 4) {   // four chunks' loads in flight; summation order stays e = 0, 1, 2, ...
    float2 ml[4];
    float a[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t slot = slot0 + (e + u) * stride;
      ml[u] = ws_ml[slot];
      a[u] = ws_acc[slot * D + d];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float w = __builtin_amdgcn_exp2f(ml[u].x - m_star);
      denom = fmaf(w, ml[u].y, denom);
      num = fmaf(w, a[u], num);
    }
  }
  for (; e < n; ++e) {
    const size_t slot = slot0 + e * stride;
    const float2 ml = ws_ml[slot];
    const float w = __builtin_amdgcn_exp2f(ml.x - m_star);
    denom = fmaf(w, ml.y, denom);
    num = fmaf(w, ws_acc[slot * D + d], num);
  }
  const size_t oh = static_cast<size_t>(seq) * Hq + hq;
  store_out<T>(out + oh * D + d, n > 0 ? num / denom : 0.0f);
  if (lse != nullptr && d == 0)
    lse[oh] = n > 0 ? (m_star + __builtin_amdgcn_logf(denom)) * kLn2 : -INFINITY;
}

// Merge for the flat slot stream: segment (seq, kv head) occupies slots [a, a+npg) and was
// touched by the wavefronts a/share .. (a+npg-1)/share; the partial of (wavefront w,
// segment s) sits at index w + s.  A segment inside one share was stored by its wavefront
// already; an empty sequence gets its zeros here.
template <bool PRESCAN>
__global__ __launch_bounds__(256) void attn_merge_flat_kernel(const int32_t* __restrict__ ctx_len,
                                                              const int32_t* __restrict__ hdr,
                                                              const int32_t* __restrict__ seq_pg,
                                                              const float2* __restrict__ ws_ml,
                                                              const float* __restrict__ ws_acc,
                                                              uint16_t* __restrict__ out,
                                                              float* __restrict__ lse, int C, int Hq,
                                                              int Hkv, int g, int max_tokens) {
  // one workgroup per (sequence, kv head); a thread owns four head_dim indices of one head
  __shared__ int s_before[256 / kWave], s_all[256 / kWave];
  const int seq = blockIdx.x, kvh = blockIdx.y;
  int share, npg, pg0;
  if (PRESCAN) {
    share = hdr[1];
    pg0 = seq_pg[seq];
    npg = seq_pg[seq + 1] - pg0;
  } else {
    // pages before this sequence and in total, from ctx_len (the same counts the split
    // kernel's wavefronts derived their cursors from)
    int before = 0, all = 0;
    for (int i = threadIdx.x; i < C; i += 256) {
      const int pgs = attn_pages_of(ctx_len, i, max_tokens);
      all += pgs;
      before += i < seq ? pgs : 0;
    }
    before = wave_sum_i(before);
    all = wave_sum_i(all);
    if ((threadIdx.x & (kWave - 1)) == 0) {
      s_before[threadIdx.x / kWave] = before;
      s_all[threadIdx.x / kWave] = all;
    }
    __syncthreads();
    pg0 = 0;
    int pages = 0;
#pragma unroll
    for (int w = 0; w < 256 / kWave; ++w) {
      pg0 += s_before[w];
      pages += s_all[w];
    }
    const int total = pages * Hkv;
    share = total > 0 ? (total + kAttnWaves - 1) / kAttnWaves : 1;
    npg = attn_pages_of(ctx_len, seq, max_tokens);
  }
  const int64_t a = static_cast<int64_t>(pg0) * Hkv + static_cast<int64_t>(kvh) * npg;
  const int seg = seq * Hkv + kvh;
  const int w0 = npg > 0 ? static_cast<int>(a / share) : 0;
  const int n = npg > 0 ? static_cast<int>((a + npg - 1) / share) - w0 + 1 : 0;
  if (n == 1) return;   // stored by the one wavefront that saw it
  for (int idx = threadIdx.x; idx < g * (kD / 4); idx += 256) {
    const int h = idx / (kD / 4), d4 = idx - h * (kD / 4);
    const size_t slot0 = (static_cast<size_t>(w0) + seg) * g + h;   // consecutive wavefronts: stride g
    float m_star = -INFINITY;
    float denom = 0.0f;
    float4 num = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    constexpr int kFast = 6;
    if (n <= kFast) {
      // the usual case: all partials in flight at once (one round trip), then the same
      // arithmetic in the same order as the loop below
      float2 ml[kFast];
      float4 x[kFast];
#pragma unroll
      for (int e = 0; e < kFast; ++e) {
        const size_t slot = slot0 + static_cast<size_t>(e < n ? e : 0) * g;
        ml[e] = ws_ml[slot];
        x[e] = *reinterpret_cast<const float4*>(ws_acc + slot * kD + 4 * d4);
      }
#pragma unroll
      for (int e = 0; e < kFast; ++e)
        if (e < n) m_star = fmaxf(m_star, ml[e].x);
#pragma unroll
      for (int e = 0; e < kFast; ++e) {
        if (e < n) {
          const float w = __builtin_amdgcn_exp2f(ml[e].x - m_star);
          denom = fmaf(w, ml[e].y, denom);
          num.x = fmaf(w, x[e].x, num.x);
          num.y = fmaf(w, x[e].y, num.y);
          num.z = fmaf(w, x[e].z, num.z);
          num.w = fmaf(w, x[e].w, num.w);
        }
      }
    } else {
      for (int e = 0; e < n; ++e) m_star = fmaxf(m_star, ws_ml[slot0 + static_cast<size_t>(e) * g].x);
      for (int e = 0; e < n; ++e) {
        const size_t slot = slot0 + static_cast<size_t>(e) * g;
        const float2 ml = ws_ml[slot];
        const float4 x = *reinterpret_cast<const float4*>(ws_acc + slot * kD + 4 * d4);
        const float w = __builtin_amdgcn_exp2f(ml.x - m_star);
        denom = fmaf(w, ml.y, denom);
        num.x = fmaf(w, x.x, num.x);
        num.y = fmaf(w, x.y, num.y);
        num.z = fmaf(w, x.z, num.z);
        num.w = fmaf(w, x.w, num.w);
      }
    }
    const size_t oh = static_cast<size_t>(seq) * Hq + kvh * g + h;
    ushort4 r = make_ushort4(0, 0, 0, 0);
    if (n > 0) {
      r.x = f32_to_bf16(num.x / denom);
      r.y = f32_to_bf16(num.y / denom);
      r.z = f32_to_bf16(num.z / denom);
      r.w = f32_to_bf16(num.w / denom);
    }
    *reinterpret_cast<ushort4*>(out + oh * kD + 4 * d4) = r;
    if (lse != nullptr && d4 == 0)
      lse[oh] = n > 0 ? (m_star + __builtin_amdgcn_logf(denom)) * kLn2 : -INFINITY;
  }
}

// --------------------------------------------------------------------------
// host launcher
// --------------------------------------------------------------------------
int launch_decode_attn(const void* q, const void* k_cache, const void* v_cache,
                       const int32_t* block_table, const int32_t* ctx_len, void* out, float* lse,
                       void* workspace, int C, int Hq, int Hkv, int D, int page_size,
                       int max_pages, float scale, int dtype, hipStream_t stream) {
  const int g = Hq / Hkv;
  const AttnWorkspace w = attn_workspace_layout(C, Hq, Hkv, D, page_size, max_pages);
  char* ws = static_cast<char*>(workspace);
  int32_t* hdr = reinterpret_cast<int32_t*>(ws + w.hdr);
  int32_t* seq_off = reinterpret_cast<int32_t*>(ws + w.seq_off);
  int2* list = reinterpret_cast<int2*>(ws + w.list);
  float2* ws_ml = reinterpret_cast<float2*>(ws + w.ml);
  float* ws_acc = reinterpret_cast<float*>(ws + w.acc);
  const int64_t max_tokens64 = static_cast<int64_t>(max_pages) * page_size;
  const int max_tokens = static_cast<int>(max_tokens64);
  const float scale_log2e = scale * kLog2e;

  // the flat slot stream packs the kv head in 8 bits and the sequence in 17
  const bool tuned = dtype == 1 && D == kD && page_size == kP && Hkv <= 256 && C < kAttnMaxSeqTuned &&
                     static_cast<int64_t>(C) * max_pages * Hkv < (1ll << 31);
  if (tuned) {
    int4* start = reinterpret_cast<int4*>(list);   // kAttnWaves start cursors (the list area is larger)
    const bool prescan = C > kAttnMaxSeqInKernelCursor;
    if (prescan) {
      COPRIS_PRE("attn_scan_kernel");
      hipLaunchKernelGGL(attn_scan_kernel, dim3(1), dim3(kListThreads), 0, stream, ctx_len, C,
                         max_tokens, Hkv, hdr, seq_off, start);
      COPRIS_POST("attn_scan_kernel");
    }
    COPRIS_PRE("attn_split_flat_kernel");
    if (prescan) {
      hipLaunchKernelGGL((attn_split_flat_kernel<3, true>), dim3(kAttnWaves), dim3(64), 0, stream,
                         static_cast<const uint16_t*>(q), static_cast<const u32x4*>(k_cache),
                         static_cast<const u32x4*>(v_cache), block_table, ctx_len, hdr, start, ws_ml,
                         ws_acc, static_cast<uint16_t*>(out), lse, C, Hq, Hkv, g, max_pages, max_tokens,
                         scale_log2e);
    } else {
      hipLaunchKernelGGL((attn_split_flat_kernel<3, false>), dim3(kAttnWaves), dim3(64), 0, stream,
                         static_cast<const uint16_t*>(q), static_cast<const u32x4*>(k_cache),
                         static_cast<const u32x4*>(v_cache), block_table, ctx_len, hdr, start, ws_ml,
                         ws_acc, static_cast<uint16_t*>(out), lse, C, Hq, Hkv, g, max_pages, max_tokens,
                         scale_log2e);
    }
    COPRIS_POST("attn_split_flat_kernel");
    COPRIS_PRE("attn_merge_flat_kernel");
    if (prescan) {
      hipLaunchKernelGGL(attn_merge_flat_kernel<true>, dim3(C, Hkv), dim3(256), 0, stream, ctx_len, hdr,
                         seq_off, ws_ml, ws_acc, static_cast<uint16_t*>(out), lse, C, Hq, Hkv, g,
                         max_tokens);
    } else {
      hipLaunchKernelGGL(attn_merge_flat_kernel<false>, dim3(C, Hkv), dim3(256), 0, stream, ctx_len, hdr,
                         seq_off, ws_ml, ws_acc, static_cast<uint16_t*>(out), lse, C, Hq, Hkv, g,
                         max_tokens);
    }
    COPRIS_POST("attn_merge_flat_kernel");
    return 0;
  }

  COPRIS_PRE("attn_worklist_kernel");
  hipLaunchKernelGGL(attn_worklist_kernel, dim3(1), dim3(kListThreads), 0, stream, ctx_len, C,
                     max_tokens, hdr, seq_off, list);
  COPRIS_POST("attn_worklist_kernel");
  {
    const dim3 grid(static_cast<unsigned>(w.max_list * Hkv));
#define COPRIS_GENERIC(T, DD)                                                                   \
  hipLaunchKernelGGL((attn_split_generic_kernel<T, DD>), grid, dim3(256), 0, stream,            \
                     static_cast<const T*>(q), static_cast<const T*>(k_cache),                  \
                     static_cast<const T*>(v_cache), block_table, ctx_len, hdr, list, ws_ml,    \
                     ws_acc, Hq, Hkv, g, page_size, max_pages, max_tokens, scale_log2e)
    COPRIS_PRE("attn_split_generic_kernel");
    if (dtype == 0 && D == 64) COPRIS_GENERIC(float, 64);
    else if (dtype == 0 && D == 128) COPRIS_GENERIC(float, 128);
    else if (dtype == 1 && D == 64) COPRIS_GENERIC(uint16_t, 64);
    else COPRIS_GENERIC(uint16_t, 128);
#undef COPRIS_GENERIC
    COPRIS_POST("attn_split_generic_kernel");
  }
  COPRIS_PRE("attn_merge_kernel");
  if (dtype == 0) {
    hipLaunchKernelGGL(attn_merge_kernel<float>, dim3(C, Hq), dim3(D), 0, stream, seq_off, ws_ml,
                       ws_acc, static_cast<float*>(out), lse, Hq, Hkv, g, D);
  } else {
    hipLaunchKernelGGL(attn_merge_kernel<uint16_t>, dim3(C, Hq), dim3(D), 0, stream, seq_off,
                       ws_ml, ws_acc, static_cast<uint16_t*>(out), lse, Hq, Hkv, g, D);
  }
  COPRIS_POST("attn_merge_kernel");
  return 0;
}

}  // namespace copris
