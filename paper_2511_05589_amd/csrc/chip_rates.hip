// Stand-alone measurement of two chip rates the kernel designs lean on (not part of
// libcopris.so; build and run:
//   hipcc --offload-arch=gfx950 -O3 -o /tmp/chip_rates paper_2511_05589_amd/csrc/chip_rates.hip && /tmp/chip_rates
// ):
//   * the sustained rate of the two bf16 matrix instructions (independent accumulators, operands
//     in registers, no memory traffic) for 1 .. 8 waves per SIMD;
//   * the LDS read bandwidth of a CU for 128-bit reads, 64-bit reads and the transposing
//     64-bit read, with conflict-free addresses.
// Every access stays inside the arrays declared here.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

#define CHECK(x)                                                                  \
  do {                                                                            \
    hipError_t e_ = (x);                                                          \
    if (e_ != hipSuccess) {                                                       \
      fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                     \
      return 1;                                                                   \
    }                                                                             \
  } while (0)

constexpr int kCUs = 256;
constexpr double kClock = 2.4e9;

template <int SHAPE>
__global__ __launch_bounds__(256) void mfma_kernel(float* out, int iters, uint32_t seed) {
  const u32x4 ra = {seed * (threadIdx.x + 1), seed + 3, seed ^ 0x3f803f80u, seed};
  const bf16x8 a = __builtin_bit_cast(bf16x8, ra), b = __builtin_bit_cast(bf16x8, ra);
  float s = 0.f;
  if (SHAPE == 16) {
    f32x4 c[8];
    for (int i = 0; i < 8; ++i) c[i] = f32x4{0, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 8; ++i) c[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c[i], 0, 0, 0);
    }
    for (int i = 0; i < 8; ++i) s += c[i][0] + c[i][3];
  } else {
    f32x16 c[4];
    for (int i = 0; i < 4; ++i)
      for (int r = 0; r < 16; ++r) c[i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 4; ++i) c[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[i], 0, 0, 0);
    }
    for (int i = 0; i < 4; ++i) s += c[i][0] + c[i][15];
  }
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// MODE 128: ds_read_b128, lane-linear.  64: ds_read_b64, lane-linear.  65: ds_read_b64_tr_b16,
// a group of 16 lanes reading four rows x 32 bytes, the rows' pieces in different banks.
template <int MODE>
__global__ __launch_bounds__(256) void lds_kernel(unsigned* out, int iters) {
  __shared__ __attribute__((aligned(1024))) char smem[32768];
  for (int i = threadIdx.x; i < 8192; i += 256) reinterpret_cast<unsigned*>(smem)[i] = i;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(smem)) + wave * 4096;
  unsigned acc = 0;
  if (MODE == 128) {
    const uint32_t a = lds0 + lane * 16;
    for (int it = 0; it < iters; ++it) {
      u32x4 x0, x1, x2, x3;
      asm volatile(
          "ds_read_b128 %0, %4 offset:0\n\tds_read_b128 %1, %4 offset:1024\n\tds_read_b128 %2, %4 offset:2048\n\t"
          "ds_read_b128 %3, %4 offset:3072\n\ts_waitcnt lgkmcnt(0)"
          : "=&v"(x0), "=&v"(x1), "=&v"(x2), "=&v"(x3)
          : "v"(a)
          : "memory");
      acc += x0[0] + x1[1] + x2[2] + x3[3];
    }
  } else if (MODE == 64) {
    const uint32_t a = lds0 + lane * 8;
    for (int it = 0; it < iters; ++it) {
      s16x4 x0, x1, x2, x3;
      asm volatile(
          "ds_read_b64 %0, %4 offset:0\n\tds_read_b64 %1, %4 offset:512\n\tds_read_b64 %2, %4 offset:1024\n\t"
          "ds_read_b64 %3, %4 offset:1536\n\ts_waitcnt lgkmcnt(0)"
          : "=&v"(x0), "=&v"(x1), "=&v"(x2), "=&v"(x3)
          : "v"(a)
          : "memory");
      acc += x0[0] + x1[1] + x2[2] + x3[3];
    }
  } else {
    const int i16 = lane & 15, g = lane >> 4;
    const int row = 4 * (g >> 1) + (i16 >> 2);
    const int piece = (g & 1) ^ (row & 3) ^ (4 * (g & 1));   // lanes 0..31 cover all 64 banks
    const uint32_t a = lds0 + row * 256 + piece * 32 + (i16 & 3) * 8;
    for (int it = 0; it < iters; ++it) {
      s16x4 x0, x1, x2, x3;
      asm volatile(
          "ds_read_b64_tr_b16 %0, %4 offset:0\n\tds_read_b64_tr_b16 %1, %4 offset:2048\n\t"
          "ds_read_b64_tr_b16 %2, %4 offset:0\n\tds_read_b64_tr_b16 %3, %4 offset:2048\n\ts_waitcnt lgkmcnt(0)"
          : "=&v"(x0), "=&v"(x1), "=&v"(x2), "=&v"(x3)
          : "v"(a)
          : "memory");
      acc += x0[0] + x1[1] + x2[2] + x3[3];
    }
  }
  out[blockIdx.x * 256 + threadIdx.x] = acc;
}

template <typename F>
int timed(F launch, float* ms) {
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  launch(100);
  CHECK(hipDeviceSynchronize());
  CHECK(hipEventRecord(e0));
  launch(20000);
  CHECK(hipEventRecord(e1));
  CHECK(hipEventSynchronize(e1));
  CHECK(hipEventElapsedTime(ms, e0, e1));
  CHECK(hipEventDestroy(e0));
  CHECK(hipEventDestroy(e1));
  return 0;
}

template <int SHAPE>
int run_mfma(const char* name, int waves_per_simd, uint32_t seed, float* d) {
  const int grid = kCUs * waves_per_simd;
  float ms;
  if (timed([&](int iters) { hipLaunchKernelGGL(mfma_kernel<SHAPE>, dim3(grid), dim3(256), 0, 0, d, iters, seed); }, &ms)) return 1;
  const double per = SHAPE == 16 ? 8.0 * 16 * 16 * 32 * 2 : 4.0 * 32 * 32 * 16 * 2;
  printf("%-24s %d wave(s) per SIMD, %s operands: %7.0f TFLOP/s\n", name, waves_per_simd, seed ? "random" : "zero  ",
         per * 20000 * 4.0 * grid / ms / 1e9);
  return 0;
}

template <int MODE>
int run_lds(const char* name, int waves_per_simd, unsigned* d) {
  const int grid = kCUs * waves_per_simd;
  float ms;
  if (timed([&](int iters) { hipLaunchKernelGGL(lds_kernel<MODE>, dim3(grid), dim3(256), 0, 0, d, iters); }, &ms)) return 1;
  const double bytes = (MODE == 128 ? 4096.0 : 2048.0) * 20000 * 4.0 * grid;   // four instructions per wave and iteration
  printf("%-24s %d wave(s) per SIMD: %6.1f TB/s chip-wide = %4.0f B per CU and clock (at 2.4 GHz)\n", name, waves_per_simd,
         bytes / ms / 1e9, bytes / kCUs / (ms * 1e-3 * kClock));
  return 0;
}

int main() {
  void* d;
  CHECK(hipMalloc(&d, static_cast<size_t>(kCUs) * 8 * 256 * sizeof(float)));
  for (uint32_t seed : {0u, 0x12345u}) {
    for (int w : {1, 2, 4, 8})
      if (run_mfma<16>("v_mfma_f32_16x16x32_bf16", w, seed, static_cast<float*>(d))) return 1;
    for (int w : {1, 2, 4})
      if (run_mfma<32>("v_mfma_f32_32x32x16_bf16", w, seed, static_cast<float*>(d))) return 1;
  }
  for (int w : {1, 2, 4})
    if (run_lds<128>("ds_read_b128", w, static_cast<unsigned*>(d))) return 1;
  for (int w : {1, 2, 4})
    if (run_lds<64>("ds_read_b64", w, static_cast<unsigned*>(d))) return 1;
  for (int w : {1, 2, 4})
    if (run_lds<65>("ds_read_b64_tr_b16", w, static_cast<unsigned*>(d))) return 1;
  CHECK(hipFree(d));
  return 0;
}
