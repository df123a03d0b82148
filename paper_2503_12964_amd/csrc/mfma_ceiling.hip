// Measured ceiling of the bf16 matrix pipe on the GPU at hand: a loop of nothing but
// independent v_mfma_f32_32x32x16_bf16 instructions (8 accumulators per wavefront, two
// wavefronts per SIMD, no memory or LDS traffic), sustained for a few seconds.  Run once
// with constant operands and once with random ones: the matrix pipe draws more power when
// its inputs toggle, and the chip lowers its clock to stay inside its power limit, so the
// rate an attention kernel with real data can approach is the second figure, not the
// first.  A third loop of nothing but v_exp_f32 gives the rate of the softmax's exponentials
// (the secondary ceiling of an attention kernel: one exponential per score, and per score
// again in each of the two backward kernels).  Prints one JSON line.  Standalone program;
// not part of the library.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <vector>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define CHECK(x)                                                                   \
  do {                                                                             \
    hipError_t e_ = (x);                                                           \
    if (e_ != hipSuccess) {                                                        \
      fprintf(stderr, "mfma_ceiling: %s at line %d\n", hipGetErrorString(e_), __LINE__); \
      exit(1);                                                                     \
    }                                                                              \
  } while (0)

constexpr int kThreads = 256;
constexpr int kOperandSets = 4;

__global__ __launch_bounds__(kThreads) void mfma_loop(const bf16x8* __restrict__ src,
                                                      float* __restrict__ sink, int iters) {
  bf16x8 a[kOperandSets], b[kOperandSets];
  for (int i = 0; i < kOperandSets; ++i) {
    a[i] = src[(2 * i) * kThreads + threadIdx.x];
    b[i] = src[(2 * i + 1) * kThreads + threadIdx.x];
  }
  f32x16 acc[8];
  for (int n = 0; n < 8; ++n)
    for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int n = 0; n < 8; ++n)
      acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[n & 3], b[(n + (n >> 2)) & 3], acc[n], 0, 0, 0);
  }
  float s = 0.f;
  for (int n = 0; n < 8; ++n)
    for (int r = 0; r < 16; ++r) s += acc[n][r];
  if (s == 12345.678f) sink[threadIdx.x] = s;   // keeps the loop alive; practically never true
}

// Eight independent chains of y = 2^(-y) per lane (converges to 0.64; the rate does not depend
// on the values), two wavefronts per SIMD.
__global__ __launch_bounds__(kThreads) void exp_loop(float* __restrict__ sink, int iters) {
  float y[8];
  for (int n = 0; n < 8; ++n) y[n] = 0.1f * (float)(n + 1) + 1e-3f * (float)threadIdx.x;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int n = 0; n < 8; ++n) y[n] = __builtin_amdgcn_exp2f(-y[n]);
  }
  float s = 0.f;
  for (int n = 0; n < 8; ++n) s += y[n];
  if (s == 12345.678f) sink[threadIdx.x] = s;
}

// Exponentials per second (in units of 1e12), one timed batch of launches after a warm-up.
static double exp_rate_tera(float* sink) {
  const int iters = 20000, grid = 2048, launches = 10;
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  exp_loop<<<grid, kThreads>>>(sink, iters);
  CHECK(hipEventRecord(e0));
  for (int i = 0; i < launches; ++i) exp_loop<<<grid, kThreads>>>(sink, iters);
  CHECK(hipEventRecord(e1));
  CHECK(hipEventSynchronize(e1));
  float ms = 0.f;
  CHECK(hipEventElapsedTime(&ms, e0, e1));
  CHECK(hipEventDestroy(e0));
  CHECK(hipEventDestroy(e1));
  return (double)launches * grid * kThreads * iters * 8 / (ms * 1e-3) / 1e12;
}

// Sustained TFLOP/s over the second half of `seconds` of back-to-back launches.
static double sustained_tflops(const void* src, float* sink, double seconds) {
  const int iters = 40000, grid = 512, launches = 10;
  const double flops = (double)launches * grid * (kThreads / 64) * iters * 8 * (2.0 * 32 * 32 * 16);
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  const auto t0 = std::chrono::steady_clock::now();
  double sum = 0.0;
  int n = 0;
  for (;;) {
    const double t = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    if (t >= seconds) break;
    CHECK(hipEventRecord(e0));
    for (int i = 0; i < launches; ++i)
      mfma_loop<<<grid, kThreads>>>(static_cast<const bf16x8*>(src), sink, iters);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    if (t >= 0.5 * seconds) { sum += flops / (ms * 1e-3) / 1e12; ++n; }
  }
  CHECK(hipEventDestroy(e0));
  CHECK(hipEventDestroy(e1));
  return n ? sum / n : 0.0;
}

int main(int argc, char** argv) {
  const double seconds = argc > 1 ? atof(argv[1]) : 1.5;
  const size_t n_elems = (size_t)2 * kOperandSets * kThreads * 8;
  std::vector<unsigned short> host(n_elems);
  void* src = nullptr;
  float* sink = nullptr;
  CHECK(hipMalloc(&src, n_elems * 2));
  CHECK(hipMalloc(&sink, kThreads * sizeof(float)));
  double rate[2];
  for (int random = 0; random < 2; ++random) {
    unsigned x = 12345u;
    for (auto& e : host) {
      x = x * 1664525u + 1013904223u;   // random sign, mantissa and an exponent in [2^-7, 1]
      const unsigned sign = (x >> 31) << 15, expo = 120u + ((x >> 20) & 7u), mant = (x >> 9) & 0x7fu;
      e = random ? (unsigned short)(sign | (expo << 7) | mant) : (unsigned short)0x3f80;   // else 1.0
    }
    CHECK(hipMemcpy(src, host.data(), n_elems * 2, hipMemcpyHostToDevice));
    rate[random] = sustained_tflops(src, sink, seconds);
  }
  const double exp_tera = exp_rate_tera(sink);
  printf("{\"constant_operands_tflops\": %.1f, \"random_operands_tflops\": %.1f, \"seconds_each\": %.2f, "
         "\"exp2_only_tera_per_s\": %.2f}\n",
         rate[0], rate[1], seconds, exp_tera);
  CHECK(hipFree(src));
  CHECK(hipFree(sink));
  return 0;
}
