// Measurement aid: what the gfx950 matrix cores sustain with no data movement at all.
// Every wavefront issues back-to-back independent v_mfma_f32_32x32x16_bf16 on register
// operands; the run is repeated with constant operands and with pseudo-random bf16 operands
// (switching activity, and with it power and clock, depends on the data).
//
//   mfma_peak [milliseconds per measurement, default 200]
//
// Prints one line per case: achieved TFLOP/s, the fraction of the 2500 TFLOP/s nominal peak, and
// the shader clock the loop ran at (cycle counter over the constant-rate wall counter, both read
// by one wavefront at the start and at the end of its loop).
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define CHECK(x)                                                                   \
  do {                                                                             \
    hipError_t e_ = (x);                                                           \
    if (e_ != hipSuccess) {                                                        \
      fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
      return 1;                                                                    \
    }                                                                              \
  } while (0)

constexpr int NACC = 8;   // independent accumulators per wavefront (no dependent issue)

template <bool RANDOM>
__global__ __launch_bounds__(256) void mfma_loop(float* out, int iters, long long* ticks) {
  const long long c0 = clock64(), w0 = wall_clock64();
  f32x16 acc[NACC];
  for (int i = 0; i < NACC; ++i)
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  bf16x8 a, b, a2, b2;
  unsigned seed = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
  for (int i = 0; i < 8; ++i) {
    if (RANDOM) {
      seed = seed * 1664525u + 1013904223u;
      a[i] = (__bf16)(((int)(seed >> 16) % 2001 - 1000) / 1000.f);
      seed = seed * 1664525u + 1013904223u;
      b[i] = (__bf16)(((int)(seed >> 16) % 2001 - 1000) / 1000.f);
    } else {
      a[i] = (__bf16)1.0f;
      b[i] = (__bf16)1.0f;
    }
  }
  for (int i = 0; i < 8; ++i) {
    a2[i] = b[7 - i];
    b2[i] = a[7 - i];
  }
  for (int it = 0; it < iters; it += 2) {
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, b2, acc[i], 0, 0, 0);
  }
  float s = 0.f;
  for (int i = 0; i < NACC; ++i)
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    ticks[0] = clock64() - c0;
    ticks[1] = wall_clock64() - w0;
  }
}

template <bool RANDOM>
static int measure(const char* name, float* out, long long* ticks, double wall_khz, int ncu, double target_ms) {
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  const int blocks = ncu * 2;   // two workgroups of four wavefronts per compute unit
  int iters = 2000;
  double tf = 0.0;
  for (int rep = 0; rep < 4; ++rep) {   // the first repetitions size the run and warm the clocks
    CHECK(hipEventRecord(e0));
    hipLaunchKernelGGL(mfma_loop<RANDOM>, dim3(blocks), dim3(256), 0, 0, out, iters, ticks);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double flop = (double)blocks * 4 * iters * NACC * 32.0 * 32.0 * 16.0 * 2.0;
    tf = flop / ms / 1e9;
    if (rep < 3) iters = (int)(iters * target_ms / (ms > 1e-3 ? ms : 1e-3)) / 2 * 2 + 2;
    else {
      long long h[2] = {0, 1};
      CHECK(hipMemcpy(h, ticks, sizeof(h), hipMemcpyDeviceToHost));
      printf("%-28s %8.1f ms  %7.1f TFLOP/s  %.3f of 2500   shader clock %.0f MHz\n", name, ms, tf, tf / 2500.0,
             (double)h[0] / (double)h[1] * wall_khz / 1e3);
    }
  }
  return 0;
}

int main(int argc, char** argv) {
  const double target_ms = argc > 1 ? atof(argv[1]) : 200.0;
  hipDeviceProp_t prop;
  CHECK(hipGetDeviceProperties(&prop, 0));
  const int ncu = prop.multiProcessorCount;
  float* out = nullptr;
  long long* ticks = nullptr;
  int wall_khz = 100000;
  CHECK(hipDeviceGetAttribute(&wall_khz, hipDeviceAttributeWallClockRate, 0));
  CHECK(hipMalloc(&out, (size_t)ncu * 2 * 256 * sizeof(float)));
  CHECK(hipMalloc(&ticks, 2 * sizeof(long long)));
  printf("%s, %d compute units\n", prop.gcnArchName, ncu);
  if (measure<false>("constant operands", out, ticks, wall_khz, ncu, target_ms)) return 1;
  if (measure<true>("random bf16 operands", out, ticks, wall_khz, ncu, target_ms)) return 1;
  CHECK(hipFree(out));
  CHECK(hipFree(ticks));
  return 0;
}
