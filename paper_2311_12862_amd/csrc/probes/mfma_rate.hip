// Matrix-core rate probe for gfx950 (a developer tool, not part of the library): every wave of a
// full-chip grid issues independent 16x16x32 bf16 MFMAs back to back, nothing else.  The run gives
// the rate the matrix cores sustain (against the published dense peak that the roofline fractions
// use) and, from the shader clock counter against the wall clock, the clock the chip holds while
// they are busy.  No memory is touched except one 8-byte store per wave at the end.
#include <hip/hip_runtime.h>
#include <cstdio>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kAcc = 16;  // independent accumulators per wave

__global__ void __launch_bounds__(256) k_mfma(int iters, long long* __restrict__ ticks, int n_out) {
  f32x4 acc[kAcc];
  for (int i = 0; i < kAcc; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  bf16x8 a, b;
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(float)(threadIdx.x % 3);
    b[i] = (__bf16)(float)(threadIdx.x % 5);
  }
  const long long t0 = clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < kAcc; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
  }
  const long long t1 = clock64();
  float s = 0.f;
  for (int i = 0; i < kAcc; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  const int w = (int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6);
  if ((threadIdx.x & 63) == 0 && w < n_out) ticks[w] = (t1 - t0) + (s == 12345.678f ? 1 : 0);
}

int main() {
  const int cus = 256, wgs_per_cu = 2, iters = 20000;
  const int wgs = cus * wgs_per_cu, waves = wgs * 4;
  long long* d_ticks;
  if (hipMalloc(&d_ticks, waves * sizeof(long long)) != hipSuccess) return 2;
  hipEvent_t e0, e1;
  hipEventCreate(&e0);
  hipEventCreate(&e1);
  for (int rep = 0; rep < 3; ++rep) {
    hipEventRecord(e0, 0);
    hipLaunchKernelGGL(k_mfma, dim3(wgs), dim3(256), 0, 0, iters, d_ticks, waves);
    hipEventRecord(e1, 0);
    if (hipEventSynchronize(e1) != hipSuccess) { printf("launch failed\n"); return 3; }
    float ms = 0.f;
    hipEventElapsedTime(&ms, e0, e1);
    long long t = 0;
    hipMemcpy(&t, d_ticks, sizeof(t), hipMemcpyDeviceToHost);
    const double flop = (double)waves * iters * kAcc * 16.0 * 16.0 * 32.0 * 2.0;
    printf("run %d: %.3f ms, %.1f TFLOP/s dense bf16 (%d waves, 2 per SIMD); wave 0: %lld counter ticks = %.1f per MFMA; "
           "counter rate %.1f MHz\n",
           rep, ms, flop / (ms * 1e-3) / 1e12, waves, t, (double)t / ((double)iters * kAcc), (double)t / (ms * 1e3));
    fflush(stdout);
  }
  return 0;
}
