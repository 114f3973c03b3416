// Measured peaks of the GPU the library runs on, for roofline reports: what a plain streaming
// copy moves through HBM and what back-to-back matrix instructions sustain.  Both are quoted
// beside the published figures (8 TB/s, 2.5 PFLOP/s dense fp16 / bf16), never instead of them.
#include "common.h"

namespace spc {
namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// dst[i] = src[i], 16 bytes per thread and step, grid-stride: one read and one write per byte
__global__ void __launch_bounds__(256) k_stream_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, long long n) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// every wave issues independent 16x16x32 fp16 MFMAs back to back, nothing else
constexpr int kAcc = 16;
__global__ void __launch_bounds__(256) k_mfma_rate(int iters, float* __restrict__ sink) {
  f32x4 acc[kAcc];
  for (int i = 0; i < kAcc; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  f16x8 a, b;
  for (int i = 0; i < 8; ++i) {
    a[i] = (_Float16)(float)(threadIdx.x % 3);
    b[i] = (_Float16)(float)(threadIdx.x % 5);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < kAcc; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
  for (int i = 0; i < kAcc; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  if (s == 12345.678f) sink[0] = s;  // (keeps the loop alive)
}

struct EventPair {
  hipEvent_t a = nullptr, b = nullptr;
  ~EventPair() {
    if (a) (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
  }
};

}  // namespace
}  // namespace spc

using namespace spc;

extern "C" SPCONV_API int spconv_measure_peaks(double* hbm_copy_gbs, double* mfma_f16_tflops, void* stream) {
  StreamScope scope((hipStream_t)stream);
  hipStream_t st = (hipStream_t)stream;
  EventPair ev;
  SPC_HIP(hipEventCreate(&ev.a));
  SPC_HIP(hipEventCreate(&ev.b));
  if (hbm_copy_gbs) {
    // 1 GiB each way: four times the 256 MB last-level cache, so the bytes come from and go to HBM
    const size_t bytes = (size_t)1 << 30;
    DevBuf src, dst;
    SPC_TRY(src.alloc(bytes));
    SPC_TRY(dst.alloc(bytes));
    SPC_HIP(hipMemsetAsync(src.p, 1, bytes, st));
    const long long n = (long long)(bytes / 16);
    float best = 1e30f;
    for (int rep = 0; rep < 4; ++rep) {  // (the first run also warms the launch)
      SPC_HIP(hipEventRecord(ev.a, st));
      hipLaunchKernelGGL(k_stream_copy, dim3(256 * 32), dim3(256), 0, st, src.as<uint4>(), dst.as<uint4>(), n);
      SPC_LAUNCH_CHECK();
      SPC_HIP(hipEventRecord(ev.b, st));
      SPC_HIP(hipEventSynchronize(ev.b));
      float ms = 0.f;
      SPC_HIP(hipEventElapsedTime(&ms, ev.a, ev.b));
      if (rep > 0 && ms < best) best = ms;
    }
    *hbm_copy_gbs = 2.0 * (double)bytes / ((double)best * 1e-3) / 1e9;  // bytes read + bytes written
  }
  if (mfma_f16_tflops) {
    DevBuf sink;
    SPC_TRY(sink.alloc(16));
    const int wgs = 256 * 2, iters = 20000;  // two waves per SIMD
    float best = 1e30f;
    for (int rep = 0; rep < 3; ++rep) {
      SPC_HIP(hipEventRecord(ev.a, st));
      hipLaunchKernelGGL(k_mfma_rate, dim3(wgs), dim3(256), 0, st, iters, sink.as<float>());
      SPC_LAUNCH_CHECK();
      SPC_HIP(hipEventRecord(ev.b, st));
      SPC_HIP(hipEventSynchronize(ev.b));
      float ms = 0.f;
      SPC_HIP(hipEventElapsedTime(&ms, ev.a, ev.b));
      if (rep > 0 && ms < best) best = ms;
    }
    const double flop = (double)wgs * 4 * iters * kAcc * 16.0 * 16.0 * 32.0 * 2.0;
    *mfma_f16_tflops = flop / ((double)best * 1e-3) / 1e12;
  }
  return SPCONV_OK;
}
