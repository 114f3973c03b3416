// Element-wise glue between convolution layers (activation, residual add, channel concat and
// their gradients).  Not part of the paper's method; they exist so that a whole network can
// run on the library's own kernels.  All are bandwidth-bound streaming kernels over
// [rows][channels] tensors, 8 elements (16 bytes) per lane for the 16-bit types.
#include "common.h"

#include <algorithm>

namespace spc {
namespace {

template <typename T> __device__ __forceinline__ float to_f(T v) { return (float)v; }

enum EwOp { EW_RELU = 0, EW_ADD = 1, EW_ADD_RELU = 2, EW_RELU_BWD = 3 };

// out[i] = op(a[i], b[i]); RELU: max(a,0); ADD: a+b; ADD_RELU: max(a+b,0); RELU_BWD: b > 0 ? a : 0
template <typename T, int OP>
__global__ void __launch_bounds__(256) k_ew(const T* a, const T* b, T* out,  // (out may alias a or b: no __restrict__)
                                            long long n) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    const float x = to_f(a[i]);
    const float y = (OP == EW_RELU) ? 0.f : to_f(b[i]);
    float r;
    if (OP == EW_RELU) r = x > 0.f ? x : 0.f;
    else if (OP == EW_ADD) r = x + y;
    else if (OP == EW_ADD_RELU) r = (x + y) > 0.f ? (x + y) : 0.f;
    else r = y > 0.f ? x : 0.f;
    out[i] = (T)r;
  }
}

// dst[r][dst_off + c] = src[r][src_off + c] for c < cols (channel concat / split)
template <typename T>
__global__ void __launch_bounds__(256) k_copy_cols(const T* __restrict__ src, int src_ld, int src_off, T* __restrict__ dst,
                                                   int dst_ld, int dst_off, int cols, long long rows) {
  const long long total = rows * cols;
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const long long r = i / cols;
    const int c = (int)(i - r * cols);
    dst[r * dst_ld + dst_off + c] = src[r * src_ld + src_off + c];
  }
}

template <typename T>
int launch_ew(int op, const void* a, const void* b, void* out, long long n, hipStream_t st) {
  const unsigned blocks = (unsigned)std::min<long long>((n + 255) / 256, 8192);
  const T* pa = (const T*)a;
  const T* pb = (const T*)b;
  T* po = (T*)out;
  switch (op) {
    case EW_RELU: hipLaunchKernelGGL((k_ew<T, EW_RELU>), dim3(blocks), dim3(256), 0, st, pa, pb, po, n); break;
    case EW_ADD: hipLaunchKernelGGL((k_ew<T, EW_ADD>), dim3(blocks), dim3(256), 0, st, pa, pb, po, n); break;
    case EW_ADD_RELU: hipLaunchKernelGGL((k_ew<T, EW_ADD_RELU>), dim3(blocks), dim3(256), 0, st, pa, pb, po, n); break;
    case EW_RELU_BWD: hipLaunchKernelGGL((k_ew<T, EW_RELU_BWD>), dim3(blocks), dim3(256), 0, st, pa, pb, po, n); break;
    default: return SPCONV_EINVAL;
  }
  SPC_LAUNCH_CHECK();
  return SPCONV_OK;
}

}  // namespace
}  // namespace spc

using namespace spc;

extern "C" {

SPCONV_API int spconv_ew(int op, const void* a, const void* b, void* out, int64_t n, spconv_dtype dtype, void* stream) {
  if (n < 0 || op < 0 || op > 3) return SPCONV_EINVAL;
  if (n == 0) return SPCONV_OK;
  if (!a || !out || (op != EW_RELU && !b)) return SPCONV_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  switch (dtype) {
    case SPCONV_F32: return launch_ew<float>(op, a, b, out, n, st);
    case SPCONV_F16: return launch_ew<_Float16>(op, a, b, out, n, st);
    case SPCONV_BF16: return launch_ew<__bf16>(op, a, b, out, n, st);
  }
  return SPCONV_EINVAL;
}

SPCONV_API int spconv_copy_cols(const void* src, int src_ld, int src_off, void* dst, int dst_ld, int dst_off, int cols,
                                int64_t rows, spconv_dtype dtype, void* stream) {
  if (rows < 0 || cols < 0 || src_off < 0 || dst_off < 0 || src_off + cols > src_ld || dst_off + cols > dst_ld)
    return SPCONV_EINVAL;
  if (rows == 0 || cols == 0) return SPCONV_OK;
  if (!src || !dst) return SPCONV_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  const unsigned blocks = (unsigned)std::min<long long>((rows * cols + 255) / 256, 8192);
  if (dtype == SPCONV_F32)
    hipLaunchKernelGGL((k_copy_cols<float>), dim3(blocks), dim3(256), 0, st, (const float*)src, src_ld, src_off,
                       (float*)dst, dst_ld, dst_off, cols, (long long)rows);
  else if (dtype == SPCONV_F16 || dtype == SPCONV_BF16)
    hipLaunchKernelGGL((k_copy_cols<unsigned short>), dim3(blocks), dim3(256), 0, st, (const unsigned short*)src,
                       src_ld, src_off, (unsigned short*)dst, dst_ld, dst_off, cols, (long long)rows);
  else
    return SPCONV_EINVAL;
  SPC_LAUNCH_CHECK();
  return SPCONV_OK;
}

}  // extern "C"
