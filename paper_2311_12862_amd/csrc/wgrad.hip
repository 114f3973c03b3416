// Weight-gradient kernels (Sections 4.2, 6.2): dW[k] = sum over present pairs
// (n, j = M[n][k]) of x[j]^T . dy[n].
//
// The reduction runs over output rows, which is the long inner loop the paper
// singles out.  Here a workgroup takes one offset k and a range of rows from
// the offset-major map, compacts the present pairs of 256 rows at a time into
// an LDS ring with a wave ballot and a four-entry prefix, and feeds the matrix
// cores dense batches of 128 pairs: no multiply is spent on absent
// neighbours, whatever the row order, so wgrad needs no sorted map.  Both
// operands are gathered row-wise and transposed on their way into LDS
// (the MFMA wants the reduction index contiguous per lane).  Each work item
// writes an fp32 partial tile; a second kernel adds the tiles of each offset
// in a fixed order, so results are bit-reproducible.
#include "common.h"

namespace spc {
namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <typename T> struct Mfma;
template <> struct Mfma<_Float16> {
  typedef f16x8 vec;
  static __device__ __forceinline__ f32x4 run(vec a, vec b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
  }
};
template <> struct Mfma<__bf16> {
  typedef bf16x8 vec;
  static __device__ __forceinline__ f32x4 run(vec a, vec b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
};

struct WgradParams {
  const void* feats;   // [n_in][C_in]
  const void* dout;    // [n_out][C_out]
  const int* map_k;    // [V][rows_pad]
  const WgradItem* items;
  float* partial;      // [n_items][C_in][C_out]
  long long rows_pad;
  int C_in, C_out;
};

constexpr int WG_BK = 128;             // pairs per MFMA batch
constexpr int WG_LD = WG_BK + 8;       // LDS pitch of the transposed operand tiles
constexpr int WG_RING = 512;

template <typename T>
__global__ void __launch_bounds__(256) k_wgrad(const WgradParams p) {
  typedef typename Mfma<T>::vec vec8;
  __shared__ __align__(16) unsigned short XT[64 * WG_LD];  // [ci][pair]
  __shared__ __align__(16) unsigned short DT[64 * WG_LD];  // [co][pair]
  __shared__ int ringN[WG_RING], ringJ[WG_RING];
  __shared__ int wave_cnt[4];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const WgradItem item = p.items[blockIdx.x];
  const int ci0 = blockIdx.y * 64, co0 = blockIdx.z * 64;
  const unsigned short* feats = reinterpret_cast<const unsigned short*>(p.feats);
  const unsigned short* dout = reinterpret_cast<const unsigned short*>(p.dout);
  const int* col = p.map_k + (long long)item.k * p.rows_pad;

  f32x4 acc[4];
#pragma unroll
  for (int nb = 0; nb < 4; ++nb) acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int seg = tid % 8, q0 = tid / 8;

  auto batch = [&](int head, int cnt) {
    // gather the two operands of up to WG_BK pairs and store them transposed
#pragma unroll
    for (int ps = 0; ps < WG_BK / 32; ++ps) {
      const int q = q0 + ps * 32;
      uint4 vx = make_uint4(0, 0, 0, 0), vd = make_uint4(0, 0, 0, 0);
      if (q < cnt) {
        const int n = ringN[(head + q) & (WG_RING - 1)], j = ringJ[(head + q) & (WG_RING - 1)];
        if (ci0 + seg * 8 < p.C_in)
          vx = *reinterpret_cast<const uint4*>(feats + (long long)j * p.C_in + ci0 + seg * 8);
        if (co0 + seg * 8 < p.C_out)
          vd = *reinterpret_cast<const uint4*>(dout + (long long)n * p.C_out + co0 + seg * 8);
      }
      const unsigned wx[4] = {vx.x, vx.y, vx.z, vx.w}, wd[4] = {vd.x, vd.y, vd.z, vd.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        XT[(seg * 8 + 2 * i) * WG_LD + q] = (unsigned short)(wx[i] & 0xFFFFu);
        XT[(seg * 8 + 2 * i + 1) * WG_LD + q] = (unsigned short)(wx[i] >> 16);
        DT[(seg * 8 + 2 * i) * WG_LD + q] = (unsigned short)(wd[i] & 0xFFFFu);
        DT[(seg * 8 + 2 * i + 1) * WG_LD + q] = (unsigned short)(wd[i] >> 16);
      }
    }
    __syncthreads();
    const unsigned short* a = XT + (wave * 16 + (lane & 15)) * WG_LD + (lane >> 4) * 8;
    const unsigned short* b = DT + (lane & 15) * WG_LD + (lane >> 4) * 8;
    const int steps = (cnt + 31) / 32;
    for (int ks = 0; ks < steps; ++ks) {
      const vec8 af = *reinterpret_cast<const vec8*>(a + ks * 32);
#pragma unroll
      for (int nb = 0; nb < 4; ++nb) {
        const vec8 bf = *reinterpret_cast<const vec8*>(b + nb * 16 * WG_LD + ks * 32);
        acc[nb] = Mfma<T>::run(af, bf, acc[nb]);
      }
    }
    __syncthreads();
  };

  int head = 0, tail = 0;
  const unsigned long long lt = (1ull << lane) - 1ull;
  for (int base = item.row_begin; base < item.row_end; base += 256) {
    const int n = base + tid;
    const int j = (n < item.row_end) ? col[n] : -1;
    const bool valid = j >= 0;
    const unsigned long long bal = __ballot(valid);
    if (lane == 0) wave_cnt[wave] = __popcll(bal);
    __syncthreads();
    int off = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int c = wave_cnt[w];
      off += (w < wave) ? c : 0;
      total += c;
    }
    if (valid) {
      const int pos = (tail + off + __popcll(bal & lt)) & (WG_RING - 1);
      ringN[pos] = n;
      ringJ[pos] = j;
    }
    tail += total;
    __syncthreads();
    while (tail - head >= WG_BK) {
      batch(head, WG_BK);
      head += WG_BK;
    }
  }
  if (tail > head) batch(head, tail - head);

  float* dst = p.partial + (long long)item.slot * p.C_in * p.C_out;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int ci = ci0 + wave * 16 + (lane >> 4) * 4 + r;
    if (ci >= p.C_in) continue;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      const int co = co0 + nb * 16 + (lane & 15);
      if (co < p.C_out) dst[(long long)ci * p.C_out + co] = acc[nb][r];
    }
  }
}

// fp32 path: 16 rows at a time, absent neighbours contribute zeros.
__global__ void __launch_bounds__(256) k_wgrad_f32(const WgradParams p) {
  __shared__ float Xs[16][64 + 4];
  __shared__ float Ds[16][64 + 4];
  const int tid = threadIdx.x;
  const WgradItem item = p.items[blockIdx.x];
  const int ci0 = blockIdx.y * 64, co0 = blockIdx.z * 64;
  const float* feats = reinterpret_cast<const float*>(p.feats);
  const float* dout = reinterpret_cast<const float*>(p.dout);
  const int* col = p.map_k + (long long)item.k * p.rows_pad;
  const int ty = tid / 16, tx = tid % 16;
  const int q = tid / 16, seg4 = (tid % 16) * 4;
  float acc[4][4] = {};
  for (int base = item.row_begin; base < item.row_end; base += 16) {
    const int n = base + q;
    const int j = (n < item.row_end) ? col[n] : -1;
    float4 vx = make_float4(0.f, 0.f, 0.f, 0.f), vd = vx;
    if (j >= 0) {
      if (ci0 + seg4 < p.C_in) vx = *reinterpret_cast<const float4*>(feats + (long long)j * p.C_in + ci0 + seg4);
      if (co0 + seg4 < p.C_out) vd = *reinterpret_cast<const float4*>(dout + (long long)n * p.C_out + co0 + seg4);
    }
    *reinterpret_cast<float4*>(&Xs[q][seg4]) = vx;
    *reinterpret_cast<float4*>(&Ds[q][seg4]) = vd;
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = Xs[r][ty * 4 + i];
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) b[jj] = Ds[r][tx * 4 + jj];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) acc[i][jj] = fmaf(a[i], b[jj], acc[i][jj]);
    }
    __syncthreads();
  }
  float* dst = p.partial + (long long)item.slot * p.C_in * p.C_out;
  for (int i = 0; i < 4; ++i) {
    const int ci = ci0 + ty * 4 + i;
    if (ci >= p.C_in) continue;
    for (int jj = 0; jj < 4; ++jj) {
      const int co = co0 + tx * 4 + jj;
      if (co < p.C_out) dst[(long long)ci * p.C_out + co] = acc[i][jj];
    }
  }
}

// dW[k][e] = sum of the partial tiles of offset k, in item order
__global__ void __launch_bounds__(256) k_wgrad_reduce(const float* __restrict__ partial, const int* __restrict__ seg,
                                                      int elems, float* __restrict__ dw) {
  const int e4 = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (e4 >= elems) return;
  const int k = blockIdx.y;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int it = seg[k]; it < seg[k + 1]; ++it) {
    const float4 v = *reinterpret_cast<const float4*>(partial + (long long)it * elems + e4);
    s.x += v.x;
    s.y += v.y;
    s.z += v.z;
    s.w += v.w;
  }
  *reinterpret_cast<float4*>(dw + (long long)k * elems + e4) = s;
}

}  // namespace

int wgrad_run(spconv_kmap* km, const WgradPlan& wp, const void* feats, const void* dout, int C_in, int C_out,
              spconv_dtype dtype, float* dweights, hipStream_t st) {
  const int V = km->V;
  const int elems = C_in * C_out;
  if (wp.n_items > 0) {
    SPC_TRY(km->scratch.reserve((size_t)wp.n_items * elems * sizeof(float)));
    WgradParams p{};
    p.feats = feats;
    p.dout = dout;
    p.map_k = wp.map_k.as<int>();
    p.items = wp.items.as<WgradItem>();
    p.partial = km->scratch.as<float>();
    p.rows_pad = km->out_side.rows_pad;
    p.C_in = C_in;
    p.C_out = C_out;
    dim3 grid((unsigned)wp.n_items, (unsigned)ceil_div(C_in, 64), (unsigned)ceil_div(C_out, 64));
    switch (dtype) {
      case SPCONV_F32: hipLaunchKernelGGL(k_wgrad_f32, grid, dim3(256), 0, st, p); break;
      case SPCONV_F16: hipLaunchKernelGGL((k_wgrad<_Float16>), grid, dim3(256), 0, st, p); break;
      case SPCONV_BF16: hipLaunchKernelGGL((k_wgrad<__bf16>), grid, dim3(256), 0, st, p); break;
    }
    SPC_LAUNCH_CHECK();
  }
  dim3 rgrid((unsigned)ceil_div(elems / 4, 256), (unsigned)V);
  hipLaunchKernelGGL(k_wgrad_reduce, rgrid, dim3(256), 0, st, km->scratch.as<float>(), wp.seg.as<int>(), elems,
                     dweights);
  SPC_LAUNCH_CHECK();
  return SPCONV_OK;
}

}  // namespace spc
