// Weight-gradient kernels (Sections 4.2, 6.2): dW[k] = sum over present pairs
// (n, j = M[n][k]) of x[j]^T . dy[n].
//
// The reduction runs over output rows, the long inner loop the paper singles
// out.  Here it walks the compacted pair list of one offset (the
// weight-stationary view of the map, Section 2.2.1), so no multiply is spent
// on absent neighbours and the row order of the map does not matter.  A
// workgroup owns a 64 x 64 tile of dW[k] and a range of pairs.  Per batch of 64
// pairs it gathers 64 rows of x and of dy (16-byte segments, out-of-range
// buffer loads for the ragged tail), one batch ahead of the matrix cores, and
// stores them row-major in LDS; the MFMA operands need the reduction index
// (the pair) contiguous per lane, which the CDNA4 transposing LDS read
// (ds_read_b64_tr_b16) delivers without a software transpose.  Each work item
// writes an fp32 partial tile; a second kernel adds the tiles of each offset
// in item order, so results are bit-reproducible.
#include "common.h"

#include <atomic>

namespace spc {
namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <typename T> struct Mfma;
template <> struct Mfma<_Float16> {
  static __device__ __forceinline__ f32x4 run(s16x8 a, s16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0,
                                                  0);
  }
};
template <> struct Mfma<__bf16> {
  static __device__ __forceinline__ f32x4 run(s16x8 a, s16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                   0, 0);
  }
};

struct WgradParams {
  const void* feats;   // [n_in][C_in]
  const void* dout;    // [n_out][C_out]
  const int2* pairs;   // (n, j), offset-major
  const WgradItem* items;
  const int* item_seg; // [V+2], [V] = number of items
  float* partial;      // [max_items][C_in][C_out]
  unsigned feats_bytes, dout_bytes, pairs_bytes;
  int C_in, C_out, V;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ uint4 buf_load16(__amdgpu_buffer_rsrc_t r, unsigned byte_off) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ int2 buf_load8(__amdgpu_buffer_rsrc_t r, unsigned byte_off) {
  const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, byte_off, 0, 0);
  return make_int2((int)v.x, (int)v.y);
}

constexpr int WG_BK = 64;   // pairs per batch

// Transposing read: the 16 lanes of a group together fetch a 4 (rows) x 16 (columns) block,
// lane a pointing at row a/4, columns 4*(a%4)..+3; lane a receives column a of the block,
// i.e. four consecutive rows of one channel.  Two reads give the 8 reduction steps of a lane.
template <int LD>
__device__ __forceinline__ s16x8 read_frag(const unsigned short* tile, int row0, int col0, int lane) {
  const int a = lane & 15, g = lane >> 4;
  const unsigned short* p = tile + (row0 + 8 * g + (a >> 2)) * LD + col0 + 4 * (a & 3);
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4*)(p));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4*)(p + 4 * LD));
  return s16x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
}

// TILE x TILE outputs of dW[k] per workgroup (32, 64 or 128); each of the four waves owns a
// TILE/2 x TILE/2 quadrant as QB x QB MFMA blocks.  A larger tile gathers every pair's rows
// fewer times when the layer has more than 64 channels.
template <typename T, int TILE>
__global__ void __launch_bounds__(256) k_wgrad(const WgradParams p) {
  constexpr int QB = TILE / 32;        // 16 x 16 blocks per quadrant side
  constexpr int LD = TILE + 16;        // LDS row pitch in 2-byte elements: 8 words mod 32, so that the
                                       // four rows a transposing read touches fall on disjoint banks
  constexpr int SEGS = TILE / 8;       // 16-byte segments per staged row
  constexpr int PASSES = WG_BK * SEGS / 256;
  constexpr int RPP = 256 / SEGS;      // pair rows covered per pass
  extern __shared__ __align__(16) unsigned char smem_w[];
  unsigned short* Xs = reinterpret_cast<unsigned short*>(smem_w);  // [2][pair][ci]
  unsigned short* Ds = Xs + 2 * WG_BK * LD;                        // [2][pair][co]

  const int n_items = p.item_seg[p.V];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ci0 = blockIdx.y * TILE, co0 = blockIdx.z * TILE;
  // the grid is bounded; a workgroup takes items blockIdx.x, blockIdx.x + gridDim.x, ...
  for (int item_id = blockIdx.x; item_id < n_items; item_id += gridDim.x) {
  const WgradItem item = p.items[item_id];
  const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(p.feats, p.feats_bytes);
  const __amdgpu_buffer_rsrc_t d_rsrc = make_rsrc(p.dout, p.dout_bytes);
  const __amdgpu_buffer_rsrc_t p_rsrc = make_rsrc(p.pairs, p.pairs_bytes);
  const unsigned x_row = (unsigned)p.C_in * 2u, d_row = (unsigned)p.C_out * 2u;

  const int wci = (wave >> 1) * (TILE / 2), wco = (wave & 1) * (TILE / 2);
  f32x4 acc[QB][QB];
#pragma unroll
  for (int i = 0; i < QB; ++i)
#pragma unroll
    for (int j = 0; j < QB; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // staging: thread (q, seg) moves segment seg (8 channels) of pair rows q, q + RPP, ...
  const int seg = tid % SEGS, q0 = tid / SEGS;
  const bool x_ok = ci0 + seg * 8 < p.C_in, d_ok = co0 + seg * 8 < p.C_out;
  const int n_batches = (item.pair_end - item.pair_begin + WG_BK - 1) / WG_BK;

  int2 pr[PASSES];            // pair indices of the batch after next
  uint4 rx[PASSES], rd[PASSES];  // rows of the next batch
  auto load_pairs = [&](int batch) {
#pragma unroll
    for (int h = 0; h < PASSES; ++h) {
      const int e = item.pair_begin + batch * WG_BK + q0 + RPP * h;
      pr[h] = buf_load8(p_rsrc, (batch < n_batches && e < item.pair_end) ? (unsigned)e * 8u : 0xFFFFFFFFu);
    }
  };
  auto load_rows = [&](int batch) {
#pragma unroll
    for (int h = 0; h < PASSES; ++h) {
      const int e = item.pair_begin + batch * WG_BK + q0 + RPP * h;
      const bool live = batch < n_batches && e < item.pair_end;
      rx[h] = buf_load16(x_rsrc, (live && x_ok) ? (unsigned)pr[h].y * x_row + (unsigned)(ci0 + seg * 8) * 2u
                                                 : 0xFFFFFFFFu);
      rd[h] = buf_load16(d_rsrc, (live && d_ok) ? (unsigned)pr[h].x * d_row + (unsigned)(co0 + seg * 8) * 2u
                                                 : 0xFFFFFFFFu);
    }
  };
  auto store_rows = [&](int buf) {
#pragma unroll
    for (int h = 0; h < PASSES; ++h) {
      *reinterpret_cast<uint4*>(Xs + (buf * WG_BK + q0 + RPP * h) * LD + seg * 8) = rx[h];
      *reinterpret_cast<uint4*>(Ds + (buf * WG_BK + q0 + RPP * h) * LD + seg * 8) = rd[h];
    }
  };

  load_pairs(0);
  load_rows(0);
  load_pairs(1);
  store_rows(0);
  __syncthreads();
  for (int b = 0; b < n_batches; ++b) {
    load_rows(b + 1);   // out-of-range (zero, no traffic) past the last batch
    load_pairs(b + 2);
    const unsigned short* xs = Xs + (b & 1) * WG_BK * LD;
    const unsigned short* ds = Ds + (b & 1) * WG_BK * LD;
#pragma unroll
    for (int ks = 0; ks < WG_BK / 32; ++ks) {
      s16x8 af[QB], bf[QB];
#pragma unroll
      for (int i = 0; i < QB; ++i) af[i] = read_frag<LD>(xs, ks * 32, wci + i * 16, lane);
#pragma unroll
      for (int j = 0; j < QB; ++j) bf[j] = read_frag<LD>(ds, ks * 32, wco + j * 16, lane);
#pragma unroll
      for (int i = 0; i < QB; ++i)
#pragma unroll
        for (int j = 0; j < QB; ++j) acc[i][j] = Mfma<T>::run(af[i], bf[j], acc[i][j]);
    }
    store_rows((b + 1) & 1);
    __syncthreads();
  }

  float* dst = p.partial + (long long)item_id * p.C_in * p.C_out;
#pragma unroll
  for (int i = 0; i < QB; ++i)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int ci = ci0 + wci + i * 16 + (lane >> 4) * 4 + r;
      if (ci >= p.C_in) continue;
#pragma unroll
      for (int j = 0; j < QB; ++j) {
        const int co = co0 + wco + j * 16 + (lane & 15);
        if (co < p.C_out) dst[(long long)ci * p.C_out + co] = acc[i][j][r];
      }
    }
  __syncthreads();  // the LDS tiles are reused by the next item
  }
}

// fp32 path: plain FMA arithmetic, 16 pairs at a time.
__global__ void __launch_bounds__(256) k_wgrad_f32(const WgradParams p) {
  __shared__ float Xs[16][64 + 4];
  __shared__ float Ds[16][64 + 4];
  if ((int)blockIdx.x >= p.item_seg[p.V]) return;
  const int tid = threadIdx.x;
  const WgradItem item = p.items[blockIdx.x];
  const int ci0 = blockIdx.y * 64, co0 = blockIdx.z * 64;
  const float* feats = reinterpret_cast<const float*>(p.feats);
  const float* dout = reinterpret_cast<const float*>(p.dout);
  const int ty = tid / 16, tx = tid % 16;
  const int q = tid / 16, seg4 = (tid % 16) * 4;
  float acc[4][4] = {};
  for (int base = item.pair_begin; base < item.pair_end; base += 16) {
    const int e = base + q;
    float4 vx = make_float4(0.f, 0.f, 0.f, 0.f), vd = vx;
    if (e < item.pair_end) {
      const int2 pr = p.pairs[e];
      if (ci0 + seg4 < p.C_in) vx = *reinterpret_cast<const float4*>(feats + (long long)pr.y * p.C_in + ci0 + seg4);
      if (co0 + seg4 < p.C_out) vd = *reinterpret_cast<const float4*>(dout + (long long)pr.x * p.C_out + co0 + seg4);
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
  float* dst = p.partial + (long long)blockIdx.x * p.C_in * p.C_out;
  for (int i = 0; i < 4; ++i) {
    const int ci = ci0 + ty * 4 + i;
    if (ci >= p.C_in) continue;
    for (int jj = 0; jj < 4; ++jj) {
      const int co = co0 + tx * 4 + jj;
      if (co < p.C_out) dst[(long long)ci * p.C_out + co] = acc[i][jj];
    }
  }
}

// dW[k][e] = sum of the partial tiles of offset k.  A workgroup covers 64 float4 columns; its four
// waves take the items of the offset round-robin (four loads in flight each) and their sums are
// added in wave order, so the order of additions is fixed and results are bit-reproducible.
__global__ void __launch_bounds__(256) k_wgrad_reduce(const float* __restrict__ partial,
                                                      const int* __restrict__ item_seg, int elems,
                                                      float* __restrict__ dw) {
  __shared__ float4 part[4][64];
  const int col = threadIdx.x & 63, stripe = threadIdx.x >> 6;
  const int e4 = (blockIdx.x * 64 + col) * 4;
  const int k = blockIdx.y;
  const int first = item_seg[k], last = item_seg[k + 1];
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (e4 < elems) {
    int it = first + stripe;
    for (; it + 12 < last; it += 16) {
      float4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4*>(partial + (long long)(it + 4 * u) * elems + e4);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        s.x += v[u].x;
        s.y += v[u].y;
        s.z += v[u].z;
        s.w += v[u].w;
      }
    }
    for (; it < last; it += 4) {
      const float4 v = *reinterpret_cast<const float4*>(partial + (long long)it * elems + e4);
      s.x += v.x;
      s.y += v.y;
      s.z += v.z;
      s.w += v.w;
    }
  }
  part[stripe][col] = s;
  __syncthreads();
  if (stripe == 0 && e4 < elems) {
    float4 t = part[0][col];
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      t.x += part[w][col].x;
      t.y += part[w][col].y;
      t.z += part[w][col].z;
      t.w += part[w][col].w;
    }
    *reinterpret_cast<float4*>(dw + (long long)k * elems + e4) = t;
  }
}

}  // namespace

int wgrad_run(spconv_kmap* km, const WgradPlan& wp, const void* feats, const void* dout, int C_in, int C_out,
              spconv_dtype dtype, float* dweights, hipStream_t st) {
  const int V = km->V;
  const int elems = C_in * C_out;
  const size_t e = dtype == SPCONV_F32 ? 4 : 2;
  const uint64_t feats_bytes = (uint64_t)km->n_in * C_in * e, dout_bytes = (uint64_t)km->n_out * C_out * e;
  const uint64_t pairs_bytes = (uint64_t)std::max<int64_t>(wp.pairs_cap, 0) * 8;
  if (dtype != SPCONV_F32 && (feats_bytes >= 0xFFFFC000ull || dout_bytes >= 0xFFFFC000ull || pairs_bytes >= 0xFFFFC000ull))
    return SPCONV_EINVAL;  // buffer descriptors address 32 bits
  SPC_TRY(km->scratch.reserve((size_t)wp.max_items * elems * sizeof(float)));
  WgradParams p{};
  p.feats = feats;
  p.dout = dout;
  p.pairs = wp.pairs.as<int2>();
  p.items = wp.items.as<WgradItem>();
  p.item_seg = wp.item_seg.as<int>();
  p.partial = km->scratch.as<float>();
  p.feats_bytes = (unsigned)feats_bytes;
  p.dout_bytes = (unsigned)dout_bytes;
  p.pairs_bytes = (unsigned)pairs_bytes;
  p.C_in = C_in;
  p.C_out = C_out;
  p.V = V;
  if (wp.pairs_cap > 0) {
    if (dtype == SPCONV_F32) {
      dim3 grid((unsigned)wp.max_items, (unsigned)ceil_div(C_in, 64), (unsigned)ceil_div(C_out, 64));
      hipLaunchKernelGGL(k_wgrad_f32, grid, dim3(256), 0, st, p);
    } else {
      // 128 x 128 tiles as soon as a 64 x 64 tile would gather every pair's rows more than once
      // (and 32 x 32 tiles for layers of at most 32 channels, whose rows would otherwise be half padding)
      const int tile = (C_in > 64 || C_out > 64) ? 128 : ((C_in > 32 || C_out > 32) ? 64 : 32);
      const unsigned tiles = (unsigned)(ceil_div(C_in, tile) * ceil_div(C_out, tile));
      const unsigned gx = (unsigned)std::min<int64_t>(wp.max_items, std::max<unsigned>(64u, 512u / tiles));
      dim3 grid(gx, (unsigned)ceil_div(C_in, tile), (unsigned)ceil_div(C_out, tile));
      const size_t smem = (size_t)2 * 2 * WG_BK * (tile + 16) * 2;
      static std::atomic<bool> attr_set{false};  // (set twice by racing threads at worst: the calls are idempotent)
      if (!attr_set.load(std::memory_order_acquire)) {
        SPC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_wgrad<_Float16, 128>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)((size_t)8 * WG_BK * 144)));
        SPC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_wgrad<__bf16, 128>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)((size_t)8 * WG_BK * 144)));
        attr_set.store(true, std::memory_order_release);
      }
      if (dtype == SPCONV_F16) {
        if (tile == 32) hipLaunchKernelGGL((k_wgrad<_Float16, 32>), grid, dim3(256), smem, st, p);
        else if (tile == 64) hipLaunchKernelGGL((k_wgrad<_Float16, 64>), grid, dim3(256), smem, st, p);
        else hipLaunchKernelGGL((k_wgrad<_Float16, 128>), grid, dim3(256), smem, st, p);
      } else {
        if (tile == 32) hipLaunchKernelGGL((k_wgrad<__bf16, 32>), grid, dim3(256), smem, st, p);
        else if (tile == 64) hipLaunchKernelGGL((k_wgrad<__bf16, 64>), grid, dim3(256), smem, st, p);
        else hipLaunchKernelGGL((k_wgrad<__bf16, 128>), grid, dim3(256), smem, st, p);
      }
    }
    SPC_LAUNCH_CHECK();
  }
  dim3 rgrid((unsigned)ceil_div(elems / 4, 64), (unsigned)V);
  hipLaunchKernelGGL(k_wgrad_reduce, rgrid, dim3(256), 0, st, km->scratch.as<float>(), wp.item_seg.as<int>(), elems,
                     dweights);
  SPC_LAUNCH_CHECK();
  return SPCONV_OK;
}

}  // namespace spc
