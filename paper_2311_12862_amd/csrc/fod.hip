// Fetch-on-demand dataflow (Section 2.2.2) for forward and input gradient, block-fused over the
// kernel offsets: the second dataflow of the design space (Sections 4.1, 6.1).
//
// The map is walked in its weight-stationary form, the per-offset pair lists
// M_delta = {(n, j) : M[n][k] = j} that the weight-gradient kernel also uses, cut into work
// items of at most BM pairs of one offset.  A workgroup takes one item and BN output channels:
// it fetches the BM input rows of its pairs on demand (raw buffer loads, one 64-channel chunk
// ahead of the matrix cores, staged through LDS), multiplies them by the matching chunk of
// W[k] (forward) or W[k]^T (input gradient), and adds the BM x BN products to the rows of an
// fp32 accumulator with atomic adds: outputs reached through several offsets are written by
// several workgroups, which is the write-back contention the paper names.  No multiply is
// spent on an absent neighbour; the price is sum_k |M_k| / N_out times the output traffic,
// the zero-fill of the accumulator and one rounding pass to the output type.
//
// Every access a map entry steers goes through a buffer descriptor (gathered rows, pair
// list, accumulator), so a wrong index reads zeros or drops the add instead of faulting; the
// offsets of the adds are always multiples of four bytes.
#include "common.h"

#include <algorithm>

namespace spc {
namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

struct FodParams {
  const void* feats;     // gathered tensor: x [n_in][C_in] (forward) or dy [n_out][C_out] (input gradient)
  const void* weights;   // [V][C_in][C_out]
  float* acc;            // [rows_dst][c_out] fp32, zero before the launch
  const int2* pairs;     // (output row n, input row j), offset-major
  const WgradItem* items;
  const int* item_seg;   // [V] = number of items
  unsigned feats_bytes, pairs_bytes, acc_bytes;
  int V, C_in, C_out;
  int c_red, c_out;      // reduced / produced channel counts
  int dgrad;
};

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

template <int BM, int BN, int KC> struct FodSmem {
  static constexpr int LDA = KC + 16;  // rows with the reduction index contiguous; a pitch of 32 B mod 64 B keeps the
                                       // 16-byte fragment reads of 8 rows x 2 column groups (one LDS pass) on distinct banks
  static constexpr int LDB = BN + 16;  // forward weight rows: output channel contiguous; pitch = 8 words mod 32
  static constexpr size_t a_bytes = (size_t)BM * LDA * 2;
  static constexpr size_t b_fwd = (size_t)KC * LDB * 2, b_dgrad = (size_t)BN * LDA * 2;
  static constexpr size_t b_bytes = b_fwd > b_dgrad ? b_fwd : b_dgrad;
  static constexpr size_t total = a_bytes + b_bytes + (size_t)2 * BM * 4;
};

template <typename T, int BM, int BN, int KC>
__global__ void __launch_bounds__(256) k_fod(const FodParams p) {
  typedef FodSmem<BM, BN, KC> S;
  typedef typename Mfma<T>::vec vec8;
  constexpr int LDA = S::LDA, LDB = S::LDB;
  constexpr int WM = BM / 2, WN = BN / 2;  // the four waves tile the BM x BN products 2 x 2
  constexpr int MB = WM / 16, NB = WN / 16;
  constexpr int SEG = KC / 8;              // 16-byte segments per staged row
  constexpr int A_RPP = 256 / SEG;
  constexpr int A_PASSES = BM / A_RPP;
  constexpr int B_PASSES = (KC * BN / 8 + 255) / 256;
  constexpr int BF_RPP = 2048 / BN;        // forward: reduction rows covered per pass

  const int item_id = blockIdx.x;
  if (item_id >= p.item_seg[p.V]) return;  // the grid is sized by a bound on the item count

  extern __shared__ __align__(16) unsigned char smem_f[];
  unsigned short* As = reinterpret_cast<unsigned short*>(smem_f);
  unsigned short* Bs = reinterpret_cast<unsigned short*>(smem_f + S::a_bytes);
  int* srcS = reinterpret_cast<int*>(smem_f + S::a_bytes + S::b_bytes);
  int* dstS = srcS + BM;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave >> 1, wave_n = wave & 1;
  const int n0 = blockIdx.y * BN;
  const WgradItem item = p.items[item_id];
  int cnt = item.pair_end - item.pair_begin;
  if (cnt > BM) cnt = BM;  // items are cut to at most BM pairs by the plan
  const int c_red = p.c_red;
  const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(p.feats, p.feats_bytes);
  const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(p.weights, (unsigned)((size_t)p.V * p.C_in * p.C_out * 2));
  const __amdgpu_buffer_rsrc_t p_rsrc = make_rsrc(p.pairs, p.pairs_bytes);
  const __amdgpu_buffer_rsrc_t o_rsrc = make_rsrc(p.acc, p.acc_bytes);
  const unsigned row_bytes = (unsigned)c_red * 2u;
  const unsigned wk = (unsigned)item.k * (unsigned)(p.C_in * p.C_out) * 2u;

  // the pairs of this item: row to fetch, row to add to (-1 past the end of the item)
  for (int r = tid; r < BM; r += 256) {
    const bool live = r < cnt;
    const int2 pr = buf_load8(p_rsrc, live ? (unsigned)(item.pair_begin + r) * 8u : 0xFFFFFFFFu);
    srcS[r] = live ? (p.dgrad ? pr.x : pr.y) : -1;
    dstS[r] = live ? (p.dgrad ? pr.y : pr.x) : -1;
  }
  __syncthreads();

  f32x4 acc[MB][NB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int n_chunks = (c_red + KC - 1) / KC;
  uint4 ra[A_PASSES], rb[B_PASSES];
  const int a_seg = tid % SEG, a_row = tid / SEG;

  auto load_regs = [&](int chunk) {
    const unsigned col = (unsigned)(chunk * KC + a_seg * 8);
#pragma unroll
    for (int ps = 0; ps < A_PASSES; ++ps) {
      const int idx = srcS[a_row + ps * A_RPP];
      // idx = -1 wraps to just below 2^32: out of range, reads zeros
      ra[ps] = buf_load16(x_rsrc, col < (unsigned)c_red ? (unsigned)idx * row_bytes + col * 2u : 0xFFFFFFFFu);
    }
    if (!p.dgrad) {  // rows of W[k]: reduction channel ci, 8 output channels per load
      const int nseg = tid % (BN / 8), kk0 = tid / (BN / 8);
#pragma unroll
      for (int ps = 0; ps < B_PASSES; ++ps) {
        const int kk = kk0 + ps * BF_RPP;
        const int ci = chunk * KC + kk, co = n0 + nseg * 8;
        const bool ok = kk < KC && ci < p.C_in && co < p.C_out;
        rb[ps] = buf_load16(w_rsrc, ok ? wk + (unsigned)(ci * p.C_out + co) * 2u : 0xFFFFFFFFu);
      }
    } else {  // rows of W[k]: produced channel ci, 8 reduction channels (co) per load
#pragma unroll
      for (int ps = 0; ps < B_PASSES; ++ps) {
        const int n = a_row + ps * A_RPP;
        const int ci = n0 + n, co = chunk * KC + a_seg * 8;
        const bool ok = n < BN && ci < p.C_in && co < p.C_out;
        rb[ps] = buf_load16(w_rsrc, ok ? wk + (unsigned)(ci * p.C_out + co) * 2u : 0xFFFFFFFFu);
      }
    }
  };
  auto store_lds = [&]() {
#pragma unroll
    for (int ps = 0; ps < A_PASSES; ++ps)
      *reinterpret_cast<uint4*>(As + (a_row + ps * A_RPP) * LDA + a_seg * 8) = ra[ps];
    if (!p.dgrad) {  // stored as loaded, [ci][co]; the transposing LDS read does the rest
      const int nseg = tid % (BN / 8), kk0 = tid / (BN / 8);
#pragma unroll
      for (int ps = 0; ps < B_PASSES; ++ps) {
        const int kk = kk0 + ps * BF_RPP;
        if (kk < KC) *reinterpret_cast<uint4*>(Bs + kk * LDB + nseg * 8) = rb[ps];
      }
    } else {
#pragma unroll
      for (int ps = 0; ps < B_PASSES; ++ps) {
        const int n = a_row + ps * A_RPP;
        if (n < BN) *reinterpret_cast<uint4*>(Bs + n * LDA + a_seg * 8) = rb[ps];
      }
    }
  };

  load_regs(0);
  store_lds();
  __syncthreads();

  const int fa = lane & 15, fg = lane >> 4;
  for (int chunk = 0; chunk < n_chunks; ++chunk) {
    // the next chunk travels while this one is on the matrix cores (past the last chunk the
    // channel test makes every load out of range: zeros, no traffic)
    load_regs(chunk + 1);
    const unsigned short* a = As + (wave_m * WM + fa) * LDA + fg * 8;
#pragma unroll
    for (int ks = 0; ks < KC / 32; ++ks) {
      vec8 bf[NB];
      if (!p.dgrad) {
        // 16 lanes fetch a 4 x 16 block of [ci][co] and each receives one column: 4 reduction
        // steps of its output channel; two reads give the lane's 8 steps (ci = 8*fg .. 8*fg+7)
        const unsigned short* b = Bs + (ks * 32 + 8 * fg + (fa >> 2)) * LDB + wave_n * WN + 4 * (fa & 3);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4*)(b + nb * 16));
          const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4*)(b + nb * 16 + 4 * LDB));
          const s16x8 v = {lo4[0], lo4[1], lo4[2], lo4[3], hi4[0], hi4[1], hi4[2], hi4[3]};
          bf[nb] = __builtin_bit_cast(vec8, v);
        }
      } else {
        const unsigned short* b = Bs + (wave_n * WN + fa) * LDA + fg * 8;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) bf[nb] = *reinterpret_cast<const vec8*>(b + nb * 16 * LDA + ks * 32);
      }
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        if (wave_m * WM + mb * 16 < cnt) {  // blocks past the item's last pair hold zeros only
          const vec8 af = *reinterpret_cast<const vec8*>(a + mb * 16 * LDA + ks * 32);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = Mfma<T>::run(af, bf[nb], acc[mb][nb]);
        }
      }
    }
    __syncthreads();  // everyone is done reading this chunk's tiles
    store_lds();
    __syncthreads();
  }

  // scatter: the lane holds rows 4*(lane/16)+r, column lane%16 of each 16 x 16 block; 16 lanes add
  // to 64 contiguous bytes of one accumulator row
  const int c_out = p.c_out;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    if (wave_m * WM + mb * 16 >= cnt) continue;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int drow = dstS[wave_m * WM + mb * 16 + (lane >> 4) * 4 + r];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const int col = n0 + wave_n * WN + nb * 16 + (lane & 15);
        // Lanes of rows past the item's end (-1) and of columns past the tensor issue nothing.
        // (An atomic needs a 4-byte aligned address whether or not it is in range, so the
        // out-of-range offset 0xFFFFFFFF that serves the loads must never reach one.)
        if (drow >= 0 && col < c_out)
          __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_f32(
              acc[mb][nb][r], o_rsrc, ((unsigned)drow * (unsigned)c_out + (unsigned)col) * 4u, 0, 0);
      }
    }
  }
}

// fp32 fetch-on-demand (the precision of the paper's own dataflow comparison, Section 6.1): plain
// FMA arithmetic, an item of up to 64 pairs x 64 output channels per workgroup, 4 x 4 products per
// thread, the reduction in chunks of 16 channels through LDS; products added to the accumulator's
// rows with the same atomics as the 16-bit kernel.
constexpr int FF_BM = 64, FF_BN = 64, FF_KC = 16;
__global__ void __launch_bounds__(256) k_fod_f32(const FodParams p) {
  __shared__ float As[FF_BM][FF_KC + 1];
  __shared__ float Bs[FF_KC][FF_BN + 4];
  __shared__ int srcS[FF_BM], dstS[FF_BM];
  const int item_id = blockIdx.x;
  if (item_id >= p.item_seg[p.V]) return;  // the grid is sized by a bound on the item count
  const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
  const int n0 = blockIdx.y * FF_BN;
  const WgradItem item = p.items[item_id];
  int cnt = item.pair_end - item.pair_begin;
  if (cnt > FF_BM) cnt = FF_BM;  // items are cut to at most 64 pairs by the plan
  const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(p.feats, p.feats_bytes);
  const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(p.weights, (unsigned)((size_t)p.V * p.C_in * p.C_out * 4));
  const __amdgpu_buffer_rsrc_t p_rsrc = make_rsrc(p.pairs, p.pairs_bytes);
  const __amdgpu_buffer_rsrc_t o_rsrc = make_rsrc(p.acc, p.acc_bytes);
  const int c_red = p.c_red;
  const unsigned row_bytes = (unsigned)c_red * 4u;
  const unsigned wk = (unsigned)item.k * (unsigned)(p.C_in * p.C_out) * 4u;
  if (tid < FF_BM) {
    const bool live = tid < cnt;
    const int2 pr = buf_load8(p_rsrc, live ? (unsigned)(item.pair_begin + tid) * 8u : 0xFFFFFFFFu);
    srcS[tid] = live ? (p.dgrad ? pr.x : pr.y) : -1;
    dstS[tid] = live ? (p.dgrad ? pr.y : pr.x) : -1;
  }
  __syncthreads();
  float acc[4][4] = {};
  const int n_chunks = (c_red + FF_KC - 1) / FF_KC;
  for (int chunk = 0; chunk < n_chunks; ++chunk) {
    {  // A: 64 rows x 16 floats, one 16-byte load per thread (a dead row or channel reads zeros)
      const int r = tid / 4, seg = tid % 4;
      const int idx = srcS[r];
      const unsigned col = (unsigned)(chunk * FF_KC + seg * 4);
      const uint4 v = buf_load16(x_rsrc, col < (unsigned)c_red ? (unsigned)idx * row_bytes + col * 4u : 0xFFFFFFFFu);
      As[r][seg * 4 + 0] = __uint_as_float(v.x);
      As[r][seg * 4 + 1] = __uint_as_float(v.y);
      As[r][seg * 4 + 2] = __uint_as_float(v.z);
      As[r][seg * 4 + 3] = __uint_as_float(v.w);
    }
    if (!p.dgrad) {  // B[kk][n] = W[k][ci = chunk*KC + kk][co = n0 + n]
      const int kk = tid / 16, n4 = (tid % 16) * 4;
      const int ci = chunk * FF_KC + kk, co = n0 + n4;
      const uint4 v = buf_load16(w_rsrc, (ci < p.C_in && co < p.C_out) ? wk + (unsigned)(ci * p.C_out + co) * 4u : 0xFFFFFFFFu);
      Bs[kk][n4 + 0] = __uint_as_float(v.x);
      Bs[kk][n4 + 1] = __uint_as_float(v.y);
      Bs[kk][n4 + 2] = __uint_as_float(v.z);
      Bs[kk][n4 + 3] = __uint_as_float(v.w);
    } else {  // B[kk][n] = W[k][ci = n0 + n][co = chunk*KC + kk]
      const int n = tid / 4, kk4 = (tid % 4) * 4;
      const int ci = n0 + n, co = chunk * FF_KC + kk4;
      const uint4 v = buf_load16(w_rsrc, (ci < p.C_in && co < p.C_out) ? wk + (unsigned)(ci * p.C_out + co) * 4u : 0xFFFFFFFFu);
      Bs[kk4 + 0][n] = __uint_as_float(v.x);
      Bs[kk4 + 1][n] = __uint_as_float(v.y);
      Bs[kk4 + 2][n] = __uint_as_float(v.z);
      Bs[kk4 + 3][n] = __uint_as_float(v.w);
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < FF_KC; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[ty * 4 + i][kk];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  const int c_out = p.c_out;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int drow = dstS[ty * 4 + i];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + tx * 4 + j;
      // (lanes of dead rows and of columns past the tensor issue nothing: an atomic needs an aligned
      // address whether or not it is in range)
      if (drow >= 0 && col < c_out)
        __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_f32(acc[i][j], o_rsrc,
                                                        ((unsigned)drow * (unsigned)c_out + (unsigned)col) * 4u, 0, 0);
    }
  }
}

__global__ void __launch_bounds__(256) k_zero_f4(float4* __restrict__ dst, long long n4) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride)
    dst[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

template <typename T, int BM, int BN, int KC>
int launch_fod(const FodParams& p, dim3 grid, hipStream_t st) {
  typedef FodSmem<BM, BN, KC> S;
  static_assert(S::total <= 64 * 1024, "fits the default dynamic LDS limit");
  hipLaunchKernelGGL((k_fod<T, BM, BN, KC>), grid, dim3(256), S::total, st, p);
  SPC_LAUNCH_CHECK();
  return SPCONV_OK;
}

template <typename T, int BM, int BN>
int launch_fod_kc(const FodParams& p, int kc, dim3 grid, hipStream_t st) {
  return kc == 64 ? launch_fod<T, BM, BN, 64>(p, grid, st) : launch_fod<T, BM, BN, 32>(p, grid, st);
}

template <typename T, int BM>
int launch_fod_bn(const FodParams& p, int bn, int kc, dim3 grid, hipStream_t st) {
  switch (bn) {
    case 32: return launch_fod_kc<T, BM, 32>(p, kc, grid, st);
    case 64: return launch_fod_kc<T, BM, 64>(p, kc, grid, st);
    case 128: return launch_fod_kc<T, BM, 128>(p, kc, grid, st);
  }
  return SPCONV_EINVAL;
}

template <typename T>
int launch_fod_bm(const FodParams& p, int bm, int bn, int kc, dim3 grid, hipStream_t st) {
  switch (bm) {
    case 64: return launch_fod_bn<T, 64>(p, bn, kc, grid, st);
    case 128: return launch_fod_bn<T, 128>(p, bn, kc, grid, st);
  }
  return SPCONV_EINVAL;
}

}  // namespace

bool fod_supported(const spconv_kmap* km, int dgrad, int C_in, int C_out, spconv_dtype dtype) {
  if (dtype != SPCONV_F16 && dtype != SPCONV_BF16 && dtype != SPCONV_F32) return false;
  const int64_t rows_src = dgrad ? km->n_out : km->n_in, rows_dst = dgrad ? km->n_in : km->n_out;
  const int c_red = dgrad ? C_out : C_in, c_dst = dgrad ? C_in : C_out;
  const uint64_t e = dtype == SPCONV_F32 ? 4 : 2;
  // buffer descriptors address 32 bits
  return (uint64_t)rows_src * c_red * e < 0xFFFFC000ull && (uint64_t)km->V * C_in * C_out * e < 0xFFFFC000ull && (uint64_t)rows_dst * c_dst * 4 < 0xFFFFC000ull &&
         (uint64_t)km->n_out * km->V * 8 < 0xFFFFC000ull;
}

int fod_run(spconv_kmap* km, const WgradPlan& wp, const IgemmArgs& a, int tile_m, void* dst, hipStream_t st) {
  if (tile_m != 64 && tile_m != 128) return SPCONV_EINVAL;
  if (a.dtype == SPCONV_F32 && tile_m != FF_BM) return SPCONV_EINVAL;  // the fp32 kernel has one tile shape
  if (wp.target_pairs != tile_m) return SPCONV_EINVAL;  // one work item is one tile of pairs
  if (wp.max_items >= (1 << 20)) return SPCONV_EINVAL;  // the plan's item table is capped there
  if (!fod_supported(km, a.dgrad, a.C_in, a.C_out, a.dtype)) return SPCONV_EINVAL;
  const int64_t rows_src = a.dgrad ? km->n_out : km->n_in, rows_dst = a.dgrad ? km->n_in : km->n_out;
  if (rows_dst == 0) return SPCONV_OK;
  FodParams p{};
  p.c_red = a.dgrad ? a.C_out : a.C_in;
  p.c_out = a.dgrad ? a.C_in : a.C_out;
  const size_t acc_bytes = (size_t)rows_dst * p.c_out * sizeof(float);
  SPC_TRY(km->scratch.reserve(acc_bytes));
  {
    const long long n4 = (long long)(acc_bytes / 16);  // channel counts are multiples of 8
    const unsigned blocks = (unsigned)std::min<long long>(ceil_div(n4, 256), 4096);
    hipLaunchKernelGGL(k_zero_f4, dim3(blocks), dim3(256), 0, st, km->scratch.as<float4>(), n4);
    SPC_LAUNCH_CHECK();
  }
  if (wp.pairs_cap > 0 && rows_src > 0) {
    p.feats = a.feats;
    p.weights = a.weights;
    p.acc = km->scratch.as<float>();
    p.pairs = wp.pairs.as<int2>();
    p.items = wp.items.as<WgradItem>();
    p.item_seg = wp.item_seg.as<int>();
    p.feats_bytes = (unsigned)((uint64_t)rows_src * p.c_red * (a.dtype == SPCONV_F32 ? 4 : 2));
    p.pairs_bytes = (unsigned)((uint64_t)wp.pairs_cap * 8);
    p.acc_bytes = (unsigned)acc_bytes;
    p.V = km->V;
    p.C_in = a.C_in;
    p.C_out = a.C_out;
    p.dgrad = a.dgrad;
    if (a.dtype == SPCONV_F32) {
      dim3 grid((unsigned)wp.max_items, (unsigned)ceil_div(p.c_out, FF_BN));
      hipLaunchKernelGGL(k_fod_f32, grid, dim3(256), 0, st, p);
      SPC_LAUNCH_CHECK();
      return split_reduce(km->scratch.as<float>(), 1, rows_dst, p.c_out, a.dtype, dst, st);
    }
    int bn = a.tile_n;
    if (bn == 0) bn = p.c_out <= 32 ? 32 : (p.c_out <= 64 ? 64 : 128);
    if (bn != 32 && bn != 64 && bn != 128) return SPCONV_EINVAL;
    const int kc = (p.c_red % 64 == 0) ? 64 : 32;
    dim3 grid((unsigned)wp.max_items, (unsigned)ceil_div(p.c_out, bn));
    if (a.dtype == SPCONV_F16) SPC_TRY(launch_fod_bm<_Float16>(p, tile_m, bn, kc, grid, st));
    else SPC_TRY(launch_fod_bm<__bf16>(p, tile_m, bn, kc, grid, st));
  }
  return split_reduce(km->scratch.as<float>(), 1, rows_dst, p.c_out, a.dtype, dst, st);
}

}  // namespace spc
