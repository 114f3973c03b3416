// Implicit-GEMM sparse convolution kernels (Sections 2.2.3, 3.1, 3.2, 4.1):
// forward and input-gradient with workgroup tiles, for channel counts whose
// weights do not fit in LDS, plus the fp32 path.
//
// One workgroup owns BM consecutive rows of the (possibly bitmask-sorted)
// output-stationary map and BN output channels.  The tile's map slab is copied
// to LDS once (the addressing that Section 3.2 hoists out of the inner loop),
// the loop over kernel offsets visits only offsets whose bit is set in the
// tile's mask, and every 16-row MFMA block of a wave skips offsets none of its
// rows has (the lock-step unit of Section 2.2.3 is a 16-row block here, not a
// 32-thread warp).  Gathered feature rows and the weight slice of the next step
// are loaded into registers (raw buffer loads: an absent neighbour is an
// out-of-range offset that reads as zero, no branch) while the current step
// runs on the matrix cores out of a single LDS stage; the small LDS footprint
// lets several workgroups share a CU and hide each other's load latency.
// Forward weights are stored as they arrive ([ci][co]) and read with the
// transposing LDS read, so no software transpose is needed.  The map is padded
// to whole tiles so that no map access needs a bounds check (Section 3.2).
#include "common.h"

#include <atomic>

namespace spc {
namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct IgemmParams {
  const void* feats;
  const void* weights;
  void* out;
  float* partial;
  const int* map[kMaxSplit];
  const int* perm[kMaxSplit];
  const unsigned* tilemask[kMaxSplit];
  int lo[kMaxSplit], width[kMaxSplit];
  long long rows;
  int parts, V;
  int c_red, c_out;  // reduced / produced channel counts
  int C_in, C_out;   // of the layer
  int dgrad, mirror;
  int heavy_first;   // sorted maps: tiles late in the sort order hold the most offsets; start them first
  unsigned feats_bytes;  // size of the gathered tensor (16-bit kernels address it through a buffer descriptor)
  // sizes of the tables that a tile index reaches (read through range-checked buffer descriptors:
  // beyond the end zeros, no access): each part's map, the permutation (rows_pad entries), the tile masks
  unsigned map_part_bytes[kMaxSplit];
  unsigned rows_pad_bytes, tiles_bytes;
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

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

// Raw buffer loads: an absent neighbour (index -1) or a channel past the end becomes an
// out-of-range offset, which returns zeros without touching memory and without a branch.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ uint4 buf_load16(__amdgpu_buffer_rsrc_t r, unsigned byte_off) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// LDS plan of the tiled kernel.  One stage of operands (the next stage waits in registers):
// more workgroups fit on a CU, and they hide each other's load latency.
// Pitches (in 2-byte elements) of the rows whose reduction index is contiguous (gathered rows, and
// the weight rows of the input gradient).  Measured on gfx950: one pass of a 16-byte LDS read
// serves 8 rows x 2 column groups, so a pitch of 32 B mod 64 B (KC + 16 elements) is free of bank
// conflicts (19 clk per wave instruction with four waves reading) while KC + 8 costs two passes
// (32 clk).  The wider pitch is used unless it would cost a resident workgroup per CU.
template <int BM, int BN, int KC, bool DGRAD> struct IgemmSmem {
  static constexpr int LDB = BN + 16;  // forward weight rows: output channel contiguous; pitch = 8 words mod 32
  static constexpr size_t map_bytes = (size_t)BM * 27 * 4;
  static constexpr size_t perm_bytes = (size_t)BM * 4;
  static constexpr size_t kLdsPerCu = 160 * 1024;
  static constexpr size_t total_with(int lda, int ldbd) {
    return (size_t)BM * lda * 2 + (DGRAD ? (size_t)BN * ldbd * 2 : (size_t)KC * LDB * 2) + map_bytes + perm_bytes;
  }
  static constexpr size_t fit(int lda, int ldbd) { return kLdsPerCu / total_with(lda, ldbd); }
  static constexpr int LDA = fit(KC + 16, KC + 8) == fit(KC + 8, KC + 8) ? KC + 16 : KC + 8;
  static constexpr int LDBD = fit(LDA, KC + 16) == fit(LDA, KC + 8) ? KC + 16 : KC + 8;
  static constexpr size_t a_bytes = (size_t)BM * LDA * 2;
  static constexpr size_t b_bytes = DGRAD ? (size_t)BN * LDBD * 2 : (size_t)KC * LDB * 2;
  static constexpr size_t total = a_bytes + b_bytes + map_bytes + perm_bytes;
};

// DGRAD is a template parameter: as a run-time flag the compiler issued the LDS reads of both
// operand layouts and awaited the unused ones.
template <typename T, int BM, int BN, int KC, int NW, bool DGRAD>
__global__ void __launch_bounds__(NW * 64) k_igemm(const IgemmParams p) {
  typedef IgemmSmem<BM, BN, KC, DGRAD> S;
  typedef typename Mfma<T>::vec vec8;
  constexpr int LDA = S::LDA, LDB = S::LDB, LDBD = S::LDBD;
  // the NW (4 or 8) waves tile the workgroup's BM x BN outputs (NW/2) x 2
  constexpr int NT = NW * 64;        // threads
  constexpr int WM = BM / (NW / 2);  // rows per wave
  constexpr int WN = BN / 2;         // columns per wave
  constexpr int MB = WM / 16;        // 16-row MFMA blocks per wave
  constexpr int NB = WN / 16;        // 16-column MFMA blocks per wave
  constexpr int SEG = KC / 8;   // 16-byte segments per staged A row
  constexpr int A_RPP = NT / SEG;
  constexpr int A_PASSES = BM / A_RPP;
  constexpr int B_PASSES = (KC * BN / 8 + NT - 1) / NT;
  constexpr int BF_RPP = NT * 8 / BN;  // forward: reduction rows covered per pass

  extern __shared__ __align__(16) unsigned char smem[];
  unsigned short* As = reinterpret_cast<unsigned short*>(smem);
  unsigned short* Bs = reinterpret_cast<unsigned short*>(smem + S::a_bytes);
  int* mapS = reinterpret_cast<int*>(smem + S::a_bytes + S::b_bytes);
  int* permS = reinterpret_cast<int*>(smem + S::a_bytes + S::b_bytes + S::map_bytes);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave >> 1, wave_n = wave & 1;
  const int part = blockIdx.z;
  const long long tile = p.heavy_first ? (long long)gridDim.x - 1 - blockIdx.x : blockIdx.x;
  const int n0 = blockIdx.y * BN;
  const int width = p.width[part], lo = p.lo[part];
  const long long row0 = tile * BM;
  const unsigned tmask = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(make_rsrc(p.tilemask[part], p.tiles_bytes),
                                                                       (unsigned)tile * 4u, 0, 0);
  const int c_red = p.c_red;
  const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(p.feats, p.feats_bytes);
  const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(p.weights, (unsigned)((size_t)p.V * p.C_in * p.C_out * 2));
  const unsigned row_bytes = (unsigned)c_red * 2u, slice_bytes = (unsigned)(p.C_in * p.C_out) * 2u;

  {  // map slab and output rows of this tile: every load is issued before the first one is awaited
    // (the slab is BM * width consecutive ints; tiles start on 256-byte boundaries)
    // through a buffer descriptor over the part's map that ends with the slab: a load past the
    // end returns zeros, so no load sits behind a branch and all of them are in flight together
    constexpr int SLAB_IT = (BM * 27 / 4 + NT - 1) / NT;
    const int n4 = BM * width / 4;
    const unsigned slab_begin = (unsigned)(row0 * width) * 4u, slab_end = slab_begin + (unsigned)n4 * 16u;
    const __amdgpu_buffer_rsrc_t m_rsrc =
        make_rsrc(p.map[part], slab_end < p.map_part_bytes[part] ? slab_end : p.map_part_bytes[part]);
    uint4 slab[SLAB_IT];
#pragma unroll
    for (int i = 0; i < SLAB_IT; ++i) slab[i] = buf_load16(m_rsrc, slab_begin + (unsigned)(tid + NT * i) * 16u);
    const int* pm = p.perm[part];
    const __amdgpu_buffer_rsrc_t p_rsrc = make_rsrc(pm, p.rows_pad_bytes);
    for (int r = tid; r < BM; r += NT) {
      const long long g = row0 + r;
      permS[r] = pm ? __builtin_amdgcn_raw_buffer_load_b32(p_rsrc, (unsigned)g * 4u, 0, 0) : (g < p.rows ? (int)g : -1);
    }
#pragma unroll
    for (int i = 0; i < SLAB_IT; ++i) {
      const int e = tid + NT * i;
      if (e < n4) reinterpret_cast<uint4*>(mapS)[e] = slab[i];
    }
  }
  __syncthreads();

  // per-block offset masks: bit c set iff some row of the 16-row block has neighbour c
  unsigned blk_mask[MB];
  {
#pragma unroll
    for (int m0 = 0; m0 < WM; m0 += 64) {  // 64 rows per round, one per lane
      unsigned bits = 0;
      if (m0 + lane < WM) {
        // all 27 reads are issued at once; entries past `width` belong to the next row or to the
        // unused end of the slab's LDS and are masked off
        const int* mr = mapS + (wave_m * WM + m0 + lane) * width;
#pragma unroll
        for (int c = 0; c < 27; ++c) bits |= (mr[c] >= 0 ? 1u : 0u) << c;
        bits &= (1u << width) - 1u;
      }
      bits |= __shfl_xor(bits, 1);
      bits |= __shfl_xor(bits, 2);
      bits |= __shfl_xor(bits, 4);
      bits |= __shfl_xor(bits, 8);
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (m0 / 16 + j < MB) blk_mask[m0 / 16 + j] = __builtin_amdgcn_readlane(bits, j * 16);
    }
  }

  f32x4 acc[MB][NB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int n_chunks = (c_red + KC - 1) / KC;
  const int total = __popc(tmask) * n_chunks;

  // operands on their way: the weights of the next step, the gathered rows of the next two
  uint4 ra0[A_PASSES] = {}, ra1[A_PASSES] = {}, rb0[B_PASSES] = {};
  const int a_seg = tid % SEG, a_row = tid / SEG;

  auto load_a = [&](uint4* ra, int c, int chunk) {
    // all map entries are read before the first load is issued (one LDS latency, not one per load)
    int idx[A_PASSES];
#pragma unroll
    for (int ps = 0; ps < A_PASSES; ++ps) idx[ps] = mapS[(a_row + ps * A_RPP) * width + c];
    const unsigned col = (unsigned)(chunk * KC + a_seg * 8);
#pragma unroll
    for (int ps = 0; ps < A_PASSES; ++ps) {
      // idx = -1 wraps to just below 2^32: out of range
      ra[ps] = buf_load16(x_rsrc, col < (unsigned)c_red ? (unsigned)idx[ps] * row_bytes + col * 2u : 0xFFFFFFFFu);
    }
  };
  auto load_b = [&](uint4* rb, int c, int chunk) {
    const int k = lo + c;
    const unsigned wk = (unsigned)(p.mirror ? p.V - 1 - k : k) * slice_bytes;
    if constexpr (!DGRAD) {  // rows of W[k]: reduction channel ci, 8 output channels per load
      const int nseg = tid % (BN / 8), kk0 = tid / (BN / 8);
#pragma unroll
      for (int ps = 0; ps < B_PASSES; ++ps) {
        const int kk = kk0 + ps * BF_RPP;
        const int ci = chunk * KC + kk, co = n0 + nseg * 8;
        const bool ok = kk < KC && ci < p.C_in && co < p.C_out;
        rb[ps] = buf_load16(w_rsrc, ok ? wk + (unsigned)(ci * p.C_out + co) * 2u : 0xFFFFFFFFu);
      }
    } else {  // rows of W[k]: output channel n = ci, 8 reduction channels (co) per load
#pragma unroll
      for (int ps = 0; ps < B_PASSES; ++ps) {
        const int n = a_row + ps * A_RPP;
        const int ci = n0 + n, co = chunk * KC + a_seg * 8;
        const bool ok = n < BN && ci < p.C_in && co < p.C_out;
        rb[ps] = buf_load16(w_rsrc, ok ? wk + (unsigned)(ci * p.C_out + co) * 2u : 0xFFFFFFFFu);
      }
    }
  };

  auto store_lds = [&](const uint4* ra, const uint4* rb) {
#pragma unroll
    for (int ps = 0; ps < A_PASSES; ++ps)
      *reinterpret_cast<uint4*>(As + (a_row + ps * A_RPP) * LDA + a_seg * 8) = ra[ps];
    if constexpr (!DGRAD) {  // forward: stored as loaded, [ci][co]; the transposing LDS read does the rest
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
        if (n < BN) *reinterpret_cast<uint4*>(Bs + n * LDBD + a_seg * 8) = rb[ps];
      }
    }
  };

  const int fa = lane & 15, fg = lane >> 4;
  // one step (offset c, one chunk of the reduction) out of the LDS tiles
  auto compute = [&](int c) {
    const unsigned short* a = As + (wave_m * WM + fa) * LDA + fg * 8;
#pragma unroll
    for (int ks = 0; ks < KC / 32; ++ks) {
      vec8 bf[NB];
      if constexpr (!DGRAD) {
        // 16 lanes fetch a 4 x 16 block of [ci][co] and each receives one column: 4 reduction
        // steps of its output channel; two reads give the lane's 8 steps (ci = 8*fg .. 8*fg+7)
        const unsigned short* b = Bs + (ks * 32 + 8 * fg + (fa >> 2)) * LDB + wave_n * WN + 4 * (fa & 3);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4*)(b + nb * 16));
          const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4*)(b + nb * 16 + 4 * LDB));
          typedef short s16x8 __attribute__((ext_vector_type(8)));
          const s16x8 v = {lo4[0], lo4[1], lo4[2], lo4[3], hi4[0], hi4[1], hi4[2], hi4[3]};
          bf[nb] = __builtin_bit_cast(vec8, v);
        }
      } else {
        const unsigned short* b = Bs + (wave_n * WN + fa) * LDBD + fg * 8;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) bf[nb] = *reinterpret_cast<const vec8*>(b + nb * 16 * LDBD + ks * 32);
      }
      // every fragment read of the step is issued before the first MFMA waits for one (a read
      // inside the per-block branch would be awaited right where it is issued); only the
      // MFMAs of a block without this offset are skipped
      vec8 af[MB];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) af[mb] = *reinterpret_cast<const vec8*>(a + mb * 16 * LDA + ks * 32);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        if ((blk_mask[mb] >> c) & 1u) {
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = Mfma<T>::run(af[mb], bf[nb], acc[mb][nb]);
        }
      }
    }
  };

  // The steps in order: set bits of the tile mask, ascending, each with its chunks.  One step lives
  // in LDS.  The weight tile of the next step (an L2 hit) is loaded one step ahead; the gathered
  // rows, which mostly come from beyond L2, two steps ahead, alternating between two register
  // sets so that a set in flight is never copied (a copy would wait for it).
  struct Cursor {  // walks the steps
    unsigned rem;
    int c, chunk, left;
  };
  auto cursor_begin = [&]() {
    Cursor q{tmask, 0, 0, total};
    if (total > 0) {
      q.c = __ffs((int)q.rem) - 1;
      q.rem &= q.rem - 1;
    }
    return q;
  };
  auto cursor_next = [&](Cursor& q) {
    --q.left;
    if (++q.chunk == n_chunks) {
      q.chunk = 0;
      q.c = q.rem ? __ffs((int)q.rem) - 1 : 0;
      q.rem &= q.rem - 1;
    }
  };
  Cursor qa = cursor_begin(), qb = cursor_begin();  // next step whose rows / weights are to be issued
  int c_lds = 0, c_regs = 0;  // offsets of the step in LDS and of the step whose weights are in registers
  auto issue_a = [&](uint4* ra) {
    if (qa.left > 0) {
      load_a(ra, qa.c, qa.chunk);
      cursor_next(qa);
    }
  };
  auto issue_b = [&]() {
    if (qb.left > 0) {
      load_b(rb0, qb.c, qb.chunk);
      c_regs = qb.c;
      cursor_next(qb);
    }
  };
  // one step: `cur` holds the rows of the next step (issued a step ago), `nxt` receives those of
  // the step after it; returns true after the last step
  auto step = [&](uint4* cur, uint4* nxt, int it) {
    issue_b();
    issue_a(nxt);
    compute(c_lds);
    if (it + 1 >= total) return true;
    __syncthreads();  // everyone is done reading this step's tiles
    store_lds(cur, rb0);
    c_lds = c_regs;
    __syncthreads();
    return false;
  };
  if (total > 0) {
    issue_b();
    issue_a(ra0);
    issue_a(ra1);
    store_lds(ra0, rb0);
    c_lds = c_regs;
  }
  __syncthreads();
  for (int it = 0; it < total; it += 2) {
    if (step(ra1, ra0, it)) break;
    if (step(ra0, ra1, it + 1)) break;
  }

  // D layout of the 16x16 MFMA: lane holds rows 4*(lane/16)+r, column lane%16
  const int c_out = p.c_out;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int orow = permS[wave_m * WM + mb * 16 + (lane >> 4) * 4 + r];
      if (orow < 0) continue;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const int col = n0 + wave_n * WN + nb * 16 + (lane & 15);
        if (col >= c_out) continue;
        const float v = acc[mb][nb][r];
        if (p.partial)
          p.partial[((long long)part * p.rows + orow) * c_out + col] = v;
        else
          reinterpret_cast<T*>(p.out)[(long long)orow * c_out + col] = (T)v;
      }
    }
  }
}

// fp32 path: plain FMA arithmetic, 64 x 64 tile, 4 x 4 outputs per thread.
constexpr int F32_BM = 64, F32_BN = 64, F32_KC = 16;

__global__ void __launch_bounds__(256) k_igemm_f32(const IgemmParams p) {
  __shared__ float As[F32_BM][F32_KC + 1];
  __shared__ float Bs[F32_KC][F32_BN + 4];
  __shared__ int mapS[F32_BM * 27];
  __shared__ int permS[F32_BM];
  const int tid = threadIdx.x;
  const int part = blockIdx.z;
  const long long tile = blockIdx.x;
  const int n0 = blockIdx.y * F32_BN;
  const int width = p.width[part], lo = p.lo[part];
  const long long row0 = tile * F32_BM;
  const unsigned tmask = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(make_rsrc(p.tilemask[part], p.tiles_bytes),
                                                                       (unsigned)tile * 4u, 0, 0);
  const float* feats = reinterpret_cast<const float*>(p.feats);
  const float* wts = reinterpret_cast<const float*>(p.weights);
  const int c_red = p.c_red;
  {
    const __amdgpu_buffer_rsrc_t m_rsrc = make_rsrc(p.map[part], p.map_part_bytes[part]);
    const unsigned slab_begin = (unsigned)(row0 * width) * 4u;
    for (int e = tid; e < F32_BM * width; e += 256)
      mapS[e] = __builtin_amdgcn_raw_buffer_load_b32(m_rsrc, slab_begin + (unsigned)e * 4u, 0, 0);
    const int* pm = p.perm[part];
    if (tid < F32_BM) {
      const long long g = row0 + tid;
      permS[tid] = pm ? __builtin_amdgcn_raw_buffer_load_b32(make_rsrc(pm, p.rows_pad_bytes), (unsigned)g * 4u, 0, 0)
                      : (g < p.rows ? (int)g : -1);
    }
  }
  __syncthreads();
  const int ty = tid / 16, tx = tid % 16;
  float acc[4][4] = {};
  const int n_chunks = (c_red + F32_KC - 1) / F32_KC;
  unsigned m_rem = tmask;
  while (m_rem) {
    const int c = __ffs((int)m_rem) - 1;
    m_rem &= m_rem - 1;
    const int k = lo + c;
    const long long wk = (long long)(p.mirror ? p.V - 1 - k : k) * p.C_in * p.C_out;
    for (int chunk = 0; chunk < n_chunks; ++chunk) {
      {  // A: 64 rows x 16 floats, one float4 per thread
        const int r = tid / 4, seg = tid % 4;
        const int idx = mapS[r * width + c];
        const int col = chunk * F32_KC + seg * 4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (idx >= 0 && col < c_red) v = *reinterpret_cast<const float4*>(feats + (long long)idx * c_red + col);
        As[r][seg * 4 + 0] = v.x;
        As[r][seg * 4 + 1] = v.y;
        As[r][seg * 4 + 2] = v.z;
        As[r][seg * 4 + 3] = v.w;
      }
      if (!p.dgrad) {  // B[kk][n] = W[k][ci = chunk*KC + kk][co = n0 + n]
        const int kk = tid / 16, n4 = (tid % 16) * 4;
        const int ci = chunk * F32_KC + kk, co = n0 + n4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ci < p.C_in && co < p.C_out) v = *reinterpret_cast<const float4*>(wts + wk + (long long)ci * p.C_out + co);
        Bs[kk][n4 + 0] = v.x;
        Bs[kk][n4 + 1] = v.y;
        Bs[kk][n4 + 2] = v.z;
        Bs[kk][n4 + 3] = v.w;
      } else {  // B[kk][n] = W[k][ci = n0 + n][co = chunk*KC + kk]
        const int n = tid / 4, kk4 = (tid % 4) * 4;
        const int ci = n0 + n, co = chunk * F32_KC + kk4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ci < p.C_in && co < p.C_out) v = *reinterpret_cast<const float4*>(wts + wk + (long long)ci * p.C_out + co);
        Bs[kk4 + 0][n] = v.x;
        Bs[kk4 + 1][n] = v.y;
        Bs[kk4 + 2][n] = v.z;
        Bs[kk4 + 3][n] = v.w;
      }
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < F32_KC; ++kk) {
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
  }
  const int c_out = p.c_out;
  for (int i = 0; i < 4; ++i) {
    const int orow = permS[ty * 4 + i];
    if (orow < 0) continue;
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + tx * 4 + j;
      if (col >= c_out) continue;
      if (p.partial)
        p.partial[((long long)part * p.rows + orow) * c_out + col] = acc[i][j];
      else
        reinterpret_cast<float*>(p.out)[(long long)orow * c_out + col] = acc[i][j];
    }
  }
}

// out[e] = sum over parts of partial[part][e], rounded once to the output type (Section 4.1)
template <typename T>
__global__ void __launch_bounds__(256) k_split_reduce(const float* __restrict__ partial, int parts, long long elems,
                                                      T* __restrict__ out) {
  const long long e4 = ((long long)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (e4 >= elems) return;
  float4 s = *reinterpret_cast<const float4*>(partial + e4);
  for (int q = 1; q < parts; ++q) {
    const float4 v = *reinterpret_cast<const float4*>(partial + (long long)q * elems + e4);
    s.x += v.x;
    s.y += v.y;
    s.z += v.z;
    s.w += v.w;
  }
  out[e4 + 0] = (T)s.x;
  out[e4 + 1] = (T)s.y;
  out[e4 + 2] = (T)s.z;
  out[e4 + 3] = (T)s.w;
}

template <typename T, int BM, int BN, int KC, int NW>
int launch_igemm(const IgemmParams& p, dim3 grid, hipStream_t st) {
  typedef IgemmSmem<BM, BN, KC, false> SF;
  typedef IgemmSmem<BM, BN, KC, true> SD;
  static_assert(BM * (KC / 8) >= NW * 64, "every thread stages at least one segment of the gathered rows");
  static std::atomic<bool> attr_set{false};  // (set twice by racing threads at worst: the calls are idempotent)
  auto fwd = k_igemm<T, BM, BN, KC, NW, false>;
  auto dgr = k_igemm<T, BM, BN, KC, NW, true>;
  if (!attr_set.load(std::memory_order_acquire)) {
    SPC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(fwd), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)SF::total));
    SPC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(dgr), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)SD::total));
    attr_set.store(true, std::memory_order_release);
  }
  if (p.dgrad)
    hipLaunchKernelGGL(dgr, grid, dim3(NW * 64), SD::total, st, p);
  else
    hipLaunchKernelGGL(fwd, grid, dim3(NW * 64), SF::total, st, p);
  SPC_LAUNCH_CHECK();
  return SPCONV_OK;
}

template <typename T, int BM, int BN>
int launch_kc(const IgemmParams& p, int kc, int nw, dim3 grid, hipStream_t st) {
  if constexpr (BM >= 128) {
    if (nw == 8)
      return kc == 64 ? launch_igemm<T, BM, BN, 64, 8>(p, grid, st) : launch_igemm<T, BM, BN, 32, 8>(p, grid, st);
  }
  return kc == 64 ? launch_igemm<T, BM, BN, 64, 4>(p, grid, st) : launch_igemm<T, BM, BN, 32, 4>(p, grid, st);
}

template <typename T, int BM>
int launch_bn(const IgemmParams& p, int bn, int kc, int nw, dim3 grid, hipStream_t st) {
  switch (bn) {
    case 32: return launch_kc<T, BM, 32>(p, kc, nw, grid, st);
    case 64: return launch_kc<T, BM, 64>(p, kc, nw, grid, st);
    case 128: return launch_kc<T, BM, 128>(p, kc, nw, grid, st);
  }
  return SPCONV_EINVAL;
}

template <typename T>
int launch_bm(const IgemmParams& p, int bm, int bn, int kc, int nw, dim3 grid, hipStream_t st) {
  switch (bm) {
    case 64: return launch_bn<T, 64>(p, bn, kc, nw, grid, st);
    case 128: return launch_bn<T, 128>(p, bn, kc, nw, grid, st);
    case 256: return launch_bn<T, 256>(p, bn, kc, nw, grid, st);
  }
  return SPCONV_EINVAL;
}

}  // namespace

namespace {
// dynamic LDS of the tiled 16-bit kernel for a tile shape it is built for (0: no such kernel)
template <int BM, int BN> size_t tile_lds_kc(int kc, bool dgrad) {
  if (kc == 64) return dgrad ? IgemmSmem<BM, BN, 64, true>::total : IgemmSmem<BM, BN, 64, false>::total;
  if (kc == 32) return dgrad ? IgemmSmem<BM, BN, 32, true>::total : IgemmSmem<BM, BN, 32, false>::total;
  return 0;
}
template <int BM> size_t tile_lds_bn(int bn, int kc, bool dgrad) {
  switch (bn) {
    case 32: return tile_lds_kc<BM, 32>(kc, dgrad);
    case 64: return tile_lds_kc<BM, 64>(kc, dgrad);
    case 128: return tile_lds_kc<BM, 128>(kc, dgrad);
  }
  return 0;
}
size_t tile_lds_bytes(int bm, int bn, int kc, bool dgrad) {
  switch (bm) {
    case 64: return tile_lds_bn<64>(bn, kc, dgrad);
    case 128: return tile_lds_bn<128>(bn, kc, dgrad);
    case 256: return tile_lds_bn<256>(bn, kc, dgrad);
  }
  return 0;
}
}  // namespace

int igemm_tile_shape(int V, int n_split, int64_t rows, int64_t rows_src, int c_red, int c_out, int tile_m, int tile_n,
                     bool f32, bool dgrad, TileShape* s) {
  *s = TileShape{};
  const int q = f32 ? 4 : 8;
  if (rows < 1 || rows_src < 0 || c_red < q || c_out < q || c_red % q || c_out % q) return SPCONV_EINVAL;
  if (f32) tile_m = F32_BM;
  PlanShape ps;
  SPC_TRY(plan_shape(V, rows, n_split, tile_m, &ps));
  if ((uint64_t)ps.rows_pad * 27 * 4 >= 0xFFFF0000ull) return SPCONV_EINVAL;  // maps are read through 32-bit buffer offsets
  s->bm = tile_m;
  if (f32) {
    s->bn = F32_BN;
    s->kc = F32_KC;
    s->nw = 4;
    s->threads = 256;
    s->lds_bytes = sizeof(float) * (F32_BM * (F32_KC + 1) + F32_KC * (F32_BN + 4)) + sizeof(int) * (F32_BM * 27 + F32_BM);
    s->grid[0] = (unsigned)ps.n_tiles;
    s->grid[1] = (unsigned)ceil_div(c_out, F32_BN);
    s->grid[2] = (unsigned)ps.parts;
    return SPCONV_OK;
  }
  const uint64_t bytes = (uint64_t)rows_src * c_red * 2;
  if (bytes >= 0xFFFFC000ull) return SPCONV_EINVAL;  // buffer descriptors address 32 bits
  s->feats_bytes = (unsigned)bytes;
  int bn = tile_n;
  if (bn == 0) bn = c_out <= 32 ? 32 : (c_out <= 64 ? 64 : 128);
  if (bn != 32 && bn != 64 && bn != 128) return SPCONV_EINVAL;
  s->bn = bn;
  s->kc = (c_red % 64 == 0) ? 64 : 32;
  // Eight waves per workgroup where the reduction runs in 32-channel chunks (channel counts that
  // are not multiples of 64) on tiles of 128 rows or more: the steps are short there and twice the
  // waves hide their load latency (300k voxels, 96 -> 96: 150 us against 219 us); with 64-channel
  // chunks four waves with larger per-wave tiles are faster (256 -> 256: 602 us against 696 us).
  s->nw = (s->kc == 32 && tile_m >= 128) ? 8 : 4;
  s->threads = s->nw * 64;
  s->lds_bytes = tile_lds_bytes(tile_m, bn, s->kc, dgrad);
  if (s->lds_bytes == 0 || s->lds_bytes > 160 * 1024) return SPCONV_EINVAL;
  s->grid[0] = (unsigned)ps.n_tiles;
  s->grid[1] = (unsigned)ceil_div(c_out, bn);
  s->grid[2] = (unsigned)ps.parts;
  return SPCONV_OK;
}

int igemm_run(const spconv_kmap* km, const SideMap& side, const IgemmPlan& plan, const IgemmArgs& a,
              hipStream_t st) {
  if (plan.rows == 0) return SPCONV_OK;
  IgemmParams p{};
  p.feats = a.feats;
  p.weights = a.weights;
  p.out = a.out;
  p.partial = a.partial;
  p.rows = plan.rows;
  p.parts = plan.parts;
  p.V = km->V;
  p.C_in = a.C_in;
  p.C_out = a.C_out;
  p.dgrad = a.dgrad;
  p.mirror = a.mirror;
  p.c_red = a.dgrad ? a.C_out : a.C_in;
  p.c_out = a.dgrad ? a.C_in : a.C_out;
  const int64_t rows_src = (&side == &km->out_side) ? km->n_in : km->n_out;
  TileShape sh;
  SPC_TRY(igemm_tile_shape(km->V, plan.n_split, plan.rows, rows_src, p.c_red, p.c_out, plan.tile_m, a.tile_n,
                           a.dtype == SPCONV_F32, a.dgrad != 0, &sh));
  if (sh.bm != plan.tile_m || sh.grid[0] != (unsigned)plan.n_tiles) return SPCONV_EINVAL;  // (the plan was cut for another tile height)
  const int64_t tiles_alloc = plan.n_tiles > 0 ? plan.n_tiles : 1;
  for (int i = 0; i < plan.parts; ++i) {
    p.lo[i] = plan.lo[i];
    p.width[i] = plan.width[i];
    p.tilemask[i] = plan.tilemask.as<unsigned>() + (size_t)i * tiles_alloc;
    if (plan.n_split == 0) {
      p.map[i] = side.map.as<int>();
      p.perm[i] = nullptr;
    } else {
      p.map[i] = plan.maps.as<int>() + plan.map_off[i];
      p.perm[i] = plan.perm.as<int>() + (size_t)i * plan.rows_pad;
    }
    p.map_part_bytes[i] = (unsigned)((uint64_t)plan.rows_pad * plan.width[i] * 4);
  }
  p.rows_pad_bytes = (unsigned)((uint64_t)plan.rows_pad * 4);
  p.tiles_bytes = (unsigned)((uint64_t)plan.n_tiles * 4);
  p.feats_bytes = sh.feats_bytes;
  dim3 grid(sh.grid[0], sh.grid[1], sh.grid[2]);
  if (a.dtype == SPCONV_F32) {
    hipLaunchKernelGGL(k_igemm_f32, grid, dim3(256), 0, st, p);
    SPC_LAUNCH_CHECK();
    return SPCONV_OK;
  }
  // tiles late in a bitmask-sorted order hold the most offsets: they start first, so that the
  // grid does not end on its longest workgroups
  p.heavy_first = plan.n_split > 0 ? 1 : 0;
  if (a.dtype == SPCONV_F16) return launch_bm<_Float16>(p, plan.tile_m, sh.bn, sh.kc, sh.nw, grid, st);
  return launch_bm<__bf16>(p, plan.tile_m, sh.bn, sh.kc, sh.nw, grid, st);
}

int split_reduce(const float* partial, int parts, int64_t rows, int c, spconv_dtype dtype, void* out,
                 hipStream_t st) {
  const long long elems = (long long)rows * c;
  if (elems == 0) return SPCONV_OK;
  const unsigned blocks = (unsigned)ceil_div(elems / 4, 256);
  switch (dtype) {
    case SPCONV_F32:
      hipLaunchKernelGGL((k_split_reduce<float>), dim3(blocks), dim3(256), 0, st, partial, parts, elems, (float*)out);
      break;
    case SPCONV_F16:
      hipLaunchKernelGGL((k_split_reduce<_Float16>), dim3(blocks), dim3(256), 0, st, partial, parts, elems,
                         (_Float16*)out);
      break;
    case SPCONV_BF16:
      hipLaunchKernelGGL((k_split_reduce<__bf16>), dim3(blocks), dim3(256), 0, st, partial, parts, elems,
                         (__bf16*)out);
      break;
  }
  SPC_LAUNCH_CHECK();
  return SPCONV_OK;
}

}  // namespace spc
