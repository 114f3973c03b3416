// Implicit-GEMM forward / input-gradient for small channel counts: weights
// resident in LDS, one wave per 16-row block, no workgroup barriers in the loop.
//
// At 64 channels the layer is bound by memory latency, not by the matrix
// cores, so this kernel is organised around keeping loads in flight rather
// than around large MFMA tiles:
//   * the weight slices of all offsets of this part (Section 4.1's split) for
//     BN output channels stay in the CU's 160 KB LDS for the life of the
//     workgroup (stored reduction-index-contiguous, 16-byte chunks XOR-swizzled
//     so that fragment reads do not collide on banks);
//   * each wave owns whole 16-row blocks of the (possibly bitmask-sorted) map;
//     a lane fetches its MFMA A-fragment (8 consecutive channels of one
//     gathered row) straight from global memory into registers, predicated on
//     the neighbour being present, several offsets ahead of the MFMAs that
//     consume it;
//   * offsets whose bit is clear in the block's mask are skipped: the lock-step
//     unit of Section 2.2.3 is the 16-row block;
//   * the block's map rows are staged in a per-wave LDS slab (the hoisted
//     addressing of Section 3.2), and output rows leave through the same slab
//     as whole 16-byte segments.
#include "common.h"

#include <atomic>

#include <algorithm>
#include <cstdlib>

namespace spc {
namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <typename T> struct MfmaW;
template <> struct MfmaW<_Float16> {
  static __device__ __forceinline__ f32x4 run(uint4 a, uint4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0,
                                                  0);
  }
};
template <> struct MfmaW<__bf16> {
  static __device__ __forceinline__ f32x4 run(uint4 a, uint4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                   0, 0);
  }
};

struct WaveParams {
  const void* feats;
  const void* weights;
  void* out;
  float* partial;
  const int* map[kMaxSplit];
  const int* perm[kMaxSplit];
  const unsigned* blkmask[kMaxSplit];
  const unsigned* rowmask;  // unsorted maps: per-row masks; the 16-row block mask is their OR (no plan kernel)
  int lo[kMaxSplit], width[kMaxSplit];
  long long rows, n_blocks;
  int parts, V;
  int c_red, c_out;
  int C_in, C_out;
  int dgrad, mirror;
  int slab_bytes;  // per-wave LDS slab: map rows, then the output staging tile
  int map_bytes;   // size of the map part of the slab
  unsigned feats_bytes;  // size of the gathered tensor, < 2^32 - 16 KiB
  unsigned map_part_bytes[kMaxSplit];  // sizes of the tables a plan index reaches: each part's map,
  unsigned rows_pad_bytes;             //   the permutation and the row masks (rows_pad entries),
  unsigned blocks_bytes;               //   the block masks (n_blocks entries)
  int quad;     // gathers issued by quads of lanes per row and permuted to the operand layout
  int xcd_ranges;  // blocks are dealt to the 8 XCDs as contiguous ranges (gridDim.x is a multiple of 8)
};

// physical 16-byte chunk of logical chunk q in weight row n (row pitch = 4*KS chunks)
template <int KS> __device__ __forceinline__ int swz(int q, int n) {
  if ((4 * KS) % 8 == 0) return (q & ~7) | ((q ^ n) & 7);
  return (q & ~3) | ((q ^ (n >> 1)) & 3);
}


typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Raw buffer descriptor over [base, base + bytes): loads beyond the end return zeros and touch
// no memory, which turns "neighbour absent" (index -1) into an out-of-range offset instead of a
// branch, so that every load is issued unconditionally and the wait counters stay countable.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ uint4 buf_load16(__amdgpu_buffer_rsrc_t r, unsigned byte_off) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}

constexpr int kLoopUnroll = 3;  // trips through the DEPTH slots per loop iteration (see the offset loop)
constexpr int kMapVecs = 7;  // ceil(16 rows * 27 offsets / 64 lanes)

// DEPTH = offsets whose A-fragments are in flight per wave.  DEPTH 8 needs more than the 128
// registers a 16-wave workgroup leaves per lane, so it runs with 8 waves.
template <typename T, int KS, int NB, int DEPTH, bool QUAD>
__global__ void __launch_bounds__(DEPTH > 4 ? 512 : 1024) k_igemm_wave(const WaveParams p) {
  constexpr int BN = NB * 16;
  constexpr int ROW_CHUNKS = 4 * KS;        // 16-byte chunks per weight row
  constexpr int ROW_HALFS = 32 * KS;
  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform, and known to be
  const int n_waves = blockDim.x >> 6;
  const int arow = lane & 15, aq = lane >> 4;  // fragment row and 8-channel group within a k-step
  const int part = blockIdx.z;
  const int n0 = blockIdx.y * BN;
  const int width = p.width[part], lo = p.lo[part];
  const int c_red = p.c_red, c_out = p.c_out;

  unsigned short* Ws = reinterpret_cast<unsigned short*>(smem);  // [width][BN][ROW_HALFS] swizzled
  unsigned char* slab = smem + (size_t)width * BN * ROW_HALFS * 2 + (size_t)wave * p.slab_bytes;
  int* mapW = reinterpret_cast<int*>(slab);

  const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(p.weights, (unsigned)((size_t)p.V * p.C_in * p.C_out * 2));
  const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(p.feats, p.feats_bytes);

  // Blocks of this workgroup: b = j * gridDim.x + blockIdx.x, j < nj, handed to its waves one at
  // a time in descending j (a bitmask-sorted map has its widest masks at the end, so the heaviest
  // blocks go first and the tail of the kernel is made of light ones).  A wave's first ticket is
  // its index; further ones come from a counter in LDS.
  __shared__ unsigned next_ticket;
  // With p.xcd_ranges the blocks are cut into eight contiguous ranges, one per XCD (workgroups go
  // to the XCDs round-robin by their index), and a workgroup takes every (gridDim.x / 8)-th block
  // of its XCD's range: with rows whose sort key starts with a spatial slab, an XCD's gathers stay
  // within one eighth of the input, which its 4 MB L2 holds.
  const int n_rng = p.xcd_ranges ? 8 : 1;
  const int rng = p.xcd_ranges ? (int)(blockIdx.x & 7) : 0;
  const int wi = p.xcd_ranges ? (int)(blockIdx.x >> 3) : (int)blockIdx.x;  // workgroup within the range
  const int wpr = (int)gridDim.x / n_rng;                                    // workgroups per range
  const long long rlo = p.n_blocks * rng / n_rng, rhi = p.n_blocks * (rng + 1) / n_rng;
  const int nj = rhi - rlo > wi ? (int)((rhi - rlo - wi + wpr - 1) / wpr) : 0;
  auto block_of = [&](int t) { return rlo + (long long)(nj - 1 - t) * wpr + wi; };
  const bool has_work = wave < nj;
  if (tid == 0) next_ticket = (unsigned)n_waves;
  const unsigned row_bytes = (unsigned)c_red * 2u;
  const int map_len = 16 * width;
  const int* map_part = p.map[part];
  const int* pm = p.perm[part];
  const unsigned* bmask = p.blkmask[part];
  T* stage = reinterpret_cast<T*>(slab + p.map_bytes);

  // per-lane constants of the offset loop
  // With QUAD a gathered row is loaded by a quad of adjacent lanes (lane / 4 = row of the block,
  // lane % 4 = 16-byte chunk of the k-step): the four requests of a quad fall into one cache line
  // and travel as one, where the MFMA operand layout itself (lane % 16 = row) sends sixteen rows
  // per quarter-wave and every 16-byte piece on its own (measured on random 128-byte rows out of
  // an L2-resident array: 21 TB/s against 8 TB/s).  consume() then moves each dword to the lane
  // the MFMA wants it in with one cross-lane permute (8 per offset: they pay on bitmask-sorted
  // maps, whose blocks hold few absent rows, and cost more than they save on unsorted ones).
  constexpr unsigned kAbsent = 0xFFFF0000u;  // byte offset that is out of range with any lane offset added
  const int grow = QUAD ? lane >> 2 : arow, gq = QUAD ? lane & 3 : aq;  // gather role: block row, chunk of a k-step
  const unsigned lane_map = (unsigned)(grow * width) * 4u;  // this lane's map row in the slab
  const int frag_src = (4 * arow + aq) * 4;  // (byte address of) the lane that gathered this lane's MFMA fragment
  unsigned lane_col[KS];  // the 8 channels this lane gathers of a row (bytes), or out of range
  unsigned lane_b[KS];    // this lane's weight chunk within an offset's slice (bytes, first 16 columns)
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const unsigned col = (unsigned)(ks * 4 + gq) * 8u;
    lane_col[ks] = col < (unsigned)c_red ? col * 2u : 0x80000000u;
    lane_b[ks] = (unsigned)(arow * ROW_HALFS + swz<KS>(ks * 4 + aq, arow) * 8) * 2u;
  }

  // registers holding the next block's map rows, mask and output rows
  int mreg[kMapVecs];
  unsigned bm_next = 0;
  int orow_next = -1;
  // Every table that a block index reaches is read through a range-checked buffer descriptor
  // (beyond the end: zeros, no access), like the gathered rows: a wrong index cannot fault.
  auto prefetch_block = [&](long long b) {
    const __amdgpu_buffer_rsrc_t m_rsrc = make_rsrc(map_part, p.map_part_bytes[part]);
    const unsigned mbase = (unsigned)(b * map_len) * 4u;
#pragma unroll
    for (int i = 0; i < kMapVecs; ++i) {
      const int e = lane + 64 * i;
      mreg[i] = __builtin_amdgcn_raw_buffer_load_b32(m_rsrc, e < map_len ? mbase + (unsigned)e * 4u : 0xFFFFFFFFu, 0, 0);
    }
    const unsigned g4 = (unsigned)(b * 16 + arow) * 4u;
    if (p.rowmask)  // OR-reduced when the block starts
      bm_next = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(make_rsrc(p.rowmask, p.rows_pad_bytes), g4, 0, 0);
    else
      bm_next = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(make_rsrc(bmask, p.blocks_bytes), (unsigned)b * 4u, 0, 0);
    const long long g = b * 16 + arow;
    if (pm)
      orow_next = __builtin_amdgcn_raw_buffer_load_b32(make_rsrc(pm, p.rows_pad_bytes), g4, 0, 0);
    else
      orow_next = g < p.rows ? (int)g : -1;
  };

  uint4 fr[DEPTH][KS];
  int cc[DEPTH];
  unsigned m = 0;
  // Always issues KS loads: with no offset left they are out-of-range loads (zeros, no traffic).
  // The slab holds byte offsets of the gathered rows (kAbsent for a missing neighbour).
  auto issue = [&](int s) {
    const int c = m ? __ffs((int)m) - 1 : -1;
    m &= m - 1;  // 0 stays 0
    cc[s] = c;
    unsigned rowb = kAbsent;
    if (c >= 0) rowb = *reinterpret_cast<const unsigned*>(slab + lane_map + (unsigned)c * 4u);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) fr[s][ks] = buf_load16(x_rsrc, rowb + lane_col[ks]);
  };
  // Publishes the prefetched block in the wave's slab, takes the ticket of the block after it and
  // starts that block's prefetch, then puts the first DEPTH offsets in flight.
  int t_next = 0;
  auto start_block = [&]() {
#pragma unroll
    for (int i = 0; i < kMapVecs; ++i) {
      const int e = lane + 64 * i;
      if (e < map_len) mapW[e] = mreg[i] < 0 ? (int)kAbsent : (int)((unsigned)mreg[i] * row_bytes);
    }
    unsigned bm = bm_next;
    if (p.rowmask) {  // lanes 0..15 (and their three copies) hold the rows' masks
      bm |= __shfl_xor(bm, 1);
      bm |= __shfl_xor(bm, 2);
      bm |= __shfl_xor(bm, 4);
      bm |= __shfl_xor(bm, 8);
    }
    m = __builtin_amdgcn_readfirstlane(bm);
    unsigned t = 0;
    if (lane == 0) t = atomicAdd(&next_ticket, 1u);
    t_next = (int)__builtin_amdgcn_readfirstlane(t);
    prefetch_block(block_of(t_next < nj ? t_next : nj - 1));
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) issue(s);
  };

  // the first block's map rows travel while the weights are being staged
  if (has_work) prefetch_block(block_of(wave));

  // ---- weights of this part -> LDS (once per workgroup), kFill loads in flight per thread
  constexpr int kFill = 8;
  {
    const unsigned slice = (unsigned)(p.C_in * p.C_out * 2);
    if (p.dgrad) {
      // B[kk = co][n = ci] = W[k][ci][co]: rows of W are already reduction-contiguous
      const int chunks = width * BN * ROW_CHUNKS;
      for (int e0 = tid; e0 < chunks; e0 += kFill * blockDim.x) {
        uint4 v[kFill];
#pragma unroll
        for (int u = 0; u < kFill; ++u) {
          const int e = e0 + u * blockDim.x;
          const int q = e % ROW_CHUNKS, n = (e / ROW_CHUNKS) % BN, c = e / (ROW_CHUNKS * BN);
          const int k = lo + c;
          const int ci = n0 + n, co = q * 8;
          const bool ok = e < chunks && ci < p.C_in && co < p.C_out;
          const unsigned off = (unsigned)(p.mirror ? p.V - 1 - k : k) * slice + (unsigned)(ci * p.C_out + co) * 2u;
          v[u] = buf_load16(w_rsrc, ok ? off : 0xFFFFFFFFu);
        }
#pragma unroll
        for (int u = 0; u < kFill; ++u) {
          const int e = e0 + u * blockDim.x;
          const int q = e % ROW_CHUNKS, n = (e / ROW_CHUNKS) % BN, c = e / (ROW_CHUNKS * BN);
          if (e < chunks)
            *reinterpret_cast<uint4*>(Ws + ((size_t)(c * BN + n) * ROW_CHUNKS + swz<KS>(q, n)) * 8) = v[u];
        }
      }
    } else {
      // B[kk = ci][n = co] = W[k][ci][co].  A thread takes four consecutive ci of one group of 8
      // output channels (four 16-byte loads), transposes the 4 x 8 block in registers and writes
      // each output channel's four reduction steps with one 8-byte store (2-byte stores made this
      // fill 1.7 us slower than the input gradient's, whose rows are copied as they are).
      constexpr int kQuad = kFill / 4;  // 4-row groups in flight per thread
      const int groups = width * (ROW_HALFS / 4) * (BN / 8);
      for (int e0 = tid; e0 < groups; e0 += kQuad * blockDim.x) {
        uint4 v[kQuad][4];
#pragma unroll
        for (int u = 0; u < kQuad; ++u) {
          const int e = e0 + u * blockDim.x;
          const int ng = e % (BN / 8), k4 = (e / (BN / 8)) % (ROW_HALFS / 4), c = e / ((BN / 8) * (ROW_HALFS / 4));
          const int k = lo + c;
          const int co = n0 + ng * 8;
          const unsigned base = (unsigned)(p.mirror ? p.V - 1 - k : k) * slice;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int ci = k4 * 4 + r;
            const bool ok = e < groups && ci < p.C_in && co < p.C_out;
            v[u][r] = buf_load16(w_rsrc, ok ? base + (unsigned)(ci * p.C_out + co) * 2u : 0xFFFFFFFFu);
          }
        }
#pragma unroll
        for (int u = 0; u < kQuad; ++u) {
          const int e = e0 + u * blockDim.x;
          if (e >= groups) continue;
          const int ng = e % (BN / 8), k4 = (e / (BN / 8)) % (ROW_HALFS / 4), c = e / ((BN / 8) * (ROW_HALFS / 4));
          const int kk = k4 * 4;
          const unsigned w[4][4] = {{v[u][0].x, v[u][0].y, v[u][0].z, v[u][0].w},
                                    {v[u][1].x, v[u][1].y, v[u][1].z, v[u][1].w},
                                    {v[u][2].x, v[u][2].y, v[u][2].z, v[u][2].w},
                                    {v[u][3].x, v[u][3].y, v[u][3].z, v[u][3].w}};
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const int n = ng * 8 + i;
            const int sh = (i & 1) * 16;
            const unsigned h0 = (w[0][i >> 1] >> sh) & 0xFFFFu, h1 = (w[1][i >> 1] >> sh) & 0xFFFFu;
            const unsigned h2 = (w[2][i >> 1] >> sh) & 0xFFFFu, h3 = (w[3][i >> 1] >> sh) & 0xFFFFu;
            *reinterpret_cast<uint2*>(Ws + ((size_t)(c * BN + n) * ROW_CHUNKS + swz<KS>(kk >> 3, n)) * 8 + (kk & 7)) =
                make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
          }
        }
      }
    }
  }
  __syncthreads();  // weights visible
  if (!has_work) return;

  for (int t_cur = wave; t_cur < nj; t_cur = t_next) {
    const int orow_cur = orow_next;
    start_block();
    f32x4 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto consume = [&](int s) {
      const unsigned char* wk = smem + (unsigned)cc[s] * (unsigned)(BN * ROW_HALFS * 2);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        uint4 af = fr[s][ks];
        if constexpr (QUAD) {  // gather layout -> MFMA A-fragment layout
          af.x = (unsigned)__builtin_amdgcn_ds_bpermute(frag_src, (int)fr[s][ks].x);
          af.y = (unsigned)__builtin_amdgcn_ds_bpermute(frag_src, (int)fr[s][ks].y);
          af.z = (unsigned)__builtin_amdgcn_ds_bpermute(frag_src, (int)fr[s][ks].z);
          af.w = (unsigned)__builtin_amdgcn_ds_bpermute(frag_src, (int)fr[s][ks].w);
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const uint4 bf = *reinterpret_cast<const uint4*>(wk + lane_b[ks] + nb * (16 * ROW_HALFS * 2));
          acc[nb] = MfmaW<T>::run(af, bf, acc[nb]);
        }
      }
    };

    // The exits leave the loop directly (not through its latch), so that the wait-count
    // bookkeeping at the loop head sees only the steady state: DEPTH - 1 slots in flight.
    for (;;) {
#pragma unroll
      for (int rep = 0; rep < kLoopUnroll; ++rep) {
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
          if (cc[s] < 0) goto offsets_done;
          consume(s);
          issue(s);
        }
      }
    }
  offsets_done:

    // ---- output rows
    if (p.partial) {
      // fp32 partial sums: lane holds rows 4*(lane/16)+r, column lane%16 of each 16-column block
      int o4[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) o4[r] = __shfl(orow_cur, aq * 4 + r);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (o4[r] < 0) continue;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const int col = n0 + nb * 16 + arow;
          if (col < c_out) p.partial[((long long)part * p.rows + o4[r]) * c_out + col] = acc[nb][r];
        }
      }
    } else {
      // stage the 16 x BN tile in the wave's slab, then write whole 16-byte segments of each row
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) stage[(aq * 4 + r) * BN + nb * 16 + arow] = (T)acc[nb][r];
      __builtin_amdgcn_wave_barrier();
      constexpr int SEGS = BN / 8;  // 16-byte segments per staged row
#pragma unroll
      for (int i = 0; i < (16 * SEGS + 63) / 64; ++i) {
        const int e = lane + 64 * i;
        const int r = e / SEGS, sg = e % SEGS;
        const int o = __shfl(orow_cur, r & 15);
        if (e < 16 * SEGS && o >= 0 && n0 + sg * 8 < c_out)
          *reinterpret_cast<uint4*>(reinterpret_cast<T*>(p.out) + (long long)o * c_out + n0 + sg * 8) =
              *reinterpret_cast<const uint4*>(stage + r * BN + sg * 8);
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
}

template <typename T, int KS, int NB, int DEPTH, bool QUAD>
int launch_wave_q(const WaveParams& p, dim3 grid, int threads, size_t smem, hipStream_t st) {
  static std::atomic<size_t> attr_bytes{0};  // largest dynamic LDS size announced for this instance so far
  auto fn = k_igemm_wave<T, KS, NB, DEPTH, QUAD>;
  if (smem > attr_bytes.load(std::memory_order_acquire)) {
    SPC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)smem));
    attr_bytes.store(smem, std::memory_order_release);
  }
  hipLaunchKernelGGL(fn, grid, dim3(threads), smem, st, p);
  SPC_LAUNCH_CHECK();
  return SPCONV_OK;
}

template <typename T, int KS, int NB, int DEPTH>
int launch_wave_d(const WaveParams& p, dim3 grid, int threads, size_t smem, hipStream_t st) {
  if (p.quad) return launch_wave_q<T, KS, NB, DEPTH, true>(p, grid, threads, smem, st);
  return launch_wave_q<T, KS, NB, DEPTH, false>(p, grid, threads, smem, st);
}

template <typename T, int KS, int NB>
int launch_wave(const WaveParams& p, dim3 grid, int threads, size_t smem, hipStream_t st) {
  if constexpr (KS <= 2) {
    if (threads <= 512) return launch_wave_d<T, KS, NB, 8>(p, grid, threads, smem, st);
  }
  return launch_wave_d<T, KS, NB, 4>(p, grid, threads, smem, st);
}

template <typename T, int KS>
int launch_wave_nb(int nb, const WaveParams& p, dim3 grid, int threads, size_t smem, hipStream_t st) {
  switch (nb) {
    case 1: return launch_wave<T, KS, 1>(p, grid, threads, smem, st);
    case 2: return launch_wave<T, KS, 2>(p, grid, threads, smem, st);
    case 4: return launch_wave<T, KS, 4>(p, grid, threads, smem, st);
  }
  return SPCONV_EINVAL;
}

template <typename T>
int launch_wave_ks(int ks, int nb, const WaveParams& p, dim3 grid, int threads, size_t smem, hipStream_t st) {
  switch (ks) {
    case 1: return launch_wave_nb<T, 1>(nb, p, grid, threads, smem, st);
    case 2: return launch_wave_nb<T, 2>(nb, p, grid, threads, smem, st);
    case 3: return launch_wave_nb<T, 3>(nb, p, grid, threads, smem, st);
    case 4: return launch_wave_nb<T, 4>(nb, p, grid, threads, smem, st);
  }
  return SPCONV_EINVAL;
}

constexpr size_t kLdsBudget = 160 * 1024 - 64;  // (64 bytes for the static ticket counter)

size_t map_bytes_for(int max_width) { return (size_t)round_up((int64_t)16 * max_width * 4, 16); }

size_t slab_bytes_for(int max_width, int bn, int parts) {
  return map_bytes_for(max_width) + (parts == 1 ? (size_t)16 * bn * 2 : 0);
}

}  // namespace

// Largest BN in {64, 32, 16} (or exactly tile_n) for which the weights of the widest part plus
// the per-wave slabs of at least 8 waves fit in LDS; 0 if none does.
int igemm_wave_pick_bn(int V, int n_split, int c_red, int c_out, int tile_n, int* waves_out) {
  if (c_red > 128 || n_split > V) return 0;  // (every part needs at least one offset)
  const int ks = (c_red + 31) / 32;
  const int parts = std::max(1, n_split);
  int max_width = 0;
  for (int i = 0; i < parts; ++i) max_width = std::max(max_width, (i + 1) * V / parts - i * V / parts);
  const int cands[3] = {64, 32, 16};
  for (int bn : cands) {
    if (tile_n != 0 && bn != tile_n) continue;
    if (tile_n == 0 && bn > 16 && bn >= 2 * c_out) continue;  // no point in a tile twice as wide as the layer
    // unsorted maps: two 32-column tiles beat one of 64 (100k voxels, 32 -> 64: 24.3 us against 26.7 us)
    if (tile_n == 0 && bn == 64 && n_split == 0) continue;
    const size_t w = (size_t)max_width * bn * ks * 64;
    const size_t slab = slab_bytes_for(max_width, bn, parts);
    for (int waves : {16, 8}) {
      if (w + (size_t)waves * slab <= kLdsBudget) {
        if (waves_out) *waves_out = waves;
        return bn;
      }
    }
  }
  return 0;
}

int igemm_wave_shape(int V, int n_split, int64_t rows, int64_t rows_src, int c_red, int c_out, int tile_n,
                     WaveShape* s) {
  *s = WaveShape{};
  if (rows < 1 || rows_src < 0 || c_red < 8 || c_out < 8 || c_red % 8 || c_out % 8) return SPCONV_EINVAL;
  PlanShape ps;
  SPC_TRY(plan_shape(V, rows, n_split, 16, &ps));
  const uint64_t feats_bytes = (uint64_t)rows_src * c_red * 2;
  // buffer descriptors address 32 bits; "absent" is the byte offset 0xFFFF0000, and lanes beyond a
  // channel count that is not a multiple of 32 add 2^31 to stay out of range
  if (feats_bytes >= (c_red % 32 ? 0x7FFF0000ull : 0xFFFF0000ull)) return SPCONV_EINVAL;
  s->feats_bytes = (unsigned)feats_bytes;
  int waves = 8;
  s->bn = igemm_wave_pick_bn(V, n_split, c_red, c_out, tile_n, &waves);
  if (s->bn == 0) return SPCONV_EINVAL;
  s->waves = waves;
  s->threads = waves * 64;
  s->ks = (c_red + 31) / 32;
  for (int i = 0; i < ps.parts; ++i) s->max_width = std::max(s->max_width, ps.width[i]);
  // the map, the permutation and the masks are read through 32-bit buffer offsets as well
  if ((uint64_t)ps.rows_pad * s->max_width * 4 >= 0xFFFF0000ull) return SPCONV_EINVAL;
  s->slab_bytes = (int)slab_bytes_for(s->max_width, s->bn, ps.parts);
  s->map_bytes = (int)map_bytes_for(s->max_width);
  s->lds_bytes = (size_t)s->max_width * s->bn * s->ks * 64 + (size_t)waves * s->slab_bytes;
  if (s->lds_bytes > kLdsBudget) return SPCONV_EINVAL;
  const int n_tiles_n = (int)ceil_div(c_out, s->bn);
  // persistent workgroups: about one per CU over all (n-tile, part) slices, each wave gets >= 1 block
  int64_t per_slice = std::max<int64_t>(1, 256 / ((int64_t)n_tiles_n * ps.parts));
  per_slice = std::min<int64_t>(per_slice, ceil_div(ps.n_tiles, waves));
  if (per_slice > 8) per_slice = per_slice / 8 * 8;  // (whole rounds over the eight XCDs)
  s->grid[0] = (unsigned)per_slice;
  s->grid[1] = (unsigned)n_tiles_n;
  s->grid[2] = (unsigned)ps.parts;
  return SPCONV_OK;
}

int igemm_wave_run(const spconv_kmap* km, const SideMap& side, const IgemmPlan& plan, const IgemmArgs& a,
                   hipStream_t st) {
  if (plan.rows == 0) return SPCONV_OK;
  if (plan.tile_m != 16 || a.dtype == SPCONV_F32) return SPCONV_EINVAL;
  WaveParams p{};
  p.feats = a.feats;
  p.weights = a.weights;
  p.out = a.out;
  p.partial = a.partial;
  p.rows = plan.rows;
  p.n_blocks = plan.n_tiles;
  p.parts = plan.parts;
  p.V = km->V;
  p.C_in = a.C_in;
  p.C_out = a.C_out;
  p.dgrad = a.dgrad;
  p.mirror = a.mirror;
  p.c_red = a.dgrad ? a.C_out : a.C_in;
  p.c_out = a.dgrad ? a.C_in : a.C_out;
  const int64_t rows_src = (&side == &km->out_side) ? km->n_in : km->n_out;
  WaveShape sh;
  SPC_TRY(igemm_wave_shape(km->V, plan.n_split, plan.rows, rows_src, p.c_red, p.c_out, a.tile_n, &sh));
  p.feats_bytes = sh.feats_bytes;
  const int64_t tiles_alloc = plan.n_tiles > 0 ? plan.n_tiles : 1;
  for (int i = 0; i < plan.parts; ++i) {
    p.lo[i] = plan.lo[i];
    p.width[i] = plan.width[i];
    p.blkmask[i] = plan.tilemask.as<unsigned>() + (size_t)i * tiles_alloc;
    if (plan.n_split == 0) {
      p.map[i] = side.map.as<int>();
      p.perm[i] = nullptr;
      p.rowmask = side.mask.as<unsigned>();
    } else {
      p.map[i] = plan.maps.as<int>() + plan.map_off[i];
      p.perm[i] = plan.perm.as<int>() + (size_t)i * plan.rows_pad;
    }
    p.map_part_bytes[i] = (unsigned)((uint64_t)plan.rows_pad * plan.width[i] * 4);
  }
  p.rows_pad_bytes = (unsigned)((uint64_t)plan.rows_pad * 4);
  p.blocks_bytes = (unsigned)((uint64_t)plan.n_tiles * 4);
  p.slab_bytes = sh.slab_bytes;
  p.map_bytes = sh.map_bytes;
  p.xcd_ranges = plan.slabs && sh.grid[0] % 8 == 0;  // (contiguous ranges of a purely bitmask-sorted order are unequal work)
  p.quad = plan.n_split > 0;
  dim3 grid(sh.grid[0], sh.grid[1], sh.grid[2]);
  if (a.dtype == SPCONV_F16) return launch_wave_ks<_Float16>(sh.ks, sh.bn / 16, p, grid, sh.threads, sh.lds_bytes, st);
  return launch_wave_ks<__bf16>(sh.ks, sh.bn / 16, p, grid, sh.threads, sh.lds_bytes, st);
}

}  // namespace spc
