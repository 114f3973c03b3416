// Mapping work that depends on the dataflow parameters (Sections 2.2.3, 3.2,
// 4.1): per-split bitmask argsort, offline map reordering and padding,
// per-tile mask reduction, the offset-major map and work list of wgrad, and
// the executed-MAC count of a configuration.
#include "common.h"

#include <algorithm>
#include <new>

namespace spc {
namespace {

inline unsigned blocks_for(int64_t n, int per_block) { return (unsigned)ceil_div(n > 0 ? n : 1, per_block); }

// Spatial slabs in front of the bitmask keys of large maps.  A bitmask-sorted block gathers rows
// from all over the scene, so every XCD of the chip pulls most of the input through its own 4 MB
// L2 (measured on the 100k-voxel scan: 54 MB fetched for 12.8 MB of features).  With the rows cut
// into kSlabs slabs along the longest axis and the bitmask order kept inside each slab, the
// kernels hand each XCD a contiguous range of the order, i.e. about one slab: its gathers stay
// within an eighth of the input plus a one-voxel halo.  Any order gives the same result; the
// price is a little more lock-step redundancy (1.23 -> 1.43 executed / valid on that scan).
constexpr int kSlabBits = 3, kSlabs = 1 << kSlabBits;
// Measured on the 100k-voxel scan, 64 -> 64: beyond-L2 traffic of the forward kernel 66.7 -> 43 MB
// (1.82 x -> 1.17 x the compulsory bytes), kernel time 20.9 -> 23.2 us: the kernel is bound by the
// length of a wave's per-offset chain, not by that traffic, so the extra block-offsets cost more
// than the L2 hits return.  Slabs are therefore kept for inputs that no longer fit the 256 MB
// last-level cache comfortably.
constexpr int kSlabMinRows = 1 << 20;
constexpr int kBoundsBlocks = 64;

// partial[b][0..2] = min, partial[b][3..5] = max of (x, y, z) over the rows block b visits
__global__ void __launch_bounds__(256)
    k_coord_bounds(const int4* __restrict__ coords, int rows, int* __restrict__ partial) {
  __shared__ int red[4][6];
  int lo[3] = {0x7FFFFFFF, 0x7FFFFFFF, 0x7FFFFFFF}, hi[3] = {(int)0x80000000, (int)0x80000000, (int)0x80000000};
  for (int r = blockIdx.x * blockDim.x + threadIdx.x; r < rows; r += gridDim.x * blockDim.x) {
    const int4 c = coords[r];  // (b, x, y, z)
    lo[0] = min(lo[0], c.y), lo[1] = min(lo[1], c.z), lo[2] = min(lo[2], c.w);
    hi[0] = max(hi[0], c.y), hi[1] = max(hi[1], c.z), hi[2] = max(hi[2], c.w);
  }
#pragma unroll
  for (int a = 0; a < 3; ++a)
    for (int o = 32; o > 0; o >>= 1) {
      lo[a] = min(lo[a], __shfl_xor(lo[a], o));
      hi[a] = max(hi[a], __shfl_xor(hi[a], o));
    }
  const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
  if (lane == 0)
    for (int a = 0; a < 3; ++a) red[wib][a] = lo[a], red[wib][3 + a] = hi[a];
  __syncthreads();
  if (threadIdx.x < 6) {
    const int a = threadIdx.x;
    int v = red[0][a];
    for (int w = 1; w < 4; ++w) v = a < 3 ? min(v, red[w][a]) : max(v, red[w][a]);
    partial[blockIdx.x * 6 + a] = v;
  }
}

// key[r] = bits [lo, lo+width) of mask[r], below the row's slab if coords is given; val[r] = r
__global__ void __launch_bounds__(256)
    k_split_keys(const unsigned* __restrict__ mask, int rows, int lo, int width, const int4* __restrict__ coords,
                 const int* __restrict__ partial, int n_partial, unsigned* __restrict__ key, int* __restrict__ val) {
  __shared__ int s_axis, s_lo, s_ext;
  if (coords) {
    if (threadIdx.x < 64) {  // the first wave folds the partial bounds and picks the longest axis
      int mn[3], mx[3];
      for (int a = 0; a < 3; ++a) {
        int l = 0x7FFFFFFF, h = (int)0x80000000;
        for (int b = threadIdx.x; b < n_partial; b += 64) {
          l = min(l, partial[b * 6 + a]);
          h = max(h, partial[b * 6 + 3 + a]);
        }
        for (int o = 32; o > 0; o >>= 1) {
          l = min(l, __shfl_xor(l, o));
          h = max(h, __shfl_xor(h, o));
        }
        mn[a] = l, mx[a] = h;
      }
      if (threadIdx.x == 0) {
        int axis = 0;
        for (int a = 1; a < 3; ++a)
          if ((long long)mx[a] - mn[a] > (long long)mx[axis] - mn[axis]) axis = a;
        s_axis = axis;
        s_lo = mn[axis];
        s_ext = (int)min((long long)mx[axis] - mn[axis] + 1, (long long)0x7FFFFFFF);
      }
    }
    __syncthreads();
  }
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= rows) return;
  unsigned k = (mask[r] >> lo) & ((1u << width) - 1u);
  if (coords) {
    const int4 c = coords[r];
    const int v = s_axis == 0 ? c.y : s_axis == 1 ? c.z : c.w;
    const long long slab = ((long long)v - s_lo) * kSlabs / s_ext;  // 0 .. kSlabs-1
    k |= (unsigned)slab << width;
  }
  key[r] = k;
  val[r] = r;
}

// ---- bitmask argsort in few launches (maps of up to kSortMaxWgs * kSortWg rows) ----
// Stable least-significant-digit radix sort of (key, row): one launch per digit, and one in front
// that clears three counters.  A workgroup owns kSortWg consecutive items, each of its four waves
// a quarter.  It counts its items per digit value, publishes the counts as a row of the matrix
// hist[workgroup][value], and waits until every workgroup of the launch has done so (all of them
// are resident: at most kSortMaxWgs workgroups on 256 CUs; the wait is bounded all the same, and a
// wait that runs out fails the sort).  It then finds its own offsets by summing the rows in front
// of it (a coalesced read of at most 256 KB, in place of a scan launch) and ranks its items with
// ballots as the general sort does.  The first digit's keys come straight from the masks, the last
// digit writes only the row order.
constexpr int kSortWg = 2048, kSortWaves = 4, kSortThreads = 64 * kSortWaves;
constexpr int kSortWave = kSortWg / kSortWaves, kSortSteps = kSortWave / 64;
constexpr int kSortMaxWgs = 64;
constexpr int kSortMaxBits = 10, kSortMaxBins = 1 << kSortMaxBits;
constexpr unsigned kSortSpinLimit = 1u << 20;  // polls of the arrival counter (about a second)
// head of the counter buffer: arrive[16 * pass], error at [48]
constexpr int kSortSyncWords = 64;
constexpr int kSortRound = 32;  // matrix rows a thread reads at a time

struct MaskKeys {
  const unsigned* mask;
  const int4* coords;  // null: no slabs
  const int* partial;  // kBoundsBlocks partial bounds
  int lo, width;
};

// the first wave folds the partial bounds and picks the longest axis: slab[0..2] = axis, lowest
// coordinate, extent
__device__ __forceinline__ void fold_bounds(const int* __restrict__ partial, int n_partial, int* slab) {
  if (threadIdx.x < 64) {
    int mn[3], mx[3];
    for (int a = 0; a < 3; ++a) {
      int l = 0x7FFFFFFF, h = (int)0x80000000;
      for (int b = threadIdx.x; b < n_partial; b += 64) {
        l = min(l, partial[b * 6 + a]);
        h = max(h, partial[b * 6 + 3 + a]);
      }
      for (int o = 32; o > 0; o >>= 1) {
        l = min(l, __shfl_xor(l, o));
        h = max(h, __shfl_xor(h, o));
      }
      mn[a] = l, mx[a] = h;
    }
    if (threadIdx.x == 0) {
      int axis = 0;
      for (int a = 1; a < 3; ++a)
        if ((long long)mx[a] - mn[a] > (long long)mx[axis] - mn[axis]) axis = a;
      slab[0] = axis;
      slab[1] = mn[axis];
      slab[2] = (int)min((long long)mx[axis] - mn[axis] + 1, (long long)0x7FFFFFFF);
    }
  }
}

// bits [lo, lo + width) of the row's mask, below the row's slab if there are slabs
__device__ __forceinline__ unsigned mask_key(const MaskKeys& mk, const int* slab, int r) {
  unsigned k = (mk.mask[r] >> mk.lo) & ((1u << mk.width) - 1u);
  if (mk.coords) {
    const int4 c = mk.coords[r];
    const int v = slab[0] == 0 ? c.y : slab[0] == 1 ? c.z : c.w;
    k |= (unsigned)(((long long)v - slab[1]) * kSlabs / slab[2]) << mk.width;  // slab 0 .. kSlabs-1
  }
  return k;
}

__global__ void __launch_bounds__(64) k_msort_clear(unsigned* __restrict__ sync) { sync[threadIdx.x] = 0; }

// KEYS: a plain sort of 32-bit keys (no rows travel with them; every digit writes the keys).
template <bool FIRST, bool LAST, bool KEYS = false>
__global__ void __launch_bounds__(kSortThreads)
    k_msort_pass(MaskKeys mk, const unsigned* __restrict__ kin, const int* __restrict__ vin,
                 unsigned* __restrict__ kout, int* __restrict__ vout, int rows, int shift, int bits,
                 unsigned* hist, unsigned* arrive, unsigned* error, unsigned error_bit) {
  __shared__ unsigned off[kSortWaves][kSortMaxBins];  // wave counts, then the waves' running places within the workgroup
  __shared__ unsigned first[kSortMaxBins];   // the workgroup's first place per digit value
  __shared__ unsigned part[2][kSortThreads][4];       // partial sums of the matrix rows: [before | total][thread][digit of quad]
  __shared__ unsigned wave_sum[kSortWaves];
  __shared__ int slab[3];
  const int wib = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bins = 1 << bits;
  const int begin = blockIdx.x * kSortWg + wib * kSortWave;
  for (int d = threadIdx.x; d < kSortWaves * kSortMaxBins; d += kSortThreads) (&off[0][0])[d] = 0;
  if (FIRST && mk.coords) fold_bounds(mk.partial, kBoundsBlocks, slab);
  if (FIRST) __syncthreads();
  // all of the wave's items are fetched up front (the ranking steps depend on each other)
  unsigned kreg[kSortSteps];
  int vreg[kSortSteps];
#pragma unroll
  for (int s = 0; s < kSortSteps; ++s) {
    const int i = begin + s * 64 + lane;
    kreg[s] = 0;
    vreg[s] = i;
    if (i < rows) {
      kreg[s] = FIRST ? mask_key(mk, slab, i) : kin[i];
      if (!FIRST && !KEYS) vreg[s] = vin[i];
    }
  }
  __syncthreads();
#pragma unroll
  for (int s = 0; s < kSortSteps; ++s)
    if (begin + s * 64 + lane < rows) atomicAdd(&off[wib][(kreg[s] >> shift) & (unsigned)(bins - 1)], 1u);
  __syncthreads();
  // publish this workgroup's counts (whole quads: the readers take four at a time); the wave
  // counts become the waves' first places within the workgroup's share of each digit value
  for (int d = threadIdx.x; d < (bins > 4 ? bins : 4); d += kSortThreads) {
    unsigned run = 0;
    for (int w = 0; w < kSortWaves; ++w) {
      const unsigned c = off[w][d];
      off[w][d] = run;
      run += c;
    }
    hist[(size_t)blockIdx.x * kSortMaxBins + d] = run;
  }
  // The way a grid-wide barrier is built: workgroup barrier, then one thread releases at device
  // scope (which covers what the workgroup's threads wrote before the barrier) and counts the
  // workgroup in; after the wait it acquires at device scope in front of a second workgroup barrier.
  __syncthreads();
  if (threadIdx.x == 0) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __hip_atomic_fetch_add(arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // While the other workgroups arrive: every item's place within the workgroup's share of its
  // digit value (ballots find the lanes with equal digits; the rank is the number of such lanes
  // below; the wave's running places live in LDS).
  const unsigned long long lt = (1ull << lane) - 1ull;
  unsigned lpos[kSortSteps];
#pragma unroll
  for (int s = 0; s < kSortSteps; ++s) {
    const bool valid = begin + s * 64 + lane < rows;
    const unsigned d = (kreg[s] >> shift) & (unsigned)(bins - 1);
    unsigned long long peers = __ballot(valid);
    for (int b = 0; b < bits; ++b) {
      const bool bit = (d >> b) & 1u;
      const unsigned long long bal = __ballot(bit);
      peers &= bit ? bal : ~bal;
    }
    const unsigned rank = (unsigned)__popcll(peers & lt);
    unsigned pos = 0;
    if (valid) pos = off[wib][d];
    __builtin_amdgcn_wave_barrier();  // every lane has read its place before a leader advances it
    if (valid && rank == 0) off[wib][d] = pos + (unsigned)__popcll(peers);
    __builtin_amdgcn_wave_barrier();
    lpos[s] = pos + rank;
  }
  if (threadIdx.x == 0) {
    unsigned polls = 0;
    while (__hip_atomic_load(arrive, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < gridDim.x) {
      if (++polls > kSortSpinLimit) {
        atomicOr(error, error_bit);
        break;
      }
      __builtin_amdgcn_s_sleep(2);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // the other workgroups' counts are read below
  }
  __syncthreads();
  // First places of this workgroup.  The matrix rows are summed by all threads: thread (g, q)
  // takes the four digit values of quad q in the rows w = g, g + ng, ...; before = items in the
  // workgroups in front, total = in all workgroups.
  const int nq = bins >= 4 ? bins / 4 : 1, ng = kSortThreads / nq;
  {
    const int q = threadIdx.x % nq, g = threadIdx.x / nq;
    unsigned before[4] = {0, 0, 0, 0}, total[4] = {0, 0, 0, 0};
    const unsigned* col = hist + 4 * q;
    // (rounds of kSortRound loads, all in flight together: the rows come from memory, and a load
    // that waits for the one before it costs a round trip each)
    for (int w0 = g; w0 < (int)gridDim.x; w0 += kSortRound * ng) {
      uint4 h[kSortRound];
#pragma unroll
      for (int i = 0; i < kSortRound; ++i) {
        const int w = w0 + i * ng;
        h[i] = make_uint4(0u, 0u, 0u, 0u);
        if (w < (int)gridDim.x) h[i] = *reinterpret_cast<const uint4*>(col + (size_t)w * kSortMaxBins);
      }
#pragma unroll
      for (int i = 0; i < kSortRound; ++i) {
        const unsigned hv[4] = {h[i].x, h[i].y, h[i].z, h[i].w};
        const bool front = w0 + i * ng < (int)blockIdx.x;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          total[j] += hv[j];
          before[j] += front ? hv[j] : 0u;
        }
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      part[0][threadIdx.x][j] = before[j];
      part[1][threadIdx.x][j] = total[j];
    }
  }
  __syncthreads();
  unsigned before[4] = {0, 0, 0, 0}, total[4] = {0, 0, 0, 0};
  const int d0 = 4 * threadIdx.x;  // thread t < nq owns digit values 4t .. 4t+3
  if (threadIdx.x < nq) {
    for (int g = 0; g < ng; ++g)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        before[j] += part[0][g * nq + threadIdx.x][j];
        total[j] += part[1][g * nq + threadIdx.x][j];
      }
  }
  const unsigned mine = total[0] + total[1] + total[2] + total[3];
  unsigned incl = mine;  // inclusive scan of the threads' sums
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const unsigned up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  if (lane == 63) wave_sum[wib] = incl;
  __syncthreads();
  unsigned base = incl - mine;
  for (int w = 0; w < wib; ++w) base += wave_sum[w];
  if (threadIdx.x < nq) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      first[d0 + j] = base + before[j];  // first place of digit value d0 + j for this workgroup
      base += total[j];
    }
  }
  __syncthreads();
#pragma unroll
  for (int s = 0; s < kSortSteps; ++s) {
    const bool valid = begin + s * 64 + lane < rows;
    const unsigned key = kreg[s];
    const unsigned pos = first[(key >> shift) & (unsigned)(bins - 1)] + lpos[s];
    if (valid && pos < (unsigned)rows) {  // (always below rows when the counters are consistent)
      if (!KEYS) vout[pos] = vreg[s];
      if (!LAST || KEYS) kout[pos] = key;
    }
  }
}

// Offline reordering (Section 3.2) of one part of the map, and the OR of each tile's keys.  A
// workgroup takes 256 consecutive places of the order (a whole number of tiles): perm_out[r] =
// row at place r (-1 in the padding), reordered[r][c] = map[perm[r]][lo + c], tilemask[t] = OR of
// the keys of tile t's rows.  If the sort reported a failed wait (*error != 0) the rows stay in map
// order: any order gives the same results, an order that is no permutation would not.
__global__ void __launch_bounds__(256)
    k_reorder_tiles(const int* __restrict__ map, const unsigned* __restrict__ mask, int V,
                    const int* __restrict__ sorted_rows, const unsigned* __restrict__ error, int rows, int lo,
                    int width, int tile_m, long long n_tiles, int* __restrict__ reordered,
                    int* __restrict__ perm_out, unsigned* __restrict__ tilemask) {
  __shared__ int src_of[256];
  __shared__ unsigned wave_or[4];
  const long long r = (long long)blockIdx.x * 256 + threadIdx.x;
  const bool failed = error && *error != 0;
  const int src = r < rows ? (failed ? (int)r : sorted_rows[r]) : -1;
  src_of[threadIdx.x] = src;
  if (blockIdx.y == 0) perm_out[r] = src;
  unsigned m = src >= 0 ? (mask[src] >> lo) & (width >= 32 ? 0xFFFFFFFFu : ((1u << width) - 1u)) : 0u;
  const int span = tile_m < 64 ? tile_m : 64;
  for (int o = span >> 1; o > 0; o >>= 1) m |= __shfl_xor(m, o);
  if ((threadIdx.x & 63) == 0) wave_or[threadIdx.x >> 6] = m;
  __syncthreads();
  if (blockIdx.y == 0 && threadIdx.x % tile_m == 0) {
    const long long t = r / tile_m;
    unsigned all = m;
    for (int w = 1; w < tile_m / 64; ++w) all |= wave_or[(threadIdx.x >> 6) + w];
    if (t < n_tiles) tilemask[t] = all;
  }
  // one thread per entry of the block's 256 x width entries (consecutive threads, consecutive
  // addresses); the workgroups of one blockIdx.x share them.  e / width for e < 6912 by a multiply:
  // (e + 0.5) / width stays 0.5 / 27 away from every integer, far beyond the rounding of the product.
  int* dst = reordered + (long long)blockIdx.x * 256 * width;
  const float inv_width = 1.0f / (float)width;
  for (int e = threadIdx.x + 256 * blockIdx.y; e < 256 * width; e += 256 * gridDim.y) {
    const int rr = (int)(((float)e + 0.5f) * inv_width);
    const int sr = src_of[rr];
    dst[e] = sr >= 0 ? map[(long long)sr * V + lo + (e - rr * width)] : -1;
  }
}

// tilemask[t] = OR over the tile's rows of their split keys.  One wave per tile.
// perm == nullptr: rows in map order.
__global__ void __launch_bounds__(256)
    k_tile_mask(const unsigned* __restrict__ mask, const int* __restrict__ perm, long long rows, int tile_m, int lo,
                int width, long long n_tiles, unsigned* __restrict__ tilemask) {
  const int lane = threadIdx.x & 63;
  const long long t = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  if (t >= n_tiles) return;
  unsigned m = 0;
  for (int i = lane; i < tile_m; i += 64) {
    const long long r = t * tile_m + i;
    if (r < rows) {
      const int src = perm ? perm[r] : (int)r;
      if (src >= 0) m |= mask[src];
    }
  }
  for (int o = 32; o > 0; o >>= 1) m |= __shfl_xor(m, o);
  if (lane == 0) tilemask[t] = (m >> lo) & (width >= 32 ? 0xFFFFFFFFu : ((1u << width) - 1u));
}

// executed MAC units: for every group of `group` consecutive (sorted) rows,
// popcount(OR of keys) * real rows in the group
__global__ void __launch_bounds__(256)
    k_mac_units(const unsigned* __restrict__ mask, const int* __restrict__ perm, long long rows, int group, int lo,
                int width, unsigned long long* __restrict__ executed) {
  const long long g = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long r0 = g * group;
  unsigned long long mine = 0;
  if (r0 < rows) {
    unsigned m = 0;
    int real = 0;
    for (int i = 0; i < group; ++i) {
      const long long r = r0 + i;
      if (r < rows) {
        const int src = perm ? perm[r] : (int)r;
        if (src >= 0) {
          m |= mask[src];
          ++real;
        }
      }
    }
    m = (m >> lo) & (width >= 32 ? 0xFFFFFFFFu : ((1u << width) - 1u));
    mine = (unsigned long long)__popc(m) * (unsigned long long)real;
  }
  for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o);
  if ((threadIdx.x & 63) == 0 && mine) atomicAdd(executed, mine);
}

// Per-offset pair counts of chunks of wave_rows rows (a multiple of 256): counts[k][chunk].  A
// workgroup takes one chunk, each of its four waves a quarter of it (more waves in flight than one
// wave per chunk, same number of counters to scan).  A ballot per offset turns the 64 masks held by
// the lanes into that offset's count; lane k keeps the running count of offset k.
__device__ __forceinline__ unsigned count_offsets(const unsigned* __restrict__ mask, long long rows, long long first,
                                                  int steps, int V, int lane) {
  unsigned mine = 0;
  for (int it = 0; it < steps; ++it) {
    const long long r = first + it * 64 + lane;
    const unsigned m = r < rows ? mask[r] : 0u;
    for (int k = 0; k < V; ++k) {
      const unsigned long long bal = __ballot((m >> k) & 1u);
      if (lane == k) mine += (unsigned)__popcll(bal);
    }
  }
  return mine;
}

__global__ void __launch_bounds__(256)
    k_pair_count(const unsigned* __restrict__ mask, long long rows, int V, int n_chunks, int wave_rows,
                 unsigned* __restrict__ counts) {
  __shared__ unsigned part[4][32];
  const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
  const long long w = blockIdx.x;
  if (w >= n_chunks) return;
  const int sub = wave_rows / 4;
  const unsigned mine = count_offsets(mask, rows, w * wave_rows + (long long)wib * sub, sub / 64, V, lane);
  if (lane < 32) part[wib][lane] = lane < V ? mine : 0u;
  __syncthreads();
  if (wib == 0 && lane < V) counts[(long long)lane * n_chunks + w] = part[0][lane] + part[1][lane] + part[2][lane] + part[3][lane];
  if (w == 0 && threadIdx.x == 63) counts[(long long)V * n_chunks] = 0;  // the slot that will receive the total
}

// Cuts every offset's pair range into ceil(count / target) nearly equal work items.  Called by a
// whole workgroup; begin_of(k) returns the scanned pair offset of offset k (k = V: the total).
template <typename BeginOf>
__device__ __forceinline__ void make_items(BeginOf begin_of, int V, unsigned target, int max_items, int* seg,
                                           WgradItem* items, int* item_seg) {
  __shared__ unsigned s_begin[33], s_cnt[33], s_first[34];
  const int lane = threadIdx.x;
  if (lane < 64) {  // the first wave works out the per-offset figures
    const unsigned begin = lane <= V ? begin_of(lane) : 0u;
    const unsigned next = __shfl_down(begin, 1);
    const unsigned cnt = lane < V ? next - begin : 0u;
    if (lane <= V) seg[lane] = (int)begin;
    const unsigned pieces = cnt ? (cnt + target - 1) / target : 0u;
    unsigned incl = pieces;
    for (int o = 1; o < 64; o <<= 1) {
      const unsigned up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    unsigned first = incl - pieces;
    if (first > (unsigned)max_items) first = (unsigned)max_items;
    if (lane <= V) {
      s_begin[lane] = begin;
      s_cnt[lane] = cnt;
      s_first[lane] = first;
      item_seg[lane] = (int)first;
    }
    if (lane == V) {
      s_first[V + 1] = first;
      item_seg[V + 1] = (int)first;
    }
  }
  __syncthreads();
  const unsigned n_items = s_first[V];
  for (unsigned i = lane; i < n_items; i += blockDim.x) {
    int k = 0;
    while (k + 1 < V && s_first[k + 1] <= i) ++k;
    const unsigned c = s_cnt[k], pc = s_first[k + 1] - s_first[k], q = i - s_first[k];
    // c * q / pc with c = a * pc + r
    const unsigned a = c / pc, r = c - a * pc;
    WgradItem w;
    w.k = k;
    w.pair_begin = (int)(s_begin[k] + a * q + (unsigned)(((unsigned long long)r * q) / pc));
    w.pair_end = (int)(s_begin[k] + a * (q + 1) + (unsigned)(((unsigned long long)r * (q + 1)) / pc));
    w.pad = 0;
    items[i] = w;
  }
}

// Most chunks for which the fill kernel adds up the per-chunk counts by itself: 64 lanes x steps.
constexpr int kSelfScanSteps = 10;
constexpr int kSelfScanChunks = 64 * kSelfScanSteps;

// Writes the pairs (n, M[n][k]) of every offset in row order.  A workgroup takes one chunk: each
// wave recounts its quarter, so that it knows where its rows start inside the chunk's range of
// every offset.  The 64 map rows of a step are first copied to LDS with coalesced loads that are
// all in flight together; the per-offset ballots then rank the present entries.  No pair is
// written past pairs_cap.
// Where the chunk's range starts: with SELF_SCAN the workgroup adds up the raw per-chunk counts
// itself (every offset's total, and the part of it that the chunks before this one hold; 27 x
// chunks counters, read from L2 by every workgroup, which is cheaper than a scan launch in between
// while there are a few hundred chunks), and workgroup 0 also cuts the work items; otherwise
// `counts` was scanned before the launch and the items are made elsewhere.
template <int V, bool SELF_SCAN>
__global__ void __launch_bounds__(256)
    k_pair_fill(const int* __restrict__ map, const unsigned* __restrict__ mask, long long rows, int n_chunks,
                int wave_rows, const unsigned* __restrict__ counts, int2* __restrict__ pairs, long long pairs_cap,
                unsigned target, int max_items, int* __restrict__ seg, WgradItem* __restrict__ items,
                int* __restrict__ item_seg) {
  __shared__ int slab[4][64 * V];
  __shared__ unsigned part[4][32];
  __shared__ unsigned s_before[32], s_total[32], s_seg[34];
  const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
  const long long w = blockIdx.x;
  if (w >= n_chunks) return;
  const int sub = wave_rows / 4;
  const long long first = w * wave_rows + (long long)wib * sub;
  // a wave per offset (wib, wib + 4, ...), lanes over the chunks; every counter load is issued
  // before the first is used
  constexpr int KPW = (V + 3) / 4;
  unsigned cv[SELF_SCAN ? KPW : 1][SELF_SCAN ? kSelfScanSteps : 1];
  if constexpr (SELF_SCAN) {
#pragma unroll
    for (int q = 0; q < KPW; ++q) {
      const int k = wib + 4 * q;
#pragma unroll
      for (int i = 0; i < kSelfScanSteps; ++i) {
        const int j = lane + 64 * i;
        cv[q][i] = (k < V && j < n_chunks) ? counts[(long long)k * n_chunks + j] : 0u;
      }
    }
  }
  const unsigned mine = count_offsets(mask, rows, first, sub / 64, V, lane);
  if (lane < 32) part[wib][lane] = lane < V ? mine : 0u;
  if constexpr (SELF_SCAN) {
#pragma unroll
    for (int q = 0; q < KPW; ++q) {
      const int k = wib + 4 * q;
      unsigned tot = 0, bef = 0;
#pragma unroll
      for (int i = 0; i < kSelfScanSteps; ++i) {
        tot += cv[q][i];
        if (lane + 64 * i < w) bef += cv[q][i];
      }
      for (int o = 32; o > 0; o >>= 1) {
        tot += __shfl_xor(tot, o);
        bef += __shfl_xor(bef, o);
      }
      if (lane == 0 && k < V) {
        s_total[k] = tot;
        s_before[k] = bef;
      }
    }
    __syncthreads();
    if (wib == 0) {  // where each offset's pairs begin: exclusive scan of the totals; [V] = all pairs
      const unsigned t = lane < V ? s_total[lane] : 0u;
      unsigned incl = t;
      for (int o = 1; o < 64; o <<= 1) {
        const unsigned up = __shfl_up(incl, o);
        if (lane >= o) incl += up;
      }
      if (lane <= V) s_seg[lane] = incl - t;
    }
  }
  __syncthreads();
  unsigned base = 0;  // lane k: next slot of offset k
  if (lane < V) {
    if constexpr (SELF_SCAN)
      base = s_seg[lane] + s_before[lane];
    else
      base = counts[(long long)lane * n_chunks + w];
    for (int i = 0; i < wib; ++i) base += part[i][lane];
  }
  if constexpr (SELF_SCAN) {
    if (w == 0) make_items([&](int k) { return s_seg[k]; }, V, target, max_items, seg, items, item_seg);
  }
  const unsigned long long lt = (1ull << lane) - 1ull;
  int* ms = slab[wib];
  for (int it = 0; it < sub / 64; ++it) {
    const long long r0 = first + it * 64;
    if (r0 >= rows) break;
    const long long r = r0 + lane;
    const unsigned m = r < rows ? mask[r] : 0u;
    // rows r0 .. r0+63 are contiguous in the padded map (rows_pad is a multiple of 256)
    const int* src = map + r0 * V;
    int tmp[V];
#pragma unroll
    for (int i = 0; i < V; ++i) tmp[i] = src[lane + 64 * i];
#pragma unroll
    for (int i = 0; i < V; ++i) ms[lane + 64 * i] = tmp[i];
    __builtin_amdgcn_wave_barrier();
    for (int k = 0; k < V; ++k) {
      const bool bit = (m >> k) & 1u;
      const unsigned long long bal = __ballot(bit);
      const unsigned slot = __shfl(base, k) + (unsigned)__popcll(bal & lt);
      if (bit && (long long)slot < pairs_cap) pairs[slot] = make_int2((int)r, ms[lane * V + k]);
      if (lane == k) base += (unsigned)__popcll(bal);
    }
    __builtin_amdgcn_wave_barrier();
  }
}

__global__ void __launch_bounds__(256)
    k_make_items(const unsigned* __restrict__ scanned, int V, int n_waves, unsigned target, int max_items,
                 int* __restrict__ seg, WgradItem* __restrict__ items, int* __restrict__ item_seg) {
  make_items([&](int k) { return scanned[(long long)k * n_waves]; }, V, target, max_items, seg, items, item_seg);
}

}  // namespace

// Sorts n 32-bit keys of key_bits significant bits with the one-launch-per-digit sort above (at
// most kSortMaxWgs * kSortWg keys: SPCONV_EINVAL beyond, and the caller takes the general sort).
// A wait that runs out sets error_bit in *error_word (device memory that the caller reads back
// later): the keys are then not sorted and the caller must sort them again.
int msort_keys_u32(uint32_t* key_a, uint32_t* key_b, int64_t n, int key_bits, unsigned* error_word, unsigned error_bit,
                   hipStream_t st, int* in_b) {
  *in_b = 0;
  if (n <= 1 || key_bits <= 0) return SPCONV_OK;
  const int n_wg = (int)ceil_div(n, kSortWg);
  if (n_wg > kSortMaxWgs || key_bits > 32) return SPCONV_EINVAL;
  DevBuf hist;
  const size_t hist_elems = (size_t)n_wg * kSortMaxBins;
  const int passes = (key_bits + kSortMaxBits - 1) / kSortMaxBits;
  const int bits = (key_bits + passes - 1) / passes;
  SPC_TRY(hist.alloc((kSortSyncWords + (size_t)passes * hist_elems) * sizeof(uint32_t)));
  unsigned* sync = hist.as<unsigned>();
  hipLaunchKernelGGL(k_msort_clear, dim3(1), dim3(kSortSyncWords), 0, st, sync);
  SPC_LAUNCH_CHECK();
  const MaskKeys none{};
  int shift = 0;
  for (int p = 0; p < passes; ++p) {  // (passes <= 4: arrival counters at sync[16 p], p < 4)
    const int b = shift + bits <= key_bits ? bits : key_bits - shift;
    const unsigned* kin = *in_b ? key_b : key_a;
    unsigned* kout = *in_b ? key_a : key_b;
    hipLaunchKernelGGL((k_msort_pass<false, false, true>), dim3((unsigned)n_wg), dim3(kSortThreads), 0, st, none, kin,
                       (const int*)nullptr, kout, (int*)nullptr, (int)n, shift, b,
                       sync + kSortSyncWords + (size_t)p * hist_elems, sync + 16 * p, error_word, error_bit);
    SPC_LAUNCH_CHECK();
    *in_b ^= 1;
    shift += b;
  }
  return SPCONV_OK;
}

int plan_shape(int V, int64_t rows, int n_split, int tile_m, PlanShape* s) {
  // every part needs at least one offset (a K = 1 map has a single one): the kernels index the
  // last column of a part's map
  if (V < 1 || V > 27 || rows < 0 || n_split < 0 || n_split > kMaxSplit || n_split > V) return SPCONV_EINVAL;
  if (tile_m != 16 && tile_m != 64 && tile_m != 128 && tile_m != 256) return SPCONV_EINVAL;
  *s = PlanShape{};
  s->parts = std::max(1, n_split);
  s->rows_pad = round_up(rows > 0 ? rows : 1, kRowPad);  // a multiple of every tile height: tiles never run past the map
  s->n_tiles = ceil_div(rows, tile_m);
  size_t off = 0;
  for (int i = 0; i < s->parts; ++i) {
    s->lo[i] = (int)(((int64_t)i * V) / s->parts);
    s->width[i] = (int)(((int64_t)(i + 1) * V) / s->parts) - s->lo[i];
    s->map_off[i] = off;
    off += (size_t)s->rows_pad * s->width[i];
  }
  s->map_elems = off;
  return SPCONV_OK;
}

int plan_get(spconv_kmap* km, SideMap& side, int n_split, int tile_m, hipStream_t st, IgemmPlan** out) {
  const bool force_slabs = (tile_m & kPlanSlabs) != 0 && n_split > 0;
  auto key = std::make_pair(n_split, n_split > 0 ? tile_m : (tile_m & ~kPlanSlabs));
  tile_m &= ~kPlanSlabs;
  PlanShape sh;
  SPC_TRY(plan_shape(km->V, side.rows, n_split, tile_m, &sh));
  if (side.rows > 0 && sh.rows_pad != side.rows_pad) return SPCONV_EINVAL;  // (the map was padded by the same rule)
  auto it = side.plans.find(key);
  if (it != side.plans.end()) {
    *out = it->second.get();
    return SPCONV_OK;
  }
  std::unique_ptr<IgemmPlan> p(new (std::nothrow) IgemmPlan);
  if (!p) return SPCONV_ENOMEM;
  const int V = km->V;
  p->n_split = n_split;
  p->tile_m = tile_m;
  p->parts = sh.parts;
  p->rows = side.rows;
  p->rows_pad = sh.rows_pad;
  p->n_tiles = sh.n_tiles;
  for (int i = 0; i < p->parts; ++i) {
    p->lo[i] = sh.lo[i];
    p->width[i] = sh.width[i];
    p->map_off[i] = sh.map_off[i];
  }
  const size_t off = sh.map_elems;
  const int64_t tiles_alloc = std::max<int64_t>(1, p->n_tiles);
  SPC_TRY(p->tilemask.alloc((size_t)p->parts * tiles_alloc * sizeof(unsigned)));
  const unsigned tile_blocks = blocks_for(tiles_alloc, 4);
  if (n_split == 0) {
    // (16-row blocks are the wave kernel's; it ORs the row masks itself, so no launch here)
    if (p->n_tiles > 0 && tile_m != 16) {
      hipLaunchKernelGGL(k_tile_mask, dim3(tile_blocks), dim3(256), 0, st, side.mask.as<unsigned>(),
                         (const int*)nullptr, (long long)p->rows, tile_m, 0, V, (long long)p->n_tiles,
                         p->tilemask.as<unsigned>());
      SPC_LAUNCH_CHECK();
    }
  } else {
    SPC_TRY(p->maps.alloc(off * sizeof(int)));
    SPC_TRY(p->perm.alloc((size_t)p->parts * p->rows_pad * sizeof(int)));
    if (p->rows > 0) {
      // the coordinates of the side's rows (slabs need them; a width of 27 + 3 bits still fits the key)
      const DevBuf& crd = (&side == &km->out_side) ? (km->submanifold() ? km->in_coords : km->out_coords)
                                                    : ((km->transposed && km->stride == 1) ? km->out_coords : km->in_coords);
      const bool slabs = (force_slabs || p->rows >= kSlabMinRows) && crd.p && crd.bytes >= (size_t)p->rows * 16;
      p->slabs = slabs;
      DevBuf bounds;
      if (slabs) {
        SPC_TRY(bounds.alloc((size_t)kBoundsBlocks * 6 * sizeof(int)));
        hipLaunchKernelGGL(k_coord_bounds, dim3(kBoundsBlocks), dim3(256), 0, st, crd.as<int4>(), (int)p->rows,
                           bounds.as<int>());
        SPC_LAUNCH_CHECK();
      }
      DevBuf key_a, key_b, val_a, val_b, hist;
      const size_t n = (size_t)p->rows;
      const int n_wg = (int)ceil_div(p->rows, kSortWg);
      const bool few_launches = n_wg <= kSortMaxWgs;
      SPC_TRY(key_a.alloc(n * 4));
      SPC_TRY(key_b.alloc(n * 4));
      SPC_TRY(val_a.alloc(n * 4));
      SPC_TRY(val_b.alloc(n * 4));
      const size_t hist_elems = (size_t)n_wg * kSortMaxBins;
      SPC_TRY(hist.alloc((few_launches ? kSortSyncWords + 3 * hist_elems : sort_hist_elems(p->rows)) * sizeof(uint32_t)));
      for (int i = 0; i < p->parts; ++i) {
        const int key_bits = p->width[i] + (slabs ? kSlabBits : 0);
        const int* sorted_rows = nullptr;
        if (few_launches) {
          const MaskKeys mk{side.mask.as<unsigned>(), slabs ? crd.as<int4>() : (const int4*)nullptr, bounds.as<int>(),
                            p->lo[i], p->width[i]};
          const int passes = (key_bits + kSortMaxBits - 1) / kSortMaxBits;  // <= 3: key_bits <= 30
          const int bits = (key_bits + passes - 1) / passes;
          unsigned* sync = hist.as<unsigned>();
          unsigned* h[3] = {sync + kSortSyncWords, sync + kSortSyncWords + hist_elems,
                            sync + kSortSyncWords + 2 * hist_elems};
          unsigned *ka = key_a.as<unsigned>(), *kb = key_b.as<unsigned>();
          int *va = val_a.as<int>(), *vb = val_b.as<int>();
          const dim3 grid((unsigned)n_wg), block(kSortThreads);
          const int rows_i = (int)p->rows;
          const int b_last = key_bits - (passes - 1) * bits;  // width of the last digit
          unsigned* err = sync + 48;
          hipLaunchKernelGGL(k_msort_clear, dim3(1), dim3(kSortSyncWords), 0, st, sync);
          SPC_LAUNCH_CHECK();
          if (passes == 1) {
            hipLaunchKernelGGL((k_msort_pass<true, true>), grid, block, 0, st, mk, (const unsigned*)nullptr,
                               (const int*)nullptr, (unsigned*)nullptr, vb, rows_i, 0, bits, h[0], sync, err, 1u);
            sorted_rows = vb;
          } else if (passes == 2) {
            hipLaunchKernelGGL((k_msort_pass<true, false>), grid, block, 0, st, mk, (const unsigned*)nullptr,
                               (const int*)nullptr, kb, vb, rows_i, 0, bits, h[0], sync, err, 1u);
            SPC_LAUNCH_CHECK();
            hipLaunchKernelGGL((k_msort_pass<false, true>), grid, block, 0, st, mk, (const unsigned*)kb,
                               (const int*)vb, (unsigned*)nullptr, va, rows_i, bits, b_last, h[1], sync + 16, err, 1u);
            sorted_rows = va;
          } else {
            hipLaunchKernelGGL((k_msort_pass<true, false>), grid, block, 0, st, mk, (const unsigned*)nullptr,
                               (const int*)nullptr, kb, vb, rows_i, 0, bits, h[0], sync, err, 1u);
            SPC_LAUNCH_CHECK();
            hipLaunchKernelGGL((k_msort_pass<false, false>), grid, block, 0, st, mk, (const unsigned*)kb,
                               (const int*)vb, ka, va, rows_i, bits, bits, h[1], sync + 16, err, 1u);
            SPC_LAUNCH_CHECK();
            hipLaunchKernelGGL((k_msort_pass<false, true>), grid, block, 0, st, mk, (const unsigned*)ka,
                               (const int*)va, (unsigned*)nullptr, vb, rows_i, 2 * bits, b_last, h[2], sync + 32, err, 1u);
            sorted_rows = vb;
          }
          SPC_LAUNCH_CHECK();
        } else {
          hipLaunchKernelGGL(k_split_keys, dim3(blocks_for(p->rows, 256)), dim3(256), 0, st,
                             side.mask.as<unsigned>(), (int)p->rows, p->lo[i], p->width[i],
                             slabs ? crd.as<int4>() : (const int4*)nullptr, bounds.as<int>(), kBoundsBlocks,
                             key_a.as<unsigned>(), val_a.as<int>());
          SPC_LAUNCH_CHECK();
          int in_b = 0;
          SPC_TRY(radix_sort_u32(key_a.as<uint32_t>(), key_b.as<uint32_t>(), val_a.as<int32_t>(), val_b.as<int32_t>(),
                                 p->rows, key_bits, hist.as<uint32_t>(), st, &in_b));
          sorted_rows = in_b ? val_b.as<int>() : val_a.as<int>();
        }
        int* perm_i = p->perm.as<int>() + (size_t)i * p->rows_pad;
        hipLaunchKernelGGL(k_reorder_tiles, dim3((unsigned)(p->rows_pad / 256), 8), dim3(256), 0, st, side.map.as<int>(),
                           side.mask.as<unsigned>(), V, sorted_rows,
                           few_launches ? (const unsigned*)(hist.as<unsigned>() + 48) : (const unsigned*)nullptr,
                           (int)p->rows, p->lo[i], p->width[i], tile_m,
                           (long long)p->n_tiles, p->maps.as<int>() + p->map_off[i], perm_i,
                           p->tilemask.as<unsigned>() + (size_t)i * tiles_alloc);
        SPC_LAUNCH_CHECK();
      }
      // the sort temporaries return to the pool while the stream may still use them;
      // later users are ordered behind on the same stream
    }
  }
  *out = p.get();
  side.plans[key] = std::move(p);
  return SPCONV_OK;
}

int plan_mac_units(spconv_kmap* km, SideMap& side, IgemmPlan* plan, int group_rows, hipStream_t st,
                   int64_t* executed) {
  (void)km;
  *executed = 0;
  if (plan->rows == 0) return SPCONV_OK;
  DevBuf acc;
  SPC_TRY(acc.alloc(8));
  SPC_HIP(hipMemsetAsync(acc.p, 0, 8, st));
  const int64_t groups = ceil_div(plan->rows, group_rows);
  for (int i = 0; i < plan->parts; ++i) {
    const int* perm = plan->n_split ? plan->perm.as<int>() + (size_t)i * plan->rows_pad : nullptr;
    hipLaunchKernelGGL(k_mac_units, dim3(blocks_for(groups, 256)), dim3(256), 0, st, side.mask.as<unsigned>(),
                       perm, (long long)plan->rows, group_rows, plan->lo[i], plan->width[i],
                       acc.as<unsigned long long>());
    SPC_LAUNCH_CHECK();
  }
  unsigned long long h = 0;
  SPC_HIP(hipMemcpyAsync(&h, acc.p, 8, hipMemcpyDeviceToHost, st));
  SPC_HIP(hipStreamSynchronize(st));
  *executed = (int64_t)h;
  return SPCONV_OK;
}

int wplan_get(spconv_kmap* km, int64_t target_pairs, hipStream_t st, WgradPlan** out) {
  const int64_t requested = target_pairs;  // (the cache key; the item size may be raised below)
  auto it = km->wplans.find(target_pairs);
  if (it != km->wplans.end()) {
    *out = it->second.get();
    return SPCONV_OK;
  }
  // The pair count is known after a synchronous submanifold build.  While an asynchronous build is
  // pending, sizes come from the bound n_out * V (surplus workgroups exit at once); maps built with
  // stride > 1 count their pairs here (one synchronisation).
  if (km->n_pairs < 0 && !km->pending) SPC_TRY(kmap_count_pairs(km, st, nullptr));
  std::unique_ptr<WgradPlan> p(new (std::nothrow) WgradPlan);
  if (!p) return SPCONV_ENOMEM;
  const int V = km->V;
  const SideMap& side = km->out_side;
  p->pairs_cap = km->n_pairs >= 0 ? km->n_pairs : km->n_out * V;
  // At most 2^20 work items: a smaller request is raised to the item size that covers every pair
  // (the item cutter gives later offsets no item once the list is full, which would drop pairs).
  constexpr int64_t kMaxItems = 1 << 20;
  if (V + ceil_div(p->pairs_cap, target_pairs) > kMaxItems) target_pairs = ceil_div(p->pairs_cap, kMaxItems - V);
  p->target_pairs = target_pairs;
  p->max_items = (int)(V + ceil_div(p->pairs_cap, target_pairs));
  // rows per chunk (one workgroup, a quarter per wave): 256, or the next power of two up to 2048
  // that lets the fill kernel add up the counters itself
  int wave_rows = 256;
  while (ceil_div(km->n_out, wave_rows) > kSelfScanChunks && wave_rows < 2048) wave_rows *= 2;
  const int n_waves = (int)std::max<int64_t>(1, ceil_div(km->n_out, wave_rows));  // chunks
  const size_t n_counts = (size_t)V * n_waves + 1;  // the extra counter ends up holding the total
  const size_t n_sums = scan_sums_elems((int64_t)n_counts);
  DevBuf counts;
  SPC_TRY(counts.alloc((n_counts + n_sums) * sizeof(unsigned)));
  SPC_TRY(p->pairs.alloc(std::max<size_t>(1, (size_t)p->pairs_cap) * sizeof(int2)));
  SPC_TRY(p->seg.alloc((size_t)(V + 1) * sizeof(int)));
  SPC_TRY(p->items.alloc((size_t)p->max_items * sizeof(WgradItem)));
  SPC_TRY(p->item_seg.alloc((size_t)(V + 2) * sizeof(int)));
  const unsigned blocks = (unsigned)n_waves;  // one workgroup per chunk
  hipLaunchKernelGGL(k_pair_count, dim3(blocks), dim3(256), 0, st, side.mask.as<unsigned>(), (long long)km->n_out, V,
                     n_waves, wave_rows, counts.as<unsigned>());
  SPC_LAUNCH_CHECK();
  // Up to kSelfScanChunks chunks the fill kernel adds up the raw counts itself; beyond that (its
  // reads grow with the square of the chunk count) they are scanned by launches of their own.
  const bool self_scan = n_waves <= kSelfScanChunks;
  if (!self_scan) {
    SPC_TRY(scan_u32_inplace(counts.as<uint32_t>(), (int64_t)n_counts, counts.as<uint32_t>() + n_counts, st));
    hipLaunchKernelGGL(k_make_items, dim3(1), dim3(256), 0, st, counts.as<unsigned>(), V, n_waves,
                       (unsigned)target_pairs, p->max_items, p->seg.as<int>(), p->items.as<WgradItem>(),
                       p->item_seg.as<int>());
    SPC_LAUNCH_CHECK();
  }
  const int* mp = side.map.as<int>();
  const unsigned* mk = side.mask.as<unsigned>();
  const long long cap = (long long)std::max<int64_t>(1, p->pairs_cap);  // elements the pair buffer holds
#define SPC_FILL(VV, SELF)                                                                                       \
  hipLaunchKernelGGL((k_pair_fill<VV, SELF>), dim3(blocks), dim3(256), 0, st, mp, mk, (long long)km->n_out,       \
                     n_waves, wave_rows, counts.as<unsigned>(), p->pairs.as<int2>(), cap, (unsigned)target_pairs, \
                     p->max_items, p->seg.as<int>(), p->items.as<WgradItem>(), p->item_seg.as<int>())
  if (V == 27) {
    if (self_scan) SPC_FILL(27, true); else SPC_FILL(27, false);
  } else if (V == 25) {  // a plane of a K = 5 map
    if (self_scan) SPC_FILL(25, true); else SPC_FILL(25, false);
  } else if (V == 8) {
    if (self_scan) SPC_FILL(8, true); else SPC_FILL(8, false);
  } else {
    if (self_scan) SPC_FILL(1, true); else SPC_FILL(1, false);
  }
#undef SPC_FILL
  SPC_LAUNCH_CHECK();
  *out = p.get();
  km->wplans[requested] = std::move(p);
  return SPCONV_OK;
}

}  // namespace spc
