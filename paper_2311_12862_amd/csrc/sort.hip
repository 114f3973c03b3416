// Stable least-significant-digit radix sort built from wavefront primitives.
//
// Each wave owns a contiguous run of kItemsPerWave items.  A pass is three
// launches: per-wave digit histograms (LDS atomics, wave-private counters),
// one exclusive scan over the [digit][wave] matrix, and a scatter in which a
// wave ranks its 64 items per step with ballots (lanes with equal digits find
// each other from one ballot per digit bit; the rank is the number of peers in
// lower lanes) against wave-private running offsets held in LDS.  Used for
// putting the output coordinates of strided maps into their canonical order,
// and for the bitmask argsort of Sections 2.2.3 / 4.1 on maps too large for
// the one-launch-per-digit sort in plan.hip.
#include "common.h"

#include <atomic>

namespace spc {
namespace {

constexpr int kItemsPerWave = 512;
constexpr int kMaxBits = 10;
constexpr int kMaxBins = 1 << kMaxBits;

template <typename KeyT>
__global__ void __launch_bounds__(256) k_radix_hist(const KeyT* __restrict__ keys, long long n, int shift, int bits,
                                                    unsigned* __restrict__ hist, int n_waves, int ipw) {
  __shared__ unsigned cnt[4][kMaxBins];
  const int wib = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long long w = (long long)blockIdx.x * 4 + wib;
  const int bins = 1 << bits;
  for (int d = lane; d < bins; d += 64) cnt[wib][d] = 0;
  __syncthreads();
  if (w < n_waves) {
    const long long begin = w * ipw;
    const long long end = begin + ipw < n ? begin + ipw : n;
    for (long long i = begin + lane; i < end; i += 64)
      atomicAdd(&cnt[wib][(unsigned)(keys[i] >> shift) & (unsigned)(bins - 1)], 1u);
  }
  __syncthreads();
  if (w < n_waves)
    for (int d = lane; d < bins; d += 64) hist[(long long)d * n_waves + w] = cnt[wib][d];
}

// Exclusive scan of `elems` counters in place.  A workgroup of 1024 threads scans one tile of
// 8192 counters through LDS so that global accesses are coalesced: each thread scans 8
// consecutive counters (LDS index skewed by one word per 32 to stay off bank conflicts) and a
// wave-shuffle scan combines the threads.  One tile: a single launch.  More: every tile is
// scanned by its own workgroup, the tile totals are scanned by one more launch, and a third
// adds each tile's offset.
constexpr int kScanPer = 8;
constexpr int kScanTile = 1024 * kScanPer;
constexpr int kScanBigPer = 32;  // one workgroup alone scans up to 32768 counters (135 KB of LDS)
constexpr int kScanBig = 1024 * kScanBigPer;
__device__ __forceinline__ int scan_skew(int x) { return x + (x >> 5); }
template <int PER> constexpr size_t scan_lds_bytes() { return (size_t)(1024 * PER + 1024 * PER / 32 + 8) * 4; }

template <int kScanPer>
__global__ void __launch_bounds__(1024) k_scan_tile(unsigned* __restrict__ data, long long elems,
                                                    unsigned* __restrict__ tile_sums) {
  constexpr int kScanTile = 1024 * kScanPer;
  extern __shared__ unsigned tile[];
  __shared__ unsigned wave_sum[16];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const long long base = (long long)blockIdx.x * kScanTile;
#pragma unroll
  for (int i = 0; i < kScanPer; ++i) {
    const long long g = base + i * 1024 + t;
    tile[scan_skew(i * 1024 + t)] = g < elems ? data[g] : 0u;
  }
  __syncthreads();
  unsigned v[kScanPer], sum = 0;
#pragma unroll
  for (int i = 0; i < kScanPer; ++i) {
    v[i] = tile[scan_skew(t * kScanPer + i)];
    sum += v[i];
  }
  unsigned incl = sum;  // inclusive scan across the wave
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const unsigned up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  if (lane == 63) wave_sum[wave] = incl;
  __syncthreads();
  unsigned before = 0;
  for (int w = 0; w < wave; ++w) before += wave_sum[w];
  unsigned run = before + incl - sum;
#pragma unroll
  for (int i = 0; i < kScanPer; ++i) {
    tile[scan_skew(t * kScanPer + i)] = run;
    run += v[i];
  }
  if (t == 1023 && tile_sums) tile_sums[blockIdx.x] = run;  // the tile's total
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kScanPer; ++i) {
    const long long g = base + i * 1024 + t;
    if (g < elems) data[g] = tile[scan_skew(i * 1024 + t)];
  }
}

__global__ void __launch_bounds__(1024) k_scan_add(unsigned* __restrict__ data, long long elems,
                                                   const unsigned* __restrict__ tile_offs) {
  const unsigned off = tile_offs[blockIdx.x];
  const long long base = (long long)blockIdx.x * kScanTile;
#pragma unroll
  for (int i = 0; i < kScanPer; ++i) {
    const long long g = base + i * 1024 + threadIdx.x;
    if (g < elems) data[g] += off;
  }
}

template <typename KeyT, bool HAS_VAL>
__global__ void __launch_bounds__(256)
    k_radix_scatter(const KeyT* __restrict__ kin, KeyT* __restrict__ kout, const int* __restrict__ vin,
                    int* __restrict__ vout, long long n, int shift, int bits, const unsigned* __restrict__ hist,
                    int n_waves, int ipw) {
  __shared__ unsigned off[4][kMaxBins];
  const int wib = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long long w = (long long)blockIdx.x * 4 + wib;
  const int bins = 1 << bits;
  if (w < n_waves)
    for (int d = lane; d < bins; d += 64) off[wib][d] = hist[(long long)d * n_waves + w];
  __syncthreads();
  if (w >= n_waves) return;
  const long long begin = w * ipw;
  const long long end = begin + ipw < n ? begin + ipw : n;
  const unsigned long long lt = (1ull << lane) - 1ull;
  // all of the wave's keys (and values) are fetched up front: the ranking steps below depend on
  // each other through the running offsets, and a load inside them would expose its latency
  // once per step
  constexpr int STEPS = kItemsPerWave / 64;
  KeyT kreg[STEPS];
  int vreg[STEPS];
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    const long long i = begin + s * 64 + lane;
    kreg[s] = i < end ? kin[i] : (KeyT)0;
    if (HAS_VAL) vreg[s] = i < end ? vin[i] : 0;
  }
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    const long long i = begin + s * 64 + lane;
    const bool valid = i < end;
    const KeyT key = kreg[s];
    const unsigned d = (unsigned)(key >> shift) & (unsigned)(bins - 1);
    unsigned long long peers = __ballot(valid);
    for (int b = 0; b < bits; ++b) {
      const bool bit = (d >> b) & 1u;
      const unsigned long long bal = __ballot(bit);
      peers &= bit ? bal : ~bal;
    }
    const unsigned rank = (unsigned)__popcll(peers & lt);
    unsigned pos = 0;
    if (valid) pos = off[wib][d];
    __builtin_amdgcn_wave_barrier();  // every lane has read its offset before a leader advances it
    if (valid && rank == 0) off[wib][d] = pos + (unsigned)__popcll(peers);
    __builtin_amdgcn_wave_barrier();
    if (valid) {
      kout[pos + rank] = key;
      if (HAS_VAL) vout[pos + rank] = vreg[s];
    }
  }
}

// the histogram matrix is followed by the scan's tile-total scratch
size_t hist_matrix_elems(int64_t n) { return (size_t)ceil_div(n > 0 ? n : 1, kItemsPerWave) * kMaxBins; }
uint32_t* hist_sums_of(uint32_t* hist, int64_t n) { return hist + hist_matrix_elems(n); }

template <typename KeyT, bool HAS_VAL>
int radix_pass(const KeyT* kin, KeyT* kout, const int* vin, int* vout, int64_t n, int shift, int bits,
               uint32_t* hist, hipStream_t st) {
  // (Longer runs per wave would shrink the [digit][wave] matrix to what one scan launch handles,
  // but the serial steps of a wave cost more than the launches saved: measured 40 % slower.)
  const int ipw = kItemsPerWave;
  const int n_waves = (int)ceil_div(n, ipw);
  const unsigned blocks = (unsigned)ceil_div(n_waves, 4);
  hipLaunchKernelGGL((k_radix_hist<KeyT>), dim3(blocks), dim3(256), 0, st, kin, (long long)n, shift, bits, hist,
                     n_waves, ipw);
  SPC_LAUNCH_CHECK();
  SPC_TRY(scan_u32_inplace(hist, ((int64_t)n_waves) << bits, hist_sums_of(hist, n), st));
  hipLaunchKernelGGL((k_radix_scatter<KeyT, HAS_VAL>), dim3(blocks), dim3(256), 0, st, kin, kout, vin, vout,
                     (long long)n, shift, bits, hist, n_waves, ipw);
  SPC_LAUNCH_CHECK();
  return SPCONV_OK;
}

}  // namespace

// `sums` must hold scan_sums_elems(elems) counters of scratch.
size_t scan_sums_elems(int64_t elems) { return (size_t)ceil_div(elems > 0 ? elems : 1, kScanTile); }

int scan_u32_inplace(uint32_t* data, int64_t elems, uint32_t* sums, hipStream_t st) {
  if (elems <= 0) return SPCONV_OK;
  const int64_t tiles = ceil_div(elems, kScanTile);
  if (tiles == 1) {
    hipLaunchKernelGGL((k_scan_tile<kScanPer>), dim3(1), dim3(1024), scan_lds_bytes<kScanPer>(), st, data,
                       (long long)elems, (unsigned*)nullptr);
    SPC_LAUNCH_CHECK();
    return SPCONV_OK;
  }
  if (elems <= kScanBig) {
    static std::atomic<bool> attr_set{false};  // (set twice by racing threads at worst: the calls are idempotent)
    if (!attr_set.load(std::memory_order_acquire)) {
      SPC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_scan_tile<kScanBigPer>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)scan_lds_bytes<kScanBigPer>()));
      attr_set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((k_scan_tile<kScanBigPer>), dim3(1), dim3(1024), scan_lds_bytes<kScanBigPer>(), st, data,
                       (long long)elems, (unsigned*)nullptr);
    SPC_LAUNCH_CHECK();
    return SPCONV_OK;
  }
  if (tiles > kScanTile) return SPCONV_EINVAL;  // 67M counters: far beyond what the callers produce
  hipLaunchKernelGGL((k_scan_tile<kScanPer>), dim3((unsigned)tiles), dim3(1024), scan_lds_bytes<kScanPer>(), st, data,
                     (long long)elems, sums);
  SPC_LAUNCH_CHECK();
  hipLaunchKernelGGL((k_scan_tile<kScanPer>), dim3(1), dim3(1024), scan_lds_bytes<kScanPer>(), st, sums,
                     (long long)tiles, (unsigned*)nullptr);
  SPC_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_scan_add, dim3((unsigned)tiles), dim3(1024), 0, st, data, (long long)elems, sums);
  SPC_LAUNCH_CHECK();
  return SPCONV_OK;
}

size_t sort_hist_elems(int64_t n) { return hist_matrix_elems(n) + scan_sums_elems((int64_t)hist_matrix_elems(n)); }

int radix_sort_u32(uint32_t* key_a, uint32_t* key_b, int32_t* val_a, int32_t* val_b, int64_t n, int key_bits,
                   uint32_t* hist, hipStream_t st, int* in_b) {
  *in_b = 0;
  if (n <= 1 || key_bits <= 0) return SPCONV_OK;
  const int passes = (key_bits + kMaxBits - 1) / kMaxBits;
  const int bits = (key_bits + passes - 1) / passes;  // even digit widths, each <= kMaxBits
  int shift = 0;
  for (int p = 0; p < passes; ++p) {
    const int b = (shift + bits <= key_bits) ? bits : key_bits - shift;
    const bool fwd = (*in_b == 0);
    if (val_a)
      SPC_TRY((radix_pass<uint32_t, true>(fwd ? key_a : key_b, fwd ? key_b : key_a, fwd ? val_a : val_b,
                                          fwd ? val_b : val_a, n, shift, b, hist, st)));
    else  // keys only
      SPC_TRY((radix_pass<uint32_t, false>(fwd ? key_a : key_b, fwd ? key_b : key_a, nullptr, nullptr, n, shift, b,
                                           hist, st)));
    *in_b ^= 1;
    shift += b;
  }
  return SPCONV_OK;
}

int radix_sort_u64(uint64_t* key_a, uint64_t* key_b, int64_t n, uint64_t varying, uint32_t* hist, hipStream_t st,
                   int* in_b) {
  *in_b = 0;
  if (n <= 1) return SPCONV_OK;
  // Digits are taken over maximal runs of bit positions that contain a varying bit,
  // cut into pieces of at most kMaxBits; constant bits in between cost nothing.
  int pos = 0;
  while (pos < 64) {
    if (!((varying >> pos) & 1ull)) {
      ++pos;
      continue;
    }
    int top = pos;
    for (int b = pos; b < 64 && b < pos + kMaxBits; ++b)
      if ((varying >> b) & 1ull) top = b;
    const int bits = top - pos + 1;
    if (*in_b == 0)
      SPC_TRY((radix_pass<unsigned long long, false>((unsigned long long*)key_a, (unsigned long long*)key_b,
                                                     nullptr, nullptr, n, pos, bits, hist, st)));
    else
      SPC_TRY((radix_pass<unsigned long long, false>((unsigned long long*)key_b, (unsigned long long*)key_a,
                                                     nullptr, nullptr, n, pos, bits, hist, st)));
    *in_b ^= 1;
    pos += bits;
  }
  return SPCONV_OK;
}

}  // namespace spc
