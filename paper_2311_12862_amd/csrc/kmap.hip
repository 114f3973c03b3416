// Kernel-map construction: coordinate hash table, output-coordinate
// generation for strided maps, neighbour probe, neighbour bitmask, and the
// input-side (transposed) table that dgrad of strided maps walks.
//
// The paper counts these mapping operations as a cost centre (Sections 4.2,
// 6.1, 6.3) but gives no algorithm for them; the design below is this
// library's own.  Submanifold 3x3x3 maps, the common case, hash runs of four
// cells along z (one 32-byte entry per run) and read 13.5 entries per voxel,
// each row writing its own map row and mask.  The other maps use one 16-byte
// slot per key (64-bit packed coordinate + row index) in an open-addressing
// table at load factor <= 0.5 and one probe lane per (output row, offset), so
// that map writes are contiguous per wave and the bitmask comes from a wave
// ballot; stride-2 3x3x3 maps are filled from the input side; K = 5 maps are
// held as five planes of 25 offsets.
#include "common.h"

#include <chrono>
#include <thread>

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

namespace spc {
namespace {

constexpr unsigned long long kEmpty = ~0ull;

enum : unsigned long long { FLAG_RANGE = 1, FLAG_DUP = 2, FLAG_FULL = 4, FLAG_SORT = 8 };  // SORT: a sort's bounded wait ran out
constexpr int kRetryGeneralSort = 1;  // (internal) build again with the general sort

// Control block read back by the host at the build's synchronisation point.  The pair counter
// is spread over 64 cache lines (one atomic per probe workgroup) so that the adds do not queue
// up on one address.
constexpr int kPairSlots = 64;
struct Ctl {
  unsigned long long flags, count, pad[14];
  unsigned long long pairs[kPairSlots * 16];
  unsigned long long key_or[kPairSlots * 16], key_and[kPairSlots * 16];  // spread like pairs
  unsigned long long entries[kPairSlots * 16];  // present map entries, counted from the finished map
  unsigned tick[kPairSlots * 16];  // arrivals per pair slot (submanifold probe)
  unsigned tick_top, pad2[15];     // pair slots whose workgroups have all arrived
};

// What a submanifold build hands to the host: written by the probe straight into pinned host
// memory, so that no copy has to be enqueued behind the build.
// What an asynchronous build leaves in pinned host memory, in one 8-byte word so that one store
// publishes it: bit 63 = written, bits 48..55 = error flags, bits 0..47 = pair count.
struct HostResult {
  unsigned long long word;
};
constexpr unsigned long long kHostReady = 1ull << 63;

__device__ __forceinline__ bool coord_ok(int b, int x, int y, int z) {
  return (unsigned)b <= 65534u && (unsigned)(x + 32768) <= 65535u && (unsigned)(y + 32768) <= 65535u &&
         (unsigned)(z + 32768) <= 65535u;
}

// (b, x, y, z) -> 64-bit key whose unsigned order is the lexicographic order of (b, x, y, z).
__device__ __forceinline__ unsigned long long pack_key(int b, int x, int y, int z) {
  return ((unsigned long long)(unsigned)b << 48) | ((unsigned long long)(unsigned)(x + 32768) << 32) |
         ((unsigned long long)(unsigned)(y + 32768) << 16) | (unsigned long long)(unsigned)(z + 32768);
}

// The table is an array of buckets of four 16-byte slots (one 64-byte line).  A key hashes to a
// bucket; insertion takes the first free slot of the bucket, in order, and moves on to the next
// bucket when all four are taken.  A lookup reads one line per step (four loads in flight) and
// stops at the first empty slot; at load <= 0.5 a second step is rare.
__device__ __forceinline__ unsigned hash_bucket(unsigned long long key, int log_cap) {
  return (unsigned)((key * 0x9E3779B97F4A7C15ull) >> (64 - (log_cap - 2)));
}

// 0: inserted, 1: key already there, 2: table full (cannot happen at load <= 0.5)
__device__ __forceinline__ int table_insert(unsigned long long* tab, int log_cap, unsigned long long key,
                                            int val, unsigned* slot_out) {
  const unsigned bucket_mask = (1u << (log_cap - 2)) - 1u;
  unsigned b = hash_bucket(key, log_cap);
  for (unsigned it = 0; it <= bucket_mask; ++it) {
    for (unsigned i = 0; i < 4; ++i) {
      const unsigned s = b * 4 + i;
      const unsigned long long old = atomicCAS(&tab[2 * (size_t)s], kEmpty, key);
      if (old == kEmpty) {
        tab[2 * (size_t)s + 1] = (unsigned long long)(unsigned)val;
        if (slot_out) *slot_out = s;
        return 0;
      }
      if (old == key) {
        if (slot_out) *slot_out = s;
        return 1;
      }
    }
    b = (b + 1) & bucket_mask;
  }
  return 2;
}

__device__ __forceinline__ int table_find(const unsigned long long* tab, int log_cap, unsigned long long key,
                                          unsigned* slot_out) {
  const unsigned bucket_mask = (1u << (log_cap - 2)) - 1u;
  unsigned b = hash_bucket(key, log_cap);
  for (unsigned it = 0; it <= bucket_mask; ++it) {
    const ulonglong2* line = reinterpret_cast<const ulonglong2*>(tab) + (size_t)b * 4;
    const ulonglong2 e0 = line[0], e1 = line[1], e2 = line[2], e3 = line[3];  // four loads in flight
    if (e0.x == key) {
      if (slot_out) *slot_out = b * 4;
      return (int)(unsigned)e0.y;
    }
    if (e0.x == kEmpty) return -1;
    if (e1.x == key) {
      if (slot_out) *slot_out = b * 4 + 1;
      return (int)(unsigned)e1.y;
    }
    if (e1.x == kEmpty) return -1;
    if (e2.x == key) {
      if (slot_out) *slot_out = b * 4 + 2;
      return (int)(unsigned)e2.y;
    }
    if (e2.x == kEmpty) return -1;
    if (e3.x == key) {
      if (slot_out) *slot_out = b * 4 + 3;
      return (int)(unsigned)e3.y;
    }
    if (e3.x == kEmpty) return -1;
    b = (b + 1) & bucket_mask;
  }
  return -1;
}

__device__ __forceinline__ int floor_div(int a, int s) {
  int q = a / s;
  return (a % s != 0 && a < 0) ? q - 1 : q;
}

__global__ void k_ctl_init(Ctl* ctl) {
  if (threadIdx.x == 0) {
    ctl->flags = 0;
    ctl->count = 0;
  }
  ctl->pairs[threadIdx.x * 16] = 0;  // launched with kPairSlots threads
  ctl->entries[threadIdx.x * 16] = 0;
  ctl->key_or[threadIdx.x * 16] = 0;
  ctl->key_and[threadIdx.x * 16] = ~0ull;
}

// Insert key(p_j) -> j for every input row; flags range and duplicate errors.
__global__ void __launch_bounds__(256) k_insert_rows(const int4* __restrict__ coords, int n,
                                                     unsigned long long* tab, int log_cap, Ctl* ctl,
                                                     int4* __restrict__ keep) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  const int4 c = coords[j];
  keep[j] = c;  // the kmap's own copy of the caller's rows
  if (!coord_ok(c.x, c.y, c.z, c.w)) {
    atomicOr(&ctl->flags, FLAG_RANGE);
    return;
  }
  const int r = table_insert(tab, log_cap, pack_key(c.x, c.y, c.z, c.w), j, nullptr);
  if (r == 1) atomicOr(&ctl->flags, FLAG_DUP);
  if (r == 2) atomicOr(&ctl->flags, FLAG_FULL);
}

// Coarse coordinates floor(p / s): de-duplicate through a second table, append each
// new key to ukeys (order arbitrary; sorted afterwards), and reduce OR / AND of the
// keys so that the host knows which key bytes vary.
__global__ void __launch_bounds__(256) k_coarse_unique(const int4* __restrict__ coords, int n, int stride,
                                                       unsigned long long* tab, int log_cap,
                                                       unsigned long long* __restrict__ ukeys, Ctl* ctl,
                                                       int4* __restrict__ keep) {
  __shared__ unsigned long long s_or[4], s_and[4];
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  bool fresh = false;
  unsigned long long key = 0, k_or = 0, k_and = ~0ull;
  if (j < n) {
    const int4 c = coords[j];
    if (keep) keep[j] = c;  // the kmap's own copy of the caller's rows (builds without a fine table)
    if (!coord_ok(c.x, c.y, c.z, c.w)) atomicOr(&ctl->flags, FLAG_RANGE);
    if (coord_ok(c.x, c.y, c.z, c.w)) {
      key = pack_key(c.x, floor_div(c.y, stride), floor_div(c.z, stride), floor_div(c.w, stride));
      const int r = table_insert(tab, log_cap, key, 0, nullptr);
      fresh = (r == 0);
      if (r == 2) atomicOr(&ctl->flags, FLAG_FULL);
      k_or = key;
      k_and = key;
    }
  }
  // workgroup-aggregated append: one counter atomic per workgroup, ranks from ballots
  __shared__ unsigned wave_cnt[4];
  __shared__ unsigned long long block_base;
  const unsigned long long bal = __ballot(fresh);
  if (lane == 0) wave_cnt[wave] = (unsigned)__popcll(bal);
  for (int o = 32; o > 0; o >>= 1) {
    k_or |= __shfl_xor(k_or, o);
    k_and &= __shfl_xor(k_and, o);
  }
  if (lane == 0) {
    s_or[wave] = k_or;
    s_and[wave] = k_and;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned total = wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
    block_base = total ? atomicAdd(&ctl->count, (unsigned long long)total) : 0ull;
    const int slot = (blockIdx.x % kPairSlots) * 16;
    atomicOr(&ctl->key_or[slot], s_or[0] | s_or[1] | s_or[2] | s_or[3]);
    atomicAnd(&ctl->key_and[slot], s_and[0] & s_and[1] & s_and[2] & s_and[3]);
  }
  __syncthreads();
  if (fresh) {
    unsigned before = 0;
    for (int w = 0; w < wave; ++w) before += wave_cnt[w];
    ukeys[block_base + before + __popcll(bal & ((1ull << lane) - 1ull))] = key;
  }
}

// Candidate outputs of a dilated stride-1 map: q = p - delta for every input p and offset delta
// (Equation 1 with P_out = every point that reads at least one input), de-duplicated and appended
// like the coarse points above.  One thread per (input row, offset).
template <int K>
__global__ void __launch_bounds__(256) k_dilate_unique(const int4* __restrict__ coords, long long n,
                                                       unsigned long long* tab, int log_cap,
                                                       unsigned long long* __restrict__ ukeys, Ctl* ctl) {
  constexpr int V = K * K * K, R = (K - 1) / 2;
  __shared__ unsigned long long s_or[4], s_and[4];
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long j = t / V;
  const int k = (int)(t - j * V);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  bool fresh = false;
  unsigned long long key = 0, k_or = 0, k_and = ~0ull;
  if (j < n) {
    const int4 c = coords[j];
    const int qx = c.y - (k / (K * K) - R), qy = c.z - ((k / K) % K - R), qz = c.w - (k % K - R);
    if (coord_ok(c.x, c.y, c.z, c.w)) {  // (an invalid input row is flagged by the insert kernel)
      if (!coord_ok(c.x, qx, qy, qz)) {
        atomicOr(&ctl->flags, FLAG_RANGE);  // an output beside the packable range
      } else {
        key = pack_key(c.x, qx, qy, qz);
        const int r = table_insert(tab, log_cap, key, 0, nullptr);
        fresh = (r == 0);
        if (r == 2) atomicOr(&ctl->flags, FLAG_FULL);
        k_or = key;
        k_and = key;
      }
    }
  }
  __shared__ unsigned wave_cnt[4];
  __shared__ unsigned long long block_base;
  const unsigned long long bal = __ballot(fresh);
  if (lane == 0) wave_cnt[wave] = (unsigned)__popcll(bal);
  for (int o = 32; o > 0; o >>= 1) {
    k_or |= __shfl_xor(k_or, o);
    k_and &= __shfl_xor(k_and, o);
  }
  if (lane == 0) {
    s_or[wave] = k_or;
    s_and[wave] = k_and;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned total = wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
    block_base = total ? atomicAdd(&ctl->count, (unsigned long long)total) : 0ull;
    const int slot = (blockIdx.x % kPairSlots) * 16;
    atomicOr(&ctl->key_or[slot], s_or[0] | s_or[1] | s_or[2] | s_or[3]);
    atomicAnd(&ctl->key_and[slot], s_and[0] & s_and[1] & s_and[2] & s_and[3]);
  }
  __syncthreads();
  if (fresh) {
    unsigned before = 0;
    for (int w = 0; w < wave; ++w) before += wave_cnt[w];
    ukeys[block_base + before + __popcll(bal & ((1ull << lane) - 1ull))] = key;
  }
}

__global__ void __launch_bounds__(256) k_decode_keys(const unsigned long long* __restrict__ keys, int n,
                                                     int4* __restrict__ coords) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const unsigned long long k = keys[i];
  int4 c;
  c.x = (int)(k >> 48);
  c.y = (int)((k >> 32) & 0xFFFF) - 32768;
  c.z = (int)((k >> 16) & 0xFFFF) - 32768;
  c.w = (int)(k & 0xFFFF) - 32768;
  coords[i] = c;
}

// After sorting the unique coarse keys: store each key's rank as its table value.
__global__ void __launch_bounds__(256) k_assign_rank(const unsigned long long* __restrict__ keys, int n,
                                                     unsigned long long* tab, int log_cap) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  unsigned slot = 0;
  if (table_find(tab, log_cap, keys[i], &slot) >= 0) tab[2 * (size_t)slot + 1] = (unsigned long long)(unsigned)i;
}

// One lane per (row, offset).  A wave covers 64 / V rows, so that its V-lane
// groups write contiguous map entries and a single ballot yields the bitmasks.
//   TRANSPOSED = false: row coords are output points q; look up s*q + delta.
//   TRANSPOSED = true : row coords are fine points f; look up (f - delta) / s if divisible.
template <int K, bool TRANSPOSED>
__global__ void __launch_bounds__(256) k_probe(const int4* __restrict__ rows, int n_rows, int stride,
                                               const unsigned long long* __restrict__ tab, int log_cap,
                                               int* __restrict__ map, unsigned* __restrict__ mask, Ctl* ctl) {
  __shared__ unsigned wave_pairs[4];
  constexpr int V = K * K * K;
  constexpr int RPW = 64 / V;
  constexpr int R = (K - 1) / 2;
  const int lane = threadIdx.x & 63;
  const long long wave = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int sub = lane / V, k = lane - sub * V;
  const long long row = wave * RPW + sub;
  const bool active = (sub < RPW) && (row < n_rows);
  int found = -1;
  if (active) {
    const int4 c = rows[row];
    const int dx = k / (K * K) - R, dy = (k / K) % K - R, dz = k % K - R;
    int tx, ty, tz;
    bool ok = true;
    if (!TRANSPOSED) {
      tx = stride * c.y + dx;
      ty = stride * c.z + dy;
      tz = stride * c.w + dz;
    } else {
      const int fx = c.y - dx, fy = c.z - dy, fz = c.w - dz;
      tx = floor_div(fx, stride);
      ty = floor_div(fy, stride);
      tz = floor_div(fz, stride);
      ok = (tx * stride == fx) && (ty * stride == fy) && (tz * stride == fz);
    }
    if (ok && coord_ok(c.x, tx, ty, tz)) found = table_find(tab, log_cap, pack_key(c.x, tx, ty, tz), nullptr);
    map[row * V + k] = found;
  }
  const unsigned long long bal = __ballot(found >= 0);
  if (active && k == 0) mask[row] = (unsigned)((bal >> (sub * V)) & ((1ull << V) - 1ull));
  // number of present pairs: one atomic per workgroup
  if (lane == 0) wave_pairs[threadIdx.x >> 6] = (unsigned)__popcll(bal);
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned n = wave_pairs[0] + wave_pairs[1] + wave_pairs[2] + wave_pairs[3];
    if (n) atomicAdd(&ctl->pairs[(blockIdx.x % kPairSlots) * 16], (unsigned long long)n);
  }
}

// K = 5, submanifold: the 125 offsets as five x-planes of 25 (dx = g - 2; offset j of a plane is
// dy = j / 5 - 2, dz = j % 5 - 2), one map and one 25-bit mask array per plane.  blockIdx.y is the
// plane; one lane per (row, offset of the plane), two rows per wave.
struct Planes5 {
  int* map[5];
  unsigned* mask[5];
};
constexpr int kPlaneSlots = 12;  // pair-count slots per plane (5 x 12 <= kPairSlots)
__global__ void __launch_bounds__(256)
    k_probe_planes5(const int4* __restrict__ rows, int n_rows, const unsigned long long* __restrict__ tab, int log_cap,
                    Planes5 pl, Ctl* ctl) {
  __shared__ unsigned wave_pairs[4];
  constexpr int VP = 25, RPW = 2;
  const int g = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const long long wave = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int sub = lane / VP, k = lane - sub * VP;
  const long long row = wave * RPW + sub;
  const bool active = (sub < RPW) && (row < n_rows);
  int found = -1;
  if (active) {
    const int4 c = rows[row];
    const int tx = c.y + g - 2, ty = c.z + k / 5 - 2, tz = c.w + k % 5 - 2;
    if (coord_ok(c.x, c.y, c.z, c.w) && coord_ok(c.x, tx, ty, tz))
      found = table_find(tab, log_cap, pack_key(c.x, tx, ty, tz), nullptr);
    pl.map[g][row * VP + k] = found;
  }
  const unsigned long long bal = __ballot(found >= 0);
  if (active && k == 0) pl.mask[g][row] = (unsigned)((bal >> (sub * VP)) & ((1ull << VP) - 1ull));
  if (lane == 0) wave_pairs[threadIdx.x >> 6] = (unsigned)__popcll(bal);
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned n = wave_pairs[0] + wave_pairs[1] + wave_pairs[2] + wave_pairs[3];
    if (n) atomicAdd(&ctl->pairs[(g * kPlaneSlots + blockIdx.x % kPlaneSlots) * 16], (unsigned long long)n);
  }
}

// Strided 3x3x3 map built from the input side.  Input p meets output q exactly when
// p = s*q + delta with delta in {-1, 0, 1}^3 (Eq. 1 with stride s), so per axis q is floor(p/s)
// (delta = p - s*q, if that is <= 1) or floor(p/s) + 1 (delta = p - s*q, if that is >= -1): at most
// 2x2x2 candidates, tried by 8 lanes per input row, each one lookup of q's rank in the table of
// coarse points.  At stride 2 that is 3.4 lookups per input on average, against 27 per output when
// probing from the output side.  The map was preset to -1; the masks are derived from it
// afterwards.  Plain stores: duplicate input rows write one entry twice, which shows as fewer
// present entries in the finished map than hits counted here.
__global__ void __launch_bounds__(256)
    k_scatter_down3(const int4* __restrict__ rows, int n_rows, int stride, const unsigned long long* __restrict__ tab,
                    int log_cap, int* __restrict__ map, Ctl* ctl) {
  __shared__ unsigned wave_pairs[4];
  constexpr int V = 27;
  const int lane = threadIdx.x & 63;
  const long long wave = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const long long row = wave * 8 + (lane >> 3);
  const int cand = lane & 7;
  bool found = false;
  if (row < n_rows) {
    const int4 c = rows[row];
    if (coord_ok(c.x, c.y, c.z, c.w)) {
      const int pc[3] = {c.y, c.z, c.w};
      int q[3], d[3];
      bool ok = true;
#pragma unroll
      for (int a = 0; a < 3; ++a) {
        const int up = (cand >> (2 - a)) & 1;
        q[a] = floor_div(pc[a], stride) + up;
        d[a] = pc[a] - stride * q[a];
        ok = ok && d[a] >= -1 && d[a] <= 1;
      }
      if (ok && coord_ok(c.x, q[0], q[1], q[2])) {
        const int n = table_find(tab, log_cap, pack_key(c.x, q[0], q[1], q[2]), nullptr);
        if (n >= 0) {
          const int k = ((d[0] + 1) * 3 + (d[1] + 1)) * 3 + (d[2] + 1);
          map[(long long)n * V + k] = (int)row;
          found = true;
        }
      }
    }
  }
  const unsigned long long bal = __ballot(found);
  if (lane == 0) wave_pairs[threadIdx.x >> 6] = (unsigned)__popcll(bal);
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned n = wave_pairs[0] + wave_pairs[1] + wave_pairs[2] + wave_pairs[3];
    if (n) atomicAdd(&ctl->pairs[(blockIdx.x % kPairSlots) * 16], (unsigned long long)n);
  }
}

// Plain fills (in place of memset calls, which must stay out of anything a caller may capture).
// The K = 1 map of a row set: row r meets itself; rows of the padding meet nothing.
__global__ void __launch_bounds__(256) k_identity_map(int* __restrict__ map, unsigned* __restrict__ mask,
                                                      long long rows, long long rows_pad) {
  const long long r = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= rows_pad) return;
  map[r] = r < rows ? (int)r : -1;
  mask[r] = r < rows ? 1u : 0u;
}

__global__ void __launch_bounds__(256) k_fill_u32(unsigned* __restrict__ dst, long long n, unsigned v) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = v;
}

// One launch that prepares a submanifold build: fills the table with ones (every key empty,
// every cell -1) and clears the control block.
__global__ void __launch_bounds__(256) k_build_init(ulonglong2* __restrict__ tab, long long words, Ctl* ctl) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  for (long long i = t; i < words; i += stride) tab[i] = make_ulonglong2(kEmpty, kEmpty);
  if (blockIdx.x == 0) {
    if (threadIdx.x == 0) {
      ctl->flags = 0;
      ctl->count = 0;
    }
    if (threadIdx.x < kPairSlots) {
      ctl->pairs[threadIdx.x * 16] = 0;
      ctl->tick[threadIdx.x * 16] = 0;
    }
    if (threadIdx.x == 0) ctl->tick_top = 0;
  }
}

// ---- submanifold 3x3x3 build over a table of z-runs ----
// One table entry holds four cells that are neighbours along z: the key is (b, x, y, z >> 2) and
// rows[z & 3] the input row there.  A voxel's three neighbours in a column (x + dx, y + dy,
// z - 1 .. z + 1) lie in one entry, or in two when the range crosses a multiple of four, so the
// whole 27-neighbourhood takes 13.5 entry reads on average (as many as the 13 single-voxel lookups
// that the symmetry M[n][k] = j <=> M[j][26 - k] = n leaves), and every read returns up to three
// neighbours.  Each row then writes its own 27 map entries and its own mask: no entry of another
// row is touched, so the map needs no preset and the masks no atomics.
struct RunSlot {
  unsigned long long key;
  int rows[4];
  unsigned long long pad;
};
static_assert(sizeof(RunSlot) == 32, "two entries per 64-byte line");

// (32-bit mixing: a 64-bit multiply costs several times as many instructions, and the probe hashes
// twice per lane)
__device__ __forceinline__ unsigned hash_slot(unsigned long long key, int log_cap) {
  unsigned h = (unsigned)key * 0x9E3779B1u ^ (unsigned)(key >> 32) * 0x85EBCA77u;
  h ^= h >> 15;
  return (h * 0xC2B2AE3Du) >> (32 - log_cap);
}

// The table arrives filled with ones: every key empty, every cell -1.  Duplicate rows store into
// one cell; the probe notices, because one of them no longer finds itself there.
__global__ void __launch_bounds__(256) k_insert_runs(const int4* __restrict__ coords, int n, RunSlot* tab, int log_cap,
                                                     Ctl* ctl, int4* __restrict__ keep) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  const int4 c = coords[j];
  keep[j] = c;  // the kmap's own copy of the caller's rows
  if (!coord_ok(c.x, c.y, c.z, c.w)) {
    atomicOr(&ctl->flags, FLAG_RANGE);
    return;
  }
  const unsigned long long key = pack_key(c.x, c.y, c.z, c.w >> 2);
  const unsigned slot_mask = (1u << log_cap) - 1u;
  unsigned s = hash_slot(key, log_cap);
  for (unsigned it = 0; it <= slot_mask; ++it) {
    const unsigned long long old = atomicCAS(&tab[s].key, kEmpty, key);
    if (old == kEmpty || old == key) {
      tab[s].rows[c.w & 3] = j;
      return;
    }
    s = (s + 1) & slot_mask;
  }
  atomicOr(&ctl->flags, FLAG_FULL);
}

// Finishes a lookup whose first entry (slot s) is already loaded: a = key and cells 0, 1.  FULL
// also fetches cells 2, 3.
template <bool FULL>
__device__ __forceinline__ void run_resolve(const RunSlot* tab, int log_cap, unsigned long long key, unsigned s,
                                            uint4 a, int cells[4]) {
  const unsigned slot_mask = (1u << log_cap) - 1u;
  for (unsigned it = 0; it <= slot_mask; ++it) {
    const unsigned long long k = (unsigned long long)a.x | ((unsigned long long)a.y << 32);
    if (k == key) {
      cells[0] = (int)a.z;
      cells[1] = (int)a.w;
      if (FULL) {
        const uint2 b = *reinterpret_cast<const uint2*>(&tab[s].rows[2]);
        cells[2] = (int)b.x;
        cells[3] = (int)b.y;
      }
      return;
    }
    if (k == kEmpty) return;
    s = (s + 1) & slot_mask;
    a = *reinterpret_cast<const uint4*>(tab + s);
  }
}

// The workgroup that arrives last sums the pair counters and writes the result into pinned host
// memory.  A pair slot is one 64-bit counter: pairs in its low 40 bits, arrivals above, so that one
// atomic both adds the workgroup's pairs and tells it whether it was the slot's last (a second
// level counts the finished slots: no address sees more than gridDim/64 or 64 atomics).  Called by
// the first wave only, after the others have left: two returning atomics in a row, awaited by the
// whole workgroup, kept every wave of the probe resident for 7 us.  Every value the last workgroup
// reads was produced by an atomic whose return its producer waited for before counting itself in,
// and is read with an atomic, so no cache write-back is needed.
__device__ __forceinline__ void publish_pairs(unsigned wg_pairs, Ctl* ctl, HostResult* host) {
  constexpr unsigned long long kArrive = 1ull << 40;
  int last = 0;
  if (threadIdx.x == 0) {
    const unsigned slot = blockIdx.x % kPairSlots;
    const unsigned long long before = atomicAdd(&ctl->pairs[slot * 16], (unsigned long long)wg_pairs + kArrive);
    const unsigned slot_wgs = (gridDim.x - slot + kPairSlots - 1) / kPairSlots;
    const unsigned used_slots = gridDim.x < (unsigned)kPairSlots ? gridDim.x : (unsigned)kPairSlots;
    if ((unsigned)(before >> 40) + 1 == slot_wgs) last = atomicAdd(&ctl->tick_top, 1u) + 1 == used_slots;
  }
  last = __builtin_amdgcn_readfirstlane(last);
  if (last) {
    unsigned long long v = atomicAdd(&ctl->pairs[threadIdx.x * 16], 0ull) & (kArrive - 1);  // kPairSlots == 64 lanes
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    if (threadIdx.x == 0)
      host->word = kHostReady | ((unsigned long long)(ctl->flags & 0xFFu) << 48) | (v & 0xFFFFFFFFFFFFull);
  }
}

__device__ __forceinline__ unsigned spread3(unsigned g) {  // bit c of 9 -> bit 3c
  g = (g | (g << 16)) & 0x030000FFu;
  g = (g | (g << 8)) & 0x0300F00Fu;
  g = (g | (g << 4)) & 0x030C30C3u;
  return (g | (g << 2)) & 0x09249249u;
}

// Nine lanes per row, one per column (dx, dy); seven rows per wave.  Rows of the padding
// (n_rows <= row < rows_pad) get an empty neighbourhood.
__global__ void __launch_bounds__(256)
    k_probe_runs3(const int4* __restrict__ rows, int n_rows, long long rows_pad, const RunSlot* __restrict__ tab,
                  int log_cap, int* __restrict__ map, unsigned* __restrict__ mask, Ctl* ctl, HostResult* host) {
  __shared__ unsigned wave_pairs[4];
  constexpr int V = 27, LPR = 9, RPW = 7;
  const int lane = threadIdx.x & 63;
  const long long wave = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int sub = lane / LPR, col = lane - sub * LPR;
  const long long row = wave * RPW + sub;
  const bool active = (sub < RPW) && (row < rows_pad);
  int nb[3] = {-1, -1, -1};
  if (active && row < n_rows) {
    const int4 c = rows[row];
    const int tx = c.y + col / 3 - 1, ty = c.z + col % 3 - 1;
    // The cells z - 1, z, z + 1 are three in a row of the window [run q_lo | run q_lo + 1], starting
    // at (z - 1) & 3: of the upper run only cells 0 and 1 can be needed, which come with its key.
    // (z itself is in range, so the runs' indices fit the key's field; cells beside the range are
    // dropped below.  A row beside the range fails the build; its neighbourhood stays empty.)
    const int q_lo = (c.w - 1) >> 2, i0 = (c.w - 1) & 3;
    if (coord_ok(c.x, c.y, c.z, c.w) && coord_ok(c.x, tx, ty, c.w)) {
      const unsigned long long key_lo = pack_key(c.x, tx, ty, q_lo), key_hi = key_lo + 1;
      const unsigned s_lo = hash_slot(key_lo, log_cap), s_hi = hash_slot(key_hi, log_cap);
      const uint4 a_lo = *reinterpret_cast<const uint4*>(tab + s_lo);
      const uint2 b_lo = *reinterpret_cast<const uint2*>(&tab[s_lo].rows[2]);
      // (the kernel is bound by the number of read requests a CU keeps in flight: the upper run is
      // only read where the window reaches into it)
      uint4 a_hi = make_uint4(~0u, ~0u, 0u, 0u);
      if (i0 >= 2) a_hi = *reinterpret_cast<const uint4*>(tab + s_hi);  // all in flight
      int w[8] = {-1, -1, -1, -1, -1, -1, -1, -1};
      {
        const unsigned long long k = (unsigned long long)a_lo.x | ((unsigned long long)a_lo.y << 32);
        if (k == key_lo) {
          w[0] = (int)a_lo.z;
          w[1] = (int)a_lo.w;
          w[2] = (int)b_lo.x;
          w[3] = (int)b_lo.y;
        } else if (k != kEmpty) {
          run_resolve<true>(tab, log_cap, key_lo, s_lo, a_lo, w);
        }
      }
      if (i0 >= 2) run_resolve<false>(tab, log_cap, key_hi, s_hi, a_hi, w + 4);
      const bool b1 = i0 & 1, b2 = i0 & 2;
#pragma unroll
      for (int d = 0; d < 3; ++d) {
        const int v = b2 ? (b1 ? w[3 + d] : w[2 + d]) : (b1 ? w[1 + d] : w[d]);
        nb[d] = coord_ok(c.x, tx, ty, c.w + d - 1) ? v : -1;
      }
      // a row that does not find itself at its own place shares it with another row
      if (col == 4 && nb[1] != (int)row) atomicOr(&ctl->flags, FLAG_DUP);
    }
  }
  if (active) {
    int* dst = map + row * V + 3 * col;
    dst[0] = nb[0];
    dst[1] = nb[1];
    dst[2] = nb[2];
  }
  const unsigned long long b0 = __ballot(nb[0] >= 0), b1 = __ballot(nb[1] >= 0), b2 = __ballot(nb[2] >= 0);
  if (active && col == 0) {
    const int sh = sub * LPR;
    mask[row] = spread3((unsigned)(b0 >> sh) & 0x1FFu) | (spread3((unsigned)(b1 >> sh) & 0x1FFu) << 1) |
                (spread3((unsigned)(b2 >> sh) & 0x1FFu) << 2);
  }
  if (lane == 0) wave_pairs[threadIdx.x >> 6] = (unsigned)(__popcll(b0) + __popcll(b1) + __popcll(b2));
  __syncthreads();
  if (threadIdx.x >= 64) return;
  publish_pairs(wave_pairs[0] + wave_pairs[1] + wave_pairs[2] + wave_pairs[3], ctl, host);
}

// T[j][k] = n for every present pair M[n][k] = j.
__global__ void __launch_bounds__(256) k_scatter_in_side(const int* __restrict__ map, long long n_entries, int V,
                                                         int* __restrict__ tmap) {
  const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n_entries) return;
  const int j = map[e];
  if (j >= 0) {
    const long long n = e / V;
    const int k = (int)(e - n * V);
    tmap[(long long)j * V + k] = (int)n;
  }
}

template <int V>
__global__ void __launch_bounds__(256) k_mask_from_map(const int* __restrict__ map, int n_rows,
                                                       unsigned* __restrict__ mask, Ctl* ctl) {
  __shared__ unsigned wave_cnt[4];
  constexpr int RPW = 64 / V;
  const int lane = threadIdx.x & 63;
  const long long wave = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int sub = lane / V, k = lane - sub * V;
  const long long row = wave * RPW + sub;
  const bool active = (sub < RPW) && (row < n_rows);
  const bool hit = active && map[row * V + k] >= 0;
  const unsigned long long bal = __ballot(hit);
  if (active && k == 0) mask[row] = (unsigned)((bal >> (sub * V)) & ((1ull << V) - 1ull));
  if (!ctl) return;  // (uniform) otherwise count the present entries, one atomic per workgroup
  if (lane == 0) wave_cnt[threadIdx.x >> 6] = (unsigned)__popcll(bal);
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned n = wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
    if (n) atomicAdd(&ctl->entries[(blockIdx.x % kPairSlots) * 16], (unsigned long long)n);
  }
}

// The unique coarse keys vary in a few bit ranges only (per 16-bit field: lowest to highest
// varying bit).  Squeezing those ranges together gives a dense key of usually <= 32 bits whose
// order is the order of the full keys, so the sort moves half the bytes in half the passes.
struct BitRuns {
  int n, total;
  int pos[4], len[4], out[4];
  unsigned long long base;  // the constant bits
};
__global__ void __launch_bounds__(256) k_compress_keys(const unsigned long long* __restrict__ keys, int n, BitRuns r,
                                                       unsigned* __restrict__ out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const unsigned long long k = keys[i];
  unsigned c = 0;
  for (int j = 0; j < r.n; ++j) c |= (unsigned)((k >> r.pos[j]) & ((1ull << r.len[j]) - 1ull)) << r.out[j];
  out[i] = c;
}
// Sorted dense keys -> coordinates of the coarse points, and each key's rank as its table value.
__global__ void __launch_bounds__(256) k_expand_keys(const unsigned* __restrict__ dense, int n, BitRuns r,
                                                     int4* __restrict__ coords, unsigned long long* tab,
                                                     int log_cap) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const unsigned c = dense[i];
  unsigned long long k = r.base;
  for (int j = 0; j < r.n; ++j) k |= ((unsigned long long)((c >> r.out[j]) & ((1u << r.len[j]) - 1u))) << r.pos[j];
  int4 q;
  q.x = (int)(k >> 48);
  q.y = (int)((k >> 32) & 0xFFFF) - 32768;
  q.z = (int)((k >> 16) & 0xFFFF) - 32768;
  q.w = (int)(k & 0xFFFF) - 32768;
  coords[i] = q;
  if (tab) {
    unsigned slot = 0;
    if (table_find(tab, log_cap, k, &slot) >= 0) tab[2 * (size_t)slot + 1] = (unsigned long long)(unsigned)i;
  }
}

// Per-offset pair counts from the bitmasks.
__global__ void __launch_bounds__(256) k_count_pairs(const unsigned* __restrict__ mask, int n_rows,
                                                     unsigned long long* __restrict__ counts) {
  __shared__ unsigned cnt[32];
  if (threadIdx.x < 32) cnt[threadIdx.x] = 0;
  __syncthreads();
  for (long long r = (long long)blockIdx.x * blockDim.x + threadIdx.x; r < n_rows;
       r += (long long)gridDim.x * blockDim.x) {
    unsigned m = mask[r];
    while (m) {
      const int k = __ffs((int)m) - 1;
      m &= m - 1;
      atomicAdd(&cnt[k], 1u);
    }
  }
  __syncthreads();
  if (threadIdx.x < 32 && cnt[threadIdx.x]) atomicAdd(&counts[threadIdx.x], (unsigned long long)cnt[threadIdx.x]);
}

int log2_capacity(int64_t n) {
  int lc = 10;
  while ((1ll << lc) < 2 * n) ++lc;
  return lc;
}

inline unsigned blocks_for(int64_t n, int per_block) { return (unsigned)ceil_div(n > 0 ? n : 1, per_block); }

template <int K>
int launch_probe(bool transposed, const int4* rows, int64_t n_rows, int stride, const unsigned long long* tab,
                 int log_cap, int* map, unsigned* mask, Ctl* ctl, hipStream_t st) {
  constexpr int V = K * K * K;
  constexpr int RPW = 64 / V;
  const int64_t waves = ceil_div(n_rows, RPW);
  const unsigned blocks = blocks_for(waves, 4);
  if (transposed)
    hipLaunchKernelGGL((k_probe<K, true>), dim3(blocks), dim3(256), 0, st, rows, (int)n_rows, stride, tab, log_cap,
                       map, mask, ctl);
  else
    hipLaunchKernelGGL((k_probe<K, false>), dim3(blocks), dim3(256), 0, st, rows, (int)n_rows, stride, tab,
                       log_cap, map, mask, ctl);
  SPC_LAUNCH_CHECK();
  return SPCONV_OK;
}

int fill_u32(void* dst, int64_t n, unsigned v, hipStream_t st) {
  if (n <= 0) return SPCONV_OK;
  hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)std::min<int64_t>(ceil_div(n, 256), 2048)), dim3(256), 0, st,
                     static_cast<unsigned*>(dst), (long long)n, v);
  SPC_LAUNCH_CHECK();
  return SPCONV_OK;
}

// Allocates map and masks; presets the padding rows (no neighbours), or every row when the
// builder only writes the entries that are present.
int alloc_side(SideMap& side, int64_t rows, int V, hipStream_t st, bool preset_all = false) {
  side.rows = rows;
  side.rows_pad = round_up(rows > 0 ? rows : 1, kRowPad);
  SPC_TRY(side.map.alloc((size_t)side.rows_pad * V * sizeof(int)));
  SPC_TRY(side.mask.alloc((size_t)side.rows_pad * sizeof(unsigned)));
  const int64_t first = preset_all ? 0 : rows;
  SPC_TRY(fill_u32(side.map.as<int>() + first * V, (side.rows_pad - first) * V, 0xFFFFFFFFu, st));
  SPC_TRY(fill_u32(side.mask.as<unsigned>() + first, side.rows_pad - first, 0u, st));
  return SPCONV_OK;
}

// Pool of pinned control blocks.  The probe's last workgroup stores the result word; the host finds
// out by reading the word, so nothing is recorded on the stream behind the probe (an event there
// delayed the next kernel by 5.6 us).
struct HostCtl {
  HostResult res;
  HostResult* dev;  // device-side address of res
};

std::mutex g_host_mu;
std::vector<HostCtl*> g_host_free;

HostCtl* host_ctl_acquire() {
  {
    std::lock_guard<std::mutex> lk(g_host_mu);
    if (!g_host_free.empty()) {
      HostCtl* h = g_host_free.back();
      g_host_free.pop_back();
      return h;
    }
  }
  void* p = nullptr;
  if (hipHostMalloc(&p, sizeof(HostCtl), hipHostMallocDefault) != hipSuccess) {
    (void)hipGetLastError();
    return nullptr;
  }
  HostCtl* h = static_cast<HostCtl*>(p);
  void* dp = nullptr;
  if (hipHostGetDevicePointer(&dp, p, 0) != hipSuccess) {
    (void)hipGetLastError();
    (void)hipHostFree(p);
    return nullptr;
  }
  h->dev = &static_cast<HostCtl*>(dp)->res;
  return h;
}

// Waits (briefly, yielding) for the result word of a block to be written.
bool host_ctl_ready(const HostCtl* h, double max_seconds) {
  const volatile unsigned long long* w = &h->res.word;
  const auto t0 = std::chrono::steady_clock::now();
  while (!(*w & kHostReady)) {
    if (std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() > max_seconds) return false;
    std::this_thread::yield();
  }
  return true;
}

void host_ctl_release(HostCtl* h) {
  std::lock_guard<std::mutex> lk(g_host_mu);
  g_host_free.push_back(h);
}

// Reads the control block back through a pinned staging buffer (one per process) and
// synchronises the stream.
int read_ctl(const Ctl* ctl, Ctl* host, hipStream_t st) {
  static std::mutex mu;
  static Ctl* pinned = nullptr;
  std::lock_guard<std::mutex> lk(mu);
  if (!pinned) {
    void* p = nullptr;
    if (hipHostMalloc(&p, sizeof(Ctl), hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      p = nullptr;
    }
    pinned = static_cast<Ctl*>(p);
  }
  Ctl* dst = pinned ? pinned : host;
  SPC_HIP(hipMemcpyAsync(dst, ctl, sizeof(Ctl), hipMemcpyDeviceToHost, st));
  SPC_HIP(hipStreamSynchronize(st));
  if (pinned) *host = *pinned;
  return SPCONV_OK;
}

int flags_status(const Ctl& h) {
  if (h.flags & FLAG_RANGE) return SPCONV_ERANGE;
  if (h.flags & FLAG_DUP) return SPCONV_EDUP;
  if (h.flags & FLAG_FULL) return SPCONV_ENOMEM;
  return SPCONV_OK;
}

}  // namespace
int kmap_status_impl(spconv_kmap* km, hipStream_t st, bool wait_stream);
namespace {

// Submanifold 3x3x3 build: init, insert, probe (whose last workgroup publishes the result to
// pinned host memory).
int build_submanifold3(spconv_kmap* km, const int4* rows, int64_t N, bool async, hipStream_t st) {
  const int V = 27;
  DevBuf ctl_buf, tab, own_rows;
  SPC_TRY(ctl_buf.alloc(sizeof(Ctl)));
  Ctl* ctl = ctl_buf.as<Ctl>();
  const int lc = log2_capacity(N);  // entries >= 2 N >= twice the z-runs
  SPC_TRY(tab.alloc(sizeof(RunSlot) << lc));
  SPC_TRY(own_rows.alloc((size_t)N * 16));
  SideMap& side = km->out_side;
  side.rows = N;
  side.rows_pad = round_up(N, kRowPad);
  SPC_TRY(side.map.alloc((size_t)side.rows_pad * V * sizeof(int)));
  SPC_TRY(side.mask.alloc((size_t)side.rows_pad * sizeof(unsigned)));
  const long long words = 2ll << lc;  // 16-byte words of the table, all set to ones
  const unsigned init_blocks = (unsigned)std::min<int64_t>(ceil_div(words, 256), 4096);
  hipLaunchKernelGGL(k_build_init, dim3(init_blocks), dim3(256), 0, st, tab.as<ulonglong2>(), words,
                     ctl);
  SPC_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_insert_runs, dim3(blocks_for(N, 256)), dim3(256), 0, st, rows, (int)N, tab.as<RunSlot>(), lc,
                     ctl, own_rows.as<int4>());
  SPC_LAUNCH_CHECK();
  HostCtl* hc = host_ctl_acquire();
  if (!hc) return SPCONV_ENOMEM;
  hc->res.word = 0;  // (pinned memory: visible to the kernel launched below)
  hipLaunchKernelGGL(k_probe_runs3, dim3(blocks_for(ceil_div(side.rows_pad, 7), 4)), dim3(256), 0, st, rows, (int)N,
                     (long long)side.rows_pad, tab.as<RunSlot>(), lc, side.map.as<int>(), side.mask.as<unsigned>(),
                     ctl, hc->dev);
  const bool ok = hipGetLastError() == hipSuccess;
  if (!ok) {
    (void)hipGetLastError();
    (void)hipStreamSynchronize(st);
    host_ctl_release(hc);
    return SPCONV_EHIP;
  }
  km->n_in = km->n_out = N;
  side.ready = true;
  km->pending_host = hc;
  km->pending = true;
  km->n_pairs = -1;
  // (ctl_buf returns to the pool here; reuse is ordered behind the probe on this stream)
  if (!async) SPC_TRY(kmap_status_impl(km, st, true));
  std::swap(km->in_coords.p, own_rows.p);  // P_out == P_in: out_coords stays empty
  std::swap(km->in_coords.bytes, own_rows.bytes);
  return SPCONV_OK;
}

// K = 5 submanifold build: one table of the rows, one probe launch over the five planes, one read of
// the control block (flags and the planes' pair counts).
int build_submanifold5(spconv_kmap* km, const int4* rows, int64_t N, hipStream_t st) {
  constexpr int VP = 25;
  DevBuf ctl_buf, tab, own_rows;
  SPC_TRY(ctl_buf.alloc(sizeof(Ctl)));
  Ctl* ctl = ctl_buf.as<Ctl>();
  hipLaunchKernelGGL(k_ctl_init, dim3(1), dim3(kPairSlots), 0, st, ctl);
  SPC_LAUNCH_CHECK();
  const int lc = log2_capacity(N);
  SPC_TRY(tab.alloc((size_t)16 << lc));
  SPC_TRY(fill_u32(tab.p, (int64_t)4 << lc, 0xFFFFFFFFu, st));
  SPC_TRY(own_rows.alloc((size_t)N * 16));
  hipLaunchKernelGGL(k_insert_rows, dim3(blocks_for(N, 256)), dim3(256), 0, st, rows, (int)N,
                     tab.as<unsigned long long>(), lc, ctl, own_rows.as<int4>());
  SPC_LAUNCH_CHECK();
  Planes5 pl{};
  for (int g = 0; g < 5; ++g) {
    std::unique_ptr<spconv_kmap> sub(new (std::nothrow) spconv_kmap(
        std::make_shared<SideMap>(), std::make_shared<SideMap>(), km->in_coords_ref, km->out_coords_ref));
    if (!sub) return SPCONV_ENOMEM;
    sub->K = 5;
    sub->V = VP;
    sub->n_in = sub->n_out = N;
    sub->build_stream = sub->last_stream = st;
    SPC_TRY(alloc_side(sub->out_side, N, VP, st));
    sub->out_side.ready = true;
    pl.map[g] = sub->out_side.map.as<int>();
    pl.mask[g] = sub->out_side.mask.as<unsigned>();
    km->groups.push_back(std::move(sub));
  }
  hipLaunchKernelGGL(k_probe_planes5, dim3(blocks_for(ceil_div(N, 2), 4), 5), dim3(256), 0, st, rows, (int)N,
                     tab.as<unsigned long long>(), lc, pl, ctl);
  SPC_LAUNCH_CHECK();
  Ctl h{};
  SPC_TRY(read_ctl(ctl, &h, st));
  std::swap(km->in_coords.p, own_rows.p);  // P_out == P_in: out_coords stays empty
  std::swap(km->in_coords.bytes, own_rows.bytes);
  km->n_in = km->n_out = N;
  km->n_pairs = 0;
  for (int g = 0; g < 5; ++g) {
    int64_t n = 0;
    for (int i = 0; i < kPlaneSlots; ++i) n += (int64_t)h.pairs[(g * kPlaneSlots + i) * 16];
    km->groups[g]->n_pairs = n;
    km->n_pairs += n;
  }
  km->build_status = flags_status(h);
  return km->build_status;
}

}  // namespace

struct HostCtlHandle {
  // the probe must have written the block before it is handed to another build
  static void finish(void* p) {
    HostCtl* hc = static_cast<HostCtl*>(p);
    if (!host_ctl_ready(hc, 0.05)) (void)hipDeviceSynchronize();
    host_ctl_release(hc);
  }
};

// wait_stream: wait for the whole stream (the synchronous build: everything on it is the build);
// otherwise only for the probe's result word.
int kmap_status_impl(spconv_kmap* km, hipStream_t st, bool wait_stream) {
  if (!km->pending) return km->build_status;
  HostCtl* hc = static_cast<HostCtl*>(km->pending_host);
  if (wait_stream) {
    SPC_HIP(hipStreamSynchronize(st));
  } else if (!host_ctl_ready(hc, 0.002)) {
    // not there yet: wait for the stream the build runs on instead of spinning
    SPC_HIP(hipStreamSynchronize(km->build_stream));
  }
  if (!host_ctl_ready(hc, 1.0)) {  // the probe never ran to its end
    (void)hipDeviceSynchronize();
    km->pending = false;
    km->pending_host = nullptr;
    host_ctl_release(hc);
    km->build_status = SPCONV_EHIP;
    return SPCONV_EHIP;
  }
  const unsigned long long word = hc->res.word;
  Ctl h{};
  h.flags = (unsigned)((word >> 48) & 0xFFu);
  const int status = flags_status(h);
  km->n_pairs = (int64_t)(word & 0xFFFFFFFFFFFFull);
  km->pending = false;
  km->pending_host = nullptr;
  host_ctl_release(hc);
  km->build_status = status;  // kept: whoever resolved the build (a pair count, a tuner), spconv_kmap_status still reports it
  return status;
}

int kmap_status(spconv_kmap* km, hipStream_t st) { return kmap_status_impl(km, st, false); }

namespace {
int kmap_build_impl(const int32_t* coords, int64_t N, int K, int stride, int transposed, bool async, hipStream_t st,
                    spconv_kmap** out, bool dilate, bool few_launch_sort);
}
int kmap_build(const int32_t* coords, int64_t N, int K, int stride, int transposed, bool async, hipStream_t st,
               spconv_kmap** out, bool dilate) {
  const int status = kmap_build_impl(coords, N, K, stride, transposed, async, st, out, dilate, true);
  if (status != kRetryGeneralSort) return status;
  return kmap_build_impl(coords, N, K, stride, transposed, async, st, out, dilate, false);
}
namespace {
int kmap_build_impl(const int32_t* coords, int64_t N, int K, int stride, int transposed, bool async, hipStream_t st,
                    spconv_kmap** out, bool dilate, bool few_launch_sort) {
  std::unique_ptr<spconv_kmap> km(new (std::nothrow) spconv_kmap);
  if (!km) return SPCONV_ENOMEM;
  km->K = K;
  km->V = K * K * K;
  km->stride = stride;
  km->transposed = transposed;
  km->dilated = dilate ? 1 : 0;
  km->build_stream = st;
  km->last_stream = st;
  const int V = km->V;
  // builds whose output (or, transposed, input) set is derived from the caller's rows: the coarse
  // points of a strided map, or the dilated set of a stride-1 map
  const bool needs_coarse = stride > 1 || dilate;
  const int64_t cand = dilate ? N * V : N;  // most points that derivation can yield

  if (N == 0) {
    km->n_in = km->n_out = 0;
    km->n_pairs = 0;
    SPC_TRY(km->in_coords.alloc(16));
    SPC_TRY(km->out_coords.alloc(16));
    SPC_TRY(alloc_side(km->out_side, 0, V, st));
    km->out_side.ready = true;
    *out = km.release();
    return SPCONV_OK;
  }

  const int4* rows = reinterpret_cast<const int4*>(coords);
  if (K == 5) {  // (submanifold only: the entry points refuse other K = 5 maps)
    SPC_TRY(build_submanifold5(km.get(), rows, N, st));  // (range and duplicate errors: no kmap, as for every synchronous build)
    *out = km.release();
    return SPCONV_OK;
  }
  if (K == 3 && stride == 1 && !transposed && !dilate) {
    SPC_TRY(build_submanifold3(km.get(), rows, N, async, st));
    *out = km.release();
    return SPCONV_OK;
  }
  DevBuf ctl_buf, tab_fine, tab_coarse, ukeys_a, ukeys_b, hist;
  SPC_TRY(ctl_buf.alloc(sizeof(Ctl)));
  Ctl* ctl = ctl_buf.as<Ctl>();
  hipLaunchKernelGGL(k_ctl_init, dim3(1), dim3(kPairSlots), 0, st, ctl);
  SPC_LAUNCH_CHECK();

  // Stride-2 3x3x3 maps are built from the input side and need no table of the fine points.  (Only
  // stride 2: there every input row meets the output floor(p/2), so every row writes at least one
  // entry and duplicate rows cannot escape the entry count; at larger strides some rows write none.)
  const bool from_inputs = (K == 3 && stride == 2 && !transposed && !dilate);
  // fine table: key(p_j) -> j.  Also the duplicate / range check of the caller's rows.
  const int lc_fine = log2_capacity(N);
  // the caller's rows are kept: they are P_in (and P_out for stride 1), or the fine output set
  DevBuf own_rows;
  SPC_TRY(own_rows.alloc((size_t)N * 16));
  if (!from_inputs) {
    SPC_TRY(tab_fine.alloc((size_t)16 << lc_fine));
    SPC_TRY(fill_u32(tab_fine.p, (int64_t)4 << lc_fine, 0xFFFFFFFFu, st));
    hipLaunchKernelGGL(k_insert_rows, dim3(blocks_for(N, 256)), dim3(256), 0, st, rows, (int)N,
                       tab_fine.as<unsigned long long>(), lc_fine, ctl, own_rows.as<int4>());
    SPC_LAUNCH_CHECK();
  }

  Ctl h{};
  int64_t U = 0;
  DevBuf coarse_rows;
  const int lc_coarse = dilate ? log2_capacity(cand) : lc_fine;
  if (needs_coarse) {
    SPC_TRY(tab_coarse.alloc((size_t)16 << lc_coarse));
    SPC_TRY(fill_u32(tab_coarse.p, (int64_t)4 << lc_coarse, 0xFFFFFFFFu, st));
    SPC_TRY(ukeys_a.alloc((size_t)cand * 8));
    SPC_TRY(ukeys_b.alloc((size_t)cand * 8));
    if (dilate) {
      const unsigned blocks = blocks_for(cand, 256);
      if (K == 3)
        hipLaunchKernelGGL(k_dilate_unique<3>, dim3(blocks), dim3(256), 0, st, rows, (long long)N,
                           tab_coarse.as<unsigned long long>(), lc_coarse, ukeys_a.as<unsigned long long>(), ctl);
      else
        hipLaunchKernelGGL(k_dilate_unique<1>, dim3(blocks), dim3(256), 0, st, rows, (long long)N,
                           tab_coarse.as<unsigned long long>(), lc_coarse, ukeys_a.as<unsigned long long>(), ctl);
    } else {
      hipLaunchKernelGGL(k_coarse_unique, dim3(blocks_for(N, 256)), dim3(256), 0, st, rows, (int)N, stride,
                         tab_coarse.as<unsigned long long>(), lc_coarse, ukeys_a.as<unsigned long long>(), ctl,
                         from_inputs ? own_rows.as<int4>() : nullptr);
    }
    SPC_LAUNCH_CHECK();
  }
  if (needs_coarse) {
    // the one synchronisation of a strided build: error flags, U, varying key bits
    SPC_TRY(read_ctl(ctl, &h, st));
    SPC_TRY(flags_status(h));
    U = (int64_t)h.count;
    SPC_TRY(hist.alloc(sort_hist_elems(U) * sizeof(uint32_t)));
    int in_b = 0;
    unsigned long long key_or = 0, key_and = ~0ull;
    for (int i = 0; i < kPairSlots; ++i) {
      key_or |= h.key_or[i * 16];
      key_and &= h.key_and[i * 16];
    }
    const unsigned long long varying = key_or ^ key_and;
    BitRuns runs{};
    runs.base = key_and & ~varying;
    for (int f = 0; f < 4; ++f) {
      const unsigned v = (unsigned)((varying >> (16 * f)) & 0xFFFFu);
      if (!v) continue;
      int lo = 0, hi = 15;
      while (!((v >> lo) & 1u)) ++lo;
      while (!((v >> hi) & 1u)) --hi;
      runs.pos[runs.n] = 16 * f + lo;
      runs.len[runs.n] = hi - lo + 1;
      runs.out[runs.n] = runs.total;
      runs.total += hi - lo + 1;
      // (bits inside a span that do not vary travel with the dense key; base must not repeat them)
      runs.base &= ~(((1ull << (hi - lo + 1)) - 1ull) << (16 * f + lo));
      ++runs.n;
    }
    SPC_TRY(coarse_rows.alloc((size_t)U * 16));
    const bool want_rank = transposed || from_inputs;
    if (runs.total <= 32) {
      // ukeys_b's N * 8 bytes hold both dense key buffers
      uint32_t* dense_a = ukeys_b.as<uint32_t>();
      uint32_t* dense_b = dense_a + cand;
      hipLaunchKernelGGL(k_compress_keys, dim3(blocks_for(U, 256)), dim3(256), 0, st,
                         ukeys_a.as<unsigned long long>(), (int)U, runs, dense_a);
      SPC_LAUNCH_CHECK();
      // Builds that read the control block once more at their end (stride-2 3x3x3) sort with one
      // launch per digit; should one of its bounded waits run out, that read shows it and the
      // build is done again with the general sort.
      int sorted = SPCONV_EINVAL;
      if (few_launch_sort && from_inputs)
        sorted = msort_keys_u32(dense_a, dense_b, U, runs.total, reinterpret_cast<unsigned*>(&ctl->flags),
                                (unsigned)FLAG_SORT, st, &in_b);
      if (sorted == SPCONV_EINVAL)
        sorted = radix_sort_u32(dense_a, dense_b, nullptr, nullptr, U, runs.total, hist.as<uint32_t>(), st, &in_b);
      SPC_TRY(sorted);
      hipLaunchKernelGGL(k_expand_keys, dim3(blocks_for(U, 256)), dim3(256), 0, st, in_b ? dense_b : dense_a, (int)U,
                         runs, coarse_rows.as<int4>(),
                         want_rank ? tab_coarse.as<unsigned long long>() : (unsigned long long*)nullptr, lc_coarse);
      SPC_LAUNCH_CHECK();
    } else {
      SPC_TRY(radix_sort_u64(ukeys_a.as<uint64_t>(), ukeys_b.as<uint64_t>(), U, varying, hist.as<uint32_t>(), st,
                             &in_b));
      const unsigned long long* sorted = in_b ? ukeys_b.as<unsigned long long>() : ukeys_a.as<unsigned long long>();
      hipLaunchKernelGGL(k_decode_keys, dim3(blocks_for(U, 256)), dim3(256), 0, st, sorted, (int)U,
                         coarse_rows.as<int4>());
      SPC_LAUNCH_CHECK();
      if (want_rank) {
        hipLaunchKernelGGL(k_assign_rank, dim3(blocks_for(U, 256)), dim3(256), 0, st, sorted, (int)U,
                           tab_coarse.as<unsigned long long>(), lc_coarse);
        SPC_LAUNCH_CHECK();
      }
    }
  }

  int status = SPCONV_OK;
  if (from_inputs) {
    km->n_in = N;
    km->n_out = U;
    SPC_TRY(alloc_side(km->out_side, U, V, st, true));
    hipLaunchKernelGGL(k_scatter_down3, dim3(blocks_for(ceil_div(N, 8), 4)), dim3(256), 0, st, rows, (int)N, stride,
                       tab_coarse.as<unsigned long long>(), lc_coarse, km->out_side.map.as<int>(), ctl);
    SPC_LAUNCH_CHECK();
    hipLaunchKernelGGL((k_mask_from_map<27>), dim3(blocks_for(ceil_div(U, 2), 4)), dim3(256), 0, st,
                       km->out_side.map.as<int>(), (int)U, km->out_side.mask.as<unsigned>(), ctl);
    SPC_LAUNCH_CHECK();
  } else if (!transposed) {
    km->n_in = N;
    km->n_out = needs_coarse ? U : N;
    const int4* qrows = needs_coarse ? coarse_rows.as<int4>() : rows;
    SPC_TRY(alloc_side(km->out_side, km->n_out, V, st));
    int* mp = km->out_side.map.as<int>();
    unsigned* mk = km->out_side.mask.as<unsigned>();
    const unsigned long long* tf = tab_fine.as<unsigned long long>();
    // (a dilated map probes like any other stride-1 map, from its derived output points)
    status = K == 3   ? launch_probe<3>(false, qrows, km->n_out, stride, tf, lc_fine, mp, mk, ctl, st)
             : K == 2 ? launch_probe<2>(false, qrows, km->n_out, stride, tf, lc_fine, mp, mk, ctl, st)
                      : launch_probe<1>(false, qrows, km->n_out, stride, tf, lc_fine, mp, mk, ctl, st);
    SPC_TRY(status);
  } else {
    km->n_in = needs_coarse ? U : N;
    km->n_out = N;
    const unsigned long long* tab = needs_coarse ? tab_coarse.as<unsigned long long>()
                                                 : tab_fine.as<unsigned long long>();
    SPC_TRY(alloc_side(km->out_side, km->n_out, V, st));
    int* mp = km->out_side.map.as<int>();
    unsigned* mk = km->out_side.mask.as<unsigned>();
    const int lc = needs_coarse ? lc_coarse : lc_fine;
    status = K == 3   ? launch_probe<3>(true, rows, N, stride, tab, lc, mp, mk, ctl, st)
             : K == 2 ? launch_probe<2>(true, rows, N, stride, tab, lc, mp, mk, ctl, st)
                      : launch_probe<1>(true, rows, N, stride, tab, lc, mp, mk, ctl, st);
    SPC_TRY(status);
  }
  km->out_side.ready = true;

  if (!needs_coarse || from_inputs) {  // (from_inputs: duplicate rows only show up in the scatter)
    SPC_TRY(read_ctl(ctl, &h, st));
    int64_t pairs = 0, entries = 0;  // the probe ran before this synchronisation: its pair count is final
    for (int i = 0; i < kPairSlots; ++i) pairs += (int64_t)h.pairs[i * 16];
    for (int i = 0; i < kPairSlots; ++i) entries += (int64_t)h.entries[i * 16];
    if (from_inputs && entries != pairs) h.flags |= FLAG_DUP;  // two rows wrote one entry
    if (h.flags & FLAG_SORT) return kRetryGeneralSort;
    SPC_TRY(flags_status(h));
    km->n_pairs = pairs;
  }

  // coordinate sets kept for the export calls and for the next layer of a network
  if (!transposed) {
    if (needs_coarse) {
      std::swap(km->in_coords.p, own_rows.p);
      std::swap(km->in_coords.bytes, own_rows.bytes);
      std::swap(km->out_coords.p, coarse_rows.p);
      std::swap(km->out_coords.bytes, coarse_rows.bytes);
    } else {
      std::swap(km->in_coords.p, own_rows.p);
      std::swap(km->in_coords.bytes, own_rows.bytes);  // P_out == P_in: out_coords stays empty
    }
  } else {
    std::swap(km->out_coords.p, own_rows.p);
    std::swap(km->out_coords.bytes, own_rows.bytes);
    if (needs_coarse) {
      std::swap(km->in_coords.p, coarse_rows.p);
      std::swap(km->in_coords.bytes, coarse_rows.bytes);
    }  // stride 1: P_in == the caller's rows: in_coords stays empty
  }
  // temporaries (tables, key lists) go back to the pool here; the stream has either been
  // synchronised (stride 1) or later work on it is ordered after the kernels that read them
  *out = km.release();
  return SPCONV_OK;
}
}  // namespace

int kmap_build_in_side(spconv_kmap* km, hipStream_t st) {
  if (km->in_side.ready) return SPCONV_OK;
  const int V = km->V;
  SPC_TRY(alloc_side(km->in_side, km->n_in, V, st));
  if (km->n_in > 0) {
    SPC_TRY(fill_u32(km->in_side.map.p, km->in_side.rows_pad * V, 0xFFFFFFFFu, st));
    const long long entries = (long long)km->n_out * V;
    if (entries > 0) {
      hipLaunchKernelGGL(k_scatter_in_side, dim3(blocks_for(entries, 256)), dim3(256), 0, st,
                         km->out_side.map.as<int>(), entries, V, km->in_side.map.as<int>());
      SPC_LAUNCH_CHECK();
    }
    const int64_t rpw = 64 / V;
    const unsigned blocks = blocks_for(ceil_div(km->n_in, rpw), 4);
    const int* tm = km->in_side.map.as<int>();
    unsigned* tk = km->in_side.mask.as<unsigned>();
    if (V == 27)
      hipLaunchKernelGGL((k_mask_from_map<27>), dim3(blocks), dim3(256), 0, st, tm, (int)km->n_in, tk, (Ctl*)nullptr);
    else if (V == 8)
      hipLaunchKernelGGL((k_mask_from_map<8>), dim3(blocks), dim3(256), 0, st, tm, (int)km->n_in, tk, (Ctl*)nullptr);
    else
      hipLaunchKernelGGL((k_mask_from_map<1>), dim3(blocks), dim3(256), 0, st, tm, (int)km->n_in, tk, (Ctl*)nullptr);
    SPC_LAUNCH_CHECK();
  }
  km->in_side.ready = true;
  return SPCONV_OK;
}

// The kmap of the transposed convolution that pairs with src: the same pairs with inputs and
// outputs exchanged.  Its output-stationary table is src's input-side table and the other way
// round, so no table is built and nothing is probed: one scatter pass (unless src has its input
// side already) and device-to-device copies.
int kmap_pointwise(spconv_kmap* src, int on_outputs, hipStream_t st, spconv_kmap** out) {
  if (src->pending) SPC_TRY(kmap_status(src, st));  // a failed build has no rows to stand on
  std::unique_ptr<spconv_kmap> km(new (std::nothrow) spconv_kmap);
  if (!km) return SPCONV_ENOMEM;
  const int64_t rows = on_outputs ? src->n_out : src->n_in;
  km->K = 1;
  km->V = 1;
  km->stride = 1;
  km->transposed = 0;
  km->n_in = km->n_out = km->n_pairs = rows;
  km->build_stream = st;
  km->last_stream = st;
  SideMap& side = km->out_side;
  side.rows = rows;
  side.rows_pad = round_up(rows > 0 ? rows : 1, kRowPad);
  SPC_TRY(side.map.alloc((size_t)side.rows_pad * sizeof(int)));
  SPC_TRY(side.mask.alloc((size_t)side.rows_pad * sizeof(unsigned)));
  hipLaunchKernelGGL(k_identity_map, dim3(blocks_for(side.rows_pad, 256)), dim3(256), 0, st, side.map.as<int>(),
                     side.mask.as<unsigned>(), (long long)rows, (long long)side.rows_pad);
  SPC_LAUNCH_CHECK();
  side.ready = true;
  // Which buffer of src holds that side's rows: a kmap keeps the caller's rows and, for stride > 1,
  // the coarse set; with stride 1 the two sets are one (in_coords of a forward kmap, out_coords of
  // a transposed one).
  const DevBuf* from;
  if (!src->transposed)
    from = (on_outputs && (src->stride > 1 || src->dilated)) ? &src->out_coords : &src->in_coords;
  else
    from = (!on_outputs && src->stride > 1) ? &src->in_coords : &src->out_coords;
  if (rows == 0 || !from->p) {
    SPC_TRY(km->in_coords.alloc(16));
  } else {
    SPC_TRY(km->in_coords.alloc((size_t)rows * 16));
    SPC_HIP(hipMemcpyAsync(km->in_coords.p, from->p, (size_t)rows * 16, hipMemcpyDeviceToDevice, st));
  }
  *out = km.release();
  return SPCONV_OK;
}

int kmap_transpose(spconv_kmap* src, hipStream_t st, spconv_kmap** out) {
  if (src->dilated) return SPCONV_EINVAL;  // (no build call returns the transposed partner of a dilated map)
  if (src->pending) SPC_TRY(kmap_status(src, st));  // a failed build has no transpose
  SPC_TRY(kmap_build_in_side(src, st));
  // The transposed convolution's output-stationary table is the source's input-side table and the
  // other way round, and its coordinate sets are the source's with the roles exchanged: the two
  // kmaps share all four buffers (and whatever plans get cached on the tables); nothing is copied.
  // A kmap keeps the caller's rows and, for stride > 1, the coarse set; with stride 1 the two sets
  // are one and only the caller's rows are kept (in_coords of a forward kmap, out_coords of a
  // transposed one), the other buffer stays empty.
  auto none = []() { return std::make_shared<DevBuf>(); };
  std::shared_ptr<DevBuf> in_rows, out_rows;
  if (!src->transposed) {
    out_rows = src->in_coords_ref;
    in_rows = src->stride > 1 ? src->out_coords_ref : none();
  } else {
    in_rows = src->out_coords_ref;
    out_rows = src->stride > 1 ? src->in_coords_ref : none();
  }
  std::unique_ptr<spconv_kmap> km(new (std::nothrow) spconv_kmap(src->in_ref, src->out_ref, in_rows, out_rows));
  if (!km) return SPCONV_ENOMEM;
  km->K = src->K;
  km->V = src->V;
  km->stride = src->stride;
  km->transposed = src->transposed ? 0 : 1;
  km->n_in = src->n_out;
  km->n_out = src->n_in;
  km->n_pairs = src->n_pairs;
  km->build_stream = st;
  km->last_stream = st;
  *out = km.release();
  return SPCONV_OK;
}

int kmap_count_pairs(spconv_kmap* km, hipStream_t st, int64_t* per_k) {
  if (km->pending && !per_k) return kmap_status(km, st) == SPCONV_EHIP ? SPCONV_EHIP : SPCONV_OK;
  unsigned long long h[32] = {0};
  if (km->n_out > 0) {
    DevBuf counts;
    SPC_TRY(counts.alloc(32 * sizeof(unsigned long long)));
    SPC_TRY(fill_u32(counts.p, 64, 0u, st));
    const unsigned blocks = (unsigned)std::min<int64_t>(ceil_div(km->n_out, 256), 1024);
    hipLaunchKernelGGL(k_count_pairs, dim3(blocks), dim3(256), 0, st, km->out_side.mask.as<unsigned>(),
                       (int)km->n_out, counts.as<unsigned long long>());
    SPC_LAUNCH_CHECK();
    SPC_HIP(hipMemcpyAsync(h, counts.p, sizeof(h), hipMemcpyDeviceToHost, st));
    SPC_HIP(hipStreamSynchronize(st));
  }
  int64_t total = 0;
  for (int k = 0; k < km->V; ++k) {
    total += (int64_t)h[k];
    if (per_k) per_k[k] = (int64_t)h[k];
  }
  km->n_pairs = total;
  return SPCONV_OK;
}

namespace {
// The 125-bit mask of a K = 5 row from its planes' 25-bit masks: bit k of the row's mask is bit
// k % 32 of word k / 32, and k = 25 g + j.
__global__ void __launch_bounds__(256) k_join_masks5(Planes5 pl, long long rows, uint4* __restrict__ dst) {
  const long long r = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= rows) return;
  unsigned long long lo = 0, hi = 0;  // bits 0..63, 64..127
#pragma unroll
  for (int g = 0; g < 5; ++g) {
    const unsigned long long m = pl.mask[g][r];
    const int at = 25 * g;
    if (at < 64) {
      lo |= m << at;
      if (at + 25 > 64) hi |= m >> (64 - at);
    } else {
      hi |= m << (at - 64);
    }
  }
  dst[r] = make_uint4((unsigned)lo, (unsigned)(lo >> 32), (unsigned)hi, (unsigned)(hi >> 32));
}
}  // namespace

int kmap_export_mask_words(const spconv_kmap* km, uint32_t* dst, hipStream_t st) {
  if (km->groups.size() != 5) return SPCONV_EINVAL;
  Planes5 pl{};
  for (int g = 0; g < 5; ++g) pl.mask[g] = km->groups[(size_t)g]->out_side.mask.as<unsigned>();
  hipLaunchKernelGGL(k_join_masks5, dim3(blocks_for(km->n_out, 256)), dim3(256), 0, st, pl, (long long)km->n_out,
                     reinterpret_cast<uint4*>(dst));
  SPC_LAUNCH_CHECK();
  return SPCONV_OK;
}

}  // namespace spc

spconv_kmap::~spconv_kmap() {
  if (pending_host) {  // the copy into the pinned block must have landed before the block is reused
    spc::HostCtlHandle::finish(pending_host);
  }
}
