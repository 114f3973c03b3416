// Shared declarations of the library's translation units (host side).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <map>
#include <memory>
#include <vector>

#include "spconv.h"

namespace spc {

constexpr int kMaxSplit = 4;
constexpr int kRowPad = 256;  // map rows are padded to a multiple of the largest tile_m
constexpr int kWave = 64;
constexpr int kPlanSlabs = 0x10000;  // or-ed into the tile height of a plan key: sort keys start with a spatial slab

int hip_fail(hipError_t e, const char* what, const char* file, int line);
#define SPC_HIP(expr)                                                        \
  do {                                                                       \
    hipError_t e__ = (expr);                                                 \
    if (e__ != hipSuccess) return ::spc::hip_fail(e__, #expr, __FILE__, __LINE__); \
  } while (0)
#define SPC_TRY(expr)               \
  do {                              \
    int s__ = (expr);               \
    if (s__ != SPCONV_OK) return s__; \
  } while (0)
#define SPC_LAUNCH_CHECK() SPC_HIP(hipGetLastError())

void* dev_alloc(size_t bytes);
void dev_free(void* p);
// Names the stream that the pool's requests and returns of this thread belong to.
class StreamScope {
 public:
  explicit StreamScope(hipStream_t st);
  ~StreamScope();
  StreamScope(const StreamScope&) = delete;
  StreamScope& operator=(const StreamScope&) = delete;

 private:
  hipStream_t saved_;
};

// Owning device buffer (grow-only when used as scratch).
struct DevBuf {
  void* p = nullptr;
  size_t bytes = 0;
  DevBuf() = default;
  DevBuf(const DevBuf&) = delete;
  DevBuf& operator=(const DevBuf&) = delete;
  ~DevBuf() { release(); }
  void release() {
    if (p) dev_free(p);
    p = nullptr;
    bytes = 0;
  }
  int alloc(size_t n) {  // exact size, contents undefined
    release();
    if (n == 0) n = 16;
    p = dev_alloc(n);
    if (!p) return SPCONV_ENOMEM;
    bytes = n;
    return SPCONV_OK;
  }
  int reserve(size_t n) { return (n <= bytes && p) ? SPCONV_OK : alloc(n); }
  template <typename T> T* as() const { return reinterpret_cast<T*>(p); }
};

inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Plan of the implicit-GEMM kernels for one side of the map (output rows for
// fwd, input rows for dgrad), one split count and one tile height.
struct IgemmPlan {
  int n_split = 0;  // 0 = unsorted
  int tile_m = 128;
  int parts = 1;  // max(1, n_split)
  int64_t rows = 0, rows_pad = 0, n_tiles = 0;
  int lo[kMaxSplit] = {0}, width[kMaxSplit] = {0};
  size_t map_off[kMaxSplit] = {0};  // element offsets into maps
  DevBuf maps;      // reordered maps, part i: int32 [rows_pad][width[i]]  (unused when n_split == 0)
  DevBuf perm;      // int32 [parts][rows_pad]                              (unused when n_split == 0)
  DevBuf tilemask;  // uint32 [parts][n_tiles] bits relative to lo[i]
  bool slabs = false;  // sort keys start with a spatial slab: contiguous ranges of the order are spatially compact
};

struct WgradItem {
  int32_t k, pair_begin, pair_end, pad;  // pairs [pair_begin, pair_end) of offset k; item i writes partial tile i
};

// Weight-stationary view of the map for wgrad: the present pairs of each offset, compacted
// in row order (the M_delta of Section 2.2.1), cut into work items of about target_pairs.
struct WgradPlan {
  int64_t target_pairs = 0;
  int max_items = 0;  // launch bound: V + ceil(n_pairs / target_pairs)
  DevBuf pairs;       // int2 [pairs_cap]: (output row n, input row j), offset-major
  int64_t pairs_cap = 0;  // n_pairs, or the bound n_out * V while an asynchronous build is pending
  DevBuf seg;         // int32 [V+1]: pairs of offset k are seg[k]..seg[k+1]
  DevBuf items;       // WgradItem [max_items]
  DevBuf item_seg;    // int32 [V+2]: items of offset k are item_seg[k]..item_seg[k+1]; [V+1] = n_items
};

struct SideMap {      // one output-stationary table: rows x V
  int64_t rows = 0, rows_pad = 0;
  DevBuf map;         // int32 [rows_pad][V]
  DevBuf mask;        // uint32 [rows_pad]
  bool ready = false;
  std::map<std::pair<int, int>, std::unique_ptr<IgemmPlan>> plans;  // (n_split, tile_m)
};

}  // namespace spc

struct spconv_kmap {
  int K = 3, V = 27, stride = 1, transposed = 0;
  int dilated = 0;  // stride 1 with P_out = every point that has an input in its neighbourhood (not P_in)
  int64_t n_in = 0, n_out = 0, n_pairs = -1;
  hipStream_t build_stream = nullptr;
  hipStream_t last_stream = nullptr;  // stream of the most recent call that used this kmap
  // coordinate sets, reference-counted like the tables (a transposed partner holds the same two)
  std::shared_ptr<spc::DevBuf> in_coords_ref, out_coords_ref;
  spc::DevBuf& in_coords;
  spc::DevBuf& out_coords;
  // The two tables are reference-counted: a kmap and the kmap of its paired transposed
  // convolution hold the same two tables with the roles exchanged (spconv_kmap_transpose).
  std::shared_ptr<spc::SideMap> out_ref, in_ref;
  spc::SideMap& out_side;  // M: rows = n_out, entries index input rows
  spc::SideMap& in_side;   // T: rows = n_in, T[j][k] = n  <=>  M[n][k] = j (built on demand)
  spconv_kmap()
      : in_coords_ref(std::make_shared<spc::DevBuf>()), out_coords_ref(std::make_shared<spc::DevBuf>()),
        in_coords(*in_coords_ref), out_coords(*out_coords_ref), out_ref(std::make_shared<spc::SideMap>()),
        in_ref(std::make_shared<spc::SideMap>()), out_side(*out_ref), in_side(*in_ref) {}
  spconv_kmap(std::shared_ptr<spc::SideMap> out_table, std::shared_ptr<spc::SideMap> in_table,
              std::shared_ptr<spc::DevBuf> in_rows, std::shared_ptr<spc::DevBuf> out_rows)
      : in_coords_ref(std::move(in_rows)), out_coords_ref(std::move(out_rows)), in_coords(*in_coords_ref),
        out_coords(*out_coords_ref), out_ref(std::move(out_table)), in_ref(std::move(in_table)), out_side(*out_ref),
        in_side(*in_ref) {}
  spconv_kmap(const spconv_kmap&) = delete;
  spconv_kmap& operator=(const spconv_kmap&) = delete;
  std::map<int64_t, std::unique_ptr<spc::WgradPlan>> wplans;  // by target_pairs
  // K = 5 (125 offsets): the kmap is held as its five x-planes, each a submanifold map of 25 offsets
  // (dx = g - 2) over the same rows, so that masks, sort keys and tile masks stay 32-bit words and
  // every kernel runs on a plane as it runs on a 27-offset map; the planes' results are summed like
  // the parts of a split.  Offset k of the whole map is offset k % 25 of plane k / 25.
  std::vector<std::unique_ptr<spconv_kmap>> groups;
  spc::DevBuf scratch;    // split partial sums / wgrad partial tiles
  // build whose status was not read yet: the pinned block the probe kernel publishes flags and
  // pair count to, with the event that marks the probe's completion
  void* pending_host = nullptr;
  bool pending = false;
  int build_status = SPCONV_OK;  // verdict of the build once resolved: every later spconv_kmap_status returns it
  ~spconv_kmap();
  bool submanifold() const { return stride == 1 && !transposed && !dilated; }
};

namespace spc {

// ---- kmap.hip
int kmap_build(const int32_t* coords, int64_t N, int K, int stride, int transposed, bool async, hipStream_t st,
               spconv_kmap** out, bool dilate = false);
int kmap_status(spconv_kmap* km, hipStream_t st);  // resolves a pending asynchronous build (synchronises)
int kmap_build_in_side(spconv_kmap* km, hipStream_t st);
int kmap_count_pairs(spconv_kmap* km, hipStream_t st, int64_t* per_k /*[V] or null*/);
int kmap_export_mask_words(const spconv_kmap* km, uint32_t* dst, hipStream_t st);  // K = 5: [n_out][4]
int kmap_transpose(spconv_kmap* src, hipStream_t st, spconv_kmap** out);
int kmap_pointwise(spconv_kmap* src, int on_outputs, hipStream_t st, spconv_kmap** out);

// ---- sort.hip
// Stable LSD radix sort of n (key, value) pairs on key bits [0, key_bits).
// keys/vals are ping-pong buffers of n elements each; *in_b tells where the
// result ended up (0: buffer a, 1: buffer b).  hist must hold
// sort_hist_elems(n) uint32.
size_t sort_hist_elems(int64_t n);
// plan.hip: one launch per digit, at most 131072 keys (SPCONV_EINVAL beyond); see there for error_word
int msort_keys_u32(uint32_t* key_a, uint32_t* key_b, int64_t n, int key_bits, unsigned* error_word, unsigned error_bit,
                   hipStream_t st, int* in_b);
// Exclusive scan in place; `sums` is scratch of scan_sums_elems(elems) counters.
size_t scan_sums_elems(int64_t elems);
int scan_u32_inplace(uint32_t* data, int64_t elems, uint32_t* sums, hipStream_t st);
int radix_sort_u32(uint32_t* key_a, uint32_t* key_b, int32_t* val_a, int32_t* val_b, int64_t n,
                   int key_bits, uint32_t* hist, hipStream_t st, int* in_b);
// Keys only, 64-bit, on the digit positions whose bits are set in `varying`.
int radix_sort_u64(uint64_t* key_a, uint64_t* key_b, int64_t n, uint64_t varying, uint32_t* hist,
                   hipStream_t st, int* in_b);

// ---- launch arithmetic.  Everything a launch derives from the layer's shape is computed by these
// host functions and by nothing else (the run functions call them), so that it can be checked on
// the CPU: spconv_describe_launch reports it, and a test walks the index formulas of the kernels
// over a grid of shapes.  They return SPCONV_EINVAL for shapes the kernels do not take.
struct PlanShape {  // plan_get: parts of the offset range, padded rows, tiles
  int parts = 1;
  int lo[kMaxSplit] = {0}, width[kMaxSplit] = {0};
  size_t map_off[kMaxSplit] = {0};  // element offsets of the parts' reordered maps
  size_t map_elems = 0;             // all parts together
  int64_t rows_pad = 0, n_tiles = 0;
};
int plan_shape(int V, int64_t rows, int n_split, int tile_m, PlanShape* s);

struct WaveShape {  // igemm_wave_run (kernel 1)
  int bn = 0, waves = 0, ks = 0, max_width = 0, threads = 0;
  int slab_bytes = 0, map_bytes = 0;
  size_t lds_bytes = 0;
  unsigned grid[3] = {0, 0, 0};
  unsigned feats_bytes = 0;
};
int igemm_wave_shape(int V, int n_split, int64_t rows, int64_t rows_src, int c_red, int c_out, int tile_n,
                     WaveShape* s);

struct TileShape {  // igemm_run (kernel 2 and the fp32 kernel)
  int bm = 0, bn = 0, kc = 0, nw = 0, threads = 0;
  size_t lds_bytes = 0;
  unsigned grid[3] = {0, 0, 0};
  unsigned feats_bytes = 0;
};
int igemm_tile_shape(int V, int n_split, int64_t rows, int64_t rows_src, int c_red, int c_out, int tile_m, int tile_n,
                     bool f32, bool dgrad, TileShape* s);

// ---- plan.hip
// tile_m may carry kPlanSlabs (a plan of its own in the cache)
int plan_get(spconv_kmap* km, SideMap& side, int n_split, int tile_m, hipStream_t st, IgemmPlan** out);
int plan_mac_units(spconv_kmap* km, SideMap& side, IgemmPlan* plan, int group_rows, hipStream_t st,
                   int64_t* executed);
int wplan_get(spconv_kmap* km, int64_t target_pairs, hipStream_t st, WgradPlan** out);

// ---- igemm.hip
struct IgemmArgs {
  const void* feats;    // [rows_src][c_red]
  const void* weights;  // [V][C_in][C_out] (always the forward layout)
  void* out;            // [rows][c_out_eff] in dtype, or nullptr when partial sums are used
  float* partial;       // [parts][rows][c_out_eff] fp32: the kernels write partial sums whenever this is set
  int C_in, C_out;      // of the layer (forward orientation)
  int dgrad;            // 0: reduce over C_in, produce C_out.  1: reduce over C_out, produce C_in
  int mirror;           // weight slice of map column k is V-1-k (dgrad on the submanifold map itself)
  spconv_dtype dtype;
  int tile_n;           // 0 = auto
};
int igemm_run(const spconv_kmap* km, const SideMap& side, const IgemmPlan& plan, const IgemmArgs& a,
              hipStream_t st);
// ---- igemm_wave.hip (weights resident in LDS; plan tile_m must be 16)
int igemm_wave_pick_bn(int V, int n_split, int c_red, int c_out, int tile_n, int* waves_out);
int igemm_wave_run(const spconv_kmap* km, const SideMap& side, const IgemmPlan& plan, const IgemmArgs& a,
                   hipStream_t st);
int split_reduce(const float* partial, int parts, int64_t rows, int c, spconv_dtype dtype, void* out,
                 hipStream_t st);

// ---- fod.hip (fetch-on-demand dataflow; wp must have been cut into items of tile_m pairs)
bool fod_supported(const spconv_kmap* km, int dgrad, int C_in, int C_out, spconv_dtype dtype);
int fod_run(spconv_kmap* km, const WgradPlan& wp, const IgemmArgs& a, int tile_m, void* dst, hipStream_t st);

// ---- wgrad.hip
int wgrad_run(spconv_kmap* km, const WgradPlan& wp, const void* feats, const void* dout, int C_in,
              int C_out, spconv_dtype dtype, float* dweights, hipStream_t st);

}  // namespace spc
