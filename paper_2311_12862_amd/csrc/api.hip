// C ABI entry points: argument checks, plan look-up, dispatch, the device
// memory pool and the tuner.  No arithmetic of the method lives here.
#include "common.h"

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

namespace spc {

static thread_local char g_hip_err[512] = "";

int hip_fail(hipError_t e, const char* what, const char* file, int line) {
  std::snprintf(g_hip_err, sizeof(g_hip_err), "%s: %s (%s:%d)", hipGetErrorString(e), what, file, line);
  (void)hipGetLastError();  // clear the sticky error so that later calls report their own
  return SPCONV_EHIP;
}

// ---- device memory: user callbacks, else a small caching pool over hipMalloc.
// Blocks handed back are reused by later requests of a similar size.  Nothing waits for the
// kernels that used a block: reuse is safe because it is ordered by the stream, so a block is
// only handed to a request made for the stream it was last used on.  Every entry point names
// that stream for the duration of the call (StreamScope).
namespace {
std::mutex g_mem_mu;
void* (*g_user_alloc)(size_t, void*, void*) = nullptr;
void (*g_user_free)(void*, void*, void*) = nullptr;
void* g_user_ctx = nullptr;

struct Block {
  void* p;
  size_t bytes;
  hipStream_t stream;  // the stream whose work last touched the block
};
thread_local hipStream_t t_stream = nullptr;
std::vector<Block> g_free_blocks;
std::map<void*, size_t> g_live;
size_t g_pooled_bytes = 0;
constexpr size_t kPoolLimit = (size_t)8 << 30;

void pool_trim_locked() {
  for (auto& b : g_free_blocks) (void)hipFree(b.p);
  g_free_blocks.clear();
  g_pooled_bytes = 0;
}
}  // namespace

StreamScope::StreamScope(hipStream_t st) : saved_(t_stream) { t_stream = st; }
StreamScope::~StreamScope() { t_stream = saved_; }

void* dev_alloc(size_t bytes) {
  std::lock_guard<std::mutex> lk(g_mem_mu);
  if (g_user_alloc) return g_user_alloc(bytes, (void*)t_stream, g_user_ctx);  // the stream of the call in progress
  bytes = (size_t)round_up((int64_t)bytes, 256);
  int best = -1;
  for (int i = 0; i < (int)g_free_blocks.size(); ++i) {
    const size_t b = g_free_blocks[i].bytes;
    if (g_free_blocks[i].stream != t_stream) continue;
    if (b >= bytes && b <= bytes + bytes / 2 + 4096 && (best < 0 || b < g_free_blocks[best].bytes)) best = i;
  }
  if (best >= 0) {
    Block blk = g_free_blocks[best];
    g_free_blocks.erase(g_free_blocks.begin() + best);
    g_pooled_bytes -= blk.bytes;
    g_live[blk.p] = blk.bytes;
    return blk.p;
  }
  void* p = nullptr;
  if (hipMalloc(&p, bytes) != hipSuccess) {
    (void)hipGetLastError();
    pool_trim_locked();
    if (hipMalloc(&p, bytes) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
  }
  g_live[p] = bytes;
  return p;
}

void dev_free(void* p) {
  if (!p) return;
  std::lock_guard<std::mutex> lk(g_mem_mu);
  if (g_user_free && g_live.find(p) == g_live.end()) {
    g_user_free(p, (void*)t_stream, g_user_ctx);
    return;
  }
  auto it = g_live.find(p);
  if (it == g_live.end()) return;
  const size_t bytes = it->second;
  g_live.erase(it);
  if (g_pooled_bytes + bytes > kPoolLimit) {
    (void)hipFree(p);
    return;
  }
  g_free_blocks.push_back({p, bytes, t_stream});
  g_pooled_bytes += bytes;
}

namespace {

bool dtype_ok(int d) { return d == SPCONV_F32 || d == SPCONV_F16 || d == SPCONV_BF16; }

int check_channels(int C_in, int C_out, spconv_dtype dtype) {
  const int q = dtype == SPCONV_F32 ? 4 : 8;
  if (C_in <= 0 || C_out <= 0 || C_in % q || C_out % q || C_in > 4096 || C_out > 4096) return SPCONV_EINVAL;
  return SPCONV_OK;
}

// Normalised copy of the caller's config.
int resolve_config(const spconv_config* cfg, spconv_dtype dtype, spconv_config* out) {
  spconv_config c{};
  if (cfg) c = *cfg;
  if (c.n_split < 0 || c.n_split > kMaxSplit) return SPCONV_EINVAL;
  if (c.tile_m == 0) c.tile_m = 128;
  if (c.tile_m != 64 && c.tile_m != 128 && c.tile_m != 256) return SPCONV_EINVAL;
  if (c.tile_n != 0 && c.tile_n != 16 && c.tile_n != 32 && c.tile_n != 64 && c.tile_n != 128) return SPCONV_EINVAL;
  if (c.wgrad_pairs < 0 || c.kernel < 0 || c.kernel > 3 || (c.flags & ~SPCONV_FLAG_SLABS)) return SPCONV_EINVAL;
  if (c.kernel == 3) {  // fetch-on-demand: unsorted pair lists, tiles of 64 or 128 pairs (fp32: 64)
    if (cfg->tile_m == 0) c.tile_m = 64;
    if (c.n_split != 0 || c.tile_m == 256 || c.tile_n == 16) return SPCONV_EINVAL;
    if (dtype == SPCONV_F32 && c.tile_m != 64) return SPCONV_EINVAL;
  } else if (dtype == SPCONV_F32) {  // the fp32 implicit-GEMM kernel has one tile shape
    c.tile_m = 64;
    c.kernel = 2;
  }
  *out = c;
  return SPCONV_OK;
}

// Tile height of the plan a configuration uses, as the plan cache keys it.
int plan_tile(const spconv_config& c, bool wave) {
  return (wave ? 16 : c.tile_m) | ((c.flags & SPCONV_FLAG_SLABS) && c.n_split > 0 ? kPlanSlabs : 0);
}

// Which table an op walks, and with which weight indexing.
struct OpSide {
  SideMap* side;
  int dgrad, mirror;
};

int side_for(spconv_kmap* km, spconv_op op, hipStream_t st, OpSide* o) {
  if (op == SPCONV_OP_FWD) {
    *o = {&km->out_side, 0, 0};
    return SPCONV_OK;
  }
  if (km->submanifold()) {  // M[n][k] = j  <=>  M[j][V-1-k] = n: dgrad walks M itself with mirrored weights
    *o = {&km->out_side, 1, 1};
    return SPCONV_OK;
  }
  SPC_TRY(kmap_build_in_side(km, st));
  *o = {&km->in_side, 1, 0};
  return SPCONV_OK;
}

int64_t auto_wgrad_pairs(spconv_kmap* km, int C_in, int C_out) {
  const int tile = (C_in > 64 || C_out > 64) ? 128 : 64;
  const int64_t tiles = ceil_div(C_in, tile) * ceil_div(C_out, tile);
  const int64_t want_items = std::max<int64_t>(32, 1536 / tiles);
  const int64_t pairs = km->n_pairs > 0 ? km->n_pairs : km->n_out * 4;  // unknown while a build is pending
  return std::max<int64_t>(1024, ceil_div(pairs, want_items));
}

// Which kernel runs a forward / dgrad call and on which tiles: the caller's configuration with
// the automatic choices filled in.  Pure host arithmetic (spconv_describe_launch reports it).
struct KernelChoice {
  bool wave = false;  // kernel 1 (weights resident in LDS) instead of kernel 2 (workgroup tiles)
  int tile_m = 0;     // plan tile height: 16 for kernel 1
  int tile_n = 0;     // as passed to the kernel (0: its own default)
};
int choose_kernel(int V, int64_t rows_dst, int c_red, int c_cols, spconv_dtype dtype, bool tile_m_given,
                  const spconv_config& c, KernelChoice* out) {
  KernelChoice k;
  int tile_m = c.tile_m;
  if (!tile_m_given && dtype != SPCONV_F32) {
    // automatic tile height (measured on unsorted maps, 10k .. 300k rows): 128 rows when that still
    // leaves several workgroups per CU, or when the reduction is long (>= 128 channels) and there
    // are enough rows for a workgroup per CU anyway; 64 rows otherwise
    tile_m = (ceil_div(rows_dst, 128) * ceil_div(c_cols, 128) >= 2048 || (rows_dst >= 25000 && c_red >= 128)) ? 128 : 64;
  }
  if (c.kernel != 2 && dtype != SPCONV_F32) {
    const int bn = igemm_wave_pick_bn(V, c.n_split, c_red, c_cols, c.tile_n, nullptr);
    k.wave = bn > 0;
    if (!k.wave && c.kernel == 1) return SPCONV_EINVAL;
    // Automatic choice: the LDS-resident kernel gathers the input once per column tile.  It wins
    // while the output is at most two tiles wide (64 -> 64 is 2 x 32) and, beyond that, while
    // tiles x reduced channels x rows stays small: few rows leave the tiled kernel without enough
    // workgroups, many rows make the repeated gathers the larger cost (measured: 100k rows,
    // 64 -> 256 in eight tiles 89 us against 114 us; 128 -> 128 in eight 16-column tiles 160 us
    // against 131 us; 10k rows, 128 -> 128 25 us against 41 us; 300k rows, 64 -> 128 213 us
    // against 171 us).
    if (k.wave && c.kernel == 0) {
      const int64_t tiles = ceil_div(c_cols, bn);
      if (tiles > 2 && (double)tiles * c_red * (double)rows_dst > 6e7) k.wave = false;
    }
  }
  if (!k.wave && c.tile_n == 16) return SPCONV_EINVAL;
  k.tile_m = k.wave ? 16 : tile_m;
  k.tile_n = c.tile_n;
  // few row tiles: 64-column tiles double the workgroups of the tiled kernel (10k rows, 256 -> 256:
  // 91 us against 104 us)
  if (!k.wave && c.tile_n == 0 && dtype != SPCONV_F32 && tile_m == 64 && c_cols > 64 &&
      ceil_div(rows_dst, 64) * ceil_div(c_cols, 128) < 400)
    k.tile_n = 64;
  *out = k;
  return SPCONV_OK;
}

// ---- the fixed scratch array of the entry point that allocates nothing --------------------
// Split partial sums of spconv_fwd_noalloc live here instead of in a buffer of the kmap.  In
// host code the array's name is only a stand-in: the device address comes from
// hipGetSymbolAddress, once per device (each GPU holds its own copy), with that device current.
constexpr size_t kStaticScratchBytes = (size_t)SPCONV_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out) {
  int dev = -1;
  SPC_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return SPCONV_EINVAL;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    SPC_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return SPCONV_EHIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return SPCONV_OK;
}

// prepared_only: the call may not allocate.  Plans are looked up, never built (SPCONV_ENOPLAN when
// missing), and split partial sums go to the fixed scratch array (SPCONV_ELIMIT beyond its size).
// K = 5: forward / dgrad as the sum over the five 25-offset planes.  Every plane runs like a kmap of
// its own (its plan, the kernel and tiles chosen for 25 offsets) and writes fp32 partial sums; one
// reduction adds the parts of all planes and rounds once (Section 4.1's split reduction, over planes
// as well as over mask splits).  Plane g holds the offsets 25 g .. 25 g + 24, so its weights are
// that slice; dgrad on the submanifold map mirrors the offset, 124 - k, which is offset 24 - j of
// plane 4 - g.
int run_planes(spconv_op op, const void* src, const void* weights, spconv_kmap* km, int C_in, int C_out,
               spconv_dtype dtype, const spconv_config* cfg, const spconv_config& c_in, void* dst, hipStream_t st) {
  const int64_t rows = km->n_out;
  const int dgrad = op == SPCONV_OP_DGRAD;
  const int c_red = dgrad ? C_out : C_in, c_dst = dgrad ? C_in : C_out;
  const size_t e = dtype == SPCONV_F32 ? 4 : 2;
  const int n_planes = (int)km->groups.size();
  struct Launch {
    IgemmPlan* plan;
    bool wave;
    int tile_n;
  };
  std::vector<Launch> ls((size_t)n_planes);
  int parts_total = 0;
  for (int g = 0; g < n_planes; ++g) {
    spconv_kmap* sub = km->groups[(size_t)g].get();
    sub->last_stream = st;
    spconv_config c = c_in;
    KernelChoice kc;
    SPC_TRY(choose_kernel(sub->V, rows, c_red, c_dst, dtype, cfg && cfg->tile_m != 0, c, &kc));
    c.tile_m = kc.wave ? c.tile_m : kc.tile_m;
    SPC_TRY(plan_get(sub, sub->out_side, c.n_split, plan_tile(c, kc.wave), st, &ls[(size_t)g].plan));
    ls[(size_t)g].wave = kc.wave;
    ls[(size_t)g].tile_n = kc.tile_n;
    parts_total += ls[(size_t)g].plan->parts;
  }
  SPC_TRY(km->scratch.reserve((size_t)parts_total * rows * c_dst * sizeof(float)));
  int part0 = 0;
  for (int g = 0; g < n_planes; ++g) {
    spconv_kmap* sub = km->groups[(size_t)g].get();
    const int wg = dgrad ? n_planes - 1 - g : g;
    IgemmArgs a{};
    a.feats = src;
    a.weights = static_cast<const char*>(weights) + (size_t)wg * sub->V * C_in * C_out * e;
    a.C_in = C_in;
    a.C_out = C_out;
    a.dgrad = dgrad;
    a.mirror = dgrad;
    a.dtype = dtype;
    a.tile_n = ls[(size_t)g].tile_n;
    a.out = nullptr;
    a.partial = km->scratch.as<float>() + (size_t)part0 * rows * c_dst;
    const IgemmPlan& plan = *ls[(size_t)g].plan;
    SPC_TRY(ls[(size_t)g].wave ? igemm_wave_run(sub, sub->out_side, plan, a, st) : igemm_run(sub, sub->out_side, plan, a, st));
    part0 += plan.parts;
  }
  return split_reduce(km->scratch.as<float>(), parts_total, rows, c_dst, dtype, dst, st);
}

int run_igemm_op(spconv_op op, const void* src, const void* weights, spconv_kmap* km, int C_in, int C_out,
                 spconv_dtype dtype, const spconv_config* cfg, void* dst, hipStream_t st,
                 bool prepared_only = false) {
  if (!km || !dtype_ok(dtype)) return SPCONV_EINVAL;
  SPC_TRY(check_channels(C_in, C_out, dtype));
  km->last_stream = st;
  const int64_t rows_dst = op == SPCONV_OP_FWD ? km->n_out : km->n_in;
  if (rows_dst == 0) return SPCONV_OK;
  if (!src || !weights || !dst) return SPCONV_EINVAL;
  spconv_config c;
  SPC_TRY(resolve_config(cfg, dtype, &c));
  if (!km->groups.empty()) {
    if (prepared_only || c.kernel == 3) return SPCONV_EINVAL;
    return run_planes(op, src, weights, km, C_in, C_out, dtype, cfg, c, dst, st);
  }
  if (c.kernel == 3) {  // fetch-on-demand dataflow over the weight-stationary pair lists
    if (prepared_only) return SPCONV_EINVAL;
    const int dgrad = op == SPCONV_OP_DGRAD;
    if (!fod_supported(km, dgrad, C_in, C_out, dtype)) return SPCONV_EINVAL;
    WgradPlan* wp = nullptr;
    SPC_TRY(wplan_get(km, c.tile_m, st, &wp));
    IgemmArgs a{};
    a.feats = src;
    a.weights = weights;
    a.C_in = C_in;
    a.C_out = C_out;
    a.dgrad = dgrad;
    a.dtype = dtype;
    a.tile_n = c.tile_n;
    return fod_run(km, *wp, a, c.tile_m, dst, st);
  }
  OpSide os;
  if (prepared_only) {
    if (op != SPCONV_OP_FWD) return SPCONV_EINVAL;
    os = {&km->out_side, 0, 0};
  } else {
    SPC_TRY(side_for(km, op, st, &os));
  }
  const int c_red = os.dgrad ? C_out : C_in;
  const int c_cols = os.dgrad ? C_in : C_out;
  KernelChoice kc;
  SPC_TRY(choose_kernel(km->V, rows_dst, c_red, c_cols, dtype, cfg && cfg->tile_m != 0, c, &kc));
  const bool wave = kc.wave;
  c.tile_m = wave ? c.tile_m : kc.tile_m;
  IgemmPlan* plan = nullptr;
  if (prepared_only) {
    if (c.n_split > km->V) return SPCONV_EINVAL;
    auto it = os.side->plans.find(std::make_pair((int)c.n_split, plan_tile(c, wave)));
    if (it == os.side->plans.end()) return SPCONV_ENOPLAN;
    plan = it->second.get();
  } else {
    SPC_TRY(plan_get(km, *os.side, c.n_split, plan_tile(c, wave), st, &plan));
  }
  IgemmArgs a{};
  a.feats = src;
  a.weights = weights;
  a.C_in = C_in;
  a.C_out = C_out;
  a.dgrad = os.dgrad;
  a.mirror = os.mirror;
  a.dtype = dtype;
  a.tile_n = kc.tile_n;
  const int c_dst = os.dgrad ? C_in : C_out;
  if (plan->parts > 1) {
    const size_t need = (size_t)plan->parts * plan->rows * c_dst * sizeof(float);
    if (prepared_only) {
      if (need > kStaticScratchBytes) return SPCONV_ELIMIT;
      void* ptr = nullptr;
      SPC_TRY(static_scratch(&ptr));
      a.partial = reinterpret_cast<float*>(ptr);
    } else {
      SPC_TRY(km->scratch.reserve(need));
      a.partial = km->scratch.as<float>();
    }
    a.out = nullptr;
    SPC_TRY(wave ? igemm_wave_run(km, *os.side, *plan, a, st) : igemm_run(km, *os.side, *plan, a, st));
    return split_reduce(a.partial, plan->parts, plan->rows, c_dst, dtype, dst, st);
  }
  a.out = dst;
  return wave ? igemm_wave_run(km, *os.side, *plan, a, st) : igemm_run(km, *os.side, *plan, a, st);
}

}  // namespace
}  // namespace spc

using namespace spc;

extern "C" {

SPCONV_API int spconv_build_kmap(const int32_t* coords, int64_t N, int K, int stride, int transposed, void* stream,
                      spconv_kmap** out) {
  StreamScope scope((hipStream_t)stream);
  if (!out) return SPCONV_EINVAL;
  *out = nullptr;
  if (N < 0 || N > (int64_t)0x7FFFFF00 / 32 || (N > 0 && !coords)) return SPCONV_EINVAL;
  if (K != 1 && K != 2 && K != 3 && K != 5) return SPCONV_EINVAL;
  if (K == 2 && stride != 2) return SPCONV_EINVAL;  // the even kernel is the non-overlapping 2x2x2 / stride-2 layer
  if (K == 5 && (stride != 1 || transposed)) return SPCONV_EINVAL;  // K = 5: submanifold maps only
  if (stride < 1 || stride > 64) return SPCONV_EINVAL;
  if (transposed != 0 && transposed != 1) return SPCONV_EINVAL;
  return kmap_build(coords, N, K, stride, transposed, false, (hipStream_t)stream, out);
}

SPCONV_API int spconv_build_kmap_async(const int32_t* coords, int64_t N, int K, int stride, int transposed,
                                       void* stream, spconv_kmap** out) {
  StreamScope scope((hipStream_t)stream);
  if (!out) return SPCONV_EINVAL;
  *out = nullptr;
  if (N < 0 || N > (int64_t)0x7FFFFF00 / 32 || (N > 0 && !coords)) return SPCONV_EINVAL;
  if (K != 1 && K != 2 && K != 3) return SPCONV_EINVAL;
  if (K == 2 && stride != 2) return SPCONV_EINVAL;  // the even kernel is the non-overlapping 2x2x2 / stride-2 layer
  if (stride < 1 || stride > 64) return SPCONV_EINVAL;
  if (transposed != 0 && transposed != 1) return SPCONV_EINVAL;
  return kmap_build(coords, N, K, stride, transposed, true, (hipStream_t)stream, out);
}

SPCONV_API int spconv_build_kmap_dilated(const int32_t* coords, int64_t N, int K, void* stream, spconv_kmap** out) {
  StreamScope scope((hipStream_t)stream);
  if (!out) return SPCONV_EINVAL;
  *out = nullptr;
  // the candidate set holds up to K^3 points per input row
  if (N < 0 || N > (int64_t)0x7FFFFF00 / 32 / 27 || (N > 0 && !coords)) return SPCONV_EINVAL;
  if (K != 1 && K != 3) return SPCONV_EINVAL;
  return kmap_build(coords, N, K, 1, 0, false, (hipStream_t)stream, out, true);
}

SPCONV_API int spconv_kmap_pointwise(spconv_kmap* km, int on_outputs, void* stream, spconv_kmap** out) {
  StreamScope scope((hipStream_t)stream);
  if (!out) return SPCONV_EINVAL;
  *out = nullptr;
  if (!km || (on_outputs != 0 && on_outputs != 1)) return SPCONV_EINVAL;
  km->last_stream = (hipStream_t)stream;
  return kmap_pointwise(km, on_outputs, (hipStream_t)stream, out);
}

SPCONV_API int spconv_kmap_transpose(spconv_kmap* km, void* stream, spconv_kmap** out) {
  StreamScope scope((hipStream_t)stream);
  if (!out) return SPCONV_EINVAL;
  *out = nullptr;
  if (!km || !km->groups.empty()) return SPCONV_EINVAL;
  km->last_stream = (hipStream_t)stream;
  return kmap_transpose(km, (hipStream_t)stream, out);
}

SPCONV_API int spconv_kmap_status(spconv_kmap* km, void* stream) {
  StreamScope scope((hipStream_t)stream);
  if (!km) return SPCONV_EINVAL;
  return kmap_status(km, (hipStream_t)stream);
}

SPCONV_API int spconv_kmap_sizes(const spconv_kmap* km, int64_t* n_in, int64_t* n_out, int64_t* n_pairs) {
  if (!km) return SPCONV_EINVAL;
  if (n_in) *n_in = km->n_in;
  if (n_out) *n_out = km->n_out;
  if (n_pairs) {
    if (km->n_pairs < 0) SPC_TRY(kmap_count_pairs(const_cast<spconv_kmap*>(km), km->build_stream, nullptr));
    *n_pairs = km->n_pairs;
  }
  return SPCONV_OK;
}

SPCONV_API int spconv_kmap_out_coords(const spconv_kmap* km, int32_t* dst, void* stream) {
  StreamScope scope((hipStream_t)stream);
  if (!km || (!dst && km->n_out > 0)) return SPCONV_EINVAL;
  if (km->n_out == 0) return SPCONV_OK;
  const DevBuf& b = km->submanifold() ? km->in_coords : km->out_coords;
  SPC_HIP(hipMemcpyAsync(dst, b.p, (size_t)km->n_out * 16, hipMemcpyDeviceToDevice, (hipStream_t)stream));
  return SPCONV_OK;
}

SPCONV_API int spconv_kmap_in_coords(const spconv_kmap* km, int32_t* dst, void* stream) {
  StreamScope scope((hipStream_t)stream);
  if (!km || (!dst && km->n_in > 0)) return SPCONV_EINVAL;
  if (km->n_in == 0) return SPCONV_OK;
  const DevBuf& b = (km->transposed && km->stride == 1 && !km->dilated) ? km->out_coords : km->in_coords;
  SPC_HIP(hipMemcpyAsync(dst, b.p, (size_t)km->n_in * 16, hipMemcpyDeviceToDevice, (hipStream_t)stream));
  return SPCONV_OK;
}

SPCONV_API int spconv_kmap_export(const spconv_kmap* km, int32_t* dst, void* stream) {
  StreamScope scope((hipStream_t)stream);
  if (!km || (!dst && km->n_out > 0)) return SPCONV_EINVAL;
  if (km->n_out == 0) return SPCONV_OK;
  if (!km->groups.empty()) {  // K = 5: column 25 g + j of the whole map is column j of plane g
    const size_t n_planes = km->groups.size();
    for (size_t g = 0; g < n_planes; ++g) {
      const spconv_kmap& sub = *km->groups[g];
      SPC_HIP(hipMemcpy2DAsync(dst + g * sub.V, (size_t)km->V * sizeof(int32_t), sub.out_side.map.p,
                               (size_t)sub.V * sizeof(int32_t), (size_t)sub.V * sizeof(int32_t), (size_t)km->n_out,
                               hipMemcpyDeviceToDevice, (hipStream_t)stream));
    }
    return SPCONV_OK;
  }
  SPC_HIP(hipMemcpyAsync(dst, km->out_side.map.p, (size_t)km->n_out * km->V * sizeof(int32_t),
                         hipMemcpyDeviceToDevice, (hipStream_t)stream));
  return SPCONV_OK;
}

SPCONV_API int spconv_kmap_export_mask(const spconv_kmap* km, uint32_t* dst, void* stream) {
  StreamScope scope((hipStream_t)stream);
  if (!km || (!dst && km->n_out > 0)) return SPCONV_EINVAL;
  if (km->n_out == 0) return SPCONV_OK;
  if (!km->groups.empty()) return kmap_export_mask_words(km, dst, (hipStream_t)stream);
  SPC_HIP(hipMemcpyAsync(dst, km->out_side.mask.p, (size_t)km->n_out * sizeof(uint32_t), hipMemcpyDeviceToDevice,
                         (hipStream_t)stream));
  return SPCONV_OK;
}

SPCONV_API int spconv_kmap_prepare(spconv_kmap* km, spconv_op op, const spconv_config* cfg, void* stream) {
  StreamScope scope((hipStream_t)stream);
  if (!km || op < SPCONV_OP_FWD || op > SPCONV_OP_WGRAD) return SPCONV_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  km->last_stream = st;
  if (!km->groups.empty()) {
    for (auto& sub : km->groups) SPC_TRY(spconv_kmap_prepare(sub.get(), op, cfg, stream));
    return SPCONV_OK;
  }
  spconv_config c;
  SPC_TRY(resolve_config(cfg, SPCONV_F16, &c));
  if (op == SPCONV_OP_WGRAD) {
    if (c.wgrad_pairs == 0) return SPCONV_EINVAL;  // the automatic choice needs the channel counts
    WgradPlan* wp = nullptr;
    return wplan_get(km, c.wgrad_pairs, st, &wp);
  }
  if (c.kernel == 3) {
    WgradPlan* wp = nullptr;
    return wplan_get(km, c.tile_m, st, &wp);
  }
  OpSide os;
  SPC_TRY(side_for(km, op, st, &os));
  IgemmPlan* plan = nullptr;
  return plan_get(km, *os.side, c.n_split, plan_tile(c, c.kernel == 1), st, &plan);
}

SPCONV_API int spconv_kmap_drop_plans(spconv_kmap* km) {
  if (!km) return SPCONV_EINVAL;
  StreamScope scope(km->last_stream);
  SPC_HIP(hipDeviceSynchronize());
  km->out_side.plans.clear();
  km->in_side.plans.clear();
  if (km->in_ref.use_count() == 1) {  // (a transposed partner uses this table as its own map)
    km->in_side.map.release();
    km->in_side.mask.release();
    km->in_side.ready = false;
  }
  km->wplans.clear();
  for (auto& sub : km->groups) {
    sub->out_side.plans.clear();
    sub->wplans.clear();
  }
  return SPCONV_OK;
}

SPCONV_API int spconv_kmap_export_perm(spconv_kmap* km, spconv_op op, const spconv_config* cfg, int split, int32_t* dst,
                            void* stream) {
  StreamScope scope((hipStream_t)stream);
  if (!km || !dst || (op != SPCONV_OP_FWD && op != SPCONV_OP_DGRAD)) return SPCONV_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  spconv_config c;
  SPC_TRY(resolve_config(cfg, SPCONV_F16, &c));
  if (!km->groups.empty()) {  // parts of plane 0, then of plane 1, ...
    if (c.n_split == 0 || split < 0 || split >= c.n_split * (int)km->groups.size()) return SPCONV_EINVAL;
    return spconv_kmap_export_perm(km->groups[split / c.n_split].get(), op, cfg, split % c.n_split, dst, stream);
  }
  if (c.n_split == 0 || split < 0 || split >= c.n_split) return SPCONV_EINVAL;
  OpSide os;
  SPC_TRY(side_for(km, op, st, &os));
  IgemmPlan* plan = nullptr;
  SPC_TRY(plan_get(km, *os.side, c.n_split, plan_tile(c, false), st, &plan));
  if (plan->rows == 0) return SPCONV_OK;
  SPC_HIP(hipMemcpyAsync(dst, plan->perm.as<int>() + (size_t)split * plan->rows_pad,
                         (size_t)plan->rows * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
  return SPCONV_OK;
}

SPCONV_API int spconv_kmap_mac_units(spconv_kmap* km, spconv_op op, const spconv_config* cfg, int64_t* executed,
                          int64_t* effective, void* stream) {
  StreamScope scope((hipStream_t)stream);
  if (!km || !executed || !effective || (op != SPCONV_OP_FWD && op != SPCONV_OP_DGRAD)) return SPCONV_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  spconv_config c;
  SPC_TRY(resolve_config(cfg, SPCONV_F16, &c));
  if (!km->groups.empty()) {
    *executed = *effective = 0;
    for (auto& sub : km->groups) {
      int64_t ex = 0, ef = 0;
      SPC_TRY(spconv_kmap_mac_units(sub.get(), op, cfg, &ex, &ef, stream));
      *executed += ex;
      *effective += ef;
    }
    return SPCONV_OK;
  }
  if (km->n_pairs < 0) SPC_TRY(kmap_count_pairs(km, st, nullptr));
  *effective = km->n_pairs;
  if (c.kernel == 3) {  // fetch-on-demand walks the pair lists: nothing but valid pairs is multiplied
    *executed = km->n_pairs;
    return SPCONV_OK;
  }
  OpSide os;
  SPC_TRY(side_for(km, op, st, &os));
  IgemmPlan* plan = nullptr;
  SPC_TRY(plan_get(km, *os.side, c.n_split, plan_tile(c, false), st, &plan));
  return plan_mac_units(km, *os.side, plan, 16, st, executed);
}

SPCONV_API void spconv_kmap_destroy(spconv_kmap* km) {
  if (!km) return;
  StreamScope scope(km->last_stream);  // its blocks go back to the pool of the stream that used them last
  delete km;
}

SPCONV_API int spconv_fwd(const void* feats, const void* weights, spconv_kmap* km, int C_in, int C_out, spconv_dtype dtype,
               const spconv_config* cfg, void* out, void* stream) {
  StreamScope scope((hipStream_t)stream);
  return run_igemm_op(SPCONV_OP_FWD, feats, weights, km, C_in, C_out, dtype, cfg, out, (hipStream_t)stream);
}

SPCONV_API int spconv_fwd_noalloc(const void* feats, const void* weights, spconv_kmap* km, int C_in, int C_out,
                                  spconv_dtype dtype, const spconv_config* cfg, void* out, void* stream) {
  return run_igemm_op(SPCONV_OP_FWD, feats, weights, km, C_in, C_out, dtype, cfg, out, (hipStream_t)stream, true);
}

SPCONV_API int spconv_dgrad(const void* dout, const void* weights, spconv_kmap* km, int C_in, int C_out, spconv_dtype dtype,
                 const spconv_config* cfg, void* din, void* stream) {
  StreamScope scope((hipStream_t)stream);
  return run_igemm_op(SPCONV_OP_DGRAD, dout, weights, km, C_in, C_out, dtype, cfg, din, (hipStream_t)stream);
}

SPCONV_API int spconv_wgrad(const void* feats, const void* dout, spconv_kmap* km, int C_in, int C_out, spconv_dtype dtype,
                 const spconv_config* cfg, float* dweights, void* stream) {
  StreamScope scope((hipStream_t)stream);
  if (!km || !dtype_ok(dtype) || !dweights) return SPCONV_EINVAL;
  SPC_TRY(check_channels(C_in, C_out, dtype));
  if ((km->n_out > 0 && km->n_in > 0) && (!feats || !dout)) return SPCONV_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  spconv_config c;
  SPC_TRY(resolve_config(cfg, dtype, &c));
  km->last_stream = st;
  if (!km->groups.empty()) {  // each plane fills its own 25 slices of dW
    for (size_t g = 0; g < km->groups.size(); ++g) {
      spconv_kmap* sub = km->groups[g].get();
      SPC_TRY(spconv_wgrad(feats, dout, sub, C_in, C_out, dtype, cfg, dweights + g * (size_t)sub->V * C_in * C_out, stream));
    }
    return SPCONV_OK;
  }
  if (km->n_pairs < 0 && !km->pending) SPC_TRY(kmap_count_pairs(km, st, nullptr));
  const int64_t target = c.wgrad_pairs > 0 ? c.wgrad_pairs : auto_wgrad_pairs(km, C_in, C_out);
  WgradPlan* wp = nullptr;
  SPC_TRY(wplan_get(km, target, st, &wp));
  return wgrad_run(km, *wp, feats, dout, C_in, C_out, dtype, dweights, st);
}

SPCONV_API int spconv_tune(spconv_kmap* km, int C_in, int C_out, spconv_dtype dtype, spconv_op op, int layers_sharing_kmap,
                spconv_config* best, float* best_us, void* stream) {
  StreamScope scope((hipStream_t)stream);
  if (!km || !best || !dtype_ok(dtype) || op < SPCONV_OP_FWD || op > SPCONV_OP_WGRAD || layers_sharing_kmap < 1)
    return SPCONV_EINVAL;
  if (!km->groups.empty()) return SPCONV_EINVAL;  // (K = 5 kmaps run the automatic or the caller's configuration)
  SPC_TRY(check_channels(C_in, C_out, dtype));
  hipStream_t st = (hipStream_t)stream;
  const size_t e = dtype == SPCONV_F32 ? 4 : 2;
  const int64_t n_in = std::max<int64_t>(km->n_in, 1), n_out = std::max<int64_t>(km->n_out, 1);
  DevBuf x, y, w, dw;
  SPC_TRY(x.alloc((size_t)n_in * C_in * e));
  SPC_TRY(y.alloc((size_t)n_out * C_out * e));
  SPC_TRY(w.alloc((size_t)km->V * C_in * C_out * e));
  SPC_TRY(dw.alloc((size_t)km->V * C_in * C_out * 4));
  SPC_HIP(hipMemsetAsync(x.p, 0, x.bytes, st));  // zeros are valid numbers in every dtype
  SPC_HIP(hipMemsetAsync(y.p, 0, y.bytes, st));
  SPC_HIP(hipMemsetAsync(w.p, 0, w.bytes, st));
  struct Events {  // destroyed on every way out
    hipEvent_t a = nullptr, b = nullptr;
    ~Events() {
      if (a) (void)hipEventDestroy(a);
      if (b) (void)hipEventDestroy(b);
    }
  } ev;
  SPC_HIP(hipEventCreate(&ev.a));
  SPC_HIP(hipEventCreate(&ev.b));
  const hipEvent_t e0 = ev.a, e1 = ev.b;

  std::vector<spconv_config> cands;
  if (op == SPCONV_OP_WGRAD) {
    if (km->n_pairs < 0) SPC_TRY(kmap_count_pairs(km, st, nullptr));
    const int64_t base = auto_wgrad_pairs(km, C_in, C_out);
    for (int64_t f : {1, 2, 4}) {
      spconv_config c{};
      c.wgrad_pairs = (int32_t)std::min<int64_t>(base * f / 2 + 512, 0x7FFFFFFF);
      cands.push_back(c);
    }
  } else {
    const int tiles[3] = {64, 128, 256};
    const int c_red = op == SPCONV_OP_DGRAD ? C_out : C_in, c_dst = op == SPCONV_OP_DGRAD ? C_in : C_out;
    if (fod_supported(km, op == SPCONV_OP_DGRAD, C_in, C_out, dtype))
      for (int tm : {64, 128}) {  // the fetch-on-demand dataflow (its mapping: the pair lists)
        if (dtype == SPCONV_F32 && tm != 64) continue;
        spconv_config c{};
        c.kernel = 3;
        c.tile_m = tm;
        cands.push_back(c);
      }
    for (int s = 0; s <= kMaxSplit && s <= km->V; ++s) {  // (a part needs at least one offset)
      for (int t = 0; t < (dtype == SPCONV_F32 ? 1 : 3); ++t) {
        spconv_config c{};
        c.n_split = s;
        c.tile_m = tiles[t];
        c.kernel = 2;
        cands.push_back(c);
      }
      if (dtype == SPCONV_F32) continue;
      for (int tn : {64, 32, 16}) {
        if (tn >= 2 * c_dst && tn > 16) continue;
        if (igemm_wave_pick_bn(km->V, s, c_red, c_dst, tn, nullptr) == 0) continue;
        spconv_config c{};
        c.n_split = s;
        c.kernel = 1;
        c.tile_n = tn;
        cands.push_back(c);
      }
    }
  }
  int status = SPCONV_OK;
  float best_t = 1e30f;
  auto run_once = [&](const spconv_config& c) -> int {
    switch (op) {
      case SPCONV_OP_FWD: return spconv_fwd(x.p, w.p, km, C_in, C_out, dtype, &c, y.p, st);
      case SPCONV_OP_DGRAD: return spconv_dgrad(y.p, w.p, km, C_in, C_out, dtype, &c, x.p, st);
      default: return spconv_wgrad(x.p, y.p, km, C_in, C_out, dtype, &c, dw.as<float>(), st);
    }
  };
  auto elapsed = [&](float* ms) {
    (void)hipEventRecord(e1, st);
    (void)hipEventSynchronize(e1);
    (void)hipEventElapsedTime(ms, e0, e1);
  };
  for (const auto& c : cands) {
    // mapping time: building the plan from scratch (best of two), timed apart from the kernel
    float t_map = 1e30f;
    for (int rep = 0; rep < 2 && status == SPCONV_OK; ++rep) {
      (void)spconv_kmap_drop_plans(km);
      (void)hipEventRecord(e0, st);
      if (op == SPCONV_OP_WGRAD) {
        WgradPlan* wp = nullptr;
        status = wplan_get(km, c.wgrad_pairs, st, &wp);
      } else {
        status = spconv_kmap_prepare(km, op, &c, st);
      }
      float ms = 0.f;
      elapsed(&ms);
      t_map = std::min(t_map, ms);
    }
    if (status != SPCONV_OK) break;
    // kernel time: warm, best of three groups of five
    status = run_once(c);
    if (status != SPCONV_OK) break;
    float t_k = 1e30f;
    for (int grp = 0; grp < 3; ++grp) {
      (void)hipEventRecord(e0, st);
      for (int r = 0; r < 5; ++r) (void)run_once(c);
      float ms = 0.f;
      elapsed(&ms);
      t_k = std::min(t_k, ms / 5.f);
    }
    const float t = t_k + t_map / (float)layers_sharing_kmap;
    if (t < best_t) {
      best_t = t;
      *best = c;
    }
  }
  if (status == SPCONV_OK && best_us) *best_us = best_t * 1000.f;
  return status;
}

// ---- group tuner (Section 4.2): the layers that share a kmap take one map structure --------
namespace {

struct GroupTimer {
  spconv_kmap* km;
  spconv_dtype dtype;
  hipStream_t st;
  DevBuf x, y, w, dw;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  ~GroupTimer() {
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  }
  float elapsed_ms() {
    float ms = 0.f;
    (void)hipEventRecord(e1, st);
    (void)hipEventSynchronize(e1);
    (void)hipEventElapsedTime(&ms, e0, e1);
    return ms;
  }
  int run(spconv_op op, int ci, int co, const spconv_config& c) {
    switch (op) {
      case SPCONV_OP_FWD: return spconv_fwd(x.p, w.p, km, ci, co, dtype, &c, y.p, st);
      case SPCONV_OP_DGRAD: return spconv_dgrad(y.p, w.p, km, ci, co, dtype, &c, x.p, st);
      default: return spconv_wgrad(x.p, y.p, km, ci, co, dtype, &c, dw.as<float>(), st);
    }
  }
  // warm kernel time in microseconds: best of two groups of four launches
  int kernel_us(spconv_op op, int ci, int co, const spconv_config& c, float* us) {
    SPC_TRY(run(op, ci, co, c));
    float best = 1e30f;
    for (int grp = 0; grp < 2; ++grp) {
      (void)hipEventRecord(e0, st);
      for (int r = 0; r < 4; ++r) SPC_TRY(run(op, ci, co, c));
      best = std::min(best, elapsed_ms() / 4.f);
    }
    *us = best * 1000.f;
    return SPCONV_OK;
  }
  // time to build the plan of c from scratch, in microseconds (best of two)
  int mapping_us(spconv_op op, const spconv_config& c, float* us) {
    float best = 1e30f;
    for (int rep = 0; rep < 2; ++rep) {
      SPC_TRY(spconv_kmap_drop_plans(km));
      (void)hipEventRecord(e0, st);
      if (op == SPCONV_OP_WGRAD) {
        WgradPlan* wp = nullptr;
        SPC_TRY(wplan_get(km, c.wgrad_pairs, st, &wp));
      } else {
        SPC_TRY(spconv_kmap_prepare(km, op, &c, st));
      }
      best = std::min(best, elapsed_ms());
    }
    *us = best * 1000.f;
    return SPCONV_OK;
  }
};

struct SplitChoice {                    // one op, one split count, every layer of the group
  std::vector<spconv_config> cfg;       // fastest kernel / tile per distinct layer shape
  float us = 1e30f;                     // sum over the layers + mapping of the plans they use
};

}  // namespace

SPCONV_API int spconv_tune_group(spconv_kmap* km, const spconv_layer_shape* layers, int n_layers, spconv_dtype dtype,
                                 int training, int bind_fwd_dgrad, spconv_config* fwd, spconv_config* dgrad,
                                 spconv_config* wgrad, float* group_us, void* stream) {
  StreamScope scope((hipStream_t)stream);
  if (!km || !layers || n_layers < 1 || !fwd || !dtype_ok(dtype)) return SPCONV_EINVAL;
  if (!km->groups.empty()) return SPCONV_EINVAL;
  if (training && (!dgrad || !wgrad)) return SPCONV_EINVAL;
  int max_ci = 0, max_co = 0;
  std::vector<std::pair<int, int>> shapes;  // distinct shapes
  std::vector<int> shape_of(n_layers), count;
  for (int i = 0; i < n_layers; ++i) {
    SPC_TRY(check_channels(layers[i].c_in, layers[i].c_out, dtype));
    max_ci = std::max(max_ci, layers[i].c_in);
    max_co = std::max(max_co, layers[i].c_out);
    const auto sh = std::make_pair(layers[i].c_in, layers[i].c_out);
    size_t j = 0;
    while (j < shapes.size() && shapes[j] != sh) ++j;
    if (j == shapes.size()) {
      shapes.push_back(sh);
      count.push_back(0);
    }
    shape_of[i] = (int)j;
    ++count[j];
  }
  GroupTimer t;
  t.km = km;
  t.dtype = dtype;
  t.st = (hipStream_t)stream;
  const size_t e = dtype == SPCONV_F32 ? 4 : 2;
  SPC_TRY(t.x.alloc((size_t)std::max<int64_t>(km->n_in, 1) * max_ci * e));
  SPC_TRY(t.y.alloc((size_t)std::max<int64_t>(km->n_out, 1) * max_co * e));
  SPC_TRY(t.w.alloc((size_t)km->V * max_ci * max_co * e));
  SPC_TRY(t.dw.alloc((size_t)km->V * max_ci * max_co * 4));
  SPC_HIP(hipMemsetAsync(t.x.p, 0, t.x.bytes, t.st));  // zeros are valid numbers in every dtype
  SPC_HIP(hipMemsetAsync(t.y.p, 0, t.y.bytes, t.st));
  SPC_HIP(hipMemsetAsync(t.w.p, 0, t.w.bytes, t.st));
  SPC_HIP(hipEventCreate(&t.e0));
  SPC_HIP(hipEventCreate(&t.e1));
  km->last_stream = t.st;

  const int max_split = std::min(kMaxSplit, km->V);
  // The map structures a group can take: implicit GEMM on an unsorted map or on 1..max_split sorted
  // splits (choices 0..max_split), or the fetch-on-demand dataflow on the pair lists (the last choice).
  const int n_choices = max_split + 2, fod_choice = max_split + 1;
  // fwd / dgrad: for every map structure, the fastest kernel and tile of each layer shape, plus the
  // mapping time of every plan (structure, tile height) those choices need, paid once per group
  auto tune_op = [&](spconv_op op, std::vector<SplitChoice>* out) -> int {
    out->assign(n_choices, SplitChoice{});
    for (int s = 0; s < n_choices; ++s) {
      const bool fod = s == fod_choice;
      if (fod) {
        bool ok = true;
        for (const auto& sh : shapes) ok = ok && fod_supported(km, op == SPCONV_OP_DGRAD, sh.first, sh.second, dtype);
        if (!ok) continue;  // stays at its initial, never-chosen time
      }
      SplitChoice& ch = (*out)[s];
      ch.cfg.resize(shapes.size());
      float total = 0.f;
      std::vector<int> plan_keys;  // tile heights whose plans are used (16 = kernel 1)
      for (size_t j = 0; j < shapes.size(); ++j) {
        const int ci = shapes[j].first, co = shapes[j].second;
        const int c_red = op == SPCONV_OP_DGRAD ? co : ci, c_dst = op == SPCONV_OP_DGRAD ? ci : co;
        std::vector<spconv_config> cands;
        for (int tm : {64, 128, 256}) {
          if (fod ? (tm == 256 || (dtype == SPCONV_F32 && tm != 64)) : (dtype == SPCONV_F32 && tm != 64)) continue;
          spconv_config c{};
          c.n_split = fod ? 0 : s;
          c.tile_m = tm;
          c.kernel = fod ? 3 : 2;
          cands.push_back(c);
        }
        if (dtype != SPCONV_F32 && !fod)
          for (int tn : {64, 32, 16}) {
            if (tn >= 2 * c_dst && tn > 16) continue;
            if (igemm_wave_pick_bn(km->V, s, c_red, c_dst, tn, nullptr) == 0) continue;
            spconv_config c{};
            c.n_split = s;
            c.kernel = 1;
            c.tile_n = tn;
            cands.push_back(c);
          }
        float best = 1e30f;
        for (const auto& c : cands) {
          float us = 0.f;
          SPC_TRY(t.kernel_us(op, ci, co, c, &us));
          if (us < best) {
            best = us;
            ch.cfg[j] = c;
          }
        }
        total += best * (float)count[j];
        const int key = ch.cfg[j].kernel == 1 ? 16 : ch.cfg[j].tile_m;
        if (std::find(plan_keys.begin(), plan_keys.end(), key) == plan_keys.end()) plan_keys.push_back(key);
      }
      for (int key : plan_keys) {
        spconv_config c{};
        c.n_split = fod ? 0 : s;
        c.kernel = fod ? 3 : (key == 16 ? 1 : 2);
        c.tile_m = key == 16 ? 0 : key;
        float us = 0.f;
        SPC_TRY(t.mapping_us(op, c, &us));
        total += us;
      }
      ch.us = total;
    }
    return SPCONV_OK;
  };

  std::vector<SplitChoice> f, d;
  SPC_TRY(tune_op(SPCONV_OP_FWD, &f));
  int sf = 0, sd = 0;
  float total = 0.f;
  if (!training) {
    for (int s = 1; s < n_choices; ++s)
      if (f[s].us < f[sf].us) sf = s;
    total = f[sf].us;
  } else {
    SPC_TRY(tune_op(SPCONV_OP_DGRAD, &d));
    if (bind_fwd_dgrad) {
      for (int s = 1; s < n_choices; ++s)
        if (f[s].us + d[s].us < f[sf].us + d[sf].us) sf = s;
      sd = sf;
    } else {
      for (int s = 1; s < n_choices; ++s) {
        if (f[s].us < f[sf].us) sf = s;
        if (d[s].us < d[sd].us) sd = s;
      }
    }
    total = f[sf].us + d[sd].us;
  }
  for (int i = 0; i < n_layers; ++i) {
    fwd[i] = f[sf].cfg[shape_of[i]];
    if (training) dgrad[i] = d[sd].cfg[shape_of[i]];
  }
  if (training) {
    // wgrad walks the weight-stationary pair lists, whose only parameter is the pairs per work
    // item: one value for the group, so that the lists are built once
    if (km->n_pairs < 0) SPC_TRY(kmap_count_pairs(km, t.st, nullptr));
    float best = 1e30f;
    int32_t best_pairs = 0;
    for (int32_t pairs : {768, 1536, 3072, 6144}) {
      spconv_config c{};
      c.wgrad_pairs = pairs;
      float sum = 0.f, us = 0.f;
      SPC_TRY(t.mapping_us(SPCONV_OP_WGRAD, c, &us));
      sum += us;
      for (size_t j = 0; j < shapes.size(); ++j) {
        SPC_TRY(t.kernel_us(SPCONV_OP_WGRAD, shapes[j].first, shapes[j].second, c, &us));
        sum += us * (float)count[j];
      }
      if (sum < best) {
        best = sum;
        best_pairs = pairs;
      }
    }
    for (int i = 0; i < n_layers; ++i) {
      wgrad[i] = spconv_config{};
      wgrad[i].wgrad_pairs = best_pairs;
    }
    total += best;
  }
  if (group_us) *group_us = total;
  return SPCONV_OK;
}

SPCONV_API int spconv_describe_launch(int K, int64_t rows, int64_t rows_src, int C_red, int C_cols, spconv_dtype dtype,
                                      const spconv_config* cfg, int dgrad, spconv_launch_info* out) {
  if (!out || !dtype_ok(dtype) || (K != 1 && K != 2 && K != 3 && K != 5) || rows < 0 || rows_src < 0 || (dgrad != 0 && dgrad != 1))
    return SPCONV_EINVAL;
  std::memset(out, 0, sizeof(*out));
  SPC_TRY(check_channels(C_red, C_cols, dtype));
  spconv_config c;
  SPC_TRY(resolve_config(cfg, dtype, &c));
  if (c.kernel == 3) return SPCONV_EINVAL;  // (fetch-on-demand launches are sized by the pair lists, not by these shapes)
  const int V = K == 5 ? 25 : K * K * K;  // K = 5 launches once per 25-offset plane: the launch of one plane
  if (c.n_split > V) return SPCONV_EINVAL;
  if (rows == 0) return SPCONV_OK;  // nothing is launched
  KernelChoice kc;
  SPC_TRY(choose_kernel(V, rows, C_red, C_cols, dtype, cfg && cfg->tile_m != 0, c, &kc));
  PlanShape ps;
  SPC_TRY(plan_shape(V, rows, c.n_split, kc.tile_m, &ps));
  out->kernel = kc.wave ? 1 : 2;
  out->tile_m = kc.tile_m;
  out->parts = ps.parts;
  out->rows_pad = ps.rows_pad;
  out->n_tiles = ps.n_tiles;
  for (int i = 0; i < ps.parts; ++i) {
    out->lo[i] = ps.lo[i];
    out->width[i] = ps.width[i];
    out->map_elems[i] = (int64_t)ps.rows_pad * (c.n_split == 0 ? V : ps.width[i]);
  }
  out->sorted = c.n_split > 0;
  if (kc.wave) {
    WaveShape w;
    SPC_TRY(igemm_wave_shape(V, c.n_split, rows, rows_src, C_red, C_cols, kc.tile_n, &w));
    out->tile_n = w.bn;
    out->k_steps = w.ks;
    out->waves = w.waves;
    out->threads = w.threads;
    out->lds_bytes = (int64_t)w.lds_bytes;
    out->slab_bytes = w.slab_bytes;
    out->slab_map_bytes = w.map_bytes;
    for (int i = 0; i < 3; ++i) out->grid[i] = (int32_t)w.grid[i];
    out->xcd_ranges = ((c.flags & SPCONV_FLAG_SLABS) || rows >= (1 << 20)) && c.n_split > 0 && w.grid[0] % 8 == 0;
  } else {
    TileShape t;
    SPC_TRY(igemm_tile_shape(V, c.n_split, rows, rows_src, C_red, C_cols, kc.tile_m, kc.tile_n, dtype == SPCONV_F32,
                             dgrad != 0, &t));
    out->tile_m = t.bm;
    out->tile_n = t.bn;
    out->k_steps = t.kc;
    out->waves = t.nw;
    out->threads = t.threads;
    out->lds_bytes = (int64_t)t.lds_bytes;
    for (int i = 0; i < 3; ++i) out->grid[i] = (int32_t)t.grid[i];
  }
  return SPCONV_OK;
}

SPCONV_API int spconv_set_allocator(void* (*alloc)(size_t, void*, void*), void (*free_)(void*, void*, void*), void* user) {
  if ((alloc == nullptr) != (free_ == nullptr)) return SPCONV_EINVAL;
  std::lock_guard<std::mutex> lk(g_mem_mu);
  g_user_alloc = alloc;
  g_user_free = free_;
  g_user_ctx = user;
  return SPCONV_OK;
}

SPCONV_API const char* spconv_strerror(int status) {
  switch (status) {
    case SPCONV_OK: return "ok";
    case SPCONV_EINVAL: return "invalid argument";
    case SPCONV_ERANGE: return "coordinate outside the packable range";
    case SPCONV_EDUP: return "duplicate input coordinate";
    case SPCONV_ENOMEM: return "out of memory";
    case SPCONV_ESHAPE: return "channel or row counts do not fit";
    case SPCONV_EHIP: return "HIP call failed";
    case SPCONV_ENOPLAN: return "no prepared plan for this configuration (call spconv_kmap_prepare first)";
    case SPCONV_ELIMIT: return "partial sums exceed the fixed scratch array of the allocation-free entry point";
  }
  return "unknown status";
}

SPCONV_API const char* spconv_last_hip_error(void) { return g_hip_err; }

SPCONV_API int spconv_version(void) { return 100; }

}  // extern "C"
