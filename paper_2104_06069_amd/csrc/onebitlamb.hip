// libonebitlamb: host side of the C ABI (include/onebitlamb.h) -- context, tile tables, argument
// validation and kernel launches.  The kernels live in ob_kernels.h.
//
// Build flags that the arithmetic depends on: -ffp-contract=off (one rounding per operation) and
// hipcc's default correctly rounded fp32 divide/sqrt; never -ffast-math.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <mutex>
#include <new>
#include <string>
#include <type_traits>
#include <vector>

#include "ob_kernels.h"
#include "onebitlamb.h"

using namespace obk;

namespace {

// 128-bit accesses per thread per array in the plain N-sized kernels: tiles of 1024 elements measured
// ~7 % faster than 4096 on MI355X (ratio and update kernels at 6.4-6.5 TB/s instead of 6.0).  The
// kernels with a per-layer barrier share the segment arrays of this tiling, so it is fixed at 1.
constexpr int U_MAIN = 1;
constexpr int U_SRV = 1;    // ... in the kernels over the single server chunk
// ... in the single-pass server kernel (zb stays in registers): the smallest of these whose tiles of
// the served chunk all fit on the device at once (more, smaller workgroups hide the W dependent
// additions per element better)
constexpr int U_SRV_RES[] = {1, 2, 4};   // (8 would need registers that cost more slots than it saves tiles)
#ifndef OB_U_RES
#define OB_U_RES 16
#endif
constexpr int U_RES = OB_U_RES;   // ... in the single-pass worker compression (z stays in registers)
// workgroups per CU the single-pass compression kernel is built for: 5 lets the instantiation with
// momentum scaling spill its layer cursor (touched only in tiles that meet a layer boundary) instead
// of dropping to 4 (measured 3 % faster; without momentum scaling the kernel fits 5 anyway)
#ifndef OB_RES_MINW
#define OB_RES_MINW 5
#endif
#ifndef OB_G_RES
#define OB_G_RES 2
#endif
constexpr int G_RES = OB_G_RES;    // the single-pass kernel issues its loads G_RES accesses at a time
constexpr int TILE_MAIN = SPAN * U_MAIN;
constexpr int TILE_SRV = SPAN * U_SRV;
constexpr int TILE_RES = SPAN * U_RES;
#ifndef OB_U_LB
#define OB_U_LB 8
#endif
constexpr int U_LB = OB_U_LB;  // ... in the fused ratio+update kernel (v_frozen and signs stay in registers)
constexpr int TILE_LB = SPAN * U_LB;
#ifndef OB_U_WU
#define OB_U_WU 8
#endif
// 1: the ratio+update kernel streams its tile and fetches x after the layer's coefficient is known
// (k_ratios_apply_stream; half the registers per element across the barrier), OB_G_LB spans at a time
#ifndef OB_LB_STREAM
#define OB_LB_STREAM 0
#endif
#ifndef OB_G_LB
#define OB_G_LB 2
#endif
// safety margin, in tiles, under 80 % of the device's workgroup slots for the largest layer a
// barrier kernel takes
#ifndef OB_SPLIT_MARGIN
#define OB_SPLIT_MARGIN 8
#endif
constexpr int U_WU = OB_U_WU;  // ... in the single-pass warmup kernel (u and x stay in registers)
constexpr int TILE_WU = SPAN * U_WU;
#ifndef OB_BIG_MIN_TILES
#define OB_BIG_MIN_TILES 64   // a layer outside the barrier kernel with at least that many whole 8192-element tiles
#endif
#ifndef OB_G_WU
#define OB_G_WU 2
#endif
constexpr int G_WU = OB_G_WU;        // the single-pass warmup kernel issues its loads G_WU accesses at a time

enum KernelId {
  KID_MOMENTUM_Z = 0,
  KID_COMPRESS_RESIDENT,
  KID_CHUNK_SCALE,
  KID_SIGN_PACK,
  KID_COMPRESS_DEFERRED,
  KID_SERVER_AVG,
  KID_SERVER_SCALE,
  KID_SERVER_PACK,
  KID_SERVER_RESIDENT,
  KID_RATIOS_PASS,
  KID_RATIOS_FINALIZE,
  KID_APPLY,
  KID_RATIOS_APPLY_RESIDENT,
  KID_RATIOS_APPLY_HIST,
  KID_VARIANCE_DENSE,
  KID_VARIANCE_TERMS,
  KID_RATIOS_BIG_HIST,
  KID_MOMENTUM_DENSE,
  KID_ERROR_DENSE,
  KID_MOMENTUM_SCALE,
  KID_WARMUP_MOMENTS,
  KID_WARMUP_COEFF,
  KID_WARMUP_APPLY,
  KID_WARMUP_RESIDENT,
  KID_FILL,
  KID_COPY,
  KID_COUNT
};
const char* const kKernelNames[KID_COUNT] = {
    "momentum_z_sumsq", "compress_resident", "chunk_scale",     "sign_pack_error", "compress_deferred", "server_unpack_avg",
    "server_scale",     "server_sign_pack", "server_resident", "ratios_pass",     "ratios_finalize",
    "decompress_apply", "ratios_apply_resident", "ratios_apply_hist", "variance_dense", "variance_terms", "ratios_big_hist", "momentum_dense", "error_dense", "momentum_scale", "warmup_moments",   "warmup_coeff",    "warmup_apply",
    "warmup_resident",  "fill",            "copy"};

struct ProfRec {
  int kid;
  hipEvent_t e0, e1;
};

// Split of the work between a kernel with a per-layer barrier and the plain kernels.  The barrier
// kernel takes "listed" tiles: the TILE_LB tiles that lie wholly inside one layer, for every layer
// whose such tiles all fit on the device at once (80 % of that kernel's workgroup slots).  The
// plain kernels take every other 1024-element tile that holds parameters ("rest" tiles: layers
// that are too large, the spans where layers meet, small tensors), and finish the layers that
// have no listed tile.  (Listing only the last tiles of a layer that is too large was measured:
// a run of layers that each fill the device to the limit stalls at every barrier, and the kernel
// fell from 5.8 to 3.5 TB/s on a GPT-1.3B-shaped list.)
struct LayerSplit {
  bool on = false;          // at least one tile is listed
  int n_fused_tiles = 0;    // listed TILE_LB tiles
  int n_rest_tiles = 0;     // TILE_MAIN tiles outside them that hold parameters
  int64_t n_layers = 0;     // layers with listed tiles
  int64_t n_params = 0;     // parameters in listed tiles
  int* d_fused_tiles = nullptr;
  int* d_n_listed = nullptr;               // [L] listed tiles of each layer
  int* d_list_begin = nullptr;             // [L] index in d_fused_tiles of the layer's first listed tile
  int* d_seg_first = nullptr;              // [L] first / one past the last segment (TILE_MAIN tiling) that the
  int* d_seg_end = nullptr;                //     layer's listed tiles cover
  float* d_listed_max = nullptr;           // [n_fused_tiles] partial results of the listed tiles
  double* d_listed_sums = nullptr;         // [2*n_fused_tiles]
  int tile = 0;             // elements per listed tile
  int tpc = 0;              // such tiles per chunk
  int* d_rest_tiles = nullptr;
  // The layers that are too large for the barrier kernel: their TILE_LB tiles ("big" tiles) take the
  // ratio pass with the variance in deferred form (ob_lamb_ratios_apply_hist only)
  bool big_on = false;                     // there are such tiles (and no wait has expired)
  int n_big_tiles = 0;
  int64_t n_big_params = 0;
  int* d_big_tiles = nullptr;
  int n_rest_ratio_tiles = 0;              // TILE_MAIN tiles outside the listed and the big tiles
  int* d_rest_ratio_tiles = nullptr;
  int n_cov_tiles = 0;                     // TILE_MAIN tiles inside the listed or the big tiles
  int* d_cov_tiles = nullptr;
  unsigned char* d_has_listed = nullptr;   // [L] 1 for layers that the barrier kernel finishes
  unsigned long long* d_counter = nullptr; // [L * CTR_STRIDE] (generation << 32) | arrivals
  unsigned long long* d_flag = nullptr;    // [L] (generation << 32) | payload
};

}  // namespace

struct ob_lamb_ctx {
  // configuration
  int64_t L = 0, N = 0, n_pad = 0, n_c = 0;
  int32_t W = 1, server_chunk = 0;
  float beta1, beta2, beta3, eta, c_min, c_max, r_min, r_max, r_thr, wd;
  float omb1, omb2, omb3, one_m_thr, one_p_thr, invW;
  // tiling
  int tpc = 0;        // TILE_MAIN tiles per chunk
  int n_tiles = 0;    // W * tpc
  int tpc_srv = 0;    // TILE_SRV tiles of the server chunk
  int n_segs = 0;     // (tile, layer) segments
  // device memory
  int device = -1;
  int64_t* d_off = nullptr;       // [L+2]
  int* d_first_layer = nullptr;   // [n_tiles]
  int* d_tile_seg0 = nullptr;     // [n_tiles+1]
  int* d_seg_layer = nullptr;     // [n_segs]
  int* d_layer_seg0 = nullptr;    // [L+1]
  double* d_partials = nullptr;   // [n_tiles]
  double* d_partials_srv = nullptr;  // [tpc_srv]
  double* d_seg_sums = nullptr;   // [2*n_segs]
  double* d_sigma = nullptr;      // [L] per-layer RMS (momentum-scale generation)
  float* d_seg_max = nullptr;     // [n_segs] per-segment max(v_frozen/v_fresh)
  // (chunk, layer) pairs and the per-step values of the variance in deferred form (VTerms)
  int n_pairs = 0;
  int* d_pair_base = nullptr;     // [W+1]
  int* d_pair_lfirst = nullptr;   // [W]
  int* d_pair_c = nullptr;        // [n_pairs]
  int* d_pair_l = nullptr;        // [n_pairs]
  float* d_vterms = nullptr;      // [(VF_MAX_OLD+1) * n_pairs * 2]
  // single-pass worker compression (k_compress_resident)
  bool resident = false;          // selected at create when the device can hold 2 chunks of tiles
  int tpc_res = 0, n_tiles_res = 0;
  int* d_first_layer_res = nullptr;        // [n_tiles_res]
  double* d_partials_res = nullptr;        // [n_tiles_res]
  unsigned long long* d_counter = nullptr; // [W * CTR_STRIDE] (generation << 32) | arrivals
  unsigned long long* d_flag = nullptr;    // [W] (generation << 32) | scale bits
  unsigned int* d_errflag = nullptr;       // [1] raised when a bounded wait expired
  // single-pass server kernel (k_server_resident): selected at create when all of its workgroups
  // fit on the device at once
  int u_srv_res = 0;                           // its tile size in 1024-element spans; 0: not used
  int tpc_srv_res = 0;                         // such tiles of the server chunk
  double* d_partials_srv_res = nullptr;        // [tpc_srv_res]
  unsigned long long* d_counter_srv = nullptr; // [CTR_STRIDE]
  unsigned long long* d_flag_srv = nullptr;    // [1]
  int spin_limit = OB_SPIN_LIMIT_DEFAULT;
  // kernels with a per-layer barrier (k_ratios_apply_resident, k_warmup_resident): their common
  // tiling (TILE_LB; the segment arrays are those of the TILE_MAIN tiling) and, for each, the split
  // of the work between it and the plain kernels
  LayerSplit sp_apply;                     // ob_lamb_ratios_apply
  LayerSplit sp_warm;                      // ob_lamb_warmup_step
  size_t device_bytes = 0;                 // device memory this context holds (tables + workspace)
  // diagnostics
  bool profile = false;
  std::vector<ProfRec> prof;
  std::string hip_err;
};

namespace {

bool hip_ok(ob_lamb_ctx* ctx, hipError_t e, const char* what) {
  if (e == hipSuccess) return true;
  if (ctx) ctx->hip_err = std::string(what) + ": " + hipGetErrorString(e);
  return false;
}

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

struct Launch {
  ob_lamb_ctx* ctx;
  hipStream_t stream;
  bool ok = true;
  Launch(ob_lamb_ctx* c, void* s) : ctx(c), stream(reinterpret_cast<hipStream_t>(s)) {}
  // A timing record for the coming launch (profile mode).  record_start: also record its first
  // event on the stream now (device copies); kernels hand both events to the launch instead, which
  // stamps them with the kernel's own start and end on the device.
  bool begin(int kid, bool record_start) {
    if (!ctx->profile || !ok) return false;
    ProfRec r;
    r.kid = kid;
    ok = hip_ok(ctx, hipEventCreate(&r.e0), "hipEventCreate") &&
         hip_ok(ctx, hipEventCreate(&r.e1), "hipEventCreate") &&
         (!record_start || hip_ok(ctx, hipEventRecord(r.e0, stream), "hipEventRecord"));
    if (ok) ctx->prof.push_back(r);
    return ok;
  }
  void end(const char* name, bool record_stop) {
    if (!ok) return;
    ok = hip_ok(ctx, hipGetLastError(), name);
    if (ok && ctx->profile && record_stop)
      ok = hip_ok(ctx, hipEventRecord(ctx->prof.back().e1, stream), "hipEventRecord");
  }
};

#define OB_LAUNCH_B(la, kid, kernel, grid, block, ...)                            \
  do {                                                                            \
    if ((la).ok && (grid) > 0) {                                                  \
      if ((la).begin(kid, false))                                                 \
        hipExtLaunchKernelGGL(kernel, dim3((unsigned)(grid)), dim3(block), 0, (la).stream, \
                              (la).ctx->prof.back().e0, (la).ctx->prof.back().e1, 0, __VA_ARGS__); \
      else if ((la).ok)                                                           \
        hipLaunchKernelGGL(kernel, dim3((unsigned)(grid)), dim3(block), 0, (la).stream, __VA_ARGS__); \
      (la).end(kKernelNames[kid], false);                                         \
    }                                                                             \
  } while (0)
#define OB_LAUNCH(la, kid, kernel, grid, ...) OB_LAUNCH_B(la, kid, kernel, grid, BLOCK, __VA_ARGS__)

template <class T>
bool upload(ob_lamb_ctx* ctx, T** dst, const std::vector<T>& src) {
  const size_t bytes = src.size() * sizeof(T);
  if (!hip_ok(ctx, hipMalloc(reinterpret_cast<void**>(dst), bytes ? bytes : sizeof(T)), "hipMalloc")) return false;
  ctx->device_bytes += bytes ? bytes : sizeof(T);
  if (bytes && !hip_ok(ctx, hipMemcpy(*dst, src.data(), bytes, hipMemcpyHostToDevice), "hipMemcpy")) return false;
  return true;
}

template <class T>
bool alloc_zero(ob_lamb_ctx* ctx, T** dst, size_t count) {
  const size_t bytes = (count ? count : 1) * sizeof(T);
  if (!hip_ok(ctx, hipMalloc(reinterpret_cast<void**>(dst), bytes), "hipMalloc")) return false;
  ctx->device_bytes += bytes;
  return hip_ok(ctx, hipMemset(*dst, 0, bytes), "hipMemset");
}

ob_status check_common(const ob_lamb_ctx* ctx, const ob_lamb_state* st) {
  if (!ctx || !st) return OB_ERR_NULL;
  // the context's tables live on the device it was created on
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != ctx->device) return OB_ERR_ARG;
  return OB_OK;
}

#define REQUIRE_PTR(p)                    \
  do {                                    \
    if ((p) == nullptr) return OB_ERR_NULL; \
    if (misaligned(p)) return OB_ERR_ALIGN; \
  } while (0)

// ---- small helpers for the entry points -------------------------------------------------------

LayerTab layer_tab(const ob_lamb_ctx* ctx, const ob_lamb_state* st, const int* first_layer) {
  LayerTab lt;
  lt.mom_scale = st->mom_scale;
  lt.off = ctx->d_off;
  lt.first_layer = first_layer;
  lt.L = (int)ctx->L;
  return lt;
}

// Calls f(std::bool_constant<a>, std::bool_constant<b>) so that kernels can take a and b as
// template arguments.
template <class F>
void dispatch2(bool a, bool b, F f) {
  if (a) {
    if (b) f(std::true_type{}, std::true_type{});
    else f(std::true_type{}, std::false_type{});
  } else {
    if (b) f(std::false_type{}, std::true_type{});
    else f(std::false_type{}, std::false_type{});
  }
}

// Calls f(std::bool_constant<a>).
template <class F>
void dispatch1(bool a, F f) {
  if (a) f(std::true_type{});
  else f(std::false_type{});
}

// Gradient argument of the _lp entry points -> kernel argument; *lp: 16-bit source.
ob_status grad_source(const void* grad, int dtype, float scale, GradSrc* gs, bool* lp) {
  if (!grad) return OB_ERR_NULL;
  if (misaligned(grad)) return OB_ERR_ALIGN;
  if (dtype != OB_F32 && dtype != OB_F16 && dtype != OB_BF16) return OB_ERR_ARG;
  if (dtype == OB_F32 && scale != 1.0f) return OB_ERR_ARG;
  if (!std::isfinite(scale)) return OB_ERR_ARG;
  gs->p = grad;
  gs->scale = scale;
  gs->bf16 = (dtype == OB_BF16) ? 1 : 0;
  *lp = (dtype != OB_F32);
  return OB_OK;
}

// 16-bit parameter copy of the _lp entry points (NULL: none).
struct XLp {
  void* p = nullptr;
  int bf16 = 0;
};
ob_status x_lp_target(void* x_lp, int dtype, XLp* out) {
  out->p = nullptr;
  out->bf16 = 0;
  if (!x_lp) return OB_OK;
  if (dtype != OB_F16 && dtype != OB_BF16) return OB_ERR_ARG;
  if (misaligned(x_lp)) return OB_ERR_ALIGN;
  out->p = x_lp;
  out->bf16 = (dtype == OB_BF16) ? 1 : 0;
  return OB_OK;
}

// The momentum source of a call: dense st->m if given, else the 1-bit form.
ob_status momentum_source(const ob_lamb_state* st, bool* packed, PackedMom* pm) {
  pm->bits = nullptr;
  pm->scales = nullptr;
  if (st->m) {
    if (misaligned(st->m)) return OB_ERR_ALIGN;
    *packed = false;
    return OB_OK;
  }
  if (!st->m_packed || !st->m_scales) return OB_ERR_NULL;
  if (misaligned(st->m_packed)) return OB_ERR_ALIGN;
  *packed = true;
  pm->bits = st->m_packed;
  pm->scales = st->m_scales;
  return OB_OK;
}

// Tables of one tiling of the padded buffer (tiles of `tile` elements inside each chunk): the layer
// of each tile's first element (L = padding), the (tile, layer) segments in position order and
// their grouping by layer.
struct Tiling {
  int64_t tpc = 0, n_tiles = 0;
  std::vector<int> first, tile_seg0, seg_layer, layer_seg0;
};

bool build_tiling(int64_t tile, int64_t n_c, int64_t W, int64_t L, const std::vector<int64_t>& h_off,
                  Tiling* out) {
  out->tpc = (n_c + tile - 1) / tile;
  out->n_tiles = out->tpc * W;
  if (out->n_tiles > 0x7fffffff) return false;
  out->first.resize((size_t)out->n_tiles);
  out->tile_seg0.resize((size_t)out->n_tiles + 1);
  out->seg_layer.clear();
  out->layer_seg0.assign((size_t)L + 1, 0);
  for (int64_t t = 0; t < out->n_tiles; ++t) {
    const int64_t c = t / out->tpc, b = t % out->tpc;
    const int64_t tile0 = c * n_c + b * tile;
    const int64_t tile1 = std::min(tile0 + tile, (c + 1) * n_c);
    // first layer: the non-empty layer that holds tile0 (binary search on the offsets)
    int64_t lo = 0, hi = L + 1;  // h_off[lo] <= tile0 < h_off[hi]
    while (hi - lo > 1) {
      const int64_t mid = (lo + hi) / 2;
      if (h_off[(size_t)mid] <= tile0) lo = mid; else hi = mid;
    }
    out->first[(size_t)t] = (int)lo;  // lo == L when tile0 >= N
    out->tile_seg0[(size_t)t] = (int)out->seg_layer.size();
    for (int64_t l = lo; l < L && h_off[(size_t)l] < tile1; ++l) {
      const int64_t a = std::max(h_off[(size_t)l], tile0), e = std::min(h_off[(size_t)l + 1], tile1);
      if (e > a) out->seg_layer.push_back((int)l);
    }
  }
  out->tile_seg0[(size_t)out->n_tiles] = (int)out->seg_layer.size();
  std::vector<int> count((size_t)L, 0);  // segments are ordered by position, hence grouped by layer
  for (int l : out->seg_layer) ++count[(size_t)l];
  for (int64_t l = 0; l < L; ++l)
    out->layer_seg0[(size_t)l + 1] = out->layer_seg0[(size_t)l] + count[(size_t)l];
  return true;
}

// The host side of one LayerSplit: which tiles the barrier kernel takes and what is left.
struct SplitPlan {
  std::vector<unsigned char> has_listed;   // [L] 1 for layers that the barrier kernel finishes
  std::vector<int> fused_tiles, rest_tiles, n_listed, list_begin, seg_first, seg_end;
  std::vector<unsigned char> covered;      // [TILE_MAIN tiles] 1 inside a listed tile
  std::vector<int> big_tiles, rest_ratio_tiles;
  std::vector<unsigned char> covered_big;  // [TILE_MAIN tiles] 1 inside a big tile
  int64_t n_layers = 0, n_params = 0, n_big_params = 0;
};

// tl / tm: the barrier kernel's tiling (tiles of tile_lb elements) and the TILE_MAIN tiling;
// max_tiles: the largest number of tiles of one layer the barrier kernel may hold (0: it is not
// used).  No HIP call.
void plan_split(const Tiling& tl, int64_t tile_lb, const Tiling& tm, const std::vector<int64_t>& h_off,
                int64_t n_c, int64_t L, int64_t max_tiles, SplitPlan* pl) {
  pl->has_listed.assign((size_t)L, 0);
  pl->n_listed.assign((size_t)L, 0);
  pl->list_begin.assign((size_t)L, 0);
  pl->seg_first.assign((size_t)L, 0);
  pl->seg_end.assign((size_t)L, 0);
  pl->covered.assign((size_t)tm.n_tiles, 0);
  auto tile_range = [&](int64_t t, int64_t* tile0, int64_t* tile1) {
    const int64_t c = t / tl.tpc, b = t % tl.tpc;
    *tile0 = c * n_c + b * tile_lb;
    *tile1 = std::min(*tile0 + tile_lb, (c + 1) * n_c);
  };
  // tiles inside one layer, per layer in position order
  std::vector<std::vector<int>> inside((size_t)L);
  for (int64_t t = 0; t < tl.n_tiles; ++t) {
    int64_t tile0, tile1;
    tile_range(t, &tile0, &tile1);
    const int l = tl.first[(size_t)t];
    if (l < L && tile1 <= h_off[(size_t)l + 1]) inside[(size_t)l].push_back((int)t);
  }
  for (int64_t l = 0; l < L; ++l) {
    const std::vector<int>& in = inside[(size_t)l];
    const size_t n = in.size();
    if (n == 0 || n > (size_t)max_tiles) continue;   // (max_tiles = 0: no layer is listed)
    pl->has_listed[(size_t)l] = 1;
    pl->n_listed[(size_t)l] = (int)n;
    pl->list_begin[(size_t)l] = (int)pl->fused_tiles.size();
    pl->n_layers += 1;
    for (size_t j = 0; j < n; ++j) {
      const int64_t t = in[j];
      int64_t tile0, tile1;
      tile_range(t, &tile0, &tile1);
      pl->fused_tiles.push_back((int)t);
      pl->n_params += tile1 - tile0;
      const int64_t c = t / tl.tpc, b = t % tl.tpc;
      const int64_t span0 = c * tm.tpc + b * (tile_lb / TILE_MAIN);
      const int64_t nspan = (tile1 - tile0 + TILE_MAIN - 1) / TILE_MAIN;
      for (int64_t j2 = 0; j2 < nspan; ++j2) pl->covered[(size_t)(span0 + j2)] = 1;
      // each of these spans lies inside the layer: one segment each, consecutive
      if (j == 0) pl->seg_first[(size_t)l] = tm.tile_seg0[(size_t)span0];
      pl->seg_end[(size_t)l] = tm.tile_seg0[(size_t)(span0 + nspan)];
    }
  }
  // big tiles: the whole tiles of the layers that hold many of them but are not listed
  pl->covered_big.assign((size_t)tm.n_tiles, 0);
  for (int64_t l = 0; l < L; ++l) {   // (also when no layer is listed: the pass needs no barrier)
    const std::vector<int>& in = inside[(size_t)l];
    if (pl->has_listed[(size_t)l] || in.size() < (size_t)OB_BIG_MIN_TILES) continue;
    for (int t : in) {
      int64_t tile0, tile1;
      tile_range(t, &tile0, &tile1);
      pl->big_tiles.push_back(t);
      pl->n_big_params += tile1 - tile0;
      const int64_t c = t / tl.tpc, b = t % tl.tpc;
      const int64_t span0 = c * tm.tpc + b * (tile_lb / TILE_MAIN);
      const int64_t nspan = (tile1 - tile0 + TILE_MAIN - 1) / TILE_MAIN;
      for (int64_t j2 = 0; j2 < nspan; ++j2) pl->covered_big[(size_t)(span0 + j2)] = 1;
    }
  }
  for (int64_t t = 0; t < tm.n_tiles; ++t)
    if (!pl->covered[(size_t)t] && tm.tile_seg0[(size_t)t + 1] > tm.tile_seg0[(size_t)t]) {
      pl->rest_tiles.push_back((int)t);
      if (!pl->covered_big[(size_t)t]) pl->rest_ratio_tiles.push_back((int)t);
    }
}

// Plans and uploads one LayerSplit.
bool build_split(ob_lamb_ctx* ctx, const Tiling& tl, int tile_lb, const Tiling& tm,
                 const std::vector<int64_t>& h_off, int64_t max_tiles, LayerSplit* sp) {
  const int64_t L = ctx->L;
  SplitPlan pl;
  plan_split(tl, tile_lb, tm, h_off, ctx->n_c, L, max_tiles, &pl);
  sp->tile = tile_lb;
  sp->tpc = (int)tl.tpc;
  sp->n_layers = pl.n_layers;
  sp->n_params = pl.n_params;
  sp->on = !pl.fused_tiles.empty();
  sp->n_fused_tiles = (int)pl.fused_tiles.size();
  sp->n_rest_tiles = (int)pl.rest_tiles.size();
  std::vector<int> cov;
  for (int64_t t = 0; t < tm.n_tiles; ++t)
    if (pl.covered[(size_t)t] || pl.covered_big[(size_t)t]) cov.push_back((int)t);
  sp->n_cov_tiles = (int)cov.size();
  sp->n_big_tiles = (int)pl.big_tiles.size();
  sp->big_on = sp->n_big_tiles > 0;
  sp->n_big_params = pl.n_big_params;
  sp->n_rest_ratio_tiles = (int)pl.rest_ratio_tiles.size();
  return upload(ctx, &sp->d_cov_tiles, cov) && upload(ctx, &sp->d_big_tiles, pl.big_tiles) &&
         upload(ctx, &sp->d_rest_ratio_tiles, pl.rest_ratio_tiles) && upload(ctx, &sp->d_fused_tiles, pl.fused_tiles) && upload(ctx, &sp->d_n_listed, pl.n_listed) &&
         upload(ctx, &sp->d_list_begin, pl.list_begin) && upload(ctx, &sp->d_seg_first, pl.seg_first) &&
         upload(ctx, &sp->d_seg_end, pl.seg_end) && alloc_zero(ctx, &sp->d_listed_max, pl.fused_tiles.size()) &&
         alloc_zero(ctx, &sp->d_listed_sums, 2 * pl.fused_tiles.size()) &&
         upload(ctx, &sp->d_rest_tiles, pl.rest_tiles) && upload(ctx, &sp->d_has_listed, pl.has_listed) &&
         alloc_zero(ctx, &sp->d_counter, (size_t)L * CTR_STRIDE) && alloc_zero(ctx, &sp->d_flag, (size_t)L);
}

void free_split(LayerSplit* sp) {
  void* ptrs[] = {sp->d_fused_tiles, sp->d_n_listed, sp->d_list_begin, sp->d_seg_first, sp->d_seg_end,
                  sp->d_listed_max,  sp->d_listed_sums, sp->d_rest_tiles, sp->d_cov_tiles, sp->d_big_tiles,
                  sp->d_rest_ratio_tiles,
                  sp->d_has_listed,  sp->d_counter,  sp->d_flag};
  for (void* p : ptrs)
    if (p) (void)hipFree(p);
}

ListedTiles listed_tiles(const ob_lamb_ctx* ctx, const LayerSplit& sp) {
  ListedTiles lt;
  lt.tile_list = sp.d_fused_tiles; lt.list_begin = sp.d_list_begin; lt.n_listed = sp.d_n_listed;
  lt.seg_first = sp.d_seg_first; lt.seg_end = sp.d_seg_end; lt.layer_seg0 = ctx->d_layer_seg0;
  lt.n_c = ctx->n_c; lt.tpc = sp.tpc; lt.tpc_span = ctx->tpc;
  return lt;
}

// Largest number of one layer's tiles that a barrier kernel with `per_cu` resident workgroups per
// CU may hold: 80 % of the device's slots, or the configuration's fused_max_tiles if that is lower
// (cap; 0 = none).
int64_t split_max_tiles(int per_cu, int cus, int32_t cap) {
  int64_t max_tiles = (4 * (int64_t)per_cu * cus) / 5 - OB_SPLIT_MARGIN;
  if (cap > 0 && cap < max_tiles) max_tiles = cap;
  return max_tiles < 0 ? 0 : max_tiles;
}

// Launches of the plain ratio pass and finalize kernels.  tiles: the 1024-element tiles to cover
// (NULL: all, in order), n_launch_tiles of them; layers with done_elsewhere[l] != 0 (NULL: none) are
// left to be finished by the kernel with the per-layer barrier.
void launch_ratios(Launch& la, ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                   const float* server_scales, bool packed_m, const PackedMom& pm, const int* tiles,
                   int n_launch_tiles, const unsigned char* done_elsewhere, bool finalize) {
  RatioArgs ra;
  ra.packed = packed_all; ra.sscales = server_scales; ra.m = st->m; ra.pm = pm;
  ra.v_fresh = st->v_fresh; ra.v_frozen = st->v_frozen;
  ra.beta1 = ctx->beta1; ra.omb1 = ctx->omb1; ra.beta2 = ctx->beta2; ra.omb2 = ctx->omb2;
  const LayerTab lt = layer_tab(ctx, st, ctx->d_first_layer);
  dispatch2(st->mom_scale != nullptr, packed_m, [&](auto hk, auto pk) {
    OB_LAUNCH(la, KID_RATIOS_PASS, (k_ratios_pass<U_MAIN, decltype(hk)::value, decltype(pk)::value>),
              n_launch_tiles, ra, ctx->d_seg_max, ctx->n_c, ctx->tpc, lt, ctx->d_tile_seg0, ctx->d_seg_layer,
              tiles);
  });
  if (finalize)
    OB_LAUNCH_B(la, KID_RATIOS_FINALIZE, k_ratios_finalize, (int)ctx->L, FBLOCK, ctx->d_seg_max,
                ctx->d_layer_seg0, st->c_avg, st->r_prev, st->coeff_c, ctx->one_m_thr, ctx->one_p_thr,
                ctx->r_min, ctx->r_max, done_elsewhere);
}

ApplyArgs apply_args(const ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                     const float* server_scales, float lr, const XLp& xl) {
  ApplyArgs aa;
  aa.packed = packed_all; aa.sscales = server_scales; aa.v_frozen = st->v_frozen; aa.x = st->x;
  aa.m = st->m; aa.coeff_c = st->coeff_c; aa.lr = lr; aa.eta = ctx->eta;
  aa.x_lp = xl.p; aa.x_lp_bf16 = xl.bf16;
  return aa;
}

void launch_apply(Launch& la, ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                  const float* server_scales, float lr, const int* tiles, int n_launch_tiles, const XLp& xl) {
  const ApplyArgs aa = apply_args(ctx, st, packed_all, server_scales, lr, xl);
  const LayerTab lt = layer_tab(ctx, st, ctx->d_first_layer);
  dispatch2(st->mom_scale != nullptr, st->m != nullptr, [&](auto hk, auto wm) {
    dispatch1(xl.p != nullptr, [&](auto lx) {
      OB_LAUNCH(la, KID_APPLY,
                (k_decompress_apply<U_MAIN, decltype(hk)::value, decltype(wm)::value, decltype(lx)::value>),
                n_launch_tiles, aa, ctx->n_c, ctx->tpc, lt, tiles);
    });
  });
}

// commit of the 1-bit momentum (see ob_lamb_decompress_apply)
void commit_packed_momentum(Launch& la, ob_lamb_ctx* ctx, const ob_lamb_state* st,
                                   const uint32_t* packed_all, const float* server_scales) {
  if (!(st->m_packed && st->m_packed != packed_all)) return;
  la.begin(KID_COPY, true);
  if (la.ok)
    la.ok = hip_ok(ctx, hipMemcpyAsync(st->m_packed, packed_all, (size_t)ctx->n_pad / 8,
                                       hipMemcpyDeviceToDevice, la.stream), "hipMemcpyAsync") &&
            hip_ok(ctx, hipMemcpyAsync(st->m_scales, server_scales, (size_t)ctx->W * sizeof(float),
                                       hipMemcpyDeviceToDevice, la.stream), "hipMemcpyAsync");
  la.end("copy", true);
}

ob_status check_ratios_args(const ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                                   const float* server_scales) {
  if (ob_status s = check_common(ctx, st)) return s;
  REQUIRE_PTR(packed_all); REQUIRE_PTR(st->v_fresh); REQUIRE_PTR(st->v_frozen);
  if (!server_scales || !st->c_avg || !st->r_prev || !st->coeff_c) return OB_ERR_NULL;
  return OB_OK;
}

ob_status check_apply_args(const ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                                  const float* server_scales, float lr) {
  if (ob_status s = check_common(ctx, st)) return s;
  REQUIRE_PTR(packed_all); REQUIRE_PTR(st->x); REQUIRE_PTR(st->v_frozen);
  if (!server_scales || !st->coeff_c) return OB_ERR_NULL;
  if (!std::isfinite(lr)) return OB_ERR_ARG;
  if (st->m && misaligned(st->m)) return OB_ERR_ALIGN;
  if (!st->m && !st->m_packed) return OB_ERR_NULL;  // the momentum has to be committed somewhere
  if (st->m_packed && !st->m_scales) return OB_ERR_NULL;
  if (st->m_packed && misaligned(st->m_packed)) return OB_ERR_ALIGN;
  return OB_OK;
}

}  // namespace

extern "C" {

int64_t ob_lamb_padded_len_for(int64_t n, int32_t W) {
  if (n < 0 || W < 1) return 0;
  const int64_t q = 256 * (int64_t)W;
  const int64_t r = ((n + q - 1) / q) * q;
  return r > 0 ? r : q;
}

const char* ob_lamb_status_string(ob_status s) {
  switch (s) {
    case OB_OK: return "ok";
    case OB_ERR_NULL: return "required pointer is NULL";
    case OB_ERR_ARG: return "invalid argument";
    case OB_ERR_ALIGN: return "device pointer not 16-byte aligned";
    case OB_ERR_STATE: return "invalid state";
    case OB_ERR_HIP: return "HIP runtime error";
    case OB_ERR_SIZE: return "size exceeds the capacity of the static scratch";
  }
  return "unknown status";
}

const char* ob_lamb_last_hip_error(const ob_lamb_ctx* ctx) { return ctx ? ctx->hip_err.c_str() : ""; }

static ob_status create_ctx(const ob_lamb_config* cfg, ob_lamb_ctx** out);

ob_status ob_lamb_create(const ob_lamb_config* cfg, ob_lamb_ctx** out) {
  // the host tables are std::vectors: a failed allocation must not leave the C ABI as an exception
  try {
    return create_ctx(cfg, out);
  } catch (const std::bad_alloc&) {
    if (out) *out = nullptr;
    return OB_ERR_ARG;
  }
}

static ob_status check_config(const ob_lamb_config* cfg) {
  if (!cfg || !cfg->layer_offsets) return OB_ERR_NULL;
  const int64_t L = cfg->num_layers;
  if (L < 1 || L > (int64_t)1 << 24 || cfg->num_workers < 1 || cfg->num_workers > 65536) return OB_ERR_ARG;
  if (cfg->server_chunk < 0 || cfg->server_chunk >= cfg->num_workers) return OB_ERR_ARG;
  if (cfg->layer_offsets[0] != 0) return OB_ERR_ARG;
  for (int64_t l = 0; l < L; ++l)
    if (cfg->layer_offsets[l + 1] < cfg->layer_offsets[l]) return OB_ERR_ARG;
  const int64_t N = cfg->layer_offsets[L];
  if (N < 1 || N > ((int64_t)1 << 40)) return OB_ERR_ARG;
  const float fl[] = {cfg->beta1, cfg->beta2, cfg->beta3, cfg->eta, cfg->c_min, cfg->c_max,
                      cfg->r_min, cfg->r_max, cfg->r_threshold, cfg->weight_decay};
  for (float f : fl)
    if (!std::isfinite(f)) return OB_ERR_ARG;
  if (cfg->c_min > cfg->c_max || cfg->r_min > cfg->r_max) return OB_ERR_ARG;
  if ((cfg->flags & ~OB_CFG_NO_BARRIERS) != 0u || cfg->fused_max_tiles < 0 || cfg->spin_limit < OB_SPIN_NONE)
    return OB_ERR_ARG;
  return OB_OK;
}

// Offsets with the sentinel the per-element paths rely on.
static std::vector<int64_t> host_offsets(const ob_lamb_config* cfg) {
  const int64_t L = cfg->num_layers;
  std::vector<int64_t> h_off((size_t)L + 2);
  for (int64_t l = 0; l <= L; ++l) h_off[(size_t)l] = cfg->layer_offsets[l];
  h_off[(size_t)L + 1] = std::numeric_limits<int64_t>::max();
  return h_off;
}

ob_status ob_lamb_plan_split(const ob_lamb_config* cfg, int64_t max_tiles, uint8_t* span_owner,
                             int32_t* layer_listed) {
  if (ob_status s = check_config(cfg)) return s;
  if (!span_owner || !layer_listed) return OB_ERR_NULL;
  if (max_tiles < 0) return OB_ERR_ARG;
  try {
    const int64_t L = cfg->num_layers, W = cfg->num_workers;
    const int64_t n_c = ob_lamb_padded_len_for(cfg->layer_offsets[L], cfg->num_workers) / W;
    const std::vector<int64_t> h_off = host_offsets(cfg);
    Tiling tm, tl;
    if (!build_tiling(TILE_MAIN, n_c, W, L, h_off, &tm) || !build_tiling(TILE_LB, n_c, W, L, h_off, &tl))
      return OB_ERR_ARG;
    SplitPlan pl;
    plan_split(tl, TILE_LB, tm, h_off, n_c, L, max_tiles, &pl);
    for (int64_t t = 0; t < tm.n_tiles; ++t) span_owner[t] = pl.covered[(size_t)t] ? 2 : 0;
    for (int t : pl.rest_tiles) span_owner[t] = 1;
    for (int64_t l = 0; l < L; ++l) layer_listed[l] = pl.n_listed[(size_t)l];
    return OB_OK;
  } catch (const std::bad_alloc&) {
    return OB_ERR_ARG;
  }
}

ob_status ob_lamb_plan_big_tiles(const ob_lamb_config* cfg, int64_t max_tiles, uint8_t* span_big) {
  if (ob_status s = check_config(cfg)) return s;
  if (!span_big) return OB_ERR_NULL;
  if (max_tiles < 0) return OB_ERR_ARG;
  try {
    const int64_t L = cfg->num_layers, W = cfg->num_workers;
    const int64_t n_c = ob_lamb_padded_len_for(cfg->layer_offsets[L], cfg->num_workers) / W;
    const std::vector<int64_t> h_off = host_offsets(cfg);
    Tiling tm, tl;
    if (!build_tiling(TILE_MAIN, n_c, W, L, h_off, &tm) || !build_tiling(TILE_LB, n_c, W, L, h_off, &tl))
      return OB_ERR_ARG;
    SplitPlan pl;
    plan_split(tl, TILE_LB, tm, h_off, n_c, L, max_tiles, &pl);
    for (int64_t t = 0; t < tm.n_tiles; ++t) span_big[t] = pl.covered_big[(size_t)t] ? 1 : 0;
    return OB_OK;
  } catch (const std::bad_alloc&) {
    return OB_ERR_ARG;
  }
}

namespace { ob_status static_scratch(double** out); }

static ob_status create_ctx(const ob_lamb_config* cfg, ob_lamb_ctx** out) {
  if (out) *out = nullptr;
  if (!out) return OB_ERR_NULL;
  if (ob_status s = check_config(cfg)) return s;
  {
    // set-up time is also when this device's copy of the static scratch array (used by
    // ob_lamb_server_reduce_static, which must not do anything but launch) is looked up
    double* unused = nullptr;
    if (ob_status s = static_scratch(&unused)) return s;
  }
  const int64_t L = cfg->num_layers;
  const int64_t N = cfg->layer_offsets[L];

  ob_lamb_ctx* ctx = new (std::nothrow) ob_lamb_ctx();
  if (!ctx) return OB_ERR_ARG;
  struct Guard {   // frees the context and what it holds on every path that does not hand it over
    ob_lamb_ctx* c;
    ~Guard() { ob_lamb_destroy(c); }
  } guard{ctx};
  ctx->L = L;
  ctx->N = N;
  ctx->W = cfg->num_workers;
  ctx->server_chunk = cfg->server_chunk;
  ctx->n_pad = ob_lamb_padded_len_for(N, ctx->W);
  ctx->n_c = ctx->n_pad / ctx->W;
  ctx->beta1 = cfg->beta1; ctx->beta2 = cfg->beta2; ctx->beta3 = cfg->beta3;
  ctx->eta = cfg->eta; ctx->c_min = cfg->c_min; ctx->c_max = cfg->c_max;
  ctx->r_min = cfg->r_min; ctx->r_max = cfg->r_max; ctx->r_thr = cfg->r_threshold;
  ctx->wd = cfg->weight_decay;
  ctx->omb1 = 1.0f - ctx->beta1;
  ctx->omb2 = 1.0f - ctx->beta2;
  ctx->omb3 = 1.0f - ctx->beta3;
  ctx->one_m_thr = 1.0f - ctx->r_thr;
  ctx->one_p_thr = 1.0f + ctx->r_thr;
  ctx->invW = 1.0f / (float)ctx->W;

  const int64_t tpc_srv = (ctx->n_c + TILE_SRV - 1) / TILE_SRV;
  if (tpc_srv > 0x7fffffff) return OB_ERR_ARG;
  ctx->tpc_srv = (int)tpc_srv;

  const std::vector<int64_t> h_off = host_offsets(cfg);
  Tiling tm, tl, tw;
  if (!build_tiling(TILE_MAIN, ctx->n_c, ctx->W, L, h_off, &tm) ||
      !build_tiling(TILE_LB, ctx->n_c, ctx->W, L, h_off, &tl) ||
      !build_tiling(TILE_WU, ctx->n_c, ctx->W, L, h_off, &tw))
    return OB_ERR_ARG;
  const int64_t n_tiles = tm.n_tiles;
  ctx->tpc = (int)tm.tpc;
  ctx->n_tiles = (int)tm.n_tiles;
  ctx->n_segs = (int)tm.seg_layer.size();
  const std::vector<int>&first = tm.first, &tile_seg0 = tm.tile_seg0, &seg_layer = tm.seg_layer,
                        &layer_seg0 = tm.layer_seg0;

  // single-pass worker compression: its own (larger) tiles and the layer of each tile's start
  const int64_t tpc_res = (ctx->n_c + TILE_RES - 1) / TILE_RES;
  ctx->tpc_res = (int)tpc_res;
  ctx->n_tiles_res = (int)(tpc_res * ctx->W);
  std::vector<int> first_res((size_t)ctx->n_tiles_res);
  for (int64_t t = 0; t < ctx->n_tiles_res; ++t) {
    const int64_t tile0 = (t / tpc_res) * ctx->n_c + (t % tpc_res) * TILE_RES;
    int64_t lo = 0, hi = L + 1;
    while (hi - lo > 1) {
      const int64_t mid = (lo + hi) / 2;
      if (h_off[(size_t)mid] <= tile0) lo = mid; else hi = mid;
    }
    first_res[(size_t)t] = (int)lo;
  }

  bool ok = hip_ok(ctx, hipGetDevice(&ctx->device), "hipGetDevice");
  if (ok) {
    // The single-pass kernel needs a whole chunk's workgroups on the device at once (see the
    // kernel's comment); it is used only when they fill at most 80 % of the device's workgroup
    // slots (it still beats two passes at 61 % on MI355X), else the two-pass kernels run.
    int per_cu = 0, cus = 0;
    ok = hip_ok(ctx, hipOccupancyMaxActiveBlocksPerMultiprocessor(
                         &per_cu, k_compress_resident<U_RES, G_RES, true, false>, BLOCK, 0),
                "hipOccupancyMaxActiveBlocksPerMultiprocessor") &&
         hip_ok(ctx, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, ctx->device),
                "hipDeviceGetAttribute");
    // every instantiation is built for at least OB_RES_MINW workgroups per CU (its launch bounds); count
    // no more than that, whatever this one reaches
    const int64_t slots = (int64_t)std::min(per_cu, OB_RES_MINW) * cus;
    // a lower bound of the device-side waits (tests of the expiry path: with OB_SPIN_NONE every wait
    // gives up without polling, all kernels still run to their end)
    if (cfg->spin_limit == OB_SPIN_NONE) ctx->spin_limit = 0;
    else if (cfg->spin_limit > 0 && cfg->spin_limit < ctx->spin_limit) ctx->spin_limit = cfg->spin_limit;
    const bool two_pass = (cfg->flags & OB_CFG_TWO_PASS_COMPRESS) != 0;
    ctx->resident = ok && !two_pass && 5 * (tpc_res + 8) <= 4 * slots;
    // the single-pass server kernel: same rule for the one chunk it covers
    int per_cu_s[3] = {0, 0, 0};
    ok = ok &&
         hip_ok(ctx, hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_s[0], k_server_resident<U_SRV_RES[0]>, BLOCK, 0),
                "hipOccupancyMaxActiveBlocksPerMultiprocessor") &&
         hip_ok(ctx, hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_s[1], k_server_resident<U_SRV_RES[1]>, BLOCK, 0),
                "hipOccupancyMaxActiveBlocksPerMultiprocessor") &&
         hip_ok(ctx, hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_s[2], k_server_resident<U_SRV_RES[2]>, BLOCK, 0),
                "hipOccupancyMaxActiveBlocksPerMultiprocessor");
    // the tile table of the chunk's partials is sized for the smallest tile
    ctx->tpc_srv_res = (int)((ctx->n_c + SPAN - 1) / SPAN);
    for (int i = 0; ok && i < 3 && ctx->u_srv_res == 0 && !two_pass; ++i) {
      const int64_t tiles = (ctx->n_c + (int64_t)SPAN * U_SRV_RES[i] - 1) / ((int64_t)SPAN * U_SRV_RES[i]);
      if (5 * (tiles + 8) <= 4 * (int64_t)per_cu_s[i] * cus) ctx->u_srv_res = U_SRV_RES[i];
    }
  }
  // the two kernels with a per-layer barrier: which layers each of them takes.  The slot count is
  // the kernel's launch bound (every instantiation reaches it), whatever the one queried reaches.
  if (ok) {
    int per_cu_a = 0, per_cu_w = 0, cus = 0;
    ok = hip_ok(ctx, hipOccupancyMaxActiveBlocksPerMultiprocessor(
#if OB_LB_STREAM
                         &per_cu_a, k_ratios_apply_stream<U_LB, OB_G_LB, true>, BLOCK, 0),
#else
                         &per_cu_a, k_ratios_apply_resident<U_LB, true>, BLOCK, 0),
#endif
                "hipOccupancyMaxActiveBlocksPerMultiprocessor") &&
         hip_ok(ctx, hipOccupancyMaxActiveBlocksPerMultiprocessor(
                         &per_cu_w, k_warmup_resident<U_WU, G_WU, 0, false>, BLOCK, 0),
                "hipOccupancyMaxActiveBlocksPerMultiprocessor") &&
         hip_ok(ctx, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, ctx->device),
                "hipDeviceGetAttribute");
    int per_cu_h = 0;   // the same tiles go through the kernel with the variance in deferred form
    ok = ok && hip_ok(ctx, hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_h, k_ratios_apply_hist<true, false>, BLOCK, 0),
                      "hipOccupancyMaxActiveBlocksPerMultiprocessor");
    per_cu_a = std::min(per_cu_a, per_cu_h);
    const int64_t max_a = (cfg->flags & OB_CFG_NO_FUSED_APPLY)
                              ? 0 : split_max_tiles(std::min(per_cu_a, OB_LB_MINW), cus, cfg->fused_max_tiles);
    const int64_t max_w = (cfg->flags & OB_CFG_TWO_PASS_WARMUP)
                              ? 0 : split_max_tiles(std::min(per_cu_w, OB_WU_MINW), cus, cfg->fused_max_tiles);
    ok = ok && build_split(ctx, tl, TILE_LB, tm, h_off, max_a, &ctx->sp_apply) &&
         build_split(ctx, tw, TILE_WU, tm, h_off, max_w, &ctx->sp_warm);
  }
  ok = ok && upload(ctx, &ctx->d_first_layer_res, first_res) &&
       alloc_zero(ctx, &ctx->d_partials_res, (size_t)ctx->n_tiles_res) &&
       alloc_zero(ctx, &ctx->d_counter, (size_t)ctx->W * CTR_STRIDE) && alloc_zero(ctx, &ctx->d_flag, (size_t)ctx->W) &&
       alloc_zero(ctx, &ctx->d_errflag, 1) &&
       alloc_zero(ctx, &ctx->d_partials_srv_res, (size_t)ctx->tpc_srv_res) &&
       alloc_zero(ctx, &ctx->d_counter_srv, (size_t)CTR_STRIDE) && alloc_zero(ctx, &ctx->d_flag_srv, 1);
  ok = ok && upload(ctx, &ctx->d_off, h_off) && upload(ctx, &ctx->d_first_layer, first) &&
       upload(ctx, &ctx->d_tile_seg0, tile_seg0) && upload(ctx, &ctx->d_seg_layer, seg_layer) &&
       upload(ctx, &ctx->d_layer_seg0, layer_seg0) &&
       alloc_zero(ctx, &ctx->d_partials, (size_t)n_tiles) &&
       alloc_zero(ctx, &ctx->d_partials_srv, (size_t)tpc_srv) &&
       alloc_zero(ctx, &ctx->d_seg_sums, 2 * (size_t)ctx->n_segs) &&
       alloc_zero(ctx, &ctx->d_sigma, (size_t)L) &&
       alloc_zero(ctx, &ctx->d_seg_max, (size_t)ctx->n_segs);
  if (ok) {
    // the layers that meet each chunk (empty layers in between included; a chunk that lies in the
    // padding has none)
    std::vector<int> pair_base((size_t)ctx->W + 1, 0), pair_lfirst((size_t)ctx->W, 0), pair_c, pair_l;
    int64_t l = 0;
    for (int64_t c = 0; c < ctx->W; ++c) {
      const int64_t c0 = c * ctx->n_c, c1 = std::min((c + 1) * ctx->n_c, N);
      pair_base[(size_t)c] = (int)pair_c.size();
      if (c0 < N) {
        while (h_off[(size_t)l + 1] <= c0) ++l;      // the layer that holds element c0
        pair_lfirst[(size_t)c] = (int)l;
        for (int64_t q = l; q < L && h_off[(size_t)q] < c1; ++q) {
          pair_c.push_back((int)c);
          pair_l.push_back((int)q);
        }
      }
    }
    pair_base[(size_t)ctx->W] = (int)pair_c.size();
    ctx->n_pairs = (int)pair_c.size();
    ok = upload(ctx, &ctx->d_pair_base, pair_base) && upload(ctx, &ctx->d_pair_lfirst, pair_lfirst) &&
         upload(ctx, &ctx->d_pair_c, pair_c) && upload(ctx, &ctx->d_pair_l, pair_l) &&
         alloc_zero(ctx, &ctx->d_vterms, (size_t)(VF_MAX_OLD + 1) * (size_t)ctx->n_pairs * 2);
  }
  ok = ok && hip_ok(ctx, hipDeviceSynchronize(), "hipDeviceSynchronize");
  if (!ok) return OB_ERR_HIP;
  guard.c = nullptr;
  *out = ctx;
  return OB_OK;
}

void ob_lamb_destroy(ob_lamb_ctx* ctx) {
  if (!ctx) return;
  for (auto& r : ctx->prof) {
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  void* ptrs[] = {ctx->d_off, ctx->d_first_layer, ctx->d_tile_seg0, ctx->d_seg_layer, ctx->d_layer_seg0,
                  ctx->d_partials, ctx->d_partials_srv, ctx->d_seg_sums, ctx->d_seg_max, ctx->d_sigma,
                  ctx->d_first_layer_res, ctx->d_partials_res, ctx->d_counter, ctx->d_flag, ctx->d_errflag,
                  ctx->d_partials_srv_res, ctx->d_counter_srv, ctx->d_flag_srv, ctx->d_pair_base,
                  ctx->d_pair_lfirst, ctx->d_pair_c, ctx->d_pair_l, ctx->d_vterms};
  for (void* p : ptrs)
    if (p) (void)hipFree(p);
  free_split(&ctx->sp_apply);
  free_split(&ctx->sp_warm);
  delete ctx;
}

int64_t ob_lamb_num_params(const ob_lamb_ctx* ctx) { return ctx ? ctx->N : 0; }
int64_t ob_lamb_padded_len(const ob_lamb_ctx* ctx) { return ctx ? ctx->n_pad : 0; }
int64_t ob_lamb_chunk_len(const ob_lamb_ctx* ctx) { return ctx ? ctx->n_c : 0; }
size_t ob_lamb_workspace_bytes(const ob_lamb_ctx* ctx) { return ctx ? ctx->device_bytes : 0; }

ob_status ob_lamb_warmup_step_lp(ob_lamb_ctx* ctx, const ob_lamb_state* st, const void* grad,
                                 ob_dtype grad_dtype, float grad_scale, float lr, void* x_lp,
                                 ob_dtype x_dtype, void* hip_stream) {
  if (ob_status s = check_common(ctx, st)) return s;
  GradSrc gs;
  bool lpg = false;
  if (ob_status s = grad_source(grad, grad_dtype, grad_scale, &gs, &lpg)) return s;
  XLp xl;
  if (ob_status s = x_lp_target(x_lp, x_dtype, &xl)) return s;
  REQUIRE_PTR(st->x); REQUIRE_PTR(st->m); REQUIRE_PTR(st->v_fresh);
  if (!st->c_avg || !st->coeff_c) return OB_ERR_NULL;
  if (!std::isfinite(lr)) return OB_ERR_ARG;
  Launch la(ctx, hip_stream);
  const LayerTab lt = layer_tab(ctx, st, ctx->d_first_layer);
  auto moments = [&](const int* tiles, int n_launch_tiles) {
    dispatch1(lpg, [&](auto lg) {
      OB_LAUNCH(la, KID_WARMUP_MOMENTS, (k_warmup_moments<U_MAIN, decltype(lg)::value ? 1 : 0>), n_launch_tiles,
                gs, st->m, st->v_fresh, st->x, ctx->d_seg_sums, ctx->n_c, ctx->tpc, ctx->beta1, ctx->omb1,
                ctx->beta2, ctx->omb2, ctx->eta, ctx->wd, lt, ctx->d_tile_seg0, ctx->d_seg_layer, tiles);
    });
  };
  auto coeff = [&](const unsigned char* done_elsewhere) {
    OB_LAUNCH_B(la, KID_WARMUP_COEFF, k_warmup_coeff, (int)ctx->L, FBLOCK, ctx->d_seg_sums, ctx->d_layer_seg0,
                st->coeff_c, st->c_avg, ctx->c_min, ctx->c_max, ctx->beta3, ctx->omb3, done_elsewhere);
  };
  auto apply = [&](const int* tiles, int n_launch_tiles) {
    dispatch1(xl.p != nullptr, [&](auto lx) {
      OB_LAUNCH(la, KID_WARMUP_APPLY, (k_warmup_apply<U_MAIN, decltype(lx)::value>), n_launch_tiles, st->m,
                st->v_fresh, st->x, st->coeff_c, ctx->n_c, ctx->tpc, lr, ctx->eta, ctx->wd, lt, xl.p, xl.bf16,
                tiles);
    });
  };
  LayerSplit& sp = ctx->sp_warm;
  if (!sp.on) {   // two passes over everything
    moments(nullptr, ctx->n_tiles);
    coeff(nullptr);
    apply(nullptr, ctx->n_tiles);
    return la.ok ? OB_OK : OB_ERR_HIP;
  }
  // 1. moments and partial sums of everything outside the listed tiles; the layers without listed
  //    tiles get their c here (an empty layer too), the sums of the others wait in seg_sums
  moments(sp.d_rest_tiles, sp.n_rest_tiles);
  if (sp.n_layers < ctx->L) coeff(sp.d_has_listed);
  // 2. the listed tiles: moments, layer barrier, update
  WarmSync ws;
  ws.seg_sums = ctx->d_seg_sums; ws.listed_sums = sp.d_listed_sums; ws.lt = listed_tiles(ctx, sp);
  ws.counter = sp.d_counter; ws.flag = sp.d_flag; ws.errflag = ctx->d_errflag;
  ws.spin_limit = ctx->spin_limit;
  ws.coeff_c = st->coeff_c; ws.c_avg = st->c_avg;
  ws.c_min = ctx->c_min; ws.c_max = ctx->c_max; ws.beta3 = ctx->beta3; ws.omb3 = ctx->omb3;
  dispatch2(lpg, xl.p != nullptr, [&](auto lg, auto lx) {
    OB_LAUNCH(la, KID_WARMUP_RESIDENT,
              (k_warmup_resident<U_WU, G_WU, decltype(lg)::value ? 1 : 0, decltype(lx)::value>), sp.n_fused_tiles,
              gs, st->m, st->v_fresh, st->x, ws, ctx->beta1, ctx->omb1, ctx->beta2, ctx->omb2, ctx->eta, ctx->wd,
              lr, lt, xl.p, xl.bf16);
  });
  // 3. update of everything outside the listed tiles, with the coefficients of steps 1 and 2
  apply(sp.d_rest_tiles, sp.n_rest_tiles);
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_warmup_step(ob_lamb_ctx* ctx, const ob_lamb_state* st, const float* grad, float lr,
                              void* hip_stream) {
  return ob_lamb_warmup_step_lp(ctx, st, grad, OB_F32, 1.0f, lr, nullptr, OB_F32, hip_stream);
}

ob_status ob_lamb_freeze(ob_lamb_ctx* ctx, const ob_lamb_state* st, void* hip_stream) {
  if (ob_status s = check_common(ctx, st)) return s;
  REQUIRE_PTR(st->v_fresh); REQUIRE_PTR(st->v_frozen);
  if (!st->r_prev) return OB_ERR_NULL;
  Launch la(ctx, hip_stream);
  la.begin(KID_COPY, true);
  if (la.ok)
    la.ok = hip_ok(ctx, hipMemcpyAsync(st->v_frozen, st->v_fresh, (size_t)ctx->n_pad * sizeof(float),
                                       hipMemcpyDeviceToDevice, la.stream), "hipMemcpyAsync");
  la.end("copy", true);
  OB_LAUNCH(la, KID_FILL, k_fill, (int)((ctx->L + BLOCK - 1) / BLOCK), st->r_prev, ctx->L, 1.0f);
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_compress_local_lp(ob_lamb_ctx* ctx, const ob_lamb_state* st, const void* grad,
                                    ob_dtype grad_dtype, float grad_scale, uint32_t* packed_out,
                                    float* scales_out, void* hip_stream) {
  if (ob_status s = check_common(ctx, st)) return s;
  GradSrc gs;
  bool lpg = false;
  if (ob_status s = grad_source(grad, grad_dtype, grad_scale, &gs, &lpg)) return s;
  REQUIRE_PTR(st->err_worker); REQUIRE_PTR(packed_out);
  if (!scales_out) return OB_ERR_NULL;
  bool packed_m = false;
  PackedMom pm;
  if (ob_status s = momentum_source(st, &packed_m, &pm)) return s;
  if (packed_m && st->m_packed == packed_out) return OB_ERR_ARG;  // would be overwritten while read
  if ((st->own_packed_in == nullptr) != (st->own_scale_in == nullptr)) return OB_ERR_NULL;
  if (st->own_packed_in && misaligned(st->own_packed_in)) return OB_ERR_ALIGN;
  OwnCopy oc;
  oc.packed = st->own_packed_in; oc.scale = st->own_scale_in; oc.chunk = ctx->server_chunk;
  Launch la(ctx, hip_stream);
  PackedErr pe;
  pe.bits = st->err_packed; pe.scales = st->err_scales;
  if ((st->err_packed == nullptr) != (st->err_scales == nullptr)) return OB_ERR_NULL;
  if (st->err_packed) {
    // deferred error: the whole call is one streaming pass plus the scales -- no barrier, no second pass
    if (misaligned(st->err_packed)) return OB_ERR_ALIGN;
    if (packed_m && st->m_packed == st->err_packed) return OB_ERR_ARG;
    const LayerTab lt = layer_tab(ctx, st, ctx->d_first_layer);
    dispatch2(st->mom_scale != nullptr, packed_m, [&](auto hk, auto pk) {
      dispatch1(lpg, [&](auto lg) {
        OB_LAUNCH(la, KID_COMPRESS_DEFERRED,
                  (k_momentum_z_sumsq<U_MAIN, decltype(hk)::value, decltype(pk)::value,
                                      decltype(lg)::value ? 1 : 0, true>),
                  ctx->n_tiles, gs, st->m, pm, st->err_worker, ctx->d_partials, ctx->n_c, ctx->tpc,
                  ctx->beta1, ctx->omb1, lt, pe, packed_out, oc);
      });
    });
    OB_LAUNCH_B(la, KID_CHUNK_SCALE, k_chunk_scale, ctx->W, FBLOCK, ctx->d_partials, ctx->tpc, ctx->n_c, scales_out,
                oc.scale, oc.chunk);
    return la.ok ? OB_OK : OB_ERR_HIP;
  }
  if (ctx->resident) {
    ChunkSync cs;
    cs.partials = ctx->d_partials_res;
    cs.counter = ctx->d_counter;
    cs.flag = ctx->d_flag;
    cs.errflag = ctx->d_errflag;
    cs.spin_limit = ctx->spin_limit;
    const LayerTab lt = layer_tab(ctx, st, ctx->d_first_layer_res);
    dispatch2(st->mom_scale != nullptr, packed_m, [&](auto hk, auto pk) {
      dispatch1(lpg, [&](auto lg) {
        OB_LAUNCH(la, KID_COMPRESS_RESIDENT,
                  (k_compress_resident<U_RES, G_RES, decltype(hk)::value, decltype(pk)::value, OB_RES_MINW,
                                       decltype(lg)::value ? 1 : 0>),
                  ctx->n_tiles_res, gs, st->m, pm, st->err_worker, packed_out, scales_out, cs, ctx->n_c,
                  ctx->tpc_res, ctx->beta1, ctx->omb1, lt, oc);
      });
    });
    return la.ok ? OB_OK : OB_ERR_HIP;
  }
  const LayerTab lt = layer_tab(ctx, st, ctx->d_first_layer);
  dispatch2(st->mom_scale != nullptr, packed_m, [&](auto hk, auto pk) {
    dispatch1(lpg, [&](auto lg) {
      OB_LAUNCH(la, KID_MOMENTUM_Z,
                (k_momentum_z_sumsq<U_MAIN, decltype(hk)::value, decltype(pk)::value, decltype(lg)::value ? 1 : 0>),
                ctx->n_tiles, gs, st->m, pm, st->err_worker, ctx->d_partials, ctx->n_c, ctx->tpc,
                ctx->beta1, ctx->omb1, lt, pe, packed_out, oc);
    });
  });
  OB_LAUNCH_B(la, KID_CHUNK_SCALE, k_chunk_scale, ctx->W, FBLOCK, ctx->d_partials, ctx->tpc, ctx->n_c, scales_out,
              (float*)nullptr, 0);
  OB_LAUNCH(la, KID_SIGN_PACK, (k_sign_pack_error<U_MAIN>), ctx->n_tiles, st->err_worker, packed_out,
            scales_out, ctx->n_c, ctx->tpc);
  if (oc.packed) {   // the two-pass form copies the rank's own chunk afterwards
    const int64_t wpc = ctx->n_c / 32;
    la.begin(KID_COPY, true);
    if (la.ok)
      la.ok = hip_ok(ctx, hipMemcpyAsync(oc.packed, packed_out + (int64_t)oc.chunk * wpc, (size_t)wpc * 4,
                                         hipMemcpyDeviceToDevice, la.stream), "hipMemcpyAsync") &&
              hip_ok(ctx, hipMemcpyAsync(oc.scale, scales_out + oc.chunk, sizeof(float),
                                         hipMemcpyDeviceToDevice, la.stream), "hipMemcpyAsync");
    la.end("copy", true);
  }
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_compress_local(ob_lamb_ctx* ctx, const ob_lamb_state* st, const float* grad,
                                 uint32_t* packed_out, float* scales_out, void* hip_stream) {
  return ob_lamb_compress_local_lp(ctx, st, grad, OB_F32, 1.0f, packed_out, scales_out, hip_stream);
}

ob_status ob_lamb_server_reduce(ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_in,
                                const float* scales_in, uint32_t* packed_out, float* scale_out,
                                void* hip_stream) {
  if (ob_status s = check_common(ctx, st)) return s;
  REQUIRE_PTR(packed_in); REQUIRE_PTR(packed_out); REQUIRE_PTR(st->err_server);
  if (!scales_in || !scale_out) return OB_ERR_NULL;
  // the kernels address packed_in with 32-bit byte offsets
  if ((int64_t)ctx->W * (ctx->n_c / 8) >= ((int64_t)1 << 31)) return OB_ERR_SIZE;
  Launch la(ctx, hip_stream);
  if ((st->srv_err_packed == nullptr) != (st->srv_err_scale == nullptr)) return OB_ERR_NULL;
  if (st->srv_err_packed) {
    // deferred server error: one pass over the chunk plus its scale -- no barrier, no second pass
    if (misaligned(st->srv_err_packed)) return OB_ERR_ALIGN;
    if (st->srv_err_packed == packed_out) return OB_ERR_ARG;
    OB_LAUNCH(la, KID_SERVER_AVG, (k_server_unpack_avg<U_SRV, true>), ctx->tpc_srv, packed_in, scales_in,
              st->err_server, ctx->d_partials_srv, ctx->n_c, (int)ctx->W, ctx->invW, st->srv_err_packed,
              st->srv_err_scale, packed_out);
    OB_LAUNCH_B(la, KID_SERVER_SCALE, k_chunk_scale, 1, FBLOCK, ctx->d_partials_srv, ctx->tpc_srv, ctx->n_c, scale_out,
                st->srv_err_scale, 0);
    return la.ok ? OB_OK : OB_ERR_HIP;
  }
  if (ctx->u_srv_res) {
    ChunkSync cs;
    cs.partials = ctx->d_partials_srv_res;
    cs.counter = ctx->d_counter_srv;
    cs.flag = ctx->d_flag_srv;
    cs.errflag = ctx->d_errflag;
    cs.spin_limit = ctx->spin_limit;
    const int64_t tile = (int64_t)SPAN * ctx->u_srv_res;
    const int tiles = (int)((ctx->n_c + tile - 1) / tile);
    auto launch = [&](auto u) {
      OB_LAUNCH(la, KID_SERVER_RESIDENT, (k_server_resident<decltype(u)::value>), tiles, packed_in, scales_in,
                st->err_server, packed_out, scale_out, cs, ctx->n_c, (int)ctx->W, ctx->invW);
    };
    switch (ctx->u_srv_res) {
      case 1: launch(std::integral_constant<int, 1>{}); break;
      case 2: launch(std::integral_constant<int, 2>{}); break;
      default: launch(std::integral_constant<int, 4>{}); break;
    }
    return la.ok ? OB_OK : OB_ERR_HIP;
  }
  OB_LAUNCH(la, KID_SERVER_AVG, (k_server_unpack_avg<U_SRV>), ctx->tpc_srv, packed_in, scales_in,
            st->err_server, ctx->d_partials_srv, ctx->n_c, (int)ctx->W, ctx->invW, (uint32_t*)nullptr,
            (const float*)nullptr, (uint32_t*)nullptr);
  OB_LAUNCH_B(la, KID_SERVER_SCALE, k_chunk_scale, 1, FBLOCK, ctx->d_partials_srv, ctx->tpc_srv, ctx->n_c, scale_out,
              (float*)nullptr, 0);
  OB_LAUNCH(la, KID_SERVER_PACK, (k_sign_pack_error<U_SRV>), ctx->tpc_srv, st->err_server, packed_out,
            scale_out, ctx->n_c, ctx->tpc_srv);
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_layer_ratios(ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                               const float* server_scales, void* hip_stream) {
  if (ob_status s = check_ratios_args(ctx, st, packed_all, server_scales)) return s;
  bool packed_m = false;
  PackedMom pm;
  if (ob_status s = momentum_source(st, &packed_m, &pm)) return s;
  Launch la(ctx, hip_stream);
  launch_ratios(la, ctx, st, packed_all, server_scales, packed_m, pm, nullptr, ctx->n_tiles, nullptr, true);
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_decompress_apply_lp(ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                                      const float* server_scales, float lr, void* x_lp, ob_dtype x_dtype,
                                      void* hip_stream) {
  if (ob_status s = check_apply_args(ctx, st, packed_all, server_scales, lr)) return s;
  XLp xl;
  if (ob_status s = x_lp_target(x_lp, x_dtype, &xl)) return s;
  Launch la(ctx, hip_stream);
  launch_apply(la, ctx, st, packed_all, server_scales, lr, nullptr, ctx->n_tiles, xl);
  commit_packed_momentum(la, ctx, st, packed_all, server_scales);
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_decompress_apply(ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                                   const float* server_scales, float lr, void* hip_stream) {
  return ob_lamb_decompress_apply_lp(ctx, st, packed_all, server_scales, lr, nullptr, OB_F32, hip_stream);
}

ob_status ob_lamb_ratios_apply_lp(ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                                  const float* server_scales, float lr, void* x_lp, ob_dtype x_dtype,
                                  void* hip_stream) {
  if (ob_status s = check_ratios_args(ctx, st, packed_all, server_scales)) return s;
  XLp xl;
  if (ob_status s = x_lp_target(x_lp, x_dtype, &xl)) return s;
  REQUIRE_PTR(st->x);
  if (!std::isfinite(lr)) return OB_ERR_ARG;
  bool packed_m = false;
  PackedMom pm;
  pm.bits = nullptr;
  pm.scales = nullptr;
  // momentum source: dense st->m if given (then it is also where the new momentum is written),
  // else the 1-bit form of the previous step (then nothing is written: the new momentum is
  // packed_all/server_scales themselves)
  if (ob_status s = momentum_source(st, &packed_m, &pm)) return s;
  if (packed_m && st->m_packed == packed_all) return OB_ERR_ARG;
  Launch la(ctx, hip_stream);
  LayerSplit& sp = ctx->sp_apply;
  if (!sp.on || !packed_m) {
    // no tile qualifies, or the momentum is a dense array (the barrier kernel would have to hold it
    // too, which costs more than the second read of v_frozen saves): the two plain kernels
    launch_ratios(la, ctx, st, packed_all, server_scales, packed_m, pm, nullptr, ctx->n_tiles, nullptr, true);
    launch_apply(la, ctx, st, packed_all, server_scales, lr, nullptr, ctx->n_tiles, xl);
    return la.ok ? OB_OK : OB_ERR_HIP;
  }
  RatioArgs ra;
  ra.packed = packed_all; ra.sscales = server_scales; ra.m = st->m; ra.pm = pm;
  ra.v_fresh = st->v_fresh; ra.v_frozen = st->v_frozen;
  ra.beta1 = ctx->beta1; ra.omb1 = ctx->omb1; ra.beta2 = ctx->beta2; ra.omb2 = ctx->omb2;
  const ApplyArgs aa = apply_args(ctx, st, packed_all, server_scales, lr, xl);
  const bool hk = st->mom_scale != nullptr;  // (here the momentum is in 1-bit form and st->m is NULL)
  const LayerTab lt = layer_tab(ctx, st, ctx->d_first_layer);
  // 1. ratio pass over everything outside the listed tiles; its segment maxima wait in seg_max: of
  //    the layers with listed tiles for the layer barrier, of the others (the ratio of an empty layer,
  //    0, still goes through the clips) for the leading workgroups of the same launch
#if OB_LB_STREAM
  const int n_lead = 0;
#else
  const int n_lead = (sp.n_layers < ctx->L) ? (int)ctx->L : 0;   // (finished by the barrier kernel's leading workgroups)
#endif
  launch_ratios(la, ctx, st, packed_all, server_scales, packed_m, pm, sp.d_rest_tiles, sp.n_rest_tiles,
                sp.d_has_listed, n_lead == 0 && sp.n_layers < ctx->L);
  // 2. the listed tiles: ratio pass, layer barrier, update
  LayerSync ls;
  ls.seg_max = ctx->d_seg_max; ls.listed_max = sp.d_listed_max; ls.lt = listed_tiles(ctx, sp);
  ls.counter = sp.d_counter; ls.flag = sp.d_flag; ls.errflag = ctx->d_errflag;
  ls.spin_limit = ctx->spin_limit;
  ls.c_avg = st->c_avg; ls.r_prev = st->r_prev; ls.coeff_c = st->coeff_c;
  ls.one_m_thr = ctx->one_m_thr; ls.one_p_thr = ctx->one_p_thr; ls.r_min = ctx->r_min; ls.r_max = ctx->r_max;
  ls.n_lead = n_lead;
  dispatch2(hk, xl.p != nullptr, [&](auto k_, auto lx) {
#if OB_LB_STREAM
    OB_LAUNCH(la, KID_RATIOS_APPLY_RESIDENT,
              (k_ratios_apply_stream<U_LB, OB_G_LB, decltype(k_)::value, decltype(lx)::value>), sp.n_fused_tiles,
              ra, aa, ls, lt);
#else
    OB_LAUNCH(la, KID_RATIOS_APPLY_RESIDENT,
              (k_ratios_apply_resident<U_LB, decltype(k_)::value, decltype(lx)::value>), sp.n_fused_tiles + n_lead,
              ra, aa, ls, lt);
#endif
  });
  // 3. update of everything outside the listed tiles, with the coefficients of steps 1 and 2
  launch_apply(la, ctx, st, packed_all, server_scales, lr, sp.d_rest_tiles, sp.n_rest_tiles, xl);
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_ratios_apply(ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                               const float* server_scales, float lr, void* hip_stream) {
  return ob_lamb_ratios_apply_lp(ctx, st, packed_all, server_scales, lr, nullptr, OB_F32, hip_stream);
}

}  // extern "C"

namespace {
// The caller's history -> the kernels' (validated; h == NULL: none, write).
ob_status vf_history(const ob_lamb_vf_history* h, VfHist* out) {
  static_assert(OB_VF_MAX_OLD == VF_MAX_OLD, "header and kernels disagree");
  out->n_old = 0;
  out->write_v = 1;
  for (int i = 0; i < VF_MAX_OLD; ++i) {
    out->bits[i] = nullptr;
    out->scales[i] = nullptr;
  }
  if (!h) return OB_OK;
  if (h->n_old < 0 || h->n_old > OB_VF_MAX_OLD) return OB_ERR_ARG;
  for (int i = 0; i < h->n_old; ++i) {
    if (!h->bits[i] || !h->scales[i]) return OB_ERR_NULL;
    if (misaligned(h->bits[i])) return OB_ERR_ALIGN;
    out->bits[i] = h->bits[i];
    out->scales[i] = h->scales[i];
  }
  out->n_old = h->n_old;
  out->write_v = h->write_v ? 1 : 0;
  return OB_OK;
}

RatioArgs ratio_args(const ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                     const float* server_scales, const PackedMom& pm) {
  RatioArgs ra;
  ra.packed = packed_all; ra.sscales = server_scales; ra.m = st->m; ra.pm = pm;
  ra.v_fresh = st->v_fresh; ra.v_frozen = st->v_frozen;
  ra.beta1 = ctx->beta1; ra.omb1 = ctx->omb1; ra.beta2 = ctx->beta2; ra.omb2 = ctx->omb2;
  return ra;
}

VTerms vterms(const ob_lamb_ctx* ctx) {
  VTerms vt;
  vt.t = ctx->d_vterms; vt.pair_base = ctx->d_pair_base; vt.pair_lfirst = ctx->d_pair_lfirst;
  vt.pair_c = ctx->d_pair_c; vt.pair_l = ctx->d_pair_l; vt.n_pairs = ctx->n_pairs;
  return vt;
}

// the two values of every (chunk, layer) pair and step of the history, for the kernels below
void launch_variance_terms(Launch& la, ob_lamb_ctx* ctx, const ob_lamb_state* st, const RatioArgs& ra,
                           const VfHist& vh) {
  const VTerms vt = vterms(ctx);
  dispatch1(st->mom_scale != nullptr, [&](auto hk) {
    OB_LAUNCH(la, KID_VARIANCE_TERMS, (k_variance_terms<decltype(hk)::value>), (ctx->n_pairs + BLOCK - 1) / BLOCK,
              ra, vh, vt, st->mom_scale, ctx->d_vterms);
  });
}

}  // namespace

extern "C" {

ob_status ob_lamb_ratios_apply_hist_lp(ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                                       const float* server_scales, float lr, const ob_lamb_vf_history* h,
                                       void* x_lp, ob_dtype x_dtype, void* hip_stream) {
  if (ob_status s = check_ratios_args(ctx, st, packed_all, server_scales)) return s;
  XLp xl;
  if (ob_status s = x_lp_target(x_lp, x_dtype, &xl)) return s;
  REQUIRE_PTR(st->x);
  if (!std::isfinite(lr)) return OB_ERR_ARG;
  bool packed_m = false;
  PackedMom pm;
  if (ob_status s = momentum_source(st, &packed_m, &pm)) return s;
  if (!packed_m || st->m_packed == packed_all) return OB_ERR_ARG;   // the history is one of 1-bit momenta
  VfHist vh;
  if (ob_status s = vf_history(h, &vh)) return s;
  Launch la(ctx, hip_stream);
  LayerSplit& sp = ctx->sp_apply;
  if (!sp.on && !sp.big_on) {
    // no tile works from the history: the whole array is kept up to date
    launch_ratios(la, ctx, st, packed_all, server_scales, packed_m, pm, nullptr, ctx->n_tiles, nullptr, true);
    launch_apply(la, ctx, st, packed_all, server_scales, lr, nullptr, ctx->n_tiles, xl);
    return la.ok ? OB_OK : OB_ERR_HIP;
  }
  const RatioArgs ra = ratio_args(ctx, st, packed_all, server_scales, pm);
  const ApplyArgs aa = apply_args(ctx, st, packed_all, server_scales, lr, xl);
  const LayerTab lt = layer_tab(ctx, st, ctx->d_first_layer);
  // the three stages of ob_lamb_ratios_apply; the kernel with the per-layer barrier and the ratio
  // pass of the layers that are too large for it work from the history (outside their tiles the plain
  // ratio pass keeps the array up to date at every step: on 1024-element tiles that pass is bound by
  // its launch shape, not by the bytes it moves).  Without the barrier kernel (OB_CFG_NO_FUSED_APPLY)
  // every layer with enough whole tiles counts as too large: no wait anywhere, and still no rewrite
  // of the array at every step.
  // launch 1: the two values of every (chunk, layer) pair and step of the history (leading workgroups)
  // and the plain ratio pass outside the tiles that work from the history
  const int n_lead_vt = (ctx->n_pairs + BLOCK - 1) / BLOCK;
  dispatch1(st->mom_scale != nullptr, [&](auto hk) {
    OB_LAUNCH(la, KID_RATIOS_PASS, (k_ratios_pass_vterms<U_MAIN, decltype(hk)::value>),
              sp.n_rest_ratio_tiles + n_lead_vt, ra, ctx->d_seg_max, ctx->n_c, ctx->tpc, lt, ctx->d_tile_seg0,
              ctx->d_seg_layer, sp.d_rest_ratio_tiles, vh, vterms(ctx), ctx->d_vterms, n_lead_vt);
  });
  // launch 2: ratio pass of the layers that are too large for the barrier kernel, from the history
  if (sp.big_on)
    OB_LAUNCH(la, KID_RATIOS_BIG_HIST, k_ratios_big_hist, sp.n_big_tiles, ra, vh, vterms(ctx), ctx->d_seg_max,
              sp.d_big_tiles, ctx->n_c, sp.tpc, ctx->tpc, lt, ctx->d_tile_seg0);
  if (!sp.on) {
    OB_LAUNCH_B(la, KID_RATIOS_FINALIZE, k_ratios_finalize, (int)ctx->L, FBLOCK, ctx->d_seg_max,
                ctx->d_layer_seg0, st->c_avg, st->r_prev, st->coeff_c, ctx->one_m_thr, ctx->one_p_thr,
                ctx->r_min, ctx->r_max, (const unsigned char*)nullptr);
    launch_apply(la, ctx, st, packed_all, server_scales, lr, nullptr, ctx->n_tiles, xl);
    return la.ok ? OB_OK : OB_ERR_HIP;
  }
  // launch 3: the barrier kernel; its leading workgroups finish the layers without listed tiles (lines
  // 18-20 from the segment maxima that launches 1 and 2 left), the others the listed tiles
  LayerSync ls;
  ls.seg_max = ctx->d_seg_max; ls.listed_max = sp.d_listed_max; ls.lt = listed_tiles(ctx, sp);
  ls.counter = sp.d_counter; ls.flag = sp.d_flag; ls.errflag = ctx->d_errflag;
  ls.spin_limit = ctx->spin_limit;
  ls.c_avg = st->c_avg; ls.r_prev = st->r_prev; ls.coeff_c = st->coeff_c;
  ls.one_m_thr = ctx->one_m_thr; ls.one_p_thr = ctx->one_p_thr; ls.r_min = ctx->r_min; ls.r_max = ctx->r_max;
  ls.n_lead = (sp.n_layers < ctx->L) ? (int)ctx->L : 0;
  dispatch2(st->mom_scale != nullptr, xl.p != nullptr, [&](auto k_, auto lx) {
    OB_LAUNCH(la, KID_RATIOS_APPLY_HIST, (k_ratios_apply_hist<decltype(k_)::value, decltype(lx)::value>),
              sp.n_fused_tiles + ls.n_lead, ra, vh, vterms(ctx), aa, ls, lt);
  });
  launch_apply(la, ctx, st, packed_all, server_scales, lr, sp.d_rest_tiles, sp.n_rest_tiles, xl);
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_ratios_apply_hist(ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                                    const float* server_scales, float lr, const ob_lamb_vf_history* h,
                                    void* hip_stream) {
  return ob_lamb_ratios_apply_hist_lp(ctx, st, packed_all, server_scales, lr, h, nullptr, OB_F32, hip_stream);
}

ob_status ob_lamb_variance_dense(ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                                 const float* server_scales, const ob_lamb_vf_history* h, float* v_out,
                                 void* hip_stream) {
  if (ob_status s = check_common(ctx, st)) return s;
  REQUIRE_PTR(packed_all); REQUIRE_PTR(st->v_fresh); REQUIRE_PTR(st->v_frozen); REQUIRE_PTR(v_out);
  if (!server_scales) return OB_ERR_NULL;
  bool packed_m = false;
  PackedMom pm;
  if (ob_status s = momentum_source(st, &packed_m, &pm)) return s;
  if (!packed_m || st->m_packed == packed_all) return OB_ERR_ARG;
  VfHist vh;
  if (ob_status s = vf_history(h, &vh)) return s;
  vh.write_v = (v_out == st->v_fresh) ? 1 : 0;   // in place: through the array's own pointer
  Launch la(ctx, hip_stream);
  if (!vh.write_v) {   // everything outside the listed tiles is up to date in the array itself
    la.begin(KID_COPY, true);
    if (la.ok)
      la.ok = hip_ok(ctx, hipMemcpyAsync(v_out, st->v_fresh, (size_t)ctx->n_pad * sizeof(float),
                                         hipMemcpyDeviceToDevice, la.stream), "hipMemcpyAsync");
    la.end("copy", true);
  }
  LayerSplit& sp = ctx->sp_apply;
  if ((sp.on || sp.big_on) && sp.n_cov_tiles > 0) {
    const RatioArgs ra = ratio_args(ctx, st, packed_all, server_scales, pm);
    const LayerTab lt = layer_tab(ctx, st, ctx->d_first_layer);
    launch_variance_terms(la, ctx, st, ra, vh);
    OB_LAUNCH(la, KID_VARIANCE_DENSE, k_variance_dense, sp.n_cov_tiles, ra, vh, vterms(ctx),
              vh.write_v ? (float*)nullptr : v_out, ctx->n_c, ctx->tpc, lt, sp.d_cov_tiles);
  }
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_momentum_dense(ob_lamb_ctx* ctx, const ob_lamb_state* st, float* m_out, void* hip_stream) {
  if (ob_status s = check_common(ctx, st)) return s;
  REQUIRE_PTR(m_out); REQUIRE_PTR(st->m_packed);
  if (!st->m_scales) return OB_ERR_NULL;
  PackedMom pm;
  pm.bits = st->m_packed;
  pm.scales = st->m_scales;
  Launch la(ctx, hip_stream);
  const LayerTab lt = layer_tab(ctx, st, ctx->d_first_layer);
  if (st->mom_scale)
    OB_LAUNCH(la, KID_MOMENTUM_DENSE, (k_momentum_dense<U_MAIN, true>), ctx->n_tiles, pm, m_out, ctx->n_c,
              ctx->tpc, lt);
  else
    OB_LAUNCH(la, KID_MOMENTUM_DENSE, (k_momentum_dense<U_MAIN, false>), ctx->n_tiles, pm, m_out, ctx->n_c,
              ctx->tpc, lt);
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_error_dense(ob_lamb_ctx* ctx, const ob_lamb_state* st, float* err_out, void* hip_stream) {
  if (ob_status s = check_common(ctx, st)) return s;
  REQUIRE_PTR(err_out); REQUIRE_PTR(st->err_worker); REQUIRE_PTR(st->err_packed);
  if (!st->err_scales) return OB_ERR_NULL;
  PackedErr pe;
  pe.bits = st->err_packed; pe.scales = st->err_scales;
  Launch la(ctx, hip_stream);
  OB_LAUNCH(la, KID_ERROR_DENSE, k_error_dense, ctx->n_tiles, st->err_worker, pe, err_out, ctx->n_c, ctx->tpc);
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_server_error_dense(ob_lamb_ctx* ctx, const ob_lamb_state* st, float* err_out,
                                     void* hip_stream) {
  if (ob_status s = check_common(ctx, st)) return s;
  REQUIRE_PTR(err_out); REQUIRE_PTR(st->err_server); REQUIRE_PTR(st->srv_err_packed);
  if (!st->srv_err_scale) return OB_ERR_NULL;
  PackedErr pe;
  pe.bits = st->srv_err_packed; pe.scales = st->srv_err_scale;
  Launch la(ctx, hip_stream);
  // the served chunk as a one-chunk buffer
  OB_LAUNCH(la, KID_ERROR_DENSE, k_error_dense, ctx->tpc_srv, st->err_server, pe, err_out, ctx->n_c,
            ctx->tpc_srv);
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_momentum_scale(ob_lamb_ctx* ctx, const ob_lamb_state* st, void* hip_stream) {
  if (ob_status s = check_common(ctx, st)) return s;
  REQUIRE_PTR(st->m);
  if (!st->mom_scale) return OB_ERR_NULL;
  Launch la(ctx, hip_stream);
  const LayerTab lt = layer_tab(ctx, st, ctx->d_first_layer);
  constexpr int R = 8;   // tiles per workgroup
  static_assert(U_MAIN == 1, "the segment tables are those of the 1024-element tiling");
  OB_LAUNCH(la, KID_MOMENTUM_SCALE, (k_momentum_sumsq<R>), (ctx->n_tiles + R - 1) / R, st->m, ctx->d_seg_sums,
            ctx->n_c, ctx->tpc, ctx->n_tiles, lt, ctx->d_tile_seg0, ctx->d_seg_layer);
  OB_LAUNCH_B(la, KID_MOMENTUM_SCALE, k_layer_rms, (int)ctx->L, FBLOCK, ctx->d_seg_sums, ctx->d_layer_seg0,
              ctx->d_off, ctx->d_sigma);
  OB_LAUNCH_B(la, KID_MOMENTUM_SCALE, k_momentum_scale, 1, FBLOCK, ctx->d_sigma, ctx->d_off, (int)ctx->L,
              st->mom_scale);
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_check_device_status(ob_lamb_ctx* ctx, void* hip_stream) {
  if (!ctx) return OB_ERR_NULL;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  unsigned int f = 0;
  if (!hip_ok(ctx, hipStreamSynchronize(stream), "hipStreamSynchronize") ||
      !hip_ok(ctx, hipMemcpy(&f, ctx->d_errflag, sizeof(f), hipMemcpyDeviceToHost), "hipMemcpy"))
    return OB_ERR_HIP;
  if (f == 0) return OB_OK;
  // a bounded wait expired: the step that raised it produced undefined outputs.  Re-arm the
  // synchronisation state and fall back to the two-pass kernels for the rest of this context.
  ctx->resident = false;
  ctx->u_srv_res = 0;
  (void)hipMemset(ctx->d_counter_srv, 0, sizeof(unsigned long long) * CTR_STRIDE);
  (void)hipMemset(ctx->d_flag_srv, 0, sizeof(unsigned long long));
  for (LayerSplit* sp : {&ctx->sp_apply, &ctx->sp_warm}) {
    sp->on = false;
    sp->big_on = false;   // (no wait in that pass; but after an expiry every call takes the plain kernels)
    (void)hipMemset(sp->d_counter, 0, sizeof(unsigned long long) * (size_t)ctx->L * CTR_STRIDE);
    (void)hipMemset(sp->d_flag, 0, sizeof(unsigned long long) * (size_t)ctx->L);
  }
  (void)hipMemset(ctx->d_counter, 0, sizeof(unsigned long long) * (size_t)ctx->W * CTR_STRIDE);
  (void)hipMemset(ctx->d_flag, 0, sizeof(unsigned long long) * (size_t)ctx->W);
  (void)hipMemset(ctx->d_errflag, 0, sizeof(unsigned int));
  (void)hipDeviceSynchronize();
  return OB_ERR_STATE;
}

int64_t ob_lamb_fused_layers(const ob_lamb_ctx* ctx) { return (ctx && ctx->sp_apply.on) ? ctx->sp_apply.n_layers : 0; }
int64_t ob_lamb_fused_params(const ob_lamb_ctx* ctx) { return (ctx && ctx->sp_apply.on) ? ctx->sp_apply.n_params : 0; }
int64_t ob_lamb_big_tile_params(const ob_lamb_ctx* ctx) { return (ctx && ctx->sp_apply.big_on) ? ctx->sp_apply.n_big_params : 0; }
int64_t ob_lamb_warmup_fused_layers(const ob_lamb_ctx* ctx) { return (ctx && ctx->sp_warm.on) ? ctx->sp_warm.n_layers : 0; }
int64_t ob_lamb_warmup_fused_params(const ob_lamb_ctx* ctx) { return (ctx && ctx->sp_warm.on) ? ctx->sp_warm.n_params : 0; }

int32_t ob_lamb_uses_single_pass(const ob_lamb_ctx* ctx) { return (ctx && ctx->resident) ? 1 : 0; }
int32_t ob_lamb_server_single_pass(const ob_lamb_ctx* ctx) { return ctx ? ctx->u_srv_res : 0; }

ob_status ob_lamb_profile_enable(ob_lamb_ctx* ctx, int on) {
  if (!ctx) return OB_ERR_NULL;
  ctx->profile = (on != 0);
  return OB_OK;
}

int32_t ob_lamb_profile_read(ob_lamb_ctx* ctx, int32_t cap, const char** names, double* total_ms,
                             int64_t* launches) {
  if (!ctx) return 0;
  double ms[KID_COUNT] = {0};
  int64_t cnt[KID_COUNT] = {0};
  for (auto& r : ctx->prof) {
    float t = 0.0f;
    if (hipEventSynchronize(r.e1) == hipSuccess && hipEventElapsedTime(&t, r.e0, r.e1) == hipSuccess) {
      ms[r.kid] += t;
      cnt[r.kid] += 1;
    }
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  ctx->prof.clear();
  int32_t n = 0;
  for (int k = 0; k < KID_COUNT; ++k) {
    if (!cnt[k]) continue;
    if (n < cap) {
      if (names) names[n] = kKernelNames[k];
      if (total_ms) total_ms[n] = ms[k];
      if (launches) launches[n] = cnt[k];
    }
    ++n;
  }
  return n;
}

}  // extern "C"

// ---- Algorithm 1 line 10 for callers that cannot allocate -------------------------------------
// ob_lamb_server_reduce needs a context, whose creation allocates the partial sums that its
// kernels pass from the averaging pass to the scale.  This variant keeps them in a fixed array in
// the library's own device image instead: no context, no allocation of any kind.
namespace {
constexpr int64_t STATIC_MAX_CHUNK = (int64_t)1 << 25;                 // elements of the served chunk
constexpr int64_t STATIC_MAX_TILES = STATIC_MAX_CHUNK / TILE_SRV;      // 32768 partial sums = 256 KiB
}
// One copy per GPU the library runs on, alive until the process ends.  In host code this name is
// only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) double scratch[STATIC_MAX_TILES];

namespace {
constexpr int STATIC_MAX_DEVICES = 64;
std::mutex g_scratch_mu;
double* g_scratch_ptr[STATIC_MAX_DEVICES] = {};   // per device: the address of ITS copy of `scratch`

// Device address of the current device's scratch array (looked up once per device).
ob_status static_scratch(double** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return OB_ERR_HIP;
  if (dev < 0 || dev >= STATIC_MAX_DEVICES) return OB_ERR_ARG;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return OB_ERR_HIP;
    g_scratch_ptr[dev] = static_cast<double*>(p);
  }
  *out = g_scratch_ptr[dev];
  return OB_OK;
}
}  // namespace

extern "C" {

int64_t ob_lamb_static_max_chunk_len(void) { return STATIC_MAX_CHUNK; }

ob_status ob_lamb_diag_copy(const float* src, float* dst, int64_t n, void* hip_stream) {
  if (n < 0 || n > ((int64_t)1 << 40)) return OB_ERR_ARG;
  REQUIRE_PTR(src); REQUIRE_PTR(dst);
  if (n == 0) return OB_OK;
  const int64_t tiles = (n + SPAN - 1) / SPAN;
  if (tiles > 0x7fffffff) return OB_ERR_ARG;
  hipLaunchKernelGGL(k_diag_copy, dim3((unsigned)tiles), dim3(BLOCK), 0, reinterpret_cast<hipStream_t>(hip_stream),
                     src, dst, n);
  return hipGetLastError() == hipSuccess ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_server_reduce_static(int32_t num_workers, int64_t chunk_len, const uint32_t* packed_in,
                                       const float* scales_in, float* err_server, uint32_t* packed_out,
                                       float* scale_out, void* hip_stream) {
  if (num_workers < 1 || num_workers > 65536 || chunk_len < 256 || chunk_len % 256 != 0) return OB_ERR_ARG;
  if (chunk_len > STATIC_MAX_CHUNK) return OB_ERR_SIZE;
  if ((int64_t)num_workers * (chunk_len / 8) >= ((int64_t)1 << 31)) return OB_ERR_SIZE;   // 32-bit offsets into packed_in
  REQUIRE_PTR(packed_in); REQUIRE_PTR(packed_out); REQUIRE_PTR(err_server);
  if (!scales_in || !scale_out) return OB_ERR_NULL;
  double* partials = nullptr;
  if (ob_status s = static_scratch(&partials)) return s;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const int tiles = (int)((chunk_len + TILE_SRV - 1) / TILE_SRV);   // <= STATIC_MAX_TILES
  const float invW = 1.0f / (float)num_workers;
  // the three kernels of ob_lamb_server_reduce's barrier-free form; every partial that the second
  // reads has been written by the first, so the array's previous contents do not matter
  hipLaunchKernelGGL((k_server_unpack_avg<U_SRV>), dim3((unsigned)tiles), dim3(BLOCK), 0, stream, packed_in,
                     scales_in, err_server, partials, chunk_len, (int)num_workers, invW, (uint32_t*)nullptr,
                     (const float*)nullptr, (uint32_t*)nullptr);
  hipLaunchKernelGGL(k_chunk_scale, dim3(1), dim3(FBLOCK), 0, stream, partials, tiles, chunk_len, scale_out,
                     (float*)nullptr, 0);
  hipLaunchKernelGGL((k_sign_pack_error<U_SRV>), dim3((unsigned)tiles), dim3(BLOCK), 0, stream, err_server,
                     packed_out, scale_out, chunk_len, tiles);
  return hipGetLastError() == hipSuccess ? OB_OK : OB_ERR_HIP;
}

}  // extern "C"
