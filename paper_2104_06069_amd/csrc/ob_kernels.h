// Device code of libonebitlamb (gfx950): every kernel of the compression-stage step of 1-bit LAMB
// (arXiv 2104.06069, Algorithm 1) and of the LAMB warmup step (eq. (1)).  Included by
// onebitlamb.hip only.
//
// Arithmetic contract: IEEE binary32, one rounding per operation (the build passes
// -ffp-contract=off; hipcc's default divide and sqrt are correctly rounded), evaluated in the
// operation order written below; the sum-of-squares reductions accumulate in binary64 in a fixed
// order.  Never build with -ffast-math.
//
// Layout of the work.  The padded flat buffer is W chunks of n_c elements (n_c % 256 == 0).
// Every N-sized kernel runs on "tiles": tile (c, b) is elements [c*n_c + b*TILE, +TILE) clipped
// to the chunk, so a tile never crosses a chunk boundary and its length is a multiple of 256.
// A workgroup of 256 threads owns one tile; thread t touches elements tile0 + u*1024 + 4*t + k
// (u < U, k < 4) with 128-bit accesses, i.e. each wavefront-wide access covers 256 consecutive
// elements = 8 consecutive 32-bit words of a packed sign stream.
//
// Layers (tensors) are arbitrary, unaligned ranges of the flat buffer.  A host-built table gives
// the layer of each tile's first element (L = padding); a tile that lies inside one layer takes a
// vectorised path with per-tile scalars, a tile that meets a layer boundary or the end of the
// parameters takes a per-element path that walks the offset table.
//
// The momentum m_{t-1} has two sources: a dense fp32 array, or (template flag PACKED_M) the 1-bit
// form it has had since line 13 of the previous step: m[i] = (bit ? +s_c : -s_c) / k_l for
// i < N and 0 in the padding, where s_c is the previous step's server scale of chunk c.  Both give
// the same bits: the dense array holds exactly those values.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

namespace obk {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int BLOCK = 256;       // threads per workgroup (4 wavefronts of 64)
constexpr int WAVE = 64;
constexpr int SPAN = BLOCK * 4;  // elements one workgroup-wide 128-bit access covers
constexpr int FBLOCK = 1024;     // threads per workgroup of the small per-layer / per-chunk finalize kernels
#define OB_AGENT __HIP_MEMORY_SCOPE_AGENT
// Arrival counters of different chunks / layers sit 128 bytes apart: read-modify-write atomics on one
// cache line are served one at a time (12 ns each, measured), whichever word of it they address,
// and several chunks or layers are always in flight together.
constexpr int CTR_STRIDE = 16;   // in 8-byte words
#ifndef OB_POLL_SLEEP
#define OB_POLL_SLEEP 16  // s_sleep argument (units of 64 clocks) between two polls of a barrier flag
#endif

// Every N-sized array is read once and written once per kernel: 128-bit nontemporal (streaming)
// accesses, which measure ~10 % faster than plain ones on MI355X for these patterns.
__device__ __forceinline__ v4f ld4(const float* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
}
__device__ __forceinline__ void st4(float* p, v4f v) {
  __builtin_nontemporal_store(v, reinterpret_cast<v4f*>(p));
}

// 16-bit storage of the mixed-precision variant (the paper trains in FP16, Section 6): a gradient
// may arrive as IEEE binary16 or bfloat16 and a 16-bit copy of the parameters may be written; all
// arithmetic stays binary32.  GT / LPX are template flags so that the fp32-only instantiations
// keep their code.
typedef unsigned short v4h __attribute__((ext_vector_type(4)));

struct GradSrc {
  const void* __restrict__ p;   // float (GT == 0) or 16-bit patterns (GT == 1)
  float scale;                  // g = value * scale (GT == 1 only; the inverse loss scale)
  int bf16;                     // GT == 1: 0 = binary16, 1 = bfloat16
};

__device__ __forceinline__ float lp_to_float(unsigned short h, int bf16) {
  if (bf16) return __uint_as_float((unsigned int)h << 16);
  return (float)__builtin_bit_cast(_Float16, h);   // exact
}

// binary32 -> nearest 16-bit value, ties to even; NaN -> the format's canonical quiet NaN
__device__ __forceinline__ unsigned short float_to_lp(float x, int bf16) {
  if (bf16) {
    const unsigned int u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)0x7fc0;
    return (unsigned short)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
  }
  if (x != x) return (unsigned short)0x7e00;
  return __builtin_bit_cast(unsigned short, (_Float16)x);   // hardware convert, round to nearest even
}

// The thread's 4 gradient values at flat index i (a multiple of 4).
template <int GT>
__device__ __forceinline__ v4f load_grad(const GradSrc& gs, int64_t i) {
  if (GT == 0) return ld4(reinterpret_cast<const float*>(gs.p) + i);
  const v4h h = __builtin_nontemporal_load(
      reinterpret_cast<const v4h*>(reinterpret_cast<const unsigned short*>(gs.p) + i));
  v4f r;
#pragma unroll
  for (int k = 0; k < 4; ++k) r[k] = lp_to_float(h[k], gs.bf16) * gs.scale;
  return r;
}

__device__ __forceinline__ void st4_lp(void* __restrict__ base, int64_t i, v4f v, int bf16) {
  v4h h;
#pragma unroll
  for (int k = 0; k < 4; ++k) h[k] = float_to_lp(v[k], bf16);
  __builtin_nontemporal_store(h, reinterpret_cast<v4h*>(reinterpret_cast<unsigned short*>(base) + i));
}

// Sum of one double per thread over a workgroup of NT threads, in a fixed order; result valid in
// thread 0.  lds: [NT / WAVE] doubles.
template <int NT = BLOCK>
__device__ __forceinline__ double block_sum(double v, double* lds) {
#pragma unroll
  for (int o = WAVE / 2; o > 0; o >>= 1) v += __shfl_down(v, o, WAVE);
  const int lane = threadIdx.x & (WAVE - 1), wv = threadIdx.x / WAVE;
  __syncthreads();  // protects lds against the previous use
  if (lane == 0) lds[wv] = v;
  __syncthreads();
  double r = 0.0;
  if (threadIdx.x == 0) {
#pragma unroll
    for (int i = 0; i < NT / WAVE; ++i) r += lds[i];
  }
  return r;
}

// Max of one non-NaN, non-negative float per thread over a workgroup of NT threads; valid in
// thread 0.  lds: [NT / WAVE] floats.
template <int NT = BLOCK>
__device__ __forceinline__ float block_max(float v, float* lds) {
#pragma unroll
  for (int o = WAVE / 2; o > 0; o >>= 1) {
    const float w = __shfl_down(v, o, WAVE);
    v = (w > v) ? w : v;
  }
  const int lane = threadIdx.x & (WAVE - 1), wv = threadIdx.x / WAVE;
  __syncthreads();
  if (lane == 0) lds[wv] = v;
  __syncthreads();
  float r = 0.0f;
  if (threadIdx.x == 0) {
#pragma unroll
    for (int i = 0; i < NT / WAVE; ++i) r = (lds[i] > r) ? lds[i] : r;
  }
  return r;
}

// off has L+2 entries, off[L+1] = INT64_MAX, so the walk stops at L (= padding) at the latest.
__device__ __forceinline__ int walk_layer(int l, int64_t i, const int64_t* __restrict__ off) {
  while (i >= off[l + 1]) ++l;
  return l;
}

// Sign nibble of the lane's 4 elements -> the 32-bit word of its 8-lane group (in every lane of
// the group).  Element 4*lane + k of the 256-element span is bit 4*(lane%8) + k of word lane/8.
__device__ __forceinline__ unsigned int gather_word(unsigned int nibble) {
  unsigned int v = nibble << (4 * (threadIdx.x & 7));
  v |= __shfl_xor(v, 1, WAVE);
  v |= __shfl_xor(v, 2, WAVE);
  v |= __shfl_xor(v, 4, WAVE);
  return v;
}

// The lane's sign nibble from a packed stream: the bits of elements span0 + 4*threadIdx.x + k,
// span0 uniform and a multiple of 1024.
__device__ __forceinline__ unsigned int load_nibble(const uint32_t* __restrict__ packed, int64_t span0) {
  return (packed + (span0 >> 5))[threadIdx.x >> 3] >> (4 * (threadIdx.x & 7));  // bits 0..3 are the lane's
}

struct TilePos {
  int t;          // tile index (chunk-major)
  int c;          // chunk
  int64_t tile0;  // first element
  int len;        // elements in the tile (multiple of 256)
};

// Tile t of the tiling with TILE elements per tile and tpc tiles per chunk.
template <int TILE>
__device__ __forceinline__ TilePos tile_pos(int64_t n_c, int tpc, int t) {
  TilePos p;
  p.t = t;
  p.c = t / tpc;
  const int b = t - p.c * tpc;
  const int64_t in_chunk = (int64_t)b * TILE;
  p.tile0 = (int64_t)p.c * n_c + in_chunk;
  const int64_t rest = n_c - in_chunk;
  p.len = rest < TILE ? (int)rest : TILE;
  return p;
}

// Per-layer tables (device pointers) shared by the layer-aware kernels.
struct LayerTab {
  const float* __restrict__ mom_scale;   // [L] k_l of Appendix A.5.2 (only read when HAS_K)
  const int64_t* __restrict__ off;       // [L+2]
  const int* __restrict__ first_layer;   // [tiles of the launching kernel's tile size]
  int L;
};

// The layer-wise N-sized kernels take an optional tile list: the launch then covers tile
// tile_list[blockIdx.x] instead of tile blockIdx.x (the tiles outside the ones a kernel with a
// per-layer barrier handles).
__device__ __forceinline__ int listed_tile(const int* __restrict__ tile_list) {
  return tile_list ? tile_list[blockIdx.x] : (int)blockIdx.x;
}

// Momentum source in 1-bit form (only read when PACKED_M).
struct PackedMom {
  const uint32_t* __restrict__ bits;     // [N_pad/32]
  const float* __restrict__ scales;      // [W]
};

// Second destination of the worker's chunk `chunk` (see ob_lamb_state.own_packed_in); packed == NULL: none.
struct OwnCopy {
  uint32_t* packed;   // [n_c/32]
  float* scale;       // [1]
  int chunk;
};

// The worker error in deferred form (only read when DEFER): err holds z of the previous step, and
// delta = z - C[z] is formed on the fly from the previous step's own sign words and chunk scales,
// delta[i] = err[i] - (bit_i ? s_c : -s_c) -- the very subtraction of Algorithm 1 line 7, one step
// late.  With all scales 0 the array is the error itself (x - (+-0) = x).
struct PackedErr {
  const uint32_t* bits;     // [N_pad/32] this worker's own previous output (may be packed_out itself)
  const float* scales;      // [W]        ... and its scales (may be scales_out itself)
};

__device__ __forceinline__ v4f deferred_error(v4f e, unsigned int nib, float s) {
  v4f r;
#pragma unroll
  for (int k = 0; k < 4; ++k) r[k] = e[k] - (((nib >> k) & 1u) ? s : -s);
  return r;
}

// ---------------------------------------------------------------------------------------------
// z = k_l * (beta1*m + (1-beta1)*g) + err       (Algorithm 1 lines 6-7, Appendix A.5.2)
// Per-tile constants and the per-access evaluation, shared by the two-pass and single-pass kernels.
// ---------------------------------------------------------------------------------------------
template <bool HAS_K, bool PACKED_M>
struct ZTile {
  bool uniform;  // one set of constants serves the whole tile
  bool pad;      // the whole tile lies in the padding
  int l0;        // layer of the tile's first element (HAS_K)
  float kt;      // k of the tile's layer (uniform tiles)
  float bm;      // beta1 * |m| (PACKED_M; for HAS_K only on uniform tiles)
  float s_prev;  // previous server scale of the chunk (PACKED_M)
  int64_t N;
  // layer cursor of the per-element path (HAS_K, tile meets a layer boundary)
  int cur_l;
  int64_t cur_end;
  float cur_k, cur_b;
  bool cur_real;

  __device__ __forceinline__ void init(const LayerTab& lt, const PackedMom& pm, const TilePos& p,
                                       float beta1) {
    uniform = true; pad = false; l0 = 0; kt = 1.0f; bm = 0.0f; s_prev = 0.0f; N = 0;
    cur_l = 0; cur_end = 0; cur_k = 1.0f; cur_b = 0.0f; cur_real = false;
    if (PACKED_M) s_prev = pm.scales[p.c];
    if (HAS_K) {
      // k differs from layer to layer: the tile must lie inside one layer (or in the padding)
      l0 = lt.first_layer[p.t];
      uniform = (p.tile0 + p.len <= lt.off[l0 + 1]);
      pad = (l0 >= lt.L);
      if (uniform && !pad) {
        kt = lt.mom_scale[l0];
        if (PACKED_M) bm = beta1 * (s_prev / kt);
      }
      if (!uniform) {  // l0 < L here: a tile that starts in the padding is uniform
        cur_l = l0;
        cur_end = lt.off[l0 + 1];
        cur_real = true;
        cur_k = lt.mom_scale[l0];
        if (PACKED_M) cur_b = beta1 * (s_prev / cur_k);
      }
    } else if (PACKED_M) {
      // only the end of the parameters matters: the 1-bit momentum is 0 in the padding
      N = lt.off[lt.L];
      pad = (p.tile0 >= N);
      uniform = pad || (p.tile0 + p.len <= N);
      bm = beta1 * s_prev;
    }
  }

  // G, E: gradient and carried error; M: dense momentum (ignored when PACKED_M); nib: the sign
  // bits of the packed momentum (ignored otherwise); i0: flat index of the first element.
  // Calls must come in increasing i0 for one thread (the per-element path keeps a cursor).
  // KNOWN_UNIFORM: the caller has tested `uniform` itself (a copy of its loop without the other
  // paths in it).
  template <bool KNOWN_UNIFORM = false>
  __device__ __forceinline__ v4f z(const LayerTab& lt, float beta1, float omb1, v4f G, v4f M,
                                   unsigned int nib, v4f E, int64_t i0) {
    v4f r;
    if (KNOWN_UNIFORM || uniform) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        float bmk;
        if (PACKED_M) bmk = pad ? 0.0f : (((nib >> k) & 1u) ? bm : -bm);
        else bmk = beta1 * M[k];
        const float mloc = bmk + omb1 * G[k];
        r[k] = HAS_K ? kt * mloc + E[k] : mloc + E[k];
      }
    } else if (HAS_K) {
      // A thread's elements come in increasing order over the whole tile, so the layer cursor
      // only moves forward and its constants are re-formed only when a boundary is crossed.
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int64_t i = i0 + k;
        if (i >= cur_end) {
          do {
            ++cur_l;
            cur_end = lt.off[cur_l + 1];
          } while (i >= cur_end);
          cur_real = (cur_l < lt.L);
          cur_k = cur_real ? lt.mom_scale[cur_l] : 1.0f;
          if (PACKED_M) cur_b = beta1 * (s_prev / cur_k);
        }
        float bmk;
        if (PACKED_M) bmk = cur_real ? (((nib >> k) & 1u) ? cur_b : -cur_b) : 0.0f;
        else bmk = beta1 * M[k];
        const float mloc = bmk + omb1 * G[k];
        r[k] = cur_k * mloc + E[k];
      }
    } else {  // PACKED_M without k: the tile straddles the end of the parameters
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float bmk = (i0 + k < N) ? (((nib >> k) & 1u) ? bm : -bm) : 0.0f;
        r[k] = (bmk + omb1 * G[k]) + E[k];
      }
    }
    return r;
  }
};

// ---------------------------------------------------------------------------------------------
// K1  z written over err, and the tile's sum of z^2 in fp64: the first of the two passes of the
// worker compression (k_sign_pack_error is the second), or, with DEFER, all of it.
// ---------------------------------------------------------------------------------------------
// DEFER: the whole of lines 6-7 in this one pass, with no wait for the chunk's scale: the carried
// error arrives in deferred form (PackedErr), z is written over it AS the next deferred error, and
// the sign words of z are packed and written here as well (they do not depend on the scale); the
// scale itself follows from the tile partials in k_chunk_scale.  packed_out / pe.bits may be the
// same buffer: a word is read and rewritten by the same 8 lanes, in program order.
template <int U, bool HAS_K, bool PACKED_M, int GT = 0, bool DEFER = false>
__global__ __launch_bounds__(BLOCK) void k_momentum_z_sumsq(
    GradSrc g, const float* __restrict__ m, PackedMom pm,
    float* __restrict__ err, double* __restrict__ partials, int64_t n_c, int tpc, float beta1,
    float omb1, LayerTab lt, PackedErr pe, uint32_t* packed_out, OwnCopy oc) {
  constexpr int TILE = SPAN * U;
  __shared__ double lds[BLOCK / WAVE];
  const TilePos p = tile_pos<TILE>(n_c, tpc, (int)blockIdx.x);
  const int o0 = threadIdx.x * 4;
  const float se = DEFER ? pe.scales[p.c] : 0.0f;
  v4f G[U], M[U], E[U];
  unsigned int NB[U], EB[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    M[u] = 0.0f; NB[u] = 0u; EB[u] = 0u;
    if (o < p.len) {
      G[u] = load_grad<GT>(g, p.tile0 + o);
      if (PACKED_M) NB[u] = load_nibble(pm.bits, p.tile0 + u * SPAN);
      else M[u] = ld4(m + p.tile0 + o);
      if (DEFER) EB[u] = load_nibble(pe.bits, p.tile0 + u * SPAN);
      E[u] = ld4(err + p.tile0 + o);
    }
  }
  ZTile<HAS_K, PACKED_M> zt;
  zt.init(lt, pm, p, beta1);
  uint32_t* own = (DEFER && oc.packed && p.c == oc.chunk) ? oc.packed : nullptr;   // uniform
  const int64_t own_tile0 = (p.tile0 - (int64_t)p.c * n_c) >> 5;
  double acc = 0.0;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {   // uniform over the wavefront (len is a multiple of 256), as the shuffles below require
      if (DEFER) E[u] = deferred_error(E[u], EB[u], se);
      const v4f z = zt.z(lt, beta1, omb1, G[u], M[u], NB[u], E[u], p.tile0 + o);
      st4(err + p.tile0 + o, z);
      unsigned int nib = 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        acc += (double)z[k] * (double)z[k];
        if (DEFER) nib |= ((z[k] >= 0.0f) ? 1u : 0u) << k;
      }
      if (DEFER) {
        const unsigned int word = gather_word(nib);
        if ((threadIdx.x & 7) == 0) {
          const int64_t span0 = p.tile0 + u * SPAN;
          (packed_out + (span0 >> 5))[threadIdx.x >> 3] = word;
          if (own) (own + own_tile0 + u * (SPAN / 32))[threadIdx.x >> 3] = word;
        }
      }
    }
  }
  const double s = block_sum(acc, lds);
  if (threadIdx.x == 0) partials[p.t] = s;
}

// scale[c] = sqrt(sum of the chunk's tile partials / n_c), summed in a fixed order.
// own_scale (may be NULL): also receives the scale of chunk own_chunk.
__global__ __launch_bounds__(FBLOCK) void k_chunk_scale(const double* __restrict__ partials, int tpc,
                                                        int64_t n_c, float* __restrict__ scales,
                                                        float* __restrict__ own_scale, int own_chunk) {
  __shared__ double lds[FBLOCK / WAVE];
  const int c = blockIdx.x;
  double a = 0.0;
  for (int j = threadIdx.x; j < tpc; j += FBLOCK) a += partials[(int64_t)c * tpc + j];
  const double S = block_sum<FBLOCK>(a, lds);
  if (threadIdx.x == 0) {
    const float sc = (float)sqrt(S / (double)n_c);
    scales[c] = sc;
    if (own_scale && c == own_chunk) *own_scale = sc;
  }
}

// Dense view of a worker error held in deferred form: out[i] = err[i] - (bit_i ? s_c : -s_c) over the
// whole padded buffer (out may be err itself).
__global__ __launch_bounds__(BLOCK) void k_error_dense(const float* __restrict__ err, PackedErr pe,
                                                       float* __restrict__ out, int64_t n_c, int tpc) {
  const TilePos p = tile_pos<SPAN>(n_c, tpc, (int)blockIdx.x);
  const int o = threadIdx.x * 4;
  if (o >= p.len) return;
  const float se = pe.scales[p.c];
  const unsigned int nb = load_nibble(pe.bits, p.tile0);
  st4(out + p.tile0 + o, deferred_error(ld4(err + p.tile0 + o), nb, se));
}

// Sign, pack and error update of one 128-bit access held in registers (Algorithm 1 line 7/10).
// span0: flat index of the first element of the workgroup-wide access (uniform, multiple of 1024);
// the thread's elements are span0 + 4*threadIdx.x + k.
// own: if not NULL, the words are also written there at word index own_word0 + (thread's word) (the
// copy of this rank's own chunk in its server's input).
__device__ __forceinline__ void sign_pack_store(v4f z, float s, float* __restrict__ err,
                                                uint32_t* __restrict__ packed, int64_t span0,
                                                uint32_t* __restrict__ own = nullptr, int64_t own_word0 = 0) {
  unsigned int nib = 0;
  v4f e;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const bool b = (z[k] >= 0.0f);
    nib |= (b ? 1u : 0u) << k;
    e[k] = z[k] - (b ? s : -s);
  }
  st4(err + span0 + threadIdx.x * 4, e);
  const unsigned int word = gather_word(nib);
  if ((threadIdx.x & 7) == 0) {
    (packed + (span0 >> 5))[threadIdx.x >> 3] = word;
    if (own) (own + own_word0)[threadIdx.x >> 3] = word;
  }
}

// ---------------------------------------------------------------------------------------------
// K2 (two-pass path)  bits = (z >= 0), packed; err <- z - (+-scale)
// ---------------------------------------------------------------------------------------------
template <int U>
__global__ __launch_bounds__(BLOCK) void k_sign_pack_error(float* __restrict__ err,
                                                           uint32_t* __restrict__ packed,
                                                           const float* __restrict__ scales,
                                                           int64_t n_c, int tpc) {
  constexpr int TILE = SPAN * U;
  const TilePos p = tile_pos<TILE>(n_c, tpc, (int)blockIdx.x);
  const float s = scales[p.c];
  const int o0 = threadIdx.x * 4;
  v4f Z[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) Z[u] = ld4(err + p.tile0 + o);
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    // uniform over the wavefront (len is a multiple of 256), as the shuffles inside require
    if (o < p.len) sign_pack_store(Z[u], s, err, packed, p.tile0 + u * SPAN);
  }
}

// ---------------------------------------------------------------------------------------------
// Per-chunk arrival barrier of the single-pass kernels.
//
// Each workgroup of a chunk publishes one fp64 partial and arrives; the last one to arrive sums
// the chunk's partials in a fixed order, turns the sum into the scale and publishes it; the others
// wait for it.  Returns the chunk's scale to every thread.
//
// Progress: workgroups are dispatched in index order and a chunk's tiles are consecutive indices,
// so the oldest unfinished chunk always has all of its tiles resident or dispatchable provided the
// device can hold one chunk's workgroups at once; the host selects these kernels only when a
// chunk's workgroups take at most 80 % of the device's slots.
// Every wait is bounded by spin_limit polls: on expiry the workgroup raises
// *errflag, uses whatever it last read and goes on to exit, and all later waits end at once.
//
// Synchronisation uses relaxed agent-scope atomics whose payload travels in the atomic itself
// (partials: one double each; flag[c]: generation in the high word, scale bits in the low word),
// so no cache write-back/invalidate is needed; the store of the partial is complete (an explicit s_waitcnt)
// before the arrival counter is incremented.
//
// The barrier carries its own launch numbering, so a launch needs nothing from the host that
// changes from call to call (a captured launch can be replayed): counter[c] holds the generation
// in its high word and the arrivals of the running launch in its low word.  An arriving workgroup
// learns both from its fetch-add; the last one publishes the result under generation + 1 and then
// adds 2^32 - tpc to the counter (arrivals back to 0, generation + 1); the others wait for a flag
// of generation + 1.  All of it wraps harmlessly.
// ---------------------------------------------------------------------------------------------
struct ChunkSync {
  double* partials;             // [tiles of the launching kernel]
  unsigned long long* counter;  // [chunks * CTR_STRIDE] (generation << 32) | arrivals
  unsigned long long* flag;     // [chunks] (generation << 32) | bits of the scale
  unsigned int* errflag;        // [1]
  int spin_limit;
};

// Between a workgroup's publication of its payload (write-through atomic stores) and its arrival:
// the stores have been acknowledged before the arrival is issued, so whoever sees the arrival
// finds the payload.  (A release fence of workgroup scope emits no wait here, and one of agent
// scope would also write back the L2's dirty lines, i.e. the kernel's own streaming stores.)
__device__ __forceinline__ void payload_before_arrival() {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// One arrival at `counter` of a barrier with n participants: returns ((generation + 1) << 32) |
// (1 if this was the last arrival).
__device__ __forceinline__ unsigned long long barrier_arrive(unsigned long long* counter, int n) {
  const unsigned long long prev = __hip_atomic_fetch_add(counter, 1ull, __ATOMIC_RELAXED, OB_AGENT);
  const unsigned int want = (unsigned int)(prev >> 32) + 1u;
  const bool last = ((unsigned int)prev + 1u == (unsigned int)n);
  return ((unsigned long long)want << 32) | (last ? 1ull : 0ull);
}

// The last arrival's publication: flag <- (want << 32) | payload, then the counter is re-armed.
__device__ __forceinline__ unsigned long long barrier_publish(unsigned long long* flag,
                                                              unsigned long long* counter, int n,
                                                              unsigned int want, unsigned int payload) {
  const unsigned long long f = ((unsigned long long)want << 32) | (unsigned long long)payload;
  __hip_atomic_store(flag, f, __ATOMIC_RELAXED, OB_AGENT);
  (void)__hip_atomic_fetch_add(counter, (1ull << 32) - (unsigned long long)n, __ATOMIC_RELAXED, OB_AGENT);
  return f;
}

// Bounded wait (thread 0 of a workgroup) for a flag of generation `want`: at most spin_limit polls
// (0: none, the wait expires at once whatever the flag holds); returns the flag word last read (0
// if none was).  On expiry *errflag is raised; once it is raised every wait ends within 64 polls.
__device__ __forceinline__ unsigned long long barrier_wait(const unsigned long long* flag,
                                                           unsigned int want, unsigned int* errflag,
                                                           int spin_limit) {
  unsigned long long f = 0ull;
  for (int it = 0;; ++it) {
    if (it >= spin_limit) {
      atomicOr(errflag, 1u);
      break;
    }
    f = __hip_atomic_load(flag, __ATOMIC_RELAXED, OB_AGENT);
    if ((unsigned int)(f >> 32) == want) break;
    if ((it & 63) == 63 && __hip_atomic_load(errflag, __ATOMIC_RELAXED, OB_AGENT) != 0u) break;
    __builtin_amdgcn_s_sleep(OB_POLL_SLEEP);
  }
  return f;
}

__device__ __forceinline__ float chunk_barrier_scale(const ChunkSync& cs, int tile, int c, int tpc,
                                                     int64_t n_c, double part, double* lds,
                                                     unsigned long long* bc,
                                                     float* __restrict__ scale_out) {
  unsigned long long* counter = &cs.counter[(int64_t)c * CTR_STRIDE];
  if (threadIdx.x == 0) {
    __hip_atomic_store(&cs.partials[tile], part, __ATOMIC_RELAXED, OB_AGENT);
    payload_before_arrival();
    *bc = barrier_arrive(counter, tpc);
  }
  __syncthreads();
  const bool last = ((*bc & 1ull) != 0ull);
  const unsigned int want = (unsigned int)(*bc >> 32);
  __syncthreads();
  if (last) {
    // four loads in flight per thread: every waiter of the chunk is waiting for this sum (the
    // partials are >= +0, so the zeros that stand in for missing ones change nothing)
    double a = 0.0;
    const double* part_c = cs.partials + (int64_t)c * tpc;
    for (int j = threadIdx.x; j < tpc; j += 4 * BLOCK) {
      double v[4];
#pragma unroll
      for (int q = 0; q < 4; ++q)
        v[q] = (j + q * BLOCK < tpc) ? __hip_atomic_load(&part_c[j + q * BLOCK], __ATOMIC_RELAXED, OB_AGENT) : 0.0;
#pragma unroll
      for (int q = 0; q < 4; ++q) a += v[q];
    }
    const double S = block_sum(a, lds);
    if (threadIdx.x == 0) {
      const float sc = (float)sqrt(S / (double)n_c);
      scale_out[c] = sc;
      *bc = barrier_publish(&cs.flag[c], counter, tpc, want, __float_as_uint(sc));
    }
  } else if (threadIdx.x == 0) {
    *bc = barrier_wait(&cs.flag[c], want, cs.errflag, cs.spin_limit);
  }
  __syncthreads();
  return __uint_as_float((unsigned int)(*bc & 0xffffffffull));
}

// ---------------------------------------------------------------------------------------------
// K1+K2 in one pass: Algorithm 1 lines 6-7 with each input read once.  A workgroup computes z for
// its tile (U*4 registers per thread), goes through the chunk barrier, then signs, packs and writes
// the error from registers.  z never goes to memory.  Loads are issued G accesses at a time to
// bound the staging registers.
// ---------------------------------------------------------------------------------------------
template <int U, int G, bool HAS_K, bool PACKED_M, int MINW = 4, int GT = 0>
__global__ __launch_bounds__(BLOCK, MINW) void k_compress_resident(
    GradSrc g, const float* __restrict__ m, PackedMom pm,
    float* __restrict__ err, uint32_t* __restrict__ packed, float* __restrict__ scales,
    ChunkSync cs, int64_t n_c, int tpc, float beta1, float omb1, LayerTab lt, OwnCopy oc) {
  constexpr int TILE = SPAN * U;
  __shared__ double lds[BLOCK / WAVE];
  __shared__ unsigned long long bc;
  const TilePos p = tile_pos<TILE>(n_c, tpc, (int)blockIdx.x);
  const int o0 = threadIdx.x * 4;
  ZTile<HAS_K, PACKED_M> zt;
  zt.init(lt, pm, p, beta1);
  v4f Z[U];
  double acc = 0.0;
  // (Issuing the next group's loads before evaluating the current one, or a branch-free path for
  // full tiles, measured no faster: the kernel is bound by the barrier, not by load latency.)
  auto stream = [&](auto known_uniform) {
#pragma unroll
    for (int u0 = 0; u0 < U; u0 += G) {
      v4f Gr[G], M[G], E[G];
      unsigned int NB[G];
#pragma unroll
      for (int j = 0; j < G; ++j) {
        const int o = (u0 + j) * SPAN + o0;
        M[j] = 0.0f; NB[j] = 0u;
        if (o < p.len) {
          Gr[j] = load_grad<GT>(g, p.tile0 + o);
          if (PACKED_M) NB[j] = load_nibble(pm.bits, p.tile0 + (u0 + j) * SPAN);
          else M[j] = ld4(m + p.tile0 + o);
          E[j] = ld4(err + p.tile0 + o);
        }
      }
#pragma unroll
      for (int j = 0; j < G; ++j) {
        const int o = (u0 + j) * SPAN + o0;
        if (o < p.len) {
          const v4f z = zt.template z<decltype(known_uniform)::value>(lt, beta1, omb1, Gr[j], M[j], NB[j],
                                                                      E[j], p.tile0 + o);
          Z[u0 + j] = z;
#pragma unroll
          for (int k = 0; k < 4; ++k) acc += (double)z[k] * (double)z[k];
        }
      }
    }
  };
  // With k, a tile inside one layer runs a copy of the loop that holds nothing of the per-element
  // path: every tile of a chunk waits for the chunk's slowest one, and with the layer cursor of
  // that path in the same loop all tiles ran 9 % slower.
  if (HAS_K && zt.uniform) stream(std::true_type{});
  else stream(std::false_type{});
  const double part = block_sum(acc, lds);
  const float s = chunk_barrier_scale(cs, p.t, p.c, tpc, n_c, part, lds, &bc, scales);
  uint32_t* own = (oc.packed && p.c == oc.chunk) ? oc.packed : nullptr;   // uniform
  const int64_t own_tile0 = (p.tile0 - (int64_t)p.c * n_c) >> 5;           // the tile's first word within its chunk
  if (own && p.t == p.c * tpc && threadIdx.x == 0) *oc.scale = s;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) sign_pack_store(Z[u], s, err, packed, p.tile0 + u * SPAN, own, own_tile0 + u * (SPAN / 32));
  }
}

// ---------------------------------------------------------------------------------------------
// K3  server: zb = (sum_w +-s_w, sequentially) * (1/W) + err_server   (Algorithm 1 line 10)
// Workers strictly in order 0..W-1 (the fp32 sum is order dependent).  The W additions per element
// are the whole cost (the inputs are one bit per element and worker), so the loop is written for
// the vector ALU: three instructions per element and worker -- shift the worker's word so that the
// element's bit is bit 0, add that bit, moved to bit 31, to the bit pattern of -s (the carry out of
// bit 31 is dropped: bit 1 gives +s, bit 0 leaves -s; one v_lshl_add_u32), add to the accumulator --
// with no compare/select through a lane mask.  The scales come from LDS (staged SRV_STAGE at a
// time), the sign words of the next G workers are requested before those of the current G are
// consumed, and nothing inside the loop branches on the tile's shape: a wavefront whose elements lie
// beyond the tile's end skips the loop.
// ---------------------------------------------------------------------------------------------
constexpr int SRV_STAGE = 1024;   // scales held in LDS at a time
// The sign words are fetched with buffer loads: the wavefront-uniform part of the address (worker
// block, span of the tile) travels in a scalar register, the thread's part in one 32-bit register,
// so no vector instruction is spent on addresses.  Every address is inside [packed_in, packed_in +
// W*n_c/32) by construction (the descriptor's range check does not see the scalar part, so it is
// not relied on).  Offsets are 32-bit: the host admits W*n_c/8 < 2^31 bytes.
constexpr int OB_BUFFER_RSRC_WORD3 = 0x00020000;   // raw 32-bit data format word of gfx9-family descriptors

template <int U>
__device__ __forceinline__ void server_average(const uint32_t* __restrict__ packed_in,
                                               const float* __restrict__ scales_in, int64_t n_c,
                                               int W, const TilePos& p, float (&acc)[U][4],
                                               unsigned int* lds_negs /* [SRV_STAGE] */) {
  constexpr int G = (U >= 8) ? 1 : 8 / U;   // workers whose sign words are in flight together
  const int o0 = threadIdx.x * 4;
  const bool active = (o0 < p.len);   // uniform over a wavefront: len is a multiple of 256
  const int wpc_bytes = (int)(n_c >> 3);   // bytes per worker block
  // descriptor of the tile's column of packed_in: from the tile's first word to the end of the array
  const int64_t col0 = p.tile0 >> 5;
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint32_t*>(packed_in + col0), 0, (int)(((int64_t)W * (n_c >> 5) - col0) * 4), OB_BUFFER_RSRC_WORD3);
  // byte offset of the thread's word of span 0 in a worker's block; span u lies 128 bytes further.
  // The spans a partial tile lacks (only the chunk's last tile has any; uniform over the workgroup)
  // read span 0 again and their sums are never used: the words that follow the tile would lie in
  // the next worker's block and, for the last worker, beyond the end of the array.
  const int voff0 = 4 * (int)(threadIdx.x >> 3);
  int uoff[U];
#pragma unroll
  for (int u = 0; u < U; ++u) uoff[u] = (u * SPAN < p.len) ? 128 * u : 0;
  unsigned int shk[4];                // position of the thread's k-th bit in its word
#pragma unroll
  for (int k = 0; k < 4; ++k) shk[k] = 4u * (threadIdx.x & 7) + (unsigned)k;
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int k = 0; k < 4; ++k) acc[u][k] = 0.0f;
  auto add_worker = [&](const unsigned int (&word)[U], unsigned int negs) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const unsigned int t = ((word[u] >> shk[k]) << 31) + negs;   // bit ? +s : -s
        acc[u][k] = acc[u][k] + __uint_as_float(t);
      }
  };
  auto load_worker = [&](unsigned int (&word)[U], int w) {
    const int soff = w * wpc_bytes;   // uniform
#pragma unroll
    for (int u = 0; u < U; ++u)
      word[u] = (unsigned int)__builtin_amdgcn_raw_buffer_load_b32(rsrc, voff0, soff + uoff[u], 0);
  };
  for (int wb = 0; wb < W; wb += SRV_STAGE) {
    const int nb = (W - wb < SRV_STAGE) ? W - wb : SRV_STAGE;
    __syncthreads();
    for (int i = threadIdx.x; i < nb; i += BLOCK) lds_negs[i] = __float_as_uint(scales_in[wb + i]) ^ 0x80000000u;
    __syncthreads();
    if (!active) continue;
    const int full = nb - nb % G;
    unsigned int cur[G][U], nxt[G][U];
    if (full > 0) {
#pragma unroll
      for (int j = 0; j < G; ++j) load_worker(cur[j], wb + j);
    }
    for (int j0 = 0; j0 < full; j0 += G) {
      if (j0 + G < full) {
#pragma unroll
        for (int j = 0; j < G; ++j) load_worker(nxt[j], wb + j0 + G + j);
      }
#pragma unroll
      for (int j = 0; j < G; ++j) add_worker(cur[j], lds_negs[j0 + j]);
#pragma unroll
      for (int j = 0; j < G; ++j)
#pragma unroll
        for (int u = 0; u < U; ++u) cur[j][u] = nxt[j][u];
    }
    for (int j = full; j < nb; ++j) {   // the last nb % G workers
      unsigned int word[U];
      load_worker(word, wb + j);
      add_worker(word, lds_negs[j]);
    }
  }
}

// two-pass form: zb written over err_server, tile partial of sum zb^2.
// DEFER: the server error in deferred form (as for the worker, see PackedErr; here one chunk, one
// scale): err_s holds zb of the previous call, the carried error is err_s - C[zb] with the server's
// own previous output `keep` (read and rewritten in place), and the sign words of the new zb are
// written here, to packed_out and to `keep`; no second pass over the chunk is needed.
template <int U, bool DEFER = false>
__global__ __launch_bounds__(BLOCK) void k_server_unpack_avg(
    const uint32_t* __restrict__ packed_in, const float* __restrict__ scales_in,
    float* __restrict__ err_s, double* __restrict__ partials, int64_t n_c, int W, float invW,
    uint32_t* keep, const float* keep_scale, uint32_t* packed_out) {
  constexpr int TILE = SPAN * U;
  __shared__ double lds[BLOCK / WAVE];
  __shared__ unsigned int lds_negs[SRV_STAGE];
  const TilePos p = tile_pos<TILE>(n_c, (int)gridDim.x, (int)blockIdx.x);  // one chunk: c == 0
  const int o0 = threadIdx.x * 4;
  const float se = DEFER ? keep_scale[0] : 0.0f;
  float acc[U][4];
  server_average<U>(packed_in, scales_in, n_c, W, p, acc, lds_negs);
  double sq = 0.0;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {   // uniform over the wavefront, as the shuffles below require
      v4f e = ld4(err_s + p.tile0 + o);
      if (DEFER) e = deferred_error(e, load_nibble(keep, p.tile0 + u * SPAN), se);
      v4f z;
      unsigned int nib = 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        z[k] = acc[u][k] * invW + e[k];
        sq += (double)z[k] * (double)z[k];
        if (DEFER) nib |= ((z[k] >= 0.0f) ? 1u : 0u) << k;
      }
      st4(err_s + p.tile0 + o, z);
      if (DEFER) {
        const unsigned int word = gather_word(nib);
        if ((threadIdx.x & 7) == 0) {
          const int64_t w0 = (p.tile0 + u * SPAN) >> 5;
          (packed_out + w0)[threadIdx.x >> 3] = word;
          (keep + w0)[threadIdx.x >> 3] = word;
        }
      }
    }
  }
  const double s = block_sum(sq, lds);
  if (threadIdx.x == 0) partials[p.t] = s;
}

// K3+K4 in one pass: Algorithm 1 line 10 on the served chunk with zb kept in registers across the
// chunk barrier above (one chunk: c = 0, its own counter, flag and partials), instead of three
// launches and a round trip of zb through err_server.  The host selects it only when all of its
// workgroups fit on the device at once.
// Workgroups per CU the kernel is built for: 8 (at most 64 registers) for the smaller tiles; the
// 4096-element tile needs a few more registers than that and takes 7 rather than spill in its loop.
template <int U>
__global__ __launch_bounds__(BLOCK, (U >= 4 ? 7 : 8)) void k_server_resident(
    const uint32_t* __restrict__ packed_in, const float* __restrict__ scales_in,
    float* __restrict__ err_s, uint32_t* __restrict__ packed_out, float* __restrict__ scale_out,
    ChunkSync cs, int64_t n_c, int W, float invW) {
  constexpr int TILE = SPAN * U;
  __shared__ double lds[BLOCK / WAVE];
  __shared__ unsigned long long bc;
  __shared__ unsigned int lds_negs[SRV_STAGE];
  const TilePos p = tile_pos<TILE>(n_c, (int)gridDim.x, (int)blockIdx.x);  // one chunk: c == 0
  const int o0 = threadIdx.x * 4;
  float acc[U][4];
  server_average<U>(packed_in, scales_in, n_c, W, p, acc, lds_negs);
  v4f Z[U];
  double sq = 0.0;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    Z[u] = 0.0f;
    if (o < p.len) {
      const v4f e = ld4(err_s + p.tile0 + o);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        Z[u][k] = acc[u][k] * invW + e[k];
        sq += (double)Z[u][k] * (double)Z[u][k];
      }
    }
  }
  const double part = block_sum(sq, lds);
  const float s = chunk_barrier_scale(cs, p.t, 0, (int)gridDim.x, n_c, part, lds, &bc, scale_out);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) sign_pack_store(Z[u], s, err_s, packed_out, p.tile0 + u * SPAN);
  }
}

// ---------------------------------------------------------------------------------------------
// K5  per layer: global momentum, reconstructed gradient, fresh variance, max(v_frozen/v_fresh)
//     (Algorithm 1 lines 13, 15-17).  One maximum per (tile, layer) segment, no atomics.
// With the previous momentum in 1-bit form the reconstructed gradient takes only two magnitudes
// per tile, (s' - beta1 s)/(1-beta1) and (s' + beta1 s)/(1-beta1), whose squares are hoisted.
// The tile's registers and the two evaluation paths are shared with the fused ratio+update kernel.
// ---------------------------------------------------------------------------------------------
struct RatioArgs {
  const uint32_t* __restrict__ packed;   // [N_pad/32] the W recompressed chunks
  const float* __restrict__ sscales;     // [W] their scales
  const float* __restrict__ m;           // dense previous momentum (unless PACKED_M)
  PackedMom pm;                          // 1-bit previous momentum (PACKED_M)
  float* __restrict__ v_fresh;
  const float* __restrict__ v_frozen;
  float beta1, omb1, beta2, omb2;
};

template <int U, bool HAS_K, bool PACKED_M>
struct RatioTile {
  unsigned int NB[U], OB[U];
  v4f M[U], VF[U], VZ[U];

  __device__ __forceinline__ void load(const RatioArgs& ra, const TilePos& p) {
    const int o0 = threadIdx.x * 4;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int o = u * SPAN + o0;
      M[u] = 0.0f; OB[u] = 0u; NB[u] = 0u; VF[u] = 0.0f; VZ[u] = 0.0f;
      if (o < p.len) {
        NB[u] = load_nibble(ra.packed, p.tile0 + u * SPAN);
        if (PACKED_M) OB[u] = load_nibble(ra.pm.bits, p.tile0 + u * SPAN);
        else M[u] = ld4(ra.m + p.tile0 + o);
        VF[u] = ld4(ra.v_fresh + p.tile0 + o);
        VZ[u] = ld4(ra.v_frozen + p.tile0 + o);
      }
    }
  }

  // Tile inside layer l0: updates v_fresh, returns the thread's max of v_frozen/v_fresh.
  // VZ keeps v_frozen.  DEFER: the new v_fresh stays in VF for store_v_fresh() instead of being
  // stored at once (a barrier arrival that follows then does not wait for these stores).
  // ss, s_prev: new and previous server scale of the chunk; kt: k of the layer (1 without HAS_K).
  template <bool DEFER = false>
  __device__ __forceinline__ float uniform_pass(const RatioArgs& ra, const TilePos& p, float ss,
                                                float s_prev, float kt) {
    const int o0 = threadIdx.x * 4;
    const float sp = HAS_K ? ss / kt : ss;
    float t_same = 0.0f, t_diff = 0.0f;
    if (PACKED_M) {
      const float bm = ra.beta1 * (HAS_K ? s_prev / kt : s_prev);
      const float g_same = (sp - bm) / ra.omb1;     // new and old momentum of equal sign
      const float g_diff = (sp - (-bm)) / ra.omb1;  // of opposite sign
      t_same = ra.omb2 * (g_same * g_same);
      t_diff = ra.omb2 * (g_diff * g_diff);
    }
    float r = 0.0f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int o = u * SPAN + o0;
      if (o < p.len) {
        v4f vf;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          float t;
          if (PACKED_M) {
            t = (((NB[u] ^ OB[u]) >> k) & 1u) ? t_diff : t_same;
          } else {
            const float mt = ((NB[u] >> k) & 1u) ? sp : -sp;
            const float gr = (mt - ra.beta1 * M[u][k]) / ra.omb1;
            t = ra.omb2 * (gr * gr);
          }
          vf[k] = ra.beta2 * VF[u][k] + t;
          const float q = VZ[u][k] / vf[k];
          if (q > r) r = q;
        }
        if (DEFER) VF[u] = vf;
        else st4(ra.v_fresh + p.tile0 + o, vf);
      }
    }
    return r;
  }

  __device__ __forceinline__ void store_v_fresh(const RatioArgs& ra, const TilePos& p) const {
    const int o0 = threadIdx.x * 4;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int o = u * SPAN + o0;
      if (o < p.len) st4(ra.v_fresh + p.tile0 + o, VF[u]);
    }
  }

  // Tile that meets a layer boundary or the end of the parameters: element by element, leaving
  // the padding alone.  VZ is overwritten by the quotients (0 in the padding).
  __device__ __forceinline__ void element_pass(const RatioArgs& ra, const LayerTab& lt,
                                               const TilePos& p, int l0, float ss, float s_prev) {
    const int o0 = threadIdx.x * 4;
    const int64_t N = lt.off[lt.L];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int o = u * SPAN + o0;
      if (o < p.len) {
        int l = l0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int64_t i = p.tile0 + o + k;
          float q = 0.0f;
          if (i < N) {
            l = walk_layer(l, i, lt.off);
            const float kk = HAS_K ? lt.mom_scale[l] : 1.0f;
            const float sp = HAS_K ? ss / kk : ss;
            const float mt = ((NB[u] >> k) & 1u) ? sp : -sp;
            float bmk;
            if (PACKED_M) {
              const float b = ra.beta1 * (HAS_K ? s_prev / kk : s_prev);
              bmk = ((OB[u] >> k) & 1u) ? b : -b;
            } else {
              bmk = ra.beta1 * M[u][k];
            }
            const float gr = (mt - bmk) / ra.omb1;
            const float vf = ra.beta2 * VF[u][k] + ra.omb2 * (gr * gr);
            ra.v_fresh[i] = vf;
            q = VZ[u][k] / vf;
          }
          VZ[u][k] = q;
        }
      }
    }
  }

  // After element_pass: the thread's max of the quotients of elements in [a, b).
  __device__ __forceinline__ float segment_max(const TilePos& p, int64_t a, int64_t b) const {
    const int o0 = threadIdx.x * 4;
    float r = 0.0f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int o = u * SPAN + o0;
      if (o < p.len) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int64_t i = p.tile0 + o + k;
          if (i >= a && i < b && VZ[u][k] > r) r = VZ[u][k];
        }
      }
    }
    return r;
  }
};

// The ratio pass of one tile (a workgroup; lds: [BLOCK / WAVE]).
template <int U, bool HAS_K, bool PACKED_M>
__device__ __forceinline__ void ratios_pass_tile(const RatioArgs& ra, float* __restrict__ seg_max,
                                                 int64_t n_c, int tpc, const LayerTab& lt,
                                                 const int* __restrict__ tile_seg0,
                                                 const int* __restrict__ seg_layer, int tile, float* lds) {
  constexpr int TILE = SPAN * U;
  const TilePos p = tile_pos<TILE>(n_c, tpc, tile);
  const int l0 = lt.first_layer[p.t];
  if (l0 >= lt.L) return;  // tile lies in the padding (it has no segment)
  // every scalar the tile needs is requested before the streaming loads, so that nothing is
  // looked up after they return (these workgroups are short: latency counts)
  const float ss = ra.sscales[p.c];
  const float s_prev = PACKED_M ? ra.pm.scales[p.c] : 0.0f;
  const float kt = HAS_K ? lt.mom_scale[l0] : 1.0f;
  const int64_t l0_end = lt.off[l0 + 1];
  const int s0 = tile_seg0[p.t];
  RatioTile<U, HAS_K, PACKED_M> rt;
  rt.load(ra, p);
  const bool uniform = (p.tile0 + p.len <= l0_end);
  if (uniform) {
    float r = rt.uniform_pass(ra, p, ss, s_prev, kt);
    r = block_max(r, lds);
    if (threadIdx.x == 0) seg_max[s0] = r;
  } else {
    rt.element_pass(ra, lt, p, l0, ss, s_prev);
    const int s1 = tile_seg0[p.t + 1];
    for (int s = s0; s < s1; ++s) {
      const int l = seg_layer[s];
      float r = rt.segment_max(p, lt.off[l], lt.off[l + 1]);
      r = block_max(r, lds);
      if (threadIdx.x == 0) seg_max[s] = r;
    }
  }
}

template <int U, bool HAS_K, bool PACKED_M>
__global__ __launch_bounds__(BLOCK) void k_ratios_pass(RatioArgs ra, float* __restrict__ seg_max,
                                                       int64_t n_c, int tpc, LayerTab lt,
                                                       const int* __restrict__ tile_seg0,
                                                       const int* __restrict__ seg_layer,
                                                       const int* __restrict__ tile_list) {
  __shared__ float lds[BLOCK / WAVE];
  ratios_pass_tile<U, HAS_K, PACKED_M>(ra, seg_max, n_c, tpc, lt, tile_seg0, seg_layer, listed_tile(tile_list), lds);
}

// Algorithm 1 lines 18-20 for one layer given the raw ratio (thread 0 of a workgroup).
// rp, ca: r_prev[l] and c_avg[l], read by the caller (early, where their latency hides).
__device__ __forceinline__ float ratio_clip_commit(float r, int l, float rp, float ca,
                                                   float* __restrict__ r_prev,
                                                   float* __restrict__ coeff_c, float one_m_thr,
                                                   float one_p_thr, float r_min, float r_max) {
  const float lo = one_m_thr * rp, hi = one_p_thr * rp;
  r = (r > lo) ? r : lo;
  r = (r < hi) ? r : hi;
  r = (r > r_min) ? r : r_min;
  r = (r < r_max) ? r : r_max;
  r_prev[l] = r;
  const float c = r * ca;
  coeff_c[l] = c;
  return c;
}

// K6  per layer: max over the layer's segments (0 for an empty layer), then lines 18-20.
// One workgroup of NT threads per layer; lds: [NT / WAVE].
template <int NT>
__device__ __forceinline__ void ratios_finalize_layer(int l, const float* __restrict__ seg_max,
                                                      const int* __restrict__ layer_seg0,
                                                      const float* __restrict__ c_avg,
                                                      float* __restrict__ r_prev, float* __restrict__ coeff_c,
                                                      float one_m_thr, float one_p_thr, float r_min,
                                                      float r_max, float* lds) {
  const int s0 = layer_seg0[l], s1 = layer_seg0[l + 1];
  const float rp = r_prev[l], ca = c_avg[l];
  float r = 0.0f;
  // four loads in flight per thread: a tensor too large for the kernel with the per-layer barrier
  // has tens of thousands of segments, and this one workgroup walks them alone (the maxima are
  // >= +0 or NaN, so the zeros that stand in for missing ones change nothing)
  for (int s = s0 + threadIdx.x; s < s1; s += 4 * NT) {
    float q[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) q[u] = (s + u * NT < s1) ? seg_max[s + u * NT] : 0.0f;
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (q[u] > r) r = q[u];
  }
  r = block_max<NT>(r, lds);
  if (threadIdx.x == 0)
    (void)ratio_clip_commit(r, l, rp, ca, r_prev, coeff_c, one_m_thr, one_p_thr, r_min, r_max);
}

__global__ __launch_bounds__(FBLOCK) void k_ratios_finalize(const float* __restrict__ seg_max,
                                                            const int* __restrict__ layer_seg0,
                                                            const float* __restrict__ c_avg,
                                                            float* __restrict__ r_prev,
                                                            float* __restrict__ coeff_c,
                                                            float one_m_thr, float one_p_thr,
                                                            float r_min, float r_max,
                                                            const unsigned char* __restrict__ done_elsewhere) {
  __shared__ float lds[FBLOCK / WAVE];
  const int l = blockIdx.x;
  if (done_elsewhere && done_elsewhere[l]) return;  // the kernel with the per-layer barrier finishes it
  ratios_finalize_layer<FBLOCK>(l, seg_max, layer_seg0, c_avg, r_prev, coeff_c, one_m_thr, one_p_thr, r_min, r_max,
                                lds);
}

// ---------------------------------------------------------------------------------------------
// K7  x <- x - (lr*c_l) * m_t/(sqrt(v_frozen)+eta);  m <- m_t (when WRITE_M)
//     (Algorithm 1 lines 13, 21)
// ---------------------------------------------------------------------------------------------
struct ApplyArgs {
  const uint32_t* __restrict__ packed;
  const float* __restrict__ sscales;
  const float* __restrict__ v_frozen;
  float* __restrict__ x;
  float* __restrict__ m;              // written when WRITE_M
  const float* __restrict__ coeff_c;
  float lr, eta;
  void* __restrict__ x_lp;            // 16-bit copy of the updated x (LPX)
  int x_lp_bf16;
};

// Tile inside layer l0 with coefficient c: update from registers.
template <int U, bool HAS_K, bool WRITE_M, bool LPX = false>
__device__ __forceinline__ void apply_uniform(const ApplyArgs& aa, const TilePos& p, float ss,
                                              float kt, float c, const unsigned int (&NB)[U],
                                              const v4f (&VZ)[U], const v4f (&X)[U]) {
  const int o0 = threadIdx.x * 4;
  const float sp = HAS_K ? ss / kt : ss;
  const float a = aa.lr * c;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
      v4f xn, mn;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float mt = ((NB[u] >> k) & 1u) ? sp : -sp;
        const float uu = mt / (sqrtf(VZ[u][k]) + aa.eta);
        xn[k] = X[u][k] - a * uu;
        mn[k] = mt;
      }
      st4(aa.x + p.tile0 + o, xn);
      if (LPX) st4_lp(aa.x_lp, p.tile0 + o, xn, aa.x_lp_bf16);
      if (WRITE_M) st4(aa.m + p.tile0 + o, mn);
    }
  }
}

// Tile that meets a layer boundary: element by element, coefficients read from coeff_c.
template <int U, bool HAS_K, bool WRITE_M, bool LPX = false>
__device__ __forceinline__ void apply_elements(const ApplyArgs& aa, const LayerTab& lt,
                                               const TilePos& p, int l0, float ss,
                                               const unsigned int (&NB)[U], const v4f (&VZ)[U],
                                               const v4f (&X)[U]) {
  const int o0 = threadIdx.x * 4;
  const int64_t N = lt.off[lt.L];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
      int l = l0;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int64_t i = p.tile0 + o + k;
        if (i < N) {
          l = walk_layer(l, i, lt.off);
          const float sp = HAS_K ? ss / lt.mom_scale[l] : ss;
          const float a = aa.lr * aa.coeff_c[l];
          const float mt = ((NB[u] >> k) & 1u) ? sp : -sp;
          const float uu = mt / (sqrtf(VZ[u][k]) + aa.eta);
          const float xn = X[u][k] - a * uu;
          aa.x[i] = xn;
          if (LPX) reinterpret_cast<unsigned short*>(aa.x_lp)[i] = float_to_lp(xn, aa.x_lp_bf16);
          if (WRITE_M) aa.m[i] = mt;
        }
      }
    }
  }
}

template <int U, bool HAS_K, bool WRITE_M, bool LPX = false>
__global__ __launch_bounds__(BLOCK) void k_decompress_apply(ApplyArgs aa, int64_t n_c, int tpc,
                                                            LayerTab lt,
                                                            const int* __restrict__ tile_list) {
  constexpr int TILE = SPAN * U;
  const TilePos p = tile_pos<TILE>(n_c, tpc, listed_tile(tile_list));
  const int l0 = lt.first_layer[p.t];
  if (l0 >= lt.L) return;
  // scalars first (see k_ratios_pass), then the streaming loads
  const float ss = aa.sscales[p.c];
  const float kt = HAS_K ? lt.mom_scale[l0] : 1.0f;
  const float c0 = aa.coeff_c[l0];
  const int64_t l0_end = lt.off[l0 + 1];
  const int o0 = threadIdx.x * 4;
  unsigned int NB[U];
  v4f X[U], VZ[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    NB[u] = 0u; X[u] = 0.0f; VZ[u] = 0.0f;
    if (o < p.len) {
      NB[u] = load_nibble(aa.packed, p.tile0 + u * SPAN);
      VZ[u] = ld4(aa.v_frozen + p.tile0 + o);
      X[u] = ld4(aa.x + p.tile0 + o);
    }
  }
  const bool uniform = (p.tile0 + p.len <= l0_end);
  if (uniform) apply_uniform<U, HAS_K, WRITE_M, LPX>(aa, p, ss, kt, c0, NB, VZ, X);
  else apply_elements<U, HAS_K, WRITE_M, LPX>(aa, lt, p, l0, ss, NB, VZ, X);
}

// ---------------------------------------------------------------------------------------------
// K5+K6+K7 in one pass: Algorithm 1 lines 13-21 with v_frozen and the sign words read once.
// A workgroup runs the ratio pass on its tile of U 1024-element spans, keeps v_frozen and the signs
// in registers, arrives at its layer's barrier, and while the layer completes writes v_fresh,
// fetches x and forms m_t/(sqrt(v_frozen)+eta) in place of v_frozen; once the layer's coefficient
// c_t is published only a multiply and a subtract per element are left before x is stored.
//
// The kernel covers "listed" tiles: the tiles that lie inside ONE layer, for every layer whose such
// tiles all fit on the device at once (80 % of its workgroup slots).  Everything else -- layers
// that are too large, the spans where layers meet, small tensors -- goes through the plain kernels
// on 1024-element tiles: the ratio pass before this kernel (the maxima of those segments wait in
// seg_max) and the update after it.
//
// Per-layer barrier: like the per-chunk one above (same self-numbering counter and flag words),
// but the payload of a tile is its fp32 maximum of v_frozen/v_fresh (order-independent); the last
// of the layer's listed tiles to arrive reduces ALL of the layer's maxima, applies the two clips
// (lines 18-19), commits r_prev and coeff_c and publishes c_t in flag[l].  The dispatch-order
// argument of the chunk barrier applies per layer; all waits are bounded (errflag).
// ---------------------------------------------------------------------------------------------
// What the last arriver of a layer needs to find the layer's partial results: the listed tiles
// publish into an array of their own, indexed like the launch (tile_list position = blockIdx), and
// the plain kernels' segments of the layer lie before the first and after the last listed tile
// (the listed tiles of a layer are contiguous in position): [layer_seg0[l], seg_first[l]) and
// [seg_end[l], layer_seg0[l+1]) of the 1024-element tiling's segment array.
struct ListedTiles {
  const int* tile_list;         // listed tiles, by position (the launch's blockIdx -> tile)
  const int* list_begin;        // [L] index in tile_list of the layer's first listed tile
  const int* n_listed;          // [L] listed tiles of the layer
  const int* seg_first;         // [L] first segment owned by the layer's listed tiles
  const int* seg_end;           // [L] one past the last segment owned by them
  const int* layer_seg0;        // [L+1] segments of each layer
  int64_t n_c;
  int tpc, tpc_span;            // tiles of this kernel / spans per chunk
};

// The ranges of one layer, read by every workgroup at its start (uniform, next to its other
// scalars) so that the one that turns out to arrive last has them at hand.
struct LayerParts {
  int nl, lb;                 // listed tiles: tile_list[lb .. lb+nl)
  int a, s_first, s_end, b;   // plain segments: [a, s_first) and [s_end, b)
};
__device__ __forceinline__ LayerParts layer_parts(const ListedTiles& lt, int l) {
  LayerParts q;
  q.nl = lt.n_listed[l]; q.lb = lt.list_begin[l];
  q.a = lt.layer_seg0[l]; q.s_first = lt.seg_first[l]; q.s_end = lt.seg_end[l]; q.b = lt.layer_seg0[l + 1];
  return q;
}

// The last arriver's walk over a layer's partial results, strided over the workgroup's threads:
// comb(load(i)) for every listed tile of the layer (i = its position in tile_list), four loads in
// flight per thread (every waiter of the layer is waiting for this; `zero` stands in for missing
// ones and must leave comb's result unchanged), then plain(j) for every plain-kernel segment j.
template <class T, class FL, class FC, class FP>
__device__ __forceinline__ void for_layer_parts(const LayerParts& q, T zero, FL load, FC comb, FP plain) {
  for (int j = threadIdx.x; j < q.nl; j += 4 * BLOCK) {
    T v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = (j + u * BLOCK < q.nl) ? load(q.lb + j + u * BLOCK) : zero;
#pragma unroll
    for (int u = 0; u < 4; ++u) comb(v[u]);
  }
  for (int j = q.a + threadIdx.x; j < q.s_first; j += BLOCK) plain(j);
  for (int j = q.s_end + threadIdx.x; j < q.b; j += BLOCK) plain(j);
}

struct LayerSync {
  const float* seg_max;         // [segments of the 1024-element tiling] maxima left by the plain ratio pass
  float* listed_max;            // [listed tiles] maxima of this launch's tiles
  ListedTiles lt;
  unsigned long long* counter;  // [L * CTR_STRIDE] (generation << 32) | arrivals
  unsigned long long* flag;     // [L] (generation << 32) | bits of c_t
  unsigned int* errflag;
  int spin_limit;
  const float* c_avg;
  float* r_prev;
  float* coeff_c;
  float one_m_thr, one_p_thr, r_min, r_max;
  int n_lead;                   // leading workgroups of the launch, one per layer, that
                                // finish the layers without listed tiles (0: a kernel of its own has done that)
};

// Publishes the maximum r of the workgroup's listed tile (of layer l; bid: its position in
// tile_list) and arrives; if this was the
// layer's last listed tile, finishes the layer.  All threads call; r is valid in thread 0.
// lp, rp, ca: the layer's ranges, r_prev[l] and c_avg[l], read at the start of the kernel.
__device__ __forceinline__ void layer_arrive(const LayerSync& ls, int bid, int l, const LayerParts& lp, float rp,
                                             float ca, float r, float* lds, unsigned long long* bc) {
  unsigned long long* counter = &ls.counter[(int64_t)l * CTR_STRIDE];
  if (threadIdx.x == 0) {
    __hip_atomic_store(&ls.listed_max[bid], r, __ATOMIC_RELAXED, OB_AGENT);
    payload_before_arrival();
    *bc = barrier_arrive(counter, lp.nl);
  }
  __syncthreads();
  const bool last = ((*bc & 1ull) != 0ull);
  const unsigned int want = (unsigned int)(*bc >> 32);
  __syncthreads();
  if (last) {
    float q = 0.0f;
    for_layer_parts(
        lp, 0.0f,
        [&](int i) { return __hip_atomic_load(&ls.listed_max[i], __ATOMIC_RELAXED, OB_AGENT); },
        [&](float v) { if (v > q) q = v; },
        [&](int j) {
          const float v = ls.seg_max[j];   // written by an earlier kernel
          if (v > q) q = v;
        });
    q = block_max(q, lds);
    if (threadIdx.x == 0) {
      const float c = ratio_clip_commit(q, l, rp, ca, ls.r_prev, ls.coeff_c, ls.one_m_thr,
                                        ls.one_p_thr, ls.r_min, ls.r_max);
      (void)barrier_publish(&ls.flag[l], counter, lp.nl, want, __float_as_uint(c));
    }
  }
  // every thread leaves with the generation to wait for in *bc's high word (the last arriver too)
}

// Waits (bounded) until layer l's coefficient of this launch is published; returns it to all
// threads.  *bc still holds what layer_arrive left there.
__device__ __forceinline__ float layer_wait(const LayerSync& ls, int l, unsigned long long* bc) {
  __syncthreads();
  if (threadIdx.x == 0) *bc = barrier_wait(&ls.flag[l], (unsigned int)(*bc >> 32), ls.errflag, ls.spin_limit);
  __syncthreads();
  return __uint_as_float((unsigned int)(*bc & 0xffffffffull));
}

// A leading workgroup of a barrier kernel's launch (blockIdx.x < ls.n_lead, one per layer): lines 18-20 for
// layer blockIdx.x if it has no listed tile -- its segment maxima were left by earlier kernels and nothing
// in this launch reads what is written here -- in the shadow of this launch instead of in a launch of its own.
__device__ __forceinline__ void lead_finalize(const LayerSync& ls, float* lds) {
  const int l = (int)blockIdx.x;
  if (ls.lt.n_listed[l] == 0)
    ratios_finalize_layer<BLOCK>(l, ls.seg_max, ls.lt.layer_seg0, ls.c_avg, ls.r_prev, ls.coeff_c, ls.one_m_thr,
                                 ls.one_p_thr, ls.r_min, ls.r_max, lds);
}

// Instantiated for the momentum in 1-bit form only: with a dense momentum the extra array the
// tile must hold costs more (spills or occupancy) than the second read of v_frozen saves, so the
// host then takes the two-kernel path.  5 workgroups per CU (<= 96 VGPRs at U = 8) measured best:
// 4 leaves too few workgroup slots next to the ones waiting at a barrier, 6 and more spill.
#ifndef OB_LB_MINW
#define OB_LB_MINW 5
#endif
template <int U, bool HAS_K, bool LPX = false>
__global__ __launch_bounds__(BLOCK, OB_LB_MINW) void k_ratios_apply_resident(
    RatioArgs ra, ApplyArgs aa, LayerSync ls, LayerTab lt) {
  // lt.first_layer: of the 1024-element tiling
  constexpr int TILE = SPAN * U;
  __shared__ float lds[BLOCK / WAVE];
  __shared__ unsigned long long bc;
  const int bid = (int)blockIdx.x - ls.n_lead;   // position in tile_list
  if (bid < 0) {
    lead_finalize(ls, lds);
    return;
  }
  const int64_t n_c = ls.lt.n_c;
  const int tpc = ls.lt.tpc;
  const TilePos p = tile_pos<TILE>(n_c, tpc, ls.lt.tile_list[bid]);
  const int sp0 = p.c * ls.lt.tpc_span + (p.t - p.c * tpc) * U;  // the tile's first span
  const int l0 = lt.first_layer[sp0];  // the layer the tile lies in
  const float ss = ra.sscales[p.c];
  const float s_prev = ra.pm.scales[p.c];
  const float kt = HAS_K ? lt.mom_scale[l0] : 1.0f;
  const LayerParts lp = layer_parts(ls.lt, l0);
  const float rp = ls.r_prev[l0], ca = ls.c_avg[l0];
  const int o0 = threadIdx.x * 4;
  RatioTile<U, HAS_K, true> rt;
  rt.load(ra, p);
  float r = rt.template uniform_pass<true>(ra, p, ss, s_prev, kt);
  r = block_max(r, lds);
  layer_arrive(ls, bid, l0, lp, rp, ca, r, lds, &bc);   // before the stores of v_fresh: nothing to wait for
  rt.store_v_fresh(ra, p);
  v4f X[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {  // x is fetched while the layer completes
    const int o = u * SPAN + o0;
    X[u] = 0.0f;
    if (o < p.len) X[u] = ld4(aa.x + p.tile0 + o);
  }
  // m_t/(sqrt(v_frozen)+eta) does not depend on the layer's coefficient: it is formed now, in place
  // of v_frozen, so that the square root and the division run while the layer completes instead
  // of after it (the same operations on the same operands as apply_uniform's)
  const float sp = HAS_K ? ss / kt : ss;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float mt = ((rt.NB[u] >> k) & 1u) ? sp : -sp;
        float uu = mt / (sqrtf(rt.VZ[u][k]) + aa.eta);
        asm volatile("" : "+v"(uu));   // evaluated here, not sunk below the wait
        rt.VZ[u][k] = uu;
      }
    }
  }
  const float c = layer_wait(ls, l0, &bc);
  const float a = aa.lr * c;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
      v4f xn;
#pragma unroll
      for (int k = 0; k < 4; ++k) xn[k] = X[u][k] - a * rt.VZ[u][k];
      st4(aa.x + p.tile0 + o, xn);
      if (LPX) st4_lp(aa.x_lp, p.tile0 + o, xn, aa.x_lp_bf16);
    }
  }
}

// The same step for tiles of U spans with U too large to hold v_fresh, v_frozen and x of the whole
// tile at once: the ratio pass streams the tile G spans at a time (v_fresh is written back as it
// goes, the last group after the arrival) and keeps only v_frozen -- turned into
// m_t/(sqrt(v_frozen)+eta) while the layer completes -- and one sign nibble per span; x is fetched
// only after the layer's coefficient is known, G spans at a time.  Per element 4 bytes live across
// the barrier instead of 8, so a layer of twice the size fits on the device.
template <int U, int G, bool HAS_K, bool LPX = false>
__global__ __launch_bounds__(BLOCK, OB_LB_MINW) void k_ratios_apply_stream(
    RatioArgs ra, ApplyArgs aa, LayerSync ls, LayerTab lt) {
  static_assert(U % G == 0 && U % 8 == 0, "tile shape");
  constexpr int TILE = SPAN * U;
  __shared__ float lds[BLOCK / WAVE];
  __shared__ unsigned long long bc;
  const int64_t n_c = ls.lt.n_c;
  const int tpc = ls.lt.tpc;
  const TilePos p = tile_pos<TILE>(n_c, tpc, ls.lt.tile_list[blockIdx.x]);
  const int sp0 = p.c * ls.lt.tpc_span + (p.t - p.c * tpc) * U;  // the tile's first span
  const int l0 = lt.first_layer[sp0];  // the layer the tile lies in
  const float ss = ra.sscales[p.c];
  const float s_prev = ra.pm.scales[p.c];
  const float kt = HAS_K ? lt.mom_scale[l0] : 1.0f;
  const LayerParts lp = layer_parts(ls.lt, l0);
  const float rp = ls.r_prev[l0], ca = ls.c_avg[l0];
  const int o0 = threadIdx.x * 4;
  // the two magnitudes the reconstructed gradient can take (see RatioTile::uniform_pass)
  const float sp = HAS_K ? ss / kt : ss;
  const float bm = ra.beta1 * (HAS_K ? s_prev / kt : s_prev);
  const float g_same = (sp - bm) / ra.omb1;
  const float g_diff = (sp - (-bm)) / ra.omb1;
  const float t_same = ra.omb2 * (g_same * g_same);
  const float t_diff = ra.omb2 * (g_diff * g_diff);
  v4f VZ[U];
  unsigned int NBP[U / 8];   // the new momentum's sign nibbles, 8 spans to a register
  v4f VFl[G];                // fresh variance of the last group: stored after the arrival
#pragma unroll
  for (int i = 0; i < U / 8; ++i) NBP[i] = 0u;
  float r = 0.0f;
#pragma unroll
  for (int u0 = 0; u0 < U; u0 += G) {
    unsigned int NB[G], OBt[G];
    v4f VF[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int u = u0 + j, o = u * SPAN + o0;
      NB[j] = 0u; OBt[j] = 0u; VF[j] = 0.0f; VZ[u] = 0.0f;
      if (o < p.len) {
        NB[j] = load_nibble(ra.packed, p.tile0 + u * SPAN);
        OBt[j] = load_nibble(ra.pm.bits, p.tile0 + u * SPAN);
        VF[j] = ld4(ra.v_fresh + p.tile0 + o);
        VZ[u] = ld4(ra.v_frozen + p.tile0 + o);
      }
    }
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int u = u0 + j, o = u * SPAN + o0;
      if (o < p.len) {
        v4f vf;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float t = (((NB[j] ^ OBt[j]) >> k) & 1u) ? t_diff : t_same;
          vf[k] = ra.beta2 * VF[j][k] + t;
          const float q = VZ[u][k] / vf[k];
          if (q > r) r = q;
        }
        if (u0 + G < U) st4(ra.v_fresh + p.tile0 + o, vf);
        else VFl[j] = vf;
        NBP[u / 8] |= (NB[j] & 15u) << (4 * (u % 8));
      }
    }
  }
  r = block_max(r, lds);
  layer_arrive(ls, (int)blockIdx.x, l0, lp, rp, ca, r, lds, &bc);
#pragma unroll
  for (int j = 0; j < G; ++j) {
    const int o = (U - G + j) * SPAN + o0;
    if (o < p.len) st4(ra.v_fresh + p.tile0 + o, VFl[j]);
  }
  // m_t/(sqrt(v_frozen)+eta) in place of v_frozen while the layer completes (the same operations on
  // the same operands as apply_uniform's)
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float mt = ((NBP[u / 8] >> (4 * (u % 8) + k)) & 1u) ? sp : -sp;
        float uu = mt / (sqrtf(VZ[u][k]) + aa.eta);
        asm volatile("" : "+v"(uu));   // evaluated here, not sunk below the wait
        VZ[u][k] = uu;
      }
    }
  }
  const float c = layer_wait(ls, l0, &bc);
  const float a = aa.lr * c;
#pragma unroll
  for (int u0 = 0; u0 < U; u0 += G) {
    v4f X[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int o = (u0 + j) * SPAN + o0;
      X[j] = 0.0f;
      if (o < p.len) X[j] = ld4(aa.x + p.tile0 + o);
    }
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int o = (u0 + j) * SPAN + o0;
      if (o < p.len) {
        v4f xn;
#pragma unroll
        for (int k = 0; k < 4; ++k) xn[k] = X[j][k] - a * VZ[u0 + j][k];
        st4(aa.x + p.tile0 + o, xn);
        if (LPX) st4_lp(aa.x_lp, p.tile0 + o, xn, aa.x_lp_bf16);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// The fresh variance in deferred form (Algorithm 1 line 16 evaluated every step, stored every few).
//
// With the momentum in 1-bit form the reconstructed gradient of line 15 takes two magnitudes per
// (chunk, layer) and step, chosen per element by whether the momentum's sign bit flipped.  So the
// variance after a more steps follows from the variance array as last written ("base") and the
// sign words and scales of the a+1 momenta since then, by the very operations line 16 would have
// performed step by step (v <- beta2*v + t, t one of the two values of that step): the ratio of
// line 17 needs the up-to-date variance of every element in registers, but the array need not be
// rewritten each time.  A step then reads the base (4 bytes per element, as before) plus one bit
// per element and older step, and writes nothing; every few steps the caller asks for the array to
// be brought up to date (write_v) and the history starts anew.
//
// Planes, newest first: 0 = the new momentum (RatioArgs.packed / sscales), 1 = the previous one
// (RatioArgs.pm), 2 + i = VfHist.bits[i] / scales[i] for i < n_old (so bits[0] is the momentum
// before the previous one).  The base is the variance as of plane n_old + 1.
// ---------------------------------------------------------------------------------------------
constexpr int VF_MAX_OLD = 7;
struct VfHist {
  int n_old;                            // 0..VF_MAX_OLD
  int write_v;                          // store the up-to-date variance
  const uint32_t* bits[VF_MAX_OLD];     // [N_pad/32] each
  const float* scales[VF_MAX_OLD];      // [W] each
};

// The two values omb2*g^2 of one step (the operations of RatioTile::uniform_pass, in its order).
// s_new, s_old: the chunk's scale of the step's momentum and of the one before.
template <bool HAS_K>
__device__ __forceinline__ void variance_terms(const RatioArgs& ra, float s_new, float s_old, float kt,
                                               float* t_same, float* t_diff) {
  const float sp = HAS_K ? s_new / kt : s_new;
  const float bm = ra.beta1 * (HAS_K ? s_old / kt : s_old);
  const float g_same = (sp - bm) / ra.omb1;     // new and old momentum of equal sign
  const float g_diff = (sp - (-bm)) / ra.omb1;  // of opposite sign
  *t_same = ra.omb2 * (g_same * g_same);
  *t_diff = ra.omb2 * (g_diff * g_diff);
}

// bit ? a : b on the bit patterns, with the bit taken from position `pos` of `word` (two vector
// instructions: a signed one-bit field extract gives the all-ones / all-zeros mask)
__device__ __forceinline__ float select_by_bit(unsigned int word, int pos, float a, float b) {
  const unsigned int m = (unsigned int)(((int)(word << (31 - pos))) >> 31);
  return __uint_as_float((m & __float_as_uint(a)) | (~m & __float_as_uint(b)));
}

// scale of plane q (newest first) for chunk c; q is a compile-time constant where it is called
__device__ __forceinline__ float plane_scale(const RatioArgs& ra, const VfHist& h, int q, int c) {
  return q == 0 ? ra.sscales[c] : (q == 1 ? ra.pm.scales[c] : h.scales[q - 2][c]);
}
__device__ __forceinline__ const uint32_t* plane_bits(const RatioArgs& ra, const VfHist& h, int q) {
  return q == 0 ? ra.packed : (q == 1 ? ra.pm.bits : h.bits[q - 2]);
}

// The two values of every step are the same for all elements of a (chunk, layer) pair.  A small
// kernel forms them once per call for every pair and step; the N-sized kernels then fetch two
// scalars per step instead of each thread redoing four divisions per step.
// Pairs: the layers that meet chunk c, in layer order, are pairs pair_base[c] .. pair_base[c+1]-1;
// the pair of (c, l) is pair_base[c] + l - pair_lfirst[c].
struct VTerms {
  const float* __restrict__ t;   // [VF_MAX_OLD + 1 steps][n_pairs][2]: t_same, t_diff; step s (1 = newest) at s - 1
  const int* pair_base;       // [W + 1]
  const int* pair_lfirst;     // [W]
  const int* pair_c;          // [n_pairs]
  const int* pair_l;          // [n_pairs]
  int n_pairs;
};
__device__ __forceinline__ int pair_of(const VTerms& vt, int c, int l) { return vt.pair_base[c] + l - vt.pair_lfirst[c]; }

template <bool HAS_K>
__device__ __forceinline__ void variance_terms_of_pair(const RatioArgs& ra, const VfHist& h, const VTerms& vt,
                                                       const float* __restrict__ mom_scale,
                                                       float* __restrict__ out /* = vt.t */, int pr) {
  if (pr >= vt.n_pairs) return;
  const int c = vt.pair_c[pr], l = vt.pair_l[pr];
  const float kt = HAS_K ? mom_scale[l] : 1.0f;
  const int a = h.n_old + 1;
#pragma unroll
  for (int s = 1; s <= VF_MAX_OLD + 1; ++s) {
    if (s <= a) {
      float t_same, t_diff;
      variance_terms<HAS_K>(ra, plane_scale(ra, h, s - 1, c), plane_scale(ra, h, s, c), kt, &t_same, &t_diff);
      float* o = out + ((int64_t)(s - 1) * vt.n_pairs + pr) * 2;
      o[0] = t_same;
      o[1] = t_diff;
    }
  }
}

template <bool HAS_K>
__global__ __launch_bounds__(BLOCK) void k_variance_terms(RatioArgs ra, VfHist h, VTerms vt,
                                                          const float* __restrict__ mom_scale,
                                                          float* __restrict__ out /* = vt.t */) {
  variance_terms_of_pair<HAS_K>(ra, h, vt, mom_scale, out, (int)(blockIdx.x * BLOCK + threadIdx.x));
}

// k_variance_terms and k_ratios_pass (momentum in 1-bit form, tile list) in one launch: the first n_lead
// workgroups form the terms, the others run the plain ratio pass of tile_list[blockIdx.x - n_lead].
// Neither reads what the other writes; both are over before the kernels that use the terms start.
template <int U, bool HAS_K>
__global__ __launch_bounds__(BLOCK) void k_ratios_pass_vterms(RatioArgs ra, float* __restrict__ seg_max,
                                                              int64_t n_c, int tpc, LayerTab lt,
                                                              const int* __restrict__ tile_seg0,
                                                              const int* __restrict__ seg_layer,
                                                              const int* __restrict__ tile_list, VfHist h,
                                                              VTerms vt, float* __restrict__ vt_out, int n_lead) {
  __shared__ float lds[BLOCK / WAVE];
  const int bid = (int)blockIdx.x - n_lead;
  if (bid < 0) {
    variance_terms_of_pair<HAS_K>(ra, h, vt, lt.mom_scale, vt_out, (int)(blockIdx.x * BLOCK + threadIdx.x));
    return;
  }
  ratios_pass_tile<U, HAS_K, true>(ra, seg_max, n_c, tpc, lt, tile_seg0, seg_layer, tile_list[bid], lds);
}

// Dense view of a variance held in deferred form, over the 1024-element tiles inside the tiles of
// the two kernels below (each lies inside one layer): the up-to-date variance goes to the base
// array itself if h.write_v, else to vf_dense (another array, which leaves the base as it is).
__global__ __launch_bounds__(BLOCK) void k_variance_dense(RatioArgs ra, VfHist h, VTerms vt,
                                                          float* __restrict__ vf_dense, int64_t n_c, int tpc,
                                                          LayerTab lt, const int* __restrict__ tile_list) {
  const TilePos p = tile_pos<SPAN>(n_c, tpc, tile_list[blockIdx.x]);
  const int l0 = lt.first_layer[p.t];
  if (l0 >= lt.L || p.tile0 + p.len > lt.off[l0 + 1]) return;   // (not a tile of those kernels: nothing lags there)
  const int a = h.n_old + 1;   // steps to apply
  const float* tt = vt.t + (int64_t)pair_of(vt, p.c, l0) * 2;
  const int o = threadIdx.x * 4;
  if (o >= p.len) return;
  float* vf_out = h.write_v ? ra.v_fresh : vf_dense;   // uniform
  unsigned int NBq[VF_MAX_OLD + 2];   // the lane's nibble of every plane, newest first
#pragma unroll
  for (int q = 0; q < VF_MAX_OLD + 2; ++q) {
    NBq[q] = 0u;
    if (q <= a) NBq[q] = load_nibble(plane_bits(ra, h, q), p.tile0);
  }
  v4f V = ld4(ra.v_fresh + p.tile0 + o);
#pragma unroll
  for (int s = VF_MAX_OLD + 1; s >= 1; --s) {
    if (s <= a) {   // uniform: the step from plane s to plane s-1
      const float t_same = tt[(int64_t)(s - 1) * vt.n_pairs * 2], t_diff = tt[(int64_t)(s - 1) * vt.n_pairs * 2 + 1];
      const unsigned int flip = NBq[s] ^ NBq[s - 1];
#pragma unroll
      for (int k = 0; k < 4; ++k) V[k] = ra.beta2 * V[k] + select_by_bit(flip, k, t_diff, t_same);
    }
  }
  st4(vf_out + p.tile0 + o, V);
}

// The ratio pass with the variance in deferred form on 8192-element tiles that lie inside one layer,
// for the layers that are too large for the kernel with the per-layer barrier (their update still
// runs as the plain kernel).  On such tiles the pass moves bytes at the streaming rate, so reading
// the stale array and the momenta's sign words instead of rewriting the array pays; on 1024-element
// tiles it does not.  Same loads, exchange and
// walk through the steps as k_ratios_apply_hist.  The tile's maximum goes to the segment of its
// first 1024-element span, 0 to the segments of its other spans (k_ratios_finalize takes the
// maximum over all of a layer's segments).
__global__ __launch_bounds__(BLOCK, OB_LB_MINW) void k_ratios_big_hist(RatioArgs ra, VfHist h, VTerms vt, float* __restrict__ seg_max,
                                                           const int* __restrict__ big_tiles, int64_t n_c,
                                                           int tpc_big, int tpc_span, LayerTab lt,
                                                           const int* __restrict__ tile_seg0) {
  constexpr int U = 8;
  constexpr int TILE = SPAN * U;
  __shared__ float lds[BLOCK / WAVE];
  const TilePos p = tile_pos<TILE>(n_c, tpc_big, big_tiles[blockIdx.x]);
  const int sp0 = p.c * tpc_span + (p.t - p.c * tpc_big) * U;  // the tile's first span
  const int l0 = lt.first_layer[sp0];  // the layer the tile lies in (lt.first_layer: of the 1024-element tiling)
  const float* tt = vt.t + (int64_t)pair_of(vt, p.c, l0) * 2;
  const int a = h.n_old + 1;   // steps to apply
  const int o0 = threadIdx.x * 4;
  const int lane = threadIdx.x & (WAVE - 1), wv = threadIdx.x / WAVE;
  const int e0 = (lane >> 3) * SPAN + wv * (WAVE * 4) + (lane & 7) * 32;
  const bool have_word = (e0 < p.len);
  const int64_t wi = (p.tile0 + e0) >> 5;
  unsigned int Wq[VF_MAX_OLD + 2];
#pragma unroll
  for (int q = 0; q < VF_MAX_OLD + 2; ++q) {
    Wq[q] = 0u;
    if (q <= a && have_word) Wq[q] = plane_bits(ra, h, q)[wi];
  }
  v4f V[U], VZ[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    V[u] = 0.0f; VZ[u] = 0.0f;
    if (o < p.len) {
      V[u] = ld4(ra.v_fresh + p.tile0 + o);
      VZ[u] = ld4(ra.v_frozen + p.tile0 + o);
    }
  }
#pragma unroll
  for (int s = VF_MAX_OLD + 1; s >= 1; --s)
    if (s <= a) Wq[s] ^= Wq[s - 1];
  const int src = lane >> 3;
  const unsigned int sh = 4u * (lane & 7);
#pragma unroll
  for (int q = 1; q < VF_MAX_OLD + 2; ++q) {   // (plane 0 itself is not needed here: only the flips)
    if (q <= a) {   // uniform
      unsigned int packed = 0u;
#pragma unroll
      for (int u = 0; u < U; ++u) packed |= ((__shfl(Wq[q], 8 * u + src, WAVE) >> sh) & 15u) << (4 * u);
      Wq[q] = packed;
    }
  }
#pragma unroll
  for (int s = VF_MAX_OLD + 1; s >= 1; --s) {
    if (s <= a) {   // uniform: the step from plane s to plane s-1
      const float t_same = tt[(int64_t)(s - 1) * vt.n_pairs * 2], t_diff = tt[(int64_t)(s - 1) * vt.n_pairs * 2 + 1];
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int k = 0; k < 4; ++k) V[u][k] = ra.beta2 * V[u][k] + select_by_bit(Wq[s], 4 * u + k, t_diff, t_same);
    }
  }
  float r = 0.0f;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float q = VZ[u][k] / V[u][k];
        if (q > r) r = q;
      }
      if (h.write_v) st4(ra.v_fresh + p.tile0 + o, V[u]);
    }
  }
  r = block_max(r, lds);
  const int nspan = (p.len + SPAN - 1) / SPAN;
  if (threadIdx.x < nspan) seg_max[tile_seg0[sp0 + threadIdx.x]] = (threadIdx.x == 0) ? r : 0.0f;
}

// k_ratios_apply_resident with the variance in deferred form.  A wavefront's part of a tile is 64
// words of every plane (8 spans x 8 words): each lane fetches ONE word of each plane and the lanes
// then pass each other the words they need; what a lane keeps of a plane is its 8 nibbles packed
// into one register.
template <bool HAS_K, bool LPX>
__global__ __launch_bounds__(BLOCK, OB_LB_MINW) void k_ratios_apply_hist(
    RatioArgs ra, VfHist h, VTerms vt, ApplyArgs aa, LayerSync ls, LayerTab lt) {
  constexpr int U = 8;
  constexpr int TILE = SPAN * U;
  __shared__ float lds[BLOCK / WAVE];
  __shared__ unsigned long long bc;
  const int bid = (int)blockIdx.x - ls.n_lead;   // position in tile_list
  if (bid < 0) {
    lead_finalize(ls, lds);
    return;
  }
  const int tpc = ls.lt.tpc;
  const TilePos p = tile_pos<TILE>(ls.lt.n_c, tpc, ls.lt.tile_list[bid]);
  const int sp0 = p.c * ls.lt.tpc_span + (p.t - p.c * tpc) * U;  // the tile's first span
  const int l0 = lt.first_layer[sp0];  // the layer the tile lies in (lt.first_layer: of the 1024-element tiling)
  const float kt = HAS_K ? lt.mom_scale[l0] : 1.0f;
  const float ss = ra.sscales[p.c];
  const LayerParts lp = layer_parts(ls.lt, l0);
  const float rp = ls.r_prev[l0], ca = ls.c_avg[l0];
  const float* tt = vt.t + (int64_t)pair_of(vt, p.c, l0) * 2;
  const int a = h.n_old + 1;   // steps to apply
  const int o0 = threadIdx.x * 4;
  const int lane = threadIdx.x & (WAVE - 1), wv = threadIdx.x / WAVE;
  // the lane's word of each plane: span lane/8, word lane%8 of the wavefront's 8 words (256 elements) of that span
  const int e0 = (lane >> 3) * SPAN + wv * (WAVE * 4) + (lane & 7) * 32;
  const bool have_word = (e0 < p.len);   // len is a multiple of 256: a wavefront's part of a span is all there or all missing
  const int64_t wi = (p.tile0 + e0) >> 5;
  unsigned int Wq[VF_MAX_OLD + 2];
#pragma unroll
  for (int q = 0; q < VF_MAX_OLD + 2; ++q) {
    Wq[q] = 0u;
    if (q <= a && have_word) Wq[q] = plane_bits(ra, h, q)[wi];
  }
  v4f V[U], VZ[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    V[u] = 0.0f; VZ[u] = 0.0f;
    if (o < p.len) {
      V[u] = ld4(ra.v_fresh + p.tile0 + o);
      VZ[u] = ld4(ra.v_frozen + p.tile0 + o);
    }
  }
  // flips between consecutive planes, formed on the words as loaded; plane 0 stays (line 21 needs it)
#pragma unroll
  for (int s = VF_MAX_OLD + 1; s >= 1; --s)
    if (s <= a) Wq[s] ^= Wq[s - 1];
  // the lanes' own nibbles of every span, 8 to a register
  const int src = lane >> 3;               // + 8*u: the lane that holds this lane's word of span u
  const unsigned int sh = 4u * (lane & 7);
#pragma unroll
  for (int q = 0; q < VF_MAX_OLD + 2; ++q) {
    if (q <= a) {   // uniform
      unsigned int packed = 0u;
#pragma unroll
      for (int u = 0; u < U; ++u) packed |= ((__shfl(Wq[q], 8 * u + src, WAVE) >> sh) & 15u) << (4 * u);
      Wq[q] = packed;
    }
  }
#pragma unroll
  for (int s = VF_MAX_OLD + 1; s >= 1; --s) {
    if (s <= a) {   // uniform: the step from plane s to plane s-1
      const float t_same = tt[(int64_t)(s - 1) * vt.n_pairs * 2], t_diff = tt[(int64_t)(s - 1) * vt.n_pairs * 2 + 1];
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int k = 0; k < 4; ++k) V[u][k] = ra.beta2 * V[u][k] + select_by_bit(Wq[s], 4 * u + k, t_diff, t_same);
    }
  }
  float r = 0.0f;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float q = VZ[u][k] / V[u][k];
        if (q > r) r = q;
      }
    }
  }
  r = block_max(r, lds);
  layer_arrive(ls, bid, l0, lp, rp, ca, r, lds, &bc);   // before any store: nothing to wait for
  if (h.write_v) {   // uniform
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int o = u * SPAN + o0;
      if (o < p.len) st4(ra.v_fresh + p.tile0 + o, V[u]);
    }
  }
  v4f X[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {  // x is fetched while the layer completes
    const int o = u * SPAN + o0;
    X[u] = 0.0f;
    if (o < p.len) X[u] = ld4(aa.x + p.tile0 + o);
  }
  // m_t/(sqrt(v_frozen)+eta), formed in place of v_frozen while the layer completes (the same
  // operations on the same operands as apply_uniform's)
  const float sp = HAS_K ? ss / kt : ss;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float mt = ((Wq[0] >> (4 * u + k)) & 1u) ? sp : -sp;
        float uu = mt / (sqrtf(VZ[u][k]) + aa.eta);
        asm volatile("" : "+v"(uu));   // evaluated here, not sunk below the wait
        VZ[u][k] = uu;
      }
    }
  }
  const float c = layer_wait(ls, l0, &bc);
  const float al = aa.lr * c;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
      v4f xn;
#pragma unroll
      for (int k = 0; k < 4; ++k) xn[k] = X[u][k] - al * VZ[u][k];
      st4(aa.x + p.tile0 + o, xn);
      if (LPX) st4_lp(aa.x_lp, p.tile0 + o, xn, aa.x_lp_bf16);
    }
  }
}

// Dense view of a momentum held in 1-bit form: m[i] = (bit ? s_c : -s_c)/k_l for i < N (the
// padding of m is left untouched).
template <int U, bool HAS_K>
__global__ __launch_bounds__(BLOCK) void k_momentum_dense(PackedMom pm, float* __restrict__ m,
                                                          int64_t n_c, int tpc, LayerTab lt) {
  constexpr int TILE = SPAN * U;
  const TilePos p = tile_pos<TILE>(n_c, tpc, (int)blockIdx.x);
  const int l0 = lt.first_layer[p.t];
  const int L = lt.L;
  if (l0 >= L) return;
  const int o0 = threadIdx.x * 4;
  const float ss = pm.scales[p.c];
  const bool uniform = (p.tile0 + p.len <= lt.off[l0 + 1]);
  const int64_t N = lt.off[L];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
      const unsigned int nb = load_nibble(pm.bits, p.tile0 + u * SPAN);
      if (uniform) {
        const float sp = HAS_K ? ss / lt.mom_scale[l0] : ss;
        v4f mn;
#pragma unroll
        for (int k = 0; k < 4; ++k) mn[k] = ((nb >> k) & 1u) ? sp : -sp;
        st4(m + p.tile0 + o, mn);
      } else {
        int l = l0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int64_t i = p.tile0 + o + k;
          if (i < N) {
            l = walk_layer(l, i, lt.off);
            const float sp = HAS_K ? ss / lt.mom_scale[l] : ss;
            m[i] = ((nb >> k) & 1u) ? sp : -sp;
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// K8  LAMB warmup step, eq. (1)
//   a: m, v update; per (tile, layer) segment the fp64 sums of x^2 and u^2
//   b: per layer: c = clip(||x||/||u||), c_avg moving average (Algorithm 1 line 2)
//   c: x <- x - (lr*c) u, with u recomputed from the stored m, v (same operations, same value)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float lamb_u(float mn, float vn, float x, float eta, float wd) {
  float u = mn / (sqrtf(vn) + eta);
  if (wd != 0.0f) u = u + wd * x;
  return u;
}

template <int U, int GT = 0>
__global__ __launch_bounds__(BLOCK) void k_warmup_moments(
    GradSrc g, float* __restrict__ m, float* __restrict__ v,
    const float* __restrict__ x, double* __restrict__ seg_sums /* [2*n_segs] */, int64_t n_c,
    int tpc, float beta1, float omb1, float beta2, float omb2, float eta, float wd, LayerTab lt,
    const int* __restrict__ tile_seg0, const int* __restrict__ seg_layer,
    const int* __restrict__ tile_list) {
  constexpr int TILE = SPAN * U;
  __shared__ double lds[BLOCK / WAVE];
  const TilePos p = tile_pos<TILE>(n_c, tpc, listed_tile(tile_list));
  const int l0 = lt.first_layer[p.t];
  const int L = lt.L;
  if (l0 >= L) return;
  const int o0 = threadIdx.x * 4;
  const bool uniform = (p.tile0 + p.len <= lt.off[l0 + 1]);
  v4f G[U], M[U], V[U], X[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    G[u] = 0.0f; M[u] = 0.0f; V[u] = 0.0f; X[u] = 0.0f;
    if (o < p.len) {
      G[u] = load_grad<GT>(g, p.tile0 + o);
      M[u] = ld4(m + p.tile0 + o);
      V[u] = ld4(v + p.tile0 + o);
      X[u] = ld4(x + p.tile0 + o);
    }
  }
  // new moments (kept in M, V)
#pragma unroll
  for (int u = 0; u < U; ++u) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      M[u][k] = beta1 * M[u][k] + omb1 * G[u][k];
      V[u][k] = beta2 * V[u][k] + omb2 * (G[u][k] * G[u][k]);
    }
  }
  const int s0 = tile_seg0[p.t];
  if (uniform) {
    double sx = 0.0, su = 0.0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int o = u * SPAN + o0;
      if (o < p.len) {
        st4(m + p.tile0 + o, M[u]);
        st4(v + p.tile0 + o, V[u]);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float uu = lamb_u(M[u][k], V[u][k], X[u][k], eta, wd);
          sx += (double)X[u][k] * (double)X[u][k];
          su += (double)uu * (double)uu;
        }
      }
    }
    sx = block_sum(sx, lds);
    su = block_sum(su, lds);
    if (threadIdx.x == 0) {
      seg_sums[2 * (int64_t)s0] = sx;
      seg_sums[2 * (int64_t)s0 + 1] = su;
    }
  } else {
    const int64_t N = lt.off[L];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int o = u * SPAN + o0;
      if (o < p.len) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int64_t i = p.tile0 + o + k;
          if (i < N) {
            m[i] = M[u][k];
            v[i] = V[u][k];
          }
        }
      }
    }
    const int s1 = tile_seg0[p.t + 1];
    for (int s = s0; s < s1; ++s) {
      const int l = seg_layer[s];
      const int64_t a = lt.off[l], b = lt.off[l + 1];
      double sx = 0.0, su = 0.0;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int o = u * SPAN + o0;
        if (o < p.len) {
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const int64_t i = p.tile0 + o + k;
            if (i >= a && i < b) {
              const float uu = lamb_u(M[u][k], V[u][k], X[u][k], eta, wd);
              sx += (double)X[u][k] * (double)X[u][k];
              su += (double)uu * (double)uu;
            }
          }
        }
      }
      sx = block_sum(sx, lds);
      su = block_sum(su, lds);
      if (threadIdx.x == 0) {
        seg_sums[2 * (int64_t)s] = sx;
        seg_sums[2 * (int64_t)s + 1] = su;
      }
    }
  }
}

// eq. (1)'s coefficient of one layer from its sums of x^2 and u^2, and Algorithm 1 line 2
// (thread 0 of a workgroup).
// ca: c_avg[l], read by the caller (early, where its latency hides).
__device__ __forceinline__ float warmup_coeff_commit(double sx, double su, int l, float ca,
                                                     float* __restrict__ coeff_c,
                                                     float* __restrict__ c_avg, float c_min,
                                                     float c_max, float beta3, float omb3) {
  const float nx = (float)sqrt(sx), nu = (float)sqrt(su);
  float c = nx / nu;
  c = (c > c_min) ? c : c_min;
  c = (c < c_max) ? c : c_max;
  coeff_c[l] = c;
  c_avg[l] = beta3 * ca + omb3 * c;
  return c;
}

__global__ __launch_bounds__(FBLOCK) void k_warmup_coeff(const double* __restrict__ seg_sums,
                                                         const int* __restrict__ layer_seg0,
                                                         float* __restrict__ coeff_c,
                                                         float* __restrict__ c_avg, float c_min,
                                                         float c_max, float beta3, float omb3,
                                                         const unsigned char* __restrict__ done_elsewhere) {
  __shared__ double lds[FBLOCK / WAVE];
  const int l = blockIdx.x;
  if (done_elsewhere && done_elsewhere[l]) return;  // the kernel with the per-layer barrier finishes it
  const int s0 = layer_seg0[l], s1 = layer_seg0[l + 1];
  const float ca = c_avg[l];
  double sx = 0.0, su = 0.0;
  for (int s = s0 + threadIdx.x; s < s1; s += 4 * FBLOCK) {   // four pairs in flight per thread
    double vx[4], vu[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const bool in = (s + u * FBLOCK < s1);
      vx[u] = in ? seg_sums[2 * (int64_t)(s + u * FBLOCK)] : 0.0;
      vu[u] = in ? seg_sums[2 * (int64_t)(s + u * FBLOCK) + 1] : 0.0;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) { sx += vx[u]; su += vu[u]; }
  }
  sx = block_sum<FBLOCK>(sx, lds);
  su = block_sum<FBLOCK>(su, lds);
  if (threadIdx.x == 0) (void)warmup_coeff_commit(sx, su, l, ca, coeff_c, c_avg, c_min, c_max, beta3, omb3);
}

template <int U, bool LPX = false>
__global__ __launch_bounds__(BLOCK) void k_warmup_apply(
    const float* __restrict__ m, const float* __restrict__ v, float* __restrict__ x,
    const float* __restrict__ coeff_c, int64_t n_c, int tpc, float lr, float eta, float wd,
    LayerTab lt, void* __restrict__ x_lp, int x_lp_bf16, const int* __restrict__ tile_list) {
  constexpr int TILE = SPAN * U;
  const TilePos p = tile_pos<TILE>(n_c, tpc, listed_tile(tile_list));
  const int l0 = lt.first_layer[p.t];
  const int L = lt.L;
  if (l0 >= L) return;
  const int o0 = threadIdx.x * 4;
  const bool uniform = (p.tile0 + p.len <= lt.off[l0 + 1]);
  v4f M[U], V[U], X[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
      M[u] = ld4(m + p.tile0 + o);
      V[u] = ld4(v + p.tile0 + o);
      X[u] = ld4(x + p.tile0 + o);
    }
  }
  if (uniform) {
    const float a = lr * coeff_c[l0];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int o = u * SPAN + o0;
      if (o < p.len) {
        v4f xn;
#pragma unroll
        for (int k = 0; k < 4; ++k)
          xn[k] = X[u][k] - a * lamb_u(M[u][k], V[u][k], X[u][k], eta, wd);
        st4(x + p.tile0 + o, xn);
        if (LPX) st4_lp(x_lp, p.tile0 + o, xn, x_lp_bf16);
      }
    }
  } else {
    const int64_t N = lt.off[L];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int o = u * SPAN + o0;
      if (o < p.len) {
        int l = l0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int64_t i = p.tile0 + o + k;
          if (i < N) {
            l = walk_layer(l, i, lt.off);
            const float a = lr * coeff_c[l];
            const float xn = X[u][k] - a * lamb_u(M[u][k], V[u][k], X[u][k], eta, wd);
            x[i] = xn;
            if (LPX) reinterpret_cast<unsigned short*>(x_lp)[i] = float_to_lp(xn, x_lp_bf16);
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// K8 a+b+c in one pass: eq. (1) with g, m, v and x read once.  A workgroup updates the moments of
// its tile, writes them, keeps u and x in registers, publishes the tile's fp64 sums of x^2 and u^2
// and arrives at its layer's barrier; the last of the layer's listed tiles to arrive sums ALL of
// the layer's segment sums in a fixed order, forms c, commits coeff_c and c_avg (Algorithm 1 line
// 2) and publishes c; the others wait for it and then update x from registers.  Same split of the
// work as for k_ratios_apply_resident (listed tiles here; everything else through
// k_warmup_moments before, whose sums wait in seg_sums, and k_warmup_apply after), same
// synchronisation and bounded waits.
// ---------------------------------------------------------------------------------------------
struct WarmSync {
  const double* seg_sums;       // [2 * segments of the 1024-element tiling] sums left by k_warmup_moments
  double* listed_sums;          // [2 * listed tiles] sums of this launch's tiles
  ListedTiles lt;
  unsigned long long* counter;  // [L * CTR_STRIDE] (generation << 32) | arrivals
  unsigned long long* flag;     // [L] (generation << 32) | bits of c
  unsigned int* errflag;
  int spin_limit;
  float* coeff_c;
  float* c_avg;
  float c_min, c_max, beta3, omb3;
};

#ifndef OB_WU_MINW
#define OB_WU_MINW 4
#endif
template <int U, int G, int GT, bool LPX>
__global__ __launch_bounds__(BLOCK, OB_WU_MINW) void k_warmup_resident(
    GradSrc g, float* __restrict__ m, float* __restrict__ v, float* __restrict__ x, WarmSync ws,
    float beta1, float omb1, float beta2, float omb2, float eta, float wd, float lr, LayerTab lt,
    void* __restrict__ x_lp, int x_lp_bf16) {
  constexpr int TILE = SPAN * U;
  __shared__ double lds[BLOCK / WAVE];
  __shared__ unsigned long long bc;
  const int tpc = ws.lt.tpc;
  const TilePos p = tile_pos<TILE>(ws.lt.n_c, tpc, ws.lt.tile_list[blockIdx.x]);
  const int sp0 = p.c * ws.lt.tpc_span + (p.t - p.c * tpc) * U;  // the tile's first span (1024-element tiling)
  const int l0 = lt.first_layer[sp0];   // the layer the tile lies in
  const LayerParts lp = layer_parts(ws.lt, l0);
  const float ca = ws.c_avg[l0];
  const int o0 = threadIdx.x * 4;
  v4f UU[U], X[U];
  v4f Ml[G], Vl[G];   // m and v of the last group: stored after the arrival, which then waits for no store
  double sx = 0.0, su = 0.0;
#pragma unroll
  for (int u0 = 0; u0 < U; u0 += G) {
    v4f Gr[G], M[G], V[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int o = (u0 + j) * SPAN + o0;
      X[u0 + j] = 0.0f; UU[u0 + j] = 0.0f;
      if (o < p.len) {
        Gr[j] = load_grad<GT>(g, p.tile0 + o);
        M[j] = ld4(m + p.tile0 + o);
        V[j] = ld4(v + p.tile0 + o);
        X[u0 + j] = ld4(x + p.tile0 + o);
      }
    }
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int o = (u0 + j) * SPAN + o0;
      if (o < p.len) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          M[j][k] = beta1 * M[j][k] + omb1 * Gr[j][k];
          V[j][k] = beta2 * V[j][k] + omb2 * (Gr[j][k] * Gr[j][k]);
        }
        if (u0 + G < U) {
          st4(m + p.tile0 + o, M[j]);
          st4(v + p.tile0 + o, V[j]);
        } else {
          Ml[j] = M[j];
          Vl[j] = V[j];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float uu = lamb_u(M[j][k], V[j][k], X[u0 + j][k], eta, wd);
          UU[u0 + j][k] = uu;
          sx += (double)X[u0 + j][k] * (double)X[u0 + j][k];
          su += (double)uu * (double)uu;
        }
      }
    }
  }
  sx = block_sum(sx, lds);
  su = block_sum(su, lds);
  // arrive: publish the tile's sums, then count; the last arriver finishes the layer
  unsigned long long* counter = &ws.counter[(int64_t)l0 * CTR_STRIDE];
  if (threadIdx.x == 0) {
    __hip_atomic_store(&ws.listed_sums[2 * (int64_t)blockIdx.x], sx, __ATOMIC_RELAXED, OB_AGENT);
    __hip_atomic_store(&ws.listed_sums[2 * (int64_t)blockIdx.x + 1], su, __ATOMIC_RELAXED, OB_AGENT);
    payload_before_arrival();
    bc = barrier_arrive(counter, lp.nl);
  }
  __syncthreads();
  const bool last = ((bc & 1ull) != 0ull);
  const unsigned int want = (unsigned int)(bc >> 32);
  __syncthreads();
#pragma unroll
  for (int j = 0; j < G; ++j) {
    const int o = (U - G + j) * SPAN + o0;
    if (o < p.len) {
      st4(m + p.tile0 + o, Ml[j]);
      st4(v + p.tile0 + o, Vl[j]);
    }
  }
  float c;
  if (last) {
    double tx = 0.0, tu = 0.0;
    struct Sums { double x, u; };
    for_layer_parts(
        lp, Sums{0.0, 0.0},   // the sums are >= +0: adding these zeros changes nothing
        [&](int i) {
          Sums v;
          v.x = __hip_atomic_load(&ws.listed_sums[2 * (int64_t)i], __ATOMIC_RELAXED, OB_AGENT);
          v.u = __hip_atomic_load(&ws.listed_sums[2 * (int64_t)i + 1], __ATOMIC_RELAXED, OB_AGENT);
          return v;
        },
        [&](const Sums& v) { tx += v.x; tu += v.u; },
        [&](int j) {   // written by an earlier kernel
          tx += ws.seg_sums[2 * (int64_t)j];
          tu += ws.seg_sums[2 * (int64_t)j + 1];
        });
    tx = block_sum(tx, lds);
    tu = block_sum(tu, lds);
    if (threadIdx.x == 0) {
      const float cc = warmup_coeff_commit(tx, tu, l0, ca, ws.coeff_c, ws.c_avg, ws.c_min, ws.c_max,
                                           ws.beta3, ws.omb3);
      bc = barrier_publish(&ws.flag[l0], counter, lp.nl, want, __float_as_uint(cc));
    }
  } else if (threadIdx.x == 0) {
    bc = barrier_wait(&ws.flag[l0], want, ws.errflag, ws.spin_limit);
  }
  __syncthreads();
  c = __uint_as_float((unsigned int)(bc & 0xffffffffull));
  const float a = lr * c;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
      v4f xn;
#pragma unroll
      for (int k = 0; k < 4; ++k) xn[k] = X[u][k] - a * UU[u][k];
      st4(x + p.tile0 + o, xn);
      if (LPX) st4_lp(x_lp, p.tile0 + o, xn, x_lp_bf16);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Momentum-scale coefficients of Appendix A.5.2, formed once at the end of warmup.  The paper gives
// no formula; the reading taken: sigma_l = ||m_l||_2/sqrt(n_l), k_l = mean_l(sigma_l)/sigma_l over
// the non-empty layers, 1 where sigma_l = 0 or the layer is empty (every layer's RMS becomes the
// mean RMS before the fused buffer is compressed).
//   a: per (tile, layer) segment the fp64 sum of m^2
//   b: one workgroup: per-layer sigma, their mean (fixed order), k_l
// ---------------------------------------------------------------------------------------------
// A workgroup takes R consecutive tiles of the 1024-element tiling (the segment tables are the
// plain kernels'), looks up what it needs to know about all of them, then requests all of them,
// then reduces them one by one: with one 128-bit load per thread in flight, and the table look-ups
// of a tile that meets a layer boundary (three dependent loads) made for every tile after its data
// had arrived, the kernel ran at half the streaming rate.
template <int R>
__global__ __launch_bounds__(BLOCK) void k_momentum_sumsq(const float* __restrict__ m,
                                                          double* __restrict__ seg_sums,
                                                          int64_t n_c, int tpc, int n_tiles, LayerTab lt,
                                                          const int* __restrict__ tile_seg0,
                                                          const int* __restrict__ seg_layer) {
  __shared__ double lds[BLOCK / WAVE];
  const int o = threadIdx.x * 4;
  const int t0 = (int)blockIdx.x * R;
  TilePos P[R];
  int l0[R], s0[R];
  int64_t end0[R];       // end of the layer the tile starts in
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int t = (t0 + r < n_tiles) ? t0 + r : n_tiles - 1;   // (a repeated last tile is skipped below)
    P[r] = tile_pos<SPAN>(n_c, tpc, t);
    l0[r] = lt.first_layer[t];
    s0[r] = tile_seg0[t];
  }
#pragma unroll
  for (int r = 0; r < R; ++r) end0[r] = lt.off[l0[r] + 1];   // off has L+2 entries
  v4f M[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    M[r] = 0.0f;
    if (t0 + r < n_tiles && l0[r] < lt.L && o < P[r].len) M[r] = ld4(m + P[r].tile0 + o);
  }
  // the usual case: all R tiles lie inside one and the same layer -- one reduction for all of them;
  // the sum goes to the first tile's segment and the other segments contribute 0 to the layer
  bool together = (t0 + R <= n_tiles) && (l0[0] < lt.L);
#pragma unroll
  for (int r = 0; r < R; ++r)
    together = together && (l0[r] == l0[0]) && (P[r].len == SPAN) && (P[r].tile0 + SPAN <= end0[r]);
  if (together) {   // uniform
    double acc = 0.0;
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int k = 0; k < 4; ++k) acc += (double)M[r][k] * (double)M[r][k];
    acc = block_sum(acc, lds);
    if (threadIdx.x == 0) {
      seg_sums[s0[0]] = acc;
#pragma unroll
      for (int r = 1; r < R; ++r) seg_sums[s0[r]] = 0.0;
    }
    return;
  }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    if (t0 + r >= n_tiles) break;          // uniform
    if (l0[r] >= lt.L) continue;           // uniform: the tile lies in the padding (it has no segment)
    const TilePos& p = P[r];
    if (p.tile0 + p.len <= end0[r]) {      // uniform: the tile lies inside one layer, its one segment
      double acc = 0.0;
      if (o < p.len) {
#pragma unroll
        for (int k = 0; k < 4; ++k) acc += (double)M[r][k] * (double)M[r][k];
      }
      acc = block_sum(acc, lds);
      if (threadIdx.x == 0) seg_sums[s0[r]] = acc;
      continue;
    }
    const int s1 = tile_seg0[p.t + 1];
    for (int s = s0[r]; s < s1; ++s) {
      const int l = seg_layer[s];
      const int64_t a = lt.off[l], b = lt.off[l + 1];
      double acc = 0.0;
      if (o < p.len) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int64_t i = p.tile0 + o + k;
          if (i >= a && i < b) acc += (double)M[r][k] * (double)M[r][k];
        }
      }
      acc = block_sum(acc, lds);
      if (threadIdx.x == 0) seg_sums[s] = acc;
    }
  }
}

// sigma[l] (fp64 scratch, [L]) from the segment sums; one workgroup per layer.
__global__ __launch_bounds__(FBLOCK) void k_layer_rms(const double* __restrict__ seg_sums,
                                                      const int* __restrict__ layer_seg0,
                                                      const int64_t* __restrict__ off,
                                                      double* __restrict__ sigma) {
  __shared__ double lds[FBLOCK / WAVE];
  const int l = blockIdx.x;
  double a = 0.0;
  const int s1 = layer_seg0[l + 1];
  for (int s = layer_seg0[l] + threadIdx.x; s < s1; s += 4 * FBLOCK) {   // four loads in flight per thread
    double v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = (s + u * FBLOCK < s1) ? seg_sums[s + u * FBLOCK] : 0.0;
#pragma unroll
    for (int u = 0; u < 4; ++u) a += v[u];
  }
  a = block_sum<FBLOCK>(a, lds);
  if (threadIdx.x == 0) {
    const int64_t n = off[l + 1] - off[l];
    sigma[l] = (n > 0) ? sqrt(a / (double)n) : 0.0;
  }
}

// mean of sigma over the non-empty layers (one workgroup, fixed order), then k_l.
__global__ __launch_bounds__(FBLOCK) void k_momentum_scale(const double* __restrict__ sigma,
                                                           const int64_t* __restrict__ off, int L,
                                                           float* __restrict__ mom_scale) {
  __shared__ double lds[FBLOCK / WAVE];
  __shared__ double mean_s;
  double a = 0.0, cnt = 0.0;
  for (int l = threadIdx.x; l < L; l += FBLOCK) {
    if (off[l + 1] > off[l]) {
      a += sigma[l];
      cnt += 1.0;
    }
  }
  a = block_sum<FBLOCK>(a, lds);
  cnt = block_sum<FBLOCK>(cnt, lds);
  if (threadIdx.x == 0) mean_s = (cnt > 0.0) ? a / cnt : 0.0;
  __syncthreads();
  const double mean = mean_s;
  for (int l = threadIdx.x; l < L; l += FBLOCK) {
    const double s = sigma[l];
    mom_scale[l] = (s > 0.0) ? (float)(mean / s) : 1.0f;
  }
}

// Diagnostics: a plain streaming copy in the shape of the N-sized kernels above (1024-element
// tiles, one 128-bit nontemporal load and store per thread).  What it reaches is the device's
// practical streaming ceiling, against which the benchmark reports every kernel next to the
// published peak.
__global__ __launch_bounds__(BLOCK) void k_diag_copy(const float* __restrict__ src, float* __restrict__ dst,
                                                     int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * SPAN + threadIdx.x * 4;
  if (i + 4 <= n) {
    st4(dst + i, ld4(src + i));
  } else {
    for (int64_t j = i; j < n; ++j) dst[j] = src[j];
  }
}

__global__ __launch_bounds__(BLOCK) void k_fill(float* __restrict__ p, int64_t n, float v) {
  const int64_t i = (int64_t)blockIdx.x * BLOCK + threadIdx.x;
  if (i < n) p[i] = v;
}

}  // namespace obk
