// libonebitlamb: HIP kernels (gfx950) and C ABI for the compression-stage step of 1-bit LAMB
// (arXiv 2104.06069, Algorithm 1) and the LAMB warmup step (eq. (1)).
//
// Build flags that the arithmetic depends on: -ffp-contract=off (one rounding per operation) and
// hipcc's default correctly rounded fp32 divide/sqrt; never -ffast-math.
//
// Layout of the work.  The padded flat buffer is W chunks of n_c elements (n_c % 256 == 0).
// Every N-sized kernel runs on "tiles": tile (c, b) is elements [c*n_c + b*TILE, +TILE) clipped
// to the chunk, so a tile never crosses a chunk boundary and its length is a multiple of 256.
// A workgroup of 256 threads owns one tile; thread t touches elements tile0 + u*1024 + 4*t + k
// (u < U, k < 4) with 128-bit loads, i.e. each wavefront-wide access covers 256 consecutive
// elements = 8 consecutive 32-bit words of the packed sign stream.
//
// Layers (tensors) are arbitrary, unaligned ranges of the flat buffer.  A host-built table gives
// the layer of each tile's first element; a tile that lies inside one layer takes a vectorised
// path with per-tile scalars, a tile that meets a layer boundary (or the padding) takes a
// per-element path that walks the offset table.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <new>
#include <string>
#include <vector>

#include "onebitlamb.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int BLOCK = 256;          // threads per workgroup (4 wavefronts of 64)
constexpr int WAVE = 64;
constexpr int SPAN = BLOCK * 4;     // elements one workgroup-wide 128-bit access covers
constexpr int U_MAIN = 4;           // accesses per thread per array in the N-sized kernels
constexpr int U_SRV = 1;            // ... in the kernels over the single server chunk
constexpr int U_RES = 16;           // ... in the single-pass worker compression (z stays in registers)
constexpr int G_RES = 2;            // loads of the single-pass kernel are issued G_RES accesses at a time
constexpr int TILE_MAIN = SPAN * U_MAIN;
constexpr int TILE_SRV = SPAN * U_SRV;
constexpr int TILE_RES = SPAN * U_RES;
#define OB_AGENT __HIP_MEMORY_SCOPE_AGENT

// ---------------------------------------------------------------------------------------------
// device helpers
// ---------------------------------------------------------------------------------------------
// Every N-sized array is read once and written once per kernel: 128-bit nontemporal (streaming)
// accesses, which measure ~10 % faster than plain ones on MI355X for these access patterns.
__device__ __forceinline__ v4f ld4(const float* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
}
__device__ __forceinline__ void st4(float* p, v4f v) {
  __builtin_nontemporal_store(v, reinterpret_cast<v4f*>(p));
}

// Sum of one double per thread over the workgroup, in a fixed order; result valid in thread 0.
__device__ __forceinline__ double block_sum(double v, double* lds /* [BLOCK/WAVE] */) {
#pragma unroll
  for (int o = WAVE / 2; o > 0; o >>= 1) v += __shfl_down(v, o, WAVE);
  const int lane = threadIdx.x & (WAVE - 1), wv = threadIdx.x / WAVE;
  __syncthreads();  // protects lds against the previous use
  if (lane == 0) lds[wv] = v;
  __syncthreads();
  double r = 0.0;
  if (threadIdx.x == 0) {
#pragma unroll
    for (int i = 0; i < BLOCK / WAVE; ++i) r += lds[i];
  }
  return r;
}

// Max of one non-NaN, non-negative float per thread over the workgroup; valid in thread 0.
__device__ __forceinline__ float block_max(float v, float* lds /* [BLOCK/WAVE] */) {
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
    for (int i = 0; i < BLOCK / WAVE; ++i) r = (lds[i] > r) ? lds[i] : r;
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

struct TilePos {
  int c;          // chunk
  int64_t tile0;  // first element
  int len;        // elements in the tile (multiple of 256)
};

template <int TILE>
__device__ __forceinline__ TilePos tile_pos(int64_t n_c, int tpc) {
  TilePos p;
  const int t = blockIdx.x;
  p.c = t / tpc;
  const int b = t - p.c * tpc;
  const int64_t in_chunk = (int64_t)b * TILE;
  p.tile0 = (int64_t)p.c * n_c + in_chunk;
  const int64_t rest = n_c - in_chunk;
  p.len = rest < TILE ? (int)rest : TILE;
  return p;
}

// ---------------------------------------------------------------------------------------------
// K1  z = k_l*(beta1*m + (1-beta1)*g) + err  (Algorithm 1 lines 6-7, Appendix A.5.2), written over
//     err, and the tile's sum of z^2 in fp64.
// ---------------------------------------------------------------------------------------------
template <int U, bool HAS_K>
__global__ __launch_bounds__(BLOCK) void k_momentum_z_sumsq(
    const float* __restrict__ g, const float* __restrict__ m, float* __restrict__ err,
    double* __restrict__ partials, int64_t n_c, int tpc, float beta1, float omb1,
    const float* __restrict__ mom_scale, const int64_t* __restrict__ off,
    const int* __restrict__ first_layer, int L) {
  constexpr int TILE = SPAN * U;
  __shared__ double lds[BLOCK / WAVE];
  const TilePos p = tile_pos<TILE>(n_c, tpc);
  const int o0 = threadIdx.x * 4;
  v4f G[U], M[U], E[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
      G[u] = ld4(g + p.tile0 + o);
      M[u] = ld4(m + p.tile0 + o);
      E[u] = ld4(err + p.tile0 + o);
    }
  }
  bool uniform = true;
  float kt = 1.0f;
  int l0 = 0;
  if (HAS_K) {
    l0 = first_layer[blockIdx.x];
    uniform = (p.tile0 + p.len <= off[l0 + 1]);
    if (uniform && l0 < L) kt = mom_scale[l0];
  }
  double acc = 0.0;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
      v4f z;
      if (!HAS_K) {
#pragma unroll
        for (int k = 0; k < 4; ++k) z[k] = (beta1 * M[u][k] + omb1 * G[u][k]) + E[u][k];
      } else if (uniform) {
#pragma unroll
        for (int k = 0; k < 4; ++k) z[k] = kt * (beta1 * M[u][k] + omb1 * G[u][k]) + E[u][k];
      } else {
        int l = l0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          l = walk_layer(l, p.tile0 + o + k, off);
          const float kk = (l < L) ? mom_scale[l] : 1.0f;
          z[k] = kk * (beta1 * M[u][k] + omb1 * G[u][k]) + E[u][k];
        }
      }
      st4(err + p.tile0 + o, z);
#pragma unroll
      for (int k = 0; k < 4; ++k) acc += (double)z[k] * (double)z[k];
    }
  }
  const double s = block_sum(acc, lds);
  if (threadIdx.x == 0) partials[blockIdx.x] = s;
}

// scale[c] = sqrt(sum of the chunk's tile partials / n_c), summed in a fixed order.
__global__ __launch_bounds__(BLOCK) void k_chunk_scale(const double* __restrict__ partials, int tpc,
                                                       int64_t n_c, float* __restrict__ scales) {
  __shared__ double lds[BLOCK / WAVE];
  const int c = blockIdx.x;
  double a = 0.0;
  for (int j = threadIdx.x; j < tpc; j += BLOCK) a += partials[(int64_t)c * tpc + j];
  const double S = block_sum(a, lds);
  if (threadIdx.x == 0) scales[c] = (float)sqrt(S / (double)n_c);
}

// ---------------------------------------------------------------------------------------------
// K2  bits = (z >= 0), packed; err <- z - (+-scale)   (Algorithm 1 line 7 / line 10)
// ---------------------------------------------------------------------------------------------
template <int U>
__global__ __launch_bounds__(BLOCK) void k_sign_pack_error(float* __restrict__ err,
                                                           uint32_t* __restrict__ packed,
                                                           const float* __restrict__ scales,
                                                           int64_t n_c, int tpc) {
  constexpr int TILE = SPAN * U;
  const TilePos p = tile_pos<TILE>(n_c, tpc);
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
    if (o < p.len) {  // uniform over the wavefront: len is a multiple of 256
      unsigned int nib = 0;
      v4f e;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const bool b = (Z[u][k] >= 0.0f);
        nib |= (b ? 1u : 0u) << k;
        e[k] = Z[u][k] - (b ? s : -s);
      }
      st4(err + p.tile0 + o, e);
      const unsigned int word = gather_word(nib);
      if ((threadIdx.x & 7) == 0) packed[(p.tile0 + o) >> 5] = word;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// K1+K2 in one pass ("resident"): Algorithm 1 lines 6-7 with each input read once.
//
// A workgroup computes z for its tile (TILE_RES elements, 64 registers per thread), publishes the
// tile's fp64 sum of squares and then waits until the whole chunk has arrived; the last workgroup
// to arrive sums the chunk's partials in a fixed order and publishes the scale; everybody then
// signs, packs and writes the error from registers.  z never goes to memory.
//
// Progress: workgroups are dispatched in index order and a chunk's tiles are consecutive indices,
// so the oldest unfinished chunk always has all of its tiles resident or dispatchable provided the
// device can hold one chunk's workgroups at once; the host only selects this kernel when twice
// that many fit.  Every wait is bounded by spin_limit polls: on expiry the workgroup raises
// *errflag, uses whatever scale it last read and exits, and all later waits end at once.
//
// Synchronisation uses relaxed agent-scope atomics whose payload travels in the atomic itself
// (partials: one double each; flag[c]: epoch in the high word, scale bits in the low word), so no
// cache write-back/invalidate is needed; the store of the partial is complete (s_waitcnt) before
// the arrival counter is incremented.  counter[c] grows by tpc per launch; epoch numbers launches.
// ---------------------------------------------------------------------------------------------
template <int U, int G, bool HAS_K>
__global__ __launch_bounds__(BLOCK, 4) void k_compress_resident(
    const float* __restrict__ g, const float* __restrict__ m, float* __restrict__ err,
    uint32_t* __restrict__ packed, float* __restrict__ scales, double* partials,
    unsigned long long* counter, unsigned long long* flag, unsigned int* errflag, int64_t n_c,
    int tpc, float beta1, float omb1, const float* __restrict__ mom_scale,
    const int64_t* __restrict__ off, const int* __restrict__ first_layer, int L,
    unsigned int epoch, int spin_limit) {
  constexpr int TILE = SPAN * U;
  __shared__ double lds[BLOCK / WAVE];
  __shared__ unsigned long long bc;
  const TilePos p = tile_pos<TILE>(n_c, tpc);
  const int o0 = threadIdx.x * 4;
  bool uniform = true;
  float kt = 1.0f;
  int l0 = 0;
  if (HAS_K) {
    l0 = first_layer[blockIdx.x];
    uniform = (p.tile0 + p.len <= off[l0 + 1]);
    if (uniform && l0 < L) kt = mom_scale[l0];
  }
  v4f Z[U];
  double acc = 0.0;
#pragma unroll
  for (int u0 = 0; u0 < U; u0 += G) {
    v4f Gr[G], M[G], E[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int o = (u0 + j) * SPAN + o0;
      if (o < p.len) {
        Gr[j] = ld4(g + p.tile0 + o);
        M[j] = ld4(m + p.tile0 + o);
        E[j] = ld4(err + p.tile0 + o);
      }
    }
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int o = (u0 + j) * SPAN + o0;
      if (o < p.len) {
        v4f z;
        if (!HAS_K) {
#pragma unroll
          for (int k = 0; k < 4; ++k) z[k] = (beta1 * M[j][k] + omb1 * Gr[j][k]) + E[j][k];
        } else if (uniform) {
#pragma unroll
          for (int k = 0; k < 4; ++k) z[k] = kt * (beta1 * M[j][k] + omb1 * Gr[j][k]) + E[j][k];
        } else {
          int l = l0;
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            l = walk_layer(l, p.tile0 + o + k, off);
            const float kk = (l < L) ? mom_scale[l] : 1.0f;
            z[k] = kk * (beta1 * M[j][k] + omb1 * Gr[j][k]) + E[j][k];
          }
        }
        Z[u0 + j] = z;
#pragma unroll
        for (int k = 0; k < 4; ++k) acc += (double)z[k] * (double)z[k];
      }
    }
  }
  const double part = block_sum(acc, lds);
  if (threadIdx.x == 0) {
    __hip_atomic_store(&partials[blockIdx.x], part, __ATOMIC_RELAXED, OB_AGENT);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // the store is complete before the add
    const unsigned long long prev =
        __hip_atomic_fetch_add(&counter[p.c], 1ull, __ATOMIC_RELAXED, OB_AGENT);
    bc = (prev + 1ull == (unsigned long long)epoch * (unsigned long long)tpc) ? 1ull : 0ull;
  }
  __syncthreads();
  const bool last = (bc != 0ull);
  __syncthreads();
  if (last) {
    double a = 0.0;
    for (int j = threadIdx.x; j < tpc; j += BLOCK)
      a += __hip_atomic_load(&partials[(int64_t)p.c * tpc + j], __ATOMIC_RELAXED, OB_AGENT);
    const double S = block_sum(a, lds);
    if (threadIdx.x == 0) {
      const float sc = (float)sqrt(S / (double)n_c);
      scales[p.c] = sc;
      const unsigned long long f = ((unsigned long long)epoch << 32) | (unsigned long long)__float_as_uint(sc);
      __hip_atomic_store(&flag[p.c], f, __ATOMIC_RELAXED, OB_AGENT);
      bc = f;
    }
  } else if (threadIdx.x == 0) {
    unsigned long long f = 0ull;
    for (int it = 0;; ++it) {
      f = __hip_atomic_load(&flag[p.c], __ATOMIC_RELAXED, OB_AGENT);
      if ((unsigned int)(f >> 32) == epoch) break;
      if (it >= spin_limit) {
        atomicOr(errflag, 1u);
        break;
      }
      if ((it & 63) == 63 && __hip_atomic_load(errflag, __ATOMIC_RELAXED, OB_AGENT) != 0u) break;
      __builtin_amdgcn_s_sleep(2);
    }
    bc = f;
  }
  __syncthreads();
  const float s = __uint_as_float((unsigned int)(bc & 0xffffffffull));
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
      unsigned int nib = 0;
      v4f e;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const bool b = (Z[u][k] >= 0.0f);
        nib |= (b ? 1u : 0u) << k;
        e[k] = Z[u][k] - (b ? s : -s);
      }
      st4(err + p.tile0 + o, e);
      const unsigned int word = gather_word(nib);
      if ((threadIdx.x & 7) == 0) packed[(p.tile0 + o) >> 5] = word;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// K3  server: zb = (sum_w +-s_w, sequentially) * (1/W) + err_server, written over err_server, and
//     the tile's sum of zb^2   (Algorithm 1 line 10)
// ---------------------------------------------------------------------------------------------
template <int U>
__global__ __launch_bounds__(BLOCK) void k_server_unpack_avg(
    const uint32_t* __restrict__ packed_in, const float* __restrict__ scales_in,
    float* __restrict__ err_s, double* __restrict__ partials, int64_t n_c, int W, float invW) {
  constexpr int TILE = SPAN * U;
  __shared__ double lds[BLOCK / WAVE];
  const TilePos p = tile_pos<TILE>(n_c, (int)gridDim.x);  // one chunk: c == 0
  const int o0 = threadIdx.x * 4;
  const int sh = 4 * (threadIdx.x & 7);
  const int64_t wpc = n_c >> 5;  // words per worker block
  float acc[U][4];
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int k = 0; k < 4; ++k) acc[u][k] = 0.0f;
  // workers strictly in order 0..W-1 (the fp32 sum is order dependent); the loads of GROUP
  // workers are issued together so that their latencies overlap
  constexpr int GROUP = 8;
  for (int w0 = 0; w0 < W; w0 += GROUP) {
    unsigned int word[GROUP][U];
#pragma unroll
    for (int j = 0; j < GROUP; ++j) {
      const int w = (w0 + j < W) ? w0 + j : W - 1;
      const uint32_t* row = packed_in + (int64_t)w * wpc;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int o = u * SPAN + o0;
        word[j][u] = (o < p.len) ? row[(p.tile0 + o) >> 5] : 0u;
      }
    }
#pragma unroll
    for (int j = 0; j < GROUP; ++j) {
      if (w0 + j < W) {
        const float s = scales_in[w0 + j];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const unsigned int nib = word[j][u] >> sh;
#pragma unroll
          for (int k = 0; k < 4; ++k) acc[u][k] = acc[u][k] + (((nib >> k) & 1u) ? s : -s);
        }
      }
    }
  }
  double sq = 0.0;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
      const v4f e = ld4(err_s + p.tile0 + o);
      v4f z;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        z[k] = acc[u][k] * invW + e[k];
        sq += (double)z[k] * (double)z[k];
      }
      st4(err_s + p.tile0 + o, z);
    }
  }
  const double s = block_sum(sq, lds);
  if (threadIdx.x == 0) partials[blockIdx.x] = s;
}

// ---------------------------------------------------------------------------------------------
// K5  per layer: reconstructed gradient, fresh variance, max(v_frozen/v_fresh)
//     (Algorithm 1 lines 13, 15-17)
// ---------------------------------------------------------------------------------------------
template <int U, bool HAS_K>
__global__ __launch_bounds__(BLOCK) void k_ratios_pass(
    const uint32_t* __restrict__ packed, const float* __restrict__ sscales,
    const float* __restrict__ m, float* __restrict__ v_fresh, const float* __restrict__ v_frozen,
    float* __restrict__ seg_max, int64_t n_c, int tpc, float beta1, float omb1, float beta2, float omb2,
    const float* __restrict__ mom_scale, const int64_t* __restrict__ off,
    const int* __restrict__ first_layer, const int* __restrict__ tile_seg0,
    const int* __restrict__ seg_layer, int L) {
  constexpr int TILE = SPAN * U;
  __shared__ float lds[BLOCK / WAVE];
  const TilePos p = tile_pos<TILE>(n_c, tpc);
  const int l0 = first_layer[blockIdx.x];
  if (l0 >= L) return;  // tile lies in the padding (it has no segment)
  const int o0 = threadIdx.x * 4;
  const int sh = 4 * (threadIdx.x & 7);
  const float ss = sscales[p.c];
  const bool uniform = (p.tile0 + p.len <= off[l0 + 1]);
  unsigned int NB[U];
  v4f M[U], VF[U], VZ[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
      NB[u] = packed[(p.tile0 + o) >> 5] >> sh;
      M[u] = ld4(m + p.tile0 + o);
      VF[u] = ld4(v_fresh + p.tile0 + o);
      VZ[u] = ld4(v_frozen + p.tile0 + o);
    }
  }
  if (uniform) {
    const float sp = HAS_K ? ss / mom_scale[l0] : ss;
    float r = 0.0f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int o = u * SPAN + o0;
      if (o < p.len) {
        v4f vf;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float mt = ((NB[u] >> k) & 1u) ? sp : -sp;
          const float gr = (mt - beta1 * M[u][k]) / omb1;
          vf[k] = beta2 * VF[u][k] + omb2 * (gr * gr);
          const float q = VZ[u][k] / vf[k];
          if (q > r) r = q;
        }
        st4(v_fresh + p.tile0 + o, vf);
      }
    }
    r = block_max(r, lds);
    if (threadIdx.x == 0) seg_max[tile_seg0[blockIdx.x]] = r;
  } else {
    const int64_t N = off[L];
    // quotient of every element (kept in VZ), then one workgroup max per (tile, layer) segment
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
            l = walk_layer(l, i, off);
            const float sp = HAS_K ? ss / mom_scale[l] : ss;
            const float mt = ((NB[u] >> k) & 1u) ? sp : -sp;
            const float gr = (mt - beta1 * M[u][k]) / omb1;
            const float vf = beta2 * VF[u][k] + omb2 * (gr * gr);
            v_fresh[i] = vf;
            q = VZ[u][k] / vf;
          }
          VZ[u][k] = q;
        }
      }
    }
    const int s0 = tile_seg0[blockIdx.x], s1 = tile_seg0[blockIdx.x + 1];
    for (int s = s0; s < s1; ++s) {
      const int l = seg_layer[s];
      const int64_t a = off[l], b = off[l + 1];
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
      r = block_max(r, lds);
      if (threadIdx.x == 0) seg_max[s] = r;
    }
  }
}

// K6  per layer: max over the layer's segments (0 for an empty layer), then Algorithm 1 lines 18-20.
__global__ __launch_bounds__(BLOCK) void k_ratios_finalize(const float* __restrict__ seg_max,
                                                           const int* __restrict__ layer_seg0,
                                                           const float* __restrict__ c_avg,
                                                           float* __restrict__ r_prev,
                                                           float* __restrict__ coeff_c,
                                                           float one_m_thr, float one_p_thr,
                                                           float r_min, float r_max) {
  __shared__ float lds[BLOCK / WAVE];
  const int l = blockIdx.x;
  const int s0 = layer_seg0[l], s1 = layer_seg0[l + 1];
  float r = 0.0f;
  for (int s = s0 + threadIdx.x; s < s1; s += BLOCK) {
    const float q = seg_max[s];
    if (q > r) r = q;
  }
  r = block_max(r, lds);
  if (threadIdx.x == 0) {
    const float rp = r_prev[l];
    const float lo = one_m_thr * rp, hi = one_p_thr * rp;
    r = (r > lo) ? r : lo;
    r = (r < hi) ? r : hi;
    r = (r > r_min) ? r : r_min;
    r = (r < r_max) ? r : r_max;
    r_prev[l] = r;
    coeff_c[l] = r * c_avg[l];
  }
}

// ---------------------------------------------------------------------------------------------
// K7  x <- x - (lr*c_l) * m_t/(sqrt(v_frozen)+eta);  m <- m_t   (Algorithm 1 lines 13, 21)
// ---------------------------------------------------------------------------------------------
template <int U, bool HAS_K>
__global__ __launch_bounds__(BLOCK) void k_decompress_apply(
    const uint32_t* __restrict__ packed, const float* __restrict__ sscales,
    const float* __restrict__ v_frozen, float* __restrict__ x, float* __restrict__ m,
    const float* __restrict__ coeff_c, int64_t n_c, int tpc, float lr, float eta,
    const float* __restrict__ mom_scale, const int64_t* __restrict__ off,
    const int* __restrict__ first_layer, int L) {
  constexpr int TILE = SPAN * U;
  const TilePos p = tile_pos<TILE>(n_c, tpc);
  const int l0 = first_layer[blockIdx.x];
  if (l0 >= L) return;
  const int o0 = threadIdx.x * 4;
  const int sh = 4 * (threadIdx.x & 7);
  const float ss = sscales[p.c];
  const bool uniform = (p.tile0 + p.len <= off[l0 + 1]);
  unsigned int NB[U];
  v4f X[U], VZ[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
      NB[u] = packed[(p.tile0 + o) >> 5] >> sh;
      VZ[u] = ld4(v_frozen + p.tile0 + o);
      X[u] = ld4(x + p.tile0 + o);
    }
  }
  if (uniform) {
    const float sp = HAS_K ? ss / mom_scale[l0] : ss;
    const float a = lr * coeff_c[l0];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int o = u * SPAN + o0;
      if (o < p.len) {
        v4f xn, mn;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float mt = ((NB[u] >> k) & 1u) ? sp : -sp;
          const float uu = mt / (sqrtf(VZ[u][k]) + eta);
          xn[k] = X[u][k] - a * uu;
          mn[k] = mt;
        }
        st4(x + p.tile0 + o, xn);
        st4(m + p.tile0 + o, mn);
      }
    }
  } else {
    const int64_t N = off[L];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int o = u * SPAN + o0;
      if (o < p.len) {
        int l = l0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int64_t i = p.tile0 + o + k;
          if (i < N) {
            l = walk_layer(l, i, off);
            const float sp = HAS_K ? ss / mom_scale[l] : ss;
            const float a = lr * coeff_c[l];
            const float mt = ((NB[u] >> k) & 1u) ? sp : -sp;
            const float uu = mt / (sqrtf(VZ[u][k]) + eta);
            x[i] = X[u][k] - a * uu;
            m[i] = mt;
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

template <int U>
__global__ __launch_bounds__(BLOCK) void k_warmup_moments(
    const float* __restrict__ g, float* __restrict__ m, float* __restrict__ v,
    const float* __restrict__ x, double* __restrict__ seg_sums /* [2*n_segs] */, int64_t n_c,
    int tpc, float beta1, float omb1, float beta2, float omb2, float eta, float wd,
    const int64_t* __restrict__ off, const int* __restrict__ first_layer,
    const int* __restrict__ tile_seg0, const int* __restrict__ seg_layer, int L) {
  constexpr int TILE = SPAN * U;
  __shared__ double lds[BLOCK / WAVE];
  const TilePos p = tile_pos<TILE>(n_c, tpc);
  const int l0 = first_layer[blockIdx.x];
  if (l0 >= L) return;
  const int o0 = threadIdx.x * 4;
  const bool uniform = (p.tile0 + p.len <= off[l0 + 1]);
  v4f G[U], M[U], V[U], X[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int o = u * SPAN + o0;
    if (o < p.len) {
      G[u] = ld4(g + p.tile0 + o);
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
  const int s0 = tile_seg0[blockIdx.x];
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
    const int64_t N = off[L];
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
    const int s1 = tile_seg0[blockIdx.x + 1];
    for (int s = s0; s < s1; ++s) {
      const int l = seg_layer[s];
      const int64_t a = off[l], b = off[l + 1];
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

__global__ __launch_bounds__(BLOCK) void k_warmup_coeff(const double* __restrict__ seg_sums,
                                                        const int* __restrict__ layer_seg0,
                                                        float* __restrict__ coeff_c,
                                                        float* __restrict__ c_avg, float c_min,
                                                        float c_max, float beta3, float omb3) {
  __shared__ double lds[BLOCK / WAVE];
  const int l = blockIdx.x;
  const int s0 = layer_seg0[l], s1 = layer_seg0[l + 1];
  double sx = 0.0, su = 0.0;
  for (int s = s0 + threadIdx.x; s < s1; s += BLOCK) {
    sx += seg_sums[2 * (int64_t)s];
    su += seg_sums[2 * (int64_t)s + 1];
  }
  sx = block_sum(sx, lds);
  su = block_sum(su, lds);
  if (threadIdx.x == 0) {
    const float nx = (float)sqrt(sx), nu = (float)sqrt(su);
    float c = nx / nu;
    c = (c > c_min) ? c : c_min;
    c = (c < c_max) ? c : c_max;
    coeff_c[l] = c;
    c_avg[l] = beta3 * c_avg[l] + omb3 * c;
  }
}

template <int U>
__global__ __launch_bounds__(BLOCK) void k_warmup_apply(
    const float* __restrict__ m, const float* __restrict__ v, float* __restrict__ x,
    const float* __restrict__ coeff_c, int64_t n_c, int tpc, float lr, float eta, float wd,
    const int64_t* __restrict__ off, const int* __restrict__ first_layer, int L) {
  constexpr int TILE = SPAN * U;
  const TilePos p = tile_pos<TILE>(n_c, tpc);
  const int l0 = first_layer[blockIdx.x];
  if (l0 >= L) return;
  const int o0 = threadIdx.x * 4;
  const bool uniform = (p.tile0 + p.len <= off[l0 + 1]);
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
      }
    }
  } else {
    const int64_t N = off[L];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int o = u * SPAN + o0;
      if (o < p.len) {
        int l = l0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int64_t i = p.tile0 + o + k;
          if (i < N) {
            l = walk_layer(l, i, off);
            const float a = lr * coeff_c[l];
            x[i] = X[u][k] - a * lamb_u(M[u][k], V[u][k], X[u][k], eta, wd);
          }
        }
      }
    }
  }
}

__global__ __launch_bounds__(BLOCK) void k_fill(float* __restrict__ p, int64_t n, float v) {
  const int64_t i = (int64_t)blockIdx.x * BLOCK + threadIdx.x;
  if (i < n) p[i] = v;
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
enum KernelId {
  KID_MOMENTUM_Z = 0,
  KID_COMPRESS_RESIDENT,
  KID_CHUNK_SCALE,
  KID_SIGN_PACK,
  KID_SERVER_AVG,
  KID_SERVER_SCALE,
  KID_SERVER_PACK,
  KID_RATIOS_PASS,
  KID_RATIOS_FINALIZE,
  KID_APPLY,
  KID_WARMUP_MOMENTS,
  KID_WARMUP_COEFF,
  KID_WARMUP_APPLY,
  KID_FILL,
  KID_COPY,
  KID_COUNT
};
const char* const kKernelNames[KID_COUNT] = {
    "momentum_z_sumsq", "compress_resident", "chunk_scale",     "sign_pack_error", "server_unpack_avg",
    "server_scale",     "server_sign_pack", "ratios_pass",     "ratios_finalize",
    "decompress_apply", "warmup_moments",   "warmup_coeff",    "warmup_apply",
    "fill",             "copy"};

struct ProfRec {
  int kid;
  hipEvent_t e0, e1;
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
  float* d_seg_max = nullptr;     // [n_segs] per-segment max(v_frozen/v_fresh)
  // single-pass worker compression (k_compress_resident)
  bool resident = false;          // selected at create when the device can hold 2 chunks of tiles
  int tpc_res = 0, n_tiles_res = 0;
  int* d_first_layer_res = nullptr;        // [n_tiles_res]
  double* d_partials_res = nullptr;        // [n_tiles_res]
  unsigned long long* d_counter = nullptr; // [W] arrivals, monotone
  unsigned long long* d_flag = nullptr;    // [W] (epoch << 32) | scale bits
  unsigned int* d_errflag = nullptr;       // [1] raised when a bounded wait expired
  unsigned int epoch = 0;
  int spin_limit = 1 << 20;
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
  void begin(int kid) {
    if (!ctx->profile || !ok) return;
    ProfRec r;
    r.kid = kid;
    ok = hip_ok(ctx, hipEventCreate(&r.e0), "hipEventCreate") &&
         hip_ok(ctx, hipEventCreate(&r.e1), "hipEventCreate") &&
         hip_ok(ctx, hipEventRecord(r.e0, stream), "hipEventRecord");
    if (ok) ctx->prof.push_back(r);
  }
  void end(const char* name) {
    if (!ok) return;
    ok = hip_ok(ctx, hipGetLastError(), name);
    if (ok && ctx->profile) ok = hip_ok(ctx, hipEventRecord(ctx->prof.back().e1, stream), "hipEventRecord");
  }
};

#define OB_LAUNCH(la, kid, kernel, grid, ...)                                     \
  do {                                                                            \
    if ((la).ok && (grid) > 0) {                                                  \
      (la).begin(kid);                                                            \
      hipLaunchKernelGGL(kernel, dim3((unsigned)(grid)), dim3(BLOCK), 0, (la).stream, __VA_ARGS__); \
      (la).end(kKernelNames[kid]);                                                \
    }                                                                             \
  } while (0)

template <class T>
bool upload(ob_lamb_ctx* ctx, T** dst, const std::vector<T>& src) {
  const size_t bytes = src.size() * sizeof(T);
  if (!hip_ok(ctx, hipMalloc(reinterpret_cast<void**>(dst), bytes ? bytes : sizeof(T)), "hipMalloc")) return false;
  if (bytes && !hip_ok(ctx, hipMemcpy(*dst, src.data(), bytes, hipMemcpyHostToDevice), "hipMemcpy")) return false;
  return true;
}

template <class T>
bool alloc_zero(ob_lamb_ctx* ctx, T** dst, size_t count) {
  const size_t bytes = (count ? count : 1) * sizeof(T);
  if (!hip_ok(ctx, hipMalloc(reinterpret_cast<void**>(dst), bytes), "hipMalloc")) return false;
  return hip_ok(ctx, hipMemset(*dst, 0, bytes), "hipMemset");
}

ob_status check_common(const ob_lamb_ctx* ctx, const ob_lamb_state* st) {
  if (!ctx || !st) return OB_ERR_NULL;
  return OB_OK;
}

#define REQUIRE_PTR(p)                    \
  do {                                    \
    if ((p) == nullptr) return OB_ERR_NULL; \
    if (misaligned(p)) return OB_ERR_ALIGN; \
  } while (0)

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
  }
  return "unknown status";
}

const char* ob_lamb_last_hip_error(const ob_lamb_ctx* ctx) { return ctx ? ctx->hip_err.c_str() : ""; }

ob_status ob_lamb_create(const ob_lamb_config* cfg, ob_lamb_ctx** out) {
  if (out) *out = nullptr;
  if (!cfg || !out || !cfg->layer_offsets) return OB_ERR_NULL;
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

  ob_lamb_ctx* ctx = new (std::nothrow) ob_lamb_ctx();
  if (!ctx) return OB_ERR_ARG;
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

  const int64_t tpc = (ctx->n_c + TILE_MAIN - 1) / TILE_MAIN;
  const int64_t n_tiles = tpc * ctx->W;
  const int64_t tpc_srv = (ctx->n_c + TILE_SRV - 1) / TILE_SRV;
  if (n_tiles > 0x7fffffff || tpc_srv > 0x7fffffff) { delete ctx; return OB_ERR_ARG; }
  ctx->tpc = (int)tpc;
  ctx->n_tiles = (int)n_tiles;
  ctx->tpc_srv = (int)tpc_srv;

  // tile tables: layer of each tile's first element (L = padding) and the (tile, layer) segments
  const int64_t* off = cfg->layer_offsets;
  std::vector<int64_t> h_off((size_t)L + 2);
  for (int64_t l = 0; l <= L; ++l) h_off[(size_t)l] = off[l];
  h_off[(size_t)L + 1] = std::numeric_limits<int64_t>::max();
  std::vector<int> first((size_t)n_tiles), tile_seg0((size_t)n_tiles + 1), seg_layer;
  std::vector<int> layer_seg0((size_t)L + 1, 0);
  for (int64_t t = 0; t < n_tiles; ++t) {
    const int64_t c = t / tpc, b = t % tpc;
    const int64_t tile0 = c * ctx->n_c + b * TILE_MAIN;
    const int64_t tile1 = std::min(tile0 + TILE_MAIN, (c + 1) * ctx->n_c);
    // first layer: the non-empty layer that holds tile0 (binary search on off)
    int64_t lo = 0, hi = L + 1;  // h_off[lo] <= tile0 < h_off[hi]
    while (hi - lo > 1) {
      const int64_t mid = (lo + hi) / 2;
      if (h_off[(size_t)mid] <= tile0) lo = mid; else hi = mid;
    }
    first[(size_t)t] = (int)lo;  // lo == L when tile0 >= N
    tile_seg0[(size_t)t] = (int)seg_layer.size();
    for (int64_t l = lo; l < L && off[l] < tile1; ++l) {
      const int64_t a = std::max(off[l], tile0), e = std::min(off[l + 1], tile1);
      if (e > a) seg_layer.push_back((int)l);
    }
  }
  tile_seg0[(size_t)n_tiles] = (int)seg_layer.size();
  ctx->n_segs = (int)seg_layer.size();
  {
    // segments are ordered by position, hence grouped by layer
    std::vector<int> count((size_t)L, 0);
    for (int l : seg_layer) ++count[(size_t)l];
    for (int64_t l = 0; l < L; ++l) layer_seg0[(size_t)l + 1] = layer_seg0[(size_t)l] + count[(size_t)l];
  }

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
    // kernel's comment); it is used only when twice that many fit, else the two-pass kernels run.
    int per_cu = 0, cus = 0;
    ok = hip_ok(ctx, hipOccupancyMaxActiveBlocksPerMultiprocessor(
                         &per_cu, k_compress_resident<U_RES, G_RES, true>, BLOCK, 0),
                "hipOccupancyMaxActiveBlocksPerMultiprocessor") &&
         hip_ok(ctx, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, ctx->device),
                "hipDeviceGetAttribute");
    const int64_t slots = (int64_t)per_cu * cus;
    const char* env = getenv("OB_LAMB_TWO_PASS");
    ctx->resident = ok && !(env && env[0] == '1') && 2 * (tpc_res + 8) <= slots;
  }
  ok = ok && upload(ctx, &ctx->d_first_layer_res, first_res) &&
       alloc_zero(ctx, &ctx->d_partials_res, (size_t)ctx->n_tiles_res) &&
       alloc_zero(ctx, &ctx->d_counter, (size_t)ctx->W) && alloc_zero(ctx, &ctx->d_flag, (size_t)ctx->W) &&
       alloc_zero(ctx, &ctx->d_errflag, 1);
  ok = ok && upload(ctx, &ctx->d_off, h_off) && upload(ctx, &ctx->d_first_layer, first) &&
       upload(ctx, &ctx->d_tile_seg0, tile_seg0) && upload(ctx, &ctx->d_seg_layer, seg_layer) &&
       upload(ctx, &ctx->d_layer_seg0, layer_seg0) &&
       alloc_zero(ctx, &ctx->d_partials, (size_t)n_tiles) &&
       alloc_zero(ctx, &ctx->d_partials_srv, (size_t)tpc_srv) &&
       alloc_zero(ctx, &ctx->d_seg_sums, 2 * (size_t)ctx->n_segs) &&
       alloc_zero(ctx, &ctx->d_seg_max, (size_t)ctx->n_segs);
  ok = ok && hip_ok(ctx, hipDeviceSynchronize(), "hipDeviceSynchronize");
  if (!ok) {
    ob_lamb_destroy(ctx);
    return OB_ERR_HIP;
  }
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
                  ctx->d_partials, ctx->d_partials_srv, ctx->d_seg_sums, ctx->d_seg_max,
                  ctx->d_first_layer_res, ctx->d_partials_res, ctx->d_counter, ctx->d_flag, ctx->d_errflag};
  for (void* p : ptrs)
    if (p) (void)hipFree(p);
  delete ctx;
}

int64_t ob_lamb_num_params(const ob_lamb_ctx* ctx) { return ctx ? ctx->N : 0; }
int64_t ob_lamb_padded_len(const ob_lamb_ctx* ctx) { return ctx ? ctx->n_pad : 0; }
int64_t ob_lamb_chunk_len(const ob_lamb_ctx* ctx) { return ctx ? ctx->n_c : 0; }

ob_status ob_lamb_warmup_step(ob_lamb_ctx* ctx, const ob_lamb_state* st, const float* grad, float lr,
                              void* hip_stream) {
  if (ob_status s = check_common(ctx, st)) return s;
  REQUIRE_PTR(grad); REQUIRE_PTR(st->x); REQUIRE_PTR(st->m); REQUIRE_PTR(st->v_fresh);
  if (!st->c_avg || !st->coeff_c) return OB_ERR_NULL;
  if (!std::isfinite(lr)) return OB_ERR_ARG;
  Launch la(ctx, hip_stream);
  OB_LAUNCH(la, KID_WARMUP_MOMENTS, (k_warmup_moments<U_MAIN>), ctx->n_tiles, grad, st->m, st->v_fresh,
            st->x, ctx->d_seg_sums, ctx->n_c, ctx->tpc, ctx->beta1, ctx->omb1, ctx->beta2, ctx->omb2,
            ctx->eta, ctx->wd, ctx->d_off, ctx->d_first_layer, ctx->d_tile_seg0, ctx->d_seg_layer,
            (int)ctx->L);
  OB_LAUNCH(la, KID_WARMUP_COEFF, k_warmup_coeff, (int)ctx->L, ctx->d_seg_sums, ctx->d_layer_seg0,
            st->coeff_c, st->c_avg, ctx->c_min, ctx->c_max, ctx->beta3, ctx->omb3);
  OB_LAUNCH(la, KID_WARMUP_APPLY, (k_warmup_apply<U_MAIN>), ctx->n_tiles, st->m, st->v_fresh, st->x,
            st->coeff_c, ctx->n_c, ctx->tpc, lr, ctx->eta, ctx->wd, ctx->d_off, ctx->d_first_layer,
            (int)ctx->L);
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_freeze(ob_lamb_ctx* ctx, const ob_lamb_state* st, void* hip_stream) {
  if (ob_status s = check_common(ctx, st)) return s;
  REQUIRE_PTR(st->v_fresh); REQUIRE_PTR(st->v_frozen);
  if (!st->r_prev) return OB_ERR_NULL;
  Launch la(ctx, hip_stream);
  la.begin(KID_COPY);
  if (la.ok)
    la.ok = hip_ok(ctx, hipMemcpyAsync(st->v_frozen, st->v_fresh, (size_t)ctx->n_pad * sizeof(float),
                                       hipMemcpyDeviceToDevice, la.stream), "hipMemcpyAsync");
  la.end("copy");
  OB_LAUNCH(la, KID_FILL, k_fill, (int)((ctx->L + BLOCK - 1) / BLOCK), st->r_prev, ctx->L, 1.0f);
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_compress_local(ob_lamb_ctx* ctx, const ob_lamb_state* st, const float* grad,
                                 uint32_t* packed_out, float* scales_out, void* hip_stream) {
  if (ob_status s = check_common(ctx, st)) return s;
  REQUIRE_PTR(grad); REQUIRE_PTR(st->m); REQUIRE_PTR(st->err_worker); REQUIRE_PTR(packed_out);
  if (!scales_out) return OB_ERR_NULL;
  Launch la(ctx, hip_stream);
  if (ctx->resident) {
    ctx->epoch += 1;
    if (st->mom_scale)
      OB_LAUNCH(la, KID_COMPRESS_RESIDENT, (k_compress_resident<U_RES, G_RES, true>), ctx->n_tiles_res, grad,
                st->m, st->err_worker, packed_out, scales_out, ctx->d_partials_res, ctx->d_counter,
                ctx->d_flag, ctx->d_errflag, ctx->n_c, ctx->tpc_res, ctx->beta1, ctx->omb1, st->mom_scale,
                ctx->d_off, ctx->d_first_layer_res, (int)ctx->L, ctx->epoch, ctx->spin_limit);
    else
      OB_LAUNCH(la, KID_COMPRESS_RESIDENT, (k_compress_resident<U_RES, G_RES, false>), ctx->n_tiles_res, grad,
                st->m, st->err_worker, packed_out, scales_out, ctx->d_partials_res, ctx->d_counter,
                ctx->d_flag, ctx->d_errflag, ctx->n_c, ctx->tpc_res, ctx->beta1, ctx->omb1, st->mom_scale,
                ctx->d_off, ctx->d_first_layer_res, (int)ctx->L, ctx->epoch, ctx->spin_limit);
    return la.ok ? OB_OK : OB_ERR_HIP;
  }
  if (st->mom_scale)
    OB_LAUNCH(la, KID_MOMENTUM_Z, (k_momentum_z_sumsq<U_MAIN, true>), ctx->n_tiles, grad, st->m,
              st->err_worker, ctx->d_partials, ctx->n_c, ctx->tpc, ctx->beta1, ctx->omb1, st->mom_scale,
              ctx->d_off, ctx->d_first_layer, (int)ctx->L);
  else
    OB_LAUNCH(la, KID_MOMENTUM_Z, (k_momentum_z_sumsq<U_MAIN, false>), ctx->n_tiles, grad, st->m,
              st->err_worker, ctx->d_partials, ctx->n_c, ctx->tpc, ctx->beta1, ctx->omb1, st->mom_scale,
              ctx->d_off, ctx->d_first_layer, (int)ctx->L);
  OB_LAUNCH(la, KID_CHUNK_SCALE, k_chunk_scale, ctx->W, ctx->d_partials, ctx->tpc, ctx->n_c, scales_out);
  OB_LAUNCH(la, KID_SIGN_PACK, (k_sign_pack_error<U_MAIN>), ctx->n_tiles, st->err_worker, packed_out,
            scales_out, ctx->n_c, ctx->tpc);
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_server_reduce(ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_in,
                                const float* scales_in, uint32_t* packed_out, float* scale_out,
                                void* hip_stream) {
  if (ob_status s = check_common(ctx, st)) return s;
  REQUIRE_PTR(packed_in); REQUIRE_PTR(packed_out); REQUIRE_PTR(st->err_server);
  if (!scales_in || !scale_out) return OB_ERR_NULL;
  Launch la(ctx, hip_stream);
  OB_LAUNCH(la, KID_SERVER_AVG, (k_server_unpack_avg<U_SRV>), ctx->tpc_srv, packed_in, scales_in,
            st->err_server, ctx->d_partials_srv, ctx->n_c, (int)ctx->W, ctx->invW);
  OB_LAUNCH(la, KID_SERVER_SCALE, k_chunk_scale, 1, ctx->d_partials_srv, ctx->tpc_srv, ctx->n_c, scale_out);
  OB_LAUNCH(la, KID_SERVER_PACK, (k_sign_pack_error<U_SRV>), ctx->tpc_srv, st->err_server, packed_out,
            scale_out, ctx->n_c, ctx->tpc_srv);
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_layer_ratios(ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                               const float* server_scales, void* hip_stream) {
  if (ob_status s = check_common(ctx, st)) return s;
  REQUIRE_PTR(packed_all); REQUIRE_PTR(st->m); REQUIRE_PTR(st->v_fresh); REQUIRE_PTR(st->v_frozen);
  if (!server_scales || !st->c_avg || !st->r_prev || !st->coeff_c) return OB_ERR_NULL;
  Launch la(ctx, hip_stream);
  if (st->mom_scale)
    OB_LAUNCH(la, KID_RATIOS_PASS, (k_ratios_pass<U_MAIN, true>), ctx->n_tiles, packed_all, server_scales,
              st->m, st->v_fresh, st->v_frozen, ctx->d_seg_max, ctx->n_c, ctx->tpc, ctx->beta1, ctx->omb1,
              ctx->beta2, ctx->omb2, st->mom_scale, ctx->d_off, ctx->d_first_layer, ctx->d_tile_seg0,
              ctx->d_seg_layer, (int)ctx->L);
  else
    OB_LAUNCH(la, KID_RATIOS_PASS, (k_ratios_pass<U_MAIN, false>), ctx->n_tiles, packed_all, server_scales,
              st->m, st->v_fresh, st->v_frozen, ctx->d_seg_max, ctx->n_c, ctx->tpc, ctx->beta1, ctx->omb1,
              ctx->beta2, ctx->omb2, st->mom_scale, ctx->d_off, ctx->d_first_layer, ctx->d_tile_seg0,
              ctx->d_seg_layer, (int)ctx->L);
  OB_LAUNCH(la, KID_RATIOS_FINALIZE, k_ratios_finalize, (int)ctx->L, ctx->d_seg_max, ctx->d_layer_seg0,
            st->c_avg, st->r_prev, st->coeff_c, ctx->one_m_thr, ctx->one_p_thr, ctx->r_min, ctx->r_max);
  return la.ok ? OB_OK : OB_ERR_HIP;
}

ob_status ob_lamb_decompress_apply(ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                                   const float* server_scales, float lr, void* hip_stream) {
  if (ob_status s = check_common(ctx, st)) return s;
  REQUIRE_PTR(packed_all); REQUIRE_PTR(st->m); REQUIRE_PTR(st->x); REQUIRE_PTR(st->v_frozen);
  if (!server_scales || !st->coeff_c) return OB_ERR_NULL;
  if (!std::isfinite(lr)) return OB_ERR_ARG;
  Launch la(ctx, hip_stream);
  if (st->mom_scale)
    OB_LAUNCH(la, KID_APPLY, (k_decompress_apply<U_MAIN, true>), ctx->n_tiles, packed_all, server_scales,
              st->v_frozen, st->x, st->m, st->coeff_c, ctx->n_c, ctx->tpc, lr, ctx->eta, st->mom_scale,
              ctx->d_off, ctx->d_first_layer, (int)ctx->L);
  else
    OB_LAUNCH(la, KID_APPLY, (k_decompress_apply<U_MAIN, false>), ctx->n_tiles, packed_all, server_scales,
              st->v_frozen, st->x, st->m, st->coeff_c, ctx->n_c, ctx->tpc, lr, ctx->eta, st->mom_scale,
              ctx->d_off, ctx->d_first_layer, (int)ctx->L);
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
  ctx->epoch = 0;
  (void)hipMemset(ctx->d_counter, 0, sizeof(unsigned long long) * (size_t)ctx->W);
  (void)hipMemset(ctx->d_flag, 0, sizeof(unsigned long long) * (size_t)ctx->W);
  (void)hipMemset(ctx->d_errflag, 0, sizeof(unsigned int));
  (void)hipDeviceSynchronize();
  return OB_ERR_STATE;
}

int32_t ob_lamb_uses_single_pass(const ob_lamb_ctx* ctx) { return (ctx && ctx->resident) ? 1 : 0; }

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
