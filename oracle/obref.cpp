// obref -- CPU oracle for the 1-bit LAMB compression-stage step.  Test infrastructure only:
// see obref.h for what may load it and for the list of readings it fixes.
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -fno-fast-math -shared -fPIC -pthread obref.cpp -o libobref.so
// Every loop below is scalar and in the order the paper states the step; T is float for the
// oracle proper and double for the shadow the algebraic pins use.
#include "obref.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <thread>
#include <vector>

namespace {

// clip(x, a, b) := min{max{x, a}, b} as printed under eq. (1); NaN -> a.
template <class T>
inline T clip(T x, T a, T b) {
  T y = (x > a) ? x : a;
  return (y < b) ? y : b;
}

inline bool get_bit(const uint8_t* bits, int64_t i) { return (bits[i >> 3] >> (i & 7)) & 1u; }

// C[z]: sign bits and one scale, scale = ||z||_2/sqrt(n) so that the decompressed vector
// keeps the L2 norm of z (Section 2).  Error feedback of Algorithm 1 lines 7 and 10.
template <class T>
void compress_chunk(const T* z, int64_t n, uint8_t* bits, T* scale, T* err) {
  double S = 0.0;
  for (int64_t i = 0; i < n; ++i) S += (double)z[i] * (double)z[i];
  const T s = (T)std::sqrt(S / (double)n);
  for (int64_t i = 0; i < n; i += 8) {
    unsigned byte = 0;
    for (int j = 0; j < 8; ++j) {
      const T zi = z[i + j];
      const bool b = (zi >= (T)0);
      if (b) byte |= (1u << j);
      const T d = b ? s : -s;
      err[i + j] = zi - d;
    }
    bits[i >> 3] = (uint8_t)byte;
  }
  *scale = s;
}

template <class T>
void decompress_chunk(const uint8_t* bits, T scale, int64_t n, T* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = get_bit(bits, i) ? scale : -scale;
}

// Algorithm 1 lines 6-7 (+ A.5.2 momentum scaling), chunk by chunk (A.7.1).
template <class T>
void compress_local(int64_t n_pad, int64_t L, const int64_t* off, int32_t W, const T* mom_scale,
                    T beta1, const T* g, const T* m, T* err, uint8_t* bits, T* scales) {
  const T omb1 = (T)1 - beta1;
  // z = k*(beta1*m + (1-beta1)*g) + err, written over err
  for (int64_t l = 0; l < L; ++l) {
    const T k = mom_scale ? mom_scale[l] : (T)1;
    for (int64_t i = off[l]; i < off[l + 1]; ++i) {
      const T mloc = beta1 * m[i] + omb1 * g[i];
      err[i] = k * mloc + err[i];
    }
  }
  for (int64_t i = off[L]; i < n_pad; ++i) {
    const T mloc = beta1 * m[i] + omb1 * g[i];
    err[i] = mloc + err[i];
  }
  const int64_t n_c = n_pad / W;
  for (int32_t c = 0; c < W; ++c)
    compress_chunk<T>(err + c * n_c, n_c, bits + c * (n_c / 8), scales + c, err + c * n_c);
}

// Algorithm 1 line 10 on one chunk, first half: the average of the W decompressed chunks plus the
// carried server error, for elements [j0, j1) (each element is independent of the others).
template <class T>
void server_average(int64_t n_c, int32_t W, const uint8_t* bits_in, const T* scales_in,
                    T* err_server, int64_t j0, int64_t j1) {
  const T invW = (T)1 / (T)W;
  for (int64_t j = j0; j < j1; ++j) {
    T acc = (T)0;
    for (int32_t w = 0; w < W; ++w) {
      const T s = scales_in[w];
      acc = acc + (get_bit(bits_in + (int64_t)w * (n_c / 8), j) ? s : -s);
    }
    err_server[j] = acc * invW + err_server[j];
  }
}

// Algorithm 1 line 10 on one chunk.
template <class T>
void server_reduce(int64_t n_c, int32_t W, const uint8_t* bits_in, const T* scales_in,
                   T* err_server, uint8_t* bits_out, T* scale_out) {
  server_average<T>(n_c, W, bits_in, scales_in, err_server, 0, n_c);
  compress_chunk<T>(err_server, n_c, bits_out, scale_out, err_server);
}

// Algorithm 1 line 13 (+ A.5.2: divide the global momentum by the layer's coefficient), layers
// [l0, l1) (each element is independent of the others).
template <class T>
void global_momentum_layers(int64_t n_c, const int64_t* off, int64_t l0, int64_t l1,
                            const T* mom_scale, const uint8_t* bits_all, const T* server_scales,
                            T* mt) {
  for (int64_t l = l0; l < l1; ++l) {
    for (int64_t i = off[l]; i < off[l + 1]; ++i) {
      const T s = server_scales[i / n_c];
      const T d = get_bit(bits_all, i) ? s : -s;
      mt[i] = mom_scale ? d / mom_scale[l] : d;
    }
  }
}

template <class T>
void global_momentum(int64_t n_pad, int64_t L, const int64_t* off, int32_t W, const T* mom_scale,
                     const uint8_t* bits_all, const T* server_scales, T* mt) {
  global_momentum_layers<T>(n_pad / W, off, 0, L, mom_scale, bits_all, server_scales, mt);
  for (int64_t i = off[L]; i < n_pad; ++i) mt[i] = (T)0;
}

// Algorithm 1 lines 15-20.
template <class T>
void ratios_dense(int64_t L, const int64_t* off, T beta1, T beta2, T r_min, T r_max, T r_thr,
                  const T* mt, const T* m, T* v_fresh, const T* v_frozen, const T* c_avg,
                  T* r_prev, T* coeff_c) {
  const T omb1 = (T)1 - beta1;
  const T omb2 = (T)1 - beta2;
  for (int64_t l = 0; l < L; ++l) {
    T r = (T)0;
    for (int64_t i = off[l]; i < off[l + 1]; ++i) {
      const T gr = (mt[i] - beta1 * m[i]) / omb1;         // line 15
      const T vf = beta2 * v_fresh[i] + omb2 * (gr * gr);  // line 16
      v_fresh[i] = vf;
      const T q = v_frozen[i] / vf;                        // line 17 (max element)
      if (q > r) r = q;
    }
    const T lo = ((T)1 - r_thr) * r_prev[l];
    const T hi = ((T)1 + r_thr) * r_prev[l];
    r = clip<T>(r, lo, hi);       // line 18
    r = clip<T>(r, r_min, r_max); // line 19
    r_prev[l] = r;
    coeff_c[l] = r * c_avg[l];    // line 20
  }
}

// Algorithm 1 line 21; commits the global momentum (line 13).
template <class T>
void apply_dense(int64_t L, const int64_t* off, T eta, T lr, const T* mt, const T* coeff_c,
                 const T* v_frozen, T* x, T* m) {
  for (int64_t l = 0; l < L; ++l) {
    const T a = lr * coeff_c[l];
    for (int64_t i = off[l]; i < off[l + 1]; ++i) {
      const T u = mt[i] / (std::sqrt(v_frozen[i]) + eta);
      x[i] = x[i] - a * u;
      m[i] = mt[i];
    }
  }
}

// eq. (1) per tensor, then line 2 of Algorithm 1.
template <class T>
void warmup_step(int64_t L, const int64_t* off, T beta1, T beta2, T beta3, T eta, T c_min, T c_max,
                 T wd, T lr, const T* g, T* m, T* v, T* x, T* c_out, T* c_avg) {
  const T omb1 = (T)1 - beta1, omb2 = (T)1 - beta2, omb3 = (T)1 - beta3;
  std::vector<T> u;
  for (int64_t l = 0; l < L; ++l) {
    const int64_t a = off[l], n = off[l + 1] - off[l];
    u.assign((size_t)n, (T)0);
    double Sx = 0.0, Su = 0.0;
    for (int64_t j = 0; j < n; ++j) {
      const int64_t i = a + j;
      m[i] = beta1 * m[i] + omb1 * g[i];
      v[i] = beta2 * v[i] + omb2 * (g[i] * g[i]);
      T ui = m[i] / (std::sqrt(v[i]) + eta);
      if (wd != (T)0) ui = ui + wd * x[i];
      u[(size_t)j] = ui;
      Sx += (double)x[i] * (double)x[i];
      Su += (double)ui * (double)ui;
    }
    const T nx = (T)std::sqrt(Sx), nu = (T)std::sqrt(Su);
    const T c = clip<T>(nx / nu, c_min, c_max);
    const T step = lr * c;
    for (int64_t j = 0; j < n; ++j) x[a + j] = x[a + j] - step * u[(size_t)j];
    c_out[l] = c;
    c_avg[l] = beta3 * c_avg[l] + omb3 * c;
  }
}

}  // namespace

extern "C" {

int64_t obref_padded_len(int64_t n, int32_t W) {
  const int64_t q = 256 * (int64_t)W;
  return ((n + q - 1) / q) * q;
}

void obref_compress_chunk(const float* z, int64_t n, uint8_t* bits, float* scale, float* err) {
  compress_chunk<float>(z, n, bits, scale, err);
}
void obref64_compress_chunk(const double* z, int64_t n, uint8_t* bits, double* scale, double* err) {
  compress_chunk<double>(z, n, bits, scale, err);
}
void obref_decompress_chunk(const uint8_t* bits, float scale, int64_t n, float* out) {
  decompress_chunk<float>(bits, scale, n, out);
}
void obref64_decompress_chunk(const uint8_t* bits, double scale, int64_t n, double* out) {
  decompress_chunk<double>(bits, scale, n, out);
}

void obref_compress_local(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                          const float* mom_scale, float beta1, const float* g, const float* m,
                          float* err, uint8_t* bits, float* scales) {
  compress_local<float>(n_pad, L, off, W, mom_scale, beta1, g, m, err, bits, scales);
}
void obref64_compress_local(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                            const double* mom_scale, double beta1, const double* g, const double* m,
                            double* err, uint8_t* bits, double* scales) {
  compress_local<double>(n_pad, L, off, W, mom_scale, beta1, g, m, err, bits, scales);
}

void obref_server_reduce(int64_t n_c, int32_t W, const uint8_t* bits_in, const float* scales_in,
                         float* err_server, uint8_t* bits_out, float* scale_out) {
  server_reduce<float>(n_c, W, bits_in, scales_in, err_server, bits_out, scale_out);
}
void obref64_server_reduce(int64_t n_c, int32_t W, const uint8_t* bits_in, const double* scales_in,
                           double* err_server, uint8_t* bits_out, double* scale_out) {
  server_reduce<double>(n_c, W, bits_in, scales_in, err_server, bits_out, scale_out);
}

void obref_global_momentum(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                           const float* mom_scale, const uint8_t* bits_all,
                           const float* server_scales, float* mt) {
  global_momentum<float>(n_pad, L, off, W, mom_scale, bits_all, server_scales, mt);
}
void obref64_global_momentum(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                             const double* mom_scale, const uint8_t* bits_all,
                             const double* server_scales, double* mt) {
  global_momentum<double>(n_pad, L, off, W, mom_scale, bits_all, server_scales, mt);
}

void obref_ratios_dense(int64_t L, const int64_t* off, float beta1, float beta2, float r_min,
                        float r_max, float r_thr, const float* mt, const float* m, float* v_fresh,
                        const float* v_frozen, const float* c_avg, float* r_prev, float* coeff_c) {
  ratios_dense<float>(L, off, beta1, beta2, r_min, r_max, r_thr, mt, m, v_fresh, v_frozen, c_avg,
                      r_prev, coeff_c);
}
void obref64_ratios_dense(int64_t L, const int64_t* off, double beta1, double beta2, double r_min,
                          double r_max, double r_thr, const double* mt, const double* m,
                          double* v_fresh, const double* v_frozen, const double* c_avg,
                          double* r_prev, double* coeff_c) {
  ratios_dense<double>(L, off, beta1, beta2, r_min, r_max, r_thr, mt, m, v_fresh, v_frozen, c_avg,
                       r_prev, coeff_c);
}

void obref_apply_dense(int64_t L, const int64_t* off, float eta, float lr, const float* mt,
                       const float* coeff_c, const float* v_frozen, float* x, float* m) {
  apply_dense<float>(L, off, eta, lr, mt, coeff_c, v_frozen, x, m);
}
void obref64_apply_dense(int64_t L, const int64_t* off, double eta, double lr, const double* mt,
                         const double* coeff_c, const double* v_frozen, double* x, double* m) {
  apply_dense<double>(L, off, eta, lr, mt, coeff_c, v_frozen, x, m);
}

void obref_layer_ratios(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                        const float* mom_scale, float beta1, float beta2, float r_min, float r_max,
                        float r_thr, const uint8_t* bits_all, const float* server_scales,
                        const float* m, float* v_fresh, const float* v_frozen, const float* c_avg,
                        float* r_prev, float* coeff_c) {
  std::vector<float> mt((size_t)n_pad);
  global_momentum<float>(n_pad, L, off, W, mom_scale, bits_all, server_scales, mt.data());
  ratios_dense<float>(L, off, beta1, beta2, r_min, r_max, r_thr, mt.data(), m, v_fresh, v_frozen,
                      c_avg, r_prev, coeff_c);
}

void obref_decompress_apply(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                            const float* mom_scale, float eta, float lr, const uint8_t* bits_all,
                            const float* server_scales, const float* coeff_c, const float* v_frozen,
                            float* x, float* m) {
  std::vector<float> mt((size_t)n_pad);
  global_momentum<float>(n_pad, L, off, W, mom_scale, bits_all, server_scales, mt.data());
  apply_dense<float>(L, off, eta, lr, mt.data(), coeff_c, v_frozen, x, m);
}

void obref_warmup_step(int64_t L, const int64_t* off, float beta1, float beta2, float beta3,
                       float eta, float c_min, float c_max, float weight_decay, float lr,
                       const float* g, float* m, float* v, float* x, float* c_out, float* c_avg) {
  warmup_step<float>(L, off, beta1, beta2, beta3, eta, c_min, c_max, weight_decay, lr, g, m, v, x,
                     c_out, c_avg);
}
void obref64_warmup_step(int64_t L, const int64_t* off, double beta1, double beta2, double beta3,
                         double eta, double c_min, double c_max, double weight_decay, double lr,
                         const double* g, double* m, double* v, double* x, double* c_out,
                         double* c_avg) {
  warmup_step<double>(L, off, beta1, beta2, beta3, eta, c_min, c_max, weight_decay, lr, g, m, v, x,
                      c_out, c_avg);
}

namespace {
// A.5.2 (reading): sigma_l = ||m_l||_2 / sqrt(n_l), 0 for an empty layer.
double layer_sigma(const int64_t* off, int64_t l, const float* m) {
  const int64_t n = off[l + 1] - off[l];
  if (n <= 0) return 0.0;
  double S = 0.0;
  for (int64_t i = off[l]; i < off[l + 1]; ++i) S += (double)m[i] * (double)m[i];
  return std::sqrt(S / (double)n);
}

// k_l = mean(sigma over the non-empty layers, in layer order) / sigma_l; 1 where sigma_l == 0.
void momentum_scale_from_sigma(int64_t L, const int64_t* off, const double* sigma, float* mom_scale) {
  double sum = 0.0;
  int64_t cnt = 0;
  for (int64_t l = 0; l < L; ++l) {
    if (off[l + 1] - off[l] <= 0) continue;
    sum += sigma[l];
    ++cnt;
  }
  const double mean = cnt ? sum / (double)cnt : 0.0;
  for (int64_t l = 0; l < L; ++l) {
    const double s = sigma[l];
    mom_scale[l] = (s > 0.0) ? (float)(mean / s) : 1.0f;
  }
}
}  // namespace

void obref_momentum_scale(int64_t L, const int64_t* off, const float* m, float* mom_scale) {
  std::vector<double> sigma((size_t)L, 0.0);
  for (int64_t l = 0; l < L; ++l) sigma[(size_t)l] = layer_sigma(off, l, m);
  momentum_scale_from_sigma(L, off, sigma.data(), mom_scale);
}

namespace {
struct LpFormat { int ebits, fbits; };
inline LpFormat lp_format(int fmt) { return fmt == 1 ? LpFormat{5, 10} : LpFormat{8, 7}; }

// value of a 16-bit pattern: (-1)^s * 2^(e-bias) * (1 + f/2^fbits), subnormals 2^(1-bias) * f/2^fbits
double lp_value(int fmt, uint16_t b) {
  const LpFormat F = lp_format(fmt);
  const int bias = (1 << (F.ebits - 1)) - 1;
  const int s = b >> 15;
  const int e = (b >> F.fbits) & ((1 << F.ebits) - 1);
  const int f = b & ((1 << F.fbits) - 1);
  double v;
  if (e == (1 << F.ebits) - 1) v = f ? std::nan("") : INFINITY;
  else if (e == 0) v = std::ldexp((double)f, 1 - bias - F.fbits);
  else v = std::ldexp((double)((1 << F.fbits) + f), e - bias - F.fbits);
  return s ? -v : v;
}

uint16_t lp_nearest(int fmt, float x) {
  const LpFormat F = lp_format(fmt);
  const int bias = (1 << (F.ebits - 1)) - 1;
  const int emax = bias, emin = 1 - bias;
  const uint16_t exp_all = (uint16_t)(((1 << F.ebits) - 1) << F.fbits);
  if (std::isnan(x)) return (uint16_t)(exp_all | (1 << (F.fbits - 1)));
  const uint16_t sign = std::signbit(x) ? 0x8000 : 0;
  const double a = std::fabs((double)x);
  if (std::isinf(x)) return sign | exp_all;
  if (a == 0.0) return sign;
  int e;
  (void)std::frexp(a, &e);   // a = m * 2^e, m in [0.5, 1)  ->  a in [2^(e-1), 2^e)
  int ex = e - 1;
  if (ex < emin) ex = emin;  // subnormal range shares the spacing of the smallest normal binade
  // units of the last place at this exponent; nearbyint rounds ties to even (default mode)
  double q = std::nearbyint(std::ldexp(a, F.fbits - ex));
  if (q >= std::ldexp(1.0, F.fbits + 1)) { q /= 2.0; ex += 1; }   // rounded up into the next binade
  if (ex > emax) return sign | exp_all;                              // overflow -> infinity
  uint16_t bits;
  if (q < std::ldexp(1.0, F.fbits)) bits = (uint16_t)q;            // subnormal (ex == emin) or zero
  else bits = (uint16_t)(((ex + bias) << F.fbits) | ((int)q - (1 << F.fbits)));
  return sign | bits;
}
}  // namespace

void obref_lp_decode(int32_t fmt, int64_t n, const uint16_t* bits, float scale, float* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = (float)lp_value(fmt, bits[i]) * scale;
}

void obref_lp_round(int32_t fmt, int64_t n, const float* x, uint16_t* bits) {
  for (int64_t i = 0; i < n; ++i) bits[i] = lp_nearest(fmt, x[i]);
}
}  // extern "C"

// ---------------------------------------------------------------------------------------------
// Multi-threaded drivers.  They hold no arithmetic: each cuts the problem into independent pieces
// (chunks, layers, element ranges of an elementwise loop), runs the scalar routines above on the
// pieces from a pool of std::threads and leaves every output element to exactly one piece, so the
// results equal the serial entry points' bit for bit (tests pin that).  The pieces:
//   compress_local   one call of compress_local<float> per chunk, on the sub-problem "this chunk
//                    alone" (offsets clipped to the chunk; A.7.1: chunks are independent)
//   server_reduce    server_average<float> on element ranges, then compress_chunk<float> once
//   layer_ratios, decompress_apply, warmup_step   one layer at a time (lines 15-21 and eq. (1)
//                    are per layer), largest layers first
// ---------------------------------------------------------------------------------------------
namespace {

template <class F>
void run_pieces(int64_t n, int threads, F f) {
  if (threads > n) threads = (int)n;
  if (threads <= 1) {
    for (int64_t i = 0; i < n; ++i) f(i);
    return;
  }
  std::atomic<int64_t> next{0};
  auto work = [&] {
    for (;;) {
      const int64_t i = next.fetch_add(1);
      if (i >= n) break;
      f(i);
    }
  };
  std::vector<std::thread> pool;
  for (int t = 1; t < threads; ++t) pool.emplace_back(work);
  work();
  for (auto& th : pool) th.join();
}

// layer indices, largest layer first (ties: lower index first)
std::vector<int64_t> layers_by_size(int64_t L, const int64_t* off) {
  std::vector<int64_t> idx((size_t)L);
  for (int64_t l = 0; l < L; ++l) idx[(size_t)l] = l;
  std::stable_sort(idx.begin(), idx.end(), [&](int64_t a, int64_t b) {
    return off[a + 1] - off[a] > off[b + 1] - off[b];
  });
  return idx;
}

}  // namespace

extern "C" {

void obref_compress_local_mt(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                             const float* mom_scale, float beta1, const float* g, const float* m,
                             float* err, uint8_t* bits, float* scales, int32_t threads) {
  const int64_t n_c = n_pad / W;
  run_pieces(W, threads, [&](int64_t c) {
    const int64_t a = c * n_c, b = a + n_c;
    std::vector<int64_t> oc((size_t)L + 1);   // the layers as seen from inside chunk c
    for (int64_t l = 0; l <= L; ++l) oc[(size_t)l] = std::min(std::max(off[l], a), b) - a;
    compress_local<float>(n_c, L, oc.data(), 1, mom_scale, beta1, g + a, m + a, err + a,
                          bits + a / 8, scales + c);
  });
}

void obref_server_reduce_mt(int64_t n_c, int32_t W, const uint8_t* bits_in, const float* scales_in,
                            float* err_server, uint8_t* bits_out, float* scale_out, int32_t threads) {
  const int64_t piece = 1 << 16;
  const int64_t n = (n_c + piece - 1) / piece;
  run_pieces(n, threads, [&](int64_t p) {
    server_average<float>(n_c, W, bits_in, scales_in, err_server, p * piece,
                          std::min((p + 1) * piece, n_c));
  });
  compress_chunk<float>(err_server, n_c, bits_out, scale_out, err_server);
}

void obref_layer_ratios_mt(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                           const float* mom_scale, float beta1, float beta2, float r_min, float r_max,
                           float r_thr, const uint8_t* bits_all, const float* server_scales,
                           const float* m, float* v_fresh, const float* v_frozen, const float* c_avg,
                           float* r_prev, float* coeff_c, int32_t threads) {
  std::vector<float> mt((size_t)n_pad);
  const std::vector<int64_t> order = layers_by_size(L, off);
  run_pieces(L, threads, [&](int64_t k) {
    const int64_t l = order[(size_t)k];
    global_momentum_layers<float>(n_pad / W, off, l, l + 1, mom_scale, bits_all, server_scales, mt.data());
    ratios_dense<float>(1, off + l, beta1, beta2, r_min, r_max, r_thr, mt.data(), m, v_fresh, v_frozen,
                        c_avg + l, r_prev + l, coeff_c + l);
  });
}

void obref_decompress_apply_mt(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                               const float* mom_scale, float eta, float lr, const uint8_t* bits_all,
                               const float* server_scales, const float* coeff_c, const float* v_frozen,
                               float* x, float* m, int32_t threads) {
  std::vector<float> mt((size_t)n_pad);
  const std::vector<int64_t> order = layers_by_size(L, off);
  run_pieces(L, threads, [&](int64_t k) {
    const int64_t l = order[(size_t)k];
    global_momentum_layers<float>(n_pad / W, off, l, l + 1, mom_scale, bits_all, server_scales, mt.data());
    apply_dense<float>(1, off + l, eta, lr, mt.data(), coeff_c + l, v_frozen, x, m);
  });
}

void obref_warmup_step_mt(int64_t L, const int64_t* off, float beta1, float beta2, float beta3,
                          float eta, float c_min, float c_max, float weight_decay, float lr,
                          const float* g, float* m, float* v, float* x, float* c_out, float* c_avg,
                          int32_t threads) {
  const std::vector<int64_t> order = layers_by_size(L, off);
  run_pieces(L, threads, [&](int64_t k) {
    const int64_t l = order[(size_t)k];
    warmup_step<float>(1, off + l, beta1, beta2, beta3, eta, c_min, c_max, weight_decay, lr, g, m, v,
                       x, c_out + l, c_avg + l);
  });
}

void obref_momentum_scale_mt(int64_t L, const int64_t* off, const float* m, float* mom_scale,
                             int32_t threads) {
  std::vector<double> sigma((size_t)L, 0.0);
  const std::vector<int64_t> order = layers_by_size(L, off);
  run_pieces(L, threads, [&](int64_t k) {
    const int64_t l = order[(size_t)k];
    sigma[(size_t)l] = layer_sigma(off, l, m);
  });
  momentum_scale_from_sigma(L, off, sigma.data(), mom_scale);
}

}  // extern "C"
