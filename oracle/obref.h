/*
 * obref -- CPU oracle for the compression-stage step of 1-bit LAMB (arXiv 2104.06069).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  Only the tests, the smoke
 * check and the CPU-baseline leg of the benchmark may load it.  It shares no
 * code with the HIP library and includes none of its headers.
 *
 * Everything here is a plain scalar loop that takes the steps of Algorithm 1
 * (compression stage) and of eq. (1) (LAMB, warmup stage) in the paper's order.
 * Each entry point exists twice: `obref_*` computes in IEEE binary32 (one
 * rounding per operation, no fused multiply-add; the build passes
 * -ffp-contract=off), `obref64_*` is the same code instantiated in binary64
 * (the "shadow" used by the algebraic pins).  The only places where the
 * precision differs from the element type are the two sum-of-squares
 * reductions (chunk scale, LAMB norms), which accumulate in binary64.
 *
 * Readings of the paper that this file fixes (the paper is silent or
 * inconsistent on each; see the function comments):
 *   - C[z] = (sign bits, one scale), scale = ||z||_2 / sqrt(n)  (Section 2: "+-1 signs and a scale").
 *   - one scale per chunk (Appendix A.7.1: chunk-wise parameter-server equivalence).
 *   - bit i of the packed stream lives in byte i/8, bit i%8 (LSB first); 1 means +scale.
 *   - sign test is the IEEE compare z >= 0 (so +0, -0 -> 1; NaN -> 0).
 *   - server average: sequential binary32 sum over workers 0..W-1, one multiply by 1/W.
 *   - Algorithm 1 is followed literally where the proof in A.7.1 differs
 *     (no c_{t-2}/c_{t-1} factor on the carried error).
 *   - the update divides by sqrt(v_frozen) + eta; eta = 0 is Algorithm 1 line 21 as printed.
 *   - r_t^(l) = max over the layer of v_frozen/v_fresh taken with `if (q > r) r = q`
 *     starting from 0 (NaN quotients are skipped, +Inf survives and is clipped).
 *   - clip(x,a,b) = min(max(x,a),b) with max(x,a) = x > a ? x : a and
 *     min(y,b) = y < b ? y : b  (so NaN -> a).
 *
 * Parity pins (tests/test_oracle_*.py) cover every function below; none is
 * "parity unpinned".
 */
#ifndef OBREF_H
#define OBREF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Padded flat length: smallest multiple of 256*W that is >= n. */
int64_t obref_padded_len(int64_t n, int32_t num_workers);

/* ---- the compression operator C[.] on one chunk (Section 2; Algorithm 1 lines 7, 10) ----
 * z[n] -> bits[n/8] (n % 8 == 0), *scale, err[n] = z - decompress(bits, scale).
 * err may alias z. */
void obref_compress_chunk(const float* z, int64_t n, uint8_t* bits, float* scale, float* err);
void obref64_compress_chunk(const double* z, int64_t n, uint8_t* bits, double* scale, double* err);

/* out[i] = bit i ? +scale : -scale */
void obref_decompress_chunk(const uint8_t* bits, float scale, int64_t n, float* out);
void obref64_decompress_chunk(const uint8_t* bits, double scale, int64_t n, double* out);

/* ---- Algorithm 1 lines 6-7 over the whole flat buffer (all W chunks of this worker) ----
 * z = k_l * (beta1*m + (1-beta1)*g) + err ; per chunk: bits, scale, err <- z - C[z].
 * mom_scale (k_l, Appendix A.5.2) may be NULL (= 1).  Elements >= off[L] are padding: k = 1.
 * g, m, err have n_pad elements; bits n_pad/8 bytes; scales W. */
void obref_compress_local(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                          const float* mom_scale, float beta1,
                          const float* g, const float* m, float* err,
                          uint8_t* bits, float* scales);
void obref64_compress_local(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                            const double* mom_scale, double beta1,
                            const double* g, const double* m, double* err,
                            uint8_t* bits, double* scales);

/* ---- Algorithm 1 line 10 on one chunk of n_c elements ----
 * bits_in: W consecutive blocks of n_c/8 bytes (worker-major); scales_in[W].
 * zb = (sum_w +-scales_in[w]) * (1/W) + err_server ; bits_out, *scale_out, err_server <- zb - C[zb]. */
void obref_server_reduce(int64_t n_c, int32_t W, const uint8_t* bits_in, const float* scales_in,
                         float* err_server, uint8_t* bits_out, float* scale_out);
void obref64_server_reduce(int64_t n_c, int32_t W, const uint8_t* bits_in, const double* scales_in,
                           double* err_server, uint8_t* bits_out, double* scale_out);

/* ---- Algorithm 1 line 13 with A.5.2: m_t = decompress(all W server chunks) / k_l ----
 * mt[i] for i < off[L]; elements >= off[L] (padding) are set to 0. */
void obref_global_momentum(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                           const float* mom_scale, const uint8_t* bits_all,
                           const float* server_scales, float* mt);
void obref64_global_momentum(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                             const double* mom_scale, const uint8_t* bits_all,
                             const double* server_scales, double* mt);

/* ---- Algorithm 1 lines 15-20 given the global momentum mt (dense) ----
 * g = (mt - beta1*m)/(1-beta1); v_fresh = beta2*v_fresh + (1-beta2)*g*g;
 * r = max(v_frozen/v_fresh) per layer; two clips; r_prev <- r; coeff_c = r*c_avg. */
void obref_ratios_dense(int64_t L, const int64_t* off, float beta1, float beta2,
                        float r_min, float r_max, float r_thr,
                        const float* mt, const float* m, float* v_fresh, const float* v_frozen,
                        const float* c_avg, float* r_prev, float* coeff_c);
void obref64_ratios_dense(int64_t L, const int64_t* off, double beta1, double beta2,
                          double r_min, double r_max, double r_thr,
                          const double* mt, const double* m, double* v_fresh, const double* v_frozen,
                          const double* c_avg, double* r_prev, double* coeff_c);

/* ---- Algorithm 1 line 21 given mt (dense); also commits m <- mt (line 13) ----
 * x -= (lr*coeff_c[l]) * (mt / (sqrt(v_frozen) + eta)). */
void obref_apply_dense(int64_t L, const int64_t* off, float eta, float lr,
                       const float* mt, const float* coeff_c, const float* v_frozen,
                       float* x, float* m);
void obref64_apply_dense(int64_t L, const int64_t* off, double eta, double lr,
                         const double* mt, const double* coeff_c, const double* v_frozen,
                         double* x, double* m);

/* ---- the two packed-input calls: decompress, then the dense routine above ---- */
void obref_layer_ratios(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                        const float* mom_scale, float beta1, float beta2,
                        float r_min, float r_max, float r_thr,
                        const uint8_t* bits_all, const float* server_scales,
                        const float* m, float* v_fresh, const float* v_frozen,
                        const float* c_avg, float* r_prev, float* coeff_c);
void obref_decompress_apply(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                            const float* mom_scale, float eta, float lr,
                            const uint8_t* bits_all, const float* server_scales,
                            const float* coeff_c, const float* v_frozen, float* x, float* m);

/* ---- eq. (1) + Algorithm 1 line 2: one LAMB step and the moving average of c ----
 * m = b1 m + (1-b1) g; v = b2 v + (1-b2) g*g; u = m/(sqrt(v)+eta) [+ wd*x];
 * c = clip(||x||_2/||u||_2, c_min, c_max); x -= (lr*c) u; c_avg = b3 c_avg + (1-b3) c.
 * c_out[L] receives c. */
void obref_warmup_step(int64_t L, const int64_t* off, float beta1, float beta2, float beta3,
                       float eta, float c_min, float c_max, float weight_decay, float lr,
                       const float* g, float* m, float* v, float* x, float* c_out, float* c_avg);
void obref64_warmup_step(int64_t L, const int64_t* off, double beta1, double beta2, double beta3,
                         double eta, double c_min, double c_max, double weight_decay, double lr,
                         const double* g, double* m, double* v, double* x, double* c_out, double* c_avg);

/* ---- A.5.2 momentum-scale coefficients at the end of warmup (reading: the paper gives no
 * formula): sigma_l = ||m_l||_2/sqrt(n_l); k_l = mean_l(sigma_l)/sigma_l, 1 if sigma_l == 0
 * or the layer is empty; the mean runs over non-empty layers. */
void obref_momentum_scale(int64_t L, const int64_t* off, const float* m, float* mom_scale);

/* 16-bit storage formats of the mixed-precision variant (the paper trains in FP16, Section 6;
 * its volume figures are against FP16 communication).  The arithmetic stays binary32: a 16-bit
 * gradient is decoded exactly and multiplied once by grad_scale (the inverse loss scale), a
 * 16-bit copy of the parameters is the binary32 value rounded to nearest, ties to even.
 * fmt: 1 = IEEE binary16 (5 exponent bits, 10 fraction bits), 2 = bfloat16 (8, 7).
 *   obref_lp_decode: out[i] = value(bits[i]) * scale       (binary32 multiply)
 *   obref_lp_round:  bits[i] = nearest representable value of x[i] in the format; beyond the
 *                    largest finite value by half a unit or more -> infinity; every NaN ->
 *                    sign 0, all exponent bits, top fraction bit (0x7e00 / 0x7fc0).
 * Both are written from the definition of the formats (fields decoded with ldexp; rounding by
 * nearbyint on the value scaled to units of the last place), not from bit tricks. */
void obref_lp_decode(int32_t fmt, int64_t n, const uint16_t* bits, float scale, float* out);
void obref_lp_round(int32_t fmt, int64_t n, const float* x, uint16_t* bits);

/* ---- multi-threaded drivers of the float routines above (`threads` >= 1 worker threads) ----
 * No arithmetic of their own: the problem is cut into independent pieces -- chunks for
 * obref_compress_local (A.7.1: each chunk is its own parameter-server instance), element ranges of
 * the averaging loop for obref_server_reduce, layers for the per-layer routines -- and the scalar
 * routines run on the pieces in parallel.  Every output element is produced by the same operations
 * in the same order as in the serial entry point: results are bit-identical (pinned by a test).
 * They exist so that whole trajectories at the benchmark sizes finish in seconds; the serial
 * entry points remain the definition. */
void obref_compress_local_mt(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                             const float* mom_scale, float beta1, const float* g, const float* m,
                             float* err, uint8_t* bits, float* scales, int32_t threads);
void obref_server_reduce_mt(int64_t n_c, int32_t W, const uint8_t* bits_in, const float* scales_in,
                            float* err_server, uint8_t* bits_out, float* scale_out, int32_t threads);
void obref_layer_ratios_mt(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                           const float* mom_scale, float beta1, float beta2,
                           float r_min, float r_max, float r_thr,
                           const uint8_t* bits_all, const float* server_scales,
                           const float* m, float* v_fresh, const float* v_frozen,
                           const float* c_avg, float* r_prev, float* coeff_c, int32_t threads);
void obref_decompress_apply_mt(int64_t n_pad, int64_t L, const int64_t* off, int32_t W,
                               const float* mom_scale, float eta, float lr,
                               const uint8_t* bits_all, const float* server_scales,
                               const float* coeff_c, const float* v_frozen, float* x, float* m,
                               int32_t threads);
void obref_warmup_step_mt(int64_t L, const int64_t* off, float beta1, float beta2, float beta3,
                          float eta, float c_min, float c_max, float weight_decay, float lr,
                          const float* g, float* m, float* v, float* x, float* c_out, float* c_avg,
                          int32_t threads);
void obref_momentum_scale_mt(int64_t L, const int64_t* off, const float* m, float* mom_scale,
                             int32_t threads);

#ifdef __cplusplus
}
#endif
#endif
