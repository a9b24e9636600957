/*
 * libonebitlamb -- the compression-stage optimizer step of 1-bit LAMB (arXiv 2104.06069,
 * Algorithm 1) and the LAMB warmup step (eq. (1)) over one GPU's flat fp32 parameter buffer,
 * as hand-written HIP kernels for gfx950 (MI355X).
 *
 * Model of the data
 * -----------------
 * All tensors of the model are viewed as one contiguous 1-D fp32 buffer ("momentum fusion",
 * Appendix A.5.1) described by `layer_offsets` (L+1 entries, tightly packed, no alignment
 * between tensors).  "Layer" means tensor: each has its own coefficients (Section 2).
 *   N      = layer_offsets[L]            real parameters
 *   W      = num_workers                 = number of chunks of the compressed allreduce (Section 5)
 *   N_pad  = N rounded up to 256*W       length of every N-sized buffer
 *   n_c    = N_pad / W                   chunk length (a multiple of 256)
 * Elements [N, N_pad) are padding: they take part in chunk scales and error feedback like any
 * other element (with momentum-scale coefficient 1) but belong to no layer, so the ratio, the
 * parameter update and the momentum commit never touch them.  The caller zero-fills the
 * padding of every buffer once (and of each gradient).
 *
 * Compression operator C[.] (Section 2: "+-1 signs and a scale"; the paper gives no formula or
 * wire format, this library fixes them):
 *   scale = ||z||_2 / sqrt(n) per chunk (keeps the L2 norm of the chunk), accumulated in fp64;
 *   bit   = (z >= 0) as an IEEE compare (+0, -0 -> 1; NaN -> 0); 1 decodes to +scale, 0 to -scale;
 *   packed stream: element i is bit (i % 32) of the little-endian uint32 word i / 32.
 *
 * Conventions
 * -----------
 * - Pointers named in ob_lamb_state and the packed/scales/grad arguments are DEVICE pointers,
 *   owned by the caller, 16-byte aligned.  ob_lamb_config and its layer_offsets are HOST memory,
 *   copied by ob_lamb_create.
 * - Every step call validates its arguments on the host, enqueues kernels on `hip_stream`
 *   (a hipStream_t passed as void*; NULL = the default stream) and returns without
 *   synchronising.  On error nothing is enqueued and a negative ob_status is returned.
 * - All arithmetic is IEEE binary32 with one rounding per operation (no fused multiply-add),
 *   except the two sum-of-squares reductions (chunk scales, LAMB norms), which accumulate in
 *   binary64 in a fixed order: results are bit-reproducible from run to run.
 * - A context owns a small device workspace (partial sums, per-layer maxima, tile tables) on the
 *   device that was current at ob_lamb_create; step calls made with another device current return
 *   OB_ERR_ARG.  Calls on one context must not overlap in time (use one stream, or order them
 *   yourself).
 * - Call order of one compression step:
 *     ob_lamb_compress_local -> [exchange] -> ob_lamb_server_reduce -> [exchange]
 *     -> ob_lamb_layer_ratios -> ob_lamb_decompress_apply.
 *   ob_lamb_layer_ratios must precede ob_lamb_decompress_apply in the same step (the former
 *   needs the previous momentum that the latter overwrites).
 */
#ifndef ONEBITLAMB_H
#define ONEBITLAMB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ob_lamb_ctx ob_lamb_ctx; /* opaque */

typedef enum ob_status {
  OB_OK = 0,
  OB_ERR_NULL = -1,  /* a required pointer is NULL */
  OB_ERR_ARG = -2,   /* a size, offset table or hyper-parameter is invalid */
  OB_ERR_ALIGN = -3, /* a device pointer is not 16-byte aligned */
  OB_ERR_STATE = -4, /* a bounded device-side wait expired (see ob_lamb_check_device_status) */
  OB_ERR_HIP = -5,   /* a HIP runtime call failed (see ob_lamb_last_hip_error) */
  OB_ERR_SIZE = -6   /* a size exceeds a fixed capacity (ob_lamb_server_reduce, ob_lamb_server_reduce_static) */
} ob_status;

typedef struct ob_lamb_config {
  int64_t num_layers;           /* L >= 1 */
  const int64_t* layer_offsets; /* host, L+1 entries, [0] = 0, non-decreasing (empty layers allowed) */
  int32_t num_workers;          /* W >= 1 */
  int32_t server_chunk;         /* chunk this rank serves, 0..W-1 (which chunk ob_lamb_state.own_packed_in receives) */
  float beta1, beta2, beta3;    /* momentum, variance, coefficient moving average (Algorithm 1 line 1) */
  float eta;                    /* added to sqrt(v) in eq. (1) and in line 21; 0 = line 21 as printed */
  float c_min, c_max;           /* clip of LAMB's coefficient in eq. (1) (warmup only) */
  float r_min, r_max;           /* Algorithm 1 line 19 */
  float r_threshold;            /* Algorithm 1 line 18 */
  float weight_decay;           /* warmup only: u += wd * x; 0 = eq. (1) as printed */
  /* Kernel selection (all results are the same whatever is selected; 0 everywhere = the library's
   * own choice for the device).  Per context: two contexts in one process may differ. */
  uint32_t flags;               /* OB_CFG_* bits */
  int32_t fused_max_tiles;      /* > 0: the kernels with a per-layer barrier leave every layer with more
                                   than this many 8192-element tiles to the plain kernels, even if
                                   the device could hold more; 0 = the device's limit */
  int32_t spin_limit;           /* bound, in polls, of every device-side wait: 0 = the default
                                   (OB_SPIN_LIMIT_DEFAULT); > 0 = that many, at most the default;
                                   OB_SPIN_NONE = give up without polling (exists so that the expiry
                                   path can be tested without ever hanging a kernel) */
} ob_lamb_config;

/* ob_lamb_config.flags */
#define OB_CFG_TWO_PASS_COMPRESS 1u   /* ob_lamb_compress_local as two passes through memory and
                                         ob_lamb_server_reduce as three kernels: no chunk barrier */
#define OB_CFG_NO_FUSED_APPLY 2u      /* ob_lamb_ratios_apply runs the two plain kernels for every layer */
#define OB_CFG_TWO_PASS_WARMUP 4u     /* ob_lamb_warmup_step takes two passes for every layer */
#define OB_CFG_NO_BARRIERS (OB_CFG_TWO_PASS_COMPRESS | OB_CFG_NO_FUSED_APPLY | OB_CFG_TWO_PASS_WARMUP)
#define OB_SPIN_NONE (-1)
/* A poll is one 8-byte load plus a sleep of 1024 clocks; at the 2.4 GHz the device runs at, the
 * default bounds a wait at 2^20 polls = about 0.5 s (about 1 s at the lowest power state's clock). */
#define OB_SPIN_LIMIT_DEFAULT (1 << 20)

/* Device pointers, caller-owned, fp32.  N-sized arrays have N_pad elements. */
typedef struct ob_lamb_state {
  float* x;          /* [N_pad] parameters */
  float* m;          /* [N_pad] momentum: the global m_{t-1} of Algorithm 1 line 13 */
  float* v_fresh;    /* [N_pad] variance, kept up to date (eq. (1) in warmup; line 16 afterwards) */
  float* v_frozen;   /* [N_pad] v_{T_w}: variance stored at the end of warmup (line 3) */
  float* err_worker; /* [N_pad] delta^(i): this worker's compression error (line 7) */
  float* err_server; /* [n_c]   delta-bar: server error of the chunk this rank serves (line 10) */
  float* c_avg;      /* [L] moving average of LAMB's coefficient (line 2), frozen after warmup */
  float* r_prev;     /* [L] r_{t-1}^(l), starts at 1 (line 1) */
  float* coeff_c;    /* [L] out: c_t^(l); warmup: eq. (1)'s c; compression stage: line 20 */
  float* mom_scale;  /* [L] momentum-scale coefficients of Appendix A.5.2, or NULL (= all ones) */
  /* The momentum in the 1-bit form it has after Algorithm 1 line 13 (optional, see below). */
  uint32_t* m_packed; /* [N_pad/32] sign words, or NULL */
  float* m_scales;    /* [W] server scales they decode with, or NULL */
  /* Optional second destination of ob_lamb_compress_local for chunk `server_chunk` of its output:
   * the slot of this rank's own server input (block server_chunk of packed_in, entry server_chunk
   * of scales_in) that the exchange would otherwise fill with a device-to-device copy of the rank's
   * own data.  Both or neither; NULL = not written. */
  uint32_t* own_packed_in; /* [n_c/32] or NULL */
  float* own_scale_in;     /* [1] or NULL */
  /* The worker error in deferred form (optional, see below): this worker's own previous packed
   * output and its scales.  Both or neither. */
  const uint32_t* err_packed; /* [N_pad/32] or NULL */
  const float* err_scales;    /* [W] or NULL */
  /* ... and the server error in the same deferred form: the server's own previous output for the
   * chunk it serves, kept by the library's kernels in these two buffers (read AND rewritten by
   * ob_lamb_server_reduce; not the packed_out of that call).  Both or neither. */
  uint32_t* srv_err_packed;   /* [n_c/32] or NULL */
  float* srv_err_scale;       /* [1] or NULL */
} ob_lamb_state;

/* Worker error representation.  Algorithm 1 line 7 leaves delta = z - C[z] in the error buffer, and
 * C[z] needs the chunk's scale, i.e. a reduction over the whole chunk, before any delta can be
 * written: that is what forces ob_lamb_compress_local into two passes or an in-kernel barrier.  The
 * subtraction can wait until the next step instead.  With err_packed / err_scales non-NULL,
 *   - err_worker holds z of the previous call, and ob_lamb_compress_local reads the carried error as
 *     err_worker[i] - (bit_i ? +s_c : -s_c) with the bits and scales of err_packed / err_scales --
 *     the same binary32 subtraction, on the same operands, as line 7's;
 *   - it writes the new z to err_worker, its sign words to packed_out and the scales to scales_out,
 *     which are the err_packed / err_scales of the next call.  They may be the very same buffers
 *     (err_packed == packed_out, err_scales == scales_out): pass the worker's output buffers and
 *     leave them untouched between the steps.
 * The call is then ONE streaming kernel plus a W-workgroup kernel for the scales: no in-kernel
 * barrier, nothing read twice.  Results are bit-identical to the other forms.  An err_scales of all
 * zeros makes err_worker an ordinary error buffer (x - (+-0) = x): that is how a run starts, or
 * resumes from a dense error.  ob_lamb_error_dense writes the error itself, delta, to err_out
 * [N_pad] (err_out may be st->err_worker if the caller then zeroes err_scales). */
ob_status ob_lamb_error_dense(ob_lamb_ctx* ctx, const ob_lamb_state* st, float* err_out, void* hip_stream);
/* The same for Algorithm 1 line 10's server error: with srv_err_packed / srv_err_scale non-NULL,
 * err_server holds zb of the previous ob_lamb_server_reduce, the carried error is err_server -
 * C[zb] decoded from those two buffers, and the call writes the new zb to err_server and its sign
 * words to packed_out and to srv_err_packed (the new scale to scale_out and srv_err_scale): one pass
 * over the chunk plus one workgroup for the scale, no barrier.  A zero srv_err_scale makes err_server
 * an ordinary error.  ob_lamb_server_error_dense writes the error itself to err_out [n_c]. */
ob_status ob_lamb_server_error_dense(ob_lamb_ctx* ctx, const ob_lamb_state* st, float* err_out,
                                     void* hip_stream);

/* Momentum representation.  After line 13 of any compression step the global momentum is exactly
 * m[i] = (bit_i ? +s_c : -s_c) / k_l (0 in the padding), i.e. the step's packed_all/server_scales.
 * The library therefore accepts it in either form:
 *   - reads (ob_lamb_compress_local, ob_lamb_layer_ratios) use the dense array st->m if it is
 *     non-NULL, else decode (st->m_packed, st->m_scales) on the fly -- 12 bytes per parameter
 *     less HBM traffic per step, bit-identical results;
 *   - ob_lamb_decompress_apply commits the new momentum to st->m if non-NULL, and to
 *     (st->m_packed, st->m_scales) if non-NULL (a device copy of packed_all/server_scales, skipped
 *     when st->m_packed == packed_all, e.g. when the caller alternates two packed_all buffers).
 * The warmup step needs the dense array; the first compression step after warmup reads it, and a
 * caller that wants the 1-bit form passes m = NULL from that step's ob_lamb_decompress_apply on.
 * ob_lamb_momentum_dense writes the dense view of (m_packed, m_scales) into m_out [N_pad]
 * (padding left untouched) for checkpoints or inspection. */
ob_status ob_lamb_momentum_dense(ob_lamb_ctx* ctx, const ob_lamb_state* st, float* m_out,
                                 void* hip_stream);

/* Creates a context on the current HIP device: copies the configuration, builds the tile tables
 * and allocates the workspace (blocking; uses hipMalloc/hipMemcpy).  *out is NULL on error
 * (OB_ERR_ARG also when the host tables cannot be allocated). */
ob_status ob_lamb_create(const ob_lamb_config* cfg, ob_lamb_ctx** out);
/* Frees the context and its device memory (blocking).  NULL is ignored. */
void ob_lamb_destroy(ob_lamb_ctx* ctx);

int64_t ob_lamb_num_params(const ob_lamb_ctx* ctx); /* N     */
int64_t ob_lamb_padded_len(const ob_lamb_ctx* ctx); /* N_pad */
int64_t ob_lamb_chunk_len(const ob_lamb_ctx* ctx);  /* n_c   */
/* Device memory the context itself holds (tile tables, partial sums, barrier words), in bytes: a few
 * bytes per 1024 parameters.  The library allocates it in ob_lamb_create and frees it in
 * ob_lamb_destroy; it is tied to the tables built from this configuration on this device, which is
 * why it is not a caller-supplied buffer (a caller that must not allocate after start-up creates
 * its contexts at start-up; ob_lamb_server_reduce_static needs none). */
size_t ob_lamb_workspace_bytes(const ob_lamb_ctx* ctx);
/* Static helper: N_pad for given N and W without a context (0 if an argument is invalid). */
int64_t ob_lamb_padded_len_for(int64_t n, int32_t num_workers);
const char* ob_lamb_status_string(ob_status s);
/* Text of the last HIP error seen by this context ("" if none). */
const char* ob_lamb_last_hip_error(const ob_lamb_ctx* ctx);

/* eq. (1) on every layer with the already averaged gradient `grad` [N_pad], then Algorithm 1
 * line 2: m, v_fresh, x updated; coeff_c <- c_t; c_avg <- beta3*c_avg + (1-beta3)*c_t.
 * No bias correction; ||.|| is the L2 norm of the layer, x taken before the update. */
ob_status ob_lamb_warmup_step(ob_lamb_ctx* ctx, const ob_lamb_state* st, const float* grad,
                              float lr, void* hip_stream);

/* Algorithm 1 line 3, end of warmup: v_frozen <- v_fresh (over N_pad), r_prev <- 1. */
ob_status ob_lamb_freeze(ob_lamb_ctx* ctx, const ob_lamb_state* st, void* hip_stream);

/* Algorithm 1 lines 6-7 over the whole flat buffer, with Appendix A.5.2's momentum scaling:
 *   z = k_l * (beta1*m + (1-beta1)*grad) + err_worker;   per chunk c: scales_out[c], bits;
 *   err_worker <- z - C[z]   (or, in the deferred form described at ob_lamb_state, err_worker <- z).
 * grad: [N_pad] this worker's local gradient.  packed_out: [N_pad/32] words.  scales_out: [W].
 * Reads the momentum (dense or 1-bit form), does not modify it.  In the 1-bit form m_packed must
 * not be the buffer packed_out (OB_ERR_ARG). */
ob_status ob_lamb_compress_local(ob_lamb_ctx* ctx, const ob_lamb_state* st, const float* grad,
                                 uint32_t* packed_out, float* scales_out, void* hip_stream);

/* Algorithm 1 line 10 on the one chunk this rank serves:
 *   zb = (sum_{w=0..W-1, in this order} +-scales_in[w]) * (1/W) + err_server;
 *   packed_out, *scale_out = C[zb];  err_server <- zb - C[zb].
 * packed_in: W consecutive blocks of n_c/32 words, block w = what worker w sent for this chunk.
 * scales_in: [W].  packed_out: [n_c/32].  scale_out: [1].  (All device pointers; packed_out may
 * point into the packed_all buffer of the next two calls.)  packed_in must be smaller than 2 GiB
 * (W * n_c / 8 < 2^31 bytes; OB_ERR_SIZE otherwise): its kernels use 32-bit offsets into it. */
ob_status ob_lamb_server_reduce(ob_lamb_ctx* ctx, const ob_lamb_state* st,
                                const uint32_t* packed_in, const float* scales_in,
                                uint32_t* packed_out, float* scale_out, void* hip_stream);

/* Algorithm 1 lines 13-20 per layer, from the W recompressed server chunks
 * (packed_all [N_pad/32] words, server_scales [W]):
 *   m_t = decompress / k_l;  g = (m_t - beta1*m)/(1-beta1);  v_fresh <- beta2*v_fresh + (1-beta2)*g^2;
 *   r = max over the layer of v_frozen/v_fresh (NaN skipped, starts at 0);
 *   r <- clip(r, (1-thr)*r_prev, (1+thr)*r_prev); r <- clip(r, r_min, r_max);
 *   r_prev <- r;  coeff_c <- r * c_avg.
 * Updates v_fresh, r_prev, coeff_c.  Does not touch m or x. */
ob_status ob_lamb_layer_ratios(ob_lamb_ctx* ctx, const ob_lamb_state* st,
                               const uint32_t* packed_all, const float* server_scales,
                               void* hip_stream);

/* Algorithm 1 lines 13 and 21: with m_t as above and coeff_c from ob_lamb_layer_ratios,
 *   x <- x - (lr*coeff_c) * m_t / (sqrt(v_frozen) + eta);   m <- m_t. */
ob_status ob_lamb_decompress_apply(ob_lamb_ctx* ctx, const ob_lamb_state* st,
                                   const uint32_t* packed_all, const float* server_scales,
                                   float lr, void* hip_stream);

/* ob_lamb_layer_ratios followed by ob_lamb_decompress_apply in ONE call, bit-identical results.
 * Momentum: if st->m is non-NULL it is the source of m_{t-1} and receives m_t (the two kernels of
 * the separate calls run).  If it is NULL the source is (st->m_packed, st->m_scales), which must
 * not be packed_all (OB_ERR_ARG), and nothing is written -- the new momentum is
 * packed_all/server_scales themselves, to be passed as m_packed/m_scales of the next step; then,
 * for every layer that holds whole tiles of 8192 elements and whose such tiles fit on the device at
 * once (at most 80 % of its workgroup slots), a single kernel keeps v_frozen and the sign words of
 * those tiles in registers across a per-layer barrier, so they are read once instead of twice
 * (4.125 bytes per parameter less); everything outside those tiles (larger layers, small tensors,
 * the spans where layers meet) takes the two kernels, restricted to it.  Waits are bounded as for
 * ob_lamb_compress_local (ob_lamb_check_device_status).  OB_CFG_NO_FUSED_APPLY in
 * ob_lamb_config.flags forces the two-kernel path for everything, ob_lamb_config.fused_max_tiles = n
 * for every layer with more than n such tiles. */
ob_status ob_lamb_ratios_apply(ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                               const float* server_scales, float lr, void* hip_stream);
/* The fresh variance in deferred form: ob_lamb_ratios_apply for callers that keep the sign words and
 * scales of the last few global momenta (they are the steps' own packed_all / server_scales buffers).
 *
 * With the momentum in 1-bit form the reconstructed gradient of Algorithm 1 line 15 takes one of two
 * magnitudes per chunk, layer and step, chosen per element by whether the momentum's sign bit
 * flipped.  The variance after several steps therefore follows from st->v_fresh as last written and
 * the momenta since then, by the very operations line 16 performs step by step (the results are
 * bit-identical); line 17 needs the up-to-date variance of every element, but the array need not be
 * rewritten at every step.  This applies to the tiles of the single kernel with the per-layer
 * barrier (see ob_lamb_ratios_apply; ob_lamb_fused_params of them) and to the whole 8192-element
 * tiles of the layers that are too large for it (ob_lamb_big_tile_params): with write_v = 0 the call reads
 * st->v_fresh there and writes nothing to it (4 bytes per parameter less than ob_lamb_ratios_apply,
 * plus one bit per parameter and older momentum read); with write_v = 1 it brings the array up to
 * date there, after which the history starts anew (the next call passes n_old = 0).  Everywhere
 * else -- the plain kernels' elements -- st->v_fresh is rewritten at every call as by
 * ob_lamb_ratios_apply and the history is not read (on their 1024-element tiles the ratio pass is
 * bound by its launch shape, not by the bytes it moves).
 *
 * n_old: number of momenta older than the previous one (st->m_packed / st->m_scales) that have been
 * committed since write_v was last 1 (or since ob_lamb_ratios_apply / the LAMB step last wrote
 * st->v_fresh), 0..OB_VF_MAX_OLD; bits[i] / scales[i], i < n_old: their sign words [N_pad/32] and
 * scales [W], NEWEST FIRST (bits[0] is the momentum before the previous one), device pointers,
 * 16-byte aligned, read only.  h = NULL means n_old = 0, write_v = 1: ob_lamb_ratios_apply itself.
 * Requires the momentum in 1-bit form (st->m == NULL, else OB_ERR_ARG).
 * Everything else -- layers, barrier, bounded waits, what an expired wait leaves behind -- as for
 * ob_lamb_ratios_apply.  A caller's duty: between a call with write_v = 0 and the next one with
 * write_v = 1, st->v_fresh is NOT the variance; ob_lamb_variance_dense gives it. */
#define OB_VF_MAX_OLD 7
typedef struct ob_lamb_vf_history {
  int32_t n_old;
  int32_t write_v;
  const uint32_t* bits[OB_VF_MAX_OLD];
  const float* scales[OB_VF_MAX_OLD];
} ob_lamb_vf_history;
ob_status ob_lamb_ratios_apply_hist(ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                                    const float* server_scales, float lr, const ob_lamb_vf_history* h,
                                    void* hip_stream);
/* Dense view of a variance held in that form: v_out [N_pad] receives the variance as of the momentum
 * (packed_all, server_scales), given st->v_fresh, st->m_packed / st->m_scales and h exactly as they
 * were passed to the ob_lamb_ratios_apply_hist call that committed that momentum (h->write_v is
 * ignored): a device copy of st->v_fresh, then the elements that lag are brought up to date.
 * v_out may be st->v_fresh itself (no copy; the array is then up to date and the next call passes
 * n_old = 0).  For checkpoints, inspection and a return to the LAMB step. */
ob_status ob_lamb_variance_dense(ob_lamb_ctx* ctx, const ob_lamb_state* st, const uint32_t* packed_all,
                                 const float* server_scales, const ob_lamb_vf_history* h, float* v_out,
                                 void* hip_stream);

/* Host-only planning query (no HIP call, no device needed): how ob_lamb_create splits a tensor list
 * between a kernel with a per-layer barrier and the plain kernels when one layer may occupy at most
 * max_tiles of that kernel's 8192-element tiles (on a device, 80 % of the kernel's workgroup
 * slots).  span_owner: host, [W * ceil(n_c / 1024)] bytes, one per 1024-element span of the
 * padded buffer, chunk-major (the last span of a chunk may be shorter): 0 = holds no parameter
 * (padding only, no kernel visits it), 1 = plain kernels, 2 = barrier kernel.  layer_listed: host,
 * [L], number of 8192-element tiles of each layer that the barrier kernel takes (0: the layer is
 * finished by the plain kernels).  Returns OB_ERR_NULL / OB_ERR_ARG like ob_lamb_create. */
ob_status ob_lamb_plan_split(const ob_lamb_config* cfg, int64_t max_tiles, uint8_t* span_owner,
                             int32_t* layer_listed);

/* Host-only, like ob_lamb_plan_split and for the same max_tiles: span_big [W * ceil(n_c / 1024)] bytes
 * receives 1 for the 1024-element spans inside the 8192-element tiles where ob_lamb_ratios_apply_hist
 * takes the ratio pass from the history although the barrier kernel does not hold them -- the whole
 * tiles of every layer that is not listed and has at least 64 of them -- and 0 elsewhere. */
ob_status ob_lamb_plan_big_tiles(const ob_lamb_config* cfg, int64_t max_tiles, uint8_t* span_big);

/* Number of layers the single kernel of ob_lamb_ratios_apply takes part in on this device (0..L). */
int64_t ob_lamb_fused_layers(const ob_lamb_ctx* ctx);
/* ... and the number of parameters in its tiles. */
int64_t ob_lamb_fused_params(const ob_lamb_ctx* ctx);
/* Number of parameters in the 8192-element tiles of the layers that are too large for that kernel,
 * where ob_lamb_ratios_apply_hist also works from the history (ratio pass only). */
int64_t ob_lamb_big_tile_params(const ob_lamb_ctx* ctx);
/* The same two counts for ob_lamb_warmup_step, which reads g, m, v and x once (one kernel with a
 * per-layer barrier that keeps eq. (1)'s update direction and x in registers while the layer's
 * norms complete) for every layer whose tiles fit on the device, and takes two passes for the
 * rest.  OB_CFG_TWO_PASS_WARMUP in ob_lamb_config.flags forces two passes for every layer. */
int64_t ob_lamb_warmup_fused_layers(const ob_lamb_ctx* ctx);
int64_t ob_lamb_warmup_fused_params(const ob_lamb_ctx* ctx);

/* Appendix A.5.2, end of warmup: forms the momentum-scale coefficients from the dense momentum
 * st->m and writes them to st->mom_scale [L] (must be non-NULL here).  The paper gives no formula;
 * this library takes sigma_l = ||m_l||_2 / sqrt(n_l), k_l = mean(sigma) / sigma_l with the mean over
 * the non-empty layers, and k_l = 1 where sigma_l = 0 or the layer is empty, so that every layer
 * enters the fused compression with the same RMS.  fp64 accumulation, one rounding to fp32. */
ob_status ob_lamb_momentum_scale(ob_lamb_ctx* ctx, const ob_lamb_state* st, void* hip_stream);

/* ---- Mixed-precision variant: 16-bit gradient in, 16-bit copy of the parameters out ----------
 * The paper trains in FP16 (Section 6; its communication-volume figures are against FP16): the
 * backward pass hands the optimizer a 16-bit gradient, possibly multiplied by a loss scale, and the
 * forward pass reads a 16-bit copy of the parameters.  The `_lp` entry points below take and
 * produce those directly, so that no separate cast pass over N elements is needed.  State and
 * arithmetic stay binary32 and every other argument is as in the entry point of the same name:
 *   gradient   g[i] = value(grad[i]) * grad_scale    (decode exact, one binary32 multiply; pass
 *              the inverse loss scale, or 1).  grad: [N_pad] device, 16-byte aligned, of type
 *              grad_dtype; OB_F32 requires grad_scale == 1 (OB_ERR_ARG otherwise) and is then the
 *              plain entry point.
 *   parameters x_lp[i] = x[i] after the update, rounded to nearest (ties to even) in x_dtype
 *              (overflow -> infinity, NaN -> 0x7e00 / 0x7fc0), for every i that belongs to a
 *              layer; the padding of x_lp is never written.  x_lp: [N_pad] device, 16-byte
 *              aligned, or NULL for no copy (x_dtype is then ignored); OB_F32 is not accepted
 *              for a non-NULL x_lp (OB_ERR_ARG): st->x is that array. */
typedef enum ob_dtype { OB_F32 = 0, OB_F16 = 1, OB_BF16 = 2 } ob_dtype;

ob_status ob_lamb_warmup_step_lp(ob_lamb_ctx* ctx, const ob_lamb_state* st, const void* grad,
                                 ob_dtype grad_dtype, float grad_scale, float lr, void* x_lp,
                                 ob_dtype x_dtype, void* hip_stream);
ob_status ob_lamb_compress_local_lp(ob_lamb_ctx* ctx, const ob_lamb_state* st, const void* grad,
                                    ob_dtype grad_dtype, float grad_scale, uint32_t* packed_out,
                                    float* scales_out, void* hip_stream);
ob_status ob_lamb_decompress_apply_lp(ob_lamb_ctx* ctx, const ob_lamb_state* st,
                                      const uint32_t* packed_all, const float* server_scales,
                                      float lr, void* x_lp, ob_dtype x_dtype, void* hip_stream);
ob_status ob_lamb_ratios_apply_lp(ob_lamb_ctx* ctx, const ob_lamb_state* st,
                                  const uint32_t* packed_all, const float* server_scales, float lr,
                                  void* x_lp, ob_dtype x_dtype, void* hip_stream);
/* ob_lamb_ratios_apply_hist with the 16-bit copy of the parameters (h as there, x_lp / x_dtype as above). */
ob_status ob_lamb_ratios_apply_hist_lp(ob_lamb_ctx* ctx, const ob_lamb_state* st,
                                       const uint32_t* packed_all, const float* server_scales, float lr,
                                       const ob_lamb_vf_history* h, void* x_lp, ob_dtype x_dtype,
                                       void* hip_stream);

/* Kernels with an in-kernel barrier, and what happens if one of their waits expires
 * -----------------------------------------------------------------------------------
 * ob_lamb_compress_local runs as ONE kernel that keeps z in registers across a per-chunk arrival
 * barrier whenever one chunk's workgroups fill at most 80 % of the device (otherwise, or with
 * OB_CFG_TWO_PASS_COMPRESS, as two passes through memory).  ob_lamb_server_reduce,
 * ob_lamb_ratios_apply and ob_lamb_warmup_step have such a form too (per chunk / per layer).  All
 * forms compute the same operations in the same order per element; the two sum-of-squares
 * reductions add the same fp64 terms grouped by different tile sizes, so a scale or norm can differ
 * in its last binary32 bit between forms (about once in 10^8 reductions) -- within the 1e-6 bar,
 * and the sign words that depend on such a scale can then differ for elements within one unit in
 * the last place of zero.
 *
 * Progress of a barrier rests on two things the HIP programming model does not promise but the
 * hardware's dispatcher provides: workgroups start in index order, and a chunk's (layer's)
 * workgroups are all resident at once -- the host checks the second against the kernel's occupancy
 * on the device and keeps a 20 % margin.  The barrier kernels count on having the device to
 * themselves while they run: kernels of other streams or processes that keep more than a fifth of
 * the compute units busy for seconds on end can make a wait expire; shorter interference only slows
 * them down.  Every wait is bounded by ob_lamb_config.spin_limit polls (one 8-byte atomic load,
 * whose round trip to the memory side is of the order of a microsecond, plus a sleep of 1024
 * clocks = 0.43 us at 2.4 GHz): with the default of 2^20 polls a wait lasts 1.5 s at most (3 s at
 * half the clock), and once one wait has expired every other wait of the context ends within 64
 * polls, so a kernel in which a wait expires still ends about 2 s after its last workgroup started.
 *
 * An expired wait does NOT stop the kernel: the workgroup goes on with whatever the flag word last
 * held (a stale scale or coefficient), raises a device-side flag, and the step's outputs are
 * undefined.  The buffers updated in place are then corrupt and must be restored from a copy that
 * the CALLER holds -- the library keeps none:
 *   ob_lamb_compress_local   err_worker (and packed_out, scales_out)
 *   ob_lamb_server_reduce    err_server (and packed_out, scale_out)
 *   ob_lamb_ratios_apply     x, v_fresh, r_prev, coeff_c
 *   ob_lamb_warmup_step      x, m, v_fresh, c_avg, coeff_c
 * No step call returns OB_ERR_STATE by itself (none of them synchronises).  The caller learns of an
 * expiry from ob_lamb_check_device_status, which synchronises `hip_stream`, reads the flag and
 * returns OB_OK, or OB_ERR_STATE after re-arming the context to use the barrier-free kernels from
 * then on.  Call it at every point where the state is about to become irreplaceable -- before a
 * checkpoint is written, before the previous checkpoint is dropped, and at a fixed interval of steps
 * (it costs one stream synchronisation); on OB_ERR_STATE restore x, m, v_fresh, err_worker,
 * err_server, c_avg, r_prev from the last checkpoint taken after an OB_OK and redo the steps.
 * ob_lamb_uses_single_pass reports the current choice for ob_lamb_compress_local (1/0). */
ob_status ob_lamb_check_device_status(ob_lamb_ctx* ctx, void* hip_stream);
int32_t ob_lamb_uses_single_pass(const ob_lamb_ctx* ctx);
/* ob_lamb_server_reduce as one kernel with a chunk barrier (the averaged chunk stays in registers
 * between Algorithm 1 line 10's sum and its recompression): 0 if the three-kernel form is used (the
 * served chunk's workgroups do not fit on the device at once, OB_CFG_TWO_PASS_COMPRESS, or after
 * an expired wait), else the kernel's tile size in units of 1024 elements (1, 2 or 4). */
int32_t ob_lamb_server_single_pass(const ob_lamb_ctx* ctx);

/* ob_lamb_server_reduce for callers that cannot allocate device memory -- code running under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same
 * arguments' meaning (all device pointers, 16-byte aligned; num_workers = W, chunk_len = n_c, a
 * multiple of 256), but no context: the partial sums between its kernels live in a fixed array
 * inside the library's device image (256 KiB per GPU, held until the process ends), whose address
 * on a device is looked up once, by the first ob_lamb_create or the first call of this function with
 * that device current (a caller under graph capture makes one of the two before the capture
 * begins).  It calls no hipMalloc/hipFree or any allocating routine, enqueues three kernels on
 * `hip_stream` and returns without synchronising.
 *   chunk_len > ob_lamb_static_max_chunk_len() (2^25 elements), or a packed_in of 2 GiB or more
 *   -> OB_ERR_SIZE, nothing enqueued;
 *   other invalid sizes -> OB_ERR_ARG; NULL / misaligned pointers -> OB_ERR_NULL / OB_ERR_ALIGN.
 * Every call on one GPU uses that GPU's one array: calls that overlap in time on one GPU (two
 * streams, two threads) race; order them yourself.  Results equal ob_lamb_server_reduce's in its
 * three-kernel form bit for bit. */
ob_status ob_lamb_server_reduce_static(int32_t num_workers, int64_t chunk_len, const uint32_t* packed_in,
                                       const float* scales_in, float* err_server, uint32_t* packed_out,
                                       float* scale_out, void* hip_stream);
int64_t ob_lamb_static_max_chunk_len(void);

/* Diagnostics: dst[0..n) <- src[0..n) (device pointers, 16-byte aligned, not overlapping) by a plain
 * streaming kernel in the shape of the library's N-sized kernels (1024-element tiles, 128-bit
 * nontemporal accesses).  Its rate (8n bytes per launch) is the device's practical streaming
 * ceiling; the benchmark reports every kernel against it next to the published peak. */
ob_status ob_lamb_diag_copy(const float* src, float* dst, int64_t n, void* hip_stream);

/* ---- per-kernel timing (diagnostics; used by the benchmark) ----
 * While enabled, every kernel launch of this context carries a pair of HIP events that the device
 * stamps with the kernel's own start and end (hipExtLaunchKernel).
 * ob_lamb_profile_read synchronises, aggregates by kernel and clears the record.
 * Returns the number of distinct kernels; fills up to `cap` entries of each array.
 * names[i] points to a static string. */
ob_status ob_lamb_profile_enable(ob_lamb_ctx* ctx, int on);
int32_t ob_lamb_profile_read(ob_lamb_ctx* ctx, int32_t cap, const char** names,
                             double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* ONEBITLAMB_H */
