/*
 * adloco.h -- C ABI of the AdLoCo data-parallel hot path on one MI355X (gfx950).
 *
 * Two halves:
 *   1. adaptive-batch statistics: per-sample gradient squared norms of linear layers, the
 *      batch-gradient norm, the norm test / batch rule and the SwitchMode decision;
 *   2. the multi-instance DiLoCo outer step (averaged pseudo-gradient, Nesterov outer
 *      update, optional worker reset), the batch-weighted trainer merge, and the workers'
 *      fused inner optimizer step.
 *
 * Conventions (all entry points)
 *   - Return value: 0 = ADLOCO_OK, otherwise one of the ADLOCO_E* codes below.  No exception
 *     crosses this boundary.  adloco_last_error() gives a human-readable reason for the last
 *     failing call on that context (valid until the next call on it).
 *   - "device" pointers are device (HBM) addresses owned by the caller (PyTorch-ROCm
 *     allocations in the Python binding); the library never frees, reallocates or keeps
 *     them.  They must stay alive until the work enqueued on `stream` has completed.
 *     "host" pointers are ordinary host memory, read before the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All device work
 *     is enqueued on it.  When a call waits for the stream:
 *       * adloco_norm_test and adloco_inner_product_test always do (they return scalars to
 *         the host);
 *       * adloco_grad_stats, adloco_inner_products and adloco_norm_test do on the FIRST call
 *         with a new list of shapes -- number of blocks, their kinds and flags, d_in, d_out, row
 *         strides, 16-byte alignment class of a / delta, dtype, and for the statistics B and T:
 *         that call builds the tile and job tables, which allocates scratch memory, copies
 *         tables from the host and waits for the copies.  It must not be captured into a graph.
 *       * Every later call with the same shapes returns as soon as its kernels are enqueued,
 *         whatever the addresses in a, delta and grad_sum are: the pointers of a call travel in
 *         kernel arguments, nothing is allocated, copied from the host or waited for, and such
 *         a call can be captured (its pointers are part of the captured launches).
 *       * Every other call returns as soon as its kernels are enqueued.
 *   - A context owns only scratch memory (partial sums, descriptor tables, a few pinned
 *     doubles).  One context must not be used from two host threads at once, nor on two
 *     streams whose work may overlap.
 *   - Buffers must not alias unless the argument is documented "in/out".
 */
#ifndef ADLOCO_H
#define ADLOCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ------------------------------------------------------------------- */
#define ADLOCO_OK            0
#define ADLOCO_EINVAL        1  /* NULL / negative / inconsistent / misaligned argument        */
#define ADLOCO_EUNSUPPORTED  2  /* dtype, size or count outside what the kernels handle       */
#define ADLOCO_ENOMEM        3  /* scratch allocation failed                                  */
#define ADLOCO_EHIP          4  /* a HIP runtime call failed (text in adloco_last_error)      */
#define ADLOCO_ESTATE        5  /* accumulate requested on an accumulator that holds no batch */

/* ---- element types of a and delta --------------------------------------------------- */
#define ADLOCO_F32   0
#define ADLOCO_BF16  1
#define ADLOCO_F16   2   /* IEEE half: the mixed-precision setting of the paper's experiments (Section 6) */

/* ---- flags -------------------------------------------------------------------------- */
#define ADLOCO_ACCUMULATE       0x1u  /* grad_stats: continue a batch (switch mode micro-batch) */
#define ADLOCO_SUM_ONLY         0x2u  /* grad_stats: form the gradient sums only, no norms       */
#define ADLOCO_GRAD_PROVIDED    0x1u  /* linear_desc.flags: caller maintains grad_sum itself     */
/* linear_desc.flags, bits 4..7: which block of the parameters the descriptor stands for      */
#define ADLOCO_KIND_LINEAR      0x00u /* weight W [d_out, d_in] of a linear layer (the default)  */
#define ADLOCO_KIND_VECTOR      0x10u /* vector p [d_out] used element-wise: a bias or a gain    */
#define ADLOCO_KIND_EMBED       0x20u /* embedding table E [d_in, d_out], a = int32 token ids    */
#define ADLOCO_KIND_MASK        0xf0u
#define ADLOCO_BROADCAST        0x1u  /* outer_step: also write the new outer model into theta_k */
#define ADLOCO_BIASED_VAR       0x1u  /* norm_test: variance normalised by 1/B instead of 1/(B-1)*/
#define ADLOCO_ALLOW_SHRINK     0x2u  /* norm_test: raw ceil rule, requested batch may decrease   */

#define ADLOCO_MAX_INSTANCES   16     /* largest M of adloco_outer_step and S of adloco_merge    */

typedef struct adloco_ctx adloco_ctx;

/* Create / destroy a context on HIP device `device`.  adloco_create makes that device
 * current for the calling thread.  adloco_destroy frees the scratch memory (it waits for
 * the device).  adloco_last_error(NULL) returns the reason adloco_create itself failed. */
int adloco_create(adloco_ctx** out, int device);
int adloco_destroy(adloco_ctx* ctx);
const char* adloco_last_error(const adloco_ctx* ctx);

/* ------------------------------------------------------------------------------------ *
 * Gradient statistics.
 *
 * One linear layer l with weight W [d_out, d_in].  Sample i of the batch has activations
 * a_i [T, d_in] (the layer's input) and output gradients delta_i [T, d_out] (per sample,
 * NOT averaged over the batch).  Its per-sample gradient is g_i^l = sum_t delta_{i,t}
 * a_{i,t}^T, the term that the mini-batch gradient g_k = (1/b_k) sum_i grad f(x_k; xi_i)
 * of eq. 1 (Section 2.1) averages; the variance of Section 3.3.1 needs ||g_i||^2.
 * ------------------------------------------------------------------------------------ */
typedef struct {
  const void* a;          /* device [B, T, d_in], token rows a_row_stride elements apart      */
  const void* delta;      /* device [B, T, d_out], token rows delta_row_stride apart          */
  int32_t d_in, d_out;    /* >= 1                                                             */
  int64_t a_row_stride;   /* elements between consecutive tokens; 0 means d_in (contiguous)   */
  int64_t delta_row_stride; /* likewise; 0 means d_out                                        */
  float* grad_sum;        /* device [d_out, d_in] fp32, contiguous, in/out: running sum_i g_i^l
                             over the (accumulated) batch.  Written by adloco_grad_stats
                             unless ADLOCO_GRAD_PROVIDED; read by adloco_norm_test.  May be
                             NULL in adloco_grad_stats with ADLOCO_GRAD_PROVIDED.             */
  uint32_t flags;         /* ADLOCO_GRAD_PROVIDED and / or one ADLOCO_KIND_* value            */
  uint32_t reserved;      /* must be 0                                                        */
} adloco_linear_desc;

/* The other blocks of grad f(x_k; xi_i) (eq. 1 averages the gradient with respect to ALL
 * parameters) reuse the same descriptor; their norms add to the same per-sample totals:
 *
 * ADLOCO_KIND_VECTOR  a vector p [d_out] that enters a layer element-wise, y_t = p * x_t + ...
 *     g_i = sum_t delta_{i,t} * x_{i,t}.  `a` = x [B, T, d_out] (for the gain of a
 *     normalisation layer: its normalised input), or NULL for x = 1 (a bias: g_i = sum_t
 *     delta_{i,t}).  d_in must be 1; a_row_stride 0 means d_out; grad_sum is [d_out].
 * ADLOCO_KIND_EMBED   an embedding table E [d_in = V, d_out]: `a` = token ids, device int32
 *     [B, T] contiguous (a_row_stride unused); row v of g_i = sum of delta_{i,t} over the
 *     tokens with id v, so ||g_i||^2 = sum_{t,t'} [id_t = id_t'] delta_t . delta_t'.  The table
 *     gradient itself is the caller's: ADLOCO_GRAD_PROVIDED is required, grad_sum [V, d_out] is
 *     only read (by adloco_norm_test) and may be NULL in adloco_grad_stats.  T <= 8192.
 * Both kinds stream delta (and x) once; their sums run in a fixed order.  A gain and a bias that are
 * given the same delta tensor (the two vectors of a normalisation layer) are formed in one pass
 * over it.  All kernels run on `stream`, one after the other. */

/* Running accumulator of one (possibly accumulated) batch; lives in device memory, owned by
 * the caller (16 bytes, 8-byte aligned). */
typedef struct {
  double  sum_sample_sqnorm;  /* S1 = sum_i ||g_i||^2 over all samples seen so far           */
  int64_t n_samples;          /* number of samples seen so far                               */
} adloco_stats_acc;

/* adloco_grad_stats: per-sample squared gradient norms of one (micro-)batch by the Gram
 * identity  ||sum_t delta_t a_t^T||_F^2 = sum_{t,t'} (a_t . a_t')(delta_t . delta_t'),
 * plus, for every layer without ADLOCO_GRAD_PROVIDED, grad_sum (+)= sum_i delta_i^T a_i
 * (eq. 1 times b_k; Algorithm 3's "g <- g + grad L" in the accumulate branch).
 *
 *   layers   host array of n_layers descriptors (read before return), 1 <= n_layers <= 4096
 *   B, T     samples in this micro-batch and tokens per sample, >= 1 (all layers share them)
 *   dtype    ADLOCO_F32, ADLOCO_BF16 or ADLOCO_F16: element type of every a and delta
 *   per_sample_sqnorm        device [B] fp32, overwritten: sum_l ||g_i^l||^2 of this micro-batch
 *   per_layer_sample_sqnorm  device [n_layers, B] fp32, overwritten; or NULL
 *   acc      device accumulator.  Without ADLOCO_ACCUMULATE it is reset first (and grad_sum
 *            is overwritten); with it, S1, n_samples and grad_sum continue from their values
 *            (ADLOCO_ESTATE is NOT detected on the device: the flag is the caller's promise
 *            that acc and grad_sum hold the earlier micro-batches of the same batch).
 *   flags    0, ADLOCO_ACCUMULATE and / or ADLOCO_SUM_ONLY.  With ADLOCO_SUM_ONLY the call is the
 *            plain "g <- g + grad L" of Algorithm 3 for a batch whose statistics nobody asks for
 *            (every batch but the one that feeds the norm test): grad_sum (+)= sum_i delta_i^T a_i
 *            by an ordinary GEMM, nothing else is written; per_sample_sqnorm, per_layer_sample_sqnorm
 *            and acc may be NULL.
 * bf16 and fp16 inputs are multiplied exactly and accumulated in fp32 (MFMA); fp32 inputs in
 * fp32.  16-bit rows must be 2-byte aligned; 16-byte aligned rows with d % 8 == 0 take the fast
 * path, anything else a slower guarded path (same results).
 * Linear blocks that are handed the SAME activation tensor (same address, stride and d_in) with the same
 * d_out -- q / k / v or gate / up of a transformer block -- share their a_i a_i^T: the Gram kernel forms
 * it once for the group (same results up to fp32 summation order).
 * Two routes give the norms of the linear blocks.  With ADLOCO_GRAD_PROVIDED (the framework's
 * backward already holds the weight gradient) only the Gram contractions run.  When grad_sum
 * is formed here for every linear block and all of them are 16-byte aligned bf16 / fp16 with
 * T % 32 == 0, the 256 x 128 tiles of the per-sample gradients delta_i^T a_i that add up to
 * grad_sum pass through the registers one sample after the other and are squared there, so the
 * Gram contractions are not needed at all; adloco_set_tuning(ctx, "stats_variant", 0) keeps the
 * Gram kernel plus a separate gradient-sum GEMM instead.  Same results up to fp32 rounding. */
int adloco_grad_stats(adloco_ctx* ctx, const adloco_linear_desc* layers, int n_layers,
                      int B, int T, int dtype,
                      float* per_sample_sqnorm, float* per_layer_sample_sqnorm,
                      adloco_stats_acc* acc, uint32_t flags, void* stream);

/* Result of the norm test, batch rule and SwitchMode for one trainer. */
typedef struct {
  double  S1;                 /* sum_i ||g_i||^2                                               */
  double  S2;                 /* ||sum_i g_i||^2                                               */
  double  batch_grad_sqnorm;  /* ||g_k||^2 = S2 / B^2 (eq. 1)                                  */
  double  variance;           /* sigma^2_{B_k} = (S1 - S2/B)/(B-1)   (or /B if BIASED_VAR)     */
  double  stat;               /* sigma^2 / (eta^2 ||g_k||^2); NaN if undefined, +inf if g_k=0  */
  int64_t n_samples;          /* B, read from the accumulator                                  */
  int64_t b_cur;              /* echoed                                                        */
  int64_t b_req;              /* requested batch for the next outer step                       */
  int64_t b_micro;            /* micro-batch size to run with                                  */
  int64_t accum_steps;        /* ceil(b_req / b_max) when accumulating, else 1                 */
  int32_t test_passed;        /* 1 iff stat <= b_cur (eq. 4 rearranged)                        */
  int32_t accumulate;         /* 1 iff b_req > n_switch * b_max (SwitchMode)                   */
  int32_t stat_undefined;     /* 1 iff B < 2 with the unbiased variance (0/0)                  */
  int32_t reserved;           /* 0                                                             */
} adloco_norm_test_result;

/* adloco_norm_test: S2 = sum_l ||grad_sum_l||_F^2 on the device, then on the host in fp64:
 * the approximate norm test (eq. 4), the batch rule b_{k+1} = ceil(sigma^2 / (eta^2
 * ||grad F_B||^2)) (Section 3.3.1) and SwitchMode (Section 4.2; Algorithm 3).
 *   b_req = min(b_cap, max(b_cur, ceil(stat), 1))   (b_cur dropped with ADLOCO_ALLOW_SHRINK;
 *   b_cap = 0 means no ceiling);  B = 1: stat undefined, b_req = max(b_cur, 2).
 *   layers   host array; only grad_sum, d_in, d_out are used
 *   acc      device accumulator filled by adloco_grad_stats
 *   eta > 0; b_cur >= 1; b_max >= 1; n_switch >= 1; b_cap >= 0
 *   out      host, written before return.  This call waits for `stream`. */
int adloco_norm_test(adloco_ctx* ctx, const adloco_linear_desc* layers, int n_layers,
                     const adloco_stats_acc* acc, double eta, int64_t b_cur, int64_t b_max,
                     int32_t n_switch, int64_t b_cap, uint32_t flags,
                     adloco_norm_test_result* out, void* stream);

/* adloco_norm_test_noalloc: adloco_norm_test for callers that cannot allocate -- code between
 * the begin and the end of a graph capture of another stream, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels, same result; the partial sums and the device
 * copy of the block table live in a fixed device array of the library (about 1.1 MB per GPU, held
 * until the process ends) instead of scratch memory that the context allocates on demand, so the
 * call never allocates, frees or resizes anything.  Limits: n_layers <= 512 and at most 131072
 * partial sums of 16384 gradient entries each (2^31 entries when every block fills its last
 * chunk); beyond them ADLOCO_EUNSUPPORTED with the reason in adloco_last_error.  All calls on
 * one GPU share that array: two calls whose device work may overlap (other streams, other
 * contexts, other threads) race and must be ordered by the caller.  Waits for `stream`. */
int adloco_norm_test_noalloc(adloco_ctx* ctx, const adloco_linear_desc* layers, int n_layers,
                             const adloco_stats_acc* acc, double eta, int64_t b_cur, int64_t b_max,
                             int32_t n_switch, int64_t b_cap, uint32_t flags,
                             adloco_norm_test_result* out, void* stream);

/* Host-only halves of adloco_norm_test (no device, no context): the decision from given
 * S1, S2, B, and SwitchMode alone.  Same formulas, same edge conventions. */
int adloco_norm_test_decide(double S1, double S2, int64_t n_samples, double eta,
                            int64_t b_cur, int64_t b_max, int32_t n_switch, int64_t b_cap,
                            uint32_t flags, adloco_norm_test_result* out);
int adloco_switch_mode(int64_t b_req, int64_t b_max, int32_t n_switch,
                       int32_t* accumulate, int64_t* accum_steps, int64_t* b_micro);

/* ------------------------------------------------------------------------------------ *
 * adloco_outer_step: Algorithm 3's pseudo-gradient and outer update for one trainer,
 *   Delta = (1/M) sum_m (theta_outer - theta_m);   buf <- mu*buf + Delta;
 *   theta_outer <- theta_outer - lr * (nesterov ? Delta + mu*buf : buf)
 * with OuterOpt = SGD with (Nesterov) momentum (mu = 0: plain SGD, the theorems' setting),
 * and, with ADLOCO_BROADCAST, Algorithm 3's worker reset theta_m <- theta_outer.
 *   theta_outer      device [N] fp32, in/out
 *   theta_inst       HOST array of M device pointers, each [N] fp32 (written only with
 *                    ADLOCO_BROADCAST); 1 <= M <= ADLOCO_MAX_INSTANCES; no aliasing
 *   momentum         device [N] fp32 in/out; may be NULL iff mu == 0
 *   pseudo_grad_out  device [N] fp32 or NULL: receives Delta
 * N = 0 is a successful no-op.  16-byte aligned pointers take the vector path, others a
 * scalar path with the same results.  Arithmetic is fp64 in registers, rounded once. */
int adloco_outer_step(adloco_ctx* ctx, float* theta_outer, float* const* theta_inst, int M,
                      size_t N, float* momentum, double lr, double mu, int nesterov,
                      uint32_t flags, float* pseudo_grad_out, void* stream);

/* ------------------------------------------------------------------------------------ *
 * The outer step and the merge on instance DRIFTS stored in bf16.  What Algorithm 3 averages is
 * the drift d_m = x^{(t-1)} - x_m^{(t,H)} of every instance (the Delta line); kept in bf16 it costs
 * 2 bytes per instance and parameter instead of 4 -- the traffic (on one GPU: HBM bytes, across
 * GPUs: the message) that the paper's motivation is about (Sections 1 and 3.2) -- at a rounding
 * error of at most 2^-8 of the drift itself.  Outer model and momentum stay fp32.
 *
 * adloco_pack_drift: drift_out = bf16(theta_outer - theta_m): the fp32 difference rounded to
 *   nearest-even.  drift_out: device [N] bf16 bit patterns, may not overlap the inputs.
 * adloco_outer_step_drift: adloco_outer_step with Delta = (1/M) sum_m d_m read from M bf16
 *   vectors.  drift: HOST array of M device pointers, each [N] bf16 (written only with
 *   ADLOCO_BROADCAST: the worker reset x_m <- x_outer leaves every drift at zero).  All other
 *   arguments, conventions and error codes as adloco_outer_step.  Reads 8 + 2 M and writes 8 bytes
 *   per parameter (adloco_outer_step: 8 + 4 M and 8).
 * adloco_merge_drift: DoMerge (Algorithm 2) when the other trainers are known by their drifts
 *   from the representative, d_j = x_r - x_j:  x_r <- x_r - sum_{j != r} b_j d_j / sum_j b_j, which
 *   is sum_j b_j x_j / sum_j b_j.  x_rep: device [N] fp32 in/out; drift: HOST array of n_others
 *   device pointers ([N] bf16, read only); w_rep = b_r, w_others: HOST [n_others], all > 0;
 *   n_others + 1 <= ADLOCO_MAX_INSTANCES; n_others = 0 leaves x_r as it is.
 * 16-byte aligned pointers take the vector path, others a scalar path with the same results;
 * fp64 in registers, rounded once. */
int adloco_pack_drift(adloco_ctx* ctx, const float* theta_outer, const float* theta_m,
                      uint16_t* drift_out, size_t N, void* stream);
int adloco_outer_step_drift(adloco_ctx* ctx, float* theta_outer, uint16_t* const* drift, int M,
                            size_t N, float* momentum, double lr, double mu, int nesterov,
                            uint32_t flags, float* pseudo_grad_out, void* stream);
int adloco_merge_drift(adloco_ctx* ctx, float* x_rep, const uint16_t* const* drift, double w_rep,
                       const double* w_others, int n_others, size_t N, void* stream);

/* ------------------------------------------------------------------------------------ *
 * Inner-product test and augmented inner-product test (Section 3.3.2), the two alternatives to
 * the norm test.  Both need, per sample, the inner product with the batch gradient
 *   c_i = <g_i, G>,  G = sum_j g_j  (the grad_sum buffers; <g_i, g_k> = c_i / B),
 * which can only be formed once G is complete: call adloco_inner_products after
 * adloco_grad_stats has seen the whole (accumulated) batch, once per micro-batch whose a and
 * delta are still (or again) available, with ADLOCO_ACCUMULATE from the second call on.
 * ------------------------------------------------------------------------------------ */
typedef struct {
  double  sum_ip;      /* sum_i c_i  (equals ||G||^2 once every sample has been seen)           */
  double  sum_ip_sq;   /* sum_i c_i^2                                                           */
  int64_t n_samples;
  int64_t reserved;
} adloco_ip_acc;       /* device memory, caller-owned, 32 bytes, 8-byte aligned                 */

/* adloco_inner_products: c_i for the B samples of one micro-batch against the grad_sum buffers
 * of the descriptors (every kind; all grad_sum non-NULL, only read; table ids outside [0, V)
 * contribute nothing).  For 16-byte aligned bf16 linear layers with T % 32 == 0 the 256 x 128
 * tiles of each per-sample gradient delta_i^T a_i are formed by MFMA in registers and reduced
 * against the fp32 tile of G on the spot; other blocks take a plain (slow) path.  B <= 32767.
 *   per_sample_ip      device [B] fp32, overwritten: c_i
 *   per_sample_sqnorm  device [B] fp32 or NULL, overwritten: ||g_i||^2 from the explicit per-sample
 *                      gradients (a second route to adloco_grad_stats' Gram result)
 *   acc                device accumulator; reset unless ADLOCO_ACCUMULATE */
int adloco_inner_products(adloco_ctx* ctx, const adloco_linear_desc* layers, int n_layers, int B,
                          int T, int dtype, float* per_sample_ip, float* per_sample_sqnorm,
                          adloco_ip_acc* acc, uint32_t flags, void* stream);

typedef struct {
  double  S1, S2, batch_grad_sqnorm;   /* as in adloco_norm_test_result                          */
  double  var_ip;      /* Var_i <g_i, g_k>, 1/(B-1)                                              */
  double  stat_ip;     /* var_ip / (vartheta^2 ||g_k||^4)                                        */
  double  var_aug;     /* Var_i (g_i - <g_i,g_k>/||g_k||^2 g_k) = sum_i (||g_i||^2 -
                          <g_i,g_k>^2/||g_k||^2) / (B-1): the residuals average to zero          */
  double  stat_aug;    /* var_aug / (nu^2 ||g_k||^2)                                             */
  int64_t n_samples, b_cur;
  int64_t b_req_ip;    /* min(b_cap, max(b_cur, ceil(stat_ip), 1))                               */
  int64_t b_req_aug;   /* min(b_cap, max(b_cur, ceil(max(ceil(stat_ip), stat_aug)), 1))          */
  int64_t b_micro_ip, accum_steps_ip, b_micro_aug, accum_steps_aug;   /* SwitchMode of each      */
  int32_t accumulate_ip, accumulate_aug;
  int32_t stat_undefined;   /* 1 iff B < 2: both requests are max(b_cur, 2)                      */
  int32_t reserved;
} adloco_ip_test_result;

/* adloco_inner_product_test: S2 on the device as in adloco_norm_test, then both batch rules of
 * Section 3.3.2 and SwitchMode on the host in fp64.  vartheta > 0, nu > 0 (the paper's table:
 * 0.01 and 0.3).  Waits for `stream`.  adloco_inner_product_decide is the host-only half. */
int adloco_inner_product_test(adloco_ctx* ctx, const adloco_linear_desc* layers, int n_layers,
                              const adloco_stats_acc* acc, const adloco_ip_acc* ip, double vartheta,
                              double nu, int64_t b_cur, int64_t b_max, int32_t n_switch,
                              int64_t b_cap, adloco_ip_test_result* out, void* stream);
int adloco_inner_product_decide(double S1, double S2, double sum_ip, double sum_ip_sq,
                                int64_t n_samples, double vartheta, double nu, int64_t b_cur,
                                int64_t b_max, int32_t n_switch, int64_t b_cap,
                                adloco_ip_test_result* out);

/* adloco_inner_step: Algorithm 3's  x_m <- InnerOpt(x_m, g)  with InnerOpt = AdamW, the inner
 * optimizer of Section 6.1 (learning rate 4e-4, weight decay 0.1), one fused pass:
 *   g = grad_scale * grad;   x <- x - lr*weight_decay*x;
 *   m <- beta1 m + (1-beta1) g;   v <- beta2 v + (1-beta2) g^2;
 *   x <- x - lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
 *   theta        device [N] fp32, in/out: the worker's parameters x_m
 *   exp_avg      device [N] fp32, in/out: m;   exp_avg_sq  device [N] fp32, in/out: v
 *   grad         device [N] fp32, read only: a gradient SUM, e.g. the grad_sum buffers of
 *                adloco_grad_stats laid out back to back (in switch mode the sum over the
 *                accumulated micro-batches, Algorithm 3's "g <- g + grad L")
 *   grad_scale   multiplies grad: 1 / (number of samples summed) gives eq. 1's g_k
 *   step         1, 2, ...: the number of this update (bias correction); beta1, beta2 in [0,1)
 * No buffer may alias another.  N = 0 is a successful no-op.  16-byte aligned pointers take
 * the vector path, others a scalar path with the same results.  fp64 in registers, rounded
 * once.  Reads 16 and writes 12 bytes per parameter. */
int adloco_inner_step(adloco_ctx* ctx, float* theta, float* exp_avg, float* exp_avg_sq,
                      const float* grad, size_t N, double grad_scale, double lr, double beta1,
                      double beta2, double eps, double weight_decay, int64_t step, void* stream);

/* adloco_merge: DoMerge (Algorithm 2; Section 4.1.1): x_r <- sum_j b_j x_j / sum_j b_j for
 * the representative r = argmax b_j (lowest index on ties) or the given `rep`; the other
 * S-1 vectors are left untouched (the caller drops them and keeps r's optimizer state).
 *   x        HOST array of S device pointers, each [N] fp32; 1 <= S <= ADLOCO_MAX_INSTANCES
 *   weights  HOST [S], the requested batches b_j, all > 0
 *   rep      index to overwrite, or -1 for argmax
 *   rep_out  host, receives r; may be NULL */
int adloco_merge(adloco_ctx* ctx, float* const* x, const double* weights, int S, size_t N,
                 int rep, int* rep_out, void* stream);

/* adloco_check_merge: CheckMerge (Algorithm 1), host only: nothing when w = 0 or k <= 1;
 * else the w trainers with the smallest requested batch (ascending, ties by index) when
 * w <= k; else nothing.  sel_out: host [max(w,1)]; n_sel receives the count (0 or w). */
int adloco_check_merge(const int64_t* b_req, int k, int w, int* sel_out, int* n_sel);

/* ------------------------------------------------------------------------------------ *
 * adloco_round: one outer step t of Algorithm 3 for k trainers co-resident on the device,
 * as a host loop over the entry points above.  The model's forward / backward is the
 * caller's: the driver asks for it through `batch_fn`.
 *
 *   1. k > 1: M_t = CheckMerge({b_req_i}, merge_w); if non-empty DoMerge (Algorithm 2) on the
 *      trainers' outer models with weights b_req; the merged-away trainers are moved to the end
 *      of `trainers` (order of the others preserved) and *k shrinks.
 *   2. per trainer: SwitchMode(b_req_i); every worker m starts from the trainer's model
 *      (x_m <- x_Ti), then runs `inner_steps` inner steps.  Each inner step takes accum
 *      micro-batches of b_micro samples: batch_fn -> adloco_grad_stats (ADLOCO_ACCUMULATE from
 *      the second micro-batch on: Algorithm 3's "g <- g + grad L") -> adloco_inner_step with
 *      g = grad / (accum * b_micro).  After the first inner step of worker 0 the norm test gives the
 *      trainer's requested batch for the NEXT outer step ("store b_req for the next outer step"):
 *      adloco_norm_test with b_cur = accum * b_micro, the samples the statistics come from (eq. 4
 *      compares with the size of the batch at hand, which SwitchMode may have cut to b_max), then
 *      b_req_i <- max(b_req_i, result) so that the request never shrinks.  Every other batch of the
 *      outer step only needs its gradient sum (ADLOCO_SUM_ONLY).
 *   3. per trainer: Delta = (1/M) sum_m (x_Ti - x_m), x_Ti <- OuterOpt(x_Ti, Delta)
 *      (adloco_outer_step).
 * Readings of the listing: the switch decision is per trainer; the accumulate branch also runs
 * `inner_steps` inner steps, each over its accumulated micro-batches; CheckMerge runs in every
 * call (a merge cadence is the caller's: pass merge_w = 0 to skip).
 * ------------------------------------------------------------------------------------ */
typedef struct {
  float*  theta;        /* device [N] fp32: worker parameters x_m (overwritten from the trainer) */
  float*  exp_avg;      /* device [N] fp32: AdamW first moment, carried across rounds            */
  float*  exp_avg_sq;   /* device [N] fp32: AdamW second moment                                   */
  float*  grad;         /* device [N] fp32: the grad_sum buffers of the layer list, back to back,
                           in list order (layer l at grad + sum of the sizes before it)          */
  int64_t step;         /* inner steps done so far (bias correction); in/out                      */
} adloco_worker;

typedef struct {
  float*            theta_outer;        /* device [N] fp32: x_Ti, in/out                        */
  float*            momentum;           /* device [N] fp32: OuterOpt momentum (NULL iff mu = 0) */
  adloco_worker*    workers;            /* host array of n_workers workers                      */
  int32_t           n_workers;          /* 1 .. ADLOCO_MAX_INSTANCES                            */
  int32_t           reserved;           /* 0                                                    */
  int64_t           b_req;              /* requested batch, in/out                              */
  adloco_stats_acc* acc;                /* device accumulator (16 bytes)                        */
  float*            per_sample_sqnorm;  /* device [b_max] fp32 scratch for the per-sample norms */
  void*             user;               /* handed to batch_fn                                   */
} adloco_trainer;

typedef struct {
  int32_t T;             /* tokens per sample                                                  */
  int32_t dtype;         /* ADLOCO_F32 / ADLOCO_BF16 / ADLOCO_F16 of every a, delta            */
  int32_t inner_steps;   /* H >= 1                                                             */
  int32_t n_switch;      /* SwitchMode multiplier n (the paper uses 2)                         */
  int32_t merge_w;       /* w of CheckMerge; 0: no merging in this call                        */
  int32_t nesterov;      /* OuterOpt: 1 Nesterov momentum, 0 heavy ball                        */
  int64_t b_max;         /* micro-batch (memory) cap                                           */
  int64_t b_cap;         /* ceiling on b_req, 0 = none                                         */
  double  eta;           /* norm test                                                          */
  double  lr_inner, beta1, beta2, eps, weight_decay;   /* InnerOpt = AdamW                     */
  double  lr_outer, mu_outer;                          /* OuterOpt                             */
} adloco_round_config;

/* Runs the model of worker `worker` of the trainer that owns `user` at parameters `theta`
 * (device) on `b` fresh samples and describes the result: on entry layers[l] holds d_in, d_out,
 * grad_sum, flags of the template; the callback fills a, delta and the row strides (device
 * tensors [b, T, .] that stay valid until the next callback for this trainer), and for blocks
 * with ADLOCO_GRAD_PROVIDED maintains grad_sum itself: it STORES its gradient sum there when
 * micro_step is 0 (the driver does not clear such blocks between inner steps) and adds to it when
 * micro_step > 0.  Device work of the callback
 * must be ordered before later work on `stream`.  Return 0, or non-zero to abort the round. */
typedef int (*adloco_batch_fn)(void* user, int32_t worker, int32_t inner_step, int32_t micro_step,
                               int64_t b, const float* theta, adloco_linear_desc* layers,
                               int32_t n_layers, void* stream);

typedef struct {
  int64_t b_req_used;    /* the requested batch this round ran with                             */
  int64_t b_micro;       /* SwitchMode: micro-batch size                                        */
  int64_t accum_steps;   /* SwitchMode: micro-batches per inner step                            */
  int32_t accumulate;    /* SwitchMode: 1 iff gradient accumulation was on                      */
  int32_t merged_from;   /* number of trainers merged into this one in step 1 (0: none)         */
  adloco_norm_test_result test;   /* the norm test that produced the new b_req                  */
} adloco_round_report;

/*   trainers   host array of *k trainers, reordered in place when a merge happens
 *   k          in: number of trainers (>= 1); out: number left
 *   layers     host template of n_layers descriptors: d_in, d_out, flags (a, delta, grad_sum
 *              ignored); the blocks' sizes must add up to N
 *   reports    host [k_in] or NULL; reports[i] belongs to trainers[i] after the call
 * Returns ADLOCO_ESTATE when batch_fn fails. */
int adloco_round(adloco_ctx* ctx, const adloco_round_config* cfg, adloco_trainer* trainers, int* k,
                 const adloco_linear_desc* layers, int n_layers, size_t N, adloco_batch_fn batch_fn,
                 adloco_round_report* reports, void* stream);

/* Library version (major*10000 + minor*100 + patch). */
int adloco_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ADLOCO_H */
