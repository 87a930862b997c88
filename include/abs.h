/*
 * abs.h -- C ABI of the adaptive-batch-size local-gradient hot path for MI355X (gfx950).
 *
 * M worker replicas of one MLP live side by side in device memory.  Each call of
 * abs_local_step() makes every replica take one local optimizer step on its own
 * mini-batch and leaves behind the statistics that the batch-size tests need;
 * abs_average_replicas() is the model average that ends a communication round.
 * The operations are those of the paper "Communication-Efficient Adaptive Batch Size
 * Strategies for Distributed Local Gradient Methods" (Lau, Li, Xu, Liu, Kolar):
 * its Sec. 3 (problem, Local SGD), Sec. 4 (norm test, batch-size rule) and Alg. 1 / Alg. 2
 * of its appendix "Main Algorithm".  All M workers are simulated on one GPU; the average
 * is an in-device mean, not a collective.
 *
 * Conventions
 *  - Every function returns an abs_status and never throws or aborts across the ABI.
 *    On error, out-parameters are left untouched and abs_last_error() describes it.
 *  - "host" / "device" on a pointer says where the memory lives.  The caller owns every
 *    buffer it passes in (dataset, labels, indices, workspace, stream); the library
 *    borrows the device pointers for the lifetime of the context and owns only the
 *    abs_ctx object (plus a few hundred bytes of pinned host memory for the read-back of
 *    the statistics).  The library allocates no device memory: all of it is carved from
 *    the caller's workspace (abs_workspace_bytes says how much).
 *  - abs_local_step and abs_average_replicas are asynchronous on the context's stream.
 *    The *_test calls return once the statistics of the most recent step have reached the host; the
 *    statistics are the step's last launch, so every kernel of that step has finished by then (work
 *    enqueued after the step, e.g. an average, may still be running).  The get/set calls synchronise
 *    the stream.
 *  - One context per host thread and stream; calls on one context are not re-entrant.
 *  - Parameter vector layout (x0, get/set_params, get_grad): layer-major; for each layer
 *    the weight W_l row-major [out_l x in_l], then (if has_bias) the bias [out_l].
 *  - Per-sample loss is softmax cross-entropy of the last layer's outputs (natural log);
 *    the backprop signals are those of the per-sample loss, not divided by the batch size.
 */
#ifndef ABS_H_
#define ABS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct abs_ctx abs_ctx;

typedef enum {
  ABS_OK = 0,
  ABS_EINVAL = 1,       /* bad argument (range, NULL, alignment) */
  ABS_ENOMEM = 2,       /* workspace (or one of its pieces) too small; host allocation failed */
  ABS_ESTATE = 3,       /* call out of order (e.g. a test before any local step) */
  ABS_EHIP = 4,         /* a HIP runtime call failed (or an unexpected internal error) */
  ABS_EUNSUPPORTED = 5  /* shape the kernels do not cover */
} abs_status;

enum { ABS_ACT_NONE = 0, ABS_ACT_RELU = 1, ABS_ACT_GELU = 2 };   /* GELU: exact erf form */
enum { ABS_OPT_SGD = 0, ABS_OPT_SHB = 1, ABS_OPT_ADAMW = 2,   /* Adam = AdamW with weight_decay 0 */
       ABS_OPT_ADAGRAD = 3 };                                   /* v <- v + g^2 ; x <- x - lr g / (sqrt v + eps) */
enum { ABS_PREC_F32 = 0,    /* fp32 operands and accumulation */
       ABS_PREC_BF16 = 1 }; /* bf16 operands, fp32 accumulation, fp32 master weights */
enum { ABS_STATS_NORM = 1,  /* sum_i ||g_i||^2 and ||gbar||^2 (norm test) */
       ABS_STATS_IP = 2 };  /* also sum_i <g_i,gbar> and its square (inner-product tests) */

typedef struct {
  int n_layers;            /* L >= 1 linear layers */
  const int *dims;         /* host, L+1 entries: dims[0] inputs ... dims[L] classes.
                              In ABS_PREC_BF16 dims[0..L-1] must be multiples of 8. */
  int act;                 /* ABS_ACT_* applied after every layer but the last */
  int has_bias;
  int prec;                /* ABS_PREC_* */
  int M;                   /* number of worker replicas, >= 1 */
  int b_cap;               /* largest local batch size any call will use, >= 2 */
  int opt;                 /* ABS_OPT_* : the inner optimizer ("or other inner optimizers", Alg. 1) */
  float momentum;          /* SHB:  v <- momentum v + g ; x <- x - lr v */
  float beta1, beta2, eps, weight_decay;  /* AdamW, decoupled decay, bias-corrected moments */
  int stats_mask;          /* ABS_STATS_* bits gathered by every local step */
  void *hip_stream;        /* hipStream_t of the caller (NULL = the null stream) */
  void *workspace;         /* device, 256-byte aligned, caller-allocated */
  size_t workspace_bytes;
} abs_config;

/* One worker's statistics and test outcome for the most recent local step. */
typedef struct {
  int b;                   /* local batch size the statistics were gathered on */
  double sum_sq;           /* S1 = sum_i ||g_i||^2 over the batch (per-sample gradients) */
  double gbar_sq;          /* S2 = ||gbar||^2, gbar = local batch gradient, eq. (batch_grad) */
  double sum_q;            /* S4 = sum_i <g_i, gbar>            (0 unless ABS_STATS_IP) */
  double sum_q2;           /* S3 = sum_i <g_i, gbar>^2          (0 unless ABS_STATS_IP) */
  double loss_sum;         /* sum_i f_i over the batch */
  double var;              /* batch variance of the tested quantity, eq. (def_var) */
  double var_perp;         /* variance of the components orthogonal to gbar (augmented test) */
  double lhs, rhs;         /* the two sides of the tested inequality */
  double ratio;            /* the quantity whose ceiling is T */
  long long T;             /* test statistic, Alg. 1: ceil(ratio) */
  int pass;                /* 1 if the condition holds (batch size need not grow) */
} abs_test_result;

/* Device bytes abs_init_replicas needs in cfg->workspace for a dataset of N samples. */
abs_status abs_workspace_bytes(const abs_config *cfg, int64_t N, size_t *bytes /*host*/);

/*
 * Create the M replicas, all equal to x0 (Alg. 1, "initial model parameters x_{0,0}^m = x_0").
 *   x0_host : host, n_params floats in the layout above.
 *   X_dev   : device, float [N x dims[0]] row-major, the (shared, i.i.d.) training set.
 *   y_dev   : device, int32 [N] labels in [0, dims[L]).
 * Both stay borrowed until abs_destroy.  Optimizer state starts at zero.
 */
abs_status abs_init_replicas(const abs_config *cfg, const float *x0_host, const float *X_dev,
                             const int32_t *y_dev, int64_t N, abs_ctx **out /*host*/);

/*
 * One local step of all M workers (the body of Alg. 1's inner loop): gather the batch,
 * forward, per-sample backprop signals, the local batch gradient of eq. (batch_grad), the
 * statistics selected by stats_mask, then the optimizer update with learning rate lr.
 * The statistics refer to the gradient at the iterate *before* the update.
 *   idx_dev : device, int32 [M x b], row m = the sample indices of worker m's batch
 *             ("sample the local batch uniformly", with replacement; drawn by the caller).
 *   b       : local batch size, the same for every worker (the paper's practical rule gives
 *             all workers the maximum), 2 <= b <= b_cap.
 * Per-sample gradients are never formed: ||g_i||^2 = sum_l ||delta_i^l||^2 (||a_i^{l-1}||^2 + 1)
 * and <g_i,gbar> = sum_l delta_i^l . (Gbar_l a_i^{l-1} + betabar_l).
 */
abs_status abs_local_step(abs_ctx *ctx, const int32_t *idx_dev, int b, float lr);

/*
 * abs_local_step for callers that repeat a batch size (for those that cannot afford the launch overhead of
 * some forty kernels per step: small models, small batches).  The first step at a given b runs directly, the
 * second is captured into a HIP graph, later ones replay it; one small launch in front of the graph carries
 * idx_dev, lr and the optimizer's step-dependent scalars into fixed device locations.  Results are bitwise
 * those of abs_local_step.  Graphs of up to 8 batch sizes are kept (least recently used dropped).  Steps are
 * run directly, without capture, while abs_profile_enable is on or when the context uses the legacy default
 * stream (stream capture needs a created stream); abs_graph_count tells how many graphs exist.
 */
abs_status abs_local_step_graphed(abs_ctx *ctx, const int32_t *idx_dev, int b, float lr);
abs_status abs_graph_count(const abs_ctx *ctx, int *n /*host*/);

/*
 * The same step as abs_local_step, with the batch of b samples processed in micro-batches of
 * micro_b <= b_cap samples ("gradient accumulation", Sec. 6, for batches whose activations do
 * not fit): b may exceed b_cap.  The gradient, S1 and the loss accumulate over the micro-batches
 * and S2 is taken from the finished gradient; the inner products <g_i, gbar> need the gradient
 * of the whole batch, so with ABS_STATS_IP the forward and backward passes run a second time.
 * One optimizer update follows.  The result equals abs_local_step on the whole batch up to the
 * order of floating-point additions.
 *   idx_dev : device, int32 [M x b] (row stride b).   b % micro_b must not be 1.
 * abs_get_per_sample afterwards returns the values of the micro-batches that lie wholly inside
 * the first b_cap samples (all of them when b <= b_cap).
 */
abs_status abs_local_step_accumulated(abs_ctx *ctx, const int32_t *idx_dev, int b, int micro_b, float lr);

/*
 * The same step with one local batch size per worker (eq. (test_stat) gives each worker its own
 * b^m before the practical rule takes their maximum; Sec. 3 allows heterogeneous workers).
 *   idx_dev : device, int32 [M x ldi]; worker m uses the first b_host[m] entries of row m.
 *   b_host  : host, M entries, each in [2, b_cap]; ldi >= max_m b_host[m].  The array is copied
 *             during the call and may be reused at once.
 * Worker m's batch gradient is the mean over its own b^m samples and its statistics are taken
 * over those samples only.  abs_cross_worker_test refuses a ragged step (Alg. 2 assumes equal b).
 */
abs_status abs_local_step_ragged(abs_ctx *ctx, const int32_t *idx_dev, int ldi, const int *b_host /*host*/,
                                 float lr);

/*
 * Approximate local norm test, eqs. (approx_norm_local) and (test_stat), per worker:
 *   Var = (S1 - b S2)/(b-1)  [eq. (def_var)],  condition Var/b <= eta^2 S2,
 *   T = ceil(Var / (eta^2 S2)).   0 < eta < 1.   A zero batch gradient gives T = b, pass = 1.
 *   out : host, M entries.
 */
abs_status abs_norm_test(abs_ctx *ctx, double eta, abs_test_result *out);

/* The same test with one constant per worker (eta^m of eq. (approx_norm_local)); eta: host, M entries. */
abs_status abs_norm_test_per_worker(abs_ctx *ctx, const double *eta /*host*/, abs_test_result *out);

/*
 * The same test with the finite-population factor of Sec. 4.1's estimate of delta_B^2 (a batch
 * of b drawn from n samples without replacement): Var is multiplied by (n - b)/(n - 1), taken
 * at the current b, before the comparison and the ceiling.  n_total >= b, n_total >= 2.
 * n_total == b gives Var = 0 (the batch is the whole population), so the rule keeps b.
 */
abs_status abs_norm_test_fpc(abs_ctx *ctx, double eta, int64_t n_total, abs_test_result *out);

/*
 * Inner-product test of the adaptive-sampling literature the paper cites (named at the end
 * of its Sec. 4.1), applied per worker to its own batch:
 *   Var_q = sample variance of q_i = <g_i,gbar>;  condition Var_q/b <= theta^2 S2^2;
 *   T_ip = ceil(Var_q / (theta^2 S2^2)).
 * With nu > 0 (augmented test) also Var_perp = (S1 - S3/S2)/(b-1), condition
 * Var_perp/b <= nu^2 S2, and T = max(T_ip, ceil(Var_perp/(nu^2 S2))).  nu <= 0: plain test.
 * Needs ABS_STATS_IP in stats_mask.   out : host, M entries.
 */
abs_status abs_inner_product_test(abs_ctx *ctx, double theta, double nu, abs_test_result *out);

/*
 * Once-per-round norm test of Alg. 2 from the M local batch gradients of the most recent
 * local step: Var = b/(M-1) sum_m ||g^m - gbar||^2, T = ceil(Var / (M eta^2 ||gbar||^2)),
 * gbar the mean over workers.  Needs M >= 2.  out : host, ONE entry (sum_sq = sum_m ||g^m||^2,
 * gbar_sq = ||gbar||^2).
 */
abs_status abs_cross_worker_test(abs_ctx *ctx, double eta, abs_test_result *out);

/*
 * Batch-size rule, pure host function: b_next^m = min(b_cap, max(T^m, b_cur^m)) (Alg. 1);
 * with sync_max != 0 every worker gets the maximum over workers (display after eq. test_stat).
 *   res, b_cur, b_next : host, M entries each.
 */
abs_status abs_next_batch_size(const abs_test_result *res, int M, const int *b_cur, int b_cap,
                               int sync_max, int *b_next);

/* Model average that ends a round, eq. (local_sgd_alt): x^m <- (1/M) sum_m x^m for all m.
 * Only the parameters are averaged; optimizer state stays local. */
abs_status abs_average_replicas(abs_ctx *ctx);

/*
 * Where the optimizer step of the weights is applied (ABS_PREC_BF16; on by default): inside the epilogue of the
 * weight-gradient contraction (Alg. 1's "local step" fused into "compute the local batch gradient"), instead of
 * storing the fp32 gradient and streaming it through a separate update.  At small local batch sizes, where a step is
 * bound by the bytes moved per parameter, this removes 8 of 26 bytes per parameter (heavy ball).  ||gbar||^2 is then
 * summed from per-wavefront partial sums left by the epilogues, and the statistics, tests and parameters are those of
 * the separate update up to the order of the additions in ||gbar||^2 (parameters: bit for bit).  The fp32 gradient of
 * the weights is not stored by such a step; abs_get_grad and abs_cross_worker_test form it on demand from the layer
 * inputs and backprop signals the step left in the workspace (the same contractions with a plain epilogue: the very
 * entries the step applied), which costs one more pass of the weight-gradient contractions.  A caller that reads the
 * gradient after every step (Alg. 2 with H = 1) may prefer on = 0.  A layer whose weight gradient splits its
 * reduction over the batch (few output tiles, long batches) takes its step in the launch that adds the slices;
 * abs_local_step_accumulated, which keeps the gradient in memory between micro-batches, always updates separately,
 * as does a net with a layer width that is no multiple of 4.  on != 0 with ABS_PREC_F32: ABS_EUNSUPPORTED.
 */
abs_status abs_set_fused_update(abs_ctx *ctx, int on);

/*
 * How the inner products q_i = <g_i, gbar> of the inner-product test are formed (ABS_PREC_BF16 with ABS_STATS_IP;
 * ignored otherwise).  Steps with b <= b_max (every worker's b^m for a ragged step) use
 *   <g_i, g_j> = sum_l (delta_i^l . delta_j^l)(a_i^{l-1} . a_j^{l-1} + [bias]),   q_i = (1/b) sum_j <g_i, g_j>,
 * i.e. the b x b Gram matrices of the layer inputs and backprop signals (the per-sample gradient of a layer is the
 * outer product delta_i a_i^T), which reads b (in + out) values per layer instead of every parameter; longer
 * batches contract the stored bf16 copy of Gbar with the activations (cost linear in b).  Both are the same sum
 * in exact arithmetic.  In the Gram form Gbar is never rounded to bf16 on its way into the product, so q_i differs
 * from the other form's by that rounding (relative 2^-9 per entry of Gbar, far less in the sums).
 * b_max in [0, 256]; 0 switches the Gram form off; the default is 256 (measured on config 3: the Gram form is the faster one for every b up to there).  abs_local_step_accumulated always uses the
 * contraction with Gbar.
 */
abs_status abs_set_gram_ip_max_batch(abs_ctx *ctx, int b_max);

/*
 * Counters of Alg. 1: rounds = k, the communication rounds completed (one per abs_average_replicas,
 * "k <- k + 1"); local_steps = optimizer steps taken by every worker; samples = B, the local batch
 * sizes actually used, summed over workers and local steps ("B <- B + sum_m sum_h b^m").
 * Host integers kept by the context; no GPU call, no synchronisation.  Any out pointer may be NULL.
 */
abs_status abs_get_counters(const abs_ctx *ctx, long long *rounds, long long *local_steps, long long *samples);

/* Parity helpers (synchronising).  m in [0, M); buffers are host, n_params floats. */
abs_status abs_get_params(abs_ctx *ctx, int m, float *out_host);
abs_status abs_set_params(abs_ctx *ctx, int m, const float *in_host);
abs_status abs_get_grad(abs_ctx *ctx, int m, float *out_host);    /* last local batch gradient */
/* Optimizer state of worker m (local to a worker, never averaged: "synchronizing only the models", Sec. 6):
 * which = 0: heavy-ball buffer v / AdamW second moment / AdaGrad accumulator; which = 1: AdamW first moment. */
abs_status abs_get_opt_state(abs_ctx *ctx, int m, int which, float *out_host);
/* Per-sample ||g_i||^2 (and <g_i,gbar> if gathered; else q_host may be NULL) of worker m
 * for the most recent step: host, b floats each (b^m after a ragged step; see
 * abs_local_step_accumulated for what an accumulated step keeps). */
abs_status abs_get_per_sample(abs_ctx *ctx, int m, float *n_host, float *q_host);

/* Linear scaling of the learning rate with the batch size (Sec. 6.1): lr_ref * b / b_ref. */
abs_status abs_lr_linear_scaling(double lr_ref, int64_t b, int64_t b_ref, double *lr /*host*/);

/* Learning-rate schedule of the paper's experiments (Sec. 6.1): linear warm-up to `peak` over the
 * first warmup_steps local steps (lr = peak (step+1)/warmup_steps), then cosine decay to `floor`,
 * reached at total_steps.  Pure host function; abs_local_step takes the rate per call. */
abs_status abs_lr_schedule(long long step, long long total_steps, long long warmup_steps, double peak,
                           double floor, double *lr /*host*/);

/* Number of parameters of cfg's network (host only, no GPU call). */
abs_status abs_n_params(const abs_config *cfg, int64_t *n /*host*/);

/*
 * Statistics and averaging alone, on caller-supplied layer inputs and backprop signals
 * (no model run): for each of M replicas and L stacked linear layers without bias,
 *   a_dev[l]     : device, bf16 [M x b x in_l],  delta_dev[l] : device, bf16 [M x b x out_l]
 * computes Gbar_l = delta^T a / b (fp32, into workspace), n_i, S1, S2, q_i, S3, S4 with the
 * same kernels as abs_local_step.   out : host, M entries (b, sum_sq, gbar_sq, sum_q, sum_q2).
 *   n_out_dev, q_out_dev : device, float [M x b] (either may be NULL).
 *   gbar_out_dev : device, float, sum_l out_l*in_l per replica, replica-major (may be NULL).
 */
abs_status abs_layer_stats(int L, const int *in_dims, const int *out_dims, int M, int b,
                           const void *const *a_dev, const void *const *delta_dev,
                           void *workspace, size_t workspace_bytes, void *hip_stream,
                           abs_test_result *out, float *n_out_dev, float *q_out_dev,
                           float *gbar_out_dev);
abs_status abs_layer_stats_workspace_bytes(int L, const int *in_dims, const int *out_dims,
                                           int M, int b, size_t *bytes);

/* Mean over M replicas of a bf16 parameter block, written back to all M (fp32 sum in
 * replica order, one rounding):  params_dev : device, bf16 [M x n]; n multiple of 8.
 * scratch_dev : device, n bf16 values, 16-byte aligned, caller-owned, or NULL.  With a scratch buffer a
 * large block is averaged in two passes (read all replicas, then write all replicas); the result is the
 * same bit for bit, HBM serves the two pure streams faster than their mixture. */
abs_status abs_average_bf16(void *params_dev, int M, int64_t n, void *scratch_dev, void *hip_stream);

/*
 * abs_average_bf16 for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the mean buffer of the two-pass form is a 32 MiB array that is part of
 * the library's code object (each GPU the library runs on holds it until the process ends), so the call
 * allocates nothing and takes no scratch pointer.  Same kernels, same result bit for bit as abs_average_bf16
 * with a scratch buffer.   n <= 16 Mi (16 777 216) bf16 values per replica, else ABS_EINVAL.
 * All calls on one GPU share that GPU's buffer: calls that overlap on one GPU (different streams or host
 * threads) race; calls on one stream are ordered and safe.  The buffer's address is resolved on the first call
 * on a device (make that call outside any stream capture).
 */
abs_status abs_average_bf16_static(void *params_dev, int M, int64_t n, void *hip_stream);

/*
 * Per-kernel timing (measurement aid; not part of the method).  While enabled, every kernel
 * launch of abs_local_step / abs_average_replicas is bracketed by two HIP events on the
 * context's stream.  abs_profile_read synchronises, folds the elapsed times into per-kernel
 * totals (accumulated since abs_profile_enable) and returns one entry per kernel class that ran:
 * calls, total milliseconds, and the algorithmic work of those calls (flops for the matrix-core
 * GEMMs: 2 m n k per replica, with the largest b^m for every replica after a ragged step; bytes
 * for the bandwidth-bound kernels).   out : host.
 */
typedef struct {
  char name[32];
  long long calls;
  double total_ms, flops, bytes;
} abs_profile_entry;
abs_status abs_profile_enable(abs_ctx *ctx, int on);
abs_status abs_profile_read(abs_ctx *ctx, int max_entries, abs_profile_entry *out, int *n_entries);
/* Suspend (paused != 0) or resume the bracketing without synchronising and without clearing the totals, so
 * that a caller can sample some steps of a timed run and leave the others unperturbed (two events per
 * launch cost a few microseconds, which matters when a whole step takes a few hundred). */
abs_status abs_profile_pause(abs_ctx *ctx, int paused);

/* Plain device-to-device copy kernel (one 16-byte vector per thread), bytes a multiple of 16,
 * both pointers 16-byte aligned.  It moves a known number of bytes, so its hardware-counter
 * readings are the reference that the counters of the other kernels are scaled by. */
abs_status abs_copy_probe(const void *src_dev, void *dst_dev, int64_t bytes, void *hip_stream);

abs_status abs_destroy(abs_ctx *ctx);
const char *abs_last_error(const abs_ctx *ctx);   /* ctx may be NULL: last error of this thread */

#ifdef __cplusplus
}
#endif
#endif /* ABS_H_ */
