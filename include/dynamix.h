/*
 * dynamix.h -- C ABI of the per-step gradient aggregate + statistics path on one MI355X.
 *
 * Setting (paper: Background, "Distributed machine learning systems"; Problem Formulation,
 * "Action space and batch size adjustment"; Algorithm 1, the gradient-and-model-update step and the
 * metric-collection step of a training iteration): K bulk-synchronous data-parallel
 * workers hold a full model replica each, worker k computes its gradient g_k on a batch of its
 * own size b_k (an integer the agent moves inside [32, 1024]), and at the barrier the gradients
 * are combined.  The agent's state carries gradient statistics (Problem Formulation, "Training
 * Statistical Efficiency Metrics": sigma_norm, sigma_norm^2; reward term
 * -eta (sigma_norm^2 + sigma_norm)).  The paper prints no formula for the combination or the
 * statistics; this library uses the mean over the global batch and the standard estimators:
 *
 *   B = sum_k b_k            G_i = (sum_k b_k g_ki) / B
 *   n_k = sum_i g_ki^2       A = sum_i G_i^2       d_k = sum_i (g_ki - G_i)^2
 *   T = (sum_k b_k d_k)/(K-1)   (0 when K == 1; unbiased trace of the per-example covariance)
 *
 * One call makes a single streaming pass over the K gradient buffers and produces G and one
 * statistics record for the whole vector plus one per caller-defined contiguous segment
 * (layer).  Everything runs in HIP kernels enqueued on the caller's stream; the call never
 * synchronises the device or the stream.
 *
 * Plain C: no C++ types and no exceptions cross this boundary.
 */
#ifndef DYNAMIX_H
#define DYNAMIX_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Storage type of the gradient buffers.  Every stored value is widened exactly (fp16
 * subnormals included); accumulation is fp32 per lane and fp64 across blocks for all three; the
 * aggregate is always written as fp32.
 * Non-finite inputs propagate per IEEE 754 and are not trapped: an Inf or NaN in worker k's
 * buffer makes worker_sqnorm[k] (and only that worker's) non-finite, which serves as the
 * overflow flag of loss-scaled fp16 training; the aggregate, its norm and all deviations are
 * then non-finite too in the records that cover the element. */
typedef enum { DYNAMIX_F32 = 0, DYNAMIX_BF16 = 1, DYNAMIX_F16 = 2 } dynamix_dtype;

typedef enum {
    DYNAMIX_OK = 0,
    DYNAMIX_ERR_NULL = 1,     /* a required pointer (or one of the K gradient pointers) is NULL */
    DYNAMIX_ERR_ARG = 2,      /* K < 1, K > DYNAMIX_K_MAX, P < 1, a batch size <= 0, bad dtype */
    DYNAMIX_ERR_SEGMENTS = 3, /* offsets do not start at 0, are not strictly increasing, or do not end at P */
    DYNAMIX_ERR_ALIGN = 4,    /* a gradient pointer or out_agg is not 16-byte aligned, or out_stats not 8-byte */
    DYNAMIX_ERR_NOMEM = 5,    /* the library could not allocate its workspace */
    DYNAMIX_ERR_HIP = 6,      /* a HIP runtime call failed (launch, copy, device query) */
    DYNAMIX_ERR_CAPACITY = 7  /* dynamix_grad_aggregate_stats_static: the shape needs more than
                                 DYNAMIX_STATIC_SCRATCH_BYTES of workspace */
} dynamix_status;

enum { DYNAMIX_K_MAX = 256 };       /* most workers per call: pointers and weights travel in the kernel arguments */
enum { DYNAMIX_K_MAX_ONE_SWEEP = 64 }; /* up to here every gradient byte is read once; above, twice (see below) */
enum { DYNAMIX_K_MAX_STATEFUL = 32 }; /* most workers for the fused updates that carry optimizer state */
enum { DYNAMIX_STATIC_SCRATCH_BYTES = 4 << 20 }; /* workspace of dynamix_grad_aggregate_stats_static */
enum { DYNAMIX_STATS_HEAD = 8 };    /* scalars in front of the per-worker entries of a record */

/* Positions inside one statistics record of DYNAMIX_STATS_HEAD + 2K doubles. */
enum {
    DYNAMIX_STAT_AGG_SQNORM = 0,          /* A = sum_i G_i^2 */
    DYNAMIX_STAT_TR_SIGMA = 1,            /* T */
    DYNAMIX_STAT_AGG_SQNORM_UNBIASED = 2, /* A - T/B, unbiased |E g|^2 */
    DYNAMIX_STAT_NOISE_SCALE = 3,         /* T / (A - T/B); IEEE division, never clamped */
    DYNAMIX_STAT_NOISE_SCALE_BIASED = 4,  /* T / A */
    DYNAMIX_STAT_SIGMA2_NORM = 5,         /* T / (B A): variance of G over its squared norm */
    DYNAMIX_STAT_SIGMA_NORM = 6,          /* sqrt(max(0, sigma2_norm)) */
    DYNAMIX_STAT_COUNT = 7                /* elements covered by the record */
    /* [8 .. 8+K)     worker_sqnorm[k]     = n_k
       [8+K .. 8+2K)  worker_dev_sqnorm[k] = d_k */
};

/*
 * Weighted aggregation of K workers' gradients fused with the statistics above
 * (Algorithm 1: gradient synchronisation and metric collection of one training iteration).
 *
 * grads            HOST array of K DEVICE pointers.  grads[k] holds P elements of `dtype`,
 *                  contiguous, 16-byte aligned, read-only for the call, owned by the caller.
 *                  The K buffers are independent allocations; none may overlap out_agg.
 *                  (Speed only: with 8 to 32 workers the kernel reads interleaved 256-byte
 *                  chunks, which keeps equally placed buffers, e.g. allocations a multiple of
 *                  16 MB apart, from meeting in the same memory channels; it does so when every
 *                  gradient buffer and the output start on 256-byte boundaries, and falls back to
 *                  consecutive 4 KB tiles, up to 8 % slower for such placements, when one does
 *                  not.)
 * batch_sizes      HOST array of K per-worker batch sizes b_k, each > 0.
 * K, P             number of workers (1..DYNAMIX_K_MAX) and elements per gradient (>= 1).
 *                  Up to DYNAMIX_K_MAX_ONE_SWEEP workers the K values of an element stay in
 *                  registers until its aggregate is known and every gradient byte is read from
 *                  memory once.  Above, they do not fit: the kernel then sweeps the gradients
 *                  twice, 32 block iterations at a time (first G and its norm, G parked on chip
 *                  and written in one burst; then n_k and d_k, sixteen workers at a time), and
 *                  the memory traffic is 2 K P sizeof(dtype) read + 4 P written.  Same results,
 *                  same reproducibility; the fused model updates are not available there
 *                  (DYNAMIX_ERR_ARG).
 * dtype            a dynamix_dtype.
 * segment_offsets  HOST array, or NULL.  NULL: one record for [0, P) only.  Otherwise strictly
 *                  increasing element offsets that start at 0; the array ends at the first
 *                  entry equal to P (S+1 entries for S segments; segments need no alignment).
 * out_agg          DEVICE, P floats, 16-byte aligned, caller-owned; receives G.  NULL skips
 *                  the write (statistics only).
 * out_stats        DEVICE, dynamix_stats_count(K, S) doubles, caller-owned.  Record 0 covers
 *                  [0, P); records 1..S the segments (present only with segment_offsets).
 * stream           a hipStream_t passed as void*; NULL is the default stream.
 *
 * Host arrays are consumed before the call returns.  Arguments are validated before the first
 * HIP call; on any error nothing is enqueued and a dynamix_status other than DYNAMIX_OK is
 * returned.  Results are valid once the caller has synchronised `stream`.  The first call with
 * a shape on a stream also allocates and uploads the plan; every later one only launches
 * kernels.  A call may be recorded into a HIP graph (stream capture): it then carries the upload
 * of its tables with it, as a few small kernels, so the graph is complete in itself.  The
 * allocation of a first call is not graph material: make one call with the shape before the
 * capture, or use dynamix_grad_aggregate_stats_static.  A recorded call refers to the library's
 * workspace for its shape: dynamix_release_cached(), or 128 other shapes used since, free it, and
 * a graph that holds such a call must not be replayed afterwards.  Non-finite inputs
 * propagate by IEEE rules.  The library keeps a small workspace per (device, stream, shape),
 * allocated on the first call with that shape and reused afterwards; two calls that share it
 * must be ordered on that stream.  For fixed inputs, shape and device the results are bitwise
 * reproducible (fixed-order reductions, no atomics); the order of the sums, not the aggregate,
 * depends on whether all buffers start on 256-byte boundaries.
 */
int dynamix_grad_aggregate_stats(const void* const* grads, const int32_t* batch_sizes,
                                 int32_t K, int64_t P, int32_t dtype,
                                 const int64_t* segment_offsets, float* out_agg,
                                 double* out_stats, void* stream);

/* Same operation with the number of segments given explicitly: segment_offsets holds
 * num_segments + 1 entries (num_segments == 0 requires segment_offsets == NULL). */
int dynamix_grad_aggregate_stats_ex(const void* const* grads, const int32_t* batch_sizes,
                                    int32_t K, int64_t P, int32_t dtype,
                                    const int64_t* segment_offsets, int64_t num_segments,
                                    float* out_agg, double* out_stats, void* stream);

/*
 * dynamix_grad_aggregate_stats_ex for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same
 * kernels, same results bit for bit, but the library's workspace (plan tables, tail counter,
 * partial sums) lies in a static device array of DYNAMIX_STATIC_SCRATCH_BYTES (4 MiB, held by every
 * GPU the library runs on until the process ends) instead of an allocation per shape.  The call
 * makes no hipMalloc, hipFree or other allocating call, not even the first time: the tables reach
 * the device in kernel arguments, on `stream`.  Returns DYNAMIX_ERR_CAPACITY, before anything is
 * enqueued, when tables plus partial sums exceed the array: 48 bytes per piece of the work
 * decomposition (dynamix_plan_describe counts them; about 5 per block plus one per segment) plus
 * 8 (2K + 1) per piece for its partial sums plus 24 per segment; the paper-sized shapes need
 * 0.2 to 0.8 MiB, K = 64 with 3000 segments still fits.
 * All calls on one GPU share the one array, which keeps the tables of the last shape (a call
 * with the same shape as the one before only launches the two kernels; another shape is uploaded
 * in place): calls on the same GPU must not overlap, whatever their streams; the caller orders
 * them (one stream, or events).  That holds for replays of a graph the call was recorded into as
 * well; a recorded call uploads its tables at every replay, and from the first recording on
 * every call on that GPU does (the host can no longer know what a replay left in the array).
 * The caller still owns inputs and outputs.
 */
int dynamix_grad_aggregate_stats_static(const void* const* grads, const int32_t* batch_sizes,
                                        int32_t K, int64_t P, int32_t dtype,
                                        const int64_t* segment_offsets, int64_t num_segments,
                                        float* out_agg, double* out_stats, void* stream);

/*
 * The same pass with the model update fused in (Algorithm 1, the model-update half of its
 * gradient step): instead of writing G, the kernel applies plain stochastic gradient descent with
 * L2 weight decay in place,
 *     params[i] <- params[i] - lr * (G_i + weight_decay * params[i]),
 * which saves the write of G and the optimizer's later read of it.  params: DEVICE, P floats,
 * 16-byte aligned, read and written; it may not overlap any gradient buffer.  lr and weight_decay
 * are plain floats (NaN is an argument error).  Everything else, including out_stats, is as for
 * dynamix_grad_aggregate_stats_ex; the statistics are those of the gradients and do not depend
 * on params.  The update is evaluated in fp32 as fma(-lr, fma(weight_decay, p, G), p).
 */
int dynamix_grad_aggregate_stats_sgd(const void* const* grads, const int32_t* batch_sizes,
                                     int32_t K, int64_t P, int32_t dtype,
                                     const int64_t* segment_offsets, int64_t num_segments,
                                     float* params, float lr, float weight_decay,
                                     double* out_stats, void* stream);

/*
 * The pass with a model update that carries optimizer state fused in (Algorithm 1, the
 * model-update half of its gradient step; the paper trains with SGD and with Adam, "Evaluation",
 * experimental setup, and prints no update rule: the rules below are the published ones the common
 * frameworks implement).  The state vectors travel through the pass as further streams, read and
 * rewritten in place like params, so neither G nor the state makes an extra round trip through
 * HBM.  params and every state vector: DEVICE, P floats, 16-byte aligned, not overlapping each
 * other or any gradient buffer.  K <= DYNAMIX_K_MAX_STATEFUL (above, the K gradient vectors of a
 * lane and the state leave no registers; DYNAMIX_ERR_ARG; from 25 workers on the kernels load 8
 * bytes per lane instead of 16, which costs some read bandwidth).  Statistics, segments, stream,
 * validation and error behaviour as for dynamix_grad_aggregate_stats_ex; the statistics are those
 * of the gradients (these kernels take fewer vectors per block iteration, so the partial sums are
 * added in another order than in the plain call).  All arithmetic of the updates is fp32 (fused multiply-adds,
 * IEEE division and square root), constants that depend only on the scalars are formed once on the
 * host in double.
 *
 * dynamix_grad_aggregate_stats_sgd_momentum -- heavy-ball momentum, zero dampening:
 *     g = G_i + weight_decay p_i;   buf_i <- momentum buf_i + g;
 *     p_i <- p_i - lr (nesterov ? g + momentum buf_i : buf_i)
 * A zero momentum_buf makes the first step plain SGD.
 *
 * dynamix_grad_aggregate_stats_adam -- Adam with bias correction, step = t >= 1 (the caller
 * counts); 0 <= beta < 1:
 *     g = G_i + weight_decay p_i            (decoupled != 0: g = G_i and p_i <- p_i (1 - lr weight_decay) first)
 *     m_i <- beta1 m_i + (1 - beta1) g;     v_i <- beta2 v_i + (1 - beta2) g^2
 *     p_i <- p_i - lr (m_i / (1 - beta1^t)) / (sqrt(v_i / (1 - beta2^t)) + eps)
 */
int dynamix_grad_aggregate_stats_sgd_momentum(const void* const* grads, const int32_t* batch_sizes,
                                              int32_t K, int64_t P, int32_t dtype,
                                              const int64_t* segment_offsets, int64_t num_segments,
                                              float* params, float* momentum_buf, float lr,
                                              float weight_decay, float momentum, int32_t nesterov,
                                              double* out_stats, void* stream);
int dynamix_grad_aggregate_stats_adam(const void* const* grads, const int32_t* batch_sizes, int32_t K,
                                      int64_t P, int32_t dtype, const int64_t* segment_offsets,
                                      int64_t num_segments, float* params, float* exp_avg,
                                      float* exp_avg_sq, float lr, float beta1, float beta2, float eps,
                                      float weight_decay, int32_t decoupled, int64_t step,
                                      double* out_stats, void* stream);

/* Doubles needed for out_stats: (1 + S) * (DYNAMIX_STATS_HEAD + 2K); S = 0 without segments.
 * Returns -1 for K outside 1..DYNAMIX_K_MAX or S < 0. */
int64_t dynamix_stats_count(int32_t K, int64_t num_segments);

/*
 * Diagnostic, pure host arithmetic (no HIP call, usable without a GPU): the work decomposition
 * the library uses for this shape on a device that keeps `max_blocks` blocks resident.
 * The range of vectors (what a lane loads at a time: 16 bytes up to 32 workers, 8 up to 48, 4
 * above) is dealt to blocks as contiguous spans of equal cost and cut at segment boundaries into
 * pieces; each piece yields one partial statistics record.  Up to `capacity` pieces are written
 * to pieces_out as six int64 each: first vector, end vector, vectors per block iteration, first
 * element, end element (elements of the first and last vector outside this range belong to the
 * neighbouring segment and are masked), owning block.  Returns the number of pieces, or minus a
 * dynamix_status.
 */
int64_t dynamix_plan_describe(int32_t K, int64_t P, int32_t dtype, const int64_t* segment_offsets,
                              int64_t num_segments, int64_t max_blocks, int64_t* pieces_out,
                              int64_t capacity);

/* Static, NUL-terminated description of a dynamix_status value. */
const char* dynamix_status_string(int status);

/*
 * Aggregation over one adjustment cycle.  The paper's agent decides every k iterations on
 * metrics aggregated over those k iterations (System Architecture; Problem Formulation, "State
 * representation"), its state carries sigma_norm and sigma_norm^2, and its reward for adaptive
 * optimizers carries -eta (sigma_norm^2 + sigma_norm) and, for every worker, the batch size
 * regulariser -delta (log2 BatchSize - 5) ("Reward function design").  The paper does not say how
 * the k iterations are combined; this library takes the arithmetic mean of every entry of the
 * statistics record and, beside it, ratios formed from the mean sums.
 *
 * dynamix_cycle_accumulate: window[i] += stats[i] for i < count and window[count] += 1 (the
 * number of iterations in the window); with first != 0 the window is overwritten instead
 * (window := stats, counter := 1), which starts a cycle.  stats is the out_stats of an aggregate
 * call (DEVICE, count doubles); window is DEVICE, count + 1 doubles, caller-owned.
 *
 * dynamix_cycle_summary: for each of the 1 + S records (R = DYNAMIX_STATS_HEAD + 2K doubles in
 * the window, R + 4 in `summary`):
 *   [0, R)  mean over the accumulated iterations of every entry of the record
 *   [R+0]   pooled noise scale   mean(T) / (mean(A) - mean(T)/B)
 *   [R+1]   pooled sigma2_norm   mean(T) / (B mean(A))
 *   [R+2]   pooled sigma_norm    sqrt(max(0, [R+1]))
 *   [R+3]   optimizer penalty    -eta (mean(sigma2_norm) + mean(sigma_norm))
 * and after the last record K doubles, the regulariser -delta (log2 b_k - 5) of every worker.
 * summary: DEVICE, dynamix_cycle_summary_count(K, S) = (1+S)(R+4) + K doubles.  batch_sizes: HOST,
 * K entries > 0, constant over the cycle.  Both calls only enqueue work on `stream`, validate
 * before any HIP call and return a dynamix_status.
 */
int     dynamix_cycle_accumulate(const double* stats, int64_t count, double* window, int32_t first,
                                 void* stream);
int     dynamix_cycle_summary(const double* window, int32_t K, int64_t num_segments,
                              const int32_t* batch_sizes, double eta, double delta,
                              double* summary, void* stream);
int64_t dynamix_cycle_summary_count(int32_t K, int64_t num_segments);

/*
 * Host side of an adjustment cycle (no device work; every pointer below is a HOST pointer).
 * Every k iterations the paper's agent maps each worker's state to one of five batch size
 * adjustments with a policy whose parameters all workers share, pi_theta(a | s_i, s_global)
 * (Problem Formulation, "Reinforcement learning framework"), the batch size moves by that
 * amount and is clamped to [x_min, x_max] = [32, 1024] ("Action space and batch size adjustment";
 * Algorithm 1, the action and batch-size steps), and the reward is
 *     r = A_mean + alpha max(0, dA) - beta T_iter - delta (log2 b - 5)   [- eta (sigma2_norm + sigma_norm)
 *                                                                         with adaptive optimizers]
 * ("Reward function design").  The paper gives neither the network's shape nor any coefficient:
 * both are arguments.  The network here is a multi-layer perceptron with tanh between layers and
 * a softmax over the five actions; training it is outside this library.
 *
 * dynamix_policy_weight_count: floats a network with num_layers >= 2 layer sizes needs: for each
 *   pair of consecutive sizes (in, out) a row-major out x in matrix followed by out biases; -1
 *   for invalid sizes.
 * dynamix_policy_forward: states is K rows of layer_sizes[0] floats (a worker's local state
 *   followed by the global state); the last layer size must be DYNAMIX_NUM_ACTIONS; probs
 *   receives K rows of DYNAMIX_NUM_ACTIONS action probabilities (sums in double, outputs float).
 * dynamix_policy_choose: actions[k] = index into DYNAMIX_ACTIONS; uniforms == NULL picks the
 *   most probable action (the first of equals), otherwise uniforms[k] in [0, 1) is the caller's
 *   random draw and the index is the inverse of the cumulative distribution there (the library
 *   draws no random numbers itself).
 * dynamix_batch_sizes_step: next[k] = max(min(b[k] + DYNAMIX_ACTIONS[actions[k]], b_max), b_min).
 * dynamix_cycle_rewards: the reward above per worker; sigma2_norm and sigma_norm are the cycle
 *   means from dynamix_cycle_summary (global record, entries DYNAMIX_STAT_SIGMA2_NORM and
 *   DYNAMIX_STAT_SIGMA_NORM of the means), used only when adaptive_optimizer != 0.
 * dynamix_discounted_return: sum_t gamma^t rewards[t] over count cycles.
 * dynamix_policy_update: one gradient-ascent step of the shared parameters on n recorded
 *   decisions (Algorithm 1, the policy-update step), weights <- weights + lr * gradient of the
 *   mean objective, evaluated before the step and returned in *objective (may be NULL):
 *     DYNAMIX_POLICY_RETURN_WEIGHTED  mean_j signal[j] log pi(a_j | s_j): the paper's simplified
 *                                     rule, the cumulative reward as the weight of each decision,
 *                                     no clipping and no advantage estimate; old_probs unused
 *     DYNAMIX_POLICY_CLIPPED          mean_j min(r_j signal[j], clip(r_j, 1-eps, 1+eps) signal[j]),
 *                                     r_j = pi(a_j | s_j) / old_probs[j], the clipped surrogate
 *                                     of the paper's PPO objective with signal = the advantage
 *   states: n rows as for dynamix_policy_forward; actions: n indices; signal: n doubles;
 *   old_probs: n probabilities the old policy gave the taken actions.  Gradients by
 *   back-propagation in double; the optimizer around it (learning-rate schedule, epochs over the
 *   batch) is the caller's.
 * All return a dynamix_status except the two that return a count or a value.
 */
enum { DYNAMIX_NUM_ACTIONS = 5 };
enum { DYNAMIX_POLICY_RETURN_WEIGHTED = 0, DYNAMIX_POLICY_CLIPPED = 1 };
#define DYNAMIX_ACTIONS {-100, -25, 0, 25, 100}
int64_t dynamix_policy_weight_count(const int32_t* layer_sizes, int32_t num_layers);
int     dynamix_policy_forward(const float* weights, const int32_t* layer_sizes, int32_t num_layers,
                               const float* states, int32_t K, float* probs);
int     dynamix_policy_choose(const float* probs, int32_t K, const float* uniforms, int32_t* actions);
int     dynamix_batch_sizes_step(const int32_t* batch_sizes, const int32_t* actions, int32_t K,
                                 int32_t b_min, int32_t b_max, int32_t* next_batch_sizes);
int     dynamix_cycle_rewards(const double* mean_accuracy, const double* accuracy_gain,
                              const double* iteration_time, const int32_t* batch_sizes, int32_t K,
                              double alpha, double beta, double delta, double eta, double sigma2_norm,
                              double sigma_norm, int32_t adaptive_optimizer, double* rewards);
double  dynamix_discounted_return(const double* rewards, int64_t count, double gamma);
int     dynamix_policy_update(float* weights, const int32_t* layer_sizes, int32_t num_layers,
                              const float* states, const int32_t* actions, const double* signal,
                              const float* old_probs, int64_t n, int32_t mode, double clip_eps,
                              double lr, double* objective);

/*
 * Kernel timing (profiling aid).  dynamix_timing_begin(capacity) creates `capacity` slots of HIP
 * events (capacity 0 switches timing off and frees them).  While slots remain, every call to the
 * aggregate entry points records three events on its stream: before the streaming pass, between
 * the two kernels, after the final reduction.  dynamix_timing_count() is the number of slots
 * used.  Once the stream has been synchronised, dynamix_timing_read(i, ...) returns the two
 * kernel durations of the i-th timed call in milliseconds (DYNAMIX_ERR_HIP if that call has not
 * finished, DYNAMIX_ERR_ARG for an unused slot).  The events themselves cost the stream about ten
 * microseconds per timed call; dynamix_timing_every(n) has only every n-th call timed, counted
 * from the dynamix_timing_begin that follows (n >= 1; the default is every call).
 */
int     dynamix_timing_begin(int32_t capacity);
int     dynamix_timing_every(int32_t n);
int32_t dynamix_timing_count(void);
int     dynamix_timing_read(int32_t index, float* stream_pass_ms, float* final_reduce_ms);

/*
 * Measurement aid, not part of the path: plain streaming kernels in the launch shape and access
 * pattern of the streaming pass (one block of 256 threads per compute unit, contiguous span per
 * block, 128-bit non-temporal buffer accesses) with no arithmetic, to measure what the memory
 * system gives such a kernel.  `buffers`: HOST array of `count` DEVICE pointers, 256-byte aligned,
 * `bytes` each (a multiple of 4096 is used).  Modes:
 *   DYNAMIX_PROBE_READ         read `count` (1, 2, 4, 8, 16 or 32) buffers, 4 KB tiles in order
 *   DYNAMIX_PROBE_READ_SPREAD  the same in the interleaved 256-byte chunks of the streaming pass
 *   DYNAMIX_PROBE_READ_SPREAD_128B, _512B  the same with chunks of 128 and 512 bytes (32 and 8
 *                              units of 4 KB per load instruction of a block instead of 16)
 *   DYNAMIX_PROBE_WRITE        count == 1: write buffers[0]
 *   DYNAMIX_PROBE_COPY         count == 2: buffers[1] := buffers[0]
 * Every probe kernel reserves more than half of a compute unit's LDS, so two probes launched
 * together on two streams with n and (compute units - n) blocks run on disjoint units: that is
 * how reading beside writing is measured.  Only enqueues one kernel on `stream`; validates first.
 */
enum { DYNAMIX_PROBE_READ = 0, DYNAMIX_PROBE_READ_SPREAD = 1, DYNAMIX_PROBE_WRITE = 2,
       DYNAMIX_PROBE_COPY = 3, DYNAMIX_PROBE_READ_SPREAD_128B = 4, DYNAMIX_PROBE_READ_SPREAD_512B = 5 };
int dynamix_hbm_probe(const void* const* buffers, int32_t count, int64_t bytes, int32_t mode,
                      int32_t blocks, void* stream);

/*
 * Environment: DYNAMIX_MAX_BLOCKS=n (n >= 1) caps the number of blocks the streaming pass is
 * launched with; it is read whenever a plan is built (first call for a shape).  A tuning and
 * testing aid: results do not depend on it beyond the order of the fp64 partial sums.
 * DYNAMIX_SPREAD=0 keeps the streaming pass on consecutive tiles also where it would interleave
 * chunks (see `grads` above); read at every call; same kind of aid.
 * DYNAMIX_TAIL_PERMILLE=n (0..500) sets the share of every block's span that is cut into short
 * pieces for whichever block is free (default 30, for spans of 64 block iterations or more; 0
 * turns it off) and DYNAMIX_TAIL_MIN=n the length of the shortest of them in block iterations
 * (default 2); read when a plan is built; same kind of aid: every piece yields its own partial
 * sums, so results do not depend on which block took which.
 */

/* Frees every cached plan and workspace.  The caller must have synchronised all streams that
 * were used with the library.  Returns a dynamix_status. */
int dynamix_release_cached(void);

#ifdef __cplusplus
}
#endif
#endif /* DYNAMIX_H */
