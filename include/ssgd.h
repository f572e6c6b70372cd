/*
 * ssgd.h - C ABI of the MI355X library that simulates straggler-aware
 * distributed SGD with P virtual workers on one GPU.
 *
 * The calls follow the problem statement of "Slow and Stale Gradients Can Win
 * the Race" (arXiv 2003.10579): a parameter server with P workers (Sec. 2.1),
 * mini-batch size m, learning rate eta, K workers or mini-batches waited for
 * per update (Sec. 2.2), i.i.d. random compute delays per worker and
 * mini-batch (Sec. 3.1), the expected runtime per iteration (Sec. 2.3, Sec. 3)
 * and AdaSync (Sec. 6).
 *
 * Conventions
 *  - Pointers are tagged DEVICE (address in the memory of the current HIP
 *    device) or HOST.  The library never takes ownership of a caller buffer.
 *  - Every call returns an ssgd_status; nothing throws or aborts across the
 *    ABI.  On an error `ssgd_last_error` gives a static or context-owned text.
 *  - A context is bound to the HIP device that was current in ssgd_create and
 *    to the stream given there.  It is not thread-safe; distinct contexts are
 *    independent.
 *  - Determinism: identical arguments give identical delays, selections,
 *    staleness counts and clock values, bit for bit.
 */
#ifndef SSGD_H
#define SSGD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ssgd_ctx ssgd_ctx; /* opaque, library-owned */

typedef enum {
    SSGD_OK = 0,
    SSGD_EINVAL = 1,  /* bad argument; nothing was changed */
    SSGD_ENOMEM = 2,  /* a device or host allocation failed */
    SSGD_EDEVICE = 3, /* a HIP call or a kernel reported an error */
    SSGD_ESTATE = 4   /* call not valid in the context's current state */
} ssgd_status;

/* Loss f(w, xi) behind the objective F(w) = (1/N) sum_n f(w, xi_n) (Eq. (1)).
 * Parameter vector layout (fp32):
 *   SSGD_LSQ      f = (x.w - y)^2 / 2                 w[d]
 *   SSGD_SOFTMAX  f = -log softmax(W x + b)_y         W[classes][d], b[classes]
 *   SSGD_MLP2     two-layer ReLU network + softmax    W1[hidden][d], b1[hidden],
 *                                                     W2[classes][hidden], b2[classes] */
typedef enum { SSGD_LSQ = 0, SSGD_SOFTMAX = 1, SSGD_MLP2 = 2 } ssgd_model_kind;

/* The four variants of Sec. 2.2. */
typedef enum {
    SSGD_K_SYNC = 0,       /* Eq. (2): first K of P workers, the rest are cancelled */
    SSGD_K_BATCH_SYNC = 1, /* first K mini-batches; a finished worker starts another at w_j */
    SSGD_K_ASYNC = 2,      /* Eq. (3): first K of P workers, nobody is cancelled, stale w */
    SSGD_K_BATCH_ASYNC = 3 /* first K mini-batches, nobody is cancelled: a worker that pushes re-reads the
                              current parameters and starts its next mini-batch at once.  Fixed K or
                              AdaSync mode 1.  Linear models: d % 4 == 0, at most 15 classes,
                              K <= 64 (any m); MLP2: its usual limits, K <= 256;
                              else SSGD_EINVAL */
} ssgd_variant;

/* Delay X of one mini-batch on one worker (Sec. 3.1).
 *   SSGD_EXP          X = E / rate,          E ~ Exp(1)   (rate = mu, E[X] = 1/mu)
 *   SSGD_SHIFTED_EXP  X = shift + E / rate                (Lemma 4)
 *   SSGD_PARETO       X = scale * exp(E / alpha)          (Pareto(alpha, scale), Fig. 5)
 *   SSGD_TABLE        X = table[(((version * P) + worker) * R + ordinal) mod table_len],
 *                     R = 1 for K-sync / K-async, Kmax + 1 for the batch variants.
 *                     `table` is a HOST pointer, copied in ssgd_create. */
typedef enum { SSGD_EXP = 0, SSGD_SHIFTED_EXP = 1, SSGD_PARETO = 2, SSGD_TABLE = 3 } ssgd_delay_kind;

typedef struct {
    int32_t kind; /* ssgd_delay_kind */
    double shift, rate, alpha, scale;
    const float *table; /* HOST, SSGD_TABLE only */
    int64_t table_len;
} ssgd_delay_dist;

typedef struct {
    int32_t kind; /* ssgd_model_kind */
    int32_t d, classes, hidden;
    int32_t bf16;    /* SSGD_MLP2: 1 = bf16 operands, fp32 accumulation, in the two
                        contractions over d; must be 0 for the linear models */
    const float *X;  /* DEVICE, N x d row-major fp32; must outlive the context and stay unchanged:
                      * SSGD_MLP2 keeps its values rounded to bf16, taken when the context is made */
    const void *y;   /* DEVICE, float[N] (LSQ) or int32[N] labels in [0, classes) */
    int64_t N;       /* 1 <= N < 2^32 */
} ssgd_model;

/* AdaSync (Sec. 6): how K changes between updates.
 *   mode 0  K fixed
 *   mode 1  windows of `window` updates; if the mean training loss of a window is
 *           above (1 - rel_tol) times that of the window before, K doubles (<= Kmax)
 *   mode 2  Algorithm 1: whenever the clock crosses a multiple of interval_t and
 *           K < Kmax, K = K0 sqrt(F(w_0) / F(w_start)), rounded, never decreasing
 *   mode 3  the K-sync rule of App. D: K^2/(P-K) = K0^2/(P-K0) F(w_0)/F(w_start)
 * F is estimated by the mean mini-batch loss of the contributors. */
typedef struct {
    int32_t mode, K0, Kmax, window;
    double rel_tol, interval_t;
} ssgd_adasync;

/* Create `replicas` independent simulations (same data, same w_0, delays and
 * mini-batches keyed by the replica index) of `variant` with P workers that
 * waits for K, mini-batch size m, learning rate lr.  All P workers start at
 * time 0 with w_0 (zeros; uniform(-1/sqrt(fan_in), 1/sqrt(fan_in)) weights for
 * the MLP).  `hip_stream` is a hipStream_t (NULL = default stream); all work
 * is enqueued there.  `adasync` may be NULL (mode 0).
 * Limits: 1 <= K <= P <= 256 for K-sync / K-async, 1 <= K <= 256 for the batch
 * variants, m >= 1, d >= 1, classes <= 16 for SOFTMAX; MLP2 needs bf16 = 1, m <= 64,
 * d % 128 == 0, hidden % 128 == 0, and with several replicas a fixed K or AdaSync mode 1;
 * SSGD_K_BATCH_ASYNC has the limits given with the enumeration.  Invalid arguments give
 * SSGD_EINVAL and leave *out untouched. */
ssgd_status ssgd_create(const ssgd_model *model, int32_t P, int32_t K, int32_t m, int32_t variant,
                        const ssgd_delay_dist *dist, double lr, uint64_t seed, int32_t replicas,
                        const ssgd_adasync *adasync, void *hip_stream, ssgd_ctx **out);

/* Perform J further parameter-server updates in every replica: delays,
 * K-of-P selection, mini-batch gradients at the (possibly stale) parameters each
 * contributor read, w_{j+1} = w_j - (lr/K) sum_l g_l.  Appends to the trace.
 * Returns after the work has completed on the stream.  The library may use further
 * streams of its own (default priority; they start after the work queued on
 * `hip_stream` and that stream waits for them) and, for one replica of SSGD_MLP2,
 * two short-lived host threads that launch kernels during the call. */
ssgd_status ssgd_run(ssgd_ctx *ctx, int64_t J);

/* Make room in the trace for `updates` further updates now, so that later ssgd_run
 * calls up to that total do not reallocate it. */
ssgd_status ssgd_reserve_trace(ssgd_ctx *ctx, int64_t updates);

/* One update; additionally writes the averaged gradient (1/K) sum_l g_l that the
 * update applied, for replica 0, to agg_grad_out (DEVICE, |w| floats, nullable). */
ssgd_status ssgd_step(ssgd_ctx *ctx, float *agg_grad_out);

/* Number of parameters |w| of the context's model. */
int64_t ssgd_param_count(const ssgd_ctx *ctx);
/* Updates done so far, current K, and the row width Kmax of the trace arrays. */
int64_t ssgd_updates_done(const ssgd_ctx *ctx);
int32_t ssgd_current_K(const ssgd_ctx *ctx, int32_t replica);
int32_t ssgd_trace_width(const ssgd_ctx *ctx);

/* Copy updates [from, from+n) of one replica's trace to HOST arrays (each
 * nullable): t[n] clock after the update (fp64), loss[n] mean mini-batch loss of
 * the contributors, K[n], and n x Kmax matrices (unused entries -1) of the
 * contributing workers in arrival order, their staleness j - tau, and the
 * ordinal of the contributed mini-batch. */
ssgd_status ssgd_get_trace(ssgd_ctx *ctx, int32_t replica, int64_t from, int64_t n, double *t,
                           float *loss, int32_t *K, int32_t *sel_workers, int32_t *staleness,
                           int32_t *ordinal);

/* Copy the current parameters of one replica to w_out (HOST, |w| floats). */
ssgd_status ssgd_get_params(ssgd_ctx *ctx, int32_t replica, float *w_out);
/* Overwrite the current parameters of one replica from w_in (HOST, |w| floats).
 * Gradients of mini-batches already in flight keep the parameters they read. */
ssgd_status ssgd_set_params(ssgd_ctx *ctx, int32_t replica, const float *w_in);
/* Force K for the following updates (1 <= K <= Kmax); AdaSync keeps running. */
ssgd_status ssgd_force_K(ssgd_ctx *ctx, int32_t K);

/* The objective F(w) = (1/N) sum_n f(w, xi_n) of Eq. (1) over the whole data set at the replica's
 * current parameters (what the paper's error-versus-time curves plot), one streaming pass over
 * X.  loss_out: HOST.  Linear models need d % 4 == 0 (else SSGD_EINVAL) and evaluate in fp32
 * with fp64 sums.  The two-layer network evaluates with the forward pass of its trainer (inputs,
 * W1 and W2 at their bf16 values, fp32 accumulation), through temporary device buffers that the
 * call allocates and frees (SSGD_ENOMEM if they do not fit); mini-batches in flight are untouched. */
ssgd_status ssgd_full_loss(ssgd_ctx *ctx, int32_t replica, double *loss_out);

/* The gradient of that objective, grad F(w) = (1/N) sum_n grad f(w, xi_n), at the replica's current
 * parameters: the quantity in which the staleness bound (fifth assumption of Sec. 4.1) is stated
 * (E||grad F(w_j) - grad F(w_tau)||^2 <= gamma E||grad F(w_j)||^2).  grad_out: HOST, |w| floats in the
 * layout of the parameters.  Two passes over X in fp32 with fp64 sums over chunks of samples, through
 * temporary device buffers (SSGD_ENOMEM if they do not fit).  Linear models need d % 4 == 0, else
 * SSGD_EINVAL.  The two-layer network: with the arithmetic of its training gradients (bf16 operands in
 * the two large contractions, fp32 accumulation), the data set in blocks of up to 256 x 64 rows that are
 * added on the host in fp64; parameters, trace and mini-batches in flight are untouched. */
ssgd_status ssgd_full_gradient(ssgd_ctx *ctx, int32_t replica, float *grad_out);

/* ssgd_full_gradient for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same kernels in the same launch shape,
 * hence the same values bit for bit, but the intermediate results (16 floats per sample and up to
 * 64 partial gradients) live in a static device array of the library, 4 Mi floats = 16 MiB that every
 * GPU the library runs on holds until the process ends, and the gradient is written to
 * grad_out_device (DEVICE, |w| floats, layout of the parameters).  The call allocates and frees
 * nothing, copies nothing to the host and does not wait: the work is enqueued on the context's stream
 * and the result is complete when that stream reaches the end of it.  Data sets that need more than
 * the array holds (16 N + min(64, ceil(N / 256)) * classes * (d + 1) floats > 4 Mi) give SSGD_EINVAL,
 * as do the shapes ssgd_full_gradient refuses.  All calls on one GPU, from any context, share that
 * GPU's array: calls that overlap on one GPU (different streams or threads) race; calls on one stream
 * are ordered.  Nothing in the array has to be zero at entry: a call writes every word before it
 * reads it, so the contents left by an earlier, larger call do not matter. */
ssgd_status ssgd_full_gradient_static(ssgd_ctx *ctx, int32_t replica, float *grad_out_device);

/* The mini-batch each worker of a K-async run has in flight (Sec. 2.2: a worker that is not
 * among the K selected keeps computing on the parameters it read): version read tau_i, ordinal,
 * absolute finish time f_i.  HOST arrays of P entries, each nullable.  SSGD_EINVAL for the
 * synchronous variants, which restart every worker at every update. */
ssgd_status ssgd_get_workers(ssgd_ctx *ctx, int32_t replica, int32_t *tau, int32_t *ord, double *finish);

/* Snapshot and resume.  A snapshot holds everything later updates depend on: the trace so far,
 * update count, simulated clock, current K and the AdaSync bookkeeping, every worker's tau_i and
 * f_i, the parameters, and the gradients (linear models) or gradient factors (MLP) of the
 * mini-batches in flight, which were taken at parameters that no longer exist.  It is an opaque
 * HOST buffer of ssgd_state_bytes() bytes (the size grows with the trace); ssgd_set_state accepts
 * it only on a context created with the same model shape, P, m, variant, replicas, seed and
 * AdaSync mode and only if its size fits the number of updates its header states (else
 * SSGD_EINVAL, context unchanged), replaces that context's state and trace, and the updates that
 * follow are those the original context would have run.  A device error while the state is
 * copied leaves the context unusable (SSGD_ESTATE from then on).  The data set is not part of
 * the snapshot. */
ssgd_status ssgd_state_bytes(ssgd_ctx *ctx, int64_t *bytes);
ssgd_status ssgd_get_state(ssgd_ctx *ctx, void *host_buf, int64_t bytes);
ssgd_status ssgd_set_state(ssgd_ctx *ctx, const void *host_buf, int64_t bytes);

/* Monte-Carlo estimate of the runtime per iteration T (Sec. 2.3, Lemmas 1-3;
 * the simulation behind Fig. 6).  Trial r draws P fresh delays; for every K in
 * [Kmin, Kmax] the variant's event process is run for chain_len updates from that
 * fresh start and T_l (l = 1..chain_len) is recorded; for SSGD_K_BATCH_ASYNC (Lemma 5)
 * the pushes of all workers form one sequence for every K and update l is push l K.
 * P <= 256, chain_len <= 4096, for SSGD_K_BATCH_ASYNC chain_len * Kmax <= 7500 (else
 * SSGD_EINVAL).  Outputs are HOST arrays of
 * (Kmax-Kmin+1) x chain_len entries: mean and unbiased variance of T_l, and
 * (nullable) the raw sums `sum` and `sumsq`; per_trial (HOST, nullable,
 * trials x (Kmax-Kmin+1) x chain_len fp64) receives every trial's T_l. */
ssgd_status ssgd_runtime_mc(int32_t variant, int32_t P, int32_t Kmin, int32_t Kmax,
                            const ssgd_delay_dist *dist, int64_t trial0, int64_t trials,
                            int32_t chain_len, uint64_t seed, void *hip_stream, double *mean,
                            double *var, double *sum, double *sumsq, double *per_trial);

/* Delays and mini-batch indices as the library draws them (DEVICE kernels, HOST
 * outputs), for bit-exact checks: n delays for raw 32-bit words, and the m sample
 * ids of the mini-batch (replica, worker, ordinal, version). */
ssgd_status ssgd_debug_delays(const ssgd_delay_dist *dist, const uint32_t *bits, int64_t n, float *out);
ssgd_status ssgd_debug_batch(uint64_t seed, uint32_t replica, uint32_t worker, uint32_t ordinal,
                             uint32_t version, int32_t m, int64_t N, uint32_t *out);

/* Measurement aid (the achievable ceiling that Sec. 6-style throughput figures of the HBM-bound paths are
 * set against): `passes` plain streaming reads of `bytes` bytes at `data` (DEVICE, 16-byte aligned), timed
 * with HIP events on hip_stream; *bytes_per_s (HOST) receives bytes read per second.  The buffer is only
 * read.  SSGD_EINVAL for a null or misaligned buffer, bytes < 16 or passes < 1. */
ssgd_status ssgd_stream_read_rate(const void *data, int64_t bytes, int32_t passes, void *hip_stream,
                                  double *bytes_per_s);

/* Text of the last error of a context (ctx may be NULL: last error of a call
 * that has no context).  Valid until the next call on that context. */
const char *ssgd_last_error(const ssgd_ctx *ctx);

/* Average duration in milliseconds (HIP events on the context's stream) of the
 * gradient kernel launches of the last ssgd_run, and their number. */
ssgd_status ssgd_last_kernel_ms(const ssgd_ctx *ctx, double *avg_ms, int64_t *launches);

void ssgd_destroy(ssgd_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* SSGD_H */
