/*
 * netmax.h - C ABI of the MI355X (gfx950) NetMax iteration library.
 *
 * One NetMax iteration (arXiv 2009.05766, Algorithm 2 and Section IV,
 * Eq. (c0)/(c1)) over M worker model copies resident in one GPU's HBM.  For
 * every worker i, all from the copies of the previous iteration t:
 *
 *     m_i       ~ row i of the policy matrix P                (Algorithm 2, peer selection)
 *     g_i       = grad f(x_i^t ; batch_i^t)                   (Algorithm 2, first-step update)
 *     v_i^{t+1} = mu v_i^t + g_i + wd x_i^t                   (momentum SGD, Section V-A)
 *     h_i       = x_i^t - alpha v_i^{t+1}                     (Eq. (c0))
 *     x_i^{t+1} = h_i - w_i (h_i - x_{m_i}^t)                 (Eq. (c1))
 *     w_i       = alpha rho (d_{i,m_i} + d_{m_i,i}) / (2 p_{i,m_i}),  0 if m_i = i
 *
 * Conventions
 *   - Plain C.  Every call returns a netmax_status; netmax_last_error() gives the text.
 *   - "host" pointers are ordinary CPU memory, read during the call only.
 *     "device" pointers are HIP device memory owned by the caller, who keeps it
 *     alive while the context uses it.  The library owns only its own tables and
 *     scratch (thresholds, weights, batch indices, activations, partial sums).
 *   - Matrices over workers (x, v, g) are M x ld floats, ld >= D a multiple of
 *     NETMAX_TILE, base pointers 16-byte aligned, in the WORKER-INTERLEAVED TILE
 *     LAYOUT: [ld / NETMAX_TILE tiles][M workers][NETMAX_TILE floats], i.e. column j
 *     of worker i is element ((j / NETMAX_TILE) * M + i) * NETMAX_TILE + j % NETMAX_TILE.
 *     (All workers' copies of a column tile are contiguous, so the mix kernel sweeps
 *     HBM linearly and finds a peer's row next to the worker's own.)  netmax_pack
 *     and netmax_unpack convert from and to row-major.  Columns D..ld-1 are padding
 *     and stay 0.
 *   - Kernels are enqueued on the hipStream_t given at init and calls return
 *     without waiting, except netmax_consensus_dist, netmax_set_policy,
 *     netmax_set_lr, netmax_get_tables and netmax_destroy, which synchronise
 *     that stream.
 *   - The iteration number is an argument: all random draws are counter based
 *     (Philox4x32-10, key = (seed_lo, seed_hi ^ stream), counter = (block, worker,
 *     iter_lo, iter_hi)), so any iteration can be replayed.
 */
#ifndef NETMAX_H
#define NETMAX_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NETMAX_MAX_LAYERS 7
#define NETMAX_TILE 2048 /* floats per column tile and worker */

typedef struct netmax_ctx netmax_ctx; /* opaque, library-owned */

typedef enum {
    NETMAX_OK = 0,
    NETMAX_EINVAL = 1,      /* null pointer, M < 2, bad shape, bad alignment, invalid row of P */
    NETMAX_EINFEASIBLE = 2, /* a selectable pair has mix weight >= 1 (strict mode: > 1/2, i.e. violates (o3)) */
    NETMAX_ESTATE = 3,      /* state or data not bound, or call does not fit the model kind */
    NETMAX_EDEVICE = 4,     /* a HIP call failed */
    NETMAX_ENOMEM = 5
} netmax_status;

typedef enum { NETMAX_FLAT = 0, NETMAX_MLP = 1 } netmax_model;
typedef enum { NETMAX_F32 = 0, NETMAX_BF16 = 1 } netmax_dtype;
/* Second-step weight.  NETMAX_MIX_POLICY: w_im = alpha rho (d_im + d_mi) / (2 p_im), Algorithm 2 (a rarely chosen
 * peer weighs more).  NETMAX_MIX_FIXED: the same weight for every drawn pair, the gossip / AD-PSGD averaging that
 * Section III-D and Section V-H run under the same peer-selection policy (fixed_weight = 1/2 is plain averaging). */
typedef enum { NETMAX_MIX_POLICY = 0, NETMAX_MIX_FIXED = 1 } netmax_mix_mode;

typedef struct {
    int32_t M;         /* workers, 2 .. 4096 */
    int64_t D;         /* parameters per worker */
    int64_t ld;        /* padded number of columns of x, v, g: >= D, multiple of NETMAX_TILE */
    int32_t model;     /* netmax_model. FLAT: the local gradient is synthetic N(0, grad_sigma^2) noise.
                          MLP: ReLU perceptron with softmax cross-entropy; one layer = softmax regression */
    int32_t n_layers;  /* MLP only: 1 .. NETMAX_MAX_LAYERS */
    int64_t dims[NETMAX_MAX_LAYERS + 1]; /* MLP only: layer widths, D must equal sum(dims[l]*dims[l+1] + dims[l+1]).
                          Parameter layout inside a row: per layer W row-major [in][out], then b [out] */
    int32_t batch;     /* MLP only: samples per worker and iteration, 1 .. 1024 */
    int32_t gemm_in;   /* netmax_dtype of the feature matrix and of the GEMM operands (accumulation is fp32) */
    float lr;          /* alpha */
    float momentum;    /* mu; 0 = plain SGD */
    float weight_decay;
    float rho;         /* consensus weight of Eq. (1) */
    float grad_sigma;  /* FLAT only */
    uint64_t seed;
    int32_t strict_o3; /* nonzero: require w <= 1/2 for every selectable pair: constraint (o3) taken with >=, as
                          netmax_generate_policy takes it (links on the bound have w = 1/2); a relative 1e-6 is
                          allowed for a rho that was rounded to single precision */
    const double *P;   /* host, M*M row-major; p_im = probability that worker i selects m (Section II-B) */
    const uint8_t *adj;/* host, M*M neighbourhood indicators d_im, or NULL = complete graph without self loops */
    void *stream;      /* hipStream_t, NULL = the null stream */
    int32_t mix_mode;  /* netmax_mix_mode */
    float fixed_weight;/* NETMAX_MIX_FIXED only: in [0, 1) */
} netmax_config;

/* Builds the context: validates the configuration, turns P into 32-bit fixed-point cumulative
 * thresholds (row i: C[m] = round(2^32 sum_{j<=m} p_ij), forced to 2^32 from the last positive
 * entry on) and the mix-weight table w_im (Algorithm 2, second-step update), uploads both and
 * allocates the library's scratch.  On failure *out is NULL and netmax_last_error(NULL) has the text.
 * Rows of P must be non-negative and sum to 1 within 1e-9. */
int netmax_init(netmax_ctx **out, const netmax_config *cfg);

/* Host-only part of netmax_init, usable without a GPU: validates P (and adj) and writes the tables that
 * netmax_init would upload.  thresholds_host: uint32 [M][M]; last_host: int32 [M]; w_host: float [M][M];
 * all host memory owned by the caller.  Returns NETMAX_OK, NETMAX_EINVAL or NETMAX_EINFEASIBLE; the text is
 * available from netmax_last_error(NULL). */
int netmax_build_tables(int32_t M, const double *P, const uint8_t *adj, float lr, float rho, int32_t strict_o3,
                        int32_t mix_mode, float fixed_weight, uint32_t *thresholds_host, int32_t *last_host,
                        float *w_host);

/* Communication policy generation (Algorithm 3; Section III-C; Appendix A), host only, no GPU needed.
 * t_host: host double [M][M], t_im = iteration time of worker i when it pulls from m (the diagonal is ignored:
 * d_ii = 0 in Eq. (d3)); adj as in netmax_config; alpha = learning rate; K, R = grid sizes of the outer
 * (rho = k 0.5 / (alpha K), k = 1..K) and inner (tbar = L + r (U - L) / R, r = 1..R) search; eps in (0,1) scales
 * T_convergence = tbar ln(eps) / ln(lambda_2).  For every grid point the row-separable linear program
 * min sum p_ii s.t. (o2)-(o5) is solved ((o3) with >=; among the optimal points the one with the least-squares
 * distance to the lower bounds of (o3)), lambda_2 is the second largest eigenvalue of Y_P (Eq. (d2)).
 * Outputs (host): P_out double [M][M], rho_out; optional tbar_out, lambda2_out, t_conv_out of the winner.
 * Returns NETMAX_OK, NETMAX_EINVAL, or NETMAX_EINFEASIBLE if no grid point is feasible. */
int netmax_generate_policy(int32_t M, const double *t_host, const uint8_t *adj, double alpha, int32_t K, int32_t R,
                           double eps, double *P_out, double *rho_out, double *tbar_out, double *lambda2_out,
                           double *t_conv_out);

/* A new policy and weight from the monitor takes effect at the next iteration (Algorithm 2, "received
 * new policy").  P: host, M*M.  The tables are rebuilt; on error the old ones stay in force. */
int netmax_set_policy(netmax_ctx *ctx, const double *P, float rho);

/* Changes alpha (learning-rate decay, Section V-A) and rebuilds w, which depends on it. */
int netmax_set_lr(netmax_ctx *ctx, float lr);

/* Binds the caller's state, all device float M x ld in the tile layout: x_a holds x^t for the next iteration to run and
 * x_b receives x^{t+1} (the two swap roles after every netmax_mix); v is the momentum buffer (the caller
 * zeroes it for v^0 = 0), g receives the gradients. */
int netmax_bind_state(netmax_ctx *ctx, float *x_a, float *x_b, float *v, float *g);

/* MLP only.  feats: device, [n_total][dims[0]] row-major, float or bfloat16 as cfg.gemm_in says;
 * labels: device int32 [n_total], values in [0, dims[n_layers]); shard_off: host int64 [M+1], worker i
 * owns rows shard_off[i] .. shard_off[i+1]-1 (each shard non-empty, at most 2^31-1 rows). */
int netmax_bind_data(netmax_ctx *ctx, const void *feats, const int32_t *labels, const int64_t *shard_off);

/* Layout conversion on the context's stream.  rows_dev: device float, row-major [M][row_ld], row_ld >= D;
 * tiled_dev: device float M x ld in the tile layout.  netmax_pack copies the first D columns of every row
 * and zeroes the padding; netmax_unpack writes the first D columns of every row. */
int netmax_pack(netmax_ctx *ctx, const float *rows_dev, int64_t row_ld, float *tiled_dev);
int netmax_unpack(netmax_ctx *ctx, const float *tiled_dev, float *rows_dev, int64_t row_ld);

/* Peer selection of Algorithm 2 for all workers at iteration `iter`: worker i draws word 0 of block 0 of
 * stream 0 and takes the first m whose cumulative threshold exceeds it.  peers_dev: device int32 [M]. */
int netmax_sample_peers(netmax_ctx *ctx, uint64_t iter, int32_t *peers_dev);

/* MLP only.  The batch D_{i,n} of Eq. (a5): B draws with replacement per worker; draw b is word b%4 of
 * block b/4 of stream 1 mapped to floor(u n_i / 2^32).  idx_dev: device int32 [M][batch], shard-local rows.
 * netmax_local_step makes the same draws itself; this entry point exposes them. */
int netmax_sample_batch(netmax_ctx *ctx, uint64_t iter, int32_t *idx_dev);

/* Fills g from the current parameters: the stochastic gradient of Algorithm 2's first-step update.
 * MLP: mean cross-entropy gradient of each worker's own weights on its own batch (grouped GEMMs, one
 * group per worker).  FLAT: g[i][j] = grad_sigma * N(0,1) by Box-Muller on block j/4 of stream 2 with
 * u = ((word >> 9) + 0.5) 2^-23; words (0,1) give elements j, j+1 and words (2,3) give j+2, j+3.
 * Padding columns of g are set to 0. */
int netmax_local_step(netmax_ctx *ctx, uint64_t iter);

/* Momentum apply and mix (Eq. (c0), (c1)) for all workers with the given peers (device int32 [M], each in
 * [0, M); an index outside that range is treated as a self draw); reads x^t, g, v and the peers' rows of x^t, writes x^{t+1} and v, then swaps the roles of the two
 * parameter buffers.  `iter` is recorded for netmax_iteration(). */
int netmax_mix(netmax_ctx *ctx, uint64_t iter, const int32_t *peers_dev);

/* n_iters whole iterations (netmax_sample_peers, netmax_local_step, netmax_mix for iter = first_iter, first_iter + 1,
 * ...) enqueued from one call; peers_dev (device int32 [M]) receives each iteration's peers in turn.  With
 * use_graph != 0 an iteration is recorded once per direction of the parameter ping-pong into a HIP graph and
 * replayed (the iteration number then lives in a device cell that the graph advances), which removes the launch
 * overhead that dominates small models; this needs a context created on a non-default stream (the null stream
 * cannot be captured), else NETMAX_ESTATE.  The graphs are dropped when buffers, data or the learning rate change.
 * Results are identical to the individual calls.
 * Small softmax-regression models (one layer, float features, at most 32 classes, parameters and batch within a
 * workgroup's LDS) run whole iterations inside ONE kernel, one workgroup per worker: without use_graph all n_iters
 * iterations are one cooperative launch with a device-wide barrier after every iteration (when all M workgroups fit
 * the device at once, else one launch per iteration); with use_graph the replayed graph holds that kernel.  Same
 * results bit for bit: netmax_local_step runs the same gradient code for such models and every kernel applies the
 * update with the same instructions.  Should a workgroup ever wait at the barrier in vain, the kernel still ends, the
 * parameters are invalid and the next netmax_consensus_dist returns NETMAX_EDEVICE. */
int netmax_run(netmax_ctx *ctx, uint64_t first_iter, int32_t n_iters, int32_t *peers_dev, int32_t use_graph);

/* netmax_run with the second-step update (Eq. (c0)/(c1)) applied by the weight-gradient kernels themselves: for the
 * layers that run on the bf16 matrix-core kernels the product dW = A^T dZ is not written to g; the kernel that
 * computes it reads x, v and the peer's x and writes x' and v' of those columns directly (Algorithm 2's two update
 * steps on the gradient while it is still in registers).  A reduced mix covers all other columns.  x' and v' are
 * the same as without fusion; g then holds only the columns the fused kernels do not cover.  on = 0 switches back.
 * For flat models the fused variant generates the synthetic gradient inside the update kernel (g is still written,
 * with the same values; its read by the update is what is saved).
 * Affects netmax_run only (netmax_local_step and netmax_mix stay separate steps).  NETMAX_ESTATE for perceptron
 * models without such a layer.  Waits for the stream and drops captured graphs. */
int netmax_set_fusion(netmax_ctx *ctx, int32_t on);

/* The device-wide barrier of the multi-iteration launches of netmax_run (small models, above) polls a counter; a
 * workgroup that has polled `polls` times without seeing all others arrive raises the context's fault flag and goes
 * on, so that the kernel always ends (default 2^24 polls, seconds; the barrier itself takes microseconds).  This call
 * sets that number and clears the fault flag; it waits for the stream.  polls = 0 makes every workgroup that is not the
 * last to arrive give up at once: the way to exercise the failure path (netmax_consensus_dist then returns
 * NETMAX_EDEVICE and the parameters are not valid) without making anything wait. */
int netmax_set_barrier_patience(netmax_ctx *ctx, int64_t polls);

/* ---- Asynchronous schedule (Section II-B, Eq. (c2)-(c4)) ----------------------------------------------------
 * The workers do not step together: in global step k one worker i_k is active, pulls from m_k ~ P[i_k, :], takes
 * its local step and mixes; every other copy stays as it is, x^{k+1} = D^k (x^k - alpha g^k).  A worker whose
 * iterations take tbar_i = sum_m t_im p_im d_im on average (Eq. (d3)) is the active one with probability
 * p_i = (1 / tbar_i) / sum_m (1 / tbar_m) (Eq. (d4)).
 *
 * netmax_activity: host helper, p_act_out[i] = p_i from iteration times t (host double [M][M], diagonal ignored),
 * policy P (host double [M][M]) and adj (host, may be NULL).  NETMAX_EINVAL if a worker's mean time is not positive.
 * netmax_mean_times: host helper, tbar_out[i] = tbar_i of Eq. (d3) (host double [M]) and, if rate_out is not NULL,
 * sum_i 1 / tbar_i, the number of global steps per unit of time (the normaliser of Eq. (d4)).  Same arguments and
 * error as netmax_activity.
 * netmax_set_activity: installs p_act (host double [M], non-negative, sum 1 within 1e-9) as 32-bit cumulative
 * thresholds, as for a policy row.
 * netmax_async_run: global steps first_step .. first_step + n_steps - 1 on the context's stream.  Step k draws i_k
 * from word 0 of Philox stream 3 at counter (0, 0, k) and m_k from stream 0 at counter (0, i_k, k); the gradient
 * of the active worker uses iteration number k in its counters.  active_dev / peers_dev: device int32 [n_steps],
 * caller-owned, receive i_k and m_k.  x (the current buffer) and v are updated in place, no buffer flip; the active
 * worker's row of g receives its gradient (only that worker's gradient is computed).  Consecutive steps that cannot
 * see each other (no worker active twice, no pull from a row written earlier in the group, no write to a row pulled
 * earlier) run as one batch of launches of up to 32 steps; the host finds these groups by repeating the draws, which
 * are integer work on the same tables.  The result is that of the strictly sequential schedule.
 * Needs netmax_bind_state, netmax_set_activity and, for perceptron models, netmax_bind_data (else NETMAX_ESTATE).
 * Returns after enqueueing. */
int netmax_activity(int32_t M, const double *t_host, const double *P_host, const uint8_t *adj, double *p_act_out);
int netmax_mean_times(int32_t M, const double *t_host, const double *P_host, const uint8_t *adj, double *tbar_out,
                      double *rate_out);
int netmax_set_activity(netmax_ctx *ctx, const double *p_act);
int netmax_async_run(netmax_ctx *ctx, uint64_t first_step, uint64_t n_steps, int32_t *active_dev, int32_t *peers_dev);

/* Worker-side time bookkeeping of Algorithm 2 (UpdateTimeVector) against a simulated network.  For every worker i
 * with peer m = peers_dev[i]: ema_dev[i][m] = beta ema_dev[i][m] + (1 - beta) t_dev[i][m] (not for m = i) and, if
 * clock_dev is not NULL, clock_dev[i] += t_dev[i][m].  t_dev, ema_dev: device float [M][M]; clock_dev: device
 * float [M]; all caller-owned.  ema_dev is what the monitor would collect (Algorithm 1) and hand to
 * netmax_generate_policy. */
int netmax_update_times(netmax_ctx *ctx, const int32_t *peers_dev, const float *t_dev, float beta, float *ema_dev,
                        float *clock_dev);

/* The same bookkeeping for global steps of the asynchronous schedule, taken in order: for s = 0 .. n_steps - 1 with
 * i = active_dev[s], m = peers_dev[s]: ema_dev[i][m] = beta ema_dev[i][m] + (1 - beta) t_dev[i][m] (not for m = i),
 * clock_dev[i] += t_dev[i][m].  active_dev, peers_dev: device int32 [n_steps], as netmax_async_run fills them. */
int netmax_update_times_async(netmax_ctx *ctx, const int32_t *active_dev, const int32_t *peers_dev, uint64_t n_steps,
                              const float *t_dev, float beta, float *ema_dev, float *clock_dev);

/* Consensus distance sum_i ||x_i - mean_i x_i||^2 over the first D columns of the current parameters: the
 * complete-graph form of the model-difference penalty of Eq. (1).  fp64 accumulation, fixed summation
 * order.  Waits for the stream; out_host: host double. */
int netmax_consensus_dist(netmax_ctx *ctx, double *out_host);

/* The consensus distance for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Needs no context and calls no allocator: the per-block partial
 * sums that netmax_consensus_dist keeps in context-owned memory live in a fixed device array inside the library
 * (NETMAX_STATIC_PARTIALS doubles = 512 KB per GPU, held until the process ends), so ld may be at most
 * NETMAX_STATIC_MAX_LD columns; a longer matrix is rejected with NETMAX_EINVAL (text: netmax_last_error(NULL)).
 * x_dev: device float M x ld in the tile layout (ld a multiple of NETMAX_TILE, 16-byte aligned, 1 <= D <= ld,
 * 2 <= M <= 4096); cd_dev: device double [1], caller-owned, receives the same value netmax_consensus_dist returns
 * (same kernels, same summation order); stream: hipStream_t on the current device, NULL = the null stream.
 * Enqueues two kernels and returns without waiting.  All calls on one GPU share that GPU's array: calls that
 * overlap in time on one GPU (different streams, or graphs replayed side by side) race and must be serialised
 * by the caller.  Nothing has to be cleared between calls: every partial sum read is written by the same call. */
#define NETMAX_STATIC_PARTIALS 65536
#define NETMAX_STATIC_MAX_LD ((int64_t)NETMAX_STATIC_PARTIALS * 1024)
int netmax_consensus_dist_static(int32_t M, int64_t D, int64_t ld, const float *x_dev, double *cd_dev, void *stream);

/* Device pointer of the current parameters x^t (one of x_a, x_b; tile layout), NULL if nothing is bound. */
const float *netmax_params(const netmax_ctx *ctx);

/* MLP only: device float [M], mean batch loss of each worker as computed by the last netmax_local_step. */
const float *netmax_losses(const netmax_ctx *ctx);

/* MLP only: copies those M losses to out_dev (device float [M], caller-owned) on the context's stream; returns
 * without waiting. */
int netmax_read_losses(netmax_ctx *ctx, float *out_dev);

/* MLP only: the outputs of hidden layer `layer` (1 .. n_layers - 1; the ReLU outputs that feed layer `layer` + 1) of
 * the last netmax_local_step, as device float [M][batch][dims[layer]] into out_dev (caller-owned), on the context's
 * stream, without waiting.  With bf16 operands these are the stored bfloat16 activations, widened.  An entry is
 * positive exactly where the backward pass took the ReLU derivative as 1 (Algorithm 2's stochastic gradient is
 * discontinuous there, which is what run-to-run comparisons look at). */
int netmax_read_hidden(netmax_ctx *ctx, int32_t layer, float *out_dev);

/* Number of netmax_mix calls so far (the next iteration's default counter). */
uint64_t netmax_iteration(const netmax_ctx *ctx);

/* Copies the tables in force to the host (any pointer may be NULL): thresholds uint32 [M][M], index of
 * the last positive entry of each row int32 [M], mix weights float [M][M]. */
int netmax_get_tables(netmax_ctx *ctx, uint32_t *thresholds_host, int32_t *last_host, float *w_host);

/* Text of the last error of this context (ctx = NULL: of the last failed netmax_init on this thread). */
const char *netmax_last_error(const netmax_ctx *ctx);

/* Waits for the stream and frees the library's tables and scratch.  The caller's buffers are untouched. */
int netmax_destroy(netmax_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* NETMAX_H */
