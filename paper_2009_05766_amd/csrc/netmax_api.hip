// C ABI of the library (see include/netmax.h): context, host-side policy tables, argument checks and
// kernel launches.  Everything that touches model data runs in the kernels of this directory.
#include "../../include/netmax.h"
#include "kernels.h"
#include "layout.h"
#include "philox.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using namespace netmax;

struct netmax_ctx {
    netmax_config cfg{};
    std::vector<double> P;
    std::vector<uint8_t> adj;
    bool has_adj = false;
    hipStream_t stream = nullptr;
    int device = 0;
    // policy tables (device) and their host images
    uint32_t *d_thr = nullptr;
    int32_t *d_last = nullptr;
    float *d_w = nullptr;
    std::vector<uint32_t> h_thr;
    std::vector<int32_t> h_last;
    std::vector<float> h_w;
    // caller-owned state
    float *x_cur = nullptr, *x_next = nullptr, *v = nullptr, *g = nullptr;
    // caller-owned data and the library's scratch for the perceptron gradient
    const void *feats = nullptr;
    const int32_t *labels = nullptr;
    bool data_bound = false;
    int64_t *d_row0 = nullptr;
    int32_t *d_nrows = nullptr;
    int32_t *d_idx = nullptr;
    float *d_act[NETMAX_MAX_LAYERS + 1] = {};
    float *d_dz[2] = {};
    float *d_loss = nullptr;
    int32_t *d_flag = nullptr;
    uint16_t *d_hb[NETMAX_MAX_LAYERS + 1] = {};
    uint16_t *d_ht[NETMAX_MAX_LAYERS + 1] = {};
    uint16_t *d_dzb[2] = {}, *d_dzt[2] = {};
    int64_t woff[NETMAX_MAX_LAYERS + 1] = {};
    // consensus distance
    double *d_partial = nullptr, *d_cd = nullptr;
    // netmax_run with the update fused into the weight-gradient kernels: the tiles the separate mix still covers
    bool fuse = false;
    int32_t *d_fuse_tiles = nullptr;
    int n_fuse_tiles = 0;
    MixSkip fuse_skip{};
    // asynchronous schedule: thresholds of the activity probabilities p_i
    uint32_t *d_act_thr = nullptr;
    std::vector<uint32_t> h_act_thr;          // host image: the host plans the batches of independent steps from the same draws
    int act_last = -1;
    // perceptron gradients of a few listed workers (batches of the asynchronous schedule): compact copies
    int sub_cap = 0;                          // slots allocated
    float *d_xc = nullptr, *d_gc = nullptr, *d_lossc = nullptr;
    int64_t *d_row0c = nullptr;
    int32_t *d_nrowsc = nullptr;
    uint64_t iterations = 0;
    // small softmax-regression models: whole iterations in one kernel (k_small_iter.hip)
    bool small = false;                       // the model qualifies
    int small_resident = 0;                   // workgroups of that kernel the device holds at once (cooperative runs)
    unsigned *d_barrier = nullptr;            // grid-barrier counter, only ever advanced
    unsigned barrier_count = 0;               // its value once everything enqueued so far has run
    int *d_fault = nullptr;                   // raised by a workgroup that waited at the barrier in vain
    long long barrier_patience = 1ll << 24;   // polls before it gives up (seconds; the barrier itself takes microseconds)
    // graph replay (netmax_run): one captured iteration per direction of the parameter ping-pong
    float *x_first = nullptr;                 // the buffer bound as x_a: decides which graph an iteration uses
    uint64_t *d_iter = nullptr;               // device cell holding the iteration number of the next replay
    hipGraphExec_t graph_exec[2] = {nullptr, nullptr};
    const int32_t *graph_peers = nullptr;
    std::string err;
};

static thread_local std::string g_init_error;

static int fail(netmax_ctx *ctx, int code, const std::string &msg)
{
    if (ctx) ctx->err = msg; else g_init_error = msg;
    return code;
}

#define HIP_TRY(ctx, expr)                                                                         \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess)                                                                      \
            return fail(ctx, e_ == hipErrorOutOfMemory ? NETMAX_ENOMEM : NETMAX_EDEVICE,           \
                        std::string(#expr) + ": " + hipGetErrorString(e_));                        \
    } while (0)

// --------------------------------------------------------------------------------------------------
// Policy tables.  Row i of P becomes cumulative thresholds in 32-bit fixed point: the running sum of
// the row, scaled by 2^32 and rounded to nearest, with every position from the last positive entry on
// forced to 2^32 (stored as 2^32 - 1 together with `last`, which the sampler clamps to).  Entries of
// probability zero repeat the previous threshold and can never be drawn.
// The second-step weight is w_im = alpha rho (d_im + d_mi) / (2 p_im) (Algorithm 2), 0 for m = i; in the
// fixed-weight mode (gossip / AD-PSGD averaging under the same policy, Section III-D) it is one constant.
static int build_tables(int M, const double *P, const uint8_t *adj, double alpha, double rho, bool strict,
                        int mix_mode, double fixed_weight, std::vector<uint32_t> &thr, std::vector<int32_t> &last, std::vector<float> &w,
                        std::string &why)
{
    thr.assign((size_t)M * M, 0u);
    last.assign(M, 0);
    w.assign((size_t)M * M, 0.0f);
    // (o3) concerns Algorithm 2's weights.  Strict mode takes it with >=, as the policy generator does (links that
    // end on the bound get w = 1/2 exactly), with room for a rho that went through single precision.
    const bool strict_policy = strict && mix_mode == NETMAX_MIX_POLICY;
    const double limit = strict_policy ? 0.5 * (1.0 + 1e-6) : 1.0;
    char buf[200];
    for (int i = 0; i < M; ++i) {
        const double *row = P + (size_t)i * M;
        double total = 0.0;
        int tail = -1;
        for (int m = 0; m < M; ++m) {
            const double p = row[m];
            if (!(p >= 0.0) || !std::isfinite(p)) {
                snprintf(buf, sizeof buf, "P[%d][%d] = %g is not a probability", i, m, p);
                why = buf;
                return NETMAX_EINVAL;
            }
            if (p > 0.0) {
                tail = m;
                if (adj && m != i && !adj[(size_t)i * M + m]) {
                    snprintf(buf, sizeof buf, "P[%d][%d] > 0 but the workers are not neighbours (constraint (o4))", i, m);
                    why = buf;
                    return NETMAX_EINVAL;
                }
            }
            total += p;
        }
        if (tail < 0 || std::fabs(total - 1.0) > 1e-9) {
            snprintf(buf, sizeof buf, "row %d of P sums to %.12g, expected 1", i, total);
            why = buf;
            return NETMAX_EINVAL;
        }
        last[i] = tail;
        double running = 0.0;
        for (int m = 0; m < M; ++m) {
            running += row[m];
            uint64_t fixed;
            if (m >= tail) {
                fixed = 1ull << 32;
            } else {
                const double scaled = std::floor(std::ldexp(running, 32) + 0.5);
                fixed = scaled >= 4294967296.0 ? (1ull << 32) : (uint64_t)scaled;
            }
            thr[(size_t)i * M + m] = fixed > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)fixed;
            if (m != i && row[m] > 0.0) {
                const double links = adj ? (double)((adj[(size_t)i * M + m] != 0) + (adj[(size_t)m * M + i] != 0)) : 2.0;
                const double weight = mix_mode == NETMAX_MIX_FIXED ? fixed_weight : alpha * rho * links / (2.0 * row[m]);
                if (strict_policy ? !(weight <= limit) : !(weight < limit)) {
                    snprintf(buf, sizeof buf, "mix weight of pair (%d,%d) is %g, must be %s %g%s", i, m, weight,
                             strict_policy ? "at most" : "below", strict_policy ? 0.5 : 1.0, strict ? " (constraint (o3))" : "");
                    why = buf;
                    return NETMAX_EINFEASIBLE;
                }
                w[(size_t)i * M + m] = (float)weight;
            }
        }
    }
    return NETMAX_OK;
}

static int upload_tables(netmax_ctx *ctx)
{
    const size_t mm = (size_t)ctx->cfg.M * ctx->cfg.M;
    HIP_TRY(ctx, hipMemcpyAsync(ctx->d_thr, ctx->h_thr.data(), mm * sizeof(uint32_t), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipMemcpyAsync(ctx->d_last, ctx->h_last.data(), ctx->cfg.M * sizeof(int32_t), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipMemcpyAsync(ctx->d_w, ctx->h_w.data(), mm * sizeof(float), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return NETMAX_OK;
}

static int rebuild_policy(netmax_ctx *ctx, const double *P, double alpha, double rho)
{
    std::vector<uint32_t> thr;
    std::vector<int32_t> last;
    std::vector<float> w;
    std::string why;
    const int rc = build_tables(ctx->cfg.M, P, ctx->has_adj ? ctx->adj.data() : nullptr, alpha, rho,
                                ctx->cfg.strict_o3 != 0, ctx->cfg.mix_mode, (double)ctx->cfg.fixed_weight, thr, last, w,
                                why);
    if (rc != NETMAX_OK) return fail(ctx, rc, why);
    // the stream may still read the old tables: wait before they are overwritten
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    ctx->h_thr.swap(thr);
    ctx->h_last.swap(last);
    ctx->h_w.swap(w);
    return upload_tables(ctx);
}

static void drop_graphs(netmax_ctx *ctx)
{
    for (auto &g : ctx->graph_exec) {
        if (g) (void)hipGraphExecDestroy(g);
        g = nullptr;
    }
    ctx->graph_peers = nullptr;
}

static void release(netmax_ctx *ctx)
{
    drop_graphs(ctx);
    (void)hipFree(ctx->d_iter);
    (void)hipFree(ctx->d_thr); (void)hipFree(ctx->d_last); (void)hipFree(ctx->d_w);
    (void)hipFree(ctx->d_row0); (void)hipFree(ctx->d_nrows); (void)hipFree(ctx->d_idx);
    for (auto *p : ctx->d_act) (void)hipFree(p);
    (void)hipFree(ctx->d_dz[0]); (void)hipFree(ctx->d_dz[1]);
    (void)hipFree(ctx->d_loss); (void)hipFree(ctx->d_flag);
    for (auto *p : ctx->d_hb) (void)hipFree(p);
    for (auto *p : ctx->d_ht) (void)hipFree(p);
    for (auto *p : ctx->d_dzb) (void)hipFree(p);
    for (auto *p : ctx->d_dzt) (void)hipFree(p);
    (void)hipFree(ctx->d_partial); (void)hipFree(ctx->d_cd);
    (void)hipFree(ctx->d_act_thr); (void)hipFree(ctx->d_fuse_tiles);
    (void)hipFree(ctx->d_barrier); (void)hipFree(ctx->d_fault);
    (void)hipFree(ctx->d_xc); (void)hipFree(ctx->d_gc); (void)hipFree(ctx->d_lossc); (void)hipFree(ctx->d_row0c); (void)hipFree(ctx->d_nrowsc);
    delete ctx;
}

static int check_launch(netmax_ctx *ctx, const char *what)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, NETMAX_EDEVICE, std::string(what) + ": " + hipGetErrorString(e));
    return NETMAX_OK;
}

// --------------------------------------------------------------------------------------------------
extern "C" int netmax_init(netmax_ctx **out, const netmax_config *cfg)
{
    if (!out) return fail(nullptr, NETMAX_EINVAL, "out is NULL");
    *out = nullptr;
    if (!cfg || !cfg->P) return fail(nullptr, NETMAX_EINVAL, "cfg or cfg->P is NULL");
    char buf[200];
    if (cfg->M < 2 || cfg->M > 4096) return fail(nullptr, NETMAX_EINVAL, "M must be in 2..4096");
    static_assert(NETMAX_TILE == TILE, "the header and the kernels must agree on the tile size");
    if (cfg->D < 1 || cfg->ld < cfg->D || cfg->ld % TILE != 0)
        return fail(nullptr, NETMAX_EINVAL, "need 1 <= D <= ld and ld a multiple of NETMAX_TILE");
    if ((int64_t)cfg->M * (cfg->ld / 4) / 256 + 8 > (int64_t)0x7FFFFFFF)
        return fail(nullptr, NETMAX_EINVAL, "M * ld is too large for one launch");
    if (!(cfg->lr > 0.0f) || !(cfg->momentum >= 0.0f) || !(cfg->momentum < 1.0f) || !(cfg->weight_decay >= 0.0f) ||
        !(cfg->rho >= 0.0f))
        return fail(nullptr, NETMAX_EINVAL, "need lr > 0, 0 <= momentum < 1, weight_decay >= 0, rho >= 0");
    if (cfg->model != NETMAX_FLAT && cfg->model != NETMAX_MLP) return fail(nullptr, NETMAX_EINVAL, "unknown model kind");
    if (cfg->gemm_in != NETMAX_F32 && cfg->gemm_in != NETMAX_BF16) return fail(nullptr, NETMAX_EINVAL, "unknown gemm_in");
    if (cfg->mix_mode != NETMAX_MIX_POLICY && cfg->mix_mode != NETMAX_MIX_FIXED)
        return fail(nullptr, NETMAX_EINVAL, "unknown mix_mode");
    if (cfg->mix_mode == NETMAX_MIX_FIXED && (!(cfg->fixed_weight >= 0.0f) || !(cfg->fixed_weight < 1.0f)))
        return fail(nullptr, NETMAX_EINVAL, "fixed_weight must be in [0, 1)");

    netmax_ctx *ctx = new (std::nothrow) netmax_ctx;
    if (!ctx) return fail(nullptr, NETMAX_ENOMEM, "out of host memory");
    ctx->cfg = *cfg;
    ctx->cfg.P = nullptr;
    ctx->cfg.adj = nullptr;
    ctx->stream = (hipStream_t)cfg->stream;
    const int M = cfg->M;
    const size_t mm = (size_t)M * M;

    if (cfg->model == NETMAX_MLP) {
        if (cfg->n_layers < 1 || cfg->n_layers > NETMAX_MAX_LAYERS || cfg->batch < 1 || cfg->batch > 1024) {
            release(ctx);
            return fail(nullptr, NETMAX_EINVAL, "MLP needs 1 <= n_layers <= 7 and 1 <= batch <= 1024");
        }
        int64_t off = 0;
        for (int l = 0; l < cfg->n_layers; ++l) {
            if (cfg->dims[l] < 1 || cfg->dims[l + 1] < 1 || cfg->dims[l] > (1 << 24) || cfg->dims[l + 1] > (1 << 24)) {
                release(ctx);
                return fail(nullptr, NETMAX_EINVAL, "layer widths must be in 1..2^24");
            }
            ctx->woff[l] = off;
            off += cfg->dims[l] * cfg->dims[l + 1] + cfg->dims[l + 1];
        }
        if (off != cfg->D) {
            snprintf(buf, sizeof buf, "D = %lld does not match the layer widths (%lld parameters)", (long long)cfg->D,
                     (long long)off);
            release(ctx);
            return fail(nullptr, NETMAX_EINVAL, buf);
        }
    } else if (!(cfg->grad_sigma >= 0.0f)) {
        release(ctx);
        return fail(nullptr, NETMAX_EINVAL, "grad_sigma must be >= 0");
    }

    ctx->P.assign(cfg->P, cfg->P + mm);
    if (cfg->adj) {
        ctx->adj.assign(cfg->adj, cfg->adj + mm);
        ctx->has_adj = true;
    }
    std::string why;
    int rc = build_tables(M, ctx->P.data(), ctx->has_adj ? ctx->adj.data() : nullptr, (double)cfg->lr, (double)cfg->rho,
                          cfg->strict_o3 != 0, cfg->mix_mode, (double)cfg->fixed_weight, ctx->h_thr, ctx->h_last, ctx->h_w,
                          why);
    if (rc != NETMAX_OK) {
        release(ctx);
        return fail(nullptr, rc, why);
    }

#define INIT_TRY(expr)                                                                                         \
    do {                                                                                                       \
        hipError_t e_ = (expr);                                                                                \
        if (e_ != hipSuccess) {                                                                                \
            std::string m_ = std::string(#expr) + ": " + hipGetErrorString(e_);                                \
            release(ctx);                                                                                      \
            return fail(nullptr, e_ == hipErrorOutOfMemory ? NETMAX_ENOMEM : NETMAX_EDEVICE, m_);              \
        }                                                                                                      \
    } while (0)

    INIT_TRY(hipGetDevice(&ctx->device));
    INIT_TRY(prepare_mix());
    INIT_TRY(prepare_mix_synth());
    INIT_TRY(hipMalloc(&ctx->d_thr, mm * sizeof(uint32_t)));
    INIT_TRY(hipMalloc(&ctx->d_last, M * sizeof(int32_t)));
    INIT_TRY(hipMalloc(&ctx->d_w, mm * sizeof(float)));
    INIT_TRY(hipMalloc(&ctx->d_partial, (size_t)consensus_partials(cfg->ld) * sizeof(double)));
    INIT_TRY(hipMalloc(&ctx->d_cd, sizeof(double)));
    INIT_TRY(hipMalloc(&ctx->d_iter, sizeof(uint64_t)));
    prepare_kernels();
    if (cfg->model == NETMAX_MLP) {
        const size_t MB = (size_t)M * cfg->batch;
        int64_t widest = 0;
        for (int l = 1; l <= cfg->n_layers; ++l) {
            INIT_TRY(hipMalloc(&ctx->d_act[l], MB * cfg->dims[l] * sizeof(float)));
            if (cfg->dims[l] > widest) widest = cfg->dims[l];
        }
        INIT_TRY(hipMalloc(&ctx->d_dz[0], MB * widest * sizeof(float)));
        INIT_TRY(hipMalloc(&ctx->d_dz[1], MB * widest * sizeof(float)));
        if (cfg->gemm_in == NETMAX_BF16) {
            for (int l = 0; l < cfg->n_layers; ++l) {
                if (l > 0) INIT_TRY(hipMalloc(&ctx->d_hb[l], MB * cfg->dims[l] * sizeof(uint16_t)));
                if (l > 0) INIT_TRY(hipMalloc(&ctx->d_ht[l], MB * cfg->dims[l] * sizeof(uint16_t)));
            }
            for (int q = 0; q < 2; ++q) {
                INIT_TRY(hipMalloc(&ctx->d_dzb[q], MB * widest * sizeof(uint16_t)));
                INIT_TRY(hipMalloc(&ctx->d_dzt[q], MB * widest * sizeof(uint16_t)));
            }
        }
        INIT_TRY(hipMalloc(&ctx->d_idx, MB * sizeof(int32_t)));
        INIT_TRY(hipMalloc(&ctx->d_row0, M * sizeof(int64_t)));
        INIT_TRY(hipMalloc(&ctx->d_nrows, M * sizeof(int32_t)));
        INIT_TRY(hipMalloc(&ctx->d_loss, M * sizeof(float)));
        INIT_TRY(hipMalloc(&ctx->d_flag, sizeof(int32_t)));
        INIT_TRY(prepare_head());
        INIT_TRY(prepare_f32_layers());
        ctx->small = small_iter_ok(1, cfg->n_layers, cfg->gemm_in == NETMAX_BF16, cfg->batch, cfg->dims[0], cfg->dims[1], cfg->ld);
        if (ctx->small) {
            INIT_TRY(prepare_small_iter());
            ctx->small_resident = small_iter_max_resident(cfg->batch, cfg->dims[0], cfg->dims[1], cfg->ld);
            INIT_TRY(hipMalloc(&ctx->d_barrier, sizeof(unsigned)));
            INIT_TRY(hipMalloc(&ctx->d_fault, sizeof(int)));
            INIT_TRY(hipMemset(ctx->d_barrier, 0, sizeof(unsigned)));
            INIT_TRY(hipMemset(ctx->d_fault, 0, sizeof(int)));
        }
    }
#undef INIT_TRY
    rc = upload_tables(ctx);
    if (rc != NETMAX_OK) {
        g_init_error = ctx->err;
        release(ctx);
        return rc;
    }
    *out = ctx;
    return NETMAX_OK;
}

extern "C" int netmax_build_tables(int32_t M, const double *P, const uint8_t *adj, float lr, float rho, int32_t strict_o3,
                                   int32_t mix_mode, float fixed_weight, uint32_t *thresholds_host, int32_t *last_host,
                                   float *w_host)
{
    if (M < 2 || M > 4096 || !P || !thresholds_host || !last_host || !w_host || !(lr > 0.0f) || !(rho >= 0.0f) ||
        (mix_mode != NETMAX_MIX_POLICY && mix_mode != NETMAX_MIX_FIXED) ||
        (mix_mode == NETMAX_MIX_FIXED && (!(fixed_weight >= 0.0f) || !(fixed_weight < 1.0f))))
        return fail(nullptr, NETMAX_EINVAL, "bad argument");
    std::vector<uint32_t> thr;
    std::vector<int32_t> last;
    std::vector<float> w;
    std::string why;
    const int rc = build_tables(M, P, adj, (double)lr, (double)rho, strict_o3 != 0, mix_mode, (double)fixed_weight, thr,
                                last, w, why);
    if (rc != NETMAX_OK) return fail(nullptr, rc, why);
    memcpy(thresholds_host, thr.data(), thr.size() * sizeof(uint32_t));
    memcpy(last_host, last.data(), last.size() * sizeof(int32_t));
    memcpy(w_host, w.data(), w.size() * sizeof(float));
    return NETMAX_OK;
}

extern "C" int netmax_destroy(netmax_ctx *ctx)
{
    if (!ctx) return NETMAX_OK;
    (void)hipStreamSynchronize(ctx->stream);
    release(ctx);
    return NETMAX_OK;
}

extern "C" const char *netmax_last_error(const netmax_ctx *ctx) { return ctx ? ctx->err.c_str() : g_init_error.c_str(); }

extern "C" int netmax_set_policy(netmax_ctx *ctx, const double *P, float rho)
{
    if (!ctx) return NETMAX_EINVAL;
    if (!P || !(rho >= 0.0f)) return fail(ctx, NETMAX_EINVAL, "P is NULL or rho < 0");
    const int rc = rebuild_policy(ctx, P, (double)ctx->cfg.lr, (double)rho);
    if (rc != NETMAX_OK) return rc;
    ctx->P.assign(P, P + (size_t)ctx->cfg.M * ctx->cfg.M);
    ctx->cfg.rho = rho;
    return NETMAX_OK;
}

extern "C" int netmax_set_lr(netmax_ctx *ctx, float lr)
{
    if (!ctx) return NETMAX_EINVAL;
    if (!(lr > 0.0f)) return fail(ctx, NETMAX_EINVAL, "lr must be > 0");
    const int rc = rebuild_policy(ctx, ctx->P.data(), (double)lr, (double)ctx->cfg.rho);
    if (rc != NETMAX_OK) return rc;
    ctx->cfg.lr = lr;
    drop_graphs(ctx);                          // alpha is an argument of the captured mix kernel
    return NETMAX_OK;
}

extern "C" int netmax_bind_state(netmax_ctx *ctx, float *x_a, float *x_b, float *v, float *g)
{
    if (!ctx) return NETMAX_EINVAL;
    if (!x_a || !x_b || !v || !g) return fail(ctx, NETMAX_EINVAL, "a state pointer is NULL");
    if (x_a == x_b) return fail(ctx, NETMAX_EINVAL, "x_a and x_b must be different buffers");
    for (const void *p : {(const void *)x_a, (const void *)x_b, (const void *)v, (const void *)g})
        if ((uintptr_t)p % 16 != 0) return fail(ctx, NETMAX_EINVAL, "state pointers must be 16-byte aligned");
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    drop_graphs(ctx);
    ctx->x_cur = ctx->x_first = x_a;
    ctx->x_next = x_b;
    ctx->v = v;
    ctx->g = g;
    return NETMAX_OK;
}

// Counts labels outside [0, C): one pass over the label array, any violation raises the flag.
__global__ void __launch_bounds__(256) check_labels_kernel(int64_t n, int32_t C, const int32_t *__restrict__ labels,
                                                           int32_t *__restrict__ flag)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n && (labels[t] < 0 || labels[t] >= C)) atomicOr(flag, 1);
}

extern "C" int netmax_bind_data(netmax_ctx *ctx, const void *feats, const int32_t *labels, const int64_t *shard_off)
{
    if (!ctx) return NETMAX_EINVAL;
    if (ctx->cfg.model != NETMAX_MLP) return fail(ctx, NETMAX_ESTATE, "data can only be bound to an MLP context");
    if (!feats || !labels || !shard_off) return fail(ctx, NETMAX_EINVAL, "a data pointer is NULL");
    const int M = ctx->cfg.M;
    std::vector<int64_t> row0(M);
    std::vector<int32_t> nrows(M);
    if (shard_off[0] < 0) return fail(ctx, NETMAX_EINVAL, "shard_off[0] < 0");
    for (int i = 0; i < M; ++i) {
        const int64_t n = shard_off[i + 1] - shard_off[i];
        if (n < 1 || n > 0x7FFFFFFFLL) return fail(ctx, NETMAX_EINVAL, "every shard needs 1 .. 2^31-1 rows");
        row0[i] = shard_off[i];
        nrows[i] = (int32_t)n;
    }
    const int64_t n_total = shard_off[M];
    if (n_total > 0x7FFFFFFFLL * 256) return fail(ctx, NETMAX_EINVAL, "too many rows");
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    HIP_TRY(ctx, hipMemcpyAsync(ctx->d_row0, row0.data(), M * sizeof(int64_t), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipMemcpyAsync(ctx->d_nrows, nrows.data(), M * sizeof(int32_t), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipMemsetAsync(ctx->d_flag, 0, sizeof(int32_t), ctx->stream));
    hipLaunchKernelGGL(check_labels_kernel, dim3((unsigned)((n_total + 255) / 256)), dim3(256), 0, ctx->stream, n_total,
                       (int32_t)ctx->cfg.dims[ctx->cfg.n_layers], labels, ctx->d_flag);
    int rc = check_launch(ctx, "check_labels");
    if (rc != NETMAX_OK) return rc;
    int32_t flag = 0;
    HIP_TRY(ctx, hipMemcpyAsync(&flag, ctx->d_flag, sizeof flag, hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    if (flag) return fail(ctx, NETMAX_EINVAL, "a label is outside [0, number of classes)");
    drop_graphs(ctx);
    ctx->feats = feats;
    ctx->labels = labels;
    ctx->data_bound = true;
    return NETMAX_OK;
}

extern "C" int netmax_pack(netmax_ctx *ctx, const float *rows_dev, int64_t row_ld, float *tiled_dev)
{
    if (!ctx) return NETMAX_EINVAL;
    if (!rows_dev || !tiled_dev || row_ld < ctx->cfg.D) return fail(ctx, NETMAX_EINVAL, "NULL pointer or row_ld < D");
    launch_pack(ctx->stream, ctx->cfg.M, ctx->cfg.D, ctx->cfg.ld, rows_dev, row_ld, tiled_dev);
    return check_launch(ctx, "pack");
}

extern "C" int netmax_unpack(netmax_ctx *ctx, const float *tiled_dev, float *rows_dev, int64_t row_ld)
{
    if (!ctx) return NETMAX_EINVAL;
    if (!rows_dev || !tiled_dev || row_ld < ctx->cfg.D) return fail(ctx, NETMAX_EINVAL, "NULL pointer or row_ld < D");
    launch_unpack(ctx->stream, ctx->cfg.M, ctx->cfg.D, tiled_dev, rows_dev, row_ld);
    return check_launch(ctx, "unpack");
}

// The three phases of one iteration, enqueued on the context's stream (no argument checks, no pointer flip).
static int enqueue_sample_peers(netmax_ctx *ctx, const IterRef &iter, int32_t *peers_dev)
{
    launch_sample_peers(ctx->stream, ctx->cfg.M, ctx->d_thr, ctx->d_last, ctx->cfg.seed, iter, peers_dev);
    return check_launch(ctx, "sample_peers");
}

// Peer draw and local step of one iteration inside netmax_run: perceptrons that take the kernel-by-kernel path draw
// peers and batch rows in one launch.
static int enqueue_draws_and_local_step(netmax_ctx *ctx, const IterRef &iter, int32_t *peers_dev);

static MlpPlan make_plan(const netmax_ctx *ctx)
{
    const netmax_config &c = ctx->cfg;
    MlpPlan p{};
    p.M = c.M; p.n_layers = c.n_layers; p.B = c.batch; p.ld = c.ld; p.bf16 = (c.gemm_in == NETMAX_BF16);
    for (int l = 0; l <= c.n_layers; ++l) {
        p.dims[l] = c.dims[l]; p.woff[l] = ctx->woff[l]; p.act[l] = ctx->d_act[l];
        p.hb[l] = ctx->d_hb[l]; p.ht[l] = ctx->d_ht[l];
    }
    for (int q = 0; q < 2; ++q) { p.dzb[q] = ctx->d_dzb[q]; p.dzt[q] = ctx->d_dzt[q]; }
    p.feats = ctx->feats; p.labels = ctx->labels; p.row0 = ctx->d_row0; p.idx = ctx->d_idx;
    p.dz[0] = ctx->d_dz[0]; p.dz[1] = ctx->d_dz[1]; p.loss = ctx->d_loss;
    return p;
}

static MixArgs mix_args(const netmax_ctx *ctx, const int32_t *peers_dev)
{
    const netmax_config &c = ctx->cfg;
    return MixArgs{ctx->x_cur, ctx->v, ctx->x_next, peers_dev, ctx->d_w, c.lr, c.momentum, c.weight_decay};
}

// Small softmax-regression models: n_iters whole iterations (or, grad_only, one batch draw + loss + gradient) in one
// launch of the one-workgroup-per-worker kernel.  No pointer flip here.
static SmallIterLaunch small_launch(netmax_ctx *ctx, const IterRef &iter, int n_iters, bool grad_only, int32_t *peers_dev)
{
    const netmax_config &c = ctx->cfg;
    SmallIterLaunch a{};
    a.M = c.M; a.B = c.batch; a.din = c.dims[0]; a.dout = c.dims[1]; a.D = c.D; a.ld = c.ld;
    a.feats = (const float *)ctx->feats; a.labels = ctx->labels; a.row0 = ctx->d_row0; a.n_rows = ctx->d_nrows;
    a.thr = ctx->d_thr; a.last = ctx->d_last; a.w = ctx->d_w;
    a.x_first = ctx->x_cur; a.x_second = ctx->x_next; a.V = ctx->v; a.G = ctx->g; a.loss = ctx->d_loss;
    a.peers = peers_dev; a.idx = ctx->d_idx;
    a.alpha = c.lr; a.mu = c.momentum; a.wd = c.weight_decay; a.seed = c.seed; a.iter = iter; a.n_iters = n_iters;
    a.grad_only = grad_only ? 1 : 0;
    a.barrier = ctx->d_barrier; a.barrier_base = ctx->barrier_count; a.fault = ctx->d_fault;
    a.workers = nullptr; a.n_workers = 0;
    a.patience = ctx->barrier_patience;
    return a;
}

static int enqueue_small(netmax_ctx *ctx, const IterRef &iter, int n_iters, bool grad_only, int32_t *peers_dev, bool cooperative)
{
    const SmallIterLaunch a = small_launch(ctx, iter, n_iters, grad_only, peers_dev);
    const hipError_t e = launch_small_iter(ctx->stream, a, cooperative ? 1 : 0);
    if (e != hipSuccess) return fail(ctx, NETMAX_EDEVICE, std::string("small-model iteration kernel: ") + hipGetErrorString(e));
    if (n_iters > 1) ctx->barrier_count += (unsigned)(n_iters - 1) * (unsigned)ctx->cfg.M;
    return NETMAX_OK;
}

// fused_peers != nullptr: the matrix-core layers apply the update to their weight columns themselves (netmax_run
// after netmax_set_fusion); enqueue_mix then covers the remaining columns only.
// batch_drawn: the batch rows of this iteration are in d_idx already.
static int enqueue_local_step(netmax_ctx *ctx, const IterRef &iter, const int32_t *fused_peers = nullptr, bool batch_drawn = false)
{
    const netmax_config &c = ctx->cfg;
    if (c.model == NETMAX_FLAT) {
        if (fused_peers) return NETMAX_OK;           // the fused update generates the gradient itself
        launch_synth_grad(ctx->stream, c.M, c.D, c.ld, c.grad_sigma, c.seed, iter, ctx->g);
        return check_launch(ctx, "synth_grad");
    }
    if (ctx->small) return enqueue_small(ctx, iter, 1, true, nullptr, false);
    if (!batch_drawn) launch_sample_batch(ctx->stream, c.M, c.batch, ctx->d_nrows, c.seed, iter, ctx->d_idx);
    const MlpPlan p = make_plan(ctx);
    if (fused_peers) {
        const MixArgs mx = mix_args(ctx, fused_peers);
        launch_mlp_grad(ctx->stream, p, ctx->x_cur, ctx->g, &mx);
    } else {
        launch_mlp_grad(ctx->stream, p, ctx->x_cur, ctx->g);
    }
    return check_launch(ctx, "mlp_grad");
}

static int enqueue_draws_and_local_step(netmax_ctx *ctx, const IterRef &iter, int32_t *peers_dev)
{
    const netmax_config &c = ctx->cfg;
    const int32_t *fused_peers = ctx->fuse ? peers_dev : nullptr;
    if (c.model == NETMAX_FLAT || ctx->small) {
        const int rc = enqueue_sample_peers(ctx, iter, peers_dev);
        return rc != NETMAX_OK ? rc : enqueue_local_step(ctx, iter, fused_peers);
    }
    launch_sample_iteration(ctx->stream, c.M, ctx->d_thr, ctx->d_last, peers_dev, c.batch, ctx->d_nrows, ctx->d_idx, c.seed, iter);
    const int rc = check_launch(ctx, "sample_iteration");
    return rc != NETMAX_OK ? rc : enqueue_local_step(ctx, iter, fused_peers, true);
}

static int enqueue_mix(netmax_ctx *ctx, const int32_t *peers_dev, bool fused = false, const IterRef &iter = IterRef{0, nullptr})
{
    const netmax_config &c = ctx->cfg;
    if (fused && c.model == NETMAX_FLAT)
        launch_mix_synth(ctx->stream, c.M, c.D, c.ld, ctx->x_cur, ctx->g, ctx->v, ctx->x_next, peers_dev, ctx->d_w, c.lr,
                         c.momentum, c.weight_decay, c.grad_sigma, c.seed, iter);
    else if (fused)
        launch_mix_subset(ctx->stream, c.M, ctx->d_fuse_tiles, ctx->n_fuse_tiles, ctx->fuse_skip, ctx->x_cur, ctx->g, ctx->v,
                          ctx->x_next, peers_dev, ctx->d_w, c.lr, c.momentum, c.weight_decay);
    else
        launch_mix(ctx->stream, c.M, c.ld, ctx->x_cur, ctx->g, ctx->v, ctx->x_next, peers_dev, ctx->d_w, c.lr, c.momentum,
                   c.weight_decay);
    return check_launch(ctx, "mix");
}

static void flip(netmax_ctx *ctx)
{
    float *t = ctx->x_cur;
    ctx->x_cur = ctx->x_next;
    ctx->x_next = t;
    ctx->iterations += 1;
}

extern "C" int netmax_sample_peers(netmax_ctx *ctx, uint64_t iter, int32_t *peers_dev)
{
    if (!ctx) return NETMAX_EINVAL;
    if (!peers_dev) return fail(ctx, NETMAX_EINVAL, "peers_dev is NULL");
    return enqueue_sample_peers(ctx, IterRef{iter, nullptr}, peers_dev);
}

extern "C" int netmax_sample_batch(netmax_ctx *ctx, uint64_t iter, int32_t *idx_dev)
{
    if (!ctx) return NETMAX_EINVAL;
    if (ctx->cfg.model != NETMAX_MLP || !ctx->data_bound) return fail(ctx, NETMAX_ESTATE, "no data bound");
    if (!idx_dev) return fail(ctx, NETMAX_EINVAL, "idx_dev is NULL");
    launch_sample_batch(ctx->stream, ctx->cfg.M, ctx->cfg.batch, ctx->d_nrows, ctx->cfg.seed, IterRef{iter, nullptr}, idx_dev);
    return check_launch(ctx, "sample_batch");
}

extern "C" int netmax_local_step(netmax_ctx *ctx, uint64_t iter)
{
    if (!ctx) return NETMAX_EINVAL;
    if (!ctx->x_cur) return fail(ctx, NETMAX_ESTATE, "no state bound");
    if (ctx->cfg.model == NETMAX_MLP && !ctx->data_bound) return fail(ctx, NETMAX_ESTATE, "no data bound");
    return enqueue_local_step(ctx, IterRef{iter, nullptr});
}

extern "C" int netmax_mix(netmax_ctx *ctx, uint64_t iter, const int32_t *peers_dev)
{
    if (!ctx) return NETMAX_EINVAL;
    if (!ctx->x_cur) return fail(ctx, NETMAX_ESTATE, "no state bound");
    if (!peers_dev) return fail(ctx, NETMAX_EINVAL, "peers_dev is NULL");
    (void)iter;
    const int rc = enqueue_mix(ctx, peers_dev);
    if (rc != NETMAX_OK) return rc;
    flip(ctx);
    return NETMAX_OK;
}

// One iteration (sample, local step, mix, advance the iteration cell) recorded into a HIP graph for the
// current direction of the parameter ping-pong.  Every kernel argument is fixed: the iteration number is read
// from the device cell.
static int capture_iteration(netmax_ctx *ctx, int dir, int32_t *peers_dev)
{
    hipGraph_t graph = nullptr;
    HIP_TRY(ctx, hipStreamBeginCapture(ctx->stream, hipStreamCaptureModeThreadLocal));
    const IterRef it{0, ctx->d_iter};
    int rc;
    if (ctx->small && !ctx->fuse) {
        rc = enqueue_small(ctx, it, 1, false, peers_dev, false);
    } else {
        rc = enqueue_draws_and_local_step(ctx, it, peers_dev);
        if (rc == NETMAX_OK) rc = enqueue_mix(ctx, peers_dev, ctx->fuse, it);
    }
    if (rc == NETMAX_OK) {
        launch_bump_iteration(ctx->stream, ctx->d_iter);
        rc = check_launch(ctx, "bump_iteration");
    }
    const hipError_t e = hipStreamEndCapture(ctx->stream, &graph);
    if (rc != NETMAX_OK) {
        if (graph) (void)hipGraphDestroy(graph);
        return rc;
    }
    if (e != hipSuccess) return fail(ctx, NETMAX_EDEVICE, std::string("hipStreamEndCapture: ") + hipGetErrorString(e));
    const hipError_t ei = hipGraphInstantiate(&ctx->graph_exec[dir], graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (ei != hipSuccess) {
        ctx->graph_exec[dir] = nullptr;
        return fail(ctx, NETMAX_EDEVICE, std::string("hipGraphInstantiate: ") + hipGetErrorString(ei));
    }
    return NETMAX_OK;
}

extern "C" int netmax_run(netmax_ctx *ctx, uint64_t first_iter, int32_t n_iters, int32_t *peers_dev, int32_t use_graph)
{
    if (!ctx) return NETMAX_EINVAL;
    if (!ctx->x_cur) return fail(ctx, NETMAX_ESTATE, "no state bound");
    if (ctx->cfg.model == NETMAX_MLP && !ctx->data_bound) return fail(ctx, NETMAX_ESTATE, "no data bound");
    if (!peers_dev || n_iters < 0) return fail(ctx, NETMAX_EINVAL, "peers_dev is NULL or n_iters < 0");
    if (!use_graph && ctx->small && !ctx->fuse) {
        // whole iterations inside one kernel; as many per launch as a cooperative launch allows (all workgroups
        // resident), else one launch per iteration
        const bool coop = ctx->small_resident >= ctx->cfg.M;
        int32_t k = 0;
        while (k < n_iters) {
            const int32_t n = coop ? std::min<int32_t>(n_iters - k, 1 << 20) : 1;
            const int rc = enqueue_small(ctx, IterRef{first_iter + (uint64_t)k, nullptr}, n, false, peers_dev, coop && n > 1);
            if (rc != NETMAX_OK) return rc;
            for (int32_t q = 0; q < n; ++q) flip(ctx);
            k += n;
        }
        return NETMAX_OK;
    }
    if (!use_graph) {
        for (int32_t k = 0; k < n_iters; ++k) {
            const IterRef it{first_iter + (uint64_t)k, nullptr};
            int rc = enqueue_draws_and_local_step(ctx, it, peers_dev);
            if (rc == NETMAX_OK) rc = enqueue_mix(ctx, peers_dev, ctx->fuse, it);
            if (rc != NETMAX_OK) return rc;
            flip(ctx);
        }
        return NETMAX_OK;
    }
    if (!ctx->stream) return fail(ctx, NETMAX_ESTATE, "graph replay needs a non-default stream (the null stream cannot be captured)");
    if (ctx->graph_peers != peers_dev) drop_graphs(ctx);
    launch_set_iteration(ctx->stream, ctx->d_iter, first_iter);
    int rc = check_launch(ctx, "set_iteration");
    if (rc != NETMAX_OK) return rc;
    for (int32_t k = 0; k < n_iters; ++k) {
        const int dir = ctx->x_cur == ctx->x_first ? 0 : 1;
        if (!ctx->graph_exec[dir]) {
            rc = capture_iteration(ctx, dir, peers_dev);
            if (rc != NETMAX_OK) return rc;
            ctx->graph_peers = peers_dev;
        }
        HIP_TRY(ctx, hipGraphLaunch(ctx->graph_exec[dir], ctx->stream));
        flip(ctx);
    }
    return NETMAX_OK;
}

// ---- the update fused into the weight-gradient kernels ---------------------------------------------------

extern "C" int netmax_set_fusion(netmax_ctx *ctx, int32_t on)
{
    if (!ctx) return NETMAX_EINVAL;
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    drop_graphs(ctx);
    if (!on) { ctx->fuse = false; return NETMAX_OK; }
    const netmax_config &c = ctx->cfg;
    if (c.model == NETMAX_FLAT) {                    // the gradient generator moves into the update kernel
        ctx->fuse = true;
        return NETMAX_OK;
    }
    const MlpPlan p = make_plan(ctx);
    MixSkip skip{};
    for (int l = 0; l < c.n_layers; ++l)
        if (mfma_layer_ok(p, l)) {
            if (skip.n == MIX_MAX_SKIP) return fail(ctx, NETMAX_ESTATE, "too many layers");
            skip.lo[skip.n] = ctx->woff[l];
            skip.hi[skip.n] = ctx->woff[l] + (int64_t)c.dims[l] * c.dims[l + 1];
            ++skip.n;
        }
    if (skip.n == 0) return fail(ctx, NETMAX_ESTATE, "no layer of this model runs on the matrix-core kernels");
    // tiles with at least one column outside the ranges (four columns at a time, as the kernel tests them)
    std::vector<int32_t> tiles;
    const int64_t n_tiles = c.ld / NETMAX_TILE;
    for (int64_t t = 0; t < n_tiles; ++t) {
        const int64_t lo = t * NETMAX_TILE, hi = lo + NETMAX_TILE;
        bool covered = false;
        for (int r = 0; r < skip.n; ++r) covered |= (skip.lo[r] <= lo && hi <= skip.hi[r]);
        if (!covered) tiles.push_back((int32_t)t);
    }
    (void)hipFree(ctx->d_fuse_tiles);
    ctx->d_fuse_tiles = nullptr;
    if (!tiles.empty()) {
        HIP_TRY(ctx, hipMalloc(&ctx->d_fuse_tiles, tiles.size() * sizeof(int32_t)));
        HIP_TRY(ctx, hipMemcpy(ctx->d_fuse_tiles, tiles.data(), tiles.size() * sizeof(int32_t), hipMemcpyHostToDevice));
    }
    ctx->n_fuse_tiles = (int)tiles.size();
    ctx->fuse_skip = skip;
    ctx->fuse = true;
    return NETMAX_OK;
}

// ---- asynchronous schedule ---------------------------------------------------------------------------

extern "C" int netmax_activity(int32_t M, const double *t_host, const double *P_host, const uint8_t *adj, double *p_act_out)
{
    if (M < 1 || !t_host || !P_host || !p_act_out) return NETMAX_EINVAL;
    double total = 0.0;
    for (int i = 0; i < M; ++i) {
        double tbar = 0.0;                                   // Eq. (d3); d_ii = 0
        for (int m = 0; m < M; ++m)
            if (m != i && (!adj || adj[(size_t)i * M + m])) tbar += t_host[(size_t)i * M + m] * P_host[(size_t)i * M + m];
        if (!(tbar > 0.0) || !std::isfinite(tbar)) return NETMAX_EINVAL;
        p_act_out[i] = 1.0 / tbar;
        total += p_act_out[i];
    }
    for (int i = 0; i < M; ++i) p_act_out[i] /= total;       // Eq. (d4)
    return NETMAX_OK;
}

extern "C" int netmax_mean_times(int32_t M, const double *t_host, const double *P_host, const uint8_t *adj, double *tbar_out,
                                 double *rate_out)
{
    if (M < 1 || !t_host || !P_host || !tbar_out) return NETMAX_EINVAL;
    double rate = 0.0;
    for (int i = 0; i < M; ++i) {
        double tbar = 0.0;                                   // Eq. (d3); d_ii = 0
        for (int m = 0; m < M; ++m)
            if (m != i && (!adj || adj[(size_t)i * M + m])) tbar += t_host[(size_t)i * M + m] * P_host[(size_t)i * M + m];
        if (!(tbar > 0.0) || !std::isfinite(tbar)) return NETMAX_EINVAL;
        tbar_out[i] = tbar;
        rate += 1.0 / tbar;                                  // the normaliser of Eq. (d4)
    }
    if (rate_out) *rate_out = rate;
    return NETMAX_OK;
}

extern "C" int netmax_set_activity(netmax_ctx *ctx, const double *p_act)
{
    if (!ctx) return NETMAX_EINVAL;
    if (!p_act) return fail(ctx, NETMAX_EINVAL, "p_act is NULL");
    const int M = ctx->cfg.M;
    double total = 0.0;
    int tail = -1;
    for (int i = 0; i < M; ++i) {
        if (!(p_act[i] >= 0.0) || !std::isfinite(p_act[i])) return fail(ctx, NETMAX_EINVAL, "an activity probability is negative or not finite");
        if (p_act[i] > 0.0) tail = i;
        total += p_act[i];
    }
    if (tail < 0 || std::fabs(total - 1.0) > 1e-9) return fail(ctx, NETMAX_EINVAL, "the activity probabilities do not sum to 1");
    std::vector<uint32_t> thr(M);
    double running = 0.0;
    for (int i = 0; i < M; ++i) {                            // the same fixed-point thresholds as a policy row
        running += p_act[i];
        uint64_t fixed;
        if (i >= tail) {
            fixed = 1ull << 32;
        } else {
            const double scaled = std::floor(std::ldexp(running, 32) + 0.5);
            fixed = scaled >= 4294967296.0 ? (1ull << 32) : (uint64_t)scaled;
        }
        thr[i] = fixed > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)fixed;
    }
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));         // a running step may still read the old thresholds
    if (!ctx->d_act_thr) HIP_TRY(ctx, hipMalloc(&ctx->d_act_thr, (size_t)M * sizeof(uint32_t)));
    HIP_TRY(ctx, hipMemcpy(ctx->d_act_thr, thr.data(), (size_t)M * sizeof(uint32_t), hipMemcpyHostToDevice));
    ctx->h_act_thr = thr;
    ctx->act_last = tail;
    return NETMAX_OK;
}

// Number of thresholds <= u, clamped to the last positive entry: the draw of the kernels, on the host.
static int host_draw(const uint32_t *row, int n, int last, uint32_t u)
{
    const int pos = (int)(std::upper_bound(row, row + n, u) - row);
    return pos < last ? pos : last;
}

constexpr int ASYNC_MAX_BATCH = 32;

// The gradients of the n listed workers (device list `workers`, consecutive global steps from k0) into the compact
// matrix d_gc: their rows and shard descriptors are gathered, the grouped kernels run on n groups.
static int enqueue_subset_gradient(netmax_ctx *ctx, const int32_t *workers, int n, uint64_t k0)
{
    const netmax_config &c = ctx->cfg;
    if (!ctx->sub_cap) {
        const int cap = std::min<int>(c.M, ASYNC_MAX_BATCH);
        HIP_TRY(ctx, hipMalloc(&ctx->d_xc, (size_t)cap * c.ld * sizeof(float)));
        HIP_TRY(ctx, hipMalloc(&ctx->d_gc, (size_t)cap * c.ld * sizeof(float)));
        HIP_TRY(ctx, hipMalloc(&ctx->d_lossc, (size_t)cap * sizeof(float)));
        HIP_TRY(ctx, hipMalloc(&ctx->d_row0c, (size_t)cap * sizeof(int64_t)));
        HIP_TRY(ctx, hipMalloc(&ctx->d_nrowsc, (size_t)cap * sizeof(int32_t)));
        ctx->sub_cap = cap;
    }
    launch_gather_shards(ctx->stream, c.M, n, workers, ctx->d_row0, ctx->d_nrows, ctx->d_row0c, ctx->d_nrowsc);
    launch_sample_batch_subset(ctx->stream, n, c.batch, workers, ctx->d_nrowsc, c.seed, k0, ctx->d_idx);
    launch_gather_rows(ctx->stream, c.M, n, c.ld, workers, ctx->x_cur, ctx->d_xc);
    MlpPlan p = make_plan(ctx);
    p.M = n;
    p.row0 = ctx->d_row0c;
    p.loss = ctx->d_lossc;
    launch_mlp_grad(ctx->stream, p, ctx->d_xc, ctx->d_gc);
    launch_scatter_loss(ctx->stream, c.M, n, workers, ctx->d_lossc, ctx->d_loss);
    return check_launch(ctx, "subset gradient");
}

extern "C" int netmax_async_run(netmax_ctx *ctx, uint64_t first_step, uint64_t n_steps, int32_t *active_dev, int32_t *peers_dev)
{
    if (!ctx) return NETMAX_EINVAL;
    if (!active_dev || !peers_dev) return fail(ctx, NETMAX_EINVAL, "active_dev or peers_dev is NULL");
    if (n_steps > (1ull << 31)) return fail(ctx, NETMAX_EINVAL, "more than 2^31 steps in one call");
    if (!ctx->x_cur) return fail(ctx, NETMAX_ESTATE, "netmax_bind_state has not been called");
    if (ctx->act_last < 0) return fail(ctx, NETMAX_ESTATE, "netmax_set_activity has not been called");
    const netmax_config &c = ctx->cfg;
    if (c.model == NETMAX_MLP && !ctx->data_bound) return fail(ctx, NETMAX_ESTATE, "netmax_bind_data has not been called");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    if (n_steps == 0) return NETMAX_OK;
    launch_async_draw(ctx->stream, c.M, ctx->d_act_thr, ctx->act_last, ctx->d_thr, ctx->d_last, c.seed, first_step, n_steps,
                      active_dev, peers_dev);
    int rc = check_launch(ctx, "async_draw");
    // The host repeats the draws (integer work on the same tables) and cuts the run into batches of consecutive
    // steps that cannot see each other: a step joins the batch unless its active worker was active or pulled
    // from earlier in the batch, or it pulls from a worker that was active.  A batch is one set of launches.
    const int cap = std::min<int>(c.M, ASYNC_MAX_BATCH);
    std::vector<uint8_t> wrote(c.M, 0), read(c.M, 0);
    std::vector<int> touched;
    uint64_t s0 = 0;
    while (s0 < n_steps && rc == NETMAX_OK) {
        int n = 0;
        touched.clear();
        while (s0 + n < n_steps && n < cap) {
            const uint64_t k = first_step + s0 + n;
            const int i = host_draw(ctx->h_act_thr.data(), c.M, ctx->act_last, draw_block(c.seed, STREAM_ACTIVE, 0u, 0u, k).a);
            const int m = host_draw(ctx->h_thr.data() + (size_t)i * c.M, c.M, ctx->h_last[i],
                                    draw_block(c.seed, STREAM_PEER, 0u, (uint32_t)i, k).a);
            if (n > 0 && (wrote[i] || read[i] || wrote[m])) break;
            wrote[i] = 1;
            read[m] = 1;
            touched.push_back(i);
            touched.push_back(m);
            ++n;
        }
        for (int q : touched) wrote[q] = read[q] = 0;
        const uint64_t k0 = first_step + s0;
        int source = 0;
        if (c.model == NETMAX_MLP) {
            if (ctx->small) {
                SmallIterLaunch a = small_launch(ctx, IterRef{k0, nullptr}, 1, true, nullptr);
                a.workers = active_dev + s0;
                a.n_workers = n;
                const hipError_t e = launch_small_iter(ctx->stream, a, 0);
                if (e != hipSuccess) return fail(ctx, NETMAX_EDEVICE, std::string("small-model gradient kernel: ") + hipGetErrorString(e));
                source = 1;
            } else {
                rc = enqueue_subset_gradient(ctx, active_dev + s0, n, k0);
                if (rc != NETMAX_OK) break;
                source = 2;
            }
        }
        launch_async_rows(ctx->stream, source, c.M, c.D, c.ld, ctx->x_cur, ctx->v, ctx->g, ctx->d_gc, n, active_dev + s0,
                          peers_dev + s0, ctx->d_w, c.lr, c.momentum, c.weight_decay, c.grad_sigma, c.seed, k0);
        rc = check_launch(ctx, "async_rows");
        s0 += (uint64_t)n;
    }
    if (rc == NETMAX_OK) ctx->iterations = first_step + n_steps;
    return rc;
}

extern "C" int netmax_update_times(netmax_ctx *ctx, const int32_t *peers_dev, const float *t_dev, float beta,
                                   float *ema_dev, float *clock_dev)
{
    if (!ctx) return NETMAX_EINVAL;
    if (!peers_dev || !t_dev || !ema_dev || !(beta >= 0.0f) || !(beta <= 1.0f))
        return fail(ctx, NETMAX_EINVAL, "NULL pointer or beta outside [0, 1]");
    launch_update_times(ctx->stream, ctx->cfg.M, peers_dev, t_dev, beta, ema_dev, clock_dev);
    return check_launch(ctx, "update_times");
}

extern "C" int netmax_update_times_async(netmax_ctx *ctx, const int32_t *active_dev, const int32_t *peers_dev, uint64_t n_steps,
                                         const float *t_dev, float beta, float *ema_dev, float *clock_dev)
{
    if (!ctx) return NETMAX_EINVAL;
    if (!active_dev || !peers_dev || !t_dev || !ema_dev || !(beta >= 0.0f) || !(beta <= 1.0f) || n_steps > (1ull << 31))
        return fail(ctx, NETMAX_EINVAL, "NULL pointer, beta outside [0, 1] or more than 2^31 steps");
    if (n_steps == 0) return NETMAX_OK;
    launch_async_times(ctx->stream, ctx->cfg.M, (int64_t)n_steps, active_dev, peers_dev, t_dev, beta, ema_dev, clock_dev);
    return check_launch(ctx, "update_times_async");
}

extern "C" int netmax_consensus_dist(netmax_ctx *ctx, double *out_host)
{
    if (!ctx) return NETMAX_EINVAL;
    if (!ctx->x_cur) return fail(ctx, NETMAX_ESTATE, "no state bound");
    if (!out_host) return fail(ctx, NETMAX_EINVAL, "out_host is NULL");
    const netmax_config &c = ctx->cfg;
    launch_consensus(ctx->stream, c.M, c.D, c.ld, ctx->x_cur, ctx->d_partial, ctx->d_cd);
    const int rc = check_launch(ctx, "consensus");
    if (rc != NETMAX_OK) return rc;
    HIP_TRY(ctx, hipMemcpyAsync(out_host, ctx->d_cd, sizeof(double), hipMemcpyDeviceToHost, ctx->stream));
    int fault = 0;
    if (ctx->d_fault) HIP_TRY(ctx, hipMemcpyAsync(&fault, ctx->d_fault, sizeof fault, hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    if (fault) return fail(ctx, NETMAX_EDEVICE, "a multi-iteration launch of netmax_run lost its grid barrier: the parameters are not valid");
    return NETMAX_OK;
}

// ---- consensus distance without any allocation ------------------------------------------------------------
// The partial sums live in a fixed device array.  In host code the array's name is only a handle for the symbol
// lookup: its device address differs per GPU, is asked for once per device and kept; kernels get that address.
static_assert((int64_t)NETMAX_STATIC_PARTIALS * CONSENSUS_COLS == NETMAX_STATIC_MAX_LD, "header limits must agree");
static __device__ __align__(256) double scratch[NETMAX_STATIC_PARTIALS];

constexpr int STATIC_MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static double *g_scratch_ptr[STATIC_MAX_DEVICES] = {};

// Device address of `scratch` on the current device (looked up on the first call per device).
static int scratch_of_current_device(double **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(nullptr, NETMAX_EDEVICE, std::string("hipGetDevice: ") + hipGetErrorString(e));
    if (dev < 0 || dev >= STATIC_MAX_DEVICES) return fail(nullptr, NETMAX_EDEVICE, "device index out of range");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(nullptr, NETMAX_EDEVICE, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
        g_scratch_ptr[dev] = (double *)p;
    }
    *out = g_scratch_ptr[dev];
    return NETMAX_OK;
}

extern "C" int netmax_consensus_dist_static(int32_t M, int64_t D, int64_t ld, const float *x_dev, double *cd_dev, void *stream)
{
    if (!x_dev || !cd_dev) return fail(nullptr, NETMAX_EINVAL, "x_dev or cd_dev is NULL");
    if (M < 2 || M > 4096) return fail(nullptr, NETMAX_EINVAL, "M must be in 2..4096");
    if (D < 1 || ld < D || ld % TILE != 0) return fail(nullptr, NETMAX_EINVAL, "need 1 <= D <= ld and ld a multiple of NETMAX_TILE");
    if ((uintptr_t)x_dev % 16 != 0 || (uintptr_t)cd_dev % 8 != 0) return fail(nullptr, NETMAX_EINVAL, "x_dev must be 16-byte and cd_dev 8-byte aligned");
    if (ld > NETMAX_STATIC_MAX_LD || consensus_partials(ld) > NETMAX_STATIC_PARTIALS) {
        char buf[160];
        snprintf(buf, sizeof buf, "ld = %lld exceeds NETMAX_STATIC_MAX_LD = %lld columns (the fixed scratch array)",
                 (long long)ld, (long long)NETMAX_STATIC_MAX_LD);
        return fail(nullptr, NETMAX_EINVAL, buf);
    }
    double *partial = nullptr;
    const int rc = scratch_of_current_device(&partial);
    if (rc != NETMAX_OK) return rc;
    launch_consensus((hipStream_t)stream, M, D, ld, x_dev, partial, cd_dev);
    return check_launch(nullptr, "consensus (static scratch)");
}

extern "C" int netmax_set_barrier_patience(netmax_ctx *ctx, int64_t polls)
{
    if (!ctx) return NETMAX_EINVAL;
    if (polls < 0) return fail(ctx, NETMAX_EINVAL, "polls must be >= 0");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    ctx->barrier_patience = polls;
    if (ctx->d_fault) HIP_TRY(ctx, hipMemset(ctx->d_fault, 0, sizeof(int)));
    return NETMAX_OK;
}

extern "C" const float *netmax_params(const netmax_ctx *ctx) { return ctx ? ctx->x_cur : nullptr; }
extern "C" const float *netmax_losses(const netmax_ctx *ctx) { return ctx ? ctx->d_loss : nullptr; }

extern "C" int netmax_read_losses(netmax_ctx *ctx, float *out_dev)
{
    if (!ctx) return NETMAX_EINVAL;
    if (ctx->cfg.model != NETMAX_MLP) return fail(ctx, NETMAX_ESTATE, "only perceptron models have losses");
    if (!out_dev) return fail(ctx, NETMAX_EINVAL, "out_dev is NULL");
    HIP_TRY(ctx, hipMemcpyAsync(out_dev, ctx->d_loss, (size_t)ctx->cfg.M * sizeof(float), hipMemcpyDeviceToDevice, ctx->stream));
    return NETMAX_OK;
}

extern "C" int netmax_read_hidden(netmax_ctx *ctx, int32_t layer, float *out_dev)
{
    if (!ctx) return NETMAX_EINVAL;
    const netmax_config &c = ctx->cfg;
    if (c.model != NETMAX_MLP) return fail(ctx, NETMAX_ESTATE, "only perceptron models have hidden layers");
    if (layer < 1 || layer >= c.n_layers) return fail(ctx, NETMAX_EINVAL, "layer must be in 1 .. n_layers - 1");
    if (!out_dev) return fail(ctx, NETMAX_EINVAL, "out_dev is NULL");
    const int64_t n = (int64_t)c.M * c.batch * c.dims[layer];
    if (c.gemm_in == NETMAX_BF16) {
        launch_widen_bf16(ctx->stream, n, ctx->d_hb[layer], out_dev);
        return check_launch(ctx, "read_hidden");
    }
    HIP_TRY(ctx, hipMemcpyAsync(out_dev, ctx->d_act[layer], (size_t)n * sizeof(float), hipMemcpyDeviceToDevice, ctx->stream));
    return NETMAX_OK;
}

extern "C" uint64_t netmax_iteration(const netmax_ctx *ctx) { return ctx ? ctx->iterations : 0; }

extern "C" int netmax_get_tables(netmax_ctx *ctx, uint32_t *thresholds_host, int32_t *last_host, float *w_host)
{
    if (!ctx) return NETMAX_EINVAL;
    const size_t mm = (size_t)ctx->cfg.M * ctx->cfg.M;
    // read back what the device holds, so the caller sees the tables the kernels use
    if (thresholds_host) HIP_TRY(ctx, hipMemcpyAsync(thresholds_host, ctx->d_thr, mm * sizeof(uint32_t), hipMemcpyDeviceToHost, ctx->stream));
    if (last_host) HIP_TRY(ctx, hipMemcpyAsync(last_host, ctx->d_last, ctx->cfg.M * sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream));
    if (w_host) HIP_TRY(ctx, hipMemcpyAsync(w_host, ctx->d_w, mm * sizeof(float), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return NETMAX_OK;
}
