/*
 * CPU oracle of one NetMax iteration over M worker model copies.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * tests, the smoke check and the benchmark's CPU-baseline leg compare the GPU
 * library against.  It shares no code with the GPU library and nothing in the
 * product path may call it.
 *
 * What it follows (NetMax paper, arXiv 2009.05766):
 *   - Algorithm 2 ("NetMax at worker node i"): draw a peer m with probability
 *     p_im, first-step update with the local gradient, second-step update with
 *     the pulled peer model;
 *   - Section IV, Eq. (c0)/(c1): x_i^{k+1/2} = x_i^k - alpha g_i^k and
 *     x_i^{k+1} = x_i^{k+1/2} - alpha rho gamma_im (x_i^{k+1/2} - x_m^k), with
 *     gamma_im = (d_im + d_mi) / (2 p_im) as defined just before Eq. (c0);
 *   - Section V-A "Configurations": momentum SGD (momentum 0.9, weight decay) as
 *     the first-step optimiser;
 *   - Eq. (1): the pairwise model-difference penalty, whose complete-graph form
 *     is the consensus distance returned here;
 *   - Section II-B, Eq. (c2)-(c4), (d3), (d4): the asynchronous schedule with one
 *     active worker per global step (ora_activity, ora_async_draw,
 *     ora_async_apply);
 *   - Algorithm 2, UpdateTimeVector: smoothed iteration times (ora_update_times).
 * In the synchronous functions all M workers step once per iteration and read
 * the copies of the previous iteration (the pulled x_m is the peer's copy from
 * before its own update).
 *
 * Arithmetic: state is stored as float; every element of a result is computed
 * in double from the float inputs and rounded to float once.  Integer work
 * (thresholds, Philox, peer and batch indices) is exact.
 *
 * Pins (tests/test_oracle_*.py): Philox known answers; threshold row sums and
 * boundary sweeps; chi-square of peer draws; two-step form == convex form;
 * fixed point of identical copies; M=2 closed forms; expectation over the peer
 * draw == one step of Eq. (a4)/(a5); single active worker == D^k of Eq. (c4);
 * momentum apply == torch.optim.SGD; gradients == finite differences and
 * torch.autograd (fp64); consensus distance == brute-force pair sum; smoothed
 * times == geometric closed form; asynchronous step == the active worker's row
 * of the synchronous step == D^k (x - alpha g), draw frequencies, one-step
 * second moment == x^T Y_P x of Eq. (d2).
 * Full trajectories of the five synthetic workloads have no published values:
 * parity unpinned in absolute terms for those (GPU vs oracle only).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 1;

/* Number of host threads the per-worker loops use (1 = single-threaded). Returns what is in effect. */
int ora_set_threads(int n)
{
#ifdef _OPENMP
    if (n < 1) n = 1;
    g_threads = n;
#else
    (void)n;
    g_threads = 1;
#endif
    return g_threads;
}

/* ------------------------------------------------------------------ Philox4x32-10
 * Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3" (SC'11).
 * Counter 4 x u32, key 2 x u32, ten rounds; the key is bumped by the Weyl
 * constants before every round but the first. */
void ora_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        if (r > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Draws of the method: key = (seed_lo, seed_hi ^ stream), counter = (blk, worker, iter_lo, iter_hi).
 * stream 0: peer choice, 1: batch indices, 2: synthetic gradient. */
static void draw(uint64_t seed, uint32_t stream, uint32_t blk, uint32_t worker, uint64_t iter, uint32_t out[4])
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) ^ stream };
    uint32_t ctr[4] = { blk, worker, (uint32_t)iter, (uint32_t)(iter >> 32) };
    ora_philox4x32_10(ctr, key, out);
}

/* ------------------------------------------------------------------ policy tables
 * Row i of P (Section II-B "Probability": p_im is the probability that worker i
 * selects m) becomes 32-bit fixed-point cumulative thresholds:
 *   C[m] = round(2^32 * sum_{j<=m} p_ij), forced to 2^32 from the last positive
 *   entry on, stored clamped to 2^32-1.
 * Returns 0, or 1 if a row has a negative entry, no positive entry, or a sum
 * that is off 1 by more than 1e-9. */
int ora_thresholds(int M, const double *P, uint32_t *T, int32_t *last)
{
    for (int i = 0; i < M; ++i) {
        const double *p = P + (size_t)i * M;
        int l = -1;
        double c = 0.0;
        for (int m = 0; m < M; ++m) {
            if (!(p[m] >= 0.0)) return 1;
            if (p[m] > 0.0) l = m;
            c += p[m];
        }
        if (l < 0 || fabs(c - 1.0) > 1e-9) return 1;
        last[i] = l;
        c = 0.0;
        for (int m = 0; m < M; ++m) {
            c += p[m];
            double s = floor(c * 4294967296.0 + 0.5);
            uint64_t C = s >= 4294967296.0 ? 4294967296ull : (uint64_t)s;
            if (m >= l) C = 4294967296ull;
            T[(size_t)i * M + m] = C > 4294967295ull ? 4294967295u : (uint32_t)C;
        }
    }
    return 0;
}

/* Peer of a uniform 32-bit word u: the first m whose cumulative threshold exceeds u. */
int32_t ora_peer_of_word(int M, const uint32_t *Trow, int32_t last, uint32_t u)
{
    int32_t m = 0;
    while (m < M && Trow[m] <= u) ++m;
    return m < last ? m : last;
}

/* Algorithm 2, "select a neighbor m with probability p_im": one draw per worker and iteration. */
void ora_sample_peers(int M, const uint32_t *T, const int32_t *last, uint64_t seed, uint64_t iter, int32_t *peer)
{
    for (int i = 0; i < M; ++i) {
        uint32_t r[4];
        draw(seed, 0u, 0u, (uint32_t)i, iter, r);
        peer[i] = ora_peer_of_word(M, T + (size_t)i * M, last[i], r[0]);
    }
}

/* Second-step weight of Algorithm 2 / Eq. (c1): w_im = alpha rho (d_im + d_mi) / (2 p_im);
 * 0 on the diagonal (a worker that draws itself only takes its local step) and where p_im = 0.
 * adj may be NULL: complete graph without self loops. */
void ora_mix_weights(int M, const double *P, const uint8_t *adj, double alpha, double rho, double *w)
{
    for (int i = 0; i < M; ++i)
        for (int m = 0; m < M; ++m) {
            double p = P[(size_t)i * M + m];
            double dim = adj ? (double)(adj[(size_t)i * M + m] != 0) : 1.0;
            double dmi = adj ? (double)(adj[(size_t)m * M + i] != 0) : 1.0;
            w[(size_t)i * M + m] = (m == i || p <= 0.0) ? 0.0 : alpha * rho * (dim + dmi) / (2.0 * p);
        }
}

/* The fixed-weight variant: the gossip / AD-PSGD update that Section III-D and Section V-H run under the same
 * peer-selection policy uses one weight for every pulled model (1/2 = plain averaging of the two copies). */
void ora_mix_weights_fixed(int M, const double *P, double weight, double *w)
{
    for (int i = 0; i < M; ++i)
        for (int m = 0; m < M; ++m)
            w[(size_t)i * M + m] = (m == i || P[(size_t)i * M + m] <= 0.0) ? 0.0 : weight;
}

/* ------------------------------------------------------------------ batch indices
 * "sampled dataset D_{i,n} from D_i" (Eq. (a5)): B draws with replacement from the
 * worker's shard; draw b uses word b%4 of block b/4 of stream 1 and maps it to
 * floor(u * n_i / 2^32). idx is [M][B], local to the shard. */
void ora_sample_batch(int M, int B, const int64_t *shard_off, uint64_t seed, uint64_t iter, int32_t *idx)
{
    for (int i = 0; i < M; ++i) {
        uint64_t n = (uint64_t)(shard_off[i + 1] - shard_off[i]);
        for (int b = 0; b < B; ++b) {
            uint32_t r[4];
            draw(seed, 1u, (uint32_t)(b / 4), (uint32_t)i, iter, r);
            idx[(size_t)i * B + b] = (int32_t)(((uint64_t)r[b % 4] * n) >> 32);
        }
    }
}

/* ------------------------------------------------------------------ synthetic gradient
 * g[i][j] = sigma * N(0,1) (stands in for a CNN's stochastic gradient, cf. the additive-noise
 * assumption of Section IV).  Block j/4 of stream 2 gives four words; u = ((word >> 9) + 0.5) 2^-23,
 * a 24-bit value strictly inside (0,1) that single precision also holds exactly;
 * Box-Muller on (u0,u1) gives elements j, j+1 and on (u2,u3) elements j+2, j+3. Columns >= D are 0.
 * G holds the window of columns col0 .. col0+ld-1 of the full matrix (col0 a multiple of 4; 0 = whole rows);
 * D counts valid columns inside the window. */
void ora_synth_grad(int M, int64_t D, int64_t ld, int64_t col0, double sigma, uint64_t seed, uint64_t iter, float *G)
{
    const double two_pi = 6.283185307179586476925286766559;
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int i = 0; i < M; ++i) {
        float *g = G + (size_t)i * ld;
        for (int64_t j0 = 0; j0 < ld; j0 += 4) {
            uint32_t r[4];
            double z[4];
            draw(seed, 2u, (uint32_t)((col0 + j0) / 4), (uint32_t)i, iter, r);
            for (int h = 0; h < 2; ++h) {
                double u0 = ((double)(r[2 * h] >> 9) + 0.5) * (1.0 / 8388608.0);
                double u1 = ((double)(r[2 * h + 1] >> 9) + 0.5) * (1.0 / 8388608.0);
                double rad = sqrt(-2.0 * log(u0));
                z[2 * h] = rad * cos(two_pi * u1);
                z[2 * h + 1] = rad * sin(two_pi * u1);
            }
            for (int e = 0; e < 4 && j0 + e < ld; ++e)
                g[j0 + e] = (j0 + e < D) ? (float)(sigma * z[e]) : 0.0f;
        }
    }
}

/* ------------------------------------------------------------------ local gradient
 * Mean cross-entropy gradient of a ReLU multilayer perceptron (one layer = softmax
 * regression) for ONE worker on its sampled batch: the "nabla f(x_i; D_{i,n})" of
 * Algorithm 2's first-step update.  params / grad use the flat layout: per layer
 * W row-major [in][out], then b [out].  feats rows are float, or bfloat16 bit
 * patterns when feats_bf16 != 0; rows are indexed by idx[b] (shard-local rows of
 * `feats`, which points at the worker's shard).  Everything is accumulated in
 * double; grad is rounded to float once.  Returns the mean loss.
 *
 * operands_bf16 != 0 selects the arithmetic that the bf16 workload prescribes
 * ("bf16 inputs, fp32 accumulate, fp32 master weights"): both operands of every
 * matrix product (activations, weights, back-propagated errors) are rounded to
 * float and then to bfloat16 (nearest even) before they are multiplied; sums,
 * biases, ReLU and softmax stay in double.  With operands_bf16 == 0 the result is
 * the exact-arithmetic gradient. */
static double feat_at(const void *feats, int bf16, size_t k)
{
    if (!bf16) return (double)((const float *)feats)[k];
    uint32_t bits = (uint32_t)((const uint16_t *)feats)[k] << 16;
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
}

/* value of x after rounding to float and then to bfloat16, round-to-nearest-even */
double ora_round_bf16(double x)
{
    float f = (float)x;
    uint32_t b;
    memcpy(&b, &f, 4);
    b += 0x7FFFu + ((b >> 16) & 1u);
    b &= 0xFFFF0000u;
    memcpy(&f, &b, 4);
    return (double)f;
}

static inline double opnd(double x, int bf16) { return bf16 ? ora_round_bf16(x) : x; }

/* The operands of a matrix product as the chosen arithmetic sees them: n values, each rounded to bfloat16 when
 * rb != 0, as doubles (rounding is a function of the element alone, so it is done once per matrix here instead of
 * once per use; the products and their order are unchanged). */
static double *operands_f32(const float *x, size_t n, int rb)
{
    double *r = (double *)malloc(sizeof(double) * (n ? n : 1));
    for (size_t k = 0; k < n; ++k) r[k] = opnd((double)x[k], rb);
    return r;
}

static double *operands_f64(const double *x, size_t n, int rb)
{
    double *r = (double *)malloc(sizeof(double) * (n ? n : 1));
    for (size_t k = 0; k < n; ++k) r[k] = opnd(x[k], rb);
    return r;
}

/* Forward pass of one worker's batch.  a[0] = the batch rows, a[l] = ReLU output of layer l-1, a[n_layers] = logits;
 * Wop[l] = layer l's weights as operands.  z_hidden (may be NULL) receives the pre-activations of the hidden layers,
 * layer after layer, each [B][dims[l+1]]. */
static void forward_mlp(int n_layers, const int64_t *dims, const float *params, const void *feats, int feats_bf16,
                        int rb, const int32_t *idx, int B, double **a, double **Wop, size_t *woff, double *z_hidden)
{
    const int64_t d0 = dims[0];
    for (int b = 0; b < B; ++b)
        for (int64_t k = 0; k < d0; ++k)
            a[0][(size_t)b * d0 + k] = feat_at(feats, feats_bf16, (size_t)idx[b] * d0 + k);
    size_t off = 0;
    for (int l = 0; l < n_layers; ++l) {
        const int64_t din = dims[l], dout = dims[l + 1];
        const float *W = params + off, *bias = W + din * dout;
        woff[l] = off;
        off += (size_t)(din * dout + dout);
        Wop[l] = operands_f32(W, (size_t)(din * dout), rb);
        double *xin = operands_f64(a[l], (size_t)B * din, rb);
        for (int b = 0; b < B; ++b) {
            double *z = a[l + 1] + (size_t)b * dout;
            for (int64_t o = 0; o < dout; ++o) z[o] = 0.0;
            for (int64_t k = 0; k < din; ++k) {
                const double x = xin[(size_t)b * din + k];
                const double *Wk = Wop[l] + k * dout;
                for (int64_t o = 0; o < dout; ++o) z[o] += x * Wk[o];
            }
            for (int64_t o = 0; o < dout; ++o) z[o] += (double)bias[o];
            if (l + 1 < n_layers) {
                if (z_hidden) {
                    for (int64_t o = 0; o < dout; ++o) z_hidden[(size_t)b * dout + o] = z[o];
                }
                for (int64_t o = 0; o < dout; ++o) z[o] = z[o] > 0.0 ? z[o] : 0.0;
            }
        }
        if (z_hidden && l + 1 < n_layers) z_hidden += (size_t)B * dout;
        free(xin);
    }
}

double ora_grad_mlp(int n_layers, const int64_t *dims, const float *params, const void *feats, int feats_bf16,
                    int operands_bf16, const int32_t *labels, const int32_t *idx, int B, float *grad)
{
    const int rb = operands_bf16;
    int64_t maxw = 0;
    for (int l = 0; l <= n_layers; ++l) if (dims[l] > maxw) maxw = dims[l];
    double **a = (double **)malloc(sizeof(double *) * (n_layers + 1));
    for (int l = 0; l <= n_layers; ++l) a[l] = (double *)malloc(sizeof(double) * B * dims[l]);
    double **Wop = (double **)malloc(sizeof(double *) * n_layers);
    size_t *woff = (size_t *)malloc(sizeof(size_t) * n_layers);
    double *dz = (double *)malloc(sizeof(double) * B * maxw);
    double *da = (double *)malloc(sizeof(double) * B * maxw);
    forward_mlp(n_layers, dims, params, feats, feats_bf16, rb, idx, B, a, Wop, woff, NULL);

    /* softmax cross-entropy, mean over the batch */
    const int64_t C = dims[n_layers];
    double loss = 0.0;
    for (int b = 0; b < B; ++b) {
        const double *z = a[n_layers] + (size_t)b * C;
        double mx = z[0], s = 0.0;
        for (int64_t o = 1; o < C; ++o) if (z[o] > mx) mx = z[o];
        for (int64_t o = 0; o < C; ++o) s += exp(z[o] - mx);
        const int32_t y = labels[idx[b]];
        loss += -(z[y] - mx - log(s));
        for (int64_t o = 0; o < C; ++o)
            dz[(size_t)b * C + o] = (exp(z[o] - mx) / s - (o == y ? 1.0 : 0.0)) / (double)B;
    }
    loss /= (double)B;
    /* backward */
    for (int l = n_layers - 1; l >= 0; --l) {
        const int64_t din = dims[l], dout = dims[l + 1];
        float *gW = grad + woff[l], *gb = gW + din * dout;
        double *acc = (double *)calloc((size_t)dout, sizeof(double));
        double *xin = operands_f64(a[l], (size_t)B * din, rb);
        double *dzo = operands_f64(dz, (size_t)B * dout, rb);
        /* gW = a_l^T dz */
        for (int64_t k = 0; k < din; ++k) {
            memset(acc, 0, sizeof(double) * dout);
            for (int b = 0; b < B; ++b) {
                const double x = xin[(size_t)b * din + k];
                const double *d = dzo + (size_t)b * dout;
                for (int64_t o = 0; o < dout; ++o) acc[o] += x * d[o];
            }
            for (int64_t o = 0; o < dout; ++o) gW[k * dout + o] = (float)acc[o];
        }
        /* gb = column sums of dz (no product: not rounded) */
        memset(acc, 0, sizeof(double) * dout);
        for (int b = 0; b < B; ++b)
            for (int64_t o = 0; o < dout; ++o) acc[o] += dz[(size_t)b * dout + o];
        for (int64_t o = 0; o < dout; ++o) gb[o] = (float)acc[o];
        free(acc);
        if (l > 0) {
            /* da = dz W^T, then through the ReLU: derivative 1 where the activation is positive, else 0 */
            for (int b = 0; b < B; ++b) {
                const double *d = dzo + (size_t)b * dout;
                for (int64_t k = 0; k < din; ++k) {
                    const double *Wk = Wop[l] + k * dout;
                    double s = 0.0;
                    for (int64_t o = 0; o < dout; ++o) s += d[o] * Wk[o];
                    da[(size_t)b * din + k] = a[l][(size_t)b * din + k] > 0.0 ? s : 0.0;
                }
            }
            double *t = dz; dz = da; da = t;
        }
        free(xin); free(dzo);
    }
    for (int l = 0; l <= n_layers; ++l) free(a[l]);
    for (int l = 0; l < n_layers; ++l) free(Wop[l]);
    free(a); free(Wop); free(dz); free(da); free(woff);
    return loss;
}

/* The pre-activations z = a W + b of the hidden layers of one worker's batch, in the arithmetic ora_grad_mlp uses:
 * z_hidden receives layer after layer, each [B][dims[l+1]] (l = 0 .. n_layers-2).  Their signs are the ReLU
 * decisions of the gradient; the tests count where another implementation decides differently. */
void ora_hidden_mlp(int n_layers, const int64_t *dims, const float *params, const void *feats, int feats_bf16,
                    int operands_bf16, const int32_t *idx, int B, double *z_hidden)
{
    double **a = (double **)malloc(sizeof(double *) * (n_layers + 1));
    for (int l = 0; l <= n_layers; ++l) a[l] = (double *)malloc(sizeof(double) * B * dims[l]);
    double **Wop = (double **)malloc(sizeof(double *) * n_layers);
    size_t *woff = (size_t *)malloc(sizeof(size_t) * n_layers);
    forward_mlp(n_layers, dims, params, feats, feats_bf16, operands_bf16, idx, B, a, Wop, woff, z_hidden);
    for (int l = 0; l <= n_layers; ++l) free(a[l]);
    for (int l = 0; l < n_layers; ++l) free(Wop[l]);
    free(a); free(Wop); free(woff);
}

/* All workers' hidden pre-activations: Z is [M][sum over hidden layers of B * dims[l+1]]. */
void ora_local_hidden(int M, int64_t ld, int n_layers, const int64_t *dims, const float *X, const void *feats,
                      int feats_bf16, int operands_bf16, const int64_t *shard_off, const int32_t *idx, int B, double *Z)
{
    size_t per = 0;
    for (int l = 0; l + 1 < n_layers; ++l) per += (size_t)B * dims[l + 1];
    const size_t esz = feats_bf16 ? 2 : 4;
#pragma omp parallel for num_threads(g_threads) schedule(dynamic, 1)
    for (int i = 0; i < M; ++i) {
        const char *f = (const char *)feats + (size_t)shard_off[i] * dims[0] * esz;
        ora_hidden_mlp(n_layers, dims, X + (size_t)i * ld, f, feats_bf16, operands_bf16, idx + (size_t)i * B, B,
                       Z + (size_t)i * per);
    }
}

/* All workers: gradient of worker i from row i of X into row i of G (padding columns set to 0).
 * feats/labels hold all shards; shard_off[M+1] delimits them; idx is [M][B]. loss (may be NULL) is [M]. */
void ora_local_grad(int M, int64_t ld, int n_layers, const int64_t *dims, const float *X, const void *feats,
                    int feats_bf16, int operands_bf16, const int32_t *labels, const int64_t *shard_off, const int32_t *idx, int B,
                    float *G, double *loss)
{
    int64_t D = 0;
    for (int l = 0; l < n_layers; ++l) D += dims[l] * dims[l + 1] + dims[l + 1];
    const size_t esz = feats_bf16 ? 2 : 4;
#pragma omp parallel for num_threads(g_threads) schedule(dynamic, 1)
    for (int i = 0; i < M; ++i) {
        const char *f = (const char *)feats + (size_t)shard_off[i] * dims[0] * esz;
        double L = ora_grad_mlp(n_layers, dims, X + (size_t)i * ld, f, feats_bf16, operands_bf16, labels + shard_off[i],
                                idx + (size_t)i * B, B, G + (size_t)i * ld);
        for (int64_t j = D; j < ld; ++j) G[(size_t)i * ld + j] = 0.0f;
        if (loss) loss[i] = L;
    }
}

/* ------------------------------------------------------------------ momentum apply + mix
 * For every worker i and parameter j, from the previous-iteration copies:
 *   v'  = mu v + g + wd x            (momentum SGD, Section V-A; v^0 = 0, mu = 0 gives plain SGD)
 *   h   = x - alpha v'               (first-step update, Algorithm 2 / Eq. (c0))
 *   x'  = h - w (h - x_peer)         (second-step update, Algorithm 2 / Eq. (c1)), w = w[i][peer_i]
 * x_peer is the peer's row of Xcur, i.e. its copy before this iteration.  V is updated in place. */
void ora_mix(int M, int64_t ld, const float *Xcur, const float *G, float *V, float *Xnext, const int32_t *peer,
             const double *w, double alpha, double mu, double wd)
{
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int i = 0; i < M; ++i) {
        const int32_t m = peer[i];
        const double wi = w[(size_t)i * M + m];
        const float *x = Xcur + (size_t)i * ld, *xp = Xcur + (size_t)m * ld, *g = G + (size_t)i * ld;
        float *v = V + (size_t)i * ld, *xn = Xnext + (size_t)i * ld;
        for (int64_t j = 0; j < ld; ++j) {
            const double vn = mu * (double)v[j] + (double)g[j] + wd * (double)x[j];
            const float vf = (float)vn;           /* the stored momentum is what the next iteration reads */
            const double h = (double)x[j] - alpha * (double)vf;
            xn[j] = (float)(h - wi * (h - (double)xp[j]));
            v[j] = vf;
        }
    }
}

/* The same update written as the convex combination of Eq. (c1), second line:
 * x' = (1 - w)(x - alpha v') + w x_peer.  Used only to pin ora_mix. */
void ora_mix_convex(int M, int64_t ld, const float *Xcur, const float *G, float *V, float *Xnext,
                    const int32_t *peer, const double *w, double alpha, double mu, double wd)
{
    for (int i = 0; i < M; ++i) {
        const int32_t m = peer[i];
        const double wi = w[(size_t)i * M + m];
        for (int64_t j = 0; j < ld; ++j) {
            const size_t q = (size_t)i * ld + j;
            const double vn = mu * (double)V[q] + (double)G[q] + wd * (double)Xcur[q];
            const float vf = (float)vn;
            Xnext[q] = (float)((1.0 - wi) * ((double)Xcur[q] - alpha * (double)vf) + wi * (double)Xcur[(size_t)m * ld + j]);
            V[q] = vf;
        }
    }
}

/* ------------------------------------------------------------------ asynchronous schedule
 * Section II-B and Eq. (c2)-(c4): the workers do not step together.  In global step k exactly one worker i_k is
 * active.  A worker whose iterations take tbar_i = sum_m t_im p_im d_im on average (Eq. (d3)) is the active one
 * with probability p_i = (1 / tbar_i) / sum_m (1 / tbar_m) (Eq. (d4)).  It pulls from m_k ~ P[i_k, :], takes
 * its local step and mixes; every other copy stays: x^{k+1} = D^k (x^k - alpha g^k), g^k zero outside row i_k.
 *
 * Draws: i_k is found from word 0 of stream 3 at counter (0, 0, k) against the 32-bit cumulative thresholds of
 * (p_i) (built like a policy row); m_k as in the synchronous schedule, stream 0 at counter (0, i_k, k). */
void ora_activity(int M, const double *t, const double *P, const uint8_t *adj, double *p_act)
{
    double total = 0.0;
    for (int i = 0; i < M; ++i) {
        double tbar = 0.0;
        for (int m = 0; m < M; ++m) {
            const double d = (m == i) ? 0.0 : (adj ? (double)(adj[(size_t)i * M + m] != 0) : 1.0);
            tbar += t[(size_t)i * M + m] * P[(size_t)i * M + m] * d;
        }
        p_act[i] = 1.0 / tbar;
        total += p_act[i];
    }
    for (int i = 0; i < M; ++i) p_act[i] /= total;
}

void ora_async_draw(int M, const uint32_t *Tact, int32_t last_act, const uint32_t *T, const int32_t *last,
                    uint64_t seed, uint64_t k, int32_t *i_out, int32_t *m_out)
{
    uint32_t r[4];
    draw(seed, 3u, 0u, 0u, k, r);
    const int32_t i = ora_peer_of_word(M, Tact, last_act, r[0]);
    draw(seed, 0u, 0u, (uint32_t)i, k, r);
    *i_out = i;
    *m_out = ora_peer_of_word(M, T + (size_t)i * M, last[i], r[0]);
}

/* The active worker's update, in place: row i of X and V from its gradient g (one row) and row m of X. */
void ora_async_apply(int M, int64_t ld, float *X, float *V, const float *g, int i, int m, double w, double alpha,
                     double mu, double wd)
{
    (void)M;
    float *x = X + (size_t)i * ld, *v = V + (size_t)i * ld;
    const float *xp = X + (size_t)m * ld;
    for (int64_t j = 0; j < ld; ++j) {
        const double vn = mu * (double)v[j] + (double)g[j] + wd * (double)x[j];
        const float vf = (float)vn;
        const double h = (double)x[j] - alpha * (double)vf;
        const double xpj = (m == i) ? 0.0 : (double)xp[j];          /* w = 0 for a self selection */
        x[j] = (float)(h - w * (h - xpj));
        v[j] = vf;
    }
}

/* ------------------------------------------------------------------ iteration-time bookkeeping
 * Algorithm 2, UpdateTimeVector: after an iteration with peer m the worker records the iteration time t_im and
 * smooths it, T_i[m] <- beta T_i[m] + (1 - beta) t_im (exponential moving average, T_i starts at 0); the
 * monitor later collects the matrix [T_i[m]] (Algorithm 1).  Here the recorded time comes from a given matrix
 * t (a simulated network); clock[i] accumulates the time worker i has spent (t_ii for a self selection).
 * ema and clock are float and updated in place; clock may be NULL. */
void ora_update_times(int M, const int32_t *peer, const float *t, double beta, float *ema, float *clock)
{
    for (int i = 0; i < M; ++i) {
        const int32_t m = peer[i];
        const size_t e = (size_t)i * M + m;
        if (m != i) ema[e] = (float)(beta * (double)ema[e] + (1.0 - beta) * (double)t[e]);
        if (clock) clock[i] = (float)((double)clock[i] + (double)t[e]);
    }
}

/* The same bookkeeping for the asynchronous schedule: the global steps are taken in order, step s concerns only its
 * active worker active[s] and the peer peers[s] it pulled from. */
void ora_update_times_async(int M, int64_t n_steps, const int32_t *active, const int32_t *peers, const float *t,
                            double beta, float *ema, float *clock)
{
    for (int64_t s = 0; s < n_steps; ++s) {
        const int32_t i = active[s], m = peers[s];
        const size_t e = (size_t)i * M + m;
        if (m != i) ema[e] = (float)(beta * (double)ema[e] + (1.0 - beta) * (double)t[e]);
        if (clock) clock[i] = (float)((double)clock[i] + (double)t[e]);
    }
}

/* ------------------------------------------------------------------ consensus distance
 * CD = sum_i || x_i - xbar ||^2, xbar = (1/M) sum_i x_i, over the first D columns: the
 * complete-graph form of the model-difference penalty of Eq. (1)
 * ( = (1/2M) sum_i sum_m ||x_i - x_m||^2 ). */
double ora_consensus_dist(int M, int64_t D, int64_t ld, const float *X)
{
    double cd = 0.0;
    for (int64_t j = 0; j < D; ++j) {
        double mean = 0.0;
        for (int i = 0; i < M; ++i) mean += (double)X[(size_t)i * ld + j];
        mean /= (double)M;
        for (int i = 0; i < M; ++i) {
            const double d = (double)X[(size_t)i * ld + j] - mean;
            cd += d * d;
        }
    }
    return cd;
}
