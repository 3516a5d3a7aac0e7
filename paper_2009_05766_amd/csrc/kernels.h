// Internal launch interface between the C ABI (netmax_api.hip) and the gfx950 kernels.
// X, V, G are in the worker-interleaved tile layout of layout.h; ld is a multiple of TILE.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "philox.h"   // IterRef: iteration number by value or from a device cell

namespace netmax {


// Peer selection of Algorithm 2: one Philox draw per worker against fixed-point cumulative thresholds.
void launch_sample_peers(hipStream_t s, int M, const uint32_t *thr, const int32_t *last, uint64_t seed,
                         const IterRef &iter, int32_t *peer);

// Batch draws (with replacement) for every worker; n_rows[i] = shard size of worker i.
void launch_sample_batch(hipStream_t s, int M, int B, const int32_t *n_rows, uint64_t seed, const IterRef &iter,
                         int32_t *idx);
// both draws of an iteration in one launch
void launch_sample_iteration(hipStream_t s, int M, const uint32_t *thr, const int32_t *last, int32_t *peer, int B,
                             const int32_t *n_rows, int32_t *idx, uint64_t seed, const IterRef &iter);

// g[i][j] = sigma * N(0,1) from Philox + Box-Muller; padding columns are zeroed.
void launch_synth_grad(hipStream_t s, int M, int64_t D, int64_t ld, float sigma, uint64_t seed, const IterRef &iter,
                       float *G);

// Asynchronous schedule: all (active worker, peer) draws of a run, and the in-place update of one worker's row.
void launch_async_draw(hipStream_t s, int M, const uint32_t *act_thr, int act_last, const uint32_t *thr, const int32_t *last,
                       uint64_t seed, uint64_t first, uint64_t n_steps, int32_t *active, int32_t *peers);
// A batch of n_steps consecutive global steps (numbers k0, k0 + 1, ...) whose rows do not overlap.  source 0: flat model,
// gradient generated; 1: read from the active worker's row of G; 2: read from slot s of the compact matrix Gc.
void launch_async_rows(hipStream_t s, int source, int M, int64_t D, int64_t ld, float *X, float *V, float *G, const float *Gc,
                       int n_steps, const int32_t *active, const int32_t *peers, const float *w, float alpha, float mu, float wd,
                       float sigma, uint64_t seed, uint64_t k0);
// Subset runs of the perceptron gradient (asynchronous schedule): rows of listed workers into a compact matrix, their
// shard descriptors, their batch draws (slot s at iteration first_iter + s), their losses back.
void launch_gather_rows(hipStream_t s, int M, int n, int64_t ld, const int32_t *workers, const float *X, float *Xc);
void launch_gather_shards(hipStream_t s, int M, int n, const int32_t *workers, const int64_t *row0, const int32_t *n_rows,
                          int64_t *row0_c, int32_t *n_rows_c);
void launch_scatter_loss(hipStream_t s, int M, int n, const int32_t *workers, const float *loss_c, float *loss);
void launch_sample_batch_subset(hipStream_t s, int n, int B, const int32_t *workers, const int32_t *n_rows_c, uint64_t seed,
                                uint64_t first_iter, int32_t *idx);

void launch_async_times(hipStream_t s, int M, int64_t n_steps, const int32_t *active, const int32_t *peers, const float *t,
                        float beta, float *ema, float *clock);

// Iteration-time bookkeeping of Algorithm 2 (UpdateTimeVector) against a given time matrix.
void launch_update_times(hipStream_t s, int M, const int32_t *peer, const float *t, float beta, float *ema, float *clock);

// The device cell of the iteration number used by graph replays: set it, advance it by one.
void launch_set_iteration(hipStream_t s, uint64_t *cell, uint64_t value);
void launch_bump_iteration(hipStream_t s, uint64_t *cell);

// One-time kernel attributes (LDS limits); call once per process before the first launch.
void prepare_kernels();

// Momentum apply + mix, Eq. (c0)/(c1), for all workers.
void launch_mix(hipStream_t s, int M, int64_t ld, const float *Xcur, const float *G, float *V, float *Xnext,
                const int32_t *peer, const float *w, float alpha, float mu, float wd);
// Once per device before the first launch_mix: lets the kernel be launched with its large (unused) LDS request.
hipError_t prepare_mix();
hipError_t prepare_mix_synth();      // the same for launch_mix_synth

// Flat models: the synthetic gradient generated inside the update (g is still written).
void launch_mix_synth(hipStream_t s, int M, int64_t D, int64_t ld, const float *Xcur, float *G, float *V, float *Xnext,
                      const int32_t *peer, const float *w, float alpha, float mu, float wd, float sigma, uint64_t seed,
                      const IterRef &iter);

// The same update for a list of column tiles only, leaving out up to MIX_MAX_SKIP column ranges (multiples of four
// columns) that another kernel has already updated.  tiles: device [n_tiles_listed].
constexpr int MIX_MAX_SKIP = 8;
struct MixSkip { int n; int64_t lo[MIX_MAX_SKIP], hi[MIX_MAX_SKIP]; };
void launch_mix_subset(hipStream_t s, int M, const int32_t *tiles, int n_listed, const MixSkip &skip, const float *Xcur,
                       const float *G, float *V, float *Xnext, const int32_t *peer, const float *w, float alpha, float mu,
                       float wd);

// Consensus distance: per-block partial sums (double), then a fixed-order final sum into out_dev[0].
// partial must hold consensus_partials(ld) doubles: one per CONSENSUS_COLS columns.
constexpr int CONSENSUS_COLS = 1024;
int consensus_partials(int64_t ld);
void launch_consensus(hipStream_t s, int M, int64_t D, int64_t ld, const float *X, double *partial,
                      double *out_dev);

// Layout conversion between row-major [M][row_ld] and the tile layout (columns >= cols read as / are left 0).
void launch_pack(hipStream_t s, int M, int64_t cols, int64_t ld, const float *rows, int64_t row_ld, float *tiled);
void launch_unpack(hipStream_t s, int M, int64_t cols, const float *tiled, float *rows, int64_t row_ld);

// out[k] = bfloat16 in[k] as float, k < n.
void launch_widen_bf16(hipStream_t s, int64_t n, const uint16_t *in, float *out);

// Whole iterations of a small softmax-regression model in one kernel, one workgroup per worker (k_small_iter.hip).
// grad_only: batch draw, loss and gradient only (G, loss, idx); otherwise also the peer draw (peers) and the update
// (x_second, V).  n_iters > 1 needs a cooperative launch: x_first / x_second swap roles after every iteration and
// the workgroups meet at a barrier (counter `barrier`, which the launch advances by (n_iters - 1) * M from
// barrier_base); *fault is raised if a workgroup waited in vain.
struct SmallIterLaunch {
    int M, B; int64_t din, dout, D, ld;
    const float *feats; const int32_t *labels; const int64_t *row0; const int32_t *n_rows;
    const uint32_t *thr; const int32_t *last; const float *w;
    float *x_first, *x_second, *V, *G, *loss; int32_t *peers, *idx;
    float alpha, mu, wd; uint64_t seed; IterRef iter; int n_iters, grad_only;
    unsigned *barrier; unsigned barrier_base; int *fault;
    const int32_t *workers; int n_workers;   // grad_only: one workgroup per listed worker (device list), slot s at iteration iter + s
    long long patience;                      // polls of the barrier counter before a workgroup gives up and raises *fault
};
bool small_iter_ok(int model_is_mlp, int n_layers, int bf16, int B, int64_t din, int64_t dout, int64_t ld);
hipError_t prepare_small_iter();
int small_iter_max_resident(int B, int64_t din, int64_t dout, int64_t ld);
hipError_t launch_small_iter(hipStream_t s, const SmallIterLaunch &a, int cooperative);

// Workgroup id -> (worker, block inside the worker's GEMM).  Workgroup ids are dealt round-robin to the 8
// XCDs; all blocks of one worker are placed on the same XCD, next to each other, so the operand every
// block of that worker re-reads (its activations / back-propagated errors) comes from HBM once and from
// that XCD's L2 afterwards.  Returns false for the padding ids beyond the last worker.
constexpr int MF_XCD = 8;
__device__ __forceinline__ bool decode_group(unsigned bid, unsigned blocks_per_worker, int M, int &g, unsigned &local)
{
    const unsigned xcd = bid % MF_XCD, slot = bid / MF_XCD;
    const unsigned round = slot / blocks_per_worker;
    local = slot - round * blocks_per_worker;
    g = (int)(round * MF_XCD + xcd);
    return g < M;
}
inline unsigned grouped_grid(int M, unsigned blocks_per_worker)
{
    return (unsigned)((M + MF_XCD - 1) / MF_XCD * MF_XCD) * blocks_per_worker;
}

// Per-worker MLP / softmax-regression gradient (grouped GEMMs).
struct MlpPlan {
    int M, n_layers, B;
    int64_t dims[8];
    int64_t woff[8];        // offset of layer l's W inside a parameter row; the bias follows the matrix
    int64_t ld;
    int bf16;               // operands rounded to bfloat16 (features are stored as bfloat16)
    const void *feats;      // [n_total][dims[0]]
    const int32_t *labels;  // [n_total]
    const int64_t *row0;    // device [M]: first feature row of each worker's shard
    const int32_t *idx;     // device [M][B] shard-local batch rows
    float *act[8];          // act[l], l = 1..n_layers: [M][B][dims[l]] post-activation (logits for the last)
    float *dz[2];           // two ping-pong buffers [M][B][max width]
    float *loss;            // [M]
    // bf16 operands only: bfloat16 copies of activations and back-propagated errors, in both orientations
    uint16_t *hb[8];        // hb[l], l = 1..n_layers-1: [M][B][dims[l]]
    uint16_t *ht[8];        // ht[l], l = 1..n_layers-1: [M][dims[l]][B] (the first layer's weight gradient gathers its A^T from the data rows)
    uint16_t *dzb[2];       // [M][B][max width]
    uint16_t *dzt[2];       // [M][max width][B]
};
// What the second-step update needs besides the gradient: passed to the gradient code when the weight-gradient
// kernels of the matrix-core layers apply the update themselves instead of writing the gradient.
struct MixArgs {
    const float *Xcur; float *V, *Xnext; const int32_t *peer; const float *w; float alpha, mu, wd;
};
// fuse != nullptr: layers accepted by mfma_layer_ok() do not write their weight gradient to G; they write
// x' and v' of their weight columns (Eq. (c0)/(c1)) straight from the product.
void launch_mlp_grad(hipStream_t s, const MlpPlan &p, const float *X, float *G, const MixArgs *fuse = nullptr);

// Matrix-core kernels (k_grad_mfma.hip) for layers that mfma_layer_ok() accepts.
bool mfma_layer_ok(const MlpPlan &p, int l);
void launch_fwd_mfma(hipStream_t s, const MlpPlan &p, int l, const float *X);
// also writes the bias gradient of layer l - 1 into G; want_f32: keep the fp32 copy of the error as well
void launch_dgrad_mfma(hipStream_t s, const MlpPlan &p, int l, const float *X, float *G, int cur, bool want_f32);
void launch_wgrad_mfma(hipStream_t s, const MlpPlan &p, int l, float *G, int cur);
void launch_wgrad_mix_mfma(hipStream_t s, const MlpPlan &p, int l, int cur, const MixArgs &mix);
// Last layer with at most 32 outputs.
bool mfma_small_last_ok(const MlpPlan &p);
// also: softmax cross-entropy on the logits (loss, dZ, the last layer's bias gradient, the gradient's padding)
void launch_fwd_small(hipStream_t s, const MlpPlan &p, const float *X, float *G);
void launch_wgrad_small(hipStream_t s, const MlpPlan &p, float *G, int cur);
void launch_dgrad_small(hipStream_t s, const MlpPlan &p, const float *X, float *G, int cur, bool want_f32);

// Layers on fp32 operands with a batch of 32 or 64 rows and a multiple of 32 outputs (k_grad_f32.hip): forward pass
// and weight gradient that read W / write dW exactly once with many loads in flight.
bool fwd_f32_ok(const MlpPlan &p, int l);
bool wgrad_f32_ok(const MlpPlan &p, int l);
hipError_t prepare_f32_layers();
void launch_fwd_f32(hipStream_t s, const MlpPlan &p, int l, const float *X);
void launch_wgrad_f32(hipStream_t s, const MlpPlan &p, int l, float *G, const float *dz);

// Last layer with at most 16 classes on fp32 operands above a hidden layer (k_grad_head.hip): one kernel from the
// last hidden activation to the error of that layer: logits, loss, dW, db, dH and the column sums of dH.
bool head_ok(const MlpPlan &p);
hipError_t prepare_head();
void launch_head(hipStream_t s, const MlpPlan &p, const float *X, float *G);

}  // namespace netmax
