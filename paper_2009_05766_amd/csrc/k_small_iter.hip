// Whole NetMax iterations of a small softmax-regression model in ONE kernel (Algorithm 2, all of its steps): one
// workgroup per worker draws its peer and its batch, computes logits, loss and gradient with the worker's parameters
// and batch rows held in LDS, and applies the momentum step and the mix (Eq. (c0), (c1)) against the peer's copy of the
// previous iteration.  Models of this size are bound by launch latency (six dependent launches of a few microseconds
// each otherwise); here an iteration is one launch, or, launched cooperatively, one grid barrier inside a launch that
// runs many iterations.
//
// Three modes share the code, so their results agree bit for bit:
//   GRAD      batch draw, loss, gradient -> G (netmax_local_step; the mix kernel then applies the same update function)
//   STEP      peer draw + GRAD + update  -> Xnext, V, G (one iteration per launch; also what a captured graph replays)
//   the same with n_iters > 1: cooperative launch, all workgroups resident, a barrier after every iteration.
//
// Arithmetic: fp32, fixed order.  Forward: eight lanes share a batch row, lane s takes the features k = s, s + 8, ...
// in increasing order, the eight partial sums are added in halves.  Weight gradient: one thread per four features
// and four classes, batch rows in increasing order.  Shapes that tile (at most 16 classes, a batch of 16, 32 or 64
// rows, features a multiple of 256 / (batch / 16)) take both products on v_mfma_f32_16x16x4_f32 instead (exact fp32 products, fp32
// accumulation; lane l supplies A[l % 16][l / 16] and B[l / 16][l % 16] and receives D[4 (l / 16) + v][l % 16]): the
// vector units are then left with the softmax and the update.
//
// The kernel lives on latency, so little is waited for that could have been asked for earlier: the peer's row and
// the own momentum are requested before the gradient is computed and used after it; the draws of the NEXT iteration
// depend on (seed, iteration, worker) only, so its labels are requested before the forward pass and its batch rows
// after the update, and both arrive while this iteration finishes and waits at the barrier; the new parameters
// stay in LDS, only the peer's row is read again after the barrier.  (Requests are placed where few registers are
// live: held across the forward pass they starve its inner loop of registers.)
#include "kernels.h"
#include "layout.h"
#include "philox.h"
#include "vec.h"

namespace netmax {

constexpr int SI_THREADS = 512, SI_WAVES = SI_THREADS / 64;
constexpr int SI_SPLIT = 8;                 // lanes that share one batch row in the forward pass
constexpr int SI_MAX_OUT = 32;              // classes
constexpr int SI_LDS_LIMIT = 150 * 1024;
constexpr int SI_BURST = 8;                 // loads a thread has in flight while it fills LDS
constexpr int SI_UPD = 4;                   // vectors of x_peer and v per thread and pass of the update

struct SmallIterArgs {
    int M, B, din, dout;
    int64_t D, ld;
    const float *feats; const int32_t *labels; const int64_t *row0; const int32_t *n_rows;
    const uint32_t *thr; const int32_t *last; const float *w;
    float *x_first, *x_second;              // x_first holds x^t of the first iteration of the launch
    float *V, *G, *loss;
    int32_t *peers, *idx;
    float alpha, mu, wd;
    uint64_t seed;
    IterRef iter;                           // number of the first iteration
    int n_iters, grad_only;
    unsigned *barrier; unsigned barrier_base; int *fault;
    const int32_t *workers;                 // grad_only: workgroup s works for worker workers[s] at iteration iter + s (NULL: s, iter)
    long long patience;                     // polls of the barrier counter before a workgroup gives up
};

// The matrix-instruction form of the two products: classes padded to one 16-wide tile, 16-row tiles of the batch, the
// the waves split the features of the forward pass evenly in groups of 64 (no bounds test in any loop).
static bool small_iter_mm(int B, int64_t din, int64_t dout)
{
    return dout <= 16 && (B == 16 || B == 32 || B == 64) && din % (64 * SI_WAVES / (B / 16)) == 0;     // every wave's part: whole groups of 64 features
}
static int small_iter_cap(int B, int64_t din, int64_t dout)
{
    if (small_iter_mm(B, din, dout)) return 16;
    return dout <= 8 ? 8 : (dout <= 16 ? 16 : SI_MAX_OUT);
}
constexpr int SI_MM_PAD = 4;                // floats behind a batch row in that form: sixteen rows read together meet all banks
constexpr int SI_MM_PART = SI_WAVES * 16 * 16;   // floats of partial logits: one 16 x 16 tile per wave

static size_t small_iter_lds(int B, int din, int dout, int64_t ld)
{
    const bool mm = small_iter_mm(B, din, dout);
    const size_t pitch = (size_t)din + (mm ? SI_MM_PAD : SI_SPLIT), cap = (size_t)small_iter_cap(B, din, dout);
    return (2 * (size_t)ld + ((size_t)din + 1) * (cap + 4) + (size_t)B * pitch + (size_t)B * cap + (size_t)B + (mm ? SI_MM_PART : 0)) * sizeof(float) +
           (4 * (size_t)B + 2) * sizeof(int32_t);
}

// All workgroups of the grid have arrived (and their stores are visible to each other) when this returns true.  A
// workgroup that polls `patience` times without seeing the others raises *fault and goes on, so the kernel always ends.
__device__ __forceinline__ void grid_barrier(unsigned *counter, unsigned target, int *fault, long long patience)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");        // this wave's stores, device wide
    __syncthreads();
    if (threadIdx.x == 0) {
        __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        long long polls = 0;
        while ((int)(__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
            if (++polls > patience) {
                *fault = 1;
                break;
            }
            __builtin_amdgcn_s_sleep(4);
        }
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");        // drop what this compute unit cached of the others' rows
}

// j / d for 0 <= j < 2^32 / d, with magic = ceil(2^32 / d).
__device__ __forceinline__ int div_magic(int j, uint32_t magic) { return (int)__umulhi((uint32_t)j, magic); }
static __device__ __host__ __forceinline__ uint32_t magic_of(int d) { return (uint32_t)((0x100000000ull + (uint32_t)d - 1) / (uint32_t)d); }

// The value that lane (l ^ MASK) holds, MASK in {1, 2, 4}, by data-parallel-primitive moves inside the vector unit
// (no trip through the LDS crossbar as a general lane shuffle takes): quad permutations [1,0,3,2] and [2,3,0,1] for
// 1 and 2; for 4 the mirror of each group of eight lanes (l -> l ^ 7) followed by the reversal of each quad (^ 3).
template <int MASK>
__device__ __forceinline__ float xor_lane(float v)
{
    static_assert(MASK == 1 || MASK == 2 || MASK == 4, "lane distances inside a group of eight");
    int x = __float_as_int(v);
    if (MASK == 1) x = __builtin_amdgcn_update_dpp(x, x, 0xB1, 0xF, 0xF, false);
    if (MASK == 2) x = __builtin_amdgcn_update_dpp(x, x, 0x4E, 0xF, 0xF, false);
    if (MASK == 4) {
        x = __builtin_amdgcn_update_dpp(x, x, 0x141, 0xF, 0xF, false);
        x = __builtin_amdgcn_update_dpp(x, x, 0x1B, 0xF, 0xF, false);
    }
    return __int_as_float(x);
}

// The value, hidden from the optimiser: what is computed from it inside a loop is computed there, not once before
// the loop (address arithmetic of all phases kept in registers across the whole iteration starves the inner loops).
__device__ __forceinline__ int opaque(int v)
{
    asm volatile("" : "+v"(v));
    return v;
}

// CAP: classes the unrolled loops cover: dout <= CAP, CAP in {8, 16, 32}.  RT > 0: the two products on matrix
// instructions, RT = batch / 16 tiles of batch rows (CAP = 16, shapes accepted by small_iter_mm()).
template <int CAP, int RT = 0>
__global__ void __launch_bounds__(SI_THREADS) small_softmax_iteration_kernel(SmallIterArgs p)
{
    constexpr bool MM = RT > 0;
    static_assert(!MM || CAP == 16, "the matrix-instruction form pads the classes to one 16-wide tile");
    extern __shared__ __attribute__((aligned(16))) unsigned char si_smem[];
    constexpr int SI_DEPTH = CAP <= 16 ? 4 : 2;               // steps of an inner product whose LDS reads are in flight together
    constexpr int OWN = CAP / SI_SPLIT;                       // classes a lane owns after the reduction of a row
    constexpr int WP = CAP + 4;                               // floats per padded row of W: the eight rows a wave reads
                                                              // together then lie in different LDS banks
    const int t0 = threadIdx.x;
    const int i = p.workers ? p.workers[blockIdx.x] : (int)blockIdx.x;
    if ((unsigned)i >= (unsigned)p.M) return;
    const int pitch = p.din + (MM ? SI_MM_PAD : SI_SPLIT);
    float *xl = reinterpret_cast<float *>(si_smem);           // [ld]  the worker's parameters (W row-major [din][dout], b)
    float *gl = xl + p.ld;                                    // [ld]  its gradient
    float *wp = gl + p.ld;                                    // [din + 1][WP] W and then b with rows padded by zeros to
                                                              //       CAP classes: the inner loops run without a bounds test
    float *dz = wp + ((size_t)p.din + 1) * WP;                // [B][CAP], zeros beyond dout (16-byte aligned rows)
    float *xs = dz + (size_t)p.B * CAP;                       // [B][pitch] batch rows
    float *lb = xs + (size_t)p.B * pitch;                     // [B] per-row loss
    float *part = lb + p.B;                                   // MM: [parts of the features][B][16] partial logits
    int32_t *ib = reinterpret_cast<int32_t *>(part + (MM ? SI_MM_PART : 0));   // [2][B] batch rows (shard-local) of this and the next iteration
    int32_t *yl = ib + 2 * p.B;                               // [2][B] their labels
    int32_t *cnt = yl + 2 * p.B;                              // [2] thresholds of the peer draw that are <= u
    const uint64_t iter0 = iteration_of(p.iter) + (p.workers ? (uint64_t)blockIdx.x : 0ull);
    const int n_vec = (int)(p.ld >> 2);
    const float invB = 1.0f / (float)p.B;
    const uint32_t n_i = (uint32_t)p.n_rows[i];
    const int64_t r0 = p.row0[i];
    const int last_i = p.grad_only ? 0 : p.last[i];
    const float *shard = p.feats + (size_t)r0 * p.din;
    const uint32_t *thr_row = p.thr + (size_t)i * p.M;
    const uint32_t magic_out = magic_of(p.dout);
    const bool vec_rows = (p.din & 3) == 0;                   // batch rows as 128-bit pieces, else element by element
    const int row_units = vec_rows ? p.din >> 2 : p.din, feat_units = p.B * row_units;
    const uint32_t magic_row = magic_of(row_units);

    // The batch draw of one iteration: thread b < B draws its own row (word b % 4 of block b / 4 of stream 1), stores
    // it and returns the row's label (still in flight).
    auto draw_batch = [&](int t, uint64_t iter, int buf) -> int32_t {
        if (t >= p.B) return 0;
        const Words4 r = draw_block(p.seed, STREAM_BATCH, (uint32_t)t >> 2, (uint32_t)i, iter);
        const uint32_t word = (t & 3) == 0 ? r.a : ((t & 3) == 1 ? r.b : ((t & 3) == 2 ? r.c : r.d));
        const int32_t v = (int32_t)__umulhi(word, n_i);
        ib[buf * p.B + t] = v;
        p.idx[(size_t)i * p.B + t] = v;
        return p.labels[r0 + v];
    };
    // The peer draw: the peer is the number of thresholds of the row that are <= u (they do not decrease), clamped
    // to the last positive entry; the threads count their share, the waves add up in LDS.
    auto count_hits = [&](int t, int q, uint32_t threshold, uint32_t u, int buf) {
        const unsigned long long hit = __ballot(q < p.M && threshold <= u);
        if ((t & 63) == 0 && hit) atomicAdd(&cnt[buf], (int)__popcll(hit));
    };
    auto count_thresholds = [&](int t, uint64_t iter, int buf, uint32_t first) {   // first: thr_row[t], read earlier
        const uint32_t u = draw_block(p.seed, STREAM_PEER, 0u, (uint32_t)i, iter).a;
        count_hits(t, t, first, u, buf);
        for (int q0 = SI_THREADS; q0 < p.M; q0 += SI_THREADS) {
            const int q = q0 + t;
            count_hits(t, q, thr_row[q < p.M ? q : 0], u, buf);
        }
    };
    // Requests the first SI_BURST pieces per thread of the batch rows listed in ib[buf].
    auto request_rows = [&](int t, int buf, f32x4 (&r)[SI_BURST]) {
#pragma unroll
        for (int e = 0; e < SI_BURST; ++e) {
            const int q = e * SI_THREADS + t, qc = q < feat_units ? q : 0;     // unconditional, see the update's requests
            const int b = div_magic(qc, magic_row), c = qc - b * row_units;
            const float *src = shard + (size_t)ib[buf * p.B + b] * p.din;
            if (vec_rows) r[e] = load4(src + 4 * c); else r[e][0] = src[c];
        }
    };
    auto store_piece = [&](int q, const f32x4 &v) {
        const int b = div_magic(q, magic_row), c = q - b * row_units;
        float *dst = xs + (size_t)b * pitch;
        if (vec_rows) { dst[4 * c] = v[0]; dst[4 * c + 1] = v[1]; dst[4 * c + 2] = v[2]; dst[4 * c + 3] = v[3]; }
        else dst[c] = v[0];
    };
    // Four neighbouring parameters into LDS: the flat copy and the padded rows.
    auto keep_params = [&](int q, const f32x4 &v) {
        *reinterpret_cast<f32x4 *>(xl + (size_t)q * 4) = v;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int j = q * 4 + c;
            if (j < (int)p.D) {
                const int k = div_magic(j, magic_out);        // row din holds the bias
                wp[(size_t)k * WP + (j - k * p.dout)] = v[c];
            }
        }
    };

    // ---- before the first iteration: parameters, draws and batch rows, all requested before any is waited for
    const int t = t0;
    f32x4 rf[SI_BURST], rpar[SI_BURST];
#pragma unroll
    for (int e = 0; e < SI_BURST; ++e) {
        const int q = e * SI_THREADS + t;
        rpar[e] = load4(p.x_first + tiled_offset(p.M, i, (int64_t)(q < n_vec ? q : 0) * 4));
    }
    if (t < 2) cnt[t] = 0;
    int32_t label = draw_batch(t, iter0, 0);
    __syncthreads();
    const uint32_t thr_own = p.grad_only ? 0u : thr_row[t0 < p.M ? t0 : 0];      // the row does not change during a launch
    if (!p.grad_only) count_thresholds(t, iter0, 0, thr_own);
    request_rows(t, 0, rf);
#pragma unroll
    for (int e = 0; e < SI_BURST; ++e) {
        const int q = e * SI_THREADS + t;
        if (q < n_vec) keep_params(q, rpar[e]);
    }
    for (int q = SI_BURST * SI_THREADS + t; q < n_vec; q += SI_THREADS)
        keep_params(q, load4(p.x_first + tiled_offset(p.M, i, (int64_t)q * 4)));
    for (int q = t; q < (p.din + 1) * (CAP - p.dout); q += SI_THREADS) {       // the padding of every row
        const int k = q / (CAP - p.dout);
        wp[(size_t)k * WP + p.dout + (q - k * (CAP - p.dout))] = 0.0f;
    }
    if (t < p.B) yl[t] = label;
    for (int64_t j = p.D + t; j < p.ld; j += SI_THREADS) gl[j] = 0.0f;     // the padding behind the gradient: written here only

    for (int it = 0; it < p.n_iters; ++it) {
        const uint64_t iter = iter0 + (uint64_t)it;
        const int cur = it & 1, nxt = cur ^ 1;
        const bool more = it + 1 < p.n_iters;
        const int t = opaque(t0);
        float *Xcur = cur ? p.x_second : p.x_first;
        float *Xnext = cur ? p.x_first : p.x_second;
        // ---- this iteration's batch rows into LDS (the first pieces were requested an iteration ago)
#pragma unroll
        for (int e = 0; e < SI_BURST; ++e) {
            const int q = e * SI_THREADS + t;
            if (q < feat_units) store_piece(q, rf[e]);
        }
        for (int q = SI_BURST * SI_THREADS + t; q < feat_units; q += SI_THREADS) {
            const int b = div_magic(q, magic_row), c = q - b * row_units;
            const float *src = shard + (size_t)ib[cur * p.B + b] * p.din;
            f32x4 v;
            if (vec_rows) v = load4(src + 4 * c); else v[0] = src[c];
            store_piece(q, v);
        }

        __syncthreads();
        // ---- the peer
        int m = i;
        if (!p.grad_only) {
            const int c = cnt[cur];
            m = c < last_i ? c : last_i;
            if (t == 0) p.peers[i] = m;
        }
        // the next iteration's batch draw (its labels travel while this iteration computes)
        if (more) {
            if (t == 0) cnt[nxt] = 0;
            label = draw_batch(t, iter + 1, nxt);
        }
        if constexpr (MM) {
            // ---- forward on matrix instructions: wave = (16-row tile of the batch, part of the features); four steps
            // of sixteen features are read from LDS together, then multiplied
            const int t = opaque(t0);
            const int lane = t & 63, wave = t >> 6, r = lane & 15, q = lane >> 4;
            constexpr int BT = MM ? RT : 1, KP = SI_WAVES / BT;
            const int KW = p.din / KP, rt = wave % BT, kp = wave / BT;
            const float *xrow = xs + (size_t)(16 * rt + r) * pitch + kp * KW + 4 * q;
            const float *wcol = wp + (size_t)(kp * KW + 4 * q) * WP + r;
            f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
            for (int k0 = 0; k0 < KW; k0 += 64) {
                f32x4 a[4];
                float b[4][4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    a[u] = *reinterpret_cast<const f32x4 *>(xrow + k0 + 16 * u);
#pragma unroll
                    for (int j = 0; j < 4; ++j) b[u][j] = wcol[(size_t)(k0 + 16 * u + j) * WP];
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u][j], b[u][j], acc, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) part[(size_t)(kp * p.B + 16 * rt + 4 * q + v) * 16 + r] = acc[v];
            __syncthreads();
            // ---- the parts added in order, bias, softmax, loss, dZ: sixteen lanes per batch row, one class each
            const float *bias = wp + (size_t)p.din * WP;
            for (int e = t; e < p.B * 16; e += SI_THREADS) {
                const int b = e >> 4, c = e & 15;
                float z = part[(size_t)b * 16 + c];
#pragma unroll
                for (int kk = 1; kk < KP; ++kk) z += part[(size_t)(kk * p.B + b) * 16 + c];
                const bool real = c < p.dout;
                z = real ? z + bias[c] : -INFINITY;
                float mx = z;
                mx = fmaxf(mx, xor_lane<1>(mx));
                mx = fmaxf(mx, xor_lane<2>(mx));
                mx = fmaxf(mx, xor_lane<4>(mx));
                mx = fmaxf(mx, __shfl_xor(mx, 8, 16));
                const float ex = real ? expf(z - mx) : 0.0f;
                float sum = ex;
                sum += xor_lane<1>(sum);
                sum += xor_lane<2>(sum);
                sum += xor_lane<4>(sum);
                sum += __shfl_xor(sum, 8, 16);
                const int y = yl[cur * p.B + b];
                dz[(size_t)b * CAP + c] = real ? (ex * (1.0f / sum) - (c == y ? 1.0f : 0.0f)) * invB : 0.0f;
                if (c == y) lb[b] = logf(sum) - (z - mx);
            }
        } else {
        // ---- forward, softmax, loss, dZ: eight lanes per batch row; lane s adds the features s, s + 8, ... in order,
        // the lanes then add their partial sums in halves, so that each ends up owning OWN classes of the row
        {
            const int t = opaque(t0);
            const int sub = t & (SI_SPLIT - 1);
            const int own0 = ((sub >> 2) & 1) * (CAP / 2) + ((sub >> 1) & 1) * (CAP / 4) + (sub & 1) * (CAP / 8);
            const float *bias = wp + (size_t)p.din * WP;
            for (int b0 = 0; b0 < p.B; b0 += SI_THREADS / SI_SPLIT) {
                const int b = b0 + t / SI_SPLIT;
                const bool row_ok = b < p.B;
                float acc[CAP];
#pragma unroll
                for (int o = 0; o < CAP; ++o) acc[o] = 0.0f;
                if (row_ok) {
                    // SI_DEPTH steps at a time: all their LDS reads are requested, then all their products are added
                    for (int k0 = sub; k0 < p.din; k0 += SI_SPLIT * SI_DEPTH) {
                        float x[SI_DEPTH];
                        f32x4 wv[SI_DEPTH][CAP / 4];
#pragma unroll
                        for (int u = 0; u < SI_DEPTH; ++u) {
                            const int k = k0 + u * SI_SPLIT;
                            const bool in = k < p.din;
                            x[u] = in ? xs[(size_t)b * pitch + k] : 0.0f;
                            const f32x4 *wk = reinterpret_cast<const f32x4 *>(wp + (size_t)(in ? k : 0) * WP);
#pragma unroll
                            for (int o4 = 0; o4 < CAP / 4; ++o4) wv[u][o4] = wk[o4];
                        }
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int u = 0; u < SI_DEPTH; ++u)
#pragma unroll
                            for (int o4 = 0; o4 < CAP / 4; ++o4)
#pragma unroll
                                for (int c = 0; c < 4; ++c) acc[4 * o4 + c] = fmaf(x[u], wv[u][o4][c], acc[4 * o4 + c]);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                // halving exchange over the lane bits 4, 2, 1: a lane keeps the half its bit selects and adds the partner's
                {
                    const bool up4 = (sub & 4) != 0, up2 = (sub & 2) != 0, up1 = (sub & 1) != 0;
#pragma unroll
                    for (int j = 0; j < CAP / 2; ++j)
                        acc[j] = (up4 ? acc[j + CAP / 2] : acc[j]) + xor_lane<4>(up4 ? acc[j] : acc[j + CAP / 2]);
#pragma unroll
                    for (int j = 0; j < CAP / 4; ++j)
                        acc[j] = (up2 ? acc[j + CAP / 4] : acc[j]) + xor_lane<2>(up2 ? acc[j] : acc[j + CAP / 4]);
#pragma unroll
                    for (int j = 0; j < CAP / 8; ++j)
                        acc[j] = (up1 ? acc[j + CAP / 8] : acc[j]) + xor_lane<1>(up1 ? acc[j] : acc[j + CAP / 8]);
                }
                float z[OWN], mx = -INFINITY;
#pragma unroll
                for (int j = 0; j < OWN; ++j) {
                    z[j] = acc[j] + bias[own0 + j];
                    if (own0 + j < p.dout) mx = fmaxf(mx, z[j]);
                }
                mx = fmaxf(mx, xor_lane<1>(mx));
                mx = fmaxf(mx, xor_lane<2>(mx));
                mx = fmaxf(mx, xor_lane<4>(mx));
                const int y = row_ok ? yl[cur * p.B + b] : 0;
                float ex[OWN], sum = 0.0f, zy = 0.0f;
#pragma unroll
                for (int j = 0; j < OWN; ++j) {
                    ex[j] = own0 + j < p.dout ? expf(z[j] - mx) : 0.0f;
                    sum += ex[j];
                    zy += own0 + j == y ? z[j] : 0.0f;
                }
                sum += xor_lane<1>(sum);
                sum += xor_lane<2>(sum);
                sum += xor_lane<4>(sum);
                zy += xor_lane<1>(zy);
                zy += xor_lane<2>(zy);
                zy += xor_lane<4>(zy);
                if (row_ok) {
                    const float inv = 1.0f / sum;
#pragma unroll
                    for (int j = 0; j < OWN; ++j)
                        dz[(size_t)b * CAP + own0 + j] =
                            own0 + j < p.dout ? (ex[j] * inv - (own0 + j == y ? 1.0f : 0.0f)) * invB : 0.0f;
                    if (sub == 0) lb[b] = logf(sum) - (zy - mx);
                }
            }
        }
        }
        __syncthreads();
        // the peer's row and the own momentum are requested before the gradient is computed and used after it
        f32x4 rxp[SI_UPD], rv[SI_UPD];
        if (!p.grad_only) {
            const int t = opaque(t0);
#pragma unroll
            for (int e = 0; e < SI_UPD; ++e) {
                // unconditional (beyond the end: the first vector again, never used): a load under a branch is
                // waited for where the branches join, one round trip per pair instead of one for all
                const int q = e * SI_THREADS + t, qc = q < n_vec ? q : 0;
                rxp[e] = load4(Xcur + tiled_offset(p.M, m, (int64_t)qc * 4));
                rv[e] = load4(p.V + tiled_offset(p.M, i, (int64_t)qc * 4));
            }
        }
        if (more) count_thresholds(t, iter + 1, nxt, thr_own);
        // ---- gradient into LDS: dW[k][o] = sum_b x[b][k] dz[b][o], db[o] = sum_b dz[b][o] (batch rows in order), padding 0
        if constexpr (MM) {
            // a wave takes sixteen features at a time; the batch is the contraction (step s, lane group q: row 4 s + q)
            const int t = opaque(t0);
            const int lane = t & 63, wave = t >> 6, r = lane & 15, q = lane >> 4;
            constexpr int STEPS = MM ? 4 * RT : 1;           // batch / 4
            float bz[STEPS];
#pragma unroll
            for (int s4 = 0; s4 < STEPS; ++s4) bz[s4] = dz[(size_t)(4 * s4 + q) * CAP + r];
            for (int kt = wave; kt < (p.din >> 4); kt += SI_THREADS / 64) {
                float av[STEPS];
#pragma unroll
                for (int s4 = 0; s4 < STEPS; ++s4) av[s4] = xs[(size_t)(4 * s4 + q) * pitch + 16 * kt + r];
                __builtin_amdgcn_sched_barrier(0);
                f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int s4 = 0; s4 < STEPS; ++s4) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[s4], bz[s4], acc, 0, 0, 0);
                if (r < p.dout) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) gl[(size_t)(16 * kt + 4 * q + v) * p.dout + r] = acc[v];
                }
            }
            if (wave == SI_THREADS / 64 - 1) {
                // db = column sums of dZ: the same product with a row of ones in place of the features
                f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
                const float one = r == 0 ? 1.0f : 0.0f;
#pragma unroll
                for (int s4 = 0; s4 < STEPS; ++s4) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(one, bz[s4], acc, 0, 0, 0);
                if (q == 0 && r < p.dout) gl[(size_t)p.din * p.dout + r] = acc[0];
            }
            if (wave == 0) {
                // the loss: the rows' terms added by one wave in a fixed tree
                float l = lane < p.B ? lb[lane] : 0.0f;
#pragma unroll
                for (int m2 = 32; m2 > 0; m2 >>= 1) l += __shfl_xor(l, m2);
                if (lane == 0) p.loss[i] = l * invB;
            }
        } else {
            constexpr int OG = CAP / 4;                       // groups of four classes
            const int t = opaque(t0);
            const int og = t % OG, n_kg = (p.din + 3) >> 2;
            for (int kg = t / OG; kg < n_kg; kg += SI_THREADS / OG) {
                float acc[4][4];
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[a][c] = 0.0f;
                for (int b0 = 0; b0 < p.B; b0 += SI_DEPTH) {
                    float xv[SI_DEPTH][4];
                    f32x4 dv[SI_DEPTH];
#pragma unroll
                    for (int u = 0; u < SI_DEPTH; ++u) {
                        const int b = b0 + u < p.B ? b0 + u : p.B - 1;
                        const float *xr = xs + (size_t)b * pitch + 4 * kg;    // the row's pad keeps 4 kg + 3 inside it
#pragma unroll
                        for (int a = 0; a < 4; ++a) xv[u][a] = xr[a];
                        dv[u] = *reinterpret_cast<const f32x4 *>(dz + (size_t)b * CAP + 4 * og);
                        if (b0 + u >= p.B) dv[u] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int u = 0; u < SI_DEPTH; ++u)
#pragma unroll
                        for (int a = 0; a < 4; ++a)
#pragma unroll
                            for (int c = 0; c < 4; ++c) acc[a][c] = fmaf(xv[u][a], dv[u][c], acc[a][c]);
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        if (4 * kg + a < p.din && 4 * og + c < p.dout) gl[(size_t)(4 * kg + a) * p.dout + 4 * og + c] = acc[a][c];
            }
        }
        if (!MM && t < CAP) {                                 // the bias gradient
            float s = 0.0f;
#pragma unroll 8
            for (int b = 0; b < p.B; ++b) s += dz[(size_t)b * CAP + t];
            if (t < p.dout) gl[(size_t)p.din * p.dout + t] = s;
        }
        if (!MM && t == SI_THREADS - 1) {                     // batch rows in order
            float s = 0.0f;
#pragma unroll 8
            for (int b = 0; b < p.B; ++b) s += lb[b];
            p.loss[i] = s * invB;
        }
        __syncthreads();
        // ---- gradient to memory; momentum step and mix (Eq. (c0), (c1)) against the peer's previous copy; the new
        // parameters stay in LDS for the next iteration
        const float wi = p.grad_only ? 0.0f : p.w[(size_t)i * p.M + m];
        for (int q0 = 0; q0 < n_vec; q0 += SI_THREADS * SI_UPD) {
            if (q0 > 0 && !p.grad_only) {                     // beyond what was requested ahead
#pragma unroll
                for (int e = 0; e < SI_UPD; ++e) {
                    const int q = q0 + e * SI_THREADS + t, qc = q < n_vec ? q : 0;
                    rxp[e] = load4(Xcur + tiled_offset(p.M, m, (int64_t)qc * 4));
                    rv[e] = load4(p.V + tiled_offset(p.M, i, (int64_t)qc * 4));
                }
            }
#pragma unroll
            for (int e = 0; e < SI_UPD; ++e) {
                const int q = q0 + e * SI_THREADS + t;
                if (q < n_vec) {
                    const int64_t j = (int64_t)q * 4;
                    const size_t own = tiled_offset(p.M, i, j);
                    const f32x4 g = *reinterpret_cast<const f32x4 *>(gl + j);
                    store4(p.G + own, g);
                    if (!p.grad_only) {
                        const f32x4 x = *reinterpret_cast<const f32x4 *>(xl + j);
                        f32x4 xn, vn;
                        momentum_mix4(x, rv[e], g, rxp[e], wi, p.alpha, p.mu, p.wd, xn, vn);
                        store4(Xnext + own, xn);
                        store4(p.V + own, vn);
                        if (more) keep_params(q, xn);
                    }
                }
            }
        }
        if (more) {
            request_rows(t, nxt, rf);                         // the next iteration's batch rows travel across the barrier
            if (t < p.B) yl[nxt * p.B + t] = label;
            grid_barrier(p.barrier, p.barrier_base + (unsigned)(it + 1) * (unsigned)p.M, p.fault, p.patience);
        }
    }
}

bool small_iter_ok(int model_is_mlp, int n_layers, int bf16, int B, int64_t din, int64_t dout, int64_t ld)
{
    return model_is_mlp && n_layers == 1 && !bf16 && dout <= SI_MAX_OUT && din <= 4096 && ld <= 32768 &&
           small_iter_lds(B, (int)din, (int)dout, ld) <= (size_t)SI_LDS_LIMIT;
}

static const void *small_iter_kernel(int B, int64_t din, int64_t dout)
{
    if (small_iter_mm(B, din, dout)) {
        if (B == 16) return reinterpret_cast<const void *>(small_softmax_iteration_kernel<16, 1>);
        if (B == 32) return reinterpret_cast<const void *>(small_softmax_iteration_kernel<16, 2>);
        return reinterpret_cast<const void *>(small_softmax_iteration_kernel<16, 4>);
    }
    if (dout <= 8) return reinterpret_cast<const void *>(small_softmax_iteration_kernel<8>);
    if (dout <= 16) return reinterpret_cast<const void *>(small_softmax_iteration_kernel<16>);
    return reinterpret_cast<const void *>(small_softmax_iteration_kernel<SI_MAX_OUT>);
}

hipError_t prepare_small_iter()
{
    const void *kernels[] = {reinterpret_cast<const void *>(small_softmax_iteration_kernel<8>),
                             reinterpret_cast<const void *>(small_softmax_iteration_kernel<16>),
                             reinterpret_cast<const void *>(small_softmax_iteration_kernel<SI_MAX_OUT>),
                             reinterpret_cast<const void *>(small_softmax_iteration_kernel<16, 1>),
                             reinterpret_cast<const void *>(small_softmax_iteration_kernel<16, 2>),
                             reinterpret_cast<const void *>(small_softmax_iteration_kernel<16, 4>)};
    for (const void *k : kernels) {
        const hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, SI_LDS_LIMIT);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// cooperative != 0: every workgroup must be resident (the caller has checked M against small_iter_max_resident()).
hipError_t launch_small_iter(hipStream_t s, const SmallIterLaunch &a, int cooperative)
{
    SmallIterArgs p{};
    p.M = a.M; p.B = a.B; p.din = (int)a.din; p.dout = (int)a.dout; p.D = a.D; p.ld = a.ld;
    p.feats = a.feats; p.labels = a.labels; p.row0 = a.row0; p.n_rows = a.n_rows;
    p.thr = a.thr; p.last = a.last; p.w = a.w;
    p.x_first = a.x_first; p.x_second = a.x_second; p.V = a.V; p.G = a.G; p.loss = a.loss; p.peers = a.peers; p.idx = a.idx;
    p.alpha = a.alpha; p.mu = a.mu; p.wd = a.wd; p.seed = a.seed; p.iter = a.iter; p.n_iters = a.n_iters;
    p.grad_only = a.grad_only; p.barrier = a.barrier; p.barrier_base = a.barrier_base; p.fault = a.fault;
    p.workers = a.grad_only ? a.workers : nullptr;
    p.patience = a.patience;
    const unsigned groups = p.workers ? (unsigned)a.n_workers : (unsigned)a.M;
    const size_t lds = small_iter_lds(a.B, p.din, p.dout, a.ld);
    void *args[] = {&p};
    if (cooperative)
        return hipLaunchCooperativeKernel(small_iter_kernel(a.B, a.din, a.dout), dim3(groups), dim3(SI_THREADS), args, (unsigned)lds, s);
    return hipLaunchKernel(small_iter_kernel(a.B, a.din, a.dout), dim3(groups), dim3(SI_THREADS), args, lds, s);
}

// How many workgroups of the kernel fit on the device at once with this much LDS each (0 if unknown).
int small_iter_max_resident(int B, int64_t din, int64_t dout, int64_t ld)
{
    int per_cu = 0, dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
    if (!prop.cooperativeLaunch) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, small_iter_kernel(B, din, dout), SI_THREADS,
                                                     small_iter_lds(B, (int)din, (int)dout, ld)) != hipSuccess)
        return 0;
    return per_cu * prop.multiProcessorCount;
}

}  // namespace netmax
