// Last layer of a ReLU perceptron with few classes on fp32 operands, from the last hidden activation h to the error
// handed to the layer below (the stochastic gradient of Algorithm 2's first-step update, its part above the last
// hidden layer): logits = h W + b, softmax cross-entropy (mean loss, dZ = (softmax - onehot) / B), dW = h^T dZ,
// db = column sums of dZ, dH = (dZ W^T) masked by h > 0, and the column sums of dH = the bias gradient of the layer
// below.  The general kernels take five dependent launches of a few microseconds each for this; small perceptrons are
// bound by exactly that latency.  Here it is two:
//
//   head_logits_kernel  one workgroup per worker and 16 batch rows; its four waves split the hidden units, add their
//                       partial logits through LDS in wave order, then sixteen lanes per row do the softmax
//   head_grads_kernel   one workgroup per worker and 64 hidden units; a wave takes sixteen of them: sixteen rows of
//                       dW and sixteen columns of dH from one set of loads of h (the order of the contraction over
//                       the batch in dW is chosen so that the lanes hold the 16 x B block of h exactly as the result
//                       block of dH, which needs it for the ReLU mask)
//
// so that h is read once by each, by many compute units (one kernel that did everything per worker had a single
// compute unit pull 200 KB and took 14.6 us at 16 workers, 512 hidden units; these take 4 to 5 us each).
// The three products run on v_mfma_f32_16x16x4_f32 with the class dimension padded to one 16-wide tile (lane l
// supplies A[l % 16][l / 16] and B[l / 16][l % 16] and receives D[4 (l / 16) + v][l % 16], v = 0..3); the operands
// from W are loaded straight into that layout (a wave's load is 4 rows of W = 4 C contiguous floats).
// No load sits under a branch: where a bound has to be respected the index is clamped and the value discarded.
#include "kernels.h"
#include "layout.h"
#include "vec.h"

namespace netmax {

constexpr int HD_THREADS = 256, HD_WAVES = HD_THREADS / 64;
constexpr int HD_CP = 16;                       // padded class dimension
constexpr int HD_ZP = 20;                       // floats per row of dZ in LDS: the four row groups (16 rows apart) that a
                                                // wave reads at once fall into different banks
constexpr int HD_MAX_H = 1024;
constexpr int HD_KCHUNK = 128;                  // hidden units of one wave's part whose loads are in flight together

struct HeadArgs {
    const float *h;                 // [M][B][H] activation of the last hidden layer
    const float *X; float *G;       // parameters and gradient, tile layout
    const int32_t *labels; const int64_t *row0; const int32_t *idx;
    float *logits;                  // [M][B][C]
    float *dz;                      // [M][B][C]
    float *row_loss;                // [M][B] loss of every batch row (between the two kernels)
    float *dh;                      // [M][B][H]
    float *loss;                    // [M]
    int M, B, H, C;
    int64_t woff;                   // W [H][C] of the last layer inside a parameter row, its bias behind it
    int64_t boff_below;             // bias of the layer below
    int64_t D, ld;
};

__device__ __forceinline__ f32x4 mfma_16x16x4(float a, float b, f32x4 acc) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc, 0, 0, 0); }

// Grid: (B / 16, workers).
__global__ void __launch_bounds__(HD_THREADS) head_logits_kernel(HeadArgs p)
{
    __shared__ float part[HD_WAVES][16][HD_CP];
    const int B = p.B, H = p.H, C = p.C;
    const int g = blockIdx.y, rt = blockIdx.x, t = threadIdx.x, lane = t & 63, r = lane & 15, q = lane >> 4;
    const int kp = __builtin_amdgcn_readfirstlane(t >> 6);
    const int KW = H / HD_WAVES, k_begin = kp * KW, k_end = k_begin + KW;
    const float *a_ptr = p.h + ((size_t)g * B + 16 * rt + r) * H + 4 * q;
    const bool real = r < C;
    const int64_t wbase = p.woff + (real ? r : 0);
    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int k0 = k_begin; k0 < k_end; k0 += HD_KCHUNK) {
        f32x4 a[HD_KCHUNK / 16];
        float b[HD_KCHUNK / 16][4];
#pragma unroll
        for (int i = 0; i < HD_KCHUNK / 16; ++i) {
            const int kc = k0 + 16 * i < k_end ? k0 + 16 * i : k_begin;       // past the end: the first step again, unused
            a[i] = *reinterpret_cast<const f32x4 *>(a_ptr + kc);
#pragma unroll
            for (int j = 0; j < 4; ++j) b[i][j] = p.X[tiled_offset(p.M, g, wbase + (int64_t)(kc + 4 * q + j) * C)];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < HD_KCHUNK / 16; ++i)
            if (k0 + 16 * i < k_end) {
#pragma unroll
                for (int j = 0; j < 4; ++j) acc = mfma_16x16x4(a[i][j], real ? b[i][j] : 0.0f, acc);
            }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) part[kp][4 * q + v][r] = acc[v];
    __syncthreads();
    // the parts added in order, bias, softmax cross-entropy: sixteen lanes per batch row, one class each
    const int row = t >> 4, c = t & 15, b_row = 16 * rt + row;
    const bool cls = c < C;
    const float bias = p.X[tiled_offset(p.M, g, p.woff + (int64_t)H * C + (cls ? c : 0))];
    const int y = p.labels[p.row0[g] + p.idx[(size_t)g * B + b_row]];
    float z = ((part[0][row][c] + part[1][row][c]) + part[2][row][c]) + part[3][row][c];
    z = cls ? z + bias : -INFINITY;
    float mx = z;
#pragma unroll
    for (int m = 1; m < 16; m <<= 1) mx = fmaxf(mx, __shfl_xor(mx, m, 16));
    const float ex = cls ? expf(z - mx) : 0.0f;
    float sum = ex;
#pragma unroll
    for (int m = 1; m < 16; m <<= 1) sum += __shfl_xor(sum, m, 16);
    if (cls) {
        const size_t e = ((size_t)g * B + b_row) * C + c;
        p.logits[e] = z;
        p.dz[e] = (ex * (1.0f / sum) - (c == y ? 1.0f : 0.0f)) * (1.0f / (float)B);
    }
    if (c == y) p.row_loss[(size_t)g * B + b_row] = logf(sum) - (z - mx);
}

// RT: 16-row tiles of the batch (1, 2 or 4).  Grid: (ceil(H / 64), workers).
template <int RT>
__global__ void __launch_bounds__(HD_THREADS) head_grads_kernel(HeadArgs p)
{
    constexpr int B = 16 * RT, tp = B + 16;      // tp: pitch of the transposed dZ, rows 16 apart in banks
    __shared__ float dzs[B][HD_ZP];              // dZ, columns C .. 15 zero
    __shared__ float dzt[HD_CP][tp];             // its transpose
    const int H = p.H, C = p.C;
    const int g = blockIdx.y, t = threadIdx.x, lane = t & 63, r = lane & 15, q = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const bool first = blockIdx.x == 0;          // the workgroup that also writes what does not split by hidden units
    const int KT = H >> 4, kt = (int)blockIdx.x * HD_WAVES + wave;
    const int ktc = kt < KT ? kt : 0;            // waves past the end repeat the first block and store nothing
    const float *hg = p.h + (size_t)g * B * H;
    float *dhg = p.dh + (size_t)g * B * H;
    const int64_t boff = p.woff + (int64_t)H * C;
    // requests: this wave's 16 columns of h (all batch rows), its 16 rows of W, and dZ
    float hv[RT][4];                             // h[16 i + 4 q + v][16 kt + r]
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) hv[i][v] = hg[(16 * i + 4 * q + v) * H + 16 * ktc + r];
    float wv[4];                                 // W[16 kt + r][4 s + q]
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const float w = p.X[tiled_offset(p.M, g, p.woff + (int64_t)(16 * ktc + r) * C + (4 * s + q < C ? 4 * s + q : 0))];
        wv[s] = 4 * s + q < C ? w : 0.0f;
    }
    float zv[B * HD_CP / HD_THREADS];
#pragma unroll
    for (int u = 0; u < B * HD_CP / HD_THREADS; ++u) {
        const int e = t + u * HD_THREADS, row = e >> 4, c = e & 15;
        const float d = p.dz[((size_t)g * B + row) * C + (c < C ? c : 0)];
        zv[u] = c < C ? d : 0.0f;
    }
    float lrow = 0.0f;
    if (first && wave == 0) lrow = lane < B ? p.row_loss[(size_t)g * B + lane] : 0.0f;
#pragma unroll
    for (int u = 0; u < B * HD_CP / HD_THREADS; ++u) {
        const int e = t + u * HD_THREADS, row = e >> 4, c = e & 15;
        dzs[row][c] = zv[u];
        dzt[c][row] = zv[u];
    }
    __syncthreads();
    if (first) {
        if (wave == 0) {
#pragma unroll
            for (int m = 32; m > 0; m >>= 1) lrow += __shfl_xor(lrow, m);
            if (lane == 0) p.loss[g] = lrow / (float)B;
        }
        for (int64_t e = t; e < p.ld - p.D; e += HD_THREADS) p.G[tiled_offset(p.M, g, p.D + e)] = 0.0f;
        // db = column sums of dZ: the product below with a row of ones in place of h^T
        if (wave == HD_WAVES - 1) {
            f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
            const float one = r == 0 ? 1.0f : 0.0f;
#pragma unroll
            for (int s = 0; s < B / 4; ++s) acc = mfma_16x16x4(one, dzs[4 * s + q][r], acc);
            if (q == 0 && r < C) p.G[tiled_offset(p.M, g, boff + r)] = acc[0];
        }
    }
    if (kt >= KT) return;
    // ---- dW = h^T dZ, rows 16 kt .. 16 kt + 15: the batch is the contraction, taken in the order in which the lanes hold h
    {
        f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int i = 0; i < RT; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc = mfma_16x16x4(hv[i][v], dzs[16 * i + 4 * q + v][r], acc);
        if (r < C) {
#pragma unroll
            for (int v = 0; v < 4; ++v) p.G[tiled_offset(p.M, g, p.woff + (int64_t)(16 * kt + 4 * q + v) * C + r)] = acc[v];
        }
    }
    // ---- dH = (dZ W^T) where h > 0, columns 16 kt .. 16 kt + 15 of all batch rows, and its column sums
    {
        float colsum = 0.0f;
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int s = 0; s < 4; ++s) acc = mfma_16x16x4(dzt[4 * s + q][16 * i + r], wv[s], acc);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float d = hv[i][v] > 0.0f ? acc[v] : 0.0f;
                dhg[(16 * i + 4 * q + v) * H + 16 * kt + r] = d;
                colsum += d;
            }
        }
        colsum += __shfl_xor(colsum, 16);
        colsum += __shfl_xor(colsum, 32);
        if (q == 0) p.G[tiled_offset(p.M, g, p.boff_below + 16 * kt + r)] = colsum;
    }
}

// fp32 operands, a hidden layer below, at most 16 classes, a batch of 16, 32 or 64 rows, and a hidden width that the
// four waves of the logits kernel divide evenly in steps of sixteen.
bool head_ok(const MlpPlan &p)
{
    const int L = p.n_layers;
    if (p.bf16 || L < 2 || p.M > 65535) return false;
    const int64_t H = p.dims[L - 1], C = p.dims[L];
    const int B = p.B;
    if (C < 1 || C > HD_CP) return false;
    if (B != 16 && B != 32 && B != 64) return false;
    return H >= 64 && H <= HD_MAX_H && H % (16 * HD_WAVES) == 0;
}

hipError_t prepare_head() { return hipSuccess; }

void launch_head(hipStream_t s, const MlpPlan &p, const float *X, float *G)
{
    const int L = p.n_layers;
    HeadArgs a;
    a.h = p.act[L - 1]; a.X = X; a.G = G; a.labels = p.labels; a.row0 = p.row0; a.idx = p.idx;
    a.logits = p.act[L]; a.dz = p.dz[0]; a.dh = p.dz[1]; a.loss = p.loss;
    a.M = p.M; a.B = p.B; a.H = (int)p.dims[L - 1]; a.C = (int)p.dims[L];
    a.row_loss = p.dz[0] + (size_t)p.M * p.B * a.C;          // behind dZ: the buffer holds M x B x (widest layer) floats
    a.woff = p.woff[L - 1];
    a.boff_below = p.woff[L - 2] + p.dims[L - 2] * p.dims[L - 1];
    a.D = p.woff[L - 1] + p.dims[L - 1] * p.dims[L] + p.dims[L]; a.ld = p.ld;
    const dim3 block(HD_THREADS);
    hipLaunchKernelGGL(head_logits_kernel, dim3((unsigned)(a.B / 16), (unsigned)p.M), block, 0, s, a);
    const dim3 grid((unsigned)((a.H / 16 + HD_WAVES - 1) / HD_WAVES), (unsigned)p.M);
    switch (a.B / 16) {
    case 1: hipLaunchKernelGGL(head_grads_kernel<1>, grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL(head_grads_kernel<2>, grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL(head_grads_kernel<4>, grid, block, 0, s, a); break;
    }
}

}  // namespace netmax
