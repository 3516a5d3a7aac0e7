// Last layer of a ReLU perceptron with few classes on fp32 operands, from the last hidden activation h to the error
// handed to the layer below, in one kernel (the stochastic gradient of Algorithm 2's first-step update, its part
// above the last hidden layer): logits = h W + b, softmax cross-entropy (mean loss, dZ = (softmax - onehot) / B),
// dW = h^T dZ, db = column sums of dZ, dH = (dZ W^T) masked by h > 0, and the column sums of dH = the bias gradient
// of the layer below.  These are five dependent launches of a few microseconds each when done by the general
// kernels; small perceptrons are bound by exactly that latency.
//
// Workgroups of sixteen waves; a worker has one workgroup per 256 columns of h.  Each of them computes all logits and
// dZ (every column of h enters them); the products that follow split by columns of h: a wave takes sixteen of them,
// the matching sixteen rows of dW and sixteen columns of dH.  The three products run on v_mfma_f32_16x16x4_f32 with the
// class dimension padded to one 16-wide tile (lane l supplies A[l % 16][l / 16] and B[l / 16][l % 16] and receives
// D[4 (l / 16) + v][l % 16], v = 0..3).  W (with zero columns up to 16) and dZ (in both orientations) live in LDS.
// Every value of h a lane needs is requested when the kernel starts: the 16 x B block of h that a wave uses for dW
// is held by its lanes exactly as the result block of dH is (the order of the contraction over the batch is
// chosen that way), so one set of loads serves the product and the ReLU mask.
#include "kernels.h"
#include "layout.h"
#include "vec.h"

namespace netmax {

constexpr int HD_THREADS = 1024, HD_WAVES = HD_THREADS / 64;
constexpr int HD_CP = 16;                       // padded class dimension
constexpr int HD_WP = 20, HD_ZP = 20;           // floats per row of W and of dZ in LDS: the row groups that the four lane
                                                // groups of a wave read at once, 4 or 64 rows apart, fall into different banks
constexpr int HD_MAX_B = 64, HD_MAX_H = 1024;

struct HeadArgs {
    const float *h;                 // [M][B][H] activation of the last hidden layer
    const float *X; float *G;       // parameters and gradient, tile layout
    const int32_t *labels; const int64_t *row0; const int32_t *idx;
    float *logits;                  // [M][B][C]
    float *dz;                      // [M][B][C]
    float *dh;                      // [M][B][H]
    float *loss;                    // [M]
    int M, B, H, C;
    int64_t woff;                   // W [H][C] of the last layer inside a parameter row, its bias behind it
    int64_t boff_below;             // bias of the layer below
    int64_t D, ld;
};

static size_t head_lds_bytes(int B, int H)
{
    return sizeof(float) * ((size_t)H * HD_WP + 256 * HD_CP + (size_t)B * HD_ZP + (size_t)HD_CP * (B + 16) + HD_MAX_B);
}

__device__ __forceinline__ f32x4 mfma_16x16x4(float a, float b, f32x4 acc) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc, 0, 0, 0); }

// RT: 16-row tiles of the batch (1, 2 or 4).  Grid: (workers, ceil(H / 256)).
template <int RT>
__global__ void __launch_bounds__(HD_THREADS) head_kernel(HeadArgs p)
{
    extern __shared__ __attribute__((aligned(16))) float head_smem[];
    constexpr int B = 16 * RT;
    constexpr int KP = HD_WAVES / RT;            // parts of the contraction over H in the first product
    const int H = p.H, C = p.C;
    constexpr int tp = B + 16;                   // pitch of the transposed dZ: rows 16 apart in banks
    float *W = head_smem;                        // [H][HD_WP], columns C .. 15 zero
    float *part = W + (size_t)H * HD_WP;         // [KP][B][16] partial logits (KP * B = 256)
    float *dzs = part + 256 * HD_CP;             // [B][HD_ZP] dZ, columns C .. 15 zero
    float *dzt = dzs + B * HD_ZP;                // [16][tp] its transpose
    float *red = dzt + HD_CP * tp;               // [HD_MAX_B] loss per batch row
    const int g = blockIdx.x, t = threadIdx.x, lane = t & 63, r = lane & 15, q = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const bool first = blockIdx.y == 0;          // the workgroup that also writes what does not split by columns of h
    const float *hg = p.h + (size_t)g * B * H;
    float *dhg = p.dh + (size_t)g * B * H;
    const int64_t boff = p.woff + (int64_t)H * C;

    // ---- requests: the wave's part of h for the logits (row tile rt, part kp of H; eight steps of sixteen columns at
    // a time) and its 16 columns x B rows for the products after the softmax
    const int rt = wave % RT, kp = wave / RT, KW = H / KP, k_begin = kp * KW, k_end = k_begin + KW;
    const float *a_ptr = hg + (16 * rt + r) * H + 4 * q;
    f32x4 a[8];
    auto load_a = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (k0 + 16 * i < k_end) a[i] = *reinterpret_cast<const f32x4 *>(a_ptr + k0 + 16 * i);
    };
    load_a(k_begin);
    const int KT = H >> 4, kt = (int)blockIdx.y * HD_WAVES + wave;
    float hv[RT][4];                             // h[16 i + 4 q + v][16 kt + r]
    if (kt < KT) {
#pragma unroll
        for (int i = 0; i < RT; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) hv[i][v] = hg[(16 * i + 4 * q + v) * H + 16 * kt + r];
    }
    // W into LDS, eight requests per thread in flight (H * 16 is a multiple of the workgroup size)
    for (int e0 = t; e0 < H * HD_CP; e0 += 8 * HD_THREADS) {
        float w[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int e = e0 + u * HD_THREADS, k = e >> 4, c = e & 15;
            w[u] = (e < H * HD_CP && c < C) ? p.X[tiled_offset(p.M, g, p.woff + (int64_t)k * C + c)] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int e = e0 + u * HD_THREADS;
            if (e < H * HD_CP) W[(e >> 4) * HD_WP + (e & 15)] = w[u];
        }
    }
    __syncthreads();
    // ---- logits
    {
        f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int k0 = k_begin; k0 < k_end; k0 += 128) {
            if (k0 != k_begin) load_a(k0);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (k0 + 16 * i < k_end) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc = mfma_16x16x4(a[i][j], W[(k0 + 16 * i + 4 * q + j) * HD_WP + r], acc);
                }
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) part[((kp * B) + 16 * rt + 4 * q + v) * HD_CP + r] = acc[v];
    }
    __syncthreads();
    // ---- the parts added in order, bias, softmax cross-entropy: sixteen lanes per batch row, one class each
    for (int e = t; e < B * HD_CP; e += HD_THREADS) {
        const int row = e >> 4, c = e & 15;
        float z = part[row * HD_CP + c];
        for (int kk = 1; kk < KP; ++kk) z += part[(kk * B + row) * HD_CP + c];
        const bool real = c < C;
        if (real) {
            z += p.X[tiled_offset(p.M, g, boff + c)];
            if (first) p.logits[((size_t)g * B + row) * C + c] = z;
        } else {
            z = -INFINITY;
        }
        float mx = z;
#pragma unroll
        for (int m = 1; m < 16; m <<= 1) mx = fmaxf(mx, __shfl_xor(mx, m, 16));
        const float ex = real ? expf(z - mx) : 0.0f;
        float sum = ex;
#pragma unroll
        for (int m = 1; m < 16; m <<= 1) sum += __shfl_xor(sum, m, 16);
        const int y = p.labels[p.row0[g] + p.idx[(size_t)g * B + row]];
        const float inv = 1.0f / sum, invB = 1.0f / (float)B;
        const float d = real ? (ex * inv - (c == y ? 1.0f : 0.0f)) * invB : 0.0f;
        dzs[row * HD_ZP + c] = d;
        dzt[c * tp + row] = d;
        if (real && first) p.dz[((size_t)g * B + row) * C + c] = d;
        if (c == y) red[row] = logf(sum) - (z - mx);
    }
    __syncthreads();
    if (first) {
        if (wave == 0) {
            float l = 0.0f;
            for (int row = lane; row < B; row += 64) l += red[row];
#pragma unroll
            for (int m = 32; m > 0; m >>= 1) l += __shfl_xor(l, m);
            if (lane == 0) p.loss[g] = l / (float)B;
        }
        for (int64_t e = t; e < p.ld - p.D; e += HD_THREADS) p.G[tiled_offset(p.M, g, p.D + e)] = 0.0f;
        // db = column sums of dZ: the product below with a row of ones in place of h^T
        if (wave == HD_WAVES - 1) {
            f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
            const float one = r == 0 ? 1.0f : 0.0f;
#pragma unroll
            for (int s = 0; s < B / 4; ++s) acc = mfma_16x16x4(one, dzs[(4 * s + q) * HD_ZP + r], acc);
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
            for (int v = 0; v < 4; ++v) acc = mfma_16x16x4(hv[i][v], dzs[(16 * i + 4 * q + v) * HD_ZP + r], acc);
        if (r < C) {
#pragma unroll
            for (int v = 0; v < 4; ++v) p.G[tiled_offset(p.M, g, p.woff + (int64_t)(16 * kt + 4 * q + v) * C + r)] = acc[v];
        }
    }
    // ---- dH = (dZ W^T) where h > 0, columns 16 kt .. 16 kt + 15 of all batch rows, and its column sums
    {
        float b[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) b[s] = W[(16 * kt + r) * HD_WP + 4 * s + q];
        float colsum = 0.0f;
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int s = 0; s < 4; ++s) acc = mfma_16x16x4(dzt[(4 * s + q) * tp + 16 * i + r], b[s], acc);
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

// fp32 operands, a hidden layer below, at most 16 classes, a batch of 16, 32 or 64 rows, and a hidden width that
// the sixteen waves divide evenly in both products.
bool head_ok(const MlpPlan &p)
{
    const int L = p.n_layers;
    if (p.bf16 || L < 2) return false;
    const int64_t H = p.dims[L - 1], C = p.dims[L];
    const int B = p.B;
    if (C < 1 || C > HD_CP) return false;
    if (B != 16 && B != 32 && B != 64) return false;
    const int KP = HD_WAVES / (B / 16);
    if (H < 16 || H > HD_MAX_H || H % (16 * KP) != 0) return false;
    return true;
}

hipError_t prepare_head()
{
    const int bytes = (int)head_lds_bytes(HD_MAX_B, HD_MAX_H);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(head_kernel<1>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void *>(head_kernel<2>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void *>(head_kernel<4>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    return e;
}

void launch_head(hipStream_t s, const MlpPlan &p, const float *X, float *G)
{
    const int L = p.n_layers;
    HeadArgs a;
    a.h = p.act[L - 1]; a.X = X; a.G = G; a.labels = p.labels; a.row0 = p.row0; a.idx = p.idx;
    a.logits = p.act[L]; a.dz = p.dz[0]; a.dh = p.dz[1]; a.loss = p.loss;
    a.M = p.M; a.B = p.B; a.H = (int)p.dims[L - 1]; a.C = (int)p.dims[L];
    a.woff = p.woff[L - 1];
    a.boff_below = p.woff[L - 2] + p.dims[L - 2] * p.dims[L - 1];
    a.D = p.woff[L - 1] + p.dims[L - 1] * p.dims[L] + p.dims[L]; a.ld = p.ld;
    const dim3 grid((unsigned)p.M, (unsigned)((a.H / 16 + HD_WAVES - 1) / HD_WAVES)), block(HD_THREADS);
    const size_t lds = head_lds_bytes(a.B, a.H);
    switch (a.B / 16) {
    case 1: hipLaunchKernelGGL(head_kernel<1>, grid, block, lds, s, a); break;
    case 2: hipLaunchKernelGGL(head_kernel<2>, grid, block, lds, s, a); break;
    default: hipLaunchKernelGGL(head_kernel<4>, grid, block, lds, s, a); break;
    }
}

}  // namespace netmax
