// Softmax cross-entropy on the logits of one worker, by one workgroup (any size up to 1024 threads, at least the batch):
// dz = (softmax - onehot) / B, the mean loss, the column sums of dz (the last layer's bias gradient) and the zeros of
// the padding behind the worker's gradient.  A function of its own because two kernels end with it: the one that only
// does this, and the last-layer forward kernel of the matrix-core path, whose workgroup holds all logits of its worker.
#pragma once
#include "bf16.h"
#include "kernels.h"
#include "layout.h"

namespace netmax {

struct SoftmaxArgs {
    int B; int64_t C; const float *logits; const int32_t *labels; const int64_t *row0; const int32_t *idx;
    float *dz; uint16_t *dz_bf16, *dz_bf16_t;      // the bfloat16 copies (both orientations) are optional
    float *loss; int M; int64_t boff, D, ld; float *G;
};

inline SoftmaxArgs softmax_args(const MlpPlan &p, float *G)
{
    const int L = p.n_layers;
    const bool bf = p.bf16 != 0;
    SoftmaxArgs a;
    a.B = p.B; a.C = p.dims[L]; a.logits = p.act[L]; a.labels = p.labels; a.row0 = p.row0; a.idx = p.idx;
    a.dz = p.dz[0]; a.dz_bf16 = bf ? p.dzb[0] : nullptr; a.dz_bf16_t = bf ? p.dzt[0] : nullptr;
    a.loss = p.loss; a.M = p.M; a.boff = p.woff[L - 1] + p.dims[L - 1] * p.dims[L];
    a.D = a.boff + p.dims[L]; a.ld = p.ld; a.G = G;
    return a;
}

// One thread per batch row; the workgroup then adds up the columns of dz (batch rows in a fixed order).
__device__ __forceinline__ void softmax_xent_block(const SoftmaxArgs &a, int g)
{
    const int B = a.B, M = a.M;
    const int64_t C = a.C, boff = a.boff, D = a.D, ld = a.ld;
    const float *logits = a.logits; const int32_t *labels = a.labels; const int64_t *row0 = a.row0; const int32_t *idx = a.idx;
    float *dz = a.dz; uint16_t *dz_bf16 = a.dz_bf16, *dz_bf16_t = a.dz_bf16_t; float *loss = a.loss, *G = a.G;
    __shared__ float red[1024];
    const int b = threadIdx.x;
    float l = 0.0f;
    if (b < B) {
        const float *z = logits + ((size_t)g * B + b) * C;
        float *d = dz + ((size_t)g * B + b) * C;
        float mx = z[0];
        for (int64_t o = 1; o < C; ++o) mx = fmaxf(mx, z[o]);
        float sum = 0.0f;
        for (int64_t o = 0; o < C; ++o) sum += expf(z[o] - mx);
        const int y = labels[row0[g] + idx[(size_t)g * B + b]];
        l = logf(sum) - (z[y] - mx);
        const float inv = 1.0f / sum, invB = 1.0f / (float)B;
        for (int64_t o = 0; o < C; ++o) {
            const float v = (expf(z[o] - mx) * inv - (o == y ? 1.0f : 0.0f)) * invB;
            d[o] = v;
            if (dz_bf16) {
                const uint16_t h = (uint16_t)bf16_bits(v);
                dz_bf16[((size_t)g * B + b) * C + o] = h;
                dz_bf16_t[((size_t)g * C + o) * B + b] = h;
            }
        }
    }
    red[b] = l;
    __syncthreads();                 // also: every row of dz is written
    for (int stride = 512; stride > 0; stride >>= 1) {
        if (b < stride && b + stride < (int)blockDim.x) red[b] += red[b + stride];
        __syncthreads();
    }
    if (b == 0) loss[g] = red[0] / (float)B;
    for (int64_t e = b; e < ld - D; e += blockDim.x) G[tiled_offset(M, g, D + e)] = 0.0f;
    // column sums of dz.  With few classes the rows are split over P groups of threads (rows part, part + P, ...),
    // whose partial sums are then added in the order of the groups; otherwise one thread per column.
    const int nt = (int)blockDim.x;
    if (C <= nt / 2) {
        const int c = (int)C, P = nt / c;
        __syncthreads();             // red[0] has been read
        if (b < c * P) {
            const int o = b % c, part = b / c;
            float s = 0.0f;
            for (int r = part; r < B; r += P) s += dz[((size_t)g * B + r) * C + o];
            red[b] = s;
        }
        __syncthreads();
        if (b < c) {
            float s = 0.0f;
            for (int part = 0; part < P; ++part) s += red[part * c + b];
            G[tiled_offset(M, g, boff + b)] = s;
        }
    } else {
        for (int64_t o = b; o < C; o += nt) {
            float s = 0.0f;
            for (int r = 0; r < B; ++r) s += dz[((size_t)g * B + r) * C + o];
            G[tiled_offset(M, g, boff + o)] = s;
        }
    }
}


}  // namespace netmax
