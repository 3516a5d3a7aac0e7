// Per-worker gradient of a ReLU perceptron with softmax cross-entropy (one layer = softmax regression):
// the stochastic gradient of Algorithm 2's first-step update, for all workers at once.  Every GEMM is
// grouped, one group per worker, because each worker multiplies its own batch with its own weights.
//
// This file holds the general tiled kernels (any shape, fp32 matrix instructions).  With bf16 operands the inputs of
// every product are rounded to bfloat16 first and accumulated in fp32.
#include "bf16.h"
#include "kernels.h"
#include "layout.h"
#include "softmax_xent.h"

#include <type_traits>

namespace netmax {

constexpr int GEMM_THREADS = 256;
typedef float gemm_acc __attribute__((ext_vector_type(16)));
constexpr int MAX_BATCH = 1024;

// Where the input of a layer comes from: the gathered data rows (fp32 or bfloat16 storage) for the first
// layer, else the previous layer's activation (fp32, or its stored bfloat16 copy when the operands are bf16).
enum : int { IN_GATHER_F32 = 0, IN_GATHER_BF16 = 1, IN_ACT_F32 = 2, IN_ACT_BF16 = 3 };

__device__ __forceinline__ float as_float(uint32_t u) { return __builtin_bit_cast(float, u); }
// Operands are rounded to bfloat16 exactly when the layer inputs are stored as bfloat16 (the odd kinds): a property
// of the instantiation, so the fp32 kernels carry no rounding code.
template <int KIND> __device__ __forceinline__ float operand(float x)
{
    if constexpr ((KIND & 1) != 0) return round_bf16(x);
    else return x;
}

// Input of layer l for worker g, batch row r, feature k.  bits<KIND>() is one unconditional load (the caller
// passes coordinates inside the operand), value<KIND>() turns what was loaded into the multiplicand.
struct LayerInput {
    const void *feats; const int64_t *row0; const int32_t *idx; const float *act_prev;
    const uint16_t *act_prev_bf16;
    int B; int64_t din; int kind;
    // rows: the worker's batch as absolute data rows (row0[g] + idx[g][b]), staged in LDS by the kernel
    template <int KIND> __device__ __forceinline__ uint32_t bits(int g, int r, int64_t k, const int64_t *rows) const
    {
        if constexpr (KIND == IN_GATHER_F32) return ((const uint32_t *)feats)[rows[r] * din + k];
        else if constexpr (KIND == IN_GATHER_BF16) return ((const uint16_t *)feats)[rows[r] * din + k];
        else if constexpr (KIND == IN_ACT_F32) return ((const uint32_t *)act_prev)[((size_t)g * B + r) * din + k];
        else return act_prev_bf16[((size_t)g * B + r) * din + k];
    }
    template <int KIND> __device__ __forceinline__ float value(uint32_t u) const
    {
        if constexpr (KIND == IN_GATHER_BF16 || KIND == IN_ACT_BF16) return as_float(u << 16);
        else return as_float(u);
    }
    // the same element as bits(): element index of feature 0 of batch row r, and the load of index + k
    template <int KIND> __device__ __forceinline__ int64_t row_index(int g, int r, const int64_t *rows) const
    {
        if constexpr (KIND == IN_GATHER_F32 || KIND == IN_GATHER_BF16) return rows[r] * din;
        else return ((int64_t)g * B + r) * din;
    }
    template <int KIND> __device__ __forceinline__ uint32_t load_index(int64_t index) const
    {
        if constexpr (KIND == IN_GATHER_F32) return ((const uint32_t *)feats)[index];
        else if constexpr (KIND == IN_GATHER_BF16) return ((const uint16_t *)feats)[index];
        else if constexpr (KIND == IN_ACT_F32) return ((const uint32_t *)act_prev)[index];
        else return act_prev_bf16[index];
    }
};

// tiled_offset() with one 32 x 32 -> 64 bit multiply-add: j + (((j >> 11) (M - 1) + i) << 11); needs j < 2^43
__device__ __forceinline__ size_t tiled_offset_quick(int M, int i, int64_t j)
{
    const uint64_t t = (uint64_t)(uint32_t)(j >> TILE_SHIFT) * (uint32_t)(M - 1) + (uint32_t)i;
    return (size_t)j + (size_t)(t << TILE_SHIFT);
}

// Z = A W + b, optional ReLU.  rows = batch, cols = dout, K = din.
struct FwdProblem {
    static constexpr bool A_K_FAST = true, B_C_FAST = true;
    LayerInput in; const float *X; int64_t woff, din, dout; int M, B, relu; float *out;
    uint16_t *out_bf16, *out_bf16_t;     // optional bfloat16 copies: [B][dout] and transposed [dout][B]
    __device__ int rows() const { return B; }
    __device__ int64_t cols() const { return dout; }
    __device__ int64_t depth() const { return din; }
    __device__ const LayerInput &input() const { return in; }
    template <int AK> __device__ uint32_t a_bits(int g, int64_t r, int64_t k, const int64_t *rows) const
    {
        return in.bits<AK>(g, (int)r, k, rows);
    }
    template <int AK> __device__ float a_val(uint32_t u) const { return in.value<AK>(u); }
    __device__ uint32_t b_bits(int g, int64_t k, int64_t c) const
    {
        return ((const uint32_t *)X)[tiled_offset(M, g, woff + k * dout + c)];
    }
    template <int AK> __device__ float b_val(uint32_t u) const { return operand<AK>(as_float(u)); }
    // the operands as base + k * step: what does not depend on the contraction index is computed once per thread
    static constexpr bool A_AFFINE = true;
    template <int AK> __device__ int64_t a_base(int g, int64_t r, const int64_t *rows) const { return in.row_index<AK>(g, (int)r, rows); }
    __device__ int64_t a_step() const { return 1; }
    template <int AK> __device__ uint32_t a_at(int64_t index) const { return in.load_index<AK>(index); }
    __device__ int64_t b_base(int g, int64_t c) const { return woff + c; }
    __device__ int64_t b_step() const { return dout; }
    __device__ uint32_t b_at(int g, int64_t index) const { return ((const uint32_t *)X)[tiled_offset_quick(M, g, index)]; }
    __device__ void store(int g, int64_t r, int64_t c, float acc) const
    {
        float z = acc + X[tiled_offset(M, g, woff + din * dout + c)];
        if (relu) z = z > 0.0f ? z : 0.0f;
        if (out) out[((size_t)g * B + r) * dout + c] = z;
        if (out_bf16) {
            const uint16_t h = (uint16_t)bf16_bits(z);
            out_bf16[((size_t)g * B + r) * dout + c] = h;
            out_bf16_t[((size_t)g * dout + c) * B + r] = h;
        }
    }
};

// dA = (dZ W^T) * [A > 0].  rows = batch, cols = din, K = dout.
struct DgradProblem {
    static constexpr bool A_K_FAST = true, B_C_FAST = false;
    const float *dz; const float *X; const float *act; const uint16_t *act_bf16; int64_t woff, din, dout;
    int M, B; float *out; uint16_t *out_bf16, *out_bf16_t;
    __device__ int rows() const { return B; }
    __device__ int64_t cols() const { return din; }
    __device__ int64_t depth() const { return dout; }
    __device__ LayerInput input() const { return LayerInput{}; }
    template <int AK> __device__ uint32_t a_bits(int g, int64_t r, int64_t k, const int64_t *) const
    {
        return ((const uint32_t *)dz)[((size_t)g * B + r) * dout + k];
    }
    template <int AK> __device__ float a_val(uint32_t u) const { return operand<AK>(as_float(u)); }
    __device__ uint32_t b_bits(int g, int64_t k, int64_t c) const
    {
        return ((const uint32_t *)X)[tiled_offset(M, g, woff + c * dout + k)];
    }
    template <int AK> __device__ float b_val(uint32_t u) const { return operand<AK>(as_float(u)); }
    static constexpr bool A_AFFINE = true;
    template <int AK> __device__ int64_t a_base(int g, int64_t r, const int64_t *) const { return ((int64_t)g * B + r) * dout; }
    __device__ int64_t a_step() const { return 1; }
    template <int AK> __device__ uint32_t a_at(int64_t index) const { return ((const uint32_t *)dz)[index]; }
    __device__ int64_t b_base(int g, int64_t c) const { return woff + c * dout; }
    __device__ int64_t b_step() const { return 1; }
    __device__ uint32_t b_at(int g, int64_t index) const { return ((const uint32_t *)X)[tiled_offset_quick(M, g, index)]; }
    __device__ void store(int g, int64_t r, int64_t c, float acc) const
    {
        const size_t q = ((size_t)g * B + r) * din + c;
        const bool on = act_bf16 ? bf16_positive(act_bf16[q]) : act[q] > 0.0f;
        const float d = on ? acc : 0.0f;
        out[q] = d;
        if (out_bf16) {
            const uint16_t h = (uint16_t)bf16_bits(d);
            out_bf16[q] = h;
            out_bf16_t[((size_t)g * din + c) * B + r] = h;
        }
    }
};

// dW = A^T dZ.  rows = din, cols = dout, K = batch.
struct WgradProblem {
    static constexpr bool A_K_FAST = false, B_C_FAST = true;
    LayerInput in; const float *dz; int64_t woff, din, dout; int M, B; float *G;
    __device__ int64_t rows() const { return din; }
    __device__ int64_t cols() const { return dout; }
    __device__ int64_t depth() const { return B; }
    __device__ const LayerInput &input() const { return in; }
    template <int AK> __device__ uint32_t a_bits(int g, int64_t r, int64_t k, const int64_t *rows) const
    {
        return in.bits<AK>(g, (int)k, r, rows);
    }
    template <int AK> __device__ float a_val(uint32_t u) const { return in.value<AK>(u); }
    __device__ uint32_t b_bits(int g, int64_t k, int64_t c) const
    {
        return ((const uint32_t *)dz)[((size_t)g * B + k) * dout + c];
    }
    template <int AK> __device__ float b_val(uint32_t u) const { return operand<AK>(as_float(u)); }
    static constexpr bool A_AFFINE = false;      // the batch row of contraction index k is looked up (gathered data)
    template <int AK> __device__ int64_t a_base(int, int64_t, const int64_t *) const { return 0; }
    __device__ int64_t a_step() const { return 0; }
    template <int AK> __device__ uint32_t a_at(int64_t) const { return 0u; }
    __device__ int64_t b_base(int g, int64_t c) const { return (int64_t)g * B * dout + c; }
    __device__ int64_t b_step() const { return dout; }
    __device__ uint32_t b_at(int, int64_t index) const { return ((const uint32_t *)dz)[index]; }
    __device__ void store(int g, int64_t r, int64_t c, float acc) const
    {
        G[tiled_offset(M, g, woff + r * dout + c)] = acc;
    }
};

// 64 x 64 output tile per workgroup (32 x 32 in the SMALL variant), one 32 x 32 quadrant per wave on v_mfma_f32_32x32x2_f32 (fp32 operands,
// exact products, fp32 accumulation), K in steps of 32 through LDS.  Lane l of the instruction supplies
// A[row l % 32][k = l / 32] and B[k = l / 32][col l % 32] and holds D[8 (v / 4) + 4 (l / 32) + v % 4][l % 32]
// in result register v.  The operands of the
// next step are fetched into registers while the current step is multiplied.  Every fetch is a run of
// unconditional loads: coordinates beyond the operand are clamped into it and the value is replaced by zero
// afterwards, the operand's kind AK is a template parameter and the worker's batch rows are resolved once into
// LDS, so that no load waits for a branch or for another load.
template <class Problem, int AK, bool SMALL = false>
__global__ void __launch_bounds__(GEMM_THREADS) grouped_gemm_kernel(Problem p)
{
    // SMALL: a 32 x 32 output tile; the four waves split every step's contraction indices between them (wave w takes
    // k = 8 w .. 8 w + 7) and their partial tiles are added through LDS at the end, in the order of the waves.  Four
    // times as many workgroups with a quarter of the matrix instructions per step each: for few, long problems.
    constexpr int TM = SMALL ? 32 : 64, TN = SMALL ? 32 : 64;
    constexpr int TK = SMALL ? 64 : 32;      // contraction indices per step
    __shared__ float As[TK][TM + 4];
    __shared__ float Bs[TK][TN + 4];
    __shared__ int64_t s_rows[MAX_BATCH];
    const int g = blockIdx.z, tid = threadIdx.x;
    const int64_t row0 = (int64_t)blockIdx.y * TM, col0 = (int64_t)blockIdx.x * TN;
    const int64_t R = p.rows(), C = p.cols(), K = p.depth();
    const int lane = tid & 63, wave = tid >> 6, wm = SMALL ? 0 : wave >> 1, wn = SMALL ? 0 : wave & 1;
    if (AK == IN_GATHER_F32 || AK == IN_GATHER_BF16) {
        const LayerInput in = p.input();
        for (int b = tid; b < in.B; b += GEMM_THREADS) s_rows[b] = in.row0[g] + in.idx[(size_t)g * in.B + b];
        __syncthreads();
    }
    constexpr int A_PER = (TM * TK) / GEMM_THREADS, B_PER = (TN * TK) / GEMM_THREADS;
    uint32_t ra[A_PER], rb[B_PER];
    unsigned a_ok = 0, b_ok = 0;          // bit q: element q of the fetch lies inside the operand
    // per element of a fetch: its index at contraction index kk (its own offset inside a step; row / column clamped
    // into the operand), so that a step only adds k0 * step, the same number for the whole workgroup
    int64_t a_idx[A_PER], b_idx[B_PER];
    unsigned a_in = 0, b_in = 0;          // bit q: the row / column of element q exists
    const int64_t a_step = p.a_step(), b_step = p.b_step();
#pragma unroll
    for (int q = 0; q < A_PER; ++q) {
        const int e = tid + q * GEMM_THREADS;
        const int r = Problem::A_K_FAST ? e / TK : e % TM, kk = Problem::A_K_FAST ? e % TK : e / TM;
        const int64_t rr = row0 + r;
        a_in |= (unsigned)(rr < R) << q;
        a_idx[q] = Problem::A_AFFINE ? p.template a_base<AK>(g, rr < R ? rr : R - 1, s_rows) + kk * a_step : 0;
    }
#pragma unroll
    for (int q = 0; q < B_PER; ++q) {
        const int e = tid + q * GEMM_THREADS;
        const int c = Problem::B_C_FAST ? e % TN : e / TK, kk = Problem::B_C_FAST ? e / TN : e % TK;
        const int64_t cc = col0 + c;
        b_in |= (unsigned)(cc < C) << q;
        b_idx[q] = p.b_base(g, cc < C ? cc : C - 1) + kk * b_step;
    }
    // full = std::true_type: every contraction index of the step is below K, nothing to clamp or mask along K
    auto fetch = [&](int64_t k0, auto full) {
        constexpr bool FULL = decltype(full)::value;
        a_ok = FULL ? a_in : 0u;
        b_ok = FULL ? b_in : 0u;
        const int64_t a_k0 = k0 * a_step, b_k0 = k0 * b_step;
#pragma unroll
        for (int q = 0; q < A_PER; ++q) {
            const int e = tid + q * GEMM_THREADS;
            const int r = Problem::A_K_FAST ? e / TK : e % TM, kk = Problem::A_K_FAST ? e % TK : e / TM;
            const int64_t kq = k0 + kk, kc = (FULL || kq < K) ? kq : K - 1;
            if (!FULL) a_ok |= (unsigned)(((a_in >> q) & 1u) && kq < K) << q;
            if constexpr (Problem::A_AFFINE) {
                ra[q] = p.template a_at<AK>(FULL ? a_idx[q] + a_k0 : a_idx[q] + (kc - kk) * a_step);
            } else {
                const int64_t rr = row0 + r;
                ra[q] = p.template a_bits<AK>(g, rr < R ? rr : R - 1, kc, s_rows);
            }
        }
#pragma unroll
        for (int q = 0; q < B_PER; ++q) {
            const int e = tid + q * GEMM_THREADS;
            const int kk = Problem::B_C_FAST ? e / TN : e % TK;
            const int64_t kq = k0 + kk, kc = (FULL || kq < K) ? kq : K - 1;
            if (!FULL) b_ok |= (unsigned)(((b_in >> q) & 1u) && kq < K) << q;
            rb[q] = p.b_at(g, FULL ? b_idx[q] + b_k0 : b_idx[q] + (kc - kk) * b_step);
        }
    };
    auto fetch_step = [&](int64_t k0) {
        if (k0 + TK <= K) fetch(k0, std::true_type{});
        else fetch(k0, std::false_type{});
    };
    gemm_acc acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    fetch_step(0);
    for (int64_t k0 = 0; k0 < K; k0 += TK) {
        __syncthreads();                       // the previous step's reads of LDS are done
#pragma unroll
        for (int q = 0; q < A_PER; ++q) {
            const int e = tid + q * GEMM_THREADS;
            int kk, r;
            if (Problem::A_K_FAST) { kk = e % TK; r = e / TK; } else { r = e % TM; kk = e / TM; }
            const float v = p.template a_val<AK>(ra[q]);
            As[kk][r] = ((a_ok >> q) & 1u) ? v : 0.0f;
        }
#pragma unroll
        for (int q = 0; q < B_PER; ++q) {
            const int e = tid + q * GEMM_THREADS;
            int kk, c;
            if (Problem::B_C_FAST) { c = e % TN; kk = e / TN; } else { kk = e % TK; c = e / TK; }
            const float v = p.template b_val<AK>(rb[q]);
            Bs[kk][c] = ((b_ok >> q) & 1u) ? v : 0.0f;
        }
        __syncthreads();
        if (k0 + TK < K) fetch_step(k0 + TK);
        constexpr int K_PER_WAVE = SMALL ? TK / 4 : TK;
#pragma unroll
        for (int kk = 0; kk < K_PER_WAVE; kk += 2) {
            const int k = (SMALL ? wave * K_PER_WAVE : 0) + kk + (lane >> 5);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(As[k][32 * wm + (lane & 31)], Bs[k][32 * wn + (lane & 31)], acc, 0, 0, 0);
        }
    }
    if constexpr (SMALL) {
        __shared__ float part[4][32][33];
#pragma unroll
        for (int v = 0; v < 16; ++v) part[wave][8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)][lane & 31] = acc[v];
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = tid + j * GEMM_THREADS, r = e >> 5, c = e & 31;
            const float sum = ((part[0][r][c] + part[1][r][c]) + part[2][r][c]) + part[3][r][c];
            if (row0 + r < R && col0 + c < C) p.store(g, row0 + r, col0 + c, sum);
        }
    } else {
    const int64_t cc = col0 + 32 * wn + (lane & 31);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int64_t rr = row0 + 32 * wm + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (rr < R && cc < C) p.store(g, rr, cc, acc[v]);
    }
    }
}

// Forward pass of a layer with few outputs (at most 32: the classifier layer), any input width and kind.  The tiled
// kernel above would use one 64-column tile per worker for it, most of it padding, on M workgroups.  Here a
// workgroup takes 16 batch rows of one worker; 16 threads share a row and split the contraction index between them
// (thread q takes k = q, q + 16, ...).  The weights of a chunk of the contraction are a run of consecutive
// parameters (rows of W are dout long), copied to LDS as they lie; all loads of a chunk are requested before the
// first is used.  The 16 partial sums of a row are added in a fixed butterfly order.  Products and sums in fp32.
constexpr int NARROW_ROWS = 16, NARROW_SPLIT = 16, NARROW_THREADS = NARROW_ROWS * NARROW_SPLIT, NARROW_WEIGHTS = 2048;
template <int AK, int CP>       // CP: outputs padded to 16 or 32
__global__ void __launch_bounds__(NARROW_THREADS) fwd_narrow_kernel(FwdProblem p)
{
    constexpr int CHUNK = NARROW_WEIGHTS / CP;                 // contraction indices per chunk
    constexpr int PER = CHUNK / NARROW_SPLIT, W_PER = NARROW_WEIGHTS / NARROW_THREADS;
    __shared__ float Wl[NARROW_WEIGHTS + CP];                   // CP more: the padded columns of the last row read on
    __shared__ int64_t s_row[NARROW_ROWS];
    const int g = blockIdx.y, tid = threadIdx.x, r = tid / NARROW_SPLIT, q = tid % NARROW_SPLIT;
    const int b = blockIdx.x * NARROW_ROWS + r;
    const int C = (int)p.dout;
    if (tid < NARROW_ROWS) {
        const int bb = blockIdx.x * NARROW_ROWS + tid;
        const int bq = bb < p.B ? bb : p.B - 1;              // rows beyond the batch repeat the last one and are not stored
        const LayerInput &in = p.in;
        s_row[tid] = (AK == IN_GATHER_F32 || AK == IN_GATHER_BF16) ? (in.row0[g] + in.idx[(size_t)g * in.B + bq]) * in.din
                                                                   : ((int64_t)g * in.B + bq) * in.din;
    }
    if (tid < CP) Wl[NARROW_WEIGHTS + tid] = 0.0f;
    __syncthreads();
    const int64_t a_row = s_row[r];
    float acc[CP];
#pragma unroll
    for (int c = 0; c < CP; ++c) acc[c] = 0.0f;
    // Chunks are small (8 loads of each kind per thread) and every loop over them is unrolled completely, so that the
    // staged values stay in registers; clamped unconditional loads, no predicates.
    for (int64_t k0 = 0; k0 < p.din; k0 += CHUNK) {
        const int n = (int)(p.din - k0 < CHUNK ? p.din - k0 : CHUNK), n_w = n * C;
        uint32_t av[PER], wv[W_PER];
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int kk = q + u * NARROW_SPLIT;
            av[u] = p.in.template load_index<AK>(a_row + k0 + (kk < n ? kk : n - 1));
        }
        const int64_t w0 = p.woff + k0 * p.dout;               // first parameter of the chunk
#pragma unroll
        for (int u = 0; u < W_PER; ++u) {
            const int e = tid + u * NARROW_THREADS;
            wv[u] = ((const uint32_t *)p.X)[tiled_offset_quick(p.M, g, w0 + (e < n_w ? e : n_w - 1))];
        }
        __syncthreads();                                       // the previous chunk has been used
#pragma unroll
        for (int u = 0; u < W_PER; ++u) {
            const int e = tid + u * NARROW_THREADS;
            Wl[e < n_w ? e : n_w - 1] = p.template b_val<AK>(wv[u]);     // clamped slots all hold the last weight
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int kk = q + u * NARROW_SPLIT;
            const float a = kk < n ? p.template a_val<AK>(av[u]) : 0.0f;
            const float *wk = Wl + (kk < n ? kk : 0) * C;
            // columns from C on multiply whatever follows the row (finite numbers); those sums are never stored
#pragma unroll
            for (int c = 0; c < CP; ++c) acc[c] = fmaf(a, wk[c], acc[c]);
        }
    }
    // the 16 partial sums of a row sit in 16 neighbouring lanes: butterfly over lane distances 8, 4, 2, 1
#pragma unroll
    for (int c = 0; c < CP; ++c)
#pragma unroll
        for (int d = NARROW_SPLIT / 2; d > 0; d >>= 1) acc[c] += __shfl_xor(acc[c], d, 64);
    if (b < p.B) {
#pragma unroll
        for (int c0 = 0; c0 < CP; c0 += NARROW_SPLIT) {        // thread q stores columns q, q + 16
            float v = 0.0f;
#pragma unroll
            for (int c = 0; c < NARROW_SPLIT; ++c) v = (c == q) ? acc[c0 + c] : v;
            if (c0 + q < C) p.store(g, b, c0 + q, v);
        }
    }
}

template <int CP> static void launch_fwd_narrow_kind(hipStream_t s, const FwdProblem &p, int kind, dim3 grid)
{
    const dim3 block(NARROW_THREADS);
    switch (kind) {
    case IN_GATHER_F32: hipLaunchKernelGGL((fwd_narrow_kernel<IN_GATHER_F32, CP>), grid, block, 0, s, p); break;
    case IN_GATHER_BF16: hipLaunchKernelGGL((fwd_narrow_kernel<IN_GATHER_BF16, CP>), grid, block, 0, s, p); break;
    case IN_ACT_F32: hipLaunchKernelGGL((fwd_narrow_kernel<IN_ACT_F32, CP>), grid, block, 0, s, p); break;
    default: hipLaunchKernelGGL((fwd_narrow_kernel<IN_ACT_BF16, CP>), grid, block, 0, s, p); break;
    }
}
static void launch_fwd_narrow(hipStream_t s, const FwdProblem &p, int kind, int groups)
{
    const dim3 grid((unsigned)((p.B + NARROW_ROWS - 1) / NARROW_ROWS), (unsigned)groups);
    if (p.dout <= 16) launch_fwd_narrow_kind<16>(s, p, kind, grid);
    else launch_fwd_narrow_kind<32>(s, p, kind, grid);
}

template <class Problem> static dim3 gemm_grid(int groups, int64_t rows, int64_t cols, int tile = 64)
{
    return dim3((unsigned)((cols + tile - 1) / tile), (unsigned)((rows + tile - 1) / tile), (unsigned)groups);
}

static void launch_gemm(hipStream_t s, const DgradProblem &p, int kind, int groups, int64_t rows, int64_t cols)
{
    const dim3 grid = gemm_grid<DgradProblem>(groups, rows, cols);
    if (kind == IN_ACT_BF16) hipLaunchKernelGGL((grouped_gemm_kernel<DgradProblem, IN_ACT_BF16>), grid, dim3(GEMM_THREADS), 0, s, p);
    else hipLaunchKernelGGL((grouped_gemm_kernel<DgradProblem, IN_ACT_F32>), grid, dim3(GEMM_THREADS), 0, s, p);
}

// depth: the contraction length.  Few tiles and a long contraction (a small batch against a wide layer): the 32 x 32
// variant, whose four waves share each step, puts four times as many workgroups on the chip.
template <class Problem>
static void launch_gemm(hipStream_t s, const Problem &p, int kind, int groups, int64_t rows, int64_t cols, int64_t depth)
{
    dim3 grid = gemm_grid<Problem>(groups, rows, cols);
    const bool small = (int64_t)grid.x * grid.y * grid.z < 256 && depth >= 128;
    if (small) grid = gemm_grid<Problem>(groups, rows, cols, 32);
#define NETMAX_GEMM(KIND)                                                                                        \
    do {                                                                                                         \
        if (small) hipLaunchKernelGGL((grouped_gemm_kernel<Problem, KIND, true>), grid, dim3(GEMM_THREADS), 0, s, p);  \
        else hipLaunchKernelGGL((grouped_gemm_kernel<Problem, KIND, false>), grid, dim3(GEMM_THREADS), 0, s, p);       \
    } while (0)
    switch (kind) {
    case IN_GATHER_F32: NETMAX_GEMM(IN_GATHER_F32); break;
    case IN_GATHER_BF16: NETMAX_GEMM(IN_GATHER_BF16); break;
    case IN_ACT_F32: NETMAX_GEMM(IN_ACT_F32); break;
    default: NETMAX_GEMM(IN_ACT_BF16); break;
    }
#undef NETMAX_GEMM
}

// Softmax cross-entropy on the logits (softmax_xent.h): one workgroup per worker.
__global__ void __launch_bounds__(1024) softmax_xent_kernel(SoftmaxArgs a) { softmax_xent_block(a, blockIdx.x); }

// db = column sums of dZ.  One workgroup = one worker x 64 outputs; the batch rows are dealt to four groups of
// threads (rows r, r + 4, ...), whose partial sums are added in the order of the groups.
__global__ void __launch_bounds__(256)
bias_grad_kernel(int M, int B, int64_t dout, const float *__restrict__ dz, int64_t boff,
                 float *__restrict__ G)
{
    __shared__ float part[4][64];
    const int g = blockIdx.y, lane_c = threadIdx.x & 63, rg = threadIdx.x >> 6;
    const int64_t c = (int64_t)blockIdx.x * 64 + lane_c;
    float s = 0.0f;
    if (c < dout)
        for (int b = rg; b < B; b += 4) s += dz[((size_t)g * B + b) * dout + c];
    part[rg][lane_c] = s;
    __syncthreads();
    if (rg == 0 && c < dout) G[tiled_offset(M, g, boff + c)] = ((part[0][lane_c] + part[1][lane_c]) + part[2][lane_c]) + part[3][lane_c];
}

void launch_mlp_grad(hipStream_t s, const MlpPlan &p, const float *X, float *G, const MixArgs *fuse)
{
    const int L = p.n_layers;
    const bool bf = p.bf16 != 0;
    bool fast[8] = {};
    for (int l = 0; l < L; ++l) fast[l] = mfma_layer_ok(p, l);
    const bool small_last = mfma_small_last_ok(p);
    const bool head = head_ok(p);
    auto input_of = [&](int l) {
        LayerInput in;
        in.feats = p.feats; in.row0 = p.row0; in.idx = p.idx;
        in.act_prev = (l > 0 && !bf) ? p.act[l] : nullptr;
        in.act_prev_bf16 = (l > 0 && bf) ? p.hb[l] : nullptr;
        in.B = p.B; in.din = p.dims[l];
        in.kind = l == 0 ? (bf ? IN_GATHER_BF16 : IN_GATHER_F32) : (bf ? IN_ACT_BF16 : IN_ACT_F32);
        return in;
    };
    // forward.  With bf16 operands the hidden activations are kept as bfloat16 only (both orientations).
    for (int l = 0; l < L; ++l) {
        const bool last = (l + 1 == L);
        if (fast[l] && !last) {
            launch_fwd_mfma(s, p, l, X);
            continue;
        }
        if (last && small_last) {
            launch_fwd_small(s, p, X, G);
            continue;
        }
        if (last && head) break;         // the head kernel below starts from the last hidden activation
        if (fwd_f32_ok(p, l)) {
            launch_fwd_f32(s, p, l, X);
            continue;
        }
        FwdProblem f;
        f.in = input_of(l); f.X = X; f.M = p.M; f.woff = p.woff[l]; f.din = p.dims[l]; f.dout = p.dims[l + 1];
        f.B = p.B; f.relu = !last;
        f.out = (last || !bf) ? p.act[l + 1] : nullptr;
        f.out_bf16 = (bf && !last) ? p.hb[l + 1] : nullptr;
        f.out_bf16_t = (bf && !last) ? p.ht[l + 1] : nullptr;
        // few outputs: the tiled kernel would pad them to a 64-column tile on one workgroup per worker
        if (f.dout <= 32) launch_fwd_narrow(s, f, f.in.kind, p.M);
        else launch_gemm(s, f, f.in.kind, p.M, p.B, f.dout, f.din);
    }
    bool bias_done[8] = {};
    int cur = 0, l_top = L - 1;
    if (head) {
        // logits, loss, the last layer's gradient and the error of the last hidden layer (with its column sums)
        launch_head(s, p, X, G);
        bias_done[L - 1] = bias_done[L - 2] = true;
        l_top = L - 2;
        cur = 1;
    } else {
        // loss and dZ of the last layer
        const int sm_threads = p.B <= 64 ? 64 : (p.B <= 256 ? 256 : 1024);
        if (!small_last)             // (the last-layer forward kernel of the matrix-core path ends with it)
            hipLaunchKernelGGL(softmax_xent_kernel, dim3(p.M), dim3(sm_threads), 0, s, softmax_args(p, G));
        bias_done[L - 1] = true;     // by the kernel above
    }
    // backward
    for (int l = l_top; l >= 0; --l) {
        const int64_t din = p.dims[l], dout = p.dims[l + 1];
        if (fast[l]) {
            if (fuse) launch_wgrad_mix_mfma(s, p, l, cur, *fuse);
            else launch_wgrad_mfma(s, p, l, G, cur);
        } else if (l == L - 1 && small_last) {
            launch_wgrad_small(s, p, G, cur);
        } else if (wgrad_f32_ok(p, l)) {
            launch_wgrad_f32(s, p, l, G, p.dz[cur]);
        } else {
            WgradProblem wg;
            wg.in = input_of(l); wg.dz = p.dz[cur]; wg.M = p.M; wg.woff = p.woff[l]; wg.din = din; wg.dout = dout;
            wg.B = p.B; wg.G = G;
            launch_gemm(s, wg, wg.in.kind, p.M, din, dout, p.B);
        }
        if (!bias_done[l]) {
            hipLaunchKernelGGL(bias_grad_kernel, dim3((unsigned)((dout + 63) / 64), (unsigned)p.M), dim3(256), 0, s, p.M, p.B,
                               dout, p.dz[cur], p.woff[l] + din * dout, G);
        }
        if (l > 0) {
            if (fast[l]) {
                launch_dgrad_mfma(s, p, l, X, G, cur, !fast[l - 1]);
                bias_done[l - 1] = true;
            } else if (l == L - 1 && small_last) {
                launch_dgrad_small(s, p, X, G, cur, !fast[l - 1]);
                bias_done[l - 1] = true;
            } else {
                DgradProblem dg;
                dg.dz = p.dz[cur]; dg.X = X; dg.act = bf ? nullptr : p.act[l]; dg.act_bf16 = bf ? p.hb[l] : nullptr;
                dg.M = p.M; dg.woff = p.woff[l]; dg.din = din; dg.dout = dout; dg.B = p.B;
                dg.out = p.dz[cur ^ 1];
                dg.out_bf16 = bf ? p.dzb[cur ^ 1] : nullptr;
                dg.out_bf16_t = bf ? p.dzt[cur ^ 1] : nullptr;
                launch_gemm(s, dg, bf ? IN_ACT_BF16 : IN_ACT_F32, p.M, p.B, din);     // the kind only says whether operands are rounded
            }
            cur ^= 1;
        }
    }
}

}  // namespace netmax
