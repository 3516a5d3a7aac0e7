// Hidden layers of a perceptron on fp32 operands with a batch of 32 or 64 rows: forward pass and weight gradient (the
// stochastic gradient of Algorithm 2's first-step update).  Every worker multiplies its own batch with its own weights, so a
// weight is used by `batch` rows and by nobody else: the products are bound by how fast W streams in (forward) and dW
// streams out (weight gradient), and with few workers by how much of that is in flight.  Both kernels hand the
// operands to v_mfma_f32_32x32x2_f32 (exact fp32 products, fp32 accumulation) in the layout the loads deliver them in.
//
// Forward, Z = A W + b: a workgroup takes 32 columns of one worker's W and all batch rows; its eight waves split
// the contraction (wave w takes indices 64 s + 8 w .. + 7) and add their partial tiles through LDS in the order of the
// waves.  W is read exactly once, as 128-bit loads of whole 128-byte row pieces, and turned into the matrix
// instruction's layout through a wave-private LDS buffer (no workgroup barrier in the loop); A is read straight into
// that layout (the two lane halves take four consecutive indices each; the eight waves together read 256 contiguous
// bytes of a row per step).  Four steps of loads are in flight per wave.
//
// Weight gradient, dW = A^T dZ: a workgroup takes 32 rows of dW (32 input features) of one worker; the strip of A^T
// stays in registers (batch / 2 values per lane) and each wave multiplies it with 32-column blocks of dZ, read
// straight into the instruction's layout as 128-byte row pieces; the result leaves as 128-byte row pieces.
#include "kernels.h"
#include "layout.h"
#include "vec.h"

namespace netmax {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int F32_THREADS = 512, F32_WAVES = F32_THREADS / 64, F32_COLS = 32, F32_KS = 8, F32_DEPTH = 4;

struct LayerF32Args {
    const float *feats; const int64_t *row0; const int32_t *idx;   // gather = 1: the layer's input is the batch rows of the data
    const float *act;                                              // gather = 0: [M][B][din]
    const float *X; float *G; const float *dz;                    // parameters / gradient (tile layout); dz [M][B][dout]
    float *out;                                                    // forward: [M][B][dout]
    int64_t woff, din, dout;
    int M, B, relu, gather;
};

__device__ __forceinline__ const float *input_row(const LayerF32Args &p, int g, int b)
{
    return p.gather ? p.feats + (p.row0[g] + p.idx[(size_t)g * p.B + b]) * p.din : p.act + ((size_t)g * p.B + b) * p.din;
}

// RT: 32-row tiles of the batch (1 or 2).  Grid: grouped_grid(workers, dout / 32).
template <int RT>
__global__ void __launch_bounds__(F32_THREADS) fwd_f32_kernel(LayerF32Args p)
{
    extern __shared__ __attribute__((aligned(16))) float f32_smem[];
    // in the loop: [wave][2][F32_KS][32] staging of W; afterwards [wave][32 RT][33] partial tiles
    const int t = threadIdx.x, lane = t & 63, row = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    int g;
    unsigned cblk;
    if (!decode_group(blockIdx.x, (unsigned)(p.dout / F32_COLS), p.M, g, cblk)) return;      // a worker's blocks share an XCD (its A)
    const int64_t col0 = (int64_t)cblk * F32_COLS;
    float *stage = f32_smem + wave * (2 * F32_KS * F32_COLS);
    const float bias = p.X[tiled_offset(p.M, g, p.woff + p.din * p.dout + col0 + (t & 31))];     // for the end; requested first
    const int kr = lane >> 3, c4 = (lane & 7) * 4;               // this lane's piece of a staged W block
    const int64_t wcol = p.woff + col0 + c4;
    const int total = (int)(p.din / F32_KS);
    f32x4 fa[F32_DEPTH][RT], fw[F32_DEPTH];
    auto request_w = [&](int d, int s) {
        fw[d] = *reinterpret_cast<const f32x4 *>(p.X + tiled_offset(p.M, g, wcol + ((int64_t)s * F32_KS + kr) * p.dout));
    };
    // this wave's steps are wave, wave + 8, ...: n_mine of them.  Requests beyond the last one repeat it (in bounds, never
    // used), so that the loop over whole groups of F32_DEPTH steps has no branch and waits for exactly the loads it uses.
    const int n_mine = wave < total ? (total - wave + F32_WAVES - 1) / F32_WAVES : 0;
    const int s_last = wave + F32_WAVES * (n_mine - 1);
    // the first pieces of W do not wait for the batch-row numbers that the addresses of A depend on
    if (n_mine > 0) {
#pragma unroll
        for (int d = 0; d < F32_DEPTH; ++d) request_w(d, wave + F32_WAVES * d < s_last ? wave + F32_WAVES * d : s_last);
    }
    const float *arow[RT];
#pragma unroll
    for (int i = 0; i < RT; ++i) arow[i] = input_row(p, g, 32 * i + row) + 4 * half;
    auto request_a = [&](int d, int s) {
#pragma unroll
        for (int i = 0; i < RT; ++i) fa[d][i] = *reinterpret_cast<const f32x4 *>(arow[i] + (int64_t)s * F32_KS);
    };
    auto request_clamped = [&](int d, int s) {
        const int sc = s < s_last ? s : s_last;
        request_a(d, sc);
        request_w(d, sc);
    };
    f32x16 acc[RT];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
    auto consume = [&](int d) {
        float *buf = stage + (d & 1) * (F32_KS * F32_COLS);
        *reinterpret_cast<f32x4 *>(buf + kr * F32_COLS + c4) = fw[d];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float b = buf[(4 * half + j) * F32_COLS + row];
#pragma unroll
            for (int i = 0; i < RT; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[d][i][j], b, acc[i], 0, 0, 0);
        }
        __builtin_amdgcn_wave_barrier();
    };
    if (n_mine > 0) {
#pragma unroll
        for (int d = 0; d < F32_DEPTH; ++d) request_a(d, wave + F32_WAVES * d < s_last ? wave + F32_WAVES * d : s_last);
        int done = 0;
        for (; done + F32_DEPTH <= n_mine; done += F32_DEPTH) {
#pragma unroll
            for (int d = 0; d < F32_DEPTH; ++d) {
                consume(d);
                request_clamped(d, wave + F32_WAVES * (done + d + F32_DEPTH));
            }
        }
#pragma unroll
        for (int d = 0; d < F32_DEPTH - 1; ++d)
            if (done + d < n_mine) consume(d);
    }
    __syncthreads();                                   // every wave is done with its staging buffer
    constexpr int PP = F32_COLS + 1;
    float *part = f32_smem;
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) part[(wave * 32 * RT + 32 * i + 8 * (v >> 2) + 4 * half + (v & 3)) * PP + row] = acc[i][v];
    __syncthreads();
    const int c = t & 31;
    for (int r = t >> 5; r < 32 * RT; r += F32_THREADS / 32) {
        float z = part[r * PP + c];
#pragma unroll
        for (int w = 1; w < F32_WAVES; ++w) z += part[(w * 32 * RT + r) * PP + c];
        z += bias;
        if (p.relu) z = z > 0.0f ? z : 0.0f;
        p.out[((size_t)g * p.B + r) * p.dout + col0 + c] = z;
    }
}

static size_t fwd_f32_lds(int RT)
{
    const size_t stage = (size_t)F32_WAVES * 2 * F32_KS * F32_COLS, part = (size_t)F32_WAVES * 32 * RT * (F32_COLS + 1);
    return sizeof(float) * (stage > part ? stage : part);
}

// HB = batch / 2: values of the A^T strip per lane.  Grid: grouped_grid(workers, ceil(din / 32) * ceil(dout / (32 * 4 * WG32_TILES)));
// a wave takes WG32_TILES 32 x 32 blocks of dW, four blocks apart, with the same strip of A^T.
constexpr int WG32_THREADS = 256, WG32_WAVES = WG32_THREADS / 64, WG32_TILES = 2;
template <int HB, bool GATHER>
__global__ void __launch_bounds__(WG32_THREADS) wgrad_f32_kernel(LayerF32Args p)
{
    const int t = threadIdx.x, lane = t & 63, col = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int nct = (int)(p.dout / F32_COLS);
    const unsigned groups = (unsigned)((nct + WG32_WAVES * WG32_TILES - 1) / (WG32_WAVES * WG32_TILES));
    int g;
    unsigned local;
    if (!decode_group(blockIdx.x, (unsigned)((p.din + 31) / 32) * groups, p.M, g, local)) return;   // a worker's blocks share an XCD (its dZ)
    const int ct0 = (int)(local % groups) * (WG32_WAVES * WG32_TILES) + wave;
    if (ct0 >= nct) return;
    const int64_t f0 = (int64_t)(local / groups) * 32;
    const int64_t feat = f0 + col < p.din ? f0 + col : p.din - 1;       // rows beyond din repeat the last one and are not stored
    const float *zbase = p.dz + ((size_t)g * p.B + half) * p.dout + col;
    float a[HB], b[HB];
#pragma unroll
    for (int j = 0; j < HB; ++j) b[j] = zbase[(size_t)(2 * j) * p.dout + ct0 * F32_COLS];
    if constexpr (GATHER) {
        // all batch-row numbers first, then all values: two rounds of loads, not one per row
        int32_t rows[HB];
#pragma unroll
        for (int j = 0; j < HB; ++j) rows[j] = p.idx[(size_t)g * p.B + 2 * j + half];
        __builtin_amdgcn_sched_barrier(0);
        const float *base = p.feats + p.row0[g] * p.din + feat;
#pragma unroll
        for (int j = 0; j < HB; ++j) a[j] = base[(int64_t)rows[j] * p.din];
    } else {
        const float *base = p.act + ((size_t)g * p.B + half) * p.din + feat;
#pragma unroll
        for (int j = 0; j < HB; ++j) a[j] = base[(size_t)(2 * j) * p.din];
    }
    __builtin_amdgcn_sched_barrier(0);               // every load is requested before the first product waits for one
    for (int ct = ct0; ct < nct && ct < ct0 + WG32_WAVES * WG32_TILES; ct += WG32_WAVES) {
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
        for (int j = 0; j < HB; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[j], b[j], acc, 0, 0, 0);
        const int next = ct + WG32_WAVES;
        if (next < nct && next < ct0 + WG32_WAVES * WG32_TILES) {
#pragma unroll
            for (int j = 0; j < HB; ++j) b[j] = zbase[(size_t)(2 * j) * p.dout + next * F32_COLS];
        }
        __builtin_amdgcn_sched_barrier(0);           // the next block's loads go out before this block's stores
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t fr = f0 + 8 * (v >> 2) + 4 * half + (v & 3);
            if (fr < p.din) p.G[tiled_offset(p.M, g, p.woff + fr * p.dout + ct * F32_COLS + col)] = acc[v];
        }
    }
}

static LayerF32Args layer_f32_args(const MlpPlan &p, int l, const float *X, float *G, const float *dz)
{
    LayerF32Args a{};
    a.feats = (const float *)p.feats; a.row0 = p.row0; a.idx = p.idx; a.act = l > 0 ? p.act[l] : nullptr;
    a.X = X; a.G = G; a.dz = dz; a.out = p.act[l + 1];
    a.woff = p.woff[l]; a.din = p.dims[l]; a.dout = p.dims[l + 1];
    a.M = p.M; a.B = p.B; a.relu = l + 1 < p.n_layers; a.gather = l == 0;
    return a;
}

static bool f32_layer_common(const MlpPlan &p, int l)
{
    return !p.bf16 && (p.B == 32 || p.B == 64) && p.dims[l + 1] % F32_COLS == 0;
}

// The forward kernel reads A and W with 128-bit loads: rows of A and the pieces of W must start at multiples of 16 bytes.
bool fwd_f32_ok(const MlpPlan &p, int l)
{
    if (!f32_layer_common(p, l) || p.dims[l] % F32_KS != 0 || p.woff[l] % 4 != 0) return false;
    const void *in = l == 0 ? p.feats : (const void *)p.act[l];
    return reinterpret_cast<uintptr_t>(in) % 16 == 0;
}

bool wgrad_f32_ok(const MlpPlan &p, int l) { return f32_layer_common(p, l); }

hipError_t prepare_f32_layers()
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fwd_f32_kernel<1>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)fwd_f32_lds(1));
    if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void *>(fwd_f32_kernel<2>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)fwd_f32_lds(2));
    return e;
}

void launch_fwd_f32(hipStream_t s, const MlpPlan &p, int l, const float *X)
{
    const LayerF32Args a = layer_f32_args(p, l, X, nullptr, nullptr);
    const dim3 grid(grouped_grid(p.M, (unsigned)(a.dout / F32_COLS))), block(F32_THREADS);
    if (p.B == 32) hipLaunchKernelGGL(fwd_f32_kernel<1>, grid, block, fwd_f32_lds(1), s, a);
    else hipLaunchKernelGGL(fwd_f32_kernel<2>, grid, block, fwd_f32_lds(2), s, a);
}

void launch_wgrad_f32(hipStream_t s, const MlpPlan &p, int l, float *G, const float *dz)
{
    const LayerF32Args a = layer_f32_args(p, l, nullptr, G, dz);
    const int nct = (int)(a.dout / F32_COLS);
    const int per_group = WG32_WAVES * WG32_TILES;
    const dim3 grid(grouped_grid(p.M, (unsigned)((a.din + 31) / 32) * (unsigned)((nct + per_group - 1) / per_group))), block(WG32_THREADS);
    if (p.B == 32) {
        if (a.gather) hipLaunchKernelGGL((wgrad_f32_kernel<16, true>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((wgrad_f32_kernel<16, false>), grid, block, 0, s, a);
    } else {
        if (a.gather) hipLaunchKernelGGL((wgrad_f32_kernel<32, true>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((wgrad_f32_kernel<32, false>), grid, block, 0, s, a);
    }
}

}  // namespace netmax
