// Grouped GEMMs of the perceptron gradient on the CDNA4 matrix cores, bf16 operands / fp32 accumulate.
// One group per worker (its own batch times its own weights), so every weight is used by only `batch`
// rows: the kernels are bound by streaming the fp32 master weights from HBM and the gradient back, and
// are organised around that (128-bit loads along the weights' contiguous dimension, conversion to
// bfloat16 on the way into LDS), with v_mfma_f32_32x32x16_bf16 doing the arithmetic.
//
// Lane layout of v_mfma_f32_32x32x16_bf16 (64 lanes, l = lane):
//   A operand: 8 values A[row = l % 32][k = 8 (l / 32) + 0..7]
//   B operand: 8 values B[k = 8 (l / 32) + 0..7][col = l % 32]
//   D:        16 values D[row = 4 (l / 32) + v % 4 + 8 (v / 4)][col = l % 32], v = 0..15
#include "bf16.h"
#include "kernels.h"
#include "layout.h"
#include "softmax_xent.h"
#include "vec.h"

namespace netmax {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int MF_THREADS = 256;      // 4 waves
constexpr int MF_BM = 128, MF_BN = 128;        // weight-gradient and forward tile
// Contraction step BK of the forward and backward-data kernels: operand rows in LDS are BK + 8 bf16 long
// (16-byte aligned, conflict-free 128-bit reads).

__device__ __forceinline__ f32x16 mfma_bf16(u32x4 a, u32x4 b, f32x16 acc)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}

// tiled_offset() with one 32 x 32 -> 64 bit multiply-add: j + (((j >> 11) (M - 1) + i) << 11); needs j < 2^43
__device__ __forceinline__ size_t tiled_offset_fast(int M, int i, int64_t j)
{
    const uint64_t t = (uint64_t)(uint32_t)(j >> TILE_SHIFT) * (uint32_t)(M - 1) + (uint32_t)i;
    return (size_t)j + (size_t)(t << TILE_SHIFT);
}

__device__ __forceinline__ int d_row(int lane, int v) { return 4 * (lane >> 5) + (v & 3) + 8 * (v >> 2); }

// Position (in bf16 elements) of the 16-byte unit u of row n in an operand tile whose units are permuted
// inside each row by the row's 16-block index.  The forward kernel writes its weight tile four rows apart per
// lane (rows 4 nq + e); without the permutation those 8-byte writes meet only four bank groups (8-way
// conflict), with it the conflict is 2-way; reads of whole units stay conflict-free.
__device__ __forceinline__ int swz_unit(int n, int u) { return (u ^ ((n >> 4) & 3)) << 3; }

// One contraction step of the 128 x 128 tile from LDS: As[m][k], Bs[n][k], both k-contiguous.
// SWZ: Bs rows are stored with swz_unit().
template <int BK, bool SWZ>
__device__ __forceinline__ void tile_mma_128(const uint16_t (*As)[BK + 8], const uint16_t (*Bs)[BK + 8], int wm, int wn,
                                             int lane, f32x16 (&acc)[2][2])
{
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
        const int u = 2 * ks + (lane >> 5);
        u32x4 a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) a[i] = *reinterpret_cast<const u32x4 *>(&As[64 * wm + 32 * i + (lane & 31)][8 * u]);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = 64 * wn + 32 * j + (lane & 31);
            b[j] = *reinterpret_cast<const u32x4 *>(&Bs[n][SWZ ? swz_unit(n, u) : 8 * u]);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = mfma_bf16(a[i], b[j], acc[i][j]);
    }
}

// ---------------------------------------------------------------------------------------------------
// Leaving a 128 x 128 result tile (waves 2 x 2, 64 x 64 each, final fp32 values in acc) as bfloat16 in both
// orientations.  The matrix-instruction layout gives a lane single elements of 32 different rows; written
// straight to memory that is 2-byte and 8-byte stores.  The tile goes through LDS instead, once row-major and
// once transposed, and leaves as whole 256-byte rows in 16-byte pieces.
constexpr int ST_PITCH = 128 + 8;                      // bf16 elements per staged row (272 B)
constexpr int ST_BYTES = 128 * ST_PITCH * 2;

// T[row][col] = bf16(acc) for the whole tile (2-byte LDS writes; lanes 0..31 neighbouring columns)
__device__ __forceinline__ void stage_rows(uint16_t (*T)[ST_PITCH], int wm, int wn, int lane, const f32x16 (&acc)[2][2])
{
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                T[64 * wm + 32 * i + d_row(lane, v)][64 * wn + 32 * j + (lane & 31)] = (uint16_t)bf16_bits(acc[i][j][v]);
}
// T[col][row] = bf16(acc): four consecutive rows per 8-byte LDS write
__device__ __forceinline__ void stage_cols(uint16_t (*T)[ST_PITCH], int wm, int wn, int lane, const f32x16 (&acc)[2][2])
{
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                u32x2 packed;
                packed.x = pack_bf16x2(acc[i][j][4 * q], acc[i][j][4 * q + 1]);
                packed.y = pack_bf16x2(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                *reinterpret_cast<u32x2 *>(&T[64 * wn + 32 * j + (lane & 31)][64 * wm + 32 * i + d_row(lane, 4 * q)]) = packed;
            }
}
// 128 staged rows of `len` valid bf16 elements each -> dst + r * stride, 16 bytes per thread and piece;
// only the first n_rows rows are written.
__device__ __forceinline__ void flush_rows(const uint16_t (*T)[ST_PITCH], int t, int n_rows, int len, uint16_t *dst, size_t stride)
{
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int chunk = t + q * MF_THREADS, r = chunk >> 4, c = (chunk & 15) * 8;
        if (r < n_rows && c < len) *reinterpret_cast<u32x4 *>(dst + (size_t)r * stride + c) = *reinterpret_cast<const u32x4 *>(&T[r][c]);
    }
}
// out[(g B + row) ld + c0 + col] and out_t[(g ld + c0 + col) B + row] from acc; all threads of the workgroup.
__device__ __forceinline__ void store_tile_bf16(uint16_t (*T)[ST_PITCH], int wm, int wn, int lane, int t, const f32x16 (&acc)[2][2],
                                                int g, int B, int64_t ld, int64_t c0, uint16_t *out, uint16_t *out_t)
{
    stage_rows(T, wm, wn, lane, acc);
    __syncthreads();
    flush_rows(T, t, B, 128, out + ((size_t)g * B) * ld + c0, (size_t)ld);
    __syncthreads();
    stage_cols(T, wm, wn, lane, acc);
    __syncthreads();
    flush_rows(T, t, 128, B, out_t + ((size_t)g * ld + c0) * B, (size_t)B);
}

// ---------------------------------------------------------------------------------------------------
// Forward: H = relu(A W + b) for one worker and one block of 128 output columns; all batch rows.
// A: gathered bf16 data rows (first layer) or the previous layer's bf16 activations [B][din].
// W: fp32 master weights [din][dout] inside the worker's parameter row (tile layout), read with 128-bit
// loads along dout, transposed 4 x 4 in registers and stored to LDS as bf16 [n][k].
// Output: bf16 activations, row-major [B][dout] and transposed [dout][B].
struct FwdMfmaArgs {
    const uint16_t *feats; const int64_t *row0; const int32_t *idx;   // first layer
    const uint16_t *a_prev;                                           // later layers: [M][B][din]
    const float *X; int64_t woff; int M, B; int64_t din, dout; int relu;
    uint16_t *out, *out_t;
};

template <bool FIRST, int BK>
__device__ __forceinline__ void fwd_mfma_body(const FwdMfmaArgs &p)
{
    constexpr int PITCH = BK + 8;
    constexpr int A_CH = MF_BM * BK / 8 / MF_THREADS;      // 16-byte chunks of A per thread and step
    constexpr int CPR = BK / 8;                            // chunks per A row
    constexpr int W_BL = BK / 32;                          // 4 (k) x 4 (n) blocks of W per thread and step
    // operand tiles during the contraction, the staging tile of the result afterwards
    constexpr int OPERAND_BYTES = (MF_BM + MF_BN) * PITCH * 2;
    __shared__ __attribute__((aligned(16))) unsigned char smem[OPERAND_BYTES > ST_BYTES ? OPERAND_BYTES : ST_BYTES];
    uint16_t (*As)[PITCH] = reinterpret_cast<uint16_t (*)[PITCH]>(smem);
    uint16_t (*Bs)[PITCH] = reinterpret_cast<uint16_t (*)[PITCH]>(smem + MF_BM * PITCH * 2);
    uint16_t (*T)[ST_PITCH] = reinterpret_cast<uint16_t (*)[ST_PITCH]>(smem);
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    int g;
    unsigned nblk;
    if (!decode_group(blockIdx.x, (unsigned)(p.dout / MF_BN), p.M, g, nblk)) return;
    const int64_t n0 = (int64_t)nblk * MF_BN;

    const uint16_t *a_src[A_CH];
    int a_row[A_CH], a_k[A_CH];
#pragma unroll
    for (int c = 0; c < A_CH; ++c) {
        const int chunk = t + c * MF_THREADS;
        a_row[c] = chunk / CPR;
        a_k[c] = (chunk % CPR) * 8;
        if (a_row[c] < p.B) {
            const int64_t row = FIRST ? p.row0[g] + p.idx[(size_t)g * p.B + a_row[c]] : (int64_t)g * p.B + a_row[c];
            a_src[c] = (FIRST ? p.feats : p.a_prev) + row * p.din + a_k[c];
        } else {
            a_src[c] = nullptr;
        }
    }
    // W: 4 (k) x 4 (n) blocks per thread.  One contraction step moves every load by BK rows of W =
    // BK * dout columns of the parameter row, a whole number of layout tiles (dout is a multiple of 128),
    // so the pointers advance by a constant.
    const int kg = t >> 5, nq = t & 31;
    const float *w_src[W_BL][4];
#pragma unroll
    for (int q = 0; q < W_BL; ++q)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            w_src[q][r] = p.X + tiled_offset(p.M, g, p.woff + n0 + 4 * nq + (int64_t)(4 * (kg + 8 * q) + r) * p.dout);
    const size_t w_step = (size_t)BK * (size_t)p.dout * (size_t)p.M;

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    u32x4 ra[A_CH];
    f32x4_t rw[W_BL][4];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int c = 0; c < A_CH; ++c)
            ra[c] = a_src[c] ? *reinterpret_cast<const u32x4 *>(a_src[c] + k0) : (u32x4){0u, 0u, 0u, 0u};
#pragma unroll
        for (int q = 0; q < W_BL; ++q)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                rw[q][r] = *reinterpret_cast<const f32x4_t *>(w_src[q][r]);
                w_src[q][r] += w_step;
            }
    };
    auto stash = [&]() {
#pragma unroll
        for (int c = 0; c < A_CH; ++c) *reinterpret_cast<u32x4 *>(&As[a_row[c]][a_k[c]]) = ra[c];
#pragma unroll
        for (int q = 0; q < W_BL; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e) {   // column n = 4 nq + e gets its four consecutive k
                u32x2 packed;
                packed.x = pack_bf16x2(rw[q][0][e], rw[q][1][e]);
                packed.y = pack_bf16x2(rw[q][2][e], rw[q][3][e]);
                const int n = 4 * nq + e, k4 = kg + 8 * q;       // k4: index of the group of four k
                *reinterpret_cast<u32x2 *>(&Bs[n][swz_unit(n, k4 >> 1) + 4 * (k4 & 1)]) = packed;
            }
    };

    fetch(0);
    for (int64_t k0 = 0; k0 < p.din; k0 += BK) {
        __syncthreads();            // the previous step's reads of LDS are done
        stash();
        __syncthreads();
        if (k0 + BK < p.din) fetch(k0 + BK);   // overlaps with the matrix instructions below
        tile_mma_128<BK, true>(As, Bs, wm, wn, lane, acc);
    }

    // epilogue: bias, ReLU, then bf16 in both layouts through LDS
    const float *bias = p.X;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int64_t col = n0 + 64 * wn + 32 * j + (lane & 31);
        const float bcol = bias[tiled_offset(p.M, g, p.woff + p.din * p.dout + col)];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float z = acc[i][j][v] + bcol;
                acc[i][j][v] = (p.relu && !(z > 0.0f)) ? 0.0f : z;
            }
    }
    __syncthreads();                 // the last step's reads of the operand tiles are done
    store_tile_bf16(T, wm, wn, lane, t, acc, g, p.B, p.dout, n0, p.out, p.out_t);
}

template <bool FIRST>
__global__ void __launch_bounds__(MF_THREADS) __attribute__((amdgpu_waves_per_eu(4, 4))) fwd_mfma_kernel(FwdMfmaArgs p)
{
    fwd_mfma_body<FIRST, 32>(p);
}
// ---------------------------------------------------------------------------------------------------
// Shared tail of the backward-data kernels.  The workgroup holds dA for all batch rows (waves 2 x 2, each
// 64 rows x 64 columns in acc[i][j]) of `c0 .. c0 + 127`: applies the ReLU mask of the layer's input, writes
// the error as bf16 [B][din] and transposed [din][B] (fp32 [B][din] too if out_f32 is given) and, because all
// rows of a column are here, the column sums = the bias gradient of the layer below, in a fixed order.
struct DgradOut {
    const uint16_t *act;          // bf16 activations of this layer's input [M][B][din] (ReLU mask)
    float *out_f32; uint16_t *out, *out_t;
    float *G; int64_t boff;       // bias gradient of the layer below: G[tile layout, boff + column]
};

// BURST: how many of the eight pieces of the activation tile a thread requests at a time (0: see below).
template <int BURST>
__device__ __forceinline__ void dgrad_tail(const DgradOut &o, int M, int g, int B, int64_t din, int64_t c0, int wm, int wn,
                                           int lane, int t, f32x16 (&acc)[2][2], uint16_t (*T)[ST_PITCH], float (*red)[2][64])
{
    const int wave = 2 * wm + wn;
    // the activations under the tile (ReLU mask) come in as whole rows
    // (all eight requested before the first is stored, rows past the batch clamped: a load under a bounds test is
    // waited for where the branches join, one round trip per load)
    if constexpr (BURST == 0) {
        // one piece at a time, each under its bounds test: for the kernel whose registers are all taken by the tile
        // (requesting the pieces together made it spill more and run 4 % slower)
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int chunk = t + q * MF_THREADS, r = chunk >> 4, c = (chunk & 15) * 8;
            if (r < B) *reinterpret_cast<u32x4 *>(&T[r][c]) = *reinterpret_cast<const u32x4 *>(o.act + ((size_t)g * B + r) * din + c0 + c);
        }
    } else {
#pragma unroll
    for (int q0 = 0; q0 < 8; q0 += (BURST > 0 ? BURST : 8)) {
        u32x4 mask_rows[BURST > 0 ? BURST : 1];
#pragma unroll
        for (int q = 0; q < BURST; ++q) {
            const int chunk = t + (q0 + q) * MF_THREADS, r = chunk >> 4, c = (chunk & 15) * 8;
            mask_rows[q] = *reinterpret_cast<const u32x4 *>(o.act + ((size_t)g * B + (r < B ? r : B - 1)) * din + c0 + c);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < BURST; ++q) {
            const int chunk = t + (q0 + q) * MF_THREADS, r = chunk >> 4, c = (chunk & 15) * 8;
            if (r < B) *reinterpret_cast<u32x4 *>(&T[r][c]) = mask_rows[q];
        }
    }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int cl = 64 * wn + 32 * j + (lane & 31);
        float csum = 0.0f;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = 64 * wm + 32 * i + d_row(lane, v);
                const float d = (row < B && bf16_positive(T[row][cl])) ? acc[i][j][v] : 0.0f;
                acc[i][j][v] = d;
                csum += d;
            }
        red[wave][j][lane] = csum;
    }
    if (o.out_f32) {                 // only when the layer below runs on the general fp32-input kernels
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = 64 * wm + 32 * i + d_row(lane, v);
                    if (row < B) o.out_f32[((size_t)g * B + row) * din + c0 + 64 * wn + 32 * j + (lane & 31)] = acc[i][j][v];
                }
    }
    __syncthreads();                 // every mask is read before the tile is overwritten
    store_tile_bf16(T, wm, wn, lane, t, acc, g, B, din, c0, o.out, o.out_t);
    if (t < 128) {                   // red[] was complete before the barriers above
        const int cwn = t >> 6, cj = (t >> 5) & 1, cl = t & 31;
        float sum = 0.0f;
#pragma unroll
        for (int cwm = 0; cwm < 2; ++cwm)
#pragma unroll
            for (int half = 0; half < 2; ++half) sum += red[2 * cwm + cwn][cj][cl + 32 * half];
        o.G[tiled_offset(M, g, o.boff + c0 + t)] = sum;
    }
}

// Backward through a layer: dA = (dZ W^T) * [A > 0] for one worker, all batch rows and 128 input features
// (the output columns).  dZ: bf16 [B][dout]; W rows are contiguous along the contraction index, so they go
// to LDS untransposed (128-byte row pieces per step).
struct DgradMfmaArgs {
    const uint16_t *dz; const float *X; int64_t woff; int M, B; int64_t din, dout;
    DgradOut o;
};

template <int BK>
__device__ __forceinline__ void dgrad_mfma_body(const DgradMfmaArgs &p)
{
    constexpr int PITCH = BK + 8;
    constexpr int A_CH = MF_BM * BK / 8 / MF_THREADS;      // 16-byte chunks of dZ per thread and step
    constexpr int CPR = BK / 8;
    constexpr int W_CH = MF_BN * BK / 4 / MF_THREADS;      // 16-byte chunks of W per thread and step
    constexpr int WPR = BK / 4;
    constexpr int OPERAND_BYTES = (MF_BM + MF_BN) * PITCH * 2;
    __shared__ __attribute__((aligned(16))) unsigned char smem[OPERAND_BYTES > ST_BYTES ? OPERAND_BYTES : ST_BYTES];
    uint16_t (*As)[PITCH] = reinterpret_cast<uint16_t (*)[PITCH]>(smem);
    uint16_t (*Bs)[PITCH] = reinterpret_cast<uint16_t (*)[PITCH]>(smem + MF_BM * PITCH * 2);
    uint16_t (*T)[ST_PITCH] = reinterpret_cast<uint16_t (*)[ST_PITCH]>(smem);
    __shared__ float red[4][2][64];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    int g;
    unsigned cblk;
    if (!decode_group(blockIdx.x, (unsigned)(p.din / MF_BN), p.M, g, cblk)) return;
    const int64_t c0 = (int64_t)cblk * MF_BN;     // first input feature (output column) of this block

    const uint16_t *a_src[A_CH];
    int a_row[A_CH], a_k[A_CH];
#pragma unroll
    for (int c = 0; c < A_CH; ++c) {
        const int chunk = t + c * MF_THREADS;
        a_row[c] = chunk / CPR;
        a_k[c] = (chunk % CPR) * 8;
        a_src[c] = a_row[c] < p.B ? p.dz + ((size_t)g * p.B + a_row[c]) * p.dout + a_k[c] : nullptr;
    }
    // W: 16-byte chunks, feature row = chunk / WPR, k offset 4 * (chunk % WPR)
    int w_row[W_CH], w_k[W_CH];
    int64_t w_col[W_CH];
#pragma unroll
    for (int r = 0; r < W_CH; ++r) {
        const int chunk = t + r * MF_THREADS;
        w_row[r] = chunk / WPR;
        w_k[r] = 4 * (chunk % WPR);
        w_col[r] = p.woff + (c0 + w_row[r]) * p.dout + w_k[r];
    }
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    u32x4 ra[A_CH];
    f32x4_t rw[W_CH];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int c = 0; c < A_CH; ++c)
            ra[c] = a_src[c] ? *reinterpret_cast<const u32x4 *>(a_src[c] + k0) : (u32x4){0u, 0u, 0u, 0u};
#pragma unroll
        for (int r = 0; r < W_CH; ++r) rw[r] = *reinterpret_cast<const f32x4_t *>(p.X + tiled_offset(p.M, g, w_col[r] + k0));
    };
    auto stash = [&]() {
#pragma unroll
        for (int c = 0; c < A_CH; ++c) *reinterpret_cast<u32x4 *>(&As[a_row[c]][a_k[c]]) = ra[c];
#pragma unroll
        for (int r = 0; r < W_CH; ++r) {
            u32x2 packed;
            packed.x = pack_bf16x2(rw[r][0], rw[r][1]);
            packed.y = pack_bf16x2(rw[r][2], rw[r][3]);
            *reinterpret_cast<u32x2 *>(&Bs[w_row[r]][w_k[r]]) = packed;
        }
    };

    // The contraction starts at a different offset in every workgroup and wraps around: at any moment the
    // workgroups then read different parts of their weight rows, which spreads the requests over the memory
    // channels (all rows of W start at multiples of 4 dout bytes, the same offset in every row would meet
    // the same few channels).
    const int n_steps = (int)(p.dout / BK);
    const int shift = (int)((cblk * 5u + (unsigned)g * 3u) % (unsigned)n_steps);
    auto k_of = [&](int s) { int q = s + shift; if (q >= n_steps) q -= n_steps; return (int64_t)q * BK; };
    fetch(k_of(0));
    for (int s = 0; s < n_steps; ++s) {
        __syncthreads();
        stash();
        __syncthreads();
        if (s + 1 < n_steps) fetch(k_of(s + 1));
        tile_mma_128<BK, false>(As, Bs, wm, wn, lane, acc);
    }
    __syncthreads();                 // the last step's reads of the operand tiles are done
    dgrad_tail<0>(p.o, p.M, g, p.B, p.din, c0, wm, wn, lane, t, acc, T, red);
}

__global__ void __launch_bounds__(MF_THREADS) __attribute__((amdgpu_waves_per_eu(4, 4))) dgrad_mfma_kernel(DgradMfmaArgs p)
{
    dgrad_mfma_body<32>(p);
}

// ---------------------------------------------------------------------------------------------------
// Weight gradient: dW = A^T dZ for one worker and a strip of rows of W.  The contraction runs over
// the batch (<= 128), so whole operand blocks fit in LDS: the strip's A^T block [rows][B] is loaded once,
// then the workgroup walks along the strip in blocks of 128 columns; the dZ^T block of the next step is
// fetched into registers while the matrix instructions of the current one run.  Both operands are the
// transposed bf16 copies (batch-contiguous), read with coalesced 128-bit loads.  The fp32 product leaves
// straight from the accumulators as 128-byte row pieces (non-temporal) into the gradient row.
struct WgradMfmaArgs {
    const uint16_t *a_t, *dz_t; int M, B; int64_t din, dout, woff; float *G;
    const uint16_t *feats; const int64_t *row0; const int32_t *idx;      // first layer: A^T is gathered from the data rows
};

constexpr int WG_PITCH = 128 + 8;            // bf16 elements per operand row in LDS (272 B)

// The strip's A^T block [ROWS][B] into LDS.  Layers above the first read it from the transposed bf16 activations
// (batch-contiguous rows, whole 16-byte chunks).  The first layer (feats != nullptr) takes it from the data rows of
// the worker's batch themselves: every batch row holds the strip's ROWS features as ROWS * 2 contiguous bytes; a
// thread loads eight of them and scatters them into eight rows of the block.  Neighbouring lanes take neighbouring
// batch rows (the same feature chunk): their 2-byte LDS writes fall into one row of the block, and the eight chunks
// of a data row's line are fetched from memory once and hit in the cache afterwards.
template <int ROWS>
__device__ __forceinline__ void load_at_block(uint16_t (*At)[WG_PITCH], int t, int g, int B, int64_t din, int64_t r0,
                                              const uint16_t *a_t, const uint16_t *feats, const int64_t *row0,
                                              const int32_t *idx)
{
    // No load sits under a branch (one under a bounds test is waited for where the branches join: a round trip per
    // load instead of one for all): indices past the end are clamped and what they load is not stored.
    if (feats) {
        constexpr int KC = ROWS / 8;                             // 16-byte chunks of a batch row inside the strip
        constexpr int N = KC * 128 / MF_THREADS;                 // chunks per thread at the largest batch
        const int n = KC * B;
        int kcs[N], bs[N];
        int32_t rows[N];
#pragma unroll
        for (int q = 0; q < N; ++q) {
            const int c = t + q * MF_THREADS, cc = c < n ? c : n - 1;
            kcs[q] = cc / B;
            bs[q] = cc - kcs[q] * B;
            rows[q] = idx[(size_t)g * B + bs[q]];                // all batch-row numbers first, then all rows
        }
        const uint16_t *base = feats + (size_t)row0[g] * din + r0;
        u32x4 v[N];
#pragma unroll
        for (int q = 0; q < N; ++q) v[q] = *reinterpret_cast<const u32x4 *>(base + (size_t)rows[q] * din + 8 * kcs[q]);
#pragma unroll
        for (int q = 0; q < N; ++q) {
            if (t + q * MF_THREADS < n) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    At[8 * kcs[q] + 2 * e][bs[q]] = (uint16_t)(v[q][e] & 0xFFFFu);
                    At[8 * kcs[q] + 2 * e + 1][bs[q]] = (uint16_t)(v[q][e] >> 16);
                }
            }
        }
        return;
    }
    const int chunks_per_row = B >> 3;
    const uint16_t *a_src = a_t + ((size_t)g * din + r0) * B;
    constexpr int N = ROWS * 16 / MF_THREADS;                    // chunks per thread at the largest batch
    const int n = ROWS * chunks_per_row;
    int rws[N], cols[N];
    u32x4 v[N];
#pragma unroll
    for (int q = 0; q < N; ++q) {
        const int c = t + q * MF_THREADS, cc = c < n ? c : n - 1;
        rws[q] = cc / chunks_per_row;
        cols[q] = (cc - rws[q] * chunks_per_row) * 8;
        v[q] = *reinterpret_cast<const u32x4 *>(a_src + (size_t)rws[q] * B + cols[q]);
    }
#pragma unroll
    for (int q = 0; q < N; ++q)
        if (t + q * MF_THREADS < n) *reinterpret_cast<u32x4 *>(&At[rws[q]][cols[q]]) = v[q];
}

// STRIP: rows of W per workgroup (128 or 64), BN: columns per block step (128 or 64); waves 2 x 2, each
// STRIP / 2 rows x BN / 2 columns.
constexpr int WG_STAGE_PITCH = 132;                  // floats per row of the staged output block
template <int STRIP, int BN>
__device__ __forceinline__ void wgrad_mfma_body(const WgradMfmaArgs &p)
{
    constexpr int RI = STRIP / 64;                               // 32-row tiles per wave
    constexpr int CJ = BN / 64;                                  // 32-column tiles per wave
    constexpr int Z_CHUNKS = BN * 128 / 8 / MF_THREADS;
    __shared__ __attribute__((aligned(16))) uint16_t At[STRIP][WG_PITCH];
    __shared__ __attribute__((aligned(16))) uint16_t Zt[BN][WG_PITCH];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    const unsigned nx = (unsigned)(p.dout / BN), ny = (unsigned)(p.din / STRIP);
    int g;
    unsigned strip;
    if (!decode_group(blockIdx.x, ny, p.M, g, strip)) return;
    const int64_t r0 = (int64_t)strip * STRIP;
    const int chunks_per_row = p.B >> 3;                        // 16-byte chunks; at most 16
    const uint16_t *z_src = p.dz_t + (size_t)g * p.dout * p.B;
    load_at_block<STRIP>(At, t, g, p.B, p.din, r0, p.a_t, p.feats, p.row0, p.idx);
    int c_row[Z_CHUNKS], c_col[Z_CHUNKS];
#pragma unroll
    for (int q = 0; q < Z_CHUNKS; ++q) {
        const int c = t + q * MF_THREADS;
        c_row[q] = c / chunks_per_row;
        c_col[q] = (c - c_row[q] * chunks_per_row) * 8;
    }
    const int n_chunks = BN * chunks_per_row;
    const int64_t lane_col = p.woff + (r0 + 32 * RI * wm + 4 * (lane >> 5)) * p.dout + 32 * CJ * wn + (lane & 31);
    u32x4 rz[Z_CHUNKS];
    auto fetch_z = [&](unsigned nb) {
#pragma unroll
        for (int q = 0; q < Z_CHUNKS; ++q)
            if (t + q * MF_THREADS < n_chunks)
                rz[q] = *reinterpret_cast<const u32x4 *>(z_src + ((size_t)nb * BN + c_row[q]) * p.B + c_col[q]);
    };
    fetch_z(0);

    for (unsigned nb = 0; nb < nx; ++nb) {
        __syncthreads();                                        // the previous block's reads of Zt are done
#pragma unroll
        for (int q = 0; q < Z_CHUNKS; ++q)
            if (t + q * MF_THREADS < n_chunks) *reinterpret_cast<u32x4 *>(&Zt[c_row[q]][c_col[q]]) = rz[q];
        __syncthreads();
        if (nb + 1 < nx) fetch_z(nb + 1);

        f32x16 acc[RI][CJ];
#pragma unroll
        for (int i = 0; i < RI; ++i)
#pragma unroll
            for (int j = 0; j < CJ; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
        for (int b0 = 0; b0 < p.B; b0 += 16) {
            const int kofs = b0 + 8 * (lane >> 5);
            u32x4 a[RI], b[CJ];
#pragma unroll
            for (int i = 0; i < RI; ++i) a[i] = *reinterpret_cast<const u32x4 *>(&At[32 * RI * wm + 32 * i + (lane & 31)][kofs]);
#pragma unroll
            for (int j = 0; j < CJ; ++j) b[j] = *reinterpret_cast<const u32x4 *>(&Zt[32 * CJ * wn + 32 * j + (lane & 31)][kofs]);
#pragma unroll
            for (int i = 0; i < RI; ++i)
#pragma unroll
                for (int j = 0; j < CJ; ++j) acc[i][j] = mfma_bf16(a[i], b[j], acc[i][j]);
        }
        if constexpr (STRIP == 64 && BN == 128) {
            // The block goes through LDS (the space of the dZ^T block, which every wave has finished reading) and
            // leaves as whole 512-byte row pieces, 16 bytes per lane, in one burst of stores per workgroup (measured:
            // 15 us less per iteration of the 3072-1024-1024 perceptron than 4-byte stores straight from the accumulators).
            float (*T)[WG_STAGE_PITCH] = reinterpret_cast<float (*)[WG_STAGE_PITCH]>(&Zt[0][0]);
            static_assert(sizeof(float) * 64 * WG_STAGE_PITCH <= sizeof(uint16_t) * BN * WG_PITCH, "the staged block fits the operand block");
            __syncthreads();
#pragma unroll
            for (int j = 0; j < CJ; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) T[32 * wm + d_row(lane, v)][64 * wn + 32 * j + (lane & 31)] = acc[0][j][v];
            __syncthreads();
            const int cq = (t & 31) * 4, r_in = t >> 5;              // 32 lanes along the 128 columns, 8 rows per pass
#pragma unroll
            for (int pass = 0; pass < 8; ++pass) {
                const int row = pass * 8 + r_in;
                const int64_t jj = p.woff + (r0 + row) * p.dout + (int64_t)nb * BN + cq;
                __builtin_nontemporal_store(*reinterpret_cast<const f32x4_t *>(&T[row][cq]),
                                            reinterpret_cast<f32x4_t *>(p.G + tiled_offset_fast(p.M, g, jj)));
            }
        } else {
        // column index inside the parameter row = lane part (fixed) + a part that is the same for the whole wave
#pragma unroll
        for (int i = 0; i < RI; ++i)
#pragma unroll
            for (int j = 0; j < CJ; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int64_t uni = (int64_t)(32 * i + (v & 3) + 8 * (v >> 2)) * p.dout + (int64_t)nb * BN + 32 * j;
                    __builtin_nontemporal_store(acc[i][j][v], p.G + tiled_offset_fast(p.M, g, lane_col + uni));
                }
        }
    }
}

// 64-row strips: 51 KB of LDS, three workgroups per compute unit, whose arithmetic and store phases overlap
// better than those of two workgroups with 128-row strips (measured: 13 % less time for both layers of the
// 3072-1024-1024 perceptron).
constexpr int WG_STRIP = 64;
__global__ void __launch_bounds__(MF_THREADS) __attribute__((amdgpu_waves_per_eu(3, 3))) wgrad_mfma_kernel(WgradMfmaArgs p)
{
    wgrad_mfma_body<WG_STRIP, 128>(p);
}

// ---------------------------------------------------------------------------------------------------
// Weight gradient with the second-step update applied in place of the store: one workgroup = one worker and one
// 64-row x 128-column block of W.  The product dW = A^T dZ of the block is computed as above, turned through LDS
// into rows, and every thread then updates four neighbouring parameters: v' = mu v + dW + wd x, h = x - alpha v',
// x' = h - w (h - x_peer) (Eq. (c0), (c1)) with 128-bit loads and stores.  The gradient never goes to memory.
// Workgroups are ordered block by block: all M workers of a block run side by side on one XCD (as the mix kernel
// orders its tiles), so the block a worker pulls from its peer is in that XCD's L2.
struct WgradMixArgs {
    const uint16_t *a_t, *dz_t; int M, B; int64_t din, dout, woff;
    MixArgs mix;
    const uint16_t *feats; const int64_t *row0; const int32_t *idx;      // first layer: A^T is gathered from the data rows
};
constexpr int WM_ROWS = 64, WM_COLS = 128;
constexpr int WM_TILE_PITCH = WM_COLS + 4;           // floats per staged row

__global__ void __launch_bounds__(MF_THREADS) __attribute__((amdgpu_waves_per_eu(3, 3))) wgrad_mix_mfma_kernel(WgradMixArgs p)
{
    constexpr int OPERAND_BYTES = (WM_ROWS + WM_COLS) * WG_PITCH * 2, TILE_BYTES = WM_ROWS * WM_TILE_PITCH * 4;
    __shared__ __attribute__((aligned(16))) unsigned char smem[OPERAND_BYTES > TILE_BYTES ? OPERAND_BYTES : TILE_BYTES];
    uint16_t (*At)[WG_PITCH] = reinterpret_cast<uint16_t (*)[WG_PITCH]>(smem);
    uint16_t (*Zt)[WG_PITCH] = reinterpret_cast<uint16_t (*)[WG_PITCH]>(smem + WM_ROWS * WG_PITCH * 2);
    float (*T)[WM_TILE_PITCH] = reinterpret_cast<float (*)[WM_TILE_PITCH]>(smem);
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    // workgroup id -> (block, worker): ids are dealt round-robin to the XCDs; a block's workers are consecutive slots
    const unsigned nbx = (unsigned)(p.dout / WM_COLS), blocks = nbx * (unsigned)(p.din / WM_ROWS);
    const unsigned xcd = blockIdx.x % MF_XCD, slot = blockIdx.x / MF_XCD;
    const unsigned blk = (slot / (unsigned)p.M) * MF_XCD + xcd;
    const int g = (int)(slot % (unsigned)p.M);
    if (blk >= blocks) return;
    const int64_t r0 = (int64_t)(blk / nbx) * WM_ROWS, n0 = (int64_t)(blk % nbx) * WM_COLS;
    const int chunks_per_row = p.B >> 3;
    const uint16_t *z_src = p.dz_t + ((size_t)g * p.dout + n0) * p.B;
    load_at_block<WM_ROWS>(At, t, g, p.B, p.din, r0, p.a_t, p.feats, p.row0, p.idx);
#pragma unroll
    for (int q = 0; q < WM_COLS * 16 / MF_THREADS; ++q) {
        const int c = t + q * MF_THREADS, row = c / chunks_per_row, col = (c - row * chunks_per_row) * 8;
        if (c < WM_COLS * chunks_per_row)
            *reinterpret_cast<u32x4 *>(&Zt[row][col]) = *reinterpret_cast<const u32x4 *>(z_src + (size_t)row * p.B + col);
    }
    __syncthreads();
    f32x16 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;
    for (int b0 = 0; b0 < p.B; b0 += 16) {
        const int kofs = b0 + 8 * (lane >> 5);
        const u32x4 a = *reinterpret_cast<const u32x4 *>(&At[32 * wm + (lane & 31)][kofs]);
#pragma unroll
        for (int j = 0; j < 2; ++j)
            acc[j] = mfma_bf16(a, *reinterpret_cast<const u32x4 *>(&Zt[64 * wn + 32 * j + (lane & 31)][kofs]), acc[j]);
    }
    __syncthreads();                 // the operand tiles are read; their space becomes the staging tile
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) T[32 * wm + d_row(lane, v)][64 * wn + 32 * j + (lane & 31)] = acc[j][v];
    __syncthreads();

    const MixArgs &mx = p.mix;
    int m = mx.peer[g];
    if ((unsigned)m >= (unsigned)p.M) m = g;
    const float wi = mx.w[(size_t)g * p.M + m];
    const int cq = (t & 31) * 4, r_in = t >> 5;          // 32 lanes along the 128 columns, 8 rows per pass
#pragma unroll 2
    for (int pass = 0; pass < WM_ROWS / 8; ++pass) {
        const int row = pass * 8 + r_in;
        const int64_t j = p.woff + (r0 + row) * p.dout + n0 + cq;
        const size_t own = tiled_offset_fast(p.M, g, j), other = tiled_offset_fast(p.M, m, j);
        const f32x4_t x = *reinterpret_cast<const f32x4_t *>(mx.Xcur + own);
        const f32x4_t xp = *reinterpret_cast<const f32x4_t *>(mx.Xcur + other);
        const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(mx.V + own));
        const f32x4_t gr = *reinterpret_cast<const f32x4_t *>(&T[row][cq]);
        f32x4_t xn, vn;
        momentum_mix4(x, v, gr, xp, wi, mx.alpha, mx.mu, mx.wd, xn, vn);
        __builtin_nontemporal_store(xn, reinterpret_cast<f32x4_t *>(mx.Xnext + own));
        __builtin_nontemporal_store(vn, reinterpret_cast<f32x4_t *>(mx.V + own));
    }
}

// ---------------------------------------------------------------------------------------------------
// Last layer with few classes (dout <= 32): the same three products with the class dimension padded to
// one 32-wide matrix-instruction tile.  The weight matrix is tiny (din x dout), the work is bound by
// reading / writing the [B][din] activations and errors.

// logits = A W + b.  One workgroup per worker; W^T goes to LDS as bf16 [32][din], each wave takes 32
// batch rows and reads its A operands straight from the bf16 activations.
struct FwdSmallArgs {
    const uint16_t *a_prev; const float *X; int64_t woff; int M, B; int64_t din, dout; float *out;
    SoftmaxArgs sm;                  // what follows the logits in the same workgroup
};
constexpr int SMALL_MAX_DIN = 2048;

__global__ void __launch_bounds__(MF_THREADS) fwd_small_mfma_kernel(FwdSmallArgs p)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t Wt[];      // [32][din + 8]
    const int g = blockIdx.x, t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int din = (int)p.din, dout = (int)p.dout, pitch = din + 8;
    // rows dout .. 31 of Wt are the zero padding of the class dimension
    for (int e = t + dout * pitch / 2; e < 32 * pitch / 2; e += MF_THREADS) reinterpret_cast<uint32_t *>(Wt)[e] = 0u;
    // W[k][n] -> Wt[n][k]: the din x dout block is contiguous in the parameter row and starts at a multiple of four
    // columns, so it is read as float4 (a float4 never straddles a layout tile)
    {
        // eight pieces per thread are requested together (past the end: the first piece again, not stored)
        const unsigned n_w = (unsigned)(din * dout), udout = (unsigned)dout;
        for (unsigned base = 4u * t; base < n_w; base += 8u * 4u * MF_THREADS) {
            f32x4_t w[8];
#pragma unroll
            for (unsigned u = 0; u < 8; ++u) {
                const unsigned e4 = base + u * 4u * MF_THREADS;
                w[u] = *reinterpret_cast<const f32x4_t *>(p.X + tiled_offset(p.M, g, p.woff + (e4 < n_w ? e4 : 0u)));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (unsigned u = 0; u < 8; ++u) {
                const unsigned e4 = base + u * 4u * MF_THREADS;
                if (e4 < n_w) {
#pragma unroll
                    for (unsigned c = 0; c < 4; ++c) {
                        const unsigned e = e4 + c, k = e / udout, n = e - k * udout;
                        Wt[n * pitch + k] = (uint16_t)bf16_bits(w[u][c]);
                    }
                }
            }
        }
    }
    __syncthreads();
    for (int m0 = 32 * wave; m0 < p.B; m0 += 32 * (MF_THREADS / 64)) {
        const uint16_t *a_ptr = p.a_prev + ((size_t)g * p.B + m0 + (lane & 31)) * p.din + 8 * (lane >> 5);
        const uint16_t *b_ptr = Wt + (lane & 31) * pitch + 8 * (lane >> 5);
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
        // din is a multiple of 128: eight steps of loads are issued before their matrix instructions
        for (int k0 = 0; k0 < din; k0 += 128) {
            u32x4 a[8];
#pragma unroll
            for (int s = 0; s < 8; ++s) a[s] = *reinterpret_cast<const u32x4 *>(a_ptr + k0 + 16 * s);
            __builtin_amdgcn_sched_barrier(0);             // or the loads are interleaved with the instructions that wait for them
#pragma unroll
            for (int s = 0; s < 8; ++s) acc = mfma_bf16(a[s], *reinterpret_cast<const u32x4 *>(b_ptr + k0 + 16 * s), acc);
            __builtin_amdgcn_sched_barrier(0);
        }
        const int col = lane & 31;
        if (col < dout) {
            const float bcol = p.X[tiled_offset(p.M, g, p.woff + (int64_t)din * dout + col)];
#pragma unroll
            for (int v = 0; v < 16; ++v) p.out[((size_t)g * p.B + m0 + d_row(lane, v)) * p.dout + col] = acc[v] + bcol;
        }
    }
    // the workgroup holds all logits of its worker: loss, dZ and the last layer's bias gradient follow at once
    __syncthreads();
    softmax_xent_block(p.sm, g);
}

// dW = A^T dZ with dout <= 32: one workgroup = one worker x 128 rows of W, one 32-row tile per wave;
// both operands come straight from the transposed bf16 copies.
struct WgradSmallArgs {
    const uint16_t *a_t, *dz_t; int M, B; int64_t din, dout, woff; float *G;
};

__global__ void __launch_bounds__(MF_THREADS) wgrad_small_mfma_kernel(WgradSmallArgs p)
{
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    int g;
    unsigned strip;
    if (!decode_group(blockIdx.x, (unsigned)(p.din / 128), p.M, g, strip)) return;
    const int64_t r0 = (int64_t)strip * 128 + 32 * wave;
    const uint16_t *a_ptr = p.a_t + ((size_t)g * p.din + r0 + (lane & 31)) * p.B + 8 * (lane >> 5);
    const int n = lane & 31;
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    // the batch is at most 128: all eight steps' operands are requested before the first product (steps past the batch
    // and classes past dout repeat a valid address and are masked)
    const uint16_t *b_ok = p.dz_t + ((size_t)g * p.dout + (n < p.dout ? n : 0)) * p.B + 8 * (lane >> 5);
    const uint32_t keep = n < p.dout ? 0xFFFFFFFFu : 0u;
    u32x4 av[8], bv[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const int b0 = 16 * s < p.B ? 16 * s : 0;
        av[s] = *reinterpret_cast<const u32x4 *>(a_ptr + b0);
        bv[s] = *reinterpret_cast<const u32x4 *>(b_ok + b0);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < 8; ++s)
        if (16 * s < p.B) acc = mfma_bf16(av[s], (u32x4){bv[s][0] & keep, bv[s][1] & keep, bv[s][2] & keep, bv[s][3] & keep}, acc);
    if (n < p.dout) {
#pragma unroll
        for (int v = 0; v < 16; ++v)
            p.G[tiled_offset(p.M, g, p.woff + (r0 + d_row(lane, v)) * p.dout + n)] = acc[v];
    }
}

// dA = (dZ W^T) * [A > 0] with dout <= 32: the contraction is one or two matrix-instruction steps.
// One workgroup = one worker x 128 input features x all batch rows; waves 2 x 2, 64 x 64 each.
struct DgradSmallArgs {
    const uint16_t *dz; const float *X; int64_t woff; int M, B; int64_t din, dout;
    DgradOut o;
};

__global__ void __launch_bounds__(MF_THREADS) dgrad_small_mfma_kernel(DgradSmallArgs p)
{
    __shared__ __attribute__((aligned(16))) uint16_t T[128][ST_PITCH];
    __shared__ float red[4][2][64];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    int g;
    unsigned cblk;
    if (!decode_group(blockIdx.x, (unsigned)(p.din / 128), p.M, g, cblk)) return;
    const int64_t c0 = (int64_t)cblk * 128;
    const int steps = p.dout <= 16 ? 1 : 2;
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    for (int s = 0; s < steps; ++s) {
        const int nbase = 16 * s + 8 * (lane >> 5);
        u32x4 a[2], b[2];
        // All 32 values are requested before any is used: unconditional loads (row / class clamped into the operand,
        // the value masked afterwards; a load under the bounds test, or selected by it, is waited for one by one).
        uint32_t zr[2][8];
        float xr[2][8];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = 64 * wm + 32 * i + (lane & 31);
            const uint16_t *zrow = p.dz + ((size_t)g * p.B + (row < p.B ? row : p.B - 1)) * p.dout;
#pragma unroll
            for (int e = 0; e < 8; ++e) zr[i][e] = zrow[nbase + e < p.dout ? nbase + e : 0];
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t feat = c0 + 64 * wn + 32 * j + (lane & 31);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                xr[j][e] = p.X[tiled_offset(p.M, g, p.woff + feat * p.dout + (nbase + e < p.dout ? nbase + e : 0))];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = 64 * wm + 32 * i + (lane & 31);
            uint32_t h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] = zr[i][e] & ((row < p.B && nbase + e < p.dout) ? 0xFFFFu : 0u);
            a[i] = (u32x4){h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            float w[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) w[e] = __uint_as_float(__float_as_uint(xr[j][e]) & (nbase + e < p.dout ? 0xFFFFFFFFu : 0u));
            b[j] = (u32x4){pack_bf16x2(w[0], w[1]), pack_bf16x2(w[2], w[3]), pack_bf16x2(w[4], w[5]), pack_bf16x2(w[6], w[7])};
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = mfma_bf16(a[i], b[j], acc[i][j]);
    }
    dgrad_tail<8>(p.o, p.M, g, p.B, p.din, c0, wm, wn, lane, t, acc, T, red);
}

// ---------------------------------------------------------------------------------------------------
bool mfma_layer_ok(const MlpPlan &p, int l)
{
    const int64_t din = p.dims[l], dout = p.dims[l + 1];
    return p.bf16 && p.B % 32 == 0 && p.B <= 128 && din % 128 == 0 && dout % 128 == 0 && p.woff[l] % 4 == 0;
}

// the last layer when it has at most 32 outputs (see the "few classes" kernels above)
bool mfma_small_last_ok(const MlpPlan &p)
{
    const int l = p.n_layers - 1;
    const int64_t din = p.dims[l], dout = p.dims[l + 1];
    return p.bf16 && l > 0 && dout <= 32 && p.B % 32 == 0 && p.B <= 128 && din % 128 == 0 && din <= SMALL_MAX_DIN &&
           p.woff[l] % 4 == 0;
}

void prepare_kernels()
{

    // fwd_small_mfma_kernel keeps W^T in more than the default 64 KB of dynamic LDS
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(fwd_small_mfma_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 32 * (SMALL_MAX_DIN + 8) * 2);
}

// Outputs of the backward-data kernel of layer l: the error of layer l - 1 and that layer's bias gradient.
static DgradOut dgrad_out(const MlpPlan &p, int l, int cur, float *G, bool want_f32)
{
    DgradOut o;
    o.act = p.hb[l]; o.out_f32 = want_f32 ? p.dz[cur ^ 1] : nullptr; o.out = p.dzb[cur ^ 1]; o.out_t = p.dzt[cur ^ 1];
    o.G = G; o.boff = p.woff[l - 1] + p.dims[l - 1] * p.dims[l];
    return o;
}

void launch_fwd_small(hipStream_t s, const MlpPlan &p, const float *X, float *G)
{
    const int l = p.n_layers - 1;
    FwdSmallArgs a;
    a.a_prev = p.hb[l]; a.X = X; a.woff = p.woff[l]; a.M = p.M; a.B = p.B; a.din = p.dims[l]; a.dout = p.dims[l + 1];
    a.out = p.act[l + 1];
    a.sm = softmax_args(p, G);
    const size_t lds = (size_t)32 * (a.din + 8) * sizeof(uint16_t);
    hipLaunchKernelGGL(fwd_small_mfma_kernel, dim3(p.M), dim3(MF_THREADS), lds, s, a);
}

void launch_wgrad_small(hipStream_t s, const MlpPlan &p, float *G, int cur)
{
    const int l = p.n_layers - 1;
    WgradSmallArgs a;
    a.a_t = p.ht[l]; a.dz_t = p.dzt[cur]; a.M = p.M; a.B = p.B; a.din = p.dims[l]; a.dout = p.dims[l + 1];
    a.woff = p.woff[l]; a.G = G;
    hipLaunchKernelGGL(wgrad_small_mfma_kernel, dim3(grouped_grid(p.M, (unsigned)(a.din / 128))), dim3(MF_THREADS), 0, s, a);
}

void launch_dgrad_small(hipStream_t s, const MlpPlan &p, const float *X, float *G, int cur, bool want_f32)
{
    const int l = p.n_layers - 1;
    DgradSmallArgs a;
    a.dz = p.dzb[cur]; a.X = X; a.woff = p.woff[l]; a.M = p.M; a.B = p.B; a.din = p.dims[l]; a.dout = p.dims[l + 1];
    a.o = dgrad_out(p, l, cur, G, want_f32);
    hipLaunchKernelGGL(dgrad_small_mfma_kernel, dim3(grouped_grid(p.M, (unsigned)(a.din / 128))), dim3(MF_THREADS), 0, s, a);
}

void launch_fwd_mfma(hipStream_t s, const MlpPlan &p, int l, const float *X)
{
    FwdMfmaArgs a;
    a.feats = (const uint16_t *)p.feats; a.row0 = p.row0; a.idx = p.idx; a.a_prev = l > 0 ? p.hb[l] : nullptr;
    a.X = X; a.woff = p.woff[l]; a.M = p.M; a.B = p.B; a.din = p.dims[l]; a.dout = p.dims[l + 1];
    a.relu = (l + 1 < p.n_layers); a.out = p.hb[l + 1]; a.out_t = p.ht[l + 1];
    const dim3 grid(grouped_grid(p.M, (unsigned)(a.dout / MF_BN)));
    if (l == 0) hipLaunchKernelGGL(fwd_mfma_kernel<true>, grid, dim3(MF_THREADS), 0, s, a);
    else hipLaunchKernelGGL(fwd_mfma_kernel<false>, grid, dim3(MF_THREADS), 0, s, a);
}

void launch_dgrad_mfma(hipStream_t s, const MlpPlan &p, int l, const float *X, float *G, int cur, bool want_f32)
{
    DgradMfmaArgs a;
    a.dz = p.dzb[cur]; a.X = X; a.woff = p.woff[l]; a.M = p.M; a.B = p.B; a.din = p.dims[l]; a.dout = p.dims[l + 1];
    a.o = dgrad_out(p, l, cur, G, want_f32);
    hipLaunchKernelGGL(dgrad_mfma_kernel, dim3(grouped_grid(p.M, (unsigned)(a.din / MF_BN))), dim3(MF_THREADS), 0, s, a);
}

void launch_wgrad_mix_mfma(hipStream_t s, const MlpPlan &p, int l, int cur, const MixArgs &mix)
{
    WgradMixArgs a;
    a.a_t = p.ht[l]; a.dz_t = p.dzt[cur]; a.M = p.M; a.B = p.B; a.din = p.dims[l]; a.dout = p.dims[l + 1];
    a.woff = p.woff[l]; a.mix = mix;
    a.feats = l == 0 ? (const uint16_t *)p.feats : nullptr; a.row0 = p.row0; a.idx = p.idx;
    const unsigned blocks = (unsigned)((a.din / WM_ROWS) * (a.dout / WM_COLS));
    const unsigned grid = (blocks + MF_XCD - 1) / MF_XCD * MF_XCD * (unsigned)p.M;
    hipLaunchKernelGGL(wgrad_mix_mfma_kernel, dim3(grid), dim3(MF_THREADS), 0, s, a);
}

void launch_wgrad_mfma(hipStream_t s, const MlpPlan &p, int l, float *G, int cur)
{
    WgradMfmaArgs a;
    a.a_t = p.ht[l]; a.dz_t = p.dzt[cur]; a.M = p.M; a.B = p.B; a.din = p.dims[l]; a.dout = p.dims[l + 1];
    a.woff = p.woff[l]; a.G = G;
    a.feats = l == 0 ? (const uint16_t *)p.feats : nullptr; a.row0 = p.row0; a.idx = p.idx;
    hipLaunchKernelGGL(wgrad_mfma_kernel, dim3(grouped_grid(p.M, (unsigned)(a.din / WG_STRIP))), dim3(MF_THREADS), 0, s, a);
}

}  // namespace netmax
