// Bias gradient of the layer Y = X W^T + 1 b^T (Sec. 4.1: the backward pass multiplies by the
// transposed operands; the bias term's adjoint is the column sum): db[j] = sum_i dY[i][j].
//
// HBM-bound: every element of dY is read once.  One workgroup owns a strip of 32 columns (one
// 128-byte line per row) of one output and walks all rows of its source blocks: 8 lanes cover a
// row's 32 columns with one 16-byte load each, the 32 row lanes of the workgroup take every 32nd row.
// Each thread accumulates in double (FP32 accumulation over tens of thousands of rows would miss the
// 1e-6 bar by an order of magnitude on same-sign data), the row lanes' sums are added in a fixed order
// through LDS and rounded once: no atomics, the same bits on every run.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "norm_kernels.hpp"      // wave_sum
#include "stream_kernels.hpp"

namespace jg {

struct ColSumOut {
    const float* src[2];   // source blocks stacked by rows (4-way: the two row halves of a column half); rows x cols, dense
    float* dst[2];         // where the cols sums go (4-way: the bias slice is held by both ranks of the column)
    int nsrc, ndst;
};

struct ColSumGroup {
    ColSumOut o[kMaxBlocks];
    int nout;
    int rows, cols;        // shape of every source block
};

constexpr int COLSUM_THREADS = 256;
constexpr int COLSUM_STRIP = 32;     // columns per workgroup

// grid: x = column strip, y = output.  VEC: cols % 4 == 0 and every source 16-byte aligned.
template <bool VEC>
__global__ __launch_bounds__(COLSUM_THREADS) void colsum_f32(const ColSumGroup g)
{
    constexpr int LANES = VEC ? COLSUM_STRIP / 4 : COLSUM_STRIP;     // threads across a strip
    constexpr int ROW_LANES = COLSUM_THREADS / LANES;                // 32, or 8
    constexpr int W = VEC ? 4 : 1;                                   // columns per thread
    __shared__ double part[ROW_LANES][COLSUM_STRIP + 1];
    const ColSumOut& O = g.o[blockIdx.y];
    const int tid = threadIdx.x;
    const int cl = tid % LANES, rl = tid / LANES;
    const int col = blockIdx.x * COLSUM_STRIP + cl * W;
    double s[W];
#pragma unroll
    for (int q = 0; q < W; ++q) s[q] = 0.0;
    if (col < g.cols) {      // (VEC: cols % 4 == 0, so a thread's four columns are all inside or all outside)
        for (int b = 0; b < O.nsrc; ++b) {
            const float* src = O.src[b] + col;
#pragma unroll 4
            for (int r = rl; r < g.rows; r += ROW_LANES) {
                if (VEC) {
                    const vf4 v = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(src + (int64_t)r * g.cols));
                    s[0] += (double)v.x;
                    s[W > 1 ? 1 : 0] += (double)v.y;
                    s[W > 2 ? 2 : 0] += (double)v.z;
                    s[W > 3 ? 3 : 0] += (double)v.w;
                } else {
                    s[0] += (double)src[(int64_t)r * g.cols];
                }
            }
        }
    }
#pragma unroll
    for (int q = 0; q < W; ++q) part[rl][cl * W + q] = s[q];
    __syncthreads();
    if (tid < COLSUM_STRIP) {
        const int c = blockIdx.x * COLSUM_STRIP + tid;
        if (c < g.cols) {
            double t = 0.0;
#pragma unroll
            for (int r = 0; r < ROW_LANES; ++r) t += part[r][tid];
            const float y = (float)t;
            for (int d = 0; d < O.ndst; ++d) O.dst[d][c] = y;
        }
    }
}

inline hipError_t launch_colsum_group(const ColSumGroup& g, hipStream_t stream)
{
    if (g.nout <= 0 || g.cols <= 0) return hipSuccess;      // (rows == 0: the sums are zero and are written)
    bool vec = (g.cols & 3) == 0;
    for (int i = 0; i < g.nout; ++i)
        for (int b = 0; b < g.o[i].nsrc; ++b)
            if ((uintptr_t)g.o[i].src[b] & 15) vec = false;
    dim3 grid((g.cols + COLSUM_STRIP - 1) / COLSUM_STRIP, g.nout, 1);
    if (vec) hipLaunchKernelGGL(colsum_f32<true>, grid, dim3(COLSUM_THREADS), 0, stream, g);
    else hipLaunchKernelGGL(colsum_f32<false>, grid, dim3(COLSUM_THREADS), 0, stream, g);
    return hipGetLastError();
}

// Row sums: dst[i] = sum over the columns of all source blocks (side by side) of row i.  This is the gradient of a
// bias that goes with the row (the token) instead of the column: the second layer of the token-mixing MLP
// (Sec. 5: the transposed layer and the layer after it) adds b2[t] to every channel of token t.
// One wavefront per row; each lane walks the row in steps of 64 (vectors of four where the layout allows), double
// accumulators, the lanes' sums added in a fixed order, rounded once.
struct RowSumOut {
    const float* src[2];   // source blocks side by side (the two column halves of a row range); rows x cols, dense
    float* dst;            // rows sums
    int nsrc;
};

struct RowSumGroup {
    RowSumOut o[kMaxBlocks];
    int nout;
    int rows, cols;        // shape of every source block
};

constexpr int ROWSUM_THREADS = 256;
constexpr int ROWSUM_ROWS_PER_WG = ROWSUM_THREADS / 64;

// grid: x = group of rows, y = output.  VEC: cols % 4 == 0 and every source 16-byte aligned.
template <bool VEC>
__global__ __launch_bounds__(ROWSUM_THREADS) void rowsum_f32(const RowSumGroup g)
{
    const RowSumOut& O = g.o[blockIdx.y];
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * ROWSUM_ROWS_PER_WG + (threadIdx.x >> 6);
    if (row >= g.rows) return;      // (whole wavefronts leave together; nothing below waits on another wavefront)
    double s = 0.0;
    for (int b = 0; b < O.nsrc; ++b) {
        const float* src = O.src[b] + (int64_t)row * g.cols;
        if (VEC) {
            const vf4* v = reinterpret_cast<const vf4*>(src);
            const int nvec = g.cols >> 2;
#pragma unroll 4
            for (int c = lane; c < nvec; c += 64) {
                const vf4 x = __builtin_nontemporal_load(v + c);
                s += ((double)x.x + (double)x.y) + ((double)x.z + (double)x.w);
            }
        } else {
            for (int c = lane; c < g.cols; c += 64) s += (double)src[c];
        }
    }
    s = wave_sum(s);
    if (lane == 0) O.dst[row] = (float)s;
}

inline hipError_t launch_rowsum_group(const RowSumGroup& g, hipStream_t stream)
{
    if (g.nout <= 0 || g.rows <= 0) return hipSuccess;      // (cols == 0: the sums are zero and are written)
    bool vec = (g.cols & 3) == 0;
    for (int i = 0; i < g.nout; ++i)
        for (int b = 0; b < g.o[i].nsrc; ++b)
            if ((uintptr_t)g.o[i].src[b] & 15) vec = false;
    dim3 grid((g.rows + ROWSUM_ROWS_PER_WG - 1) / ROWSUM_ROWS_PER_WG, g.nout, 1);
    if (vec) hipLaunchKernelGGL(rowsum_f32<true>, grid, dim3(ROWSUM_THREADS), 0, stream, g);
    else hipLaunchKernelGGL(rowsum_f32<false>, grid, dim3(ROWSUM_THREADS), 0, stream, g);
    return hipGetLastError();
}

}  // namespace jg
