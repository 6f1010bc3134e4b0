// Bias gradient of the layer Y = X W^T + 1 b^T (Sec. 4.1: the backward pass multiplies by the
// transposed operands; the bias term's adjoint is the column sum): db[j] = sum_i dY[i][j].
//
// HBM-bound: every element of dY is read once.  A workgroup owns a strip of 32 columns (one 128-byte
// line per row) of one output and a range of the rows of its source blocks: 8 lanes cover a row's 32
// columns with one 16-byte load each, the 32 row lanes take every 32nd row of the range.  Each thread
// accumulates in double (FP32 accumulation over tens of thousands of rows would miss the 1e-6 bar by an
// order of magnitude on same-sign data) and the row lanes' sums are added in a fixed order through LDS.
// A layer's few thousand columns give too few strips for 256 compute units (one workgroup per strip
// reached 3.1 TB/s: a compute unit keeps only so many cache lines in flight), so the rows are cut into
// `parts` ranges when the caller provides a workspace: every workgroup then leaves its 32 sums as doubles
// there and a second small kernel adds a column's parts in ascending order and rounds once.  No atomics:
// the same bits on every run.
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
    int parts;             // row ranges per source block (1: one workgroup per strip writes the result itself)
    int part_rows;         // rows per range
    double* partial;       // parts > 1: nout x parts x cols sums
};

constexpr int COLSUM_THREADS = 256;
constexpr int COLSUM_STRIP = 32;     // columns per workgroup

// grid: x = column strip, y = output, z = row range.  VEC: cols % 4 == 0 and every source 16-byte aligned.
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
    const int r_begin = blockIdx.z * g.part_rows, r_end = min(g.rows, r_begin + g.part_rows);
    double s[W];
#pragma unroll
    for (int q = 0; q < W; ++q) s[q] = 0.0;
    if (col < g.cols) {      // (VEC: cols % 4 == 0, so a thread's four columns are all inside or all outside)
        for (int b = 0; b < O.nsrc; ++b) {
            const float* src = O.src[b] + col;
#pragma unroll 4
            for (int r = r_begin + rl; r < r_end; r += ROW_LANES) {
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
            if (g.parts > 1) {
                g.partial[((int64_t)blockIdx.y * g.parts + blockIdx.z) * g.cols + c] = t;
            } else {
                const float y = (float)t;
                for (int d = 0; d < O.ndst; ++d) O.dst[d][c] = y;
            }
        }
    }
}

// Second stage: column c of output blockIdx.y = its parts in ascending order, rounded once.
__global__ __launch_bounds__(COLSUM_THREADS) void colsum_join_f32(const ColSumGroup g)
{
    const ColSumOut& O = g.o[blockIdx.y];
    const int c = blockIdx.x * COLSUM_THREADS + threadIdx.x;
    if (c >= g.cols) return;
    const double* p = g.partial + (int64_t)blockIdx.y * g.parts * g.cols + c;
    double t = 0.0;
    for (int k = 0; k < g.parts; ++k) t += p[(int64_t)k * g.cols];
    const float y = (float)t;
    for (int d = 0; d < O.ndst; ++d) O.dst[d][c] = y;
}

// Row ranges a column-sum launch is cut into: enough workgroups for about four per compute unit, ranges of at
// least 64 rows, at most kColParts.
constexpr int kColParts = 64;
inline int col_parts(int rows, int cols, int nout, int strip)
{
    const int64_t strips = (int64_t)((cols + strip - 1) / strip) * nout;
    int parts = (int)((1024 + strips - 1) / strips);
    if (parts > rows / 64) parts = rows / 64;
    if (parts > kColParts) parts = kColParts;
    return parts < 1 ? 1 : parts;
}
inline size_t colsum_workspace_bytes(int rows, int cols, int nout)
{
    const int parts = col_parts(rows, cols, nout, COLSUM_STRIP);
    return parts > 1 ? (size_t)nout * parts * cols * sizeof(double) : 0;
}

// workspace (may be null, 8-byte aligned): colsum_workspace_bytes(rows, cols, nout) bytes enable the two-stage form
inline hipError_t launch_colsum_group(ColSumGroup g, hipStream_t stream, void* workspace = nullptr, size_t workspace_bytes = 0)
{
    if (g.nout <= 0 || g.cols <= 0) return hipSuccess;      // (rows == 0: the sums are zero and are written)
    bool vec = (g.cols & 3) == 0;
    for (int i = 0; i < g.nout; ++i)
        for (int b = 0; b < g.o[i].nsrc; ++b)
            if ((uintptr_t)g.o[i].src[b] & 15) vec = false;
    g.parts = col_parts(g.rows, g.cols, g.nout, COLSUM_STRIP);
    if (!workspace || workspace_bytes < colsum_workspace_bytes(g.rows, g.cols, g.nout)) g.parts = 1;
    g.part_rows = g.parts > 1 ? ((g.rows + g.parts - 1) / g.parts + 31) / 32 * 32 : g.rows;
    if (g.parts > 1) g.parts = (g.rows + g.part_rows - 1) / g.part_rows;
    g.partial = static_cast<double*>(workspace);
    dim3 grid((g.cols + COLSUM_STRIP - 1) / COLSUM_STRIP, g.nout, g.parts);
    if (vec) hipLaunchKernelGGL(colsum_f32<true>, grid, dim3(COLSUM_THREADS), 0, stream, g);
    else hipLaunchKernelGGL(colsum_f32<false>, grid, dim3(COLSUM_THREADS), 0, stream, g);
    if (g.parts > 1)
        hipLaunchKernelGGL(colsum_join_f32, dim3((g.cols + COLSUM_THREADS - 1) / COLSUM_THREADS, g.nout, 1),
                           dim3(COLSUM_THREADS), 0, stream, g);
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
