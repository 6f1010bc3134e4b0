// Streaming (HBM-bound) kernels of the Jigsaw linear layer: strided block copies
// (shard, gather, 4-way weight-block hand-off) and the separate partial-sum combine
// (the "+" of Eqs. (2) and (4) when it is not fused into the GEMM epilogue).
//
// Every kernel moves each element exactly once (one read per source, one write)
// with 128-bit accesses when shapes and pointers allow it, 32-bit otherwise.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace jg {

constexpr int kMaxBlocks = 4;        // blocks (ranks) per grouped launch
constexpr int COPY_THREADS = 256;
constexpr int COPY_ROWS = 8;         // rows per workgroup

struct CopyBlock {
    const float* src;   // rows x cols, leading dimension lds_
    float* dst;         // rows x cols, leading dimension ldd
    int64_t ld_src, ld_dst;
};

struct CopyGroup {
    CopyBlock b[kMaxBlocks];
    int nblocks;
    int rows, cols;     // common shape
    int vec_ok;         // cols, both leading dimensions multiples of 4 and all pointers 16-B aligned
    int col_chunks;     // ceil(cols / (4 * COPY_THREADS))
};

// grid: x = row chunk * col_chunks + column chunk, y = block
__global__ __launch_bounds__(COPY_THREADS) void copy2d_f32(const CopyGroup g)
{
    const CopyBlock& B = g.b[blockIdx.y];
    const int cchunk = blockIdx.x % g.col_chunks;
    const int row0 = (blockIdx.x / g.col_chunks) * COPY_ROWS;
    const int row1 = min(row0 + COPY_ROWS, g.rows);
    if (g.vec_ok) {
        const int c4 = cchunk * COPY_THREADS + threadIdx.x;
        if (c4 * 4 >= g.cols) return;
        float4 v[COPY_ROWS];
#pragma unroll
        for (int r = 0; r < COPY_ROWS; ++r)
            if (row0 + r < row1)
                v[r] = *reinterpret_cast<const float4*>(B.src + (int64_t)(row0 + r) * B.ld_src + c4 * 4);
#pragma unroll
        for (int r = 0; r < COPY_ROWS; ++r)
            if (row0 + r < row1)
                *reinterpret_cast<float4*>(B.dst + (int64_t)(row0 + r) * B.ld_dst + c4 * 4) = v[r];
    } else {
        // scalar path: the x extent of the grid was sized for 4 columns per thread
        const int c0 = (cchunk * COPY_THREADS + threadIdx.x) * 4;
        for (int r = row0; r < row1; ++r)
            for (int c = c0; c < min(c0 + 4, g.cols); ++c)
                B.dst[(int64_t)r * B.ld_dst + c] = B.src[(int64_t)r * B.ld_src + c];
    }
}

inline hipError_t launch_copy_group(CopyGroup& g, hipStream_t stream)
{
    if (g.rows <= 0 || g.cols <= 0 || g.nblocks <= 0) return hipSuccess;
    int vec = (g.cols & 3) == 0;
    for (int i = 0; i < g.nblocks; ++i) {
        if (((uintptr_t)g.b[i].src & 15) || ((uintptr_t)g.b[i].dst & 15) || (g.b[i].ld_src & 3) ||
            (g.b[i].ld_dst & 3))
            vec = 0;
    }
    g.vec_ok = vec;
    const int per_block_cols = COPY_THREADS * 4;
    g.col_chunks = (g.cols + per_block_cols - 1) / per_block_cols;
    const int64_t nx = (int64_t)g.col_chunks * ((g.rows + COPY_ROWS - 1) / COPY_ROWS);
    if (nx > 0x7fffffff) return hipErrorInvalidValue;
    dim3 grid((unsigned)nx, g.nblocks, 1);
    hipLaunchKernelGGL(copy2d_f32, grid, dim3(COPY_THREADS), 0, stream, g);
    return hipGetLastError();
}

// ---- separate combine: y = kept + received (+ bias), dense n_rows x n_cols each ----
struct CombineBlock {
    const float* kept;
    const float* recv;
    const float* bias;   // length cols or nullptr
    float* y;
};

struct CombineGroup {
    CombineBlock b[kMaxBlocks];
    int nblocks;
    int rows, cols;      // all four arrays dense (leading dimension = cols)
    int vec_ok;
    int col_chunks;
};

__global__ __launch_bounds__(COPY_THREADS) void combine_f32(const CombineGroup g)
{
    const CombineBlock& B = g.b[blockIdx.y];
    const int cchunk = blockIdx.x % g.col_chunks;
    const int row0 = (blockIdx.x / g.col_chunks) * COPY_ROWS;
    const int row1 = min(row0 + COPY_ROWS, g.rows);
    if (g.vec_ok) {
        const int c4 = cchunk * COPY_THREADS + threadIdx.x;
        if (c4 * 4 >= g.cols) return;
        float4 bj = make_float4(0.f, 0.f, 0.f, 0.f);
        if (B.bias) bj = *reinterpret_cast<const float4*>(B.bias + c4 * 4);
        float4 a[COPY_ROWS], b[COPY_ROWS];
#pragma unroll
        for (int r = 0; r < COPY_ROWS; ++r)
            if (row0 + r < row1) {
                const int64_t o = (int64_t)(row0 + r) * g.cols + c4 * 4;
                a[r] = *reinterpret_cast<const float4*>(B.kept + o);
                b[r] = *reinterpret_cast<const float4*>(B.recv + o);
            }
#pragma unroll
        for (int r = 0; r < COPY_ROWS; ++r)
            if (row0 + r < row1) {
                const int64_t o = (int64_t)(row0 + r) * g.cols + c4 * 4;
                float4 y;
                y.x = a[r].x + b[r].x + bj.x;
                y.y = a[r].y + b[r].y + bj.y;
                y.z = a[r].z + b[r].z + bj.z;
                y.w = a[r].w + b[r].w + bj.w;
                *reinterpret_cast<float4*>(B.y + o) = y;
            }
    } else {
        const int c0 = (cchunk * COPY_THREADS + threadIdx.x) * 4;
        for (int r = row0; r < row1; ++r)
            for (int c = c0; c < min(c0 + 4, g.cols); ++c) {
                const int64_t o = (int64_t)r * g.cols + c;
                B.y[o] = B.kept[o] + B.recv[o] + (B.bias ? B.bias[c] : 0.f);
            }
    }
}

inline hipError_t launch_combine_group(CombineGroup& g, hipStream_t stream)
{
    if (g.rows <= 0 || g.cols <= 0 || g.nblocks <= 0) return hipSuccess;
    int vec = (g.cols & 3) == 0;
    for (int i = 0; i < g.nblocks; ++i) {
        if (((uintptr_t)g.b[i].kept & 15) || ((uintptr_t)g.b[i].recv & 15) ||
            ((uintptr_t)g.b[i].y & 15) || (g.b[i].bias && ((uintptr_t)g.b[i].bias & 15)))
            vec = 0;
    }
    g.vec_ok = vec;
    const int per_block_cols = COPY_THREADS * 4;
    g.col_chunks = (g.cols + per_block_cols - 1) / per_block_cols;
    const int64_t nx = (int64_t)g.col_chunks * ((g.rows + COPY_ROWS - 1) / COPY_ROWS);
    if (nx > 0x7fffffff) return hipErrorInvalidValue;
    dim3 grid((unsigned)nx, g.nblocks, 1);
    hipLaunchKernelGGL(combine_f32, grid, dim3(COPY_THREADS), 0, stream, g);
    return hipGetLastError();
}

}  // namespace jg
