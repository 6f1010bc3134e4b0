// Patch rearrangement of the encoder and decoder (Sec. 5 "Encoding and decoding layers": a
// convolution whose kernel equals its stride is computed by reshaping the input into
// non-overlapping patches and applying a linear layer).  The patch matrix of a [C, H, W] field
// has one row per patch, t = py * (W / p) + px, and one column per (channel, offset in the patch),
// f = c * p * p + dy * p + dx, holding field[c, py * p + dy, px * p + dx].  These kernels move
// between the field and the per-rank blocks of that matrix directly, so the matrix itself is
// never stored whole: each rank's block is read from (written to) its part of the field, the way
// Sec. 5 "Data loading" lets every rank read its own partition.
//
// HBM-bound, each element moved once.  One thread moves one 16-byte piece of a patch row (four
// consecutive dx, contiguous in the field when p is a multiple of 4), or one element otherwise;
// consecutive threads walk a row of the block, so the block side is accessed in 1 KiB runs and the
// field side in runs of p elements.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "stream_kernels.hpp"

namespace jg {

struct PatchGroup {
    float* block[kMaxBlocks];   // dense rows x cols blocks of the patch matrix (one per rank)
    int row0[kMaxBlocks];       // first patch (row of the matrix) of each block
    int col0[kMaxBlocks];       // first feature (column) of each block
    int nblocks;
    int rows, cols;
    float* field;               // C x H x W, dense
    int H, W, p, wp;            // wp = W / p patches per field row
    uint32_t units_per_row, units;
};

// grid: x = unit / COPY_THREADS, y = block.  TO_FIELD: block -> field (decoder), else field -> block.
template <bool TO_FIELD, bool VEC>
__global__ __launch_bounds__(COPY_THREADS) void patch_copy_f32(const PatchGroup g)
{
    const uint32_t i = blockIdx.x * (uint32_t)COPY_THREADS + threadIdx.x;
    if (i >= g.units) return;
    const int b = blockIdx.y;
    const uint32_t row = i / g.units_per_row;
    const uint32_t u = i - row * g.units_per_row;
    const int f = g.col0[b] + (int)u * (VEC ? 4 : 1);
    const int t = g.row0[b] + (int)row;
    const int pp = g.p * g.p;
    const int c = f / pp, rem = f - c * pp;
    const int dy = rem / g.p, dx = rem - dy * g.p;
    const int py = t / g.wp, px = t - py * g.wp;
    float* in_field = g.field + ((int64_t)c * g.H + (py * g.p + dy)) * g.W + (px * g.p + dx);
    float* in_block = g.block[b] + (int64_t)row * g.cols + (int64_t)u * (VEC ? 4 : 1);
    if (VEC) {
        if (TO_FIELD)
            __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const vf4*>(in_block)),
                                        reinterpret_cast<vf4*>(in_field));
        else
            __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const vf4*>(in_field)),
                                        reinterpret_cast<vf4*>(in_block));
    } else {
        if (TO_FIELD) *in_field = *in_block;
        else *in_block = *in_field;
    }
}

// Preconditions (checked by the C-ABI layer): p >= 1 divides H and W; every block lies inside the
// (H / p) * (W / p) x (C * p * p) matrix; rows * cols < 2^31.
inline hipError_t launch_patch_group(PatchGroup g, bool to_field, hipStream_t stream)
{
    if (g.rows <= 0 || g.cols <= 0 || g.nblocks <= 0) return hipSuccess;
    bool vec = (g.p % 4) == 0 && (g.cols % 4) == 0 && (g.W % 4) == 0 && ((uintptr_t)g.field & 15) == 0;
    for (int i = 0; i < g.nblocks; ++i)
        if (((uintptr_t)g.block[i] & 15) || (g.col0[i] & 3)) vec = false;
    g.units_per_row = (uint32_t)(vec ? g.cols / 4 : g.cols);
    const int64_t units = (int64_t)g.rows * g.units_per_row;
    if (units >= kMaxUnitsPerLaunch) return hipErrorInvalidValue;
    g.units = (uint32_t)units;
    const dim3 grid((g.units + COPY_THREADS - 1) / COPY_THREADS, g.nblocks, 1);
    if (to_field) {
        if (vec) hipLaunchKernelGGL((patch_copy_f32<true, true>), grid, dim3(COPY_THREADS), 0, stream, g);
        else hipLaunchKernelGGL((patch_copy_f32<true, false>), grid, dim3(COPY_THREADS), 0, stream, g);
    } else {
        if (vec) hipLaunchKernelGGL((patch_copy_f32<false, true>), grid, dim3(COPY_THREADS), 0, stream, g);
        else hipLaunchKernelGGL((patch_copy_f32<false, false>), grid, dim3(COPY_THREADS), 0, stream, g);
    }
    return hipGetLastError();
}

}  // namespace jg
