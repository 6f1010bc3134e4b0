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
// consecutive dx, contiguous in the field when p is a multiple of 4), or one element otherwise.
// Which piece matters: a patch row is only p elements long in the field (32 bytes for p = 8), and
// the p * p elements of one (patch, channel) are only 4 p * p bytes long in the block, so walking
// either side in its own order leaves the other with quarter-line accesses (measured 2.4 TB/s).
// patch_copy_tiled_f32 therefore gives a wavefront all the rows of a few neighbouring patches of
// one channel: lanes ordered (dy, patch, piece) read whole 128-byte lines of the field (neighbouring
// patches continue each other's rows) and, between them, write whole (patch, channel) runs of the
// block.  It serves p = 4, 8, 16; patch_copy_f32 serves every other case.
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
    // tiled kernel: a wavefront = G patches x p rows x q pieces (q = p / 4, G * p * q = 64)
    int q, G, groups;           // groups = ceil(rows / G) wavefronts per channel of the block
    int channels;               // cols / (p * p)
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

// grid: x = wavefront index / 4 (4 wavefronts per workgroup), y = block
template <bool TO_FIELD>
__global__ __launch_bounds__(COPY_THREADS) void patch_copy_tiled_f32(const PatchGroup g)
{
    const int b = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int64_t wv = (int64_t)blockIdx.x * (COPY_THREADS / 64) + (threadIdx.x >> 6);
    const int cl = (int)(wv / g.groups);              // channel of the block
    if (cl >= g.channels) return;
    const int grp = (int)(wv - (int64_t)cl * g.groups);
    const int ch = lane % g.q;                        // 16-byte piece of the patch row
    const int pl = (lane / g.q) % g.G;                // patch of the group
    const int dy = lane / (g.q * g.G);
    const int row = grp * g.G + pl;                   // row of the block
    if (row >= g.rows) return;
    const int t = g.row0[b] + row;
    const int pp = g.p * g.p;
    const int c = g.col0[b] / pp + cl;
    const int py = t / g.wp, px = t - py * g.wp;
    float* in_field = g.field + ((int64_t)c * g.H + (py * g.p + dy)) * g.W + (px * g.p + ch * 4);
    float* in_block = g.block[b] + (int64_t)row * g.cols + (cl * pp + dy * g.p + ch * 4);
    if (TO_FIELD)
        __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const vf4*>(in_block)),
                                    reinterpret_cast<vf4*>(in_field));
    else
        __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const vf4*>(in_field)),
                                    reinterpret_cast<vf4*>(in_block));
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
    const int pp = g.p * g.p;
    bool tiled = vec && (g.p == 4 || g.p == 8 || g.p == 16) && (g.cols % pp) == 0;
    for (int i = 0; i < g.nblocks; ++i)
        if (g.col0[i] % pp) tiled = false;
    if (tiled) {
        g.q = g.p / 4;
        g.G = 64 / (g.p * g.q);
        g.groups = (g.rows + g.G - 1) / g.G;
        g.channels = g.cols / pp;
        const int64_t waves = (int64_t)g.groups * g.channels;
        const dim3 tgrid((unsigned)((waves + COPY_THREADS / 64 - 1) / (COPY_THREADS / 64)), g.nblocks, 1);
        if (to_field) hipLaunchKernelGGL((patch_copy_tiled_f32<true>), tgrid, dim3(COPY_THREADS), 0, stream, g);
        else hipLaunchKernelGGL((patch_copy_tiled_f32<false>), tgrid, dim3(COPY_THREADS), 0, stream, g);
        return hipGetLastError();
    }
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
