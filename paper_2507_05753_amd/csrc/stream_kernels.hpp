// Streaming (HBM-bound) kernels of the Jigsaw linear layer: strided block copies
// (shard, gather, 4-way weight-block hand-off) and the separate partial-sum combine
// (the "+" of Eqs. (2) and (4) when it is not fused into the GEMM epilogue).
//
// Every kernel moves each element exactly once (one read per source, one write).
// One thread moves one 16-byte vector (or one float when shapes or pointers rule out
// 128-bit accesses); consecutive threads walk consecutive vectors of a row, so a
// wavefront reads and writes 1 KiB runs.  Large single-use tensors (activations,
// outputs, partial products) move with non-temporal loads and stores so that they do
// not displace what the GEMM re-reads; small tensors the GEMM is about to read
// (weight blocks, bias) use ordinary cached accesses.
#pragma once

#include <hip/hip_runtime.h>

#include "epilogue.hpp"
#include <stdint.h>

namespace jg {

constexpr int kMaxBlocks = 4;        // blocks (ranks) per grouped launch
constexpr int COPY_THREADS = 256;
constexpr int64_t kMaxUnitsPerLaunch = (int64_t)1 << 31;   // 32-bit unit index inside a launch

typedef float vf4 __attribute__((ext_vector_type(4)));

struct CopyBlock {
    const float* src;   // rows x cols, leading dimension ld_src
    float* dst;         // rows x cols, leading dimension ld_dst
    int64_t ld_src, ld_dst;
};

struct CopyGroup {
    CopyBlock b[kMaxBlocks];
    int nblocks;
    int rows, cols;     // common shape
    int vec_ok;         // cols, both leading dimensions multiples of 4 and all pointers 16-B aligned
    int nontemporal;    // 1: single-use data, bypass-style accesses; 0: cached accesses
    uint32_t units_per_row;   // cols / 4 (vector path) or cols (scalar path)
    uint32_t units;           // rows * units_per_row
};

// grid: x = unit index / COPY_THREADS, y = block
template <bool VEC, bool NT>
__global__ __launch_bounds__(COPY_THREADS) void copy2d_f32(const CopyGroup g)
{
    const CopyBlock& B = g.b[blockIdx.y];
    const uint32_t i = blockIdx.x * (uint32_t)COPY_THREADS + threadIdx.x;
    if (i >= g.units) return;
    const uint32_t row = i / g.units_per_row;
    const uint32_t c = i - row * g.units_per_row;
    if (VEC) {
        const vf4* src = reinterpret_cast<const vf4*>(B.src + (int64_t)row * B.ld_src) + c;
        vf4* dst = reinterpret_cast<vf4*>(B.dst + (int64_t)row * B.ld_dst) + c;
        if (NT) __builtin_nontemporal_store(__builtin_nontemporal_load(src), dst);
        else *dst = *src;
    } else {
        B.dst[(int64_t)row * B.ld_dst + c] = B.src[(int64_t)row * B.ld_src + c];
    }
}

inline hipError_t launch_copy_group(CopyGroup g, hipStream_t stream)
{
    if (g.rows <= 0 || g.cols <= 0 || g.nblocks <= 0) return hipSuccess;
    int vec = (g.cols & 3) == 0;
    for (int i = 0; i < g.nblocks; ++i) {
        if (((uintptr_t)g.b[i].src & 15) || ((uintptr_t)g.b[i].dst & 15) || (g.b[i].ld_src & 3) ||
            (g.b[i].ld_dst & 3))
            vec = 0;
    }
    g.vec_ok = vec;
    g.units_per_row = (uint32_t)(vec ? g.cols / 4 : g.cols);
    // a launch indexes its units with 32 bits: very tall blocks go in several row ranges
    const int64_t max_rows = kMaxUnitsPerLaunch / g.units_per_row;
    const int total_rows = g.rows;
    for (int64_t r0 = 0; r0 < total_rows; r0 += max_rows) {
        CopyGroup part = g;
        part.rows = (int)((total_rows - r0 < max_rows) ? total_rows - r0 : max_rows);
        for (int i = 0; i < g.nblocks; ++i) {
            part.b[i].src = g.b[i].src + r0 * g.b[i].ld_src;
            part.b[i].dst = g.b[i].dst + r0 * g.b[i].ld_dst;
        }
        part.units = (uint32_t)((int64_t)part.rows * part.units_per_row);
        dim3 grid((part.units + COPY_THREADS - 1) / COPY_THREADS, g.nblocks, 1);
        if (vec && g.nontemporal)
            hipLaunchKernelGGL((copy2d_f32<true, true>), grid, dim3(COPY_THREADS), 0, stream, part);
        else if (vec)
            hipLaunchKernelGGL((copy2d_f32<true, false>), grid, dim3(COPY_THREADS), 0, stream, part);
        else
            hipLaunchKernelGGL((copy2d_f32<false, false>), grid, dim3(COPY_THREADS), 0, stream, part);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---- separate combine: y = act(kept + received (+ bias)) (+ residual), dense rows x cols each ----
struct CombineBlock {
    const float* kept;
    const float* recv;
    const float* bias;   // length cols or nullptr
    float* y;
    const float* residual;   // dense like y, or nullptr
};

struct CombineGroup {
    CombineBlock b[kMaxBlocks];
    int nblocks;
    int rows, cols;      // all arrays dense (leading dimension = cols)
    int vec_ok;
    uint32_t units_per_row;
    uint32_t units;
    int act;             // kActNone / kActGelu
};

__global__ __launch_bounds__(COPY_THREADS) void combine_f32(const CombineGroup g)
{
    const CombineBlock& B = g.b[blockIdx.y];
    const uint32_t i = blockIdx.x * (uint32_t)COPY_THREADS + threadIdx.x;
    if (i >= g.units) return;
    const uint32_t c = i % g.units_per_row;
    if (g.vec_ok) {
        const vf4 a = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(B.kept) + i);
        const vf4 r = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(B.recv) + i);
        vf4 y = a + r;   // same order as the fused epilogue: (kept + received) + bias
        if (B.bias) y += reinterpret_cast<const vf4*>(B.bias)[c];
        if (g.act) y = vf4{activate(y.x, g.act), activate(y.y, g.act), activate(y.z, g.act), activate(y.w, g.act)};
        if (B.residual) y += __builtin_nontemporal_load(reinterpret_cast<const vf4*>(B.residual) + i);
        __builtin_nontemporal_store(y, reinterpret_cast<vf4*>(B.y) + i);
    } else {
        float y = B.kept[i] + B.recv[i];
        if (B.bias) y += B.bias[c];
        y = activate(y, g.act);
        if (B.residual) y += B.residual[i];
        B.y[i] = y;
    }
}

inline hipError_t launch_combine_group(CombineGroup g, hipStream_t stream)
{
    if (g.rows <= 0 || g.cols <= 0 || g.nblocks <= 0) return hipSuccess;
    int vec = (g.cols & 3) == 0;
    for (int i = 0; i < g.nblocks; ++i) {
        if (((uintptr_t)g.b[i].kept & 15) || ((uintptr_t)g.b[i].recv & 15) ||
            ((uintptr_t)g.b[i].y & 15) || (g.b[i].bias && ((uintptr_t)g.b[i].bias & 15)) ||
            (g.b[i].residual && ((uintptr_t)g.b[i].residual & 15)))
            vec = 0;
    }
    g.vec_ok = vec;
    g.units_per_row = (uint32_t)(vec ? g.cols / 4 : g.cols);
    const int unit_floats = vec ? 4 : 1;
    const int64_t max_rows = kMaxUnitsPerLaunch / g.units_per_row;
    const int total_rows = g.rows;
    for (int64_t r0 = 0; r0 < total_rows; r0 += max_rows) {
        CombineGroup part = g;
        part.rows = (int)((total_rows - r0 < max_rows) ? total_rows - r0 : max_rows);
        const int64_t off = r0 * g.units_per_row * unit_floats;
        for (int i = 0; i < g.nblocks; ++i) {
            part.b[i].kept = g.b[i].kept + off;
            part.b[i].recv = g.b[i].recv + off;
            part.b[i].y = g.b[i].y + off;
            if (g.b[i].residual) part.b[i].residual = g.b[i].residual + off;
        }
        part.units = (uint32_t)((int64_t)part.rows * part.units_per_row);
        dim3 grid((part.units + COPY_THREADS - 1) / COPY_THREADS, g.nblocks, 1);
        hipLaunchKernelGGL(combine_f32, grid, dim3(COPY_THREADS), 0, stream, part);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace jg
