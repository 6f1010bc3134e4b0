// Shard step of the reduced-precision modes: a rank's block of an FP32 tensor is written as
// bfloat16 (the upper half of the FP32 bit pattern, rounded to nearest, ties to even), optionally
// followed in every row by the bfloat16 rounding of what the first rounding left over
// (x = hi + lo + a remainder below 2^-17 |x|; the difference x - hi is exact in FP32).
//
// HBM-bound: 4 bytes read and 2 (4 with the lo plane) written per element.  One thread converts
// 8 consecutive elements of a row: two 16-byte loads, one 16-byte store per plane.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "stream_kernels.hpp"

namespace jg {

struct CvtBlock {
    const float* src;     // rows x cols, leading dimension ld_src (floats)
    uint16_t* dst;        // rows of planes * plane bfloat16: [hi(0..cols) pad | lo(0..cols) pad]
    int64_t ld_src;
};

struct CvtGroup {
    CvtBlock b[kMaxBlocks];
    int nblocks;
    int rows, cols;       // common shape; cols is a multiple of 8
    int planes;           // 1: hi only; 2: [hi | lo] in every row
    int plane;            // elements from one plane of a row to the next (>= cols; the padding is not written)
    uint32_t units_per_row, units;   // units of 8 elements
};

__device__ __forceinline__ uint32_t bf16_bits(float x)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    if ((u & 0x7F800000u) == 0x7F800000u)                  // infinity stays, NaN keeps a set fraction bit
        return (u >> 16) | ((u & 0x007FFFFFu) ? 0x40u : 0u);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ float bf16_value(uint32_t bits) { return __builtin_bit_cast(float, bits << 16); }

typedef uint32_t vu4 __attribute__((ext_vector_type(4)));

// grid: x = unit / COPY_THREADS, y = block
template <bool VEC>
__global__ __launch_bounds__(COPY_THREADS) void cvt_bf16(const CvtGroup g)
{
    const CvtBlock& B = g.b[blockIdx.y];
    const uint32_t i = blockIdx.x * (uint32_t)COPY_THREADS + threadIdx.x;
    if (i >= g.units) return;
    const uint32_t row = i / g.units_per_row;
    const uint32_t c = (i - row * g.units_per_row) * 8;
    const float* src = B.src + (int64_t)row * B.ld_src + c;
    float x[8];
    if (VEC) {
        const vf4 a = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(src));
        const vf4 b = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(src) + 1);
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) x[k] = src[k];
    }
    uint32_t hi[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) hi[k] = bf16_bits(x[k]);
    uint16_t* dst = B.dst + (int64_t)row * g.plane * g.planes + c;
    *reinterpret_cast<vu4*>(dst) = vu4{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16)};
    if (g.planes == 2) {
        uint32_t lo[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) lo[k] = bf16_bits(x[k] - bf16_value(hi[k]));
        *reinterpret_cast<vu4*>(dst + g.plane) =
            vu4{lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16), lo[6] | (lo[7] << 16)};
    }
}

// Preconditions: cols % 8 == 0; every dst 16-byte aligned.
inline hipError_t launch_cvt_group(CvtGroup g, hipStream_t stream)
{
    if (g.rows <= 0 || g.cols <= 0 || g.nblocks <= 0) return hipSuccess;
    if ((g.cols & 7) || (g.plane & 7) || g.plane < g.cols) return hipErrorInvalidValue;
    bool vec = true;
    for (int i = 0; i < g.nblocks; ++i) {
        if ((uintptr_t)g.b[i].dst & 15) return hipErrorInvalidValue;
        if (((uintptr_t)g.b[i].src & 15) || (g.b[i].ld_src & 3)) vec = false;
    }
    g.units_per_row = (uint32_t)(g.cols / 8);
    const int64_t max_rows = kMaxUnitsPerLaunch / g.units_per_row;
    const int total_rows = g.rows;
    for (int64_t r0 = 0; r0 < total_rows; r0 += max_rows) {
        CvtGroup part = g;
        part.rows = (int)((total_rows - r0 < max_rows) ? total_rows - r0 : max_rows);
        for (int i = 0; i < g.nblocks; ++i) {
            part.b[i].src = g.b[i].src + r0 * g.b[i].ld_src;
            part.b[i].dst = g.b[i].dst + r0 * g.plane * g.planes;
        }
        part.units = (uint32_t)((int64_t)part.rows * part.units_per_row);
        dim3 grid((part.units + COPY_THREADS - 1) / COPY_THREADS, g.nblocks, 1);
        if (vec) hipLaunchKernelGGL(cvt_bf16<true>, grid, dim3(COPY_THREADS), 0, stream, part);
        else hipLaunchKernelGGL(cvt_bf16<false>, grid, dim3(COPY_THREADS), 0, stream, part);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace jg
