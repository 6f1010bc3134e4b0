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
    uint16_t* dst_rows = nullptr;   // cvt_bf16_transposed only, or nullptr: the untransposed rounding as well (rows of
                          // planes * plane_rows), from the same read of the source
};

struct CvtGroup {
    CvtBlock b[kMaxBlocks];
    int nblocks;
    int rows, cols;       // common shape; cols is a multiple of 8
    int planes;           // 1: hi only; 2: [hi | lo] in every row
    int plane;            // elements from one plane of a row to the next (>= cols; the padding is not written)
    int plane_rows;       // the same for CvtBlock::dst_rows
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

// The same conversion with the block transposed: dst row c holds column c of the source, dst[c][k] = bf16(src[k][c]).
// This is the shard step of the transposed layer Y = X^T W (Sec. 5) in reduced precision: the bfloat16 matrix
// kernel reads both operands along the contracted index, which for X^T W is the row index of X and W as stored, so
// the rounding pass that the mode needs anyway also lays the shard out contraction-major.
// A workgroup moves a 64 x 64 tile through LDS: FP32 reads along the source rows, 128-byte bfloat16 writes along
// the destination rows.  rows (the contracted length) and cols are arbitrary; a destination row is written up to the
// next multiple of 8 elements, with zeros past `rows`, so that the matrix kernel can contract over whole 16-byte
// chunks (a zero times a zero adds nothing).
constexpr int CVT_T_TILE = 64;

// grid: x = tile of source columns, y = tile of source rows, z = block
template <bool VEC>
__global__ __launch_bounds__(256) void cvt_bf16_transposed(const CvtGroup g)
{
    __shared__ float tile[CVT_T_TILE][CVT_T_TILE + 1];
    const CvtBlock& B = g.b[blockIdx.z];
    const int tid = threadIdx.x;
    const int c0 = blockIdx.x * CVT_T_TILE, k0 = blockIdx.y * CVT_T_TILE;
    {
        const int tk = tid >> 4, tc = (tid & 15) * 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int k = k0 + tk + 16 * i, c = c0 + tc;
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            if (k < g.rows) {
                const float* src = B.src + (int64_t)k * B.ld_src + c;
                if (VEC && c + 3 < g.cols) {
                    const vf4 a = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(src));
                    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (c + q < g.cols) v[q] = src[q];
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) tile[tk + 16 * i][tc + q] = v[q];
            if (B.dst_rows && k < g.rows && c < g.cols) {      // the same values, rounded row-major
                uint32_t hi[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) hi[q] = bf16_bits(v[q]);
                uint16_t* d = B.dst_rows + (int64_t)k * g.plane_rows * g.planes + c;
                if (c + 3 < g.cols) {       // (plane_rows and c are multiples of 4: 8-byte aligned)
                    *reinterpret_cast<uint2*>(d) = uint2{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16)};
                    if (g.planes == 2) {
                        uint32_t lo[4];
#pragma unroll
                        for (int q = 0; q < 4; ++q) lo[q] = bf16_bits(v[q] - bf16_value(hi[q]));
                        *reinterpret_cast<uint2*>(d + g.plane_rows) = uint2{lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)};
                    }
                } else {
                    for (int q = 0; q < 4 && c + q < g.cols; ++q) {
                        d[q] = (uint16_t)hi[q];
                        if (g.planes == 2) d[g.plane_rows + q] = (uint16_t)bf16_bits(v[q] - bf16_value(hi[q]));
                    }
                }
            }
        }
    }
    __syncthreads();
    const int c = c0 + (tid >> 2), kk = (tid & 3) * 16;
    if (c >= g.cols) return;
    uint16_t* dst = B.dst + (int64_t)c * g.plane * g.planes + k0 + kk;
#pragma unroll
    for (int h = 0; h < 2; ++h) {       // two chunks of 8 contracted elements (the tile holds zeros past `rows`)
        if (k0 + kk + 8 * h >= g.rows) break;       // nothing of this chunk is inside: absent
        float x[8];
        uint32_t hi[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            x[j] = tile[kk + 8 * h + j][tid >> 2];
            hi[j] = bf16_bits(x[j]);
        }
        *reinterpret_cast<vu4*>(dst + 8 * h) =
            vu4{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16)};
        if (g.planes == 2) {
            uint32_t lo[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) lo[j] = bf16_bits(x[j] - bf16_value(hi[j]));
            *reinterpret_cast<vu4*>(dst + g.plane + 8 * h) =
                vu4{lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16), lo[6] | (lo[7] << 16)};
        }
    }
}

// g.rows x g.cols: the shape of every SOURCE block; g.plane >= rows rounded up to 8 and a multiple of 8; every dst
// 16-byte aligned.  The destination has g.cols rows.
inline hipError_t launch_cvt_transposed_group(const CvtGroup& g, hipStream_t stream)
{
    if (g.rows <= 0 || g.cols <= 0 || g.nblocks <= 0) return hipSuccess;
    if ((g.plane & 7) || g.plane < (g.rows + 7) / 8 * 8) return hipErrorInvalidValue;
    bool vec = true;
    for (int i = 0; i < g.nblocks; ++i) {
        if ((uintptr_t)g.b[i].dst & 15) return hipErrorInvalidValue;
        if (g.b[i].dst_rows && (((uintptr_t)g.b[i].dst_rows & 15) || (g.plane_rows & 7) || g.plane_rows < g.cols))
            return hipErrorInvalidValue;
        if (((uintptr_t)g.b[i].src & 15) || (g.b[i].ld_src & 3)) vec = false;
    }
    const unsigned tk = (unsigned)((g.rows + CVT_T_TILE - 1) / CVT_T_TILE);
    if (tk > 65535u) return hipErrorInvalidConfiguration;
    dim3 grid((unsigned)((g.cols + CVT_T_TILE - 1) / CVT_T_TILE), tk, (unsigned)g.nblocks);
    if (vec) hipLaunchKernelGGL(cvt_bf16_transposed<true>, grid, dim3(256), 0, stream, g);
    else hipLaunchKernelGGL(cvt_bf16_transposed<false>, grid, dim3(256), 0, stream, g);
    return hipGetLastError();
}

}  // namespace jg
