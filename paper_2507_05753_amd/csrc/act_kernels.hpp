// Backward of the activation between the two layers of a mixing MLP (Sec. 3; Sec. 5 "Activation
// functions": point-wise): dA = dH * gelu'(A), gelu'(x) = Phi(x) + x phi(x), the derivative of
// x Phi(x).  HBM-bound (8 bytes read, 4 written per element); the derivative is evaluated in double
// (exp from the library, erf from a table of Taylor polynomials: see below) and the product rounded once.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "stream_kernels.hpp"

namespace jg {

struct ActBwdBlock {
    const float* a;      // pre-activation, n elements
    const float* dh;     // gradient of the activation's output
    float* da;           // gradient of the pre-activation; may be dh
};

struct ActBwdGroup {
    ActBwdBlock b[kMaxBlocks];
    int nblocks;
    int64_t n;           // elements per block
    int vec_ok;
};

// erf on [0, 4.125) from a table in LDS: 22 intervals of 3/16, in each the Taylor polynomial of degree 12 about the
// midpoint m:  erf^(n+1)(m) = (2 / sqrt(pi)) (-1)^n H_n(m) exp(-m^2)  with the Hermite recurrence H_(n+1) = 2 m H_n -
// 2 n H_(n-1).  The remainder is below 2e-17, the whole within 4e-16 of the library's erf (checked on the host over
// the range and on every float around the root of the derivative, where the sum below cancels).  The library's erf
// in double was the whole cost of this kernel (0.22 ms of arithmetic over 0.13 ms of traffic at 16200 x 4320; its
// exp is hidden under the traffic): thirteen LDS reads and twelve multiply-adds replace it.
constexpr int kErfIntervals = 22;
constexpr int kErfTerms = 13;
constexpr double kErfWidth = 0.1875;

// row i of the table: the thirteen coefficients of interval i (one thread per row, at the start of a workgroup)
__device__ inline void erf_table_row(int i, double* row)
{
    const double m = ((double)i + 0.5) * kErfWidth;
    const double e = exp(-m * m) * 1.12837916709551257390;      // 2 / sqrt(pi)
    row[0] = erf(m);
    double h_prev = 0.0, h = 1.0, factorial = 1.0, sign = 1.0;
    for (int n = 0; n < kErfTerms - 1; ++n) {
        factorial *= (double)(n + 1);
        row[n + 1] = sign * h * e / factorial;
        const double h_next = 2.0 * m * h - 2.0 * (double)n * h_prev;
        h_prev = h;
        h = h_next;
        sign = -sign;
    }
}

__device__ __forceinline__ float gelu_grad_mul(float a, float dh, const double* table)
{
    const double x = (double)a;
    const double z = fabs(x) * 0.70710678118654752440;
    double t;
    if (z < kErfIntervals * kErfWidth) {
        const int i = min((int)(z * (1.0 / kErfWidth)), kErfIntervals - 1);
        const double h = z - ((double)i + 0.5) * kErfWidth;
        const double* c = table + i * kErfTerms;
        t = c[kErfTerms - 1];
#pragma unroll
        for (int k = kErfTerms - 2; k >= 0; --k) t = fma(t, h, c[k]);
    } else {
        t = erf(z);         // the far tails, infinities and NaN: the library's, as rare as they are
    }
    const double g = 0.5 * (1.0 + copysign(t, x)) + x * exp(-0.5 * x * x) * 0.39894228040143267794;
    return (float)((double)dh * g);
}

// grid: x = workgroups that stride over the units (a unit is 4 elements when vec_ok, else 1), y = block
__global__ __launch_bounds__(COPY_THREADS) void gelu_bwd_f32(const ActBwdGroup g)
{
    __shared__ double table[kErfIntervals * kErfTerms];
    if (threadIdx.x < kErfIntervals) erf_table_row(threadIdx.x, table + threadIdx.x * kErfTerms);
    __syncthreads();
    const ActBwdBlock& B = g.b[blockIdx.y];
    const int64_t stride = (int64_t)gridDim.x * COPY_THREADS;
    if (g.vec_ok) {
        const int64_t units = g.n >> 2;
        // two units per turn: the second one's loads are in flight while the first is worked on
        for (int64_t i = (int64_t)blockIdx.x * COPY_THREADS + threadIdx.x; i < units; i += 2 * stride) {
            const int64_t j = i + stride;
            const bool two = j < units;
            const vf4 a0 = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(B.a) + i);
            const vf4 d0 = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(B.dh) + i);
            vf4 a1 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
            if (two) {
                a1 = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(B.a) + j);
                d1 = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(B.dh) + j);
            }
            const vf4 o0 = {gelu_grad_mul(a0.x, d0.x, table), gelu_grad_mul(a0.y, d0.y, table),
                            gelu_grad_mul(a0.z, d0.z, table), gelu_grad_mul(a0.w, d0.w, table)};
            reinterpret_cast<vf4*>(B.da)[i] = o0;
            if (two) {
                const vf4 o1 = {gelu_grad_mul(a1.x, d1.x, table), gelu_grad_mul(a1.y, d1.y, table),
                                gelu_grad_mul(a1.z, d1.z, table), gelu_grad_mul(a1.w, d1.w, table)};
                reinterpret_cast<vf4*>(B.da)[j] = o1;
            }
        }
    } else {
        for (int64_t i = (int64_t)blockIdx.x * COPY_THREADS + threadIdx.x; i < g.n; i += stride)
            B.da[i] = gelu_grad_mul(B.a[i], B.dh[i], table);
    }
}

inline hipError_t launch_act_bwd_group(ActBwdGroup g, hipStream_t stream)
{
    if (g.n <= 0 || g.nblocks <= 0) return hipSuccess;
    int vec = (g.n & 3) == 0;
    for (int i = 0; i < g.nblocks; ++i)
        if (((uintptr_t)g.b[i].a | (uintptr_t)g.b[i].dh | (uintptr_t)g.b[i].da) & 15) vec = 0;
    g.vec_ok = vec;
    const int64_t units = vec ? g.n / 4 : g.n;
    // a workgroup builds the table once and then walks its share of the block: about 1024 workgroups in all (four
    // per compute unit, all resident at once, so that they finish together)
    int64_t blocks = (units + COPY_THREADS - 1) / COPY_THREADS;
    const int64_t cap = (1024 + g.nblocks - 1) / g.nblocks;
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(gelu_bwd_f32, dim3((unsigned)blocks, g.nblocks, 1), dim3(COPY_THREADS), 0, stream, g);
    return hipGetLastError();
}

}  // namespace jg
