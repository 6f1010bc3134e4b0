// Backward of the activation between the two layers of a mixing MLP (Sec. 3; Sec. 5 "Activation
// functions": point-wise): dA = dH * gelu'(A), gelu'(x) = Phi(x) + x phi(x), the derivative of
// x Phi(x).  HBM-bound (8 bytes read, 4 written per element); the derivative is evaluated in double
// (erf and exp at a fraction of the time the traffic takes) and the product rounded once.
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

__device__ __forceinline__ float gelu_grad_mul(float a, float dh)
{
    const double x = (double)a;
    const double g = 0.5 * (1.0 + erf(x * 0.70710678118654752440)) + x * exp(-0.5 * x * x) * 0.39894228040143267794;
    return (float)((double)dh * g);
}

// grid: x = unit / COPY_THREADS (a unit is 4 elements when vec_ok, else 1), y = block
__global__ __launch_bounds__(COPY_THREADS) void gelu_bwd_f32(const ActBwdGroup g)
{
    const ActBwdBlock& B = g.b[blockIdx.y];
    const int64_t i = (int64_t)blockIdx.x * COPY_THREADS + threadIdx.x;
    if (g.vec_ok) {
        if (i * 4 >= g.n) return;
        const vf4 a = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(B.a) + i);
        const vf4 d = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(B.dh) + i);
        const vf4 o = {gelu_grad_mul(a.x, d.x), gelu_grad_mul(a.y, d.y), gelu_grad_mul(a.z, d.z), gelu_grad_mul(a.w, d.w)};
        reinterpret_cast<vf4*>(B.da)[i] = o;
    } else {
        if (i >= g.n) return;
        B.da[i] = gelu_grad_mul(B.a[i], B.dh[i]);
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
    const int64_t blocks = (units + COPY_THREADS - 1) / COPY_THREADS;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(gelu_bwd_f32, dim3((unsigned)blocks, g.nblocks, 1), dim3(COPY_THREADS), 0, stream, g);
    return hipGetLastError();
}

}  // namespace jg
