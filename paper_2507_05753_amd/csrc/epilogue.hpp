// What is applied to a finished output element before it is stored:
//     y = act(sum + bias) + residual
// The activation between the two linear layers of a mixing MLP is GELU (Sec. 3; Sec. 5
// "Activation functions": point-wise, so it needs no exchange and rides in the epilogue of
// the product that completes an output block).  The paper gives no formula; this is the
// defining form x * Phi(x), not the tanh approximation.
#pragma once

#include <hip/hip_runtime.h>

namespace jg {

enum { kActNone = 0, kActGelu = 1 };

__device__ __forceinline__ float gelu_f32(float x)
{
    return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f));
}

__device__ __forceinline__ float activate(float x, int act) { return act == kActGelu ? gelu_f32(x) : x; }

}  // namespace jg
