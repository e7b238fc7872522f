// The nonlinearity between the two linear layers of a feed-forward block, for the kernels that apply
// it in their epilogues.  The paper keeps the blocks of ViT / MLP-Mixer / BERT / GPT-2 as they are
// around the Monarch layers (Section 4) and does not write the nonlinearity down; those models use
// GELU, and this is the tanh form (GPT-2's):
//
//     gelu(v) = v/2 * (1 + tanh(u)) = v * s,   s = 1 / (1 + exp(-2u)),   u = sqrt(2/pi) * (v + 0.044715 v^3)
//     gelu'(v) = s + v * s * (1 - s) * d(2u)/dv
//
// fp32 throughout.  exp(-2u) is one v_exp_f32 (base 2, log2(e) folded into the polynomial).  The
// polynomial is evaluated at v clamped to [-16, 16]: beyond that s is exactly 0 or 1 in fp32, and the
// clamp keeps v^2 finite for any finite input.
#pragma once
#include <hip/hip_runtime.h>

namespace monarch {

// s(v) = 1/2 (1 + tanh u(v))
__device__ __forceinline__ float gelu_gate(float v)
{
    const float vc = __builtin_fminf(__builtin_fmaxf(v, -16.f), 16.f);
    // -2u * log2(e) = vc * (a + b vc^2):  a = -2 sqrt(2/pi) log2(e),  b = a * 0.044715
    const float w = vc * (-2.3022082f + -0.10294324f * (vc * vc));
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(w));
}

__device__ __forceinline__ float gelu_f(float v) { return v * gelu_gate(v); }

__device__ __forceinline__ float gelu_grad_f(float v)
{
    const float vc = __builtin_fminf(__builtin_fmaxf(v, -16.f), 16.f);
    const float s = gelu_gate(v);
    // d(2u)/dv = 2 sqrt(2/pi) (1 + 3 * 0.044715 v^2)
    return s + vc * (s * (1.0f - s)) * (1.5957692f + 0.21406445f * (vc * vc));
}

}  // namespace monarch
