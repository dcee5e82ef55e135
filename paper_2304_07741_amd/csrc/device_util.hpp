// Small device helpers shared by the kernels: bf16 conversion and the element-wise primitives.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace canvas {

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// Round to nearest even; NaN stays NaN.
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Element-wise primitives (Section 5): relu, abs, gelu (erf form), exp of the clamped input, sin.
__device__ __forceinline__ float unary_apply(int kind, float x, float lo, float hi) {
    switch (kind) {
    case 0: return __builtin_fmaxf(x, 0.f);
    case 1: return fabsf(x);
    case 2: return 0.5f * x * (1.f + erff(x * 0.70710678118654752f));
    case 4: return sinf(x);
    default: return expf(fminf(fmaxf(x, lo), hi));
    }
}

// Derivatives: relu'(0) = 0, sign(0) = 0, clamped exp has zero slope outside the open interval (lo, hi).
__device__ __forceinline__ float unary_grad(int kind, float x, float lo, float hi) {
    switch (kind) {
    case 0: return x > 0.f ? 1.f : 0.f;
    case 1: return x > 0.f ? 1.f : (x < 0.f ? -1.f : 0.f);
    case 2: return 0.5f * (1.f + erff(x * 0.70710678118654752f)) + x * 0.39894228040143268f * expf(-0.5f * x * x);
    case 4: return cosf(x);
    default: return (x > lo && x < hi) ? expf(x) : 0.f;
    }
}

// Blends (Section 5, Broadcast): a from the replicated LHS, b from the RHS.  kind: add, mul, sub, min, max.
__device__ __forceinline__ float binary_apply(int kind, float a, float b) {
    switch (kind) {
    case 0: return a + b;
    case 1: return a * b;
    case 2: return a - b;
    case 3: return a <= b ? a : b;
    default: return a >= b ? a : b;
    }
}
// d out / d a and d out / d b; a tie of min / max belongs to the LHS
__device__ __forceinline__ float binary_grad_lhs(int kind, float a, float b) {
    switch (kind) {
    case 0: return 1.f;
    case 1: return b;
    case 2: return 1.f;
    case 3: return a <= b ? 1.f : 0.f;
    default: return a >= b ? 1.f : 0.f;
    }
}
__device__ __forceinline__ float binary_grad_rhs(int kind, float a, float b) {
    switch (kind) {
    case 0: return 1.f;
    case 1: return a;
    case 2: return -1.f;
    case 3: return a <= b ? 0.f : 1.f;
    default: return a >= b ? 0.f : 1.f;
    }
}

}  // namespace canvas
