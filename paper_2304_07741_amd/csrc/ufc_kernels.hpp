// Element-wise middle of the pattern  x -> Unfold -> FC -> unary -> Shift -> (binary with x) -> FC:
//     v = x (*|+) shift(act(z))      and its adjoint.  bf16 tensors [N, C, H*W].
// Canvas paper, Section 5: element-wise, Shift and Broadcast primitives.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace canvas {
namespace ufc {

constexpr int kMaxSlices = 8;

struct MidParams {
    const uint16_t* x = nullptr;   // block input
    const uint16_t* z = nullptr;   // output of the first FC (pre-activation)
    const uint16_t* dv = nullptr;  // backward: gradient of v
    uint16_t* v = nullptr;         // forward output
    uint16_t* dz = nullptr;        // backward outputs: gradient of z ...
    uint16_t* dx1 = nullptr;       // ... and the part of dx that flows through the binary node
    int N = 0, C = 0, H = 0, W = 0, P = 0, upi = 0;
    uint32_t magicW = 0, magicUpi = 0;
    int act = -1;                  // -1 none, else UnaryKind
    float ulo = 0.f, uhi = 0.f;
    int bin = 1;                   // 0 add, 1 mul
    int nslices = 0;               // channel slices [c0, c1) shifted by (dh, dw); other channels are not shifted
    int c0[kMaxSlices] = {0}, c1[kMaxSlices] = {0}, dh[kMaxSlices] = {0}, dw[kMaxSlices] = {0};
};

void mid_forward(const MidParams& P, hipStream_t s);
void mid_backward(const MidParams& P, hipStream_t s);

}  // namespace ufc
}  // namespace canvas
