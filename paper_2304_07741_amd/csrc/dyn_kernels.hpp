// Per-pixel ("dynamic") window weights applied to an unfolded tensor and summed over the taps:
//     u[n, c, p] = scale * sum_t a[n, t, p] * x[n, c, p + off(t)]        (zero outside the image)
// i.e. Broadcast-multiply of a [TV]-channel tensor onto Unfold(x) [C, TV] followed by a Fold over the taps
// (Canvas paper, Section 5: Unfold, Broadcast, Fold; the Involution example of the same section), without
// materialising the unfolded tensor.  x, u and their gradients are bf16; a and its gradient fp32.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace canvas {
namespace dyn {

struct Params {
    const uint16_t* x = nullptr;   // [N, C, P] bf16
    const float* a = nullptr;      // [N, TV, P] fp32
    uint16_t* u = nullptr;         // forward output [N, C, P] bf16
    const uint16_t* du = nullptr;  // backward input
    uint16_t* dx = nullptr;        // backward: gradient of x through the unfold (bf16, overwritten)
    float* da = nullptr;           // backward: gradient of a (fp32, overwritten)
    int N = 0, C = 0, H = 0, W = 0, P = 0, upi = 0, KH = 3, KW = 3;
    float scale = 1.f;             // 1 for a sum over the taps, 1 / TV for an average
    uint32_t magicW = 0, magicUpi = 0;
};

bool supported(int KH, int KW);
void forward(const Params& P, hipStream_t s);
// One launch for both gradients of the product (they read the same du and neither fills the chip alone):
//     dx[c](p') = scale * sum_t a[t](p' - off t) * du[c](p' - off t)
//     da[t](p)  = scale * sum_c du[c](p) * x[c](p + off t)
void backward_dx_da(const Params& P, hipStream_t s);

}  // namespace dyn
}  // namespace canvas
