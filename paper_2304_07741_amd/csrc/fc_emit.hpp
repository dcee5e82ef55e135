// Launch lists of one FC-shaped contraction on the MFMA kernels, shared by the fused lowerings: picks the
// tap-major kernels (with their packed weights) where they apply, else the generic kernels.
#pragma once
#include <functional>
#include <string>
#include <vector>

#include "lowering.hpp"

namespace canvas {

// Workspace carving: returns the byte offset of a new 256-byte aligned block.
using TakeFn = std::function<int64_t(uint64_t)>;
using PtrFn = std::function<const void*(const RunArgs&)>;

struct FcOperand {
    PtrFn ptr;
    bool f32 = false;  // fp32 tensor (else bf16)
};

// y = FC(src) (forward), or, with `transposed`, the data gradient src = dy -> dst = d(source of the FC):
// then (R, Og) are the swapped dims and the FC's own weights [G][R][Og][taps] are read transposed with the
// taps flipped.  `addend_is_dst`: dst (bf16) already holds a tensor that the result is added to.
// dst is bf16 unless dst_f32.  softmax (see fc_softmax_fusable): dst receives the softmax over the outputs of each pixel.
// The launch goes to low.fwd or (backward) low.bwd; derived weight copies are registered in low.wjobs.
void emit_fc(Lowering& low, bool backward, const Dag& dag, const TakeFn& take, const std::string& name, int G, int R, int kh, int kw, int Og,
             bool transposed, int widx, FcOperand src, PtrFn dst, bool addend_is_dst, double bytes, double flops, bool dst_f32 = false,
             bool softmax = false);
// Whether emit_fc can be asked (softmax = true, dst_f32) for the softmax over the FC's outputs instead of the outputs.
bool fc_softmax_fusable(const Dag& dag, int G, int R, int kh, int kw, int Og, const FcOperand& src);

// dw[widx] = sum over (image, pixel) of dy (x) rows of src (through the window kh x kw): the kernel that writes
// one partial per workgroup goes to low.bwd, the fixed-order sum of the partials is registered in low.rjobs.
void emit_wgrad(Lowering& low, const Dag& dag, const TakeFn& take, const std::string& name, int G, int R, int kh, int kw, int Og,
                int widx, FcOperand src, FcOperand dy, double operand_bytes, double flops);

}  // namespace canvas
