// Calls on a compiled plan from inside the library: canvas_dag_forward / canvas_dag_backward with image strides.
#pragma once
#include <cstddef>
#include <cstdint>

#include "../../include/canvas_dag.h"

namespace canvas {

// True when the plan's kernels address x / dx and y / dy through an image stride, so that these tensors may be channel
// slices of wider NCHW tensors (pointer at the slice's first plane, stride of the wide tensor).
bool plan_takes_strided_io(const canvas_dag* dag);

// x_stride, y_stride: elements between consecutive images of x / dx and of y / dy, 0 = dense.  UNSUPPORTED when a stride
// is given to a plan that takes dense tensors only; otherwise as the C-ABI calls.
int plan_forward(canvas_dag* dag, const void* x, const void* const* weights, void* y, void* workspace, size_t workspace_bytes, void* stream,
                 int64_t x_stride, int64_t y_stride);
int plan_backward(canvas_dag* dag, const void* x, const void* const* weights, const void* dy, void* dx, void* const* dweights, void* workspace,
                  size_t workspace_bytes, void* stream, int64_t x_stride, int64_t y_stride);

}  // namespace canvas
