// Kernel launch wrapper.  Normally a plain launch; while a timed call is running (see
// canvas_dag_set_timing) the launch carries a start and a stop event, so that the elapsed time between
// the two is the kernel's own execution time on the device.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

namespace canvas {

struct TimingEvents {
    hipEvent_t start = nullptr, stop = nullptr;
};
extern thread_local TimingEvents g_timing;

}  // namespace canvas

#define CANVAS_LAUNCH(kernel, grid, block, shmem, stream, ...)                                                       \
    do {                                                                                                             \
        if (::canvas::g_timing.start)                                                                                \
            hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, ::canvas::g_timing.start, ::canvas::g_timing.stop, 0, \
                                  __VA_ARGS__);                                                                      \
        else                                                                                                         \
            hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);                                     \
    } while (0)
