// Sums of weight-gradient partials, several FCs per launch: every workgroup of a weight-gradient kernel writes one
// partial, and the fixed-order sums over the partials of all FCs of a DAG run as ONE launch at the end of
// the backward pass (each alone is a launch of a few microseconds on well under a megabyte).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace canvas {
namespace wreduce {

struct Job {
    const float* partial = nullptr;  // [slices][count] fp32
    float* dw = nullptr;             // [G][Og][R][TV] fp32, overwritten
    int slices = 0;
    int kind = 0;                    // 0: partials in the order of dw; 1: tap-major packed [Gm][Omp][TV][Rp] (gfc_tm_kernels.hpp)
    unsigned count = 0;              // elements per partial
    int segs = 8;                    // 2 or 8 segments of partials per element, combined through LDS in order
    unsigned blocks = 0;             // workgroups of 256 threads = 256 / segs elements each
    int G = 0, R = 0, Og = 0, TV = 1, gm = 1, Omp = 0, Rp = 0;  // kind 1 only
};

constexpr int kMaxJobs = 8;
struct Jobs {
    Job j[kMaxJobs];
    int n = 0;
};

// Fills segs and blocks from slices and count.
void plan(Job& job);

void run(const Jobs& jobs, hipStream_t s);

}  // namespace wreduce
}  // namespace canvas
