// Derived copies of FC weights, several per launch: the tap-major packed layout of gfc_tm_kernels.hpp and the
// transposed, tap-flipped layout that the generic data-gradient contraction reads.  They depend on the weights
// only, so a lowering batches all of them (forward and backward orientation) into one launch per step.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace canvas {
namespace wprep {

struct Job {
    const uint16_t* w = nullptr;  // the FC's weights [G][Og][R][TV] (transposed jobs: [G][R][Og][TV], read swapped)
    uint16_t* out = nullptr;
    int kind = 0;                 // 0: tap-major pack [Gm][Omp][TV][Rp]; 1: plain transpose [G][R][Og][TV] -> [G][Og][R][TV flipped]
    int G = 0, R = 0, Og = 0, TV = 1;
    int gm = 1, Gm = 0, Rp = 0, Omp = 0;  // kind 0 only
    int transposed = 0;           // kind 0 only
    long long total = 0;          // elements written
};

constexpr int kMaxJobs = 8;
struct Jobs {
    Job j[kMaxJobs];
    int n = 0;
};

void run(const Jobs& jobs, hipStream_t s);

}  // namespace wprep
}  // namespace canvas
