#include "wprep_kernels.hpp"

#include <algorithm>

#include "launch.hpp"

namespace canvas {
namespace wprep {

namespace {

// blockIdx.y selects the job, blockIdx.x * 256 + threadIdx.x the element it writes
__global__ __launch_bounds__(256) void k_weight_prep(Jobs jobs) {
    const Job& J = jobs.j[blockIdx.y];
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= J.total) return;
    if (J.kind == 0) {
        // wp[gmi][op][tap][rp]: block-diagonal over the gm merged groups, zero in the padding
        const int rp = (int)(i % J.Rp);
        long long t = i / J.Rp;
        const int tap = (int)(t % J.TV);
        t /= J.TV;
        const int op = (int)(t % J.Omp), gmi = (int)(t / J.Omp);
        const int sub = op / J.Og, o = op - sub * J.Og;
        const int subr = rp / J.R, row = rp - subr * J.R;
        const int g = gmi * J.gm + sub;
        uint16_t v = 0;
        if (sub < J.gm && subr == sub && g < J.G)
            v = J.transposed ? J.w[(((long long)g * J.R + row) * J.Og + o) * J.TV + (J.TV - 1 - tap)]
                             : J.w[(((long long)g * J.Og + o) * J.R + row) * J.TV + tap];
        J.out[i] = v;
    } else {
        const int tv = (int)(i % J.TV);
        long long q = i / J.TV;
        const int o = (int)(q % J.Og);
        q /= J.Og;
        const int row = (int)(q % J.R), g = (int)(q / J.R);
        J.out[i] = J.w[((long long)(g * J.Og + o) * J.R + row) * J.TV + (J.TV - 1 - tv)];
    }
}

}  // namespace

void run(const Jobs& jobs, hipStream_t s) {
    long long most = 0;
    for (int k = 0; k < jobs.n; k++) most = std::max(most, jobs.j[k].total);
    if (jobs.n > 0 && most > 0) CANVAS_LAUNCH(k_weight_prep, dim3((unsigned)((most + 255) / 256), (unsigned)jobs.n), dim3(256), 0, s, jobs);
}

}  // namespace wprep
}  // namespace canvas
