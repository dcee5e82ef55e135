#include "wprep_kernels.hpp"

#include <algorithm>

#include "launch.hpp"

namespace canvas {
namespace wprep {

namespace {

// One element of a job's output; IDX = unsigned where the job's element count allows (64-bit division is an
// instruction sequence several times as long).
template <typename IDX>
__device__ __forceinline__ void write_element(const Job& J, IDX i) {
    if (J.kind == 0) {
        // wp[gmi][op][tap][rp]: block-diagonal over the gm merged groups, zero in the padding
        const int rp = (int)(i % (IDX)J.Rp);
        IDX t = i / (IDX)J.Rp;
        const int tap = (int)(t % (IDX)J.TV);
        t /= (IDX)J.TV;
        const int op = (int)(t % (IDX)J.Omp), gmi = (int)(t / (IDX)J.Omp);
        const int sub = op / J.Og, o = op - sub * J.Og;
        const int subr = rp / J.R, row = rp - subr * J.R;
        const int g = gmi * J.gm + sub;
        uint16_t v = 0;
        if (sub < J.gm && subr == sub && g < J.G)
            v = J.transposed ? J.w[(((long long)g * J.R + row) * J.Og + o) * J.TV + (J.TV - 1 - tap)]
                             : J.w[(((long long)g * J.Og + o) * J.R + row) * J.TV + tap];
        J.out[i] = v;
    } else {
        const int tv = (int)(i % (IDX)J.TV);
        IDX q = i / (IDX)J.TV;
        const int o = (int)(q % (IDX)J.Og);
        q /= (IDX)J.Og;
        const int row = (int)(q % (IDX)J.R), g = (int)(q / (IDX)J.R);
        J.out[i] = J.w[((long long)(g * J.Og + o) * J.R + row) * J.TV + (J.TV - 1 - tv)];
    }
}

// blockIdx.y selects the job, blockIdx.x * 256 + threadIdx.x the element it writes
__global__ __launch_bounds__(256) void k_weight_prep(Jobs jobs) {
    const Job& J = jobs.j[blockIdx.y];
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= J.total) return;
    if (J.total <= 0xffffffffll) write_element<unsigned>(J, (unsigned)i);
    else write_element<unsigned long long>(J, (unsigned long long)i);
}

}  // namespace

void run(const Jobs& jobs, hipStream_t s) {
    long long most = 0;
    for (int k = 0; k < jobs.n; k++) most = std::max(most, jobs.j[k].total);
    if (jobs.n > 0 && most > 0) CANVAS_LAUNCH(k_weight_prep, dim3((unsigned)((most + 255) / 256), (unsigned)jobs.n), dim3(256), 0, s, jobs);
}

}  // namespace wprep
}  // namespace canvas
