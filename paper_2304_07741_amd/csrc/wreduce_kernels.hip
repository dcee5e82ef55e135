#include "wreduce_kernels.hpp"

#include <algorithm>

#include "launch.hpp"

namespace canvas {
namespace wreduce {

namespace {

// blockIdx.y selects the job.  Threads are numbered in the order of the partials' elements, so the elements
// of a segment read whole 128-byte lines of each partial; for the packed layout (whose element order differs
// from dw: the tap is innermost there) the padding is skipped and the small result is written scattered.
// Order of the sum of one element: the partials of a segment in ascending order, then the segments in
// ascending order -- independent of the launch.
__global__ __launch_bounds__(256) void k_reduce(Jobs jobs) {
    __shared__ float red[256];
    const Job& J = jobs.j[blockIdx.y];
    if (blockIdx.x >= J.blocks) return;  // (uniform per workgroup)
    const int el_per = 256 / J.segs;
    const int el = (int)threadIdx.x % el_per, seg = (int)threadIdx.x / el_per;
    const unsigned idx = blockIdx.x * (unsigned)el_per + (unsigned)el;
    long long e = -1;  // element of dw, if this position holds one
    if (idx < J.count) {
        if (J.kind == 0) {
            e = idx;
        } else {
            const unsigned rp = idx % (unsigned)J.Rp;
            unsigned t = idx / (unsigned)J.Rp;
            const unsigned tap = t % (unsigned)J.TV;
            t /= (unsigned)J.TV;
            const int op = (int)(t % (unsigned)J.Omp), gmi = (int)(t / (unsigned)J.Omp);
            const int sub = op / J.Og, o = op - sub * J.Og;
            const int subr = (int)rp / J.R, row = (int)rp - subr * J.R;
            const int g = gmi * J.gm + sub;
            if (sub < J.gm && subr == sub && g < J.G) e = (((long long)g * J.Og + o) * J.R + row) * J.TV + tap;
        }
    }
    float sum = 0.f;
    if (e >= 0) {
        const int per = (J.slices + J.segs - 1) / J.segs;
        const int end = min(J.slices, (seg + 1) * per);
        const float* src = J.partial + idx;
        int k = seg * per;
        for (; k + 16 <= end; k += 16) {  // sixteen independent loads in flight (a round trip to memory each), summed in slice order
            float v[16];
#pragma unroll
            for (int i = 0; i < 16; i++) v[i] = src[(long long)(k + i) * J.count];
#pragma unroll
            for (int i = 0; i < 16; i++) sum += v[i];
        }
        for (; k + 4 <= end; k += 4) {
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; i++) v[i] = src[(long long)(k + i) * J.count];
#pragma unroll
            for (int i = 0; i < 4; i++) sum += v[i];
        }
        for (; k < end; k++) sum += src[(long long)k * J.count];
    }
    red[seg * el_per + el] = sum;
    __syncthreads();
    if (seg == 0 && e >= 0) {
        float t = red[el];
        for (int i = 1; i < J.segs; i++) t += red[i * el_per + el];
        J.dw[e] = t;
    }
}

}  // namespace

void plan(Job& job) {
    job.segs = job.slices >= 32 ? 8 : 2;  // few partials: fewer, longer segments
    const unsigned el_per = 256u / (unsigned)job.segs;
    job.blocks = (job.count + el_per - 1) / el_per;
}

void run(const Jobs& jobs, hipStream_t s) {
    unsigned most = 0;
    for (int k = 0; k < jobs.n; k++) most = std::max(most, jobs.j[k].blocks);
    if (jobs.n > 0 && most > 0) CANVAS_LAUNCH(k_reduce, dim3(most, (unsigned)jobs.n), dim3(256), 0, s, jobs);
}

}  // namespace wreduce
}  // namespace canvas
