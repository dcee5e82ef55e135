// A block with C_in != C_out composed from one kernel template (Canvas paper, Section 4, "Main focus: convolutions"):
// m = max(C_in, C_out) / min(C_in, C_out) instances of the template's plan at [N, C, H, W], C = min(C_in, C_out).
// Expand (C_out = m C): every instance reads x, instance j writes channel slice j of y, dx is the sum of the instances'
// dx.  Reduce (C_in = m C): instance j reads channel slice j of x, y is the sum, instance j writes slice j of dx.
// A channel slice of an NCHW batch is strided over the images.  Plans whose kernels address their input and output through
// an image stride (the fused shift / grouped FC / unary / residual family) read and write the slices in place; the other
// plans take dense tensors: ONE launch
// regroups [N, m, C P] into m dense tensors [N, C P] or back (16-byte accesses), ONE launch adds the m dense results of
// the instances (in fp32 registers, in instance order, rounded once).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <memory>
#include <string>
#include <vector>

#include "../../include/canvas_block.h"
#include "launch.hpp"
#include "plan_calls.hpp"
#include "tile_util.hpp"

namespace canvas {
int set_last_error(int code, const std::string& msg);  // api.cpp
}

struct canvas_block {
    canvas_dag* plan = nullptr;
    canvas_block_info info;
    int64_t N = 0, C = 0, P = 0;
    int m = 1;
    bool expand = true, bf16 = false;
    bool direct = false;  // the plan's kernels take channel slices of the wide tensors as they are (image strides): no regrouping
    uint64_t plan_ws = 0, dense = 0, off_a = 0, off_b = 0;  // workspace: m plan workspaces | m dense inputs | m dense results
};

namespace canvas {
namespace block {
namespace {

using canvas::tile::u32x4;

int set_err(int code, const std::string& msg) { return canvas::set_last_error(code, msg); }
uint64_t align_up(uint64_t v) { return (v + 255) / 256 * 256; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// sliced [N][m][unit] <-> dense [m][N][unit] (instance j's dense tensor starts at j * dense_stride bytes); a unit is one
// image's slice, `upi` pieces of W bytes.  VEC: 16-byte pieces (every size a multiple of 16), else 2-byte elements.
template <bool VEC>
__global__ __launch_bounds__(256) void k_regroup(const unsigned char* __restrict__ src, unsigned char* __restrict__ dst, long long upi, int m,
                                                 long long n_images, long long dense_stride, int to_dense) {
    const long long u = (long long)blockIdx.x * 256 + threadIdx.x;
    if (u >= upi * m * n_images) return;
    constexpr int W = VEC ? 16 : 2;
    // u walks the sliced tensor: ((n * m) + j) * upi + k
    const long long nj = u / upi, k = u - nj * upi;
    const long long n = nj / m, j = nj - n * m;
    const long long sliced = u * W, dense = j * dense_stride + (n * upi + k) * W;
    const unsigned char* s = src + (to_dense ? sliced : dense);
    unsigned char* d = dst + (to_dense ? dense : sliced);
    if (VEC) *reinterpret_cast<u32x4*>(d) = *reinterpret_cast<const u32x4*>(s);
    else *reinterpret_cast<uint16_t*>(d) = *reinterpret_cast<const uint16_t*>(s);
}

// out[i] = parts[0][i] + parts[1][i] + ... (fp32, in that order), rounded to the element type once.  A thread takes 16 bytes
// of every part (8 bf16 or 4 fp32 elements; `pieces` such pieces, the parts are 256-byte aligned); the elements past the
// last whole piece go one per thread.
template <bool BF16>
__global__ __launch_bounds__(256) void k_sum(const unsigned char* __restrict__ parts, long long part_stride, int m, void* __restrict__ out,
                                             long long count, long long pieces) {
    constexpr int E = BF16 ? 8 : 4;
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i < pieces) {
        float t[E];
        for (int j = 0; j < m; j++) {
            const u32x4 v = *reinterpret_cast<const u32x4*>(parts + j * part_stride + i * 16);
#pragma unroll
            for (int e = 0; e < E; e++) {
                float f;
                if constexpr (BF16) f = (e & 1) ? canvas::tile::hi_f32(v[e >> 1]) : canvas::tile::lo_f32(v[e >> 1]);
                else f = __uint_as_float(v[e]);
                t[e] = j == 0 ? f : t[e] + f;
            }
        }
        u32x4 o;
#pragma unroll
        for (int k = 0; k < 4; k++) {
            if constexpr (BF16) o[k] = canvas::tile::pack_bf16(t[2 * k], t[2 * k + 1]);
            else o[k] = __float_as_uint(t[k]);
        }
        *reinterpret_cast<u32x4*>((unsigned char*)out + i * 16) = o;
        return;
    }
    const long long e = pieces * E + (i - pieces);
    if (e >= count) return;
    float t = 0.f;
    for (int j = 0; j < m; j++) {
        const unsigned char* p = parts + j * part_stride;
        const float v = BF16 ? __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(p)[e] << 16) : reinterpret_cast<const float*>(p)[e];
        t = j == 0 ? v : t + v;
    }
    if (BF16) reinterpret_cast<uint16_t*>(out)[e] = (uint16_t)(canvas::tile::pack_bf16(t, 0.f) & 0xffffu);
    else reinterpret_cast<float*>(out)[e] = t;
}

// all m channel slices of `sliced` ([N, m C, P]) to the m dense tensors at `dense` or back
void regroup(const canvas_block* b, const void* src, void* dst, bool to_dense, hipStream_t s) {
    const long long esz = b->bf16 ? 2 : 4;
    const long long bytes = b->C * b->P * esz;
    const bool vec = bytes % 16 == 0;
    const long long upi = vec ? bytes / 16 : bytes / 2, total = upi * b->m * b->N;
    if (total == 0) return;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (vec) CANVAS_LAUNCH(k_regroup<true>, grid, block, 0, s, (const unsigned char*)src, (unsigned char*)dst, upi, b->m, (long long)b->N, (long long)b->dense, to_dense ? 1 : 0);
    else CANVAS_LAUNCH(k_regroup<false>, grid, block, 0, s, (const unsigned char*)src, (unsigned char*)dst, upi, b->m, (long long)b->N, (long long)b->dense, to_dense ? 1 : 0);
}

void sum_instances(const canvas_block* b, const void* parts, void* out, hipStream_t s) {
    const long long count = b->N * b->C * b->P;
    if (count == 0) return;
    const long long pieces = count / (b->bf16 ? 8 : 4), threads = pieces + (count - pieces * (b->bf16 ? 8 : 4));
    const dim3 grid((unsigned)((threads + 255) / 256)), block(256);
    if (b->bf16) CANVAS_LAUNCH(k_sum<true>, grid, block, 0, s, (const unsigned char*)parts, (long long)b->dense, b->m, out, count, pieces);
    else CANVAS_LAUNCH(k_sum<false>, grid, block, 0, s, (const unsigned char*)parts, (long long)b->dense, b->m, out, count, pieces);
}

int check(const canvas_block* b, const void* x, const void* const* weights, const void* ws, size_t ws_bytes) {
    if (!b) return set_err(CANVAS_BAD_ARG, "null block handle");
    if (!x || !aligned16(x)) return set_err(CANVAS_BAD_ARG, "x must be a non-null, 16-byte aligned device pointer");
    if (b->info.n_weights > 0 && !weights) return set_err(CANVAS_BAD_ARG, "weights array is null");
    if (ws_bytes < b->info.workspace_bytes) return set_err(CANVAS_WORKSPACE_TOO_SMALL, "workspace smaller than workspace_bytes");
    if (!ws || !aligned16(ws)) return set_err(CANVAS_BAD_ARG, "workspace must be non-null and 16-byte aligned");
    return CANVAS_OK;
}

int finish() {
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return set_err(CANVAS_HIP_ERROR, std::string("kernel launch failed: ") + hipGetErrorString(e));
    return CANVAS_OK;
}

}  // namespace
}  // namespace block
}  // namespace canvas

using namespace canvas::block;

extern "C" {

int canvas_block_compile(const void* blob, size_t blob_len, const int64_t in_shape[4], int64_t c_out, canvas_dtype dt,
                         const canvas_options* opt, canvas_block** out) {
    if (!out) return set_err(CANVAS_BAD_ARG, "out is null");
    *out = nullptr;
    if (!in_shape) return set_err(CANVAS_BAD_ARG, "in_shape is null");
    if (opt && (opt->flags & CANVAS_OPT_INFERENCE)) return set_err(CANVAS_UNSUPPORTED, "a block has no inference plan");
    const int64_t c_in = in_shape[1];
    if (c_in < 1 || c_out < 1) return set_err(CANVAS_BAD_ARG, "channel counts must be positive");
    if (c_out % c_in != 0 && c_in % c_out != 0)
        return set_err(CANVAS_SHAPE_MISMATCH, "neither of C_in = " + std::to_string(c_in) + " and C_out = " + std::to_string(c_out) +
                                                  " is a multiple of the other");
    auto b = std::make_unique<canvas_block>();
    b->expand = c_out % c_in == 0;
    b->C = b->expand ? c_in : c_out;
    b->m = (int)((b->expand ? c_out : c_in) / b->C);
    const int64_t shape[4] = {in_shape[0], b->C, in_shape[2], in_shape[3]};
    int rc = canvas_dag_compile(blob, blob_len, shape, dt, opt, &b->plan);
    if (rc) return rc;
    rc = canvas_dag_query(b->plan, &b->info.plan);
    const canvas_dag_info& pi = b->info.plan;
    if (!rc && (pi.out_shape[1] != b->C || pi.out_shape[2] != 1))
        rc = set_err(CANVAS_SHAPE_MISMATCH, "the template must map [C, H, W] to [C, H, W]: its output has " + std::to_string(pi.out_shape[1]) +
                                                " channels and " + std::to_string(pi.out_shape[2]) + " taps for C = " + std::to_string(b->C));
    if (rc) {
        canvas_dag_destroy(b->plan);
        return rc;
    }
    b->N = in_shape[0];
    b->P = in_shape[2] * in_shape[3];
    b->bf16 = dt == CANVAS_BF16;
    b->dense = align_up((uint64_t)(b->N * b->C * b->P) * (b->bf16 ? 2 : 4));
    b->plan_ws = align_up(pi.workspace_bytes);
    b->off_a = b->plan_ws * (uint64_t)b->m;
    b->off_b = b->off_a + b->dense * (uint64_t)b->m;
    // (in place: 32-bit byte offsets over the wide tensors)
    b->direct = b->m > 1 && canvas::plan_takes_strided_io(b->plan) && b->N * b->C * b->m * b->P * (b->bf16 ? 2 : 4) < ((int64_t)1 << 31);
    b->info.instances = b->m;
    b->info.expand = b->expand ? 1 : 0;
    b->info.template_channels = b->C;
    b->info.n_weights = pi.n_weights;
    b->info.reserved0 = 0;
    b->info.workspace_bytes = b->off_b + b->dense * (uint64_t)b->m;
    *out = b.release();
    return CANVAS_OK;
}

int canvas_block_query(const canvas_block* block, canvas_block_info* info) {
    if (!block || !info) return set_err(CANVAS_BAD_ARG, "null argument");
    *info = block->info;
    return CANVAS_OK;
}

int canvas_block_forward(canvas_block* b, const void* x, const void* const* weights, void* y, void* workspace, size_t workspace_bytes,
                         void* stream) {
    int rc = check(b, x, weights, workspace, workspace_bytes);
    if (rc) return rc;
    if (!y || !aligned16(y)) return set_err(CANVAS_BAD_ARG, "y must be a non-null, 16-byte aligned device pointer");
    char* ws = (char*)workspace;
    const hipStream_t s = (hipStream_t)stream;
    char* A = ws + b->off_a;  // dense inputs of the instances (reduce: the slices of x, kept for backward)
    char* R = ws + b->off_b;  // dense results of the instances
    const int nw = b->info.n_weights;
    (void)hipGetLastError();
    const int64_t slice = b->C * b->P, wide = slice * b->m;      // elements of one image's slice / of one wide image
    const int64_t sbytes = slice * (b->bf16 ? 2 : 4);
    if (!b->expand && !b->direct) regroup(b, x, A, true, s);
    for (int j = 0; j < b->m; j++) {
        void* pws = ws + (uint64_t)j * b->plan_ws;
        const void* const* wj = weights ? weights + (size_t)j * nw : nullptr;
        void* rj = R + (uint64_t)j * b->dense;
        if (b->m == 1) rc = canvas_dag_forward(b->plan, x, wj, y, pws, b->plan_ws, stream);  // (the plan writes y itself)
        else if (b->direct && b->expand) rc = canvas::plan_forward(b->plan, x, wj, (char*)y + j * sbytes, pws, b->plan_ws, stream, 0, wide);
        else if (b->direct) rc = canvas::plan_forward(b->plan, (const char*)x + j * sbytes, wj, rj, pws, b->plan_ws, stream, wide, 0);
        else rc = canvas_dag_forward(b->plan, b->expand ? x : (const void*)(A + (uint64_t)j * b->dense), wj, rj, pws, b->plan_ws, stream);
        if (rc) return rc;
    }
    if (b->m > 1) {
        if (!b->expand) sum_instances(b, R, y, s);
        else if (!b->direct) regroup(b, R, y, false, s);
    }
    return finish();
}

int canvas_block_backward(canvas_block* b, const void* x, const void* const* weights, const void* dy, void* dx, void* const* dweights,
                          void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check(b, x, weights, workspace, workspace_bytes);
    if (rc) return rc;
    if (!dy || !aligned16(dy) || !dx || !aligned16(dx)) return set_err(CANVAS_BAD_ARG, "dy and dx must be non-null, 16-byte aligned device pointers");
    if (b->info.n_weights > 0 && !dweights) return set_err(CANVAS_BAD_ARG, "dweights array is null");
    char* ws = (char*)workspace;
    const hipStream_t s = (hipStream_t)stream;
    char* A = ws + b->off_a;
    char* R = ws + b->off_b;
    const int nw = b->info.n_weights;
    (void)hipGetLastError();
    const int64_t slice = b->C * b->P, wide = slice * b->m;
    const int64_t sbytes = slice * (b->bf16 ? 2 : 4);
    if (b->expand && b->m > 1 && !b->direct) regroup(b, dy, A, true, s);  // (expand: the slices of dy; reduce: A still holds the slices of x)
    for (int j = 0; j < b->m; j++) {
        void* pws = ws + (uint64_t)j * b->plan_ws;
        const void* const* wj = weights ? weights + (size_t)j * nw : nullptr;
        void* const* dwj = dweights ? dweights + (size_t)j * nw : nullptr;
        void* rj = R + (uint64_t)j * b->dense;
        if (b->m == 1) {
            rc = canvas_dag_backward(b->plan, x, wj, dy, dx, dwj, pws, b->plan_ws, stream);
        } else if (b->direct && b->expand) {
            rc = canvas::plan_backward(b->plan, x, wj, (const char*)dy + j * sbytes, rj, dwj, pws, b->plan_ws, stream, 0, wide);
        } else if (b->direct) {
            rc = canvas::plan_backward(b->plan, (const char*)x + j * sbytes, wj, dy, (char*)dx + j * sbytes, dwj, pws, b->plan_ws, stream, wide, 0);
        } else {
            const void* xj = b->expand ? x : (const void*)(A + (uint64_t)j * b->dense);
            const void* dyj = b->expand ? (const void*)(A + (uint64_t)j * b->dense) : dy;
            rc = canvas_dag_backward(b->plan, xj, wj, dyj, rj, dwj, pws, b->plan_ws, stream);
        }
        if (rc) return rc;
    }
    if (b->m > 1) {
        if (b->expand) sum_instances(b, R, dx, s);
        else if (!b->direct) regroup(b, R, dx, false, s);
    }
    return finish();
}

void canvas_block_destroy(canvas_block* block) {
    if (block) canvas_dag_destroy(block->plan);
    delete block;
}

}  // extern "C"
