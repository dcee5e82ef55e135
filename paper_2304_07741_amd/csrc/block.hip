// A block with C_in != C_out composed from one kernel template (Canvas paper, Section 4, "Main focus: convolutions"):
// m = max(C_in, C_out) / min(C_in, C_out) instances of the template's plan at [N, C, H, W], C = min(C_in, C_out).
// Expand (C_out = m C): every instance reads x, instance j writes channel slice j of y, dx is the sum of the instances'
// dx.  Reduce (C_in = m C): instance j reads channel slice j of x, y is the sum, instance j writes slice j of dx.
// A channel slice of an NCHW batch is strided over the images, the plan's kernels take dense tensors: slices are
// copied by the two kernels below (16-byte accesses), sums over the instances are kept in fp32 and rounded once.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <memory>
#include <string>
#include <vector>

#include "../../include/canvas_block.h"
#include "launch.hpp"
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
    uint64_t plan_ws = 0, off_a = 0, off_b = 0, off_sum = 0;
};

namespace {

using canvas::tile::u32x4;

int set_err(int code, const std::string& msg) { return canvas::set_last_error(code, msg); }
uint64_t align_up(uint64_t v) { return (v + 255) / 256 * 256; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// dst image n (dst_stride bytes apart, from dst_off) = src image n (src_stride apart, from src_off), `bytes` each.
// VEC: all of these are multiples of 16 and a thread moves 16 bytes; else a thread moves one 2-byte element.
template <bool VEC>
__global__ __launch_bounds__(256) void k_slice_copy(const unsigned char* __restrict__ src, unsigned char* __restrict__ dst, long long bytes,
                                                    long long src_stride, long long dst_stride, long long src_off, long long dst_off,
                                                    long long units_per_image, long long total_units) {
    const long long u = (long long)blockIdx.x * 256 + threadIdx.x;
    if (u >= total_units) return;
    const long long n = u / units_per_image, k = u - n * units_per_image;
    constexpr int W = VEC ? 16 : 2;
    const unsigned char* s = src + n * src_stride + src_off + k * W;
    unsigned char* d = dst + n * dst_stride + dst_off + k * W;
    if (VEC) *reinterpret_cast<u32x4*>(d) = *reinterpret_cast<const u32x4*>(s);
    else *reinterpret_cast<uint16_t*>(d) = *reinterpret_cast<const uint16_t*>(s);
    (void)bytes;
}

// sum (fp32) = first ? part : sum + part; on the last instance the total is also written to `out` in the element type.
template <bool BF16>
__global__ __launch_bounds__(256) void k_accumulate(const void* __restrict__ part, float* __restrict__ sum, void* __restrict__ out,
                                                    long long count, int first, int last) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    float v;
    if (BF16) v = __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(part)[i] << 16);
    else v = reinterpret_cast<const float*>(part)[i];
    const float t = first ? v : sum[i] + v;
    if (!last) {
        sum[i] = t;
    } else if (BF16) {
        reinterpret_cast<uint16_t*>(out)[i] = (uint16_t)(canvas::tile::pack_bf16(t, 0.f) & 0xffffu);
    } else {
        reinterpret_cast<float*>(out)[i] = t;
    }
}

// copies channel slice j of `sliced` ([N, m C, P]) to the dense `dense` ([N, C, P]) or back
void slice_copy(const canvas_block* b, const void* src, void* dst, int j, bool to_dense, hipStream_t s) {
    const long long esz = b->bf16 ? 2 : 4;
    const long long bytes = b->C * b->P * esz, wide = bytes * b->m;
    const bool vec = bytes % 16 == 0;
    const long long upi = vec ? bytes / 16 : bytes / 2, total = upi * b->N;
    if (total == 0) return;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    const long long so = to_dense ? j * bytes : 0, dof = to_dense ? 0 : j * bytes;
    const long long ss = to_dense ? wide : bytes, ds = to_dense ? bytes : wide;
    if (vec) CANVAS_LAUNCH(k_slice_copy<true>, grid, block, 0, s, (const unsigned char*)src, (unsigned char*)dst, bytes, ss, ds, so, dof, upi, total);
    else CANVAS_LAUNCH(k_slice_copy<false>, grid, block, 0, s, (const unsigned char*)src, (unsigned char*)dst, bytes, ss, ds, so, dof, upi, total);
}

void accumulate(const canvas_block* b, const void* part, float* sum, void* out, bool first, bool last, hipStream_t s) {
    const long long count = b->N * b->C * b->P;
    if (count == 0) return;
    const dim3 grid((unsigned)((count + 255) / 256)), block(256);
    if (b->bf16) CANVAS_LAUNCH(k_accumulate<true>, grid, block, 0, s, part, sum, out, count, first ? 1 : 0, last ? 1 : 0);
    else CANVAS_LAUNCH(k_accumulate<false>, grid, block, 0, s, part, sum, out, count, first ? 1 : 0, last ? 1 : 0);
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
    const uint64_t dense = align_up((uint64_t)(b->N * b->C * b->P) * (b->bf16 ? 2 : 4));
    b->plan_ws = align_up(pi.workspace_bytes);
    b->off_a = b->plan_ws * (uint64_t)b->m;
    b->off_b = b->off_a + dense;
    b->off_sum = b->off_b + dense;
    b->info.instances = b->m;
    b->info.expand = b->expand ? 1 : 0;
    b->info.template_channels = b->C;
    b->info.n_weights = pi.n_weights;
    b->info.reserved0 = 0;
    b->info.workspace_bytes = b->off_sum + align_up((uint64_t)(b->N * b->C * b->P) * 4);
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
    void* ta = ws + b->off_a;
    void* tb = ws + b->off_b;
    const int nw = b->info.n_weights;
    (void)hipGetLastError();
    for (int j = 0; j < b->m; j++) {
        void* pws = ws + (uint64_t)j * b->plan_ws;
        const void* const* wj = weights ? weights + (size_t)j * nw : nullptr;
        if (b->expand) {
            // (one instance: the plan writes y itself)
            rc = canvas_dag_forward(b->plan, x, wj, b->m == 1 ? y : ta, pws, b->plan_ws, stream);
            if (rc) return rc;
            if (b->m > 1) slice_copy(b, ta, y, j, false, s);
        } else {
            slice_copy(b, x, ta, j, true, s);
            rc = canvas_dag_forward(b->plan, ta, wj, tb, pws, b->plan_ws, stream);
            if (rc) return rc;
            accumulate(b, tb, (float*)(ws + b->off_sum), y, j == 0, j == b->m - 1, s);
        }
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
    void* ta = ws + b->off_a;
    void* tb = ws + b->off_b;
    const int nw = b->info.n_weights;
    (void)hipGetLastError();
    for (int j = 0; j < b->m; j++) {
        void* pws = ws + (uint64_t)j * b->plan_ws;
        const void* const* wj = weights ? weights + (size_t)j * nw : nullptr;
        void* const* dwj = dweights ? dweights + (size_t)j * nw : nullptr;
        if (b->expand) {
            if (b->m == 1) {
                rc = canvas_dag_backward(b->plan, x, wj, dy, dx, dwj, pws, b->plan_ws, stream);
                if (rc) return rc;
                continue;
            }
            slice_copy(b, dy, ta, j, true, s);
            rc = canvas_dag_backward(b->plan, x, wj, ta, tb, dwj, pws, b->plan_ws, stream);
            if (rc) return rc;
            accumulate(b, tb, (float*)(ws + b->off_sum), dx, j == 0, j == b->m - 1, s);
        } else {
            slice_copy(b, x, ta, j, true, s);
            rc = canvas_dag_backward(b->plan, ta, wj, dy, tb, dwj, pws, b->plan_ws, stream);
            if (rc) return rc;
            slice_copy(b, tb, dx, j, false, s);
        }
    }
    return finish();
}

void canvas_block_destroy(canvas_block* block) {
    if (block) canvas_dag_destroy(block->plan);
    delete block;
}

}  // extern "C"
