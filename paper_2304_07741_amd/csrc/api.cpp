// C ABI: compile / query / forward / backward / destroy.
#include <hip/hip_runtime.h>

#include <cstring>
#include <memory>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/canvas_dag.h"
#include "dag.hpp"
#include "launch.hpp"
#include "lowering.hpp"
#include "plan_calls.hpp"

struct canvas_dag {
    canvas::Dag dag;
    bool bf16 = false;
    bool inference = false;
    std::unique_ptr<canvas::Lowering> low;
    canvas_dag_info info;
    bool timing = false;
    std::vector<hipEvent_t> ev[2];  // a (start, stop) pair per launch and direction
    bool timed_once[2] = {false, false};
};

namespace {
thread_local std::string g_err;
}

// Workspace of canvas_dag_forward_static: one array per GPU, part of the library's code object, so that
// callers that may not allocate device memory still have somewhere to put the derived weights and the
// intermediates of a forward pass.  In host code this name is only a handle: the device address comes from
// hipGetSymbolAddress (static_scratch_of below) and only that address is handed to kernels.
static __device__ __align__(256) unsigned char scratch[CANVAS_STATIC_WORKSPACE_BYTES];

namespace canvas {
thread_local TimingEvents g_timing;
// the message canvas_last_error() returns, for the other translation units of the C ABI
int set_last_error(int code, const std::string& msg) {
    g_err = msg;
    return code;
}
}  // namespace canvas

namespace {

int set_err(int code, const std::string& msg) { return canvas::set_last_error(code, msg); }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_common(const canvas_dag* d, const void* x, const void* const* weights, const void* ws, size_t ws_bytes) {
    if (!d) return set_err(CANVAS_BAD_ARG, "null dag handle");
    if (!x || !aligned16(x)) return set_err(CANVAS_BAD_ARG, "x must be a non-null, 16-byte aligned device pointer");
    if (d->dag.n_weights > 0) {
        if (!weights) return set_err(CANVAS_BAD_ARG, "weights array is null");
        for (int i = 0; i < d->dag.n_weights; i++)
            if (!weights[i] || !aligned16(weights[i])) return set_err(CANVAS_BAD_ARG, "a weight pointer is null or misaligned");
    }
    if (ws_bytes < d->low->ws_bytes) return set_err(CANVAS_WORKSPACE_TOO_SMALL, "workspace smaller than workspace_bytes");
    if (d->low->ws_bytes > 0 && (!ws || !aligned16(ws))) return set_err(CANVAS_BAD_ARG, "workspace must be non-null and 16-byte aligned");
    return CANVAS_OK;
}

int finish_launches() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return set_err(CANVAS_HIP_ERROR, std::string("kernel launch failed: ") + hipGetErrorString(e));
    return CANVAS_OK;
}

void run_launches(canvas_dag* d, int backward, const canvas::RunArgs& a) {
    const auto& v = backward ? d->low->bwd : d->low->fwd;
    if (!d->timing) {
        for (const auto& l : v) l.run(a);
        return;
    }
    auto& ev = d->ev[backward];
    for (size_t i = 0; i < v.size(); i++) {
        canvas::g_timing.start = ev[2 * i];
        canvas::g_timing.stop = ev[2 * i + 1];
        v[i].run(a);
    }
    canvas::g_timing = canvas::TimingEvents();
    d->timed_once[backward] = true;
}

// Device address of this GPU's copy of `scratch`, looked up once per device with that device current.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch_of_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return set_err(CANVAS_HIP_ERROR, std::string("hipGetDevice failed: ") + hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return set_err(CANVAS_UNSUPPORTED, "device ordinal beyond the static workspace table");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return set_err(CANVAS_HIP_ERROR, std::string("hipGetSymbolAddress(static workspace) failed: ") + hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return CANVAS_OK;
}

void drop_events(canvas_dag* d) {
    for (auto& v : d->ev) {
        for (hipEvent_t e : v) (void)hipEventDestroy(e);
        v.clear();
    }
    d->timing = false;
    d->timed_once[0] = d->timed_once[1] = false;
}

}  // namespace

extern "C" {

int canvas_dag_compile(const void* blob, size_t blob_len, const int64_t in_shape[4], canvas_dtype dt,
                       const canvas_options* opt, canvas_dag** out) {
    try {
        if (!out) return set_err(CANVAS_BAD_ARG, "null output handle");
        *out = nullptr;
        if (dt != CANVAS_F32 && dt != CANVAS_BF16) return set_err(CANVAS_BAD_ARG, "unknown dtype");
        uint32_t flags = 0;
        if (opt) {
            flags = opt->flags;
            for (uint32_t r : opt->reserved)
                if (r) return set_err(CANVAS_BAD_ARG, "reserved option fields must be zero");
            if (flags & ~(CANVAS_OPT_NO_FUSION | CANVAS_OPT_INFERENCE)) return set_err(CANVAS_BAD_ARG, "unknown option flag");
        }
        auto d = std::make_unique<canvas_dag>();
        std::string err;
        int rc = canvas::parse_dag((const char*)blob, blob_len, in_shape, d->dag, err);
        if (rc != 0) return set_err(rc, err);
        d->bf16 = dt == CANVAS_BF16;
        d->low = canvas::lower(d->dag, d->bf16, (flags & CANVAS_OPT_NO_FUSION) != 0);
        d->inference = (flags & CANVAS_OPT_INFERENCE) != 0;
        if (d->inference) canvas::make_inference_plan(*d->low);

        canvas_dag_info& I = d->info;
        std::memset(&I, 0, sizeof I);
        const canvas::Dag& g = d->dag;
        I.n_nodes = (int32_t)g.nodes.size();
        I.out_node = g.out;
        I.n_weights = g.n_weights;
        I.n_launches_fwd = (int32_t)d->low->fwd.size();
        I.n_launches_bwd = (int32_t)d->low->bwd.size();
        I.n_launches_prepare = (int32_t)d->low->prep.size();
        I.fused = d->low->fused ? 1 : 0;
        I.n_fused_chains = d->low->chain_units;
        I.n_fused_nodes = d->low->chain_nodes;
        const double esz = d->bf16 ? 2.0 : 4.0;
        double wbytes = 0, wcount = 0;
        for (int k = 0; k < I.n_nodes; k++) {
            const canvas::Node& nd = g.nodes[k];
            int64_t s[5] = {g.N, nd.C, nd.T, (nd.pooled & 1) ? 1 : g.H, (nd.pooled & 2) ? 1 : g.W};
            std::memcpy(I.node_shape[k], s, sizeof s);
            if (nd.op == canvas::Op::Fc) {
                const canvas::Node& A = g.nodes[nd.a];
                int64_t K = (int64_t)(A.C / nd.groups) * A.T;
                I.weight_shape[nd.widx][0] = nd.groups;
                I.weight_shape[nd.widx][1] = nd.out / nd.groups;
                I.weight_shape[nd.widx][2] = K;
                I.weight_node[nd.widx] = k;
                if (nd.live) I.fc_flops_fwd += 2.0 * g.N * g.H * g.W * nd.out * K;
                wbytes += esz * nd.out * K;
                wcount += (double)nd.out * K;
            }
        }
        std::memcpy(I.out_shape, I.node_shape[g.out], sizeof I.out_shape);
        I.workspace_bytes = d->low->ws_bytes;
        I.min_bytes_fwd = esz * (g.numel(0) + g.numel(g.out)) + wbytes;
        I.min_bytes_bwd = esz * (2.0 * g.numel(0) + g.numel(g.out)) + wbytes + 4.0 * wcount;
        *out = d.release();
        return CANVAS_OK;
    } catch (const std::exception& e) {
        return set_err(CANVAS_UNSUPPORTED, std::string("compile failed: ") + e.what());
    }
}

int canvas_dag_query(const canvas_dag* dag, canvas_dag_info* info) {
    if (!dag || !info) return set_err(CANVAS_BAD_ARG, "null argument");
    *info = dag->info;
    return CANVAS_OK;
}

int canvas_dag_launch_desc(const canvas_dag* dag, int backward, int idx, canvas_launch_desc* out) {
    if (!dag || !out) return set_err(CANVAS_BAD_ARG, "null argument");
    const auto& v = backward ? dag->low->bwd : dag->low->fwd;
    if (idx < 0 || idx >= (int)v.size()) return set_err(CANVAS_BAD_ARG, "launch index out of range");
    std::memset(out, 0, sizeof *out);
    std::strncpy(out->name, v[idx].name.c_str(), sizeof(out->name) - 1);
    out->bytes = v[idx].bytes;
    out->flops = v[idx].flops;
    return CANVAS_OK;
}

int canvas_dag_forward(canvas_dag* dag, const void* x, const void* const* weights, void* y, void* workspace,
                       size_t workspace_bytes, void* stream) {
    return canvas::plan_forward(dag, x, weights, y, workspace, workspace_bytes, stream, 0, 0);
}

int canvas_dag_forward_static(canvas_dag* dag, const void* x, const void* const* weights, void* y, void* stream) {
    if (!dag) return set_err(CANVAS_BAD_ARG, "null dag handle");
    if (dag->low->ws_bytes > (uint64_t)CANVAS_STATIC_WORKSPACE_BYTES)
        return set_err(CANVAS_WORKSPACE_TOO_SMALL, "this plan needs " + std::to_string(dag->low->ws_bytes) +
                                                       " workspace bytes, the static workspace holds " +
                                                       std::to_string((uint64_t)CANVAS_STATIC_WORKSPACE_BYTES) +
                                                       ": use canvas_dag_forward with a workspace of the caller");
    void* ws = nullptr;
    int rc = static_scratch_of_current_device(&ws);
    if (rc) return rc;
    rc = check_common(dag, x, weights, ws, (size_t)CANVAS_STATIC_WORKSPACE_BYTES);
    if (rc) return rc;
    if (!y || !aligned16(y)) return set_err(CANVAS_BAD_ARG, "y must be a non-null, 16-byte aligned device pointer");
    canvas::RunArgs a;
    a.x = x;
    a.w = weights;
    a.y = y;
    a.ws = (char*)ws;
    a.stream = (hipStream_t)stream;
    (void)hipGetLastError();
    // an inference plan keeps its weight-only launches apart: here they run with every call, as the static
    // workspace is shared by all plans and calls on this GPU and keeps nothing between them
    for (const auto& l : dag->low->prep) l.run(a);
    run_launches(dag, 0, a);
    return finish_launches();
}

int canvas_dag_prepare(canvas_dag* dag, const void* const* weights, void* workspace, size_t workspace_bytes, void* stream) {
    if (!dag) return set_err(CANVAS_BAD_ARG, "null dag handle");
    if (!dag->inference) return set_err(CANVAS_BAD_ARG, "canvas_dag_prepare needs a plan compiled with CANVAS_OPT_INFERENCE");
    if (dag->low->prep.empty()) return CANVAS_OK;
    int rc = check_common(dag, workspace, weights, workspace, workspace_bytes);  // (no x here: the workspace stands in for the pointer check)
    if (rc) return rc;
    canvas::RunArgs a;
    a.w = weights;
    a.ws = (char*)workspace;
    a.stream = (hipStream_t)stream;
    (void)hipGetLastError();
    for (const auto& l : dag->low->prep) l.run(a);
    return finish_launches();
}

int canvas_dag_backward(canvas_dag* dag, const void* x, const void* const* weights, const void* dy, void* dx,
                        void* const* dweights, void* workspace, size_t workspace_bytes, void* stream) {
    return canvas::plan_backward(dag, x, weights, dy, dx, dweights, workspace, workspace_bytes, stream, 0, 0);
}

}  // extern "C"

namespace canvas {

bool plan_takes_strided_io(const canvas_dag* dag) { return dag && dag->low->strided_io; }

int plan_forward(canvas_dag* dag, const void* x, const void* const* weights, void* y, void* workspace, size_t workspace_bytes,
                 void* stream, int64_t x_stride, int64_t y_stride) {
    int rc = check_common(dag, x, weights, workspace, workspace_bytes);
    if (rc) return rc;
    if (!y || !aligned16(y)) return set_err(CANVAS_BAD_ARG, "y must be a non-null, 16-byte aligned device pointer");
    if ((x_stride || y_stride) && !dag->low->strided_io) return set_err(CANVAS_UNSUPPORTED, "this plan takes dense tensors only");
    RunArgs a;
    a.x = x;
    a.w = weights;
    a.y = y;
    a.ws = (char*)workspace;
    a.stream = (hipStream_t)stream;
    a.x_stride = x_stride;
    a.y_stride = y_stride;
    (void)hipGetLastError();
    run_launches(dag, 0, a);
    return finish_launches();
}

int plan_backward(canvas_dag* dag, const void* x, const void* const* weights, const void* dy, void* dx, void* const* dweights,
                  void* workspace, size_t workspace_bytes, void* stream, int64_t x_stride, int64_t y_stride) {
    if (dag && dag->inference) return set_err(CANVAS_UNSUPPORTED, "this plan was compiled for inference: it has no backward pass");
    int rc = check_common(dag, x, weights, workspace, workspace_bytes);
    if (rc) return rc;
    if (!dy || !aligned16(dy) || !dx || !aligned16(dx)) return set_err(CANVAS_BAD_ARG, "dy and dx must be non-null, 16-byte aligned device pointers");
    if (dag->dag.n_weights > 0) {
        if (!dweights) return set_err(CANVAS_BAD_ARG, "dweights array is null");
        for (int i = 0; i < dag->dag.n_weights; i++)
            if (!dweights[i] || !aligned16(dweights[i])) return set_err(CANVAS_BAD_ARG, "a dweights pointer is null or misaligned");
    }
    canvas::RunArgs a;
    a.x = x;
    a.w = weights;
    a.dy = dy;
    a.dx = dx;
    a.dw = dweights;
    a.ws = (char*)workspace;
    a.stream = (hipStream_t)stream;
    if ((x_stride || y_stride) && !dag->low->strided_io) return set_err(CANVAS_UNSUPPORTED, "this plan takes dense tensors only");
    a.x_stride = x_stride;
    a.y_stride = y_stride;
    (void)hipGetLastError();
    run_launches(dag, 1, a);
    return finish_launches();
}

}  // namespace canvas

extern "C" {

int canvas_dag_set_timing(canvas_dag* dag, int enable) {
    if (!dag) return set_err(CANVAS_BAD_ARG, "null dag handle");
    drop_events(dag);
    if (!enable) return CANVAS_OK;
    for (int b = 0; b < 2; b++) {
        size_t n = (b ? dag->low->bwd.size() : dag->low->fwd.size()) * 2;
        for (size_t i = 0; i < n; i++) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) {
                drop_events(dag);
                return set_err(CANVAS_HIP_ERROR, "hipEventCreate failed");
            }
            dag->ev[b].push_back(e);
        }
    }
    dag->timing = true;
    return CANVAS_OK;
}

int canvas_dag_get_timing(canvas_dag* dag, int backward, float* ms, int n) {
    if (!dag || !ms) return set_err(CANVAS_BAD_ARG, "null argument");
    backward = backward ? 1 : 0;
    const size_t nl = backward ? dag->low->bwd.size() : dag->low->fwd.size();
    if (!dag->timing || !dag->timed_once[backward]) return set_err(CANVAS_BAD_ARG, "no timed call to read");
    if (n != (int)nl) return set_err(CANVAS_BAD_ARG, "n must equal the number of launches");
    auto& ev = dag->ev[backward];
    for (size_t i = 0; i < nl; i++) {
        if (hipEventSynchronize(ev[2 * i + 1]) != hipSuccess) return set_err(CANVAS_HIP_ERROR, "hipEventSynchronize failed");
        if (hipEventElapsedTime(&ms[i], ev[2 * i], ev[2 * i + 1]) != hipSuccess) return set_err(CANVAS_HIP_ERROR, "hipEventElapsedTime failed");
    }
    return CANVAS_OK;
}

void canvas_dag_destroy(canvas_dag* dag) {
    if (dag) drop_events(dag);
    delete dag;
}

const char* canvas_last_error(void) { return g_err.c_str(); }

}  // extern "C"
