// A lowering turns a parsed micro-DAG into a fixed list of kernel launches for forward and backward.
// It is built once by canvas_dag_compile (host only) and replayed by canvas_dag_forward/backward.
#pragma once
#include <hip/hip_runtime.h>

#include <functional>
#include <memory>
#include <string>
#include <vector>

#include "dag.hpp"
#include "wprep_kernels.hpp"
#include "wreduce_kernels.hpp"

namespace canvas {

struct RunArgs {
    const void* x = nullptr;
    const void* const* w = nullptr;
    void* y = nullptr;
    const void* dy = nullptr;
    void* dx = nullptr;
    void* const* dw = nullptr;
    char* ws = nullptr;
    hipStream_t stream = nullptr;
    // Elements between consecutive images of x / dx and of y / dy; 0 = dense.  Only a lowering with `strided_io` reads
    // them (its input and output may then be channel slices of wider tensors).
    int64_t x_stride = 0, y_stride = 0;
};

struct Launch {
    std::string name;
    double bytes = 0;  // algorithmic bytes: every operand of the launch once
    double flops = 0;  // algorithmic flops of FC contractions
    std::function<void(const RunArgs&)> run;
    bool prep = false;  // touches only the weights (packing, widening): an inference plan runs it once, ahead of the forward calls
};

// A derived copy of the weights of FC number widx, written at byte offset `off` of the workspace.
struct WeightJob {
    wprep::Job job;  // geometry; the pointers are filled at run time
    int widx = 0;
    int64_t off = 0;
    double bytes = 0;
};

// The fixed-order sum of the weight-gradient partials of FC number widx (at byte offset `off` of the workspace).
struct ReduceJob {
    wreduce::Job job;  // geometry; the pointers are filled at run time
    int widx = 0;
    int64_t off = 0;
    double bytes = 0;
};

struct Lowering {
    bool fused = false;            // one of the whole-DAG kernel families
    bool strided_io = false;       // honours RunArgs::x_stride / y_stride
    int chain_units = 0;           // fused chains in the forward list (each is one kernel forward, one backward)
    int chain_nodes = 0;           // nodes inside them
    uint64_t ws_bytes = 0;
    std::vector<Launch> fwd, bwd;
    std::vector<WeightJob> wjobs;  // collected while lowering; batch_weight_jobs turns them into launches
    std::vector<ReduceJob> rjobs;  // likewise; batch_reduce_jobs
    std::vector<Launch> prep;  // inference plans only: the weight-only launches taken out of fwd
};

// Puts the collected weight jobs, of forward and backward alike, into one launch at the head of the forward
// list (backward runs on the weights and the workspace of the preceding forward).
void batch_weight_jobs(Lowering& low);

// Puts the collected sums of weight-gradient partials into one launch at the end of the backward list (every
// weight-gradient kernel owns its block of the workspace, so its partials stay intact until then).
void batch_reduce_jobs(Lowering& low);

// Turns a lowering into a forward-only plan: weight-only launches move to `prep`, the backward list is dropped.
void make_inference_plan(Lowering& low);

inline uint64_t align_up(uint64_t v, uint64_t a = 256) { return (v + a - 1) / a * a; }

// Lowering by units: fused chains of memory-bound primitives between the FC nodes (fuse_chains), one kernel per
// node for whatever no chain takes; fp32 tensors between units.  Handles every legal DAG.
std::unique_ptr<Lowering> lower_per_node(const Dag& dag, bool bf16, bool fuse_chains);

// Fused shift -> grouped FC -> unary chain -> (+ input); nullptr when the DAG is not of that form.
std::unique_ptr<Lowering> lower_sgfc(const Dag& dag, bool bf16);

// [Unfold] -> grouped FC -> [unary] -> Shift* -> add|mul with the input -> grouped FC, bf16 intermediates;
// nullptr when the DAG is not of that form.
std::unique_ptr<Lowering> lower_ufc(const Dag& dag, bool bf16);

// FC -> [softmax] -> broadcast-mul onto Unfold(x) -> Fold(sum|avg over taps) -> FC (per-pixel window weights);
// nullptr when the DAG is not of that form.
std::unique_ptr<Lowering> lower_dyn(const Dag& dag, bool bf16);

// Picks the lowering: fused kernel families where a pattern applies, else per node.
std::unique_ptr<Lowering> lower(const Dag& dag, bool bf16, bool no_fusion);

}  // namespace canvas
