// Planner of the fused-chain kernels: turns a set of non-FC nodes of a micro-DAG into one forward and one backward
// program of the instruction set in chain_isa.hpp.  Host only.
#pragma once
#include <string>
#include <vector>

#include "chain_isa.hpp"
#include "dag.hpp"

namespace canvas {
namespace chain {

// What an external tensor of a program is, in terms of the DAG.
enum ExtRole : int {
    kValueIn = 0,   // value of a node outside the unit (read)
    kValueOut,      // value of a node of the unit that something outside consumes (written)
    kGradIn,        // gradient of such an output node (read)
    kGradOut        // gradient of an external input (written; the lowering decides between = and +=)
};

struct ExtRef {
    int node = -1;
    ExtRole role = kValueIn;
    int store_instr = -1;  // kGradOut / kValueOut: index of the OP_ST that writes it
};

struct UnitPlan {
    std::vector<int> nodes;     // the unit, ascending
    std::vector<int> inputs;    // external nodes it reads, ascending
    std::vector<int> outputs;   // nodes of the unit that are stored, ascending
    Program fwd, bwd;
    std::vector<ExtRef> fwd_ext, bwd_ext;  // one per ext slot of the program
    double cost = 0;            // estimated work of both programs per pixel and channel (see program_cost)
};

// True when node k can be part of a fused chain at all (op, shapes, attributes).
bool chain_candidate(const Dag& dag, int k);

// Compiles the unit `nodes` (ascending node ids, all chain candidates).  `is_output(k)`: node k of the unit must be
// stored (it is the DAG's output or something outside the unit reads it).  Returns false (and says why) when the
// unit does not fit the machine: a stencil above a reduction, too many instructions, registers, passes, LDS ...
bool compile_unit(const Dag& dag, const std::vector<int>& nodes, const std::vector<bool>& is_output, UnitPlan& out, std::string& why);

// Estimated work of a program per pixel and channel of the unit, in units of one cheap lane operation: a lane of a
// tensor access counts 4, of a gradient hand-over 6, of a transcendental function 6; the whole is scaled by the pixels a
// workgroup computes per pixel it owns (the halo of backward programs) and by the length of a thread's serial walk over
// the channels beyond 16 trips.  The lowering lets a node join a chain only
// while the grown chain is not much dearer than the two chains apart.
double program_cost(const Program& pg);

// Text form of a program (for CANVAS_LOG and debugging).
std::string dump(const Program& pg);

}  // namespace chain
}  // namespace canvas
