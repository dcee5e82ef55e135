// Launcher of the fused-chain kernels (chain_isa.hpp): one launch runs one program.
#pragma once
#include <hip/hip_runtime.h>

#include "chain_isa.hpp"

namespace canvas {
namespace chain {

// Registers of the kernel instance with TM lanes (the planner must not use more).
constexpr int regs_for(int tm) { return tm <= 1 ? 8 : (tm <= 9 ? 6 : 3); }

// Largest workgroup of that instance (the tap vectors of a thread live in registers: wider lanes, fewer threads).
constexpr int max_threads_for(int tm) { return tm <= 1 ? 1024 : 512; }

// Bytes of LDS a launch of `pg` takes (persistent floats + the two hand-over buffers of OP_XADD).
inline size_t lds_bytes(const Program& pg) { return (size_t)(pg.n_persist + 2) * pg.threads * sizeof(float); }
constexpr size_t kMaxLdsBytes = 64 * 1024;

// Enqueues the program; every pointer of pg.ext must be set.  pg.tm must be 1, 9 or 25.
void run(const Program& pg, hipStream_t stream);

}  // namespace chain
}  // namespace canvas
