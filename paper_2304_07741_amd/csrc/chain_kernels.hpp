// Launcher of the fused-chain kernels (chain_isa.hpp): one launch runs one program.
#pragma once
#include <hip/hip_runtime.h>

#include "chain_isa.hpp"

namespace canvas {
namespace chain {

// Registers of the kernel instance with TM lanes (the planner must not use more).
constexpr int regs_for(int tm) { return tm <= 1 ? 10 : (tm <= 9 ? 6 : 4); }

// Pixels per thread the instances with TM lanes exist for: 16 ... 1 without taps, 4, 2 or 1 up to 9 taps, 1 beyond.
constexpr int max_vec_for(int tm) { return tm <= 1 ? 16 : (tm <= 9 ? 4 : 1); }

// Largest workgroup of that instance (the tap vectors of a thread live in registers: wider lanes, fewer threads).
constexpr int max_threads_for(int) { return 512; }
// Wavefronts per SIMD that the register allocation of an instance leaves room for (1: no requirement).  The instance with
// 9 lanes x 2 pixels came out one register above the 128 of four wavefronts; held to them it spills nothing.
constexpr int min_waves_for(int tm, int vec) { return tm > 1 && tm <= 9 && vec == 2 ? 4 : 1; }

// Channels per trip of the instance with TM lanes and `vec` pixels per thread: 16 lanes in all without taps (so that a
// thread with few pixels still has 16 independent loads in flight), 2 x 9 lanes up to 9 taps, one channel beyond.
constexpr int unroll_for(int tm, int vec) { return tm <= 1 ? 16 / vec : (tm <= 9 && vec == 1 ? 2 : 1); }

// 16-byte pieces of a register of the instance with `tm` lanes and `vec` pixels per thread (all its channels' lanes).
constexpr int reg_pieces_of(int tm, int vec) { return ((tm <= 1 ? 1 : (tm <= 9 ? 9 : 25)) * vec * unroll_for(tm, vec) + 3) / 4; }

// Bytes of LDS a thread of `pg` takes: its registers, its share of the hand-over buffer of OP_XADD, its persistent floats.
inline size_t lds_bytes_per_thread(const Program& pg) {
    return ((size_t)pg.n_regs * reg_pieces_of(pg.tm, pg.vec) * 4 + (size_t)(pg.xadd_lanes + pg.n_persist * pg.unroll) * pg.vec) * sizeof(float);
}
inline size_t lds_bytes(const Program& pg) { return lds_bytes_per_thread(pg) * pg.threads; }
constexpr size_t kMaxLdsBytes = 144 * 1024;  // of the 160 KB of a compute unit (the kernel keeps its copy of the program in LDS as well)

// Enqueues the program; every pointer of pg.ext must be set.  pg.tm must be 1, 9 or 25, pg.vec one of max_vec_for's.
void run(const Program& pg, hipStream_t stream);

}  // namespace chain
}  // namespace canvas
