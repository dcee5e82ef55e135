// Instruction set of the fused-chain kernels.
//
// A run of memory-bound primitives between FC nodes (Unfold consumed in place, Shift, element-wise, Broadcast with
// equal channel counts, Softmax over channels or taps, Folding over taps: Canvas paper, Section 5) is lowered to ONE
// forward and ONE backward kernel.  Both interpret a short program that the host planner (chain_plan.cpp) writes
// and that travels in the kernel arguments, so control flow is uniform over the whole workgroup.
//
// Machine model, per thread = per pixel of one image:
//   A            accumulator, a vector over the taps (T <= TM lanes; lane 0 only for tensors without taps)
//   R[0..NR)     registers of the same shape (operands kept while another value is computed)
//   P[...]       persistent floats of the thread, in LDS: softmax statistics and sums that run across the channel
//                loop, gradient accumulators of an external tensor within one channel
// A program is a list of passes; a pass has a prologue (run once) and a body (run for every channel of the
// workgroup's channel range).  Stencils (Shift, Unfold) never move data between threads in the forward direction:
// the planner pushes their offsets down to the loads ("this value, but of the pixel at +offset"), which is why a
// stencil may only sit above element-wise work.  In the backward direction the gradient of a shifted load belongs
// to another pixel: XADD hands it over through LDS (a gather, fixed order, deterministic).
#pragma once
#include <cstdint>

namespace canvas {
namespace chain {

constexpr int kMaxInstr = 192;
constexpr int kMaxTerms = 32;
constexpr int kMaxExt = 12;
constexpr int kMaxPass = 8;

enum Opcode : uint8_t {
    OP_LD = 0,     // A[t] = ext[a](channel, tap, pixel + offset(b) [+ window tap t]) or 0 outside the image
    OP_MASK,       // A[t] = 0 where pixel + offset(b) [+ window tap t] is outside the image
    OP_UN,         // A = unary_kind(A)
    OP_MOVR,       // R[r] = A
    OP_MOVA,       // A = R[r]
    OP_BIN,        // A = blend_kind(lhs, rhs) of A and R[r] (flags say which is which and who is a scalar)
    OP_FOLD,       // A[0] = sum | avg | max over A[0..T)
    OP_SMT,        // A = softmax over the lanes
    OP_ST,         // ext[a](channel, t, pixel) = A[t] (flag: +=) for pixels the workgroup owns
    OP_UNBX,       // A = R[r] * unary_kind'(A)                         (A: the unary's input, R[r]: gradient)
    OP_BING,       // A = d blend_kind(L, A) / d side, L = R[r]         (A: RHS value, R[r]: LHS value; T lanes)
    OP_SMTBX,      // A = A * (R[r] - sum_s R[r][s] * A[s])             (A: softmax output, R[r]: gradient)
    OP_FOLDBX,     // A[t] = gradient of the fold's input: R[r][0] spread (sum), / T (avg), to the first maximum of A (max)
    OP_PSET,       // P[a + t] = f0
    OP_PADD,       // P[a + t % b] += A[t]
    OP_PLD,        // A[t] = P[a + t]
    OP_SMCSTAT,    // running maximum P[a + t] and rescaled sum P[a + T + t] of exp(A[t] - maximum) over the channel loop
    OP_SMCAPPLY,   // A[t] = exp(A[t] - P[a + t]) / P[a + T + t]
    OP_SMCDOT,     // P[a + t] += A[t] * R[r][t]
    OP_SMCBX,      // A[t] = A[t] * (R[r][t] - P[a + t])                (A: softmax output, R[r]: gradient)
    OP_XADD,       // P[a (+ t)] += A[t] of the thread whose load at offset(b) [+ window tap t] read THIS pixel
    OP_COUNT
};

// OP_BIN flags (in `kind`, above the 3 bits of the blend kind)
constexpr uint8_t kBinRegIsLhs = 0x08;     // R[r] is the LHS (else A is)
constexpr uint8_t kBinRegScalar = 0x10;    // R[r] has one lane, replicated
constexpr uint8_t kBinAccScalar = 0x20;    // A has one lane, replicated (the result has T lanes)
// OP_BING flags
constexpr uint8_t kBingRhsSide = 0x08;     // derivative with respect to the RHS (else the LHS)
constexpr uint8_t kBingLhsScalar = 0x10;   // R[r] has one lane
constexpr uint8_t kBingRhsScalar = 0x20;   // A has one lane
// OP_LD / OP_MASK / OP_XADD flags (in `kind`)
constexpr uint8_t kWin = 0x01;             // a window level is part of the position: r = (KH << 4) | KW, lane t is tap t
constexpr uint8_t kExtTaps = 0x02;         // the external tensor has taps of its own: lane t reads tap t % T_ext
// OP_ST flags
constexpr uint8_t kStAdd = 0x01;
// extra unary kind for the planner (after the five of the DAG): negation
constexpr uint8_t kUnNeg = 16;

struct Instr {
    uint8_t op = 0, kind = 0, T = 1, r = 0;
    uint16_t a = 0, b = 0;   // b of position-dependent instructions: (first term << 8) | number of terms
    float f0 = 0.f, f1 = 0.f;
};
static_assert(sizeof(Instr) == 16, "instruction size");

// One offset of a position: applies to channels [c0, c1) only (a Shift of a channel slice).
struct Term {
    int16_t dh = 0, dw = 0;
    uint16_t c0 = 0, c1 = 0;
};

struct Ext {
    void* ptr = nullptr;   // device pointer, filled at launch
    int32_t T = 1;         // taps of the tensor (its channel count is the program's C)
    int32_t bf16 = 0;      // element type: 1 = bf16, 0 = fp32
};

struct Pass {
    uint16_t pro_begin = 0, pro_end = 0, body_begin = 0, body_end = 0;
};

struct Program {
    // geometry
    int32_t N = 0, C = 0, H = 0, W = 0;
    int32_t tile_rows = 0;     // image rows a workgroup owns
    int32_t halo_rows = 0;     // rows above and below that it recomputes for the gradient hand-over
    int32_t tiles = 0;         // workgroups per image plane = ceil(H / tile_rows)
    int32_t chunk = 0;         // channels per workgroup
    int32_t chunks = 0;        // ceil(C / chunk)
    int32_t threads = 0;       // workgroup size (a multiple of 64, >= (tile_rows + 2 * halo_rows) * W)
    int32_t n_persist = 0;     // floats of P per thread
    int32_t n_pass = 0, n_ext = 0, n_instr = 0, n_terms = 0;
    int32_t tm = 1;            // lanes the kernel instance must have (1, 9 or 25)
    Pass pass[kMaxPass];
    Ext ext[kMaxExt];
    Term term[kMaxTerms];
    Instr ins[kMaxInstr];
};
static_assert(sizeof(Program) <= 3968, "the program must fit the kernel argument buffer");

}  // namespace chain
}  // namespace canvas
