// Instruction set of the fused-chain kernels.
//
// A run of memory-bound primitives between FC nodes (Unfold consumed in place, Shift, element-wise, Broadcast with
// equal channel counts, Softmax over channels or taps, Folding over taps: Canvas paper, Section 5) is lowered to ONE
// forward and ONE backward kernel.  Both interpret a short program that the host planner (chain_plan.cpp) writes
// and that travels in the kernel arguments, so control flow is uniform over the whole workgroup.
//
// Machine model, per thread = `vec` consecutive pixels of one image plane (every lane below is `vec` floats wide):
//   A            accumulator, a vector over the taps (T <= TM lanes; lane 0 only for tensors without taps), in vector registers
//   R[0..n_regs) registers of the same shape (operands kept while another value is computed), in LDS: only A is live
//                across the interpreter's dispatch, so the compiler has no register state to shuffle between the cases
//   P[...]       persistent floats of the thread, in LDS: softmax statistics and sums that run across the channel
//                loop, gradient accumulators of an external tensor within one channel
// A program is a list of passes; a pass has a prologue (run once) and a body (run for every channel of the
// workgroup's channel range).  Stencils (Shift, Unfold) never move data between threads in the forward direction:
// the planner pushes their offsets down to the loads ("this value, but of the pixel at +offset"), which is why a
// stencil may only sit above element-wise work.  In the backward direction the gradient of a shifted load belongs
// to another pixel: XADD hands it over through LDS (a gather, fixed order, deterministic).
#pragma once
#include <cstddef>
#include <cstdint>

namespace canvas {
namespace chain {

constexpr int kMaxInstr = 184;
constexpr int kMaxTerms = 32;
constexpr int kMaxExt = 12;
constexpr int kMaxPass = 8;
constexpr int kMaxRed = 12;

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
    OP_BINLD,      // A = blend_kind(loaded, A) or (A, loaded): OP_LD and OP_BIN in one, the loaded operand never visits a register
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
// OP_BINLD: the two position flags of OP_LD, then
constexpr int kBinLdKindShift = 2;          // the blend kind, three bits
constexpr uint8_t kBinLdLoadedIsLhs = 0x20; // the loaded operand is the LHS (else A is)
constexpr uint8_t kBinLdLoadedScalar = 0x40;  // the loaded operand has one lane, replicated over A's T lanes
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
static_assert(sizeof(Ext) == 16, "tensor descriptor size");

struct Pass {
    uint16_t pro_begin = 0, pro_end = 0, body_begin = 0, body_end = 0;
    uint16_t red_begin = 0, red_end = 0;  // what the channel slices of a workgroup combine when the pass ends
    uint16_t pad[2] = {0, 0};
};

// A quantity that runs across the channel loop.  The channels of a workgroup are dealt out to `slices` groups of
// threads (slice s takes channels s, s + slices, ...), each with its own partial result in P; when the pass ends the
// partials of a pixel are combined and every slice gets the total.
struct Red {
    uint16_t slot = 0;
    uint8_t T = 1;
    uint8_t kind = 0;  // 0: softmax statistics (maximum at slot, rescaled sum at slot + T); 1: plain sums at slot
};

struct Program {
    // geometry.  A thread owns `vec` consecutive pixels of one image plane (H * W is a multiple of vec, vec <= W); the
    // plane is dealt out in tiles of `own_threads` such threads, and a workgroup computes `halo_threads` more on either
    // side of its tile (backward programs: the gradient hand-over of OP_XADD reads what neighbouring pixels computed).
    int32_t N = 0, C = 0, H = 0, W = 0;
    int32_t vec = 1;           // pixels per thread (1, 2, 4 or 8)
    int32_t own_threads = 0;   // pixel threads of a tile whose results are stored
    int32_t halo_threads = 0;  // recomputed pixel threads on either side
    int32_t tiles = 0;         // workgroups per image plane = ceil(H * W / vec / own_threads)
    int32_t chunk = 0;         // channels per workgroup
    int32_t chunks = 0;        // ceil(C / chunk)
    int32_t threads = 0;       // workgroup size = slices * pix_threads
    int32_t slices = 1;        // channel slices per workgroup
    int32_t pix_threads = 0;   // threads per slice: a multiple of 64, >= own_threads + 2 * halo_threads
    int32_t n_red = 0;
    int32_t n_persist = 0;     // floats of P per pixel
    int32_t xadd_lanes = 0;    // most lanes any OP_XADD hands over (0: the program has none)
    int32_t n_pass = 0, n_ext = 0, n_instr = 0, n_terms = 0;
    int32_t tm = 1;            // lanes the kernel instance must have (1, 9 or 25)
    int32_t fast_math = 0;     // 1: every tensor of the DAG is bf16, transcendental functions may be accurate to 1e-6 only
    int32_t n_regs = 0;        // registers R the program uses
    int32_t unroll = 1;        // channels a thread works on per trip through a pass's body (side by side, like wider lanes)
    Pass pass[kMaxPass];
    Red red[kMaxRed];
    Ext ext[kMaxExt];
    Term term[kMaxTerms];
    Instr ins[kMaxInstr];
};
static_assert(sizeof(Program) <= 3968, "the program must fit the kernel argument buffer");
static_assert(sizeof(Program) % 16 == 0 && sizeof(Instr) == 16 && offsetof(Program, ins) % 16 == 0,
              "the kernels copy the program in 16-byte pieces");

}  // namespace chain
}  // namespace canvas
