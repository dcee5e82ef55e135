// Per-thread execution of the fused-chain instruction set (see chain_isa.hpp).  Everything here is plain
// per-pixel arithmetic on the thread's own state; the one instruction that moves data between threads (OP_XADD)
// is driven by the kernel around two helpers of this file.  Primitive definitions: Canvas paper, Section 5;
// subgradient choices: relu'(0) = 0, sign(0) = 0, clipped exp flat outside the open interval, first maximum
// of a max fold, ties of min / max to the LHS.
#pragma once
#include <cmath>
#include <cstdint>
#include <cstring>

#include "chain_isa.hpp"

#if defined(__HIPCC__)
#define CHAIN_HD __host__ __device__ __forceinline__
#else
#define CHAIN_HD inline
#endif

namespace canvas {
namespace chain {

template <int TM, int NR>
struct State {
    float A[TM];
    float R[NR][TM];
};

// What a thread knows about its pixel.  Threads of the halo rows may sit outside the image (row < 0 or >= H);
// threads beyond the workgroup's rows have active == false.  Only `own` pixels are stored.
struct Thread {
    int tid = 0, n = 0, row = 0, col = 0;
    bool active = false, own = false;
};

CHAIN_HD float vm_bf16_to_f32(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

CHAIN_HD uint16_t vm_f32_to_bf16(float f) {  // round to nearest even; NaN stays NaN
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

CHAIN_HD float vm_unary(int kind, float x, float lo, float hi) {
    switch (kind) {
    case 0: return fmaxf(x, 0.f);
    case 1: return fabsf(x);
    case 2: return 0.5f * x * (1.f + erff(x * 0.70710678118654752f));
    case 4: return sinf(x);
    case kUnNeg: return -x;
    default: return expf(fminf(fmaxf(x, lo), hi));
    }
}

CHAIN_HD float vm_unary_grad(int kind, float x, float lo, float hi) {
    switch (kind) {
    case 0: return x > 0.f ? 1.f : 0.f;
    case 1: return x > 0.f ? 1.f : (x < 0.f ? -1.f : 0.f);
    case 2: return 0.5f * (1.f + erff(x * 0.70710678118654752f)) + x * 0.39894228040143268f * expf(-0.5f * x * x);
    case 4: return cosf(x);
    case kUnNeg: return -1.f;
    default: return (x > lo && x < hi) ? expf(x) : 0.f;
    }
}

CHAIN_HD float vm_blend(int kind, float a, float b) {
    switch (kind) {
    case 0: return a + b;
    case 1: return a * b;
    case 2: return a - b;
    case 3: return a <= b ? a : b;
    default: return a >= b ? a : b;
    }
}

CHAIN_HD float vm_blend_grad(int kind, bool rhs_side, float a, float b) {
    switch (kind) {
    case 0: return 1.f;
    case 1: return rhs_side ? a : b;
    case 2: return rhs_side ? -1.f : 1.f;
    case 3: return (a <= b) != rhs_side ? 1.f : 0.f;
    default: return (a >= b) != rhs_side ? 1.f : 0.f;
    }
}

// Sum of the offsets of a position for channel c: terms [b >> 8, (b >> 8) + (b & 255)) that cover c.
CHAIN_HD void vm_offset(const Program& pg, uint16_t b, int c, int& dh, int& dw) {
    dh = 0;
    dw = 0;
    const int first = b >> 8, cnt = b & 255;
    for (int k = 0; k < cnt; k++) {
        const Term& t = pg.term[first + k];
        if (c >= (int)t.c0 && c < (int)t.c1) {
            dh += t.dh;
            dw += t.dw;
        }
    }
}

#if defined(CHAIN_VM_BOUNDS)  // host builds of the interpreter only: every access checked against the tensor's size
#include <cstdio>
#include <cstdlib>
#define CHAIN_VM_CHECK(pg, e, idx)                                                                            \
    do {                                                                                                      \
        if ((idx) < 0 || (idx) >= (int64_t)(pg).N * (pg).C * (e).T * (pg).H * (pg).W) {                       \
            std::fprintf(stderr, "chain vm: index %lld outside a tensor of %d taps\n", (long long)(idx), (int)(e).T); \
            std::abort();                                                                                     \
        }                                                                                                     \
    } while (0)
#else
#define CHAIN_VM_CHECK(pg, e, idx) ((void)0)
#endif

CHAIN_HD float vm_load(const Program& pg, const Ext& e, int64_t idx) {
    CHAIN_VM_CHECK(pg, e, idx);
    return e.bf16 ? vm_bf16_to_f32(((const uint16_t*)e.ptr)[idx]) : ((const float*)e.ptr)[idx];
}

#define CHAIN_LANES(T) _Pragma("unroll") for (int t = 0; t < TM; t++) if (t < (T))

// Runs `body` with X bound to register r (r is uniform: one branch, no dynamic register indexing).
#define CHAIN_WITH_REG(st, r, X, ...)                                    \
    do {                                                                 \
        _Pragma("unroll") for (int rr_ = 0; rr_ < NR; rr_++) if (rr_ == (int)(r)) { \
            float* X = (st).R[rr_];                                      \
            __VA_ARGS__                                                  \
        }                                                                \
    } while (0)

// Every instruction except OP_XADD.  Pm: this thread's persistent floats, element k at Pm[k * pstride].
template <int TM, int NR>
CHAIN_HD void vm_exec(const Program& pg, const Instr& I, int c, const Thread& th, State<TM, NR>& st, float* Pm, int pstride) {
    float* A = st.A;
    const int T = I.T;
    const int H = pg.H, W = pg.W;
    switch (I.op) {
    case OP_LD: {
        int dh, dw;
        vm_offset(pg, I.b, c, dh, dw);
        const Ext& e = pg.ext[I.a];
        const int64_t plane = (int64_t)H * W;
        const int64_t base = ((int64_t)th.n * pg.C + c) * e.T;
        if (I.kind & kWin) {
            const int KH = I.r >> 4, KW = I.r & 15;
            CHAIN_LANES(T) {
                const int hh = th.row + dh + t / KW - KH / 2, ww = th.col + dw + t % KW - KW / 2;
                const bool in = th.active && hh >= 0 && hh < H && ww >= 0 && ww < W;
                A[t] = in ? vm_load(pg, e, base * plane + (int64_t)hh * W + ww) : 0.f;
            }
        } else {
            const int hh = th.row + dh, ww = th.col + dw;
            const bool in = th.active && hh >= 0 && hh < H && ww >= 0 && ww < W;
            const int64_t pix = (int64_t)hh * W + ww;
            CHAIN_LANES(T) {
                const int te = (I.kind & kExtTaps) ? (t < e.T ? t : t % e.T) : 0;
                A[t] = in ? vm_load(pg, e, (base + te) * plane + pix) : 0.f;
            }
        }
        break;
    }
    case OP_MASK: {
        int dh, dw;
        vm_offset(pg, I.b, c, dh, dw);
        if (I.kind & kWin) {
            const int KH = I.r >> 4, KW = I.r & 15;
            CHAIN_LANES(T) {
                const int hh = th.row + dh + t / KW - KH / 2, ww = th.col + dw + t % KW - KW / 2;
                if (!(hh >= 0 && hh < H && ww >= 0 && ww < W)) A[t] = 0.f;
            }
        } else {
            const int hh = th.row + dh, ww = th.col + dw;
            if (!(hh >= 0 && hh < H && ww >= 0 && ww < W)) CHAIN_LANES(T) A[t] = 0.f;
        }
        break;
    }
    case OP_UN:
        CHAIN_LANES(T) A[t] = vm_unary(I.kind, A[t], I.f0, I.f1);
        break;
    case OP_MOVR:
        CHAIN_WITH_REG(st, I.r, X, CHAIN_LANES(T) X[t] = A[t];);
        break;
    case OP_MOVA:
        CHAIN_WITH_REG(st, I.r, X, CHAIN_LANES(T) A[t] = X[t];);
        break;
    case OP_BIN: {
        const int kind = I.kind & 7;
        const bool reg_lhs = I.kind & kBinRegIsLhs, reg_sc = I.kind & kBinRegScalar, acc_sc = I.kind & kBinAccScalar;
        const float a0 = A[0];
        CHAIN_WITH_REG(st, I.r, X, CHAIN_LANES(T) {
            const float rv = reg_sc ? X[0] : X[t], av = acc_sc ? a0 : A[t];
            A[t] = reg_lhs ? vm_blend(kind, rv, av) : vm_blend(kind, av, rv);
        });
        break;
    }
    case OP_FOLD: {
        float s = A[0];
        _Pragma("unroll") for (int t = 1; t < TM; t++) if (t < T) {
            if (I.kind == 2) s = A[t] > s ? A[t] : s;
            else s += A[t];
        }
        if (I.kind == 1) s /= (float)T;
        A[0] = s;
        break;
    }
    case OP_SMT: {
        float m = A[0];
        _Pragma("unroll") for (int t = 1; t < TM; t++) if (t < T) m = fmaxf(m, A[t]);
        float z = 0.f;
        CHAIN_LANES(T) {
            A[t] = expf(A[t] - m);
            z += A[t];
        }
        CHAIN_LANES(T) A[t] = A[t] / z;
        break;
    }
    case OP_ST: {
        if (!th.own) break;
        const Ext& e = pg.ext[I.a];
        const int64_t plane = (int64_t)H * W;
        const int64_t base = ((int64_t)th.n * pg.C + c) * e.T;
        const int64_t pix = (int64_t)th.row * W + th.col;
        CHAIN_LANES(T) {
            const int64_t idx = (base + t) * plane + pix;
            CHAIN_VM_CHECK(pg, e, idx);
            if (e.bf16) ((uint16_t*)e.ptr)[idx] = vm_f32_to_bf16(A[t]);
            else if (I.kind & kStAdd) ((float*)e.ptr)[idx] += A[t];
            else ((float*)e.ptr)[idx] = A[t];
        }
        break;
    }
    case OP_UNBX:
        CHAIN_WITH_REG(st, I.r, X, CHAIN_LANES(T) A[t] = X[t] * vm_unary_grad(I.kind, A[t], I.f0, I.f1););
        break;
    case OP_BING: {
        const int kind = I.kind & 7;
        const bool rhs_side = I.kind & kBingRhsSide, l_sc = I.kind & kBingLhsScalar, r_sc = I.kind & kBingRhsScalar;
        const float a0 = A[0];
        CHAIN_WITH_REG(st, I.r, X, CHAIN_LANES(T) A[t] = vm_blend_grad(kind, rhs_side, l_sc ? X[0] : X[t], r_sc ? a0 : A[t]););
        break;
    }
    case OP_SMTBX:
        CHAIN_WITH_REG(st, I.r, X, {
            float dot = 0.f;
            CHAIN_LANES(T) dot += X[t] * A[t];
            CHAIN_LANES(T) A[t] = A[t] * (X[t] - dot);
        });
        break;
    case OP_FOLDBX:
        CHAIN_WITH_REG(st, I.r, X, {
            const float g = X[0];
            if (I.kind == 2) {
                int best = 0;
                float m = A[0];
                _Pragma("unroll") for (int t = 1; t < TM; t++) if (t < T && A[t] > m) {
                    m = A[t];
                    best = t;
                }
                CHAIN_LANES(T) A[t] = t == best ? g : 0.f;
            } else {
                const float v = I.kind == 1 ? g / (float)T : g;
                CHAIN_LANES(T) A[t] = v;
            }
        });
        break;
    case OP_PSET:
        CHAIN_LANES(T) Pm[(I.a + t) * pstride] = I.f0;
        break;
    case OP_PADD:
        CHAIN_LANES(T) Pm[(I.a + (t < (int)I.b ? t : t % (int)I.b)) * pstride] += A[t];
        break;
    case OP_PLD:
        CHAIN_LANES(T) A[t] = Pm[(I.a + t) * pstride];
        break;
    case OP_SMCSTAT:
        CHAIN_LANES(T) {
            float& m = Pm[(I.a + t) * pstride];
            float& z = Pm[(I.a + T + t) * pstride];
            const float v = A[t];
            if (v > m) {
                z = z * expf(m - v) + 1.f;  // (m = -inf at the first channel: z = 0 * 0 + 1)
                m = v;
            } else {
                z += expf(v - m);
            }
        }
        break;
    case OP_SMCAPPLY:
        CHAIN_LANES(T) A[t] = expf(A[t] - Pm[(I.a + t) * pstride]) / Pm[(I.a + T + t) * pstride];
        break;
    case OP_SMCDOT:
        CHAIN_WITH_REG(st, I.r, X, CHAIN_LANES(T) Pm[(I.a + t) * pstride] += A[t] * X[t];);
        break;
    case OP_SMCBX:
        CHAIN_WITH_REG(st, I.r, X, CHAIN_LANES(T) A[t] = A[t] * (X[t] - Pm[(I.a + t) * pstride]););
        break;
    default: break;
    }
}

// OP_XADD, lane t: the thread index (inside the workgroup) whose load at offset [+ window tap t] read this
// thread's pixel, or -1 when there is none (outside the image, or outside the rows the workgroup computes: the
// planner sizes the halo so that this never happens to a pixel the workgroup owns).
CHAIN_HD int vm_xadd_source(const Program& pg, const Instr& I, int dh, int dw, int t, const Thread& th, int row_first, int rows) {
    int oh = dh, ow = dw;
    if (I.kind & kWin) {
        const int KH = I.r >> 4, KW = I.r & 15;
        oh += t / KW - KH / 2;
        ow += t % KW - KW / 2;
    }
    const int sr = th.row - oh, sc = th.col - ow;
    if (!th.active || sc < 0 || sc >= pg.W || sr < 0 || sr >= pg.H || sr < row_first || sr >= row_first + rows) return -1;
    return (sr - row_first) * pg.W + sc;
}

}  // namespace chain
}  // namespace canvas
