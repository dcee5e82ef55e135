// Pattern match and lowering for
//     x -> [Unfold] -> grouped FC -> [unary] -> Shift* -> binary(add|mul) with x -> [Fold over one tap]* -> grouped FC -> output
// (the shape of a sampled kernel that mixes a spatial aggregation with a gate on the block input; Canvas
// paper, Section 5 primitives and the sampled structures of Section 6).  All intermediates stay bf16:
//     forward   z = FC1(unfold x);  v = x (*|+) shift(act z);  y = FC2(v)
//     backward  dW2 = dy . v;  dv = FC2^T dy;  (dz, dx_direct) = adjoint of the middle;
//               dW1 = dz . unfold x;  dx = FC1^T dz (through the Unfold adjoint) + dx_direct
// Both contractions run on the MFMA grouped-FC kernels, the Unfold is never materialised.
#include <algorithm>
#include <functional>
#include <vector>

#include "fc_emit.hpp"
#include "gfc_kernels.hpp"
#include "lowering.hpp"
#include "ufc_kernels.hpp"

namespace canvas {

std::unique_ptr<Lowering> lower_ufc(const Dag& dag, bool bf16) {
    if (!bf16) return nullptr;
    const int n = (int)dag.nodes.size();
    for (int k = 0; k < n; k++)
        if (!dag.nodes[k].live || dag.nodes[k].pooled) return nullptr;  // (no tensor with folded spatial dims in this pattern)
    const int C = dag.nodes[0].C, Pn = dag.P();
    int k = 1, prev = 0;
    int KH = 1, KW = 1;
    if (k < n && dag.nodes[k].op == Op::Unfold) {
        const Node& u = dag.nodes[k];
        if (u.a != 0 || u.kh > 7 || u.kw > 7) return nullptr;
        KH = u.kh;
        KW = u.kw;
        prev = k++;
    }
    if (k >= n || dag.nodes[k].op != Op::Fc || dag.nodes[k].a != prev) return nullptr;
    const Node fc1 = dag.nodes[k];
    if (fc1.out != C) return nullptr;
    prev = k++;
    ufc::MidParams M;
    if (k < n && dag.nodes[k].op == Op::Unary) {
        const Node& u = dag.nodes[k];
        if (u.a != prev) return nullptr;
        // z is kept in bf16.  Rounding never changes a sign, so the decisions of relu and abs are those of the
        // unrounded z; the clip bounds of expclip sit at arbitrary values that rounding can cross, which
        // would flip gradients between exp(z) and 0: such DAGs take the per-node lowering (fp32 z).
        if (u.kind == kExpClip) return nullptr;
        M.act = u.kind;
        M.ulo = u.lo;
        M.uhi = u.hi;
        prev = k++;
    }
    std::vector<bool> shifted(C, false);
    while (k < n && dag.nodes[k].op == Op::Shift) {
        const Node& s = dag.nodes[k];
        if (s.a != prev || s.T != 1) return nullptr;
        if ((s.dh != 0 || s.dw != 0) && s.c1 > s.c0) {
            if (M.nslices == ufc::kMaxSlices) return nullptr;
            for (int c = s.c0; c < s.c1; c++) {
                if (shifted[c]) return nullptr;  // two zero-filling shifts of one channel do not compose into one
                shifted[c] = true;
            }
            M.c0[M.nslices] = s.c0;
            M.c1[M.nslices] = s.c1;
            M.dh[M.nslices] = s.dh;
            M.dw[M.nslices] = s.dw;
            M.nslices++;
        }
        prev = k++;
    }
    if (k >= n || dag.nodes[k].op != Op::Binary) return nullptr;
    {
        const Node& b = dag.nodes[k];
        const bool with_input = (b.a == 0 && b.b == prev) || (b.a == prev && b.b == 0);
        if (!with_input || prev == 0 || (b.kind != kAdd && b.kind != kMul) || b.C != C || b.T != 1) return nullptr;
        M.bin = b.kind == kMul ? 1 : 0;
        prev = k++;
    }
    while (k < n && dag.nodes[k].op == Op::Fold && !dag.nodes[k].axis_c && !dag.nodes[k].axis_hw && dag.nodes[dag.nodes[k].a].T == 1) {  // a fold over one tap is the identity
        if (dag.nodes[k].a != prev) return nullptr;
        prev = k++;
    }
    if (k >= n || dag.nodes[k].op != Op::Fc || dag.nodes[k].a != prev) return nullptr;
    const Node fc2 = dag.nodes[k];
    prev = k++;
    if (k != n || dag.out != prev) return nullptr;
    // the input may feed only the head of the chain and the binary node
    int uses = 0;
    for (int j = 1; j < n; j++) uses += (dag.nodes[j].a == 0) + (dag.nodes[j].b == 0 && dag.nodes[j].op == Op::Binary);
    if (uses != 2) return nullptr;
    // 32-bit byte offsets through buffer descriptors
    const int O2 = fc2.out;
    if ((int64_t)dag.N * std::max(C, O2) * Pn * 2 >= ((int64_t)1 << 31) || dag.W < 4 || (int64_t)dag.N * Pn >= ((int64_t)1 << 28)) return nullptr;

    const int G1 = fc1.groups, G2 = fc2.groups;
    const int K1 = (C / G1) * KH * KW, K2 = C / G2;
    M.N = dag.N;
    M.C = C;
    M.H = dag.H;
    M.W = dag.W;
    M.P = Pn;
    M.upi = (Pn + 7) / 8;
    M.magicW = gfc::magic_u32(dag.W);
    M.magicUpi = gfc::magic_u32(M.upi);
    if ((int64_t)dag.N * C * M.upi >= ((int64_t)1 << 31)) return nullptr;

    auto low = std::make_unique<Lowering>();
    low->fused = true;
    const int64_t nw1 = (int64_t)C * K1, nw2 = (int64_t)O2 * K2;
    const double act = 2.0 * dag.numel(0), outb = 2.0 * dag.numel(dag.out);
    uint64_t off = 0;
    auto take = [&](uint64_t bytes) {
        const uint64_t o = off;
        off += align_up(bytes);
        return (int64_t)o;
    };
    const int64_t oz = take((uint64_t)act), ov = take((uint64_t)act), odv = take((uint64_t)act), odz = take((uint64_t)act);
    const int w1 = fc1.widx, w2 = fc2.widx;
    const double fl1 = 2.0 * dag.N * Pn * (double)C * K1, fl2 = 2.0 * dag.N * Pn * (double)O2 * K2;

    const int TV = KH * KW;
    const TakeFn takef = take;
    const FcOperand in_x{[](const RunArgs& a) { return a.x; }, false};
    const FcOperand in_dy{[](const RunArgs& a) { return a.dy; }, false};
    auto ws_at = [](int64_t o) { return [=](const RunArgs& a) { return (const void*)(a.ws + o); }; };
    emit_fc(*low, false, dag, takef, TV > 1 ? "ufc_fc1_unfold" : "ufc_fc1", G1, C / G1, KH, KW, C / G1, false, w1, in_x, ws_at(oz), false,
            2.0 * act + 2.0 * nw1, fl1);
    low->fwd.push_back({"ufc_mid_fwd", 3.0 * act, 0, [=](const RunArgs& a) {
                            ufc::MidParams R = M;
                            R.x = (const uint16_t*)a.x;
                            R.z = (const uint16_t*)(a.ws + oz);
                            R.v = (uint16_t*)(a.ws + ov);
                            ufc::mid_forward(R, a.stream);
                        }});
    emit_fc(*low, false, dag, takef, "ufc_fc2", G2, C / G2, 1, 1, O2 / G2, false, w2, FcOperand{ws_at(ov), false},
            [](const RunArgs& a) { return (const void*)a.y; }, false, act + outb + 2.0 * nw2, fl2);

    // backward (forward must have run with the same workspace: z and v are read back, and left intact)
    emit_wgrad(*low, dag, takef, "ufc_fc2_wgrad", G2, C / G2, 1, 1, O2 / G2, w2, FcOperand{ws_at(ov), false}, in_dy, act + outb, fl2);
    emit_fc(*low, true, dag, takef, "ufc_fc2_dgrad", G2, O2 / G2, 1, 1, C / G2, true, w2, in_dy, ws_at(odv), false, act + outb + 2.0 * nw2, fl2);
    low->bwd.push_back({"ufc_mid_bwd", (M.bin ? 5.0 : 4.0) * act, 0, [=](const RunArgs& a) {
                            ufc::MidParams R = M;
                            R.x = (const uint16_t*)a.x;
                            R.z = (const uint16_t*)(a.ws + oz);
                            R.dv = (const uint16_t*)(a.ws + odv);
                            R.dz = (uint16_t*)(a.ws + odz);
                            R.dx1 = (uint16_t*)a.dx;  // completed by the data gradient of FC1 below
                            ufc::mid_backward(R, a.stream);
                        }});
    emit_wgrad(*low, dag, takef, TV > 1 ? "ufc_fc1_wgrad_unfold" : "ufc_fc1_wgrad", G1, C / G1, KH, KW, C / G1, w1, in_x,
               FcOperand{ws_at(odz), false}, 2.0 * act, fl1);
    // mid_backward left dx_direct in dx; the data gradient of FC1 (through the Unfold adjoint) adds to it
    emit_fc(*low, true, dag, takef, TV > 1 ? "ufc_fc1_dgrad_unfold" : "ufc_fc1_dgrad", G1, C / G1, KH, KW, C / G1, true, w1,
            FcOperand{ws_at(odz), false}, [](const RunArgs& a) { return (const void*)a.dx; }, true, 3.0 * act + 2.0 * nw1, fl1);
    low->ws_bytes = off;
    return low;
}

}  // namespace canvas
