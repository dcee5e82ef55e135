// Pattern match and lowering for per-pixel window weights (the Involution form of the Canvas paper, Section 5):
//     l = FC1(x) [TV channels];  a = softmax_C(l) (optional);  U = Unfold(x) [C, TV];
//     m = a (broadcast-mul) U;  u = Fold_{sum|avg over taps}(m);  y = FC2(u)
// with TV = KH*KW, so that the broadcast pairs channel t of a with tap t of U.  With a Group view [G, C/G] on x
// (and hence on l, a and U) the blend runs inside each group: l has G*TV channels and channel g*TV + t meets
// tap t of the channels of group g; (image, group) pairs are then independent, and the kernels see N*G
// "images" of C/G channels.  The unfolded tensor and the product m are never materialised:
//     forward   l (fp32), a (fp32), u (bf16) -> y
//     backward  dW2 = dy . u;  du = FC2^T dy;  dx = dyn^T(a, du) and da = sum_c du . U (one launch);  dl = softmax'(a, da);
//               dW1 = dl . x;  dx += FC1^T dl
#include <algorithm>

#include "dyn_kernels.hpp"
#include "fc_emit.hpp"
#include "lowering.hpp"
#include "ref_kernels.hpp"

namespace canvas {

std::unique_ptr<Lowering> lower_dyn(const Dag& dag, bool bf16) {
    if (!bf16) return nullptr;
    const int n = (int)dag.nodes.size();
    for (int k = 0; k < n; k++)
        if (!dag.nodes[k].live || dag.nodes[k].pooled) return nullptr;  // (no tensor with folded spatial dims in this pattern)
    // the nodes in any valid order: exactly one of each kind (softmax optional)
    int ifc1 = -1, isoft = -1, iunf = -1, ibin = -1, ifold = -1, ifc2 = -1;
    for (int k = 1; k < n; k++) {
        const Node& nd = dag.nodes[k];
        int* slot = nullptr;
        switch (nd.op) {
        case Op::Fc: slot = nd.a == 0 ? &ifc1 : &ifc2; break;
        case Op::Softmax: slot = &isoft; break;
        case Op::Unfold: slot = &iunf; break;
        case Op::Binary: slot = &ibin; break;
        case Op::Fold: slot = &ifold; break;
        default: return nullptr;
        }
        if (*slot >= 0) return nullptr;
        *slot = k;
    }
    if (ifc1 < 0 || iunf < 0 || ibin < 0 || ifold < 0 || ifc2 < 0) return nullptr;
    const Node &fc1 = dag.nodes[ifc1], &unf = dag.nodes[iunf], &bin = dag.nodes[ibin], &fold = dag.nodes[ifold], &fc2 = dag.nodes[ifc2];
    const int C = dag.nodes[0].C, TV = unf.kh * unf.kw, Pn = dag.P();
    if (dag.nodes[0].T != 1 || unf.a != 0 || !dyn::supported(unf.kh, unf.kw)) return nullptr;
    const int Gb = bin.bgroups, TVa = Gb * TV;  // groups of the blend, channels of l and a
    if (fc1.a != 0 || fc1.out != TVa || C % Gb || (Gb > 1 && fc1.groups != Gb)) return nullptr;
    int alast = ifc1;
    if (isoft >= 0) {
        const Node& sm = dag.nodes[isoft];
        if (sm.a != ifc1 || sm.kind != kAxisC) return nullptr;
        alast = isoft;
    }
    // LHS [TV, 1] onto RHS [C, TV]: with C != TV the broadcast index (c*TV + t) % TV = t pairs channel t with tap t
    // (inside each group when Gb > 1: C/Gb channels)
    if (bin.kind != kMul || bin.a != alast || bin.b != iunf || C / Gb == TV) return nullptr;
    if (fold.a != ibin || fold.axis_c || fold.axis_hw || (fold.kind != kSum && fold.kind != kAvg)) return nullptr;
    if (fc2.a != ifold || dag.out != ifc2) return nullptr;
    // every intermediate has exactly the one consumer of the pattern
    for (int k = 1; k < n; k++) {
        const Node& nd = dag.nodes[k];
        auto uses = [&](int v) { return (nd.a == v) + (nd.op == Op::Binary && nd.b == v); };
        if (k != isoft && k != ibin && uses(ifc1)) return nullptr;
        if (isoft >= 0 && k != ibin && uses(isoft)) return nullptr;
        if (k != ibin && uses(iunf)) return nullptr;
        if (k != ifold && uses(ibin)) return nullptr;
        if (k != ifc2 && uses(ifold)) return nullptr;
        if (k != ifc1 && k != iunf && uses(0)) return nullptr;
    }
    const int O2 = fc2.out, G1 = fc1.groups, G2 = fc2.groups;
    if ((int64_t)dag.N * std::max(C, O2) * Pn * 2 >= ((int64_t)1 << 31) || (int64_t)dag.N * TVa * Pn * 4 >= ((int64_t)1 << 31) || dag.W < 4 ||
        (int64_t)dag.N * Pn >= ((int64_t)1 << 28))
        return nullptr;
    const int upi = (Pn + 7) / 8;
    if ((int64_t)dag.N * C * upi >= ((int64_t)1 << 31) || (int64_t)dag.N * Gb * upi * upi >= ((int64_t)1 << 32) ||
        (int64_t)dag.N * Gb >= ((int64_t)1 << 24))
        return nullptr;

    dyn::Params D;
    D.N = dag.N * Gb;
    D.C = C / Gb;
    D.H = dag.H;
    D.W = dag.W;
    D.P = Pn;
    D.upi = upi;
    D.KH = unf.kh;
    D.KW = unf.kw;
    D.scale = fold.kind == kAvg ? 1.f / (float)TV : 1.f;
    auto magic = [](uint32_t d) { return d <= 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) + d - 1) / d); };
    D.magicW = magic((uint32_t)dag.W);
    D.magicUpi = magic((uint32_t)upi);

    auto low = std::make_unique<Lowering>();
    low->fused = true;
    uint64_t off = 0;
    const TakeFn take = [&off](uint64_t bytes) {
        const uint64_t o = off;
        off += align_up(bytes);
        return (int64_t)o;
    };
    const double act = 2.0 * dag.numel(0), outb = 2.0 * dag.numel(dag.out), ab = 4.0 * dag.N * TVa * Pn;
    const int64_t ol = take((uint64_t)ab), oa = isoft >= 0 ? take((uint64_t)ab) : ol;  // logits, softmax output (fp32)
    const int64_t ou = take((uint64_t)act), odu = take((uint64_t)act);
    const int64_t oda = take((uint64_t)ab), odl = isoft >= 0 ? take((uint64_t)ab) : oda;
    // the gradient of the logits once more in bf16: the data gradient of FC1 then runs on the bf16 MFMA kernel (its
    // result is rounded to bf16 anyway); the weight gradient keeps the fp32 copy
    const int64_t odl16 = isoft >= 0 ? take((uint64_t)(ab / 2)) : -1;
    const int w1 = fc1.widx, w2 = fc2.widx;
    const int64_t nw1 = (int64_t)TVa * (C / G1), nw2 = (int64_t)O2 * (C / G2);
    const double fl1 = 2.0 * dag.N * Pn * (double)nw1, fl2 = 2.0 * dag.N * Pn * (double)nw2;
    const double fld = 2.0 * dag.N * Pn * (double)C * TV;
    const int64_t N = dag.N;
    const bool soft = isoft >= 0;
    auto ws_at = [](int64_t o) { return [=](const RunArgs& a) { return (const void*)(a.ws + o); }; };
    const FcOperand in_x{[](const RunArgs& a) { return a.x; }, false};
    const FcOperand in_dy{[](const RunArgs& a) { return a.dy; }, false};

    // the softmax over the few channels of FC1 is the epilogue of FC1 where all of them are in one tile
    const bool sm_in_fc1 = soft && fc_softmax_fusable(dag, G1, C / G1, 1, 1, TVa / G1, in_x);
    emit_fc(*low, false, dag, take, sm_in_fc1 ? "dyn_fc1_softmax" : "dyn_fc1", G1, C / G1, 1, 1, TVa / G1, false, w1, in_x,
            ws_at(sm_in_fc1 ? oa : ol), false, act + ab + 2.0 * nw1, fl1, true, sm_in_fc1);
    if (soft && !sm_in_fc1)
        low->fwd.push_back({"dyn_softmax", 2.0 * ab, 0, [=](const RunArgs& a) {
                                ref::softmax_fwd((const float*)(a.ws + ol), (float*)(a.ws + oa), N, TVa, 1, Pn, 1, a.stream);
                            }});
    low->fwd.push_back({"dyn_apply", 2.0 * act + ab, fld, [=](const RunArgs& a) {
                            dyn::Params Q = D;
                            Q.x = (const uint16_t*)a.x;
                            Q.a = (const float*)(a.ws + oa);
                            Q.u = (uint16_t*)(a.ws + ou);
                            dyn::forward(Q, a.stream);
                        }});
    emit_fc(*low, false, dag, take, "dyn_fc2", G2, C / G2, 1, 1, O2 / G2, false, w2, FcOperand{ws_at(ou), false},
            [](const RunArgs& a) { return (const void*)a.y; }, false, act + outb + 2.0 * nw2, fl2);

    // backward (forward must have run with the same workspace: a and u are read back)
    emit_wgrad(*low, dag, take, "dyn_fc2_wgrad", G2, C / G2, 1, 1, O2 / G2, w2, FcOperand{ws_at(ou), false}, in_dy, act + outb, fl2);
    emit_fc(*low, true, dag, take, "dyn_fc2_dgrad", G2, O2 / G2, 1, 1, C / G2, true, w2, in_dy, ws_at(odu), false, act + outb + 2.0 * nw2, fl2);
    low->bwd.push_back({"dyn_apply_dx_da", 3.0 * act + 2.0 * ab, 2.0 * fld, [=](const RunArgs& a) {
                            dyn::Params Q = D;
                            Q.x = (const uint16_t*)a.x;
                            Q.a = (const float*)(a.ws + oa);
                            Q.du = (const uint16_t*)(a.ws + odu);
                            Q.dx = (uint16_t*)a.dx;
                            Q.da = (float*)(a.ws + oda);
                            dyn::backward_dx_da(Q, a.stream);
                        }});
    if (soft)
        low->bwd.push_back({"dyn_softmax_bwd", 3.0 * ab, 0, [=](const RunArgs& a) {
                                ref::softmax_bwd((const float*)(a.ws + oa), (const float*)(a.ws + oda), (float*)(a.ws + odl), N, TVa, 1, Pn, 1, 0,
                                                 a.stream, (uint16_t*)(a.ws + odl16));
                            }});
    emit_wgrad(*low, dag, take, "dyn_fc1_wgrad", G1, C / G1, 1, 1, TVa / G1, w1, in_x, FcOperand{ws_at(odl), true}, act + ab, fl1);
    // the data gradient of FC1 adds to the dx that dyn_apply_dx_da has written
    emit_fc(*low, true, dag, take, "dyn_fc1_dgrad", G1, TVa / G1, 1, 1, C / G1, true, w1,
            soft ? FcOperand{ws_at(odl16), false} : FcOperand{ws_at(odl), true},
            [](const RunArgs& a) { return (const void*)a.dx; }, true, 2.0 * act + ab + 2.0 * nw1, fl1);
    low->ws_bytes = off;
    return low;
}

}  // namespace canvas
