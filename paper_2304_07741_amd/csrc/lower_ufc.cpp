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

#include "gfc_kernels.hpp"
#include "gfc_tm_kernels.hpp"
#include "lowering.hpp"
#include "ufc_kernels.hpp"

namespace canvas {

std::unique_ptr<Lowering> lower_ufc(const Dag& dag, bool bf16) {
    if (!bf16) return nullptr;
    const int n = (int)dag.nodes.size();
    for (int k = 0; k < n; k++)
        if (!dag.nodes[k].live) return nullptr;
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
    while (k < n && dag.nodes[k].op == Op::Fold && dag.nodes[dag.nodes[k].a].T == 1) {  // a fold over one tap is the identity
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
    gfc::Params F1 = gfc::shape(dag.N, G1, C / G1, KH, KW, C / G1, dag.H, dag.W);
    gfc::Params F2 = gfc::shape(dag.N, G2, C / G2, 1, 1, O2 / G2, dag.H, dag.W);
    F1.src_f32 = F2.src_f32 = 0;
    F1.dst_f32 = F2.dst_f32 = 0;
    F1.dy_f32 = F2.dy_f32 = 0;
    gfc::Params W1 = F1, W2 = F2;
    gfc::prepare_wgrad(W1);
    gfc::prepare_wgrad(W2);
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
    const int64_t nw1 = (int64_t)C * F1.K, nw2 = (int64_t)O2 * F2.K;
    const double act = 2.0 * dag.numel(0), outb = 2.0 * dag.numel(dag.out);
    uint64_t off = 0;
    auto take = [&](uint64_t bytes) {
        const uint64_t o = off;
        off += align_up(bytes);
        return (int64_t)o;
    };
    const int64_t oz = take((uint64_t)act), ov = take((uint64_t)act), odv = take((uint64_t)act), odz = take((uint64_t)act);
    const int64_t op1 = take((uint64_t)W1.slices * nw1 * 4), op2 = take((uint64_t)W2.slices * nw2 * 4);
    low->ws_bytes = off;
    const int w1 = fc1.widx, w2 = fc2.widx;
    const double fl1 = 2.0 * dag.N * Pn * (double)C * F1.K, fl2 = 2.0 * dag.N * Pn * (double)O2 * F2.K;

    // One FC-shaped contraction (forward, or a data gradient when `transposed`): the tap-major kernels
    // with a weight-packing launch in front where they apply, else the generic kernel (whose data
    // gradient wants the weights transposed first).
    using Ptr = std::function<const void*(const RunArgs&)>;
    auto emit_fc = [&](std::vector<Launch>& list, const std::string& name, int G, int R, int kh, int kw, int Og, bool transposed, int widx,
                       Ptr src, Ptr dst, bool addend_is_dst, double bytes, double flops) {
        const int64_t nw = (int64_t)G * Og * R * kh * kw;
        // (1x1 contractions with enough tiles to fill the chip stay on the generic kernel: measured faster there)
        if (gfctm::supported(dag.N, G, R, kh, kw, Og, dag.H, dag.W) &&
            (kh * kw > 1 || gfctm::shape(dag.N, G, R, kh, kw, Og, dag.H, dag.W).ksplit > 1)) {
            const gfctm::Params T = gfctm::shape(dag.N, G, R, kh, kw, Og, dag.H, dag.W);
            const bool identity = !transposed && T.TV == 1 && T.gm == 1 && T.Rp == R && T.Omp == Og;
            const int64_t opk = identity ? -1 : take((uint64_t)gfctm::packed_elems(T) * 2);
            if (!identity)
                list.push_back({name + "_pack_w", 2.0 * nw + 2.0 * gfctm::packed_elems(T), 0, [=](const RunArgs& a) {
                                    gfctm::pack_weights((const uint16_t*)a.w[widx], (uint16_t*)(a.ws + opk), T, transposed, a.stream);
                                }});
            list.push_back({name, bytes, flops, [=](const RunArgs& a) {
                                gfctm::Params Q = T;
                                Q.src = (const uint16_t*)src(a);
                                Q.wp = identity ? (const uint16_t*)a.w[widx] : (const uint16_t*)(a.ws + opk);
                                Q.dst = const_cast<void*>(dst(a));
                                Q.addend = addend_is_dst ? (const uint16_t*)dst(a) : nullptr;  // each lane reads the elements it then overwrites
                                gfctm::forward(Q, a.stream);
                            }});
            return;
        }
        gfc::Params F = gfc::shape(dag.N, G, R, kh, kw, Og, dag.H, dag.W);
        F.src_f32 = 0;
        F.dst_f32 = 0;
        gfc::prepare_forward(F);
        const int64_t owt = transposed ? take((uint64_t)nw * 2) : -1;
        if (transposed)  // here (R, Og) are already the swapped dims: the FC's own weights are [G][R][Og][taps]
            list.push_back({name + "_transpose_w", 4.0 * nw, 0, [=](const RunArgs& a) {
                                gfc::transpose_weights((const uint16_t*)a.w[widx], (uint16_t*)(a.ws + owt), G, R, Og, kh * kw, a.stream);
                            }});
        list.push_back({name, bytes, flops, [=](const RunArgs& a) {
                            gfc::Params Q = F;
                            Q.src = src(a);
                            Q.w = transposed ? (const uint16_t*)(a.ws + owt) : (const uint16_t*)a.w[widx];
                            Q.dst = const_cast<void*>(dst(a));
                            Q.addend = addend_is_dst ? (const uint16_t*)dst(a) : nullptr;
                            gfc::forward(Q, a.stream);
                        }});
    };
    const int TV = KH * KW;
    emit_fc(low->fwd, TV > 1 ? "ufc_fc1_unfold" : "ufc_fc1", G1, C / G1, KH, KW, C / G1, false, w1,
            [](const RunArgs& a) { return a.x; }, [=](const RunArgs& a) { return (const void*)(a.ws + oz); }, false, 2.0 * act + 2.0 * nw1, fl1);
    low->fwd.push_back({"ufc_mid_fwd", 3.0 * act, 0, [=](const RunArgs& a) {
                            ufc::MidParams R = M;
                            R.x = (const uint16_t*)a.x;
                            R.z = (const uint16_t*)(a.ws + oz);
                            R.v = (uint16_t*)(a.ws + ov);
                            ufc::mid_forward(R, a.stream);
                        }});
    emit_fc(low->fwd, "ufc_fc2", G2, C / G2, 1, 1, O2 / G2, false, w2, [=](const RunArgs& a) { return (const void*)(a.ws + ov); },
            [](const RunArgs& a) { return (const void*)a.y; }, false, act + outb + 2.0 * nw2, fl2);

    // backward (forward must have run with the same workspace: z and v are read back, and left intact)
    const int s1 = W1.slices, s2 = W2.slices;
    low->bwd.push_back({"ufc_fc2_wgrad", act + outb + 4.0 * s2 * nw2, fl2, [=](const RunArgs& a) {
                            gfc::Params R = W2;
                            R.src = a.ws + ov;
                            R.dy = a.dy;
                            R.partial = (float*)(a.ws + op2);
                            gfc::wgrad_partial(R, a.stream);
                        }});
    low->bwd.push_back({"ufc_fc2_wgrad_reduce", 4.0 * (s2 + 1) * nw2, 0, [=](const RunArgs& a) {
                            gfc::wgrad_reduce((const float*)(a.ws + op2), (float*)a.dw[w2], s2, nw2, a.stream);
                        }});
    emit_fc(low->bwd, "ufc_fc2_dgrad", G2, O2 / G2, 1, 1, C / G2, true, w2, [](const RunArgs& a) { return a.dy; },
            [=](const RunArgs& a) { return (const void*)(a.ws + odv); }, false, act + outb + 2.0 * nw2, fl2);
    low->bwd.push_back({"ufc_mid_bwd", (M.bin ? 5.0 : 4.0) * act, 0, [=](const RunArgs& a) {
                            ufc::MidParams R = M;
                            R.x = (const uint16_t*)a.x;
                            R.z = (const uint16_t*)(a.ws + oz);
                            R.dv = (const uint16_t*)(a.ws + odv);
                            R.dz = (uint16_t*)(a.ws + odz);
                            R.dx1 = (uint16_t*)a.dx;  // completed by the data gradient of FC1 below
                            ufc::mid_backward(R, a.stream);
                        }});
    if (TV > 1 && gfctm::supported(dag.N, G1, C / G1, KH, KW, C / G1, dag.H, dag.W)) {
        gfctm::Params T = gfctm::shape(dag.N, G1, C / G1, KH, KW, C / G1, dag.H, dag.W);
        gfctm::prepare_wgrad(T);
        const int ts = gfctm::wgrad_slices(T);
        const int64_t pk = gfctm::packed_elems(T);
        const int64_t opt = take((uint64_t)ts * pk * 4);
        low->bwd.push_back({"ufc_fc1_wgrad_unfold", 2.0 * act + 4.0 * ts * pk, fl1, [=](const RunArgs& a) {
                                gfctm::Params R = T;
                                R.src = (const uint16_t*)a.x;
                                R.dy = (const uint16_t*)(a.ws + odz);
                                R.partial = (float*)(a.ws + opt);
                                gfctm::wgrad_partial(R, a.stream);
                            }});
        low->bwd.push_back({"ufc_fc1_wgrad_reduce", 4.0 * ts * pk + 4.0 * nw1, 0, [=](const RunArgs& a) {
                                gfctm::Params R = T;
                                R.partial = (float*)(a.ws + opt);
                                gfctm::wgrad_reduce(R, (float*)a.dw[w1], a.stream);
                            }});
    } else {
        low->bwd.push_back({KH * KW > 1 ? "ufc_fc1_wgrad_unfold" : "ufc_fc1_wgrad", 2.0 * act + 4.0 * s1 * nw1, fl1, [=](const RunArgs& a) {
                                gfc::Params R = W1;
                                R.src = a.x;
                                R.dy = a.ws + odz;
                                R.partial = (float*)(a.ws + op1);
                                gfc::wgrad_partial(R, a.stream);
                            }});
        low->bwd.push_back({"ufc_fc1_wgrad_reduce", 4.0 * (s1 + 1) * nw1, 0, [=](const RunArgs& a) {
                                gfc::wgrad_reduce((const float*)(a.ws + op1), (float*)a.dw[w1], s1, nw1, a.stream);
                            }});
    }
    // mid_backward left dx_direct in dx; the data gradient of FC1 (through the Unfold adjoint) adds to it
    emit_fc(low->bwd, TV > 1 ? "ufc_fc1_dgrad_unfold" : "ufc_fc1_dgrad", G1, C / G1, KH, KW, C / G1, true, w1,
            [=](const RunArgs& a) { return (const void*)(a.ws + odz); }, [](const RunArgs& a) { return (const void*)a.dx; }, true,
            3.0 * act + 2.0 * nw1, fl1);
    low->ws_bytes = off;
    return low;
}

}  // namespace canvas
