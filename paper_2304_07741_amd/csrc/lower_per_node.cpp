// Lowering by units, for every legal DAG.  The DAG is cut at its FC nodes; the runs of memory-bound primitives
// between them are grown, one node at a time in topological order, into fused chains (chain_plan.hpp: one forward
// and one backward kernel per chain, nothing inside a chain is materialised, an Unfold is never written out); a
// node joins the chain of one of its operands as long as the grown chain still compiles (a stencil above a
// reduction, a blend across channel counts, too many taps, registers, instructions or LDS end a chain).  What no
// chain takes (folds over space or channels, joint softmax, grouped blends ...) is one kernel per node, and so is
// everything when fusion is switched off.  FC nodes run on the MFMA kernels (bf16 dtype) or the plain ones.
// Tensors that cross a unit boundary live in the workspace as fp32 [N, C, T, H, W] together with their gradients;
// x, y, dy and dx are read and written in place, in their own type, wherever the unit at that end can do so.
#include "lowering.hpp"
#include "chain_kernels.hpp"
#include "chain_plan.hpp"
#include "gfc_kernels.hpp"
#include "ref_kernels.hpp"

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <stdexcept>

namespace canvas {

namespace {

struct Layout {
    std::vector<int64_t> val, grad, wf;  // byte offsets into the workspace; -1 = not in the workspace
    std::vector<int64_t> wt, part;       // per fc (bf16 path): transposed weights, weight-gradient partials
    uint64_t total = 0;
};

const char* op_name(Op op) {
    switch (op) {
    case Op::Unfold: return "unfold";
    case Op::Shift: return "shift";
    case Op::Fc: return "fc";
    case Op::Unary: return "unary";
    case Op::Binary: return "binary";
    case Op::Softmax: return "softmax";
    case Op::Fold: return "fold";
    case Op::Group: return "group";
    default: return "input";
    }
}

}  // namespace

namespace {

struct Unit {
    bool chain = false;
    std::vector<int> nodes;       // ascending
    chain::UnitPlan plan;         // chain units
};

// A program ready to launch: the pointers of its external tensors are resolved per call.
struct Binding {
    int node = -1;
    chain::ExtRole role = chain::kValueIn;
    int where = 0;   // 0 = workspace offset `off` (fp32), 1 = x, 2 = y, 3 = dy, 4 = dx (the caller's tensors, in the DAG's dtype)
    int64_t off = 0;
};

void run_program(const chain::Program& pg0, const std::vector<Binding>& bind, bool bf16, const RunArgs& a) {
    chain::Program pg = pg0;
    pg.fast_math = bf16 ? 1 : 0;
    for (size_t i = 0; i < bind.size(); i++) {
        const Binding& b = bind[i];
        switch (b.where) {
        case 0: pg.ext[i].ptr = a.ws + b.off; pg.ext[i].bf16 = 0; break;
        case 1: pg.ext[i].ptr = const_cast<void*>(a.x); pg.ext[i].bf16 = bf16; break;
        case 2: pg.ext[i].ptr = a.y; pg.ext[i].bf16 = bf16; break;
        case 3: pg.ext[i].ptr = const_cast<void*>(a.dy); pg.ext[i].bf16 = bf16; break;
        default: pg.ext[i].ptr = a.dx; pg.ext[i].bf16 = bf16; break;
        }
    }
    chain::run(pg, a.stream);
}

}  // namespace

std::unique_ptr<Lowering> lower_per_node(const Dag& dag, bool bf16, bool fuse_chains) {
    auto low = std::make_unique<Lowering>();
    const int n = (int)dag.nodes.size();
    const int P = dag.P();
    const int64_t N = dag.N;
    Layout lay;
    lay.val.assign(n, -1);
    lay.grad.assign(n, -1);
    lay.wf.assign(dag.n_weights, -1);
    uint64_t off = 0;
    auto take = [&](int64_t numel) {
        uint64_t o = off;
        off += align_up((uint64_t)numel * 4);
        return (int64_t)o;
    };
    // bf16 path: FC nodes run on MFMA and read an Unfold operand implicitly.  An Unfold whose every
    // consumer is such an FC is never materialised (no value, no gradient, no launch).
    auto bytes_ok = [&](int64_t numel) { return numel * 4 < ((int64_t)1 << 31); };
    bool mfma = bf16 && dag.W >= 4 && (int64_t)dag.N * dag.P() < ((int64_t)1 << 28);
    for (int k = 1; k < n && mfma; k++) {
        const Node& f = dag.nodes[k];
        if (!f.live || f.op != Op::Fc) continue;
        const Node& A = dag.nodes[f.a];
        const int srcn = A.op == Op::Unfold ? A.a : f.a;  // the larger of the two possible operands is f.a
        mfma = bytes_ok(dag.numel(f.a)) && bytes_ok(dag.numel(srcn)) && bytes_ok(dag.numel(k)) &&
               bytes_ok((int64_t)f.out * (A.C / f.groups) * A.T);
    }
    std::vector<bool> virt(n, false);
    if (mfma) {
        for (int k = 1; k < n; k++) {
            const Node& u = dag.nodes[k];
            if (!u.live || u.op != Op::Unfold || u.kh > 7 || u.kw > 7) continue;
            bool only_fc = true;
            for (int j = k + 1; j < n; j++) {
                const Node& c = dag.nodes[j];
                if (!c.live) continue;
                if ((c.a == k || c.b == k) && c.op != Op::Fc) only_fc = false;
            }
            virt[k] = only_fc && dag.out != k;
        }
    }
    // which fc nodes use the MFMA kernels (32-bit buffer offsets must cover their tensors; a 1 x 1 image has no
    // 8-pixel units: the plain kernels take it)
    std::vector<bool> fc_mfma(n, false);
    for (int k = 1; k < n; k++)
        if (dag.nodes[k].live && dag.nodes[k].op == Op::Fc) fc_mfma[k] = mfma && !dag.nodes[k].pooled;

    // ---------------------------------------------------------------- units
    std::vector<std::vector<int>> consumers(n);
    for (int k = 1; k < n; k++) {
        const Node& nd = dag.nodes[k];
        if (!nd.live) continue;
        consumers[nd.a].push_back(k);
        if (nd.b >= 0 && nd.b != nd.a) consumers[nd.b].push_back(k);
    }
    std::vector<Unit> units;
    std::vector<int> unit_of(n, -1);
    auto outputs_of = [&](const std::vector<int>& nodes) {
        std::vector<bool> in(n, false), outp(n, false);
        for (int k : nodes) in[k] = true;
        for (int k : nodes) {
            if (k == dag.out) outp[k] = true;
            for (int c : consumers[k])
                if (!in[c]) outp[k] = true;
        }
        return outp;
    };
    const bool log = std::getenv("CANVAS_LOG") != nullptr;
    for (int k = 1; k < n; k++) {
        const Node& nd = dag.nodes[k];
        if (!nd.live || virt[k]) continue;
        bool placed = false;
        if (fuse_chains && chain::chain_candidate(dag, k)) {
            // the chains of the operands, latest first; joining chain u needs every operand inside u or produced before u runs
            std::vector<int> cands;
            for (int o : {nd.b, nd.a})
                if (o > 0 && unit_of[o] >= 0 && units[unit_of[o]].chain && std::find(cands.begin(), cands.end(), unit_of[o]) == cands.end())
                    cands.push_back(unit_of[o]);
            std::sort(cands.rbegin(), cands.rend());
            for (int u : cands) {
                bool ok = true;
                for (int o : {nd.a, nd.b})
                    if (o > 0 && !virt[o] && unit_of[o] != u && unit_of[o] > u) ok = false;
                if (!ok) continue;
                std::vector<int> grown = units[u].nodes;
                grown.push_back(k);
                chain::UnitPlan plan;
                std::string why;
                if (chain::compile_unit(dag, grown, outputs_of(grown), plan, why)) {
                    units[u].nodes = grown;
                    units[u].plan = plan;
                    unit_of[k] = u;
                    placed = true;
                    break;
                }
                if (log) std::fprintf(stderr, "canvas: node %d does not join chain %d: %s\n", k, u, why.c_str());
            }
            if (!placed) {
                chain::UnitPlan plan;
                std::string why;
                std::vector<int> alone{k};
                if (chain::compile_unit(dag, alone, outputs_of(alone), plan, why)) {
                    Unit U;
                    U.chain = true;
                    U.nodes = alone;
                    U.plan = plan;
                    units.push_back(U);
                    unit_of[k] = (int)units.size() - 1;
                    placed = true;
                } else if (log) {
                    std::fprintf(stderr, "canvas: node %d takes a kernel of its own: %s\n", k, why.c_str());
                }
            }
        }
        if (!placed) {
            Unit U;
            U.nodes = {k};
            units.push_back(U);
            unit_of[k] = (int)units.size() - 1;
        }
    }
    // Full recomputation makes a long chain dearer than its parts (every unary's adjoint evaluates its operand again,
    // every softmax over channels adds passes).  A grown chain is therefore cut in two, at the place that pays most,
    // while the halves together cost less than four fifths of the whole, and the halves are looked at again.  A cut
    // materialises what crosses it: across a tensor with taps (an unfolded tensor, which a chain otherwise never
    // writes) it is only made when the halves cost less than two fifths of the whole, which in practice means a
    // softmax over channels of an unfolded tensor, whose passes each recompute the whole window.
    for (size_t u = 0; u < units.size(); u++) {
        if (!units[u].chain || units[u].nodes.size() < 2) continue;
        std::string why;
        chain::UnitPlan whole;
        if (!chain::compile_unit(dag, units[u].nodes, outputs_of(units[u].nodes), whole, why)) continue;
        const std::vector<int> nodes = units[u].nodes;
        double best = whole.cost;
        size_t cut = 0;
        for (size_t i = 1; i < nodes.size(); i++) {
            const std::vector<int> A(nodes.begin(), nodes.begin() + i), Bn(nodes.begin() + i, nodes.end());
            bool taps = false;
            for (int k : Bn)
                for (int o : {dag.nodes[k].a, dag.nodes[k].b})
                    if (o > 0 && std::find(A.begin(), A.end(), o) != A.end() && dag.nodes[o].T != 1) taps = true;
            chain::UnitPlan pa, pb;
            if (!chain::compile_unit(dag, A, outputs_of(A), pa, why) || !chain::compile_unit(dag, Bn, outputs_of(Bn), pb, why)) continue;
            const double apart = (pa.cost + pb.cost) / (taps ? 0.4 : 0.8);  // (as if the whole had to be that much dearer)
            if (apart < best) {
                best = apart;
                cut = i;
            }
        }
        if (cut == 0) continue;
        if (log) std::fprintf(stderr, "canvas: chain %zu cut after %zu of %zu nodes: weighted cost %.0f apart, %.0f whole\n", u, cut, nodes.size(), best, whole.cost);
        Unit B;
        B.chain = true;
        B.nodes.assign(nodes.begin() + cut, nodes.end());
        units[u].nodes.assign(nodes.begin(), nodes.begin() + cut);
        units.insert(units.begin() + u + 1, B);
        for (size_t v = 0; v < units.size(); v++)
            for (int k : units[v].nodes) unit_of[k] = (int)v;
        u--;  // (the first half again, then the second)
    }
    // a unit was last compiled when it last grew, against the consumers known then; later nodes may have joined
    // other units, which never removes an output, but a later joiner of THIS unit may have: compile the final sets
    for (Unit& U : units)
        if (U.chain) {
            std::string why;
            if (!chain::compile_unit(dag, U.nodes, outputs_of(U.nodes), U.plan, why)) throw std::runtime_error("chain unit no longer compiles: " + why);
            low->chain_units++;
            low->chain_nodes += (int)U.nodes.size();
            if (log) {
                std::string ids;
                for (int k : U.nodes) ids += " " + std::to_string(k);
                std::fprintf(stderr, "canvas: chain of %zu nodes [%s ] cost fwd %.1f bwd %.1f\n%s%s", U.nodes.size(), ids.c_str(),
                             chain::program_cost(U.plan.fwd), chain::program_cost(U.plan.bwd), chain::dump(U.plan.fwd).c_str(), chain::dump(U.plan.bwd).c_str());
            }
        }
    // materialised nodes: everything outside a chain, and the stored nodes of a chain
    std::vector<bool> mat(n, false);
    for (const Unit& U : units) {
        if (!U.chain) mat[U.nodes[0]] = true;
        else
            for (int o : U.plan.outputs) mat[o] = true;
    }
    // who can use the caller's tensors in place: chains (any dtype) and MFMA FC nodes (bf16)
    auto in_place = [&](int k) { return k > 0 && unit_of[k] >= 0 && (units[unit_of[k]].chain || fc_mfma[k]); };
    // x: read in place by chains and by MFMA FC nodes (also through a virtual Unfold); a widened copy only for the others
    bool need_x32 = dag.out == 0;
    for (int c : consumers[0]) {
        if (virt[c]) continue;  // (its consumers are MFMA FC nodes)
        if (!in_place(c)) need_x32 = true;
    }
    // y and dy: in place when the output node is produced by such a unit and nothing else reads it
    const bool y_direct = in_place(dag.out) && consumers[dag.out].empty();
    // dx: in place when exactly one unit writes the gradient of x and it can
    int x_writers = 0;
    bool x_writer_ok = true;
    {
        std::vector<int> seen;
        for (int c : consumers[0]) {
            if (virt[c]) {
                for (int f : consumers[c]) x_writers++, x_writer_ok = x_writer_ok && fc_mfma[f];
                continue;
            }
            const int u = unit_of[c];
            if (units[u].chain) {
                if (std::find(seen.begin(), seen.end(), u) != seen.end()) continue;
                seen.push_back(u);
            }
            x_writers++;
            x_writer_ok = x_writer_ok && in_place(c);
        }
    }
    const bool dx_direct = x_writers == 1 && x_writer_ok;
    for (int k = 0; k < n; k++) {
        if (!dag.nodes[k].live || virt[k]) continue;
        if (k == 0) {
            if (bf16 && need_x32) lay.val[0] = take(dag.numel(0));
            if (!dx_direct) lay.grad[0] = take(dag.numel(0));
            continue;
        }
        if (!mat[k]) continue;
        if (k == dag.out && y_direct) continue;  // value in y, gradient in dy
        lay.val[k] = take(dag.numel(k));
        lay.grad[k] = take(dag.numel(k));
    }
    std::vector<int64_t> wnumel(dag.n_weights);
    for (int i = 0; i < dag.n_weights; i++) {
        const Node& f = dag.nodes[dag.weight_node[i]];
        const Node& A = dag.nodes[f.a];
        wnumel[i] = (int64_t)f.out * (A.C / f.groups) * A.T;
    }
    // MFMA contraction parameters of fc node k (forward orientation); src pointer filled at run time
    auto fc_params = [&](int k) {
        const Node& f = dag.nodes[k];
        const bool v = virt[f.a];
        const Node& U = dag.nodes[f.a];
        const int srcn = v ? U.a : f.a;
        const Node& S = dag.nodes[srcn];
        gfc::Params Q = gfc::shape(dag.N, f.groups, (S.C / f.groups) * S.T, v ? U.kh : 1, v ? U.kw : 1, f.out / f.groups, dag.H, dag.W);
        return Q;
    };
    auto fc_src = [&](int k) { return virt[dag.nodes[k].a] ? dag.nodes[dag.nodes[k].a].a : dag.nodes[k].a; };

    // geometry of the weight-gradient launch of MFMA fc node k (operand types decide its tile shape)
    auto wgrad_params = [&](int k) {
        gfc::Params Q = fc_params(k);
        Q.src_f32 = fc_src(k) == 0 ? 0 : 1;
        Q.dy_f32 = (k == dag.out && y_direct) ? 0 : 1;
        gfc::prepare_wgrad(Q);
        return Q;
    };
    lay.wt.assign(dag.n_weights, -1);
    lay.part.assign(dag.n_weights, -1);
    for (int i = 0; i < dag.n_weights; i++) {
        const int k = dag.weight_node[i];
        const Node& f = dag.nodes[k];
        if (!f.live) continue;
        if (!fc_mfma[k]) {
            if (bf16) lay.wf[i] = take(wnumel[i]);
            continue;
        }
        lay.wt[i] = (int64_t)off;
        off += align_up((uint64_t)wnumel[i] * 2);
        const gfc::Params Q = wgrad_params(k);
        const int64_t slices = gfc::wgrad_partials(Q);
        lay.part[i] = (int64_t)off;
        off += align_up((uint64_t)slices * wnumel[i] * 4);
    }
    low->ws_bytes = off;
    const double esz = bf16 ? 2.0 : 4.0;

    // pointer resolvers
    auto val = [lay](const RunArgs& a, int k) -> const float* {
        return lay.val[k] >= 0 ? (const float*)(a.ws + lay.val[k]) : (const float*)a.x;
    };
    auto valw = [lay](const RunArgs& a, int k) -> float* { return (float*)(a.ws + lay.val[k]); };
    auto grad = [lay](const RunArgs& a, int k) -> float* { return (float*)(a.ws + lay.grad[k]); };
    auto wptr = [lay, bf16](const RunArgs& a, int i) -> const float* {
        return bf16 ? (const float*)(a.ws + lay.wf[i]) : (const float*)a.w[i];
    };

    // ---------------------------------------------------------------- forward
    if (bf16) {
        int64_t ne = dag.numel(0);
        if (lay.val[0] >= 0) low->fwd.push_back({"widen_x", ne * 6.0, 0, [=](const RunArgs& a) { ref::widen_bf16(a.x, valw(a, 0), ne, a.stream); }});
        for (int i = 0; i < dag.n_weights; i++) {
            if (lay.wf[i] < 0) continue;  // MFMA fc nodes read the bf16 weights as they are
            int64_t nw = wnumel[i];
            int64_t o = lay.wf[i];
            low->fwd.push_back({"widen_w", nw * 6.0, 0, [=](const RunArgs& a) { ref::widen_bf16(a.w[i], (float*)(a.ws + o), nw, a.stream); }, true});
        }
    }
    // where an external tensor of a chain program lives
    auto bind = [&](const std::vector<chain::ExtRef>& ext) {
        std::vector<Binding> b(ext.size());
        for (size_t i = 0; i < ext.size(); i++) {
            const int e = ext[i].node;
            b[i].node = e;
            b[i].role = ext[i].role;
            switch (ext[i].role) {
            case chain::kValueIn:
                if (e == 0) b[i].where = 1;
                else b[i].off = lay.val[e];
                break;
            case chain::kValueOut:
                if (e == dag.out && y_direct) b[i].where = 2;
                else b[i].off = lay.val[e];
                break;
            case chain::kGradIn:
                if (e == dag.out && y_direct) b[i].where = 3;
                else b[i].off = lay.grad[e];
                break;
            case chain::kGradOut:
                if (e == 0 && dx_direct) b[i].where = 4;
                else b[i].off = lay.grad[e];
                break;
            }
            if (b[i].where == 0 && b[i].off < 0) throw std::runtime_error("chain: an external tensor without a buffer");
        }
        return b;
    };
    auto ext_bytes = [&](const std::vector<Binding>& b) {
        double t = 0;
        for (const Binding& e : b) t += (e.where == 0 ? 4.0 : esz) * dag.numel(e.node);
        return t;
    };
    for (size_t ui = 0; ui < units.size(); ui++) {
        const Unit& U = units[ui];
        if (U.chain) {
            const chain::Program pg = U.plan.fwd;
            const std::vector<Binding> b = bind(U.plan.fwd_ext);
            low->fwd.push_back({"chain_fwd", ext_bytes(b), 0, [=](const RunArgs& a) { run_program(pg, b, bf16, a); }});
            continue;
        }
        const int k = U.nodes[0];
        const Node nd = dag.nodes[k];
        const Node A = dag.nodes[nd.a];
        Launch L;
        L.name = std::string("node_") + op_name(nd.op) + "_fwd";
        L.bytes = 4.0 * (dag.numel(nd.a) + dag.numel(k));
        switch (nd.op) {
        case Op::Unfold:
            L.run = [=](const RunArgs& a) { ref::unfold_fwd(val(a, nd.a), valw(a, k), N * A.C, A.T, nd.kh, nd.kw, dag.H, dag.W, a.stream); };
            break;
        case Op::Shift:
            L.run = [=](const RunArgs& a) {
                ref::shift(val(a, nd.a), valw(a, k), N, nd.C, nd.T, dag.H, dag.W, nd.dh, nd.dw, nd.c0, nd.c1, 0, a.stream);
            };
            break;
        case Op::Fc: {
            int G = nd.groups, Og = nd.out / G, K = (A.C / G) * A.T;
            L.flops = 2.0 * N * dag.Pk(k) * nd.out * K;
            if (fc_mfma[k]) {
                gfc::Params Q = fc_params(k);
                const int srcn = fc_src(k);
                const bool src_x = srcn == 0;  // the caller's bf16 input is read directly
                const bool to_y = k == dag.out && y_direct;  // the output node: written as bf16 where the caller wants it
                Q.src_f32 = src_x ? 0 : 1;
                Q.dst_f32 = to_y ? 0 : 1;
                gfc::prepare_forward(Q);
                L.name = Q.TV > 1 ? "gfc_fwd_unfold" : "gfc_fwd";
                L.bytes = (src_x ? 2.0 : 4.0) * dag.numel(srcn) + (to_y ? 2.0 : 4.0) * dag.numel(k) + 2.0 * wnumel[nd.widx];
                const int widx = nd.widx;
                L.run = [=](const RunArgs& a) {
                    gfc::Params R = Q;
                    R.src = src_x ? a.x : (const void*)val(a, srcn);
                    R.w = (const uint16_t*)a.w[widx];
                    R.dst = to_y ? a.y : (void*)valw(a, k);
                    gfc::forward(R, a.stream);
                };
                break;
            }
            L.bytes += 4.0 * wnumel[nd.widx];
            const int Pn = dag.Pk(k);
            L.run = [=](const RunArgs& a) { ref::fc_fwd(val(a, nd.a), wptr(a, nd.widx), valw(a, k), N, G, Og, K, Pn, a.stream); };
            break;
        }
        case Op::Unary: {
            int64_t ne = dag.numel(k);
            L.run = [=](const RunArgs& a) { ref::unary_fwd(val(a, nd.a), valw(a, k), ne, nd.kind, nd.lo, nd.hi, a.stream); };
            break;
        }
        case Op::Binary: {
            const Node B = dag.nodes[nd.b];
            L.bytes = 4.0 * (dag.numel(nd.a) + dag.numel(nd.b) + dag.numel(k));
            const int Pn = dag.Pk(k), PL = dag.Pk(nd.a);
            // a common Group dim: (image, group) pairs are independent, each blends [CL/G, TL] onto [CR/G, TR]
            const int Gb = nd.bgroups;
            // lhs=pixels: the [H*W, 1, 1, 1] LHS is a one-channel full-size tensor to the kernel
            const int CLk = nd.lhs_pixels ? 1 : A.C / Gb, TLk = nd.lhs_pixels ? 1 : A.T, PLk = nd.lhs_pixels ? Pn : PL;
            // an LHS that has folded away one spatial dim the result still has is replicated along it
            const int lost = A.pooled & ~nd.pooled, Wd = dag.Wk(k);
            const int rep = nd.lhs_pixels || lost == 3 || lost == 0 ? 0 : lost;
            L.run = [=](const RunArgs& a) {
                ref::binary_fwd(val(a, nd.a), val(a, nd.b), valw(a, k), N * Gb, CLk, TLk, B.C / Gb, B.T, Pn, PLk, rep, Wd, nd.kind, a.stream);
            };
            break;
        }
        case Op::Group: {  // (live only as the output: a copy of the viewed tensor)
            int64_t ne = dag.numel(k);
            L.run = [=](const RunArgs& a) { ref::copy_f32(val(a, nd.a), valw(a, k), ne, a.stream); };
            break;
        }
        case Op::Softmax:
            {
                const int Pn = dag.Pk(k);
                if (nd.kind >= kAxisH) {  // rows of every (image, channel, tap) plane: along W or the whole plane contiguous, along H strided by W
                    const int Hn = dag.Hk(k), Wn = dag.Wk(k);
                    const int len = nd.kind == kAxisH ? Hn : (nd.kind == kAxisW ? Wn : Hn * Wn), inner = nd.kind == kAxisH ? Wn : 1;
                    const int64_t rows = (int64_t)N * nd.C * nd.T * Pn / len;
                    L.run = [=](const RunArgs& a) { ref::softmax_rows_fwd(val(a, nd.a), valw(a, k), rows, len, inner, a.stream); };
                    break;
                }
                L.run = [=](const RunArgs& a) { ref::softmax_fwd(val(a, nd.a), valw(a, k), N, nd.C, nd.T, Pn, nd.kind == kAxisCT ? 2 : (nd.kind == kAxisC ? 1 : 0), a.stream); };
            }
            break;
        case Op::Fold:
            if (nd.axis_c) {
                const int64_t TP = (int64_t)A.T * dag.Pk(nd.a);
                const int Cg = A.C / nd.groups;
                L.name = "node_cfold_fwd";
                L.run = [=](const RunArgs& a) { ref::cfold_fwd(val(a, nd.a), valw(a, k), N * nd.groups, Cg, TP, nd.kind, a.stream); };
            } else if (nd.axis_hw == 1) {
                // over H alone: the H rows of a plane are "channels" of Wi elements each to the channel-fold kernel
                const int Hi = dag.Hk(nd.a), Wi = dag.Wk(nd.a);
                L.name = "node_hfold_fwd";
                L.run = [=](const RunArgs& a) { ref::cfold_fwd(val(a, nd.a), valw(a, k), N * A.C * A.T, Hi, Wi, nd.kind, a.stream); };
            } else if (nd.axis_hw) {
                // over W alone: every image row is a plane of Wi pixels; over both: every (channel, tap) plane
                const int Hi = dag.Hk(nd.a), Wi = dag.Wk(nd.a);
                const int64_t rows = N * A.C * A.T * (nd.axis_hw == 2 ? Hi : 1);
                const int len = nd.axis_hw == 2 ? Wi : Hi * Wi;
                L.name = "node_pool_fwd";
                L.run = [=](const RunArgs& a) { ref::pool_fwd(val(a, nd.a), valw(a, k), rows, len, nd.kind, a.stream); };
            } else {
                const int Pn = dag.Pk(k);
                L.run = [=](const RunArgs& a) { ref::fold_fwd(val(a, nd.a), valw(a, k), N * A.C, A.T, Pn, nd.kind, a.stream); };
            }
            break;
        default: break;
        }
        low->fwd.push_back(std::move(L));
    }
    if (!y_direct) {
        int64_t ne = dag.numel(dag.out);
        int o = dag.out;
        if (bf16) low->fwd.push_back({"narrow_y", ne * 6.0, 0, [=](const RunArgs& a) { ref::narrow_bf16(val(a, o), a.y, ne, a.stream); }});
        else low->fwd.push_back({"copy_y", ne * 8.0, 0, [=](const RunArgs& a) { ref::copy_f32(val(a, o), (float*)a.y, ne, a.stream); }});
    }

    // --------------------------------------------------------------- backward
    std::vector<bool> written(n, false);
    if (!y_direct) {
        int64_t ne = dag.numel(dag.out);
        int o = dag.out;
        if (bf16) low->bwd.push_back({"widen_dy", ne * 6.0, 0, [=](const RunArgs& a) { ref::widen_bf16(a.dy, grad(a, o), ne, a.stream); }});
        else low->bwd.push_back({"copy_dy", ne * 8.0, 0, [=](const RunArgs& a) { ref::copy_f32((const float*)a.dy, grad(a, o), ne, a.stream); }});
        written[o] = true;
    }
    for (int ui = (int)units.size() - 1; ui >= 0; ui--) {
        const Unit& U = units[ui];
        if (U.chain) {
            chain::Program pg = U.plan.bwd;
            const std::vector<Binding> b = bind(U.plan.bwd_ext);
            for (size_t i = 0; i < b.size(); i++)
                if (b[i].role == chain::kGradOut) {
                    // the first writer of a gradient overwrites, later ones add (fp32 buffers only)
                    if (written[b[i].node]) pg.ins[U.plan.bwd_ext[i].store_instr].kind |= chain::kStAdd;
                    written[b[i].node] = true;
                }
            low->bwd.push_back({"chain_bwd", ext_bytes(b), 0, [=](const RunArgs& a) { run_program(pg, b, bf16, a); }});
            continue;
        }
        const int k = U.nodes[0];
        const Node nd = dag.nodes[k];
        const Node A = dag.nodes[nd.a];
        if (nd.op == Op::Fc && fc_mfma[k]) {
            const int srcn = fc_src(k), widx = nd.widx;
            const bool src_x = srcn == 0;
            const bool from_dy = k == dag.out && y_direct;   // the output node: its gradient is the caller's dy
            const bool to_dx = src_x && dx_direct;           // the only writer of dx: written in place, in bf16
            const int acc_s = written[srcn] ? 1 : 0;
            const double flops = 2.0 * N * P * nd.out * (double)(wnumel[widx] / nd.out);
            // weight gradient: partial sums over slices of the (image, pixel) range, then a fixed-order sum
            const gfc::Params Q = wgrad_params(k);
            const int64_t poff = lay.part[widx], toff = lay.wt[widx];
            const int64_t nw = wnumel[widx];
            const int slices = gfc::wgrad_partials(Q);
            low->bwd.push_back({Q.TV > 1 ? "gfc_wgrad_unfold" : "gfc_wgrad", (src_x ? 2.0 : 4.0) * dag.numel(srcn) + 4.0 * dag.numel(k) + 4.0 * slices * nw, flops,
                                [=](const RunArgs& a) {
                                    gfc::Params R = Q;
                                    R.src = src_x ? a.x : (const void*)val(a, srcn);
                                    R.dy = from_dy ? a.dy : (const void*)grad(a, k);
                                    R.partial = (float*)(a.ws + poff);
                                    gfc::wgrad_partial(R, a.stream);
                                }});
            ReduceJob rj;  // (one launch at the end of the backward pass sums the partials of every FC)
            rj.job.slices = slices;
            rj.job.kind = 0;
            rj.job.count = (unsigned)nw;
            wreduce::plan(rj.job);
            rj.widx = widx;
            rj.off = poff;
            rj.bytes = 4.0 * (slices + 1) * nw;
            low->rjobs.push_back(rj);
            // data gradient: the same contraction on dy with transposed, tap-flipped weights; it writes the
            // gradient of the FC's source tensor directly (the Unfold adjoint is part of it)
            gfc::Params D = gfc::data_gradient_of(Q);
            const int Rrows = Q.R, Og = Q.Og;
            D.src_f32 = from_dy ? 0 : 1;
            D.dst_f32 = to_dx ? 0 : 1;
            D.acc = to_dx ? 0 : acc_s;
            const int G = nd.groups, TV = D.TV;
            low->bwd.push_back({"gfc_transpose_w", 4.0 * nw, 0, [=](const RunArgs& a) {
                                    gfc::transpose_weights((const uint16_t*)a.w[widx], (uint16_t*)(a.ws + toff), G, Og, Rrows, TV, a.stream);
                                }});
            low->bwd.push_back({TV > 1 ? "gfc_dgrad_unfold" : "gfc_dgrad", 4.0 * dag.numel(k) + 4.0 * dag.numel(srcn) * (1 + acc_s) + 2.0 * nw, flops,
                                [=](const RunArgs& a) {
                                    gfc::Params R = D;
                                    R.src = from_dy ? a.dy : (const void*)grad(a, k);
                                    R.w = (const uint16_t*)(a.ws + toff);
                                    R.dst = to_dx ? a.dx : (void*)grad(a, srcn);
                                    gfc::forward(R, a.stream);
                                }});
            written[srcn] = true;
            continue;
        }
        const int acc = written[nd.a] ? 1 : 0;
        Launch L;
        L.name = std::string("node_") + op_name(nd.op) + "_bwd";
        L.bytes = 4.0 * (dag.numel(nd.a) * (1 + acc) + dag.numel(k));
        switch (nd.op) {
        case Op::Unfold:
            L.run = [=](const RunArgs& a) { ref::unfold_bwd(grad(a, k), grad(a, nd.a), N * A.C, A.T, nd.kh, nd.kw, dag.H, dag.W, acc, a.stream); };
            break;
        case Op::Shift:
            L.run = [=](const RunArgs& a) {
                ref::shift(grad(a, k), grad(a, nd.a), N, nd.C, nd.T, dag.H, dag.W, -nd.dh, -nd.dw, nd.c0, nd.c1, acc, a.stream);
            };
            break;
        case Op::Fc: {
            int G = nd.groups, Og = nd.out / G, K = (A.C / G) * A.T;
            Launch D;
            D.name = "node_fc_dw";
            const int Pn = dag.Pk(k);
            D.flops = 2.0 * N * Pn * nd.out * K;
            D.bytes = 4.0 * (dag.numel(nd.a) + dag.numel(k) + wnumel[nd.widx]);
            D.run = [=](const RunArgs& a) { ref::fc_dw(grad(a, k), val(a, nd.a), (float*)a.dw[nd.widx], N, G, Og, K, Pn, a.stream); };
            low->bwd.push_back(std::move(D));
            L.name = "node_fc_dx";
            L.flops = 2.0 * N * Pn * nd.out * K;
            L.bytes += 4.0 * wnumel[nd.widx];
            L.run = [=](const RunArgs& a) { ref::fc_dx(grad(a, k), wptr(a, nd.widx), grad(a, nd.a), N, G, Og, K, Pn, acc, a.stream); };
            break;
        }
        case Op::Unary: {
            int64_t ne = dag.numel(k);
            L.bytes += 4.0 * ne;
            L.run = [=](const RunArgs& a) { ref::unary_bwd(val(a, nd.a), grad(a, k), grad(a, nd.a), ne, nd.kind, nd.lo, nd.hi, acc, a.stream); };
            break;
        }
        case Op::Binary: {
            const Node B = dag.nodes[nd.b];
            // LHS first, then RHS (which may be the same tensor and then accumulates)
            L.name = "node_binary_bwd_lhs";
            L.bytes = 4.0 * (dag.numel(nd.a) * (1 + acc) + dag.numel(k) * (nd.kind == kAdd || nd.kind == kSub ? 1 : 2));
            const int Pn = dag.Pk(k), PL = dag.Pk(nd.a), Gb = nd.bgroups;
            const int CLk = nd.lhs_pixels ? 1 : A.C / Gb, TLk = nd.lhs_pixels ? 1 : A.T, PLk = nd.lhs_pixels ? Pn : PL;
            const int lost = A.pooled & ~nd.pooled, Wd = dag.Wk(k);
            const int rep = nd.lhs_pixels || lost == 3 || lost == 0 ? 0 : lost;
            L.run = [=](const RunArgs& a) {
                ref::binary_bwd_lhs(val(a, nd.a), val(a, nd.b), grad(a, k), grad(a, nd.a), N * Gb, CLk, TLk, B.C / Gb, B.T, Pn, PLk, rep, Wd, nd.kind, acc, a.stream);
            };
            low->bwd.push_back(std::move(L));
            written[nd.a] = true;
            const int acc_r = written[nd.b] ? 1 : 0;
            Launch R;
            R.name = "node_binary_bwd_rhs";
            R.bytes = 4.0 * (dag.numel(nd.b) * (1 + acc_r) + dag.numel(k) + (nd.kind == kAdd || nd.kind == kSub ? 0 : dag.numel(nd.a)));
            R.run = [=](const RunArgs& a) {
                ref::binary_bwd_rhs(val(a, nd.a), val(a, nd.b), grad(a, k), grad(a, nd.b), N * Gb, CLk, TLk, B.C / Gb, B.T, Pn, PLk, rep, Wd, nd.kind, acc_r, a.stream);
            };
            low->bwd.push_back(std::move(R));
            written[nd.b] = true;
            continue;
        }
        case Op::Group: {  // a shift by nothing: copies, or adds to, the gradient of the viewed tensor
            const int Pn = dag.Pk(k);
            L.run = [=](const RunArgs& a) { ref::shift(grad(a, k), grad(a, nd.a), N, nd.C, nd.T, 1, Pn, 0, 0, 0, 0, acc, a.stream); };
            break;
        }
        case Op::Softmax:
            L.bytes += 4.0 * dag.numel(k);
            {
                const int Pn = dag.Pk(k);
                if (nd.kind >= kAxisH) {
                    const int Hn = dag.Hk(k), Wn = dag.Wk(k);
                    const int len = nd.kind == kAxisH ? Hn : (nd.kind == kAxisW ? Wn : Hn * Wn), inner = nd.kind == kAxisH ? Wn : 1;
                    const int64_t rows = (int64_t)N * nd.C * nd.T * Pn / len;
                    L.run = [=](const RunArgs& a) { ref::softmax_rows_bwd(val(a, k), grad(a, k), grad(a, nd.a), rows, len, inner, acc, a.stream); };
                    break;
                }
                L.run = [=](const RunArgs& a) { ref::softmax_bwd(val(a, k), grad(a, k), grad(a, nd.a), N, nd.C, nd.T, Pn, nd.kind == kAxisCT ? 2 : (nd.kind == kAxisC ? 1 : 0), acc, a.stream); };
            }
            break;
        case Op::Fold:
            L.bytes += 4.0 * dag.numel(nd.a);
            if (nd.axis_c) {
                const int64_t TP = (int64_t)A.T * dag.Pk(nd.a);
                const int Cg = A.C / nd.groups;
                L.name = "node_cfold_bwd";
                L.run = [=](const RunArgs& a) { ref::cfold_bwd(val(a, nd.a), grad(a, k), grad(a, nd.a), N * nd.groups, Cg, TP, nd.kind, acc, a.stream); };
            } else if (nd.axis_hw == 1) {
                const int Hi = dag.Hk(nd.a), Wi = dag.Wk(nd.a);
                L.name = "node_hfold_bwd";
                L.run = [=](const RunArgs& a) { ref::cfold_bwd(val(a, nd.a), grad(a, k), grad(a, nd.a), N * A.C * A.T, Hi, Wi, nd.kind, acc, a.stream); };
            } else if (nd.axis_hw) {
                const int Hi = dag.Hk(nd.a), Wi = dag.Wk(nd.a);
                const int64_t rows = N * A.C * A.T * (nd.axis_hw == 2 ? Hi : 1);
                const int len = nd.axis_hw == 2 ? Wi : Hi * Wi;
                L.name = "node_pool_bwd";
                L.run = [=](const RunArgs& a) { ref::pool_bwd(val(a, nd.a), grad(a, k), grad(a, nd.a), rows, len, nd.kind, acc, a.stream); };
            } else {
                const int Pn = dag.Pk(k);
                L.run = [=](const RunArgs& a) { ref::fold_bwd(val(a, nd.a), grad(a, k), grad(a, nd.a), N * A.C, A.T, Pn, nd.kind, acc, a.stream); };
            }
            break;
        default: break;
        }
        low->bwd.push_back(std::move(L));
        written[nd.a] = true;
    }
    for (int i = 0; i < dag.n_weights; i++) {
        if (dag.nodes[dag.weight_node[i]].live) continue;
        int64_t nw = wnumel[i];  // an fc the output does not depend on has a zero weight gradient
        low->bwd.push_back({"zero_dw", nw * 4.0, 0, [=](const RunArgs& a) { ref::fill_f32((float*)a.dw[i], 0.f, nw, a.stream); }});
    }
    if (!dx_direct) {
        int64_t ne = dag.numel(0);
        if (bf16) low->bwd.push_back({"narrow_dx", ne * 6.0, 0, [=](const RunArgs& a) { ref::narrow_bf16(grad(a, 0), a.dx, ne, a.stream); }});
        else low->bwd.push_back({"copy_dx", ne * 8.0, 0, [=](const RunArgs& a) { ref::copy_f32(grad(a, 0), (float*)a.dx, ne, a.stream); }});
    }
    (void)esz;
    return low;
}

}  // namespace canvas
