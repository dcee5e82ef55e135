// Planner of the fused-chain kernels (host only).
//
// The unit's nodes are first expanded into an instance graph: an instance is "the value of node k as seen through a
// position context", the context being the stencil offsets (Shift terms, at most one Unfold window) collected on the
// way down from a consumer.  A Shift or Unfold node itself only adds to the context of its operand and masks what
// falls outside the image; the loads at the leaves carry the total offset.  Reductions (Fold, Softmax) are only
// legal in the empty context: a stencil above a reduction would need the reduction's result at other pixels.
// Code is then emitted by demand-driven recursion, with full recomputation instead of saved values: forward
// emit_eval(instance), backward emit_grad(instance) = sum over its users of their local adjoint applied to
// emit_grad(user).  A Softmax over channels splits a program into passes over the channel range (statistics first;
// in the backward program also the sum of gradient x output that its adjoint needs).
#include "chain_plan.hpp"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <functional>
#include <map>
#include <memory>
#include <set>
#include <sstream>
#include <tuple>

#include "chain_kernels.hpp"

namespace canvas {
namespace chain {

namespace {

struct Fail {
    std::string why;
};

struct Ctx {
    std::vector<Term> terms;
    bool win = false;
    int kh = 1, kw = 1;
    bool empty() const { return terms.empty() && !win; }
    std::string key() const {
        std::ostringstream os;
        for (const Term& t : terms) os << t.dh << ',' << t.dw << ',' << t.c0 << ',' << t.c1 << ';';
        if (win) os << 'w' << kh << 'x' << kw;
        return os.str();
    }
    // how far (in pixels of the flattened plane) a read through this context can lie from the reading pixel
    int64_t reach_px(int W) const {
        int64_t r = win ? (int64_t)(kh / 2) * W + kw / 2 : 0;
        for (const Term& t : terms) r += (int64_t)std::abs((int)t.dh) * W + std::abs((int)t.dw);
        return r;
    }
};

enum InstKind { kExt, kIdent, kStencil, kUnaryI, kBinaryI, kSmT, kSmC, kFoldI, kBoxAdj };

struct Inst {
    int node = -1, ctx = 0, lanes = 1;
    InstKind kind = kExt;
    int opnd[2] = {-1, -1};
    std::vector<std::pair<int, int>> users;  // (instance, operand slot)
    int aux = -1;                            // kBoxAdj: the context of the window (see Graph::add_box_adjoints)
    int level = 0;                           // softmax-over-channels instances at or below this one (longest chain)
    int down = -1;                           // such instances above it (memo)
};

class Graph {
   public:
    Graph(const Dag& d, const std::vector<bool>& in_unit, const std::vector<bool>& is_output)
        : dag(d), in_unit_(in_unit), is_output_(is_output) {
        ctxs.push_back(Ctx());
        ctx_ids[""] = 0;
    }

    int ctx_id(const Ctx& c) {
        const std::string k = c.key();
        auto it = ctx_ids.find(k);
        if (it != ctx_ids.end()) return it->second;
        ctxs.push_back(c);
        return ctx_ids[k] = (int)ctxs.size() - 1;
    }

    int natural_lanes(int node, int ctx) const { return ctxs[ctx].win ? ctxs[ctx].kh * ctxs[ctx].kw : dag.nodes[node].T; }

    // the instance of `node` in context `ctx`; want > 0: an external tensor with fewer taps is read with lane t -> tap t % T
    int build(int node, int ctx, int want = 0) {
        const Node& nd = dag.nodes[node];
        if (ctxs[ctx].win && nd.T != 1) throw Fail{"a window over a tensor that has taps"};
        int lanes = natural_lanes(node, ctx);
        const bool external = !in_unit_[node];
        if (external && want > lanes && lanes > 1) {
            if (want % lanes) throw Fail{"tap counts of a blend do not divide"};
            lanes = want;
        }
        const auto key = std::make_tuple(node, ctx, lanes);
        auto it = memo.find(key);
        if (it != memo.end()) return it->second;
        Inst I;
        I.node = node;
        I.ctx = ctx;
        I.lanes = lanes;
        if (external) {
            I.kind = kExt;
            return add(key, I);
        }
        const bool reduction = nd.op == Op::Softmax || nd.op == Op::Fold;
        if (reduction && !ctxs[ctx].empty()) throw Fail{"a stencil above a reduction"};
        switch (nd.op) {
        case Op::Unfold: {
            if (ctxs[ctx].win) throw Fail{"nested windows"};
            Ctx c2 = ctxs[ctx];
            c2.win = true;
            c2.kh = nd.kh;
            c2.kw = nd.kw;
            I.kind = kStencil;
            I.opnd[0] = build(nd.a, ctx_id(c2));
            break;
        }
        case Op::Shift: {
            if ((nd.dh == 0 && nd.dw == 0) || nd.c0 >= nd.c1) {
                I.kind = kIdent;
                I.opnd[0] = build(nd.a, ctx);
            } else {
                Ctx c2 = ctxs[ctx];
                Term t;
                t.dh = (int16_t)nd.dh;
                t.dw = (int16_t)nd.dw;
                t.c0 = (uint16_t)nd.c0;
                t.c1 = (uint16_t)nd.c1;
                c2.terms.push_back(t);
                I.kind = kStencil;
                I.opnd[0] = build(nd.a, ctx_id(c2));
            }
            break;
        }
        case Op::Unary:
            I.kind = kUnaryI;
            I.opnd[0] = build(nd.a, ctx);
            break;
        case Op::Softmax:
            I.kind = nd.kind == kAxisC ? kSmC : kSmT;
            I.opnd[0] = build(nd.a, ctx);
            break;
        case Op::Fold:
            I.kind = kFoldI;
            I.opnd[0] = build(nd.a, ctx);
            break;
        case Op::Binary: {
            I.kind = kBinaryI;
            I.opnd[1] = build(nd.b, ctx);
            const int tr = insts[I.opnd[1]].lanes;
            if (tr != lanes) throw Fail{"blend: RHS lanes"};
            I.opnd[0] = build(nd.a, ctx, tr);
            const int tl = insts[I.opnd[0]].lanes;
            if (tl != 1 && tl != tr) throw Fail{"blend: an LHS inside the unit with fewer taps than the RHS"};
            break;
        }
        default: throw Fail{"not a chain primitive"};
        }
        return add(key, I);
    }

    int add(const std::tuple<int, int, int>& key, Inst I) {
        int lvl = 0;
        for (int s = 0; s < 2; s++)
            if (I.opnd[s] >= 0) lvl = std::max(lvl, insts[I.opnd[s]].level);
        I.level = lvl + (I.kind == kSmC ? 1 : 0);
        insts.push_back(I);
        const int id = (int)insts.size() - 1;
        for (int s = 0; s < 2; s++)
            if (I.opnd[s] >= 0) insts[I.opnd[s]].users.push_back({id, s});
        memo[key] = id;
        return id;
    }

    // Unfold followed at once by a sum / avg Fold that is an output of the unit and feeds nothing inside it is a linear
    // operator on the unfolded tensor's source (a box filter); its adjoint is the same filter applied to the incoming
    // gradient (the window is symmetric), which the pixel reads itself: a window load of dy and a fold, no hand-over of
    // T lanes to the neighbours.  Where EVERY Unfold of the unit is of that kind, each gets a pseudo user of its source's
    // own-pixel instance that stands for this adjoint in the backward program, and the leaves read through windows drop
    // out of it.  Returns whether that is so.
    bool add_box_adjoints() {
        std::vector<std::pair<int, int>> pairs;  // (unfold instance, fold instance)
        for (size_t i = 0; i < insts.size(); i++) {
            const Inst& U = insts[i];
            if (U.kind != kStencil || dag.nodes[U.node].op != Op::Unfold) continue;
            if (U.users.size() != 1) return false;
            const Inst& F = insts[U.users[0].first];
            const Node& fn = dag.nodes[F.node];
            if (F.kind != kFoldI || (fn.kind != kSum && fn.kind != kAvg) || !F.users.empty() || !is_output_[F.node] || F.ctx != 0 || U.ctx != 0)
                return false;
            pairs.push_back({(int)i, U.users[0].first});
        }
        if (pairs.empty()) return false;
        for (const auto& pr : pairs) {
            const int win_ctx = insts[insts[pr.first].opnd[0]].ctx;
            const int src = build(dag.nodes[insts[pr.first].node].a, insts[pr.first].ctx);
            if (insts[src].lanes != 1) throw Fail{"internal: the source of an unfold with taps"};
            Inst B;
            B.node = insts[pr.second].node;
            B.ctx = insts[pr.first].ctx;
            B.lanes = 1;
            B.kind = kBoxAdj;
            B.opnd[0] = src;
            B.aux = win_ctx;
            add(std::make_tuple(-1 - B.node, B.ctx, 1), B);
        }
        return true;
    }

    // softmax-over-channels instances on the longest way from instance i up to an output (i itself not counted)
    int down(int i) {
        if (insts[i].down >= 0) return insts[i].down;
        int d = 0;
        for (auto& u : insts[i].users) d = std::max(d, down(u.first) + (insts[u.first].kind == kSmC ? 1 : 0));
        return insts[i].down = d;
    }

    const Dag& dag;
    int root_ctx = 0;  // the context the unit's outputs are built in (not the empty one for a displaced unit)
    std::vector<Ctx> ctxs;
    std::map<std::string, int> ctx_ids;
    std::vector<Inst> insts;
    std::map<std::tuple<int, int, int>, int> memo;
    std::vector<bool> in_unit_, is_output_;
};

class Emitter {
   public:
    Emitter(Graph& g, int tm) : G(&g), NR(regs_for(tm)), used(regs_for(tm), false) { pg.tm = tm; }

    // Instructions may come from several instance graphs (the unit as it is, and the unit displaced by a stencil's
    // offsets: see compile_unit); `gidx` tells their instances apart in the tables below.
    void use(Graph& g, int idx) {
        G = &g;
        gidx = idx;
    }
    int gkey(int v) const { return gidx * (1 << 20) + v; }

    void emit(const Instr& I) {
        if (pg.n_instr >= kMaxInstr) throw Fail{"too many instructions"};
        pg.ins[pg.n_instr++] = I;
    }
    int alloc() {
        for (int r = 0; r < NR; r++)
            if (!used[r]) {
                used[r] = true;
                pg.n_regs = std::max(pg.n_regs, r + 1);
                return r;
            }
        throw Fail{"out of registers"};
    }
    void release(int r) { used[r] = false; }
    int persist(int n) {
        const int a = pg.n_persist;
        pg.n_persist += n;
        return a;
    }
    int ext_slot(int node, ExtRole role) {
        for (size_t i = 0; i < ext.size(); i++)
            if (ext[i].node == node && ext[i].role == role) return (int)i;
        if ((int)ext.size() >= kMaxExt) throw Fail{"too many external tensors"};
        ExtRef e;
        e.node = node;
        e.role = role;
        ext.push_back(e);
        pg.ext[ext.size() - 1].T = G->dag.nodes[node].T;
        pg.n_ext = (int)ext.size();
        return (int)ext.size() - 1;
    }
    uint16_t terms(int ctx) {
        auto it = term_of.find(gkey(ctx));
        if (it != term_of.end()) return it->second;
        const Ctx& c = G->ctxs[ctx];
        if (pg.n_terms + (int)c.terms.size() > kMaxTerms) throw Fail{"too many stencil offsets"};
        const int first = pg.n_terms;
        for (const Term& t : c.terms) pg.term[pg.n_terms++] = t;
        return term_of[gkey(ctx)] = (uint16_t)((first << 8) | (int)c.terms.size());
    }
    Instr positional(Opcode op, int ctx, int lanes) {
        Instr I;
        I.op = op;
        I.T = (uint8_t)lanes;
        I.b = terms(ctx);
        const Ctx& c = G->ctxs[ctx];
        if (c.win) {
            I.kind |= kWin;
            I.r = (uint8_t)((c.kh << 4) | c.kw);
        }
        return I;
    }
    // OP_BINLD: A (lanes) blended with the external instance i, read in place (its own lanes: `lanes`, or 1 replicated)
    Instr load_and_blend(int i, int lanes, int blend, bool loaded_is_lhs) {
        const Inst& L = G->insts[i];
        Instr I = positional(OP_BINLD, L.ctx, lanes);
        I.a = (uint16_t)ext_slot(L.node, kValueIn);
        if (G->dag.nodes[L.node].T > 1) I.kind |= kExtTaps;
        I.kind |= (uint8_t)(blend << kBinLdKindShift);
        if (loaded_is_lhs) I.kind |= kBinLdLoadedIsLhs;
        if (L.lanes == 1 && lanes > 1) I.kind |= kBinLdLoadedScalar;
        return I;
    }
    static Instr simple(Opcode op, int T, int r = 0, int kind = 0, int a = 0) {
        Instr I;
        I.op = op;
        I.T = (uint8_t)T;
        I.r = (uint8_t)r;
        I.kind = (uint8_t)kind;
        I.a = (uint16_t)a;
        return I;
    }

    // ---------------------------------------------------------------- values kept for another use
    // A value (key 2 * instance) or a gradient (key 2 * instance + 1) that `keep` names is stored in a register the
    // first time a pass body computes it and fetched from there afterwards.  `stats` records, per key, how often it was
    // computed and how many instructions one computation took: what the choice of `keep` is made from.
    struct Stat {
        int computed = 0, cost = 0;
    };
    void cached(int key0, int lanes, void (Emitter::*raw)(int), int i) {
        const int key = gkey(key0);
        auto it = held.find(key);
        if (it != held.end()) {
            emit(simple(OP_MOVA, lanes, it->second));
            return;
        }
        const int before = pg.n_instr;
        (this->*raw)(i);
        Stat& st = stats[key];
        st.computed++;
        st.cost = std::max(st.cost, pg.n_instr - before);
        if (keep.count(key)) {
            const int r = alloc();
            emit(simple(OP_MOVR, lanes, r));
            held[key] = r;
        }
    }
    void forget_graph(int idx) {  // (what a displaced copy kept is of no use to the next one)
        for (auto it = held.begin(); it != held.end();) {
            if (it->first / (1 << 20) == idx) {
                release(it->second);
                it = held.erase(it);
            } else {
                ++it;
            }
        }
    }
    void forget() {  // (a register's content does not outlive the body it was written in)
        for (auto& kv : held) release(kv.second);
        held.clear();
    }
    void eval(int i) { cached(2 * i, G->insts[i].lanes, &Emitter::eval_raw, i); }
    void grad(int i) { cached(2 * i + 1, G->insts[i].lanes, &Emitter::grad_raw, i); }

    // ---------------------------------------------------------------- forward values
    void eval_raw(int i) {
        const Inst& I = G->insts[i];
        const Node& nd = G->dag.nodes[I.node];
        switch (I.kind) {
        case kExt: {
            Instr ld = positional(OP_LD, I.ctx, I.lanes);
            ld.a = (uint16_t)ext_slot(I.node, kValueIn);
            if (nd.T > 1) ld.kind |= kExtTaps;
            emit(ld);
            break;
        }
        case kIdent: eval(I.opnd[0]); break;
        case kStencil: {
            eval(I.opnd[0]);
            const Inst& S = G->insts[I.opnd[0]];
            if (S.kind != kExt) emit(positional(OP_MASK, S.ctx, I.lanes));  // (a load checks its own position)
            break;
        }
        case kUnaryI: {
            eval(I.opnd[0]);
            Instr u = simple(OP_UN, I.lanes, 0, nd.kind);
            u.f0 = nd.lo;
            u.f1 = nd.hi;
            emit(u);
            break;
        }
        case kBinaryI: {
            const int tl = G->insts[I.opnd[0]].lanes;
            if (G->insts[I.opnd[0]].kind == kExt) {  // the LHS comes straight from memory
                eval(I.opnd[1]);
                emit(load_and_blend(I.opnd[0], I.lanes, nd.kind, true));
                break;
            }
            if (G->insts[I.opnd[1]].kind == kExt && tl == I.lanes) {  // the RHS does
                eval(I.opnd[0]);
                emit(load_and_blend(I.opnd[1], I.lanes, nd.kind, false));
                break;
            }
            eval(I.opnd[0]);
            const int r = alloc();
            emit(simple(OP_MOVR, tl, r));
            eval(I.opnd[1]);
            emit(simple(OP_BIN, I.lanes, r, nd.kind | kBinRegIsLhs | (tl == 1 && I.lanes > 1 ? kBinRegScalar : 0)));
            release(r);
            break;
        }
        case kSmT:
            eval(I.opnd[0]);
            emit(simple(OP_SMT, I.lanes));
            break;
        case kSmC:
            eval(I.opnd[0]);
            emit(simple(OP_SMCAPPLY, I.lanes, 0, 0, stat_slot(i)));
            break;
        case kFoldI:
            eval(I.opnd[0]);
            emit(simple(OP_FOLD, G->insts[I.opnd[0]].lanes, 0, nd.kind));
            break;
        case kBoxAdj: throw Fail{"internal: the value of a box adjoint"};
        }
    }

    int stat_slot(int i) {
        auto it = stat_slots.find(i);
        if (it != stat_slots.end()) return it->second;
        return stat_slots[i] = persist(2 * G->insts[i].lanes);
    }
    int dot_slot(int i) {
        auto it = dot_slots.find(i);
        if (it != dot_slots.end()) return it->second;
        return dot_slots[i] = persist(G->insts[i].lanes);
    }

    // ---------------------------------------------------------------- gradients
    // leaves d loss / d instance i in A (lanes of i)
    void grad_raw(int i) {
        const Inst& I = G->insts[i];
        bool first = true;
        int held = -1;
        auto begin_term = [&]() {
            if (!first) {
                held = alloc();
                emit(simple(OP_MOVR, I.lanes, held));
            }
        };
        auto end_term = [&]() {
            if (!first) {
                emit(simple(OP_BIN, I.lanes, held, kAdd | kBinRegIsLhs));
                release(held);
            }
            first = false;
        };
        if (I.kind != kExt && I.ctx == G->root_ctx && G->is_output_[I.node] && I.lanes == G->dag.nodes[I.node].T) {
            begin_term();
            Instr ld = positional(OP_LD, G->root_ctx, I.lanes);  // (a displaced unit reads the incoming gradient displaced)
            ld.a = (uint16_t)ext_slot(I.node, kGradIn);
            if (I.lanes > 1) ld.kind |= kExtTaps;
            emit(ld);
            end_term();
        }
        for (const auto& u : I.users) {
            begin_term();
            contribution(u.first, u.second, i);
            end_term();
        }
        if (first) throw Fail{"internal: an instance without users"};
    }

    // d loss / d (operand `slot` of user instance u), which is instance i
    void contribution(int u, int slot, int i) {
        const Inst& U = G->insts[u];
        const Inst& I = G->insts[i];
        const Node& un = G->dag.nodes[U.node];
        if (U.kind == kBoxAdj) {  // the box filter's adjoint: the same filter over the incoming gradient of the fold's output
            const Ctx& wc = G->ctxs[U.aux];
            Instr ld = positional(OP_LD, U.aux, wc.kh * wc.kw);
            ld.a = (uint16_t)ext_slot(U.node, kGradIn);
            emit(ld);
            emit(simple(OP_FOLD, wc.kh * wc.kw, 0, un.kind));
            return;
        }
        grad(u);  // A = gradient of u, U.lanes lanes
        switch (U.kind) {
        case kIdent: break;
        case kStencil:
            if (I.kind != kExt) emit(positional(OP_MASK, I.ctx, U.lanes));
            break;
        case kUnaryI: {
            const int r = alloc();
            emit(simple(OP_MOVR, U.lanes, r));
            eval(i);
            Instr b = simple(OP_UNBX, U.lanes, r, un.kind);
            b.f0 = un.lo;
            b.f1 = un.hi;
            emit(b);
            release(r);
            break;
        }
        case kBinaryI: {
            const int other = U.opnd[1 - slot];
            const int tl = G->insts[U.opnd[0]].lanes;
            const bool lhs_scalar = tl == 1 && U.lanes > 1;
            if (un.kind == kAdd || (un.kind == kSub && slot == 0)) {
            } else if (un.kind == kSub) {
                emit(simple(OP_UN, U.lanes, 0, kUnNeg));
            } else if (un.kind == kMul && G->insts[other].kind == kExt) {
                // the gradient in A times the other operand, which comes straight from memory
                emit(load_and_blend(other, U.lanes, kMul, false));
            } else if (un.kind == kMul) {
                const int r = alloc();
                emit(simple(OP_MOVR, U.lanes, r));
                eval(other);
                // A (the other operand) times the gradient in R[r]; the other operand is a scalar when it is the 1-lane LHS
                emit(simple(OP_BIN, U.lanes, r, kMul | (slot == 1 && lhs_scalar ? kBinAccScalar : 0)));
                release(r);
            } else {  // min / max: the indicator needs both operands
                const int rg = alloc();
                emit(simple(OP_MOVR, U.lanes, rg));
                eval(U.opnd[0]);
                const int rl = alloc();
                emit(simple(OP_MOVR, tl, rl));
                eval(U.opnd[1]);
                emit(simple(OP_BING, U.lanes, rl, un.kind | (slot == 1 ? kBingRhsSide : 0) | (lhs_scalar ? kBingLhsScalar : 0)));
                emit(simple(OP_BIN, U.lanes, rg, kMul));
                release(rl);
                release(rg);
            }
            if (slot == 0 && lhs_scalar) emit(simple(OP_FOLD, U.lanes, 0, kSum));  // the replicated LHS collects all lanes
            break;
        }
        case kSmT: {
            const int r = alloc();
            emit(simple(OP_MOVR, U.lanes, r));
            eval(u);
            emit(simple(OP_SMTBX, U.lanes, r));
            release(r);
            break;
        }
        case kSmC: {
            const int r = alloc();
            emit(simple(OP_MOVR, U.lanes, r));
            eval(u);
            emit(simple(OP_SMCBX, U.lanes, r, 0, dot_slot(u)));
            release(r);
            break;
        }
        case kFoldI: {
            const int r = alloc();
            emit(simple(OP_MOVR, 1, r));
            if (un.kind == kMax) eval(i);
            emit(simple(OP_FOLDBX, I.lanes, r, un.kind));
            release(r);
            break;
        }
        case kBoxAdj: break;  // (handled above)
        case kExt: throw Fail{"internal: an external tensor as a user"};
        }
    }

    void begin_pass() {
        if (pg.n_pass >= kMaxPass) throw Fail{"too many passes"};
        pg.pass[pg.n_pass].pro_begin = (uint16_t)pg.n_instr;
        pg.pass[pg.n_pass].red_begin = pg.pass[pg.n_pass].red_end = (uint16_t)pg.n_red;
    }
    // a quantity of the current pass that runs across the channel loop (the slices of a workgroup combine it at the end)
    void reduce(int slot, int T, int kind) {
        if (pg.n_red >= kMaxRed) throw Fail{"too many reductions across channels"};
        Red r;
        r.slot = (uint16_t)slot;
        r.T = (uint8_t)T;
        r.kind = (uint8_t)kind;
        pg.red[pg.n_red++] = r;
        pg.pass[pg.n_pass].red_end = (uint16_t)pg.n_red;
    }
    void begin_body() { pg.pass[pg.n_pass].pro_end = pg.pass[pg.n_pass].body_begin = (uint16_t)pg.n_instr; }
    void end_pass() {
        pg.pass[pg.n_pass++].body_end = (uint16_t)pg.n_instr;
        forget();
    }

    // the passes that collect the statistics of every softmax over channels, lowest first
    void stat_passes(const std::vector<int>& smc) {
        int top = 0;
        for (int i : smc) top = std::max(top, G->insts[i].level);
        for (int lvl = 1; lvl <= top; lvl++) {
            begin_pass();
            for (int i : smc)
                if (G->insts[i].level == lvl) {
                    Instr m = simple(OP_PSET, G->insts[i].lanes, 0, 0, stat_slot(i));
                    m.f0 = -INFINITY;
                    emit(m);
                    emit(simple(OP_PSET, G->insts[i].lanes, 0, 0, stat_slot(i) + G->insts[i].lanes));
                    reduce(stat_slot(i), G->insts[i].lanes, 0);
                }
            begin_body();
            for (int i : smc)
                if (G->insts[i].level == lvl) {
                    eval(G->insts[i].opnd[0]);
                    emit(simple(OP_SMCSTAT, G->insts[i].lanes, 0, 0, stat_slot(i)));
                }
            end_pass();
        }
    }

    Graph* G;
    int gidx = 0;
    Program pg;
    std::vector<ExtRef> ext;
    int NR;
    std::vector<bool> used;
    std::map<int, uint16_t> term_of;
    std::map<int, int> stat_slots, dot_slots;
    std::set<int> keep;
    std::map<int, int> held;
    std::map<int, Stat> stats;
    std::map<int, int64_t> reach_of;  // per OP_XADD instruction: how far (in pixels) its sources can lie
};

int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Workgroup shape for V pixels per thread and `pt` threads per slice: tile and halo, channel range and slices.
// Returns the estimated cost of the launch (arbitrary units, see set_geometry) or a negative number when it does not fit.
double geometry_for(Program& pg, const Dag& dag, int C, int64_t reach_px, bool all_channels, int V, int pt, int trips) {
    const int HW = dag.H * dag.W;
    pg.vec = V;
    pg.unroll = unroll_for(pg.tm, V);
    const int PP = HW / V;                                   // pixel threads of a plane
    const int64_t HT = (reach_px + V - 1) / V;               // halo, in pixel threads
    const int per_thread = std::max<int>(1, (int)lds_bytes_per_thread(pg));
    const int cap = (int)(std::min<int64_t>(max_threads_for(pg.tm), (int64_t)kMaxLdsBytes / per_thread) / 64 * 64);
    if (cap < 64 || pt > cap || 2 * HT >= pt) return -1;
    int own = pt - 2 * (int)HT;
    if (own >= PP) {  // the whole plane in one tile
        if (ceil_div(PP + 2 * (int)HT, 64) * 64 != pt) return -1;  // (counted once, at its own size)
        own = PP;
    } else {
        own = ceil_div(PP, ceil_div(PP, own));  // tiles evened out over the plane
    }
    pg.pix_threads = pt;
    pg.own_threads = own;
    pg.halo_threads = (int)HT;
    pg.tiles = ceil_div(PP, own);
    // channel slices: the loads of different channels are independent, so threads are worth more than trips
    const int max_slices = std::max(1, cap / pt);
    if (all_channels) {
        pg.chunk = C;
        pg.chunks = 1;
        pg.slices = std::min(max_slices, std::min(ceil_div(C, pg.unroll), 16));
    } else {
        const int S = std::max(1, std::min(std::min(max_slices, 4), ceil_div(C, pg.unroll)));
        const int chunks = ceil_div(C, S * pg.unroll * trips);
        pg.chunk = ceil_div(C, chunks);
        pg.chunks = ceil_div(C, pg.chunk);
        pg.slices = std::min(S, ceil_div(pg.chunk, pg.unroll));
    }
    pg.threads = pg.slices * pg.pix_threads;
    if (lds_bytes(pg) > kMaxLdsBytes || (int64_t)dag.N * pg.tiles * pg.chunks >= ((int64_t)1 << 31)) return -1;
    // cost: trips of a thread x what a trip costs (a fixed part for fetching and dispatching the instructions, worth
    // about eight pixels of arithmetic, plus per channel the pixels and about four pixels' worth for its narrow memory
    // accesses) x how many times over the launch fills the chip (256 compute units, about 1024 resident threads each)
    const double trips_per_thread = (double)ceil_div(pg.chunk, pg.slices * pg.unroll);
    const double threads_total = (double)dag.N * pg.tiles * pg.chunks * pg.threads;
    // (the instances with 9 lanes x 4 pixels and with 25 lanes hold more than 128 vector registers: two wavefronts per
    // SIMD, not four)
    const double resident_threads = (pg.tm > 9 || (pg.tm > 1 && V >= 4)) ? 512.0 : 1024.0;
    const double wgs_per_cu = std::max(1.0, std::min(resident_threads / pg.threads, std::floor(160.0 * 1024.0 / (double)(lds_bytes(pg) + 4352))));
    // (whole rounds: a round that a few left-over workgroups make takes as long as a full one)
    const double rounds = std::max(1.0, std::ceil(threads_total / (256.0 * wgs_per_cu * pg.threads) - 0.05));
    // (a work item also costs its set-up: the thread's position, the pass headers; worth about 6 of these units)
    return (6.0 + trips_per_thread * (8.0 + (V + 4.0) * pg.unroll)) * rounds;
}

// Pixels per thread, threads per slice and trips per thread: whatever the estimate likes best.
void set_geometry(Program& pg, const Dag& dag, int C, int64_t reach_px, bool all_channels) {
    pg.N = dag.N;
    pg.C = C;
    pg.H = dag.H;
    pg.W = dag.W;
    pg.xadd_lanes = 0;
    for (int i = 0; i < pg.n_instr; i++)
        if (pg.ins[i].op == OP_XADD) pg.xadd_lanes = std::max<int>(pg.xadd_lanes, pg.ins[i].T);
    const int HW = dag.H * dag.W;
    Program best;
    double best_cost = -1;
    for (int V = max_vec_for(pg.tm); V >= 1; V /= 2) {
        if (HW % V != 0 || dag.W < V) continue;
        for (int pt = 64; pt <= max_threads_for(pg.tm); pt += 64)
            for (int trips = 1; trips <= (all_channels ? 1 : 8); trips *= 2) {
                Program q = pg;
                const double cost = geometry_for(q, dag, C, reach_px, all_channels, V, pt, trips);
                if (cost < 0) continue;
                if (best_cost < 0 || cost < best_cost * 0.999) {  // (ties: the wider vector, the smaller workgroup, fewer trips)
                    best_cost = cost;
                    best = q;
                }
            }
    }
    if (best_cost < 0) throw Fail{"tile, halo and persistent state do not fit one workgroup"};
    pg = best;
}

}  // namespace

bool chain_candidate(const Dag& dag, int k) {
    const Node& nd = dag.nodes[k];
    if (k == 0 || !nd.live || nd.pooled || nd.T > 25 || nd.C > 65535) return false;
    const Node& A = dag.nodes[nd.a];
    if (A.pooled || A.T > 25) return false;
    switch (nd.op) {
    case Op::Unfold: return A.T == 1 && nd.kh * nd.kw <= 25 && (nd.kw == 1 || nd.kw == 3 || nd.kw == 5);
    case Op::Shift: return std::abs(nd.dh) < 32768 && std::abs(nd.dw) < 32768;
    case Op::Unary: return true;
    case Op::Binary: {
        const Node& B = dag.nodes[nd.b];
        return nd.bgroups == 1 && !nd.lhs_pixels && !B.pooled && A.C == B.C && B.T <= 25 && B.T % A.T == 0;
    }
    // (a softmax over the channels of a tensor with taps stays a kernel of its own on the materialised tensor: each of
    // its passes over the channel range would evaluate the whole window again, and backward hands T lanes over per channel
    // and pass; measured on the 200 random DAGs such chains took 1.2-2.5 ms where the kernels per node take 0.1-0.4 ms)
    case Op::Softmax: return (nd.kind == kAxisC && nd.T == 1) || nd.kind == kAxisT;
    case Op::Fold: return !nd.axis_hw && !nd.axis_c;
    default: return false;
    }
}

bool compile_unit(const Dag& dag, const std::vector<int>& nodes, const std::vector<bool>& is_output, UnitPlan& out, std::string& why) {
    try {
        if (nodes.empty()) throw Fail{"empty unit"};
        std::vector<bool> in_unit(dag.nodes.size(), false);
        for (int k : nodes) in_unit[k] = true;
        const int C = dag.nodes[nodes[0]].C;
        for (int k : nodes)
            if (dag.nodes[k].C != C) throw Fail{"channel counts differ inside the unit"};
        Graph G(dag, in_unit, is_output);
        out = UnitPlan();
        out.nodes = nodes;
        std::vector<int> out_inst;
        for (int k : nodes)
            if (is_output[k]) {
                out.outputs.push_back(k);
                out_inst.push_back(G.build(k, 0));
            }
        if (out.outputs.empty()) throw Fail{"unit without an output"};
        const bool box = G.add_box_adjoints();  // (backward only: the forward program never evaluates what this adds)
        int lanes = 1;
        std::vector<int> smc, leaves;
        for (size_t i = 0; i < G.insts.size(); i++) {
            lanes = std::max(lanes, G.insts[i].lanes);
            if (G.insts[i].kind == kSmC) smc.push_back((int)i);
            if (G.insts[i].kind == kExt) {
                if (!(box && G.ctxs[G.insts[i].ctx].win)) leaves.push_back((int)i);  // (a box adjoint replaces the way through its window)
                if (std::find(out.inputs.begin(), out.inputs.end(), G.insts[i].node) == out.inputs.end()) out.inputs.push_back(G.insts[i].node);
            }
        }
        std::sort(out.inputs.begin(), out.inputs.end());
        for (int e : out.inputs)
            if (dag.nodes[e].C != C) throw Fail{"an external tensor with another channel count"};
        auto fits32 = [&](int k) { return (int64_t)dag.N * C * std::max(dag.nodes[k].T, 1) * dag.H * dag.W * 4 < ((int64_t)1 << 31); };
        for (int k : nodes)
            if (!fits32(k)) throw Fail{"a tensor beyond 32-bit byte offsets"};
        for (int k : out.inputs)
            if (!fits32(k)) throw Fail{"a tensor beyond 32-bit byte offsets"};
        if (lanes > 25) throw Fail{"more than 25 taps"};
        const int tm = lanes <= 1 ? 1 : (lanes <= 9 ? 9 : 25);

        // ------------------------------------------------------------ displaced units
        // The gradient of a leaf that reads an external tensor through Shift offsets belongs to another pixel.  Where the
        // unit has no reduction, the pixel fetches it itself: the whole unit is instantiated once more, displaced by
        // the negated offsets (every load of it, the incoming gradient included, moves with it), and the gradient of
        // the same leaf in that copy, masked where the displaced pixel leaves the image, is what this pixel's tensor
        // element receives.  No hand-over between threads, no halo, no barrier; windows keep the hand-over (OP_XADD),
        // one displaced copy per tap would cost more than it saves.
        struct Pull {
            std::unique_ptr<Graph> g;
            int leaf = -1, mask_ctx = -1;
        };
        std::map<int, Pull> pulls;  // by leaf instance of the unit's own graph
        for (int i : leaves) {
            const Ctx& c = G.ctxs[G.insts[i].ctx];
            if (c.empty() || c.win) continue;
            try {
                Pull P;
                P.g.reset(new Graph(dag, in_unit, is_output));
                Ctx d;
                for (const Term& t : c.terms) {
                    Term n = t;
                    n.dh = (int16_t)-t.dh;
                    n.dw = (int16_t)-t.dw;
                    d.terms.push_back(n);
                }
                P.g->root_ctx = P.g->ctx_id(d);
                P.mask_ctx = P.g->root_ctx;
                for (int k : out.outputs) P.g->build(k, P.g->root_ctx);
                Ctx full = d;  // the same leaf in the displaced copy: the displacement, then the leaf's own offsets
                for (const Term& t : c.terms) full.terms.push_back(t);
                const int want_ctx = P.g->ctx_id(full);
                for (size_t j = 0; j < P.g->insts.size(); j++)
                    if (P.g->insts[j].kind == kExt && P.g->insts[j].node == G.insts[i].node && P.g->insts[j].ctx == want_ctx &&
                        P.g->insts[j].lanes == G.insts[i].lanes)
                        P.leaf = (int)j;
                if (P.leaf >= 0) pulls[i] = std::move(P);
            } catch (const Fail&) {
            }
        }
        // ------------------------------------------------------------ the two programs
        auto emit_fwd = [&](Emitter& E) {
            E.stat_passes(smc);
            E.begin_pass();
            E.begin_body();
            for (size_t o = 0; o < out.outputs.size(); o++) {
                E.eval(out_inst[o]);
                Instr st = Emitter::simple(OP_ST, dag.nodes[out.outputs[o]].T, 0, 0, E.ext_slot(out.outputs[o], kValueOut));
                E.ext[st.a].store_instr = E.pg.n_instr;
                E.emit(st);
            }
            E.end_pass();
        };
        auto emit_bwd = [&](Emitter& E) {
            E.stat_passes(smc);
            int deepest = 0;
            for (int i : smc) deepest = std::max(deepest, G.down(i));
            for (int d = 0; d <= deepest && !smc.empty(); d++) {  // the sums of gradient x output, outermost softmax first
                E.begin_pass();
                for (int i : smc)
                    if (G.down(i) == d) {
                        E.emit(Emitter::simple(OP_PSET, G.insts[i].lanes, 0, 0, E.dot_slot(i)));
                        E.reduce(E.dot_slot(i), G.insts[i].lanes, 1);
                    }
                E.begin_body();
                for (int i : smc)
                    if (G.down(i) == d) {
                        E.grad(i);
                        const int r = E.alloc();
                        E.emit(Emitter::simple(OP_MOVR, G.insts[i].lanes, r));
                        E.eval(i);
                        E.emit(Emitter::simple(OP_SMCDOT, G.insts[i].lanes, r, 0, E.dot_slot(i)));
                        E.release(r);
                    }
                E.end_pass();
            }
            E.begin_pass();
            E.begin_body();
            for (int e : out.inputs) {
                std::vector<int> mine;
                for (int i : leaves)
                    if (G.insts[i].node == e) mine.push_back(i);
                const int Te = dag.nodes[e].T;
                const int slot = E.ext_slot(e, kGradOut);
                const bool direct = mine.size() == 1 && G.insts[mine[0]].ctx == 0 && G.insts[mine[0]].lanes == Te;
                // no hand-over among the leaves: their contributions are summed in a register instead of LDS floats
                bool local = !direct;
                for (int i : mine)
                    if (G.insts[i].lanes != Te || (G.insts[i].ctx != 0 && !pulls.count(i))) local = false;
                int acc = -1, racc = -1;
                if (!direct && !local) {
                    acc = E.persist(Te);
                    E.emit(Emitter::simple(OP_PSET, Te, 0, 0, acc));
                }
                bool first_term = true;
                auto add_term = [&](int lanes) {  // A holds one more contribution
                    if (local) {
                        if (!first_term) {
                            E.emit(Emitter::simple(OP_BIN, Te, racc, kAdd | kBinRegIsLhs));
                            E.release(racc);
                            racc = -1;
                        }
                        first_term = false;
                        return;
                    }
                    Instr p = Emitter::simple(OP_PADD, lanes, 0, 0, acc);
                    p.b = (uint16_t)Te;
                    E.emit(p);
                };
                for (size_t mi = 0; mi < mine.size(); mi++) {
                    const int i = mine[mi];
                    const Inst& L = G.insts[i];
                    if (local && !first_term) {  // (the sum so far waits in a register while the next term is computed)
                        racc = E.alloc();
                        E.emit(Emitter::simple(OP_MOVR, Te, racc));
                    }
                    auto pl = pulls.find(i);
                    if (pl != pulls.end()) {  // fetched from the displaced copy of the unit
                        int idx = 1;
                        for (auto it = pulls.begin(); it != pl; ++it) idx++;
                        E.use(*pl->second.g, idx);
                        E.grad(pl->second.leaf);
                        E.emit(E.positional(OP_MASK, pl->second.mask_ctx, L.lanes));
                        E.forget_graph(idx);
                        E.use(G, 0);
                        add_term(L.lanes);
                        continue;
                    }
                    E.grad(i);
                    if (direct) break;
                    if (L.ctx == 0) {
                        add_term(L.lanes);
                    } else {
                        if (!G.ctxs[L.ctx].win && L.lanes != Te) throw Fail{"a shifted read of an external tensor with replicated taps"};
                        Instr x = E.positional(OP_XADD, L.ctx, L.lanes);
                        x.a = (uint16_t)acc;
                        if (Te > 1) x.kind |= kExtTaps;
                        E.reach_of[E.pg.n_instr] = G.ctxs[L.ctx].reach_px(dag.W);
                        E.emit(x);
                    }
                }
                if (!direct && !local) E.emit(Emitter::simple(OP_PLD, Te, 0, 0, acc));
                Instr st = Emitter::simple(OP_ST, Te, 0, 0, slot);
                E.ext[slot].store_instr = E.pg.n_instr;
                E.emit(st);
            }
            E.end_pass();
        };
        // A program is emitted with full recomputation first; then, greedily, the value or gradient whose repeated
        // computation costs the most instructions is kept in a register, as long as that shortens the program and the
        // registers last.  Returns the emitter of the shortest program that could be emitted.
        auto shortest = [&](const std::function<void(Emitter&)>& emit_program) {
            std::set<int> keep;
            auto best = std::make_shared<Emitter>(G, tm);
            emit_program(*best);  // (throws when even the plain program does not fit)
            for (int round = 0; round < regs_for(tm); round++) {
                int pick = -1, gain = 1;
                for (const auto& kv : best->stats) {
                    const int g = (kv.second.computed - 1) * (kv.second.cost - 1) - 1;  // (- the store)
                    if (!keep.count(kv.first) && g > gain) {
                        gain = g;
                        pick = kv.first;
                    }
                }
                if (pick < 0) break;
                keep.insert(pick);
                try {
                    auto E = std::make_shared<Emitter>(G, tm);
                    E->keep = keep;
                    emit_program(*E);
                    if (E->pg.n_instr >= best->pg.n_instr) break;
                    best = E;
                } catch (const Fail&) {
                    break;
                }
            }
            return best;
        };
        {
            auto E = shortest(emit_fwd);
            set_geometry(E->pg, dag, C, 0, !smc.empty());
            out.fwd = E->pg;
            out.fwd_ext = E->ext;
        }
        {
            auto E = shortest(emit_bwd);
            int64_t halo = 0;
            for (int i = 0; i < E->pg.n_instr; i++)  // (the reach of the hand-overs of the program that was chosen)
                if (E->pg.ins[i].op == OP_XADD) halo = std::max(halo, E->reach_of[i]);
            set_geometry(E->pg, dag, C, halo, !smc.empty());
            out.bwd = E->pg;
            out.bwd_ext = E->ext;
            out.cost = program_cost(out.fwd) + program_cost(out.bwd);
        }
        return true;
    } catch (const Fail& f) {
        why = f.why;
        return false;
    }
}

double program_cost(const Program& pg) {
    double sum = 0;
    for (int p = 0; p < pg.n_pass; p++)
        for (int i = pg.pass[p].body_begin; i < pg.pass[p].body_end; i++) {
            const Instr& I = pg.ins[i];
            double w = 1;
            switch (I.op) {
            case OP_LD:
            case OP_BINLD:
            case OP_ST: w = 4; break;
            case OP_XADD: w = 6; break;
            case OP_UN:
            case OP_UNBX: w = (I.kind == 0 || I.kind == 1 || I.kind == kUnNeg) ? 1 : 6; break;
            case OP_SMT:
            case OP_SMTBX:
            case OP_SMCSTAT:
            case OP_SMCAPPLY: w = 6; break;
            default: break;
            }
            sum += w * I.T;
        }
    // pixels computed per pixel owned (the halo), and the serial walk over the channels where the workgroup's shape leaves
    // a thread more than 16 trips (a program that keeps all channels in one workgroup and has no LDS left for slices)
    const double halo = (double)pg.pix_threads / std::max(1, pg.own_threads + (pg.halo_threads > 0 ? 0 : pg.pix_threads - pg.own_threads));
    const double trips = std::ceil((double)pg.chunk / std::max(1, pg.slices * pg.unroll));
    return sum * halo * std::max(1.0, trips / 16.0);
}

std::string dump(const Program& pg) {
    static const char* names[] = {"LD", "MASK", "UN", "MOVR", "MOVA", "BIN", "FOLD", "SMT", "ST", "UNBX", "BING", "SMTBX", "FOLDBX",
                                  "PSET", "PADD", "PLD", "SMCSTAT", "SMCAPPLY", "SMCDOT", "SMCBX", "XADD", "BINLD"};
    std::ostringstream os;
    os << "program: C=" << pg.C << " HxW=" << pg.H << "x" << pg.W << " vec=" << pg.vec << " own=" << pg.own_threads << " halo=" << pg.halo_threads
       << " unroll=" << pg.unroll << " tiles=" << pg.tiles << " chunk=" << pg.chunk << " slices=" << pg.slices << " threads=" << pg.threads << " persist=" << pg.n_persist
       << " lanes=" << pg.tm << "\n";
    for (int p = 0; p < pg.n_pass; p++) {
        os << " pass " << p << "\n";
        for (int i = pg.pass[p].pro_begin; i < pg.pass[p].body_end; i++) {
            const Instr& I = pg.ins[i];
            os << (i < pg.pass[p].pro_end ? "  pro  " : "  body ") << i << ": " << (I.op < OP_COUNT ? names[I.op] : "?") << " T=" << (int)I.T
               << " kind=" << (int)I.kind << " r=" << (int)I.r << " a=" << I.a << " b=" << I.b << " f0=" << I.f0 << "\n";
        }
    }
    return os.str();
}

}  // namespace chain
}  // namespace canvas
