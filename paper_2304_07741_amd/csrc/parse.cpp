// Blob parser, shape inference and legality checks (host only).
#include "dag.hpp"

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <map>
#include <sstream>

namespace canvas {
namespace {

constexpr int kOk = 0, kInvalidBlob = -1, kUnknownOp = -2, kShapeMismatch = -3, kBadArg = -4, kUnsupported = -6;
constexpr int kMaxNodes = 64;

struct Line {
    std::vector<std::string> pos;              // positional tokens
    std::map<std::string, std::string> attr;   // key=value tokens
};

bool parse_ref(const std::string& s, int& id) {
    if (s.size() < 2 || s[0] != '%') return false;
    for (size_t i = 1; i < s.size(); i++)
        if (s[i] < '0' || s[i] > '9') return false;
    if (s.size() > 8) return false;
    id = std::atoi(s.c_str() + 1);
    return true;
}

bool get_int(const Line& l, const char* key, int& v, bool required, bool& present) {
    auto it = l.attr.find(key);
    present = it != l.attr.end();
    if (!present) return !required;
    char* end = nullptr;
    long x = std::strtol(it->second.c_str(), &end, 10);
    if (end == it->second.c_str() || *end || x < -(1 << 30) || x > (1 << 30)) return false;
    v = (int)x;
    return true;
}

bool get_float(const Line& l, const char* key, float& v) {
    auto it = l.attr.find(key);
    if (it == l.attr.end()) return false;
    char* end = nullptr;
    double x = std::strtod(it->second.c_str(), &end);
    if (end == it->second.c_str() || *end) return false;
    v = (float)x;
    return true;
}

int fail(std::string& err, int lineno, const std::string& msg, int code) {
    std::ostringstream os;
    os << "blob line " << lineno << ": " << msg;
    err = os.str();
    return code;
}

}  // namespace

int parse_dag(const char* blob, size_t len, const int64_t in_shape[4], Dag& dag, std::string& err) {
    if (!blob || !in_shape) { err = "null blob or shape"; return kBadArg; }
    for (int i = 0; i < 4; i++)
        if (in_shape[i] < 1 || in_shape[i] > (1 << 24)) { err = "input shape entries must be in [1, 2^24]"; return kBadArg; }
    dag = Dag();
    dag.N = (int)in_shape[0];
    dag.H = (int)in_shape[2];
    dag.W = (int)in_shape[3];
    Node in;
    in.op = Op::Input;
    in.C = (int)in_shape[1];
    in.T = 1;
    dag.nodes.push_back(in);

    std::string text(blob, len);
    std::istringstream ss(text);
    std::string raw;
    int lineno = 0;
    bool header = false, done = false;
    while (std::getline(ss, raw)) {
        lineno++;
        std::istringstream ls(raw);
        std::string tok;
        Line l;
        bool comment = false;
        while (ls >> tok) {
            if (l.pos.empty() && l.attr.empty() && tok[0] == '#') { comment = true; break; }
            size_t eq = tok.find('=');
            if (eq != std::string::npos && eq > 0 && tok != "=") l.attr[tok.substr(0, eq)] = tok.substr(eq + 1);
            else l.pos.push_back(tok);
        }
        if (comment || (l.pos.empty() && l.attr.empty())) continue;
        if (!header) {
            if (l.pos.size() != 2 || l.pos[0] != "canvas-dag" || l.pos[1] != "1" || !l.attr.empty())
                return fail(err, lineno, "expected header 'canvas-dag 1'", kInvalidBlob);
            header = true;
            continue;
        }
        if (done) return fail(err, lineno, "text after the output line", kInvalidBlob);
        if (l.pos.empty()) return fail(err, lineno, "expected '%k = op %operand ...' or 'output %k'", kInvalidBlob);
        if (l.pos[0] == "output") {
            int id;
            if (l.pos.size() != 2 || !parse_ref(l.pos[1], id) || id >= (int)dag.nodes.size())
                return fail(err, lineno, "bad output reference", kInvalidBlob);
            dag.out = id;
            done = true;
            continue;
        }
        int id;
        if (l.pos.size() < 4 || !parse_ref(l.pos[0], id) || l.pos[1] != "=")
            return fail(err, lineno, "expected '%k = op %operand ...'", kInvalidBlob);
        if (id != (int)dag.nodes.size()) return fail(err, lineno, "node ids must be consecutive from 1", kInvalidBlob);
        if (id >= kMaxNodes) return fail(err, lineno, "too many nodes", kUnsupported);
        Node nd;
        if (!parse_ref(l.pos[3], nd.a) || nd.a >= id) return fail(err, lineno, "operand must be an earlier node", kInvalidBlob);
        const Node A = dag.nodes[nd.a];  // shape and view as named; the data is that of the viewed tensor
        auto viewed = [&](int k) {
            while (dag.nodes[k].op == Op::Group) k = dag.nodes[k].a;
            return k;
        };
        nd.a = viewed(nd.a);
        const std::string& op = l.pos[2];
        bool present;
        nd.pooled = A.pooled;  // (binary takes the RHS's below)
        nd.grp = A.grp;        // (likewise)
        if ((op == "unfold" || op == "shift") && A.pooled) return fail(err, lineno, op + " needs the spatial dims", kShapeMismatch);
        if (op == "unfold") {
            nd.op = Op::Unfold;
            if (!get_int(l, "kh", nd.kh, true, present) || !get_int(l, "kw", nd.kw, true, present))
                return fail(err, lineno, "unfold needs kh= and kw=", kInvalidBlob);
            if (nd.kh < 1 || nd.kw < 1 || nd.kh % 2 == 0 || nd.kw % 2 == 0 || nd.kh > 15 || nd.kw > 15)
                return fail(err, lineno, "unfold window must be odd and in [1, 15]", kShapeMismatch);
            if ((int64_t)A.T * nd.kh * nd.kw > 4096) return fail(err, lineno, "more than 4096 taps", kUnsupported);
            nd.C = A.C;
            nd.T = A.T * nd.kh * nd.kw;
        } else if (op == "shift") {
            nd.op = Op::Shift;
            nd.c0 = 0;
            nd.c1 = A.C;
            if (!get_int(l, "dh", nd.dh, true, present) || !get_int(l, "dw", nd.dw, true, present) ||
                !get_int(l, "c0", nd.c0, false, present) || !get_int(l, "c1", nd.c1, false, present))
                return fail(err, lineno, "shift needs dh= dw= [c0= c1=]", kInvalidBlob);
            if (nd.c0 < 0 || nd.c1 > A.C || nd.c0 > nd.c1) return fail(err, lineno, "shift slice outside the channels", kShapeMismatch);
            // a shift by the image's extent or more moves everything out: clamped, so that dh * W + dw stays a small int
            nd.dh = std::max(-dag.H, std::min(dag.H, nd.dh));
            nd.dw = std::max(-dag.W, std::min(dag.W, nd.dw));
            nd.C = A.C;
            nd.T = A.T;
        } else if (op == "group") {
            nd.op = Op::Group;
            if (!get_int(l, "groups", nd.grp, true, present)) return fail(err, lineno, "group needs groups=", kInvalidBlob);
            if (nd.grp < 1 || A.C % nd.grp) return fail(err, lineno, "group: groups must divide the channels", kShapeMismatch);
            nd.C = A.C;
            nd.T = A.T;
        } else if (op == "fc") {
            nd.op = Op::Fc;
            nd.groups = A.grp;  // a grouped operand: the FC works inside each group
            if (!get_int(l, "groups", nd.groups, false, present) || !get_int(l, "out", nd.out, true, present))
                return fail(err, lineno, "fc needs [groups=] and out=", kInvalidBlob);
            if (l.attr.count("groups") && A.grp > 1 && nd.groups != A.grp)
                return fail(err, lineno, "fc groups= contradicts the Group view of its operand", kShapeMismatch);
            if (nd.groups < 1 || nd.out < 1 || A.C % nd.groups || nd.out % nd.groups)
                return fail(err, lineno, "fc groups must divide input and output channels", kShapeMismatch);
            nd.C = nd.out;
            nd.T = 1;
            nd.widx = dag.n_weights++;
            dag.weight_node.push_back(id);
        } else if (op == "unary") {
            nd.op = Op::Unary;
            auto it = l.attr.find("op");
            if (it == l.attr.end()) return fail(err, lineno, "unary needs op=", kInvalidBlob);
            if (it->second == "relu") nd.kind = kRelu;
            else if (it->second == "abs") nd.kind = kAbs;
            else if (it->second == "gelu") nd.kind = kGelu;
            else if (it->second == "sin") nd.kind = kSin;
            else if (it->second == "expclip") {
                nd.kind = kExpClip;
                if (!get_float(l, "lo", nd.lo) || !get_float(l, "hi", nd.hi)) return fail(err, lineno, "expclip needs lo= hi=", kInvalidBlob);
                if (!(nd.lo < nd.hi)) return fail(err, lineno, "expclip needs lo < hi", kShapeMismatch);
            } else return fail(err, lineno, "unknown unary op '" + it->second + "'", kUnknownOp);
            nd.C = A.C;
            nd.T = A.T;
        } else if (op == "binary") {
            nd.op = Op::Binary;
            if (l.pos.size() < 5 || !parse_ref(l.pos[4], nd.b) || nd.b >= id)
                return fail(err, lineno, "binary needs two earlier operands", kInvalidBlob);
            auto it = l.attr.find("op");
            if (it == l.attr.end()) return fail(err, lineno, "binary needs op=", kInvalidBlob);
            if (it->second == "add") nd.kind = kAdd;
            else if (it->second == "mul") nd.kind = kMul;
            else if (it->second == "sub") nd.kind = kSub;
            else if (it->second == "min") nd.kind = kBinMin;
            else if (it->second == "max") nd.kind = kBinMax;
            else return fail(err, lineno, "unknown binary op '" + it->second + "'", kUnknownOp);
            const Node B = dag.nodes[nd.b];
            nd.b = viewed(nd.b);
            // the same Group view on both sides is a common leading dim: the rule applies to [C / G, T] inside each group
            nd.bgroups = A.grp == B.grp ? A.grp : 1;
            const int CLg = A.C / nd.bgroups, CRg = B.C / nd.bgroups;
            bool legal = (CLg == CRg) ? (B.T % A.T == 0) : (((int64_t)CRg * B.T) % ((int64_t)CLg * A.T) == 0);
            if ((A.pooled & B.pooled) != B.pooled) legal = false;  // the LHS is replicated along dims it has folded away, not the reverse
            auto al = l.attr.find("lhs");
            if (al != l.attr.end()) {
                if (al->second != "pixels") return fail(err, lineno, "binary lhs= must be pixels", kInvalidBlob);
                // [X] read as [H, W]: a common suffix with the RHS; nothing of the LHS is left to replicate along channels
                nd.lhs_pixels = true;
                nd.bgroups = 1;
                legal = A.pooled == 3 && !B.pooled && (int64_t)A.C * A.T == (int64_t)dag.H * dag.W;
            }
            nd.pooled = B.pooled;
            nd.grp = B.grp;
            if (!legal) return fail(err, lineno, "broadcast: LHS size does not divide RHS size", kShapeMismatch);
            nd.C = B.C;
            nd.T = B.T;
        } else if (op == "softmax") {
            nd.op = Op::Softmax;
            auto it = l.attr.find("axis");
            if (it == l.attr.end()) return fail(err, lineno, "softmax needs axis=", kInvalidBlob);
            if (it->second == "C") nd.kind = kAxisC;
            else if (it->second == "T") nd.kind = kAxisT;
            else if (it->second == "CT") nd.kind = kAxisCT;
            else if (it->second == "H") nd.kind = kAxisH;
            else if (it->second == "W") nd.kind = kAxisW;
            else if (it->second == "HW") nd.kind = kAxisHW;
            else return fail(err, lineno, "softmax axis must be C, T, CT, H, W or HW", kUnknownOp);
            nd.C = A.C;
            nd.T = A.T;
        } else if (op == "fold") {
            nd.op = Op::Fold;
            auto it = l.attr.find("op");
            if (it == l.attr.end()) return fail(err, lineno, "fold needs op=", kInvalidBlob);
            if (it->second == "sum") nd.kind = kSum;
            else if (it->second == "avg") nd.kind = kAvg;
            else if (it->second == "max") nd.kind = kMax;
            else return fail(err, lineno, "unknown fold op '" + it->second + "'", kUnknownOp);
            auto ax = l.attr.find("axis");
            if (ax != l.attr.end() && ax->second == "HW") nd.axis_hw = 3;
            else if (ax != l.attr.end() && ax->second == "H") nd.axis_hw = 1;
            else if (ax != l.attr.end() && ax->second == "W") nd.axis_hw = 2;
            else if (ax != l.attr.end() && ax->second == "C") nd.axis_c = 1;
            else if (ax != l.attr.end() && ax->second != "T") return fail(err, lineno, "fold axis must be T, H, W, HW or C", kUnknownOp);
            nd.C = A.C;
            if (nd.axis_c) {
                nd.groups = 1;
                if (!get_int(l, "groups", nd.groups, false, present)) return fail(err, lineno, "fold axis=C: bad groups=", kInvalidBlob);
                if (nd.groups < 1 || A.C % nd.groups) return fail(err, lineno, "fold axis=C: groups must divide the channels", kShapeMismatch);
                nd.C = nd.groups;
                nd.T = A.T;
                nd.grp = 1;
            } else if (nd.axis_hw) {
                if (A.pooled & nd.axis_hw) return fail(err, lineno, "fold: that spatial dim is already folded", kShapeMismatch);
                nd.T = A.T;
                nd.pooled = A.pooled | nd.axis_hw;
            } else {
                nd.T = 1;
            }
        } else {
            return fail(err, lineno, "unknown op '" + op + "'", kUnknownOp);
        }
        if ((int64_t)nd.C * nd.T * dag.H * dag.W * dag.N >= ((int64_t)1 << 40))
            return fail(err, lineno, "tensor too large", kUnsupported);
        dag.nodes.push_back(nd);
    }
    if (!header) { err = "empty blob: expected header 'canvas-dag 1'"; return kInvalidBlob; }
    if (dag.out < 0) { err = "blob has no output line"; return kInvalidBlob; }
    // liveness: only nodes the output depends on are computed
    dag.nodes[dag.out].live = true;
    for (int k = (int)dag.nodes.size() - 1; k >= 1; k--)
        if (dag.nodes[k].live) {
            dag.nodes[dag.nodes[k].a].live = true;
            if (dag.nodes[k].b >= 0) dag.nodes[dag.nodes[k].b].live = true;
        }
    return kOk;
}

Dag without_dead_views(const Dag& dag) {
    Dag out = dag;
    out.nodes.clear();
    std::vector<int> id(dag.nodes.size(), -1);
    for (size_t k = 0; k < dag.nodes.size(); k++) {
        const Node& nd = dag.nodes[k];
        if (nd.op == Op::Group && !nd.live) continue;
        id[k] = (int)out.nodes.size();
        Node c = nd;
        if (c.a >= 0) c.a = id[c.a];
        if (c.b >= 0) c.b = id[c.b];
        out.nodes.push_back(c);
    }
    out.out = id[dag.out];
    for (auto& w : out.weight_node) w = id[w];
    return out;
}

}  // namespace canvas
