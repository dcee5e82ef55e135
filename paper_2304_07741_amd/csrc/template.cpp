// Kernel templates: symbolic shape inference, the shape-matching solver, the global group number, the
// constraint solver and instantiation (Canvas paper, Section 6.2 and 6.3).  Host only; C ABI at the bottom.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <map>
#include <sstream>
#include <string>
#include <vector>

#include "../../include/canvas_template.h"
#include "dag.hpp"
#include "symbolic.hpp"

namespace canvas {
int set_last_error(int code, const std::string& msg);  // api.cpp
}

namespace {

using canvas::sym::Binding;
using canvas::sym::Mono;
namespace sym = canvas::sym;

enum class TOp { Input, Unfold, Shift, Fc, Unary, Binary, Softmax, Fold, Group };

struct Attr {
    std::string key, raw;
    bool symbolic = false;
    Mono m;
};

struct TNode {
    TOp op = TOp::Input;
    std::string opname;
    int a = -1, b = -1;
    std::vector<Attr> attrs;
    // inferred
    Mono C;
    std::vector<Mono> taps;
    int pooled = 0;  // mask of folded spatial dims: 1 = H, 2 = W
    Mono grp;  // 1 = no Group view
    Mono groups_used;  // fc / fold over channels / group: the group count that applies

    const Attr* find(const std::string& k) const {
        for (const auto& a : attrs)
            if (a.key == k) return &a;
        return nullptr;
    }
};

struct Constraint {
    Mono m;  // must evaluate to a positive integer
    int node;
    const char* what;
};

struct Template {
    std::vector<TNode> nodes;
    int out = -1;
    std::vector<Constraint> must_be_integer;
    std::vector<std::pair<Mono, int>> must_be_one;  // (monomial, node): lhs=pixels blends
};

int fail(int code, int lineno, const std::string& msg) {
    return canvas::set_last_error(code, lineno > 0 ? "line " + std::to_string(lineno) + ": " + msg : msg);
}

bool parse_ref(const std::string& t, int& id) {
    if (t.size() < 2 || t[0] != '%') return false;
    char* end = nullptr;
    const long v = std::strtol(t.c_str() + 1, &end, 10);
    if (*end || v < 0 || v > 1000) return false;
    id = (int)v;
    return true;
}

Mono product(const std::vector<Mono>& v) {
    Mono r;
    for (const auto& m : v) r = r * m;
    return r;
}

bool mentions_var(const Mono& m) {
    for (int j = 1; j <= sym::kMaxVars; j++)
        if (m.var_exp(j) != 0) return true;
    return false;
}

const std::map<std::string, std::vector<std::string>>& symbolic_keys() {
    static const std::map<std::string, std::vector<std::string>> k = {
        {"unfold", {"kh", "kw"}}, {"shift", {"c0", "c1"}}, {"fc", {"groups", "out"}}, {"group", {"groups"}}, {"fold", {"groups"}}};
    return k;
}

// Shapes and the list of sizes that must be integers, from the attributes as they stand.
int infer(Template& t) {
    t.must_be_integer.clear();
    t.must_be_one.clear();
    for (size_t k = 0; k < t.nodes.size(); k++) {
        TNode& nd = t.nodes[k];
        const int id = (int)k;
        if (nd.op == TOp::Input) {
            nd.C = Mono::channels();
            nd.taps.clear();
            nd.pooled = 0;
            nd.grp = Mono::one();
            continue;
        }
        const TNode& A = t.nodes[nd.a];
        nd.C = A.C;
        nd.taps = A.taps;
        nd.pooled = A.pooled;
        nd.grp = A.grp;
        auto need = [&](const char* key, Mono& out) {
            const Attr* a = nd.find(key);
            if (!a) return false;
            out = a->m;
            return true;
        };
        switch (nd.op) {
        case TOp::Unfold: {
            Mono kh, kw;
            if (!need("kh", kh) || !need("kw", kw)) return fail(CANVAS_INVALID_BLOB, 0, "node " + std::to_string(id) + ": unfold needs kh= and kw=");
            if (mentions_var(kh) || mentions_var(kw) || A.pooled)
                return fail(CANVAS_SHAPE_MISMATCH, 0, "node " + std::to_string(id) + ": a dynamic variable in a window size, or an unfold without spatial dims");
            if (!kh.is_one()) nd.taps.push_back(kh);
            if (!kw.is_one()) nd.taps.push_back(kw);
            t.must_be_integer.push_back({kh, id, "window height"});
            t.must_be_integer.push_back({kw, id, "window width"});
            break;
        }
        case TOp::Shift: {
            if (A.pooled) return fail(CANVAS_SHAPE_MISMATCH, 0, "node " + std::to_string(id) + ": shift without spatial dims");
            Mono c;
            if (need("c0", c)) t.must_be_integer.push_back({c, id, "shift c0"});
            if (need("c1", c)) t.must_be_integer.push_back({c, id, "shift c1"});
            break;
        }
        case TOp::Group: {
            Mono g;
            if (!need("groups", g)) return fail(CANVAS_INVALID_BLOB, 0, "node " + std::to_string(id) + ": group needs groups=");
            if (mentions_var(g)) return fail(CANVAS_SHAPE_MISMATCH, 0, "node " + std::to_string(id) + ": a dynamic variable as a group number");
            nd.grp = g;
            nd.groups_used = g;
            t.must_be_integer.push_back({g, id, "group number"});
            t.must_be_integer.push_back({A.C / g, id, "channels per group"});
            break;
        }
        case TOp::Fc: {
            Mono out, g = A.grp;
            if (!need("out", out)) return fail(CANVAS_INVALID_BLOB, 0, "node " + std::to_string(id) + ": fc needs out=");
            Mono stated;
            if (need("groups", stated)) {
                if (!A.grp.is_one() && !(stated == A.grp))
                    return fail(CANVAS_SHAPE_MISMATCH, 0, "node " + std::to_string(id) + ": fc groups= contradicts the Group view of its operand");
                g = stated;
            }
            if (mentions_var(g)) return fail(CANVAS_SHAPE_MISMATCH, 0, "node " + std::to_string(id) + ": a dynamic variable as a group number");
            nd.groups_used = g;
            t.must_be_integer.push_back({g, id, "fc groups"});
            t.must_be_integer.push_back({A.C / g, id, "fc input channels per group"});
            t.must_be_integer.push_back({out / g, id, "fc output channels per group"});
            nd.C = out;
            nd.taps.clear();
            break;
        }
        case TOp::Unary:
        case TOp::Softmax: break;
        case TOp::Binary: {
            const TNode& B = t.nodes[nd.b];
            if ((A.pooled & B.pooled) != B.pooled)
                return fail(CANVAS_SHAPE_MISMATCH, 0, "node " + std::to_string(id) + ": the RHS has folded a spatial dim that the LHS keeps");
            const Mono lhs = A.C * product(A.taps), rhs = B.C * product(B.taps);
            const Attr* al = nd.find("lhs");
            if (al) {
                if (al->raw != "pixels" || A.pooled != 3 || B.pooled)
                    return fail(CANVAS_SHAPE_MISMATCH, 0, "node " + std::to_string(id) + ": lhs=pixels needs a pooled LHS and a full-size RHS");
                t.must_be_one.push_back({Mono::atom(sym::aH) * Mono::atom(sym::aW) / lhs, id});
            } else {
                t.must_be_integer.push_back({rhs / lhs, id, "broadcast ratio #RHS / #LHS"});
            }
            nd.C = B.C;
            nd.taps = B.taps;
            nd.pooled = B.pooled;
            nd.grp = B.grp;
            break;
        }
        case TOp::Fold: {
            const Attr* ax = nd.find("axis");
            const std::string axis = ax ? ax->raw : "T";
            if (axis == "T") nd.taps.clear();
            else if (axis == "HW" || axis == "H" || axis == "W") {
                const int m = axis == "HW" ? 3 : (axis == "H" ? 1 : 2);
                if (A.pooled & m) return fail(CANVAS_SHAPE_MISMATCH, 0, "node " + std::to_string(id) + ": that spatial dim is already folded");
                nd.pooled = A.pooled | m;
            } else if (axis == "C") {
                Mono g = Mono::one();
                need("groups", g);
                if (mentions_var(g)) return fail(CANVAS_SHAPE_MISMATCH, 0, "node " + std::to_string(id) + ": a dynamic variable as a group number");
                nd.groups_used = g;
                t.must_be_integer.push_back({g, id, "fold groups"});
                t.must_be_integer.push_back({A.C / g, id, "folded channels per group"});
                nd.C = g;
                nd.grp = Mono::one();
            } else return fail(CANVAS_UNKNOWN_OP, 0, "node " + std::to_string(id) + ": fold axis must be T, H, W, HW or C");
            break;
        }
        default: break;
        }
        // Theorem 1 (Section 6.2): a dynamic variable only in the numerator of the channel dim, at most one
        const int v = nd.C.single_var();
        if (v < 0 || (v > 0 && nd.C.var_exp(v) != 1))
            return fail(CANVAS_SHAPE_MISMATCH, 0, "node " + std::to_string(id) + ": channel dim " + sym::to_text(nd.C) + " breaks the one-variable-in-the-numerator rule");
        t.must_be_integer.push_back({nd.C, id, "channels"});
        if (!nd.grp.is_one()) t.must_be_integer.push_back({nd.C / nd.grp, id, "channels per group of the view"});
    }
    // a size without symbols that is no integer can never become one
    for (const auto& c : t.must_be_integer)
        if (c.m.degree() == 0 && c.m.den != 1)
            return fail(CANVAS_SHAPE_MISMATCH, 0, "node " + std::to_string(c.node) + ": " + c.what + " = " + sym::to_text(c.m) + " is no integer");
    return CANVAS_OK;
}

int parse_template(const char* blob, size_t len, Template& t) {
    std::istringstream ss(std::string(blob, len));
    std::string raw;
    int lineno = 0;
    bool header = false, done = false;
    TNode in;
    in.op = TOp::Input;
    t.nodes.push_back(in);
    static const std::map<std::string, TOp> ops = {{"unfold", TOp::Unfold}, {"shift", TOp::Shift}, {"fc", TOp::Fc}, {"unary", TOp::Unary},
                                                   {"binary", TOp::Binary}, {"softmax", TOp::Softmax}, {"fold", TOp::Fold}, {"group", TOp::Group}};
    while (std::getline(ss, raw)) {
        lineno++;
        std::istringstream ls(raw);
        std::vector<std::string> tok;
        std::string w;
        while (ls >> w) tok.push_back(w);
        if (tok.empty() || tok[0][0] == '#') continue;
        if (!header) {
            if (tok.size() != 2 || tok[0] != "canvas-template" || tok[1] != "1") return fail(CANVAS_INVALID_BLOB, lineno, "expected header 'canvas-template 1'");
            header = true;
            continue;
        }
        if (done) return fail(CANVAS_INVALID_BLOB, lineno, "text after the output line");
        if (tok[0] == "output") {
            if (tok.size() != 2 || !parse_ref(tok[1], t.out) || t.out >= (int)t.nodes.size()) return fail(CANVAS_INVALID_BLOB, lineno, "bad output reference");
            done = true;
            continue;
        }
        int id;
        if (tok.size() < 4 || !parse_ref(tok[0], id) || tok[1] != "=") return fail(CANVAS_INVALID_BLOB, lineno, "expected '%k = op %operand ...'");
        if (id != (int)t.nodes.size()) return fail(CANVAS_INVALID_BLOB, lineno, "node ids must be consecutive from 1");
        if (id >= CANVAS_MAX_NODES) return fail(CANVAS_UNSUPPORTED, lineno, "too many nodes");
        TNode nd;
        auto it = ops.find(tok[2]);
        if (it == ops.end()) return fail(CANVAS_UNKNOWN_OP, lineno, "unknown op '" + tok[2] + "'");
        nd.op = it->second;
        nd.opname = tok[2];
        if (!parse_ref(tok[3], nd.a) || nd.a >= id) return fail(CANVAS_INVALID_BLOB, lineno, "operand must be an earlier node");
        size_t first_attr = 4;
        if (nd.op == TOp::Binary) {
            if (tok.size() < 5 || !parse_ref(tok[4], nd.b) || nd.b >= id) return fail(CANVAS_INVALID_BLOB, lineno, "binary needs two earlier operands");
            first_attr = 5;
        }
        const auto sk = symbolic_keys().find(nd.opname);
        for (size_t i = first_attr; i < tok.size(); i++) {
            const size_t eq = tok[i].find('=');
            if (eq == std::string::npos || eq == 0) return fail(CANVAS_INVALID_BLOB, lineno, "expected key=value, got '" + tok[i] + "'");
            Attr a;
            a.key = tok[i].substr(0, eq);
            a.raw = tok[i].substr(eq + 1);
            if (sk != symbolic_keys().end() && std::find(sk->second.begin(), sk->second.end(), a.key) != sk->second.end()) {
                a.symbolic = true;
                if (!sym::parse_mono(a.raw, a.m)) return fail(CANVAS_INVALID_BLOB, lineno, "bad size expression '" + a.raw + "'");
            }
            nd.attrs.push_back(a);
        }
        t.nodes.push_back(nd);
    }
    if (!header) return fail(CANVAS_INVALID_BLOB, 0, "empty blob: expected header 'canvas-template 1'");
    if (t.out < 0) return fail(CANVAS_INVALID_BLOB, 0, "template has no output line");
    return infer(t);
}

std::vector<int> free_vars(const Template& t) {
    bool seen[sym::kMaxVars + 1] = {};
    for (const auto& nd : t.nodes)
        for (const auto& a : nd.attrs)
            if (a.symbolic)
                for (int j = 1; j <= sym::kMaxVars; j++)
                    if (a.m.var_exp(j) != 0) seen[j] = true;
    std::vector<int> v;
    for (int j = 1; j <= sym::kMaxVars; j++)
        if (seen[j]) v.push_back(j);
    return v;
}

std::string shape_text(const TNode& nd) {
    std::string s = "[";
    if (nd.grp.is_one()) s += sym::to_text(nd.C);
    else s += sym::to_text(nd.grp) + ", " + sym::to_text(nd.C / nd.grp);
    s += " |";
    for (size_t i = 0; i < nd.taps.size(); i++) s += (i ? ", " : " ") + sym::to_text(nd.taps[i]);
    if (!nd.taps.empty()) s += " |";
    s += std::string(" ") + ((nd.pooled & 1) ? "1" : "H") + ", " + ((nd.pooled & 2) ? "1" : "W") + "]";
    return s;
}

int write_text(const std::string& s, char* buf, size_t buf_len, size_t* needed) {
    if (needed) *needed = s.size() + 1;
    if (!buf || buf_len < s.size() + 1) return canvas::set_last_error(CANVAS_BAD_ARG, "text buffer too small");
    std::memcpy(buf, s.c_str(), s.size() + 1);
    return CANVAS_OK;
}

// all factors of an all-numerator monomial (Section 6.2: "the set of all factors of x_RHS^k R_RHS")
void factors_of(const Mono& n, std::vector<Mono>& out) {
    std::vector<int64_t> divs;
    for (int64_t d = 1; d * d <= n.num; d++)
        if (n.num % d == 0) {
            divs.push_back(d);
            if (d != n.num / d) divs.push_back(n.num / d);
        }
    std::vector<Mono> cur;
    for (int64_t d : divs) cur.push_back(Mono::integer(d));
    for (int a = 0; a < sym::kAtoms; a++) {
        if (n.e[a] <= 0) continue;
        std::vector<Mono> next;
        for (const auto& m : cur) {
            Mono f = m;
            for (int k = 0; k <= n.e[a]; k++) {
                next.push_back(f);
                f = f * Mono::atom(a);
            }
        }
        cur.swap(next);
    }
    out = cur;
}

bool bind_target(const canvas_target& tg, int64_t G, Binding& b, std::string& why) {
    if (tg.C < 1 || tg.KH < 1 || tg.KW < 1 || tg.H < 1 || tg.W < 1 || G < 1) { why = "target sizes and G must be positive"; return false; }
    if (tg.C % G) { why = "G does not divide C"; return false; }
    b.v[sym::aG] = G;
    b.v[sym::aCg] = tg.C / G;
    b.v[sym::aKH] = tg.KH;
    b.v[sym::aKW] = tg.KW;
    b.v[sym::aH] = tg.H;
    b.v[sym::aW] = tg.W;
    return true;
}

// multiply-accumulates and weights of all fc nodes of one target (x bound in b)
bool cost_of(const Template& t, const Binding& b, double& flops, double& params) {
    flops = params = 0.0;
    for (const auto& nd : t.nodes) {
        if (nd.op != TOp::Fc) continue;
        const TNode& A = t.nodes[nd.a];
        const Mono w = nd.C * A.C * product(A.taps) / nd.groups_used;  // out * (C_in / G) * taps
        int64_t p, q;
        if (!sym::evaluate(w, b, p, q) || q != 1) return false;
        params += (double)p;
        flops += (double)p * ((A.pooled & 1) ? 1.0 : (double)b.v[sym::aH]) * ((A.pooled & 2) ? 1.0 : (double)b.v[sym::aW]);
    }
    return true;
}

}  // namespace

struct canvas_template {
    Template t;
};

extern "C" {

int canvas_template_parse(const void* blob, size_t blob_len, canvas_template** out) {
    if (!blob || !out) return canvas::set_last_error(CANVAS_BAD_ARG, "null blob or output pointer");
    auto h = new canvas_template();
    const int rc = parse_template((const char*)blob, blob_len, h->t);
    if (rc) {
        delete h;
        return rc;
    }
    *out = h;
    return CANVAS_OK;
}

int canvas_template_query(const canvas_template* t, canvas_template_info* info) {
    if (!t || !info) return canvas::set_last_error(CANVAS_BAD_ARG, "null argument");
    std::memset(info, 0, sizeof *info);
    info->n_nodes = (int)t->t.nodes.size();
    info->out_node = t->t.out;
    for (const auto& nd : t->t.nodes) info->n_fc += nd.op == TOp::Fc;
    const auto fv = free_vars(t->t);
    info->n_free = (int)fv.size();
    for (size_t i = 0; i < fv.size(); i++) info->free_var[i] = fv[i];
    for (const auto& nd : t->t.nodes)
        for (const auto& a : nd.attrs)
            if (a.symbolic && a.m.e[sym::aG] != a.m.e[sym::aCg]) info->uses_G = 1;  // G other than inside C = G * C/G
    return CANVAS_OK;
}

int canvas_template_node_shape(const canvas_template* t, int node, char* buf, size_t buf_len, size_t* needed) {
    if (!t || node < 0 || node >= (int)t->t.nodes.size()) return canvas::set_last_error(CANVAS_BAD_ARG, "bad template or node");
    return write_text(shape_text(t->t.nodes[node]), buf, buf_len, needed);
}

int canvas_template_substitutions(const canvas_template* t, int node, int* var, int* count, char* buf, size_t buf_len, size_t* needed) {
    if (!t || !var || !count || node < 1 || node >= (int)t->t.nodes.size() || t->t.nodes[node].op != TOp::Binary)
        return canvas::set_last_error(CANVAS_BAD_ARG, "not a binary node of this template");
    const TNode& nd = t->t.nodes[node];
    const TNode &A = t->t.nodes[nd.a], &B = t->t.nodes[nd.b];
    const int v = A.C.single_var();
    if (v <= 0) return canvas::set_last_error(CANVAS_BAD_ARG, "the LHS of this node carries no free dynamic variable");
    *var = v;
    const Mono xl = Mono::atom(sym::aX0 + v - 1);
    const Mono lhs_rest = A.C * product(A.taps) / xl;  // R_LHS
    std::vector<Mono> subs;
    if (nd.find("lhs")) {
        // laid over the pixels: #LHS must equal H * W
        const Mono only = Mono::atom(sym::aH) * Mono::atom(sym::aW) / lhs_rest;
        if (!only.has_negative_exponent() && only.den == 1) subs.push_back(only);
    } else {
        const Mono numer = B.C * product(B.taps) / lhs_rest;  // x_R^k R_RHS / R_LHS, fully simplified
        if (!numer.has_negative_exponent() && numer.den == 1 && numer.var_exp(v) == 0) factors_of(numer, subs);
    }
    std::vector<std::string> text;
    for (const auto& m : subs) text.push_back(sym::to_text(m));
    std::sort(text.begin(), text.end());
    *count = (int)text.size();
    std::string s;
    for (const auto& l : text) s += l + "\n";
    return write_text(s, buf, buf_len, needed);
}

int canvas_template_substitute(canvas_template* t, int var, const char* expr) {
    if (!t || !expr || var < 1 || var > sym::kMaxVars) return canvas::set_last_error(CANVAS_BAD_ARG, "bad template, variable or expression");
    Mono e;
    if (!sym::parse_mono(expr, e)) return canvas::set_last_error(CANVAS_INVALID_BLOB, std::string("bad size expression '") + expr + "'");
    if (e.var_exp(var) != 0) return canvas::set_last_error(CANVAS_BAD_ARG, "the expression mentions the variable it replaces");
    const auto fv = free_vars(t->t);
    if (std::find(fv.begin(), fv.end(), var) == fv.end()) return canvas::set_last_error(CANVAS_BAD_ARG, "x" + std::to_string(var) + " is not a free variable of this template");
    Template copy = t->t;
    const Mono x = Mono::atom(sym::aX0 + var - 1);
    for (auto& nd : copy.nodes)
        for (auto& a : nd.attrs) {
            if (!a.symbolic) continue;
            const int k = a.m.var_exp(var);
            for (int i = 0; i < k; i++) a.m = a.m / x * e;
            for (int i = 0; i < -k; i++) a.m = a.m * x / e;
            a.raw = sym::to_text(a.m);
        }
    const int rc = infer(copy);
    if (rc) return rc;
    t->t = copy;
    return CANVAS_OK;
}

int canvas_group_candidates(const int64_t* C, int n_targets, int64_t* out, int cap, int* count) {
    if (!C || n_targets < 1 || !count || (cap > 0 && !out)) return canvas::set_last_error(CANVAS_BAD_ARG, "bad arguments");
    int64_t g = 0;
    for (int i = 0; i < n_targets; i++) {
        if (C[i] < 1) return canvas::set_last_error(CANVAS_BAD_ARG, "channel counts must be positive");
        g = std::gcd(g, C[i]);
    }
    int n = 0;
    for (int64_t d = 2; d <= g; d++)
        if (g % d == 0) {
            if (n < cap) out[n] = d;
            n++;
        }
    *count = n;
    if (n > cap) return canvas::set_last_error(CANVAS_BAD_ARG, "candidate buffer too small");
    return CANVAS_OK;
}

int canvas_template_solve(const canvas_template* t, const canvas_target* targets, int n_targets, int64_t G, double flops_budget,
                          double params_budget, int64_t* x, canvas_solve_result* result) {
    if (!t || !targets || n_targets < 1 || !x) return canvas::set_last_error(CANVAS_BAD_ARG, "null argument or no targets");
    const Template& T = t->t;
    const auto fv = free_vars(T);
    std::vector<Binding> bind(n_targets);
    std::vector<std::vector<int64_t>> lcm(n_targets, std::vector<int64_t>(sym::kMaxVars + 1, 1));
    for (int i = 0; i < n_targets; i++) {
        std::string why;
        if (!bind_target(targets[i], G, bind[i], why)) return canvas::set_last_error(CANVAS_BAD_ARG, "target " + std::to_string(i) + ": " + why);
        for (const auto& one : T.must_be_one)
            if (!one.first.is_one())
                return canvas::set_last_error(CANVAS_SHAPE_MISMATCH, "node " + std::to_string(one.second) + ": the LHS laid over the pixels has " +
                                                                         sym::to_text(Mono::atom(sym::aH) * Mono::atom(sym::aW) / one.first) + " elements, not H*W");
        for (const auto& c : T.must_be_integer) {
            const int j = c.m.single_var();
            const std::string where = "target " + std::to_string(i) + ", node " + std::to_string(c.node) + ": " + c.what + " = " + sym::to_text(c.m);
            if (j < 0) return canvas::set_last_error(CANVAS_SHAPE_MISMATCH, where + " holds more than one dynamic variable");
            if (j > 0 && c.m.var_exp(j) < 0) return canvas::set_last_error(CANVAS_SHAPE_MISMATCH, where + ": a free variable in a denominator, substitute it first");
            int64_t p, q;
            const Mono rest = j > 0 ? c.m / Mono::atom(sym::aX0 + j - 1) : c.m;
            if (!sym::evaluate(rest, bind[i], p, q)) return canvas::set_last_error(CANVAS_SHAPE_MISMATCH, where + " cannot be evaluated");
            if (j == 0) {
                if (q != 1) return canvas::set_last_error(CANVAS_SHAPE_MISMATCH, where + " is no integer");
            } else {
                lcm[i][j] = std::lcm(lcm[i][j], q);  // p * x / q with gcd(p, q) = 1: q must divide x
            }
        }
    }
    // step 1: base values proportional to C_i, target of least C first
    int i1 = 0;
    for (int i = 1; i < n_targets; i++)
        if (targets[i].C < targets[i1].C) i1 = i;
    std::vector<std::vector<int64_t>> X(n_targets, std::vector<int64_t>(sym::kMaxVars + 1, 0));
    for (int j : fv)
        for (int i = 0; i < n_targets; i++) {
            const __int128 up = (__int128)targets[i].C * lcm[i1][j], down = (__int128)targets[i1].C * lcm[i][j];
            const int64_t k = i == i1 ? 1 : (int64_t)((up + down - 1) / down);
            X[i][j] = k * lcm[i][j];
        }
    auto net_cost = [&](double& flops, double& params) {
        flops = params = 0.0;
        for (int i = 0; i < n_targets; i++) {
            Binding b = bind[i];
            for (int j : fv) b.v[sym::aX0 + j - 1] = X[i][j];
            double f, p;
            if (!cost_of(T, b, f, p)) return false;
            flops += f;
            params += p;
        }
        return true;
    };
    double flops, params;
    if (!net_cost(flops, params)) return canvas::set_last_error(CANVAS_SHAPE_MISMATCH, "a weight shape is no integer at the base values");
    auto within = [&](double f, double p) { return (flops_budget <= 0 || f <= flops_budget) && (params_budget <= 0 || p <= params_budget); };
    if (!within(flops, params)) return canvas::set_last_error(CANVAS_UNSUPPORTED, "the base values already exceed a budget");
    int rounds = 0;
    if (flops_budget > 0 || params_budget > 0) {
        const bool by_flops = flops_budget > 0;
        for (;;) {
            // step 2: sensitivities at the current values, then doublings in ascending order
            struct Cand { double delta; int i, j; };
            std::vector<Cand> cands;
            for (int i = 0; i < n_targets; i++)
                for (int j : fv) {
                    if (X[i][j] > ((int64_t)1 << 40)) continue;
                    X[i][j] *= 2;
                    double f, p;
                    const bool ok = net_cost(f, p);
                    X[i][j] /= 2;
                    if (!ok) continue;
                    const double d = by_flops ? f - flops : p - params;
                    if (d > 0) cands.push_back({d, i, j});  // (a variable that costs nothing is left alone)
                }
            std::stable_sort(cands.begin(), cands.end(), [](const Cand& a, const Cand& b) { return a.delta < b.delta; });
            bool changed = false;
            for (const auto& c : cands) {
                X[c.i][c.j] *= 2;
                double f, p;
                if (net_cost(f, p) && within(f, p)) {
                    flops = f;
                    params = p;
                    changed = true;
                } else {
                    X[c.i][c.j] /= 2;
                }
            }
            if (!changed) break;
            rounds++;
        }
    }
    for (int i = 0; i < n_targets; i++)
        for (int j = 1; j <= sym::kMaxVars; j++) x[(size_t)i * CANVAS_MAX_VARS + j - 1] = X[i][j];
    if (result) {
        std::memset(result, 0, sizeof *result);
        result->flops = flops;
        result->params = params;
        result->rounds = rounds;
    }
    return CANVAS_OK;
}

int canvas_template_instantiate(const canvas_template* t, const canvas_target* target, int64_t G, const int64_t* x, char* buf,
                                size_t buf_len, size_t* needed) {
    if (!t || !target || !x) return canvas::set_last_error(CANVAS_BAD_ARG, "null argument");
    Binding b;
    std::string why;
    if (!bind_target(*target, G, b, why)) return canvas::set_last_error(CANVAS_BAD_ARG, why);
    for (int j : free_vars(t->t)) {
        if (x[j - 1] < 1) return canvas::set_last_error(CANVAS_BAD_ARG, "x" + std::to_string(j) + " has no positive value");
        b.v[sym::aX0 + j - 1] = x[j - 1];
    }
    std::string s = "canvas-dag 1\n";
    for (size_t k = 1; k < t->t.nodes.size(); k++) {
        const TNode& nd = t->t.nodes[k];
        s += "%" + std::to_string(k) + " = " + nd.opname + " %" + std::to_string(nd.a);
        if (nd.op == TOp::Binary) s += " %" + std::to_string(nd.b);
        for (const auto& a : nd.attrs) {
            if (!a.symbolic) {
                s += " " + a.key + "=" + a.raw;
                continue;
            }
            int64_t p, q;
            if (!sym::evaluate(a.m, b, p, q) || q != 1)
                return canvas::set_last_error(CANVAS_SHAPE_MISMATCH, "node " + std::to_string(k) + ": " + a.key + " = " + sym::to_text(a.m) + " is no integer for this target");
            s += " " + a.key + "=" + std::to_string(p);
        }
        s += "\n";
    }
    s += "output %" + std::to_string(t->t.out) + "\n";
    return write_text(s, buf, buf_len, needed);
}

void canvas_template_destroy(canvas_template* t) { delete t; }

}  // extern "C"
