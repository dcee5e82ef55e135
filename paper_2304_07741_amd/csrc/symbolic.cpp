// Monomials over the template symbols: parsing, printing, evaluation.
#include "symbolic.hpp"

#include <cstdlib>

namespace canvas {
namespace sym {

namespace {

bool parse_factor(const std::string& f, Mono& out) {
    if (f.empty()) return false;
    if (f == "C") { out = Mono::channels(); return true; }
    if (f == "G") { out = Mono::atom(aG); return true; }
    if (f == "KH") { out = Mono::atom(aKH); return true; }
    if (f == "KW") { out = Mono::atom(aKW); return true; }
    if (f == "H") { out = Mono::atom(aH); return true; }
    if (f == "W") { out = Mono::atom(aW); return true; }
    if (f[0] == 'x') {
        char* end = nullptr;
        const long j = std::strtol(f.c_str() + 1, &end, 10);
        if (end == f.c_str() + 1 || *end || j < 1 || j > kMaxVars) return false;
        out = Mono::atom(aX0 + (int)j - 1);
        return true;
    }
    char* end = nullptr;
    const long long v = std::strtoll(f.c_str(), &end, 10);
    if (end == f.c_str() || *end || v < 1 || v > (1LL << 40)) return false;
    out = Mono::integer(v);
    return true;
}

}  // namespace

bool parse_mono(const std::string& text, Mono& out) {
    out = Mono::one();
    size_t pos = 0;
    char op = '*';
    while (pos <= text.size()) {
        size_t next = text.find_first_of("*/", pos);
        if (next == std::string::npos) next = text.size();
        Mono f;
        if (!parse_factor(text.substr(pos, next - pos), f)) return false;
        out = op == '*' ? out * f : out / f;
        if (next == text.size()) break;
        op = text[next];
        pos = next + 1;
    }
    return true;
}

std::string to_text(const Mono& m) {
    // in terms of C and G: Cg = C / G
    int e[kAtoms];
    for (int i = 0; i < kAtoms; i++) e[i] = m.e[i];
    const int eC = m.e[aCg], eG = m.e[aG] - m.e[aCg];
    static const char* names[] = {"G", "C", "KH", "KW", "H", "W"};
    e[aG] = eG;
    e[aCg] = eC;
    const int order[] = {aCg, aG, aKH, aKW, aH, aW};
    std::string up, down;
    auto add = [](std::string& s, const std::string& f) {
        if (!s.empty()) s += "*";
        s += f;
    };
    if (m.num != 1) add(up, std::to_string(m.num));
    if (m.den != 1) add(down, std::to_string(m.den));
    auto emit = [&](int a, const std::string& name) {
        for (int k = 0; k < e[a]; k++) add(up, name);
        for (int k = 0; k < -e[a]; k++) add(down, name);
    };
    for (int a : order) emit(a, names[a]);
    for (int j = 1; j <= kMaxVars; j++) emit(aX0 + j - 1, "x" + std::to_string(j));
    if (up.empty()) up = "1";
    if (down.empty()) return up;
    std::string s = up;
    size_t pos = 0;
    while (pos <= down.size()) {  // a / b / c: every factor of the denominator after its own slash
        size_t next = down.find('*', pos);
        if (next == std::string::npos) next = down.size();
        s += "/" + down.substr(pos, next - pos);
        if (next == down.size()) break;
        pos = next + 1;
    }
    return s;
}

bool evaluate(const Mono& m, const Binding& b, int64_t& p, int64_t& q) {
    __int128 up = m.num, down = m.den;
    for (int i = 0; i < kAtoms; i++) {
        if (m.e[i] == 0) continue;
        if (b.v[i] <= 0) return false;
        for (int k = 0; k < (m.e[i] > 0 ? m.e[i] : -m.e[i]); k++) {
            if (m.e[i] > 0) up *= b.v[i];
            else down *= b.v[i];
            // keep the fraction reduced so that intermediate products stay small
            __int128 a = up, c = down;
            while (c) {
                const __int128 t = a % c;
                a = c;
                c = t;
            }
            up /= a;
            down /= a;
            if (up > ((__int128)1 << 62) || down > ((__int128)1 << 62)) return false;
        }
    }
    p = (int64_t)up;
    q = (int64_t)down;
    return true;
}

}  // namespace sym
}  // namespace canvas
