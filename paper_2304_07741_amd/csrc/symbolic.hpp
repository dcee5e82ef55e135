// Symbolic sizes of kernel templates (Canvas paper, Section 6.2: every dimension is numerator / denominator
// of products of C, G, K_H, K_W, H, W and dynamic variables x_j).  Host only.
#pragma once
#include <cstdint>
#include <numeric>
#include <string>
#include <vector>

namespace canvas {
namespace sym {

// atoms: the group number, the channels of one group (C = G * Cg), the window, the image, the dynamic variables
enum Atom : int { aG = 0, aCg, aKH, aKW, aH, aW, aX0 };  // aX0 + j - 1 is x_j
constexpr int kMaxVars = 8;
constexpr int kAtoms = aX0 + kMaxVars;

// (num / den) * prod atom^e, num > 0, den > 0, gcd(num, den) = 1; num == 0 marks "invalid"
struct Mono {
    int64_t num = 1, den = 1;
    int e[kAtoms] = {};

    static Mono one() { return Mono(); }
    static Mono integer(int64_t v) {
        Mono m;
        m.num = v;
        return m;
    }
    static Mono atom(int a) {
        Mono m;
        m.e[a] = 1;
        return m;
    }
    static Mono channels() {  // C = G * (C / G)
        Mono m;
        m.e[aG] = 1;
        m.e[aCg] = 1;
        return m;
    }
    void reduce() {
        const int64_t g = std::gcd(num, den);
        if (g > 1) {
            num /= g;
            den /= g;
        }
    }
    Mono operator*(const Mono& o) const {
        Mono r = *this;
        r.num *= o.num;
        r.den *= o.den;
        r.reduce();
        for (int i = 0; i < kAtoms; i++) r.e[i] += o.e[i];
        return r;
    }
    Mono operator/(const Mono& o) const {
        Mono r = *this;
        r.num *= o.den;
        r.den *= o.num;
        r.reduce();
        for (int i = 0; i < kAtoms; i++) r.e[i] -= o.e[i];
        return r;
    }
    bool operator==(const Mono& o) const {
        if (num != o.num || den != o.den) return false;
        for (int i = 0; i < kAtoms; i++)
            if (e[i] != o.e[i]) return false;
        return true;
    }
    bool is_one() const { return *this == Mono(); }
    int var_exp(int j) const { return e[aX0 + j - 1]; }
    // the one variable in it (0 when none, -1 when several or a power other than +-1)
    int single_var() const {
        int v = 0;
        for (int j = 1; j <= kMaxVars; j++)
            if (var_exp(j) != 0) {
                if (v != 0 || (var_exp(j) != 1 && var_exp(j) != -1)) return -1;
                v = j;
            }
        return v;
    }
    bool has_negative_exponent() const {
        for (int i = 0; i < kAtoms; i++)
            if (e[i] < 0) return true;
        return false;
    }
    int degree() const {
        int d = 0;
        for (int i = 0; i < kAtoms; i++) d += e[i] > 0 ? e[i] : -e[i];
        return d;
    }
};

// "x2*KW/G", "C/2", "3"; false on a syntax error
bool parse_mono(const std::string& text, Mono& out);
// canonical text: integer coefficient first, then atoms in the order C G Cg->"C/G" KH KW H W x1.., "/..." for the denominator
std::string to_text(const Mono& m);

// concrete assignment of all atoms
struct Binding {
    int64_t v[kAtoms] = {};
};
// value as a reduced fraction p / q (false on overflow or a zero atom)
bool evaluate(const Mono& m, const Binding& b, int64_t& p, int64_t& q);

}  // namespace sym
}  // namespace canvas
