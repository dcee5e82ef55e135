// Host-side micro-DAG: parsed nodes with inferred shapes (no GPU dependency).
//
// Primitive semantics follow Section 5 of the Canvas paper (table of fine-grained
// primitives); the canonical tensor form is [N, C, T, H, W] with T the number of
// unfolded taps (1 when there are none).
#pragma once
#include <cstdint>
#include <string>
#include <vector>

namespace canvas {

enum class Op : int { Input = 0, Unfold, Shift, Fc, Unary, Binary, Softmax, Fold, Group };
enum UnaryKind : int { kRelu = 0, kAbs, kGelu, kExpClip, kSin };
enum BinaryKind : int { kAdd = 0, kMul, kSub, kBinMin, kBinMax };
enum AxisKind : int { kAxisC = 0, kAxisT, kAxisCT, kAxisH, kAxisW, kAxisHW };
enum FoldKind : int { kSum = 0, kAvg, kMax };

struct Node {
    Op op = Op::Input;
    int a = -1, b = -1;          // operands (binary: a = LHS, b = RHS)
    int kh = 1, kw = 1;          // unfold window
    int dh = 0, dw = 0;          // shift offset
    int c0 = 0, c1 = 0;          // shifted channel slice [c0, c1)
    int groups = 1, out = 0;     // fc
    int kind = 0;                // UnaryKind / BinaryKind / AxisKind / FoldKind
    float lo = 0.f, hi = 0.f;    // expclip bounds
    int axis_hw = 0;             // fold: mask of the spatial dims folded by this node (1 = H, 2 = W, 3 = both), 0 = over the taps
    int axis_c = 0;              // fold: 1 = over the C / groups channels of each of `groups` channel groups
    int pooled = 0;              // mask of the spatial dims folded away so far: 1 = H ([N, C, T, 1, W]), 2 = W, 3 = both
    int grp = 1;                 // Group view of the channel dim, [grp, C / grp] (1 = none)
    bool lhs_pixels = false;     // binary: the pooled LHS has H*W elements, element p meets pixel p of every channel and tap
    int bgroups = 1;             // binary: > 1 when both operands carry this same view, the blend then runs inside each group
    int C = 0, T = 1;            // inferred shape
    int widx = -1;               // fc: index into the weight list
    bool live = false;           // reaches the output
};

struct Dag {
    std::vector<Node> nodes;     // nodes[0] is the input
    int out = -1;
    int N = 0, H = 0, W = 0;
    int n_weights = 0;
    std::vector<int> weight_node;

    int P() const { return H * W; }
    int Hk(int k) const { return (nodes[k].pooled & 1) ? 1 : H; }
    int Wk(int k) const { return (nodes[k].pooled & 2) ? 1 : W; }
    int Pk(int k) const { return Hk(k) * Wk(k); }  // pixels of node k
    int64_t numel(int k) const { return (int64_t)N * nodes[k].C * nodes[k].T * Pk(k); }
};

// Status codes mirror canvas_status in the public header.
// A Group node is a view: nodes that name it as an operand are wired to the tensor it views (and take
// the view from it), so a Group node is live only when it is the output itself.
int parse_dag(const char* blob, size_t len, const int64_t in_shape[4], Dag& dag, std::string& err);

// The DAG without its dead Group nodes, renumbered: what the lowerings work on.
Dag without_dead_views(const Dag& dag);

// Broadcast index map (Section 5, Blending primitives): the LHS element that meets RHS element (c, t).
inline void broadcast_src(int CL, int TL, int CR, int TR, int c, int t, int& cl, int& tl) {
    if (CL == CR) {
        cl = c;
        tl = t % TL;
    } else {
        int64_t j = ((int64_t)c * TR + t) % ((int64_t)CL * TL);
        cl = (int)(j / TL);
        tl = (int)(j % TL);
    }
}

}  // namespace canvas
