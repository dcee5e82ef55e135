// Pattern match and lowering for  x -> Shift* -> grouped FC -> unary{0..2} -> (binary add with x) -> output.
#include <algorithm>
#include <cstdlib>
#include <vector>

#include "lowering.hpp"
#include "sgfc_kernels.hpp"

namespace canvas {

std::unique_ptr<Lowering> lower_sgfc(const Dag& dag, bool bf16) {
    if (!bf16) return nullptr;
    const int n = (int)dag.nodes.size();
    for (int k = 0; k < n; k++)
        if (!dag.nodes[k].live || dag.nodes[k].pooled) return nullptr;  // (no tensor with folded spatial dims in this pattern)
    int k = 1, prev = 0;
    // shifts
    std::vector<int> sdh(dag.nodes[0].C, 0), sdw(dag.nodes[0].C, 0);
    std::vector<bool> shifted(dag.nodes[0].C, false);
    while (k < n && dag.nodes[k].op == Op::Shift) {
        const Node& s = dag.nodes[k];
        if (s.a != prev || s.T != 1) return nullptr;
        if (s.dh != 0 || s.dw != 0)
            for (int c = s.c0; c < s.c1; c++) {
                if (shifted[c]) return nullptr;  // two shifts with zero fill do not compose into one
                shifted[c] = true;
                sdh[c] = s.dh;
                sdw[c] = s.dw;
            }
        prev = k++;
    }
    if (k >= n || dag.nodes[k].op != Op::Fc || dag.nodes[k].a != prev) return nullptr;
    const Node fc = dag.nodes[k];
    const int C = dag.nodes[0].C, G = fc.groups, CG = C / G, OG = fc.out / G;
    if (dag.nodes[fc.a].T != 1 || CG % 16 || OG % 16 || !sgfc::supported(CG / 16, OG / 16) || G > sgfc::kMaxGroups) return nullptr;
    prev = k++;
    sgfc::Params P;
    if (k < n && dag.nodes[k].op == Op::Unary) {
        const Node& u = dag.nodes[k];
        if (u.a != prev || u.kind > kExpClip) return nullptr;  // the kernels are instantiated for relu, abs, gelu, expclip
        P.act = u.kind;
        P.ulo = u.lo;
        P.uhi = u.hi;
        prev = k++;
    }
    if (k < n && dag.nodes[k].op == Op::Binary) {
        const Node& b = dag.nodes[k];
        bool with_input = (b.a == 0 && b.b == prev) || (b.a == prev && b.b == 0);
        if (!with_input || b.kind != kAdd || fc.out != C) return nullptr;
        P.residual = 1;
        prev = k++;
    }
    if (k != n || dag.out != prev) return nullptr;
    // every FC group must see one shift
    for (int g = 0; g < G; g++) {
        for (int c = g * CG; c < (g + 1) * CG; c++)
            if (sdh[c] != sdh[g * CG] || sdw[c] != sdw[g * CG]) return nullptr;
        P.dh[g] = sdh[g * CG];
        P.dw[g] = sdw[g * CG];
    }
    const int Pn = dag.P();
    if (Pn % 8 || dag.W < 8 || (int64_t)Pn * dag.W >= ((int64_t)1 << 31)) return nullptr;
    // tensors are addressed with 32-bit byte offsets through buffer descriptors
    if ((int64_t)dag.N * std::max(C, fc.out) * Pn * 2 >= ((int64_t)1 << 31) || dag.N > 65535) return nullptr;
    if ((int64_t)dag.N * ((Pn + 127) / 128) * ((Pn + 127) / 128) >= ((int64_t)1 << 31)) return nullptr;
    // the input may only feed the first node of the chain and the residual
    for (int j = 2; j < n; j++) {
        const Node& nd = dag.nodes[j];
        bool is_res = P.residual && j == n - 1;
        if (!is_res && (nd.a == 0 || nd.b == 0)) return nullptr;
    }

    P.N = dag.N;
    P.C = C;
    P.H = dag.H;
    P.W = dag.W;
    P.P = Pn;
    P.G = G;
    P.magicW = (uint32_t)((((uint64_t)1 << 32) + dag.W - 1) / dag.W);
    P.chunks = (Pn + 127) / 128;
    P.magicChunks = (uint32_t)((((uint64_t)1 << 32) + P.chunks - 1) / P.chunks);
    P.total_tiles = (long long)dag.N * G * P.chunks;
    int tpw = 2;  // two tiles per wavefront measured best at the ResNet-18 stage-1 shape
    if (const char* e = std::getenv("CANVAS_SGFC_TPW")) tpw = std::max(1, std::atoi(e));
    P.tiles_per_wave = tpw;
    const int tiles_per_group = dag.N * P.chunks;
    P.wgs_per_group = (tiles_per_group + 4 * tpw - 1) / (4 * tpw);

    auto low = std::make_unique<Lowering>();
    low->fused = true;
    low->strided_io = true;
    const int elems = OG * CG;
    low->ws_bytes = align_up((uint64_t)G * P.wgs_per_group * elems * 4);
    const int KC = CG / 16, MO = OG / 16;
    const int widx = fc.widx;
    const int xs_dense = C * Pn, ys_dense = fc.out * Pn;
    const double act = 2.0 * dag.numel(0), wb = 2.0 * G * elems;
    const double flops = 2.0 * dag.N * Pn * fc.out * CG;
    low->fwd.push_back({"sgfc_fwd", act + 2.0 * dag.numel(dag.out) + wb, flops, [=](const RunArgs& a) {
                            sgfc::Params Q = P;
                            Q.xs = a.x_stride ? (int)a.x_stride : xs_dense;
                            Q.ys = a.y_stride ? (int)a.y_stride : ys_dense;
                            Q.x = (const uint16_t*)a.x;
                            Q.w = (const uint16_t*)a.w[widx];
                            Q.y = (uint16_t*)a.y;
                            sgfc::forward(Q, KC, MO, a.stream);
                        }});
    low->bwd.push_back({"sgfc_bwd", 2.0 * act + 2.0 * dag.numel(dag.out) + wb + 4.0 * G * P.wgs_per_group * elems, 3.0 * flops,
                        [=](const RunArgs& a) {
                            sgfc::Params Q = P;
                            Q.xs = a.x_stride ? (int)a.x_stride : xs_dense;
                            Q.ys = a.y_stride ? (int)a.y_stride : ys_dense;
                            Q.x = (const uint16_t*)a.x;
                            Q.w = (const uint16_t*)a.w[widx];
                            Q.dy = (const uint16_t*)a.dy;
                            Q.dx = (uint16_t*)a.dx;
                            Q.partial = (float*)a.ws;
                            sgfc::backward(Q, KC, MO, a.stream);
                        }});
    const int wpg = P.wgs_per_group;
    low->bwd.push_back({"sgfc_dw_reduce", 4.0 * G * elems * (wpg + 1), 0, [=](const RunArgs& a) {
                            sgfc::dw_reduce((const float*)a.ws, (float*)a.dw[widx], G, wpg, elems, a.stream);
                        }});
    return low;
}

}  // namespace canvas
