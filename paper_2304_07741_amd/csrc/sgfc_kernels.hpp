// Launchers of the fused shift -> grouped FC -> unary chain -> (+ input) kernels (bf16, NCHW).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace canvas {
namespace sgfc {

constexpr int kMaxGroups = 64;

struct Params {
    const uint16_t* x = nullptr;   // [N, C, H, W] bf16
    const uint16_t* w = nullptr;   // [G, OG, CG] bf16
    uint16_t* y = nullptr;         // [N, G*OG, H, W] bf16 (forward)
    const uint16_t* dy = nullptr;  // backward
    uint16_t* dx = nullptr;
    float* partial = nullptr;      // [G, wgs_per_group, OG*CG] fp32 partial weight gradients, one per workgroup
    int N = 0, C = 0, H = 0, W = 0, P = 0, G = 0;
    int xs = 0, ys = 0;            // elements between consecutive images of x / dx and of y / dy (C * P and G * OG * P when dense;
                                   // larger when the tensor is a channel slice of a wider one)
    int chunks = 0;                // ceil(P / 128)
    long long total_tiles = 0;     // N * G * chunks
    int wgs_per_group = 0, tiles_per_wave = 1;  // backward work split
    uint32_t magicChunks = 0;      // ceil(2^32 / chunks)
    uint32_t magicW = 0;           // ceil(2^32 / W): p / W == umulhi(p, magicW) for p * W < 2^32
    int act = -1;                  // -1: no unary node, else the UnaryKind applied to the FC output
    float ulo = 0.f, uhi = 0.f;    // expclip bounds
    int residual = 0;              // 1: the input is added to the result
    int dh[kMaxGroups] = {0}, dw[kMaxGroups] = {0};  // shift of each FC group's channels
};

// KC = CG/16, MO = OG/16
bool supported(int KC, int MO);
void forward(const Params& P, int KC, int MO, hipStream_t s);
void backward(const Params& P, int KC, int MO, hipStream_t s);
void dw_reduce(const float* partial, float* dw, int G, int n_partials, int elems, hipStream_t s);

}  // namespace sgfc
}  // namespace canvas
