// Grouped fully-connected contraction on bf16 MFMA (fp32 accumulate) for NCHW tensors, with an optional
// implicit Unfold of the operand (im2col never materialised).  Section 5 of the Canvas paper:
// Fully-connected, Group, Unfold.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace canvas {
namespace gfc {

// A "row tensor" is [N, G, R, P]: R rows (channel x materialised tap) per group, P = H*W pixels per row.
// With a virtual window KH x KW every row is seen TV = KH*KW times, shifted by the tap offset and
// zero outside the image; the contraction index is k = row*TV + tv, K = R*TV.
struct Params {
    const void* src = nullptr;    // row tensor, fp32 or bf16
    const uint16_t* w = nullptr;  // [G, Og, K] bf16
    void* dst = nullptr;          // forward: [N, G*Og, P] fp32 or bf16
    const void* dy = nullptr;     // weight gradient: [N, G*Og, P] fp32 or bf16 (dy_f32)
    const uint16_t* addend = nullptr;  // forward with bf16 dst: optional bf16 tensor added to the result
    float* partial = nullptr;     // weight gradient: [wgrad_partials(P), G*Og*K] fp32
    int N = 0, G = 0, R = 0, KH = 1, KW = 1, TV = 1, K = 0, Og = 0, H = 0, W = 0, P = 0;
    int src_f32 = 0, dst_f32 = 1, dy_f32 = 1, acc = 0;  // acc: dst += result (fp32 dst only)
    int upi = 0;                  // forward: 8-pixel units per image, ceil(P / 8)
    int otiles = 0, ktiles = 0;   // tiles of 16*MO output channels / 16*NK contraction rows
    int slices = 0, chunks32 = 0, per_slice = 0;  // weight gradient: pixel chunks of 32 split over slices
    int wtile = 2;                // weight gradient: the wavefront's dW tile is (16*wtile) x (16*wtile)
    uint32_t magicW = 0, magicTV = 0, magicKW = 0, magicC32 = 0, magicUpi = 0;
};

inline uint32_t magic_u32(uint32_t d) { return d <= 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) + d - 1) / d); }

// y[n, g*Og+o, p] (+)= sum_k w[g][o][k] * src_row(n, g, k)[p + off(k)]
void forward(const Params& P, hipStream_t s);
// partial[wg][g][o][k] = sum over the (n, p) of the workgroup's four slices of dy[n, g*Og+o, p] * src_row(n, g, k)[p + off(k)]
void wgrad_partial(const Params& P, hipStream_t s);
// number of partials wgrad_partial writes (one per workgroup of four slices); dw[e] = sum_i partial[i][e] is a
// job of wreduce_kernels.hpp
int wgrad_partials(const Params& P);
// wt[g][row][o*TV + tv] = w[g][o][row*TV + (TV-1-tv)]: the weights of the data-gradient contraction
void transpose_weights(const uint16_t* w, uint16_t* wt, int G, int Og, int R, int TV, hipStream_t s);
int choose_mo(int Og);

// Host-side set-up shared by the lowerings.  `shape` fills the geometry of a contraction whose operand has
// `rows` rows per group seen through a KH x KW window; the three `prepare_*` calls complete it for one launch kind.
Params shape(int N, int G, int rows, int KH, int KW, int Og, int H, int W);
void prepare_forward(Params& P);
// Splits the N * ceil(P/32) pixel chunks over at most 2048 slices per tile (one partial per four slices, at most 8 MB).
void prepare_wgrad(Params& P);
// Forward geometry -> geometry of the data gradient (rows and outputs swapped); use with transposed weights.
Params data_gradient_of(const Params& fwd);

}  // namespace gfc
}  // namespace canvas
