// Tap-major grouped FC on bf16 MFMA for bf16 operands and the common windows (1x1, 3x3, 5x5): the fast
// path of the contraction in gfc_kernels.hpp (same mathematics: Canvas paper, Section 5, Fully-connected,
// Group, Unfold).  The weights are first repacked so that
//   * the contraction index runs tap-major: k' = tap * Rp + row, hence one MFMA step of 16 rows has ONE
//     window tap, and the three (five) horizontal taps of a window row are served from one set of loaded
//     registers (the horizontal shift is a different static selector of the operand gather);
//   * groups with fewer than 16 rows are merged, gm = 16 / R groups per tile, into a block-diagonal weight
//     (zeros between groups), rows and outputs padded with zeros to multiples of 16.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace canvas {
namespace gfctm {

struct Params {
    const uint16_t* src = nullptr;     // row tensor [N, G, R, P] bf16
    const uint16_t* wp = nullptr;      // packed weights [Gm][Omp][TV][Rp] bf16
    void* dst = nullptr;               // forward: [N, G*Og, P] bf16 or fp32
    const uint16_t* addend = nullptr;  // forward, bf16 dst: optional tensor added before rounding
    const uint16_t* dy = nullptr;      // weight gradient: [N, G*Og, P] bf16
    float* partial = nullptr;          // weight gradient: [slices][Gm][Omp][TV][Rp] fp32
    int N = 0, H = 0, W = 0, P = 0, upi = 0;
    int G = 0, R = 0, Og = 0;          // the FC's own grouping: R rows and Og outputs per group
    int gm = 1, Gm = 0;                // groups merged per tile, merged group count ceil(G / gm)
    int Rp = 0, Omp = 0;               // rows / outputs per merged group, padded
    int KH = 1, KW = 1, TV = 1;
    int mo = 1, otiles = 1;            // 16*mo outputs per wavefront, Omp = 16*mo*otiles
    int ksplit = 1;                    // forward: wavefronts that share one tile and split its row chunks (1, 2, 4)
    int dst_f32 = 0, acc = 0;
    int softmax = 0;                   // forward: the result is the softmax over the outputs of each pixel (see softmax_fusable)
    int nsplit = 1, chunks = 0, imgs_per_split = 0;  // weight gradient: work items = chunks (32-pixel positions) x nsplit (image ranges)
    int rows = 0;                      // weight gradient by image rows: chunks = 32-column chunks of a row, ranges of (image, row) steps
    uint32_t magicW = 0, magicUpi = 0, magicW16 = 0, magicH = 0;  // exact division by W, upi, the 16-byte pieces of a weight row, H
};

// Whether the fast path covers a contraction of this geometry (bf16 operands are the caller's business).
bool supported(int N, int G, int R, int KH, int KW, int Og, int H, int W);
Params shape(int N, int G, int R, int KH, int KW, int Og, int H, int W);
// Geometry of the data gradient: rows and outputs swapped (pack the weights with transposed = true).
Params data_gradient_of(const Params& fwd);
inline int64_t packed_elems(const Params& P) { return (int64_t)P.Gm * P.Omp * P.TV * P.Rp; }

// y = FC(src) on the packed weights P.wp (packed by a job of wprep_kernels.hpp; `transposed` there gives the data
// gradient).  The weight tile of a workgroup goes through LDS where it fits (<= 72 KB).
void forward(const Params& P, hipStream_t s);
// Whether forward can apply a softmax over the outputs of each pixel to its result (P.softmax = 1, fp32 destination):
// one group, at most 16 outputs, no window.
bool softmax_fusable(const Params& P);

// Weight gradient of a windowed contraction (KH = KW = 3 or 5): by image rows for 3 x 3 windows on rows of 24 pixels
// and more, else by 32-pixel positions.  prepare_wgrad chooses and splits the work; the partials
// buffer holds wgrad_slices(P) * packed_elems(P) floats, one partial in the packed layout per workgroup; their
// fixed-order sum into dw [G][Og][R][TV] (fp32) is a job of wreduce_kernels.hpp.
void prepare_wgrad(Params& P);
int wgrad_slices(const Params& P);
void wgrad_partial(const Params& P, hipStream_t s);

}  // namespace gfctm
}  // namespace canvas
