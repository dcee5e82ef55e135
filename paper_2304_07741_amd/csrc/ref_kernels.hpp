// Launchers of the per-node fp32 kernels (unfused lowering).  All pointers are device pointers;
// `acc` != 0 adds to the destination instead of overwriting it.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace canvas {
namespace ref {

void widen_bf16(const void* in, float* out, int64_t n, hipStream_t s);
void narrow_bf16(const float* in, void* out, int64_t n, hipStream_t s);
void fill_f32(float* out, float v, int64_t n, hipStream_t s);
void copy_f32(const float* in, float* out, int64_t n, hipStream_t s);
void unfold_fwd(const float* in, float* out, int64_t NC, int Tin, int KH, int KW, int H, int W, hipStream_t s);
void unfold_bwd(const float* gout, float* gin, int64_t NC, int Tin, int KH, int KW, int H, int W, int acc, hipStream_t s);
void shift(const float* src, float* dst, int64_t N, int C, int T, int H, int W, int dh, int dw, int c0, int c1, int acc,
           hipStream_t s);
void fc_fwd(const float* x, const float* wt, float* y, int64_t N, int G, int Og, int K, int P, hipStream_t s);
void fc_dx(const float* gy, const float* wt, float* gx, int64_t N, int G, int Og, int K, int P, int acc, hipStream_t s);
void fc_dw(const float* gy, const float* x, float* dw, int64_t N, int G, int Og, int K, int P, hipStream_t s);
void unary_fwd(const float* in, float* out, int64_t n, int kind, float lo, float hi, hipStream_t s);
void unary_bwd(const float* in, const float* gout, float* gin, int64_t n, int kind, float lo, float hi, int acc, hipStream_t s);
// P: pixels of the RHS / result, Wd its width; PL: pixels of the LHS; rep: 0 = the LHS has the pixels of the result
// (PL == P) or a single one replicated over all (PL == 1), 1 = the LHS has folded H away (its pixel is p % Wd),
// 2 = it has folded W away (p / Wd)
void binary_fwd(const float* lhs, const float* rhs, float* out, int64_t N, int CL, int TL, int CR, int TR, int P, int PL, int rep, int Wd,
                int kind, hipStream_t s);
void binary_bwd_rhs(const float* lhs, const float* rhs, const float* gout, float* grhs, int64_t N, int CL, int TL, int CR, int TR, int P,
                    int PL, int rep, int Wd, int kind, int acc, hipStream_t s);
void binary_bwd_lhs(const float* lhs, const float* rhs, const float* gout, float* glhs, int64_t N, int CL, int TL, int CR, int TR, int P,
                    int PL, int rep, int Wd, int kind, int acc, hipStream_t s);
// axis_c: 1 = over channels, 0 = over taps, 2 = over both jointly
// Softmax along a spatial dim of every plane: `rows` rows of `len` elements, element k of row r at
// (r / inner) * len * inner + (r % inner) + k * inner (inner = 1: contiguous rows, i.e. along W or over a whole plane;
// inner = W: along H).  One wavefront per row, sums in a fixed butterfly order.
void softmax_rows_fwd(const float* in, float* out, int64_t rows, int len, int inner, hipStream_t s);
void softmax_rows_bwd(const float* y, const float* gout, float* gin, int64_t rows, int len, int inner, int acc, hipStream_t s);
void softmax_fwd(const float* in, float* out, int64_t N, int C, int T, int P, int axis_c, hipStream_t s);
// gin16 (optional): the same result once more, rounded to bf16
void softmax_bwd(const float* y, const float* gout, float* gin, int64_t N, int C, int T, int P, int axis_c, int acc,
                 hipStream_t s, uint16_t* gin16 = nullptr);
void fold_fwd(const float* in, float* out, int64_t NC, int T, int P, int kind, hipStream_t s);
void fold_bwd(const float* in, const float* gout, float* gin, int64_t NC, int T, int P, int kind, int acc, hipStream_t s);
// Fold over the Cg channels of each of NG (image, group) pairs; a channel is TP = taps * pixels elements
void cfold_fwd(const float* in, float* out, int64_t NG, int Cg, int64_t TP, int kind, hipStream_t s);
void cfold_bwd(const float* in, const float* gout, float* gin, int64_t NG, int Cg, int64_t TP, int kind, int acc, hipStream_t s);
// Fold over the P pixels of each of `rows` planes (kind as fold: sum, avg, max with the first maximum taking the gradient)
void pool_fwd(const float* in, float* out, int64_t rows, int P, int kind, hipStream_t s);
void pool_bwd(const float* in, const float* gout, float* gin, int64_t rows, int P, int kind, int acc, hipStream_t s);

}  // namespace ref
}  // namespace canvas
