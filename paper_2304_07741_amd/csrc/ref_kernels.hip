// Per-node kernels of the unfused lowering: one launch per primitive, every
// intermediate tensor materialised in fp32 as [N, C, T, H, W].  Each thread owns
// one element of the tensor it writes, so gradients of tensors consumed several
// times are summed by later launches adding to earlier ones (no atomics).
// Primitive definitions: Canvas paper, Section 5.
#include "ref_kernels.hpp"

#include <hip/hip_runtime.h>

#include "device_util.hpp"
#include "launch.hpp"

namespace canvas {
namespace ref {

namespace {

constexpr int kBlock = 256;

inline dim3 grid_for(int64_t total) { return dim3((unsigned)((total + kBlock - 1) / kBlock)); }

__global__ void k_bf16_to_f32(const uint16_t* __restrict__ in, float* __restrict__ out, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n) out[i] = bf16_to_f32(in[i]);
}

__global__ void k_f32_to_bf16(const float* __restrict__ in, uint16_t* __restrict__ out, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n) out[i] = f32_to_bf16(in[i]);
}

__global__ void k_fill_f32(float* __restrict__ out, float v, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n) out[i] = v;
}

__global__ void k_copy_f32(const float* __restrict__ in, float* __restrict__ out, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n) out[i] = in[i];
}

// out[n,c,t,h,w], t = ti*K + kh*KW + kw
__global__ void k_unfold_fwd(const float* __restrict__ in, float* __restrict__ out, int64_t total, int Tin, int KH, int KW,
                             int H, int W) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    int K = KH * KW, T = Tin * K;
    int w = (int)(i % W);
    int64_t r = i / W;
    int h = (int)(r % H);
    r /= H;
    int t = (int)(r % T);
    int64_t nc = r / T;
    int ti = t / K, kk = t % K, kh = kk / KW, kw = kk % KW;
    int hs = h + kh - KH / 2, ws = w + kw - KW / 2;
    float v = 0.f;
    if (hs >= 0 && hs < H && ws >= 0 && ws < W) v = in[((nc * Tin + ti) * H + hs) * W + ws];
    out[i] = v;
}

// gin[n,c,ti,h,w] (+)= sum_{kh,kw} gout[n,c,ti*K+kh*KW+kw, h-(kh-KH/2), w-(kw-KW/2)]
__global__ void k_unfold_bwd(const float* __restrict__ gout, float* __restrict__ gin, int64_t total, int Tin, int KH, int KW,
                             int H, int W, int acc) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    int K = KH * KW, T = Tin * K;
    int w = (int)(i % W);
    int64_t r = i / W;
    int h = (int)(r % H);
    r /= H;
    int ti = (int)(r % Tin);
    int64_t nc = r / Tin;
    float s = 0.f;
    for (int kh = 0; kh < KH; kh++) {
        int ho = h - (kh - KH / 2);
        if (ho < 0 || ho >= H) continue;
        for (int kw = 0; kw < KW; kw++) {
            int wo = w - (kw - KW / 2);
            if (wo < 0 || wo >= W) continue;
            s += gout[((nc * T + ti * K + kh * KW + kw) * H + ho) * W + wo];
        }
    }
    gin[i] = acc ? gin[i] + s : s;
}

// forward: dst(h,w) = src(h+dh, w+dw) on the slice; the adjoint is the same kernel with (-dh,-dw).
__global__ void k_shift(const float* __restrict__ src, float* __restrict__ dst, int64_t total, int C, int T, int H, int W,
                        int dh, int dw, int c0, int c1, int acc) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    int w = (int)(i % W);
    int64_t r = i / W;
    int h = (int)(r % H);
    r /= H;
    int64_t nc = r / T;
    int c = (int)(nc % C);
    float v;
    if (c >= c0 && c < c1) {
        int hs = h + dh, ws = w + dw;
        v = (hs >= 0 && hs < H && ws >= 0 && ws < W) ? src[(r * H + hs) * W + ws] : 0.f;
    } else {
        v = src[i];
    }
    dst[i] = acc ? dst[i] + v : v;
}

// y[n, g*Og+o, p] = sum_i W[(g*Og+o)*K + i] * x[n, g*K + i, p]   (x rows are (c,t) pairs: (g*Cg+c')*T+t = g*K+i)
__global__ void k_fc_fwd(const float* __restrict__ x, const float* __restrict__ wt, float* __restrict__ y, int64_t total,
                         int G, int Og, int K, int P) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    int p = (int)(i % P);
    int64_t r = i / P;
    int go = (int)(r % (G * Og));
    int64_t n = r / (G * Og);
    int g = go / Og;
    const float* xr = x + ((n * G + g) * (int64_t)K) * P + p;
    const float* wr = wt + (int64_t)go * K;
    float s = 0.f;
    for (int k = 0; k < K; k++) s = fmaf(wr[k], xr[(int64_t)k * P], s);
    y[i] = s;
}

// gx[n, g*K+i, p] (+)= sum_o W[(g*Og+o)*K+i] * gy[n, g*Og+o, p]
__global__ void k_fc_dx(const float* __restrict__ gy, const float* __restrict__ wt, float* __restrict__ gx, int64_t total,
                        int G, int Og, int K, int P, int acc) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    int p = (int)(i % P);
    int64_t r = i / P;
    int gi = (int)(r % (G * K));
    int64_t n = r / (G * K);
    int g = gi / K, k = gi % K;
    const float* gr = gy + ((n * G + g) * (int64_t)Og) * P + p;
    const float* wr = wt + ((int64_t)g * Og) * K + k;
    float s = 0.f;
    for (int o = 0; o < Og; o++) s = fmaf(wr[(int64_t)o * K], gr[(int64_t)o * P], s);
    gx[i] = acc ? gx[i] + s : s;
}

// dW[(g*Og+o)*K+i] = sum_{n,p} gy[n,g*Og+o,p] * x[n,g*K+i,p]; one block per weight, fixed-order tree reduction.
__global__ void k_fc_dw(const float* __restrict__ gy, const float* __restrict__ x, float* __restrict__ dw, int N, int G,
                        int Og, int K, int P) {
    __shared__ float red[kBlock];
    int64_t widx = blockIdx.x;
    int k = (int)(widx % K);
    int go = (int)(widx / K);
    int g = go / Og;
    float s = 0.f;
    int64_t M = (int64_t)N * P;
    for (int64_t m = threadIdx.x; m < M; m += kBlock) {
        int64_t n = m / P;
        int p = (int)(m % P);
        s = fmaf(gy[(n * G * Og + go) * P + p], x[((n * G + g) * (int64_t)K + k) * P + p], s);
    }
    red[threadIdx.x] = s;
    __syncthreads();
    for (int st = kBlock / 2; st > 0; st >>= 1) {
        if ((int)threadIdx.x < st) red[threadIdx.x] += red[threadIdx.x + st];
        __syncthreads();
    }
    if (threadIdx.x == 0) dw[widx] = red[0];
}

__global__ void k_unary_fwd(const float* __restrict__ in, float* __restrict__ out, int64_t n, int kind, float lo, float hi) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n) out[i] = unary_apply(kind, in[i], lo, hi);
}

__global__ void k_unary_bwd(const float* __restrict__ in, const float* __restrict__ gout, float* __restrict__ gin, int64_t n,
                            int kind, float lo, float hi, int acc) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    float g = gout[i] * unary_grad(kind, in[i], lo, hi);
    gin[i] = acc ? gin[i] + g : g;
}

__device__ inline void bsrc(int CL, int TL, int TR, int c, int t, int same_c, int& cl, int& tl) {
    if (same_c) {
        cl = c;
        tl = t % TL;
    } else {
        long long j = ((long long)c * TR + t) % ((long long)CL * TL);
        cl = (int)(j / TL);
        tl = (int)(j % TL);
    }
}

// PL: pixels of the LHS.  rep says how pixel p of the result finds its LHS pixel: 0: p itself (PL == P) or the
// one pixel of a fully pooled LHS (PL == 1); 1: p % Wd (the LHS has folded H away, PL == Wd); 2: p / Wd (the
// LHS has folded W away, PL == P / Wd).  Wd: width of the result.
__device__ __forceinline__ int lhs_pixel(int p, int PL, int rep, int Wd) {
    return rep == 1 ? p % Wd : (rep == 2 ? p / Wd : (PL == 1 ? 0 : p));
}

__global__ void k_binary_fwd(const float* __restrict__ lhs, const float* __restrict__ rhs, float* __restrict__ out,
                             int64_t total, int CL, int TL, int CR, int TR, int P, int PL, int rep, int Wd, int kind) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    int p = (int)(i % P);
    int64_t r = i / P;
    int t = (int)(r % TR);
    r /= TR;
    int c = (int)(r % CR);
    int64_t n = r / CR;
    int cl, tl;
    bsrc(CL, TL, TR, c, t, CL == CR, cl, tl);
    float a = lhs[((n * CL + cl) * TL + tl) * PL + lhs_pixel(p, PL, rep, Wd)], b = rhs[i];
    out[i] = binary_apply(kind, a, b);
}

__global__ void k_binary_bwd_rhs(const float* __restrict__ lhs, const float* __restrict__ rhs, const float* __restrict__ gout,
                                 float* __restrict__ grhs, int64_t total, int CL, int TL, int CR, int TR, int P, int PL, int rep, int Wd,
                                 int kind, int acc) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    float g = gout[i];
    if (kind != 0) {
        int p = (int)(i % P);
        int64_t r = i / P;
        int t = (int)(r % TR);
        r /= TR;
        int c = (int)(r % CR);
        int64_t n = r / CR;
        int cl, tl;
        bsrc(CL, TL, TR, c, t, CL == CR, cl, tl);
        g *= binary_grad_rhs(kind, lhs[((n * CL + cl) * TL + tl) * PL + lhs_pixel(p, PL, rep, Wd)], rhs[i]);
    }
    grhs[i] = acc ? grhs[i] + g : g;
}

// One thread per LHS element sums over the RHS elements it was replicated onto (channels / taps, and the
// pixels along the spatial dims the LHS has folded away), in a fixed order.
__global__ void k_binary_bwd_lhs(const float* __restrict__ lhs, const float* __restrict__ rhs, const float* __restrict__ gout,
                                 float* __restrict__ glhs, int64_t total, int CL, int TL, int CR, int TR, int P, int PL, int rep, int Wd,
                                 int kind, int acc) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    int pl = (int)(i % PL);
    int64_t r = i / PL;
    int tl = (int)(r % TL);
    r /= TL;
    int cl = (int)(r % CL);
    int64_t n = r / CL;
    const float a = lhs[i];
    // the pixels of the result that read this LHS pixel: pcount of them from p0 in steps of pstep
    const int p0 = rep == 2 ? pl * Wd : (PL == 1 ? 0 : pl);
    const int pcount = rep == 1 ? P / Wd : (rep == 2 ? Wd : (PL == 1 ? P : 1)), pstep = rep == 1 ? Wd : 1;
    float s = 0.f;
    if (CL == CR) {
        for (int t = tl; t < TR; t += TL)
            for (int pi = 0, p = p0; pi < pcount; pi++, p += pstep) {
                int64_t j = ((n * CR + cl) * TR + t) * P + p;
                s += kind == 0 ? gout[j] : gout[j] * binary_grad_lhs(kind, a, rhs[j]);
            }
    } else {
        long long L = (long long)CL * TL, R = (long long)CR * TR;
        for (long long f = (long long)cl * TL + tl; f < R; f += L)
            for (int pi = 0, p = p0; pi < pcount; pi++, p += pstep) {
                int64_t j = (n * R + f) * P + p;
                s += kind == 0 ? gout[j] : gout[j] * binary_grad_lhs(kind, a, rhs[j]);
            }
    }
    glhs[i] = acc ? glhs[i] + s : s;
}

constexpr int kSoftmaxRegs = 32;

// One thread per (n, outer, p); the axis is strided by `stride`, `len` long.
__global__ void k_softmax_fwd(const float* __restrict__ in, float* __restrict__ out, int64_t total, int C, int T, int P,
                              int axis_c) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    int p = (int)(i % P);
    int64_t r = i / P;
    int len, outer;
    int64_t stride, base;
    if (axis_c == 2) {  // channels and taps jointly: the [C, T] block of a pixel, stride P
        len = C * T; outer = 1;
        base = r * len * P + p;
        stride = P;
    } else if (axis_c) {
        len = C; outer = T;
        int t = (int)(r % outer);
        int64_t n = r / outer;
        base = (n * C * T + t) * P + p;
        stride = (int64_t)T * P;
    } else {
        len = T; outer = C;
        int c = (int)(r % outer);
        int64_t n = r / outer;
        base = ((n * C + c) * T) * P + p;
        stride = P;
    }
    if (len <= kSoftmaxRegs) {  // short axis (the taps of a window): one read of the axis, kept in registers
        float v[kSoftmaxRegs];
#pragma unroll
        for (int k = 0; k < kSoftmaxRegs; k++) v[k] = k < len ? in[base + k * stride] : -INFINITY;
        float m = -INFINITY;
#pragma unroll
        for (int k = 0; k < kSoftmaxRegs; k++) m = fmaxf(m, v[k]);
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < kSoftmaxRegs; k++) {
            v[k] = expf(v[k] - m);
            s += k < len ? v[k] : 0.f;
        }
        const float inv = 1.f / s;
#pragma unroll
        for (int k = 0; k < kSoftmaxRegs; k++)
            if (k < len) out[base + k * stride] = v[k] * inv;
        return;
    }
    float m = -INFINITY;
    for (int k = 0; k < len; k++) m = fmaxf(m, in[base + k * stride]);
    float s = 0.f;
    for (int k = 0; k < len; k++) s += expf(in[base + k * stride] - m);
    float inv = 1.f / s;
    for (int k = 0; k < len; k++) out[base + k * stride] = expf(in[base + k * stride] - m) * inv;
}

// Softmax along a spatial dim (Section 5, table of primitives: Softmax at any continuous dims): one wavefront per row,
// lane l takes elements l, l + 64, ...; maximum and sums cross the lanes in a fixed butterfly, so the result does not
// depend on the launch.
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v = fmaxf(v, __shfl_xor(v, d));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
    return v;
}
__global__ __launch_bounds__(256) void k_softmax_rows_fwd(const float* __restrict__ in, float* __restrict__ out, int64_t rows, int len, int inner) {
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= rows) return;  // (whole wavefronts leave: the shuffles below see all 64 lanes)
    const int lane = threadIdx.x & 63;
    const int64_t base = (r / inner) * (int64_t)len * inner + (r % inner);
    float m = -INFINITY;
    for (int k = lane; k < len; k += 64) m = fmaxf(m, in[base + (int64_t)k * inner]);
    m = wave_max(m);
    float z = 0.f;
    for (int k = lane; k < len; k += 64) z += expf(in[base + (int64_t)k * inner] - m);
    z = wave_sum(z);
    const float inv = 1.f / z;
    for (int k = lane; k < len; k += 64) out[base + (int64_t)k * inner] = expf(in[base + (int64_t)k * inner] - m) * inv;
}
__global__ __launch_bounds__(256) void k_softmax_rows_bwd(const float* __restrict__ y, const float* __restrict__ gout, float* __restrict__ gin,
                                                          int64_t rows, int len, int inner, int acc) {
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= rows) return;
    const int lane = threadIdx.x & 63;
    const int64_t base = (r / inner) * (int64_t)len * inner + (r % inner);
    float dot = 0.f;
    for (int k = lane; k < len; k += 64) dot += gout[base + (int64_t)k * inner] * y[base + (int64_t)k * inner];
    dot = wave_sum(dot);
    for (int k = lane; k < len; k += 64) {
        const int64_t i = base + (int64_t)k * inner;
        const float g = y[i] * (gout[i] - dot);
        gin[i] = acc ? gin[i] + g : g;
    }
}

// gin16 (optional): the result once more, rounded to bf16 (for a consumer that takes bf16 operands)
__global__ void k_softmax_bwd(const float* __restrict__ y, const float* __restrict__ gout, float* __restrict__ gin,
                              uint16_t* __restrict__ gin16, int64_t total, int C, int T, int P, int axis_c, int acc) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    int p = (int)(i % P);
    int64_t r = i / P;
    int len;
    int64_t stride, base;
    if (axis_c == 2) {
        len = C * T;
        base = r * len * P + p;
        stride = P;
    } else if (axis_c) {
        len = C;
        int t = (int)(r % T);
        int64_t n = r / T;
        base = (n * C * T + t) * P + p;
        stride = (int64_t)T * P;
    } else {
        len = T;
        int c = (int)(r % C);
        int64_t n = r / C;
        base = ((n * C + c) * T) * P + p;
        stride = P;
    }
    if (len <= kSoftmaxRegs) {
        float yv[kSoftmaxRegs], gv[kSoftmaxRegs];
#pragma unroll
        for (int k = 0; k < kSoftmaxRegs; k++) {
            yv[k] = k < len ? y[base + k * stride] : 0.f;
            gv[k] = k < len ? gout[base + k * stride] : 0.f;
        }
        float dot = 0.f;
#pragma unroll
        for (int k = 0; k < kSoftmaxRegs; k++) dot = fmaf(gv[k], yv[k], dot);
#pragma unroll
        for (int k = 0; k < kSoftmaxRegs; k++)
            if (k < len) {
                float g = yv[k] * (gv[k] - dot);
                if (acc) g += gin[base + k * stride];
                gin[base + k * stride] = g;
                if (gin16) gin16[base + k * stride] = f32_to_bf16(g);
            }
        return;
    }
    float dot = 0.f;
    for (int k = 0; k < len; k++) dot = fmaf(gout[base + k * stride], y[base + k * stride], dot);
    for (int k = 0; k < len; k++) {
        float g = y[base + k * stride] * (gout[base + k * stride] - dot);
        if (acc) g += gin[base + k * stride];
        gin[base + k * stride] = g;
        if (gin16) gin16[base + k * stride] = f32_to_bf16(g);
    }
}

__global__ void k_fold_fwd(const float* __restrict__ in, float* __restrict__ out, int64_t total, int T, int P, int kind) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    int p = (int)(i % P);
    int64_t nc = i / P;
    const float* src = in + nc * T * P + p;
    float a = src[0];
    for (int t = 1; t < T; t++) {
        float v = src[(int64_t)t * P];
        if (kind == 2) a = v > a ? v : a;
        else a += v;
    }
    if (kind == 1) a /= (float)T;
    out[i] = a;
}

__global__ void k_fold_bwd(const float* __restrict__ in, const float* __restrict__ gout, float* __restrict__ gin,
                           int64_t total, int T, int P, int kind, int acc) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    int p = (int)(i % P);
    int64_t nc = i / P;
    const float* src = in + nc * T * P + p;
    float* dst = gin + nc * T * P + p;
    float g = gout[i];
    int best = 0;
    if (kind == 2) {
        float a = src[0];
        for (int t = 1; t < T; t++) {
            float v = src[(int64_t)t * P];
            if (v > a) { a = v; best = t; }
        }
    } else if (kind == 1) {
        g /= (float)T;
    }
    for (int t = 0; t < T; t++) {
        float v = kind == 2 ? (t == best ? g : 0.f) : g;
        dst[(int64_t)t * P] = acc ? dst[(int64_t)t * P] + v : v;
    }
}

}  // namespace

#define LAUNCH(kern, total, ...)                                                                  \
    do {                                                                                          \
        if ((total) > 0) CANVAS_LAUNCH(kern, grid_for(total), dim3(kBlock), 0, s, __VA_ARGS__); \
    } while (0)

void widen_bf16(const void* in, float* out, int64_t n, hipStream_t s) { LAUNCH(k_bf16_to_f32, n, (const uint16_t*)in, out, n); }
void narrow_bf16(const float* in, void* out, int64_t n, hipStream_t s) { LAUNCH(k_f32_to_bf16, n, in, (uint16_t*)out, n); }
void fill_f32(float* out, float v, int64_t n, hipStream_t s) { LAUNCH(k_fill_f32, n, out, v, n); }
void copy_f32(const float* in, float* out, int64_t n, hipStream_t s) { LAUNCH(k_copy_f32, n, in, out, n); }

// Fold over the Cg channels of each channel group: one thread per output element (n, g, t, p); the channels
// of a group are Cg planes `stride` = T*P elements apart.
__global__ void k_cfold_fwd(const float* __restrict__ in, float* __restrict__ out, int64_t total, int Cg, int64_t stride, int kind) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    const int64_t ng = i / stride, rest = i - ng * stride;  // (n, g) and (t, p)
    const float* src = in + ng * Cg * stride + rest;
    float a = src[0];
    for (int c = 1; c < Cg; c++) {
        float v = src[(int64_t)c * stride];
        if (kind == 2) a = v > a ? v : a;
        else a += v;
    }
    if (kind == 1) a /= (float)Cg;
    out[i] = a;
}

__global__ void k_cfold_bwd(const float* __restrict__ in, const float* __restrict__ gout, float* __restrict__ gin, int64_t total, int Cg,
                            int64_t stride, int kind, int acc) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    const int64_t ng = i / stride, rest = i - ng * stride;
    const float* src = in + ng * Cg * stride + rest;
    float* dst = gin + ng * Cg * stride + rest;
    float g = gout[i];
    int best = 0;
    if (kind == 2) {
        float a = src[0];
        for (int c = 1; c < Cg; c++) {
            float v = src[(int64_t)c * stride];
            if (v > a) { a = v; best = c; }
        }
    } else if (kind == 1) {
        g /= (float)Cg;
    }
    for (int c = 0; c < Cg; c++) {
        float v = kind == 2 ? (c == best ? g : 0.f) : g;
        dst[(int64_t)c * stride] = acc ? dst[(int64_t)c * stride] + v : v;
    }
}

// Fold over the pixels: one workgroup per (n, c, t) plane.  Each thread folds a strided subset in pixel
// order, then a tree over the 256 threads with a fixed pairing; max keeps the lowest pixel index among equals.
__global__ __launch_bounds__(256) void k_pool_fwd(const float* __restrict__ in, float* __restrict__ out, int P, int kind) {
    __shared__ float red[256];
    const float* src = in + (int64_t)blockIdx.x * P;
    const int tid = threadIdx.x;
    float a = kind == 2 ? -INFINITY : 0.f;
    for (int p = tid; p < P; p += 256) {
        const float v = src[p];
        if (kind == 2) a = v > a ? v : a;
        else a += v;
    }
    red[tid] = a;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (tid < w) red[tid] = kind == 2 ? fmaxf(red[tid], red[tid + w]) : red[tid] + red[tid + w];
        __syncthreads();
    }
    if (tid == 0) out[blockIdx.x] = kind == 1 ? red[0] / (float)P : red[0];
}

__global__ __launch_bounds__(256) void k_pool_bwd(const float* __restrict__ in, const float* __restrict__ gout, float* __restrict__ gin, int P,
                                                  int kind, int acc) {
    __shared__ float rv[256];
    __shared__ int ri[256];
    const float* src = in + (int64_t)blockIdx.x * P;
    float* dst = gin + (int64_t)blockIdx.x * P;
    const int tid = threadIdx.x;
    float g = gout[blockIdx.x];
    int best = -1;
    if (kind == 2) {  // first maximal pixel of the plane
        float a = -INFINITY;
        int ai = 0x7fffffff;
        for (int p = tid; p < P; p += 256) {
            const float v = src[p];
            if (v > a) { a = v; ai = p; }
        }
        rv[tid] = a;
        ri[tid] = ai;
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) {
            if (tid < w) {
                const float b = rv[tid + w];
                const int bi = ri[tid + w];
                if (b > rv[tid] || (b == rv[tid] && bi < ri[tid])) { rv[tid] = b; ri[tid] = bi; }
            }
            __syncthreads();
        }
        best = ri[0];
    } else if (kind == 1) {
        g /= (float)P;
    }
    for (int p = tid; p < P; p += 256) {
        const float v = kind == 2 ? (p == best ? g : 0.f) : g;
        dst[p] = acc ? dst[p] + v : v;
    }
}

void unfold_fwd(const float* in, float* out, int64_t NC, int Tin, int KH, int KW, int H, int W, hipStream_t s) {
    int64_t total = NC * Tin * KH * KW * H * W;
    LAUNCH(k_unfold_fwd, total, in, out, total, Tin, KH, KW, H, W);
}
void unfold_bwd(const float* gout, float* gin, int64_t NC, int Tin, int KH, int KW, int H, int W, int acc, hipStream_t s) {
    int64_t total = NC * Tin * H * W;
    LAUNCH(k_unfold_bwd, total, gout, gin, total, Tin, KH, KW, H, W, acc);
}
void shift(const float* src, float* dst, int64_t N, int C, int T, int H, int W, int dh, int dw, int c0, int c1, int acc,
           hipStream_t s) {
    int64_t total = N * C * T * H * W;
    LAUNCH(k_shift, total, src, dst, total, C, T, H, W, dh, dw, c0, c1, acc);
}
void fc_fwd(const float* x, const float* wt, float* y, int64_t N, int G, int Og, int K, int P, hipStream_t s) {
    int64_t total = N * G * Og * P;
    LAUNCH(k_fc_fwd, total, x, wt, y, total, G, Og, K, P);
}
void fc_dx(const float* gy, const float* wt, float* gx, int64_t N, int G, int Og, int K, int P, int acc, hipStream_t s) {
    int64_t total = N * G * K * P;
    LAUNCH(k_fc_dx, total, gy, wt, gx, total, G, Og, K, P, acc);
}
void fc_dw(const float* gy, const float* x, float* dw, int64_t N, int G, int Og, int K, int P, hipStream_t s) {
    int64_t nw = (int64_t)G * Og * K;
    if (nw > 0) CANVAS_LAUNCH(k_fc_dw, dim3((unsigned)nw), dim3(kBlock), 0, s, gy, x, dw, (int)N, G, Og, K, P);
}
void unary_fwd(const float* in, float* out, int64_t n, int kind, float lo, float hi, hipStream_t s) {
    LAUNCH(k_unary_fwd, n, in, out, n, kind, lo, hi);
}
void unary_bwd(const float* in, const float* gout, float* gin, int64_t n, int kind, float lo, float hi, int acc, hipStream_t s) {
    LAUNCH(k_unary_bwd, n, in, gout, gin, n, kind, lo, hi, acc);
}
void binary_fwd(const float* lhs, const float* rhs, float* out, int64_t N, int CL, int TL, int CR, int TR, int P, int PL, int rep, int Wd,
                int kind, hipStream_t s) {
    int64_t total = N * CR * TR * P;
    LAUNCH(k_binary_fwd, total, lhs, rhs, out, total, CL, TL, CR, TR, P, PL, rep, Wd, kind);
}
void binary_bwd_rhs(const float* lhs, const float* rhs, const float* gout, float* grhs, int64_t N, int CL, int TL, int CR, int TR, int P,
                    int PL, int rep, int Wd, int kind, int acc, hipStream_t s) {
    int64_t total = N * CR * TR * P;
    LAUNCH(k_binary_bwd_rhs, total, lhs, rhs, gout, grhs, total, CL, TL, CR, TR, P, PL, rep, Wd, kind, acc);
}
void binary_bwd_lhs(const float* lhs, const float* rhs, const float* gout, float* glhs, int64_t N, int CL, int TL, int CR, int TR, int P,
                    int PL, int rep, int Wd, int kind, int acc, hipStream_t s) {
    int64_t total = N * CL * TL * PL;
    LAUNCH(k_binary_bwd_lhs, total, lhs, rhs, gout, glhs, total, CL, TL, CR, TR, P, PL, rep, Wd, kind, acc);
}
void cfold_fwd(const float* in, float* out, int64_t NG, int Cg, int64_t TP, int kind, hipStream_t s) {
    int64_t total = NG * TP;
    LAUNCH(k_cfold_fwd, total, in, out, total, Cg, TP, kind);
}
void cfold_bwd(const float* in, const float* gout, float* gin, int64_t NG, int Cg, int64_t TP, int kind, int acc, hipStream_t s) {
    int64_t total = NG * TP;
    LAUNCH(k_cfold_bwd, total, in, gout, gin, total, Cg, TP, kind, acc);
}
void pool_fwd(const float* in, float* out, int64_t rows, int P, int kind, hipStream_t s) {
    if (rows > 0) CANVAS_LAUNCH(k_pool_fwd, dim3((unsigned)rows), dim3(256), 0, s, in, out, P, kind);
}
void pool_bwd(const float* in, const float* gout, float* gin, int64_t rows, int P, int kind, int acc, hipStream_t s) {
    if (rows > 0) CANVAS_LAUNCH(k_pool_bwd, dim3((unsigned)rows), dim3(256), 0, s, in, gout, gin, P, kind, acc);
}
void softmax_rows_fwd(const float* in, float* out, int64_t rows, int len, int inner, hipStream_t s) {
    if (rows > 0) CANVAS_LAUNCH(k_softmax_rows_fwd, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, in, out, rows, len, inner);
}
void softmax_rows_bwd(const float* y, const float* gout, float* gin, int64_t rows, int len, int inner, int acc, hipStream_t s) {
    if (rows > 0) CANVAS_LAUNCH(k_softmax_rows_bwd, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, y, gout, gin, rows, len, inner, acc);
}
void softmax_fwd(const float* in, float* out, int64_t N, int C, int T, int P, int axis_c, hipStream_t s) {
    int64_t total = N * (axis_c == 2 ? 1 : (axis_c ? T : C)) * P;
    LAUNCH(k_softmax_fwd, total, in, out, total, C, T, P, axis_c);
}
void softmax_bwd(const float* y, const float* gout, float* gin, int64_t N, int C, int T, int P, int axis_c, int acc,
                 hipStream_t s, uint16_t* gin16) {
    int64_t total = N * (axis_c == 2 ? 1 : (axis_c ? T : C)) * P;
    LAUNCH(k_softmax_bwd, total, y, gout, gin, gin16, total, C, T, P, axis_c, acc);
}
void fold_fwd(const float* in, float* out, int64_t NC, int T, int P, int kind, hipStream_t s) {
    int64_t total = NC * P;
    LAUNCH(k_fold_fwd, total, in, out, total, T, P, kind);
}
void fold_bwd(const float* in, const float* gout, float* gin, int64_t NC, int T, int P, int kind, int acc, hipStream_t s) {
    int64_t total = NC * P;
    LAUNCH(k_fold_bwd, total, in, gout, gin, total, T, P, kind, acc);
}

}  // namespace ref
}  // namespace canvas
