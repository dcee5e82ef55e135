// Fused kernels for the pattern
//     x -> Shift (one offset per FC group) -> grouped FC -> unary -> (+ x) -> y
// on bf16 NCHW tensors: shift-convolution plus residual, the shape of the best kernel the paper
// reports for ResNet-34 (Section 8, kernel-level analysis) built from the Shift, Group,
// Fully-connected, element-wise and Broadcast primitives of Section 5.
//
// The pattern is bound by HBM traffic (8 flop per byte), so the kernels touch x, y (forward) and
// x, dy, dx (backward) once in HBM and keep everything else in registers (plus, in backward, one
// wave-private LDS tile used as a transposer):
//  * one wavefront owns a tile of 16*KC input channels x 128 pixels of one image and one FC group;
//  * every lane loads 16 bytes (8 consecutive pixels of one channel), so a load instruction covers
//    four channel rows x 256 contiguous bytes;
//  * the FC is a 16x16x16 bf16 MFMA with pixels as the N (or M) dimension.  A lane needs four
//    channels of ONE pixel per MFMA operand but holds eight pixels of four channels; eight MFMAs,
//    one per pixel offset q, take their operands from the q-th halves of the loaded registers
//    (two byte-permutes each), so no cross-lane transpose is needed;
//  * the spatial shift is an address offset of the load plus a zero mask at image borders.  All
//    tensor accesses are buffer loads/stores with the tensor size as the hardware bound, so a shifted
//    16-byte access that leaves the tensor at its two ends returns zeros instead of faulting;
//  * backward recomputes the FC output instead of saving it.  dX = W^T dz contracts over channels like
//    the forward FC; dW = dz x^T contracts over pixels, so x and dz go once through LDS to reach the
//    register distribution that contraction needs (a second pass over global memory for it, even one
//    served by L2, costs a full memory round trip per tile and was measurably slower);
//  * each wavefront writes one dW partial; a second small kernel sums them in a fixed order: no atomics;
//  * throughput is set by the bytes a SIMD keeps in flight to HBM (latency under load is several
//    microseconds), so every load of a tile is issued before any arithmetic and registers are kept
//    below 128 (4 wavefronts per SIMD).
#include "sgfc_kernels.hpp"

#include <hip/hip_runtime.h>

#include "device_util.hpp"
#include "launch.hpp"
#include "tile_util.hpp"

namespace canvas {
namespace sgfc {

namespace {

using namespace canvas::tile;

constexpr int kTilePx = 128;  // pixels per wavefront tile
constexpr int kWaves = 4;     // wavefronts per workgroup
constexpr int kActNone = -1;  // ACT template value: no unary node; otherwise a UnaryKind

// True (wave-uniform) when a tile's shifted accesses, planes starting at elements [first, last] x [p0+off, p0+off+136), leave the tensor.
__device__ __forceinline__ bool tile_near_ends(int first, int last, int p0, int off, int total_elems) {
    return first + p0 + off < 0 || last + p0 + off + kTilePx + 8 > total_elems;
}
// Elements a tensor of N images spans: `stride` apart, `planes` planes of Pn each (the last image ends with its own planes).
__device__ __forceinline__ int extent(int N, int stride, int planes, int Pn) { return (N - 1) * stride + planes * Pn; }

// Validity of the 128 pixels of a tile under a shift: bit i is 1 when tile pixel i exists (p < P) and
// its source pixel (h+dh, w+dw) lies inside the image.  magic = ceil(2^32 / W) gives h = p / W exactly.
struct TileMask {
    uint64_t lo, hi;  // pixels 0..63, 64..127
};
__device__ __forceinline__ TileMask tile_mask(int p0, int lane, const Params& P, int dh, int dw) {
    TileMask m;
    int pa = p0 + lane, pb = p0 + 64 + lane;
    int ha = (int)__umulhi((uint32_t)pa, P.magicW), wa = pa - ha * P.W;
    int hb = (int)__umulhi((uint32_t)pb, P.magicW), wb = pb - hb * P.W;
    bool va = pa < P.P && (unsigned)(ha + dh) < (unsigned)P.H && (unsigned)(wa + dw) < (unsigned)P.W;
    bool vb = pb < P.P && (unsigned)(hb + dh) < (unsigned)P.H && (unsigned)(wb + dw) < (unsigned)P.W;
    m.lo = __ballot(va);
    m.hi = __ballot(vb);
    return m;
}
// The 8 validity bits of unit u (pixels 8u..8u+7 of the tile): byte u of the 128-bit mask, picked with
// byte permutes (a dynamically indexed array would be spilled to LDS).
__device__ __forceinline__ uint32_t unit_bits(const TileMask& m, int u) {
    const uint32_t sel = 0x0c0c0c00u | (uint32_t)(u & 7);
    const uint32_t a = __builtin_amdgcn_perm((uint32_t)(m.lo >> 32), (uint32_t)m.lo, sel);
    const uint32_t b = __builtin_amdgcn_perm((uint32_t)(m.hi >> 32), (uint32_t)m.hi, sel);
    return (u & 8) ? b : a;
}


template <int ACT>
__device__ __forceinline__ float act_apply(const Params& P, float z) {
    if (ACT == kActNone) return z;
    return unary_apply(ACT, z, P.ulo, P.uhi);
}
// dz = dy * act'(z)
template <int ACT>
__device__ __forceinline__ float act_dz(const Params& P, float z, float dy) {
    if (ACT == kActNone) return dy;
    if (ACT == 0) return z > 0.f ? dy : 0.f;
    return dy * unary_grad(ACT, z, P.ulo, P.uhi);
}

// ------------------------------------------------------------------------------------------ forward
template <int KC, int MO, int ACT, bool RES>
__global__ __launch_bounds__(64 * kWaves) void k_fwd(Params P) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int chunk = blockIdx.x * kWaves + wave;
    if (chunk >= P.chunks) return;
    const int g = blockIdx.y, n = blockIdx.z;
    const int r = lane >> 4, s = lane & 15;
    constexpr int CG = 16 * KC, OG = 16 * MO;
    const int Cout = P.G * OG;
    const int p0 = chunk * kTilePx, p = p0 + 8 * s;
    const int dh = P.dh[g], dw = P.dw[g], off = dh * P.W + dw;
    const int xelems = extent(P.N, P.xs, P.C, P.P), yelems = extent(P.N, P.ys, Cout, P.P);
    const rsrc_t rx = make_rsrc(P.x, xelems * 2);
    const rsrc_t ry = make_rsrc(P.y, yelems * 2);
    const TileMask tm = tile_mask(p0, lane, P, dh, dw);
    const bool live = p < P.P;
    const uint32_t bits = live ? unit_bits(tm, s) : 0u;
    const u32x4 msk = mask_of(bits);
    const int xg = (n * P.xs + g * CG * P.P) * 2;  // byte offset of the group's first input plane

    // weights: A operand, lane holds W[g][mo*16 + s][kc*16 + 4r .. +3]
    short4_t wa[MO][KC];
#pragma unroll
    for (int mo = 0; mo < MO; mo++)
#pragma unroll
        for (int kc = 0; kc < KC; kc++) __builtin_memcpy(&wa[mo][kc], P.w + ((g * OG + mo * 16 + s) * CG + kc * 16 + 4 * r), 8);

    u32x4 xs[KC][4];
#pragma unroll
    for (int kc = 0; kc < KC; kc++)
#pragma unroll
        for (int j = 0; j < 4; j++) xs[kc][j] = bload16(rx, live ? xg + ((kc * 16 + 4 * r + j) * P.P + p + off) * 2 : kOob);
    if (tile_near_ends(xg / 2, xg / 2 + (CG - 1) * P.P, p0, off, xelems)) {
#pragma unroll
        for (int kc = 0; kc < KC; kc++)
#pragma unroll
            for (int j = 0; j < 4; j++)
                reload_if_partial(xs[kc][j], rx, live ? xg + ((kc * 16 + 4 * r + j) * P.P + p + off) * 2 : kOob, xelems * 2);
    }
    u32x4 xr[MO][4];
    if (RES) {
        const int xo = (n * P.xs + g * OG * P.P) * 2;
#pragma unroll
        for (int mo = 0; mo < MO; mo++)
#pragma unroll
            for (int j = 0; j < 4; j++) {
                xr[mo][j] = bload16_nt(rx, live ? xo + ((mo * 16 + 4 * r + j) * P.P + p) * 2 : kOob);
                pin(xr[mo][j]);
            }
    }

    float4_t acc[MO][8];
#pragma unroll
    for (int mo = 0; mo < MO; mo++)
#pragma unroll
        for (int q = 0; q < 8; q++) acc[mo][q] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kc = 0; kc < KC; kc++) {
#pragma unroll
        for (int j = 0; j < 4; j++) xs[kc][j] = xs[kc][j] & msk;
        short4_t b[8];
        gather_all(xs[kc], b);
#pragma unroll
        for (int q = 0; q < 8; q++)
#pragma unroll
            for (int mo = 0; mo < MO; mo++) acc[mo][q] = mfma16(wa[mo][kc], b[q], acc[mo][q]);  // (a group contracts 16 channels: K = 16 is the whole depth)
    }
    const int yo = (n * P.ys + g * OG * P.P) * 2;
#pragma unroll
    for (int mo = 0; mo < MO; mo++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
            float v[8];
#pragma unroll
            for (int q = 0; q < 8; q++) v[q] = act_apply<ACT>(P, acc[mo][q][j]);
            if (RES) {
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    v[2 * k] += lo_f32(xr[mo][j][k]);
                    v[2 * k + 1] += hi_f32(xr[mo][j][k]);
                }
            }
            u32x4 out;
#pragma unroll
            for (int k = 0; k < 4; k++) out[k] = pack_bf16(v[2 * k], v[2 * k + 1]);
            bstore16_nt(ry, live ? yo + ((mo * 16 + 4 * r + j) * P.P + p) * 2 : kOob, out);
        }
}

// ----------------------------------------------------------------------------------------- backward
// dx[i,p] = (residual ? dy[i,p] : 0) + sum_o W[o,i] dz[o,p-d],  dz = dy * act'(z),  z[o,p-d] = sum_i W[o,i] x[i,p]
// dW[o,i] = sum_{n,p} dz[o,p-d] x[i,p]
//
// Registers hold the tile as: lane (r = lane/16, s = lane%16) -> channels 4r+j (j = 0..3) of the 8-pixel
// unit s.  That suits z = W x and dX = W^T dz (contractions over channels).  dW contracts over pixels and
// needs channel s with runs of consecutive pixels per lane instead; x and dz are passed through a
// wave-private LDS tile ([16 channels][128 pixels], rows padded to 272 bytes) to change distribution.
constexpr int kLdsRow = 17;  // u32x4 per LDS row: 16 units + 1 pad

template <int KC, int MO, int ACT, bool RES>
__device__ __forceinline__ void bwd_tile(const Params& P, rsrc_t rx, rsrc_t rdy, rsrc_t rdx, u32x4* lds_x, u32x4* lds_dz, int n, int g,
                                         int p0, int lane, const short4_t (&wa)[MO][KC], const short4_t (&wt)[KC][MO],
                                         float4_t (&dwacc)[MO][KC]) {
    const int r = lane >> 4, s = lane & 15;
    constexpr int CG = 16 * KC, OG = 16 * MO;
    const int dh = P.dh[g], dw = P.dw[g], off = dh * P.W + dw;
    const int Cout = P.G * OG;
    const int pA = p0 + 8 * s;
    const bool liveA = pA < P.P;
    const int xg = (n * P.xs + g * CG * P.P) * 2;
    const int dyg = (n * P.ys + g * OG * P.P) * 2;
    // dy is read at p - d: validity of the shifted source uses (-dh, -dw)
    const TileMask tm = tile_mask(p0, lane, P, -dh, -dw);
    const u32x4 msk = mask_of(liveA ? unit_bits(tm, s) : 0u);

    u32x4 xa[KC][4], dya[MO][4], dyu[KC][4];
#pragma unroll
    for (int kc = 0; kc < KC; kc++)
#pragma unroll
        for (int j = 0; j < 4; j++) xa[kc][j] = bload16_nt(rx, liveA ? xg + ((kc * 16 + 4 * r + j) * P.P + pA) * 2 : kOob);
#pragma unroll
    for (int mo = 0; mo < MO; mo++)
#pragma unroll
        for (int j = 0; j < 4; j++) dya[mo][j] = bload16(rdy, liveA ? dyg + ((mo * 16 + 4 * r + j) * P.P + pA - off) * 2 : kOob);
    if (tile_near_ends(dyg / 2, dyg / 2 + (OG - 1) * P.P, p0, -off, extent(P.N, P.ys, Cout, P.P))) {
        const int dyelems = extent(P.N, P.ys, Cout, P.P);
#pragma unroll
        for (int mo = 0; mo < MO; mo++)
#pragma unroll
            for (int j = 0; j < 4; j++)
                reload_if_partial(dya[mo][j], rdy, liveA ? dyg + ((mo * 16 + 4 * r + j) * P.P + pA - off) * 2 : kOob, dyelems * 2);
    }
    // (the unshifted dy of the residual: with one 16-channel block per group it is fetched with everything else; with
    // more the registers are short, and each block's rows are fetched just ahead of its dx)
    if (RES && KC == 1) {
#pragma unroll
        for (int j = 0; j < 4; j++) {
            dyu[0][j] = bload16_nt(rdy, liveA ? dyg + ((4 * r + j) * P.P + pA) * 2 : kOob);
            pin(dyu[0][j]);
        }
    }
    // x -> LDS rows (channel 4r+j, unit s) and -> MFMA operands
    short4_t xq[KC][8];
#pragma unroll
    for (int kc = 0; kc < KC; kc++) {
#pragma unroll
        for (int j = 0; j < 4; j++) lds_x[(kc * 16 + 4 * r + j) * kLdsRow + s] = xa[kc][j];
        gather_all(xa[kc], xq[kc]);
    }

    short4_t dzq[MO][8];
#pragma unroll
    for (int mo = 0; mo < MO; mo++) {
#pragma unroll
        for (int j = 0; j < 4; j++) dya[mo][j] = dya[mo][j] & msk;
        u32x4 dzrow[4];  // dz of channel 4r+j over the unit's 8 pixels, for the LDS tile
        // steps of QS pixel offsets keep the live accumulators at 4 * QS registers (16; 8 where a group has more than
        // one 16-channel block and the tile's registers are short)
        constexpr int QS = KC > 1 ? 2 : 4;
#pragma unroll
        for (int h = 0; h < 8 / QS; h++) {
            float4_t z[QS];
#pragma unroll
            for (int q = 0; q < QS; q++) {
                z[q] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kc = 0; kc < KC; kc++) z[q] = mfma16(wa[mo][kc], xq[kc][QS * h + q], z[q]);
            }
            float d[QS][4];
#pragma unroll
            for (int j = 0; j < 4; j++) {
#pragma unroll
                for (int q = 0; q < QS; q += 2) {
                    const uint32_t w = dya[mo][j][(QS * h + q) / 2];
                    d[q][j] = act_dz<ACT>(P, z[q][j], lo_f32(w));
                    d[q + 1][j] = act_dz<ACT>(P, z[q + 1][j], hi_f32(w));
                    dzrow[j][(QS * h + q) / 2] = pack_bf16(d[q][j], d[q + 1][j]);
                }
            }
#pragma unroll
            for (int q = 0; q < QS; q++) dzq[mo][QS * h + q] = pack4(d[q][0], d[q][1], d[q][2], d[q][3]);
        }
#pragma unroll
        for (int j = 0; j < 4; j++) lds_dz[(mo * 16 + 4 * r + j) * kLdsRow + s] = dzrow[j];
    }
#pragma unroll
    for (int kc = 0; kc < KC; kc++) {
        if (RES && KC > 1) {
            asm volatile("" ::: "memory");  // (not earlier: the registers are needed until here)
#pragma unroll
            for (int j = 0; j < 4; j++) dyu[kc][j] = bload16_nt(rdy, liveA ? dyg + ((kc * 16 + 4 * r + j) * P.P + pA) * 2 : kOob);
        }
        float4_t dxs[8];
#pragma unroll
        for (int q = 0; q < 8; q++) {
            dxs[q] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int mo = 0; mo < MO; mo++) dxs[q] = mfma16(wt[kc][mo], dzq[mo][q], dxs[q]);
        }
#pragma unroll
        for (int j = 0; j < 4; j++) {
            float v[8];
#pragma unroll
            for (int q = 0; q < 8; q++) v[q] = dxs[q][j];
            if (RES) {
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    v[2 * k] += lo_f32(dyu[kc][j][k]);
                    v[2 * k + 1] += hi_f32(dyu[kc][j][k]);
                }
            }
            u32x4 out;
#pragma unroll
            for (int k = 0; k < 4; k++) out[k] = pack_bf16(v[2 * k], v[2 * k + 1]);
            bstore16_nt(rdx, liveA ? xg + ((kc * 16 + 4 * r + j) * P.P + pA) * 2 : kOob, out);
        }
    }
    // dW += dz x^T over the tile's pixels: lane reads channel s, unit 4m+r (8 consecutive pixels) of both tiles;
    // MFMA k-slot 4r+jj <-> pixel 8(4m+r) + 4*half + jj for both operands.  Lanes of dead units hold zeros.
#pragma unroll
    for (int m = 0; m < 4; m++)
#pragma unroll
        for (int mo = 0; mo < MO; mo++) {
            const u32x4 dzb = lds_dz[(mo * 16 + s) * kLdsRow + 4 * m + r];
#pragma unroll
            for (int kc = 0; kc < KC; kc++) {
                const u32x4 xb = lds_x[(kc * 16 + s) * kLdsRow + 4 * m + r];
                dwacc[mo][kc] = mfma32(as_short4(dzb[0], dzb[1]), as_short4(dzb[2], dzb[3]), as_short4(xb[0], xb[1]), as_short4(xb[2], xb[3]), dwacc[mo][kc]);
            }
        }
}

template <int KC, int MO, int ACT, bool RES>
__device__ __forceinline__ void bwd_body(const Params& P) {
    __shared__ u32x4 lds[kWaves][(KC + MO) * 16 * kLdsRow];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane >> 4, s = lane & 15;
    constexpr int CG = 16 * KC, OG = 16 * MO;
    const int g = blockIdx.y;
    const int wg = blockIdx.x;
    const int Cout = P.G * OG;
    const rsrc_t rx = make_rsrc(P.x, extent(P.N, P.xs, P.C, P.P) * 2);
    const rsrc_t rdx = make_rsrc(P.dx, extent(P.N, P.xs, P.C, P.P) * 2);
    const rsrc_t rdy = make_rsrc(P.dy, extent(P.N, P.ys, Cout, P.P) * 2);
    u32x4* lds_x = lds[wave];
    u32x4* lds_dz = lds[wave] + KC * 16 * kLdsRow;

    short4_t wa[MO][KC];  // W[o = mo*16+s][i = kc*16+4r..+3]
    short4_t wt[KC][MO];  // W[o = mo*16+4r+j][i = kc*16+s], j = 0..3
#pragma unroll
    for (int mo = 0; mo < MO; mo++)
#pragma unroll
        for (int kc = 0; kc < KC; kc++) {
            __builtin_memcpy(&wa[mo][kc], P.w + ((g * OG + mo * 16 + s) * CG + kc * 16 + 4 * r), 8);
#pragma unroll
            for (int j = 0; j < 4; j++) wt[kc][mo][j] = (short)P.w[(g * OG + mo * 16 + 4 * r + j) * CG + kc * 16 + s];
        }
    float4_t dwacc[MO][KC];
#pragma unroll
    for (int mo = 0; mo < MO; mo++)
#pragma unroll
        for (int kc = 0; kc < KC; kc++) dwacc[mo][kc] = float4_t{0.f, 0.f, 0.f, 0.f};

    const int tiles_per_group = P.N * P.chunks;
    for (int it = 0; it < P.tiles_per_wave; it++) {
        const int t = (wg * kWaves + wave) * P.tiles_per_wave + it;
        if (t >= tiles_per_group) break;
        const int n = P.chunks == 1 ? t : (int)__umulhi((uint32_t)t, P.magicChunks), chunk = t - n * P.chunks;  // magic overflows for 1
        bwd_tile<KC, MO, ACT, RES>(P, rx, rdy, rdx, lds_x, lds_dz, n, g, chunk * kTilePx, lane, wa, wt, dwacc);
    }
    // the workgroup's four wavefronts are summed in a fixed order through LDS: one partial per workgroup;
    // the reduction kernel then sums the partials in a fixed order
    __syncthreads();
    float* red = reinterpret_cast<float*>(&lds[0][0]);
#pragma unroll
    for (int mo = 0; mo < MO; mo++)
#pragma unroll
        for (int kc = 0; kc < KC; kc++)
#pragma unroll
            for (int j = 0; j < 4; j++) red[wave * (OG * CG) + (mo * 16 + 4 * r + j) * CG + kc * 16 + s] = dwacc[mo][kc][j];
    __syncthreads();
    float* part = P.partial + ((long long)g * P.wgs_per_group + wg) * (OG * CG);
    for (int e = threadIdx.x; e < OG * CG; e += 64 * kWaves) {
        float sum = red[e];
#pragma unroll
        for (int wv = 1; wv < kWaves; wv++) sum += red[wv * (OG * CG) + e];
        part[e] = sum;
    }
}

// Cheap activations fit 128 registers (4 wavefronts per SIMD); gelu and clipped exp need more.
template <int KC, int MO, int ACT, bool RES>
__global__ __launch_bounds__(64 * kWaves) __attribute__((amdgpu_waves_per_eu(4, 4))) void k_bwd(Params P) {
    bwd_body<KC, MO, ACT, RES>(P);
}
template <int KC, int MO, int ACT, bool RES>
__global__ __launch_bounds__(64 * kWaves) void k_bwd_wide(Params P) {
    bwd_body<KC, MO, ACT, RES>(P);
}
// Groups of 32 channels: two wavefronts per SIMD is what the tile's registers allow.
template <int KC, int MO, int ACT, bool RES>
__global__ __launch_bounds__(64 * kWaves) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_bwd_two(Params P) {
    bwd_body<KC, MO, ACT, RES>(P);
}

// dW[g][e] = sum over the group's partials, in order.  One block per (group, 8 elements): 128 segments of
// partials are summed by 128 threads per element and combined by a fixed-order tree in LDS.
__global__ __launch_bounds__(1024) void k_dw_reduce(const float* __restrict__ partial, float* __restrict__ dw, int n_partials,
                                                    int elems) {
    __shared__ float red[128][8];
    const int g = blockIdx.y;
    const int el = threadIdx.x & 7, seg = threadIdx.x >> 3;
    const int e = blockIdx.x * 8 + el;
    const int per = (n_partials + 127) / 128;
    float sum = 0.f;
    if (e < elems) {
        const float* src = partial + (long long)g * n_partials * elems + e;
        const int end = min(n_partials, (seg + 1) * per);
        for (int k = seg * per; k < end; k++) sum += src[(long long)k * elems];
    }
    red[seg][el] = sum;
    __syncthreads();
    for (int st = 64; st > 0; st >>= 1) {
        if (seg < st) red[seg][el] += red[seg + st][el];
        __syncthreads();
    }
    if (seg == 0 && e < elems) dw[(long long)g * elems + e] = red[0][el];
}

}  // namespace

bool supported(int KC, int MO) { return KC == MO && (KC == 1 || KC == 2); }

template <int ACT, bool RES>
static void launch_fwd(const Params& P, int W, hipStream_t s) {
    const dim3 grid((unsigned)((P.chunks + kWaves - 1) / kWaves), (unsigned)P.G, (unsigned)P.N);
    if (!P.total_tiles) return;
    if (W == 2) CANVAS_LAUNCH((k_fwd<2, 2, ACT, RES>), grid, dim3(64 * kWaves), 0, s, P);
    else CANVAS_LAUNCH((k_fwd<1, 1, ACT, RES>), grid, dim3(64 * kWaves), 0, s, P);
}
template <int ACT, bool RES>
static void launch_bwd(const Params& P, int W, hipStream_t s) {
    const dim3 grid((unsigned)P.wgs_per_group, (unsigned)P.G);
    if (!P.total_tiles) return;
    if (W == 2) CANVAS_LAUNCH((k_bwd_two<2, 2, ACT, RES>), grid, dim3(64 * kWaves), 0, s, P);
    else if (ACT == 2 || ACT == 3) CANVAS_LAUNCH((k_bwd_wide<1, 1, ACT, RES>), grid, dim3(64 * kWaves), 0, s, P);
    else CANVAS_LAUNCH((k_bwd<1, 1, ACT, RES>), grid, dim3(64 * kWaves), 0, s, P);
}

#define SGFC_DISPATCH(fn)                                                        \
    switch (P.act) {                                                             \
    case kActNone: P.residual ? fn<kActNone, true>(P, KC, s) : fn<kActNone, false>(P, KC, s); break; \
    case 0: P.residual ? fn<0, true>(P, KC, s) : fn<0, false>(P, KC, s); break;          \
    case 1: P.residual ? fn<1, true>(P, KC, s) : fn<1, false>(P, KC, s); break;          \
    case 2: P.residual ? fn<2, true>(P, KC, s) : fn<2, false>(P, KC, s); break;          \
    default: P.residual ? fn<3, true>(P, KC, s) : fn<3, false>(P, KC, s); break;         \
    }

void forward(const Params& P, int KC, int MO, hipStream_t s) {
    (void)MO;
    SGFC_DISPATCH(launch_fwd)
}

void backward(const Params& P, int KC, int MO, hipStream_t s) {
    (void)MO;
    SGFC_DISPATCH(launch_bwd)
}

void dw_reduce(const float* partial, float* dw, int G, int n_partials, int elems, hipStream_t s) {
    CANVAS_LAUNCH(k_dw_reduce, dim3((unsigned)((elems + 7) / 8), (unsigned)G), dim3(1024), 0, s, partial, dw, n_partials, elems);
}

}  // namespace sgfc
}  // namespace canvas
