// Grouped FC on bf16 MFMA with an implicit (never materialised) Unfold of the operand.
//
//   forward / data gradient:  y[n, g*Og+o, p] (+)= sum_k w[g][o][k] * row(n, g, k)[p + off(k)]
//   weight gradient:          dw[g][o][k] = sum_{n,p} dy[n, g*Og+o, p] * row(n, g, k)[p + off(k)]
//
// Canvas paper, Section 5: Fully-connected remaps all channel dims (channels of a group and taps) to a
// new channel dim, groups stay apart; Unfold is an index rearrangement U(c,kh,kw,h,w) = I(c,h+kh,w+kw),
// so the contraction reads the un-unfolded tensor at shifted addresses with zeros outside the image.
// The data gradient of an FC that consumed an Unfold is the same contraction applied to dy with
// transposed, tap-flipped weights (transpose_weights), which also folds the Unfold adjoint in.
//
// NCHW keeps pixels contiguous and the contraction index strided, while an MFMA operand wants the
// contraction index in the lane.  As in the fused shift/FC kernels, a lane loads 8 consecutive pixels of
// 4 rows and assembles the operand of pixel offset q from the q-th halves (two byte-permutes), so the
// forward tile needs no LDS.  In the weight gradient the contraction runs over pixels, which is the
// memory order of both operands: 16-byte loads are MFMA operands as they are.
#include "gfc_kernels.hpp"

#include <algorithm>

#include <hip/hip_runtime.h>

#include "launch.hpp"
#include "tile_util.hpp"

namespace canvas {
namespace gfc {

namespace {

using namespace canvas::tile;

constexpr int kWaves = 4;

__device__ __forceinline__ uint32_t div_magic(uint32_t x, uint32_t magic) { return magic ? __umulhi(x, magic) : x; }

// Validity bits of a lane's 8 consecutive pixels starting at flat pixel p (all of one image):
// rowpack byte i / colpack byte i hold, for window row i / column i, which of the 8 pixels have their
// source row / column inside the image.  Needs W >= 4 (a run of 8 pixels wraps at most twice).
struct PixGeom {
    uint64_t rowpack, colpack;
};
__device__ __forceinline__ PixGeom pix_geom(const Params& P, int p) {
    PixGeom gm;
    gm.rowpack = 0;
    gm.colpack = 0;
    const int h0 = (int)div_magic((uint32_t)p, P.magicW), w0 = p - h0 * P.W;
#pragma unroll
    for (int q = 0; q < 8; q++) {
        int c = w0 + q, h = h0;
        if (c >= P.W) { c -= P.W; h++; }
        if (c >= P.W) { c -= P.W; h++; }
        const bool inside = p + q < P.P;
        for (int i = 0; i < P.KH; i++)
            if (inside && (unsigned)(h + i - P.KH / 2) < (unsigned)P.H) gm.rowpack |= (uint64_t)1 << (8 * i + q);
        for (int i = 0; i < P.KW; i++)
            if ((unsigned)(c + i - P.KW / 2) < (unsigned)P.W) gm.colpack |= (uint64_t)1 << (8 * i + q);
    }
    return gm;
}
__device__ __forceinline__ uint32_t tap_bits(const PixGeom& gm, int khi, int kwi) {
    return (uint32_t)(gm.rowpack >> (8 * khi)) & (uint32_t)(gm.colpack >> (8 * kwi)) & 0xffu;
}

// Validity bits of the 8 pixels p..p+7 under the window offset (dh, dw), computed directly.
__device__ __forceinline__ uint32_t tap_bits_direct(const Params& P, int p, int dh, int dw) {
    int h = (int)div_magic((uint32_t)p, P.magicW), c = p - h * P.W;
    uint32_t bits = 0;
#pragma unroll
    for (int q = 0; q < 8; q++) {
        const bool v = p + q < P.P && (unsigned)(h + dh) < (unsigned)P.H && (unsigned)(c + dw) < (unsigned)P.W;
        bits |= (v ? 1u : 0u) << q;
        if (++c == P.W) { c = 0; h++; }
    }
    return bits;
}

// 8 consecutive elements at element offset `e` of a bf16 or fp32 buffer as packed bf16.  An fp32 source
// is split into hi = bf16(x) and lo = bf16(x - hi): feeding both to the MFMA keeps ~16 mantissa bits, so
// an fp32 intermediate is not degraded to bf16 just because the next node is an FC.
struct Pair8 {
    u32x4 hi, lo;
};
__device__ __forceinline__ void split2(float a, float b, Pair8& v, int k) {
    const uint32_t hi = pack_bf16(a, b);
    v.hi[k] = hi;
    v.lo[k] = pack_bf16(a - lo_f32(hi), b - hi_f32(hi));
}
// 8 consecutive elements as bf16 hi (+ lo for fp32 sources) pairs.  check_ends (wave-uniform): the 16-byte
// accesses of this wavefront may straddle an end of the buffer of `bytes` bytes -- the hardware drops such an
// access as a whole, so the lanes concerned re-read it element by element.
template <bool F32>
__device__ __forceinline__ Pair8 load8(rsrc_t r, int e, bool ok, bool check_ends, int bytes) {
    Pair8 v;
    if (!F32) {
        v.hi = bload16(r, ok ? e * 2 : kOob);
        if (check_ends) reload_if_partial(v.hi, r, ok ? e * 2 : kOob, bytes);
        v.lo = u32x4{0u, 0u, 0u, 0u};
        return v;
    }
    u32x4 a = bload16(r, ok ? e * 4 : kOob), b = bload16(r, ok ? e * 4 + 16 : kOob);
    if (check_ends) {
        reload_f32x4_if_partial(a, r, ok ? e * 4 : kOob, bytes);
        reload_f32x4_if_partial(b, r, ok ? e * 4 + 16 : kOob, bytes);
    }
    split2(__uint_as_float(a[0]), __uint_as_float(a[1]), v, 0);
    split2(__uint_as_float(a[2]), __uint_as_float(a[3]), v, 1);
    split2(__uint_as_float(b[0]), __uint_as_float(b[1]), v, 2);
    split2(__uint_as_float(b[2]), __uint_as_float(b[3]), v, 3);
    return v;
}

// ------------------------------------------------------------------------------------------- forward
// One wavefront: 16*MO output channels of one group x 16 units of 8 pixels; K in steps of 16.  Units are
// numbered across the whole batch (unit U -> image U / units_per_image), so small images (7x7, 14x14)
// still fill the tile.  Lane (r = lane/16, s = lane%16): B operand rows k = k0 + 4r + j of unit s; A
// operand w[o = 16*mo + s][k = k0 + 4r ..+3]; accumulator acc[mo][q][j] = y[o = 16*mo + 4r + j][pixel q of unit s].
template <bool F32>
struct RawChunk {
    u32x4 a[4], b[F32 ? 4 : 1];  // rows j = 0..3: 8 elements each (fp32: a = first four, b = last four)
};

template <int MO, bool SRC_F32, bool DST_F32, bool TAPS>
__global__ __launch_bounds__(64 * kWaves) void k_fwd(Params P) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // (sequence of the workgroups: the output tiles of one pixel tile, which read the same rows, then the pixel tiles,
    // whose neighbours share window halos, then the groups)
    const unsigned seq = xcd_sequence();
    const unsigned pt = seq / (unsigned)P.otiles, bx = pt % gridDim.x;
    const int tile = (int)bx * kWaves + wave;
    const int total_units = P.N * P.upi;
    if (tile * 16 >= total_units) return;
    const int g = (int)(pt / gridDim.x), ot = (int)(seq - pt * (unsigned)P.otiles);
    const int r = lane >> 4, s = lane & 15;
    const int U = tile * 16 + s;
    const bool live = U < total_units;
    const int n = live ? (int)div_magic((uint32_t)U, P.magicUpi) : 0;
    const int p = live ? (U - n * P.upi) * 8 : 0;
    const int esz = SRC_F32 ? 4 : 2;
    const int src_elems = P.N * P.G * P.R * P.P;
    const rsrc_t rs = make_rsrc(P.src, src_elems * esz);
    const rsrc_t rw = make_rsrc(P.w, P.G * P.Og * P.K * 2);
    const int row0 = (n * P.G + g) * P.R;  // first source row of this lane's image and group
    const int obase = ot * 16 * MO;

    PixGeom gm = {0, 0};
    if (TAPS) gm = pix_geom(P, p);
    const int maxoff = (P.KH / 2) * P.W + P.KW / 2;
    // wave-uniform: could a 16/32-byte access of this tile straddle an end of the source tensor?
    const int n_first = (int)div_magic((uint32_t)(tile * 16), P.magicUpi);
    const int n_last = (int)div_magic((uint32_t)min(tile * 16 + 15, total_units - 1), P.magicUpi);
    const bool near_ends = (n_first * P.G + g) * P.R * P.P - maxoff < 0 ||
                           ((n_last * P.G + g) * P.R + P.R) * P.P + 8 + maxoff > src_elems;

    float4_t acc[MO][8];
#pragma unroll
    for (int mo = 0; mo < MO; mo++)
#pragma unroll
        for (int q = 0; q < 8; q++) acc[mo][q] = float4_t{0.f, 0.f, 0.f, 0.f};

    // element offset and validity bits of row k = k0 + 4r + j for this lane's unit
    auto row_elem = [&](int k, uint32_t& bits) {
        int row = k, off = 0;
        bits = 0xffu;
        if (TAPS) {
            row = (int)div_magic((uint32_t)k, P.magicTV);
            const int tv = k - row * P.TV;
            const int khi = (int)div_magic((uint32_t)tv, P.magicKW), kwi = tv - khi * P.KW;
            off = (khi - P.KH / 2) * P.W + (kwi - P.KW / 2);
            bits = tap_bits(gm, khi, kwi);
        }
        return (row0 + row) * P.P + p + off;
    };
    auto load_raw = [&](int k0, RawChunk<SRC_F32>& c, short4_t (&wa)[MO]) {
#pragma unroll
        for (int mo = 0; mo < MO; mo++) {
            const int o = obase + mo * 16 + s;
            const int widx = ((g * P.Og + o) * P.K + k0 + 4 * r) * 2;
            uint32_t w2[2];
            if (o < P.Og && k0 + 4 * r + 3 < P.K) {
                // (the 8-byte access stays inside the weight tensor: it ends at or before the row's end)
                const auto t = __builtin_amdgcn_raw_buffer_load_b64(rw, widx, 0, 0);
                w2[0] = t[0];
                w2[1] = t[1];
            } else {
                uint32_t h[4];
#pragma unroll
                for (int i = 0; i < 4; i++)
                    h[i] = (o < P.Og && k0 + 4 * r + i < P.K) ? (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(rw, widx + 2 * i, 0, 0) : 0u;
                w2[0] = h[0] | (h[1] << 16);
                w2[1] = h[2] | (h[3] << 16);
            }
            wa[mo] = as_short4(w2[0], w2[1]);
        }
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int k = k0 + 4 * r + j;
            uint32_t bits;
            const int e = row_elem(k, bits);
            const bool ok = live && k < P.K;
            if (SRC_F32) {
                c.a[j] = bload16(rs, ok ? e * 4 : kOob);
                c.b[j & (SRC_F32 ? 3 : 0)] = bload16(rs, ok ? e * 4 + 16 : kOob);
                if (near_ends) {  // tiles at the two ends of the tensor: lanes whose access is partly outside re-read it
                    reload_f32x4_if_partial(c.a[j], rs, ok ? e * 4 : kOob, src_elems * esz);
                    reload_f32x4_if_partial(c.b[j & (SRC_F32 ? 3 : 0)], rs, ok ? e * 4 + 16 : kOob, src_elems * esz);
                }
            } else {
                c.a[j] = bload16(rs, ok ? e * 2 : kOob);
                if (near_ends) reload_if_partial(c.a[j], rs, ok ? e * 2 : kOob, src_elems * esz);
            }
        }
    };

    // One chunk of 16 contraction rows as MFMA operands: bs[q] for pixel q of the lane's unit (and bl[q], the low
    // halves of fp32 rows)
    auto operands = [&](int k0, const RawChunk<SRC_F32>& cur, short4_t (&bs)[8], short4_t (&bl)[8]) {
        u32x4 xs[4], xl[4];
#pragma unroll
        for (int j = 0; j < 4; j++) {
            if (SRC_F32) {
                Pair8 v;
                const u32x4 a = cur.a[j], b = cur.b[j & (SRC_F32 ? 3 : 0)];
                split2(__uint_as_float(a[0]), __uint_as_float(a[1]), v, 0);
                split2(__uint_as_float(a[2]), __uint_as_float(a[3]), v, 1);
                split2(__uint_as_float(b[0]), __uint_as_float(b[1]), v, 2);
                split2(__uint_as_float(b[2]), __uint_as_float(b[3]), v, 3);
                xs[j] = v.hi;
                xl[j] = v.lo;
            } else {
                xs[j] = cur.a[j];
            }
        }
        if (TAPS) {
#pragma unroll
            for (int j = 0; j < 4; j++) {
                uint32_t bits;
                (void)row_elem(k0 + 4 * r + j, bits);
                const u32x4 m = mask_of(bits);
                xs[j] = xs[j] & m;
                if (SRC_F32) xl[j] = xl[j] & m;
            }
        }
        gather_all(xs, bs);
        if (SRC_F32) gather_all(xl, bl);
    };
    if (SRC_F32) {
        // fp32 rows: the high and the low bf16 halves of a chunk meet the same weights: one K = 32 step, w | w against hi | lo
        for (int k0 = 0; k0 < P.K; k0 += 16) {
            RawChunk<SRC_F32> cur;
            short4_t wa[MO], bs[8], bl[8];
            load_raw(k0, cur, wa);
            operands(k0, cur, bs, bl);
#pragma unroll
            for (int q = 0; q < 8; q++)
#pragma unroll
                for (int mo = 0; mo < MO; mo++) acc[mo][q] = mfma32(wa[mo], wa[mo], bs[q], bl[q], acc[mo][q]);
        }
    } else {
        // bf16 rows: two chunks of 16 rows per K = 32 step (rows beyond K load as zeros, weights too)
        for (int k0 = 0; k0 < P.K; k0 += 32) {
            RawChunk<SRC_F32> c0, c1;
            short4_t w0[MO], w1[MO], b0[8], b1[8], unused[8];
            load_raw(k0, c0, w0);
            load_raw(k0 + 16, c1, w1);
            operands(k0, c0, b0, unused);
            operands(k0 + 16, c1, b1, unused);
#pragma unroll
            for (int q = 0; q < 8; q++)
#pragma unroll
                for (int mo = 0; mo < MO; mo++) acc[mo][q] = mfma32(w0[mo], w1[mo], b0[q], b1[q], acc[mo][q]);
        }
    }

    if (!live) return;
    const int nvalid = min(8, P.P - p);
    const int dsz = DST_F32 ? 4 : 2;
    const rsrc_t rd = make_rsrc(P.dst, P.N * P.G * P.Og * P.P * dsz);
#pragma unroll
    for (int mo = 0; mo < MO; mo++) {
        // What the four rows of this step are added to is read before any of them is stored: loads that follow
        // a store to the same tensor are not moved ahead of it, and would cost a memory round trip per row.
        u32x4 pre[4][2];
        const rsrc_t rad = make_rsrc(P.addend, P.N * P.G * P.Og * P.P * 2);
        if ((DST_F32 && P.acc) || (!DST_F32 && P.addend)) {
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const int o = obase + mo * 16 + 4 * r + j;
                const int e = ((n * P.G + g) * P.Og + o) * P.P + p;
                const bool ok = o < P.Og && nvalid == 8;
                if (DST_F32) {
                    pre[j][0] = bload16(rd, ok ? e * 4 : kOob);
                    pre[j][1] = bload16(rd, ok ? e * 4 + 16 : kOob);
                } else {
                    pre[j][0] = bload16(rad, ok ? e * 2 : kOob);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int o = obase + mo * 16 + 4 * r + j;
            if (o >= P.Og) continue;
            const int e = ((n * P.G + g) * P.Og + o) * P.P + p;
            float v[8];
#pragma unroll
            for (int q = 0; q < 8; q++) v[q] = acc[mo][q][j];
            if (nvalid == 8) {
                if (DST_F32) {
                    u32x4 lo, hi;
                    if (P.acc) {
                        lo = pre[j][0];
                        hi = pre[j][1];
#pragma unroll
                        for (int k = 0; k < 4; k++) {
                            v[k] += __uint_as_float(lo[k]);
                            v[4 + k] += __uint_as_float(hi[k]);
                        }
                    }
#pragma unroll
                    for (int k = 0; k < 4; k++) {
                        lo[k] = __float_as_uint(v[k]);
                        hi[k] = __float_as_uint(v[4 + k]);
                    }
                    bstore16(rd, e * 4, lo);
                    bstore16(rd, e * 4 + 16, hi);
                } else {
                    if (P.addend) {  // bf16 tensor of the output's shape added before rounding
                        const u32x4 ad = pre[j][0];
#pragma unroll
                        for (int k = 0; k < 4; k++) {
                            v[2 * k] += lo_f32(ad[k]);
                            v[2 * k + 1] += hi_f32(ad[k]);
                        }
                    }
                    u32x4 out;
#pragma unroll
                    for (int k = 0; k < 4; k++) out[k] = pack_bf16(v[2 * k], v[2 * k + 1]);
                    bstore16(rd, e * 2, out);
                }
            } else {
#pragma unroll
                for (int q = 0; q < 8; q++) {
                    if (q >= nvalid) break;
                    if (DST_F32) {
                        float* d = reinterpret_cast<float*>(P.dst) + e + q;
                        *d = P.acc ? *d + v[q] : v[q];
                    } else {
                        float t = v[q];
                        if (P.addend) t += __uint_as_float((uint32_t)P.addend[e + q] << 16);
                        reinterpret_cast<uint16_t*>(P.dst)[e + q] = (uint16_t)(pack_bf16(t, 0.f) & 0xffffu);
                    }
                }
            }
        }
    }
}

// ----------------------------------------------------------------------------------- weight gradient
// One wavefront: a 16*MO x 16*NK tile of dw[g] over a slice of the (image, pixel) range, 32 pixels per
// step.  Lane (r, s) loads pixels 8r..8r+7 of the step from dy row o = 16*mo + s and from operand row
// k = 16*nk + s: the two halves of each 16-byte load are the A / B operands of two MFMAs whose
// contraction slot 4r+jj is pixel 8r + 4*half + jj.  Result: lane holds dw[o = 16*mo + 4r + jj][k = 16*nk + s].
template <int MO, int NK, bool SRC_F32, bool DY_F32, bool TAPS>
__global__ __launch_bounds__(64 * kWaves) void k_wgrad(Params P) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int slice = blockIdx.x * kWaves + wave;
    const bool active = slice < P.slices;  // (no early exit: every wavefront takes part in the workgroup sum below)
    const int g = blockIdx.z;
    const int ot = blockIdx.y / P.ktiles, kt = blockIdx.y - ot * P.ktiles;
    const int r = lane >> 4, s = lane & 15;
    const int esz = SRC_F32 ? 4 : 2;
    const int src_elems = P.N * P.G * P.R * P.P;
    const rsrc_t rs = make_rsrc(P.src, src_elems * esz);
    const rsrc_t rdy = make_rsrc(P.dy, P.N * P.G * P.Og * P.P * (DY_F32 ? 4 : 2));
    const int obase = ot * 16 * MO, kbase = kt * 16 * NK;

    // this lane's operand rows: fixed source row, tap offset and window position per nk
    int krow[NK], koff[NK], khi[NK], kwi[NK];
    bool kok[NK];
#pragma unroll
    for (int nk = 0; nk < NK; nk++) {
        const int k = kbase + nk * 16 + s;
        kok[nk] = k < P.K;
        krow[nk] = k;
        koff[nk] = 0;
        khi[nk] = kwi[nk] = 0;
        if (TAPS) {
            krow[nk] = (int)div_magic((uint32_t)k, P.magicTV);
            const int tv = k - krow[nk] * P.TV;
            khi[nk] = (int)div_magic((uint32_t)tv, P.magicKW);
            kwi[nk] = tv - khi[nk] * P.KW;
            koff[nk] = (khi[nk] - P.KH / 2) * P.W + (kwi[nk] - P.KW / 2);
        }
    }
    float4_t acc[MO][NK];
#pragma unroll
    for (int mo = 0; mo < MO; mo++)
#pragma unroll
        for (int nk = 0; nk < NK; nk++) acc[mo][nk] = float4_t{0.f, 0.f, 0.f, 0.f};

    const int c_begin = active ? slice * P.per_slice : 0, c_end = active ? min(P.N * P.chunks32, c_begin + P.per_slice) : 0;
    int n = (int)div_magic((uint32_t)c_begin, P.magicC32);
    int pc = c_begin - n * P.chunks32;
    const int maxoff = (P.KH / 2) * P.W + P.KW / 2;
    for (int c = c_begin; c < c_end; c++) {
        const int p = pc * 32 + 8 * r;
        const bool live = p < P.P;
        const int nvalid = live ? min(8, P.P - p) : 0;
        const int row0 = (n * P.G + g) * P.R;
        const bool near_ends = row0 * P.P + pc * 32 - maxoff < 0 || (row0 + P.R - 1) * P.P + pc * 32 + 40 + maxoff > src_elems ||
                               ((n * P.G + g) * P.Og + P.Og - 1) * P.P + pc * 32 + 40 > P.N * P.G * P.Og * P.P;
        const u32x4 mvalid = mask_of(nvalid >= 8 ? 0xffu : ((1u << nvalid) - 1u));
        Pair8 a[MO], b[NK];  // dy is fp32: hi + lo; the operand rows too when they are fp32
#pragma unroll
        for (int mo = 0; mo < MO; mo++) {
            const int o = obase + mo * 16 + s;
            const bool ok = live && o < P.Og;
            const int e = ((n * P.G + g) * P.Og + o) * P.P + p;
            a[mo] = load8<DY_F32>(rdy, e, ok, near_ends, P.N * P.G * P.Og * P.P * (DY_F32 ? 4 : 2));
            a[mo].hi = a[mo].hi & mvalid;
            a[mo].lo = a[mo].lo & mvalid;
        }
#pragma unroll
        for (int nk = 0; nk < NK; nk++) {
            const bool ok = live && kok[nk];
            const int e = (row0 + krow[nk]) * P.P + p + koff[nk];
            b[nk] = load8<SRC_F32>(rs, e, ok, near_ends, src_elems * (SRC_F32 ? 4 : 2));
            if (TAPS) {
                const u32x4 m = mask_of(live ? tap_bits_direct(P, p, khi[nk] - P.KH / 2, kwi[nk] - P.KW / 2) : 0u);
                b[nk].hi = b[nk].hi & m;
                b[nk].lo = b[nk].lo & m;
            }
        }
#pragma unroll
        for (int mo = 0; mo < MO; mo++)
#pragma unroll
            for (int nk = 0; nk < NK; nk++) {
                float4_t c = acc[mo][nk];  // (8 pixels per lane and operand: one K = 32 step each)
                c = mfma32(a[mo].hi, b[nk].hi, c);
                if (DY_F32) c = mfma32(a[mo].lo, b[nk].hi, c);
                if (SRC_F32) c = mfma32(a[mo].hi, b[nk].lo, c);
                acc[mo][nk] = c;
            }
        if (++pc == P.chunks32) { pc = 0; n++; }
    }
    // sum of the workgroup's four wavefronts (consecutive slices of the same tile) in a fixed order,
    // (w0 + w2) + (w1 + w3), through LDS: one partial per workgroup
    __shared__ float red[2][MO * NK * 4][64];
    auto put = [&](int slot) {
#pragma unroll
        for (int mo = 0; mo < MO; mo++)
#pragma unroll
            for (int nk = 0; nk < NK; nk++)
#pragma unroll
                for (int jj = 0; jj < 4; jj++) red[slot][(mo * NK + nk) * 4 + jj][lane] = acc[mo][nk][jj];
    };
    auto add = [&](int slot) {
#pragma unroll
        for (int mo = 0; mo < MO; mo++)
#pragma unroll
            for (int nk = 0; nk < NK; nk++)
#pragma unroll
                for (int jj = 0; jj < 4; jj++) acc[mo][nk][jj] += red[slot][(mo * NK + nk) * 4 + jj][lane];
    };
    if (wave >= 2) put(wave - 2);
    __syncthreads();
    if (wave < 2) add(wave);
    __syncthreads();
    if (wave == 1) put(0);
    __syncthreads();
    if (wave != 0) return;
    add(0);
    float* part = P.partial + (long long)blockIdx.x * P.G * P.Og * P.K;
#pragma unroll
    for (int mo = 0; mo < MO; mo++)
#pragma unroll
        for (int nk = 0; nk < NK; nk++)
#pragma unroll
            for (int jj = 0; jj < 4; jj++) {
                const int o = obase + mo * 16 + 4 * r + jj, k = kbase + nk * 16 + s;
                if (o < P.Og && k < P.K) part[((long long)g * P.Og + o) * P.K + k] = acc[mo][nk][jj];
            }
}

// 64 x 64 tile of dW per wavefront for bf16 operands without a window, 64 pixels per step.  The operand rows are
// loaded the way memory likes it -- one instruction covers 8 rows x 128 contiguous bytes -- and turned into the MFMA
// layout (lane (r, s): row s, pixels 8r .. 8r+7 of a 32-pixel half) through a wavefront-private LDS tile of
// 64 rows x (128 + 16) bytes, first dy, then x through the same rows.  (With the loads in the MFMA layout an
// instruction touched 16 rows x 64 bytes, and the kernel was bound by the address pipeline: 27 -> 20 us for the
// same bytes when only the shape of the loads was changed.)  The four wavefronts of a workgroup (consecutive
// slices of the same tile) are summed through the same LDS in a fixed order: one partial per workgroup.
__global__ __launch_bounds__(64 * kWaves) void k_wgrad64(Params P) {
    constexpr int MO = 4, NK = 4, kRow = 144;
    __shared__ __align__(16) unsigned char lds[kWaves * 64 * kRow];
    static_assert(sizeof(lds) >= 2 * MO * NK * 4 * 64 * sizeof(float), "the cross-wavefront sum reuses the tiles");
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int slice = blockIdx.x * kWaves + wave;
    const bool active = slice < P.slices;  // (no early exit: every wavefront takes part in the workgroup sum below)
    const int g = blockIdx.z;
    const int ot = blockIdx.y / P.ktiles, kt = blockIdx.y - ot * P.ktiles;
    const int r = lane >> 4, s = lane & 15;
    const int lrow = lane >> 3, lseg = lane & 7;  // shape of the loads: 8 rows x 8 pieces of 16 bytes
    const int src_elems = P.N * P.G * P.R * P.P, dy_elems = P.N * P.G * P.Og * P.P;
    const rsrc_t rs = make_rsrc(P.src, src_elems * 2);
    const rsrc_t rdy = make_rsrc(P.dy, dy_elems * 2);
    const int obase = ot * 64, kbase = kt * 64;
    unsigned char* mine = lds + wave * 64 * kRow;

    float4_t acc[MO][NK];
#pragma unroll
    for (int mo = 0; mo < MO; mo++)
#pragma unroll
        for (int nk = 0; nk < NK; nk++) acc[mo][nk] = float4_t{0.f, 0.f, 0.f, 0.f};

    // steps of 64 pixels: P.chunks32 counts them here
    const int c_begin = active ? slice * P.per_slice : 0, c_end = active ? min(P.N * P.chunks32, c_begin + P.per_slice) : 0;
    int n = (int)div_magic((uint32_t)c_begin, P.magicC32);
    int pc = c_begin - n * P.chunks32;
    for (int c = c_begin; c < c_end; c++) {
        const int px0 = pc * 64;
        const int row0 = (n * P.G + g) * P.R, orow0 = (n * P.G + g) * P.Og;
        const bool near_ends = (row0 + P.R - 1) * P.P + px0 + 72 > src_elems || (orow0 + P.Og - 1) * P.P + px0 + 72 > dy_elems;
        const int pl = px0 + lseg * 8;
        u32x4 ra[8], rb[8];
#pragma unroll
        for (int k = 0; k < 8; k++) {
            const int o = obase + 8 * k + lrow;
            ra[k] = load8<false>(rdy, (orow0 + o) * P.P + pl, pl < P.P && o < P.Og, near_ends, dy_elems * 2).hi;
        }
#pragma unroll
        for (int k = 0; k < 8; k++) {
            const int kr = kbase + 8 * k + lrow;
            rb[k] = load8<false>(rs, (row0 + kr) * P.P + pl, pl < P.P && kr < P.K, near_ends, src_elems * 2).hi;
        }
        u32x4 a[2][MO], b[2][NK];
#pragma unroll
        for (int k = 0; k < 8; k++) *reinterpret_cast<u32x4*>(mine + (8 * k + lrow) * kRow + lseg * 16) = ra[k];
#pragma unroll
        for (int h = 0; h < 2; h++) {
            // (a 16-byte piece that begins inside the plane may run past its end into the next row: masked here, on dy)
            const int nvalid = max(0, min(8, P.P - (px0 + h * 32 + 8 * r)));
            const u32x4 mvalid = mask_of((1u << nvalid) - 1u);
#pragma unroll
            for (int mo = 0; mo < MO; mo++)
                a[h][mo] = *reinterpret_cast<const u32x4*>(mine + (mo * 16 + s) * kRow + h * 64 + r * 16) & mvalid;
        }
#pragma unroll
        for (int k = 0; k < 8; k++) *reinterpret_cast<u32x4*>(mine + (8 * k + lrow) * kRow + lseg * 16) = rb[k];
#pragma unroll
        for (int h = 0; h < 2; h++)
#pragma unroll
            for (int nk = 0; nk < NK; nk++) b[h][nk] = *reinterpret_cast<const u32x4*>(mine + (nk * 16 + s) * kRow + h * 64 + r * 16);
#pragma unroll
        for (int h = 0; h < 2; h++) {
            if (h == 1 && px0 + 32 >= P.P) continue;  // (wave-uniform: the plane ends in the first half)
#pragma unroll
            for (int mo = 0; mo < MO; mo++)
#pragma unroll
                for (int nk = 0; nk < NK; nk++) {
                    float4_t t = acc[mo][nk];
                    t = mfma32(a[h][mo], b[h][nk], t);
                    acc[mo][nk] = t;
                }
        }
        if (++pc == P.chunks32) { pc = 0; n++; }
    }
    // sum of the four wavefronts in a fixed order, (w0 + w2) + (w1 + w3)
    __syncthreads();  // every wavefront has left its tile
    float (*red)[MO * NK * 4][64] = reinterpret_cast<float (*)[MO * NK * 4][64]>(lds);
    auto put = [&](int slot) {
#pragma unroll
        for (int mo = 0; mo < MO; mo++)
#pragma unroll
            for (int nk = 0; nk < NK; nk++)
#pragma unroll
                for (int jj = 0; jj < 4; jj++) red[slot][(mo * NK + nk) * 4 + jj][lane] = acc[mo][nk][jj];
    };
    auto add = [&](int slot) {
#pragma unroll
        for (int mo = 0; mo < MO; mo++)
#pragma unroll
            for (int nk = 0; nk < NK; nk++)
#pragma unroll
                for (int jj = 0; jj < 4; jj++) acc[mo][nk][jj] += red[slot][(mo * NK + nk) * 4 + jj][lane];
    };
    if (wave >= 2) put(wave - 2);
    __syncthreads();
    if (wave < 2) add(wave);
    __syncthreads();
    if (wave == 1) put(0);
    __syncthreads();
    if (wave != 0) return;
    add(0);
    float* part = P.partial + (long long)blockIdx.x * P.G * P.Og * P.K;
#pragma unroll
    for (int mo = 0; mo < MO; mo++)
#pragma unroll
        for (int nk = 0; nk < NK; nk++)
#pragma unroll
            for (int jj = 0; jj < 4; jj++) {
                const int o = obase + mo * 16 + 4 * r + jj, k = kbase + nk * 16 + s;
                if (o < P.Og && k < P.K) part[((long long)g * P.Og + o) * P.K + k] = acc[mo][nk][jj];
            }
}

__global__ void k_transpose_weights(const uint16_t* __restrict__ w, uint16_t* __restrict__ wt, int G, int Og, int R, int TV) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long total = (long long)G * R * Og * TV;
    if (i >= total) return;
    const int tv = (int)(i % TV);
    long long q = i / TV;
    const int o = (int)(q % Og);
    q /= Og;
    const int row = (int)(q % R), g = (int)(q / R);
    wt[i] = w[((long long)(g * Og + o) * R + row) * TV + (TV - 1 - tv)];
}

template <int MO>
void launch_fwd(const Params& P, hipStream_t s) {
    const int tiles = (P.N * P.upi + 15) / 16;
    const dim3 grid((unsigned)((tiles + kWaves - 1) / kWaves), (unsigned)(P.G * P.otiles));
    const dim3 block(64 * kWaves);
    const bool taps = P.TV > 1;
#define GFC_FWD(SF, DF, TP) CANVAS_LAUNCH((k_fwd<MO, SF, DF, TP>), grid, block, 0, s, P)
    if (P.src_f32) {
        if (P.dst_f32) { if (taps) GFC_FWD(true, true, true); else GFC_FWD(true, true, false); }
        else { if (taps) GFC_FWD(true, false, true); else GFC_FWD(true, false, false); }
    } else {
        if (P.dst_f32) { if (taps) GFC_FWD(false, true, true); else GFC_FWD(false, true, false); }
        else { if (taps) GFC_FWD(false, false, true); else GFC_FWD(false, false, false); }
    }
#undef GFC_FWD
}

}  // namespace

int choose_mo(int Og) { return Og <= 16 ? 1 : (Og <= 32 ? 2 : 4); }

Params shape(int N, int G, int rows, int KH, int KW, int Og, int H, int W) {
    Params Q;
    Q.N = N;
    Q.G = G;
    Q.R = rows;
    Q.KH = KH;
    Q.KW = KW;
    Q.TV = KH * KW;
    Q.K = rows * Q.TV;
    Q.Og = Og;
    Q.H = H;
    Q.W = W;
    Q.P = H * W;
    Q.upi = (Q.P + 7) / 8;
    Q.magicUpi = magic_u32(Q.upi);
    Q.magicW = magic_u32(W);
    Q.magicTV = magic_u32(Q.TV);
    Q.magicKW = magic_u32(Q.KW);
    return Q;
}

void prepare_forward(Params& P) {
    const int mo = 16 * choose_mo(P.Og);
    P.otiles = (P.Og + mo - 1) / mo;
}

void prepare_wgrad(Params& P) {
    // bf16 operands without a window and at least 64 x 64 weights per group: 64 x 64 tiles (each loaded
    // register feeds four MFMAs instead of two); set src_f32 / dy_f32 before this call
    P.wtile = (!P.src_f32 && !P.dy_f32 && P.TV == 1 && P.Og >= 64 && P.K >= 64) ? 4 : 2;
    P.otiles = (P.Og + 16 * P.wtile - 1) / (16 * P.wtile);
    P.ktiles = (P.K + 16 * P.wtile - 1) / (16 * P.wtile);
    const int chunk_px = P.wtile == 4 ? 64 : 32;  // pixels per step of a wavefront
    P.chunks32 = (P.P + chunk_px - 1) / chunk_px;
    P.magicC32 = magic_u32(P.chunks32);
    const int64_t wnumel = (int64_t)P.G * P.Og * P.K;
    const int64_t tiles = (int64_t)P.G * P.otiles * P.ktiles;
    const int64_t steps = (int64_t)P.N * P.chunks32;
    // at most 2048 slices per tile and about 4 k wavefronts in all;
    // one partial per workgroup of kWaves slices, at most 8 MB of partials (16 MB measured slower: the
    // partials are written once and read once more by the sum)
    int64_t slices = std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(steps, 2048), (4096 + tiles - 1) / std::max<int64_t>(1, tiles)));
    slices = std::max<int64_t>(1, std::min<int64_t>(slices, kWaves * (((int64_t)8 << 20) / std::max<int64_t>(1, wnumel * 4))));
    const int64_t per = std::max<int64_t>(1, (steps + slices - 1) / slices);
    P.per_slice = (int)per;
    P.slices = (int)((steps + per - 1) / per);
}

Params data_gradient_of(const Params& fwd) {
    Params D = fwd;
    D.R = fwd.Og;
    D.Og = fwd.R;
    D.K = fwd.Og * fwd.TV;
    prepare_forward(D);
    return D;
}

void forward(const Params& P, hipStream_t s) {
    if (P.N * P.G * P.Og * P.P == 0 || P.K == 0) return;
    switch (choose_mo(P.Og)) {
    case 1: launch_fwd<1>(P, s); break;
    case 2: launch_fwd<2>(P, s); break;
    default: launch_fwd<4>(P, s); break;
    }
}

void wgrad_partial(const Params& P, hipStream_t s) {
    if (P.slices == 0) return;
    const dim3 grid((unsigned)((P.slices + kWaves - 1) / kWaves), (unsigned)(P.otiles * P.ktiles), (unsigned)P.G);
    const dim3 block(64 * kWaves);
    const bool taps = P.TV > 1;
#define GFC_WG(SF, DF) \
    do { if (taps) CANVAS_LAUNCH((k_wgrad<2, 2, SF, DF, true>), grid, block, 0, s, P); else CANVAS_LAUNCH((k_wgrad<2, 2, SF, DF, false>), grid, block, 0, s, P); } while (0)
    if (P.wtile == 4) {
        CANVAS_LAUNCH(k_wgrad64, grid, block, 0, s, P);
        return;
    }
    if (P.src_f32) { if (P.dy_f32) GFC_WG(true, true); else GFC_WG(true, false); }
    else { if (P.dy_f32) GFC_WG(false, true); else GFC_WG(false, false); }
#undef GFC_WG
}

int wgrad_partials(const Params& P) { return (P.slices + kWaves - 1) / kWaves; }


void transpose_weights(const uint16_t* w, uint16_t* wt, int G, int Og, int R, int TV, hipStream_t s) {
    const long long total = (long long)G * R * Og * TV;
    if (total > 0) CANVAS_LAUNCH(k_transpose_weights, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, w, wt, G, Og, R, TV);
}

}  // namespace gfc
}  // namespace canvas
