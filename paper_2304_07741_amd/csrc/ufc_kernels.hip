// v = x (*|+) shift(act(z)) and its adjoint, one thread per 8 consecutive pixels of one channel
// (16-byte bf16 accesses).  The shift is an address offset plus a zero mask applied AFTER the
// activation (Shift zero-fills its own output, whatever act(0) is).  Memory-bound: forward reads x, z
// and writes v; backward reads dv, x, z (dv and x at two positions, the second served by cache) and
// writes dz and dx1.
#include "ufc_kernels.hpp"

#include <type_traits>

#include "device_util.hpp"
#include "launch.hpp"
#include "tile_util.hpp"

namespace canvas {
namespace ufc {

namespace {

using namespace canvas::tile;

__device__ __forceinline__ uint32_t div_magic(uint32_t x, uint32_t magic) { return magic ? __umulhi(x, magic) : x; }

// bit q: pixel p+q exists and its source (h+dh, w+dw) is inside the image
__device__ __forceinline__ uint32_t shift_bits(const MidParams& P, int p, int dh, int dw) {
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

__device__ __forceinline__ void unpack8(const u32x4& v, float (&f)[8]) {
#pragma unroll
    for (int k = 0; k < 4; k++) {
        f[2 * k] = lo_f32(v[k]);
        f[2 * k + 1] = hi_f32(v[k]);
    }
}

__device__ __forceinline__ u32x4 load8(rsrc_t r, int e, int bytes) {
    u32x4 v = bload16(r, e * 2);
    reload_if_partial(v, r, e * 2, bytes);
    return v;
}

__device__ __forceinline__ void store8(rsrc_t r, uint16_t* base, int e, const float (&f)[8], int nvalid) {
    if (nvalid == 8) {
        u32x4 out;
#pragma unroll
        for (int k = 0; k < 4; k++) out[k] = pack_bf16(f[2 * k], f[2 * k + 1]);
        bstore16_nt(r, e * 2, out);
    } else {
#pragma unroll
        for (int q = 0; q < 8; q++)
            if (q < nvalid) base[e + q] = (uint16_t)(pack_bf16(f[q], 0.f) & 0xffffu);
    }
}

struct Unit {
    int plane, p, dh, dw, nvalid;
    bool live;
};
__device__ __forceinline__ Unit decode(const MidParams& P) {
    Unit u;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long total = (long long)P.N * P.C * P.upi;
    u.live = idx < total;
    const uint32_t i = u.live ? (uint32_t)idx : 0u;
    const int nc = (int)div_magic(i, P.magicUpi);
    u.p = ((int)i - nc * P.upi) * 8;
    u.plane = nc * P.P;
    const int c = nc % P.C;
    u.dh = u.dw = 0;
    for (int k = 0; k < P.nslices; k++)
        if (c >= P.c0[k] && c < P.c1[k]) {
            u.dh = P.dh[k];
            u.dw = P.dw[k];
        }
    u.nvalid = min(8, P.P - u.p);
    return u;
}

// Normal CDF and density at z.  erfc by the rational-times-Gaussian approximation of Abramowitz and Stegun,
// formula 7.1.26 (absolute error of erf below 1.5e-7, far below the bf16 rounding of every tensor these
// kernels write); the Gaussian is shared with the density, so gelu and its derivative at one point cost one
// exponential and one reciprocal.  (The fp32 per-node kernels use erff.)
__device__ __forceinline__ void normal_parts(float z, float& cdf, float& pdf) {
    const float t = __builtin_amdgcn_rcpf(1.f + 0.3275911f * 0.70710678f * fabsf(z));
    const float e = __expf(-0.5f * z * z);
    const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
    const float tail = 0.5f * poly * e;  // 0.5 * erfc(|z| / sqrt 2)
    cdf = z >= 0.f ? 1.f - tail : tail;
    pdf = 0.39894228f * e;
}

// ACT: -1 none, else UnaryKind (relu 0, abs 1, gelu 2, sin 4)
template <int ACT>
__device__ __forceinline__ float act_apply(float z) {
    if constexpr (ACT == 2) {
        float cdf, pdf;
        normal_parts(z, cdf, pdf);
        return z * cdf;
    } else if constexpr (ACT < 0) {
        return z;
    } else {
        return unary_apply(ACT, z, 0.f, 0.f);
    }
}
template <int ACT>
__device__ __forceinline__ float act_grad(float z) {
    if constexpr (ACT == 2) {
        float cdf, pdf;
        normal_parts(z, cdf, pdf);
        return cdf + z * pdf;
    } else if constexpr (ACT < 0) {
        return 1.f;
    } else {
        return unary_grad(ACT, z, 0.f, 0.f);
    }
}

template <int ACT, int BIN>
__global__ __launch_bounds__(256) void k_mid_fwd(MidParams P) {
    const Unit u = decode(P);
    if (!u.live) return;
    const int bytes = P.N * P.C * P.P * 2;
    const rsrc_t rx = make_rsrc(P.x, bytes), rz = make_rsrc(P.z, bytes), rv = make_rsrc(P.v, bytes);
    const int off = u.dh * P.W + u.dw;
    const uint32_t bits = shift_bits(P, u.p, u.dh, u.dw);
    float x[8], z[8], v[8];
    unpack8(load8(rx, u.plane + u.p, bytes), x);
    unpack8(load8(rz, u.plane + u.p + off, bytes), z);
#pragma unroll
    for (int q = 0; q < 8; q++) {
        float t = act_apply<ACT>(z[q]);
        t = ((bits >> q) & 1u) ? t : 0.f;
        v[q] = BIN ? x[q] * t : x[q] + t;
    }
    store8(rv, P.v, u.plane + u.p, v, u.nvalid);
}

template <int ACT, int BIN>
__global__ __launch_bounds__(256) void k_mid_bwd(MidParams P) {
    const Unit u = decode(P);
    if (!u.live) return;
    const int bytes = P.N * P.C * P.P * 2;
    const rsrc_t rx = make_rsrc(P.x, bytes), rz = make_rsrc(P.z, bytes), rdv = make_rsrc(P.dv, bytes);
    const rsrc_t rdz = make_rsrc(P.dz, bytes), rdx = make_rsrc(P.dx1, bytes);
    const int off = u.dh * P.W + u.dw;
    const uint32_t bits_f = shift_bits(P, u.p, u.dh, u.dw);    // t_s(p) reads z(p + d)
    const uint32_t bits_b = shift_bits(P, u.p, -u.dh, -u.dw);  // dt(p) receives g(p - d)
    float dv[8], zs[8], z[8], dvb[8], xb[8], dx1[8], dz[8];
    unpack8(load8(rdv, u.plane + u.p, bytes), dv);
    unpack8(load8(rz, u.plane + u.p, bytes), z);
    if (off != 0) {  // (channels that are not shifted read every tensor once)
        unpack8(load8(rz, u.plane + u.p + off, bytes), zs);
        unpack8(load8(rdv, u.plane + u.p - off, bytes), dvb);
    }
    if (BIN) unpack8(load8(rx, u.plane + u.p - off, bytes), xb);
#pragma unroll
    for (int q = 0; q < 8; q++) {
        const float zq = z[q], zsq = off != 0 ? zs[q] : zq;
        float t, d;
        if constexpr (ACT == 2) {
            float cdf, pdf;
            normal_parts(zq, cdf, pdf);
            d = cdf + zq * pdf;
            if (off != 0) {
                float cdf_s, pdf_s;
                normal_parts(zsq, cdf_s, pdf_s);
                t = zsq * cdf_s;
            } else {
                t = zq * cdf;
            }
        } else {
            t = act_apply<ACT>(zsq);
            d = act_grad<ACT>(zq);
        }
        t = ((bits_f >> q) & 1u) ? t : 0.f;
        dx1[q] = BIN ? dv[q] * t : dv[q];
        const float dvq = off != 0 ? dvb[q] : dv[q];
        float g = BIN ? dvq * xb[q] : dvq;
        g = ((bits_b >> q) & 1u) ? g : 0.f;
        dz[q] = g * d;
    }
    store8(rdx, P.dx1, u.plane + u.p, dx1, u.nvalid);
    store8(rdz, P.dz, u.plane + u.p, dz, u.nvalid);
}

template <typename F>
void by_act(int act, F f) {
    switch (act) {
    case 0: f(std::integral_constant<int, 0>()); break;
    case 1: f(std::integral_constant<int, 1>()); break;
    case 2: f(std::integral_constant<int, 2>()); break;
    case 4: f(std::integral_constant<int, 4>()); break;
    default: f(std::integral_constant<int, -1>()); break;
    }
}

}  // namespace

void mid_forward(const MidParams& P, hipStream_t s) {
    const long long total = (long long)P.N * P.C * P.upi;
    if (total <= 0) return;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (P.bin) by_act(P.act, [&](auto a) { CANVAS_LAUNCH((k_mid_fwd<decltype(a)::value, 1>), grid, block, 0, s, P); });
    else by_act(P.act, [&](auto a) { CANVAS_LAUNCH((k_mid_fwd<decltype(a)::value, 0>), grid, block, 0, s, P); });
}

void mid_backward(const MidParams& P, hipStream_t s) {
    const long long total = (long long)P.N * P.C * P.upi;
    if (total <= 0) return;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (P.bin) by_act(P.act, [&](auto a) { CANVAS_LAUNCH((k_mid_bwd<decltype(a)::value, 1>), grid, block, 0, s, P); });
    else by_act(P.act, [&](auto a) { CANVAS_LAUNCH((k_mid_bwd<decltype(a)::value, 0>), grid, block, 0, s, P); });
}

}  // namespace ufc
}  // namespace canvas
