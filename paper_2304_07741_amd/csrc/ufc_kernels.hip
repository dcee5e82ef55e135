// v = x (*|+) shift(act(z)) and its adjoint, one thread per 8 consecutive pixels of one channel
// (16-byte bf16 accesses).  The shift is an address offset plus a zero mask applied AFTER the
// activation (Shift zero-fills its own output, whatever act(0) is).  Memory-bound: forward reads x, z
// and writes v; backward reads dv, x, z (dv and x at two positions, the second served by cache) and
// writes dz and dx1.
#include "ufc_kernels.hpp"

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
        float t = P.act < 0 ? z[q] : unary_apply(P.act, z[q], P.ulo, P.uhi);
        t = ((bits >> q) & 1u) ? t : 0.f;
        v[q] = P.bin ? x[q] * t : x[q] + t;
    }
    store8(rv, P.v, u.plane + u.p, v, u.nvalid);
}

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
    unpack8(load8(rz, u.plane + u.p + off, bytes), zs);
    unpack8(load8(rz, u.plane + u.p, bytes), z);
    unpack8(load8(rdv, u.plane + u.p - off, bytes), dvb);
    if (P.bin) unpack8(load8(rx, u.plane + u.p - off, bytes), xb);
#pragma unroll
    for (int q = 0; q < 8; q++) {
        float t = P.act < 0 ? zs[q] : unary_apply(P.act, zs[q], P.ulo, P.uhi);
        t = ((bits_f >> q) & 1u) ? t : 0.f;
        dx1[q] = P.bin ? dv[q] * t : dv[q];
        float g = P.bin ? dvb[q] * xb[q] : dvb[q];
        g = ((bits_b >> q) & 1u) ? g : 0.f;
        dz[q] = P.act < 0 ? g : g * unary_grad(P.act, z[q], P.ulo, P.uhi);
    }
    store8(rdx, P.dx1, u.plane + u.p, dx1, u.nvalid);
    store8(rdz, P.dz, u.plane + u.p, dz, u.nvalid);
}

}  // namespace

void mid_forward(const MidParams& P, hipStream_t s) {
    const long long total = (long long)P.N * P.C * P.upi;
    if (total > 0) CANVAS_LAUNCH(k_mid_fwd, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, P);
}

void mid_backward(const MidParams& P, hipStream_t s) {
    const long long total = (long long)P.N * P.C * P.upi;
    if (total > 0) CANVAS_LAUNCH(k_mid_bwd, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, P);
}

}  // namespace ufc
}  // namespace canvas
