// One thread owns 8 consecutive pixels (a 16-byte bf16 access).  Window rows are read as the 8 pixels plus
// two on either side; a tap is used only where its source pixel lies inside the image (a select, so what
// the out-of-image positions hold never matters).  All three kernels are memory/latency-bound
// element-wise passes; the channel sum of the gradient of a is a fixed-order butterfly over 16 lanes.
#include "dyn_kernels.hpp"

#include "launch.hpp"
#include "tile_util.hpp"

namespace canvas {
namespace dyn {

namespace {

using namespace canvas::tile;

__device__ __forceinline__ uint32_t div_magic(uint32_t x, uint32_t magic) { return magic ? __umulhi(x, magic) : x; }

// elements e-2 .. e+9 of a bf16 buffer of `total` elements, as floats (0 where outside the buffer).  The two
// elements on either side of the lane's own 8 are loaded as two more 4-byte accesses (NB = 0), or, where the
// lanes 16 below / above hold the adjacent units (NB = 16), taken from their registers, and only the first and
// last quarter of the wavefront load them.  Where a neighbour holds another plane the pixels concerned lie
// outside the image and are never selected by the caller.
template <int NB>
__device__ __forceinline__ void load12(rsrc_t r, int e, int total, float (&f)[12]) {
    uint32_t d[6];
    const int lane = threadIdx.x & 63;
    const bool first = lane < 16, last = lane >= 48;
    const bool inside = e - 2 >= 0 && e + 10 <= total;
    uint32_t edge = 0;
    if (inside) {
        const u32x4 m = bload16(r, e * 2);
        if constexpr (NB == 0) {
            d[0] = __builtin_amdgcn_raw_buffer_load_b32(r, (e - 2) * 2, 0, 0);
            d[5] = __builtin_amdgcn_raw_buffer_load_b32(r, (e + 8) * 2, 0, 0);
        } else {
            edge = __builtin_amdgcn_raw_buffer_load_b32(r, first ? (e - 2) * 2 : (last ? (e + 8) * 2 : kOob), 0, 0);
        }
#pragma unroll
        for (int k = 0; k < 4; k++) d[k + 1] = m[k];
    } else {  // at an end of the tensor: a multi-byte access that straddles the end would be dropped as a whole
#pragma unroll
        for (int k = 0; k < 6; k++) {
            const int i = e - 2 + 2 * k;
            const uint32_t lo = (unsigned)i < (unsigned)total ? (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r, i * 2, 0, 0) : 0u;
            const uint32_t hi = (unsigned)(i + 1) < (unsigned)total ? (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r, (i + 1) * 2, 0, 0) : 0u;
            d[k] = (lo & 0xffffu) | (hi << 16);
        }
    }
    if constexpr (NB == 16) {
        // the last dword of the lane 16 below, the first dword of the lane 16 above
        uint32_t below = (uint32_t)__builtin_amdgcn_ds_bpermute(((lane + 48) & 63) * 4, (int)d[4]);
        uint32_t above = (uint32_t)__builtin_amdgcn_ds_bpermute(((lane + 16) & 63) * 4, (int)d[1]);
        below = first ? edge : below;
        above = last ? edge : above;
        if (inside) {
            d[0] = below;
            d[5] = above;
        }
    }
#pragma unroll
    for (int k = 0; k < 6; k++) {
        f[2 * k] = lo_f32(d[k]);
        f[2 * k + 1] = hi_f32(d[k]);
    }
}
// elements e .. e+7 of an fp32 buffer
__device__ __forceinline__ void load8f(rsrc_t r, int e, int total, float (&f)[8]) {
    if (e >= 0 && e + 8 <= total) {
        const u32x4 a = bload16(r, e * 4), b = bload16(r, e * 4 + 16);
#pragma unroll
        for (int k = 0; k < 4; k++) {
            f[k] = __uint_as_float(a[k]);
            f[4 + k] = __uint_as_float(b[k]);
        }
    } else {
#pragma unroll
        for (int k = 0; k < 8; k++)
            f[k] = (unsigned)(e + k) < (unsigned)total ? __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (e + k) * 4, 0, 0)) : 0.f;
    }
}
__device__ __forceinline__ void store8_bf16(rsrc_t r, uint16_t* base, int e, const float (&f)[8], int nvalid) {
    if (nvalid == 8) {
        u32x4 out;
#pragma unroll
        for (int k = 0; k < 4; k++) out[k] = pack_bf16(f[2 * k], f[2 * k + 1]);
        bstore16(r, e * 2, out);
    } else {
#pragma unroll
        for (int q = 0; q < 8; q++)
            if (q < nvalid) base[e + q] = (uint16_t)(pack_bf16(f[q], 0.f) & 0xffffu);
    }
}

struct Pix {
    int h[8], w[8];
};
__device__ __forceinline__ Pix pixels(const Params& P, int p) {
    Pix g;
    int h = (int)div_magic((uint32_t)p, P.magicW), c = p - h * P.W;
#pragma unroll
    for (int q = 0; q < 8; q++) {
        g.h[q] = h;
        g.w[q] = c;
        if (++c == P.W) { c = 0; h++; }
    }
    return g;
}

// One thread: 8 pixels of CPT consecutive channels of one image.  The window weights a (fp32, read by every
// channel of the image) are loaded once per tap and used for the CPT channels: with one channel per thread
// the re-reads of a from L2 set the time of these kernels.
template <int KH, int KW, int CPT>
__global__ __launch_bounds__(256) void k_fwd(Params P) {
    constexpr int HH = KH / 2, HW = KW / 2, TV = KH * KW;
    const int CG = (P.C + CPT - 1) / CPT;
    unsigned bx, by;
    xcd_order(bx, by);  // (neighbouring blocks read overlapping window rows)
    const long long idx = (long long)bx * 256 + threadIdx.x;
    if (idx >= (long long)P.N * CG * P.upi) return;
    const int ng = (int)div_magic((uint32_t)idx, P.magicUpi);
    const int p = ((int)idx - ng * P.upi) * 8;
    const int n = ng / CG, c0 = (ng - n * CG) * CPT;
    const int xtotal = P.N * P.C * P.P, atotal = P.N * TV * P.P;
    const rsrc_t rx = make_rsrc(P.x, xtotal * 2), ra = make_rsrc(P.a, atotal * 4), ru = make_rsrc(P.u, xtotal * 2);
    const Pix g = pixels(P, p);
    float acc[CPT][8];
#pragma unroll
    for (int k = 0; k < CPT; k++)
#pragma unroll
        for (int q = 0; q < 8; q++) acc[k][q] = 0.f;
#pragma unroll 1  // one window row at a time in flight: keeps the kernel small enough for several waves per SIMD
    for (int kh = 0; kh < KH; kh++) {
        float xr[CPT][12];
#pragma unroll
        for (int k = 0; k < CPT; k++) load12<0>(rx, (n * P.C + min(c0 + k, P.C - 1)) * P.P + p + (kh - HH) * P.W, xtotal, xr[k]);
#pragma unroll
        for (int kw = 0; kw < KW; kw++) {
            float a[8];
            load8f(ra, (n * TV + kh * KW + kw) * P.P + p, atotal, a);
#pragma unroll
            for (int q = 0; q < 8; q++) {
                const bool v = (unsigned)(g.h[q] + kh - HH) < (unsigned)P.H && (unsigned)(g.w[q] + kw - HW) < (unsigned)P.W;
                const float aq = v ? a[q] : 0.f;
#pragma unroll
                for (int k = 0; k < CPT; k++) acc[k][q] += aq * xr[k][q + kw - HW + 2];
            }
        }
    }
#pragma unroll
    for (int k = 0; k < CPT; k++) {
        if (c0 + k >= P.C) break;
#pragma unroll
        for (int q = 0; q < 8; q++) acc[k][q] *= P.scale;
        store8_bf16(ru, P.u, (n * P.C + c0 + k) * P.P + p, acc[k], min(8, P.P - p));
    }
}

template <int KH, int KW, int CPT>
__device__ __forceinline__ void bwd_dx_block(const Params& P, unsigned bx) {
    constexpr int HH = KH / 2, HW = KW / 2, TV = KH * KW;
    const int CG = (P.C + CPT - 1) / CPT;
    const long long idx = (long long)bx * 256 + threadIdx.x;
    if (idx >= (long long)P.N * CG * P.upi) return;
    const int ng = (int)div_magic((uint32_t)idx, P.magicUpi);
    const int p = ((int)idx - ng * P.upi) * 8;
    const int n = ng / CG, c0 = (ng - n * CG) * CPT;
    const int xtotal = P.N * P.C * P.P, atotal = P.N * TV * P.P;
    const rsrc_t rdu = make_rsrc(P.du, xtotal * 2), ra = make_rsrc(P.a, atotal * 4), rdx = make_rsrc(P.dx, xtotal * 2);
    const Pix g = pixels(P, p);
    float acc[CPT][8];
#pragma unroll
    for (int k = 0; k < CPT; k++)
#pragma unroll
        for (int q = 0; q < 8; q++) acc[k][q] = 0.f;
#pragma unroll 1
    for (int kh = 0; kh < KH; kh++) {
        // pixel p' receives tap t from the output pixel p' - off(t): that pixel must be inside the image
        float dr[CPT][12];
#pragma unroll
        for (int k = 0; k < CPT; k++) load12<0>(rdu, (n * P.C + min(c0 + k, P.C - 1)) * P.P + p - (kh - HH) * P.W, xtotal, dr[k]);
#pragma unroll
        for (int kw = 0; kw < KW; kw++) {
            float a[8];
            load8f(ra, (n * TV + kh * KW + kw) * P.P + p - (kh - HH) * P.W - (kw - HW), atotal, a);
#pragma unroll
            for (int q = 0; q < 8; q++) {
                const bool v = (unsigned)(g.h[q] - (kh - HH)) < (unsigned)P.H && (unsigned)(g.w[q] - (kw - HW)) < (unsigned)P.W;
                const float aq = v ? a[q] : 0.f;
#pragma unroll
                for (int k = 0; k < CPT; k++) acc[k][q] += aq * dr[k][q - (kw - HW) + 2];
            }
        }
    }
#pragma unroll
    for (int k = 0; k < CPT; k++) {
        if (c0 + k >= P.C) break;
#pragma unroll
        for (int q = 0; q < 8; q++) acc[k][q] *= P.scale;
        store8_bf16(rdx, P.dx, (n * P.C + c0 + k) * P.P + p, acc[k], min(8, P.P - p));
    }
}

// block = 16 units x 16 channel slices (lane % 16 = slice: channels slice, slice + 16, ...) of one window row
template <int KH, int KW>
__device__ __forceinline__ void bwd_da_block(const Params& P, unsigned bx, unsigned kh_of_block) {
    constexpr int HH = KH / 2, HW = KW / 2, TV = KH * KW;
    const int cs = threadIdx.x & 15;
    const long long U = (long long)bx * 16 + (threadIdx.x >> 4);
    const bool live = U < (long long)P.N * P.upi;
    const int n = live ? (int)div_magic((uint32_t)U, P.magicUpi) : 0;
    const int p = live ? ((int)U - n * P.upi) * 8 : 0;
    const int xtotal = P.N * P.C * P.P, atotal = P.N * TV * P.P;
    const rsrc_t rdu = make_rsrc(P.du, xtotal * 2), rx = make_rsrc(P.x, xtotal * 2);
    const Pix g = pixels(P, p);
    const int nvalid = min(8, P.P - p);
    {
        const int kh = (int)kh_of_block;  // one window row per block: KH times the parallelism, the rows are independent
        float acc[KW][8];
#pragma unroll
        for (int kw = 0; kw < KW; kw++)
#pragma unroll
            for (int q = 0; q < 8; q++) acc[kw][q] = 0.f;
        for (int c = cs; c < P.C; c += 16) {
            const int plane = (n * P.C + c) * P.P;
            float d[12], xr[12];
            load12<16>(rdu, plane + p, xtotal, d);
            load12<16>(rx, plane + p + (kh - HH) * P.W, xtotal, xr);
#pragma unroll
            for (int kw = 0; kw < KW; kw++)
#pragma unroll
                for (int q = 0; q < 8; q++) {
                    const bool v = (unsigned)(g.h[q] + kh - HH) < (unsigned)P.H && (unsigned)(g.w[q] + kw - HW) < (unsigned)P.W;
                    acc[kw][q] += v ? d[q + 2] * xr[q + kw - HW + 2] : 0.f;
                }
        }
        // sum over the 16 slices: butterfly with a fixed pairing, every lane ends with the total
#pragma unroll
        for (int kw = 0; kw < KW; kw++)
#pragma unroll
            for (int q = 0; q < 8; q++) {
                float v = acc[kw][q];
#pragma unroll
                for (int m = 1; m < 16; m <<= 1) v += __shfl_xor(v, m, 16);
                acc[kw][q] = v * P.scale;
            }
        // lane kw of the unit's 16 stores tap (kh, kw)
#pragma unroll
        for (int kw = 0; kw < KW; kw++)
            if (live && cs == kw) {
                const int e = (n * TV + kh * KW + kw) * P.P + p;
                if (nvalid == 8) {
                    float4* out = reinterpret_cast<float4*>(P.da + e);
                    if ((e & 3) == 0) {
                        out[0] = make_float4(acc[kw][0], acc[kw][1], acc[kw][2], acc[kw][3]);
                        out[1] = make_float4(acc[kw][4], acc[kw][5], acc[kw][6], acc[kw][7]);
                    } else {
#pragma unroll
                        for (int q = 0; q < 8; q++) P.da[e + q] = acc[kw][q];
                    }
                } else {
#pragma unroll
                    for (int q = 0; q < 8; q++)
                        if (q < nvalid) P.da[e + q] = acc[kw][q];
                }
            }
    }
    (void)atotal;
}

// The two gradients of the window product in one launch: dx = dyn^T(a, du) and da = sum_c du . U read the same du and
// neither fills the chip alone.  The first da_blocks blocks of the sequence (units x window rows, the longer job) work
// on da, the rest on dx.
template <int KH, int KW, int CPT>
__global__ __launch_bounds__(256) void k_bwd_dx_da(Params P, unsigned da_blocks_x) {
    unsigned seq, unused;
    xcd_order(seq, unused);  // (neighbouring blocks read overlapping window rows)
    const unsigned da_blocks = da_blocks_x * KH;
    if (seq < da_blocks) {
        // (the KH blocks of the same units read the same du and overlapping rows of x: neighbours in the sequence)
        const unsigned units = seq / KH;
        bwd_da_block<KH, KW>(P, units, seq - units * KH);
    } else {
        bwd_dx_block<KH, KW, CPT>(P, seq - da_blocks);
    }
}

template <typename F33, typename F55>
void dispatch(const Params& P, F33 f33, F55 f55) {
    if (P.KH == 3) f33();
    else f55();
}

}  // namespace

bool supported(int KH, int KW) { return (KH == 3 && KW == 3) || (KH == 5 && KW == 5); }

// channels per thread: 4 where that still leaves a wavefront per SIMD, else 1
static int channels_per_thread(const Params& P) { return (long long)P.N * ((P.C + 3) / 4) * P.upi >= 65536 ? 4 : 1; }

void forward(const Params& P, hipStream_t s) {
    const int cpt = channels_per_thread(P);
    const long long total = (long long)P.N * ((P.C + cpt - 1) / cpt) * P.upi;
    if (total == 0) return;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (cpt == 4)
        dispatch(P, [&] { CANVAS_LAUNCH((k_fwd<3, 3, 4>), grid, block, 0, s, P); }, [&] { CANVAS_LAUNCH((k_fwd<5, 5, 4>), grid, block, 0, s, P); });
    else
        dispatch(P, [&] { CANVAS_LAUNCH((k_fwd<3, 3, 1>), grid, block, 0, s, P); }, [&] { CANVAS_LAUNCH((k_fwd<5, 5, 1>), grid, block, 0, s, P); });
}

void backward_dx_da(const Params& P, hipStream_t s) {
    const int cpt = channels_per_thread(P);
    const long long total = (long long)P.N * ((P.C + cpt - 1) / cpt) * P.upi;
    const long long units = (long long)P.N * P.upi;
    if (total == 0) return;
    const unsigned dx_blocks = (unsigned)((total + 255) / 256), da_x = (unsigned)((units + 15) / 16);
    const dim3 grid(dx_blocks + da_x * (unsigned)P.KH), block(256);
    if (cpt == 4)
        dispatch(P, [&] { CANVAS_LAUNCH((k_bwd_dx_da<3, 3, 4>), grid, block, 0, s, P, da_x); },
                 [&] { CANVAS_LAUNCH((k_bwd_dx_da<5, 5, 4>), grid, block, 0, s, P, da_x); });
    else
        dispatch(P, [&] { CANVAS_LAUNCH((k_bwd_dx_da<3, 3, 1>), grid, block, 0, s, P, da_x); },
                 [&] { CANVAS_LAUNCH((k_bwd_dx_da<5, 5, 1>), grid, block, 0, s, P, da_x); });
}

}  // namespace dyn
}  // namespace canvas
