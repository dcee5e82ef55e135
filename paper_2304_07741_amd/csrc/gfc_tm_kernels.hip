// Tap-major grouped FC on bf16 MFMA (see gfc_tm_kernels.hpp for the packed weight layout).
//
// Forward / data gradient, one wavefront = 16*MO outputs of one merged group x 16 units of 8 consecutive
// pixels (units numbered across the batch).  Lane (r = lane / 16, s = lane % 16) owns unit s and the
// rows 4r..4r+3 of each 16-row chunk.  For one (row chunk, window row kh) it loads, per row, the 8 pixels
// of its unit at vertical offset (kh - KH/2) * W plus two pixels on either side; the MFMA operand of
// source pixel i is assembled from the halves of the four rows' registers with two byte-permutes (the
// contraction index must sit in the lane, NCHW keeps pixels contiguous instead), and the tap (kh, kw)
// uses operand q + kw - KW/2 for output pixel q: the horizontal taps share loads and gathers.
// Zero padding of the window: a vertical mask on the loaded registers (skipped when no lane of the
// wavefront needs it) and a per-(pixel, kw) horizontal mask on the operand.
// Loads of the next (chunk, kh) group are in flight while the current one is multiplied.
#include "gfc_tm_kernels.hpp"

#include <algorithm>

#include <hip/hip_runtime.h>

#include "launch.hpp"
#include "tile_util.hpp"

namespace canvas {
namespace gfctm {

namespace {

using namespace canvas::tile;

constexpr int kWaves = 4;

__device__ __forceinline__ uint32_t div_magic(uint32_t x, uint32_t magic) { return magic ? __umulhi(x, magic) : x; }

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int MO, int KW>
struct Group {
    uint32_t d[4][KW > 1 ? 6 : 4];  // per row: [pixels -2,-1] pixels 0..7 [pixels 8,9]
    short4_t a[KW][MO];             // weights of the KW taps of this window row
};

template <int MO, int KH, int KW, bool DST_F32>
__global__ __launch_bounds__(64 * kWaves) void k_fwd(Params P) {
    constexpr int TV = KH * KW, HW = KW / 2, HH = KH / 2;
    constexpr bool HALO = KW > 1;
    constexpr int ND = HALO ? 6 : 4;   // dwords per row
    constexpr int E0 = HALO ? 2 : 0;   // index of pixel 0 in the row's element array
    static_assert(HW <= 2, "halo of two pixels");
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tile = blockIdx.x * kWaves + wave;
    const int total_units = P.N * P.upi;
    if (tile * 16 >= total_units) return;
    const int gmi = blockIdx.y / P.otiles, ot = blockIdx.y - gmi * P.otiles;
    const int gcount = min(P.gm, P.G - gmi * P.gm);
    const int Rm = gcount * P.R, Om = gcount * P.Og;
    const int r = lane >> 4, s = lane & 15;
    const int U = tile * 16 + s;
    const bool live = U < total_units;
    const int n = live ? (int)div_magic((uint32_t)U, P.magicUpi) : 0;
    const int p = live ? (U - n * P.upi) * 8 : 0;
    const int rows_img = P.G * P.R;
    const int src_elems = P.N * rows_img * P.P;
    const rsrc_t rs = make_rsrc(P.src, src_elems * 2);
    const rsrc_t rw = make_rsrc(P.wp, P.Gm * P.Omp * TV * P.Rp * 2);
    const int grow0 = gmi * P.gm * P.R;                      // first row of the merged group within an image
    const int ebase = (n * rows_img + grow0 + 4 * r) * P.P + p;  // element (row 4r, pixel p) of this lane
    const int wbase = ((gmi * P.Omp + ot * 16 * MO + s) * TV * P.Rp + 4 * r) * 2;
    const int nrc = P.Rp >> 4;
    const bool padrows = (Rm & 15) != 0;

    // wave-uniform: could a multi-byte access of this tile straddle an end of the source tensor?  (the
    // hardware drops such an access as a whole, so those tiles read element by element)
    const int n_first = (int)div_magic((uint32_t)(tile * 16), P.magicUpi);
    const int n_last = (int)div_magic((uint32_t)min(tile * 16 + 15, total_units - 1), P.magicUpi);
    const int maxoff = HH * P.W + 2;
    const bool near_ends = (n_first * rows_img + grow0) * P.P - maxoff < 0 ||
                           (n_last * rows_img + grow0 + P.Rp) * P.P + 16 + maxoff > src_elems;

    // vertical validity of the source pixels -2..9 of this lane's unit, per window row; horizontal
    // validity of the output pixels 0..7, per window column
    uint32_t rm[KH][ND];
    bool needrow[KH];
#pragma unroll
    for (int kh = 0; kh < KH; kh++) {
        bool any = false;
#pragma unroll
        for (int k = 0; k < ND; k++) {
            const int i = 2 * k - E0;
            const bool lo = (unsigned)(p + i + (kh - HH) * P.W) < (unsigned)P.P;
            const bool hi = (unsigned)(p + i + 1 + (kh - HH) * P.W) < (unsigned)P.P;
            rm[kh][k] = (lo ? 0x0000ffffu : 0u) | (hi ? 0xffff0000u : 0u);
            any = any || !lo || !hi;
        }
        needrow[kh] = kh != HH && __builtin_amdgcn_ballot_w64(any) != 0;
    }
    uint32_t cm[8][KW];
    {
        const int h0 = (int)div_magic((uint32_t)p, P.magicW);
        int c = p - h0 * P.W;
#pragma unroll
        for (int q = 0; q < 8; q++) {
#pragma unroll
            for (int kw = 0; kw < KW; kw++) cm[q][kw] = (unsigned)(c + kw - HW) < (unsigned)P.W ? 0xffffffffu : 0u;
            if (++c == P.W) c = 0;
        }
    }

    float4_t acc[MO][8];
#pragma unroll
    for (int mo = 0; mo < MO; mo++)
#pragma unroll
        for (int q = 0; q < 8; q++) acc[mo][q] = float4_t{0.f, 0.f, 0.f, 0.f};

    // `valid` false (one group past the end): the loads touch no memory; every buffer is rewritten
    // unconditionally so that no stale value has to stay live
    auto issue = [&](int rc, int kh, bool valid, Group<MO, KW>& b) {
        const int eoff = rc * 16 * P.P + (kh - HH) * P.W;
        const int rcw = min(rc, nrc - 1);
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int e = ebase + eoff + j * P.P;
            const bool ok = valid && (!padrows || rc * 16 + 4 * r + j < Rm);
            if (!near_ends) {
                const u32x4 m = bload16(rs, ok ? e * 2 : kOob);
#pragma unroll
                for (int k = 0; k < 4; k++) b.d[j][k + E0 / 2] = m[k];
                if constexpr (HALO) {
                    b.d[j][0] = __builtin_amdgcn_raw_buffer_load_b32(rs, ok ? (e - 2) * 2 : kOob, 0, 0);
                    b.d[j][5] = __builtin_amdgcn_raw_buffer_load_b32(rs, ok ? (e + 8) * 2 : kOob, 0, 0);
                }
            } else {
#pragma unroll
                for (int k = 0; k < ND; k++) {
                    const int i = 2 * k - E0;
                    const uint32_t lo = __builtin_amdgcn_raw_buffer_load_b16(rs, ok ? (e + i) * 2 : kOob, 0, 0);
                    const uint32_t hi = __builtin_amdgcn_raw_buffer_load_b16(rs, ok ? (e + i + 1) * 2 : kOob, 0, 0);
                    b.d[j][k] = (lo & 0xffffu) | (hi << 16);
                }
            }
        }
#pragma unroll
        for (int kw = 0; kw < KW; kw++)
#pragma unroll
            for (int mo = 0; mo < MO; mo++) {
                const auto t = __builtin_amdgcn_raw_buffer_load_b64(rw, wbase, ((mo * 16 * TV + kh * KW + kw) * P.Rp + rcw * 16) * 2, 0);
                b.a[kw][mo] = as_short4(t[0], t[1]);
            }
    };

    auto consume = [&](int kh, Group<MO, KW>& b) {
        if (needrow[kh]) {
#pragma unroll
            for (int j = 0; j < 4; j++)
#pragma unroll
                for (int k = 0; k < ND; k++) b.d[j][k] &= rm[kh][k];
        }
        // operand of source pixel i = t - E0: rows 4r..4r+3 of that pixel
        u32x2 op[2 * ND];
#pragma unroll
        for (int t = E0 - HW; t < E0 + 8 + HW; t++) {
            const uint32_t sel = (t & 1) ? 0x07060302u : 0x05040100u;
            op[t][0] = __builtin_amdgcn_perm(b.d[1][t >> 1], b.d[0][t >> 1], sel);
            op[t][1] = __builtin_amdgcn_perm(b.d[3][t >> 1], b.d[2][t >> 1], sel);
        }
#pragma unroll
        for (int kw = 0; kw < KW; kw++)
#pragma unroll
            for (int q = 0; q < 8; q++) {
                u32x2 o = op[q + kw - HW + E0];
                if (kw != HW) {
                    o[0] &= cm[q][kw];
                    o[1] &= cm[q][kw];
                }
                const short4_t bq = as_short4(o[0], o[1]);
#pragma unroll
                for (int mo = 0; mo < MO; mo++) acc[mo][q] = mfma16(b.a[kw][mo], bq, acc[mo][q]);
            }
    };

    // groups g = (row chunk, kh); each statically unrolled slot owns one buffer, the next group's loads
    // are issued before the current group is multiplied
    constexpr int UNR = KH > 1 ? KH : 2;
    Group<MO, KW> buf[UNR];
    const int NG = nrc * KH;
    issue(0, 0, true, buf[0]);
    for (int it = 0; it * UNR < NG; it++) {
#pragma unroll
        for (int u = 0; u < UNR; u++) {
            const int g = it * UNR + u;
            if (KH > 1 || g < NG) {
                const int khn = KH > 1 ? (u + 1) % KH : 0;
                const int rcn = KH > 1 ? (u + 1 == KH ? it + 1 : it) : g + 1;
                issue(rcn, khn, g + 1 < NG, buf[(u + 1) % UNR]);
                __builtin_amdgcn_sched_barrier(0);
                consume(KH > 1 ? u : 0, buf[u]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    if (!live) return;
    const int nvalid = min(8, P.P - p);
    const int outs_img = P.G * P.Og;
    const int dst_elems = P.N * outs_img * P.P;
    const rsrc_t rd = make_rsrc(P.dst, dst_elems * (DST_F32 ? 4 : 2));
#pragma unroll
    for (int mo = 0; mo < MO; mo++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int o = ot * 16 * MO + mo * 16 + 4 * r + j;
            if (o >= Om) continue;
            const int e = (n * outs_img + gmi * P.gm * P.Og + o) * P.P + p;
            float v[8];
#pragma unroll
            for (int q = 0; q < 8; q++) v[q] = acc[mo][q][j];
            if (nvalid == 8) {
                if (DST_F32) {
                    u32x4 lo, hi;
                    if (P.acc) {
                        lo = bload16(rd, e * 4);
                        hi = bload16(rd, e * 4 + 16);
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
                        const u32x4 ad = bload16(make_rsrc(P.addend, dst_elems * 2), e * 2);
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

// wp[gmi][op][tap][rp]: block-diagonal over the gm merged groups, zero in the padding
__global__ void k_pack_weights(const uint16_t* __restrict__ w, uint16_t* __restrict__ wp, int G, int R, int Og, int TV, int gm, int Gm,
                               int Rp, int Omp, int transposed) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long total = (long long)Gm * Omp * TV * Rp;
    if (i >= total) return;
    const int rp = (int)(i % Rp);
    long long t = i / Rp;
    const int tap = (int)(t % TV);
    t /= TV;
    const int op = (int)(t % Omp), gmi = (int)(t / Omp);
    const int sub = op / Og, o = op - sub * Og;
    const int subr = rp / R, row = rp - subr * R;
    const int g = gmi * gm + sub;
    uint16_t v = 0;
    if (sub < gm && subr == sub && g < G)
        v = transposed ? w[(((long long)g * R + row) * Og + o) * TV + (TV - 1 - tap)] : w[(((long long)g * Og + o) * R + row) * TV + tap];
    wp[i] = v;
}

// One tile per wavefront.  (Measured on MI355X: persistent wavefronts that walk over several tiles and
// issue the next tile's first loads early, with or without cache-line touches ahead, were not faster.)
template <int MO, int KH, int KW, bool DST_F32>
void launch_fwd_k(const Params& P, hipStream_t s) {
    const int tiles = (P.N * P.upi + 15) / 16;
    const int gx = (tiles + kWaves - 1) / kWaves;
    CANVAS_LAUNCH((k_fwd<MO, KH, KW, DST_F32>), dim3((unsigned)gx, (unsigned)(P.Gm * P.otiles)), dim3(64 * kWaves), 0, s, P);
}

template <int MO, bool DST_F32>
void launch_fwd(const Params& P, hipStream_t s) {
    if (P.KH == 1) launch_fwd_k<MO, 1, 1, DST_F32>(P, s);
    else if constexpr (MO <= 2) {
        if (P.KH == 3) launch_fwd_k<MO, 3, 3, DST_F32>(P, s);
        else launch_fwd_k<MO, 5, 5, DST_F32>(P, s);
    }
}

}  // namespace

bool supported(int N, int G, int R, int KH, int KW, int Og, int H, int W) {
    if (!((KH == 1 && KW == 1) || (KH == 3 && KW == 3) || (KH == 5 && KW == 5))) return false;
    if (W < 4 || N <= 0 || G <= 0 || R <= 0 || Og <= 0) return false;
    const int64_t P = (int64_t)H * W, upi = (P + 7) / 8;
    // 32-bit byte offsets; exact magic-number division of unit and pixel indices
    if (N * (int64_t)G * std::max(R, Og) * P * 4 >= ((int64_t)1 << 31)) return false;
    if (N * upi * upi >= ((int64_t)1 << 32) || P * W >= ((int64_t)1 << 32)) return false;
    const Params Q = shape(N, G, R, KH, KW, Og, H, W);
    return packed_elems(Q) * 2 < ((int64_t)1 << 31);
}

Params shape(int N, int G, int R, int KH, int KW, int Og, int H, int W) {
    Params Q;
    Q.N = N;
    Q.H = H;
    Q.W = W;
    Q.P = H * W;
    Q.upi = (Q.P + 7) / 8;
    Q.G = G;
    Q.R = R;
    Q.Og = Og;
    Q.KH = KH;
    Q.KW = KW;
    Q.TV = KH * KW;
    Q.gm = R < 16 ? std::max(1, std::min(G, 16 / R)) : 1;
    Q.Gm = (G + Q.gm - 1) / Q.gm;
    Q.Rp = (Q.gm * R + 15) / 16 * 16;
    const int Om = Q.gm * Og;
    Q.mo = Om <= 16 ? 1 : (Om <= 32 || KW > 1 ? 2 : 4);  // windows: the buffers of two groups leave room for 32 outputs
    // small problems: more, narrower wavefront tiles rather than idle SIMDs
    const int64_t tiles = ((int64_t)N * Q.upi + 15) / 16;
    while (Q.mo > 1 && tiles * Q.Gm * ((Om + 16 * Q.mo - 1) / (16 * Q.mo)) < 2048) Q.mo /= 2;
    Q.otiles = (Om + 16 * Q.mo - 1) / (16 * Q.mo);
    Q.Omp = Q.otiles * 16 * Q.mo;
    auto magic = [](uint32_t d) { return d <= 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) + d - 1) / d); };
    Q.magicW = magic((uint32_t)W);
    Q.magicUpi = magic((uint32_t)Q.upi);
    return Q;
}

Params data_gradient_of(const Params& f) { return shape(f.N, f.G, f.Og, f.KH, f.KW, f.R, f.H, f.W); }

void pack_weights(const uint16_t* w, uint16_t* wp, const Params& P, bool transposed, hipStream_t s) {
    const long long total = packed_elems(P);
    if (total > 0)
        CANVAS_LAUNCH(k_pack_weights, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, w, wp, P.G, P.R, P.Og, P.TV, P.gm, P.Gm, P.Rp,
                      P.Omp, transposed ? 1 : 0);
}

void forward(const Params& P, hipStream_t s) {
    if ((int64_t)P.N * P.G * P.Og * P.P == 0) return;
    if (P.dst_f32) {
        switch (P.mo) {
        case 1: launch_fwd<1, true>(P, s); break;
        case 2: launch_fwd<2, true>(P, s); break;
        default: launch_fwd<4, true>(P, s); break;
        }
    } else {
        switch (P.mo) {
        case 1: launch_fwd<1, false>(P, s); break;
        case 2: launch_fwd<2, false>(P, s); break;
        default: launch_fwd<4, false>(P, s); break;
        }
    }
}

}  // namespace gfctm
}  // namespace canvas
