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

template <int MO, int KW, bool WL>
struct Group {
    uint32_t d[4][KW > 1 ? 6 : 4];      // per row: [pixels -2,-1] pixels 0..7 [pixels 8,9]
    short4_t a[WL ? 1 : KW][WL ? 1 : MO];  // weights of the KW taps of this window row (WL: read from LDS when used)
};

// Dynamic LDS of k_fwd: the weight tile of the workgroup (WL) and, after the K loop, the split-K sums (KS > 1).
extern __shared__ __align__(16) unsigned char lds_dyn[];

// KS > 1: the KS wavefronts that share a tile split its row chunks (chunk c goes to wavefront c % KS) and
// their accumulators are added through LDS in a fixed order; for contractions with many channels on
// few pixels, where one wavefront per tile would leave most SIMDs idle on a long serial K loop.
// WL: the workgroup first copies its weight tile (16*MO outputs x all taps and rows of the merged group: one
// contiguous block of the packed layout) into LDS with coalesced 16-byte loads, and the MFMA A operands are
// read from there.  Read straight from memory, an A operand load touches 16 lines for 512 bytes, and those
// loads were a third of the kernel time of the many-channel shapes.  Rows are padded by 16 bytes in LDS: the
// 16 rows that one read touches then fall into different banks.
// SM (16 outputs at most, fp32 result, no window): the result is the softmax over the outputs of each pixel instead
// of the sums themselves -- the per-pixel window weights of an Involution-like kernel (Section 5 of the paper) are
// an FC followed by a softmax over its few channels, and the softmax alone was a launch as long as the FC.  One
// wavefront of the tile then collects all of its sums (they are 4 x 8 values per lane), the outputs of a pixel sit
// in the lanes 16 and 32 apart, and maximum and sum cross them by lane exchanges.
template <int MO, int KH, int KW, bool DST_F32, int KS, bool WL, bool SM = false>
__global__ __launch_bounds__(64 * kWaves) void k_fwd(Params P) {
    static_assert(!SM || (MO == 1 && KH == 1 && KW == 1 && DST_F32), "softmax epilogue: one output tile, fp32, no window");
    constexpr int TV = KH * KW, HW = KW / 2, HH = KH / 2;
    constexpr bool HALO = KW > 1;
    constexpr int ND = HALO ? 6 : 4;   // dwords per row
    constexpr int E0 = HALO ? 2 : 0;   // index of pixel 0 in the row's element array
    static_assert(HW <= 2, "halo of two pixels");
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Sequence of the workgroups: the output tiles of one pixel tile first (they read the same rows: with x fastest the
    // 1x1 FC of 512 channels fetched its input 8 times, once per output tile), then the pixel tiles (neighbours share
    // window halos), then the merged groups.
    const unsigned seq = xcd_sequence();
    const unsigned otiles_u = (unsigned)P.otiles, pt = seq / otiles_u;
    const unsigned bx = pt % gridDim.x;
    const int tile = (int)bx * (kWaves / KS) + wave / KS, ks = wave % KS;
    const int total_units = P.N * P.upi;
    const bool active = tile * 16 < total_units;
    if constexpr (KS == 1 && !WL) {
        if (!active) return;
    }
    const int gmi = (int)(pt / gridDim.x), ot = (int)(seq - pt * otiles_u);
    const int gcount = min(P.gm, P.G - gmi * P.gm);
    const int Rm = gcount * P.R, Om = gcount * P.Og;
    const int r = lane >> 4, s = lane & 15;
    const int U = tile * 16 + s;
    const bool live = active && U < total_units;
    const int n = live ? (int)div_magic((uint32_t)U, P.magicUpi) : 0;
    const int p = live ? (U - n * P.upi) * 8 : 0;
    const int rows_img = P.G * P.R;
    const int src_elems = P.N * rows_img * P.P;
    const rsrc_t rs = make_rsrc(P.src, src_elems * 2);
    const rsrc_t rw = make_rsrc(P.wp, P.Gm * P.Omp * TV * P.Rp * 2);
    const int grow0 = gmi * P.gm * P.R;                      // first row of the merged group within an image
    const int ebase = (n * rows_img + grow0 + 4 * r) * P.P + p;  // element (row 4r, pixel p) of this lane
    // the same of the first and the last lane of this lane's row of 16 (their units may lie in other images)
    const int eb_first = __builtin_amdgcn_ds_bpermute((lane & 48) * 4, ebase);
    const int eb_last = __builtin_amdgcn_ds_bpermute(((lane & 48) + 15) * 4, ebase);
    const int wbase = ((gmi * P.Omp + ot * 16 * MO + s) * TV * P.Rp + 4 * r) * 2;
    const int nrc = P.Rp >> 4;
    const bool padrows = (Rm & 15) != 0;
    const int wstride = TV * P.Rp * 2 + 16;  // bytes per output row of the tile in LDS
    if constexpr (WL) {
        const int wrow16 = TV * P.Rp / 8;    // 16-byte pieces per output row
        const int npieces = 16 * MO * wrow16;
        const int tbase = (gmi * P.Omp + ot * 16 * MO) * TV * P.Rp * 2;
        constexpr int B = 8;  // loads in flight per thread
        for (int i0 = (int)threadIdx.x; i0 < npieces; i0 += B * 64 * kWaves) {
            u32x4 v[B];
#pragma unroll
            for (int u = 0; u < B; u++) {
                const int i = i0 + u * 64 * kWaves;
                v[u] = bload16(rw, i < npieces ? tbase + i * 16 : kOob);
            }
#pragma unroll
            for (int u = 0; u < B; u++) {
                const int i = i0 + u * 64 * kWaves;
                if (i < npieces) {
                    const int row = (int)div_magic((uint32_t)i, P.magicW16);
                    *reinterpret_cast<u32x4*>(lds_dyn + row * wstride + (i - row * wrow16) * 16) = v[u];
                }
            }
        }
        __syncthreads();
        if constexpr (KS == 1) {
            if (!active) return;
        }
    }

    // wave-uniform: could a multi-byte access of this tile straddle an end of the source tensor?  (the
    // hardware drops such an access as a whole; the lanes concerned re-read element by element)
    const int n_first = (int)div_magic((uint32_t)min(tile * 16, total_units - 1), P.magicUpi);
    const int n_last = (int)div_magic((uint32_t)min(tile * 16 + 15, total_units - 1), P.magicUpi);
    const int maxoff = HH * P.W + 2;
    const bool near_ends = (n_first * rows_img + grow0) * P.P - maxoff < 0 ||
                           (n_last * rows_img + grow0 + P.Rp) * P.P + 16 + maxoff > src_elems;

    // vertical validity of the source pixels -2..9 of this lane's unit, per window row (below); horizontal
    // validity of the output pixels 0..7, per window column
    // (rows: only whether any lane of the wavefront needs a mask is kept; the masks themselves are built where they
    // are applied, in the few tiles that touch the first or last image rows)
    bool needrow[KH];
#pragma unroll
    for (int kh = 0; kh < KH; kh++) {
        const int dk = (kh - HH) * P.W;
        const bool any = p - E0 + dk < 0 || p + 2 * ND - E0 - 1 + dk >= P.P;
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

    // `valid` false (one group past the end): the loads touch no memory; with a window every buffer is
    // rewritten unconditionally so that no stale value has to stay live
    auto issue = [&](int rc, int kh, bool valid, Group<MO, KW, WL>& b) {
        if (KH == 1 && !valid) return;  // (wave-uniform; with a window the unconditional form measured faster)
        const int eoff = rc * 16 * P.P + (kh - HH) * P.W;
        const int rcw = min(rc, nrc - 1);
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int e = ebase + eoff + j * P.P;
            const bool ok = valid && (!padrows || rc * 16 + 4 * r + j < Rm);
            const int bo = ok ? e * 2 : kOob;
            u32x4 m = bload16(rs, bo);
            if (near_ends) reload_if_partial(m, rs, bo, src_elems * 2);  // only lanes whose access is partly outside re-read
#pragma unroll
            for (int k = 0; k < 4; k++) b.d[j][k + E0 / 2] = m[k];
        }
        if constexpr (HALO) {
            // The two pixels on either side of a unit are the neighbouring lanes' registers (units are consecutive
            // pixels) and are fetched by a lane shift when the group is consumed; only the first and the last
            // lane of a row of 16 have no such neighbour.  Their 2 x 4 values (left / right edge of the rows
            // 4r .. 4r+3) are loaded by ONE instruction: lane s = j loads the left edge of row j, lane s = 8 + j
            // the right edge, and the group's consumer hands them to lanes 0 and 15.
            const int jl = s & 3;
            const bool okl = valid && (!padrows || rc * 16 + 4 * r + jl < Rm);
            const int el = (s < 4 ? eb_first - E0 : eb_last + 8) + eoff + jl * P.P;
            const int eo = okl && (s < 4 || (s >= 8 && s < 12)) ? el * 2 : kOob;
            uint32_t edge = __builtin_amdgcn_raw_buffer_load_b32(rs, eo, 0, 0);
            if (near_ends) reload_pair_if_partial(edge, rs, eo, src_elems * 2);
            b.d[0][0] = edge;
        }
        if constexpr (!WL) {
#pragma unroll
            for (int kw = 0; kw < KW; kw++)
#pragma unroll
                for (int mo = 0; mo < MO; mo++) {
                    const auto t = __builtin_amdgcn_raw_buffer_load_b64(rw, wbase, ((mo * 16 * TV + kh * KW + kw) * P.Rp + rcw * 16) * 2, 0);
                    b.a[kw][mo] = as_short4(t[0], t[1]);
                }
        }
    };

    struct Pending {
        short4_t wa[MO];
        short4_t b[8];
    } pend;
    auto consume = [&](int rc, int kh, Group<MO, KW, WL>& b, int phase) {
        short4_t wa[KW][MO];  // A operands: outputs 16 * mo + s, rows 4r .. 4r+3 of the chunk, tap (kh, kw)
#pragma unroll
        for (int kw = 0; kw < KW; kw++)
#pragma unroll
            for (int mo = 0; mo < MO; mo++) {
                if constexpr (WL) {
                    const u32x2 t = *reinterpret_cast<const u32x2*>(lds_dyn + (mo * 16 + s) * wstride +
                                                                     ((kh * KW + kw) * P.Rp + rc * 16 + 4 * r) * 2);
                    wa[kw][mo] = as_short4(t[0], t[1]);
                } else {
                    wa[kw][mo] = b.a[kw][mo];
                }
            }
        if constexpr (HALO) {
            // row_shr:1 / row_shl:1 within the 16 lanes of a row; a lane without a source keeps the loaded edge value
            const uint32_t loaded = b.d[0][0];
#pragma unroll
            for (int j = 0; j < 4; j++) {
                // lane 0 of the row takes the left edge of row j from lane j, lane 15 the right edge from lane 8 + j
                const uint32_t edge = (uint32_t)__builtin_amdgcn_ds_bpermute(((lane & 48) + (s == 15 ? 8 : 0) + j) * 4, (int)loaded);
                b.d[j][0] = (uint32_t)__builtin_amdgcn_update_dpp((int)edge, (int)b.d[j][4], 0x111, 0xf, 0xf, false);
                b.d[j][5] = (uint32_t)__builtin_amdgcn_update_dpp((int)edge, (int)b.d[j][1], 0x101, 0xf, 0xf, false);
            }
        }
        if (needrow[kh]) {
#pragma unroll
            for (int k = 0; k < ND; k++) {
                const int i = 2 * k - E0 + (kh - HH) * P.W;
                const bool lo = (unsigned)(p + i) < (unsigned)P.P, hi = (unsigned)(p + i + 1) < (unsigned)P.P;
                const uint32_t m = (lo ? 0x0000ffffu : 0u) | (hi ? 0xffff0000u : 0u);
#pragma unroll
                for (int j = 0; j < 4; j++) b.d[j][k] &= m;
            }
        }
        // operand of source pixel i = t - E0: rows 4r..4r+3 of that pixel
        u32x2 op[2 * ND];
#pragma unroll
        for (int t = E0 - HW; t < E0 + 8 + HW; t++) {
            const uint32_t sel = (t & 1) ? 0x07060302u : 0x05040100u;
            op[t][0] = __builtin_amdgcn_perm(b.d[1][t >> 1], b.d[0][t >> 1], sel);
            op[t][1] = __builtin_amdgcn_perm(b.d[3][t >> 1], b.d[2][t >> 1], sel);
        }
        // operand of output pixel q for window column kw (its source pixel q + kw - HW, zero where that leaves the image row)
        auto bop = [&](int q, int kw) {
            u32x2 o = op[q + kw - HW + E0];
            if (kw != HW) {
                o[0] &= cm[q][kw];
                o[1] &= cm[q][kw];
            }
            return as_short4(o[0], o[1]);
        };
        if constexpr (KW == 1) {
            // no window: two row chunks of 16 make one K = 32 step.  phase 0 keeps this chunk's operands, phase 1
            // multiplies the kept chunk and this one, phase 2 (a last chunk without a partner) multiplies alone.
            if (phase == 0) {
#pragma unroll
                for (int mo = 0; mo < MO; mo++) pend.wa[mo] = wa[0][mo];
#pragma unroll
                for (int q = 0; q < 8; q++) pend.b[q] = bop(q, 0);
            } else if (phase == 1) {
#pragma unroll
                for (int q = 0; q < 8; q++) {
                    const short4_t bq = bop(q, 0);
#pragma unroll
                    for (int mo = 0; mo < MO; mo++) acc[mo][q] = mfma32(pend.wa[mo], wa[0][mo], pend.b[q], bq, acc[mo][q]);
                }
            } else {
#pragma unroll
                for (int q = 0; q < 8; q++)
#pragma unroll
                    for (int mo = 0; mo < MO; mo++) acc[mo][q] = mfma32(wa[0][mo], short4_t{0, 0, 0, 0}, bop(q, 0), short4_t{0, 0, 0, 0}, acc[mo][q]);
            }
        } else {
            // every accumulator is complete before, and is first used after, a stretch of wait states longer than the
            // longest MFMA takes to write its result (the empty asm statements tie the accumulators to this point
            // without stopping the scheduler from moving loads across)
            auto shape_fence = [&]() {
#pragma unroll
                for (int mo = 0; mo < MO; mo++)
#pragma unroll
                    for (int q = 0; q < 8; q++) asm volatile("" : "+v"(acc[mo][q]));
                asm volatile("s_nop 15\n\ts_nop 7");
#pragma unroll
                for (int mo = 0; mo < MO; mo++)
#pragma unroll
                    for (int q = 0; q < 8; q++) asm volatile("" : "+v"(acc[mo][q]));
            };
            if constexpr (KW == 3) {
                // a 3-wide window row: columns 0 and 1 are one K = 32 step (same 16 rows, two taps), column 2 a K = 16
                // step.  An accumulator that went from one of the two MFMA shapes straight into the other came back
                // wrong (measured on gfx950 with this compiler: y of every 3 x 3 contraction off by tens of percent;
                // correct as soon as the two were apart).  So all K = 16 steps come first, then all K = 32 steps, and
                // each block is fenced (below).
                shape_fence();
#pragma unroll
                for (int q = 0; q < 8; q++) {
                    const short4_t b2 = bop(q, 2);
#pragma unroll
                    for (int mo = 0; mo < MO; mo++) acc[mo][q] = mfma16(wa[2][mo], b2, acc[mo][q]);
                }
                shape_fence();
#pragma unroll
                for (int q = 0; q < 8; q++) {
                    const short4_t b0 = bop(q, 0), b1 = bop(q, 1);
#pragma unroll
                    for (int mo = 0; mo < MO; mo++) acc[mo][q] = mfma32(wa[0][mo], wa[1][mo], b0, b1, acc[mo][q]);
                }
            } else {
                // (5 x 5: the wider operands would cost the registers that keep two wavefronts per SIMD)
#pragma unroll
                for (int q = 0; q < 8; q++)
#pragma unroll
                    for (int kw = 0; kw < KW; kw++) {
                        const short4_t bq = bop(q, kw);
#pragma unroll
                        for (int mo = 0; mo < MO; mo++) acc[mo][q] = mfma16(wa[kw][mo], bq, acc[mo][q]);
                    }
            }
        }
    };

    // Output rows of the tile as T = 4 * MO "row slots" t = 4 * mo + j (output 16 * mo + 4 * r + j of this lane, 8 pixels
    // each); this wavefront finishes the TF slots from t0 on (all of them when KS == 1, see below).
    constexpr int T = 4 * MO, TF = SM ? T : T / KS;
    static_assert(T % KS == 0, "row slots divide among the wavefronts of a tile");
    const int t0 = KS > 1 && !SM ? ks * TF : 0;
    const int nvalid = min(8, P.P - p);
    const int outs_img = P.G * P.Og;
    const int dst_elems = P.N * outs_img * P.P;
    const rsrc_t rad = make_rsrc(P.addend, dst_elems * 2);
    // A bf16 tensor that is added to the result (windowed data gradients) is fetched now, so that it has arrived
    // when the K loop ends; 3 x 3 windows only: there the registers do not cost a wavefront of occupancy.
    constexpr bool EARLY = !DST_F32 && KH == 3 && TF <= 8;
    u32x4 early[EARLY ? TF : 1];
    if constexpr (EARLY) {
#pragma unroll
        for (int i = 0; i < TF; i++) {
            const int t = t0 + i;
            const int o = ot * 16 * MO + (t >> 2) * 16 + 4 * r + (t & 3);
            const int e = (n * outs_img + gmi * P.gm * P.Og + o) * P.P + p;
            early[i] = bload16(rad, P.addend && live && o < Om && nvalid == 8 ? e * 2 : kOob);
        }
    }

    // groups g = (row chunk, kh); each statically unrolled slot owns one buffer, the next group's loads
    // are issued before the current group is multiplied
    constexpr int UNR = KH > 1 ? KH : 2;
    Group<MO, KW, WL> buf[UNR];
    const int nrc_mine = active && ks < nrc ? (nrc - ks + KS - 1) / KS : 0;  // this wavefront's chunks: ks, ks + KS, ...
    const int NG = nrc_mine * KH;
    issue(ks, 0, NG > 0, buf[0]);
    for (int it = 0; it * UNR < NG; it++) {
#pragma unroll
        for (int u = 0; u < UNR; u++) {
            const int g = it * UNR + u;
            if (KH > 1 || g < NG) {
                const int khn = KH > 1 ? (u + 1) % KH : 0;
                const int rcn = KH > 1 ? (u + 1 == KH ? it + 1 : it) : g + 1;  // index among this wavefront's chunks
                issue(ks + rcn * KS, khn, g + 1 < NG, buf[(u + 1) % UNR]);
                __builtin_amdgcn_sched_barrier(0);
                // (no window: UNR == 2, the chunks of an iteration are the two halves of a K = 32 step)
                consume(ks + (KH > 1 ? it : g) * KS, KH > 1 ? u : 0, buf[u], KW > 1 ? 2 : (u == 0 ? (g + 1 < NG ? 0 : 2) : 1));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // KS == 1: the wavefront owns all row slots.  KS > 1: wavefront f of the tile finishes slots
    // [f * T / KS, (f + 1) * T / KS): in round v every wavefront w hands the slots of wavefront (w + v) % KS over
    // through LDS, so each finisher adds its partners' sums in the fixed order own, w-1, w-2, ... and the
    // additions and stores of a tile are spread over its KS wavefronts.
    float fin[TF][8];
    if constexpr (SM && KS > 1) {
        // the first wavefront of the tile adds its partners' sums in the fixed order 1, 2, ... and finishes all rows
        typedef float Red[KS - 1][T * 8][64];
        Red* red = reinterpret_cast<Red*>(lds_dyn);
        if constexpr (WL) __syncthreads();
        const int sub = wave / KS;
        if (ks > 0) {
#pragma unroll
            for (int i = 0; i < T; i++)
#pragma unroll
                for (int q = 0; q < 8; q++) red[sub][ks - 1][i * 8 + q][lane] = acc[i >> 2][q][i & 3];
        }
        __syncthreads();
        if (ks > 0) return;
#pragma unroll
        for (int i = 0; i < T; i++)
#pragma unroll
            for (int q = 0; q < 8; q++) {
                float t = acc[i >> 2][q][i & 3];
#pragma unroll
                for (int d = 0; d < KS - 1; d++) t += red[sub][d][i * 8 + q][lane];
                fin[i][q] = t;
            }
    } else if constexpr (KS == 1) {
#pragma unroll
        for (int i = 0; i < TF; i++)
#pragma unroll
            for (int q = 0; q < 8; q++) fin[i][q] = acc[i >> 2][q][i & 3];
    } else {
        // (the sums reuse the LDS of the weight tile: every wavefront has left the K loop first)
        typedef float Red[KS][TF * 8][64];
        Red* red = reinterpret_cast<Red*>(lds_dyn);
        if constexpr (WL) __syncthreads();
        const int sub = wave / KS;
#pragma unroll
        for (int d = 0; d < KS; d++)
            if (d == ks) {
#pragma unroll
                for (int i = 0; i < TF; i++)
#pragma unroll
                    for (int q = 0; q < 8; q++) fin[i][q] = acc[(d * TF + i) >> 2][q][(d * TF + i) & 3];
            }
#pragma unroll
        for (int v = 1; v < KS; v++) {
            const int dst = (ks + v) % KS;
#pragma unroll
            for (int d = 0; d < KS; d++)
                if (d == dst) {
#pragma unroll
                    for (int i = 0; i < TF; i++)
#pragma unroll
                        for (int q = 0; q < 8; q++) red[sub][d][i * 8 + q][lane] = acc[(d * TF + i) >> 2][q][(d * TF + i) & 3];
                }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < TF; i++)
#pragma unroll
                for (int q = 0; q < 8; q++) fin[i][q] += red[sub][ks][i * 8 + q][lane];
            if (v + 1 < KS) __syncthreads();
        }
    }
    if (!live) return;
    if constexpr (SM) {
        // row slot i of lane (r, s) is output 4r + i of the unit's pixels: the Om outputs of a pixel are spread over the
        // lanes r = 0..3 of the same s (16 and 32 lanes apart)
#pragma unroll
        for (int q = 0; q < 8; q++) {
            float m = -INFINITY;
#pragma unroll
            for (int i = 0; i < T; i++)
                if (4 * r + i < Om) m = fmaxf(m, fin[i][q]);
            m = fmaxf(m, __shfl_xor(m, 16));
            m = fmaxf(m, __shfl_xor(m, 32));
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < T; i++) {
                fin[i][q] = 4 * r + i < Om ? expf(fin[i][q] - m) : 0.f;
                sum += fin[i][q];
            }
            sum += __shfl_xor(sum, 16);
            sum += __shfl_xor(sum, 32);
            const float inv = 1.f / sum;
#pragma unroll
            for (int i = 0; i < T; i++) fin[i][q] *= inv;
        }
    }
    const rsrc_t rd = make_rsrc(P.dst, dst_elems * (DST_F32 ? 4 : 2));
    // What the rows are added to is read, four rows at a time, before any of the four is stored: loads that
    // follow a store to the same tensor are not moved ahead of it, and would cost a memory round trip per row.
    constexpr int RB = TF < 4 ? TF : 4;
    const bool adds = (DST_F32 && P.acc) || (!DST_F32 && !EARLY && P.addend);
#pragma unroll
    for (int i0 = 0; i0 < TF; i0 += RB) {
    u32x4 pre[RB][2];
    if (adds) {
#pragma unroll
        for (int b = 0; b < RB; b++) {
            const int t = t0 + i0 + b;
            const int o = ot * 16 * MO + (t >> 2) * 16 + 4 * r + (t & 3);
            const int e = (n * outs_img + gmi * P.gm * P.Og + o) * P.P + p;
            const bool ok = o < Om && nvalid == 8;
            if (DST_F32) {
                pre[b][0] = bload16(rd, ok ? e * 4 : kOob);
                pre[b][1] = bload16(rd, ok ? e * 4 + 16 : kOob);
            } else {
                pre[b][0] = bload16(rad, ok ? e * 2 : kOob);
            }
        }
    }
#pragma unroll
    for (int b = 0; b < RB; b++) {
        const int i = i0 + b;
        const int t = t0 + i;
        const int o = ot * 16 * MO + (t >> 2) * 16 + 4 * r + (t & 3);
        if (o >= Om) continue;
        const int e = (n * outs_img + gmi * P.gm * P.Og + o) * P.P + p;
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; q++) v[q] = fin[i][q];
        if (nvalid == 8) {
            if (DST_F32) {
                u32x4 lo, hi;
                if (P.acc) {
                    lo = pre[b][0];
                    hi = pre[b][1];
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
                    const u32x4 ad = EARLY ? early[EARLY ? i : 0] : pre[b][0];
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
                    float tq = v[q];
                    if (P.addend) tq += __uint_as_float((uint32_t)P.addend[e + q] << 16);
                    reinterpret_cast<uint16_t*>(P.dst)[e + q] = (uint16_t)(pack_bf16(tq, 0.f) & 0xffffu);
                }
            }
        }
    }
    }
}

// ----------------------------------------------------------------------------------- weight gradient
// dwp[gmi][o'][tap][row'] = sum over (image, pixel) of dy[o'](p) * x[row'](p + off(tap)), zero outside the image.
// The contraction runs over pixels, the memory order of both operands, so 16-byte loads are MFMA operands
// as they are: lane (r, s) holds pixels 8r..8r+7 of a 32-pixel chunk, of dy row 16*mo + s (A) and of x row
// 16*rc + s (B); result lane holds dw[o' = 16*mo + 4r + jj][row' = 16*rc + s].
// A wavefront owns one chunk POSITION inside the image and walks over a range of images, so everything
// that depends on the position -- the zero-padding masks -- is computed once.  Per image and window row it
// loads the x pixels of its unit plus two on either side; the horizontal taps are funnel shifts of those
// registers.  Horizontal validity (a property of the output pixel) masks dy, once per window column;
// vertical validity masks x, only in chunks that touch the first / last image rows.
// The four wavefronts of a workgroup take four consecutive (image range, position) items of the same
// (group, output tile, row chunk); their sums are added through LDS in a fixed order: one partial per workgroup.
template <int MO, int KH, int KW>
struct Step {
    u32x4 dy[MO];
    uint32_t x[KH][6];  // per window row: [pixels -2,-1] pixels 0..7 [pixels 8,9]
};

template <int MO, int KH, int KW>
__global__ __launch_bounds__(64 * kWaves) void k_wgrad(Params P) {
    constexpr int TV = KH * KW, HW = KW / 2, HH = KH / 2;
    constexpr int NE = MO * TV * 4;  // accumulator floats per lane
    static_assert(HW >= 1 && HW <= 2, "windows with a halo of one or two pixels");
    __shared__ float red[2][NE][64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane >> 4, s = lane & 15;
    const int nrc = P.Rp >> 4;
    const int rc = blockIdx.y % nrc;
    const int got = blockIdx.y / nrc;
    const int otiles = P.Omp / (16 * MO);
    const int gmi = got / otiles, ot = got - gmi * otiles;
    const int gcount = min(P.gm, P.G - gmi * P.gm);
    const int Rm = gcount * P.R, Om = gcount * P.Og;
    const int items = P.chunks * P.nsplit;
    const int item = blockIdx.x * kWaves + wave;
    const bool active = item < items;
    const int isplit = active ? item / P.chunks : 0;
    const int pc = active ? item - isplit * P.chunks : 0;
    const int i0 = isplit * P.imgs_per_split;
    const int i1 = active ? min(P.N, i0 + P.imgs_per_split) : i0;

    const int rows_img = P.G * P.R, outs_img = P.G * P.Og;
    const int src_elems = P.N * rows_img * P.P, dy_elems = P.N * outs_img * P.P;
    const rsrc_t rs = make_rsrc(P.src, src_elems * 2);
    const rsrc_t rdy = make_rsrc(P.dy, dy_elems * 2);
    const int grow0 = gmi * P.gm * P.R, gout0 = gmi * P.gm * P.Og;
    const int p = pc * 32 + 8 * r;
    const bool livepx = p < P.P;
    const int nvalid = livepx ? min(8, P.P - p) : 0;
    const int maxoff = HH * P.W + 2;

    // per-lane constants: element offsets inside an image, load enables, masks
    int edy[MO];
    bool dyok[MO];
#pragma unroll
    for (int mo = 0; mo < MO; mo++) {
        const int o = ot * 16 * MO + mo * 16 + s;
        dyok[mo] = livepx && o < Om;
        edy[mo] = (gout0 + o) * P.P + p;
    }
    const int row = rc * 16 + s;
    const bool xok = livepx && row < Rm;
    const int ex = (grow0 + row) * P.P + p;

    u32x4 dymask[KW];  // pixel exists and its source column under window column kw is inside the image
    {
        const int h0 = (int)div_magic((uint32_t)min(p, P.P - 1), P.magicW);
        int c = min(p, P.P - 1) - h0 * P.W;
        uint32_t bits[KW];
#pragma unroll
        for (int kw = 0; kw < KW; kw++) bits[kw] = 0;
#pragma unroll
        for (int q = 0; q < 8; q++) {
#pragma unroll
            for (int kw = 0; kw < KW; kw++)
                if (q < nvalid && (unsigned)(c + kw - HW) < (unsigned)P.W) bits[kw] |= 1u << q;
            if (++c == P.W) c = 0;
        }
#pragma unroll
        for (int kw = 0; kw < KW; kw++) dymask[kw] = mask_of(bits[kw]);
    }
    bool needrow[KH];
#pragma unroll
    for (int kh = 0; kh < KH; kh++) {
        const int first = p - 2 + (kh - HH) * P.W, last = p + 9 + (kh - HH) * P.W;
        needrow[kh] = kh != HH && __builtin_amdgcn_ballot_w64(livepx && (first < 0 || last >= P.P)) != 0;
    }

    float4_t acc[MO][TV];
#pragma unroll
    for (int mo = 0; mo < MO; mo++)
#pragma unroll
        for (int t = 0; t < TV; t++) acc[mo][t] = float4_t{0.f, 0.f, 0.f, 0.f};

    auto issue = [&](int n, bool valid, Step<MO, KH, KW>& st) {
        // wave-uniform: could a multi-byte access of this step straddle an end of a tensor?  (the hardware
        // drops such an access as a whole; the lanes concerned re-read element by element)
        const int xrow0 = n * rows_img + grow0 + rc * 16, yrow0 = n * outs_img + gout0 + ot * 16 * MO;
        const bool near_ends = xrow0 * P.P + pc * 32 - maxoff < 0 || (xrow0 + 16) * P.P + pc * 32 + 48 + maxoff > src_elems ||
                               (yrow0 + 16 * MO) * P.P + pc * 32 + 40 > dy_elems;
        const int nx = n * rows_img * P.P, ny = n * outs_img * P.P;
#pragma unroll
        for (int mo = 0; mo < MO; mo++) {
            const bool ok = valid && dyok[mo];
            const int e = ny + edy[mo];
            st.dy[mo] = bload16(rdy, ok ? e * 2 : kOob);
            if (near_ends) reload_if_partial(st.dy[mo], rdy, ok ? e * 2 : kOob, dy_elems * 2);
        }
#pragma unroll
        for (int kh = 0; kh < KH; kh++) {
            const bool ok = valid && xok;
            const int bo = ok ? (nx + ex + (kh - HH) * P.W) * 2 : kOob;
            u32x4 m = bload16(rs, bo);
            // the two pixels on either side of the lane's 8 are its neighbours' (lanes 16 below / above hold the
            // adjacent pixels of the same row) and are fetched from them when the step is consumed; the first and
            // the last quarter of the wavefront have no such neighbour and load them, both in one instruction
            const int eo = ok ? (r == 0 ? bo - 4 : (r == 3 ? bo + 16 : kOob)) : kOob;
            uint32_t edge = __builtin_amdgcn_raw_buffer_load_b32(rs, eo, 0, 0);
            if (near_ends) {  // only lanes whose access is partly outside re-read, element by element
                reload_if_partial(m, rs, bo, src_elems * 2);
                reload_pair_if_partial(edge, rs, eo, src_elems * 2);
            }
#pragma unroll
            for (int k = 0; k < 4; k++) st.x[kh][k + 1] = m[k];
            st.x[kh][0] = edge;
        }
    };

    auto consume = [&](Step<MO, KH, KW>& st) {
#pragma unroll
        for (int kh = 0; kh < KH; kh++) {
            const uint32_t edge = st.x[kh][0];
            const uint32_t below = (uint32_t)__builtin_amdgcn_ds_bpermute(((lane + 48) & 63) * 4, (int)st.x[kh][4]);  // lane - 16
            const uint32_t above = (uint32_t)__builtin_amdgcn_ds_bpermute(((lane + 16) & 63) * 4, (int)st.x[kh][1]);  // lane + 16
            st.x[kh][0] = r == 0 ? edge : below;
            st.x[kh][5] = r == 3 ? edge : above;
        }
#pragma unroll
        for (int kh = 0; kh < KH; kh++)
            if (needrow[kh]) {
#pragma unroll
                for (int k = 0; k < 6; k++) {
                    const int i = 2 * k - 2;
                    const bool lo = (unsigned)(p + i + (kh - HH) * P.W) < (unsigned)P.P;
                    const bool hi = (unsigned)(p + i + 1 + (kh - HH) * P.W) < (unsigned)P.P;
                    st.x[kh][k] &= (lo ? 0x0000ffffu : 0u) | (hi ? 0xffff0000u : 0u);
                }
            }
#pragma unroll
        for (int kw = 0; kw < KW; kw++) {
            u32x4 a[MO];
#pragma unroll
            for (int mo = 0; mo < MO; mo++) a[mo] = st.dy[mo] & dymask[kw];
#pragma unroll
            for (int kh = 0; kh < KH; kh++) {
                // pixels dw .. dw + 7 of the row registers (element index of pixel 0 is 2)
                const int dw = kw - HW;
                uint32_t xs[4];
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    const int e0 = 2 * k + 2 + dw;  // first element of output dword k
                    xs[k] = (e0 & 1) ? __builtin_amdgcn_alignbit(st.x[kh][(e0 >> 1) + 1], st.x[kh][e0 >> 1], 16) : st.x[kh][e0 >> 1];
                }
#pragma unroll
                for (int mo = 0; mo < MO; mo++) {
                    float4_t c = acc[mo][kh * KW + kw];
                    c = mfma32(as_short4(a[mo][0], a[mo][1]), as_short4(a[mo][2], a[mo][3]), as_short4(xs[0], xs[1]), as_short4(xs[2], xs[3]), c);
                    acc[mo][kh * KW + kw] = c;
                }
            }
        }
    };

    if constexpr (KH <= 3) {
        // two images per trip: the loads of the next image are in flight while this one is multiplied
        Step<MO, KH, KW> st[2];
        issue(i0, i0 < i1, st[0]);
        for (int n = i0; n < i1; n += 2) {
            issue(n + 1, n + 1 < i1, st[1]);
            __builtin_amdgcn_sched_barrier(0);
            consume(st[0]);
            __builtin_amdgcn_sched_barrier(0);
            issue(n + 2, n + 2 < i1, st[0]);
            __builtin_amdgcn_sched_barrier(0);
            if (n + 1 < i1) consume(st[1]);
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
        // 5x5: 100 accumulator registers; one image in flight keeps the kernel under 256 registers
        Step<MO, KH, KW> st;
        for (int n = i0; n < i1; n++) {
            issue(n, true, st);
            consume(st);
        }
    }

    // sum of the workgroup's four wavefronts in a fixed order: (w0 + w2) + (w1 + w3), through LDS
    auto put = [&](int slot) {
#pragma unroll
        for (int mo = 0; mo < MO; mo++)
#pragma unroll
            for (int t = 0; t < TV; t++)
#pragma unroll
                for (int jj = 0; jj < 4; jj++) red[slot][(mo * TV + t) * 4 + jj][lane] = acc[mo][t][jj];
    };
    auto add = [&](int slot) {
#pragma unroll
        for (int mo = 0; mo < MO; mo++)
#pragma unroll
            for (int t = 0; t < TV; t++)
#pragma unroll
                for (int jj = 0; jj < 4; jj++) acc[mo][t][jj] += red[slot][(mo * TV + t) * 4 + jj][lane];
    };
    if (wave >= 2) put(wave - 2);
    __syncthreads();
    if (wave < 2) add(wave);
    __syncthreads();
    if (wave == 1) put(0);
    __syncthreads();
    if (wave == 0) {
        add(0);
        float* part = P.partial + (long long)blockIdx.x * P.Gm * P.Omp * TV * P.Rp;
#pragma unroll
        for (int mo = 0; mo < MO; mo++)
#pragma unroll
            for (int t = 0; t < TV; t++)
#pragma unroll
                for (int jj = 0; jj < 4; jj++) {
                    const int o = ot * 16 * MO + mo * 16 + 4 * r + jj;
                    part[((long long)(gmi * P.Omp + o) * TV + t) * P.Rp + rc * 16 + s] = acc[mo][t][jj];
                }
    }
}

// The same for 3 x 3 windows on images whose rows fill most of one or several 32-pixel chunks: a wavefront owns
// a chunk of COLUMNS and walks down the image rows (a step = one row of one image).  Row h + 1 of x at step
// h is row h of step h + 1: after the first step of an image only ONE new x row is loaded per step, and the two
// others are the previous step's registers (the kernel above fetches three row pieces per step, and its loads
// were more than half of its time at 56 x 56).  A row is inside the image or not as a whole, so a row outside
// is simply not loaded (zeros) and no vertical masks exist; columns beyond the row's end hold the next row's
// pixels and are masked on dy together with the horizontal validity of each window column.
template <int MO>
__global__ __launch_bounds__(64 * kWaves) void k_wgrad_rows(Params P) {
    constexpr int KH = 3, KW = 3, TV = 9, HW = 1;
    constexpr int NE = MO * TV * 4;
    __shared__ float red[2][NE][64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane >> 4, s = lane & 15;
    const int nrc = P.Rp >> 4;
    const int rc = blockIdx.y % nrc;
    const int got = blockIdx.y / nrc;
    const int otiles = P.Omp / (16 * MO);
    const int gmi = got / otiles, ot = got - gmi * otiles;
    const int gcount = min(P.gm, P.G - gmi * P.gm);
    const int Rm = gcount * P.R, Om = gcount * P.Og;
    const int items = P.chunks * P.nsplit;  // column chunks x ranges of (image, row) steps
    const int item = blockIdx.x * kWaves + wave;
    const bool active = item < items;
    const int isplit = active ? item / P.chunks : 0;
    const int qc = active ? item - isplit * P.chunks : 0;
    const int t0 = isplit * P.imgs_per_split;
    const int t1 = active ? min(P.N * P.H, t0 + P.imgs_per_split) : t0;

    const int rows_img = P.G * P.R, outs_img = P.G * P.Og;
    const int src_elems = P.N * rows_img * P.P, dy_elems = P.N * outs_img * P.P;
    const rsrc_t rs = make_rsrc(P.src, src_elems * 2);
    const rsrc_t rdy = make_rsrc(P.dy, dy_elems * 2);
    const int grow0 = gmi * P.gm * P.R, gout0 = gmi * P.gm * P.Og;
    const int c = qc * 32 + 8 * r;  // first column of this lane
    const bool livepx = c < P.W;

    int edy[MO];
    bool dyok[MO];
#pragma unroll
    for (int mo = 0; mo < MO; mo++) {
        const int o = ot * 16 * MO + mo * 16 + s;
        dyok[mo] = livepx && o < Om;
        edy[mo] = (gout0 + o) * P.P + c;
    }
    const int row = rc * 16 + s;
    const bool xok = livepx && row < Rm;
    const int ex = (grow0 + row) * P.P + c;

    u32x4 dymask[KW];  // column exists and its source column under window column kw is inside the image
#pragma unroll
    for (int kw = 0; kw < KW; kw++) {
        uint32_t bits = 0;
#pragma unroll
        for (int q = 0; q < 8; q++)
            if (c + q < P.W && (unsigned)(c + q + kw - HW) < (unsigned)P.W) bits |= 1u << q;
        dymask[kw] = mask_of(bits);
    }

    float4_t acc[MO][TV];
#pragma unroll
    for (int mo = 0; mo < MO; mo++)
#pragma unroll
        for (int t = 0; t < TV; t++) acc[mo][t] = float4_t{0.f, 0.f, 0.f, 0.f};

    struct RowStep {
        u32x4 dy[MO];
        uint32_t x[KH][6];  // per window row: [2 pixels left | the lane's 8 pixels | 2 pixels right]
    };

    // x row `hr` of image n (a row outside the image: zeros) -> its 8 pixels in x[1..4], the edge pixels of the first /
    // last quarter of the wavefront in x[0] (see the kernel above)
    auto load_row = [&](int n, int hr, bool valid, bool near_ends, uint32_t (&x)[6]) {
        const bool ok = valid && xok && (unsigned)hr < (unsigned)P.H;
        const int bo = ok ? (n * rows_img * P.P + ex + hr * P.W) * 2 : kOob;
        u32x4 m = bload16(rs, bo);
        const int eo = ok ? (r == 0 ? bo - 4 : (r == 3 ? bo + 16 : kOob)) : kOob;
        uint32_t edge = __builtin_amdgcn_raw_buffer_load_b32(rs, eo, 0, 0);
        if (near_ends) {  // only lanes whose access is partly outside re-read, element by element
            reload_if_partial(m, rs, bo, src_elems * 2);
            reload_pair_if_partial(edge, rs, eo, src_elems * 2);
        }
#pragma unroll
        for (int k = 0; k < 4; k++) x[k + 1] = m[k];
        x[0] = edge;
    };
    // `first`: the step opens an image (or the wavefront's range): all three x rows are loaded; else rows h - 1 and h
    // are the previous step's rows h and h + 1
    auto issue = [&](int t, bool valid, bool first, RowStep& st, const RowStep& prev) {
        const int n = (int)div_magic((uint32_t)t, P.magicH), h = t - n * P.H;
        // wave-uniform: could an access of this step straddle an end of a tensor?
        const int xrow0 = n * rows_img + grow0 + rc * 16, yrow0 = n * outs_img + gout0 + ot * 16 * MO;
        const int px = h * P.W + qc * 32;
        const bool near_ends = xrow0 * P.P + px - P.W - 2 < 0 || (xrow0 + 16) * P.P + px + P.W + 48 > src_elems ||
                               (yrow0 + 16 * MO) * P.P + px + 40 > dy_elems;
#pragma unroll
        for (int mo = 0; mo < MO; mo++) {
            const bool ok = valid && dyok[mo];
            const int bo = ok ? (n * outs_img * P.P + edy[mo] + h * P.W) * 2 : kOob;
            st.dy[mo] = bload16(rdy, bo);
            if (near_ends) reload_if_partial(st.dy[mo], rdy, bo, dy_elems * 2);
        }
        if (first) {
            load_row(n, h - 1, valid, near_ends, st.x[0]);
            load_row(n, h, valid, near_ends, st.x[1]);
        } else {
#pragma unroll
            for (int k = 0; k < 6; k++) {
                st.x[0][k] = prev.x[1][k];
                st.x[1][k] = prev.x[2][k];
            }
        }
        load_row(n, h + 1, valid, near_ends, st.x[2]);
    };
    // the two pixels on either side of the lane's 8: its neighbours' (lanes 16 below / above), or the loaded edge
    auto halo = [&](uint32_t (&x)[6]) {
        const uint32_t edge = x[0];
        const uint32_t below = (uint32_t)__builtin_amdgcn_ds_bpermute(((lane + 48) & 63) * 4, (int)x[4]);
        const uint32_t above = (uint32_t)__builtin_amdgcn_ds_bpermute(((lane + 16) & 63) * 4, (int)x[1]);
        x[0] = r == 0 ? edge : below;
        x[5] = r == 3 ? edge : above;
    };
    auto finish = [&](bool first, RowStep& st) {
        if (first) {
            halo(st.x[0]);
            halo(st.x[1]);
        }
        halo(st.x[2]);
    };
    auto multiply = [&](RowStep& st) {
#pragma unroll
        for (int kw = 0; kw < KW; kw++) {
            u32x4 a[MO];
#pragma unroll
            for (int mo = 0; mo < MO; mo++) a[mo] = st.dy[mo] & dymask[kw];
#pragma unroll
            for (int kh = 0; kh < KH; kh++) {
                const int dw = kw - HW;
                uint32_t xs[4];
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    const int e0 = 2 * k + 2 + dw;  // first element of output dword k (element index of pixel 0 is 2)
                    xs[k] = (e0 & 1) ? __builtin_amdgcn_alignbit(st.x[kh][(e0 >> 1) + 1], st.x[kh][e0 >> 1], 16) : st.x[kh][e0 >> 1];
                }
#pragma unroll
                for (int mo = 0; mo < MO; mo++) {
                    float4_t cc = acc[mo][kh * KW + kw];
                    cc = mfma32(as_short4(a[mo][0], a[mo][1]), as_short4(a[mo][2], a[mo][3]), as_short4(xs[0], xs[1]), as_short4(xs[2], xs[3]), cc);
                    acc[mo][kh * KW + kw] = cc;
                }
            }
        }
    };
    auto opens_image = [&](int t) { return t - (int)div_magic((uint32_t)t, P.magicH) * P.H == 0; };

    // two steps per trip: the loads of the next step are in flight while this one is multiplied
    RowStep st[2];
    bool first0 = true, first1 = false;
    issue(t0, t0 < t1, true, st[0], st[0]);
    for (int t = t0; t < t1; t += 2) {
        finish(first0, st[0]);
        first1 = opens_image(t + 1);
        issue(t + 1, t + 1 < t1, first1, st[1], st[0]);
        __builtin_amdgcn_sched_barrier(0);
        multiply(st[0]);
        __builtin_amdgcn_sched_barrier(0);
        if (t + 1 < t1) {
            finish(first1, st[1]);
            first0 = opens_image(t + 2);
            issue(t + 2, t + 2 < t1, first0, st[0], st[1]);
            __builtin_amdgcn_sched_barrier(0);
            multiply(st[1]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // sum of the workgroup's four wavefronts in a fixed order: (w0 + w2) + (w1 + w3), through LDS
    auto put = [&](int slot) {
#pragma unroll
        for (int mo = 0; mo < MO; mo++)
#pragma unroll
            for (int t = 0; t < TV; t++)
#pragma unroll
                for (int jj = 0; jj < 4; jj++) red[slot][(mo * TV + t) * 4 + jj][lane] = acc[mo][t][jj];
    };
    auto add = [&](int slot) {
#pragma unroll
        for (int mo = 0; mo < MO; mo++)
#pragma unroll
            for (int t = 0; t < TV; t++)
#pragma unroll
                for (int jj = 0; jj < 4; jj++) acc[mo][t][jj] += red[slot][(mo * TV + t) * 4 + jj][lane];
    };
    if (wave >= 2) put(wave - 2);
    __syncthreads();
    if (wave < 2) add(wave);
    __syncthreads();
    if (wave == 1) put(0);
    __syncthreads();
    if (wave == 0) {
        add(0);
        float* part = P.partial + (long long)blockIdx.x * P.Gm * P.Omp * TV * P.Rp;
#pragma unroll
        for (int mo = 0; mo < MO; mo++)
#pragma unroll
            for (int t = 0; t < TV; t++)
#pragma unroll
                for (int jj = 0; jj < 4; jj++) {
                    const int o = ot * 16 * MO + mo * 16 + 4 * r + jj;
                    part[((long long)(gmi * P.Omp + o) * TV + t) * P.Rp + rc * 16 + s] = acc[mo][t][jj];
                }
    }
}

// One tile per wavefront (KS = 1) or per KS wavefronts.  (Measured on MI355X: persistent wavefronts that
// walk over several tiles and issue the next tile's first loads early, with or without cache-line
// touches ahead, were not faster than letting the hardware scheduler balance one-tile workgroups; nor was
// a 1x1 variant that keeps three groups of loads in flight instead of one.)
template <int MO, int KH, int KW, bool DST_F32, bool WL>
void launch_fwd_w(const Params& P, unsigned lds_w, hipStream_t s) {
    const int tiles = (P.N * P.upi + 15) / 16;
    const dim3 block(64 * kWaves);
    const unsigned gy = (unsigned)(P.Gm * P.otiles);
    // split-K sums: kWaves / KS tiles x KS wavefronts x (4 * MO / KS) row slots x 8 pixels x 64 lanes, fp32
    const unsigned red = P.ksplit > 1 ? (unsigned)(kWaves * (4 * MO / P.ksplit) * 8 * 64 * 4) : 0u;
    const unsigned lds = std::max(lds_w, red);
    if (P.ksplit == 4) CANVAS_LAUNCH((k_fwd<MO, KH, KW, DST_F32, 4, WL>), dim3((unsigned)tiles, gy), block, lds, s, P);
    else if (P.ksplit == 2) CANVAS_LAUNCH((k_fwd<MO, KH, KW, DST_F32, 2, WL>), dim3((unsigned)((tiles + 1) / 2), gy), block, lds, s, P);
    else CANVAS_LAUNCH((k_fwd<MO, KH, KW, DST_F32, 1, WL>), dim3((unsigned)((tiles + kWaves - 1) / kWaves), gy), block, lds, s, P);
}

// FC + softmax over its (at most 16) outputs: one output tile, fp32 result, no window
template <bool WL>
void launch_fwd_softmax_w(const Params& P, unsigned lds_w, hipStream_t s) {
    const int tiles = (P.N * P.upi + 15) / 16;
    const dim3 block(64 * kWaves);
    const unsigned gy = (unsigned)(P.Gm * P.otiles);
    // the partners' sums: kWaves / KS tiles x (KS - 1) wavefronts x 4 row slots x 8 pixels x 64 lanes, fp32
    const unsigned red = P.ksplit > 1 ? (unsigned)(kWaves / P.ksplit * (P.ksplit - 1) * 32 * 64 * 4) : 0u;
    const unsigned lds = std::max(lds_w, red);
    if (P.ksplit == 4) CANVAS_LAUNCH((k_fwd<1, 1, 1, true, 4, WL, true>), dim3((unsigned)tiles, gy), block, lds, s, P);
    else if (P.ksplit == 2) CANVAS_LAUNCH((k_fwd<1, 1, 1, true, 2, WL, true>), dim3((unsigned)((tiles + 1) / 2), gy), block, lds, s, P);
    else CANVAS_LAUNCH((k_fwd<1, 1, 1, true, 1, WL, true>), dim3((unsigned)((tiles + kWaves - 1) / kWaves), gy), block, lds, s, P);
}

template <int MO, int KH, int KW, bool DST_F32>
void launch_fwd_k(const Params& P, hipStream_t s) {
    // the weight tile of a workgroup goes through LDS where two workgroups' tiles fit a compute unit
    const unsigned lds_w = 16u * MO * (unsigned)(P.TV * P.Rp * 2 + 16);
    if (lds_w <= 72u * 1024u) launch_fwd_w<MO, KH, KW, DST_F32, true>(P, lds_w, s);
    else launch_fwd_w<MO, KH, KW, DST_F32, false>(P, 0u, s);
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
    if (Q.mo == 4) {
        // 64 outputs per wavefront need ~200 registers (two wavefronts per SIMD, 2 048 at once), 32 outputs ~124 (four,
        // 4 096): where the launch with 64 needs a second round of wavefronts and the one with 32 fits at once, 32 are
        // faster although the source is read once more
        const int64_t tiles16 = ((int64_t)N * Q.upi + 15) / 16 * Q.Gm;
        const int64_t w4 = tiles16 * ((Om + 63) / 64), w2 = tiles16 * ((Om + 31) / 32);
        if (w4 > 2048 && w2 <= 4096) Q.mo = 2;
    }
    Q.otiles = (Om + 16 * Q.mo - 1) / (16 * Q.mo);
    // few tiles with a long K loop: split the row chunks of a tile over 2 or 4 wavefronts
    const int64_t waves = (((int64_t)N * Q.upi + 15) / 16) * Q.Gm * Q.otiles;
    const int nrc = Q.Rp / 16;
    Q.ksplit = 1;
    // (only while all wavefronts are resident at once, two per SIMD: a second round of wavefronts costs more than the
    // longer K loop; C=128, 28x28, N=128, 64 outputs per tile: 1 568 wavefronts unsplit 13.8 us, 3 136 split by two 17.1 us,
    // 3 136 of 32 outputs 18.0 us)
    if (waves * 2 <= 2048 && nrc >= 2) Q.ksplit = 2;
    if (waves * 4 <= 2048 && nrc >= 4) Q.ksplit = 4;
    Q.Omp = Q.otiles * 16 * Q.mo;
    auto magic = [](uint32_t d) { return d <= 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) + d - 1) / d); };
    Q.magicW = magic((uint32_t)W);
    Q.magicUpi = magic((uint32_t)Q.upi);
    Q.magicW16 = magic((uint32_t)(Q.TV * Q.Rp / 8));
    Q.magicH = magic((uint32_t)H);
    return Q;
}

Params data_gradient_of(const Params& f) { return shape(f.N, f.G, f.Og, f.KH, f.KW, f.R, f.H, f.W); }

// outputs per wavefront tile of the weight gradient, in units of 16 (its accumulators are MO x taps)
static int wgrad_mo(const Params& P) { return P.KH == 3 && P.Omp % 32 == 0 ? 2 : 1; }

void prepare_wgrad(Params& P) {
    // 3 x 3 windows on rows that fill at least 3/4 of their 32-column chunks: by image rows (k_wgrad_rows), where a
    // step is one row of one image; else by 32-pixel positions, where a step is one image
    const int qchunks = (P.W + 31) / 32;
    P.rows = P.KH == 3 && P.KW == 3 && P.W >= 24 && 4 * P.W >= 3 * 32 * qchunks ? 1 : 0;
    P.chunks = P.rows ? qchunks : (P.P + 31) / 32;
    const int64_t steps = P.rows ? (int64_t)P.N * P.H : P.N;
    const int64_t tiles = (int64_t)P.Gm * (P.Omp / (16 * wgrad_mo(P))) * (P.Rp / 16);
    const int64_t packed = packed_elems(P);
    // about 3.5 k wavefronts (by rows: 2 k, measured); partials at most max(4 MB, 30 % of the operand bytes)
    const int64_t waves = P.rows ? 2048 : 3584;
    int64_t nsplit = std::max<int64_t>(1, std::min<int64_t>(steps, (waves + P.chunks * tiles - 1) / (P.chunks * tiles)));
    const int64_t operand_bytes = (int64_t)P.N * P.G * (P.R + P.Og) * P.P * 2;
    const int64_t cap = std::max<int64_t>((int64_t)4 << 20, operand_bytes * 3 / 10);
    nsplit = std::max<int64_t>(1, std::min<int64_t>(nsplit, kWaves * cap / (packed * 4 * P.chunks)));
    int64_t per = (steps + nsplit - 1) / nsplit;
    if (P.rows) {
        // a range of steps that begins inside an image reloads its three rows: ranges are whole images, or the
        // smallest divisor of the image height that is at least the number wanted, so that none straddles two images
        if (per >= P.H) {
            per = (per + P.H / 2) / P.H * P.H;
        } else {
            int64_t d = per;
            while (P.H % d) d++;
            per = d;
        }
    }
    P.imgs_per_split = (int)per;
    P.nsplit = (int)((steps + per - 1) / per);
}

int wgrad_slices(const Params& P) { return (P.chunks * P.nsplit + kWaves - 1) / kWaves; }

void wgrad_partial(const Params& P, hipStream_t s) {
    const int mo = wgrad_mo(P);
    const dim3 grid((unsigned)wgrad_slices(P), (unsigned)(P.Gm * (P.Omp / (16 * mo)) * (P.Rp / 16)));
    const dim3 block(64 * kWaves);
    if (P.rows) {
        if (mo == 1) CANVAS_LAUNCH((k_wgrad_rows<1>), grid, block, 0, s, P);
        else CANVAS_LAUNCH((k_wgrad_rows<2>), grid, block, 0, s, P);
    } else if (P.KH == 3) {
        if (mo == 1) CANVAS_LAUNCH((k_wgrad<1, 3, 3>), grid, block, 0, s, P);
        else CANVAS_LAUNCH((k_wgrad<2, 3, 3>), grid, block, 0, s, P);
    } else {
        CANVAS_LAUNCH((k_wgrad<1, 5, 5>), grid, block, 0, s, P);
    }
}

bool softmax_fusable(const Params& P) { return P.G == 1 && P.Og <= 16 && P.KH == 1 && P.KW == 1; }

void forward(const Params& P, hipStream_t s) {
    if ((int64_t)P.N * P.G * P.Og * P.P == 0) return;
    if (P.softmax) {  // (the caller has checked softmax_fusable and set dst_f32)
        const unsigned lds_w = 16u * (unsigned)(P.TV * P.Rp * 2 + 16);
        if (lds_w <= 72u * 1024u) launch_fwd_softmax_w<true>(P, lds_w, s);
        else launch_fwd_softmax_w<false>(P, 0u, s);
        return;
    }
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
