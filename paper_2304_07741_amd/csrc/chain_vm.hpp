// Per-thread execution of the fused-chain instruction set (see chain_isa.hpp).  A thread owns V consecutive pixels of
// one image plane; a value is T x V floats (lane t * V + v = tap t of pixel v), so one interpreted instruction works
// on 8 to 25 elements and every tensor access is one vector access of V elements.  Everything here is per-pixel
// arithmetic on the thread's own state; the one instruction that moves data between threads (OP_XADD) is driven by the
// kernel around two helpers of this file.  Primitive definitions: Canvas paper, Section 5; subgradient choices:
// relu'(0) = 0, sign(0) = 0, clipped exp flat outside the open interval, first maximum of a max fold, ties of
// min / max to the LHS.
//
// The file compiles for the device (raw buffer accesses) and for the host (checked scalar accesses), so that the
// interpreter can be run on the CPU, workgroup by workgroup, against the same programs.
#pragma once
#include <cmath>
#include <cstdint>
#include <cstring>

#include "chain_isa.hpp"

#if defined(__HIP_DEVICE_COMPILE__)
#include "tile_util.hpp"
#endif

#if defined(__HIPCC__)
#define CHAIN_HD __host__ __device__ __forceinline__
#else
#define CHAIN_HD inline
#endif

namespace canvas {
namespace chain {

template <int TM, int V, int U>
struct State {
    float A[U * TM * V];
};

// 16-byte pieces of a register R[r] (lanes floats, rounded up); piece q of register r of thread i is at float
// ((r * pieces + q) * threads + i) * 4 of the register area, so that a wavefront's access is one contiguous run.
constexpr int reg_pieces(int lanes) { return (lanes + 3) / 4; }

// What a thread knows about its pixels.  p0 is the plane index of its first pixel (a multiple of V; threads of the
// halo may lie before the plane or behind it: active == false); only `own` threads store.
struct Thread {
    int ptid = 0, n = 0, p0 = 0, row0 = 0, col0 = 0;
    bool active = false, own = false;
};

// Geometry in uniform registers.
struct Geo {
    int H = 0, W = 0, C = 0, HW = 0, N = 0;
    int npx = 0;  // pixels a slice of the workgroup computes = pix_threads * V
    bool whole_rows = false;  // W is a multiple of V: the V pixels of a thread never straddle two image rows
};

// Each case of the dispatch begins with an empty volatile asm statement: the cases are small, and without it the
// compiler executes the arithmetic of ALL of them for every instruction and selects the result.
#if defined(__HIP_DEVICE_COMPILE__)
#define CHAIN_CASE asm volatile("")
#else
#define CHAIN_CASE ((void)0)
#endif

// The program is interpreted from LDS, whose loads land in vector registers: the compiler cannot know that every
// lane read the same word.  vm_u() tells it (one v_readfirstlane), so that instruction fields, tensor descriptors and
// geometry live in scalar registers and the dispatch on them is a scalar branch.
#if defined(__HIP_DEVICE_COMPILE__)
CHAIN_HD int vm_u(int v) { return __builtin_amdgcn_readfirstlane(v); }
#else
CHAIN_HD int vm_u(int v) { return v; }
#endif
// A 16-byte instruction, made uniform.
CHAIN_HD Instr vm_fetch(const Instr& src) {
    uint32_t w[4];
    memcpy(w, &src, 16);
    for (int k = 0; k < 4; k++) w[k] = (uint32_t)vm_u((int)w[k]);
    Instr I;
    memcpy(&I, w, 16);
    return I;
}
#if defined(__HIPCC__)
// The same for an instruction that has already been read as four dwords.
__device__ __forceinline__ Instr vm_uniform(const uint4& raw) {
    uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
    for (int k = 0; k < 4; k++) w[k] = (uint32_t)vm_u((int)w[k]);
    Instr I;
    memcpy(&I, w, 16);
    return I;
}
#endif
CHAIN_HD Geo vm_geo(const Program& pg) {
    Geo g;
    g.H = vm_u(pg.H);
    g.W = vm_u(pg.W);
    g.C = vm_u(pg.C);
    g.N = vm_u(pg.N);
    g.HW = g.H * g.W;
    g.npx = vm_u(pg.pix_threads) * vm_u(pg.vec);
    g.whole_rows = g.W % vm_u(pg.vec) == 0;
    return g;
}

CHAIN_HD float vm_bf16_to_f32(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}
CHAIN_HD float vm_bits_to_f32(uint32_t u) {
    float f;
    memcpy(&f, &u, 4);
    return f;
}
CHAIN_HD uint32_t vm_f32_to_bits(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    return u;
}

CHAIN_HD uint16_t vm_f32_to_bf16(float f) {  // round to nearest even; NaN stays NaN
    uint32_t u = vm_f32_to_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// ---------------------------------------------------------------------------------------------------- tensors
// A tensor of the program in uniform registers.  Element indices are 32-bit (the planner only admits tensors below
// 2^31 bytes) and may lie outside the tensor (a shifted access at the first or last image): such elements read as
// zero on the device and as NaN on the host, and are masked by the caller either way.
struct Tensor {
#if defined(__HIP_DEVICE_COMPILE__)
    tile::rsrc_t rs;
#else
    void* ptr = nullptr;
#endif
    int bytes = 0;
    int T = 1;
    int bf16 = 0;
};

CHAIN_HD Tensor vm_tensor(const Program& pg, const Geo& g, int a) {
    uint32_t w[4];
    memcpy(w, &pg.ext[a], 16);
    for (int k = 0; k < 4; k++) w[k] = (uint32_t)vm_u((int)w[k]);
    Tensor t;
    t.T = (int)w[2];
    t.bf16 = (int)w[3];
    t.bytes = g.N * g.C * t.T * g.HW * (t.bf16 ? 2 : 4);
    void* p = (void*)(((uint64_t)w[1] << 32) | w[0]);
#if defined(__HIP_DEVICE_COMPILE__)
    t.rs = tile::make_rsrc(p, t.bytes);
#else
    t.ptr = p;
#endif
    return t;
}

#if defined(__HIP_DEVICE_COMPILE__)
typedef uint32_t vm_u32x2 __attribute__((ext_vector_type(2)));

// V elements that begin at element `elem`.  ALIGNED: elem is a multiple of V (so is every tensor's size), the access
// is wholly inside or wholly outside the tensor and no piece of it needs a second look.
template <int V, bool ALIGNED>
__device__ __forceinline__ void vm_load(const Tensor& e, int elem, float* out) {
    if (e.bf16) {
        const int o = elem * 2;
        if (V % 8 == 0) {
#pragma unroll
            for (int q = 0; q < V / 8; q++) {
                tile::u32x4 d = tile::bload16(e.rs, o + 16 * q);
                if (!ALIGNED && tile::straddles_an_end(o + 16 * q, 16, e.bytes)) {
                    // (rare: a shifted vector across the very start or end of the tensor; the empty asm keeps the
                    // compiler from computing the element addresses of this branch ahead of it, for every access)
                    int o2 = o + 16 * q;
                    asm volatile("" : "+v"(o2));
#pragma unroll
                    for (int k = 0; k < 4; k++) d[k] = tile::elem_b16(e.rs, o2 + 4 * k, e.bytes) | (tile::elem_b16(e.rs, o2 + 4 * k + 2, e.bytes) << 16);
                }
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    out[8 * q + 2 * k] = tile::lo_f32(d[k]);
                    out[8 * q + 2 * k + 1] = tile::hi_f32(d[k]);
                }
            }
        } else if (V == 4) {
            vm_u32x2 d = __builtin_amdgcn_raw_buffer_load_b64(e.rs, o, 0, 0);
            if (!ALIGNED && tile::straddles_an_end(o, 8, e.bytes)) {
#pragma unroll
                for (int k = 0; k < 2; k++) d[k] = tile::elem_b16(e.rs, o + 4 * k, e.bytes) | (tile::elem_b16(e.rs, o + 4 * k + 2, e.bytes) << 16);
            }
#pragma unroll
            for (int k = 0; k < 2; k++) {
                out[2 * k] = tile::lo_f32(d[k]);
                out[2 * k + 1] = tile::hi_f32(d[k]);
            }
        } else if (V == 2) {
            uint32_t d = __builtin_amdgcn_raw_buffer_load_b32(e.rs, o, 0, 0);
            if (!ALIGNED) tile::reload_pair_if_partial(d, e.rs, o, e.bytes);
            out[0] = tile::lo_f32(d);
            out[1] = tile::hi_f32(d);
        } else {
#pragma unroll
            for (int v = 0; v < V; v++) out[v] = tile::lo_f32(tile::elem_b16(e.rs, o + 2 * v, e.bytes));
        }
    } else {
        const int o = elem * 4;
        if (V % 4 == 0) {
#pragma unroll
            for (int q = 0; q < V / 4; q++) {
                tile::u32x4 d = tile::bload16(e.rs, o + 16 * q);
                if (!ALIGNED && tile::straddles_an_end(o + 16 * q, 16, e.bytes)) {
                    int o2 = o + 16 * q;
                    asm volatile("" : "+v"(o2));
#pragma unroll
                    for (int k = 0; k < 4; k++) d[k] = tile::elem_b32(e.rs, o2 + 4 * k, e.bytes);
                }
#pragma unroll
                for (int k = 0; k < 4; k++) out[4 * q + k] = __uint_as_float(d[k]);
            }
        } else {
#pragma unroll
            for (int v = 0; v < V; v++) out[v] = __uint_as_float(tile::elem_b32(e.rs, o + 4 * v, e.bytes));
        }
    }
}

// V elements to element `elem` (always inside the tensor and a multiple of V: only owned pixels are stored).
template <int V>
__device__ __forceinline__ void vm_store(const Tensor& e, int elem, const float* in, bool add) {
    if (e.bf16) {
        const int o = elem * 2;
        if (V % 8 == 0) {
#pragma unroll
            for (int q = 0; q < V / 8; q++) {
                tile::u32x4 d;
#pragma unroll
                for (int k = 0; k < 4; k++) d[k] = tile::pack_bf16(in[8 * q + 2 * k], in[8 * q + 2 * k + 1]);
                tile::bstore16_nt(e.rs, o + 16 * q, d);
            }
        } else if (V == 4) {
            vm_u32x2 d;
#pragma unroll
            for (int k = 0; k < 2; k++) d[k] = tile::pack_bf16(in[2 * k], in[2 * k + 1]);
            __builtin_amdgcn_raw_buffer_store_b64(d, e.rs, o, 0, 0);
        } else if (V == 2) {
            __builtin_amdgcn_raw_buffer_store_b32(tile::pack_bf16(in[0], in[1]), e.rs, o, 0, 0);
        } else {
            __builtin_amdgcn_raw_buffer_store_b16((uint16_t)(tile::pack_bf16(in[0], 0.f) & 0xffffu), e.rs, o, 0, 0);
        }
    } else {
        const int o = elem * 4;
        float v[V];
        if (add) {
            vm_load<V, true>(e, elem, v);
#pragma unroll
            for (int k = 0; k < V; k++) v[k] += in[k];
        } else {
#pragma unroll
            for (int k = 0; k < V; k++) v[k] = in[k];
        }
        if (V % 4 == 0) {
#pragma unroll
            for (int q = 0; q < V / 4; q++) {
                tile::u32x4 d;
#pragma unroll
                for (int k = 0; k < 4; k++) d[k] = __float_as_uint(v[4 * q + k]);
                tile::bstore16_nt(e.rs, o + 16 * q, d);
            }
        } else {
#pragma unroll
            for (int k = 0; k < V; k++) __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v[k]), e.rs, o + 4 * k, 0, 0);
        }
    }
}
#else
// Host: element by element, checked.  An element outside the tensor reads as NaN, so that a missing mask shows in
// the results; a store outside the tensor is a bug of the planner and aborts.
#include <cstdio>
#include <cstdlib>
template <int V, bool ALIGNED>
inline void vm_load(const Tensor& e, int elem, float* out) {
    const int64_t n = e.bytes / (e.bf16 ? 2 : 4);
    if (ALIGNED && elem % V != 0) {
        std::fprintf(stderr, "chain vm: an aligned load of %d elements at %d\n", V, elem);
        std::abort();
    }
    for (int v = 0; v < V; v++) {
        const int64_t i = (int64_t)elem + v;
        if (i < 0 || i >= n) out[v] = NAN;
        else out[v] = e.bf16 ? vm_bf16_to_f32(((const uint16_t*)e.ptr)[i]) : ((const float*)e.ptr)[i];
    }
}
template <int V>
inline void vm_store(const Tensor& e, int elem, const float* in, bool add) {
    const int64_t n = e.bytes / (e.bf16 ? 2 : 4);
    if (elem < 0 || (int64_t)elem + V > n || elem % V) {
        std::fprintf(stderr, "chain vm: store of %d elements at %d outside a tensor of %lld\n", V, elem, (long long)n);
        std::abort();
    }
    for (int v = 0; v < V; v++) {
        if (e.bf16) ((uint16_t*)e.ptr)[elem + v] = vm_f32_to_bf16(in[v]);
        else if (add) ((float*)e.ptr)[elem + v] += in[v];
        else ((float*)e.ptr)[elem + v] = in[v];
    }
}
#endif

// ---------------------------------------------------------------------------------------------------- arithmetic
// The element-wise functions, one per kind: the dispatch on the kind happens once per instruction, outside the loops
// over the lanes (a switch inside the loop costs a scalar branch tree per element).
CHAIN_HD float vm_gelu(float x) { return 0.5f * x * (1.f + erff(x * 0.70710678118654752f)); }
CHAIN_HD float vm_gelu_grad(float x) { return 0.5f * (1.f + erff(x * 0.70710678118654752f)) + x * 0.39894228040143268f * expf(-0.5f * x * x); }
CHAIN_HD float vm_sign(float x) { return x > 0.f ? 1.f : (x < 0.f ? -1.f : 0.f); }
// Normal CDF and density for programs of bf16 DAGs (Program::fast_math): erfc by the rational-times-Gaussian
// approximation of Abramowitz and Stegun, formula 7.1.26 (absolute error of erf below 1.5e-7, five orders below the
// tolerance of a bf16 DAG); the Gaussian is shared with the density, so gelu or its derivative costs one exponential
// and one division.  fp32 DAGs keep erff.  Exponential and reciprocal of such programs are the hardware's (base-2
// exponential of x * log2 e: relative error about 1e-7 * (1 + |x|), results below 2^-126 are 0; reciprocal to one unit
// in the last place): a fifth of the instructions of expf and of a division.
#if defined(__HIP_DEVICE_COMPILE__)
CHAIN_HD float vm_exp_fast(float x) { return __expf(x); }
CHAIN_HD float vm_rcp_fast(float x) { return __builtin_amdgcn_rcpf(x); }
#else
CHAIN_HD float vm_exp_fast(float x) { return expf(x); }
CHAIN_HD float vm_rcp_fast(float x) { return 1.f / x; }
#endif
CHAIN_HD void vm_normal_parts(float z, float& cdf, float& pdf) {
    const float t = vm_rcp_fast(1.f + 0.3275911f * 0.70710678f * fabsf(z));
    const float e = vm_exp_fast(-0.5f * z * z);
    const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
    const float tail = 0.5f * poly * e;  // 0.5 * erfc(|z| / sqrt 2)
    cdf = z >= 0.f ? 1.f - tail : tail;
    pdf = 0.39894228f * e;
}
CHAIN_HD float vm_gelu_fast(float x) {
    float cdf, pdf;
    vm_normal_parts(x, cdf, pdf);
    return x * cdf;
}
CHAIN_HD float vm_gelu_grad_fast(float x) {
    float cdf, pdf;
    vm_normal_parts(x, cdf, pdf);
    return cdf + x * pdf;
}

// Sum of the offsets of a position for channel c: terms [b >> 8, (b >> 8) + (b & 255)) that cover c.
CHAIN_HD void vm_offset(const Program& pg, uint16_t b, int c, int& dh, int& dw) {
    dh = 0;
    dw = 0;
    const int first = b >> 8, cnt = b & 255;
    for (int k = 0; k < cnt; k++) {
        uint32_t w[2];
        memcpy(w, &pg.term[first + k], 8);
        const int off = vm_u((int)w[0]), rng = vm_u((int)w[1]);  // (dh, dw) and (c0, c1) as packed halves
        if (c >= (rng & 0xffff) && c < (int)((uint32_t)rng >> 16)) {
            dh += (int16_t)(off & 0xffff);
            dw += (int16_t)((uint32_t)off >> 16);
        }
    }
}

// Row and column of tap t of a KH x KW window (t is a compile-time constant after unrolling, KW is uniform: the
// windows the planner admits are 1, 3 or 5 wide).
CHAIN_HD void vm_tap(int t, int KH, int KW, int& oh, int& ow) {
    const int kh = KW == 3 ? t / 3 : (KW == 5 ? t / 5 : t);
    oh = kh - KH / 2;
    ow = t - kh * KW - KW / 2;
}

// Lanes of a value: channel u < U of the trip, tap t < T (T is uniform: 1, or the taps of a window), pixel v < V.
// The body sees e = (u * TM + t) * V + v and l = t * V + v.
#define CHAIN_EACH(T, e, l, ...)                                                          \
    do {                                                                                  \
        if (TM == 1 || (T) == 1) {                                                        \
            _Pragma("unroll") for (int u_ = 0; u_ < U; u_++) {                            \
                _Pragma("unroll") for (int l = 0; l < V; l++) {                           \
                    const int e = u_ * TM * V + l;                                        \
                    __VA_ARGS__                                                           \
                }                                                                         \
            }                                                                             \
        } else {                                                                          \
            _Pragma("unroll") for (int u_ = 0; u_ < U; u_++) {                            \
                _Pragma("unroll") for (int t_ = 0; t_ < TM; t_++) if (t_ < (T)) {         \
                    _Pragma("unroll") for (int v_ = 0; v_ < V; v_++) {                    \
                        const int l = t_ * V + v_;                                        \
                        const int e = u_ * TM * V + l;                                    \
                        __VA_ARGS__                                                       \
                    }                                                                     \
                }                                                                         \
            }                                                                             \
        }                                                                                 \
    } while (0)

// Register r (uniform) of all U channels <-> X: lanes [0, T * V) of every channel.  Rm: piece 0 of register 0 of this
// thread; rstride: floats between pieces (threads * 4); a register is its U * TM * V lanes in pieces of four.
template <int TM, int V, int U>
CHAIN_HD void vm_reg_read(const float* Rm, int rstride, int r, int T, float* X) {
    constexpr int L = U * TM * V, Q = reg_pieces(L);
    const float* src = Rm + r * Q * rstride;
#pragma unroll
    for (int q = 0; q < Q; q++) {
        bool needed = false;
#pragma unroll
        for (int k = 0; k < 4; k++)
            if (q * 4 + k < L && (q * 4 + k) % (TM * V) < T * V) needed = true;
        if (needed) {
            float w[4];
            memcpy(w, src + q * rstride, 16);
#pragma unroll
            for (int k = 0; k < 4; k++)
                if (q * 4 + k < L) X[q * 4 + k] = w[k];
        }
    }
}
template <int TM, int V, int U>
CHAIN_HD void vm_reg_write(float* Rm, int rstride, int r, int T, const float* X) {
    constexpr int L = U * TM * V, Q = reg_pieces(L);
    float* dst = Rm + r * Q * rstride;
#pragma unroll
    for (int q = 0; q < Q; q++) {
        bool needed = false;
#pragma unroll
        for (int k = 0; k < 4; k++)
            if (q * 4 + k < L && (q * 4 + k) % (TM * V) < T * V) needed = true;
        if (needed) {
            float w[4];
#pragma unroll
            for (int k = 0; k < 4; k++) w[k] = q * 4 + k < L ? X[q * 4 + k] : 0.f;
            memcpy(dst + q * rstride, w, 16);
        }
    }
}

// Which of the thread's V pixels see the image at offset (oh, ow): bit v of the result.  The thread's pixels are a run
// of at most two image rows (V <= W), so the valid ones are at most two runs of bits: no per-pixel arithmetic.
CHAIN_HD uint32_t vm_bits(int lo, int hi) {  // bits [lo, hi), 0 <= lo, hi <= 32
    const uint32_t upto_hi = hi >= 32 ? 0xffffffffu : ((1u << hi) - 1u);
    return hi > lo ? (upto_hi & ~((1u << lo) - 1u)) : 0u;
}
// x where bit v of m is set, else +0 (two bit operations instead of a compare and a select).
CHAIN_HD float vm_keep(float x, uint32_t m, int v) { return vm_bits_to_f32(vm_f32_to_bits(x) & (0u - ((m >> v) & 1u))); }
template <int V>
CHAIN_HD uint32_t vm_valid(const Geo& g, const Thread& th, int oh, int ow) {
    if (!th.active) return 0;
    if (g.whole_rows) {
        // all V pixels lie in row0 (col0 is a multiple of V): the row is inside or not as a whole, and columns fall off only
        // at the row's first pixels (to the left) or last pixels (to the right)
        if ((unsigned)(th.row0 + oh) >= (unsigned)g.H) return 0;
        const int first = -(th.col0 + ow), behind = g.W - th.col0 - ow;
        return vm_bits(first > 0 ? first : 0, behind < V ? behind : V);
    }
    const int n1 = g.W - th.col0 < V ? g.W - th.col0 : V;  // pixels [0, n1) lie in row0, [n1, V) in row0 + 1
    const int first = -(th.col0 + ow), behind = g.W - th.col0 - ow;  // pixel v of row0 has column v - first; valid for first <= v < behind
    uint32_t m = 0;
    if ((unsigned)(th.row0 + oh) < (unsigned)g.H) m |= vm_bits(first > 0 ? first : 0, behind < n1 ? behind : n1);
    if (n1 < V && (unsigned)(th.row0 + 1 + oh) < (unsigned)g.H) {
        // pixel v of row0 + 1 has column v - n1, displaced v - n1 + ow = v - behind + ... : valid for behind <= v < behind + W
        const int lo2 = behind > n1 ? behind : n1, hi2 = behind + g.W < V ? behind + g.W : V;
        m |= vm_bits(lo2, hi2);
    }
    return m;
}

// out[v] = tensor(plane, pixel p0 + v displaced by (oh, ow)), 0 outside the image.  Without displacement nothing is
// masked: what a thread outside the plane reads (zeros, or pixels of another plane) is never stored nor handed over.
template <int V>
CHAIN_HD void vm_load_at(const Tensor& e, const Geo& g, const Thread& th, int plane, int oh, int ow, float* out) {
    if (oh == 0 && ow == 0) {
        vm_load<V, true>(e, plane * g.HW + th.p0, out);
    } else {
        float raw[V];
        vm_load<V, false>(e, plane * g.HW + th.p0 + oh * g.W + ow, raw);
        const uint32_t m = vm_valid<V>(g, th, oh, ow);
#pragma unroll
        for (int v = 0; v < V; v++) out[v] = vm_keep(raw[v], m, v);
    }
}

#if defined(__HIP_DEVICE_COMPILE__)
// The T = KH * KW taps of a window of a bf16 tensor, displaced by (dh, dw), for the thread's V pixels of plane `chan`:
// out[t * V + v], 0 outside the image.  All loads are issued before the first is looked at: one round trip to memory
// for the T taps, not T (tap by tap, each load was followed by its own wait: the fix-up of an access that straddles an
// end of the tensor may overwrite what was loaded).  KHC x KWC: the window as constants (tap geometry folds, the taps
// of a window row share the row test and the taps of a window column the column mask), or 0 x 0 for the window (KH, KW).
template <int TM, int V, int KHC, int KWC>
__device__ __forceinline__ void vm_ld_window_bf16(const Tensor& e, const Geo& g, const Thread& th, int chan, int dh, int dw, int KH, int KW, int T,
                                                  float* out) {
    constexpr int D = V == 1 ? 1 : V / 2;
    if (KHC > 0) {
        KH = KHC;
        KW = KWC;
        T = KHC * KWC;
    }
    uint32_t raw[TM][D];
    int off[TM];
    // Threads that never cross an image row: a tap's row is inside the image or not as a whole (outside, the load is
    // sent to the offset that reads zeros), and its columns fall off at the row's ends only.
    const bool by_rows = g.whole_rows;
    const int centre_off = (chan * g.HW + th.p0) * 2;
#pragma unroll
    for (int t = 0; t < TM; t++)
        if (t < T) {
            int oh, ow;
            vm_tap(t, KH, KW, oh, ow);
            off[t] = centre_off + ((dh + oh) * g.W + dw + ow) * 2;
            if (V == 1) {  // (one element: inside the image or not)
                const bool inside = th.active && (unsigned)(th.row0 + dh + oh) < (unsigned)g.H && (unsigned)(th.col0 + dw + ow) < (unsigned)g.W;
                off[t] = inside ? off[t] : tile::kOob;
            } else if (by_rows) {
                const bool row_inside = th.active && (unsigned)(th.row0 + dh + oh) < (unsigned)g.H;
                off[t] = row_inside ? off[t] : tile::kOob;
            }
            // (each tap's offset in a register of its own: a negative base register plus the tap's distance as the
            // instruction's immediate offset is not what the bounds check expects)
            asm volatile("" : "+v"(off[t]));
            if (V == 4) {
                const vm_u32x2 d = __builtin_amdgcn_raw_buffer_load_b64(e.rs, off[t], 0, 0);
                raw[t][0] = d[0];
                raw[t][D - 1] = d[1];
            } else if (V == 2) {
                raw[t][0] = __builtin_amdgcn_raw_buffer_load_b32(e.rs, off[t], 0, 0);
            } else {
                raw[t][0] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(e.rs, off[t], 0, 0);
            }
        }
    if (V == 1) {
#pragma unroll
        for (int t = 0; t < TM; t++)
            if (t < T) out[t] = tile::lo_f32(raw[t][0]);
        return;
    }
    // An access may straddle an end of the tensor only when the window of this thread reaches across that end: one
    // test for all taps (false for nearly every thread), then tap by tap.
    const int reach = (((KH >> 1) + (dh < 0 ? -dh : dh)) * g.W + (KW >> 1) + (dw < 0 ? -dw : dw)) * 2;
    if (centre_off - reach < 0 || centre_off + reach + 2 * V > e.bytes) {
#pragma unroll
        for (int t = 0; t < TM; t++)
            if (t < T && tile::straddles_an_end(off[t], 2 * V, e.bytes)) {
#pragma unroll
                for (int k = 0; k < D; k++)
                    raw[t][k] = tile::elem_b16(e.rs, off[t] + 4 * k, e.bytes) | (tile::elem_b16(e.rs, off[t] + 4 * k + 2, e.bytes) << 16);
            }
    }
    if (by_rows) {
        // pixel v of a tap in window column j is inside for first <= v < behind: a mask over the packed pairs, then the
        // pairs are taken apart
        constexpr int NM = KWC > 0 ? KWC : 1;
        uint32_t cm[NM][D];
#pragma unroll
        for (int t = 0; t < TM; t++)
            if (t < T) {
                int oh, ow;
                vm_tap(t, KH, KW, oh, ow);
                const int j = KWC > 0 ? ow + KWC / 2 : 0;
                if (KWC == 0 || t < KWC) {  // (first window row: the masks of its columns serve the rows below)
                    const int first = -(th.col0 + dw + ow), behind = g.W - th.col0 - dw - ow;
                    const uint32_t m = vm_bits(first > 0 ? first : 0, behind < V ? behind : V);
#pragma unroll
                    for (int k = 0; k < D; k++) {
                        const uint32_t lo = (uint32_t)((int32_t)(m << (31 - 2 * k)) >> 31), hi = (uint32_t)((int32_t)(m << (30 - 2 * k)) >> 31);
                        cm[j][k] = (lo & 0xffffu) | (hi & 0xffff0000u);
                    }
                }
#pragma unroll
                for (int k = 0; k < D; k++) {
                    const uint32_t kept = raw[t][k] & cm[j][k];
                    out[t * V + 2 * k] = tile::lo_f32(kept);
                    out[t * V + 2 * k + 1] = tile::hi_f32(kept);
                }
            }
    } else {
#pragma unroll
        for (int t = 0; t < TM; t++)
            if (t < T) {
                int oh, ow;
                vm_tap(t, KH, KW, oh, ow);
                const bool centre = dh + oh == 0 && dw + ow == 0;  // (uniform; without displacement nothing is masked)
                const uint32_t m = centre ? 0xffffffffu : vm_valid<V>(g, th, dh + oh, dw + ow);
#pragma unroll
                for (int k = 0; k < D; k++) {
                    out[t * V + 2 * k] = vm_keep(tile::lo_f32(raw[t][k]), m, 2 * k);
                    out[t * V + 2 * k + 1] = vm_keep(tile::hi_f32(raw[t][k]), m, 2 * k + 1);
                }
            }
    }
}
#endif

// What an instruction needs besides its own fields.
struct Env {
    int c = 0;        // first channel of the trip; channel u of the thread is c + u
    int h = 0;        // channels of the trip that exist (0 .. U)
    bool pro = false; // the prologue of a pass (once per workgroup item, not per channel)
    bool fast = false; // Program::fast_math
    int np = 0;       // persistent floats per pixel and channel
    int pstride = 0;  // floats between consecutive persistent floats of a thread (the workgroup's size)
    int rstride = 0;  // floats between consecutive register pieces of a thread
};

// The loads of OP_LD / OP_BINLD: lanes [0, T) of every channel of the trip into dst.
template <int TM, int V, int U>
CHAIN_HD void vm_ld(const Program& pg, const Geo& g, const Instr& I, const Env& ev, const Thread& th, float* dst, int T) {
    constexpr int TV = TM * V;
    const Tensor e = vm_tensor(pg, g, I.a);
#pragma unroll
    for (int u = 0; u < U; u++)
        if (u < ev.h) {
            int dh, dw;
            vm_offset(pg, I.b, ev.c + u, dh, dw);
            const int chan = (th.n * g.C + ev.c + u) * e.T;  // first plane of (image, channel): uniform
            if (I.kind & kWin) {
                const int KH = I.r >> 4, KW = I.r & 15;
#if defined(__HIP_DEVICE_COMPILE__)
                if ((V == 4 || V == 2 || V == 1) && e.bf16) {
                    // (the common windows with their sizes as constants: tap geometry folds, taps of one window row share
                    // the row test and taps of one window column the column masks)
                    float* out = dst + u * TV;
                    if (TM >= 9 && KH == 3 && KW == 3 && T == 9) vm_ld_window_bf16<TM, V, (TM >= 9 ? 3 : 0), (TM >= 9 ? 3 : 0)>(e, g, th, chan, dh, dw, 3, 3, 9, out);
                    else if (TM >= 25 && KH == 5 && KW == 5 && T == 25) vm_ld_window_bf16<TM, V, (TM >= 25 ? 5 : 0), (TM >= 25 ? 5 : 0)>(e, g, th, chan, dh, dw, 5, 5, 25, out);
                    else vm_ld_window_bf16<TM, V, 0, 0>(e, g, th, chan, dh, dw, KH, KW, T, out);
                    continue;
                }
#endif
#pragma unroll
                for (int t = 0; t < TM; t++)
                    if (t < T) {
                        int oh, ow;
                        vm_tap(t, KH, KW, oh, ow);
                        vm_load_at<V>(e, g, th, chan, dh + oh, dw + ow, dst + u * TV + t * V);
                    }
            } else {
#pragma unroll
                for (int t = 0; t < TM; t++)
                    if (t < T) {
                        const int te = (I.kind & kExtTaps) ? (t < e.T ? t : t % e.T) : 0;
                        vm_load_at<V>(e, g, th, chan + te, dh, dw, dst + u * TV + t * V);
                    }
            }
        }
}

// A = blend(X, A) (x_lhs) or blend(A, X), lanes [0, T) of every channel.  min and max return the same value whichever
// side is the LHS; the sides matter for sub only.
template <int TM, int V, int U>
CHAIN_HD void vm_blend_lanes(int kind, bool x_lhs, const float* X, float* A, int T) {
    switch (kind) {
    case 0: CHAIN_CASE; CHAIN_EACH(T, e, l, A[e] = X[e] + A[e];); break;
    case 1: CHAIN_CASE; CHAIN_EACH(T, e, l, A[e] = X[e] * A[e];); break;
    case 2:
        CHAIN_CASE;
        if (x_lhs) CHAIN_EACH(T, e, l, A[e] = X[e] - A[e];);
        else CHAIN_EACH(T, e, l, A[e] = A[e] - X[e];);
        break;
    case 3: CHAIN_CASE; CHAIN_EACH(T, e, l, A[e] = X[e] <= A[e] ? X[e] : A[e];); break;
    default: CHAIN_CASE; CHAIN_EACH(T, e, l, A[e] = X[e] >= A[e] ? X[e] : A[e];); break;
    }
}

// Every instruction except OP_XADD.  Pm: this thread's persistent floats.  A float that lives across the channel loop
// (softmax statistics, the sums of a softmax's adjoint: written by the prologue and the OP_SMC instructions) exists once,
// float k of pixel v at Pm[(k * V + v) * pstride]; an accumulator of one channel (OP_PSET in a body, OP_PADD, OP_PLD,
// OP_XADD) once per channel u of the trip, at Pm[((u * np + k) * V + v) * pstride].  Rm: its registers (vm_reg_read).
// TC: the lanes of the instruction as a constant (the loops over the taps then carry no test per tap), or 0 for I.T.
template <int TM, int V, int U, int TC>
CHAIN_HD void vm_exec_lanes(const Program& pg, const Geo& g, const Instr& I, const Env& ev, const Thread& th, State<TM, V, U>& st, float* Pm, float* Rm) {
    float* A = st.A;
    const int T = TC > 0 ? TC : I.T;
    const int pstride = ev.pstride, rstride = ev.rstride;
    constexpr int TV = TM * V;
    float X[U * TV];
    switch (I.op) {
    case OP_LD:
        CHAIN_CASE;
        vm_ld<TM, V, U>(pg, g, I, ev, th, A, T);
        break;
    case OP_BINLD: {
        CHAIN_CASE;
        const bool sc = I.kind & kBinLdLoadedScalar;
        vm_ld<TM, V, U>(pg, g, I, ev, th, X, sc ? 1 : T);
        if (TM > 1 && sc) CHAIN_EACH(T, e, l, X[e] = X[e - l + l % V];);
        vm_blend_lanes<TM, V, U>((I.kind >> kBinLdKindShift) & 7, (I.kind & kBinLdLoadedIsLhs) != 0, X, A, T);
        break;
    }
    case OP_MASK: {
        CHAIN_CASE;
#pragma unroll
        for (int u = 0; u < U; u++)
            if (u < ev.h) {
                int dh, dw;
                vm_offset(pg, I.b, ev.c + u, dh, dw);
                if (I.kind & kWin) {
                    const int KH = I.r >> 4, KW = I.r & 15;
#pragma unroll
                    for (int t = 0; t < TM; t++)
                        if (t < T) {
                            int oh, ow;
                            vm_tap(t, KH, KW, oh, ow);
                            const uint32_t m = vm_valid<V>(g, th, dh + oh, dw + ow);
#pragma unroll
                            for (int v = 0; v < V; v++) A[u * TV + t * V + v] = vm_keep(A[u * TV + t * V + v], m, v);
                        }
                } else {
                    const uint32_t m = vm_valid<V>(g, th, dh, dw);
#pragma unroll
                    for (int t = 0; t < TM; t++)
                        if (t < T) {
#pragma unroll
                            for (int v = 0; v < V; v++) A[u * TV + t * V + v] = vm_keep(A[u * TV + t * V + v], m, v);
                        }
                }
            }
        break;
    }
    case OP_UN:
        switch (I.kind) {
        case 0: CHAIN_CASE; CHAIN_EACH(T, e, l, A[e] = fmaxf(A[e], 0.f);); break;
        case 1: CHAIN_CASE; CHAIN_EACH(T, e, l, A[e] = fabsf(A[e]);); break;
        case 2:
            CHAIN_CASE;
            if (ev.fast) CHAIN_EACH(T, e, l, A[e] = vm_gelu_fast(A[e]););
            else CHAIN_EACH(T, e, l, A[e] = vm_gelu(A[e]););
            break;
        case 4: CHAIN_CASE; CHAIN_EACH(T, e, l, A[e] = sinf(A[e]);); break;
        case kUnNeg: CHAIN_CASE; CHAIN_EACH(T, e, l, A[e] = -A[e];); break;
        default:
            CHAIN_CASE;
            if (ev.fast) CHAIN_EACH(T, e, l, A[e] = vm_exp_fast(fminf(fmaxf(A[e], I.f0), I.f1)););
            else CHAIN_EACH(T, e, l, A[e] = expf(fminf(fmaxf(A[e], I.f0), I.f1)););
            break;
        }
        break;
    case OP_MOVR:
        CHAIN_CASE;
        vm_reg_write<TM, V, U>(Rm, rstride, I.r, T, A);
        break;
    case OP_MOVA:
        CHAIN_CASE;
        vm_reg_read<TM, V, U>(Rm, rstride, I.r, T, A);
        break;
    case OP_BIN: {
        CHAIN_CASE;
        const int kind = I.kind & 7;
        const bool reg_lhs = I.kind & kBinRegIsLhs, reg_sc = I.kind & kBinRegScalar, acc_sc = I.kind & kBinAccScalar;
        vm_reg_read<TM, V, U>(Rm, rstride, I.r, reg_sc ? 1 : T, X);
        if (TM > 1 && reg_sc) CHAIN_EACH(T, e, l, X[e] = X[e - l + l % V];);
        if (TM > 1 && acc_sc) CHAIN_EACH(T, e, l, A[e] = A[e - l + l % V];);
        vm_blend_lanes<TM, V, U>(kind, reg_lhs, X, A, T);
        break;
    }
    case OP_FOLD: {
        CHAIN_CASE;
#pragma unroll
        for (int u = 0; u < U; u++) {
            float* Au = A + u * TV;
            if (I.kind == 2) {
#pragma unroll
                for (int t = 1; t < TM; t++)
                    if (t < T) {
#pragma unroll
                        for (int v = 0; v < V; v++) Au[v] = Au[t * V + v] > Au[v] ? Au[t * V + v] : Au[v];
                    }
            } else {
#pragma unroll
                for (int t = 1; t < TM; t++)
                    if (t < T) {
#pragma unroll
                        for (int v = 0; v < V; v++) Au[v] += Au[t * V + v];
                    }
                if (I.kind == 1) {
                    // sum / T as a product with the reciprocal and one correction step from the remainder: the quotient
                    // to within one unit in the last place, a fifth of the instructions of a division per pixel
                    // (infinities and NaN come out as a division gives them)
                    const float n = (float)T;
#if defined(__HIP_DEVICE_COMPILE__)
                    const float r = 1.f / n;
#pragma unroll
                    for (int v = 0; v < V; v++) {
                        const float q = Au[v] * r;
                        Au[v] = __builtin_amdgcn_div_fixupf(fmaf(fmaf(-n, q, Au[v]), r, q), n, Au[v]);
                    }
#else
                    for (int v = 0; v < V; v++) Au[v] /= n;
#endif
                }
            }
        }
        break;
    }
    case OP_SMT: {
        CHAIN_CASE;
#pragma unroll
        for (int u = 0; u < U; u++) {
            float* Au = A + u * TV;
#pragma unroll
            for (int v = 0; v < V; v++) {
                float m = Au[v];
#pragma unroll
                for (int t = 1; t < TM; t++)
                    if (t < T) m = fmaxf(m, Au[t * V + v]);
                float z = 0.f;
                if (ev.fast) {
#pragma unroll
                    for (int t = 0; t < TM; t++)
                        if (t < T) {
                            Au[t * V + v] = vm_exp_fast(Au[t * V + v] - m);
                            z += Au[t * V + v];
                        }
                    const float rz = vm_rcp_fast(z);
#pragma unroll
                    for (int t = 0; t < TM; t++)
                        if (t < T) Au[t * V + v] = Au[t * V + v] * rz;
                    continue;
                }
#pragma unroll
                for (int t = 0; t < TM; t++)
                    if (t < T) {
                        Au[t * V + v] = expf(Au[t * V + v] - m);
                        z += Au[t * V + v];
                    }
#pragma unroll
                for (int t = 0; t < TM; t++)
                    if (t < T) Au[t * V + v] = Au[t * V + v] / z;
            }
        }
        break;
    }
    case OP_ST: {
        CHAIN_CASE;
        if (!th.own) break;
        const Tensor e = vm_tensor(pg, g, I.a);
#pragma unroll
        for (int u = 0; u < U; u++)
            if (u < ev.h) {
                const int chan = (th.n * g.C + ev.c + u) * e.T;
#pragma unroll
                for (int t = 0; t < TM; t++)
                    if (t < T) vm_store<V>(e, (chan + t) * g.HW + th.p0, A + u * TV + t * V, (I.kind & kStAdd) != 0);
            }
        break;
    }
    case OP_UNBX:
        CHAIN_CASE;
        vm_reg_read<TM, V, U>(Rm, rstride, I.r, T, X);
        switch (I.kind) {
        case 0: CHAIN_CASE; CHAIN_EACH(T, e, l, A[e] = A[e] > 0.f ? X[e] : 0.f;); break;
        case 1: CHAIN_CASE; CHAIN_EACH(T, e, l, A[e] = X[e] * vm_sign(A[e]);); break;
        case 2:
            CHAIN_CASE;
            if (ev.fast) CHAIN_EACH(T, e, l, A[e] = X[e] * vm_gelu_grad_fast(A[e]););
            else CHAIN_EACH(T, e, l, A[e] = X[e] * vm_gelu_grad(A[e]););
            break;
        case 4: CHAIN_CASE; CHAIN_EACH(T, e, l, A[e] = X[e] * cosf(A[e]);); break;
        case kUnNeg: CHAIN_CASE; CHAIN_EACH(T, e, l, A[e] = -X[e];); break;
        default:
            CHAIN_CASE;
            if (ev.fast) CHAIN_EACH(T, e, l, A[e] = (A[e] > I.f0 && A[e] < I.f1) ? X[e] * vm_exp_fast(A[e]) : 0.f;);
            else CHAIN_EACH(T, e, l, A[e] = (A[e] > I.f0 && A[e] < I.f1) ? X[e] * expf(A[e]) : 0.f;);
            break;
        }
        break;
    case OP_BING: {
        CHAIN_CASE;
        const int kind = I.kind & 7;
        const bool rhs_side = I.kind & kBingRhsSide, l_sc = I.kind & kBingLhsScalar, r_sc = I.kind & kBingRhsScalar;
        vm_reg_read<TM, V, U>(Rm, rstride, I.r, l_sc ? 1 : T, X);
        if (TM > 1 && l_sc) CHAIN_EACH(T, e, l, X[e] = X[e - l + l % V];);
        if (TM > 1 && r_sc) CHAIN_EACH(T, e, l, A[e] = A[e - l + l % V];);
        // X: the LHS value, A: the RHS value; the result is d blend / d side (a tie of min / max belongs to the LHS)
        switch (kind) {
        case 0: CHAIN_CASE; CHAIN_EACH(T, e, l, A[e] = 1.f;); break;
        case 1:
            CHAIN_CASE;
            if (!rhs_side) break;  // d (l * r) / d l = r, which A holds
            CHAIN_EACH(T, e, l, A[e] = X[e];);
            break;
        case 2:
            CHAIN_CASE;
            if (rhs_side) CHAIN_EACH(T, e, l, A[e] = -1.f;);
            else CHAIN_EACH(T, e, l, A[e] = 1.f;);
            break;
        case 3:
            CHAIN_CASE;
            if (rhs_side) CHAIN_EACH(T, e, l, A[e] = X[e] <= A[e] ? 0.f : 1.f;);
            else CHAIN_EACH(T, e, l, A[e] = X[e] <= A[e] ? 1.f : 0.f;);
            break;
        default:
            CHAIN_CASE;
            if (rhs_side) CHAIN_EACH(T, e, l, A[e] = X[e] >= A[e] ? 0.f : 1.f;);
            else CHAIN_EACH(T, e, l, A[e] = X[e] >= A[e] ? 1.f : 0.f;);
            break;
        }
        break;
    }
    case OP_SMTBX:
        CHAIN_CASE;
        vm_reg_read<TM, V, U>(Rm, rstride, I.r, T, X);
#pragma unroll
        for (int u = 0; u < U; u++) {
            float* Au = A + u * TV;
            const float* Xu = X + u * TV;
#pragma unroll
            for (int v = 0; v < V; v++) {
                float dot = 0.f;
#pragma unroll
                for (int t = 0; t < TM; t++)
                    if (t < T) dot += Xu[t * V + v] * Au[t * V + v];
#pragma unroll
                for (int t = 0; t < TM; t++)
                    if (t < T) Au[t * V + v] = Au[t * V + v] * (Xu[t * V + v] - dot);
            }
        }
        break;
    case OP_FOLDBX:
        CHAIN_CASE;
        vm_reg_read<TM, V, U>(Rm, rstride, I.r, 1, X);
        if (I.kind == 2) {
#pragma unroll
            for (int u = 0; u < U; u++) {
                float* Au = A + u * TV;
#pragma unroll
                for (int v = 0; v < V; v++) {
                    const float gr = X[u * TV + v];
                    int best = 0;
                    float m = Au[v];
#pragma unroll
                    for (int t = 1; t < TM; t++)
                        if (t < T && Au[t * V + v] > m) {
                            m = Au[t * V + v];
                            best = t;
                        }
#pragma unroll
                    for (int t = 0; t < TM; t++)
                        if (t < T) Au[t * V + v] = t == best ? gr : 0.f;
                }
            }
        } else {
            if (I.kind == 1) {
#pragma unroll
                for (int u = 0; u < U; u++)
#pragma unroll
                    for (int v = 0; v < V; v++) X[u * TV + v] = X[u * TV + v] / (float)T;
            }
            CHAIN_EACH(T, e, l, A[e] = X[e - l + l % V];);
        }
        break;
    case OP_PSET:
        CHAIN_CASE;
        if (ev.pro) {
#pragma unroll
            for (int t = 0; t < TM; t++)
                if (t < T) {
#pragma unroll
                    for (int v = 0; v < V; v++) Pm[((I.a + t) * V + v) * pstride] = I.f0;
                }
        } else {
            CHAIN_EACH(T, e, l, Pm[(((e - l) / TV * ev.np + I.a) * V + l) * pstride] = I.f0;);
        }
        break;
    case OP_PADD: {
        CHAIN_CASE;
        const int Tb = I.b;
#pragma unroll
        for (int u = 0; u < U; u++)
#pragma unroll
            for (int t = 0; t < TM; t++)
                if (t < T) {
                    const int tp = t < Tb ? t : t % Tb;
#pragma unroll
                    for (int v = 0; v < V; v++) Pm[((u * ev.np + I.a + tp) * V + v) * pstride] += A[u * TV + t * V + v];
                }
        break;
    }
    case OP_PLD:
        CHAIN_CASE;
        CHAIN_EACH(T, e, l, A[e] = Pm[(((e - l) / TV * ev.np + I.a) * V + l) * pstride];);
        break;
    case OP_SMCSTAT:
        CHAIN_CASE;
        if (ev.fast) {
            // the channels of the trip join the running maximum and sum together: one update of the pair per pixel and
            // trip, U + 1 exponentials for U channels, no branch on the data
#pragma unroll
            for (int t = 0; t < TM; t++)
                if (t < T) {
#pragma unroll
                    for (int v = 0; v < V; v++) {
                        float& m = Pm[((I.a + t) * V + v) * pstride];
                        float& z = Pm[((I.a + T + t) * V + v) * pstride];
                        const float before = m;
                        float top = before;
#pragma unroll
                        for (int u = 0; u < U; u++)
                            if (u < ev.h) top = fmaxf(top, A[u * TV + t * V + v]);
                        float sum = z * vm_exp_fast(before - top);  // (before = -inf at the first channel: 0 * 0)
#pragma unroll
                        for (int u = 0; u < U; u++)
                            if (u < ev.h) sum += vm_exp_fast(A[u * TV + t * V + v] - top);
                        m = top;
                        z = sum;
                    }
                }
            break;
        }
#pragma unroll
        for (int u = 0; u < U; u++)
            if (u < ev.h) {
#pragma unroll
                for (int t = 0; t < TM; t++)
                    if (t < T) {
#pragma unroll
                        for (int v = 0; v < V; v++) {
                            float& m = Pm[((I.a + t) * V + v) * pstride];
                            float& z = Pm[((I.a + T + t) * V + v) * pstride];
                            const float val = A[u * TV + t * V + v];
                            if (val > m) {
                                z = z * expf(m - val) + 1.f;  // (m = -inf at the first channel: z = 0 * 0 + 1)
                                m = val;
                            } else {
                                z += expf(val - m);
                            }
                        }
                    }
            }
        break;
    case OP_SMCAPPLY:
        CHAIN_CASE;
        if (ev.fast) CHAIN_EACH(T, e, l, A[e] = vm_exp_fast(A[e] - Pm[(I.a * V + l) * pstride]) * vm_rcp_fast(Pm[((I.a + T) * V + l) * pstride]););
        else CHAIN_EACH(T, e, l, A[e] = expf(A[e] - Pm[(I.a * V + l) * pstride]) / Pm[((I.a + T) * V + l) * pstride];);
        break;
    case OP_SMCDOT:
        CHAIN_CASE;
        vm_reg_read<TM, V, U>(Rm, rstride, I.r, T, X);
#pragma unroll
        for (int u = 0; u < U; u++)
            if (u < ev.h) {
#pragma unroll
                for (int t = 0; t < TM; t++)
                    if (t < T) {
#pragma unroll
                        for (int v = 0; v < V; v++) Pm[((I.a + t) * V + v) * pstride] += A[u * TV + t * V + v] * X[u * TV + t * V + v];
                    }
            }
        break;
    case OP_SMCBX:
        CHAIN_CASE;
        vm_reg_read<TM, V, U>(Rm, rstride, I.r, T, X);
        CHAIN_EACH(T, e, l, A[e] = A[e] * (X[e] - Pm[(I.a * V + l) * pstride]););
        break;
    default: break;
    }
}

// An instruction over all TM lanes of the instance (the common case of a program with taps) runs the copy of the
// dispatch whose tap loops are straight-line code.  (Not the one-pixel instances: the second copy cost them 16-18
// registers and with those a wavefront per SIMD.)
template <int TM, int V, int U>
CHAIN_HD void vm_exec(const Program& pg, const Geo& g, const Instr& I, const Env& ev, const Thread& th, State<TM, V, U>& st, float* Pm, float* Rm) {
    constexpr int TC = TM > 1 && V > 1 ? TM : 0;
    if (TC > 0 && I.T == TM) vm_exec_lanes<TM, V, U, TC>(pg, g, I, ev, th, st, Pm, Rm);
    else vm_exec_lanes<TM, V, U, 0>(pg, g, I, ev, th, st, Pm, Rm);
}

// OP_XADD of channel u, first half: the thread's lanes go to the hand-over buffer of its slice (lane t of local pixel q
// at buf[t * npx + q]).
template <int TM, int V>
CHAIN_HD void vm_xadd_write(const Geo& g, const Instr& I, const Thread& th, const float* Au, float* buf) {
#pragma unroll
    for (int t = 0; t < TM; t++)
        if (t < I.T) {
#pragma unroll
            for (int v = 0; v < V; v++) buf[t * g.npx + th.ptid * V + v] = Au[t * V + v];
        }
}

// OP_XADD of channel u, second half (after a barrier): P[a (+ t)] of every pixel of the thread collects lane t of the
// pixel whose load at offset (dh, dw) [+ window tap t] read it, if that pixel is inside the image and inside the pixels
// the slice computes (the planner sizes the halo so that an owned pixel never misses one).  Fixed order: deterministic.
// Pu: the persistent floats of this thread and channel.
template <int TM, int V>
CHAIN_HD void vm_xadd_gather(const Geo& g, const Instr& I, int dh, int dw, const Thread& th, const float* buf, float* Pu, int pstride) {
#pragma unroll
    for (int t = 0; t < TM; t++)
        if (t < I.T) {
            int oh = dh, ow = dw;
            if (I.kind & kWin) {
                int th_, tw_;
                vm_tap(t, I.r >> 4, I.r & 15, th_, tw_);
                oh += th_;
                ow += tw_;
            }
            // the source of pixel (r, c) is pixel (r - oh, c - ow)
            const uint32_t m = vm_valid<V>(g, th, -oh, -ow);
            const int slot = I.a + ((I.kind & kExtTaps) ? t : 0);
#pragma unroll
            for (int v = 0; v < V; v++) {
                const int src = th.ptid * V + v - (oh * g.W + ow);
                if (((m >> v) & 1u) && src >= 0 && src < g.npx) Pu[(slot * V + v) * pstride] += buf[t * g.npx + src];
            }
        }
}

// Combination of the slices' partial results of lane e (= t * V + v) of a Red (see chain_isa.hpp) for the pixels of
// thread `ptid`: float k of slice s is at Pbase[(k * V + v) * pstride + s * pix_threads + ptid].  kind 0 returns the
// total maximum and sum.
template <int V>
CHAIN_HD void vm_combine(const Red& R, int e, int S, int PT, const float* Pbase, int pstride, int ptid, float& v0, float& v1) {
    const float* p0 = Pbase + (R.slot * V + e) * pstride + ptid;
    if (R.kind == 0) {
        const float* p1 = Pbase + ((R.slot + R.T) * V + e) * pstride + ptid;
        float m = -INFINITY;
        for (int s = 0; s < S; s++) m = fmaxf(m, p0[s * PT]);
        float z = 0.f;
        for (int s = 0; s < S; s++) {
            const float zs = p1[s * PT];
            if (zs > 0.f) z += zs * expf(p0[s * PT] - m);  // (a slice without channels has no sum and no maximum)
        }
        v0 = m;
        v1 = z;
    } else {
        float d = 0.f;
        for (int s = 0; s < S; s++) d += p0[s * PT];
        v0 = d;
        v1 = 0.f;
    }
}

}  // namespace chain
}  // namespace canvas
