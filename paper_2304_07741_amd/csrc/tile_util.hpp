// Device helpers shared by the MFMA tile kernels: buffer addressing, bf16 packing, operand gathering,
// the border-mask table.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace canvas {
namespace tile {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __amdgpu_buffer_rsrc_t rsrc_t;

constexpr int kOob = -16;     // byte offset outside every buffer: loads give 0, stores are dropped

// Raw buffer over `bytes` bytes at p (bytes < 2^31): accesses at offsets outside [0, bytes) are discarded by hardware.
__device__ __forceinline__ rsrc_t make_rsrc(const void* p, int bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 bload16(rsrc_t r, int byte_off) { return __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0); }
__device__ __forceinline__ void bstore16(rsrc_t r, int byte_off, u32x4 v) { __builtin_amdgcn_raw_buffer_store_b128(v, r, byte_off, 0, 0); }
// Streaming variants (non-temporal hint) for data that is touched once.
__device__ __forceinline__ u32x4 bload16_nt(rsrc_t r, int byte_off) { return __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 2); }
__device__ __forceinline__ void bstore16_nt(rsrc_t r, int byte_off, u32x4 v) { __builtin_amdgcn_raw_buffer_store_b128(v, r, byte_off, 0, 2); }

// The chip's 8 XCDs (32 compute units and one L2 each) take the workgroups of a launch in turn: workgroup number b
// (x fastest, then y) runs on XCD b % 8.  Kernels whose neighbouring tiles read common data (window halos, the same
// rows for several output tiles) hand out their tiles in this order instead: XCD k works on one contiguous eighth of
// the tile sequence, so what neighbours share is found in its own L2 instead of being fetched once per XCD.
__device__ __forceinline__ unsigned xcd_sequence() {  // this workgroup's place in that order, 0 .. gridDim.x * gridDim.y - 1
    const unsigned gx = gridDim.x, total = gx * gridDim.y;
    const unsigned lin = blockIdx.y * gx + blockIdx.x;
    const unsigned xcd = lin & 7u, idx = lin >> 3, per = total >> 3, rem = total & 7u;
    return xcd * per + (xcd < rem ? xcd : rem) + idx;
}
__device__ __forceinline__ void xcd_order(unsigned& bx, unsigned& by) {  // the place as grid coordinates, x fastest
    const unsigned seq = xcd_sequence();
    by = seq / gridDim.x;
    bx = seq - by * gridDim.x;
}

// A 16-byte access that begins before the buffer is dropped as a whole by the hardware; one that runs past
// the end keeps the dwords that lie completely inside and loses the rest, including a bf16 element that
// shares its dword with the end (measured on gfx950).  Only a shifted access at the very start or end of a
// tensor can be partly out of range while holding valid pixels; the lanes concerned re-read such a register
// element by element (an element is either inside or outside).
__device__ __forceinline__ bool straddles_an_end(int byte_off, int len, int bytes) {
    return (byte_off < 0 && byte_off + len > 0) || (byte_off < bytes && byte_off + len > bytes);
}
// One element of `len` bytes at byte offset o, 0 when it is outside the buffer.  The offset handed to the
// hardware is either inside or the fixed out-of-range value: a negative base plus an immediate is never
// left to the instruction's own offset arithmetic.
__device__ __forceinline__ uint32_t elem_b16(rsrc_t r, int o, int bytes) {
    return (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r, (o >= 0 && o + 2 <= bytes) ? o : kOob, 0, 0) & 0xffffu;
}
__device__ __forceinline__ uint32_t elem_b32(rsrc_t r, int o, int bytes) {
    return __builtin_amdgcn_raw_buffer_load_b32(r, (o >= 0 && o + 4 <= bytes) ? o : kOob, 0, 0);
}
__device__ __forceinline__ void reload_if_partial(u32x4& v, rsrc_t r, int byte_off, int bytes) {
    if (straddles_an_end(byte_off, 16, bytes)) {
#pragma unroll
        for (int k = 0; k < 4; k++) v[k] = elem_b16(r, byte_off + 4 * k, bytes) | (elem_b16(r, byte_off + 4 * k + 2, bytes) << 16);
    }
}
// The same for a 4-byte access of two bf16 elements, and for a 16-byte access of four fp32 elements.
__device__ __forceinline__ void reload_pair_if_partial(uint32_t& v, rsrc_t r, int byte_off, int bytes) {
    if (straddles_an_end(byte_off, 4, bytes)) v = elem_b16(r, byte_off, bytes) | (elem_b16(r, byte_off + 2, bytes) << 16);
}
__device__ __forceinline__ void reload_f32x4_if_partial(u32x4& v, rsrc_t r, int byte_off, int bytes) {
    if (straddles_an_end(byte_off, 16, bytes)) {
#pragma unroll
        for (int k = 0; k < 4; k++) v[k] = elem_b32(r, byte_off + 4 * k, bytes);
    }
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    float2_t f = {a, b};
    bf16x2_t h = __builtin_convertvector(f, bf16x2_t);
    uint32_t u;
    __builtin_memcpy(&u, &h, 4);
    return u;
}
__device__ __forceinline__ float lo_f32(uint32_t d) { return __uint_as_float(d << 16); }
__device__ __forceinline__ float hi_f32(uint32_t d) { return __uint_as_float(d & 0xffff0000u); }
template <int Q>
__device__ __forceinline__ float elem_f32(const u32x4& v) {
    return (Q & 1) ? hi_f32(v[Q >> 1]) : lo_f32(v[Q >> 1]);
}

__device__ __forceinline__ short4_t as_short4(uint32_t lo, uint32_t hi) {
    uint32_t t[2] = {lo, hi};
    short4_t r;
    __builtin_memcpy(&r, t, 8);
    return r;
}

// Element Q (0..7) of each of four 16-byte registers -> one MFMA operand (4 bf16).
template <int Q>
__device__ __forceinline__ short4_t gather4(const u32x4& a, const u32x4& b, const u32x4& c, const u32x4& d) {
    constexpr uint32_t sel = (Q & 1) ? 0x07060302u : 0x05040100u;
    return as_short4(__builtin_amdgcn_perm(b[Q >> 1], a[Q >> 1], sel), __builtin_amdgcn_perm(d[Q >> 1], c[Q >> 1], sel));
}
__device__ __forceinline__ void gather_all(const u32x4 (&x)[4], short4_t (&out)[8]) {
    out[0] = gather4<0>(x[0], x[1], x[2], x[3]);
    out[1] = gather4<1>(x[0], x[1], x[2], x[3]);
    out[2] = gather4<2>(x[0], x[1], x[2], x[3]);
    out[3] = gather4<3>(x[0], x[1], x[2], x[3]);
    out[4] = gather4<4>(x[0], x[1], x[2], x[3]);
    out[5] = gather4<5>(x[0], x[1], x[2], x[3]);
    out[6] = gather4<6>(x[0], x[1], x[2], x[3]);
    out[7] = gather4<7>(x[0], x[1], x[2], x[3]);
}

__device__ __forceinline__ short4_t pack4(float a, float b, float c, float d) { return as_short4(pack_bf16(a, b), pack_bf16(c, d)); }

__device__ __forceinline__ float4_t mfma16(short4_t a, short4_t b, float4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b, c, 0, 0, 0);
}

// The gfx950 form with twice the contraction depth: 8 bf16 per lane and operand, K = 32.  Lane l holds row (column)
// l % 16 and the 8 contraction indices of lane group l / 16, in both operands alike, so two K = 16 operand pairs
// (a0, b0) and (a1, b1) that add into one accumulator are one K = 32 step: a0 | a1 against b0 | b1.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
__device__ __forceinline__ float4_t mfma32(short4_t a0, short4_t a1, short4_t b0, short4_t b1, float4_t c) {
    const short4_t av[2] = {a0, a1}, bv[2] = {b0, b1};
    bf16x8_t a, b;
    __builtin_memcpy(&a, av, 16);
    __builtin_memcpy(&b, bv, 16);
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
// Eight bf16 in four dwords against eight bf16 in four dwords.
__device__ __forceinline__ float4_t mfma32(const u32x4& a, const u32x4& b, float4_t c) {
    bf16x8_t av, bv;
    __builtin_memcpy(&av, &a, 16);
    __builtin_memcpy(&bv, &b, 16);
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bv, c, 0, 0, 0);
}

// kMaskLut.m[b] = the four dword masks that keep the bf16 elements whose bit is set in the 8-bit pattern b.
struct alignas(16) MaskLut {
    uint32_t m[256][4];
};
constexpr MaskLut make_mask_lut() {
    MaskLut t{};
    for (int b = 0; b < 256; b++)
        for (int k = 0; k < 4; k++)
            t.m[b][k] = (((b >> (2 * k)) & 1) ? 0x0000ffffu : 0u) | (((b >> (2 * k + 1)) & 1) ? 0xffff0000u : 0u);
    return t;
}
__device__ const MaskLut kMaskLut = make_mask_lut();

// Keeps a loaded value live at this point, so that the compiler issues its load before, not after, the
// work that follows (it would otherwise sink loads into the block that first uses them).
__device__ __forceinline__ void pin(u32x4& v) { asm volatile("" : "+v"(v)); }

// The four dword masks of an 8-bit validity pattern.
__device__ __forceinline__ u32x4 mask_of(uint32_t bits) { return reinterpret_cast<const u32x4*>(kMaskLut.m)[bits]; }

}  // namespace tile
}  // namespace canvas
