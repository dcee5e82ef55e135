// Fused-chain kernels: one workgroup = one image x one tile of the image plane (plus a halo in backward programs) x one
// range of channels; one thread = V consecutive pixels; the program (chain_isa.hpp) arrives in the kernel arguments and
// is interpreted with workgroup-uniform control flow.  A tensor access is one vector access of V elements per thread,
// coalesced along the plane (the innermost dims of NCHW); stencil offsets are address offsets of those accesses;
// reductions over taps stay in registers; the statistics of a softmax over channels and the gradient hand-over of
// shifted loads live in LDS.
#include "chain_kernels.hpp"

#include <algorithm>
#include <cstddef>

#include "chain_vm.hpp"
#include "launch.hpp"
#include "tile_util.hpp"

namespace canvas {
namespace chain {

namespace {

// The program arrives in the kernel argument buffer, which is read through the scalar cache one line at a time (and
// may live in host memory): interpreting it from there cost microseconds per instruction.  The workgroup copies what
// it needs (header, tables, the n_instr instructions in use) into LDS with one parallel round trip and interprets that.
__device__ __forceinline__ const Program& stage_program(unsigned char* sprog) {
    const uint4* src = (const uint4*)__builtin_amdgcn_kernarg_segment_ptr();
    const int n_instr = ((const int*)src)[offsetof(Program, n_instr) / 4];
    const int pieces = (int)(offsetof(Program, ins) / 16) + n_instr;
    for (int i = threadIdx.x; i < pieces; i += blockDim.x) ((uint4*)sprog)[i] = src[i];
    __syncthreads();
    return *(const Program*)sprog;
}

template <int TM, int V, int U>
__global__ __launch_bounds__(max_threads_for(TM), min_waves_for(TM, V)) void k_chain(const Program) {
    __shared__ __align__(16) unsigned char sprog[sizeof(Program)];
    const Program& pg = stage_program(sprog);
    extern __shared__ __align__(16) float lds[];
    // (geometry: read once, as scalars)
    const Geo g = vm_geo(pg);
    const int threads = vm_u(pg.threads), PT = vm_u(pg.pix_threads), S = vm_u(pg.slices);
    const int chunks = vm_u(pg.chunks), tiles = vm_u(pg.tiles), chunk = vm_u(pg.chunk);
    const int own_threads = vm_u(pg.own_threads), halo_threads = vm_u(pg.halo_threads), n_pass = vm_u(pg.n_pass);
    const int xfloats = vm_u(pg.xadd_lanes) * g.npx;             // hand-over buffer of a slice (OP_XADD)
    // LDS: registers (16-byte pieces, see vm_reg_read) | hand-over buffers | persistent floats (float k of pixel v of thread i at [(k * V + v) * threads + i])
    const int rstride = threads * 4;
    float* const Rm = lds + threadIdx.x * 4;
    float* const xbase = lds + vm_u(pg.n_regs) * reg_pieces(U * TM * V) * rstride;
    float* const Pbase = xbase + S * xfloats;
    float* const Pm = Pbase + threadIdx.x;
    const int slice = __builtin_amdgcn_readfirstlane(threadIdx.x / PT);  // (PT is a multiple of 64: uniform in a wavefront)
    float* const xbuf = xbase + slice * xfloats;
    State<TM, V, U> st;
#pragma unroll
    for (int e = 0; e < U * TM * V; e++) st.A[e] = 0.f;
    Env ev;
    ev.np = vm_u(pg.n_persist);
    ev.fast = vm_u(pg.fast_math) != 0;
    ev.pstride = threads;
    ev.rstride = rstride;
    // The workgroup stays and walks over its share of the work items (image, tile, channel range): the program is staged
    // once per workgroup, not once per item.  item = (image * tiles + tile) * chunks + chunk
    const int items = g.N * tiles * chunks;
    unsigned first, unused;
    tile::xcd_order(first, unused);  // (the tiles of an image share halos and window rows: an XCD takes neighbouring items)
    for (int item = (int)first; item < items; item += gridDim.x) {
        const int chunk_id = item % chunks;
        const int tile = (item / chunks) % tiles;
        // the workgroup's threads: `slices` groups of PT threads; a group is one thread per V pixels of the tile (+ halo)
        Thread th;
        th.ptid = threadIdx.x - slice * PT;
        th.n = item / (chunks * tiles);
        th.p0 = (tile * own_threads - halo_threads + th.ptid) * V;
        th.active = th.p0 >= 0 && th.p0 < g.HW;
        th.row0 = th.active ? th.p0 / g.W : 0;
        th.col0 = th.active ? th.p0 - th.row0 * g.W : 0;
        th.own = th.active && th.ptid >= halo_threads && th.ptid < halo_threads + own_threads;
        const int c_begin = chunk_id * chunk;
        const int c_end = c_begin + chunk < g.C ? c_begin + chunk : g.C;
        for (int ps = 0; ps < n_pass; ps++) {
            uint32_t pw[4];
            __builtin_memcpy(pw, &pg.pass[ps], 16);
            const int pro_begin = vm_u((int)pw[0]) & 0xffff, pro_end = (int)((uint32_t)vm_u((int)pw[0]) >> 16);
            const int body_begin = vm_u((int)pw[1]) & 0xffff, body_end = (int)((uint32_t)vm_u((int)pw[1]) >> 16);
            const int red_begin = vm_u((int)pw[2]) & 0xffff, red_end = (int)((uint32_t)vm_u((int)pw[2]) >> 16);
            // trip -1 is the prologue (every slice, once); then slice s takes channels c_begin + s * U ... + U - 1, the next
            // slices * U, ...: every slice makes the same number of trips (the hand-over of OP_XADD synchronises the
            // workgroup), a trip past the last channel only keeps the barriers company
            for (int c0 = c_begin - S * U; c0 < c_end; c0 += S * U) {
                ev.pro = c0 < c_begin;
                ev.c = ev.pro ? c_begin : c0 + slice * U;
                ev.h = ev.pro ? 1 : (c_end - ev.c < 0 ? 0 : (c_end - ev.c < U ? c_end - ev.c : U));
                const int i_begin = ev.pro ? pro_begin : body_begin, i_end = ev.pro ? pro_end : body_end;
                if (i_begin >= i_end) continue;
                uint4 next = *(const uint4*)&pg.ins[i_begin];
                if (ev.h <= 0) {
                    // a trip past the last channel: nothing to compute, only the barriers of the hand-overs to keep.  (A loop
                    // of its own: with this case inside the loop below, as a path on which the state passes an instruction
                    // unchanged, the compiler kept the state in two sets of registers and copied it across for every
                    // instruction.)
                    for (int i = i_begin; i < i_end; i++) {
                        const Instr I = vm_uniform(next);
                        if (i + 1 < i_end) next = *(const uint4*)&pg.ins[i + 1];
                        if (I.op != OP_XADD) continue;
                        for (int u = 0; u < U; u++) {
                            __syncthreads();
                            __syncthreads();
                        }
                    }
                    continue;
                }
                for (int i = i_begin; i < i_end; i++) {
                    const Instr I = vm_uniform(next);
                    if (i + 1 < i_end) next = *(const uint4*)&pg.ins[i + 1];  // (on its way while this instruction runs)
                    if (I.op != OP_XADD) {
                        vm_exec<TM, V, U>(pg, g, I, ev, th, st, Pm, Rm);
                        continue;
                    }
#pragma unroll
                    for (int u = 0; u < U; u++) {
                        int dh = 0, dw = 0;
                        if (u < ev.h) vm_offset(pg, I.b, ev.c + u, dh, dw);
                        __syncthreads();  // the previous hand-over has been read
                        vm_xadd_write<TM, V>(g, I, th, st.A + u * TM * V, xbuf);
                        __syncthreads();
                        if (u < ev.h) vm_xadd_gather<TM, V>(g, I, dh, dw, th, xbuf, Pm + u * ev.np * V * threads, threads);
                    }
                }
            }
            // the slices' partial statistics and sums of this pass become totals, for every slice
            if (S > 1 && red_end > red_begin) {
                __syncthreads();  // the partials are complete
                for (int k = red_begin; k < red_end; k++) {
                    uint32_t rw;
                    __builtin_memcpy(&rw, &pg.red[k], 4);
                    rw = (uint32_t)vm_u((int)rw);
                    Red R;
                    __builtin_memcpy(&R, &rw, 4);
                    for (int e = 0; e < R.T * V; e++) {
                        float v0, v1;
                        vm_combine<V>(R, e, S, PT, Pbase, threads, th.ptid, v0, v1);
                        __syncthreads();  // everyone has read the partials of this lane
                        Pm[(R.slot * V + e) * threads] = v0;
                        if (R.kind == 0) Pm[((R.slot + R.T) * V + e) * threads] = v1;
                    }
                }
                __syncthreads();  // the totals are written before the next pass adds to anything
            }
        }
    }
}

// Workgroups of a launch: every item its own workgroup while they all fit the chip at once (256 compute units, 2048
// threads each), else a grid of that size whose workgroups take equal shares.
inline unsigned grid_for(const Program& pg) {
    const int64_t items = (int64_t)pg.N * pg.tiles * pg.chunks;
    const int64_t by_lds = std::max<int64_t>(1, (160 * 1024) / (int64_t)(lds_bytes(pg) + sizeof(Program) + 256));
    const int64_t resident = 256 * std::min<int64_t>(std::max(1, 2048 / pg.threads), by_lds);
    if (items <= resident) return (unsigned)items;
    const int64_t per = (items + resident - 1) / resident;
    return (unsigned)((items + per - 1) / per);
}

template <int TM, int V>
void launch(const Program& pg, hipStream_t stream) {
    constexpr int U = unroll_for(TM, V);
    // (more than 64 KB of dynamic LDS must be asked for, once per kernel)
    static const hipError_t lds_ok = hipFuncSetAttribute((const void*)k_chain<TM, V, U>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxLdsBytes);
    (void)lds_ok;
    const dim3 grid(grid_for(pg));
    CANVAS_LAUNCH((k_chain<TM, V, U>), grid, dim3((unsigned)pg.threads), lds_bytes(pg), stream, pg);
}

}  // namespace

void run(const Program& pg, hipStream_t stream) {
    const int v = pg.vec;
    if (pg.tm <= 1) {
        if (v == 16) launch<1, 16>(pg, stream);
        else if (v == 8) launch<1, 8>(pg, stream);
        else if (v == 4) launch<1, 4>(pg, stream);
        else if (v == 2) launch<1, 2>(pg, stream);
        else launch<1, 1>(pg, stream);
    } else if (pg.tm <= 9) {
        if (v == 4) launch<9, 4>(pg, stream);
        else if (v == 2) launch<9, 2>(pg, stream);
        else launch<9, 1>(pg, stream);
    } else {
        launch<25, 1>(pg, stream);
    }
}

}  // namespace chain
}  // namespace canvas
