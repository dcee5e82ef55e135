// Fused-chain kernels: one workgroup = one image x one tile of rows (plus halo rows in backward programs) x one
// range of channels; one thread = one pixel; the program (chain_isa.hpp) arrives in the kernel arguments and is
// interpreted with workgroup-uniform control flow.  Loads are coalesced along W (the innermost dim of NCHW);
// stencil offsets are address offsets of those loads; reductions over taps stay in registers; the statistics of a
// softmax over channels and the gradient hand-over of shifted loads live in LDS.
#include "chain_kernels.hpp"

#include "chain_vm.hpp"
#include "launch.hpp"

namespace canvas {
namespace chain {

namespace {

template <int TM, int NR>
__global__ __launch_bounds__(max_threads_for(TM)) void k_chain(const Program pg) {
    extern __shared__ float lds[];
    const int threads = pg.threads;
    float* const xbuf = lds;                                  // 2 x threads: hand-over buffers of OP_XADD
    float* const Pm = lds + 2 * threads + threadIdx.x;         // this thread's persistent floats, stride `threads`
    // blockIdx.x = (image * tiles + tile) * chunks + chunk
    const int chunk_id = blockIdx.x % pg.chunks;
    const int tile = (blockIdx.x / pg.chunks) % pg.tiles;
    Thread th;
    th.tid = threadIdx.x;
    th.n = blockIdx.x / (pg.chunks * pg.tiles);
    const int rows = pg.tile_rows + 2 * pg.halo_rows;
    const int row_first = tile * pg.tile_rows - pg.halo_rows;
    const int lr = th.tid / pg.W;
    th.col = th.tid - lr * pg.W;
    th.row = row_first + lr;
    th.active = lr < rows;
    th.own = th.active && lr >= pg.halo_rows && lr < pg.halo_rows + pg.tile_rows && th.row < pg.H;
    const int c_begin = chunk_id * pg.chunk;
    const int c_end = c_begin + pg.chunk < pg.C ? c_begin + pg.chunk : pg.C;
    State<TM, NR> st;
#pragma unroll
    for (int t = 0; t < TM; t++) st.A[t] = 0.f;
#pragma unroll
    for (int r = 0; r < NR; r++)
#pragma unroll
        for (int t = 0; t < TM; t++) st.R[r][t] = 0.f;
    unsigned parity = 0;
    for (int ps = 0; ps < pg.n_pass; ps++) {
        const Pass pass = pg.pass[ps];
        for (int i = pass.pro_begin; i < pass.pro_end; i++) vm_exec<TM, NR>(pg, pg.ins[i], c_begin, th, st, Pm, threads);
        for (int c = c_begin; c < c_end; c++) {
            for (int i = pass.body_begin; i < pass.body_end; i++) {
                const Instr I = pg.ins[i];
                if (I.op != OP_XADD) {
                    vm_exec<TM, NR>(pg, I, c, th, st, Pm, threads);
                    continue;
                }
                int dh, dw;
                vm_offset(pg, I.b, c, dh, dw);
#pragma unroll
                for (int t = 0; t < TM; t++)
                    if (t < I.T) {
                        float* buf = xbuf + (parity & 1u) * threads;
                        parity++;
                        buf[th.tid] = st.A[t];
                        __syncthreads();
                        const int src = vm_xadd_source(pg, I, dh, dw, t, th, row_first, rows);
                        if (src >= 0) Pm[(I.a + ((I.kind & kExtTaps) ? t : 0)) * threads] += buf[src];
                    }
            }
        }
    }
}

template <int TM>
void launch(const Program& pg, hipStream_t stream) {
    const dim3 grid((unsigned)((int64_t)pg.N * pg.tiles * pg.chunks));
    CANVAS_LAUNCH((k_chain<TM, regs_for(TM)>), grid, dim3((unsigned)pg.threads), lds_bytes(pg), stream, pg);
}

}  // namespace

void run(const Program& pg, hipStream_t stream) {
    if (pg.tm <= 1) launch<1>(pg, stream);
    else if (pg.tm <= 9) launch<9>(pg, stream);
    else launch<25>(pg, stream);
}

}  // namespace chain
}  // namespace canvas
