#include "fc_emit.hpp"

#include "gfc_kernels.hpp"
#include "gfc_tm_kernels.hpp"

namespace canvas {

void emit_fc(Lowering& low, bool backward, const Dag& dag, const TakeFn& take, const std::string& name, int G, int R, int kh, int kw, int Og,
             bool transposed, int widx, FcOperand src, PtrFn dst, bool addend_is_dst, double bytes, double flops, bool dst_f32, bool softmax) {
    std::vector<Launch>& list = backward ? low.bwd : low.fwd;
    const int64_t nw = (int64_t)G * Og * R * kh * kw;
    if (!src.f32 && gfctm::supported(dag.N, G, R, kh, kw, Og, dag.H, dag.W)) {
        const gfctm::Params T = gfctm::shape(dag.N, G, R, kh, kw, Og, dag.H, dag.W);
        const bool identity = !transposed && T.TV == 1 && T.gm == 1 && T.Rp == R && T.Omp == Og;
        const int64_t opk = identity ? -1 : take((uint64_t)gfctm::packed_elems(T) * 2);
        if (!identity) {
            WeightJob j;
            j.job.kind = 0;
            j.job.G = T.G;
            j.job.R = T.R;
            j.job.Og = T.Og;
            j.job.TV = T.TV;
            j.job.gm = T.gm;
            j.job.Gm = T.Gm;
            j.job.Rp = T.Rp;
            j.job.Omp = T.Omp;
            j.job.transposed = transposed ? 1 : 0;
            j.job.total = gfctm::packed_elems(T);
            j.widx = widx;
            j.off = opk;
            j.bytes = 2.0 * nw + 2.0 * gfctm::packed_elems(T);
            low.wjobs.push_back(j);
        }
        list.push_back({name, bytes, flops, [=](const RunArgs& a) {
                            gfctm::Params Q = T;
                            Q.src = (const uint16_t*)src.ptr(a);
                            Q.wp = identity ? (const uint16_t*)a.w[widx] : (const uint16_t*)(a.ws + opk);
                            Q.dst = const_cast<void*>(dst(a));
                            Q.dst_f32 = dst_f32 ? 1 : 0;
                            Q.softmax = softmax ? 1 : 0;
                            Q.addend = addend_is_dst ? (const uint16_t*)dst(a) : nullptr;  // each lane reads the elements it then overwrites
                            gfctm::forward(Q, a.stream);
                        }});
        return;
    }
    gfc::Params F = gfc::shape(dag.N, G, R, kh, kw, Og, dag.H, dag.W);
    F.src_f32 = src.f32 ? 1 : 0;
    F.dst_f32 = dst_f32 ? 1 : 0;
    gfc::prepare_forward(F);
    const int64_t owt = transposed ? take((uint64_t)nw * 2) : -1;
    if (transposed) {  // (R, Og) are the swapped dims: the FC's own weights are [G][R][Og][taps]
        WeightJob j;
        j.job.kind = 1;
        j.job.G = G;
        j.job.Og = R;  // (the job reads [G][its Og][its R][TV]: the FC's own output and row counts)
        j.job.R = Og;
        j.job.TV = kh * kw;
        j.job.total = nw;
        j.widx = widx;
        j.off = owt;
        j.bytes = 4.0 * nw;
        low.wjobs.push_back(j);
    }
    list.push_back({name, bytes, flops, [=](const RunArgs& a) {
                        gfc::Params Q = F;
                        Q.src = src.ptr(a);
                        Q.w = transposed ? (const uint16_t*)(a.ws + owt) : (const uint16_t*)a.w[widx];
                        Q.dst = const_cast<void*>(dst(a));
                        Q.addend = addend_is_dst ? (const uint16_t*)dst(a) : nullptr;
                        gfc::forward(Q, a.stream);
                    }});
}

bool fc_softmax_fusable(const Dag& dag, int G, int R, int kh, int kw, int Og, const FcOperand& src) {
    return !src.f32 && gfctm::supported(dag.N, G, R, kh, kw, Og, dag.H, dag.W) &&
           gfctm::softmax_fusable(gfctm::shape(dag.N, G, R, kh, kw, Og, dag.H, dag.W));
}

void emit_wgrad(Lowering& low, const Dag& dag, const TakeFn& take, const std::string& name, int G, int R, int kh, int kw, int Og,
                int widx, FcOperand src, FcOperand dy, double operand_bytes, double flops) {
    std::vector<Launch>& list = low.bwd;
    const int64_t nw = (int64_t)G * Og * R * kh * kw;
    if (kh * kw > 1 && !src.f32 && !dy.f32 && gfctm::supported(dag.N, G, R, kh, kw, Og, dag.H, dag.W)) {
        gfctm::Params T = gfctm::shape(dag.N, G, R, kh, kw, Og, dag.H, dag.W);
        gfctm::prepare_wgrad(T);
        const int ts = gfctm::wgrad_slices(T);
        const int64_t pk = gfctm::packed_elems(T);
        const int64_t opt = take((uint64_t)ts * pk * 4);
        list.push_back({name, operand_bytes + 4.0 * ts * pk, flops, [=](const RunArgs& a) {
                            gfctm::Params Q = T;
                            Q.src = (const uint16_t*)src.ptr(a);
                            Q.dy = (const uint16_t*)dy.ptr(a);
                            Q.partial = (float*)(a.ws + opt);
                            gfctm::wgrad_partial(Q, a.stream);
                        }});
        ReduceJob rj;
        rj.job.slices = ts;
        rj.job.kind = 1;
        rj.job.count = (unsigned)pk;
        rj.job.G = T.G; rj.job.R = T.R; rj.job.Og = T.Og; rj.job.TV = T.TV;
        rj.job.gm = T.gm; rj.job.Omp = T.Omp; rj.job.Rp = T.Rp;
        wreduce::plan(rj.job);
        rj.widx = widx;
        rj.off = opt;
        rj.bytes = 4.0 * ts * pk + 4.0 * nw;
        low.rjobs.push_back(rj);
        return;
    }
    gfc::Params W = gfc::shape(dag.N, G, R, kh, kw, Og, dag.H, dag.W);
    W.src_f32 = src.f32 ? 1 : 0;
    W.dy_f32 = dy.f32 ? 1 : 0;
    gfc::prepare_wgrad(W);
    const int slices = gfc::wgrad_partials(W);
    const int64_t op = take((uint64_t)slices * nw * 4);
    list.push_back({name, operand_bytes + 4.0 * slices * nw, flops, [=](const RunArgs& a) {
                        gfc::Params Q = W;
                        Q.src = src.ptr(a);
                        Q.dy = dy.ptr(a);
                        Q.partial = (float*)(a.ws + op);
                        gfc::wgrad_partial(Q, a.stream);
                    }});
    ReduceJob rj;
    rj.job.slices = slices;
    rj.job.kind = 0;
    rj.job.count = (unsigned)nw;
    wreduce::plan(rj.job);
    rj.widx = widx;
    rj.off = op;
    rj.bytes = 4.0 * (slices + 1) * nw;
    low.rjobs.push_back(rj);
}

}  // namespace canvas
