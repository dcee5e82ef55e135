// Lowering selection.
#include "lowering.hpp"

#include <algorithm>
#include <iterator>

namespace canvas {

constexpr int64_t kMinWeightElemsForBf16Intermediates = 16;

std::unique_ptr<Lowering> lower(const Dag& full, bool bf16, bool no_fusion) {
    const Dag dag = without_dead_views(full);
    std::unique_ptr<Lowering> l;
    if (!no_fusion) {
        l = lower_sgfc(dag, bf16);
        // The two lowerings below keep C-channel intermediates in bf16 (rounding 2^-9 per element).  An element of
        // dW is a sum over all pixels whose terms can cancel; with many elements the largest one, which sets the
        // max-norm tolerance, is no cancelled sum, but a weight tensor of a few scalars has no such element.
        // Such DAGs keep fp32 intermediates (the lowering by segments).
        bool tiny_weight = false;
        for (int i = 0; i < dag.n_weights; i++) {
            const Node& f = dag.nodes[dag.weight_node[i]];
            const Node& A = dag.nodes[f.a];
            if (f.live && (int64_t)f.out * (A.C / f.groups) * A.T < kMinWeightElemsForBf16Intermediates) tiny_weight = true;
        }
        if (!l && !tiny_weight) l = lower_ufc(dag, bf16);
        if (!l && !tiny_weight) l = lower_dyn(dag, bf16);
    }
    if (!l) l = lower_per_node(dag, bf16, !no_fusion);
    batch_weight_jobs(*l);
    batch_reduce_jobs(*l);
    return l;
}

void batch_weight_jobs(Lowering& low) {
    std::vector<Launch> head;
    for (size_t first = 0; first < low.wjobs.size(); first += wprep::kMaxJobs) {
        const std::vector<WeightJob> part(low.wjobs.begin() + first,
                                          low.wjobs.begin() + std::min(low.wjobs.size(), first + (size_t)wprep::kMaxJobs));
        double bytes = 0;
        for (const auto& j : part) bytes += j.bytes;
        head.push_back({"weight_prep", bytes, 0, [part](const RunArgs& a) {
                            wprep::Jobs J;
                            for (const auto& j : part) {
                                wprep::Job& d = J.j[J.n++];
                                d = j.job;
                                d.w = (const uint16_t*)a.w[j.widx];
                                d.out = (uint16_t*)(a.ws + j.off);
                            }
                            wprep::run(J, a.stream);
                        }, true});
    }
    low.fwd.insert(low.fwd.begin(), std::make_move_iterator(head.begin()), std::make_move_iterator(head.end()));
    low.wjobs.clear();
}

void batch_reduce_jobs(Lowering& low) {
    for (size_t first = 0; first < low.rjobs.size(); first += wreduce::kMaxJobs) {
        const std::vector<ReduceJob> part(low.rjobs.begin() + first,
                                          low.rjobs.begin() + std::min(low.rjobs.size(), first + (size_t)wreduce::kMaxJobs));
        double bytes = 0;
        for (const auto& j : part) bytes += j.bytes;
        low.bwd.push_back({"wgrad_reduce", bytes, 0, [part](const RunArgs& a) {
                               wreduce::Jobs J;
                               for (const auto& j : part) {
                                   wreduce::Job& d = J.j[J.n++];
                                   d = j.job;
                                   d.partial = (const float*)(a.ws + j.off);
                                   d.dw = (float*)a.dw[j.widx];
                               }
                               wreduce::run(J, a.stream);
                           }});
    }
    low.rjobs.clear();
}

void make_inference_plan(Lowering& low) {
    std::vector<Launch> keep;
    for (auto& l : low.fwd) (l.prep ? low.prep : keep).push_back(std::move(l));
    low.fwd = std::move(keep);
    low.bwd.clear();
}

}  // namespace canvas
