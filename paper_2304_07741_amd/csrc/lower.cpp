// Lowering selection.
#include "lowering.hpp"

#include <algorithm>
#include <iterator>

namespace canvas {

std::unique_ptr<Lowering> lower(const Dag& full, bool bf16, bool no_fusion) {
    const Dag dag = without_dead_views(full);
    std::unique_ptr<Lowering> l;
    if (!no_fusion) {
        l = lower_sgfc(dag, bf16);
        if (!l) l = lower_ufc(dag, bf16);
        if (!l) l = lower_dyn(dag, bf16);
    }
    if (!l) l = lower_per_node(dag, bf16);
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
