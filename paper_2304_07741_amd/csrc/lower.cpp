// Lowering selection.
#include "lowering.hpp"

namespace canvas {

std::unique_ptr<Lowering> lower(const Dag& full, bool bf16, bool no_fusion) {
    const Dag dag = without_dead_views(full);
    if (!no_fusion) {
        if (auto l = lower_sgfc(dag, bf16)) return l;
        if (auto l = lower_ufc(dag, bf16)) return l;
        if (auto l = lower_dyn(dag, bf16)) return l;
    }
    return lower_per_node(dag, bf16);
}

void make_inference_plan(Lowering& low) {
    std::vector<Launch> keep;
    for (auto& l : low.fwd) (l.prep ? low.prep : keep).push_back(std::move(l));
    low.fwd = std::move(keep);
    low.bwd.clear();
}

}  // namespace canvas
