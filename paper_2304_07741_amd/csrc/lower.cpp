// Lowering selection.
#include "lowering.hpp"

namespace canvas {

std::unique_ptr<Lowering> lower(const Dag& dag, bool bf16, bool no_fusion) {
    (void)no_fusion;
    return lower_per_node(dag, bf16);
}

}  // namespace canvas
