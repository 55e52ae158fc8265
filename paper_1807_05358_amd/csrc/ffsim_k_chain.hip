// Chain kernels (delta simulation and search steps).
#include "ffsim_select.h"

namespace ffsim {
template <bool CACHE, bool EXT>
static chain_kernel_t chain_kernel_of(const KernelChoice& k) {
    const bool tree = k.n_groups > FLAT_GROUPS;
    if (k.wide) return tree ? k_sim_chain_steps<true, true, CACHE, EXT> : k_sim_chain_steps<true, false, CACHE, EXT>;
    return tree ? k_sim_chain_steps<false, true, CACHE, EXT> : k_sim_chain_steps<false, false, CACHE, EXT>;
}
chain_kernel_t select_chain_kernel(const KernelChoice& k) {
    if (k.ext) return k.cache ? chain_kernel_of<true, true>(k) : chain_kernel_of<false, true>(k);
    return k.cache ? chain_kernel_of<true, false>(k) : chain_kernel_of<false, false>(k);
}
}  // namespace ffsim
