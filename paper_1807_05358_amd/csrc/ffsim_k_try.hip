// Trial-mutation kernels (proposals evaluated against a chain's stored timeline).
#include "ffsim_select.h"

namespace ffsim {
template <bool CACHE, bool EXT>
static try_kernel_t try_kernel_of(const KernelChoice& k) {
    const bool tree = k.n_groups > FLAT_GROUPS;
    if (k.wide) return tree ? k_sim_chain_try<true, true, CACHE, EXT> : k_sim_chain_try<true, false, CACHE, EXT>;
    return tree ? k_sim_chain_try<false, true, CACHE, EXT> : k_sim_chain_try<false, false, CACHE, EXT>;
}
try_kernel_t select_try_kernel(const KernelChoice& k) {
    if (k.ext) return k.cache ? try_kernel_of<true, true>(k) : try_kernel_of<false, true>(k);
    return k.cache ? try_kernel_of<true, false>(k) : try_kernel_of<false, false>(k);
}
}  // namespace ffsim
