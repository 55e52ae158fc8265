// Trial-mutation kernels (proposals evaluated against a chain's stored timeline); compiled once
// per (FFSIM_EXT, FFSIM_GPN).
#include "ffsim_select.h"

#if !defined(FFSIM_EXT) || !defined(FFSIM_GPN)
#error "define FFSIM_EXT (0/1/2) and FFSIM_GPN (0/4)"
#endif

namespace ffsim {

template <bool CACHE>
static try_kernel_t try_kernel_of(const KernelChoice& k) {
    constexpr int EXT = FFSIM_EXT;
    constexpr int GPN = FFSIM_GPN;
    const bool tree = k.n_groups > FLAT_GROUPS;
    if (k.wide) return tree ? k_sim_chain_try<true, true, CACHE, EXT, GPN> : k_sim_chain_try<true, false, CACHE, EXT, GPN>;
    return tree ? k_sim_chain_try<false, true, CACHE, EXT, GPN> : k_sim_chain_try<false, false, CACHE, EXT, GPN>;
}

template <>
try_kernel_t try_kernels<FFSIM_EXT, FFSIM_GPN>(const KernelChoice& k) {
    return k.cache ? try_kernel_of<true>(k) : try_kernel_of<false>(k);
}

}  // namespace ffsim
