// Chain kernels (delta simulation and search steps); compiled once per (FFSIM_EXT, FFSIM_GPN).
#include "ffsim_select.h"

#if !defined(FFSIM_EXT) || !defined(FFSIM_GPN)
#error "define FFSIM_EXT (0/1/2) and FFSIM_GPN (0/4)"
#endif

namespace ffsim {

template <bool CACHE>
static chain_kernel_t chain_kernel_of(const KernelChoice& k) {
    constexpr int EXT = FFSIM_EXT;
    constexpr int GPN = FFSIM_GPN;
    const bool tree = k.n_groups > FLAT_GROUPS;
    if (k.wide) return tree ? k_sim_chain_steps<true, true, CACHE, EXT, GPN> : k_sim_chain_steps<true, false, CACHE, EXT, GPN>;
    return tree ? k_sim_chain_steps<false, true, CACHE, EXT, GPN> : k_sim_chain_steps<false, false, CACHE, EXT, GPN>;
}

template <>
chain_kernel_t chain_kernels<FFSIM_EXT, FFSIM_GPN>(const KernelChoice& k) {
    return k.cache ? chain_kernel_of<true>(k) : chain_kernel_of<false>(k);
}

}  // namespace ffsim
