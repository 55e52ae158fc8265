// Batch kernels; compiled once per (FFSIM_EXT, FFSIM_GPN).
#include "ffsim_select.h"

#if !defined(FFSIM_EXT) || !defined(FFSIM_GPN)
#error "define FFSIM_EXT (0/1) and FFSIM_GPN (0/4)"
#endif

namespace ffsim {

template <bool WIDE, bool STATS, bool CACHE>
static batch_kernel_t batch_kernel_of(const KernelChoice& k) {
    constexpr bool EXT = FFSIM_EXT;
    constexpr int GPN = FFSIM_GPN;
    if (k.lds_words && k.n_ops <= 16 && k.max_parts <= 16) return k_sim_batch<WIDE, true, STATS, Q_ONE16, CACHE, EXT, GPN>;
    if (k.lds_words) return k.n_ops <= 64 ? k_sim_batch<WIDE, true, STATS, Q_ONE, CACHE, EXT, GPN> : k_sim_batch<WIDE, true, STATS, Q_FLAT, CACHE, EXT, GPN>;
    return k.n_groups > FLAT_GROUPS ? k_sim_batch<WIDE, false, STATS, Q_TREE, CACHE, EXT, GPN> : k_sim_batch<WIDE, false, STATS, Q_FLAT, CACHE, EXT, GPN>;
}

template <>
batch_kernel_t batch_kernels<FFSIM_EXT, FFSIM_GPN>(const KernelChoice& k) {
    if (k.cache) {
        if (k.wide) return k.stats ? batch_kernel_of<true, true, true>(k) : batch_kernel_of<true, false, true>(k);
        return k.stats ? batch_kernel_of<false, true, true>(k) : batch_kernel_of<false, false, true>(k);
    }
    if (k.wide) return k.stats ? batch_kernel_of<true, true, false>(k) : batch_kernel_of<true, false, false>(k);
    return k.stats ? batch_kernel_of<false, true, false>(k) : batch_kernel_of<false, false, false>(k);
}

}  // namespace ffsim
