// Batch kernels; compiled once per (FFSIM_EXT, FFSIM_GPN).
#include "ffsim_select.h"

#if !defined(FFSIM_EXT) || !defined(FFSIM_GPN)
#error "define FFSIM_EXT (0/1/2) and FFSIM_GPN (0/4)"
#endif

namespace ffsim {

template <bool WIDE, bool STATS, bool CACHE>
static batch_kernel_t batch_kernel_of(const KernelChoice& k) {
    constexpr int EXT = FFSIM_EXT;
    constexpr int GPN = FFSIM_GPN;
    switch (batch_queue_shape(k)) {
        case Q_ONE16: return k_sim_batch<WIDE, true, STATS, Q_ONE16, CACHE, EXT, GPN>;
        case Q_ONE: return k_sim_batch<WIDE, true, STATS, Q_ONE, CACHE, EXT, GPN>;
        case Q_TREE: return k_sim_batch<WIDE, false, STATS, Q_TREE, CACHE, EXT, GPN>;
        default: break;
    }
    return k.lds_words ? k_sim_batch<WIDE, true, STATS, Q_FLAT, CACHE, EXT, GPN> : k_sim_batch<WIDE, false, STATS, Q_FLAT, CACHE, EXT, GPN>;
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
