// The simulation kernels are compiled in several translation units (they are many template
// instantiations); the host file picks one through these functions.
#pragma once
#include "ffsim_kernels.h"

namespace ffsim {

typedef void (*batch_kernel_t)(SimDev, const DOp*, const DEdge*, const DEdge*, const uint32_t*, const uint32_t*, const uint2*,
                               uint32_t, u64*, Counters*, unsigned char*, size_t, const uint16_t*);
typedef void (*chain_kernel_t)(SimDev, const DOp*, const DEdge*, const DEdge*, const uint32_t*, const uint32_t*, unsigned char*, size_t,
                               uint32_t, uint32_t, const uint32_t*, uint32_t, u64*, uint32_t*, SearchDev);
typedef void (*try_kernel_t)(SimDev, const DOp*, const DEdge*, const DEdge*, const uint32_t*, const uint32_t*, const unsigned char*, size_t,
                             uint32_t, uint32_t, const uint32_t*, uint32_t, u64*, const uint32_t*, uint32_t*, unsigned char*, size_t);

// What fixes the instantiation.  Batch kernels: four layouts -- task words in LDS (small graphs;
// never a queue level 2; up to 64 ops the whole queue in a register), in HBM without and with
// level 2 -- each with or without the kept per-edge set-up, the per-candidate counters, 64-bit
// sums, and the refinements of the inputs (link table, explicit devices).
struct KernelChoice {
    bool wide, lds_words, stats, cache, ext;
    uint32_t n_ops, n_groups;
};
batch_kernel_t select_batch_kernel(const KernelChoice& k);      // ffsim_k_batch.hip / ffsim_k_batch_ext.hip
batch_kernel_t select_batch_kernel_plain(const KernelChoice& k);
batch_kernel_t select_batch_kernel_ext(const KernelChoice& k);
chain_kernel_t select_chain_kernel(const KernelChoice& k);      // ffsim_k_chain.hip
try_kernel_t select_try_kernel(const KernelChoice& k);          // ffsim_k_try.hip

// shared by the two batch files
template <bool WIDE, bool STATS, bool CACHE, bool EXT>
inline batch_kernel_t batch_kernel_of(const KernelChoice& k) {
    if (k.lds_words) return k.n_ops <= 64 ? k_sim_batch<WIDE, true, STATS, Q_ONE, CACHE, EXT> : k_sim_batch<WIDE, true, STATS, Q_FLAT, CACHE, EXT>;
    return k.n_groups > FLAT_GROUPS ? k_sim_batch<WIDE, false, STATS, Q_TREE, CACHE, EXT> : k_sim_batch<WIDE, false, STATS, Q_FLAT, CACHE, EXT>;
}
template <bool EXT>
inline batch_kernel_t batch_kernel_any(const KernelChoice& k) {
    if (k.cache) {
        if (k.wide) return k.stats ? batch_kernel_of<true, true, true, EXT>(k) : batch_kernel_of<true, false, true, EXT>(k);
        return k.stats ? batch_kernel_of<false, true, true, EXT>(k) : batch_kernel_of<false, false, true, EXT>(k);
    }
    if (k.wide) return k.stats ? batch_kernel_of<true, true, false, EXT>(k) : batch_kernel_of<true, false, false, EXT>(k);
    return k.stats ? batch_kernel_of<false, true, false, EXT>(k) : batch_kernel_of<false, false, false, EXT>(k);
}

}  // namespace ffsim
