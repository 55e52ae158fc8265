// The simulation kernels are many template instantiations; they are compiled in several
// objects side by side (each kernel file once per combination of EXT and GPN), and the host
// file picks one through these functions.
#pragma once
#include "ffsim_kernels.h"

namespace ffsim {

typedef void (*batch_kernel_t)(SimDev, const DOp*, const DEdge*, const DEdge*, const uint32_t*, const uint32_t*, const uint2*,
                               uint32_t, u64*, Counters*, unsigned char*, size_t, const uint16_t*);
typedef void (*chain_kernel_t)(SimDev, const DOp*, const DEdge*, const DEdge*, const uint32_t*, const uint32_t*, unsigned char*, size_t,
                               uint32_t, uint32_t, const uint32_t*, uint32_t, u64*, uint32_t*, SearchDev);
typedef void (*try_kernel_t)(SimDev, const DOp*, const DEdge*, const DEdge*, const uint32_t*, const uint32_t*, const unsigned char*, size_t,
                             uint32_t, uint32_t, const uint32_t*, uint32_t, u64*, const uint32_t*, uint32_t*, unsigned char*, size_t);

// What fixes the instantiation inside one object.  Batch kernels: four layouts -- task words in
// LDS (small graphs; never a queue level 2; up to 64 ops the whole queue in a register, with a
// shorter form for 16 ops of 16 parts), in HBM
// without and with level 2 -- each with or without the kept per-edge set-up, the per-candidate
// counters and 64-bit sums.
struct KernelChoice {
    bool wide, lds_words, stats, cache;
    uint32_t n_ops, n_groups, max_parts;
};
// the queue shape (QueueShape) of the batch kernel that serves a graph
inline int batch_queue_shape(const KernelChoice& k) {
    if (k.lds_words && k.n_ops <= 16 && k.max_parts <= 16) return Q_ONE16;
    if (k.lds_words) return k.n_ops <= 64 ? Q_ONE : Q_FLAT;
    return k.n_groups > FLAT_GROUPS ? Q_TREE : Q_FLAT;
}
// EXT: 0 plain; 1 the refinements of the inputs (link tables, explicit devices, parameter traffic); 2 also
// training-iteration graphs (contributing edges, tied configurations).  GPN: GPUs per node the
// kernels are compiled for (4, or 0 = any).  One explicit specialisation per object.
template <int EXT, int GPN> batch_kernel_t batch_kernels(const KernelChoice& k);
template <int EXT, int GPN> chain_kernel_t chain_kernels(const KernelChoice& k);
template <int EXT, int GPN> try_kernel_t try_kernels(const KernelChoice& k);

}  // namespace ffsim
