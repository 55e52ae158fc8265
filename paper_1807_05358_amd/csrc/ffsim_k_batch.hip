// Batch kernels without the refinements of the inputs (the ones the benchmark configurations run).
#include "ffsim_select.h"

namespace ffsim {
batch_kernel_t select_batch_kernel_plain(const KernelChoice& k) { return batch_kernel_any<false>(k); }
batch_kernel_t select_batch_kernel(const KernelChoice& k) { return k.ext ? select_batch_kernel_ext(k) : select_batch_kernel_plain(k); }
}  // namespace ffsim
