// Batch kernels with the link table and / or explicit devices per task.
#include "ffsim_select.h"

namespace ffsim {
batch_kernel_t select_batch_kernel_ext(const KernelChoice& k) { return batch_kernel_any<true>(k); }
}  // namespace ffsim
