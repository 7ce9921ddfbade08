// Forward-only (inference) form of the register-chained kernel for one model shape (waves per workgroup, weight
// chunks in flight, largest group, deferred epilogues, -, forward-only, padded layer widths): benchmark workload C4
// (211:512:512:256:128:20).  The group size must be the trainer kernel's of the same shape: both read one stream.
#include "chain_kernel.h"

namespace gmi {
GMI_CHAIN_FWD_DEFINE(0, 4, 3, 4, 0, 1, 1, 224, 512, 512, 256, 128, 32)
}  // namespace gmi
