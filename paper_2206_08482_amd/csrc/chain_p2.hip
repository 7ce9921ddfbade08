// Register-chained trainer kernel compiled for one model shape (waves per workgroup, weight chunks in flight, largest group, deferred epilogues, chunks between the fetch of stored activations and their use, forward-only,
// padded layer widths): benchmark workload C4 (211:512:512:256:128:20).
#include "chain_kernel.h"

namespace gmi {
GMI_CHAIN_PART_DEFINE(2, 4, 3, 4, 0, 1, 2, 224, 512, 512, 256, 128, 32)
}  // namespace gmi
