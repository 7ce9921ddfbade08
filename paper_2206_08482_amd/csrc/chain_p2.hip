// Register-chained trainer kernel compiled for one model shape (waves per workgroup, weight chunks in flight, largest group, deferred epilogues, chunks between the fetch of stored activations and their use, forward-only,
// padded layer widths): the paper's Table 6 models 24:256:128:64:3 and 23:256:128:64:9.
#include "chain_kernel.h"

namespace gmi {
GMI_CHAIN_PART_DEFINE(2, 8, 3, 4, 0, 1, 2, 32, 256, 128, 64, 32)
}  // namespace gmi
