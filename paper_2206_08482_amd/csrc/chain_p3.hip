// Register-chained trainer kernel compiled for one model shape (waves per workgroup, weight chunks in flight, largest group, deferred epilogues, chunks between the fetch of stored activations and their use, forward-only,
// padded layer widths): the paper's Table 6 model 108:200:400:100:21.
#include "chain_kernel.h"

namespace gmi {
GMI_CHAIN_PART_DEFINE(3, 4, 3, 4, 1, 1, 0, 128, 224, 416, 128, 32)
}  // namespace gmi
