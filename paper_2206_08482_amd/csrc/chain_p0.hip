// Register-chained trainer kernel compiled for one model shape (waves per workgroup, weight chunks in flight, largest group, deferred epilogues, chunks between the fetch of stored activations and their use, forward-only,
// padded layer widths): benchmark workload C2 (60:256:128:64:8; also the paper's Anymal 48:256:128:64:12 after padding).
#include "chain_kernel.h"

namespace gmi {
GMI_CHAIN_PART_DEFINE(0, 8, 3, 4, 0, 1, 0, 64, 256, 128, 64, 32)
}  // namespace gmi
