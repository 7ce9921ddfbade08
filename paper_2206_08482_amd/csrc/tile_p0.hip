// Row-tile trainer kernel compiled for one model shape (padded layer widths): benchmark workload C4
// (211:512:512:256:128:20).
#include "tile_kernel.h"

namespace gmi {
GMI_TILE_PART_DEFINE(0, 224, 512, 512, 256, 128, 32)
}  // namespace gmi
