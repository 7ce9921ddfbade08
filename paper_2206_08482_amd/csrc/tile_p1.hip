// Row-tile trainer kernel compiled for one model shape (padded layer widths): the paper's Table 6 model
// 211:512:512:512:256:20.
#include "tile_kernel.h"

namespace gmi {
GMI_TILE_PART_DEFINE(1, 224, 512, 512, 512, 256, 32)
}  // namespace gmi
