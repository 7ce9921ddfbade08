// Forward-only row-tile kernel (agent_act / agent_value) for the 211:512:512:256:128:20 model (padded widths).
#include "tile_kernel.h"

namespace gmi {
GMI_TILE_FWD_PART_DEFINE(0, 224, 512, 512, 256, 128, 32)
}
