// Tile kernel instantiations for bf16 storage.
#include "bf_tile.inc.h"

namespace bf {

int launch_tile_op_bf16(int op, bool with_y, const TileParams& tp, const Shape& s, int grid, hipStream_t st) {
  return launch_tile_op<DT_BF16>(op, with_y, tp, s, grid, st);
}

}  // namespace bf
