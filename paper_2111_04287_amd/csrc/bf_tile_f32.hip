// Tile kernel instantiations for fp32 storage.
#include "bf_tile.inc.h"

namespace bf {

int launch_tile_op_f32(int op, bool with_y, const TileParams& tp, const Shape& s, int grid, hipStream_t st) {
  return launch_tile_op<DT_F32>(op, with_y, tp, s, grid, st);
}

}  // namespace bf
