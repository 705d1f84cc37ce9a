// Pipelined tile kernel instantiations for fp32 storage.
#include "bf_pipe.inc.h"

namespace bf {

int launch_pipe_op_f32(int op, bool with_y, const TileParams& tp, const Shape& s, int grid, hipStream_t st) {
  return launch_pipe_op<DT_F32>(op, with_y, tp, s, grid, st);
}

}  // namespace bf
