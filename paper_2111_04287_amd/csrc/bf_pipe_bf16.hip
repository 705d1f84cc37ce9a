// Pipelined tile kernel instantiations for bf16 storage.
#include "bf_pipe.inc.h"

namespace bf {

int launch_pipe_op_bf16(int op, bool with_y, const TileParams& tp, const Shape& s, int grid, hipStream_t st) {
  return launch_pipe_op<DT_BF16>(op, with_y, tp, s, grid, st);
}

}  // namespace bf
