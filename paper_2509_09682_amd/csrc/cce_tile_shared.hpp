// Constants the matrix-core kernels share with the host code that sizes their workspace.
#pragma once
#include <stdint.h>

namespace cce {

// Last-round split of a position-stationary pass at hidden size 256 (see tail_plan in cce_tile_body.hpp).
constexpr int kTailMaxSplits = 4;
constexpr int64_t kTailRows = 65536;  // rows of the partial buffer: S * tail blocks <= slots, slots * rows per block <= this

}  // namespace cce
