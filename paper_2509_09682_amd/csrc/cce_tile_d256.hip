// Matrix-core kernels of the dense cases, hidden size 256: the instantiations of cce_tile_body.hpp and their launchers.
#include "cce_tile_body.hpp"

namespace cce {

hipError_t launch_tile_d256(int pass, const TileArgs &a, hipStream_t stream) { return launch_for_d<256>(pass, a, stream); }
hipError_t launch_pos_scatter_d256(const TileArgs &a, hipStream_t stream) { return launch_pos_scatter_d<256>(a, stream); }
hipError_t launch_dh_scale_d256(const TileArgs &a, bool file_g, hipStream_t stream) { return launch_dh_scale_d<256>(a, file_g, stream); }

}  // namespace cce
