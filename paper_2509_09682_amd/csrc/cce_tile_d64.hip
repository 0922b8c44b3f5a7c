// Matrix-core kernels of the dense cases, hidden size 64: the instantiations of cce_tile_body.hpp and their launchers.
#include "cce_tile_body.hpp"

namespace cce {

hipError_t launch_tile_d64(int pass, const TileArgs &a, hipStream_t stream) { return launch_for_d<64>(pass, a, stream); }
hipError_t launch_tile_backward_d64(const TileArgs &a_dh, const TileArgs &a_de, hipStream_t stream)
{
    return launch_bwd_for_d<64>(a_dh, a_de, stream);
}
hipError_t launch_pos_scatter_d64(const TileArgs &a, hipStream_t stream) { return launch_pos_scatter_d<64>(a, stream); }
hipError_t launch_dh_scale_d64(const TileArgs &a, bool file_g, hipStream_t stream) { return launch_dh_scale_d<64>(a, file_g, stream); }

}  // namespace cce
