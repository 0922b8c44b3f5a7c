// Matrix-core kernels of the dense cases, hidden size 128: the instantiations of cce_tile_body.hpp and their launchers.
#include "cce_tile_body.hpp"

namespace cce {

hipError_t launch_tile_d128(int pass, const TileArgs &a, hipStream_t stream) { return launch_for_d<128>(pass, a, stream); }
hipError_t launch_tile_backward_d128(const TileArgs &a_dh, const TileArgs &a_de, hipStream_t stream)
{
    return launch_bwd_for_d<128>(a_dh, a_de, stream);
}
hipError_t launch_pos_scatter_d128(const TileArgs &a, hipStream_t stream) { return launch_pos_scatter_d<128>(a, stream); }
hipError_t launch_dh_scale_d128(const TileArgs &a, bool file_g, hipStream_t stream) { return launch_dh_scale_d<128>(a, file_g, stream); }

}  // namespace cce
