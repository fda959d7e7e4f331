// Explicit instantiations: row-panel variants for a gathered A (16 rows x 128 columns per compute wave).
// <compute waves, producer waves>
#include "tile_panel_kernel.hpp"
namespace tg {
template hipError_t launch_tile_panel<8, 4>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<4, 4>(const GemmParams &, hipStream_t);
}  // namespace tg
