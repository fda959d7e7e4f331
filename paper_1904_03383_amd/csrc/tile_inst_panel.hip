// Explicit instantiations: row-panel variants for a gathered A.
// <compute waves, producer waves, 16-row blocks, column groups per lane, two_level, steps of B in flight, chunk / 64>
#include "tile_panel_kernel.hpp"
namespace tg {
template hipError_t launch_tile_panel<8, 4, 1, 2, true, 1, 1, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<4, 4, 1, 2, true, 1, 1, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<4, 4, 2, 2, true, 1, 1, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<8, 4, 2, 2, false, 1, 1, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<8, 4, 2, 1, true, 1, 1, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<8, 4, 1, 1, true, 1, 1, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<4, 4, 1, 1, true, 1, 1, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<8, 4, 2, 1, true, 3, 1, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<8, 4, 1, 1, true, 3, 1, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<4, 4, 1, 1, true, 3, 1, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<8, 4, 2, 1, true, 3, 2, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<4, 4, 1, 1, true, 3, 2, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<8, 4, 2, 1, true, 3, 4, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<8, 4, 1, 1, true, 1, 1, true>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<8, 4, 2, 1, true, 1, 1, true>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<4, 4, 1, 1, true, 1, 1, true>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<8, 4, 2, 1, true, 3, 2, true>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<8, 4, 2, 1, false, 1, 1, true>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<8, 4, 2, 1, false, 3, 1, true>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<8, 4, 1, 1, false, 3, 1, true>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_panel<8, 4, 2, 1, true, 3, 1, true>(const GemmParams &, hipStream_t);
}  // namespace tg
