// Explicit instantiations: direct-to-LDS variants for 32x32 wave tiles whose fragments are fetched a whole K tile
// ahead ("_tf" names).  <BM, BN, BK, LDS stages, two_level, A mode, B mode>
#include "tile_deep_kernel.hpp"
namespace tg {
template hipError_t launch_tile_deep<64, 64, 32, 2, false, 0, 0>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_deep<64, 64, 32, 2, true, 0, 0>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_deep<64, 64, 64, 2, false, 0, 0>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_deep<64, 64, 64, 2, true, 0, 0>(const GemmParams &, hipStream_t);
}  // namespace tg
