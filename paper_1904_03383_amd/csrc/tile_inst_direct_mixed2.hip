// Explicit instantiations: direct-to-LDS variants with a gathered B, or a gathered operand next to a transposed one.
// <BM, BN, BK, WM, WN, two_level, LDS stages, wave groups along K, A mode, B mode>
#include "tile_direct_kernel.hpp"
namespace tg {
template hipError_t launch_tile_direct<64, 64, 32, 32, 32, true, 4, 1, 2, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<128, 128, 32, 64, 64, true, 3, 1, 2, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<64, 64, 32, 32, 32, true, 4, 1, 1, 2>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<128, 128, 32, 64, 64, true, 3, 1, 1, 2>(const GemmParams &, hipStream_t);
}  // namespace tg
