// Explicit instantiations: direct-to-LDS variants for transposed operands (A m-contiguous and/or B k-contiguous).
// <BM, BN, BK, WM, WN, two_level, LDS stages, wave groups along K, A mode, B mode>
#include "tile_direct_kernel.hpp"
namespace tg {
template hipError_t launch_tile_direct<64, 64, 32, 32, 32, true, 2, 1, 1, 0>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<128, 128, 32, 64, 64, true, 2, 1, 1, 0>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<128, 256, 32, 64, 128, true, 2, 1, 1, 0>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<64, 64, 32, 32, 32, true, 2, 1, 0, 1>(const GemmParams &, hipStream_t);
}  // namespace tg
