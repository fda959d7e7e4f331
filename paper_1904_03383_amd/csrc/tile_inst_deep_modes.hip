// Explicit instantiations: the "_tf" variants for transposed and element-strided operands.
// <BM, BN, BK, LDS stages, two_level, A mode, B mode>
#include "tile_deep_kernel.hpp"
namespace tg {
template hipError_t launch_tile_deep<64, 64, 32, 2, true, 1, 0>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_deep<64, 64, 32, 2, true, 0, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_deep<64, 64, 32, 2, true, 1, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_deep<64, 64, 32, 2, true, 2, 0>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_deep<64, 64, 32, 2, true, 0, 2>(const GemmParams &, hipStream_t);
}  // namespace tg
