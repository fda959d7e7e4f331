// Explicit instantiations: direct-to-LDS variants (aligned operands, k % 32 == 0, n % 4 == 0).
// <BM, BN, BK, WM, WN, two_level, LDS stages, wave groups along K>
#include "tile_direct_kernel.hpp"
namespace tg {
template hipError_t launch_tile_direct<128, 128, 32, 64, 64, false, 2, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<128, 128, 32, 64, 64, true, 2, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<128, 256, 32, 64, 128, false, 2, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<128, 256, 32, 64, 128, true, 2, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<256, 128, 32, 128, 64, false, 2, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<256, 128, 32, 128, 64, true, 2, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<128, 256, 32, 64, 128, true, 3, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<256, 128, 32, 128, 64, true, 3, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<64, 64, 32, 32, 32, false, 2, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<64, 64, 32, 32, 32, false, 4, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<64, 64, 32, 32, 32, false, 2, 2>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<64, 64, 32, 32, 32, false, 4, 2>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<256, 256, 32, 128, 128, false, 2, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<32, 256, 32, 32, 64, false, 2, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<256, 32, 32, 64, 32, false, 2, 1>(const GemmParams &, hipStream_t);
}  // namespace tg
