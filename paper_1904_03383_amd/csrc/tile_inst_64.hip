// Explicit instantiations: 64x64 workgroup tiles (four waves of 32x32) for problems too
// small to fill the chip with larger tiles.
#include "tile_kernel.hpp"
namespace tg {
template hipError_t launch_tile<64, 64, 32, 32, 32, false, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<64, 64, 32, 32, 32, true, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<128, 64, 32, 64, 32, false, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<64, 128, 32, 32, 64, false, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<32, 256, 32, 32, 64, false, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<32, 256, 32, 32, 64, true, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<256, 32, 32, 64, 32, false, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<256, 32, 32, 64, 32, true, false>(const GemmParams &, hipStream_t);
}  // namespace tg
