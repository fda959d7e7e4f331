// Explicit instantiations: 256x128 and 128x256 workgroup tiles (four waves of 128x64 / 64x128).
#include "tile_kernel.hpp"
namespace tg {
template hipError_t launch_tile<256, 128, 16, 128, 64, false, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<256, 128, 16, 128, 64, true, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<128, 256, 16, 64, 128, false, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<128, 256, 16, 64, 128, true, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<256, 128, 32, 128, 64, false, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<256, 128, 32, 128, 64, true, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<128, 256, 32, 64, 128, false, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<128, 256, 32, 64, 128, true, false>(const GemmParams &, hipStream_t);
}  // namespace tg
