// Explicit instantiations: 128x128 workgroup tiles (four waves of 64x64).
#include "tile_kernel.hpp"
namespace tg {
template hipError_t launch_tile<128, 128, 16, 64, 64, false, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<128, 128, 16, 64, 64, true, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<128, 128, 32, 64, 64, false, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<128, 128, 32, 64, 64, true, false>(const GemmParams &, hipStream_t);
}  // namespace tg
