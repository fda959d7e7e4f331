// Explicit instantiations: persistent ("stream") variants for short-K problems.
#include "tile_stream_kernel.hpp"
namespace tg {
template hipError_t launch_tile_stream<128, 128, 16, 64, 64, false, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_stream<128, 128, 32, 64, 64, false, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_stream<128, 256, 16, 64, 128, false, false>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_stream<128, 128, 16, 64, 64, false, true>(const GemmParams &, hipStream_t);
}  // namespace tg
