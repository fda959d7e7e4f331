// Explicit instantiations: row panels with A resident in LDS (short K).
#include "tile_resident_kernel.hpp"
namespace tg {
template hipError_t launch_tile_resident<16, 2, 1, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_resident<8, 2, 1, 1>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_resident<8, 2, 1, 3>(const GemmParams &, hipStream_t);
}  // namespace tg
