// Explicit instantiations: predicated variants that accept any m, n, k, leading
// dimension and pointer alignment (Sec. 4.5 of the paper: threads outside the iteration
// space are disabled by predication rather than by requiring sizes to divide).
#include "tile_kernel.hpp"
namespace tg {
template hipError_t launch_tile<128, 128, 16, 64, 64, false, true>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<128, 128, 16, 64, 64, true, true>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<64, 64, 16, 32, 32, false, true>(const GemmParams &, hipStream_t);
template hipError_t launch_tile<64, 64, 16, 32, 32, true, true>(const GemmParams &, hipStream_t);
}  // namespace tg
