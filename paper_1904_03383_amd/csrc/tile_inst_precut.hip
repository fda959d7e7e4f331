// Explicit instantiations: bf16-piece kernels whose operands are cut ahead by separate passes.
#include "tile_precut_kernel.hpp"
namespace tg {
template hipError_t launch_tile_precut<128, 256, 32, 64, 128, 6>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_precut<128, 256, 32, 64, 128, 9>(const GemmParams &, hipStream_t);
}  // namespace tg
