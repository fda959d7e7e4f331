// Explicit instantiations: workgroup-tile kernels on the bf16 matrix pipe (fp32 products from bf16 pieces).
#include "tile_pieces_kernel.hpp"
namespace tg {
template hipError_t launch_tile_pieces<128, 256, 32, 64, 128, 6>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_pieces<128, 256, 32, 64, 128, 9>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_pieces<128, 128, 32, 64, 64, 6>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_pieces<64, 64, 32, 32, 32, 6>(const GemmParams &, hipStream_t);
}  // namespace tg
