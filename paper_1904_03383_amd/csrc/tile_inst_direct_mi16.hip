// Explicit instantiations: direct-to-LDS variants with 16-row tiles (v_mfma_f32_16x16x4_f32) that gather an
// element-strided A.
// <BM, BN, BK, WM, WN, two_level, LDS stages, wave groups along K, A mode, B mode, MFMA block>
#include "tile_direct_kernel.hpp"
namespace tg {
template hipError_t launch_tile_direct<16, 256, 32, 16, 64, true, 4, 1, 2, 0, 16>(const GemmParams &, hipStream_t);
template hipError_t launch_tile_direct<16, 256, 32, 16, 64, true, 3, 1, 2, 0, 16>(const GemmParams &, hipStream_t);
}  // namespace tg
