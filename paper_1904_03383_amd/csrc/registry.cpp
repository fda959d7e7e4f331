// Table of compiled kernel variants.  The template instantiations live in the
// tile_inst_*.hip units; this file only declares and lists them.
#include "tg_internal.h"

namespace tg {

#define TG_DECL(BM, BN, BK, WM, WN, L2, EDGE) \
    extern template hipError_t launch_tile<BM, BN, BK, WM, WN, L2, EDGE>(const GemmParams &, hipStream_t);
#define TG_ROW(BM, BN, BK, WM, WN, L2, EDGE, NAME)                                              \
    {NAME, KIND_TILE, BM, BN, BK, WM, WN, L2, EDGE, false, !EDGE, (BM / WM) * (BN / WN) * 64,  \
     tile_lds_bytes<BM, BN, BK, WM, WN>(), &launch_tile<BM, BN, BK, WM, WN, L2, EDGE>},
#define TG_PROW(BM, BN, BK, WM, WN, NAME)                                                       \
    {NAME, KIND_TILE, BM, BN, BK, WM, WN, false, false, true, false, (BM / WM) * (BN / WN) * 64, \
     tile_lds_bytes<BM, BN, BK, WM, WN>(), &launch_tile_stream<BM, BN, BK, WM, WN, false, false>},
#define TG_QROW(BM, BN, BK, WM, WN, NAME)                                                       \
    {NAME, KIND_TILE, BM, BN, BK, WM, WN, false, false, true, false, (BM / WM) * (BN / WN) * 64, \
     tile_lds_bytes<BM, BN, BK, WM, WN>(), &launch_tile_stream<BM, BN, BK, WM, WN, false, true>, 0, false, 0, true},

// (BM, BN, BK, WM, WN, two_level, edge, name)
#define TG_TILE_LIST(X)                                                     \
    X(128, 128, 16, 64, 64, false, false, "t128x128x16_w64x64")             \
    X(128, 128, 16, 64, 64, true, false, "t128x128x16_w64x64_acc2")         \
    X(128, 128, 32, 64, 64, false, false, "t128x128x32_w64x64")             \
    X(128, 128, 32, 64, 64, true, false, "t128x128x32_w64x64_acc2")         \
    X(256, 128, 16, 128, 64, false, false, "t256x128x16_w128x64")           \
    X(256, 128, 16, 128, 64, true, false, "t256x128x16_w128x64_acc2")       \
    X(128, 256, 16, 64, 128, false, false, "t128x256x16_w64x128")           \
    X(128, 256, 16, 64, 128, true, false, "t128x256x16_w64x128_acc2")       \
    X(256, 128, 32, 128, 64, false, false, "t256x128x32_w128x64")           \
    X(256, 128, 32, 128, 64, true, false, "t256x128x32_w128x64_acc2")       \
    X(128, 256, 32, 64, 128, false, false, "t128x256x32_w64x128")           \
    X(128, 256, 32, 64, 128, true, false, "t128x256x32_w64x128_acc2")       \
    X(64, 64, 32, 32, 32, false, false, "t64x64x32_w32x32")                 \
    X(64, 64, 32, 32, 32, true, false, "t64x64x32_w32x32_acc2")             \
    X(128, 64, 32, 64, 32, false, false, "t128x64x32_w64x32")               \
    X(64, 128, 32, 32, 64, false, false, "t64x128x32_w32x64")               \
    X(32, 256, 32, 32, 64, false, false, "t32x256x32_w32x64")               \
    X(32, 256, 32, 32, 64, true, false, "t32x256x32_w32x64_acc2")           \
    X(256, 32, 32, 64, 32, false, false, "t256x32x32_w64x32")               \
    X(256, 32, 32, 64, 32, true, false, "t256x32x32_w64x32_acc2")           \
    X(128, 128, 16, 64, 64, false, true, "t128x128x16_w64x64_edge")         \
    X(128, 128, 16, 64, 64, true, true, "t128x128x16_w64x64_acc2_edge")     \
    X(64, 64, 16, 32, 32, false, true, "t64x64x16_w32x32_edge")             \
    X(64, 64, 16, 32, 32, true, true, "t64x64x16_w32x32_acc2_edge")

#define TG_DECL_X(BM, BN, BK, WM, WN, L2, EDGE, NAME) TG_DECL(BM, BN, BK, WM, WN, L2, EDGE)
TG_TILE_LIST(TG_DECL_X)
extern template hipError_t launch_tile_stream<128, 128, 16, 64, 64, false, false>(const GemmParams &, hipStream_t);
extern template hipError_t launch_tile_stream<128, 128, 32, 64, 64, false, false>(const GemmParams &, hipStream_t);
extern template hipError_t launch_tile_stream<128, 256, 16, 64, 128, false, false>(const GemmParams &, hipStream_t);
extern template hipError_t launch_tile_stream<128, 128, 16, 64, 64, false, true>(const GemmParams &, hipStream_t);

// direct-to-LDS variants: (BM, BN, BK, WM, WN, two_level, LDS stages, wave groups along K, name)
#define TG_DIRECT_LIST(X)                                                   \
    X(128, 128, 32, 64, 64, false, 2, 1, "d128x128x32_w64x64")                 \
    X(128, 128, 32, 64, 64, true, 2, 1, "d128x128x32_w64x64_acc2")             \
    X(128, 256, 32, 64, 128, false, 2, 1, "d128x256x32_w64x128")               \
    X(128, 256, 32, 64, 128, true, 2, 1, "d128x256x32_w64x128_acc2")           \
    X(256, 128, 32, 128, 64, false, 2, 1, "d256x128x32_w128x64")               \
    X(256, 128, 32, 128, 64, true, 2, 1, "d256x128x32_w128x64_acc2")           \
    X(128, 256, 32, 64, 128, true, 3, 1, "d128x256x32_w64x128_acc2_st3")       \
    X(256, 128, 32, 128, 64, true, 3, 1, "d256x128x32_w128x64_acc2_st3")       \
    X(256, 256, 32, 128, 128, false, 2, 1, "d256x256x32_w128x128")             \
    X(32, 256, 32, 32, 64, false, 2, 1, "d32x256x32_w32x64")                   \
    X(256, 32, 32, 64, 32, false, 2, 1, "d256x32x32_w64x32")                   \
    X(64, 64, 32, 32, 32, false, 2, 1, "d64x64x32_w32x32")                     \
    X(64, 64, 32, 32, 32, false, 4, 1, "d64x64x32_w32x32_st4")                  \
    X(64, 64, 32, 32, 32, false, 2, 2, "d64x64x32_w32x32_k2")                   \
    X(64, 64, 32, 32, 32, false, 4, 2, "d64x64x32_w32x32_k2_st4")
#define TG_DDECL(BM, BN, BK, WM, WN, L2, NS, KG, NAME) \
    extern template hipError_t launch_tile_direct<BM, BN, BK, WM, WN, L2, NS, KG>(const GemmParams &, hipStream_t);
#define TG_DROW(BM, BN, BK, WM, WN, L2, NS, KG, NAME)                                           \
    {NAME, KIND_TILE, BM, BN, BK, WM, WN, L2, false, false, false, (BM / WM) * (BN / WN) * 64 * KG, \
     NS * (BM * BK + BK * BN) * 4, &launch_tile_direct<BM, BN, BK, WM, WN, L2, NS, KG>},
TG_DIRECT_LIST(TG_DDECL)

// direct-to-LDS variants that read transposed or element-strided operands as they lie ("_ta"/"_tb": A / B given
// transposed; "_ga"/"_gb": any element strides, gathered with 4-byte loads):
// (BM, BN, BK, WM, WN, two_level, LDS stages, A mode, B mode, name)
#define TG_MODE_LIST(X)                                                          \
    X(64, 64, 32, 32, 32, true, 4, 2, 0, "d64x64x32_w32x32_acc2_st4_ga")         \
    X(32, 128, 32, 32, 32, true, 4, 2, 0, "d32x128x32_w32x32_acc2_st4_ga")       \
    X(128, 128, 32, 64, 64, true, 3, 2, 0, "d128x128x32_w64x64_acc2_st3_ga")     \
    X(128, 256, 32, 64, 128, true, 3, 2, 0, "d128x256x32_w64x128_acc2_st3_ga")   \
    X(64, 64, 32, 32, 32, true, 2, 1, 0, "d64x64x32_w32x32_acc2_ta")             \
    X(128, 128, 32, 64, 64, true, 2, 1, 0, "d128x128x32_w64x64_acc2_ta")         \
    X(128, 256, 32, 64, 128, true, 2, 1, 0, "d128x256x32_w64x128_acc2_ta")       \
    X(64, 64, 32, 32, 32, true, 2, 0, 1, "d64x64x32_w32x32_acc2_tb")             \
    X(128, 128, 32, 64, 64, true, 2, 0, 1, "d128x128x32_w64x64_acc2_tb")         \
    X(128, 256, 32, 64, 128, true, 2, 0, 1, "d128x256x32_w64x128_acc2_tb")       \
    X(64, 64, 32, 32, 32, true, 2, 1, 1, "d64x64x32_w32x32_acc2_ta_tb")          \
    X(128, 128, 32, 64, 64, true, 2, 1, 1, "d128x128x32_w64x64_acc2_ta_tb")      \
    X(128, 256, 32, 64, 128, true, 2, 1, 1, "d128x256x32_w64x128_acc2_ta_tb")    \
    X(64, 64, 32, 32, 32, true, 4, 0, 2, "d64x64x32_w32x32_acc2_st4_gb")         \
    X(128, 128, 32, 64, 64, true, 3, 0, 2, "d128x128x32_w64x64_acc2_st3_gb")     \
    X(64, 64, 32, 32, 32, true, 4, 2, 2, "d64x64x32_w32x32_acc2_st4_ga_gb")      \
    X(128, 128, 32, 64, 64, true, 3, 2, 2, "d128x128x32_w64x64_acc2_st3_ga_gb")  \
    X(64, 64, 32, 32, 32, true, 4, 2, 1, "d64x64x32_w32x32_acc2_st4_ga_tb")      \
    X(128, 128, 32, 64, 64, true, 3, 2, 1, "d128x128x32_w64x64_acc2_st3_ga_tb")  \
    X(64, 64, 32, 32, 32, true, 4, 1, 2, "d64x64x32_w32x32_acc2_st4_ta_gb")      \
    X(128, 128, 32, 64, 64, true, 3, 1, 2, "d128x128x32_w64x64_acc2_st3_ta_gb")
#define TG_MDECL(BM, BN, BK, WM, WN, L2, NS, AM, BMD, NAME) \
    extern template hipError_t launch_tile_direct<BM, BN, BK, WM, WN, L2, NS, 1, AM, BMD>(const GemmParams &, hipStream_t);
#define TG_MROW(BM, BN, BK, WM, WN, L2, NS, AM, BMD, NAME)                                      \
    {NAME, KIND_TILE, BM, BN, BK, WM, WN, L2, false, false, false, (BM / WM) * (BN / WN) * 64,  \
     NS * (BM * BK + BK * BN) * 4, &launch_tile_direct<BM, BN, BK, WM, WN, L2, NS, 1, AM, BMD>, 0, false, 0, false, AM, BMD},
TG_MODE_LIST(TG_MDECL)
// 16-row tiles on v_mfma_f32_16x16x4_f32, for a gathered A: each element of A is a cache line of its own, fetched once
// per tile column, so the widest tile that still fills the chip wins (1024 x 1024: 16 x 256 tiles are 256 workgroups)
#define TG_MI16_LIST(X)                                                          \
    X(16, 256, 32, 16, 64, true, 4, 2, 0, "d16x256x32_w16x64_acc2_st4_ga")       \
    X(16, 256, 32, 16, 64, true, 3, 2, 0, "d16x256x32_w16x64_acc2_st3_ga")
#define TG_M16DECL(BM, BN, BK, WM, WN, L2, NS, AM, BMD, NAME) \
    extern template hipError_t launch_tile_direct<BM, BN, BK, WM, WN, L2, NS, 1, AM, BMD, 16>(const GemmParams &, hipStream_t);
#define TG_M16ROW(BM, BN, BK, WM, WN, L2, NS, AM, BMD, NAME)                                    \
    {NAME, KIND_TILE, BM, BN, BK, WM, WN, L2, false, false, false, (BM / WM) * (BN / WN) * 64,  \
     NS * (BM * BK + BK * BN) * 4, &launch_tile_direct<BM, BN, BK, WM, WN, L2, NS, 1, AM, BMD, 16>, 0, false, 0, false, AM, BMD},
TG_MI16_LIST(TG_M16DECL)

// row panels of a gathered A: 16 rows by up to 1024 columns per workgroup, so that an element of A (a cache line of its
// own at a large stride) is requested once per 1024 columns; with few tile rows a K split fills the chip
// (compute waves, producer waves, 16-row blocks, column groups of four per lane, two_level, steps of B in flight,
// k per chunk / 64, persistent walk along a row panel, name)
#define TG_PANEL_LIST(X)                                       \
    X(8, 4, 1, 2, true, 1, 1, false, "g16x1024x64_w16x128_acc2_ga")      \
    X(4, 4, 1, 2, true, 1, 1, false, "g16x512x64_w16x128_acc2_ga")       \
    X(4, 4, 2, 2, true, 1, 1, false, "g32x512x64_w32x128_acc2_ga")       \
    X(8, 4, 2, 2, false, 1, 1, false, "g32x1024x64_w32x128_ga")          \
    X(8, 4, 2, 1, true, 1, 1, false, "g32x512x64_w32x64_acc2_ga")        \
    X(8, 4, 1, 1, true, 1, 1, false, "g16x512x64_w16x64_acc2_ga")        \
    X(4, 4, 1, 1, true, 1, 1, false, "g16x256x64_w16x64_acc2_ga")        \
    X(8, 4, 2, 1, true, 3, 1, false, "g32x512x64_w32x64_acc2_b3_ga")     \
    X(8, 4, 1, 1, true, 3, 1, false, "g16x512x64_w16x64_acc2_b3_ga")     \
    X(4, 4, 1, 1, true, 3, 1, false, "g16x256x64_w16x64_acc2_b3_ga")     \
    X(8, 4, 2, 1, true, 3, 2, false, "g32x512x128_w32x64_acc2_b3_ga")    \
    X(4, 4, 1, 1, true, 3, 2, false, "g16x256x128_w16x64_acc2_b3_ga")    \
    X(8, 4, 2, 1, true, 3, 4, false, "g32x512x256_w32x64_acc2_b3_ga")    \
    X(8, 4, 1, 1, true, 1, 1, true, "g16x512x64_w16x64_acc2_rw_ga")      \
    X(8, 4, 2, 1, true, 1, 1, true, "g32x512x64_w32x64_acc2_rw_ga")      \
    X(4, 4, 1, 1, true, 1, 1, true, "g16x256x64_w16x64_acc2_rw_ga")      \
    X(8, 4, 2, 1, true, 3, 2, true, "g32x512x128_w32x64_acc2_b3_rw_ga")  \
    X(8, 4, 2, 1, false, 1, 1, true, "g32x512x64_w32x64_rw_ga")          \
    X(8, 4, 2, 1, false, 3, 1, true, "g32x512x64_w32x64_b3_rw_ga")       \
    X(8, 4, 1, 1, false, 3, 1, true, "g16x512x64_w16x64_b3_rw_ga")       \
    X(8, 4, 2, 1, true, 3, 1, true, "g32x512x64_w32x64_acc2_b3_rw_ga")
#define TG_GDECL(NC, NP, RB, NQ, L2, PD, CW, RW, NAME) \
    extern template hipError_t launch_tile_panel<NC, NP, RB, NQ, L2, PD, CW, RW>(const GemmParams &, hipStream_t);
#define TG_GROW(NC, NP, RB, NQ, L2, PD, CW, RW, NAME)                                                                   \
    {NAME, KIND_TILE, 16 * RB, NC * 64 * NQ, 64 * CW, 16 * RB, 64 * NQ, L2, false, RW, false, (NC + NP) * 64, 3 * 16 * RB * (64 * CW + 8) * 4, \
     &launch_tile_panel<NC, NP, RB, NQ, L2, PD, CW, RW>, 0, false, 0, false, 2, 0},
TG_PANEL_LIST(TG_GDECL)

// row panels that keep their rows of A in LDS over the whole (short) K range: one barrier per workgroup, persistent walk
// (waves, 16-row blocks, column groups of four per lane, steps of B in flight, name)
#define TG_RESIDENT_LIST(X)                                  \
    X(16, 2, 1, 1, "g32x1024x64_w32x64_res_ga")              \
    X(8, 2, 1, 1, "g32x512x64_w32x64_res_ga")                \
    X(8, 2, 1, 3, "g32x512x64_w32x64_b3_res_ga")
#define TG_RDECL(NC, RB, NQ, PD, NAME) \
    extern template hipError_t launch_tile_resident<NC, RB, NQ, PD>(const GemmParams &, hipStream_t);
#define TG_RROW(NC, RB, NQ, PD, NAME)                                                                          \
    {NAME, KIND_TILE, 16 * RB, NC * 64 * NQ, 64, 16 * RB, 64 * NQ, false, false, true, false, NC * 64, 16 * RB * (128 + 8) * 4, \
     &launch_tile_resident<NC, RB, NQ, PD>, 0, false, 0, false, 2, 0},
TG_RESIDENT_LIST(TG_RDECL)

// direct-to-LDS variants for 32x32 wave tiles with tile-granular fragment prefetch:
// (BM, BN, BK, two_level, LDS stages, A mode, B mode, name)
#define TG_DEEP_LIST(X)                                                     \
    X(64, 64, 32, false, 2, 0, 0, "d64x64x32_w32x32_tf")                    \
    X(64, 64, 32, true, 2, 0, 0, "d64x64x32_w32x32_acc2_tf")                \
    X(64, 64, 64, false, 2, 0, 0, "d64x64x64_w32x32_tf")                    \
    X(64, 64, 64, true, 2, 0, 0, "d64x64x64_w32x32_acc2_tf")                \
    X(64, 64, 32, true, 2, 1, 0, "d64x64x32_w32x32_acc2_tf_ta")             \
    X(64, 64, 32, true, 2, 0, 1, "d64x64x32_w32x32_acc2_tf_tb")             \
    X(64, 64, 32, true, 2, 1, 1, "d64x64x32_w32x32_acc2_tf_ta_tb")          \
    X(64, 64, 32, true, 2, 2, 0, "d64x64x32_w32x32_acc2_tf_ga")             \
    X(64, 64, 32, true, 2, 0, 2, "d64x64x32_w32x32_acc2_tf_gb")
#define TG_FDECL(BM, BN, BK, L2, NS, AM, BMD, NAME) \
    extern template hipError_t launch_tile_deep<BM, BN, BK, NS, L2, AM, BMD>(const GemmParams &, hipStream_t);
#define TG_FROW(BM, BN, BK, L2, NS, AM, BMD, NAME)                                              \
    {NAME, KIND_TILE, BM, BN, BK, 32, 32, L2, false, false, false, (BM / 32) * (BN / 32) * 64, \
     NS * (BM * BK + BK * BN) * 4, &launch_tile_deep<BM, BN, BK, NS, L2, AM, BMD>, 0, false, 0, false, AM, BMD},
TG_DEEP_LIST(TG_FDECL)

// bf16-piece variants: (BM, BN, BK, WM, WN, piece products, name)
#define TG_PIECES_LIST(X)                                                   \
    X(128, 256, 32, 64, 128, 6, "e128x256x32_w64x128_x6")                   \
    X(128, 256, 32, 64, 128, 9, "e128x256x32_w64x128_x9")                   \
    X(128, 128, 32, 64, 64, 6, "e128x128x32_w64x64_x6")                     \
    X(64, 64, 32, 32, 32, 6, "e64x64x32_w32x32_x6")
#define TG_EDECL(BM, BN, BK, WM, WN, NP, NAME) \
    extern template hipError_t launch_tile_pieces<BM, BN, BK, WM, WN, NP>(const GemmParams &, hipStream_t);
#define TG_EROW(BM, BN, BK, WM, WN, NP, NAME)                                                   \
    {NAME, KIND_TILE, BM, BN, BK, WM, WN, false, false, false, false, (BM / WM) * (BN / WN) * 64, \
     2 * 3 * (BK / 8) * ((BM + 4) + (BN + 4)) * 16, &launch_tile_pieces<BM, BN, BK, WM, WN, NP>, NP},
TG_PIECES_LIST(TG_EDECL)
// the same with the operands cut ahead into a workspace image ("c" names)
#define TG_CDECL(BM, BN, BK, WM, WN, NP, NAME) \
    extern template hipError_t launch_tile_precut<BM, BN, BK, WM, WN, NP>(const GemmParams &, hipStream_t);
#define TG_CROW(BM, BN, BK, WM, WN, NP, NAME)                                                   \
    {"c" NAME, KIND_TILE, BM, BN, BK, WM, WN, false, false, false, false, (BM / WM) * (BN / WN) * 64, \
     2 * 3 * (BK / 8) * (BM + BN) * 16, &launch_tile_precut<BM, BN, BK, WM, WN, NP>, NP, true},
#define TG_PRECUT_LIST(X)                                                   \
    X(128, 256, 32, 64, 128, 6, "128x256x32_w64x128_x6")                    \
    X(128, 256, 32, 64, 128, 9, "128x256x32_w64x128_x9")
TG_PRECUT_LIST(TG_CDECL)

static const KernelInfo kTable[] = {
    TG_TILE_LIST(TG_ROW)
    TG_DIRECT_LIST(TG_DROW)
    TG_DEEP_LIST(TG_FROW)
    TG_MODE_LIST(TG_MROW)
    TG_MI16_LIST(TG_M16ROW)
    TG_PANEL_LIST(TG_GROW)
    TG_RESIDENT_LIST(TG_RROW)
    TG_PIECES_LIST(TG_EROW)
    TG_PRECUT_LIST(TG_CROW)
    TG_PROW(128, 128, 16, 64, 64, "p128x128x16_w64x64")
    TG_PROW(128, 128, 32, 64, 64, "p128x128x32_w64x64")
    TG_PROW(128, 256, 16, 64, 128, "p128x256x16_w64x128")
    TG_QROW(128, 128, 16, 64, 64, "p128x128x16_w64x64_ds")
    {"wave32", KIND_WAVE, 32, 32, 8, 32, 32, false, true, false, false, 256, 0, &launch_wave32},
    {"wave16", KIND_WAVE, 16, 16, 16, 16, 16, false, true, false, false, 256, 0, &launch_wave16},
    {"wave16x32", KIND_WAVE, 16, 32, 16, 16, 32, false, false, false, false, 256, 0, &launch_wave16w<2>},
    {"wave16x64", KIND_WAVE, 16, 64, 16, 16, 64, false, false, false, false, 256, 0, &launch_wave16w<4>},
    {"wave16k4", KIND_WAVE, 16, 16, 16, 16, 16, false, true, false, false, 256, 4096, &launch_wave16k4, 0, false, 4},
};

int num_kernels() { return (int)(sizeof(kTable) / sizeof(kTable[0])); }
const KernelInfo &kernel(int idx) { return kTable[idx]; }

}  // namespace tg
