// Internal interface between the host side (API, dispatcher, tuner) and the HIP kernels.
// Not part of the public boundary (include/tgemm.h).
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <stdint.h>

namespace tg {

// Everything a GEMM kernel launch needs.  Sizes are validated to fit in int32 by the
// API layer; element offsets are formed in 64 bits.
struct GemmParams {
    const float *A;
    const float *B;
    float *C;             // final output
    float *ws;            // split-K partial sums: [batch][splits][m][n], ld = n (nullptr if splits == 1)
    void *planes;         // piece images of A and B written by the cutting passes (kernels that cut ahead), else nullptr
    int64_t lda, ldb, ldc;
    int64_t csa, csb;     // element strides along k of A and along n of B (1 except for the strided entry point;
                          // honoured by the predicated kernels and by the direct-to-LDS kernels with operand modes 1, 2)
    int64_t strideA, strideB, strideC;
    int m, n, k;
    int nb;               // columns of B the exact-fit kernels may fetch: n, or n rounded up to a multiple of 4 when
                          // B's rows are known to have the room (an aligned copy with zero padding)
    int batch;
    int splits;           // number of K ranges; each writes its own partial product
    int ktiles_per_split; // K tiles (of the kernel's BK) per range
    int tiles_m, tiles_n; // C tiles per problem
    int group;            // tile rows per swizzle group (tile order inside one XCD's region)
    int xcd_m, xcd_n;     // 2-D split of one problem's tile grid over the 8 XCDs (xcd_m * xcd_n == 8),
                          // or 0, 0: XCDs take contiguous ranges of the linear tile order
    int flush_tiles;      // two-level accumulation: fold the MFMA accumulators into the
                          // second-level sums every this many K tiles (0 = never)
    int persistent_blocks; // > 0: launch this many workgroups (a multiple of 8) that loop over the work items
    int max_blocks_per_cu; // occupancy cap enforced through the LDS request (0 = none)
    int flags;            // kFlag* bits, computed on the host from pointers and strides
};

constexpr int kFlagVecA = 1;  // rows of A have unit element stride: four consecutive k are one 16-byte load (any 4-byte alignment)
constexpr int kFlagVecC = 2;  // n is a multiple of 4: the split-K reduction adds and stores 16-byte vectors
constexpr int kFlagVecB = 4;  // rows of B have unit element stride

typedef hipError_t (*launch_fn)(const GemmParams &, hipStream_t);

enum KernelKind { KIND_TILE = 0, KIND_WAVE = 1 };

struct KernelInfo {
    const char *name;
    KernelKind kind;
    int BM, BN, BK;      // workgroup tile (KIND_WAVE: tile of one wave, BK = k step)
    int WM, WN;          // wave tile
    bool two_level;      // has second-level accumulators (needed for long K)
    bool edge;           // predicated variant: any m, n, k, leading dimension and alignment
    bool persistent;     // workgroups loop over tiles (launch with a fixed number of workgroups per CU)
    bool k_tail;         // exact-fit variant that also takes k % BK != 0 (k % 4 == 0, k >= BK)
    int threads;
    int lds_bytes;
    launch_fn launch;
    int pieces;          // 0: fp32 MFMA; 6 or 9: every fp32 product formed from that many bf16 piece products
    bool precut;         // piece kernel whose operands are cut by separate passes into a workspace image
    int kwaves;          // KIND_WAVE: waves of a workgroup that share one tile, each with its part of K (0 = one wave per tile)
    bool defer;          // persistent variant that stores a finished tile during the next one: no split-K, aligned rows of C
    int amode, bmode;    // how the kernel reads A / B: 0 as the plain product has them (A k-contiguous, B n-contiguous,
                         // 16-byte aligned rows), 1 transposed (A m-contiguous, B k-contiguous, aligned), 2 any element strides
};

// Kernel table (registry.cpp).
int num_kernels();
const KernelInfo &kernel(int idx);

// Workgroup-tile kernels: LDS-staged, double-buffered, MFMA 32x32x2 register blocks.
template <int BM, int BN, int BK, int WM, int WN, bool TWO_LEVEL, bool EDGE>
hipError_t launch_tile(const GemmParams &p, hipStream_t s);

// Persistent form of the tile kernel: a fixed number of workgroups walk the K tiles of
// several output tiles as one stream (exact-fit shapes).
// DEFER: finished tiles are stored between the MFMAs of the workgroup's next item.
template <int BM, int BN, int BK, int WM, int WN, bool TWO_LEVEL, bool DEFER>
hipError_t launch_tile_stream(const GemmParams &p, hipStream_t s);
template <int BM, int BN, int BK, int WM, int WN>
constexpr int tile_lds_bytes();

// Same, with operand tiles loaded global -> LDS directly into a ring of NS stages (aligned operands, k % 32 == 0, n % 4 == 0);
// KG wave groups share each wave tile, every group taking 1/KG of each K tile.  AM / BMD: operand modes of A and B
// (KernelInfo::amode / bmode): transposed and element-strided operands are read as they lie, without a separate pass.
// MI: edge of the matrix instruction's block, 32 (v_mfma_f32_32x32x2_f32) or 16 (v_mfma_f32_16x16x4_f32: 16-row tiles).
template <int BM, int BN, int BK, int WM, int WN, bool TWO_LEVEL, int NS, int KG, int AM = 0, int BMD = 0, int MI = 32>
hipError_t launch_tile_direct(const GemmParams &p, hipStream_t s);

// Direct-to-LDS kernel for 32x32 wave tiles that fetches the fragments of a whole K tile one tile ahead
// (aligned operands, k % BK == 0, n % 4 == 0; operand modes AM / BMD as for launch_tile_direct).
template <int BM, int BN, int BK, int NS, bool TWO_LEVEL, int AM = 0, int BMD = 0>
hipError_t launch_tile_deep(const GemmParams &p, hipStream_t s);

// Row-panel kernel for a gathered A (any element strides of A; B plain with 16-byte rows, n % 4 == 0, k % (64 * CW) == 0):
// 16 * RB rows x 64 * NQ * NC columns per workgroup, NC compute waves that read B straight from global memory and NP
// waves that only gather A into LDS.
template <int NC, int NP, int RB, int NQ, bool TWO_LEVEL, int PD = 1, int CW = 1, bool WALK = false>
hipError_t launch_tile_panel(const GemmParams &p, hipStream_t s);
template <int NC, int RB, int NQ, int PD>
hipError_t launch_tile_resident(const GemmParams &p, hipStream_t s);

// Workgroup-tile kernel on the bf16 matrix pipe: operands cut into three bf16 pieces each, NP piece
// products per fp32 product (aligned operands, k % BK == 0, n % 4 == 0).
template <int BM, int BN, int BK, int WM, int WN, int NP>
hipError_t launch_tile_pieces(const GemmParams &p, hipStream_t s);
template <int BM, int BN, int BK>
constexpr int pieces_lds_bytes();

// The same product with the operands cut ahead: two passes write the pieces of A and B into
// GemmParams::planes (6 bytes per element, padded to whole tiles), the product kernel streams those images
// into LDS.  Any m, n, k, alignment and element stride.
template <int BM, int BN, int BK, int WM, int WN, int NP>
hipError_t launch_tile_precut(const GemmParams &p, hipStream_t s);

// One wave per 32x32 C tile, operands straight from global memory (small / batched problems).
hipError_t launch_wave32(const GemmParams &p, hipStream_t s);
hipError_t launch_wave16(const GemmParams &p, hipStream_t s);
hipError_t launch_wave16k4(const GemmParams &p, hipStream_t s);
template <int CB> hipError_t launch_wave16w(const GemmParams &p, hipStream_t s);   // 16 x 16*CB tile per wave, aligned operands

// C[b][i][j] = sum_s ws[b][s][i][j], fixed order s = 0..splits-1 (deterministic).
hipError_t launch_splitk_reduce(const GemmParams &p, hipStream_t s);

// C[b][i][j] = +0.0 on the m x n region (k == 0).
hipError_t launch_zero_fill(const GemmParams &p, hipStream_t s);

// z = alpha * x + y over n contiguous floats (bandwidth-bound streaming kernel).
hipError_t launch_saxpy(int64_t n, float alpha, const float *x, const float *y, float *z, hipStream_t s);

// dst[r * ld + c] = src[r * rs + c * cs] (rows x cols): packs an element-strided or transposed operand.
hipError_t launch_pack(const float *src, int64_t rs, int64_t cs, float *dst, int64_t ld, int rows, int cols, hipStream_t s);

// dst[r * ld + c] = src[r * rs + c] (r < rows, c < cols), +0.0 elsewhere on rows_out x ld: aligned, zero-padded copy.
hipError_t launch_pad_copy(const float *src, int64_t rs, int rows, int cols, float *dst, int64_t ld, int rows_out, hipStream_t s);
// ... of both operands in one launch
hipError_t launch_pad_copy2(const float *src_a, int64_t rs_a, int rows_a, int cols_a, float *dst_a, int64_t ld_a, int rows_out_a,
                            const float *src_b, int64_t rs_b, int rows_b, int cols_b, float *dst_b, int64_t ld_b, int rows_out_b,
                            hipStream_t s);

// The tuner's result check: copy every step-th row of C into `ref` (packed), and compare the same rows of a later
// result with it: partial[3*b + 0..2] of workgroup b = sum (c - ref)^2, sum ref^2, count of non-finite values.
constexpr int kCheckBlocks = 512;
hipError_t launch_snapshot_rows(const float *C, int64_t ldc, int64_t strideC, int batch, int m, int n, int step, float *ref,
                                hipStream_t s);
hipError_t launch_compare_rows(const float *C, int64_t ldc, int64_t strideC, int batch, int m, int n, int step, const float *ref,
                               double *partial, hipStream_t s);

// Device address, on the current device, of the library's fixed-size scratch array (static_scratch.hip).
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
hipError_t static_scratch(void **ptr);

constexpr int kLdsPerCU = 160 * 1024;  // gfx950

// Raises a kernel's dynamic LDS limit to the whole LDS of a CU, once per device (`done` holds one
// bit per device index of this process; the runtime keeps the attribute per device).
inline hipError_t allow_full_lds(const void *kernel, std::atomic<uint64_t> &done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsPerCU);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
}
constexpr int kLdsPadA = 4;  // floats added to each A row in LDS (conflict-free b128 reads)
constexpr int kLdsPadB = 8;  // floats added to each B row in LDS

// The two LDS stages of the register-staged kernels: A then B of a stage side by side, the second stage right
// after the first.
template <int BM, int BN, int BK>
constexpr int tile_stage_floats() {
    return BM * (BK + kLdsPadA) + BK * (BN + kLdsPadB);
}
template <int BM, int BN, int BK>
constexpr int tile_stage_pitch() {
    return tile_stage_floats<BM, BN, BK>();
}
template <int BM, int BN, int BK, int WM, int WN>
constexpr int tile_lds_bytes() {
    return (tile_stage_pitch<BM, BN, BK>() + tile_stage_floats<BM, BN, BK>()) * (int)sizeof(float);
}

}  // namespace tg
