// bf16-piece SGEMM for gfx950 with the operands cut ahead of the product: a pass over A and one over
// B write the three bf16 pieces of every element into a workspace, already in the order the K loop's
// LDS stages use, and the product kernel moves those images global -> LDS directly
// (global_load_lds_dwordx4): no staging registers, no cutting and no LDS write instructions in the loop.
//
// Same arithmetic as tile_pieces_kernel.hpp (matmul of Sec. 5.2 of the paper from NP = 6 or 9 products
// of bf16 pieces per fp32 product, leading products and small terms in separate fp32 accumulators);
// cutting once per element instead of once per workgroup that uses it costs 6 bytes of workspace per
// operand element and two bandwidth-bound passes, and takes 264 of the ~380 non-MFMA instructions per
// K tile out of the loop.  The passes pad every tile with zeros, so m, n and k are arbitrary here and A
// and B need no alignment, nor does C.
//
// Workspace image.  A: [problem][tile row tm][K tile kt] blocks of 3 * (BK/8) * BM 16-byte entries,
// entry (piece q, k chunk c, row r) at (q * BK/8 + c) * BM + r, holding the piece-q bf16 values of
// A[tm*BM + r][kt*BK + 8c .. 8c+7].  B: [problem][tile column tn][K tile kt] blocks of 3 * (BK/8) * BN
// entries, entry (q, c, position) holding B[kt*BK + 8c .. 8c+7][column]; positions are lane-interleaved
// per wave tile as in tile_pieces_kernel.hpp.  A block is one LDS stage image, byte for byte.
#pragma once

#include "tile_pieces_kernel.hpp"

namespace tg {

typedef __attribute__((address_space(3))) unsigned lds_u32;
typedef __attribute__((address_space(1))) const unsigned glb_u32;

template <int BM, int BN, int BK>
constexpr int precut_lds_bytes() {
    return 2 * 3 * (BK / 8) * (BM + BN) * 16;
}

// ---- the cutting passes ---------------------------------------------------------------------------

// One workgroup per (problem, tile row, K tile), in that order in a 1-D grid: BM rows x BK columns of A
// -> one block of the image.
// Thread slots (row, k chunk): 8 consecutive k of one row.  rs / cs: element strides between rows and
// along k (cs == 1 and `vec` set: 16-byte loads, at any 4-byte alignment).
template <int BM, int BK>
__global__ void __launch_bounds__(256) cut_a_kernel(const float *A, int64_t rs, int64_t cs, int64_t strideA, int m, int k,
                                                    int tiles_m, int ktiles, int vec, u32x4 *planes) {
    constexpr int NKC = BK / 8;
    const int kt = blockIdx.x % ktiles, tm = (blockIdx.x / ktiles) % tiles_m, prob = blockIdx.x / ktiles / tiles_m;
    const float *src = A + (int64_t)prob * strideA;
    u32x4 *dst = planes + (int64_t)blockIdx.x * (3 * NKC * BM);
#pragma unroll
    for (int i = 0; i < BM * NKC / 256; ++i) {
        const int f = threadIdx.x + i * 256;
        const int row = f / NKC, kc = f % NKC;
        const int gr = tm * BM + row, gk = kt * BK + kc * 8;
        float x[8];
        if (vec && gr < m && gk + 8 <= k) {
            const f32x4_a4 *q = reinterpret_cast<const f32x4_a4 *>(src + (int64_t)gr * rs + gk);
            const f32x4 lo = q[0], hi = q[1];
#pragma unroll
            for (int e = 0; e < 4; ++e) { x[e] = lo[e]; x[4 + e] = hi[e]; }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = (gr < m && gk + e < k) ? src[(int64_t)gr * rs + (int64_t)(gk + e) * cs] : 0.0f;
        }
        u32x4 pc[3];
        cut_pieces(x, pc);
#pragma unroll
        for (int q = 0; q < 3; ++q) dst[(q * NKC + kc) * BM + row] = pc[q];
    }
}

// One workgroup per (problem, tile column, K tile): BK rows x BN columns of B.  Thread slots
// (k chunk, 4 consecutive columns): 8 rows of 4 columns -> for each column the three entries of its pieces.
// rs / cs: element strides between rows (k) and along n.
template <int BN, int BK, int WN>
__global__ void __launch_bounds__(256) cut_b_kernel(const float *B, int64_t rs, int64_t cs, int64_t strideB, int k, int n,
                                                    int tiles_n, int ktiles, int vec, u32x4 *planes) {
    constexpr int NKC = BK / 8, CB = WN / 32;
    const int kt = blockIdx.x % ktiles, tn = (blockIdx.x / ktiles) % tiles_n, prob = blockIdx.x / ktiles / tiles_n;
    const float *src = B + (int64_t)prob * strideB;
    u32x4 *dst = planes + (int64_t)blockIdx.x * (3 * NKC * BN);
#pragma unroll
    for (int i = 0; i < NKC * (BN / 4) / 256; ++i) {
        const int f = threadIdx.x + i * 256;
        const int kc = f / (BN / 4), col = (f % (BN / 4)) * 4;
        const int gk = kt * BK + kc * 8, gc = tn * BN + col;
        f32x4 raw[8];
        if (vec && gk + 8 <= k && gc + 4 <= n) {
#pragma unroll
            for (int r = 0; r < 8; ++r) raw[r] = *reinterpret_cast<const f32x4_a4 *>(src + (int64_t)(gk + r) * rs + gc);
        } else {
#pragma unroll
            for (int r = 0; r < 8; ++r)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    raw[r][e] = (gk + r < k && gc + e < n) ? src[(int64_t)(gk + r) * rs + (int64_t)(gc + e) * cs] : 0.0f;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float x[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) x[r] = raw[r][e];
            u32x4 pc[3];
            cut_pieces(x, pc);
            const int j = col + e, jj = j % WN;
            const int pos = (j / WN) * WN + (jj % CB) * 32 + jj / CB;
#pragma unroll
            for (int q = 0; q < 3; ++q) dst[(q * NKC + kc) * BN + pos] = pc[q];
        }
    }
}

// ---- the product --------------------------------------------------------------------------------

template <int BM, int BN, int BK, int WM, int WN, int NP>
__global__ void __launch_bounds__((BM / WM) * (BN / WN) * 64, 1)
sgemm_tile_precut_kernel(const GemmParams p) {
    constexpr int WAVES_N = BN / WN;
    constexpr int NWAVES = (BM / WM) * (BN / WN);
    constexpr int RB = WM / 32, CB = WN / 32;
    constexpr int NKC = BK / 8, NSTEP = BK / 16;
    constexpr int A_STAGE = 3 * NKC * BM, B_STAGE = 3 * NKC * BN;       // 16-byte entries
    constexpr int A_LD = A_STAGE / (NWAVES * 64), B_LD = B_STAGE / (NWAVES * 64);
    static_assert(NP == 6 || NP == 9, "6 or 9 piece products per fp32 product");
    static_assert(BM % WM == 0 && BN % WN == 0 && WM % 32 == 0 && WN % 32 == 0, "tile shape");
    static_assert(CB == 2 || CB == 4, "wave tile width must be 64 or 128");
    static_assert(NSTEP >= 2 && NSTEP % 2 == 0, "fragment sets alternate per k step and per column block");
    static_assert(A_STAGE % (NWAVES * 64) == 0 && B_STAGE % (NWAVES * 64) == 0, "stage images must divide over the waves");

    extern __shared__ __attribute__((aligned(16))) u32x4 smem_precut[];
    u32x4 *As = smem_precut;                  // two A stages, then two B stages
    u32x4 *Bs = smem_precut + 2 * A_STAGE;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, h = lane >> 5;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    const unsigned total_work = (unsigned)p.tiles_m * (unsigned)p.tiles_n * (unsigned)p.splits * (unsigned)p.batch;
    int slice, tm, tn;
    map_workgroup(p, total_work, blockIdx.x, slice, tm, tn);
    const int prob = slice / p.splits, split = slice - prob * p.splits;
    const int m0 = tm * BM, n0 = tn * BN;

    const int kt_total = (p.k + BK - 1) / BK;
    const int kt_begin = split * p.ktiles_per_split;
    const int kt_stop = kt_begin + p.ktiles_per_split;
    const int kt_end = kt_stop < kt_total ? kt_stop : kt_total;

    // Images of this tile row / column, K tile 0; one K tile further is one stage image further.
    const u32x4 *planes_a = reinterpret_cast<const u32x4 *>(p.planes);
    const u32x4 *planes_b = planes_a + (int64_t)p.batch * p.tiles_m * kt_total * A_STAGE;
    const u32x4 *Ag = planes_a + (((int64_t)prob * p.tiles_m + tm) * kt_total) * A_STAGE;
    const u32x4 *Bg = planes_b + (((int64_t)prob * p.tiles_n + tn) * kt_total) * B_STAGE;

    // Load instruction j of a wave moves entries [slot*64, slot*64+64) of an image (A's for j < A_LD, then
    // B's), slot = j*NWAVES + wave; lane l supplies entry slot*64 + l.  Scalar image base + 32-bit lane offset.
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const unsigned lane_bytes = (unsigned)lane * 16u;
    auto issue_load = [&](const u32x4 *a_img, const u32x4 *b_img, int stage, int j) {
        if (j < A_LD) {
            const int slot = j * NWAVES + wave_u;
            __builtin_amdgcn_global_load_lds((glb_u32 *)(reinterpret_cast<const char *>(a_img + slot * 64) + lane_bytes),
                                             (lds_u32 *)(As + stage * A_STAGE + slot * 64), 16, 0, 0);
        } else {
            const int slot = (j - A_LD) * NWAVES + wave_u;
            __builtin_amdgcn_global_load_lds((glb_u32 *)(reinterpret_cast<const char *>(b_img + slot * 64) + lane_bytes),
                                             (lds_u32 *)(Bs + stage * B_STAGE + slot * 64), 16, 0, 0);
        }
    };

    f32x16 acc_hi[RB][CB], acc_lo[RB][CB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            acc_hi[rb][cb] = (f32x16)(0.0f);
            acc_lo[rb][cb] = (f32x16)(0.0f);
        }

    u32x4 a_fr[2][RB][3], b_fr[2][3];
    const int a_src = h * BM + wm * WM + li;
    const int b_src = h * BN + wn * WN + li;
    auto read_a = [&](int stage, int step, int set) {
        const u32x4 *src = As + stage * A_STAGE + a_src + step * 2 * BM;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int q = 0; q < 3; ++q) a_fr[set][rb][q] = src[q * NKC * BM + rb * 32];
    };
    auto read_b = [&](int stage, int step, int cb, int set) {
        const u32x4 *src = Bs + stage * B_STAGE + b_src + step * 2 * BN + cb * 32;
#pragma unroll
        for (int q = 0; q < 3; ++q) b_fr[set][q] = src[q * NKC * BN];
    };
    auto mfma_block = [&](int aset, int bset, int cb) {
        constexpr int order9[9][2] = {{2, 2}, {1, 2}, {2, 1}, {0, 2}, {2, 0}, {1, 1}, {0, 1}, {1, 0}, {0, 0}};
#pragma unroll
        for (int t = 9 - NP; t < 9; ++t) {
            const int qa = order9[t][0], qb = order9[t][1];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                const bf16x8 av = __builtin_bit_cast(bf16x8, a_fr[aset][rb][qa]);
                const bf16x8 bv = __builtin_bit_cast(bf16x8, b_fr[bset][qb]);
                if (t == 8) acc_hi[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc_hi[rb][cb], 0, 0, 0);
                else acc_lo[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc_lo[rb][cb], 0, 0, 0);
            }
        }
    };

    // K loop over two LDS stages.  While tile kt multiplies out of stage s, the image of tile kt+1
    // streams into stage s^1 (free since the barrier that ended tile kt-1); before the barrier that
    // ends tile kt every wave waits for its own loads (vmcnt(0)).  Past the end of the range the last
    // image is fetched again into the stage nobody reads, so every iteration is the same sequence.
    constexpr int G = NSTEP * CB;
    constexpr int N_MFMA = RB * NP;
    constexpr int N_LD = A_LD + B_LD;
    constexpr int LD_PER_GROUP = (N_LD + G - 2) / (G - 1);
    if (kt_begin < kt_end) {
        const int last = kt_end - 1;
        {
            const u32x4 *a_img = Ag + (int64_t)kt_begin * A_STAGE, *b_img = Bg + (int64_t)kt_begin * B_STAGE;
#pragma unroll
            for (int j = 0; j < N_LD; ++j) issue_load(a_img, b_img, 0, j);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __syncthreads();
        read_a(0, 0, 0);
        read_b(0, 0, 0, 0);
        int stage = 0;
        for (int kt = kt_begin; kt <= last; ++kt) {
            const int nt = kt < last ? kt + 1 : last;
            const u32x4 *a_img = Ag + (int64_t)nt * A_STAGE, *b_img = Bg + (int64_t)nt * B_STAGE;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int g = 0; g < G - 1; ++g) {
                const int step = g / CB, cb = g % CB;
                // two MFMAs first: the compiler waits for all LDS traffic before a fragment read while
                // direct loads are in flight, and the reads of the previous group had a whole group to land
                mfma_block(step & 1, cb & 1, cb);
                if (cb + 1 < CB) {
                    read_b(stage, step, cb + 1, (cb + 1) & 1);
                } else {
                    read_a(stage, step + 1, (step + 1) & 1);
                    read_b(stage, step + 1, 0, 0);
                }
#pragma unroll
                for (int i = 0; i < LD_PER_GROUP; ++i)
                    if (g * LD_PER_GROUP + i < N_LD) issue_load(a_img, b_img, stage ^ 1, g * LD_PER_GROUP + i);
                __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                       // MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 3 * RB + 3, 0);              // fragment reads (3 or 3*RB+3)
#pragma unroll
                for (int i = 0; i < LD_PER_GROUP; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                   // global -> LDS load
                }
                __builtin_amdgcn_sched_group_barrier(0x008, N_MFMA, 0);                  // the rest
                __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_s_waitcnt(0x0F70);   // this wave's share of tile kt+1 has landed
            __syncthreads();                      // everyone's has; stage s is free
            mfma_block((NSTEP - 1) & 1, (CB - 1) & 1, CB - 1);
            read_a(stage ^ 1, 0, 0);
            read_b(stage ^ 1, 0, 0, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 3 * RB + 3, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, N_MFMA, 0);
            __builtin_amdgcn_sched_barrier(0);
            stage ^= 1;
        }
    }

    // Epilogue: registers -> C (or the split-K partial).
    float *out;
    int64_t ldo;
    if (p.splits > 1) {
        out = p.ws + (int64_t)slice * p.m * p.n;
        ldo = p.n;
    } else {
        out = p.C + (int64_t)prob * p.strideC;
        ldo = p.ldc;
    }
    typedef typename vec_of<CB>::type cvec;
    const bool full_tile = m0 + BM <= p.m && n0 + BN <= p.n;
    const int col = n0 + wn * WN + li * CB;
    const bool lane_vec = col + CB <= p.n;
    const bool nt = p.splits == 1 && rows_aligned<CB>(out, ldo);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = m0 + wm * WM + rb * 32 + 8 * (v / 4) + 4 * h + (v % 4);
            cvec o;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) o[cb] = acc_hi[rb][cb][v] + acc_lo[rb][cb][v];
            float *dst = out + (int64_t)row * ldo + col;
            if (full_tile || row < p.m) store_lane<CB>(dst, o, lane_vec, col, p.n, nt);
        }
    }
}

// Bytes of the piece images of a problem set (A's, then B's).
template <int BM, int BN, int BK>
inline int64_t precut_image_bytes(int64_t batch, int64_t m, int64_t n, int64_t k) {
    const int64_t tm = (m + BM - 1) / BM, tn = (n + BN - 1) / BN, kt = (k + BK - 1) / BK;
    return batch * kt * (tm * BM + tn * BN) * 3 * (BK / 8) * 16;
}

template <int BM, int BN, int BK, int WM, int WN, int NP>
hipError_t launch_tile_precut(const GemmParams &p, hipStream_t s) {
    constexpr int threads = (BM / WM) * (BN / WN) * 64;
    constexpr int lds = precut_lds_bytes<BM, BN, BK>();
    static_assert(BM * (BK / 8) % 256 == 0 && (BK / 8) * (BN / 4) % 256 == 0, "cutting passes use 256 threads");
    if (p.planes == nullptr) return hipErrorInvalidValue;
    auto kern = sgemm_tile_precut_kernel<BM, BN, BK, WM, WN, NP>;
    static std::atomic<uint64_t> lds_limit_raised{0};
    const hipError_t attr = allow_full_lds(reinterpret_cast<const void *>(kern), lds_limit_raised);
    if (attr != hipSuccess) return attr;
    const int ktiles = (p.k + BK - 1) / BK;
    u32x4 *planes_a = reinterpret_cast<u32x4 *>(p.planes);
    u32x4 *planes_b = planes_a + (int64_t)p.batch * p.tiles_m * ktiles * (3 * (BK / 8) * BM);
    const int vec_a = (p.flags & kFlagVecA) != 0, vec_b = (p.flags & kFlagVecB) != 0;
    hipLaunchKernelGGL((cut_a_kernel<BM, BK>), dim3((unsigned)((int64_t)ktiles * p.tiles_m * p.batch)), dim3(256), 0, s, p.A, p.lda, p.csa,
                       p.strideA, p.m, p.k, p.tiles_m, ktiles, vec_a, planes_a);
    hipLaunchKernelGGL((cut_b_kernel<BN, BK, WN>), dim3((unsigned)((int64_t)ktiles * p.tiles_n * p.batch)), dim3(256), 0, s, p.B, p.ldb, p.csb,
                       p.strideB, p.k, p.n, p.tiles_n, ktiles, vec_b, planes_b);
    const int64_t blocks = (int64_t)p.tiles_m * p.tiles_n * p.splits * p.batch;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(threads), lds, s, p);
    return hipGetLastError();
}

}  // namespace tg
