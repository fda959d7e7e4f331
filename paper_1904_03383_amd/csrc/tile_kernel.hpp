// Workgroup-tile SGEMM kernel for gfx950: C tile BM x BN per workgroup, K walked in
// tiles of BK through double-buffered LDS, each wave owning a WM x WN register block
// built from v_mfma_f32_32x32x2_f32 accumulators.
//
// Computes matmul of Sec. 5.2 of the paper, C[i][j] = sum_p A[i][p] B[p][j], row-major.
// In the paper's vocabulary (Sec. 4): the BM/BN tiling are the strip-mined m and n
// dimensions mapped to BLOCK, the wave/lane decomposition is the THREAD mapping, the
// fully unrolled BK loop is UNROLL, 16-byte accesses are VECTOR, and the LDS staging is
// the SHARED temporary array with its barrier between thread nests.
//
// Register/LDS data paths (all index maps are bijections of the plain definition; only
// the order in which the k terms are added differs from the textbook loop):
//  * A tile is kept row-major in LDS with rows padded to BK+4 floats.  Lane l of a wave
//    (i = l % 32, h = l / 32) fetches with one 16-byte read the four consecutive k
//    values 8o+4h .. 8o+4h+3 of row i and feeds element t to the t-th of four MFMAs, so
//    MFMA t of k-octet o multiplies the k pair (8o+t, 8o+4+t).  B uses the same pairing.
//  * Lane column ownership is interleaved: with CB = WN/32 column blocks per wave, lane
//    i holds columns CB*i .. CB*i+CB-1 of the wave tile (column CB*i+c in block c), so a
//    B fragment is one CB*4-byte LDS read and a C row segment is one CB*4-byte store.
//  * MFMA 32x32x2 result layout: register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4,
//    column l%32 of the 32x32 block.
#pragma once

#include "tg_internal.h"

namespace tg {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int N> struct vec_of;
template <> struct vec_of<1> { typedef float type; };
template <> struct vec_of<2> { typedef f32x2 type; };
template <> struct vec_of<4> { typedef f32x4 type; };

__device__ __forceinline__ float vec_get(float v, int) { return v; }
__device__ __forceinline__ float vec_get(f32x2 v, int i) { return v[i]; }
__device__ __forceinline__ float vec_get(f32x4 v, int i) { return v[i]; }

// Workgroup id -> (slice, tile row, tile column).
// Hardware hands consecutive workgroup ids to the 8 XCDs in turn, each XCD having its own
// L2.  The first step gives XCD x one contiguous range of logical ids, so the workgroups
// resident on one XCD at a time work on neighbouring tiles; the second step orders tiles
// inside a problem in groups of `group` tile rows walked column by column, which keeps the
// set of A and B panels in flight small.  slice = problem * splits + split.
__device__ __forceinline__ void map_workgroup(const GemmParams &p, int &slice, int &tm, int &tn) {
    const unsigned W = gridDim.x, w = blockIdx.x;
    const unsigned q = W >> 3, r = W & 7u, x = w & 7u, s = w >> 3;
    const unsigned logical = x * q + (x < r ? x : r) + s;
    const unsigned T = (unsigned)p.tiles_m * (unsigned)p.tiles_n;
    const unsigned sl = logical / T;
    const unsigned t = logical - sl * T;
    const unsigned gw = (unsigned)p.group * (unsigned)p.tiles_n;
    const unsigned g = t / gw;
    const unsigned first = g * (unsigned)p.group;
    const unsigned rest = (unsigned)p.tiles_m - first;
    const unsigned gsz = rest < (unsigned)p.group ? rest : (unsigned)p.group;
    const unsigned in = t - g * gw;
    slice = (int)sl;
    tm = (int)(first + in % gsz);
    tn = (int)(in / gsz);
}

template <int BM, int BN, int BK, int WM, int WN, bool TWO_LEVEL, bool EDGE>
__global__ void __launch_bounds__((BM / WM) * (BN / WN) * 64)
sgemm_tile_kernel(const GemmParams p) {
    constexpr int WAVES_N = BN / WN;
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    constexpr int RB = WM / 32, CB = WN / 32;
    constexpr int LDA_S = BK + kLdsPadA, LDB_S = BN + kLdsPadB;
    constexpr int A_STAGE = BM * LDA_S, B_STAGE = BK * LDB_S;
    constexpr int A_LD = BM * BK / 4 / NT, B_LD = BK * BN / 4 / NT;
    static_assert(BM % WM == 0 && BN % WN == 0 && WM % 32 == 0 && WN % 32 == 0, "tile shape");
    static_assert(CB == 1 || CB == 2 || CB == 4, "wave tile width must be 32, 64 or 128");
    static_assert(BK % 8 == 0, "BK must be a multiple of 8");
    static_assert((BM * BK / 4) % NT == 0 && (BK * BN / 4) % NT == 0 && A_LD >= 1 && B_LD >= 1,
                  "tile loads must divide evenly over the workgroup");
    typedef typename vec_of<CB>::type bvec;

    extern __shared__ __attribute__((aligned(16))) float smem[];
    float *As = smem;
    float *Bs = smem + 2 * A_STAGE;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, h = lane >> 5;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    int slice, tm, tn;
    map_workgroup(p, slice, tm, tn);
    const int prob = slice / p.splits, split = slice - prob * p.splits;
    const int m0 = tm * BM, n0 = tn * BN;

    const int kt_total = (p.k + BK - 1) / BK;
    const int kt_begin = split * p.ktiles_per_split;
    const int kt_stop = kt_begin + p.ktiles_per_split;
    const int kt_end = kt_stop < kt_total ? kt_stop : kt_total;

    const float *Ag = p.A + (int64_t)prob * p.strideA + (int64_t)m0 * p.lda + (int64_t)kt_begin * BK;
    const float *Bg = p.B + (int64_t)prob * p.strideB + (int64_t)kt_begin * BK * p.ldb + n0;

    // Per-thread slots of the tile loads: slot f = tid + i*NT is one 16-byte vector.
    int a_row[A_LD], a_k[A_LD], b_row[B_LD], b_col[B_LD];
    const float *a_ptr[A_LD], *b_ptr[B_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        const int f = tid + i * NT;
        a_row[i] = f / (BK / 4);
        a_k[i] = (f % (BK / 4)) * 4;
        a_ptr[i] = Ag + (int64_t)a_row[i] * p.lda + a_k[i];
    }
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        const int f = tid + i * NT;
        b_row[i] = f / (BN / 4);
        b_col[i] = (f % (BN / 4)) * 4;
        b_ptr[i] = Bg + (int64_t)b_row[i] * p.ldb + b_col[i];
    }

    f32x4 a_reg[A_LD], b_reg[B_LD];

    auto load_global = [&](int kt) {
        // kt is the absolute K-tile index of the tile being fetched.
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            if constexpr (!EDGE) {
                a_reg[i] = *reinterpret_cast<const f32x4 *>(a_ptr[i]);
            } else {
                const bool row_ok = m0 + a_row[i] < p.m;
                const int kk = kt * BK + a_k[i];
                f32x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (row_ok && kk + e < p.k) ? a_ptr[i][e] : 0.0f;
                a_reg[i] = v;
            }
            a_ptr[i] += BK;
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            if constexpr (!EDGE) {
                b_reg[i] = *reinterpret_cast<const f32x4 *>(b_ptr[i]);
            } else {
                const bool row_ok = kt * BK + b_row[i] < p.k;
                const int cc = n0 + b_col[i];
                f32x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (row_ok && cc + e < p.n) ? b_ptr[i][e] : 0.0f;
                b_reg[i] = v;
            }
            b_ptr[i] += (int64_t)BK * p.ldb;
        }
    };

    auto store_lds = [&](int stage) {
        float *as = As + stage * A_STAGE;
        float *bs = Bs + stage * B_STAGE;
#pragma unroll
        for (int i = 0; i < A_LD; ++i)
            *reinterpret_cast<f32x4 *>(as + a_row[i] * LDA_S + a_k[i]) = a_reg[i];
#pragma unroll
        for (int i = 0; i < B_LD; ++i)
            *reinterpret_cast<f32x4 *>(bs + b_row[i] * LDB_S + b_col[i]) = b_reg[i];
    };

    f32x16 acc[RB][CB];
    f32x16 total[TWO_LEVEL ? RB : 1][TWO_LEVEL ? CB : 1];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            acc[rb][cb] = (f32x16)(0.0f);
            if constexpr (TWO_LEVEL) total[rb][cb] = (f32x16)(0.0f);
        }

    const int a_frag_off = (wm * WM + li) * LDA_S + h * 4;
    const int b_frag_off = (h * 4) * LDB_S + wn * WN + li * CB;

    auto compute = [&](int stage) {
        const float *as = As + stage * A_STAGE + a_frag_off;
        const float *bs = Bs + stage * B_STAGE + b_frag_off;
#pragma unroll
        for (int o = 0; o < BK / 8; ++o) {
            f32x4 a_frag[RB];
            bvec b_frag[4];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                a_frag[rb] = *reinterpret_cast<const f32x4 *>(as + rb * 32 * LDA_S + o * 8);
#pragma unroll
            for (int t = 0; t < 4; ++t)
                b_frag[t] = *reinterpret_cast<const bvec *>(bs + (o * 8 + t) * LDB_S);
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb)
                        acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                            a_frag[rb][t], vec_get(b_frag[t], cb), acc[rb][cb], 0, 0, 0);
        }
    };

    int since_flush = 0;
    auto maybe_flush = [&]() {
        if constexpr (TWO_LEVEL) {
            if (++since_flush == p.flush_tiles) {
                since_flush = 0;
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb) {
                        total[rb][cb] += acc[rb][cb];
                        acc[rb][cb] = (f32x16)(0.0f);
                    }
            }
        }
    };

    if (kt_begin < kt_end) {
        load_global(kt_begin);
        store_lds(0);
        __syncthreads();
        int stage = 0;
        for (int kt = kt_begin; kt < kt_end - 1; ++kt) {
            load_global(kt + 1);          // next tile travels while this one is multiplied
            // Keep the loads issued here: without this fence the scheduler sinks them below
            // the MFMA block to save registers and their latency is no longer hidden.
            __builtin_amdgcn_sched_barrier(0);
            compute(stage);
            maybe_flush();
            store_lds(stage ^ 1);
            __syncthreads();              // one barrier per K tile (see header comment of the loop)
            stage ^= 1;
        }
        compute(stage);
    }
    if constexpr (TWO_LEVEL) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) acc[rb][cb] += total[rb][cb];
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
    const int col = n0 + wn * WN + li * CB;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = m0 + wm * WM + rb * 32 + 8 * (v / 4) + 4 * h + (v % 4);
            float *dst = out + (int64_t)row * ldo + col;
            if constexpr (!EDGE) {
                bvec o;
                if constexpr (CB == 1) {
                    o = acc[rb][0][v];
                } else {
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb) o[cb] = acc[rb][cb][v];
                }
                *reinterpret_cast<bvec *>(dst) = o;
            } else {
                if (row < p.m) {
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb)
                        if (col + cb < p.n) dst[cb] = acc[rb][cb][v];
                }
            }
        }
    }
}

template <int BM, int BN, int BK, int WM, int WN, bool TWO_LEVEL, bool EDGE>
hipError_t launch_tile(const GemmParams &p, hipStream_t s) {
    constexpr int threads = (BM / WM) * (BN / WN) * 64;
    constexpr int lds = tile_lds_bytes<BM, BN, BK, WM, WN>();
    auto kern = sgemm_tile_kernel<BM, BN, BK, WM, WN, TWO_LEVEL, EDGE>;
    if (lds > 48 * 1024) {
        static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (attr != hipSuccess) return attr;
    }
    const int64_t blocks = (int64_t)p.tiles_m * p.tiles_n * p.splits * p.batch;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(threads), lds, s, p);
    return hipGetLastError();
}

}  // namespace tg
