// Workgroup-tile SGEMM for gfx950 that forms every fp32 product from bf16 pieces on the bf16
// matrix pipe (v_mfma_f32_32x32x16_bf16, 16x the fp32 MFMA's multiply rate).
//
// Computes the same matmul (Sec. 5.2 of the paper), C[i][j] = sum_p A[i][p] B[p][j], row-major,
// fp32 in and out.  Each operand element x is cut into three bf16 pieces x = x1 + x2 + x3, each
// holding the next 8 bits of the 24-bit significand (exact for every finite fp32 value whose
// pieces do not underflow).  A product of two pieces is exact in fp32, so
//   a*b = a1b1 + (a1b2 + a2b1) + (a1b3 + a2b2 + a3b1) [+ a2b3 + a3b2 + a3b3]
// with NP = 6 products leaves out only terms below 2^-23 |a*b| (less than the rounding of one fp32
// product); NP = 9 takes them all.  The leading products a1b1 run in one set of fp32 accumulators,
// all smaller ones in a second set that is added at the end: the long chain then has one rounding
// per 16 k, and the small terms round at their own, 2^-8 smaller, magnitude.
//
// Data path: every thread fetches raw fp32 operand values of the next K tile into registers
// (16-byte loads), cuts them into pieces with a handful of integer/float operations in the shadow
// of the MFMAs, and writes the pieces to LDS as three planes per operand, [piece][k chunk of 8][row]
// of 16-byte entries (8 consecutive k of one row of A / one column of B: exactly one MFMA operand of
// one lane).  LDS is double-buffered with one barrier per K tile.
// Column ownership is interleaved as in the fp32 tile kernel: lane i of a wave holds columns
// CB*i .. CB*i+CB-1 of the wave tile (CB = WN/32), so a row segment of C is one CB*4-byte store; the
// permutation costs nothing, it is applied where B's pieces are written to LDS.
//
// Exact-fit rules: 16-byte aligned operands, k % BK == 0, n % 4 == 0; m and n need not be multiples of
// the tile (edge tiles re-read the last row / vector and mask their stores).
#pragma once

#include "tile_kernel.hpp"


namespace tg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kPiecePadA = 4;   // 16-byte entries added to each k-chunk row of A's planes (conflict-free writes)
constexpr int kPiecePadB = 4;

template <int BM, int BN, int BK>
constexpr int pieces_lds_bytes() {
    return 2 * 3 * (BK / 8) * ((BM + kPiecePadA) + (BN + kPiecePadB)) * 16;
}

// The upper halves of two floats as one register: (hi16(x1) << 16) | hi16(x0).
__device__ __forceinline__ unsigned pack_upper_halves(float x0, float x1) {
    return __builtin_amdgcn_perm(__float_as_uint(x1), __float_as_uint(x0), 0x07060302u);
}

// x - (piece e of the packed pair pk), where the piece is the bf16 in half e: one dot-product
// instruction, pk . (-1, 0) + x or pk . (0, -1) + x.  The product is exact and so is the sum (the
// remainder of a truncation is representable).
// Cuts 8 values into pieces: out[p] = the p-th bf16 pieces of x[0..7], element e in half e%2 of
// register e/2 (the operand order of the MFMA).  Truncating cuts: piece and remainder keep the sign of x,
// the subtraction is exact.
// (v_dot2c_f32_bf16 could subtract a packed piece in one instruction instead of the and + sub pair; it was
// tried and is several times slower per instruction, the kernel lost 7 %.)
__device__ __forceinline__ void cut_pieces(const float (&x)[8], u32x4 (&out)[3]) {
    float r[8];
#pragma unroll
    for (int e = 0; e < 8; e += 2) out[0][e / 2] = pack_upper_halves(x[e], x[e + 1]);
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = x[e] - __uint_as_float(__float_as_uint(x[e]) & 0xffff0000u);
#pragma unroll
    for (int e = 0; e < 8; e += 2) out[1][e / 2] = pack_upper_halves(r[e], r[e + 1]);
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = r[e] - __uint_as_float(__float_as_uint(r[e]) & 0xffff0000u);
#pragma unroll
    for (int e = 0; e < 8; e += 2) out[2][e / 2] = pack_upper_halves(r[e], r[e + 1]);
}

// Columns of B per load slot: four (16-byte loads) when that still gives every thread a slot, else two, else one.
template <int BN, int BK, int NT>
constexpr int pieces_b_cols() {
    return (BK / 8) * (BN / 4) >= NT ? 4 : ((BK / 8) * (BN / 2) >= NT ? 2 : 1);
}

// Small wave tiles leave room for two waves per SIMD (two workgroups per CU cover each other's waits).
template <int BM, int BN, int BK, int WM, int WN>
constexpr int pieces_min_waves() {
    constexpr int nt = (BM / WM) * (BN / WN) * 64;
    constexpr int acc = 2 * (WM / 32) * (WN / 32) * 16;
    constexpr int frags = 2 * 3 * 4 * (WM / 32 + 1);
    constexpr int raw = (BM * BK + BK * BN) / nt;
    return acc + frags + raw + 64 <= 256 ? 2 : 1;
}

template <int BM, int BN, int BK, int WM, int WN, int NP>
__global__ void __launch_bounds__((BM / WM) * (BN / WN) * 64, (pieces_min_waves<BM, BN, BK, WM, WN>()))
sgemm_tile_pieces_kernel(const GemmParams p) {
    constexpr int WAVES_N = BN / WN;
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    constexpr int RB = WM / 32, CB = WN / 32;
    constexpr int NKC = BK / 8;            // k chunks (one MFMA operand each) per K tile
    constexpr int NSTEP = BK / 16;         // MFMA k steps per K tile
    constexpr int A_PITCH = BM + kPiecePadA, B_PITCH = BN + kPiecePadB;   // entries per k chunk
    constexpr int A_STAGE = 3 * NKC * A_PITCH, B_STAGE = 3 * NKC * B_PITCH;
    constexpr int BC = pieces_b_cols<BN, BK, NT>();   // columns of B per load slot
    constexpr int A_SL = BM * NKC / NT;          // A slots per thread: 8 consecutive k of one row
    constexpr int B_SL = NKC * (BN / BC) / NT;   // B slots per thread: 8 consecutive k of BC columns
    static_assert(NP == 6 || NP == 9, "6 or 9 piece products per fp32 product");
    static_assert(BM % WM == 0 && BN % WN == 0 && WM % 32 == 0 && WN % 32 == 0, "tile shape");
    static_assert(CB == 1 || CB == 2 || CB == 4, "wave tile width must be 32, 64 or 128");
    static_assert(NSTEP >= 2 && NSTEP % 2 == 0, "fragment sets alternate per k step and per group");
    static_assert((BM * NKC) % NT == 0 && (NKC * (BN / BC)) % NT == 0 && A_SL >= 1 && B_SL >= 1,
                  "tile loads must divide evenly over the workgroup");
    typedef typename vec_of<BC>::type braw;

    extern __shared__ __attribute__((aligned(16))) u32x4 smem_pieces[];
    u32x4 *As = smem_pieces;
    u32x4 *Bs = smem_pieces + 2 * A_STAGE;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, h = lane >> 5;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    const unsigned total_work = (unsigned)p.tiles_m * (unsigned)p.tiles_n * (unsigned)p.splits * (unsigned)p.batch;
    int slice, tm, tn;
    map_workgroup(p, total_work, blockIdx.x, slice, tm, tn);
    const int prob = slice / p.splits, split = slice - prob * p.splits;
    const int m0 = tm * BM, n0 = tn * BN;

    const int kt_total = p.k / BK;
    const int kt_begin = split * p.ktiles_per_split;
    const int kt_stop = kt_begin + p.ktiles_per_split;
    const int kt_end = kt_stop < kt_total ? kt_stop : kt_total;

    // Slots of the tile loads.  A: slot f = (row f / NKC, k chunk f % NKC): the threads of one row
    // cover BK*4 contiguous bytes.  B: slot f = (k chunk f / (BN/BC), column group f % (BN/BC)) of BC columns.
    // Rows / vectors past the end of a ragged last tile re-read the last one (in bounds, never stored).
    // Offsets are in bytes and fit 32 bits (checked on the host): scalar base + 32-bit lane offset addressing.
    unsigned a_off[A_SL], b_off[B_SL];
    int a_dst[A_SL], b_dst[B_SL][BC];
#pragma unroll
    for (int i = 0; i < A_SL; ++i) {
        const int f = tid + i * NT;
        const int row = f / NKC, kc = f % NKC;
        const int r = row < p.m - 1 - m0 ? row : p.m - 1 - m0;
        a_off[i] = ((unsigned)r * (unsigned)p.lda + (unsigned)kc * 8u) * 4u;
        a_dst[i] = kc * A_PITCH + row;
    }
#pragma unroll
    for (int i = 0; i < B_SL; ++i) {
        const int f = tid + i * NT;
        const int kc = f / (BN / BC), col = (f % (BN / BC)) * BC;
        const int c = col < p.nb - BC - n0 ? col : p.nb - BC - n0;   // (nb % 4 == 0: at least BC columns exist)
        b_off[i] = ((unsigned)(kc * 8) * (unsigned)p.ldb + (unsigned)c) * 4u;
#pragma unroll
        for (int e = 0; e < BC; ++e) {
            // tile column -> position in the plane: lane-interleaved inside the owning wave's range
            const int j = col + e, jj = j % WN;
            b_dst[i][e] = kc * B_PITCH + (j / WN) * WN + (jj % CB) * 32 + jj / CB;
        }
    }

    f32x4 a_raw[A_SL][2];
    braw b_raw[B_SL][8];

    // Raw loads of one K tile, by slot; At / Bt point at that tile.
    auto load_a_slot = [&](const float *At, int i) {
        const char *src = reinterpret_cast<const char *>(At) + a_off[i];
        a_raw[i][0] = *reinterpret_cast<const f32x4 *>(src);
        a_raw[i][1] = *reinterpret_cast<const f32x4 *>(src + 16);
    };
    auto load_b_slot = [&](const float *Bt, int i) {
#pragma unroll
        for (int r = 0; r < 8; ++r)   // (row base in scalar registers + the thread's 32-bit offset)
            b_raw[i][r] = *reinterpret_cast<const braw *>(reinterpret_cast<const char *>(Bt + (int64_t)r * p.ldb) + b_off[i]);
    };
    auto load_tile = [&](const float *At, const float *Bt) {
#pragma unroll
        for (int i = 0; i < B_SL; ++i) load_b_slot(Bt, i);
#pragma unroll
        for (int i = 0; i < A_SL; ++i) load_a_slot(At, i);
    };

    // The cut-and-store work of one K tile in units of 8 values (one LDS entry per piece): units
    // 0 .. BC*B_SL-1 are the columns of the B slots, the rest the A slots.  Once the last unit of a slot
    // is cut, its registers are free and take the same slot of the tile after (At, Bt): every load
    // then has most of a K tile's MFMAs to arrive.
    constexpr int N_UNITS = A_SL + BC * B_SL;
    auto cut_and_store = [&](int stage, int u) {
        float x[8];
        u32x4 pc[3];
        if (u < BC * B_SL) {
            const int i = u / BC, ec = u % BC;
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = vec_get(b_raw[i][e], ec);
            cut_pieces(x, pc);
            u32x4 *dst = Bs + stage * B_STAGE + b_dst[i][ec];
#pragma unroll
            for (int q = 0; q < 3; ++q) dst[q * NKC * B_PITCH] = pc[q];
        } else {
            const int i = u - BC * B_SL;
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = a_raw[i][e / 4][e % 4];
            cut_pieces(x, pc);
            u32x4 *dst = As + stage * A_STAGE + a_dst[i];
#pragma unroll
            for (int q = 0; q < 3; ++q) dst[q * NKC * A_PITCH] = pc[q];
        }
    };
    auto reload_after = [&](const float *At, const float *Bt, int u) {
        if (u < BC * B_SL) {
            if (u % BC == BC - 1) load_b_slot(Bt, u / BC);
        } else {
            load_a_slot(At, u - BC * B_SL);
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

    // Operand fragments: A for a whole k step (two sets, by step parity), B for one column block
    // (two sets, by block parity); the next set is read from LDS while the current one multiplies.
    u32x4 a_fr[2][RB][3], b_fr[2][3];
    const int a_src = h * A_PITCH + wm * WM + li;
    const int b_src = h * B_PITCH + wn * WN + li;
    auto read_a = [&](int stage, int step, int set) {
        const u32x4 *src = As + stage * A_STAGE + a_src + step * 2 * A_PITCH;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int q = 0; q < 3; ++q) a_fr[set][rb][q] = src[q * NKC * A_PITCH + rb * 32];
    };
    auto read_b = [&](int stage, int step, int cb, int set) {
        const u32x4 *src = Bs + stage * B_STAGE + b_src + step * 2 * B_PITCH + cb * 32;
#pragma unroll
        for (int q = 0; q < 3; ++q) b_fr[set][q] = src[q * NKC * B_PITCH];
    };

    // Products of one column block, smallest first; consecutive MFMAs go to different accumulators.
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

    // K loop.  Groups g = (k step, column block) of RB*NP MFMAs each; G groups per K tile.  While
    // tile kt multiplies out of stage s, the raw values of tile kt+1 are cut and written to stage s^1,
    // one unit per group, and each freed slot is refilled with tile kt+2; one barrier; during the last
    // group the first fragments of tile kt+1 are read.
    // (Measured on MI355X: an MFMA of this shape occupies the pipe for 32 cycles and up to four
    // independent vector instructions issue in its shadow at about one cycle each; beyond that every
    // further one costs its full four to five cycles.  Hence four per MFMA below.)
    constexpr int G = NSTEP * CB;
    static_assert(G % 2 == 0, "the B fragment sets alternate per group");
    constexpr int UPG = (N_UNITS + G - 2) / (G - 1);   // units per group (1 for the large tile)
    constexpr int N_MFMA = RB * NP;                    // MFMAs of one group
    // vector instructions of one group's cutting (44 per unit) spread over its MFMAs, four at least
    constexpr int VALU_PER_MFMA = (UPG * 44 + N_MFMA - 1) / N_MFMA > 4 ? (UPG * 44 + N_MFMA - 1) / N_MFMA : 4;
    constexpr int MEM_PER_MFMA = (UPG * 11 + N_MFMA - 1) / N_MFMA;   // LDS writes (3 per unit) and reloads (up to 8)
    if (kt_begin < kt_end) {
        const int last = kt_end - 1;
        const float *A0 = p.A + (int64_t)prob * p.strideA + (int64_t)m0 * p.lda;
        const float *B0 = p.B + (int64_t)prob * p.strideB + n0;
        // tile t of the operands; asking beyond the last tile of the range gives the last one (in bounds)
        auto a_tile = [&](int t) { return A0 + (int64_t)(t < last ? t : last) * BK; };
        auto b_tile = [&](int t) { return B0 + (int64_t)(t < last ? t : last) * BK * p.ldb; };
        load_tile(a_tile(kt_begin), b_tile(kt_begin));
#pragma unroll
        for (int u = 0; u < N_UNITS; ++u) cut_and_store(0, u);
        __syncthreads();
        read_a(0, 0, 0);
        read_b(0, 0, 0, 0);
        if (kt_begin < last) load_tile(a_tile(kt_begin + 1), b_tile(kt_begin + 1));
        int stage = 0;
        for (int kt = kt_begin; kt < last; ++kt) {
            const float *At = a_tile(kt + 2), *Bt = b_tile(kt + 2);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int g = 0; g < G - 1; ++g) {
                const int step = g / CB, cb = g % CB;
                if (cb + 1 < CB) {
                    read_b(stage, step, cb + 1, (g + 1) & 1);
                } else {
                    read_a(stage, step + 1, (step + 1) & 1);
                    read_b(stage, step + 1, 0, (g + 1) & 1);
                }
#pragma unroll
                for (int uu = 0; uu < UPG; ++uu) {
                    const int u = g * UPG + uu;
                    if (u < N_UNITS) {
                        cut_and_store(stage ^ 1, u);
                        reload_after(At, Bt, u);
                    }
                }
                mfma_block(step & 1, g & 1, cb);
                // every other instruction in the shadow of an MFMA: the fragment reads first, then the
                // cuts with their LDS writes and the reloads spread over the group
#pragma unroll
                for (int i = 0; i < N_MFMA; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);               // MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);               // LDS read
                    __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER_MFMA, 0);   // VALU
                    __builtin_amdgcn_sched_group_barrier(0x220, MEM_PER_MFMA, 0);    // LDS write or global load
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            __syncthreads();
            read_a(stage ^ 1, 0, 0);
            read_b(stage ^ 1, 0, 0, 0);
            mfma_block((NSTEP - 1) & 1, (G - 1) & 1, CB - 1);
            __builtin_amdgcn_sched_group_barrier(0x100, 3 * RB + 3, 0);   // the first fragments of the next tile
            __builtin_amdgcn_sched_group_barrier(0x008, N_MFMA, 0);
            __builtin_amdgcn_sched_barrier(0);
            stage ^= 1;
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int step = g / CB, cb = g % CB;
            if (cb + 1 < CB) {
                read_b(stage, step, cb + 1, (g + 1) & 1);
            } else if (step + 1 < NSTEP) {
                read_a(stage, step + 1, (step + 1) & 1);
                read_b(stage, step + 1, 0, (g + 1) & 1);
            }
            mfma_block(step & 1, g & 1, cb);
            __builtin_amdgcn_sched_barrier(0);
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
            if constexpr (CB == 1) {
                o = acc_hi[rb][0][v] + acc_lo[rb][0][v];
            } else {
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) o[cb] = acc_hi[rb][cb][v] + acc_lo[rb][cb][v];
            }
            float *dst = out + (int64_t)row * ldo + col;
            if (full_tile || row < p.m) store_lane<CB>(dst, o, lane_vec, col, p.n, nt);
        }
    }
}

template <int BM, int BN, int BK, int WM, int WN, int NP>
hipError_t launch_tile_pieces(const GemmParams &p, hipStream_t s) {
    constexpr int threads = (BM / WM) * (BN / WN) * 64;
    constexpr int lds = pieces_lds_bytes<BM, BN, BK>();
    auto kern = sgemm_tile_pieces_kernel<BM, BN, BK, WM, WN, NP>;
    static std::atomic<uint64_t> lds_limit_raised{0};
    const hipError_t attr = allow_full_lds(reinterpret_cast<const void *>(kern), lds_limit_raised);
    if (attr != hipSuccess) return attr;
    const int64_t blocks = (int64_t)p.tiles_m * p.tiles_n * p.splits * p.batch;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(threads), lds, s, p);
    return hipGetLastError();
}

}  // namespace tg
