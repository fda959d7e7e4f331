// Workgroup-tile SGEMM kernel for gfx950 whose operand tiles travel global -> LDS directly
// (global_load_lds_dwordx4), without passing through registers.  Same decomposition as
// tile_kernel.hpp (matmul of Sec. 5.2 of the paper; BLOCK / THREAD / UNROLL / VECTOR
// mapping and SHARED staging of Sec. 4); aligned operands, k a multiple of BK, n of 4.
//
// What differs from the register-staged kernel:
//  * A direct load writes the 64 lanes' 16-byte pieces to 1 KB of consecutive LDS, so rows
//    cannot be padded.  The A tile (rows of BK floats = BK/4 chunks of 16 bytes) is instead
//    stored with its chunks permuted inside each row: chunk c of row r sits at position
//    c ^ swz(r).  The lane that fills LDS position (r, q) therefore fetches chunk
//    q ^ swz(r) from global memory, and a fragment read of chunk c goes to c ^ swz(r); the
//    16 lanes of one LDS access then hit distinct bank groups.
//  * The B tile is stored row by row (k-major, BN floats per row); its fragment reads are
//    runs of consecutive floats and need no permutation.
//  * There are no staging registers and no LDS write instructions: the loads of tile kt+1
//    are issued right after the barrier that frees their stage, between the MFMAs of the
//    first octet, and are waited for (vmcnt) just before the barrier that hands over their
//    stage.  NS LDS stages form a ring, so a tile may be NS-1 K tiles in flight.
//  * KG > 1 puts KG waves on every wave tile: wave group g multiplies octets
//    [g*NO/KG, (g+1)*NO/KG) of every K tile, and the groups' accumulators are summed through
//    LDS in a fixed order at the end.  A 64x64 workgroup tile (the largest that still gives
//    1024^3 one workgroup per CU) then runs two waves per SIMD.  Measured at 1024^3 it only
//    matches the one-group kernel (21.6 us against 21.9 us): the waits it could cover are not
//    what limits that shape.
//
// Operand modes (AM for A, BMD for B): the strided matmul and the transposed layouts of Sec. 5.2 fused
// into the loader, so that no separate gather / transpose pass is needed.
//  * mode 0: the operand as the plain product has it (A row-major with k contiguous, B row-major with n
//    contiguous), described above.
//  * mode 1: the operand is given transposed.  A with unit stride along m (element (i, p) at A[i + p*csa]):
//    its tile is loaded like a B tile, k-major rows of BM floats, no permutation; a lane owns the RB
//    adjacent rows RB*i .. RB*i+RB-1 of its wave tile (row RB*i+rb in block rb), so an A fragment for
//    one k is one RB*4-byte LDS read.  B with unit stride along k (element (p, j) at B[p + j*csb]): its
//    tile is loaded like an A tile, one LDS row of BK floats per column with the chunk permutation, and
//    LDS row cb*32+i of a wave's slab holds column CB*i+cb, so the fragment reads are the conflict-free
//    ones of A while a lane still owns CB adjacent columns of C.
//  * mode 2: arbitrary element strides (element (i, p) of A at A[i*rsa + p*csa], (p, j) of B at
//    B[p*rsb + j*csb]): every lane of a 4-byte direct load fetches one element, its own cache line if the
//    stride is large, into the LDS layout of mode 0.  Nothing is staged in registers, so with NS stages
//    NS-1 K tiles of gathered lines are in flight per workgroup, which is what a gather needs: its
//    latency is that of HBM, not of L2.
// Modes other than 0 exist only in this kernel; k must still be a multiple of BK.
#pragma once

#include "tile_kernel.hpp"

namespace tg {

typedef __attribute__((address_space(3))) float lds_float;
typedef __attribute__((address_space(1))) const float glb_float;

// Chunk permutation of A rows.  For BK = 32 (8 chunks per row) it is a bijection of the
// chunk index for every row, and distinct over each aligned group of 8 rows as well as over
// the even and the odd rows of each aligned group of 16, which covers both ways 16-byte LDS
// accesses may be grouped over banks.
template <int BK>
__device__ __forceinline__ int a_swizzle(int row) {
    static_assert(BK == 32 || BK == 64, "the chunk permutation is laid out for rows of 8 or 16 chunks");
    // (rows of 64 floats all start in bank 0: the low three bits of the row spread eight consecutive rows over the
    // eight 16-byte bank groups)
    if constexpr (BK == 64) return row & 7;
    else return (row & 6) | ((row ^ (row >> 3)) & 1);
}

template <int BM, int BN, int BK, int NS>
constexpr int direct_lds_bytes() {
    return NS * (BM * BK + BK * BN) * (int)sizeof(float);
}

// The two fp32 matrix instructions.  v_mfma_f32_32x32x2_f32: lane l (i = l % 32, h = l / 32) supplies A[i][k = h]
// and B[k = h][j = i], result register v (of 16) holds row 8*(v/4) + 4*h + v%4, column i.  v_mfma_f32_16x16x4_f32:
// lane l (i = l % 16, h = l / 16) supplies A[i][k = h] and B[k = h][j = i], result register v (of 4) holds row
// 4*h + v, column i.  Either way a lane fetches the four consecutive k values 4*h .. 4*h+3 of a step of 4 * (64 / MI)
// k values at once and feeds element t to the t-th of four instructions.
template <int MI> struct mfma_shape;
template <> struct mfma_shape<32> {
    typedef f32x16 acc_t;
    static __device__ __forceinline__ acc_t mfma(float a, float b, acc_t c) { return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ int row_of(int v, int h) { return 8 * (v / 4) + 4 * h + (v % 4); }
};
template <> struct mfma_shape<16> {
    typedef f32x4 acc_t;
    static __device__ __forceinline__ acc_t mfma(float a, float b, acc_t c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ int row_of(int v, int h) { return 4 * h + v; }
};

template <int BM, int BN, int BK, int WM, int WN, bool TWO_LEVEL>
constexpr int direct_min_waves() {
    constexpr int acc = (WM * WN / 64) * (TWO_LEVEL ? 2 : 1);
    constexpr int frags = 2 * (4 * (WM / 32) + 4 * (WN / 32));
    return acc + frags + 56 <= 256 ? 2 : 1;
}

// One K tile on its way: instruction i of a wave fills LDS floats [slot*256, slot*256+256) of
// the stage (64 floats for a gathered operand), slot = i * NWAVES + wave.  a_stage / b_stage are float offsets into the
// __shared__ array.  The builtin wants address-space-qualified pointers, hence the explicit
// casts (without them the host pass drops the kernel without a diagnostic).
// (A_EL / B_EL floats per lane and instruction: 4, or 1 for a gathered operand.  The size operand of the
// builtin must be a literal, hence the two wrappers.)
// A float address at a 32-bit byte offset from a wave-uniform origin (lane offsets are kept that way, see
// at_bytes in tile_kernel.hpp: the load then takes the origin from scalar registers and a 32-bit vector offset).
__device__ __forceinline__ const float *byte_offset(const float *base, unsigned &bytes) {
    asm volatile("" : "+v"(bytes));     // (in place: the offset passes through unchanged)
    return reinterpret_cast<const float *>(reinterpret_cast<const char *>(base) + bytes);
}
// lane offset in bytes (LEAN) or in elements
template <bool LEAN>
__device__ __forceinline__ const float *lane_address(const float *base, unsigned &off) {
    if constexpr (LEAN) return byte_offset(base, off);
    else return base + off;
}

template <int EL>
__device__ __forceinline__ void direct_load(const float *g, float *l);
template <>
__device__ __forceinline__ void direct_load<4>(const float *g, float *l) {
    __builtin_amdgcn_global_load_lds((glb_float *)g, (lds_float *)l, 16, 0, 0);
}
template <>
__device__ __forceinline__ void direct_load<1>(const float *g, float *l) {
    __builtin_amdgcn_global_load_lds((glb_float *)g, (lds_float *)l, 4, 0, 0);
}
// Debug flavour of the library (compiled with TG_POISON_LDS): before a stage is refilled, every lane overwrites
// the slots that its own loads are about to fill with NaN and waits for those writes.  A kernel that read a
// stage after giving it up, or before its loads had landed, then returns NaN instead of stale but plausible
// numbers.
#ifdef TG_POISON_LDS
template <int EL>
__device__ __forceinline__ void poison_slot(float *slot, int lane) {
    if constexpr (EL == 4) *reinterpret_cast<f32x4 *>(slot + lane * 4) = (f32x4)(__builtin_nanf(""));
    else slot[lane] = __builtin_nanf("");
}
#define TG_POISON_DIRECT(a_stage, b_stage)                                                               \
    do {                                                                                                 \
        _Pragma("unroll") for (int i_ = 0; i_ < A_LD; ++i_)                                              \
            poison_slot<A_EL>(smem + (a_stage) + (i_ * NWAVES + wave) * (64 * A_EL), lane);              \
        _Pragma("unroll") for (int i_ = 0; i_ < B_LD; ++i_)                                              \
            poison_slot<B_EL>(smem + (b_stage) + (i_ * NWAVES + wave) * (64 * B_EL), lane);              \
        __builtin_amdgcn_s_waitcnt(0xC07F);   /* lgkmcnt(0) */                                           \
    } while (0)
#else
#define TG_POISON_DIRECT(a_stage, b_stage) do { } while (0)
#endif
#define TG_ISSUE_DIRECT_LOADS(a_stage, b_stage)                                                          \
    do {                                                                                                 \
        TG_POISON_DIRECT(a_stage, b_stage);                                                              \
        _Pragma("unroll") for (int i_ = 0; i_ < A_LD; ++i_)                                              \
            direct_load<A_EL>(lane_address<LEAN>(Ag, a_off[i_]), smem + (a_stage) + (i_ * NWAVES + wave) * (64 * A_EL));    \
        _Pragma("unroll") for (int i_ = 0; i_ < B_LD; ++i_)                                              \
            direct_load<B_EL>(lane_address<LEAN>(Bg, b_off[i_]), smem + (b_stage) + (i_ * NWAVES + wave) * (64 * B_EL));    \
    } while (0)

template <int BM, int BN, int BK, int WM, int WN, bool TWO_LEVEL, int NS, int KG, int AM, int BMD, int MI>
__global__ void __launch_bounds__((BM / WM) * (BN / WN) * 64 * KG, (KG > 1 ? 2 : direct_min_waves<BM, BN, BK, WM, WN, TWO_LEVEL>()))
sgemm_tile_direct_kernel(const GemmParams p) {
    constexpr int WAVES_N = BN / WN;
    constexpr int TILE_WAVES = (BM / WM) * (BN / WN);       // waves that cover the output tile once
    constexpr int NWAVES = TILE_WAVES * KG;
    constexpr int NT = NWAVES * 64;
    static_assert(MI == 32 || MI == 16, "32x32x2 or 16x16x4 matrix instructions");
    constexpr int RB = WM / MI, CB = WN / MI;                // blocks of one instruction per wave tile
    constexpr int KSTEP = 4 * (64 / MI);                     // k values of one fragment fetch: an octet (MI = 32) or 16
    constexpr int NV = MI * MI / 64;                         // results per lane and block
    typedef mfma_shape<MI> shape;
    typedef typename shape::acc_t accv;
    constexpr int A_STAGE = BM * BK, B_STAGE = BK * BN;      // floats, unpadded
    constexpr int A_EL = AM == 2 ? 1 : 4, B_EL = BMD == 2 ? 1 : 4;   // floats per lane of one load instruction
    constexpr int A_LD = BM * BK / A_EL / NT, B_LD = BK * BN / B_EL / NT;
    constexpr int NO = BK / KSTEP / KG;                     // fragment steps ("octets" below) of a K tile per wave
    static_assert(AM >= 0 && AM <= 2 && BMD >= 0 && BMD <= 2, "operand modes");
    static_assert(KG == 1 || KG == 2, "one or two wave groups along K");
    static_assert(KG == 1 || (KG - 1) * BM * BN <= NS * (BM * BK + BK * BN), "the group sum reuses the stage area");
    static_assert(BM % WM == 0 && BN % WN == 0 && WM % MI == 0 && WN % MI == 0, "tile shape");
    static_assert(CB == 1 || CB == 2 || CB == 4, "wave tile width must be 1, 2 or 4 blocks");
    static_assert(BK == 32, "BK must be 32");
    static_assert(NO >= 2 && NO % 2 == 0, "fragment sets alternate per octet");
    static_assert((BM * BK / A_EL) % NT == 0 && (BK * BN / B_EL) % NT == 0 && A_LD >= 1 && B_LD >= 1,
                  "tile loads must divide evenly over the workgroup");
    static_assert(BN % 4 == 0 && BM % 4 == 0 && (256 % BK) == 0, "one load instruction covers whole chunks and rows");
    static_assert(NS >= 2 && NS <= 4, "two to four LDS stages");
    static_assert((NS - 2) * (A_LD + B_LD) <= 63, "outstanding loads must fit the vmcnt field");
    static_assert(RB == 1 || RB == 2 || RB == 4, "wave tile height must be 1, 2 or 4 blocks");
    typedef typename vec_of<CB>::type bvec;
    typedef typename vec_of<RB>::type avec;

    extern __shared__ __attribute__((aligned(16))) float smem[];
    float *As = smem;
    float *Bs = smem + NS * A_STAGE;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    // The 128x128 wave tile (256 accumulator registers) keeps the plainer addressing: measured 249 us against 254 us at
    // 4096x4096x1024 with the leaner one, which gains 2-3 % on every other variant.
    constexpr bool LEAN = WM * WN < 128 * 128;
    // (wave id in a scalar register: the LDS targets of the direct loads are wave-uniform)
    const int wave = LEAN ? __builtin_amdgcn_readfirstlane(tid >> 6) : (tid >> 6);
    const int li = lane % MI, h = lane / MI;
    const int kg = wave / TILE_WAVES, tw = wave % TILE_WAVES;   // K group, wave inside the tile
    const int wm = tw / WAVES_N, wn = tw % WAVES_N;
    const int o_base = kg * NO;

    // One workgroup per work item (tile x slice).
    const unsigned total_work = (unsigned)p.tiles_m * (unsigned)p.tiles_n * (unsigned)p.splits * (unsigned)p.batch;
    int slice, tm, tn;
    map_workgroup(p, total_work, blockIdx.x, slice, tm, tn);
    const int prob = slice / p.splits, split = slice - prob * p.splits;
    const int m0 = tm * BM, n0 = tn * BN;

    const int kt_total = p.k / BK;
    const int kt_begin = split * p.ktiles_per_split;
    const int kt_stop = kt_begin + p.ktiles_per_split;
    const int kt_end = kt_stop < kt_total ? kt_stop : kt_total;

    // Tile origins are wave-uniform and advance per K tile; per-lane offsets are fixed.
    // (lda, ldb: row strides of A and B; csa, csb: their element strides along k and along n.)
    const int64_t a_step = AM == 0 ? (int64_t)BK : (int64_t)BK * p.csa;
    const int64_t b_step = BMD == 1 ? (int64_t)BK : (int64_t)BK * p.ldb;
    const float *Ag = p.A + (int64_t)prob * p.strideA + (int64_t)m0 * p.lda + (int64_t)kt_begin * a_step;
    const float *Bg = p.B + (int64_t)prob * p.strideB + (int64_t)kt_begin * b_step + (int64_t)n0 * (BMD == 0 ? 1 : p.csb);

    // Load instruction i of this wave fills LDS floats [slot*256, slot*256 + 256) of a stage,
    // slot = i * NWAVES + wave; lane l supplies floats slot*256 + 4l .. +3 (a gathered operand:
    // [slot*64, slot*64 + 64), lane l the float slot*64 + l).
    constexpr unsigned OFF_UNIT = LEAN ? 4u : 1u;            // lane offsets in bytes or in elements (see lane_address)
    unsigned a_off[A_LD], b_off[B_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        const int pos = ((i * NWAVES + wave) * 64 + lane) * A_EL;   // float index inside the A stage
        if constexpr (AM == 1) {
            // k-major stage: row pos / BM is one k, BM consecutive m.  Ragged last tile row: vectors past
            // the end of A re-read its last one (m % 4 == 0; in bounds, what they produce is never stored)
            const int c = pos % BM < p.m - 4 - m0 ? pos % BM : p.m - 4 - m0;
            a_off[i] = OFF_UNIT * ((unsigned)(pos / BM) * (unsigned)p.csa + (unsigned)c);
        } else {
            const int row = pos / BK;
            const int q = (pos % BK) / 4;                      // chunk position inside the row
            // ragged last tile row: LDS rows past the end of A are filled from its last row (in bounds;
            // what they produce is never stored)
            const int src_row = row < p.m - 1 - m0 ? row : p.m - 1 - m0;
            const int src_k = (q ^ a_swizzle<BK>(row)) * 4 + (AM == 2 ? pos % 4 : 0);
            a_off[i] = OFF_UNIT * ((unsigned)src_row * (unsigned)p.lda + (unsigned)src_k * (AM == 2 ? (unsigned)p.csa : 1u));
        }
    }
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        const int pos = ((i * NWAVES + wave) * 64 + lane) * B_EL;   // float index inside the B stage
        if constexpr (BMD == 1) {
            // one LDS row of BK floats per column, chunks permuted as in A's stage; LDS row cb*MI+i of a
            // wave's slab holds column CB*i+cb.  Columns past the end of B re-read its last one.
            const int row = pos / BK;
            const int q = (pos % BK) / 4;
            const int col = (row / WN) * WN + (row % MI) * CB + (row % WN) / MI;
            const int src_col = col < p.n - 1 - n0 ? col : p.n - 1 - n0;
            b_off[i] = OFF_UNIT * ((unsigned)src_col * (unsigned)p.csb + (unsigned)((q ^ a_swizzle<BK>(row)) * 4));
        } else if constexpr (BMD == 2) {
            const int c = pos % BN < p.n - 1 - n0 ? pos % BN : p.n - 1 - n0;
            b_off[i] = OFF_UNIT * ((unsigned)(pos / BN) * (unsigned)p.ldb + (unsigned)c * (unsigned)p.csb);
        } else {
            // ragged last tile column: vectors past the end of B re-read its last one (n % 4 == 0)
            const int c = pos % BN < p.nb - 4 - n0 ? pos % BN : p.nb - 4 - n0;
            b_off[i] = OFF_UNIT * ((unsigned)(pos / BN) * (unsigned)p.ldb + (unsigned)c);
        }
    }

    accv acc[RB][CB];
    accv total[TWO_LEVEL ? RB : 1][TWO_LEVEL ? CB : 1];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            acc[rb][cb] = (accv)(0.0f);
            if constexpr (TWO_LEVEL) total[rb][cb] = (accv)(0.0f);
        }

    // Fragment addressing.  A (modes 0, 2): row r = wm*WM + rb*MI + li, chunk (KSTEP/4)*o + h at position
    // ((KSTEP/4)*o + h) ^ swz(r); rb*MI does not change swz (it only looks at the low four row bits).
    // A (mode 1): k-major stage, the lane's RB adjacent rows of k = KSTEP*o + 4*h + t.
    // B (modes 0, 2): k-major stage, the lane's CB adjacent columns.  B (mode 1): as A in mode 0.
    const int a_row = wm * WM + li;
    const int a_swz = a_swizzle<BK>(a_row);                  // == a_swizzle(li): also B's rows in mode 1
    const int a_frag_off = AM == 1 ? (h * 4) * BM + wm * WM + li * RB : a_row * BK;
    const int b_frag_off = BMD == 1 ? (wn * WN + li) * BK : (h * 4) * BN + wn * WN + li * CB;

    // a_frag[set][rb][t] (modes 0, 2) or a_fragT[set][t][rb] (mode 1); b_frag[set][t][cb] (modes 0, 2) or
    // b_fragT[set][cb][t] (mode 1)
    f32x4 a_frag[2][AM == 1 ? 1 : RB];
    avec a_fragT[2][AM == 1 ? 4 : 1];
    bvec b_frag[2][BMD == 1 ? 1 : 4];
    f32x4 b_fragT[2][BMD == 1 ? CB : 1];
    constexpr int N_FRAG_RD = (AM == 1 ? 4 : RB) + (BMD == 1 ? CB : 4);   // LDS reads of one octet

    auto read_frags = [&](int stage, int o, int set) {
        const int chunk = (((KSTEP / 4) * (o_base + o) + h) ^ a_swz) * 4;
        if constexpr (AM == 1) {
            const float *as = As + stage * A_STAGE + a_frag_off + (o_base + o) * KSTEP * BM;
#pragma unroll
            for (int t = 0; t < 4; ++t)
                a_fragT[set][t] = *reinterpret_cast<const avec *>(as + t * BM);
        } else {
            const float *as = As + stage * A_STAGE + a_frag_off + chunk;
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                a_frag[set][rb] = *reinterpret_cast<const f32x4 *>(as + rb * MI * BK);
        }
        if constexpr (BMD == 1) {
            const float *bs = Bs + stage * B_STAGE + b_frag_off + chunk;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
                b_fragT[set][cb] = *reinterpret_cast<const f32x4 *>(bs + cb * MI * BK);
        } else {
            const float *bs = Bs + stage * B_STAGE + b_frag_off + (o_base + o) * KSTEP * BN;
#pragma unroll
            for (int t = 0; t < 4; ++t)
                b_frag[set][t] = *reinterpret_cast<const bvec *>(bs + t * BN);
        }
    };

    auto mfma_octet = [&](int set) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    float av, bv;
                    if constexpr (AM == 1) av = vec_get(a_fragT[set][t], rb);
                    else av = a_frag[set][rb][t];
                    if constexpr (BMD == 1) bv = b_fragT[set][cb][t];
                    else bv = vec_get(b_frag[set][t], cb);
                    acc[rb][cb] = shape::mfma(av, bv, acc[rb][cb]);
                }
    };

    int since_flush = 0;
    auto maybe_flush = [&]() {
        if constexpr (TWO_LEVEL) {
            if (since_flush == p.flush_tiles) {
                since_flush = 0;
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb) {
                        total[rb][cb] += acc[rb][cb];
                        acc[rb][cb] = (accv)(0.0f);
                        __builtin_amdgcn_sched_barrier(0);
                    }
            }
            ++since_flush;
        }
    };

    // s_waitcnt that allows kOutstanding vector-memory operations to stay in flight and waits for every LDS
    // operation of the wave (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8).
    constexpr int N_MFMA = 4 * RB * CB;
    constexpr int N_LD = A_LD + B_LD;
    constexpr int kOutstanding = (NS - 2) * N_LD;
    // The barriers of the K loop are the bare instruction behind this wait, not __syncthreads(): the fence that
    // comes with the latter makes the compiler wait for every load in flight (vmcnt(0)) before each barrier, which
    // empties a ring of more than two stages at every K tile.  What the barrier has to order is covered by the
    // wait: a direct load counts as done (vmcnt) when its data is in LDS, and the wave's own LDS reads have
    // returned (lgkmcnt(0)) before it lets the others overwrite the stage they came from.
    constexpr int kWaitTile = 0x0070 | (kOutstanding & 15) | ((kOutstanding >> 4) << 14);
    constexpr int MFMA_PER_LD = (N_MFMA - 2) / N_LD > 0 ? (N_MFMA - 2) / N_LD : 1;

    // K loop over an NS-stage ring in LDS.  During tile t (stage t % NS) the loads of tile
    // t+NS-1 are issued into the stage tile t-1 has just left; before the barrier at the end of
    // tile t a wave waits until only the NS-2 youngest tiles' loads are still in flight, i.e.
    // until its share of tile t+1 has landed.  Small tiles need the depth: a 64x64x32 tile is
    // only 16 MFMAs per wave (0.4 us), far less than a trip to L2 or HBM.  Past the end of the
    // K range the last tile is fetched again (in bounds, never read), which keeps every
    // iteration, the tail included, the same instruction sequence with the same wait counts.
    if (kt_begin < kt_end) {
        int to_load = kt_end - kt_begin;            // tiles not fetched yet
#pragma unroll
        for (int st = 0; st < NS - 1; ++st) {
            TG_ISSUE_DIRECT_LOADS(st * A_STAGE, NS * A_STAGE + st * B_STAGE);
            if (to_load > 1) {
                --to_load;
                Ag += a_step;
                Bg += b_step;
            }
        }
        __builtin_amdgcn_s_waitcnt(kWaitTile);
        __builtin_amdgcn_s_barrier();
        read_frags(0, 0, 0);
        int stage = 0, fill = NS - 1;               // stage being multiplied / stage being filled
        for (int kt = kt_begin; kt < kt_end; ++kt) {
            maybe_flush();
            __builtin_amdgcn_sched_barrier(0);
            // Every octet: two MFMAs, then the fetch of the next octet's fragments, then the
            // rest of the MFMAs.  The compiler counts direct loads as pending LDS traffic of
            // another kind, which turns every LDS wait into a full one (lgkmcnt(0)) while
            // they are in flight; with this order the full wait always falls before the
            // next fetch is issued and after the previous one had most of an octet to finish.
            // octet 0 also starts the next tile of the ring on its way.
            mfma_octet(0);
            read_frags(stage, 1, 1);
            TG_ISSUE_DIRECT_LOADS(fill * A_STAGE, NS * A_STAGE + fill * B_STAGE);
            if (to_load > 1) {
                --to_load;
                Ag += a_step;
                Bg += b_step;
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);              // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, N_FRAG_RD, 0);      // LDS reads
#pragma unroll
            for (int i = 0; i < N_LD; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);             // global -> LDS load
                __builtin_amdgcn_sched_group_barrier(0x008, MFMA_PER_LD, 0);   // MFMA
            }
            __builtin_amdgcn_sched_group_barrier(0x008, N_MFMA, 0);         // remaining MFMAs
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int o = 1; o < NO - 1; ++o) {
                mfma_octet(o & 1);
                read_frags(stage, o + 1, (o + 1) & 1);
                __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, N_FRAG_RD, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, N_MFMA, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            const int next = stage + 1 == NS ? 0 : stage + 1;
            __builtin_amdgcn_s_waitcnt(kWaitTile);   // this wave's share of the next tile is in LDS, its own LDS reads are back
            __builtin_amdgcn_s_barrier();            // everyone's is; stage `stage` is free
            mfma_octet((NO - 1) & 1);
            read_frags(next, 0, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, N_FRAG_RD, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, N_MFMA, 0);
            __builtin_amdgcn_sched_barrier(0);
            fill = stage;
            stage = next;
        }
    }
    if constexpr (TWO_LEVEL) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) acc[rb][cb] += total[rb][cb];
    }

    // Sum over the K groups: groups 1.. park their accumulators in LDS (the stage area, once
    // every load still in flight has landed and every wave has left the K loop), group 0 adds
    // them in group order and stores.
    if constexpr (KG > 1) {
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __syncthreads();
        constexpr int PER_WAVE = RB * CB * NV * 64;
        if (kg > 0) {
            float *dst = smem + ((kg - 1) * TILE_WAVES + tw) * PER_WAVE + lane;
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int v = 0; v < NV; ++v) dst[((rb * CB + cb) * NV + v) * 64] = acc[rb][cb][v];
        }
        __syncthreads();
        if (kg > 0) return;
#pragma unroll
        for (int g = 1; g < KG; ++g) {
            const float *src = smem + ((g - 1) * TILE_WAVES + tw) * PER_WAVE + lane;
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int v = 0; v < NV; ++v) acc[rb][cb][v] += src[((rb * CB + cb) * NV + v) * 64];
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
    const int col = n0 + wn * WN + li * CB;
    const bool full_tile = m0 + BM <= p.m && n0 + BN <= p.n;      // workgroup-uniform
    const bool lane_vec = col + CB <= p.n;
    const bool nt = p.splits == 1 && rows_aligned<CB>(out, ldo);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            // (a transposed A: block rb holds the rows RB*i + rb of the wave tile, i the row inside the block)
            const int in_block = shape::row_of(v, h);
            const int row = m0 + wm * WM + (AM == 1 ? in_block * RB + rb : rb * MI + in_block);
            float *dst = out + (int64_t)row * ldo + col;
            bvec o;
            if constexpr (CB == 1) {
                o = acc[rb][0][v];
            } else {
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) o[cb] = acc[rb][cb][v];
            }
            if (full_tile || row < p.m) store_lane<CB>(dst, o, lane_vec, col, p.n, nt);
        }
    }
}

template <int BM, int BN, int BK, int WM, int WN, bool TWO_LEVEL, int NS, int KG, int AM, int BMD, int MI>
hipError_t launch_tile_direct(const GemmParams &p, hipStream_t s) {
    constexpr int threads = (BM / WM) * (BN / WN) * 64 * KG;
    constexpr int lds_used = direct_lds_bytes<BM, BN, BK, NS>();
    static_assert(lds_used <= kLdsPerCU, "stages exceed the LDS of a CU");
    auto kern = sgemm_tile_direct_kernel<BM, BN, BK, WM, WN, TWO_LEVEL, NS, KG, AM, BMD, MI>;
    int lds = lds_used;
    if (p.max_blocks_per_cu > 0) {
        const int share = (kLdsPerCU / p.max_blocks_per_cu) & ~1023;
        if (share > lds) lds = share;
    }
    static std::atomic<uint64_t> lds_limit_raised{0};   // one bit per device: the attribute is kept per device
    const hipError_t attr = allow_full_lds(reinterpret_cast<const void *>(kern), lds_limit_raised);
    if (attr != hipSuccess) return attr;
    const int64_t blocks = (int64_t)p.tiles_m * p.tiles_n * p.splits * p.batch;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(threads), lds, s, p);
    return hipGetLastError();
}

}  // namespace tg
