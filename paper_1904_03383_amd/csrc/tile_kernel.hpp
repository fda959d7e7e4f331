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
//
// Two builds of the same template.  EDGE = false ("exact-fit" in names and messages): aligned
// operands and 16-byte loads with no test in the K loop; m and n need not be multiples of
// the tile (a last tile row / column re-reads the operand's last row / last vector and masks
// its stores) and k need not be a multiple of BK (the remainder goes first, as a zero-padded
// K tile).  EDGE = true: every access predicated, any size, alignment and element stride.
#pragma once

#include "tg_internal.h"

#include <type_traits>

namespace tg {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
// Four consecutive floats at any 4-byte aligned address: still one global_load_dwordx4 (global memory accesses
// need dword alignment only), so rows that are off the 16-byte grid cost no extra instructions.
typedef f32x4 f32x4_a4 __attribute__((aligned(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int N> struct vec_of;
template <> struct vec_of<1> { typedef float type; };
template <> struct vec_of<2> { typedef f32x2 type; };
template <> struct vec_of<4> { typedef f32x4 type; };

// Store of a result vector.  C itself is written once and never read back by the product, so it goes out
// with the non-temporal hint and does not displace operand panels from L2 (measured: 4096x4096x128
// 41.7 -> 40.0 us, 1024^3 23.1 -> 22.9 us, no change at 4096^3); split-K partials, which the reduction
// reads next, are stored normally.
// The destination needs 4-byte alignment only (one global_store_dwordx2/x4 either way), so rows of C that are
// off the 16-byte grid are stored the same way as aligned ones.
// (The hint is only kept by the compiler on naturally aligned vector stores: `nt` must imply that.)
template <typename V>
__device__ __forceinline__ void store_result(float *dst, V v, bool nt) {
    typedef V VA __attribute__((aligned(4)));
    if (nt) __builtin_nontemporal_store(v, reinterpret_cast<V *>(dst));
    else *reinterpret_cast<VA *>(dst) = v;
}

// Whether every lane's CB-float groups are naturally aligned in every row of the destination that starts at
// `first` (a lane's column is a multiple of CB, so this is the same for all lanes: a scalar condition).
template <int CB>
__device__ __forceinline__ bool rows_aligned(const float *first, int64_t ld) {
    return (reinterpret_cast<uintptr_t>(first) & (4 * CB - 1)) == 0 && ld % CB == 0;
}

__device__ __forceinline__ float vec_get(float v, int) { return v; }
__device__ __forceinline__ float vec_get(f32x2 v, int i) { return v[i]; }
__device__ __forceinline__ float vec_get(f32x4 v, int i) { return v[i]; }

// The CB results of one lane, columns col .. col+CB-1 of one row: one vector store where all of them exist
// (lane_vec = col + CB <= n, the same for every row of the lane), element by element in the last, partial
// group of an n that is not a multiple of CB.
template <int CB, typename V>
__device__ __forceinline__ void store_lane(float *dst, V o, bool lane_vec, int col, int n, bool nt) {
    if (lane_vec) {
        store_result(dst, o, nt);
    } else {
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
            if (col + cb < n) dst[cb] = vec_get(o, cb);
    }
}

// Address of a 16-byte vector at a 32-bit byte offset from a wave-uniform origin.  The exact-fit variants keep their
// lane offsets that way (the host checks that a tile's footprint stays below 2^30 elements): a load is then the tile
// origin in scalar registers plus a 32-bit vector offset, with no 64-bit address arithmetic and no second register
// per offset.  (The empty asm passes the offset through unchanged, in place: it keeps the widening of the offset
// next to the load; hoisted out of the K loop as a 64-bit value it would hide from instruction selection that the
// offset is a 32-bit one.)
__device__ __forceinline__ const f32x4 *at_bytes(const float *base, unsigned &bytes) {
    asm volatile("" : "+v"(bytes));
    return reinterpret_cast<const f32x4 *>(reinterpret_cast<const char *>(base) + bytes);
}

// Row of the A tile that load slot f (one 16-byte vector; BK/4 consecutive slots make a row) fetches and
// writes to LDS.  With BK = 32 eight consecutive lanes fill one padded LDS row, 32 consecutive banks.  With
// BK = 16 they fill two rows, and at a row pitch of 20 floats the rows r and r+1 overlap in four banks (a
// 2-way conflict on every ds_write_b128 of A: 16.9 % of the LDS cycles in the hardware counters); rows r
// and r+4 do not (20*4 = 80 = 16 mod 32).  So within each group of eight rows the slots take the rows in
// the order 0, 4, 1, 5, 2, 6, 3, 7.  No padding alone can do this: the second row would have to start 16
// banks after the first, i.e. at a pitch of 16 mod 32, where the fragment reads of 8 rows collide.
template <int BK>
__device__ __forceinline__ int a_slot_row(int f) {
    const int r = f / (BK / 4);
    if constexpr (BK == 16) return (r & ~7) | ((r & 1) << 2) | ((r & 7) >> 1);
    else return r;
}

// Workgroup id -> (slice, tile row, tile column);  slice = problem * splits + split.
// Hardware hands consecutive workgroup ids to the 8 XCDs in turn, and each XCD has its own
// 4 MB L2.  So that the workgroups resident on one XCD share operand panels:
//  * 2-D mode (xcd_m * xcd_n == 8, both dividing the tile grid): XCD x owns the
//    rectangular region (x / xcd_n, x % xcd_n) of every slice's tile grid, which minimises
//    the A rows plus B columns an XCD ever touches;
//  * otherwise XCD x takes one contiguous range of the linear order (slice-major).
// Inside a region (or a problem) tiles are walked in groups of `group` tile rows, column by
// column, which keeps the set of panels in flight small.
__device__ __forceinline__ void grouped_order(unsigned t, unsigned rows, unsigned cols, unsigned group,
                                              unsigned &r, unsigned &c) {
    const unsigned gw = group * cols;
    const unsigned g = t / gw;
    const unsigned first = g * group;
    const unsigned rest = rows - first;
    const unsigned gsz = rest < group ? rest : group;
    const unsigned in = t - g * gw;
    r = first + in % gsz;
    c = in / gsz;
}

// W = number of work items (tiles x slices) of the launch, w = this work item.
__device__ __forceinline__ void map_workgroup(const GemmParams &p, unsigned W, unsigned w, int &slice, int &tm,
                                              int &tn) {
    const unsigned x = w & 7u, s = w >> 3;
    const unsigned T = (unsigned)p.tiles_m * (unsigned)p.tiles_n;
    unsigned r, c;
    if (p.xcd_m != 0) {
        const unsigned per = T >> 3;                 // tiles of one slice owned by one XCD
        const unsigned sl = s / per, t = s - sl * per;
        const unsigned rm = (unsigned)p.tiles_m / (unsigned)p.xcd_m, rn = (unsigned)p.tiles_n / (unsigned)p.xcd_n;
        grouped_order(t, rm, rn, (unsigned)p.group < rm ? (unsigned)p.group : rm, r, c);
        slice = (int)sl;
        tm = (int)((x / (unsigned)p.xcd_n) * rm + r);
        tn = (int)((x % (unsigned)p.xcd_n) * rn + c);
        return;
    }
    const unsigned q = W >> 3, rem = W & 7u;
    const unsigned logical = x * q + (x < rem ? x : rem) + s;
    const unsigned sl = logical / T;
    grouped_order(logical - sl * T, (unsigned)p.tiles_m, (unsigned)p.tiles_n, (unsigned)p.group, r, c);
    slice = (int)sl;
    tm = (int)r;
    tn = (int)c;
}

// Registers: a wave tile keeps WM*WN/64 accumulator registers per lane (twice that with the
// second accumulation level), plus the staging registers of one K tile and two fragment
// sets.  When that budget fits, the kernel is compiled for two waves per SIMD (256
// registers per lane): two waves from different workgroups cover each other's barrier and
// memory waits.
template <int BM, int BN, int BK, int WM, int WN, bool TWO_LEVEL>
constexpr int min_waves_per_simd() {
    constexpr int nt = (BM / WM) * (BN / WN) * 64;
    constexpr int acc = (WM * WN / 64) * (TWO_LEVEL ? 2 : 1);
    constexpr int staging = (BM * BK + BK * BN) / nt;
    constexpr int frags = 2 * (4 * (WM / 32) + 4 * (WN / 32));
    return acc + staging + frags + 64 <= 256 ? 2 : 1;
}

template <int BM, int BN, int BK, int WM, int WN, bool TWO_LEVEL, bool EDGE>
__global__ void __launch_bounds__((BM / WM) * (BN / WN) * 64, (min_waves_per_simd<BM, BN, BK, WM, WN, TWO_LEVEL>()))
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

    // LDS: stage 0 at float 0, stage 1 at float PITCH; inside a stage A, then B.  Every LDS address a thread uses
    // is kept as a 32-bit LDS address into the stage it currently refers to and moves to the other stage with one
    // addition per K tile (of +-PITCH, a scalar that changes sign per tile): no stage index, no multiplication, no
    // address rebuilt per access.
    constexpr unsigned PITCH_BYTES = 4u * tile_stage_pitch<BM, BN, BK>();
    extern __shared__ __attribute__((aligned(16))) float smem[];
    typedef __attribute__((address_space(3))) float lds_space_float;
    const unsigned lds_base = (unsigned)(uintptr_t)(lds_space_float *)smem;
    auto lds = [](unsigned addr) { return (float *)(lds_space_float *)(uintptr_t)addr; };

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // in a scalar register: what depends only on the wave stays scalar
    const int li = lane & 31, h = lane >> 5;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    // One workgroup per work item (tile x slice).
    const unsigned total_work = (unsigned)p.tiles_m * (unsigned)p.tiles_n * (unsigned)p.splits * (unsigned)p.batch;
    const unsigned work = blockIdx.x;
    {
        int slice, tm, tn;
        map_workgroup(p, total_work, work, slice, tm, tn);
        const int prob = slice / p.splits, split = slice - prob * p.splits;
        const int m0 = tm * BM, n0 = tn * BN;

        const int kt_total = (p.k + BK - 1) / BK;
        const int kt_begin = split * p.ktiles_per_split;
        const int kt_stop = kt_begin + p.ktiles_per_split;
        const int kt_end = kt_stop < kt_total ? kt_stop : kt_total;

        // Tile origins are wave-uniform (kept in scalar registers and advanced per K tile); each
        // thread adds fixed offsets for its slots.  Fast variants use 32-bit offsets (the host
        // checks that a tile spans fewer than 2^30 elements), predicated ones 64-bit.
        // (csa, csb: element strides along k of A / along n of B, honoured by the predicated variants)
        const int64_t csa = EDGE ? p.csa : 1, csb = EDGE ? p.csb : 1;
        // Exact-fit variants with k not a multiple of BK: the k % BK leftover elements form K tile 0,
        // zero-padded on its way through the staging registers in the prologue; every later tile is
        // a full one that starts `tail` elements further on, so the K loop itself never tests k.
        // (k % 4 == 0 keeps the 16-byte alignment of the rows of A.)
        const int tail = EDGE ? 0 : p.k % BK;
        const int64_t k_begin = EDGE || tail == 0 || kt_begin == 0 ? (int64_t)kt_begin * BK : (int64_t)(kt_begin - 1) * BK + tail;
        const float *Ag = p.A + (int64_t)prob * p.strideA + (int64_t)m0 * p.lda + k_begin * csa;
        const float *Bg = p.B + (int64_t)prob * p.strideB + k_begin * p.ldb + (int64_t)n0 * csb;
        typedef typename std::conditional<EDGE, int64_t, unsigned>::type off_t;

        // Per-thread slots of the tile loads: slot f = tid + i*NT is one 16-byte vector.
        int a_row[A_LD], a_k[A_LD], b_row[B_LD], b_col[B_LD];
        off_t a_off[A_LD], b_off[B_LD];
    #pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            const int f = tid + i * NT;
            a_row[i] = a_slot_row<BK>(f);
            a_k[i] = (f % (BK / 4)) * 4;
            // exact-fit variants on a ragged last tile row: rows past the end re-read the last row
            // (in bounds; what they produce is never stored)
            const int r = EDGE ? a_row[i] : (a_row[i] < p.m - 1 - m0 ? a_row[i] : p.m - 1 - m0);
            a_off[i] = (off_t)r * (off_t)p.lda + (off_t)a_k[i] * (off_t)csa;
            if constexpr (!EDGE) a_off[i] *= 4;      // exact-fit variants: in bytes (see at_bytes)
        }
    #pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            const int f = tid + i * NT;
            b_row[i] = f / (BN / 4);
            b_col[i] = (f % (BN / 4)) * 4;
            // ... and on a ragged last tile column, vectors past the end re-read the last one (n % 4 == 0)
            const int c = EDGE ? b_col[i] : (b_col[i] < p.nb - 4 - n0 ? b_col[i] : p.nb - 4 - n0);
            b_off[i] = (off_t)b_row[i] * (off_t)p.ldb + (off_t)c * (off_t)csb;
            if constexpr (!EDGE) b_off[i] *= 4;
        }

        f32x4 a_reg[A_LD], b_reg[B_LD];
        // Fetch K tile `kt` (absolute index) into the staging registers.  The pointers then move
        // on to the next tile only if `advance` is set, so that asking again for the last tile of
        // the range (when nothing is left to prefetch) stays inside the matrices.
        // Predicated variants: a tile that lies wholly inside the matrices (the common case even
        // for ragged sizes) is fetched without per-element tests, with 16-byte loads when the
        // operand has unit element stride (host flags; the rows need not be 16-byte aligned), else
        // with four plain loads per slot; only tiles that cross an edge take the tested path.
        const bool full_m = m0 + BM <= p.m, full_n = n0 + BN <= p.n;      // workgroup-uniform
        const bool vec_a = (p.flags & kFlagVecA) != 0, vec_b = (p.flags & kFlagVecB) != 0;
        auto load_global = [&](int kt, bool advance) {
            const bool full_k = EDGE && (kt + 1) * BK <= p.k;
    #pragma unroll
            for (int i = 0; i < A_LD; ++i) {
                const float *src = EDGE ? Ag + a_off[i] : nullptr;
                if constexpr (!EDGE) {
                    a_reg[i] = *at_bytes(Ag, a_off[i]);
                } else if (full_m && full_k) {
                    if (vec_a) {
                        a_reg[i] = *reinterpret_cast<const f32x4_a4 *>(src);
                    } else {
                        f32x4 v;
    #pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = src[e * csa];
                        a_reg[i] = v;
                    }
                } else {
                    const bool row_ok = m0 + a_row[i] < p.m;
                    const int kk = kt * BK + a_k[i];
                    f32x4 v;
    #pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (row_ok && kk + e < p.k) ? src[e * csa] : 0.0f;
                    a_reg[i] = v;
                }
            }
    #pragma unroll
            for (int i = 0; i < B_LD; ++i) {
                const float *src = EDGE ? Bg + b_off[i] : nullptr;
                if constexpr (!EDGE) {
                    b_reg[i] = *at_bytes(Bg, b_off[i]);
                } else if (full_n && full_k) {
                    if (vec_b) {
                        b_reg[i] = *reinterpret_cast<const f32x4_a4 *>(src);
                    } else {
                        f32x4 v;
    #pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = src[e * csb];
                        b_reg[i] = v;
                    }
                } else {
                    const bool row_ok = kt * BK + b_row[i] < p.k;
                    const int cc = n0 + b_col[i];
                    f32x4 v;
    #pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (row_ok && cc + e < p.n) ? src[e * csb] : 0.0f;
                    b_reg[i] = v;
                }
            }
            if (advance) {
                Ag += BK * csa;
                Bg += (int64_t)BK * p.ldb;
            }
        };

        // K tile 0 of a k that leaves a remainder: only its first `tail` columns of A / rows of B exist.
        auto load_global_tail = [&](bool advance) {
            if constexpr (!EDGE) {
    #pragma unroll
                for (int i = 0; i < A_LD; ++i)
                    a_reg[i] = a_k[i] < tail ? *at_bytes(Ag, a_off[i]) : (f32x4)(0.0f);
    #pragma unroll
                for (int i = 0; i < B_LD; ++i)
                    b_reg[i] = b_row[i] < tail ? *at_bytes(Bg, b_off[i]) : (f32x4)(0.0f);
            }
            if (advance) {
                Ag += tail;
                Bg += (int64_t)tail * p.ldb;
            }
        };

        // (slot i of a thread lies a fixed number of rows below its slot 0: one address register per operand and
        // immediates, instead of an address computed per slot and tile)
        constexpr int A_SLOT_ROWS = NT / (BK / 4), B_SLOT_ROWS = NT / (BN / 4);
        static_assert(NT % (BK / 4) == 0 && A_SLOT_ROWS % 8 == 0 && NT % (BN / 4) == 0, "slots of a thread are whole rows apart");
        unsigned wr_a = lds_base + 4u * (a_row[0] * LDA_S + a_k[0]);      // this thread's slot 0 in the stage being filled
        unsigned wr_b = lds_base + 4u * (A_STAGE + b_row[0] * LDB_S + b_col[0]);
        auto store_lds = [&]() {
            float *as = lds(wr_a);
            float *bs = lds(wr_b);
#pragma unroll
            for (int i = 0; i < A_LD; ++i)
                *reinterpret_cast<f32x4 *>(as + i * A_SLOT_ROWS * LDA_S) = a_reg[i];
#pragma unroll
            for (int i = 0; i < B_LD; ++i)
                *reinterpret_cast<f32x4 *>(bs + i * B_SLOT_ROWS * LDB_S) = b_reg[i];
        };
        // Debug flavour of the library (compiled with TG_POISON_LDS): once a stage has been given up (the barrier after
        // which nobody reads it), every lane overwrites the slots it will fill next with NaN.  A kernel that read a stage
        // after giving it up, or before it was complete, then returns NaN instead of stale but plausible numbers.
        auto poison_lds = [&]() {
#ifdef TG_POISON_LDS
            float *as = lds(wr_a);
            float *bs = lds(wr_b);
#pragma unroll
            for (int i = 0; i < A_LD; ++i)
                *reinterpret_cast<f32x4 *>(as + i * A_SLOT_ROWS * LDA_S) = (f32x4)(__builtin_nanf(""));
#pragma unroll
            for (int i = 0; i < B_LD; ++i)
                *reinterpret_cast<f32x4 *>(bs + i * B_SLOT_ROWS * LDB_S) = (f32x4)(__builtin_nanf(""));
#endif
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

        unsigned rd_a = lds_base + 4u * ((wm * WM + li) * LDA_S + h * 4); // this lane's fragments in the stage being multiplied
        unsigned rd_b = lds_base + 4u * (A_STAGE + (h * 4) * LDB_S + wn * WN + li * CB);
        unsigned to_other = PITCH_BYTES;            // what takes the read addresses to the other stage (and the write addresses back)
        auto other_stage = [&]() {
            rd_a += to_other;
            rd_b += to_other;
            to_other = 0u - to_other;
            wr_a += to_other;
            wr_b += to_other;
        };

        // Operand fragments of two consecutive k-octets: while the MFMAs of octet o run from
        // one set, the LDS reads of octet o+1 fill the other.
        constexpr int NO = BK / 8;
        static_assert(NO % 2 == 0, "BK must be a multiple of 16 (fragment sets alternate per octet)");
        f32x4 a_frag[2][RB];
        bvec b_frag[2][4];

        auto read_frags = [&](int o, int set) {
            const float *as = lds(rd_a) + o * 8;
            const float *bs = lds(rd_b) + o * 8 * LDB_S;
    #pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                a_frag[set][rb] = *reinterpret_cast<const f32x4 *>(as + rb * 32 * LDA_S);
    #pragma unroll
            for (int t = 0; t < 4; ++t)
                b_frag[set][t] = *reinterpret_cast<const bvec *>(bs + t * LDB_S);
        };

        auto mfma_octet = [&](int set) {
    #pragma unroll
            for (int t = 0; t < 4; ++t)
    #pragma unroll
                for (int rb = 0; rb < RB; ++rb)
    #pragma unroll
                    for (int cb = 0; cb < CB; ++cb)
                        acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                            a_frag[set][rb][t], vec_get(b_frag[set][t], cb), acc[rb][cb], 0, 0, 0);
        };

        // Second accumulation level: after every flush_tiles K tiles the MFMA accumulators are
        // added into `total` and cleared, which bounds the length of any single fp32 running sum.
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
                            acc[rb][cb] = (f32x16)(0.0f);
                            // one block at a time keeps the temporaries of this rare path small
                            __builtin_amdgcn_sched_barrier(0);
                        }
                }
                ++since_flush;
            }
        };

        // K loop.  LDS holds two stages; the staging registers hold the tile after the one in LDS.
        // Per K tile kt (multiplied out of stage s):
        //   octets 0 .. NO-3 : fetch the fragments of the next octet, multiply the current one;
        //   octet NO-2       : the same, with the LDS writes of tile kt+1 (stage s^1) spread between
        //                      its MFMAs, so the matrix pipe keeps running while they issue;
        //   one barrier      : stage s^1 is complete, nobody reads stage s any more;
        //   octet NO-1       : fetch the first fragments of tile kt+1, start the global loads of
        //                      tile kt+2 into the (now free) staging registers, multiply.
        // A wave can have only one MFMA in flight, so every instruction that is not an MFMA is
        // placed in the shadow of one; the fences and group hints below pin that order, which the
        // scheduler would otherwise undo to save registers.
        // One barrier per K tile is enough: stage s^1 was last read before the previous barrier,
        // and stage s is not overwritten before the next one.
        // s_waitcnt encodings (gfx9: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8; all ones = not waited for)
        constexpr int kWaitLoads = 0x0F70;           // vmcnt(0)
        constexpr int kWaitOlderReads = 0xC07F | ((RB + 4) << 8);   // lgkmcnt(the reads of one octet): everything older has returned
        constexpr int N_MFMA = 4 * RB * CB;          // MFMAs of one octet
        constexpr int N_ST = A_LD + B_LD;            // LDS writes / global loads of one tile
        constexpr int MFMA_PER_ST = N_MFMA / N_ST > 0 ? N_MFMA / N_ST : 1;
        if (kt_begin < kt_end) {
            const int last = kt_end - 1;
            if (!EDGE && tail != 0 && kt_begin == 0) load_global_tail(kt_begin < last);
            else load_global(kt_begin, kt_begin < last);
            store_lds();                  // stage 0
            __syncthreads();
            read_frags(0, 0);
            wr_a += PITCH_BYTES;          // the next tile is staged in stage 1
            wr_b += PITCH_BYTES;
            {
                const int nl = kt_begin + 1 < last ? kt_begin + 1 : last;
                load_global(nl, nl < last);
            }
            for (int kt = kt_begin; kt < last; ++kt) {
                maybe_flush();                // (at the top, so the loop body below stays one block)
                __builtin_amdgcn_sched_barrier(0);
    #pragma unroll
                for (int o = 0; o < NO - 2; ++o) {
                    read_frags(o + 1, (o + 1) & 1);
                    __builtin_amdgcn_sched_barrier(0);
                    __builtin_amdgcn_s_waitcnt(kWaitOlderReads);   // one wait per octet instead of one per fragment
                    mfma_octet(o & 1);
                    __builtin_amdgcn_sched_barrier(0);
                }
                read_frags(NO - 1, (NO - 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_s_waitcnt(kWaitLoads & kWaitOlderReads);   // one wait for the staged tile instead of one per LDS write
                mfma_octet((NO - 2) & 1);
                store_lds();
    #pragma unroll
                for (int i = 0; i < N_ST; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, MFMA_PER_ST, 0);   // MFMA
                    __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);             // LDS write
                }
                __builtin_amdgcn_sched_barrier(0);
                __syncthreads();
                other_stage();                // the stage just completed is multiplied next, the one just left is filled next
                poison_lds();                 // (debug flavour only: nothing reads that stage any more)
                read_frags(0, 0);
                __builtin_amdgcn_sched_barrier(0);
                {
                    const int nl = kt + 2 < last ? kt + 2 : last;
                    load_global(nl, nl < last);
                }
                mfma_octet((NO - 1) & 1);
    #pragma unroll
                for (int i = 0; i < N_ST; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);             // global load
                    __builtin_amdgcn_sched_group_barrier(0x008, MFMA_PER_ST, 0);   // MFMA
                }
                __builtin_amdgcn_sched_barrier(0);
            }
    #pragma unroll
            for (int o = 0; o < NO - 1; ++o) {
                read_frags(o + 1, (o + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
                mfma_octet(o & 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            mfma_octet((NO - 1) & 1);
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
        const bool final_c = p.splits == 1;
        const bool lane_vec = col + CB <= p.n;
        const bool nt = final_c && rows_aligned<CB>(out, ldo);
        float *wave_tile = out + (int64_t)(m0 + wm * WM) * ldo + n0 + wn * WN;
        unsigned lane_bytes = 4u * ((unsigned)(4 * h) * (unsigned)ldo + (unsigned)(li * CB));
    #pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
    #pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = rb * 32 + 8 * (v / 4) + (v % 4);
                const int row = m0 + wm * WM + r + 4 * h;
                float *dst;
                if constexpr (EDGE) {
                    dst = out + (int64_t)row * ldo + col;
                } else {
                    // (the origin of row r of the wave tile is wave-uniform, the lane's part one 32-bit byte offset for
                    // all its stores: the host checks ldc < 2^27 for the exact-fit variants; see at_bytes for the asm)
                    asm volatile("" : "+v"(lane_bytes));
                    dst = reinterpret_cast<float *>(reinterpret_cast<char *>(wave_tile + (int64_t)r * ldo) + lane_bytes);
                }
                bvec o;
                if constexpr (CB == 1) {
                    o = acc[rb][0][v];
                } else {
    #pragma unroll
                    for (int cb = 0; cb < CB; ++cb) o[cb] = acc[rb][cb][v];
                }
                if ((full_m && full_n) || row < p.m) store_lane<CB>(dst, o, lane_vec, col, p.n, nt);
            }
        }
    }
}

template <int BM, int BN, int BK, int WM, int WN, bool TWO_LEVEL, bool EDGE>
hipError_t launch_tile(const GemmParams &p, hipStream_t s) {
    constexpr int threads = (BM / WM) * (BN / WN) * 64;
    constexpr int lds_used = tile_lds_bytes<BM, BN, BK, WM, WN>();
    auto kern = sgemm_tile_kernel<BM, BN, BK, WM, WN, TWO_LEVEL, EDGE>;
    // Occupancy cap: asking for a larger LDS allocation than the tile uses limits how many
    // workgroups share a CU (max_blocks_per_cu == 0: no cap).
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
