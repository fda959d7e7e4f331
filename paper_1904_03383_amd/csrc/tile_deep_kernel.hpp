// Direct-to-LDS SGEMM kernel for small wave tiles (32x32 per wave), gfx950: the operand fragments of a
// whole K tile are fetched one K tile ahead of the MFMAs that use them.
//
// Same product, decomposition and LDS stage layout as tile_direct_kernel.hpp (matmul of Sec. 5.2 of the
// paper; A rows chunk-permuted, B k-major, global_load_lds_dwordx4 into a ring of NS stages).  What
// differs is the register pipeline.  A 32x32 wave tile has only four MFMAs (256 cycles) per k-octet, and
// a kernel that fetches the fragments of octet o+1 while it multiplies octet o leaves an LDS read at most
// two MFMAs to come back: with four waves and the LDS-DMA writes sharing the LDS that is not enough, and
// every octet ends in a stall (1024^3 on 64x64 tiles ran at 70 % of the MFMA rate inside the loop
// whatever the wave layout, ring depth or matrix instruction; without the fragment reads it ran 2.3 us
// faster).  Here a wave keeps two register sets of all the fragments of a K tile (BK registers each):
// right after the barrier that publishes tile t+1 it issues the LDS reads of tile t+1 into one set (20 for
// BK = 32) while it multiplies tile t out of the other, BK/2 MFMAs that depend on none of those reads.
// BK = 64 halves the number of barriers per product at twice the registers and LDS (measured no gain at
// 1024^3: 21.0 us against 20.0 us; kept for the tuner).  A deeper ring (NS = 3) measured 20.4 us, and two waves per
// wave tile, each with half of every K tile and the sums joined through LDS at the end, 20.5 us (the two waves of a
// SIMD then meet the same barrier together, so neither covers the other's wait).
//
// Order of one K tile t (stage t % NS holds it; its fragments are already in registers):
//   wait: this wave's share of tile t+1 has landed, and its fragment reads of tile t have come back;
//   barrier: everyone's share of tile t+1 is in LDS, and nobody reads stage t % NS any more;
//   issue the loads of tile t+NS into stage t % NS, and the fragment reads of tile t+1;
//   16 MFMAs of tile t, interleaved with the above.
// So the global loads run NS tiles ahead of the MFMAs with NS stages.  Once the last tile of the K range
// has been requested nothing more is fetched and the waits become full ones (the tiles still in flight
// then were requested at least one tile earlier), so no load is outstanding when the wave ends.
//
// Operand modes AM / BMD as in tile_direct_kernel.hpp (0 plain, 1 transposed on the 16-byte grid, 2 any
// element strides, gathered with 4-byte loads); with one 32x32 block per wave a lane's row and column are
// simply its lane index in every mode.
//
// The barriers are the bare instruction with explicit wait counts in front, not __syncthreads(): the fence
// that comes with the latter makes the compiler wait for every load in flight (vmcnt(0)) before each barrier,
// which would empty the ring at every K tile.  What the barrier has to order is covered by the waits: a
// direct load counts as done (vmcnt) when its data is in LDS, and a wave's own LDS reads have returned
// (lgkmcnt(0)) before it lets the others overwrite the stage.
#pragma once

#include "tile_direct_kernel.hpp"

namespace tg {

template <int BM, int BN, int BK, int NS, bool TWO_LEVEL, int AM, int BMD>
__global__ void __launch_bounds__((BM / 32) * (BN / 32) * 64, (BK > 32 ? 1 : 2))
sgemm_tile_deep_kernel(const GemmParams p) {
    constexpr int WAVES_N = BN / 32;
    constexpr int NWAVES = (BM / 32) * (BN / 32);
    constexpr int NT = NWAVES * 64;
    constexpr int A_STAGE = BM * BK, B_STAGE = BK * BN;      // floats, unpadded
    constexpr int A_EL = AM == 2 ? 1 : 4, B_EL = BMD == 2 ? 1 : 4;   // floats per lane of one load instruction
    constexpr int A_LD = BM * BK / A_EL / NT, B_LD = BK * BN / B_EL / NT;
    constexpr int N_LD = A_LD + B_LD;
    constexpr int NO = BK / 8;
    static_assert(AM >= 0 && AM <= 2 && BMD >= 0 && BMD <= 2, "operand modes");
    static_assert(BK == 32 || BK == 64, "K tile of 32 or 64");
    static_assert(BM % 32 == 0 && BN % 32 == 0, "tile shape");
    static_assert((BM * BK / A_EL) % NT == 0 && (BK * BN / B_EL) % NT == 0 && A_LD >= 1 && B_LD >= 1,
                  "tile loads must divide evenly over the workgroup");
    static_assert(NS >= 2 && NS <= 4, "two to four LDS stages");
    static_assert((NS - 1) * N_LD <= 63, "outstanding loads must fit the vmcnt field");

    extern __shared__ __attribute__((aligned(16))) float smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // in a scalar register: the LDS targets of the direct loads are
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

    // (lda, ldb: row strides of A and B; csa, csb: their element strides along k and along n)
    const int64_t a_step = AM == 0 ? (int64_t)BK : (int64_t)BK * p.csa;
    const int64_t b_step = BMD == 1 ? (int64_t)BK : (int64_t)BK * p.ldb;
    const float *Ag = p.A + (int64_t)prob * p.strideA + (int64_t)m0 * p.lda + (int64_t)kt_begin * a_step;
    const float *Bg = p.B + (int64_t)prob * p.strideB + (int64_t)kt_begin * b_step + (int64_t)n0 * (BMD == 0 ? 1 : p.csb);

    // Load slots as in the direct kernel: instruction i of a wave fills LDS floats [slot*256, slot*256+256)
    // of a stage (64 floats for a gathered operand), slot = i * NWAVES + wave; rows, columns and vectors past a
    // ragged edge re-read the last valid one.  The per-lane offsets are kept in bytes, 32 bits wide (the host
    // checks that a tile's footprint stays below 4 GiB), so that a load is the wave-uniform tile origin plus a
    // 32-bit lane offset and needs no address arithmetic in the loop.
    unsigned a_off[A_LD], b_off[B_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        const int pos = ((i * NWAVES + wave) * 64 + lane) * A_EL;
        if constexpr (AM == 1) {                      // k-major stage: row pos / BM is one k, BM consecutive m
            const int c = pos % BM < p.m - 4 - m0 ? pos % BM : p.m - 4 - m0;
            a_off[i] = 4u * ((unsigned)(pos / BM) * (unsigned)p.csa + (unsigned)c);
        } else {
            const int row = pos / BK;
            const int q = (pos % BK) / 4;
            const int src_row = row < p.m - 1 - m0 ? row : p.m - 1 - m0;
            const int src_k = (q ^ a_swizzle<BK>(row)) * 4 + (AM == 2 ? pos % 4 : 0);
            a_off[i] = 4u * ((unsigned)src_row * (unsigned)p.lda + (unsigned)src_k * (AM == 2 ? (unsigned)p.csa : 1u));
        }
    }
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        const int pos = ((i * NWAVES + wave) * 64 + lane) * B_EL;
        if constexpr (BMD == 1) {                     // one LDS row of BK floats per column, chunks permuted as in A's stage
            const int row = pos / BK;
            const int q = (pos % BK) / 4;
            const int src_col = row < p.n - 1 - n0 ? row : p.n - 1 - n0;
            b_off[i] = 4u * ((unsigned)src_col * (unsigned)p.csb + (unsigned)((q ^ a_swizzle<BK>(row)) * 4));
        } else if constexpr (BMD == 2) {
            const int c = pos % BN < p.n - 1 - n0 ? pos % BN : p.n - 1 - n0;
            b_off[i] = 4u * ((unsigned)(pos / BN) * (unsigned)p.ldb + (unsigned)c * (unsigned)p.csb);
        } else {
            const int c = pos % BN < p.nb - 4 - n0 ? pos % BN : p.nb - 4 - n0;
            b_off[i] = 4u * ((unsigned)(pos / BN) * (unsigned)p.ldb + (unsigned)c);
        }
    }

    f32x16 acc = (f32x16)(0.0f);
    f32x16 total = (f32x16)(0.0f);

    const int a_row = wm * 32 + li;
    const int a_swz = a_swizzle<BK>(a_row);                  // == a_swizzle(li): also B's rows in mode 1
    const float *a_frag_base = smem + (AM == 1 ? (h * 4) * BM + a_row : a_row * BK);
    const float *b_frag_base = smem + NS * A_STAGE + (BMD == 1 ? (wn * 32 + li) * BK : (h * 4) * BN + wn * 32 + li);

    // the fragments of one K tile, element t of octet o for MFMA t of that octet: an operand whose stage keeps k
    // contiguous (A in modes 0 and 2, B in mode 1) comes as one 16-byte read per octet, the other as four 4-byte reads
    f32x4 a_frag[2][NO], b_frag[2][NO];
    constexpr int N_RD = NO * ((AM == 1 ? 4 : 1) + (BMD == 1 ? 1 : 4));   // LDS reads of one tile

    auto read_tile = [&](int stage, int set) {
        const float *as = a_frag_base + stage * A_STAGE;
        const float *bs = b_frag_base + stage * B_STAGE;
#pragma unroll
        for (int o = 0; o < NO; ++o) {
            const int chunk = ((2 * o + h) ^ a_swz) * 4;
            if constexpr (AM == 1) {
#pragma unroll
                for (int t = 0; t < 4; ++t) a_frag[set][o][t] = as[(8 * o + t) * BM];
            } else {
                a_frag[set][o] = *reinterpret_cast<const f32x4 *>(as + chunk);
            }
            if constexpr (BMD == 1) {
                b_frag[set][o] = *reinterpret_cast<const f32x4 *>(bs + chunk);
            } else {
#pragma unroll
                for (int t = 0; t < 4; ++t) b_frag[set][o][t] = bs[(8 * o + t) * BN];
            }
        }
    };

    // MFMAs first .. last-1 of a tile (in the order octet-major, t-minor)
    auto mfma_range = [&](int set, int first, int last) {
#pragma unroll
        for (int i = 0; i < 4 * NO; ++i)
            if (i >= first && i < last)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a_frag[set][i / 4][i % 4], b_frag[set][i / 4][i % 4], acc, 0, 0, 0);
    };

    // s_waitcnt encodings (gfx9: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
    constexpr int kFirst = (NS - 1) * N_LD;                 // prologue: all but the first tile may be in flight
    constexpr int kSteady = (NS - 2) * N_LD;                // loop: tile t+1 has landed, the younger ones may be in flight
    constexpr int kWaitFirst = 0x0F70 | (kFirst & 15) | ((kFirst >> 4) << 14);
    constexpr int kWaitSteady = 0x0070 | (kSteady & 15) | ((kSteady >> 4) << 14);   // and lgkmcnt(0)
    constexpr int kWaitAll = 0x0070;                        // vmcnt(0) and lgkmcnt(0)

    if (kt_begin < kt_end) {
        int to_issue = kt_end - kt_begin;           // tiles not requested yet
        auto issue = [&](int stage) {
            TG_POISON_DIRECT(stage * A_STAGE, NS * A_STAGE + stage * B_STAGE);   // (debug flavour only)
#pragma unroll
            for (int i = 0; i < A_LD; ++i)
                direct_load<A_EL>(byte_offset(Ag, a_off[i]), smem + stage * A_STAGE + (i * NWAVES + wave) * (64 * A_EL));
#pragma unroll
            for (int i = 0; i < B_LD; ++i)
                direct_load<B_EL>(byte_offset(Bg, b_off[i]), smem + NS * A_STAGE + stage * B_STAGE + (i * NWAVES + wave) * (64 * B_EL));
            --to_issue;
            Ag += a_step;
            Bg += b_step;
        };
        auto issue_a = [&](int stage) {
            TG_POISON_DIRECT(stage * A_STAGE, NS * A_STAGE + stage * B_STAGE);   // (debug flavour only)
#pragma unroll
            for (int i = 0; i < A_LD; ++i)
                direct_load<A_EL>(byte_offset(Ag, a_off[i]), smem + stage * A_STAGE + (i * NWAVES + wave) * (64 * A_EL));
            Ag += a_step;
        };
        auto issue_b = [&](int stage) {
#pragma unroll
            for (int i = 0; i < B_LD; ++i)
                direct_load<B_EL>(byte_offset(Bg, b_off[i]), smem + NS * A_STAGE + stage * B_STAGE + (i * NWAVES + wave) * (64 * B_EL));
            --to_issue;
            Bg += b_step;
        };
        auto issue_one = [&](int stage, int j) {
            if (j == 0) { TG_POISON_DIRECT(stage * A_STAGE, NS * A_STAGE + stage * B_STAGE); }
            if (j < A_LD) {
                direct_load<A_EL>(byte_offset(Ag, a_off[j]), smem + stage * A_STAGE + (j * NWAVES + wave) * (64 * A_EL));
                if (j == A_LD - 1) Ag += a_step;
            } else {
                const int i = j - A_LD;
                direct_load<B_EL>(byte_offset(Bg, b_off[i]), smem + NS * A_STAGE + stage * B_STAGE + (i * NWAVES + wave) * (64 * B_EL));
                if (i == B_LD - 1) { Bg += b_step; --to_issue; }
            }
        };
        const bool deep = to_issue >= NS;           // the K range fills the ring
#pragma unroll
        for (int st = 0; st < NS; ++st)
            if (to_issue > 0) issue(st);
        if (deep) __builtin_amdgcn_s_waitcnt(kWaitFirst);
        else __builtin_amdgcn_s_waitcnt(kWaitAll);
        __builtin_amdgcn_s_barrier();
        read_tile(0, 0);
        int stage = 0;                              // stage of the tile being multiplied

        // one K tile: `cur` holds its fragments, `nxt` receives those of the following tile
        auto step = [&](auto cur_c, auto nxt_c) {
            constexpr int cur = decltype(cur_c)::value, nxt = decltype(nxt_c)::value;
            __builtin_amdgcn_sched_barrier(0);
            const bool more = to_issue > 0;         // workgroup-uniform
            if (NS > 2 && more) __builtin_amdgcn_s_waitcnt(kWaitSteady);
            else __builtin_amdgcn_s_waitcnt(kWaitAll);
            __builtin_amdgcn_s_barrier();
            // (a ring of two: the stage of a tile is the register set of its fragments, a constant of this instance
            // of the step, and every LDS address of the tile is a register plus an immediate)
            const int cur_stage = NS == 2 ? cur : stage;
            const int next = NS == 2 ? nxt : (stage + 1 == NS ? 0 : stage + 1);
            // the first MFMA goes ahead of everything: the loads of the tile ahead (a block of its own, not issued
            // once the K range is exhausted) and the LDS reads go out in its shadow and in that of the following
            // ones, which do not depend on them
            // (measured at 1024^3, alternating in one process: 20.0 us this way, 20.4 us with the loads ahead of the
            // first MFMA, 21.7 us for the kernel that fetches fragments octet by octet)
            // (and the loads themselves are spread: a vector-memory instruction holds the wave's issue for several cycles,
            // and four or eight of them in a row let the MFMA pipe run dry.  K tiles of 32: A's loads behind the first MFMA,
            // B's behind the second; K tiles of 64: one load behind each of the first eight.  Measured against all loads
            // behind the first MFMA, alternating in one process, bit-identical: 1024^3 18.63 -> 18.19 us and 20.1 ->
            // 18.5 us, 768^3 14.6 -> 14.3 us, 2048^3 with K tiles of 64 126.9 -> 122.4 us; one load per MFMA with K tiles
            // of 32: no gain)
            constexpr int LOAD_BLOCKS = BK == 32 ? 2 : N_LD;
            if constexpr (BK == 32) {
                mfma_range(cur, 0, 1);
                if (more) issue_a(cur_stage);
                mfma_range(cur, 1, 2);
                if (more) issue_b(cur_stage);
            } else {
#pragma unroll
                for (int j = 0; j < N_LD; ++j) {
                    mfma_range(cur, j, j + 1);
                    if (more) issue_one(cur_stage, j);
                }
            }
            read_tile(next, nxt);
            mfma_range(cur, LOAD_BLOCKS, 4 * NO);
#pragma unroll
            for (int i = 0; i < N_RD; i += 2) {
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // LDS reads
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
            }
            __builtin_amdgcn_sched_barrier(0);
            stage = next;
        };
        typedef std::integral_constant<int, 0> set0;
        typedef std::integral_constant<int, 1> set1;
        // Second accumulation level: the K range is walked in chunks of flush_tiles tiles, after each of which
        // the MFMA accumulators are folded into `total` (one chunk when there is no second level).
        const int chunk = TWO_LEVEL ? p.flush_tiles : kt_end - kt_begin;
        int parity = 0;                             // which register set holds the tile to multiply next
        for (int kt = kt_begin; kt < kt_end;) {
            int left = kt_end - kt < chunk ? kt_end - kt : chunk;
            kt += left;
            if (parity && left > 0) {
                step(set1(), set0());
                parity = 0;
                --left;
            }
            for (; left >= 2; left -= 2) {
                step(set0(), set1());
                step(set1(), set0());
            }
            if (left) {
                step(set0(), set1());
                parity = 1;
            }
            if constexpr (TWO_LEVEL) {
                total += acc;
                acc = (f32x16)(0.0f);
            }
        }
    }
    if constexpr (TWO_LEVEL) acc = total;

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
    // Result register v of a lane is row 8 (v / 4) + v % 4 + 4 h of the wave's block, column li: the part that
    // depends on v is wave-uniform (a scalar row origin per store), the lane's part one 32-bit byte offset for all
    // sixteen stores (the host checks ldc < 2^27 for these kernels), so a store needs no vector address arithmetic.
    const int col = n0 + wn * 32 + li;
    const bool full_tile = m0 + BM <= p.m && n0 + BN <= p.n;      // workgroup-uniform
    const bool nt = p.splits == 1;
    float *block = out + (int64_t)(m0 + wm * 32) * ldo + n0 + wn * 32;
    unsigned lane_bytes = 4u * ((unsigned)(4 * h) * (unsigned)ldo + (unsigned)li);
    if (col < p.n) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = 8 * (v / 4) + (v % 4);
            const int row = m0 + wm * 32 + r + 4 * h;
            asm volatile("" : "+v"(lane_bytes));    // (keeps the widening of the offset next to the store, see at_bytes)
            float *dst = reinterpret_cast<float *>(reinterpret_cast<char *>(block + (int64_t)r * ldo) + lane_bytes);
            if (full_tile || row < p.m) store_result(dst, acc[v], nt);
        }
    }
}

template <int BM, int BN, int BK, int NS, bool TWO_LEVEL, int AM, int BMD>
hipError_t launch_tile_deep(const GemmParams &p, hipStream_t s) {
    constexpr int threads = (BM / 32) * (BN / 32) * 64;
    constexpr int lds_used = direct_lds_bytes<BM, BN, BK, NS>();
    static_assert(lds_used <= kLdsPerCU, "stages exceed the LDS of a CU");
    auto kern = sgemm_tile_deep_kernel<BM, BN, BK, NS, TWO_LEVEL, AM, BMD>;
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
