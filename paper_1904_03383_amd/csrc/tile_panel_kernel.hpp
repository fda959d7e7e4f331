// Row-panel SGEMM kernel for a gathered A (the strided matmul of Sec. 5.2 of the paper: consecutive
// elements of a row of A lie a fixed number of floats apart, so that at a large stride every element
// is a cache line of its own).  What such a product costs is line requests: every tile that needs an
// element requests its line again.  This kernel gives a workgroup 16 rows of A and up to 1024 columns
// of B, so an element is requested once per 1024 columns of the result, and fills the chip through a
// K split (partial products meet in the split-K reduction) where 16-row panels alone are too few.
//
// Roles inside a workgroup (the BLOCK / THREAD mapping of Sec. 4, with the SHARED temporary for A only):
//  * NP producer waves do nothing but gather.  Per chunk of 64, 128 or 256 k each fetches its rows of the panel,
//    one 4-byte direct-to-LDS load per row and 64 k (lane l fetches element k0 + l), into a ring of three LDS
//    stages, two chunks ahead of the product.  Their loads are the only ones they ever wait for, so the
//    gather queue never drains: a wave that also loaded B would have to wait for its youngest gather
//    whenever it needs an older B vector (vector-memory results return in order).
//  * NC compute waves own 16 or 32 rows x 64 or 128 columns of the result each.  B is used by one wave
//    only (a panel has a single tile row), so it does not go through LDS: per 16-k step a lane fetches one
//    or two 16-byte vectors (its 4 or 8 adjacent columns) from each of its four k rows into registers, one
//    or three 16-k steps ahead of the MFMAs, and reads its four consecutive k values of A's row with one ds_read_b128.
//  * One barrier per chunk joins the two roles: the producers arrive when the next chunk has landed,
//    the compute waves when they are done with the previous one (which frees its stage).
//
// v_mfma_f32_16x16x4_f32 operand and result layout: see mfma_shape<16> in tile_direct_kernel.hpp; the
// k pairing (MFMA t of a step multiplies k = 4h + t) and the ownership of adjacent columns by one lane
// only reorder the sum and the stores.
#pragma once

#include "tile_direct_kernel.hpp"

namespace tg {

constexpr int kPanelRows = 16;
// s_waitcnt operand that waits until at most n vector-memory operations are outstanding and for nothing else
// (gfx9: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8; all ones = not waited for)
constexpr int panel_vmcnt(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }
constexpr int kPanelStages = 3;
constexpr unsigned kPanelCUs = 256;     // MI355X: 8 XCDs of 32 CUs (a grid up to this size gives every workgroup a CU of its own)

// Workgroups are dealt to the eight XCDs in turn (workgroup w runs on XCD w % 8, each with an L2 of its own).  The
// persistent row-panel forms want the workgroups that share a row panel of A on one XCD, so that a strided A crosses
// the fabric once per panel and not once per XCD that holds one of its workgroups (2048^3 with A at stride 32, four
// workgroups per panel: 294 us with neighbours on four XCDs, 210 us for the one-tile form, whose order keeps them
// together): this is the position of workgroup w in an order that lists XCD 0's workgroups first, then XCD 1's, ...
// (grids that are not a multiple of eight keep their order).
__device__ __forceinline__ unsigned xcd_major(unsigned w, unsigned grid) {
    return (grid & 7u) == 0 ? (w & 7u) * (grid >> 3) + (w >> 3) : w;
}

// NC compute waves, NP producer waves, RB blocks of 16 rows per panel, NQ groups of four adjacent columns per lane
// (every compute wave owns 16 * RB x 64 * NQ of the result and uses a B vector RB times), TWO_LEVEL: second
// accumulation level for K ranges beyond 1024, PD: how many 16-k steps ahead of the MFMAs B is fetched (1 or 3), CW: k per
// chunk in units of 64 (the lanes of one gather instruction): a producer fills a row of a chunk with CW instructions.
// WALK: persistent launch in which a workgroup owns several neighbouring column tiles of one row panel and takes them one
// after the other with the chunk pipeline running on across the tile boundaries: while the results of one tile are
// stored the producers are two chunks into the next and B's prefetch is in its columns (one problem, one K range,
// whole tiles; the host checks).  For products with a short K, where a workgroup per tile spends as long starting and
// ending as multiplying.
template <int NC, int NP, int RB, int NQ, bool TWO_LEVEL, int PD, int CW, bool WALK>
__global__ void __launch_bounds__((NC + NP) * 64) sgemm_panel_kernel(const GemmParams p) {
    constexpr int kPanelChunk = 64 * CW;
    constexpr int kPanelPitch = kPanelChunk + 8;       // floats per row of a stage (measured at 72: 0 bank-conflict cycles on the fragment reads; 68 and 84: half of the LDS cycles)
    constexpr int STEPS = 4 * CW;                      // 16-k steps per chunk
    constexpr int BM = kPanelRows * RB;
    static_assert(BM % NP == 0, "producer waves share the rows evenly");
    static_assert(BM / NP * CW <= 63, "the gather instructions of one chunk must fit the wait counter");
    static_assert(NQ == 1 || NQ == 2, "a lane owns four or eight adjacent columns");
    static_assert(PD == 1 || PD == 3, "register sets of B: PD + 1 must divide the four steps of a chunk");
    constexpr int NSETS = PD + 1;
    constexpr int WN = 64 * NQ, BN = NC * WN;
    constexpr int NE = 4 * NQ;                   // accumulator blocks (of 16 x 16) per row block = columns per lane
    constexpr int NLD = 4 * NQ;                  // B vectors per lane and 16-k step
    constexpr int ROWS_PER_PRODUCER = BM / NP;
    constexpr int kPanelStageFloats = BM * kPanelPitch;
    __shared__ __attribute__((aligned(16))) float smem[kPanelStages * kPanelStageFloats];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const unsigned total_work = (unsigned)p.tiles_m * (unsigned)p.tiles_n * (unsigned)p.splits * (unsigned)p.batch;
    int slice, tm, tn;
    int walk = 1;                                // tiles this workgroup takes
    if constexpr (WALK) {
        walk = (int)(total_work / gridDim.x);
        const unsigned per_row = (unsigned)p.tiles_n / (unsigned)walk;
        const unsigned id = xcd_major(blockIdx.x, gridDim.x);
        slice = 0;
        tm = (int)(id / per_row);
        tn = (int)(id % per_row) * walk;
    } else {
        map_workgroup(p, total_work, blockIdx.x, slice, tm, tn);
    }
    const int prob = slice / p.splits, split = slice - prob * p.splits;
    const int m0 = tm * BM, n0 = tn * BN;
    const int ch_total = p.k / kPanelChunk;
    const int ch_begin = split * p.ktiles_per_split;
    const int ch_stop = ch_begin + p.ktiles_per_split;
    const int nch = (ch_stop < ch_total ? ch_stop : ch_total) - ch_begin;   // >= 1: the host plans no empty K range
    const int64_t k_begin = (int64_t)ch_begin * kPanelChunk;

    if (wave >= NC) {
        // ---- producer ---------------------------------------------------------------------------------
        const int pw = wave - NC;
        const float *row[ROWS_PER_PRODUCER];
#pragma unroll
        for (int i = 0; i < ROWS_PER_PRODUCER; ++i) {
            const int r = pw * ROWS_PER_PRODUCER + i;
            const int rg = m0 + r < p.m ? m0 + r : p.m - 1;   // rows past the end re-read the last one (never stored)
            row[i] = p.A + (int64_t)prob * p.strideA + (int64_t)rg * p.lda + k_begin * p.csa;
        }
        unsigned lane_bytes = 4u * (unsigned)lane * (unsigned)p.csa;   // (the host checks that a chunk spans < 2^30 elements)
        const int64_t step = (int64_t)kPanelChunk * p.csa;
        int gathered = 0;                        // chunks of the current tile asked for
        // Pacing: once the pipeline is full, a producer rests after each row's loads, so that the loads of a chunk
        // spread over about half of the time the compute waves spend on one (512 * CW * NQ * RB * NC cycles of MFMAs;
        // s_sleep counts in units of 64) instead of leaving in one burst that the compute waves' own loads of B have to
        // queue behind.  Only where the workgroup has its CU to itself (a grid of at most one workgroup per CU): with
        // several resident their bursts interleave anyway.  Same process, bit-identical, A at stride 32: 4096x1024x1024
        // 124.5 -> 114.6 us, 2048^3 209.9 -> 197.7 us, 1024^3 33.2 -> 32.4 us, 512^3 17.2 -> 16.9 us; plain operands
        // unchanged; resting for the whole of a chunk's time instead of half costs the plain products 1 %, but where
        // every element of A is a cache line of its own (stride >= 32) it is the better spread: another 0.3 - 2.5 %
        // (2048^3 185.0 -> 181.9 us, 1024^3 at stride 64 38.7 -> 37.7 us, 1024^3 at stride 32 32.4 -> 32.1 us).
        constexpr int kPaceRaw = 4 * CW * NQ * RB * NC / ROWS_PER_PRODUCER;
        constexpr int kPace = kPaceRaw < 127 ? kPaceRaw : 127;
        constexpr int kPaceFar = 2 * kPaceRaw < 127 ? 2 * kPaceRaw : 127;
        const bool far = p.csa >= 32;            // every element a cache line of its own
        const bool may_pace = kPace > 0 && gridDim.x <= kPanelCUs;
        bool paced = false;
        auto gather = [&](int stage) {
#pragma unroll
            for (int i = 0; i < ROWS_PER_PRODUCER; ++i) {
                const int r = pw * ROWS_PER_PRODUCER + i;
#pragma unroll
                for (int w = 0; w < CW; ++w)
                    direct_load<1>(byte_offset(row[i] + (int64_t)(64 * w) * p.csa, lane_bytes),
                                   smem + stage * kPanelStageFloats + r * kPanelPitch + 64 * w);
                row[i] += step;
                if (paced) {
                    if (far) __builtin_amdgcn_s_sleep(kPaceFar);
                    else __builtin_amdgcn_s_sleep(kPace);
                }
            }
            if constexpr (WALK) {
                if (++gathered == nch) {         // the next tile of the walk has the same rows of A: back to their start
                    gathered = 0;
#pragma unroll
                    for (int i = 0; i < ROWS_PER_PRODUCER; ++i) row[i] -= (int64_t)nch * step;
                }
            }
        };
        const int chunks = walk * nch;
#ifdef TG_POISON_LDS
        for (int s = 0; s < kPanelStages; ++s)
            for (int i = 0; i < ROWS_PER_PRODUCER; ++i)
                for (int w = 0; w < CW; ++w) smem[s * kPanelStageFloats + (pw * ROWS_PER_PRODUCER + i) * kPanelPitch + 64 * w + lane] = __builtin_nanf("");
        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
#endif
        gather(0);
        if (chunks > 1) gather(1);
        int stage_free = 2;                      // where chunk j + 2 goes
        paced = may_pace;
        for (int j = 0; j < chunks; ++j) {
            // chunk j has landed (the chunk after it may still be on its way)
            if (j + 1 < chunks) __builtin_amdgcn_s_waitcnt(panel_vmcnt(ROWS_PER_PRODUCER * CW));   // vmcnt(one chunk's loads)
            else __builtin_amdgcn_s_waitcnt(0x0F70);                                   // vmcnt(0)
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();        // #j: chunk j may be read; nobody reads chunk j - 1 any more
            __builtin_amdgcn_sched_barrier(0);
            if (j + 2 < chunks) {
#ifdef TG_POISON_LDS
                for (int i = 0; i < ROWS_PER_PRODUCER; ++i)
                    for (int w = 0; w < CW; ++w) smem[stage_free * kPanelStageFloats + (pw * ROWS_PER_PRODUCER + i) * kPanelPitch + 64 * w + lane] = __builtin_nanf("");
                __builtin_amdgcn_s_waitcnt(0xC07F);
#endif
                gather(stage_free);
            }
            stage_free = stage_free == kPanelStages - 1 ? 0 : stage_free + 1;
        }
        return;
    }

    // ---- compute --------------------------------------------------------------------------------------
    const int c = lane & 15, g = lane >> 4;
    const int n0w = n0 + wave * WN;
    // the lane's NQ groups of four adjacent columns; a group past the end re-reads the last four columns
    // (the width that may be fetched, nb, is a multiple of 4: n itself, or n rounded up when B is a padded copy) and
    // is not stored
    const int last = p.nb - 4;
    // B is addressed from a wave-uniform row origin (scalar registers, advanced per step) plus one 32-bit byte offset
    // per lane and column group (the host checks that 64 rows of B span fewer than 2^30 elements)
    const float *Bg = p.B + (int64_t)prob * p.strideB + k_begin * p.ldb;
    int col[NQ];
    unsigned off[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        col[q] = n0w + 4 * NQ * c + 4 * q;
        off[q] = 4u * ((unsigned)(4 * g) * (unsigned)p.ldb + (unsigned)(col[q] < last ? col[q] : last));
    }
    const int64_t step_b = 16 * p.ldb;
    int steps_left = STEPS * nch * walk;             // 16-k steps not yet fetched
    int steps_of_tile = STEPS * nch;                 // ... of the tile the prefetch is in
    const float *const B_first = Bg;

    f32x4 bq[NSETS][4][NQ];
    // vector i = NQ * t + q of a step: k row 4g + t, column group q
    auto fetch_one = [&](int set, int i) {
        const float *r = Bg + (int64_t)(i / NQ) * p.ldb;
        bq[set][i / NQ][i % NQ] = *reinterpret_cast<const f32x4 *>(byte_offset(r, off[i % NQ]));
    };
    // past the end of the K range the last step is fetched again (in bounds, never multiplied): the number of
    // loads in flight stays the same through the whole loop
    auto next_step = [&]() {
        if (steps_left > 1) {
            --steps_left;
            if (WALK && --steps_of_tile == 0) {  // on to the next tile of the walk: same K range, the next BN columns
                steps_of_tile = STEPS * nch;
                Bg = B_first;
#pragma unroll
                for (int q = 0; q < NQ; ++q) off[q] += 4u * BN;
            } else {
                Bg += step_b;
            }
        }
    };

    // two accumulation levels: every flush_tiles chunks the MFMA accumulators are folded into `total`, which bounds the
    // length of any single fp32 running sum (as in the other tile kernels)
    f32x4 acc[RB][NE], total[TWO_LEVEL ? RB : 1][TWO_LEVEL ? NE : 1];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            acc[rb][e] = (f32x4)(0.0f);
            if constexpr (TWO_LEVEL) total[rb][e] = (f32x4)(0.0f);
        }

    const float *a_lane = smem + c * kPanelPitch + 4 * g;
    f32x4 a_frag[2][RB];
    auto read_a = [&](int stage, int s, int set) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            a_frag[set][rb] = *reinterpret_cast<const f32x4 *>(a_lane + stage * kPanelStageFloats + rb * 16 * kPanelPitch + 16 * s);
    };
    // A step is 4 * NQ groups of one load (for the step PD steps on, into the register set that step will use: the steps
    // per chunk are a multiple of the sets, so step s of any chunk uses set s % NSETS) and 4 * RB independent MFMAs,
    // written in the order they are to issue and fenced: left alone, the scheduler sinks the loads to their uses and
    // waits for each in turn.  The load stands in the middle of its group, behind half of the MFMAs: a vector-memory
    // instruction holds the wave's issue for several cycles, and with the MFMA pipe freshly fed they pass unnoticed
    // (measured against the load in front of the group: 1024^3 18.45 -> 18.15 us, 4096^3 922 -> 915 us; all loads of
    // a step in front of its MFMAs: 20.3 and 955 us).
    // half h of the MFMAs of group i of step s: two of the group's four columns, every row block
    auto mfma_half = [&](int s, int i, int h) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int e = 4 * (i % NQ) + 2 * h; e < 4 * (i % NQ) + 2 * h + 2; ++e)
                acc[rb][e] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_frag[s & 1][rb][i / NQ], bq[s % NSETS][i / NQ][e / 4][e % 4],
                                                                  acc[rb][e], 0, 0, 0);
    };
    auto chunk = [&](int stage) {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();            // #j (see the producer)
        __builtin_amdgcn_sched_barrier(0);
        read_a(stage, 0, 0);
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                mfma_half(s, i, 0);
                __builtin_amdgcn_sched_barrier(0);
                fetch_one((s + PD) % NSETS, i);
                if (i == 0 && s < STEPS - 1) read_a(stage, s + 1, (s + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
                mfma_half(s, i, 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            next_step();
        }
    };

#pragma unroll
    for (int s = 0; s < PD; ++s) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) fetch_one(s, i);
        next_step();
    }
    int stage = 0;
    for (int t = 0; t < walk; ++t) {
    if (WALK && t > 0) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int e = 0; e < NE; ++e) {
                acc[rb][e] = (f32x4)(0.0f);
                if constexpr (TWO_LEVEL) total[rb][e] = (f32x4)(0.0f);
            }
    }
    int since_flush = 0;
    for (int j = 0; j < nch; ++j) {
        if constexpr (TWO_LEVEL) {
            if (since_flush == p.flush_tiles) {
                since_flush = 0;
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int e = 0; e < NE; ++e) {
                        total[rb][e] += acc[rb][e];
                        acc[rb][e] = (f32x4)(0.0f);
                    }
            }
            ++since_flush;
        }
        chunk(stage);
        stage = stage == kPanelStages - 1 ? 0 : stage + 1;
    }
    if constexpr (TWO_LEVEL) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int e = 0; e < NE; ++e) acc[rb][e] += total[rb][e];
    }

    // Epilogue: registers -> C (or the split-K partial).  Register v of block e: row 4g + v, column 4 * NQ * c + e.
    float *out;
    int64_t ldo;
    if (p.splits > 1) {
        out = p.ws + (int64_t)slice * p.m * p.n;
        ldo = p.n;
    } else {
        out = p.C + (int64_t)prob * p.strideC;
        ldo = p.ldc;
    }
    const bool nt = p.splits == 1 && rows_aligned<4>(out, ldo);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int r = m0 + 16 * rb + 4 * g + v;
            if (r >= p.m) continue;
            float *dst = out + (int64_t)r * ldo;
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int cq = col[q] + t * BN;
                if (cq >= p.n) continue;
                f32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = acc[rb][4 * q + e][v];
                // (B may have been fetched from a copy padded to a multiple of 4 columns: the last group of an n that is
                // not one leaves element by element)
                store_lane<4>(dst + cq, o, cq + 4 <= p.n, cq, p.n, nt);
            }
        }
    }
    }   // tiles of the walk
}

template <int NC, int NP, int RB, int NQ, bool TWO_LEVEL, int PD, int CW, bool WALK>
hipError_t launch_tile_panel(const GemmParams &p, hipStream_t s) {
    const int64_t blocks = WALK ? p.persistent_blocks : (int64_t)p.tiles_m * p.tiles_n * p.splits * p.batch;
    hipLaunchKernelGGL((sgemm_panel_kernel<NC, NP, RB, NQ, TWO_LEVEL, PD, CW, WALK>), dim3((unsigned)blocks), dim3((NC + NP) * 64), 0, s, p);
    return hipGetLastError();
}

}  // namespace tg
