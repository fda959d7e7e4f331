// Persistent ("stream") form of the workgroup-tile SGEMM kernel for gfx950.
//
// Same tile, LDS layout, fragment mapping and MFMA blocks as tile_kernel.hpp (matmul of
// Sec. 5.2 of the paper), exact-fit shapes only.  The difference is the outer structure: a
// fixed number of workgroups (a multiple of 8, so a work item's XCD, item % 8, is the
// workgroup's own) each take work items blockIdx.x, blockIdx.x + gridDim.x, ... and treat
// the K tiles of all their items as ONE stream.  The load side runs ahead of the compute side
// across item boundaries: while the last K tiles of one output tile are multiplied, the first
// K tiles of the next one are already being fetched and staged, so there is no per-tile
// prologue, and the C stores of one output tile drain while the next is being computed.  This
// is what short-K problems need (k = 128: only 4..8 K tiles per output tile), where a
// workgroup-per-tile launch leaves the matrix pipe idle during every prologue and epilogue.
#pragma once

#include "tile_kernel.hpp"

namespace tg {

// DEFER: a finished output tile is not stored at once; it waits in a second register set and its stores are
// issued one by one between the MFMAs of the first K tile of the workgroup's next item, so that no wave ever
// spends a phase doing nothing but stores (the last item of a workgroup is stored at the end as usual).
// These variants write C only (no split-K) and need its rows naturally aligned for their CB-float stores.
template <int BM, int BN, int BK, int WM, int WN, bool TWO_LEVEL, bool DEFER>
__global__ void __launch_bounds__((BM / WM) * (BN / WN) * 64, (min_waves_per_simd<BM, BN, BK, WM, WN, TWO_LEVEL || DEFER>()))
sgemm_tile_stream_kernel(const GemmParams p) {
    constexpr int WAVES_N = BN / WN;
    constexpr int NT = (BM / WM) * (BN / WN) * 64;
    constexpr int RB = WM / 32, CB = WN / 32;
    constexpr int LDA_S = BK + kLdsPadA, LDB_S = BN + kLdsPadB;
    constexpr int A_STAGE = BM * LDA_S, B_STAGE = BK * LDB_S;
    constexpr int A_LD = BM * BK / 4 / NT, B_LD = BK * BN / 4 / NT;
    constexpr int NO = BK / 8;
    static_assert(BM % WM == 0 && BN % WN == 0 && WM % 32 == 0 && WN % 32 == 0, "tile shape");
    static_assert(CB == 1 || CB == 2 || CB == 4, "wave tile width must be 32, 64 or 128");
    static_assert(NO % 2 == 0, "BK must be a multiple of 16 (fragment sets alternate per octet)");
    static_assert((BM * BK / 4) % NT == 0 && (BK * BN / 4) % NT == 0 && A_LD >= 1 && B_LD >= 1,
                  "tile loads must divide evenly over the workgroup");
    typedef typename vec_of<CB>::type bvec;

    // LDS as in tile_kernel.hpp: stage 0 then stage 1, A then B inside a stage; every LDS address of a thread is a
    // running 32-bit LDS address that one addition per K tile moves to the other stage.
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

    const unsigned total_work = (unsigned)p.tiles_m * (unsigned)p.tiles_n * (unsigned)p.splits * (unsigned)p.batch;
    const unsigned step = gridDim.x;
    const int kt_total = p.k / BK;

    // Per-thread slots of the tile loads: slot f = tid + i*NT is one 16-byte vector.
    int a_row[A_LD], a_k[A_LD], b_row[B_LD], b_col[B_LD];
    unsigned a_off[A_LD], b_off[B_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        const int f = tid + i * NT;
        a_row[i] = a_slot_row<BK>(f);
        a_k[i] = (f % (BK / 4)) * 4;
        a_off[i] = 4u * ((unsigned)a_row[i] * (unsigned)p.lda + (unsigned)a_k[i]);     // in bytes (see at_bytes)
    }
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        const int f = tid + i * NT;
        b_row[i] = f / (BN / 4);
        b_col[i] = (f % (BN / 4)) * 4;
        b_off[i] = 4u * ((unsigned)b_row[i] * (unsigned)p.ldb + (unsigned)b_col[i]);
    }

    // K range of a work item (slice = problem * splits + split).
    auto k_range = [&](int slice, int &prob, int &kt_begin, int &kt_end) {
        prob = slice / p.splits;
        const int split = slice - prob * p.splits;
        kt_begin = split * p.ktiles_per_split;
        const int kt_stop = kt_begin + p.ktiles_per_split;
        kt_end = kt_stop < kt_total ? kt_stop : kt_total;
    };

    // ---- load side: a cursor over (work item, K tile), wave-uniform --------------------------
    unsigned ld_work = blockIdx.x;
    const float *Ag = nullptr, *Bg = nullptr;   // origin of the tile under the cursor
    int ld_left = 0;                            // K tiles of the cursor's item not fetched yet
    auto seek = [&](unsigned w) {
        int slice, tm, tn, prob, kb, ke;
        map_workgroup(p, total_work, w, slice, tm, tn);
        k_range(slice, prob, kb, ke);
        Ag = p.A + (int64_t)prob * p.strideA + (int64_t)tm * BM * p.lda + (int64_t)kb * BK;
        Bg = p.B + (int64_t)prob * p.strideB + (int64_t)kb * BK * p.ldb + (int64_t)tn * BN;
        ld_left = ke - kb;
    };

    f32x4 a_reg[A_LD], b_reg[B_LD];
    // Fetch the tile under the cursor into the staging registers and move the cursor on.  Past
    // the end of the stream the cursor stays on its last tile (fetching it again is harmless
    // and keeps the loop body uniform).
    auto load_next = [&]() {
#pragma unroll
        for (int i = 0; i < A_LD; ++i) a_reg[i] = *at_bytes(Ag, a_off[i]);
#pragma unroll
        for (int i = 0; i < B_LD; ++i) b_reg[i] = *at_bytes(Bg, b_off[i]);
        if (ld_left > 1) {
            --ld_left;
            Ag += BK;
            Bg += (int64_t)BK * p.ldb;
        } else if (ld_work + step < total_work) {
            ld_work += step;
            seek(ld_work);
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

    // ---- compute side -------------------------------------------------------------------------
    f32x16 acc[RB][CB];
    f32x16 total[TWO_LEVEL ? RB : 1][TWO_LEVEL ? CB : 1];
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

    // A result row of a lane is row r = 32 rb + 8 (v / 4) + v % 4 (+ 4 h) of its wave tile: the origin of row r is
    // wave-uniform (scalar registers), the lane's part (4 h rows down, its column) one 32-bit byte offset for all
    // its stores (the host checks ldc < 2^27 for these kernels), so a store needs no vector address arithmetic.
    auto result_at = [&](float *wave_tile, int64_t ld, int r, unsigned &lane_bytes) {
        asm volatile("" : "+v"(lane_bytes));    // (keeps the widening of the offset next to the store, see at_bytes)
        return reinterpret_cast<float *>(reinterpret_cast<char *>(wave_tile + (int64_t)r * ld) + lane_bytes);
    };
    // The waiting tile (DEFER): its values, the origin of its wave tile, this lane's offset in it, and its row stride.
    f32x16 prev[DEFER ? RB : 1][DEFER ? CB : 1];
    float *prev_tile = nullptr;
    unsigned prev_lane = 0;
    int64_t prev_ldo = 0;
    bool have_prev = false;
    // Stores rows v = 8 * part .. 8 * part + 7 of every 32-row block of the waiting tile (RB * 8 stores).
    auto store_prev = [&](int part) {
#pragma unroll
        for (int rb = 0; rb < (DEFER ? RB : 0); ++rb) {
#pragma unroll
            for (int vv = 0; vv < 8; ++vv) {
                const int v = 8 * part + vv;
                float *dst = result_at(prev_tile, prev_ldo, rb * 32 + 8 * (v / 4) + (v % 4), prev_lane);
                bvec o;
                if constexpr (CB == 1) {
                    o = prev[rb][0][v];
                } else {
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb) o[cb] = prev[rb][cb][v];
                }
                store_result(dst, o, true);
            }
        }
    };
    constexpr int PART_STORES = RB * 8;

    constexpr int N_MFMA = 4 * RB * CB;
    constexpr int N_ST = A_LD + B_LD;
    constexpr int MFMA_PER_ST = N_MFMA / N_ST > 0 ? N_MFMA / N_ST : 1;

    // One K tile of the stream (see tile_kernel.hpp for the order of operations inside a tile).  With the drain
    // tag the stores of the waiting tile go out between its MFMAs, half with the LDS writes, half with the loads.
    // Single steps of a K tile, for the drain form below, where the order is written out instruction by instruction
    // (a sched_group_barrier pattern cannot place the stores: their address arithmetic is not in its vocabulary).
    auto mfma_one = [&](int set, int j) {   // j enumerates (t, rb, cb) in the order of mfma_octet
        const int t = j / (RB * CB), rb = (j / CB) % RB, cb = j % CB;
        acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_frag[set][rb][t], vec_get(b_frag[set][t], cb), acc[rb][cb], 0, 0, 0);
    };
    auto lds_write_one = [&](int i) {
        if (i < A_LD) *reinterpret_cast<f32x4 *>(lds(wr_a) + i * A_SLOT_ROWS * LDA_S) = a_reg[i];
        else *reinterpret_cast<f32x4 *>(lds(wr_b) + (i - A_LD) * B_SLOT_ROWS * LDB_S) = b_reg[i - A_LD];
    };
    auto load_one = [&](int i) {
        if (i < A_LD) a_reg[i] = *at_bytes(Ag, a_off[i]);
        else b_reg[i - A_LD] = *at_bytes(Bg, b_off[i - A_LD]);
    };
    auto advance_cursor = [&]() {
        if (ld_left > 1) {
            --ld_left;
            Ag += BK;
            Bg += (int64_t)BK * p.ldb;
        } else if (ld_work + step < total_work) {
            ld_work += step;
            seek(ld_work);
        }
    };
    auto store_prev_one = [&](int part, int sidx) {
        const int rb = sidx / 8, v = 8 * part + sidx % 8;
        float *dst = result_at(prev_tile, prev_ldo, rb * 32 + 8 * (v / 4) + (v % 4), prev_lane);
        bvec o;
        if constexpr (CB == 1) {
            o = prev[DEFER ? rb : 0][0][v];
        } else {
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) o[cb] = prev[DEFER ? rb : 0][cb][v];
        }
        store_result(dst, o, true);   // (DEFER variants: C only, rows naturally aligned: checked on the host)
    };

    // One K tile of the stream (see tile_kernel.hpp for the order of operations inside a tile).  With the drain
    // tag the stores of the waiting tile go out between its MFMAs, half with the LDS writes, half with the loads.
    // s_waitcnt encodings (gfx9: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8; all ones = not waited for)
    constexpr int kWaitLoads = 0x0F70;           // vmcnt(0)
    constexpr int kWaitOlderReads = 0xC07F | ((RB + 4) << 8);   // lgkmcnt(the reads of one octet): everything older has returned
    auto tile_body = [&](auto drain_tag) {
        constexpr bool DRAIN = decltype(drain_tag)::value;
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
        __builtin_amdgcn_s_waitcnt(kWaitLoads & kWaitOlderReads);   // and one for the staged tile instead of one per LDS write
        if constexpr (DRAIN) {
#pragma unroll
            for (int j = 0; j < N_MFMA; ++j) {
                mfma_one((NO - 2) & 1, j);
                if (j % MFMA_PER_ST == MFMA_PER_ST - 1 && j / MFMA_PER_ST < N_ST) lds_write_one(j / MFMA_PER_ST);
#pragma unroll
                for (int q = j * PART_STORES / N_MFMA; q < (j + 1) * PART_STORES / N_MFMA; ++q) store_prev_one(0, q);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int i = N_MFMA / MFMA_PER_ST; i < N_ST; ++i) lds_write_one(i);
        } else {
            mfma_octet((NO - 2) & 1);
            store_lds();
#pragma unroll
            for (int i = 0; i < N_ST; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, MFMA_PER_ST, 0);   // MFMA
                __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);             // LDS write
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        other_stage();                        // the stage just completed is multiplied next, the one just left is filled next
        poison_lds();                         // (debug flavour only: nothing reads that stage any more)
        read_frags(0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (DRAIN) {
#pragma unroll
            for (int j = 0; j < N_MFMA; ++j) {
                if (j % MFMA_PER_ST == 0 && j / MFMA_PER_ST < N_ST) load_one(j / MFMA_PER_ST);
                mfma_one((NO - 1) & 1, j);
#pragma unroll
                for (int q = j * PART_STORES / N_MFMA; q < (j + 1) * PART_STORES / N_MFMA; ++q) store_prev_one(1, q);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int i = N_MFMA / MFMA_PER_ST; i < N_ST; ++i) load_one(i);
            advance_cursor();
        } else {
            load_next();
            mfma_octet((NO - 1) & 1);
#pragma unroll
            for (int i = 0; i < N_ST; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);             // global load
                __builtin_amdgcn_sched_group_barrier(0x008, MFMA_PER_ST, 0);   // MFMA
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- start of the stream --------------------------------------------------------------------
    seek(ld_work);
    load_next();
    store_lds();                              // stage 0
    __syncthreads();
    read_frags(0, 0);
    wr_a += PITCH_BYTES;                      // the next tile is staged in stage 1
    wr_b += PITCH_BYTES;
    load_next();

    for (unsigned work = blockIdx.x; work < total_work; work += step) {
        int slice, tm, tn, prob, kb, ke;
        map_workgroup(p, total_work, work, slice, tm, tn);
        k_range(slice, prob, kb, ke);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                acc[rb][cb] = (f32x16)(0.0f);
                if constexpr (TWO_LEVEL) total[rb][cb] = (f32x16)(0.0f);
            }
        int since_flush = 0;

        // Every K tile of the stream runs the same body (see tile_kernel.hpp for the order of
        // operations inside a tile); the tile staged and the tile fetched may belong to the
        // next work item.
        for (int kt = kb; kt < ke; ++kt) {
            if constexpr (TWO_LEVEL) {
                if (since_flush == p.flush_tiles) {
                    since_flush = 0;
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb) {
                            total[rb][cb] += acc[rb][cb];
                            acc[rb][cb] = (f32x16)(0.0f);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                }
                ++since_flush;
            }
            __builtin_amdgcn_sched_barrier(0);
            if (DEFER && have_prev && kt == kb) {   // wave-uniform
                tile_body(std::true_type());
                have_prev = false;
            } else {
                tile_body(std::false_type());
            }
        }
        if constexpr (TWO_LEVEL) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) acc[rb][cb] += total[rb][cb];
        }

        // Epilogue of this work item: registers -> C (or the split-K partial).  The stores are
        // not waited for; they drain while the next item's tiles are multiplied.
        float *out;
        int64_t ldo;
        if (p.splits > 1) {
            out = p.ws + (int64_t)slice * p.m * p.n;
            ldo = p.n;
        } else {
            out = p.C + (int64_t)prob * p.strideC;
            ldo = p.ldc;
        }
        const bool nt = p.splits == 1 && rows_aligned<CB>(out, ldo);
        float *wave_tile = out + (int64_t)(tm * BM + wm * WM) * ldo + tn * BN + wn * WN;
        unsigned lane_bytes = 4u * ((unsigned)(4 * h) * (unsigned)ldo + (unsigned)(li * CB));
        if constexpr (DEFER) {
            // (a tile still waiting here had no successor K tile to ride on: cannot happen, every item has one)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) prev[rb][cb] = acc[rb][cb];
            prev_tile = wave_tile;
            prev_lane = lane_bytes;
            prev_ldo = ldo;
            have_prev = true;
        } else {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float *dst = result_at(wave_tile, ldo, rb * 32 + 8 * (v / 4) + (v % 4), lane_bytes);
                    bvec o;
                    if constexpr (CB == 1) {
                        o = acc[rb][0][v];
                    } else {
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb) o[cb] = acc[rb][cb][v];
                    }
                    store_result(dst, o, nt);
                }
            }
        }
    }
    if (DEFER && have_prev) {   // the workgroup's last item
        store_prev(0);
        store_prev(1);
    }
}

template <int BM, int BN, int BK, int WM, int WN, bool TWO_LEVEL, bool DEFER>
hipError_t launch_tile_stream(const GemmParams &p, hipStream_t s) {
    constexpr int threads = (BM / WM) * (BN / WN) * 64;
    constexpr int lds_used = tile_lds_bytes<BM, BN, BK, WM, WN>();
    auto kern = sgemm_tile_stream_kernel<BM, BN, BK, WM, WN, TWO_LEVEL, DEFER>;
    int lds = lds_used;
    if (p.max_blocks_per_cu > 0) {
        const int share = (kLdsPerCU / p.max_blocks_per_cu) & ~1023;
        if (share > lds) lds = share;
    }
    static std::atomic<uint64_t> lds_limit_raised{0};   // one bit per device: the attribute is kept per device
    const hipError_t attr = allow_full_lds(reinterpret_cast<const void *>(kern), lds_limit_raised);
    if (attr != hipSuccess) return attr;
    // a multiple of 8 workgroups (p.persistent_blocks), or one per item when there are fewer items
    int64_t blocks = (int64_t)p.tiles_m * p.tiles_n * p.splits * p.batch;
    if (p.persistent_blocks > 0 && p.persistent_blocks < blocks) blocks = p.persistent_blocks;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(threads), lds, s, p);
    return hipGetLastError();
}

}  // namespace tg
