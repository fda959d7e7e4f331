// Row-panel SGEMM kernel for a short K (the 4096 x 4096 x 128 product of Table 1 of the paper is the
// shape it is for): the workgroup's rows of A stay in LDS over their whole K range, so after one gather
// and one barrier no wave ever waits for another again.
//
// A workgroup owns 16 or 32 rows of A and several neighbouring column tiles of that row panel (a
// persistent launch, as the walking form of the row-panel kernel).  All waves first gather the panel
// (4-byte direct-to-LDS loads, lane l fetches element k0 + l of a row: any element stride of A), wait
// for it and meet at the only barrier.  From there every wave is on its own: it owns 64 columns of each
// tile, fetches B straight from global memory into registers a few 16-k steps ahead (B is used by one
// wave only), reads its A fragments from LDS one step ahead, and stores a finished 16 * RB x 64 block
// while the other waves of its SIMD go on multiplying: the waves drift apart, and the stores, which in
// a kernel with a barrier per K tile hold up every wave of the workgroup, hold up their own wave only.
//
// Layouts of the matrix instruction and of the stores: as in the row-panel kernel.
#pragma once

#include "tile_panel_kernel.hpp"

namespace tg {

// floats of LDS per row of the panel: k + 8 (k a multiple of 64: the pitch is 8 mod 32, which keeps the 16-byte
// fragment reads of 16 rows off each other's banks, as measured for the row-panel kernel's pitch of 72)
constexpr int resident_pitch(int k) { return k + 8; }
constexpr int kResidentMaxLds = 64 * 1024;

// NC waves, RB blocks of 16 rows per panel, NQ groups of four adjacent columns per lane, PD: how many 16-k steps ahead
// of the MFMAs B is fetched (1 or 3)
template <int NC, int RB, int NQ, int PD>
__global__ void __launch_bounds__(NC * 64) sgemm_resident_kernel(const GemmParams p) {
    constexpr int BM = kPanelRows * RB;
    static_assert(NQ == 1 || NQ == 2, "a lane owns four or eight adjacent columns");
    static_assert(PD == 1 || PD == 3, "register sets of B: PD + 1 must divide the four steps of 64 k");
    constexpr int NSETS = PD + 1;
    constexpr int WN = 64 * NQ, BN = NC * WN;
    constexpr int NE = 4 * NQ, NLD = 4 * NQ;
    extern __shared__ __attribute__((aligned(16))) float smem[];   // BM rows of resident_pitch(k) floats

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int pitch = resident_pitch(p.k);

    const unsigned tiles = (unsigned)p.tiles_m * (unsigned)p.tiles_n;
    const int walk = (int)(tiles / gridDim.x);                 // tiles this workgroup takes (the host checks that it divides)
    const unsigned per_row = (unsigned)p.tiles_n / (unsigned)walk;
    const unsigned id = xcd_major(blockIdx.x, gridDim.x);   // the workgroups of one row panel on one XCD
    const int tm = (int)(id / per_row);
    const int tn = (int)(id % per_row) * walk;
    const int m0 = tm * BM, n0 = tn * BN;
    const int nch = p.k / 64;                                  // runs of four 16-k steps

    // ---- B: a wave-uniform row origin (scalar registers) plus one 32-bit byte offset per lane and column group
    const int c = lane & 15, g = lane >> 4;
    const int n0w = n0 + wave * WN;
    const int last = p.nb - 4;
    const float *Bg = p.B;
    int col[NQ];
    unsigned off[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        col[q] = n0w + 4 * NQ * c + 4 * q;
        off[q] = 4u * ((unsigned)(4 * g) * (unsigned)p.ldb + (unsigned)(col[q] < last ? col[q] : last));
    }
    const int64_t step_b = 16 * p.ldb;
    int steps_left = 4 * nch * walk;                 // 16-k steps not yet fetched
    int steps_of_tile = 4 * nch;                     // ... of the tile the prefetch is in

    f32x4 bq[NSETS][4][NQ];
    auto fetch_one = [&](int set, int i) {
        const float *r = Bg + (int64_t)(i / NQ) * p.ldb;
        bq[set][i / NQ][i % NQ] = *reinterpret_cast<const f32x4 *>(byte_offset(r, off[i % NQ]));
    };
    // past the end of the walk the last step is fetched again (in bounds, never multiplied)
    auto next_step = [&]() {
        if (steps_left > 1) {
            --steps_left;
            if (--steps_of_tile == 0) {              // on to the next tile: same K range, the next BN columns
                steps_of_tile = 4 * nch;
                Bg = p.B;
#pragma unroll
                for (int q = 0; q < NQ; ++q) off[q] += 4u * BN;
            } else {
                Bg += step_b;
            }
        }
    };
#pragma unroll
    for (int s = 0; s < PD; ++s) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) fetch_one(s, i);
        next_step();
    }

    // ---- A: every wave gathers the rows wave, wave + NC, ... of the panel
    {
        unsigned lane_bytes = 4u * (unsigned)lane * (unsigned)p.csa;
        const int64_t run = (int64_t)64 * p.csa;
        for (int r = wave; r < BM; r += NC) {
            const int rg = m0 + r < p.m ? m0 + r : p.m - 1;    // rows past the end re-read the last one (never stored)
            const float *src = p.A + (int64_t)rg * p.lda;
            float *dst = smem + r * pitch;
#ifdef TG_POISON_LDS
            for (int w = 0; w < nch; ++w) dst[64 * w + lane] = __builtin_nanf("");
            __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
#endif
            for (int w = 0; w < nch; ++w) {
                direct_load<1>(byte_offset(src, lane_bytes), dst);
                src += run;
                dst += 64;
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0): the panel (and the first steps of B) have landed
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    }

    const float *a_lane = smem + c * pitch + 4 * g;
    const int block_floats = 16 * pitch;
    f32x4 a_frag[2][RB];
    auto read_a = [&](int k0, int set) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            a_frag[set][rb] = *reinterpret_cast<const f32x4 *>(a_lane + rb * block_floats + k0);
    };

    float *const out = p.C;
    const bool nt = rows_aligned<4>(out, p.ldc);
    f32x4 acc[RB][NE];
    read_a(0, 0);
    for (int t = 0; t < walk; ++t) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int e = 0; e < NE; ++e) acc[rb][e] = (f32x4)(0.0f);
        for (int j = 0; j < nch; ++j) {
            const int k_next = j + 1 < nch ? 64 * (j + 1) : 0;   // (after the last run: the first fragment of the next tile)
            // four steps of 4 * NQ groups of one load (for the step PD steps on) and 4 * RB independent MFMAs, in the
            // order they are to issue, fenced group by group (see the row-panel kernel; with four waves per SIMD the load
            // in front of its group is the faster place here: 36.1 us against 36.3 - 36.7 us with it in the middle)
#pragma unroll
            for (int s = 0; s < 4; ++s) {
#pragma unroll
                for (int i = 0; i < NLD; ++i) {
                    fetch_one((s + PD) % NSETS, i);
                    if (i == 0) read_a(s < 3 ? 64 * j + 16 * (s + 1) : k_next, (s + 1) & 1);
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                        for (int e = 4 * (i % NQ); e < 4 * (i % NQ) + 4; ++e)
                            acc[rb][e] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_frag[s & 1][rb][i / NQ], bq[s % NSETS][i / NQ][e / 4][e % 4],
                                                                              acc[rb][e], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
                next_step();
            }
        }
        // registers -> C.  Register v of block e: row 4g + v, column 4 * NQ * c + e.
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int r = m0 + 16 * rb + 4 * g + v;
                if (r >= p.m) continue;
                float *dst = out + (int64_t)r * p.ldc;
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const int cq = col[q] + t * BN;
                    if (cq >= p.n) continue;
                    f32x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = acc[rb][4 * q + e][v];
                    store_result(dst + cq, o, nt);
                }
            }
        }
    }
}

template <int NC, int RB, int NQ, int PD>
hipError_t launch_tile_resident(const GemmParams &p, hipStream_t s) {
    const size_t lds = (size_t)kPanelRows * RB * resident_pitch(p.k) * sizeof(float);
    if (lds > (size_t)kResidentMaxLds || p.batch != 1 || p.splits != 1) return hipErrorInvalidValue;   // (the host's validity check says why)
    hipLaunchKernelGGL((sgemm_resident_kernel<NC, RB, NQ, PD>), dim3((unsigned)p.persistent_blocks), dim3(NC * 64), lds, s, p);
    return hipGetLastError();
}

}  // namespace tg
