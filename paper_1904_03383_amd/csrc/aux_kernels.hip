// Kernels around the workgroup-tile SGEMM: the one-wave-per-tile kernel for small and
// batched problems, the deterministic split-K reduction and the k == 0 zero fill.
#include "tile_kernel.hpp"

namespace tg {

// One wave computes one 32x32 tile of C over the whole of K (matmul of Sec. 5.2 of the
// paper, per problem of a batch), reading its operands straight from global memory: with
// a single wave per tile nothing is shared between waves, so LDS staging and barriers
// would only add latency.  Four independent waves share a 256-thread workgroup.
// Lane l (i = l % 32, h = l / 32) reads A[row i][8o+4h .. 8o+4h+3] and B[8o+4h+t][col i]
// (t = 0..3) and issues four v_mfma_f32_32x32x2_f32, so MFMA t multiplies the k pair
// (8o+t, 8o+4+t).  Any m, n, k and leading dimension works: rows and columns past the edge
// are clamped to the last valid one (their products land in accumulator entries that are
// never stored), only the last k mod 8 terms are predicated.
//
// The kernel is latency bound (a few waves per CU, each waiting on its own loads), so the
// loads of up to 64 k are all issued before the first MFMA that needs them: a 32x32x64
// problem of a batch waits for memory once instead of four times.
template <int OCT>
__device__ __forceinline__ void wave32_chunk(const float *a, const float *b, int64_t ldb, f32x16 &acc) {
    f32x4 av[OCT];
    float bv[OCT][4];
#pragma unroll
    for (int o = 0; o < OCT; ++o) {
        av[o] = *reinterpret_cast<const f32x4_a4 *>(a + 8 * o);   // one 16-byte load at any 4-byte alignment
    }
#pragma unroll
    for (int o = 0; o < OCT; ++o)
#pragma unroll
        for (int t = 0; t < 4; ++t) bv[o][t] = b[(int64_t)(8 * o + t) * ldb];
    __builtin_amdgcn_sched_barrier(0);   // left alone the scheduler sinks every load to just before its use
#pragma unroll
    for (int o = 0; o < OCT; ++o)
#pragma unroll
        for (int t = 0; t < 4; ++t) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[o][t], bv[o][t], acc, 0, 0, 0);
}

__device__ __forceinline__ void wave32_body(const GemmParams &p, const float *a_row, const float *b_col, int h,
                                            f32x16 &acc) {
    // a_row and b_col already point at this lane half's k offset 4h.
    int k0 = 0;
    for (; k0 + 64 <= p.k; k0 += 64) wave32_chunk<8>(a_row + k0, b_col + (int64_t)k0 * p.ldb, p.ldb, acc);
    if (k0 + 32 <= p.k) {
        wave32_chunk<4>(a_row + k0, b_col + (int64_t)k0 * p.ldb, p.ldb, acc);
        k0 += 32;
    }
    for (; k0 + 8 <= p.k; k0 += 8) wave32_chunk<1>(a_row + k0, b_col + (int64_t)k0 * p.ldb, p.ldb, acc);
    if (k0 < p.k) {
        const int left = p.k - k0 - 4 * h;   // terms of the last, partial octet that belong to this lane half
        float a[4], b[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            a[e] = e < left ? a_row[k0 + e] : 0.0f;
            b[e] = e < left ? b_col[(int64_t)(k0 + e) * p.ldb] : 0.0f;
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[t], b[t], acc, 0, 0, 0);
    }
}

__global__ void __launch_bounds__(256) sgemm_wave32_kernel(const GemmParams p) {
    const int lane = threadIdx.x & 63;
    const int li = lane & 31, h = lane >> 5;
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    const int64_t wid = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wid >= tiles * p.batch) return;   // whole wave leaves; the kernel has no barrier
    const int prob = (int)(wid / tiles);
    const int t_in = (int)(wid - (int64_t)prob * tiles);
    const int tm = t_in / p.tiles_n, tn = t_in - tm * p.tiles_n;

    const int col = tn * 32 + li;
    const int row_c = min(tm * 32 + li, p.m - 1), col_c = min(col, p.n - 1);
    const float *a_row = p.A + (int64_t)prob * p.strideA + (int64_t)row_c * p.lda + 4 * h;
    const float *b_col = p.B + (int64_t)prob * p.strideB + (int64_t)(4 * h) * p.ldb + col_c;

    f32x16 acc = (f32x16)(0.0f);
    wave32_body(p, a_row, b_col, h, acc);

    float *c = p.C + (int64_t)prob * p.strideC;
    if (col < p.n) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = tm * 32 + 8 * (v / 4) + 4 * h + (v % 4);
            if (r < p.m) c[(int64_t)r * p.ldc + col] = acc[v];
        }
    }
}

hipError_t launch_wave32(const GemmParams &p, hipStream_t s) {
    const int64_t waves = (int64_t)p.tiles_m * p.tiles_n * p.batch;
    const int64_t blocks = (waves + 3) / 4;
    hipLaunchKernelGGL(sgemm_wave32_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p);
    return hipGetLastError();
}

// The same with one wave per 16x16 tile and v_mfma_f32_16x16x4_f32: four times as many waves, each with a
// quarter of the loads and of the MFMA work, for problems too small to give every SIMD a 32x32 tile (a batch
// of 512 products of 32x32x64 has 512 such tiles for 1024 SIMDs).  Lane l (i = l % 16, q = l / 16) supplies
// A[row i][k = q] and B[k = q][col i] to the instruction and receives rows 4q .. 4q+3 of column i.  As above
// a lane reads four consecutive k of its row at once (16c+4q .. 16c+4q+3) and feeds element t to the t-th of
// four MFMAs, which therefore multiplies the k set {16c+t, 16c+4+t, 16c+8+t, 16c+12+t}.
template <int CH>
__device__ __forceinline__ void wave16_chunk(const float *a, const float *b, int64_t ldb, f32x4 &acc) {
    f32x4 av[CH];
    float bv[CH][4];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        av[c] = *reinterpret_cast<const f32x4_a4 *>(a + 16 * c);
    }
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
        for (int t = 0; t < 4; ++t) bv[c][t] = b[(int64_t)(16 * c + t) * ldb];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
        for (int t = 0; t < 4; ++t) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[c][t], bv[c][t], acc, 0, 0, 0);
}

__device__ __forceinline__ void wave16_body(const float *a_row, const float *b_col, int64_t ldb, int klen, int q,
                                            f32x4 &acc) {
    // a_row and b_col already point at the first k of the range plus this lane quarter's offset 4q.
    int k0 = 0;
    for (; k0 + 128 <= klen; k0 += 128) wave16_chunk<8>(a_row + k0, b_col + (int64_t)k0 * ldb, ldb, acc);
    if (k0 + 64 <= klen) {
        wave16_chunk<4>(a_row + k0, b_col + (int64_t)k0 * ldb, ldb, acc);
        k0 += 64;
    }
    if (k0 + 32 <= klen) {
        wave16_chunk<2>(a_row + k0, b_col + (int64_t)k0 * ldb, ldb, acc);
        k0 += 32;
    }
    if (k0 + 16 <= klen) {
        wave16_chunk<1>(a_row + k0, b_col + (int64_t)k0 * ldb, ldb, acc);
        k0 += 16;
    }
    if (k0 < klen) {
        const int left = klen - k0 - 4 * q;   // terms of the last, partial chunk that belong to this lane quarter
        float a[4], b[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            a[e] = e < left ? a_row[k0 + e] : 0.0f;
            b[e] = e < left ? b_col[(int64_t)(k0 + e) * ldb] : 0.0f;
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[t], b[t], acc, 0, 0, 0);
    }
}

__global__ void __launch_bounds__(256) sgemm_wave16_kernel(const GemmParams p) {
    const int lane = threadIdx.x & 63;
    const int li = lane & 15, q = lane >> 4;
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    const int64_t wid = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wid >= tiles * p.batch) return;   // whole wave leaves; the kernel has no barrier
    const int prob = (int)(wid / tiles);
    const int t_in = (int)(wid - (int64_t)prob * tiles);
    const int tm = t_in / p.tiles_n, tn = t_in - tm * p.tiles_n;

    const int col = tn * 16 + li;
    const int row_c = min(tm * 16 + li, p.m - 1), col_c = min(col, p.n - 1);
    const float *a_row = p.A + (int64_t)prob * p.strideA + (int64_t)row_c * p.lda + 4 * q;
    const float *b_col = p.B + (int64_t)prob * p.strideB + (int64_t)(4 * q) * p.ldb + col_c;

    f32x4 acc = (f32x4)(0.0f);
    wave16_body(a_row, b_col, p.ldb, p.k, q, acc);

    float *c = p.C + (int64_t)prob * p.strideC;
    if (col < p.n) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int r = tm * 16 + 4 * q + v;
            if (r < p.m) c[(int64_t)r * p.ldc + col] = acc[v];
        }
    }
}

hipError_t launch_wave16(const GemmParams &p, hipStream_t s) {
    const int64_t waves = (int64_t)p.tiles_m * p.tiles_n * p.batch;
    const int64_t blocks = (waves + 3) / 4;
    hipLaunchKernelGGL(sgemm_wave16_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p);
    return hipGetLastError();
}

// Wider tiles of the same kind: a wave owns CB = 2 or 4 blocks of 16x16 side by side, lane i the CB adjacent
// columns CB*i .. CB*i+CB-1 of the 16 x 16*CB tile, so that a B fragment for all its blocks is one 8- or 16-byte
// load, a row of C leaves as full 128-byte lines and the A fragment is shared by the blocks (a quarter to a half
// of the load instructions per product).  For aligned operands (16-byte rows of A and B, n a multiple of CB).
template <int CH, int CB>
__device__ __forceinline__ void wave16w_chunk(const float *a, const float *b, int64_t ldb, f32x4 (&acc)[CB]) {
    typedef typename vec_of<CB>::type bvec;
    f32x4 av[CH];
    bvec bv[CH][4];
#pragma unroll
    for (int c = 0; c < CH; ++c) av[c] = *reinterpret_cast<const f32x4_a4 *>(a + 16 * c);
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
        for (int t = 0; t < 4; ++t) bv[c][t] = *reinterpret_cast<const bvec *>(b + (int64_t)(16 * c + t) * ldb);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < CB; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[c][t], vec_get(bv[c][t], j), acc[j], 0, 0, 0);
}

template <int CB>
__global__ void __launch_bounds__(256) sgemm_wave16w_kernel(const GemmParams p) {
    typedef typename vec_of<CB>::type bvec;
    constexpr int CHMAX = CB == 2 ? 8 : 4;   // k per round trip: 128 or 64 (96 or 80 registers of operands)
    const int lane = threadIdx.x & 63;
    const int li = lane & 15, q = lane >> 4;
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    const int64_t wid = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wid >= tiles * p.batch) return;   // whole wave leaves; the kernel has no barrier
    const int prob = (int)(wid / tiles);
    const int t_in = (int)(wid - (int64_t)prob * tiles);
    const int tm = t_in / p.tiles_n, tn = t_in - tm * p.tiles_n;

    // n is a multiple of CB, so a lane's columns are all inside or all outside; those outside re-read the last
    // CB columns (never stored), rows likewise
    const int col = tn * 16 * CB + CB * li;
    const int row_c = min(tm * 16 + li, p.m - 1), col_c = min(col, p.n - CB);
    const float *a_row = p.A + (int64_t)prob * p.strideA + (int64_t)row_c * p.lda + 4 * q;
    const float *b_col = p.B + (int64_t)prob * p.strideB + (int64_t)(4 * q) * p.ldb + col_c;

    f32x4 acc[CB];
#pragma unroll
    for (int j = 0; j < CB; ++j) acc[j] = (f32x4)(0.0f);
    int k0 = 0;
    for (; k0 + 16 * CHMAX <= p.k; k0 += 16 * CHMAX)
        wave16w_chunk<CHMAX, CB>(a_row + k0, b_col + (int64_t)k0 * p.ldb, p.ldb, acc);
    if (CHMAX == 8 && k0 + 64 <= p.k) {
        wave16w_chunk<4, CB>(a_row + k0, b_col + (int64_t)k0 * p.ldb, p.ldb, acc);
        k0 += 64;
    }
    if (k0 + 32 <= p.k) {
        wave16w_chunk<2, CB>(a_row + k0, b_col + (int64_t)k0 * p.ldb, p.ldb, acc);
        k0 += 32;
    }
    if (k0 + 16 <= p.k) {
        wave16w_chunk<1, CB>(a_row + k0, b_col + (int64_t)k0 * p.ldb, p.ldb, acc);
        k0 += 16;
    }
    if (k0 < p.k) {
        const int left = p.k - k0 - 4 * q;   // terms of the last, partial chunk that belong to this lane quarter
        float a[4];
        bvec b[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            a[e] = e < left ? a_row[k0 + e] : 0.0f;
            if (e < left) b[e] = *reinterpret_cast<const bvec *>(b_col + (int64_t)(k0 + e) * p.ldb);
            else b[e] = (bvec)(0.0f);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < CB; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[t], vec_get(b[t], j), acc[j], 0, 0, 0);
    }

    float *c = p.C + (int64_t)prob * p.strideC;
    if (col < p.n) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int r = tm * 16 + 4 * q + v;
            if (r >= p.m) continue;
            bvec o;
#pragma unroll
            for (int j = 0; j < CB; ++j) o[j] = acc[j][v];
            store_result(c + (int64_t)r * p.ldc + col, o, false);   // one vector store at any 4-byte alignment
        }
    }
}

template <int CB>
hipError_t launch_wave16w(const GemmParams &p, hipStream_t s) {
    const int64_t waves = (int64_t)p.tiles_m * p.tiles_n * p.batch;
    const int64_t blocks = (waves + 3) / 4;
    hipLaunchKernelGGL(sgemm_wave16w_kernel<CB>, dim3((unsigned)blocks), dim3(256), 0, s, p);
    return hipGetLastError();
}
template hipError_t launch_wave16w<2>(const GemmParams &, hipStream_t);
template hipError_t launch_wave16w<4>(const GemmParams &, hipStream_t);

// A few tiles with a long K (256x256x1024 has 256 tiles of 16x16 for 1024 SIMDs): the four waves of a workgroup
// share one 16x16 tile, each multiplies a quarter of K (in whole 16-k steps), the four partial tiles meet in
// LDS and wave 0 adds them in wave order, so the result does not depend on timing.
__global__ void __launch_bounds__(256) sgemm_wave16k4_kernel(const GemmParams p) {
    __shared__ f32x4 part[4][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int li = lane & 15, q = lane >> 4;
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    const int64_t wid = blockIdx.x;        // one workgroup per tile: the grid is exactly tiles * batch
    const int prob = (int)(wid / tiles);
    const int t_in = (int)(wid - (int64_t)prob * tiles);
    const int tm = t_in / p.tiles_n, tn = t_in - tm * p.tiles_n;

    const int steps = (p.k + 15) / 16, per = (steps + 3) / 4;
    const int k_begin = min(w * per * 16, p.k), k_end = min((w + 1) * per * 16, p.k);

    const int col = tn * 16 + li;
    const int row_c = min(tm * 16 + li, p.m - 1), col_c = min(col, p.n - 1);
    const float *a_row = p.A + (int64_t)prob * p.strideA + (int64_t)row_c * p.lda + k_begin + 4 * q;
    const float *b_col = p.B + (int64_t)prob * p.strideB + (int64_t)(k_begin + 4 * q) * p.ldb + col_c;

    f32x4 acc = (f32x4)(0.0f);
    wave16_body(a_row, b_col, p.ldb, k_end - k_begin, q, acc);

    part[w][lane] = acc;
    __syncthreads();
    if (w != 0) return;
    f32x4 sum = part[0][lane];
#pragma unroll
    for (int s = 1; s < 4; ++s) sum += part[s][lane];

    float *c = p.C + (int64_t)prob * p.strideC;
    if (col < p.n) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int r = tm * 16 + 4 * q + v;
            if (r < p.m) c[(int64_t)r * p.ldc + col] = sum[v];
        }
    }
}

hipError_t launch_wave16k4(const GemmParams &p, hipStream_t s) {
    const int64_t blocks = (int64_t)p.tiles_m * p.tiles_n * p.batch;
    hipLaunchKernelGGL(sgemm_wave16k4_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p);
    return hipGetLastError();
}

// C[b][i][j] = sum over s = 0..splits-1 of ws[b][s][i][j], added in that fixed order, so
// the result does not depend on scheduling (no floating-point atomics anywhere).
__global__ void __launch_bounds__(256) splitk_reduce_kernel(const GemmParams p) {
    const int64_t mn = (int64_t)p.m * p.n;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p.flags & kFlagVecC) {
        const int64_t n4 = p.n / 4;
        const int64_t total = (int64_t)p.batch * p.m * n4;
        for (int64_t idx = first; idx < total; idx += stride) {
            const int64_t b = idx / (p.m * n4);
            const int64_t rem = idx - b * p.m * n4;
            const int64_t i = rem / n4, j = (rem - i * n4) * 4;
            const float *src = p.ws + b * p.splits * mn + i * p.n + j;
            f32x4 sum = *reinterpret_cast<const f32x4 *>(src);
            for (int s = 1; s < p.splits; ++s) sum += *reinterpret_cast<const f32x4 *>(src + s * mn);
            store_result(p.C + b * p.strideC + i * p.ldc + j, sum, false);   // rows of C need no 16-byte alignment
        }
    } else {
        const int64_t total = (int64_t)p.batch * mn;
        for (int64_t idx = first; idx < total; idx += stride) {
            const int64_t b = idx / mn;
            const int64_t rem = idx - b * mn;
            const int64_t i = rem / p.n, j = rem - i * p.n;
            const float *src = p.ws + b * p.splits * mn + rem;
            float sum = src[0];
            for (int s = 1; s < p.splits; ++s) sum += src[s * mn];
            p.C[b * p.strideC + i * p.ldc + j] = sum;
        }
    }
}

hipError_t launch_splitk_reduce(const GemmParams &p, hipStream_t s) {
    const int64_t items = (p.flags & kFlagVecC) ? (int64_t)p.batch * p.m * (p.n / 4) : (int64_t)p.batch * p.m * p.n;
    int64_t blocks = (items + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p);
    return hipGetLastError();
}

__global__ void __launch_bounds__(256) zero_fill_kernel(const GemmParams p) {
    const int64_t mn = (int64_t)p.m * p.n;
    const int64_t total = (int64_t)p.batch * mn;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        const int64_t b = idx / mn;
        const int64_t rem = idx - b * mn;
        const int64_t i = rem / p.n, j = rem - i * p.n;
        p.C[b * p.strideC + i * p.ldc + j] = 0.0f;
    }
}

hipError_t launch_zero_fill(const GemmParams &p, hipStream_t s) {
    const int64_t items = (int64_t)p.batch * p.m * p.n;
    int64_t blocks = (items + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p);
    return hipGetLastError();
}

// z = alpha * x + y (axpy of Sec. 5.2 of the paper): 12 bytes of HBM traffic per element and
// one FMA, so the only thing that matters is keeping many 16-byte loads in flight.  Each
// thread handles four consecutive floats per step (dwordx4 when the three pointers are
// 16-byte aligned); the tail and unaligned vectors take the scalar path.  In the paper's terms: n strip-mined into BLOCK x THREAD x VECTOR(4).
template <bool VEC, int NT>
__global__ void __launch_bounds__(256) saxpy_kernel(int64_t n, float alpha, const float *x, const float *y, float *z) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if constexpr (VEC) {
        const int64_t n4 = n >> 2;
        const f32x4 *x4 = reinterpret_cast<const f32x4 *>(x);
        const f32x4 *y4 = reinterpret_cast<const f32x4 *>(y);
        f32x4 *z4 = reinterpret_cast<f32x4 *>(z);
        for (int64_t i = tid; i < n4; i += stride) {
            const f32x4 a = (NT & 2) ? __builtin_nontemporal_load(&x4[i]) : x4[i];
            const f32x4 b = (NT & 2) ? __builtin_nontemporal_load(&y4[i]) : y4[i];
            f32x4 r;
#pragma unroll
            for (int e = 0; e < 4; ++e) r[e] = __builtin_fmaf(alpha, a[e], b[e]);
            if (NT & 1) __builtin_nontemporal_store(r, &z4[i]);
            else z4[i] = r;
        }
        for (int64_t i = (n4 << 2) + tid; i < n; i += stride) z[i] = __builtin_fmaf(alpha, x[i], y[i]);
    } else {
        for (int64_t i = tid; i < n; i += stride) z[i] = __builtin_fmaf(alpha, x[i], y[i]);
    }
}

// In-place use (z == y or z == x) is allowed (hence no __restrict__): a thread reads an element
// before it writes the same element and no other thread touches it.
hipError_t launch_saxpy(int64_t n, float alpha, const float *x, const float *y, float *z, hipStream_t s) {
    const bool vec = ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y) | reinterpret_cast<uintptr_t>(z)) & 15u) == 0;
    const int64_t items = vec ? (n + 3) / 4 : n;
    // One 16-byte item per thread and as many workgroups as that takes: measured fastest at
    // n = 2^26 (6.0 TB/s against 5.0-5.7 TB/s for looping grids of 4..64 workgroups per CU);
    // the grid-stride loop only matters beyond 2^31 workgroups.
    int64_t blocks = (items + 255) / 256;
    if (blocks > INT32_MAX) blocks = INT32_MAX;
    if (blocks < 1) blocks = 1;
    // Non-temporal hints (NT bit 0: stores, bit 1: loads), by the size of the three vectors against the
    // 256 MB Infinity Cache.  Measured GB/s (plain / stores / loads / both):  n = 2^22: 6095 / 7898 / 6395 /
    // 7116;  2^24: 7257 / 7154 / 6377 / 6812;  2^25: 5779 / 7194 / 6709 / 6643;  2^26: 5878 / 6019 / 7032 /
    // 6602;  2^27: 5754 / 5821 / 6058 / 6274;  2^28: 6021 / 6016 / 6239 / 6435;  2^29: 6006 / 6089 / 6237 / 6456.
    const int64_t bytes = 12 * n;
    const int nt = bytes <= (int64_t)512 << 20 ? 1 : (bytes <= (int64_t)1 << 30 ? 2 : 3);
    if (!vec) hipLaunchKernelGGL((saxpy_kernel<false, 0>), dim3((unsigned)blocks), dim3(256), 0, s, n, alpha, x, y, z);
    else if (nt == 1) hipLaunchKernelGGL((saxpy_kernel<true, 1>), dim3((unsigned)blocks), dim3(256), 0, s, n, alpha, x, y, z);
    else if (nt == 2) hipLaunchKernelGGL((saxpy_kernel<true, 2>), dim3((unsigned)blocks), dim3(256), 0, s, n, alpha, x, y, z);
    else hipLaunchKernelGGL((saxpy_kernel<true, 3>), dim3((unsigned)blocks), dim3(256), 0, s, n, alpha, x, y, z);
    return hipGetLastError();
}

// dst[r * ld + c] = src[r * rs + c * cs] for a rows x cols matrix with arbitrary positive element
// strides: the gather / transpose pass in front of the unit-stride kernels for the strided
// product of Sec. 5.2.  One workgroup copies a 64 x 64 tile; all 16 loads of a thread are issued
// before the first use so that a gather (every element in its own cache line) keeps
// 4096 lines in flight per workgroup.  ALONG_ROWS: source lanes run down a column (the
// source's unit-stride direction when rs < cs, e.g. a column-major operand) and the tile is
// turned through LDS (row pitch 65 floats: conflict-free both ways) so that the writes still run
// along a row of dst.
template <bool ALONG_ROWS>
__global__ void __launch_bounds__(256) pack_kernel(const float *__restrict__ src, int64_t rs, int64_t cs,
                                                   float *__restrict__ dst, int64_t ld, int rows, int cols, int tiles_c) {
    __shared__ float tile[ALONG_ROWS ? 64 : 1][65];
    const int r0 = (int)(blockIdx.x / (unsigned)tiles_c) * 64;
    const int c0 = (int)(blockIdx.x % (unsigned)tiles_c) * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    float v[16];
#pragma unroll
    for (int it = 0; it < 16; ++it) {
        const int slow = ty + 4 * it;
        const int r = r0 + (ALONG_ROWS ? tx : slow);
        const int c = c0 + (ALONG_ROWS ? slow : tx);
        v[it] = (r < rows && c < cols) ? src[(int64_t)r * rs + (int64_t)c * cs] : 0.0f;
    }
    if constexpr (ALONG_ROWS) {
#pragma unroll
        for (int it = 0; it < 16; ++it) tile[tx][ty + 4 * it] = v[it];
        __syncthreads();
#pragma unroll
        for (int it = 0; it < 16; ++it) v[it] = tile[ty + 4 * it][tx];
    }
#pragma unroll
    for (int it = 0; it < 16; ++it) {
        const int r = r0 + ty + 4 * it, c = c0 + tx;
        if (r < rows && c < cols) dst[(int64_t)r * ld + c] = v[it];
    }
}

// dst[r * ld + c] = src[r * rs + c] for r < rows, c < cols, and +0.0 on the rest of rows_out x ld (ld a multiple
// of 4, dst 16-byte aligned): the aligned, zero-padded copy of an operand whose base, leading dimension or
// extents keep the exact-fit kernels from using 16-byte loads.  A workgroup copies 1024 vectors of 16 bytes, a thread
// four of them: its sixteen 4-byte loads (the source has no alignment to speak of) are all issued before the first
// store.  (One or four vectors per thread: the same time, 1023^3 28.3 us in all; the launch is what the copy costs.)
struct PadCopy {
    const float *src;
    int64_t rs;
    int rows, cols;
    float *dst;
    int64_t ld;
    int rows_out;
};
constexpr int kPadCopyVecs = 4;                       // per thread
constexpr int kPadCopyBlock = 256 * kPadCopyVecs;     // per workgroup

__device__ __forceinline__ void pad_copy_block(const PadCopy &d, int64_t block) {
    const int64_t vecs = d.ld / 4;
    const int64_t total = (int64_t)d.rows_out * vecs;
    f32x4 v[kPadCopyVecs];
    int64_t at[kPadCopyVecs];
#pragma unroll
    for (int j = 0; j < kPadCopyVecs; ++j) {
        const int64_t idx = block * kPadCopyBlock + j * 256 + threadIdx.x;
        const int64_t r = idx / vecs;
        const int c = (int)(idx - r * vecs) * 4;
        at[j] = idx < total ? r * d.ld + c : -1;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[j][e] = (idx < total && r < d.rows && c + e < d.cols) ? d.src[r * d.rs + c + e] : 0.0f;
    }
#pragma unroll
    for (int j = 0; j < kPadCopyVecs; ++j)
        if (at[j] >= 0) *reinterpret_cast<f32x4 *>(d.dst + at[j]) = v[j];
}

__global__ void __launch_bounds__(256) pad_copy_kernel(const PadCopy d, int64_t blocks) {
    for (int64_t b = blockIdx.x; b < blocks; b += gridDim.x) pad_copy_block(d, b);
}

// Both operands in one launch (a launch costs as much as either copy of a mid-size product): the first blocks_a
// workgroups copy A, the others B.
__global__ void __launch_bounds__(256) pad_copy2_kernel(const PadCopy a, const PadCopy b, unsigned blocks_a) {
    if (blockIdx.x < blocks_a) pad_copy_block(a, blockIdx.x);
    else pad_copy_block(b, blockIdx.x - blocks_a);
}

static int64_t pad_copy_blocks(int64_t ld, int rows_out) { return ((int64_t)rows_out * (ld / 4) + kPadCopyBlock - 1) / kPadCopyBlock; }

hipError_t launch_pad_copy(const float *src, int64_t rs, int rows, int cols, float *dst, int64_t ld, int rows_out, hipStream_t s) {
    const int64_t blocks = pad_copy_blocks(ld, rows_out);
    if (blocks <= 0) return hipSuccess;
    const PadCopy d{src, rs, rows, cols, dst, ld, rows_out};
    hipLaunchKernelGGL(pad_copy_kernel, dim3((unsigned)std::min<int64_t>(blocks, INT32_MAX)), dim3(256), 0, s, d, blocks);
    return hipGetLastError();
}

hipError_t launch_pad_copy2(const float *src_a, int64_t rs_a, int rows_a, int cols_a, float *dst_a, int64_t ld_a, int rows_out_a,
                            const float *src_b, int64_t rs_b, int rows_b, int cols_b, float *dst_b, int64_t ld_b, int rows_out_b,
                            hipStream_t s) {
    const int64_t blocks_a = pad_copy_blocks(ld_a, rows_out_a), blocks_b = pad_copy_blocks(ld_b, rows_out_b);
    if (blocks_a <= 0 || blocks_b <= 0 || blocks_a + blocks_b > INT32_MAX) {     // (one of them empty, or too many for one grid)
        hipError_t e = launch_pad_copy(src_a, rs_a, rows_a, cols_a, dst_a, ld_a, rows_out_a, s);
        return e != hipSuccess ? e : launch_pad_copy(src_b, rs_b, rows_b, cols_b, dst_b, ld_b, rows_out_b, s);
    }
    const PadCopy a{src_a, rs_a, rows_a, cols_a, dst_a, ld_a, rows_out_a}, b{src_b, rs_b, rows_b, cols_b, dst_b, ld_b, rows_out_b};
    hipLaunchKernelGGL(pad_copy2_kernel, dim3((unsigned)(blocks_a + blocks_b)), dim3(256), 0, s, a, b, (unsigned)blocks_a);
    return hipGetLastError();
}

// The tuner's result check.  snapshot_rows_kernel copies every `step`-th row of every problem's C (rows 0, step,
// 2*step, ...) into a packed reference buffer; compare_rows_kernel later compares the same rows of C with that
// reference and leaves, per workgroup, the sums of (c - ref)^2 and of ref^2 and a count of non-finite values
// (doubles; added up on the host, so no atomics are involved).
__global__ void __launch_bounds__(256) snapshot_rows_kernel(const float *__restrict__ C, int64_t ldc, int64_t strideC, int batch,
                                                            int m, int n, int step, float *__restrict__ ref) {
    const int rows = (m + step - 1) / step;
    const int64_t total = (int64_t)batch * rows * n;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t b = idx / ((int64_t)rows * n);
        const int64_t rem = idx - b * rows * n;
        const int64_t r = rem / n, j = rem - r * n;
        ref[idx] = C[b * strideC + r * step * ldc + j];
    }
}

__global__ void __launch_bounds__(256) compare_rows_kernel(const float *__restrict__ C, int64_t ldc, int64_t strideC, int batch,
                                                           int m, int n, int step, const float *__restrict__ ref,
                                                           double *__restrict__ partial) {
    __shared__ double red[3][256];
    const int rows = (m + step - 1) / step;
    const int64_t total = (int64_t)batch * rows * n;
    double d2 = 0.0, r2 = 0.0, bad = 0.0;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t b = idx / ((int64_t)rows * n);
        const int64_t rem = idx - b * rows * n;
        const int64_t r = rem / n, j = rem - r * n;
        const float c = C[b * strideC + r * step * ldc + j], f = ref[idx];
        if (!(__builtin_fabsf(c) <= 3.4e38f) || !(__builtin_fabsf(f) <= 3.4e38f)) {
            bad += 1.0;
        } else {
            const double d = (double)c - (double)f;
            d2 += d * d;
            r2 += (double)f * (double)f;
        }
    }
    red[0][threadIdx.x] = d2;
    red[1][threadIdx.x] = r2;
    red[2][threadIdx.x] = bad;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w)
            for (int q = 0; q < 3; ++q) red[q][threadIdx.x] += red[q][threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0)
        for (int q = 0; q < 3; ++q) partial[3 * blockIdx.x + q] = red[q][0];
}

hipError_t launch_snapshot_rows(const float *C, int64_t ldc, int64_t strideC, int batch, int m, int n, int step, float *ref,
                                hipStream_t s) {
    hipLaunchKernelGGL(snapshot_rows_kernel, dim3(kCheckBlocks), dim3(256), 0, s, C, ldc, strideC, batch, m, n, step, ref);
    return hipGetLastError();
}

hipError_t launch_compare_rows(const float *C, int64_t ldc, int64_t strideC, int batch, int m, int n, int step, const float *ref,
                               double *partial, hipStream_t s) {
    hipLaunchKernelGGL(compare_rows_kernel, dim3(kCheckBlocks), dim3(256), 0, s, C, ldc, strideC, batch, m, n, step, ref, partial);
    return hipGetLastError();
}

hipError_t launch_pack(const float *src, int64_t rs, int64_t cs, float *dst, int64_t ld, int rows, int cols, hipStream_t s) {
    const int64_t tiles_r = ((int64_t)rows + 63) / 64, tiles_c = ((int64_t)cols + 63) / 64;
    if (rows <= 0 || cols <= 0) return hipSuccess;
    if (tiles_r * tiles_c > INT32_MAX) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(tiles_r * tiles_c));
    if (rs < cs) hipLaunchKernelGGL(pack_kernel<true>, grid, dim3(256), 0, s, src, rs, cs, dst, ld, rows, cols, (int)tiles_c);
    else hipLaunchKernelGGL(pack_kernel<false>, grid, dim3(256), 0, s, src, rs, cs, dst, ld, rows, cols, (int)tiles_c);
    return hipGetLastError();
}

}  // namespace tg

