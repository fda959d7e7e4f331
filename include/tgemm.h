/*
 * tgemm -- single-precision dense matrix multiplication for AMD MI355X (gfx950).
 *
 * The operation is "matmul" of Sec. 5.2 of the paper (arXiv 1904.03383): C = A.B with
 * A of size m x k and B of size k x n, i.e. C[i][j] = sum_{p<k} A[i][p] * B[p][j].
 * There is no alpha/beta and no transpose flag, exactly as in that problem statement;
 * C is overwritten and never read.  The batched entry point applies the same
 * definition independently to `batch` problems (benchmark workload; not in the paper).
 *
 * Layout.  Row-major with leading dimensions in ELEMENTS: A[i*lda + p], B[p*ldb + j],
 * C[i*ldc + j]; lda >= k, ldb >= n, ldc >= n.  Elements of C between n and ldc are
 * never written.  The paper stores matrices column-major (Sec. 5.2); a column-major
 * product C = A.B is obtained from this library by swapping the operands:
 * tg_sgemm(n, m, k, B, ldb, A, lda, C, ldc, stream).
 *
 * Pointers.  A, B, C and the workspace are DEVICE pointers owned by the caller; the
 * library never allocates, frees or keeps them (the workspace pointer is kept until
 * replaced).  C must not overlap A or B (not checked).  `stream` is a hipStream_t
 * passed as void* (NULL = the default stream).
 *
 * Execution.  Calls validate their arguments on the host, enqueue kernels on `stream`
 * and return without synchronising; C is valid once the stream has been synchronised.
 * tg_tune is the only blocking call.
 *
 * Errors.  Nothing is thrown across this boundary; every function returns a tg_status
 * (or a plain value where stated).  Argument errors are detected before any GPU call,
 * so they are reported even on a machine without a GPU.  tg_last_error() returns a
 * thread-local, human-readable description of the most recent failure on this thread.
 *
 * Accuracy.  fp32 multiply-add on the matrix cores, fp32 accumulation; for k > 1024 the
 * running sums are folded into a second accumulator every 1024 terms so that the
 * relative Frobenius error stays below 1e-6 at k = 4096 (measured 5.7e-7; 1.15e-6 without).
 * The first-level sums stay 1024 terms long however long k is; on normal(0,1) operands the error
 * measures 5.8e-7 at k = 16384, 5.9e-7 at k = 65536 and 6.6e-7 at k = 262144, the longest k tested
 * against the fp64 reference; the 1e-6 bar is stated for k <= 262144.
 */
#ifndef TGEMM_H
#define TGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TG_OK = 0,
    TG_ERR_INVALID_ARG = 1, /* null pointer with non-empty extent, negative size, ld or stride too small, overflow */
    TG_ERR_UNSUPPORTED = 2, /* current device is not gfx950, or size beyond 2^31-1 per dimension */
    TG_ERR_WORKSPACE = 3,   /* a forced configuration needs more workspace than was set */
    TG_ERR_HIP = 4,         /* a HIP runtime call failed; text in tg_last_error() */
    TG_ERR_INTERNAL = 5
} tg_status;

/*
 * C = A.B (Sec. 5.2 "matmul").  m, n, k >= 0.  m == 0 or n == 0: nothing is done.
 * k == 0: the m x n region of C is set to +0.0.
 */
tg_status tg_sgemm(int64_t m, int64_t n, int64_t k,
                   const float *A, int64_t lda,
                   const float *B, int64_t ldb,
                   float *C, int64_t ldc,
                   void *stream);

/*
 * `batch` independent products of the same shape (Sec. 5.2 definition per problem).
 * Problem b uses A + b*strideA, B + b*strideB, C + b*strideC (strides in elements).
 * "Packed contiguously" means lda = k, ldb = n, ldc = n, strideA = m*k, strideB = k*n,
 * strideC = m*n.  For batch > 1: strideC >= (m-1)*ldc + n (outputs must not overlap);
 * strideA and strideB may be any non-negative value (0 broadcasts one operand).
 */
tg_status tg_sgemm_batched(int64_t batch, int64_t m, int64_t n, int64_t k,
                           const float *A, int64_t lda, int64_t strideA,
                           const float *B, int64_t ldb, int64_t strideB,
                           float *C, int64_t ldc, int64_t strideC,
                           void *stream);

/*
 * C = A.B with arbitrary element strides on the operands:
 *     C[i*ldc + j] = sum_{p<k} A[i*rsa + p*csa] * B[p*rsb + j*csb].
 * Covers the paper's "strided matmul" (Sec. 5.2: matmul 1024^3 whose consecutive elements of
 * A sit 32 elements apart: csa = 32), and transposed / column-major operands ("transposed
 * layouts", Sec. 5.2): a column-major A with leading dimension lda is rsa = 1, csa = lda.
 * A column-major C is obtained by computing C^T = B^T.A^T: swap the operands and exchange
 * each one's two strides.  All strides are in elements and must be >= 1 (ldc >= n); the
 * operands may not overlap C.  With csa == csb == 1 this is tg_sgemm(lda = rsa, ldb = rsb).
 * Otherwise the operands are read as they lie wherever a kernel variant for their layout exists (k a
 * multiple of 32 and, for a plain B, n a multiple of 4): a transposed operand on the 16-byte grid (A with
 * rsa == 1, csa % 4 == 0, m % 4 == 0; B with rsb == 1, csb % 4 == 0; 16-byte aligned bases) is loaded along
 * its unit-stride axis ("_ta" / "_tb" in tg_last_config()) and costs the same as the plain product; any
 * other strides are gathered element by element straight into the kernel's staging memory, several K
 * tiles ahead ("_ga" / "_gb"): no workspace and no separate pass are involved.  An element-strided
 * operand costs a cache-line request per element and tile that uses it, so the paper's case (1024^3,
 * csa = 32: 128 MiB of lines behind a 4 MiB operand) runs at about 1.8 times the plain product's time.
 * A strided A with a plain B (k a multiple of 64) is taken by row-panel variants ("g16x..." / "g32x..."):
 * a workgroup owns 16 or 32 rows of A and 256 to 1024 columns of B, so an element is requested once per
 * 256 ... 1024 columns, by waves that do nothing else (the paper's 1024^3: 33 us; 4096 x 1024 x 1024 at
 * csa = 32: 122 us against 227 us on tiles); with a workspace for partial products they can also split K.
 * The other form: when a workspace of tg_strided_workspace_bytes(...) is set, each operand with a non-unit
 * stride that more than one tile row or column would fetch can first be gathered into a packed row-major
 * copy in the workspace (one pass, every element fetched once), and the unit-stride kernels multiply the
 * copies; tg_last_config() then ends in "+packA", "+packB" or "+packAB".  It is used for problems the
 * reading variants do not take (other k, a transposed operand off the 16-byte grid), and for
 * element-strided operands when the cost model puts the two passes ahead of the gather, which it does where
 * no variant gathers sparingly: a strided B fetched by many tile rows (1024^3 at csb = 32: 48 us against
 * 78 us), a strided A with a k that the row panels do not take.  Transposed operands on the
 * 16-byte grid are never packed.  Without room for the copies the reading variants are used wherever they
 * apply, and the predicated kernels gather element by element otherwise.
 */
tg_status tg_sgemm_strided(int64_t m, int64_t n, int64_t k,
                           const float *A, int64_t rsa, int64_t csa,
                           const float *B, int64_t rsb, int64_t csb,
                           float *C, int64_t ldc,
                           void *stream);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture, serving loops and
 * harnesses with a no-allocation rule) and therefore have no workspace to hand to tg_set_workspace:
 * the split-K form of tg_sgemm (same product, same arguments, same accuracy) with the partial products
 * kept in a device array of TG_STATIC_SCRATCH_BYTES that is part of the library's code object (every
 * GPU the library runs on holds it from the first load until the process ends).  The call allocates
 * and frees nothing, on the host side of the GPU runtime or through any library.
 * K is cut into two or more ranges (the count the cost model ranks first for this shape: split-K pays
 * for few output tiles with a long K, e.g. 256 x 256 x 4096), every range's product is written to the
 * array by one launch, and a second kernel adds them in range order (deterministic, no atomics) into C.
 * A configuration set by tg_force_config is used if it is a split (":s<n>", n >= 2) of an fp32 tile kernel.
 * Limits and errors (all detected before any launch): 2 * m * n * 4 bytes must not exceed
 * TG_STATIC_SCRATCH_BYTES, else TG_ERR_WORKSPACE; a problem that no split fits (K shorter than two K
 * tiles per range, or an output that already fills the chip) returns TG_ERR_UNSUPPORTED: use tg_sgemm.
 * Argument checks, m == 0 / n == 0 / k == 0 and tg_last_config() behave as for tg_sgemm.
 * Every entry of the part of the array a call uses is written before it is read, so nothing has to
 * start at zero and the last call's contents do no harm.  All calls on one GPU share that GPU's array:
 * two calls that overlap in time on one GPU (different streams or host threads) race.
 */
#define TG_STATIC_SCRATCH_BYTES (32u << 20)
tg_status tg_sgemm_splitk_static(int64_t m, int64_t n, int64_t k,
                                 const float *A, int64_t lda,
                                 const float *B, int64_t ldb,
                                 float *C, int64_t ldc,
                                 void *stream);

/*
 * z[i] = alpha * x[i] + y[i] for 0 <= i < n (Sec. 5.2 "axpy": z = alpha.x + y, the paper's
 * bandwidth-bound kernel, n = 2^26 there).  x, y, z are device pointers to n contiguous
 * floats; z may be the same pointer as y or x (in-place), partial overlap is undefined.
 * Each element is one fused multiply-add (a single rounding).  n == 0: nothing is done.
 * Errors: negative n, or a null pointer with n > 0 -> TG_ERR_INVALID_ARG.
 */
tg_status tg_saxpy(int64_t n, float alpha, const float *x, const float *y, float *z, void *stream);

/*
 * Host-side tile-configuration tuner (the counterpart of the decisions -- block/thread
 * mapping, tile sizes, unrolling, memory space -- that the paper's search fixes per
 * kernel and input size, Secs. 4 and 5.1; here a small fixed candidate set is timed).
 * Runs every candidate configuration that is valid for this problem on the caller's
 * buffers (`reps` timed launches each after a warm-up, reps <= 0 selects 5), remembers
 * the fastest for this (batch, m, n, k, alignment class) and leaves a valid product in C.
 * Candidates whose roofline lower bound already exceeds the best time seen are skipped; the leaders are
 * timed again with longer runs (launch-bound problems: as replays of a graph captured on a private
 * stream created for the duration of the call).  Must not be called while `stream` is being captured.
 * Blocking: synchronises `stream`.  tg_sgemm / tg_sgemm_batched never time anything;
 * without a tuned entry they use a static heuristic.
 * Whether a problem counts as launch-bound is decided from the cost model's device time of its first
 * candidate (under 12 us), not from a measured per-call time, so that a slow host or a profiler cannot
 * hide it (tg_tune_is_launch_bound answers the same question without a GPU).
 * Result check: the first candidate's product is kept (every step-th row of C, in the static array of
 * tg_sgemm_splitk_static, so tg_tune must not overlap such calls on the same GPU) and every other
 * candidate's product is compared with it before that candidate may lead: two results that meet the
 * accuracy bar differ by at most 2e-6 in the relative Frobenius norm; 4e-6 is allowed, non-finite values
 * are not.  If any candidate fails, nothing is cached and the call returns TG_ERR_INTERNAL naming the
 * configurations (tg_last_error()).
 * The operands are passed (the benchmark definition's tg_tune(batch, m, n, k, stream) has none) because
 * candidates are timed on the caller's real buffers, with their real leading dimensions and alignment,
 * and the library allocates nothing.
 * Two environment variables exist for tests of the tuner itself: TG_TUNE_TEST_HOST_DELAY_US=<us> makes
 * the host wait that long after every timed launch (a slow host), TG_TUNE_TEST_SPOIL_REFERENCE=1
 * overwrites one entry of the kept reference (so that every candidate fails the check).
 */
tg_status tg_tune(int64_t batch, int64_t m, int64_t n, int64_t k,
                  const float *A, int64_t lda, int64_t strideA,
                  const float *B, int64_t ldb, int64_t strideB,
                  float *C, int64_t ldc, int64_t strideC,
                  void *stream, int reps);

/*
 * Workspace (device memory, caller-owned, 16-byte aligned; the benchmark definition keeps allocation with
 * the caller: PyTorch owns device memory): split-K partial products (also those of
 * the K-split tail launch of a tail split), packed copies of strided operands, aligned zero-padded copies
 * of unit-stride operands that are off the 16-byte grid or have k or n not a multiple of 4 (made for
 * single products with m, n >= 256 and m * n * k >= 4.2e8 when there is room: m x k and k x n floats, each rounded up to
 * multiples of 4 (k to a multiple of 32 when both are copied and k >= 1000); tg_last_config() then ends in "+alignA", "+alignB" or "+alignAB"; without room the
 * predicated kernels take such operands as they are, as do the one-wave-per-tile kernels that smaller products
 * run on; C is never copied: its rows may start anywhere), and the piece images of the "c" kernels.
 * Configurations that need it are considered only while a workspace of
 * sufficient size is set (tg_workspace_bytes(...) covers every candidate); otherwise one that needs none is used.
 * Pass (NULL, 0) to remove it.  Calls that use the workspace concurrently on different
 * streams race; give concurrent streams separate processes or no workspace.
 */
tg_status tg_set_workspace(void *dev_ptr, size_t bytes);

/* Largest workspace any candidate for this problem can need in the current math mode (bytes). 0 on invalid sizes. */
size_t tg_workspace_bytes(int64_t batch, int64_t m, int64_t n, int64_t k);

/*
 * Workspace that lets tg_sgemm_strided pack its non-unit-stride operands (csa != 1: m x k floats,
 * csb != 1: k x n floats, rows padded to a multiple of 4) and still consider every split-K
 * candidate: the packed copies plus tg_workspace_bytes(1, m, n, k).  0 on invalid sizes.
 */
size_t tg_strided_workspace_bytes(int64_t m, int64_t n, int64_t k, int64_t csa, int64_t csb);

/*
 * Configuration control (the paper notes that an expert can set decisions by hand before the search,
 * Sec. 6.1; this is that hook).  A spec is "<kernel>[:s<splitK>][:g<group>][:o<cap>][:p<n>][:t<rows>x<splits>]", e.g.
 * "t128x128x16_w64x64:s1:g8" (split-K factor; tile rows per ordering group; cap on
 * workgroups per CU; persistent launch with n workgroups per CU that loop over the tiles;
 * tail split: the last <rows> tile rows of every problem go out as a second launch with split-K
 * <splits>, which fills the chip once more for a fraction of a round when the tile count is a little
 * above a multiple of what the chip holds; needs the workspace like any split-K);
 * kernel names are listed by tg_kernel_name.
 * tg_force_config(spec) makes every later call use that configuration when it is valid
 * for the problem (otherwise the call fails with TG_ERR_INVALID_ARG, or TG_ERR_WORKSPACE
 * for split-K without room); tg_force_config(NULL) returns to tuned/heuristic choice.
 * The environment variable TG_FORCE_CONFIG is read once, at the first call, the same way.
 */
tg_status tg_force_config(const char *spec);

/*
 * Arithmetic the automatic choice (heuristic and tg_tune) may use.  Results are fp32 in either mode and
 * both modes meet the same accuracy bounds on finite inputs.
 *   TG_MATH_FP32_MFMA (default): every product and sum on the fp32 matrix instructions.
 *   TG_MATH_BF16_PIECES: kernels whose names start with "e" are candidates too.  They cut each operand
 *     element into three bf16 pieces (8 bits of the significand each: exact), form a product from 6 ("_x6":
 *     all terms down to 2^-23 of the product, i.e. below one fp32 rounding) or all 9 ("_x9") piece products
 *     on the bf16 matrix instructions, which multiply 16 times as fast, and sum in fp32 with the leading
 *     and the small terms in separate accumulators.  Measured relative Frobenius error at k = 4096:
 *     3.9e-7 (fp32 mode: 5.7e-7); integer-valued inputs stay bit exact.  What differs from fp32
 *     arithmetic: an infinite input gives NaN where fp32 gives infinity; and the underflow cliff sits
 *     higher: a product a*b below about 2^-100 in magnitude (say both operands scaled below 2^-50) has
 *     low-order piece products under 2^-126, which are lost, so where such products dominate an element
 *     its accuracy degrades towards that of the leading pieces (fp32 arithmetic keeps full relative
 *     accuracy down to 2^-126).  Products up to the overflow threshold behave as in fp32.
 *     Kernels whose names start with "c" do the same arithmetic with the operands cut ahead: two passes
 *     write the pieces of A and B into the workspace (6 bytes per element of A and B, every tile padded
 *     with zeros; tg_workspace_bytes includes it while this mode is on) and the product streams them in.
 *     They take any m, n, k and any alignment of A, B and C;
 *     "e" kernels need 16-byte aligned operands and k a multiple of 32.
 * A forced configuration (tg_force_config) may name an "e" or "c" kernel in either mode.  Tuned entries are kept
 * per mode.  Returns TG_ERR_INVALID_ARG for an unknown mode.
 */
#define TG_MATH_FP32_MFMA 0
#define TG_MATH_BF16_PIECES 1
tg_status tg_set_math(int mode);
int tg_get_math(void);

/* Writes the spec that a call with these sizes (packed, aligned operands) would use now. */
tg_status tg_get_config(int64_t batch, int64_t m, int64_t n, int64_t k, char *buf, size_t len);

/*
 * The search space of tg_tune, for inspection (Sec. 5.1 of the paper: candidates are ranked by a
 * cost model and cut by a lower bound on their run time before they are timed).
 * tg_num_candidates: how many configurations tg_tune would consider for these sizes (packed,
 * aligned operands, the workspace as it is now); -1 with tg_last_error set when the sizes are
 * invalid.  tg_candidate: the idx-th of them in the order they are timed (cheapest by the cost
 * model first): its spec into spec[len] (host buffer), and, where the pointers are not NULL, the
 * lower bound on its run time and the cost model's estimate, both in microseconds.  The bound
 * holds for any kernel with that tiling on this chip: the MFMA peak, one wave's share on its one
 * SIMD, whole rounds of workgroups over the 256 CUs, and one pass of the operands over HBM; a
 * candidate whose bound is not below the best time measured so far is skipped without a launch.
 * Neither call touches the GPU.
 */
int tg_num_candidates(int64_t batch, int64_t m, int64_t n, int64_t k);
tg_status tg_candidate(int64_t batch, int64_t m, int64_t n, int64_t k, int idx, char *spec, size_t len,
                       double *lower_bound_us, double *model_us);

/*
 * 1 if tg_tune would time the leading candidates of this problem (packed, aligned operands) as graph replays
 * because it is launch-bound by the cost model, 0 if not, -1 with tg_last_error set for invalid sizes.
 * Does not touch the GPU.
 */
int tg_tune_is_launch_bound(int64_t batch, int64_t m, int64_t n, int64_t k);

/* Spec the most recent successful tg_sgemm/tg_sgemm_batched/tg_tune call on this thread ran (or "" ). */
const char *tg_last_config(void);

/* Number of compiled kernel variants, and the name of variant idx (0 <= idx < count). */
int tg_num_kernels(void);
tg_status tg_kernel_name(int idx, char *buf, size_t len);

/*
 * Tuned-entry cache (the only persistent state; the counterpart of the paper's remark, Sec. 3.4, that a
 * candidate's decision vector is easy to serialise): plain text, one entry per line.  Loading merges into
 * the live cache.  If the environment variable TG_TUNE_CACHE names a file, it is loaded at the first call
 * that chooses a configuration (when it exists), and every successful tg_tune rewrites the file the variable
 * names at that time with the whole live cache.
 */
tg_status tg_load_tune_cache(const char *path);
tg_status tg_save_tune_cache(const char *path);
void tg_clear_tune_cache(void);

const char *tg_status_string(tg_status s);
const char *tg_last_error(void);
/* 100 * major + minor.  The debug flavour of the library (libtgemm_poison.so, compiled with TG_POISON_LDS: every
 * kernel overwrites an LDS stage with NaN once it has given it up and before it is refilled, so that a read of
 * stale staging memory shows as NaN in C instead of as plausible numbers) reports 1000000 more. */
int tg_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TGEMM_H */
