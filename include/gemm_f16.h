/*
 * gemm_f16.h -- C ABI of the MI355X (gfx950) f16 GEMM library.
 *
 * The operation is the one the paper's Evaluation section states and its
 * listing "Naive affine matmul" spells out: C = A B + C with all three
 * matrices row-major, A and B in IEEE binary16, no alpha/beta and no
 * transposes:
 *
 *     C[i][j] <- C[i][j] + sum_{k=0}^{K-1} A[i][k] * B[k][j]
 *
 * in the paper's two precisions: "mixed precision" (section Mixed Precision
 * Performance: f16 inputs, products accumulated in f32, C in f32) and "half
 * precision" (section Half Precision Performance: A, B and C all f16).
 *
 * Conventions common to every entry point
 *   - A, B, C are DEVICE pointers (memory of the current HIP device) owned by
 *     the caller.  A and B are only read; C is read once and written once.
 *     C must not overlap A or B.  The library allocates nothing and keeps no
 *     state between calls except the benchmarking override below (and what it
 *     has learnt once about the device: compute units, XCDs, clock rate).
 *   - lda, ldb, ldc are row pitches in ELEMENTS (lda >= K, ldb >= N,
 *     ldc >= N).  Elements between the row length and the pitch are never
 *     read for A and B beyond what an aligned 16-byte fetch inside a row's
 *     own K (resp. N) extent touches, and are never read or written for C.
 *   - Any M, N, K >= 0 up to 2^31-1 is accepted (row pitches up to 2^31-1 as
 *     well).  A problem with M == 0 or N == 0 does nothing; K == 0 leaves C
 *     unchanged.  Pointers of any 2-byte (A, B, f16 C) / 4-byte (f32 C)
 *     alignment are accepted; the fastest kernels are used when A and B are
 *     16-byte aligned with lda, ldb multiples of 8, K, N multiples of 8 and
 *     all three pitches at most 2^22 elements (beyond that a slower kernel
 *     with 64-bit addressing throughout runs).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     The call only enqueues work: it never synchronises the device, and the
 *     result is complete when the stream reaches the end of that work.
 *   - Return value: GEMM_F16_OK (0) or a negative code below.  Arguments are
 *     checked on the host before anything is enqueued; on error nothing is
 *     launched and C is untouched.  Nothing throws.
 */
#ifndef GEMM_F16_H
#define GEMM_F16_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    GEMM_F16_OK = 0,
    GEMM_F16_ERR_SIZE = -1,    /* a dimension is negative or above 2^31-1 */
    GEMM_F16_ERR_PITCH = -2,   /* lda < K, ldb < N or ldc < N (or above 2^31-1) */
    GEMM_F16_ERR_NULL = -3,    /* a needed pointer is NULL */
    GEMM_F16_ERR_LAUNCH = -4,  /* the HIP runtime refused the launch */
    GEMM_F16_ERR_CONFIG = -5,  /* unknown configuration id / bad query argument */
    GEMM_F16_ERR_ALIGN = -6,   /* C is not aligned to its element size, or A/B to 2 bytes */
    GEMM_F16_ERR_WORKSPACE = -7 /* gemm_f16_f16acc_static_workspace: more scratch memory needed than the library holds */
};

/*
 * Mixed-precision mode (paper, section Mixed Precision Performance).
 * A: M x K f16, B: K x N f16, C: M x N f32, all row-major device memory.
 * Every product a*b is formed exactly and summed in f32 on the matrix units.
 * C is read once and written once per element, outside the k loop (the paper
 * hoists the C load and store out of it: section Generating WMMA Ops and
 * More).  Where the old value of C enters the sum is the kernel's choice: the
 * large-tile kernels sum the K products starting from zero and add C last
 * (sum + C, one more f32 rounding at the end), the small-tile and any-shape
 * kernels start the accumulators from C (C + sum), and the long-k kernel adds
 * C to the running sum while its first few dozen k steps are being summed
 * ((partial sum + C) + rest; on edge tiles it adds C last).  The summation order over
 * k is the kernel's own as well; results are bit-exact wherever every partial
 * sum is exactly representable, and within the f32 rounding bound otherwise.
 *
 * Skinny problems (at most half as many 128 x 128 tiles as compute units, K >=
 * 2048, M*N small) run with the k loop cut into parts: C is not read, every
 * part adds its sum to the C in memory with hardware f32 atomic additions
 * (C0 + part + part + ...; a part that is exactly zero adds nothing, so a C
 * that gets no contribution keeps its bits).  Their order is not fixed, so that two runs may
 * differ in the last bits (never where the sums are exact), and C must lie in
 * ordinary device memory (hipMalloc: memory on which the device's
 * floating-point atomics work).  gemm_f16_query_config reports such a plan by
 * a grid that is a multiple of the tile count.  The fused form below and the
 * half-precision mode never run this way.
 */
int gemm_f16_f32acc(int64_t M, int64_t N, int64_t K,
                    const void* A, int64_t lda,
                    const void* B, int64_t ldb,
                    float* C, int64_t ldc,
                    void* stream);

/*
 * Half-precision mode (paper, section Half Precision Performance): A, B and C
 * are all f16.  gfx950 has no matrix instruction that accumulates in f16, so
 * C is widened exactly to f32, all K products are accumulated in f32 exactly
 * as in gemm_f16_f32acc, and the result is rounded to f16 ONCE, to nearest
 * even, when it is stored (values beyond the f16 range become infinities).
 * This is at least as accurate as accumulating in f16.
 */
int gemm_f16_f16acc(int64_t M, int64_t N, int64_t K,
                    const void* A, int64_t lda,
                    const void* B, int64_t ldb,
                    void* C, int64_t ldc,
                    void* stream);

/*
 * The same two operations with a fused epilogue: a per-column bias and an
 * optional ReLU applied to each result before its single store (the paper's
 * Background section, subsection Tensor Cores, names bias addition as the
 * fusion that needs the thread-data mapping of the accumulators, and its
 * Conclusion names fusion as the goal; with MFMA the mapping is documented,
 * so the epilogue is a few instructions in the store path):
 *
 *     C[i][j] <- act( C[i][j] + sum_k A[i][k] * B[k][j] + bias[j] )
 *
 * bias: N elements of C's type (f32 resp. f16) in device memory, any element
 * alignment, or NULL for no bias.  act: GEMM_F16_ACT_NONE or
 * GEMM_F16_ACT_RELU (x < 0 ? 0 : x, so NaN and -0 pass through); any other
 * value returns GEMM_F16_ERR_CONFIG.  In f32 the sum, C and the bias are added
 * in that order; in the f16 mode all three are widened exactly, added in f32
 * and rounded once.  K == 0 applies the epilogue to C alone; M == 0 or N == 0
 * does nothing.  Everything else as for the plain entry points.
 */
enum { GEMM_F16_ACT_NONE = 0, GEMM_F16_ACT_RELU = 1 };
int gemm_f16_f32acc_bias_act(int64_t M, int64_t N, int64_t K,
                             const void* A, int64_t lda,
                             const void* B, int64_t ldb,
                             float* C, int64_t ldc,
                             const float* bias, int act,
                             void* stream);
int gemm_f16_f16acc_bias_act(int64_t M, int64_t N, int64_t K,
                             const void* A, int64_t lda,
                             const void* B, int64_t ldb,
                             void* C, int64_t ldc,
                             const void* bias, int act,
                             void* stream);

/*
 * The half-precision mode for callers that can lend scratch memory (paper,
 * section Half Precision Performance; same result as gemm_f16_f16acc to the
 * bound of the mode).  Skinny problems -- few 128 x 128 tiles, a long k loop:
 * the shapes gemm_f16_f32acc cuts along k -- are bound by how fast one compute
 * unit per tile can stream the larger operand.  With a workspace of M*N
 * floats the k loop is cut into parts here too: the workspace is zeroed, the
 * parts add their f32 sums to it atomically, and a last pass stores
 * round(C + workspace) to C, the mode's one rounding (three launches on the
 * caller's stream; (16,8192,8192): 29 us against 49 unsplit, (128,128,8192):
 * 15 against 49; problems of more than 2^20 results run unsplit).
 * gemm_f16_f16acc_workspace_bytes returns the bytes that make a difference
 * for a problem (0: it would run as gemm_f16_f16acc anyway; sizes only, for
 * 16-byte aligned operands with dense rows).  workspace: device memory,
 * 16-byte aligned (else GEMM_F16_ERR_ALIGN), owned by the caller, used only
 * between the call and the completion of its work on the stream, contents
 * undefined afterwards; NULL or too small: the call runs unsplit.  Two calls
 * may share a workspace only if they are ordered on one stream.
 */
int64_t gemm_f16_f16acc_workspace_bytes(int64_t M, int64_t N, int64_t K);
int gemm_f16_f16acc_workspace(int64_t M, int64_t N, int64_t K,
                              const void* A, int64_t lda,
                              const void* B, int64_t ldb,
                              void* C, int64_t ldc,
                              void* workspace, int64_t workspace_bytes,
                              void* stream);

/*
 * gemm_f16_f16acc_workspace for callers that cannot allocate device memory and
 * have none to lend: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  The scratch memory is the library's own,
 * a fixed array of 2^20 floats (4 MB) in the library's device image on every
 * GPU it runs on, held until the process ends; the call allocates and frees
 * nothing and records no memset (the array is cleared by a small kernel).  A
 * problem whose split plan needs more than the array holds is rejected with
 * GEMM_F16_ERR_WORKSPACE (as the selector stands no plan does); problems that
 * run unsplit do not touch the array.  Every call on a GPU uses that GPU's one
 * array: calls that can overlap on one GPU (two streams, two threads) race
 * and must be ordered by the caller; gemm_f16_f16acc has no such restriction.
 * The array's address is looked up at the first call on a device (not a
 * stream operation): make that call outside a graph capture.
 */
int gemm_f16_f16acc_static_workspace(int64_t M, int64_t N, int64_t K,
                                     const void* A, int64_t lda,
                                     const void* B, int64_t ldb,
                                     void* C, int64_t ldc,
                                     void* stream);

/* Static, human-readable text for a return code. Never NULL. */
const char* gemm_strerror(int code);

/*
 * Configuration ids index one table: the product library (libgemm_f16.so) holds
 * the kernels the selector can pick; a second build of the same sources
 * (libgemm_f16_ladder.so) appends comparison kernels and ablation rows behind
 * them, which are only ever run by forcing their id.
 *
 * Tile configuration report (the paper picks the best of several thread-block
 * and warp tile combinations per problem size: Evaluation section).  When the
 * tile count of the largest tile does not fill the last round of workgroups
 * on the device, a call may run as two launches on the caller's stream: whole
 * rounds of the largest tile on the first rows of C, another configuration on
 * the rest.
 */
typedef struct gemm_f16_config {
    int32_t id;          /* index into the library's configuration table */
    int32_t block_m;     /* workgroup tile rows */
    int32_t block_n;     /* workgroup tile columns */
    int32_t block_k;     /* k extent staged in LDS per main-loop step */
    int32_t waves;       /* 64-lane wavefronts per workgroup */
    int32_t wave_m;      /* wavefront tile rows */
    int32_t wave_n;      /* wavefront tile columns */
    int32_t lds_bytes;   /* LDS bytes per workgroup */
    int64_t grid;        /* workgroups launched for the queried problem (both launches of a split) */
    int32_t split_rows;  /* 0, or: configuration `id` computes the first split_rows rows of C ... */
    int32_t id2;         /* ... and configuration id2 the remaining rows in a second launch (-1: none) */
    char name[48];       /* short label of configuration `id`, NUL-terminated */
} gemm_f16_config;

/*
 * Report the configuration the library would use for this call, without
 * launching anything.  c_is_f16 selects the mode (0: gemm_f16_f32acc,
 * 1: gemm_f16_f16acc).  Pointers are only inspected for alignment and may be
 * any value with the alignment of the real buffers.  `out` is host memory.
 */
int gemm_f16_query_config(int c_is_f16, int64_t M, int64_t N, int64_t K,
                          const void* A, int64_t lda, const void* B, int64_t ldb,
                          const void* C, int64_t ldc, gemm_f16_config* out);

/* Number of entries in the configuration table, and a description of entry
 * `id` (grid is reported as 0). */
int gemm_f16_num_configs(void);
int gemm_f16_describe_config(int id, gemm_f16_config* out);

/*
 * Benchmarking aid: force configuration `id` for every later call of this
 * process (id < 0 restores automatic selection).  A forced configuration whose
 * alignment or pitch requirements the call does not meet is ignored for that
 * call.  The launch forms made for several tiles per compute unit (names
 * ending in _chain and _stag) run the plain 256 x 256 tiling on problems with
 * too few tiles for them (and _stag on devices other than 256 compute units);
 * with a k tail (K not a multiple of 64) a forced _chain still runs chained,
 * through its k-tail instantiation, which the selector itself does not pick.
 * Not thread-safe against concurrent GEMM calls.
 */
int gemm_f16_force_config(int id);

#ifdef __cplusplus
}
#endif
#endif /* GEMM_F16_H */
