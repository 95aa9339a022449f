/*
 * atk.h -- C ABI of libatk: generalized two-stage approximate Top-K on AMD MI355X (gfx950).
 *
 * The method (arXiv 2506.04165, Section 6.1): every row of length N is split into B buckets,
 * bucket i holding the positions n with n mod B == i (Step 1); stage 1 keeps the K' greatest
 * elements of every bucket (Step 2); stage 2 returns the K greatest of the B*K' survivors in
 * descending order (Steps 3-4).  K' = 1 is the original algorithm of Section 5.
 *
 * Ordering.  The paper leaves ties open.  This library fixes one total order everywhere:
 * element a precedes element b when value(a) > value(b), or the values compare equal (so
 * -0.0 == +0.0) and index(a) < index(b).  Every result is therefore unique and can be compared
 * bit for bit.  Precondition: the input holds no NaN (behaviour with NaN is unspecified but
 * memory safe).
 *
 * Conventions for every entry point below
 *   - all data pointers are DEVICE pointers to memory owned by the caller; the library never
 *     allocates, frees or keeps device memory, and never synchronises: work is enqueued on
 *     `stream` (a hipStream_t passed as void*, NULL = the default stream) and the call returns;
 *   - `values` is row-major [rows, N] with `row_stride` elements between consecutive rows
 *     (row_stride >= N); outputs are dense row-major;
 *   - dtype: ATK_F32 = IEEE binary32; ATK_BF16 = bfloat16 and ATK_F16 = IEEE binary16 (compared
 *     after exact widening to binary32); ATK_I32 / ATK_U32 = 32-bit integers compared as such
 *     (the compute-type promotion of Section 6.3's listing); output values have the input
 *     dtype and are the stored bits of the selected elements; indices are int32 positions
 *     inside the row;
 *   - the return value is an atk_status; arguments are validated on the host before anything
 *     is launched, so every error below can be provoked without a GPU;
 *   - rows == 0 is legal and does nothing.
 *
 * Developer options (launch geometry, for experiments and tests; results never depend on them):
 * see atk_set_option.  No product call reads the environment.
 */
#ifndef ATK_H_
#define ATK_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element types of `values`.  Floating types are compared after the exact widening to binary32
 * (-0.0 equals +0.0, NaN excluded); signed and unsigned 32-bit integers are compared as such --
 * the compute-type promotion of Section 6.3's listing.  Outputs carry the stored words. */
typedef enum atk_dtype { ATK_F32 = 0, ATK_BF16 = 1, ATK_F16 = 2, ATK_I32 = 3, ATK_U32 = 4 } atk_dtype;

typedef enum atk_status {
    ATK_OK = 0,
    /* null pointer, rows < 0, N <= 0, N > 2^31 - 65536 (ATK_MAX_N), row_stride < N, B < 1, B does not divide N
     * (Section 6.3 requires equal buckets), K' < 1, K' > K (abstract: 1 <= K' <= K), K' > N/B,
     * K > B*K', K > N, K < 1, misaligned pointer */
    ATK_INVALID_ARG = 1,
    /* legal by the definition but outside what the kernels cover (see atk_approx_topk) */
    ATK_UNSUPPORTED = 2,
    ATK_WORKSPACE_TOO_SMALL = 3,
    /* a HIP call failed; atk_last_hip_error() holds its text */
    ATK_HIP_ERROR = 4
} atk_status;

/* Longest supported row, in elements. */
#define ATK_MAX_N 2147418112LL

typedef enum atk_op { ATK_OP_APPROX_TOPK = 0, ATK_OP_TOPK = 1, ATK_OP_STAGE1 = 2 } atk_op;

/*
 * Two-stage approximate Top-K (Section 6.1 Steps 1-4; stage 1 as Section 6.3, stage 2 exact).
 *   values     [rows, N] device, dtype as given
 *   K, Kprime, B   the paper's K, K' and number of buckets; 1 <= K' <= min(K, N/B), B | N,
 *                  K <= B*K'
 *   out_vals   [rows, K] device, input dtype, descending in the total order
 *   out_idx    [rows, K] device, int32
 *   workspace  device scratch of at least atk_workspace_bytes(ATK_OP_APPROX_TOPK, ...) bytes, or
 *              NULL when that is 0 (it is 0 whenever stage 2 runs fused in the stage-1 launch,
 *              i.e. when the B*K' survivors of a row fit in LDS and the rows are enough to fill
 *              the chip; otherwise survivors, or per-bucket keys of rows that several
 *              workgroups share, go through this buffer and a second launch finishes.  A
 *              buffer that is too small for the shared-row routes only switches them off)
 *              More than 16384 survivors per row (any B): stage 1 writes them to the workspace,
 *              rows cut along the bucket axis over several workgroups, and a second launch
 *              runs stage 2 on them (the unfused implementation of the paper's appendix).
 * ATK_UNSUPPORTED: K' > 32 unless K' == K (then the exact kernel runs); K > 8192 on the exact and
 * unfused routes; B > 2^24.
 */
int atk_approx_topk(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride,
                    int K, int Kprime, int B, void* out_vals, int32_t* out_idx,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * The mirrored problem, min-K: the K smallest elements of every row, smallest first, found by the
 * same two stages (stage 1 keeps the K' smallest of every bucket; Section 6.1 with the order
 * reversed).  Total order: element a precedes element b when value(a) < value(b), or the values
 * compare equal and index(a) < index(b).  Arguments, workspace, routes, limits and status codes
 * as atk_approx_topk / atk_topk (atk_workspace_bytes and atk_describe_plan answer for both).
 * The kernels are the same: every loaded value passes through the order-reversing map of its
 * type (sign flip for floating types, complement for integers) and results pass back through it.
 */
int atk_approx_mink(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride,
                    int K, int Kprime, int B, void* out_vals, int32_t* out_idx,
                    void* workspace, size_t workspace_bytes, void* stream);
int atk_mink(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride, int K,
             void* out_vals, int32_t* out_idx, void* workspace, size_t workspace_bytes, void* stream);

/*
 * atk_approx_topk for callers that cannot allocate device memory or hand over a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments
 * minus the workspace, same results.  Where atk_approx_topk would use a workspace (few-row
 * routes, survivors beyond LDS) this entry uses an array of ATK_NOALLOC_SCRATCH_BYTES that is part
 * of the library's code object (each GPU the library runs on holds its copy until the process
 * ends); it calls no allocating routine.  Problems whose survivors need more than that
 * (rows * B * K' * (element size + 4) bytes when B*K' > 16384, or 8 bytes per survivor, a lane's
 * share padded to a power of two, where the second launch ranks sorted runs; atk_workspace_bytes
 * gives the figure) are refused with ATK_WORKSPACE_TOO_SMALL; the few-row routes simply fall back to the single fused launch.
 * Nothing in the array has to start at zero (every word read was written by the same call), so
 * nothing is cleared.  All calls on one GPU share the array: calls that may overlap on one GPU
 * (different streams, other host threads) race on it -- serialise them, or use atk_approx_topk
 * with workspaces of their own.
 */
#define ATK_NOALLOC_SCRATCH_BYTES (16u << 20)
int atk_approx_topk_noalloc(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride,
                            int K, int Kprime, int B, void* out_vals, int32_t* out_idx, void* stream);

/*
 * Exact Top-K of every row under the same total order (the comparison system of Section 7; also
 * what the method reduces to at K' = K or B = 1).  Arguments as above.  ATK_UNSUPPORTED: K > 8192.
 *
 * workspace: optional device memory, 8-byte aligned.  With atk_workspace_bytes(ATK_OP_TOPK, ...)
 * bytes (0 where it does not apply: short rows, K > 1024) rows that are long against K are
 * done by the two-stage kernels at a (B, K' = 4) chosen by the library, followed by a kernel that
 * certifies each row exact (no bucket contributes K' elements to the result) or repairs it from
 * the buckets in doubt: one pass over the input at the approximate method's speed, the result is
 * the exact Top-K bit for bit.  K < 8: the two-stage kernels with K' = K, exact by construction
 * (the workspace then is what atk_approx_topk takes for those parameters: only few, long rows
 * need one, and without it the single fused launch runs).  Otherwise, and without a workspace
 * (null, or too small), a radix-selection kernel runs, which needs none.  Workspace contents need
 * not be initialised and are not preserved.  atk_describe_topk_plan says which of these a call takes.
 */
int atk_topk(const void* values, int dtype, int64_t rows, int64_t N, int64_t row_stride, int K,
             void* out_vals, int32_t* out_idx, void* workspace, size_t workspace_bytes,
             void* stream);

/*
 * Stage 1 alone (Section 6.1 Steps 1-2): the survivors, in the physical layout of Section 6.3:
 *   surv_vals  [rows, K', B] device, input dtype: plane k holds every bucket's k-th greatest
 *   surv_idx   [rows, K', B] device, int32
 * This is the first launch of the unfused path and the hook for testing stage 1 on its own.
 */
int atk_approx_topk_stage1(const void* values, int dtype, int64_t rows, int64_t N,
                           int64_t row_stride, int Kprime, int B, void* surv_vals,
                           int32_t* surv_idx, void* stream);

/* Scratch bytes the given operation needs (0 when it runs without); SIZE_MAX on illegal
 * arguments.  Host only. */
size_t atk_workspace_bytes(int op, int dtype, int64_t rows, int64_t N, int K, int Kprime, int B);

/*
 * Expected recall of the method under uniformly random placement of the Top-K (Theorem 1):
 *   1 - (B/K) * sum_{r=K'+1}^{min(K,N/B)} (r-K') C(K,r) C(N-K,N/B-r) / C(N,N/B).
 * Host only, double precision via log-gamma; returns a negative value on illegal arguments.
 */
double atk_expected_recall(int64_t N, int64_t B, int64_t K, int64_t Kprime);

/*
 * Parameter selection for a recall target (Section 6.3, appendix "Algorithm Parameter
 * Selection"): among the configurations with K' in [1, max_kprime], B a divisor of N and a
 * multiple of bucket_multiple, K' <= N/B and K <= B*K', whose expected recall (Theorem 1,
 * closed form, no Monte Carlo) is at least recall_target, the one with the fewest stage-1
 * survivors B*K' (the size of stage 2's input); on ties the smaller K'.  If none qualifies the
 * exact Top-K is returned as K' = K, B = 1.  Suggested ceilings on MI355X, where stage 1 stays
 * memory-bound: max_kprime 4 for fp32, 8 for bf16; bucket_multiple 64 (one wavefront).
 * Host only.  expected_recall_out may be NULL.
 */
int atk_select_params(int64_t N, int K, double recall_target, int max_kprime, int bucket_multiple,
                      int* Kprime_out, int* B_out, double* expected_recall_out);

/*
 * The (K', B) that atk_approx_topk_recall uses for this problem, among the configurations that
 * atk_approx_topk runs for these arguments with K' <= 4 (32-bit elements) or K' <= 8 (16-bit
 * ones) and B a multiple of 64 whose expected recall (Theorem 1) reaches the target: the shortest
 * lists for which some B keeps the survivors B*K' within a sixteenth of the row (between 512 and
 * 4096; 1024 for 16-bit rows of at most 65536 elements), with the smallest sufficient power of
 * two as B, doubled up to 1024 while the budget allows (else the smallest sufficient divisor of N) -- on this chip the list length is what
 * stage 1 pays for; when nothing fits that budget, atk_select_params' choice (the fewest
 * survivors, Section 6.3) under the same ceilings.  K' = K, B = 1 means the exact Top-K (nothing
 * approximate reaches the target); ATK_UNSUPPORTED if that is out of range too (K > 8192).
 * Host only; the last answer is cached per thread.  expected_recall_out may be NULL.
 */
int atk_recall_params(int dtype, int64_t rows, int64_t N, int K, double recall_target, int* Kprime_out,
                      int* B_out, double* expected_recall_out);

/*
 * atk_approx_topk with K' and B chosen by atk_recall_params: the paper's
 * approx_top_k(array, K, recall_target) interface (Section 6.3).  The chosen values are reported
 * through Kprime_used / B_used (may be NULL).  Size the workspace with atk_workspace_bytes for
 * the values atk_recall_params returns.
 */
int atk_approx_topk_recall(const void* values, int dtype, int64_t rows, int64_t N,
                           int64_t row_stride, int K, double recall_target, void* out_vals,
                           int32_t* out_idx, void* workspace, size_t workspace_bytes,
                           void* stream, int* Kprime_used, int* B_used);

/*
 * The same for the mirrored problem (atk_approx_mink with K' and B chosen by atk_recall_params;
 * Theorem 1 does not depend on which end of the order is asked for).
 */
int atk_approx_mink_recall(const void* values, int dtype, int64_t rows, int64_t N,
                           int64_t row_stride, int K, double recall_target, void* out_vals,
                           int32_t* out_idx, void* workspace, size_t workspace_bytes,
                           void* stream, int* Kprime_used, int* B_used);

/*
 * One-line description of how atk_topk / atk_mink run the given problem when handed the workspace
 * atk_workspace_bytes(ATK_OP_TOPK, ...) asks for: "certified B=... K'=... workspace=..." or
 * "radix threads=...".  Host only; for logs and tests.
 */
int atk_describe_topk_plan(int dtype, int64_t rows, int64_t N, int K, char* buf, size_t buflen);

/*
 * Writes a one-line description of how atk_approx_topk would run the given problem (kernel
 * variant, lanes per row, workgroup shape, LDS and workspace bytes) into buf.  Host only; for
 * logs and tests.  Returns the status atk_approx_topk would return for these arguments.
 */
int atk_describe_plan(int dtype, int64_t rows, int64_t N, int K, int Kprime, int B, char* buf,
                      size_t buflen);

/*
 * Maximum inner-product search with the matrix product fused into stage 1 (Section 7.3; appendix
 * "Matmul-fused implementation"): the rows whose approximate Top-K is wanted are the scores
 *   score[r][n] = sum_d queries[r][d] * database[n][d],   r < Q, n < N,
 * formed on the matrix cores with binary32 accumulation and consumed by the K'-list update of
 * Section 6.1 Steps 1-2 (bucket of score n = n mod B) without ever being stored; Steps 3-4 follow
 * in a second launch.  Same order and tie rule as atk_approx_topk on the score row.
 *   queries    device, [Q, D] bf16 or fp16, vectors contiguous, 16-byte aligned
 *   database   device, [N, D] same type, vectors contiguous, 16-byte aligned (vector-major, not the
 *              [D, N] operand of the paper's listing)
 *   dtype      ATK_BF16 or ATK_F16 (others: ATK_UNSUPPORTED);  D one of 64, 128, 256;  B a multiple of 32
 *              dividing N;  1 <= K' <= min(K, N/B, 4);  K <= B*K' <= 16384
 *   out_vals   device, [Q, K] binary32 scores, greatest first; a zero score is +0.0
 *   out_idx    device, [Q, K] int32 database positions
 *   workspace  device, at least atk_mips_workspace_bytes(...) bytes, 8-byte aligned; always
 *              needed (partial lists); caller-owned, may be reused after the stream reaches
 *              the end of this call
 * Precondition: finite inputs (no NaN score).  A score differs from the exactly rounded inner
 * product by the rounding of a binary32 accumulation of D products; results that hinge on
 * scores closer than that are decided by the computed scores.
 * Returns ATK_OK, ATK_INVALID_ARG, ATK_UNSUPPORTED, ATK_WORKSPACE_TOO_SMALL or ATK_HIP_ERROR;
 * asynchronous on `stream`; Q == 0 is a legal no-op.
 */
int atk_mips_approx_topk(const void* queries, const void* database, int dtype, int64_t Q, int64_t N,
                         int64_t D, int K, int Kprime, int B, float* out_vals, int32_t* out_idx,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * Fusion-aware parameter choice for atk_mips_approx_topk (named as open work in the paper's
 * conclusion): in the fused kernel every score pays about 5K'-2 vector operations (Section 6.3)
 * whatever B is, so the choice is the smallest K' <= 4 for which some legal B (a multiple of 32
 * dividing N, K <= B*K' <= 16384, K' <= N/B) reaches recall_target by Theorem 1, and for that K'
 * the smallest such B.  ATK_UNSUPPORTED when no legal configuration reaches the target.
 * Host only.  expected_recall_out may be NULL.
 */
int atk_mips_select_params(int64_t N, int K, double recall_target, int* Kprime_out, int* B_out,
                           double* expected_recall_out);

/*
 * atk_mips_approx_topk with K' and B chosen by atk_mips_select_params(N, K, recall_target); the
 * values used are reported through Kprime_used / B_used (may be NULL).  Size the workspace with
 * atk_mips_workspace_bytes for the values atk_mips_select_params returns.
 */
int atk_mips_approx_topk_recall(const void* queries, const void* database, int dtype, int64_t Q,
                                int64_t N, int64_t D, int K, double recall_target, float* out_vals,
                                int32_t* out_idx, void* workspace, size_t workspace_bytes,
                                void* stream, int* Kprime_used, int* B_used);

/* Workspace bytes atk_mips_approx_topk needs; SIZE_MAX on illegal or unsupported arguments.
 * Host only. */
size_t atk_mips_workspace_bytes(int dtype, int64_t Q, int64_t N, int64_t D, int K, int Kprime, int B);

/* Launch plan of atk_mips_approx_topk as text (tile shape, grid, segments).  Host only. */
int atk_mips_describe_plan(int dtype, int64_t Q, int64_t N, int64_t D, int K, int Kprime, int B,
                           char* buf, size_t buflen);

/*
 * Vector-ALU throughput probe (appendix "Estimating peak VPU throughput" redone for MI355X; the
 * measurement behind the ridge point of Section 2.3 that bounds K').  Streams n_words int32
 * words and applies `ops` dependent operations to each:
 *   kind 0  out[i] = y_ops where (x, y) -> (y, x + y) is applied `ops` times to (x[i], y[i])
 *   kind 1  out[i] = x[i] squared `ops` times                       (y is ignored, may be NULL)
 * with wrap-around int32 arithmetic.  x, y, out: device pointers to n_words words.
 */
int atk_valu_probe(int kind, const void* x, const void* y, void* out, size_t n_words, int ops,
                   void* stream);

/*
 * Read-only streaming probe: the memory bandwidth this chip delivers to a kernel that only reads
 * (the beta of Section 2.3's runtime model, measured rather than taken from the datasheet), as
 * the ceiling the streaming kernels are compared with.  Reads `bytes` bytes at `data` (device,
 * 16-byte aligned, a multiple of 16, below 512 GiB) once, with the loads the stage-1 kernel uses, in
 * ATK_READ_PROBE_WORDS contiguous pieces, and xors the exclusive-or of the 32-bit words of piece i
 * into checksum[i] (device, ATK_READ_PROBE_WORDS 32-bit words, which the caller sets to zero
 * beforehand; their exclusive-or is that of the whole buffer).  Asynchronous on `stream`.
 */
#define ATK_READ_PROBE_WORDS 256
int atk_read_probe(const void* data, size_t bytes, void* checksum, void* stream);

/*
 * Developer options: launch-geometry switches for experiments and tests.  Results never depend on
 * them.  Process-wide; change them only while no call is in flight.  value < 0 restores the
 * default.  Initial values may be given in the environment (read once, at the first call that
 * plans a launch): ATK_LANES_PER_ROW, ATK_SEGMENTS, ATK_SLAB, ATK_RANK_FINISH, ATK_SLAB_WIDTH,
 * ATK_SLAB_OWNERS, ATK_RANK_WGS, ATK_DEFER, ATK_NO_PACKED=1, ATK_NO_SUBWAVE=1,
 * ATK_BATCH_MIN_KP, ATK_MIPS_SEGMENTS, ATK_UNFUSED, ATK_CHUNKED, ATK_ONEPASS.
 *   "lanes_per_row"  0 = planner's choice, else a power of two <= 1024: lanes that share one row
 *   "segments"       n > 0 forces n row segments on the split route
 *   "slab"           0 never / 1 planner's choice / 2 whenever possible: slabs of 32 buckets per
 *                    workgroup (few-row route)
 *   "rank_finish"    0: stage 2 of the few-row route always runs in one workgroup per row (default 1:
 *                    spread over several workgroups that place every survivor by counting the
 *                    survivors above it, where the planner finds that applicable)
 *   "slab_width"     0 = planner's choice, else a power of two >= 32: buckets per workgroup on the
 *                    few-row route when stage 2 is spread over several workgroups
 *   "rank_wgs"       most workgroups of that second launch when survivors go through the workspace
 *   "defer"          value+step lists: 0 every element updates its list at once, 1 (default) elements
 *                    that beat a list's least entry are set aside and inserted later where the
 *                    planner finds that it pays (long buckets), 2 wherever the lists allow it
 *   "slab_owners"    0 = planner's choice, else a power of two <= 32: most lanes that share a bucket
 *                    on the few-row route
 *   "packed"         0 switches the packed-key variants (16-bit rows) off
 *   "subwave"        0 switches the several-rows-per-wavefront variants off
 *   "batch_min_kp"   list length from which sorted batches are used (default 16)
 *   "mips_segments"  n > 0 forces n segments of the database walk in atk_mips_approx_topk
 *   "unfused"        1 sends the survivors of every call through the workspace (two launches)
 *   "chunked"        1: when survivors go through the workspace, every bucket chunk's workgroup runs
 *                    stage 2 on its own survivors and passes on only its K greatest
 *   "onepass"        exact kernel: 0 always two passes over a row, 1 (default) one pass with a rising
 *                    threshold on long rows, 2 on every row it can handle
 *   "certified"      0: atk_topk / atk_mink never go through the two-stage kernels and the
 *                    certificate kernel, whatever workspace they are given
 *   "reg_rows"       0: the radix-selection kernel never keeps a short row in registers
 *   "exact_threads"  0 = planner's choice, else a power of two in [64, 1024]: lanes of a workgroup
 *                    of the radix-selection kernel
 * Returns ATK_INVALID_ARG for an unknown name or an unusable value.  Host only.
 */
int atk_set_option(const char* name, int value);

/* Static, human-readable name of a status code. */
const char* atk_status_string(int status);

/* Text of the most recent HIP error seen by this thread's calls ("" if none). */
const char* atk_last_hip_error(void);

/* Library version, e.g. "0.1.0". */
const char* atk_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ATK_H_ */
