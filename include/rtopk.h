/*
 * rtopk.h -- C ABI of the MI355X (gfx950) row-wise top-k library.
 *
 * Operation (RTop-K paper, arXiv 2409.00822, Section 3: problem statement and Algorithms 1 and 2):
 * for each of N rows of M fp32 values, select k (value, column) pairs by a binary search over a
 * threshold between the row's minimum and maximum, counting the elements at or above each midpoint.
 *
 * Common conventions for every entry point below
 * ----------------------------------------------
 *  - All data pointers are DEVICE pointers owned by the caller.  The library never allocates,
 *    frees, copies to the host or synchronises.  Work is enqueued on `stream` (a hipStream_t passed
 *    as void*; NULL means the default stream) and the call returns at once.
 *  - `in`       : [N][M] fp32, dense, row-major, row stride M, read-only, 4-byte aligned.
 *                 Rows are processed fastest when `in` is 16-byte aligned and M is a multiple of 4;
 *                 other shapes take a scalar-load path with the same results.
 *  - `out_vals` : [N][k] fp32, row-major.  out_vals[r][j] is the bit pattern of in[r][out_idx[r][j]].
 *  - `out_idx`  : [N][k] column indices, 0-based, strictly ascending within a row
 *                 (int32_t, or uint8_t in the *_u8 variants, which require M <= 256: this is the
 *                 compressed row -- k values plus k byte-wide columns -- that MaxK-GNN's sparse
 *                 aggregation consumes, Section 1 / Fig. 1).
 *  - Input and output buffers must not overlap (checked on the host: RTOPK_ERR_OVERLAP).
 *  - Ties are broken towards the lower column index.
 *  - Preconditions that are NOT checked: every input is finite and |v| < FLT_MAX / 2 (so that
 *    min + max cannot overflow).  With NaN or infinities the selection is unspecified, but the call
 *    still terminates and writes only inside the output buffers.
 *  - Return value: RTOPK_OK (0) when the work was enqueued (or N == 0: nothing to do), otherwise a
 *    negative RTOPK_ERR_* code; every argument check happens on the host before any launch, and on
 *    error nothing was enqueued.  A pending error of the caller's own earlier HIP calls is neither
 *    reported nor cleared.  Faults of the asynchronous work surface at the caller's next
 *    synchronisation, as with any HIP launch.
 *  - Limits: 1 <= k <= M <= rtopk_max_m() = 2^24 for fp32 rows with int32 columns (65536 for rows stored
 *    in 16 bits, the dense form and the backward edge; 256 in the *_u8 variants); 0 <= N; N * M and
 *    N * k must fit in int64_t.  Rows wider than 8192 columns are handled by one workgroup per row, and
 *    then N < 2^31.  Rows wider than 65536 columns are not held on chip but streamed from memory: once
 *    when k is up to about a thousand and the winners are not crowded into one sixteenth of the row,
 *    otherwise once for the minimum and maximum, once per eight search steps and, for k in the
 *    thousands, once more to write the result; a launch of fewer such rows than twice the number of
 *    compute units leaves some of them idle.
 */
#ifndef RTOPK_H_
#define RTOPK_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  RTOPK_OK = 0,
  RTOPK_ERR_NULL_POINTER = -1,  /* a data pointer is NULL while N > 0 */
  RTOPK_ERR_BAD_SHAPE = -2,     /* N < 0, M < 1, k < 1 or k > M */
  RTOPK_ERR_BAD_MAX_ITER = -3,  /* max_iter < 0 */
  RTOPK_ERR_M_TOO_LARGE = -4,   /* M > rtopk_max_m(); M > 65536 for 16-bit rows, dense form, backward edge; M > 256 for *_u8 */
  RTOPK_ERR_MISALIGNED = -5,    /* a pointer is not aligned to its element size */
  RTOPK_ERR_LAUNCH = -6,        /* the HIP runtime refused the launch */
  RTOPK_ERR_BAD_EPSILON = -7,   /* eps_rel is negative or NaN */
  RTOPK_ERR_OVERLAP = -8        /* the input shares bytes with an output, or two outputs with each other */
};

/*
 * Early-stopping selection: Algorithm 2 (Section 3.1), taken literally.
 *   lo = min(row), hi = max(row); repeat max_iter times: thres = (lo + hi) * 0.5f in fp32,
 *   cnt = #{v >= thres}, cnt < k ? hi = thres : lo = thres; emit the first k columns with v >= lo.
 * max_iter == 0 is legal and returns the first k columns.  The result is bit-identical to a scalar
 * fp32 evaluation of those steps.  Each step halves hi - lo, so after at most ~300 steps on finite fp32
 * input the rounded midpoint equals lo or hi and further steps change nothing: a max_iter above 512 is
 * run as 512, with bit-identical output (a caller may pass INT32_MAX for "no early stop").
 */
int rtopk_rowwise(const float* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, float* out_vals,
                  int32_t* out_idx, void* stream);

/*
 * Exact selection: Algorithm 1 with epsilon = 0, which Section 3.1 identifies with exact top-k.
 * The search runs until an iteration counts exactly k elements, or until no fp32 value lies strictly
 * between lo and hi; then everything >= hi is taken and the lowest columns of [lo, hi) fill up to k.
 * The result equals the plain definition of top-k with the lower column winning ties.
 */
int rtopk_rowwise_exact(const float* in, int64_t N, int32_t M, int32_t k, float* out_vals, int32_t* out_idx,
                        void* stream);

/* The same two operations writing uint8_t columns (MaxK compressed row layout); require M <= 256. */
int rtopk_rowwise_u8(const float* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, float* out_vals,
                     uint8_t* out_idx, void* stream);
int rtopk_rowwise_exact_u8(const float* in, int64_t N, int32_t M, int32_t k, float* out_vals, uint8_t* out_idx,
                           void* stream);

/*
 * Precision-bounded selection: Algorithm 1 with epsilon = eps_rel * |max(row)| (Section 3.1: epsilon
 * bounds how wide the band of undecided elements around the k-th value may stay, and with it the
 * number of steps; Appendix B, Fig. 7 sweeps it).
 * The search ends when a step counts exactly k, when hi - lo <= epsilon, or when no fp32 value lies
 * strictly between lo and hi.  Everything >= hi is then taken, and the lowest columns of [lo, hi) fill
 * up to k, so every selected value is >= (k-th largest) - epsilon and every rejected one is
 * < (k-th largest) + epsilon.  eps_rel == 0 gives exactly rtopk_rowwise_exact's output.
 *   eps_rel   : >= 0 (negative or NaN: RTOPK_ERR_BAD_EPSILON).
 *   out_iters : optional (may be NULL) device int32_t[N]; receives the exit iteration of each row's
 *               loop as Tables 1 and 5 count it: the number of midpoints evaluated when one of them
 *               counted exactly k, one more than that when the loop ended through its guard.
 */
int rtopk_rowwise_eps(const float* in, int64_t N, int32_t M, int32_t k, float eps_rel, float* out_vals,
                      int32_t* out_idx, int32_t* out_iters, void* stream);

/*
 * The k SMALLEST values per row (Section 3 states the row-wise problem for either end of the order and
 * develops the largest case only).  Defined as the two
 * operations above applied to the negated row, with the original values written out: Algorithm 2's
 * thresholds are midpoints of the negated minimum and maximum, counts are of v <= -thres.  Ties go
 * to the lower column; columns ascend; int32 columns.
 */
int rtopk_rowwise_smallest(const float* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, float* out_vals,
                           int32_t* out_idx, void* stream);
int rtopk_rowwise_exact_smallest(const float* in, int64_t N, int32_t M, int32_t k, float* out_vals, int32_t* out_idx,
                                 void* stream);

/*
 * Rows stored in 16 bits: IEEE half (_f16) or bfloat16 (_bf16), passed as raw uint16_t bit patterns.
 * The paper's method is defined in fp32 (Section 3.1); here each row is widened exactly to fp32 as
 * it is loaded and Algorithm 2 / Algorithm 1 (epsilon = 0) run on the widened row, with fp32
 * midpoints.  `in` is [N][M] and `out_vals` is [N][k], both 16-bit and 2-byte aligned (fastest when
 * `in` is 16-byte aligned and M is a multiple of 8); out_vals[r][j] is the bit pattern of
 * in[r][out_idx[r][j]].  Everything else is as for rtopk_rowwise / rtopk_rowwise_exact.
 */
int rtopk_rowwise_f16(const uint16_t* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, uint16_t* out_vals,
                      int32_t* out_idx, void* stream);
int rtopk_rowwise_exact_f16(const uint16_t* in, int64_t N, int32_t M, int32_t k, uint16_t* out_vals, int32_t* out_idx,
                            void* stream);
int rtopk_rowwise_bf16(const uint16_t* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, uint16_t* out_vals,
                       int32_t* out_idx, void* stream);
int rtopk_rowwise_exact_bf16(const uint16_t* in, int64_t N, int32_t M, int32_t k, uint16_t* out_vals,
                             int32_t* out_idx, void* stream);

/*
 * The MaxK non-linearity in dense form (Section 1 and Fig. 1: MaxK-GNN applies row-wise top-k to the
 * feature matrix before aggregation; Section 4.3 measures it inside MaxK-GNN training):
 *   out[r][c] = in[r][c] if column c is one of the k columns selected for row r, +0.0f otherwise.
 * The selected columns are exactly those of rtopk_rowwise_exact (max_iter < 0) or of
 * rtopk_rowwise with that max_iter (max_iter >= 0).  `in` and `out` are [N][M] fp32, dense,
 * row-major, 4-byte aligned (fastest when both are 16-byte aligned and M is a multiple of 4), and must
 * not overlap (RTOPK_ERR_OVERLAP).  One launch; the row is read once and written once, nothing else
 * touches memory.
 */
int rtopk_maxk_dense(const float* in, int64_t N, int32_t M, int32_t k, int32_t max_iter, float* out, void* stream);

/*
 * Backward edge of the MaxK non-linearity (Section 1 and Fig. 1: the row-wise top-k is the non-linearity
 * of a MaxK-GNN layer; Section 4.3 measures it inside MaxK-GNN training).  Forward, a row keeps its k
 * selected entries and every other entry becomes zero, so the derivative with respect to the row is
 * that 0/1 mask, and with the columns the forward pass saved the backward step is data movement:
 *
 *   rtopk_maxk_backward        : grad_in[r][c] = grad_vals[r][j] where c == idx[r][j], 0.0f elsewhere
 *                                (the gradient of the k kept values, scattered into the dense row);
 *   rtopk_maxk_backward_gather : grad_vals[r][j] = grad_out[r][idx[r][j]]
 *                                (the entries of a dense gradient row that flow back through the k kept values).
 *
 *   idx       : [N][k] columns as written by rtopk_rowwise* (int32_t, or uint8_t in the *_u8 variants,
 *               which require M <= 256), read-only.  Columns of a row must be distinct (any order); a
 *               column outside [0, M) is ignored by the scatter and yields 0.0f in the gather, so no
 *               index value can make the kernels touch memory outside the buffers.
 *   grad_vals : [N][k] fp32, row-major (input of the scatter, output of the gather).
 *   grad_in / grad_out : [N][M] fp32, dense, row-major (fastest when 16-byte aligned and M % 4 == 0).
 * All pointers are device pointers, 4-byte aligned (uint8 columns: any alignment); the dense array must
 * not overlap the others, and the gather's output must not overlap idx (RTOPK_ERR_OVERLAP).  One
 * launch per call; every byte of the inputs is read once and every byte of the output written once.
 */
int rtopk_maxk_backward(const float* grad_vals, const int32_t* idx, int64_t N, int32_t M, int32_t k, float* grad_in,
                        void* stream);
int rtopk_maxk_backward_u8(const float* grad_vals, const uint8_t* idx, int64_t N, int32_t M, int32_t k, float* grad_in,
                           void* stream);
int rtopk_maxk_backward_gather(const float* grad_out, const int32_t* idx, int64_t N, int32_t M, int32_t k,
                               float* grad_vals, void* stream);
int rtopk_maxk_backward_gather_u8(const float* grad_out, const uint8_t* idx, int64_t N, int32_t M, int32_t k,
                                  float* grad_vals, void* stream);

/* Human-readable text for a status code (static storage, never NULL). */
const char* rtopk_status_string(int status);

/* Library version, major * 10000 + minor * 100 + patch. */
int rtopk_version(void);

/* Largest supported row width M (fp32 rows, int32 columns). */
int rtopk_max_m(void);

#ifdef __cplusplus
}
#endif

#endif /* RTOPK_H_ */
