/*
 * fnn.h -- C ABI of libfnn: fast reciprocal nearest-neighbour matching between two dense
 * per-pixel descriptor maps on one AMD Instinct MI355X (gfx950).
 *
 * The three operations are the matching stage of the Speedy MASt3R paper (arXiv 2503.10017):
 *
 *   fnn_nearest       one-directional search: for every query pixel the candidate pixel with
 *                     the best score.  This is the search of Algorithm 1 / Algorithm 2
 *                     ("FastNN-Lite", section 3.4.3) with the mixed-precision rule of
 *                     Algorithm 3 ("HybridCast", section 3.4.4): descriptors may be rounded
 *                     to a 16-bit format, products are accumulated and the best candidate
 *                     is selected in fp32.
 *   fnn_reciprocal    the FastNN iteration (section 3.2.5, "FastNN Algorithm", steps 1-4):
 *                     seeds in image 1, ping-pong searches, seeds leave when they return to
 *                     where they were, the result is the set of reciprocal matches.
 *   fnn_mutual_dense  the all-pairs mutual nearest neighbours that FastNN approximates
 *                     (section 3.2.5, "Problem Context").
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - score(a, b) = sum_k a[k] * b[k]  (dist_func = negated dot product); the best candidate
 *    has the LARGEST score and, among equal scores, the LOWEST index (the strict "<" update
 *    of Algorithm 1).
 *  - A map is a row-major [n][d] array in DEVICE memory, pixel id = y * W + x, rows
 *    `row_stride` elements apart (row_stride >= d).  1 <= d <= FNN_MAX_D.
 *    n <= 2^31 - 64.  Inputs must be finite; NaN/Inf give unspecified results.
 *  - `batch` independent image pairs share shapes; maps are passed as HOST arrays of
 *    `batch` fnn_map structs (1 <= batch <= FNN_MAX_BATCH); every other array is ONE
 *    contiguous DEVICE buffer with the batch index outermost.
 *  - The caller owns every buffer.  The library allocates no device memory and touches only the
 *    outputs and `workspace` (device, >= fnn_workspace_bytes(), 256-byte aligned).  All work is
 *    enqueued on `stream` (a hipStream_t, NULL = default stream) and the call returns without
 *    waiting; outputs are valid once the stream has reached that point.  Two calls that share
 *    a workspace must be ordered by the stream.
 *  - State between calls: none that affects results.  The library keeps, per device, a small
 *    cache of launch shapes (how many workgroups of its kernels the device holds, the LDS a
 *    workgroup may be granted); it is filled under a lock by the first call on each device, so
 *    calls from several host threads and on several devices are safe.  The measurement aids of
 *    fnn_measure.h hold process-wide state of their own and are not thread-safe.
 *  - A call may be captured into a HIP graph (it launches kernels only, clears its buffers with
 *    kernels and never synchronises) once the same entry point has run eagerly on the device,
 *    which fills that cache.
 *  - The maps are read by the enqueued work and never written: keep them alive and unchanged
 *    until the stream has passed the call.  The searches work on a prepared copy of each map in
 *    the workspace (cast to the compute format, rows padded to whole 32-pixel tiles).  Two cases
 *    need no separate copy pass, and results do not depend on which way a map took:
 *    (a) the caller's array already is what the copy would be -- stored in the compute format,
 *    d in {16, 24, 32} (16-bit formats) or a multiple of 8 (FNN_F32), row_stride == d, n a
 *    multiple of 32, 16-byte aligned, the batch's maps equally spaced in memory, no flags --
 *    then fnn_nearest and fnn_reciprocal search it where it is;
 *    (b) fnn_reciprocal and (without nq_active) fnn_nearest on fp32 maps with d == 24, a
 *    16-bit compute format, no flags, rows that start on 16-byte boundaries (row_stride a
 *    multiple of 4), at least 1536 seeds or queries and enough work per pair: the first forward
 *    and the first backward search (the one search of fnn_nearest) read the caller's rows, round
 *    them on the way and leave the prepared copy behind for the passes that follow.
 *  - Errors are return codes only.  Argument errors are detected on the host before
 *    anything is enqueued (outputs untouched).  Index arrays live in device memory and are
 *    NOT range-checked: a seed or query index outside [0, n) is undefined behaviour.
 *  - `compute` selects the format the descriptors are rounded to (round-to-nearest-even)
 *    before multiplication: FNN_F16 / FNN_BF16 use the 16-bit matrix instructions,
 *    FNN_F32 multiplies unrounded fp32 values.  Accumulation and selection are fp32 in
 *    all three.  The summation order over k is unspecified.
 */
#ifndef FNN_H
#define FNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FNN_MAX_D 32
#define FNN_MAX_BATCH 64

typedef enum {
    FNN_OK = 0,
    FNN_E_NULL = 1,        /* a required pointer is NULL */
    FNN_E_SHAPE = 2,       /* batch, n, d, row_stride, nq, n_seeds out of range or inconsistent */
    FNN_E_DTYPE = 3,       /* unknown storage or compute format */
    FNN_E_RANGE = 4,       /* max_iter < 0 or another option out of range */
    FNN_E_WORKSPACE = 5,   /* workspace NULL, misaligned or smaller than fnn_workspace_bytes() */
    FNN_E_HIP = 6,         /* a HIP call or kernel launch failed */
    FNN_E_UNSUPPORTED = 7  /* valid request this build cannot serve */
} fnn_status;

typedef enum { FNN_F32 = 0, FNN_F16 = 1, FNN_BF16 = 2 } fnn_dtype;

/* One descriptor map.  `data` is a device pointer to n rows of d elements of `dtype`. */
typedef struct {
    const void* data;
    int64_t n;
    int32_t d;
    int32_t dtype;        /* fnn_dtype of the stored elements */
    int64_t row_stride;   /* in elements */
} fnn_map;

/*
 * FNN_FLAG_NORMALIZE: the maps are raw matching-head outputs (section 3.2.4, "Matching Head");
 * every descriptor is divided by its Euclidean norm before the cast to the compute format:
 * norm2 = sum_k x[k]*x[k] in fp32 (k ascending, products and sums rounded separately),
 * y[k] = x[k] / sqrt(norm2) with correctly rounded fp32 sqrt and division; an all-zero
 * descriptor stays zero.  The step is fused into the prepare pass.
 */
#define FNN_FLAG_NORMALIZE 1
/*
 * FNN_FLAG_HALF_ACCUMULATE (fnn_nearest_blocked with compute == FNN_F16 only; the other
 * entry points answer FNN_E_UNSUPPORTED): the negative control for section 3.4.4, which
 * warns against a plain fp16 computation: every product is rounded to fp16 and the sum is accumulated
 * in fp16, k ascending (IEEE binary16 multiply and add, no fused multiply-add); only the
 * selection stays in fp32.  Exists to measure how many nearest neighbours that changes.
 */
#define FNN_FLAG_HALF_ACCUMULATE 2
/*
 * FNN_FLAG_L2 (fnn_nearest, fnn_reciprocal, fnn_mutual_dense): dist_func of Algorithms 1-3 is
 * the squared Euclidean distance instead of the negated dot product -- the choice that
 * matters for maps that are NOT unit-norm.  score(a, b) = -1/2 * ||a - b||^2 over the
 * descriptors as rounded to the compute format (so "largest score, lowest index on ties"
 * is "smallest distance, lowest index on ties"); out_score / s12 / s21 hold that value,
 * ||a - b||^2 = -2 * score.  It is evaluated on the matrix cores as
 *   <a, b> - 1/2 ||a||^2 - 1/2 ||b||^2
 * with the two norm terms carried in spare channels of the prepared rows (each split into
 * two 16-bit halves for the 16-bit formats), fp32 accumulation.  ||x||^2 is the fp32 sum
 * (k ascending, squares and sums rounded separately) of the rounded channels.  Needs
 * d <= 28 (16-bit compute formats) or d <= 30 (FNN_F32), else FNN_E_SHAPE; size the
 * workspace with fnn_workspace_bytes_opts.  May be combined with FNN_FLAG_NORMALIZE.
 */
#define FNN_FLAG_L2 4
/*
 * FNN_FLAG_SPLIT (fnn_nearest, fnn_reciprocal, fnn_mutual_dense; compute must be FNN_F16, not
 * combinable with FNN_FLAG_L2, else FNN_E_UNSUPPORTED): fp32-grade scores from the 16-bit
 * matrix instructions, the precision end of the HybridCast trade-off (section 3.4.4).  Every
 * descriptor value x (after FNN_FLAG_NORMALIZE, if set) is held as two binary16 numbers,
 * hi = fp16(x) and lo = fp16(x - hi) (round to nearest even; the difference is exact in
 * fp32), and
 *   score(a, b) = sum_k ( a_hi[k] b_hi[k] + a_hi[k] b_lo[k] + a_lo[k] b_hi[k] )
 * with exact products and fp32 accumulation in unspecified order; the lo*lo term, below
 * 2^-22 of the score, is left out.  The prepared rows carry 3*d channels (image 1:
 * [hi, hi, lo], image 2: [hi, lo, hi]) padded to a multiple of 16, so a search costs three
 * times the matrix work of FNN_F16 and still less than FNN_F32; size the workspace with
 * fnn_workspace_bytes_opts.  |x| must stay below 65504.
 */
#define FNN_FLAG_SPLIT 8

typedef struct {
    int32_t compute;      /* fnn_dtype the products are formed in (see above) */
    int32_t max_iter;     /* fnn_reciprocal only: T, the iteration cap (>= 0) */
    int32_t flags;        /* bitwise OR of FNN_FLAG_* */
    int32_t reserved[5];  /* must be zero */
} fnn_opts;

/* Human-readable name of a status code (static storage). */
const char* fnn_status_string(int32_t status);

/*
 * Bytes of device workspace sufficient for any of the three operations on `batch` pairs of
 * maps with n and m pixels, d channels, at most `n_queries` queries or seeds per pair.
 * Returns 0 when the shape is invalid.
 */
size_t fnn_workspace_bytes(int32_t batch, int64_t n, int64_t m, int32_t d, int64_t n_queries, int32_t compute);
/*
 * The same for a call that will be made with `opts` (FNN_FLAG_L2 and FNN_FLAG_SPLIT widen the prepared rows);
 * fnn_workspace_bytes is this function with no flag set.  Returns 0 for invalid shapes or options.
 */
size_t fnn_workspace_bytes_opts(int32_t batch, int64_t n, int64_t m, int32_t d, int64_t n_queries,
                                const fnn_opts* opts);

/*
 * One-directional search (Algorithms 1-3).  For b < batch and q < nq:
 *   row  = q_idx ? q_idx[b*nq + q] : q                 (a pixel of src[b]; needs nq <= src.n)
 *   out_idx[b*nq + q]   = lowest j maximising score(src[b][row], tgt[b][j])
 *   out_score[b*nq + q] = that score (fp32); out_score may be NULL.
 * When nq_active (device int32[batch]) is not NULL only the first
 * min(nq_active[b], nq) queries of pair b are searched and the rest of that pair's outputs
 * are left untouched.  The N x M score matrix is never written to memory.
 */
int32_t fnn_nearest(int32_t batch, const fnn_map* src, const int32_t* q_idx, int64_t nq,
                    const int32_t* nq_active, const fnn_map* tgt, const fnn_opts* opts,
                    int32_t* out_idx, float* out_score,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * The FastNN iteration (section 3.2.5, "FastNN Algorithm").  seeds: device int32[batch][n_seeds], pixel ids of
 * d1 (duplicates allowed).  With U^0 = seeds, V^0 = NN_2(U^0), then for t = 0..max_iter-1:
 * U^{t+1} = NN_1(V^t); a seed with U^{t+1} == U^t has converged: it yields the match
 * (U^t, V^t), records iteration t and leaves; the others continue with
 * V^{t+1} = NN_2(U^{t+1}).  The loop stops when no seed is left or after max_iter
 * iterations (at most 2*max_iter searches).
 * Outputs (device):
 *   seed_i, seed_j, seed_iter  int32[batch][n_seeds]: the match of each seed and the
 *        iteration at which it converged; seed_iter == -1 marks a seed that was still moving
 *        (the convergence mask) and (seed_i, seed_j) is then its last state (U^{T-1}, V^{T-1}).
 *   pairs    int32[batch][n_seeds][2]: the matches of the converged seeds as a set, sorted
 *        by (i, j); entries past n_pairs[b] are -1.
 *   n_pairs  int32[batch].
 */
int32_t fnn_reciprocal(int32_t batch, const fnn_map* d1, const fnn_map* d2,
                       const int32_t* seeds, int64_t n_seeds, const fnn_opts* opts,
                       int32_t* seed_i, int32_t* seed_j, int32_t* seed_iter,
                       int32_t* pairs, int32_t* n_pairs,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * fnn_reciprocal for callers that cannot allocate device memory or hand over a workspace --
 * code running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, outputs and results as fnn_reciprocal, but the workspace is an array of
 * FNN_STATIC_SCRATCH_BYTES that the library itself holds on every device it is loaded on (a
 * device-side global, resident until the process ends).  The call allocates nothing: no
 * hipMalloc / hipFree and no allocating library routine; the first call on a device looks up
 * the array's address on that device (make that call outside graph capture, like the first
 * call of any entry point).
 * Limit: a call that needs more workspace than FNN_STATIC_SCRATCH_BYTES -- fnn_reciprocal's share
 * of fnn_workspace_bytes_opts(): the two prepared maps plus about 40 bytes per seed and a byte
 * per pixel -- is rejected with FNN_E_WORKSPACE before anything is enqueued (48 MiB: one
 * 512x384 pair with d = 24 in any compute format, or two such pairs in a 16-bit format, fit).
 * All calls on one device share that device's array, which keeps the previous call's contents
 * (the call clears what must start at zero itself): calls that overlap on one device -- on
 * different streams or from different host threads -- race; order them on one stream.
 */
#define FNN_STATIC_SCRATCH_BYTES ((size_t)48 << 20)
int32_t fnn_reciprocal_static(int32_t batch, const fnn_map* d1, const fnn_map* d2,
                              const int32_t* seeds, int64_t n_seeds, const fnn_opts* opts,
                              int32_t* seed_i, int32_t* seed_j, int32_t* seed_iter,
                              int32_t* pairs, int32_t* n_pairs, void* stream);

/*
 * All-pairs mutual nearest neighbours (section 3.2.5, "Problem Context").  With
 * S[i][j] = score(d1[i], d2[j]):
 *   nn12[b][i] = lowest j maximising S[i][j],  s12 = that score      (int32/float [batch][n])
 *   nn21[b][j] = lowest i maximising S[i][j],  s21 = that score      (int32/float [batch][m])
 *   pairs[b]   = the (i, nn12[i]) with nn21[nn12[i]] == i, ascending in i
 *                (int32[batch][min(n,m)][2], entries past n_pairs[b] are -1)
 * Every S[i][j] is computed once and feeds both directions, so nn12 and nn21 are consistent
 * with each other.  s12, s21 may be NULL.
 * n and m may not exceed 2^30 here (FNN_E_SHAPE).
 */
int32_t fnn_mutual_dense(int32_t batch, const fnn_map* d1, const fnn_map* d2, const fnn_opts* opts,
                         int32_t* nn12, float* s12, int32_t* nn21, float* s21,
                         int32_t* pairs, int32_t* n_pairs,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * The match set in the problem statement's own terms (section 3.1, "Problem Statement": a
 * correspondence is a pair of pixels i = (w_i, h_i), j = (w_j, h_j)), optionally thinned by
 * the confidence maps c1, c2 that the regression heads emit (section 3.2.3).  For pair b and
 * p < min(n_pairs[b], max_pairs), in input order, the match (i, j) = pairs[b][p] is KEPT iff
 *   0 <= i < n, 0 <= j < m,
 *   conf1 == NULL or conf1[b*n + i] >= min_conf1,  conf2 == NULL or conf2[b*m + j] >= min_conf2
 * (the paper names the confidence maps but prints no rule; this threshold test is this
 * library's reading; a NaN confidence drops the match), and kept matches are written
 * densely, order preserved, as
 *   out_xy[b][q] = (i mod width1, i div width1, j mod width2, j div width2);
 * rows q >= out_count[b] are set to -1.  `pairs` / `n_pairs` are the outputs of
 * fnn_reciprocal or fnn_mutual_dense (device memory, max_pairs rows per pair); the two
 * images may differ in size.  No workspace.  out_xy must not alias pairs.
 * Errors: FNN_E_NULL, FNN_E_SHAPE (batch, widths < 1, negative sizes).
 */
int32_t fnn_pairs_to_pixels(int32_t batch, const int32_t* pairs, const int32_t* n_pairs, int64_t max_pairs,
                            int64_t n, int32_t width1, int64_t m, int32_t width2, const float* conf1,
                            const float* conf2, float min_conf1, float min_conf2, int32_t* out_xy,
                            int32_t* out_count, void* stream);

/*
 * The paper's own search schedules, for comparison with fnn_nearest (same results, one image
 * pair): block_cols == 0 runs Algorithm 2 ("FastNN-Lite", section 3.4.3): a single loop over
 * blocks of block_rows queries, each scored against the WHOLE candidate map into a
 * block_rows x m block of fp32 scores in the workspace, followed by a selection kernel;
 * block_cols > 0 runs Algorithm 1 ("Original FastNN"): the double loop over blocks of
 * block_rows queries and block_cols candidates with the strict "<" running update.  Every
 * loop trip is two host-launched kernels and the score block goes through device memory --
 * the traffic the fused search avoids.  block_rows >= 1; block_cols is rounded up to a
 * multiple of 32.  out_score is required.  Workspace: fnn_blocked_workspace_bytes().
 */
size_t fnn_blocked_workspace_bytes(int64_t n, int64_t m, int32_t d, int32_t block_rows, int32_t block_cols,
                                   int32_t compute);
int32_t fnn_nearest_blocked(const fnn_map* src, const int32_t* q_idx, int64_t nq, const fnn_map* tgt,
                            const fnn_opts* opts, int32_t block_rows, int32_t block_cols,
                            int32_t* out_idx, float* out_score,
                            void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FNN_H */
