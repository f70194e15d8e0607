/*
 * CPU oracle for fast reciprocal nearest-neighbour matching -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct reference for what the GPU library computes.  It shares
 * no code with the HIP path; only tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it.
 *
 * oracle_nearest is the one-directional search of the paper's Algorithm 1 ("Original
 * FastNN", section 3.4.3) taken per pixel: an outer loop over the queries, an inner loop
 * over all candidates in ascending index order, a running best that is replaced only on a
 * STRICT improvement -- so the lowest candidate index wins ties.  The distance function is
 * the negated dot product (the paper leaves dist_func open; the workload fixes it), hence
 * "dist < min_dist" becomes "score > best".
 *
 * Arithmetic: fp32, k ascending, accumulator starts at +0.0f, no FMA contraction and no
 * reassociation (compile with -ffp-contract=off -fno-fast-math).
 */
#include <math.h>
#include <stdint.h>

/*
 * a      [k_rows][d]  queries, row-major fp32
 * b      [m_rows][d]  candidates, row-major fp32
 * idx    [k_rows]     out: lowest index of the best candidate (-1 when m_rows == 0)
 * best   [k_rows]     out: its score (-inf when m_rows == 0)
 * second [k_rows]     out: the best score among the other candidates; a tied duplicate
 *                          counts, so best-second == 0 on a tie (-inf when m_rows < 2)
 */
void oracle_nearest(const float* a, int64_t k_rows, const float* b, int64_t m_rows, int32_t d,
                    int32_t* idx, float* best, float* second)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t q = 0; q < k_rows; ++q) {
        const float* aq = a + q * (int64_t)d;
        float top = -INFINITY, runner_up = -INFINITY;
        int32_t top_j = -1;
        for (int64_t j = 0; j < m_rows; ++j) {
            const float* bj = b + j * (int64_t)d;
            float s = 0.0f;
            for (int32_t k = 0; k < d; ++k) {
                float p = aq[k] * bj[k];
                s = s + p;
            }
            if (s > top) {
                runner_up = top;
                top = s;
                top_j = (int32_t)j;
            } else if (s > runner_up) {
                runner_up = s;
            }
        }
        idx[q] = top_j;
        best[q] = top;
        second[q] = runner_up;
    }
}

/*
 * The same search with dist_func = squared Euclidean distance (the other natural reading of
 * the undefined dist_func of Algorithms 1-3; it ranks differently from the dot product when
 * the descriptors are not unit-norm).  dist = sum_k (a[k]-b[k])^2 in fp32, k ascending,
 * every difference, square and sum rounded on its own; "dist < min_dist" as printed, so the
 * lowest index wins ties.
 *
 * best / second: the smallest and second smallest distance (+inf when absent).
 */
void oracle_nearest_l2(const float* a, int64_t k_rows, const float* b, int64_t m_rows, int32_t d,
                       int32_t* idx, float* best, float* second)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t q = 0; q < k_rows; ++q) {
        const float* aq = a + q * (int64_t)d;
        float low = INFINITY, runner_up = INFINITY;
        int32_t low_j = -1;
        for (int64_t j = 0; j < m_rows; ++j) {
            const float* bj = b + j * (int64_t)d;
            float dist = 0.0f;
            for (int32_t k = 0; k < d; ++k) {
                float diff = aq[k] - bj[k];
                float sq = diff * diff;
                dist = dist + sq;
            }
            if (dist < low) {
                runner_up = low;
                low = dist;
                low_j = (int32_t)j;
            } else if (dist < runner_up) {
                runner_up = dist;
            }
        }
        idx[q] = low_j;
        best[q] = low;
        second[q] = runner_up;
    }
}

/*
 * The producer step in front of the search (paper section 3.2.4, "Matching Head": the maps
 * D1, D2 come out of the head un-normalised): every descriptor divided by its Euclidean norm.
 * norm2 = sum_k x[k]*x[k] in fp32, k ascending, every product and every sum rounded on its
 * own; y[k] = x[k] / sqrtf(norm2) (IEEE sqrt and division); an all-zero descriptor stays zero.
 */
void oracle_normalize(const float* x, int64_t rows, int32_t d, float* y)
{
    for (int64_t r = 0; r < rows; ++r) {
        const float* xr = x + r * (int64_t)d;
        float* yr = y + r * (int64_t)d;
        float norm2 = 0.0f;
        for (int32_t k = 0; k < d; ++k) {
            float sq = xr[k] * xr[k];
            norm2 = norm2 + sq;
        }
        float norm = sqrtf(norm2);
        for (int32_t k = 0; k < d; ++k) yr[k] = norm > 0.0f ? xr[k] / norm : xr[k];
    }
}

/* Number of threads the parallel loop above uses (for the benchmark's report). */
#ifdef _OPENMP
#include <omp.h>
int32_t oracle_threads(void) { return (int32_t)omp_get_max_threads(); }
#else
int32_t oracle_threads(void) { return 1; }
#endif
