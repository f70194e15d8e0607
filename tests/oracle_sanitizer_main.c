/* Driver for tests/test_oracle_sanitizers.py: runs the oracle's C routines on small inputs, including
 * empty and single-row ones, in a build with AddressSanitizer and UndefinedBehaviorSanitizer.  It
 * checks only that nothing is reported and that two closed-form results hold. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void oracle_nearest(const float*, int64_t, const float*, int64_t, int32_t, int32_t*, float*, float*);
void oracle_nearest_l2(const float*, int64_t, const float*, int64_t, int32_t, int32_t*, float*, float*);
void oracle_normalize(const float*, int64_t, int32_t, float*);

int main(void)
{
    const int shapes[][3] = {{0, 5, 3}, {5, 0, 3}, {1, 1, 1}, {7, 33, 24}, {64, 65, 32}};
    for (unsigned s = 0; s < sizeof(shapes) / sizeof(shapes[0]); ++s) {
        const int k = shapes[s][0], m = shapes[s][1], d = shapes[s][2];
        float* a = malloc(sizeof(float) * (size_t)(k * d + 1));
        float* b = malloc(sizeof(float) * (size_t)(m * d + 1));
        float* y = malloc(sizeof(float) * (size_t)(m * d + 1));
        const int rows = (k > m ? k : m) + 1;   /* the outputs also serve the m-row self search below */
        int32_t* idx = malloc(sizeof(int32_t) * (size_t)rows);
        float* best = malloc(sizeof(float) * (size_t)rows);
        float* second = malloc(sizeof(float) * (size_t)rows);
        unsigned state = 12345u + s;
        for (int i = 0; i < k * d; ++i) { state = state * 1664525u + 1013904223u; a[i] = (float)((int)(state >> 28) - 8) / 8.0f; }
        for (int i = 0; i < m * d; ++i) { state = state * 1664525u + 1013904223u; b[i] = (float)((int)(state >> 28) - 8) / 8.0f; }
        oracle_nearest(a, k, b, m, d, idx, best, second);
        for (int q = 0; q < k; ++q)
            if ((m == 0) != (idx[q] == -1) || (m > 0 && (idx[q] < 0 || idx[q] >= m))) { printf("bad index\n"); return 1; }
        oracle_nearest_l2(a, k, b, m, d, idx, best, second);
        for (int q = 0; q < k; ++q)
            if ((m == 0) != (idx[q] == -1) || (m > 0 && best[q] < 0.0f)) { printf("bad distance\n"); return 1; }
        oracle_normalize(b, m, d, y);
        /* a map searched against itself by distance finds a zero distance */
        oracle_nearest_l2(b, m, b, m, d, idx, best, second);
        for (int q = 0; q < m; ++q)
            if (best[q] != 0.0f) { printf("self distance not zero\n"); return 1; }
        free(a); free(b); free(y); free(idx); free(best); free(second);
    }
    printf("ok\n");
    return 0;
}
