/*
 * Polarized-degree stress graph (an INPUT generator; none of the method's
 * arithmetic lives here).  It imitates, in exaggerated form, the degree
 * profile the paper reports for EDA graphs (Section "Kernel Design": a few
 * extremely high-degree rows next to a mass of rows with a handful of
 * non-zeros):
 *
 *   - row i is "heavy" iff mix(seed, i) % 100 == 0                      (1 %)
 *   - light rows: d uniform in {2,3,4} distinct non-zero offsets, each
 *     uniform in [-window, +window], column = (i + offset) mod N
 *   - heavy rows: d = clip(zipf(alpha = 1.2), dmin, dmax) columns drawn
 *     i.i.d. uniform over [0, N), then sorted and de-duplicated
 *   - every row also holds its own index (self-loop); columns ascending
 *
 * The graph is directed (not symmetrised).  Everything is a pure function of
 * (seed, row), so rows can be regenerated independently on any thread.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

static uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

static uint64_t row_stream(uint64_t seed, int64_t row, uint64_t k)
{
    return mix64(mix64(mix64(seed) ^ (uint64_t)row * 0xD6E8FEB86659FD93ULL) + k);
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* Zipf(alpha) on k >= 1 through its inverse CDF, the tail sum replaced by the
   midpoint-rule integral  sum_{j>k} j^-alpha ~ (k+1/2)^(1-alpha)/(alpha-1). */
static int64_t zipf_draw(double u, double alpha, double zeta)
{
    double tail = (1.0 - u) * zeta * (alpha - 1.0);   /* want (k+.5)^(1-alpha) <= tail */
    if (tail <= 0.0) return INT64_MAX / 2;
    double k = ceil(pow(tail, -1.0 / (alpha - 1.0)) - 0.5);
    if (k < 1.0) k = 1.0;
    if (k > 9.0e15) k = 9.0e15;
    return (int64_t)k;
}

int32_t wl_stress_is_heavy(uint64_t seed, int64_t row)
{
    return row_stream(seed, row, 0) % 100 == 0;
}

/* number of draws (before de-duplication, without the self-loop) for a row */
int64_t wl_stress_draws(uint64_t seed, int64_t row, int64_t dmin, int64_t dmax)
{
    if (!wl_stress_is_heavy(seed, row))
        return 2 + (int64_t)(row_stream(seed, row, 1) % 3);
    const double alpha = 1.2, zeta = 5.591582441177751;   /* Riemann zeta(1.2) */
    double u = (double)(row_stream(seed, row, 1) >> 11) * (1.0 / 9007199254740992.0);
    int64_t z = zipf_draw(u, alpha, zeta);
    if (z < dmin) z = dmin;
    if (z > dmax) z = dmax;
    return z;
}

/*
 * Write the sorted, de-duplicated columns of one row (self-loop included)
 * into out[]; cap is the room in out[] and must be >= draws + 1.  Returns the
 * stored row length.
 */
int64_t wl_stress_row(uint64_t seed, int64_t n, int64_t row, int64_t window,
                      int64_t dmin, int64_t dmax, int32_t *out, int64_t cap)
{
    int64_t d = wl_stress_draws(seed, row, dmin, dmax);
    if (d + 1 > cap) return -1;
    int64_t m = 0;
    if (!wl_stress_is_heavy(seed, row)) {
        uint64_t k = 2;
        while (m < d) {
            int64_t off = (int64_t)(row_stream(seed, row, k++) % (uint64_t)(2 * window + 1)) - window;
            if (off == 0) continue;
            int64_t c = ((row + off) % n + n) % n;
            int dup = (c == row);
            for (int64_t t = 0; t < m && !dup; ++t) dup = (out[t] == (int32_t)c);
            if (!dup) out[m++] = (int32_t)c;
        }
    } else {
        for (int64_t t = 0; t < d; ++t)
            out[m++] = (int32_t)(row_stream(seed, row, 2 + (uint64_t)t) % (uint64_t)n);
    }
    out[m++] = (int32_t)row;
    qsort(out, (size_t)m, sizeof(int32_t), cmp_i32);
    int64_t w = 0;
    for (int64_t t = 0; t < m; ++t)
        if (w == 0 || out[w - 1] != out[t]) out[w++] = out[t];
    return w;
}

/* Pass 1: rowptr[0..n] from exact stored row lengths.  Returns nnz or -1. */
int64_t wl_stress_rowptr(uint64_t seed, int64_t n, int64_t window, int64_t dmin, int64_t dmax,
                         int64_t *rowptr)
{
    int64_t fail = 0;
    #pragma omp parallel
    {
        int64_t cap = dmax + 8;
        int32_t *buf = (int32_t *)malloc(sizeof(int32_t) * (size_t)cap);
        if (!buf) {
            #pragma omp atomic write
            fail = 1;
        } else {
            #pragma omp for schedule(dynamic, 4096)
            for (int64_t i = 0; i < n; ++i) {
                int64_t len = wl_stress_row(seed, n, i, window, dmin, dmax, buf, cap);
                rowptr[i + 1] = len;
            }
        }
        free(buf);
    }
    if (fail) return -1;
    rowptr[0] = 0;
    for (int64_t i = 0; i < n; ++i) rowptr[i + 1] += rowptr[i];
    return rowptr[n];
}

/* Pass 2: fill col[] and val[] (val = 1/row length, fp32) for a filled rowptr. */
int32_t wl_stress_fill(uint64_t seed, int64_t n, int64_t window, int64_t dmin, int64_t dmax,
                       const int64_t *rowptr, int32_t *col, float *val)
{
    int64_t fail = 0;
    #pragma omp parallel
    {
        int64_t cap = dmax + 8;
        int32_t *buf = (int32_t *)malloc(sizeof(int32_t) * (size_t)cap);
        if (!buf) {
            #pragma omp atomic write
            fail = 1;
        } else {
            #pragma omp for schedule(dynamic, 4096)
            for (int64_t i = 0; i < n; ++i) {
                int64_t len = wl_stress_row(seed, n, i, window, dmin, dmax, buf, cap);
                if (len != rowptr[i + 1] - rowptr[i]) {
                    #pragma omp atomic write
                    fail = 1;
                    continue;
                }
                memcpy(col + rowptr[i], buf, sizeof(int32_t) * (size_t)len);
                float w = 1.0f / (float)len;
                for (int64_t t = 0; t < len; ++t) val[rowptr[i] + t] = w;
            }
        }
        free(buf);
    }
    return fail ? -1 : 0;
}
