/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct statements of what the degree-split SpMM
 * path of GROOT computes, written from the paper.  Nothing here is used by
 * the product: only tests, the smoke check and the benchmark's CPU-baseline
 * leg may load this file.  It shares no code, header, table or helper with the
 * HIP library.
 *
 * Contents (each function cites the passage it follows):
 *   orc_aig_simulate      bit-parallel evaluation of an And-Inverter Graph
 *   orc_csr_nnz/_build    EDA-graph adjacency A, degree D, mean weights D^-1 A
 *   orc_spmm_f64          Y = A_hat * X row by row in fp64, plus sum of |terms|
 *   orc_spmm_t_f64, orc_csr_transpose   transposed aggregation (backward pass)
 *   orc_plan              degree classes and the stable degree sort
 *   orc_part_of_default   level-contiguous partition rule
 *   orc_regrow_*          boundary sets, crossing edges, augmented sub-graphs
 *
 * Pins (tests/, "not gpu"): the paper's two-bit multiplier example and its
 * printed node/edge counts; AIG simulation == integer product; closed-form
 * node/edge/degree counts; X = ones; dense brute force on <= 64 nodes;
 * hand-evaluated Eq. (1)-(2) sets on tiny graphs; dense transpose and the
 * adjoint identity <A x, y> = <x, A^T y> for the transposed aggregation.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#define ORC_SYMMETRIC  1u   /* store both directions of every AIG edge          */
#define ORC_SELF_LOOPS 2u   /* add (v,v) for every node                         */
#define ORC_NORM_MEAN  4u   /* weight = 1/row length (else 1)                   */
#define ORC_REGROW     1u   /* partition: add boundary nodes and crossing edges */

/* ------------------------------------------------------------------------
 * AIG evaluation (Section "Converting Netlists into Transitional Graph": an
 * AIG is a DAG of two-input ANDs whose edges may carry inverters).
 * word[v] holds 64 independent input patterns, one per bit.  PIs take their
 * word from pi_words in id order; an AND is the conjunction of its two
 * (possibly complemented) fanin words; a PO copies its (possibly
 * complemented) driver.  Returns 0, or -1 if a fanin does not precede its
 * node.
 * ------------------------------------------------------------------------ */
int32_t orc_aig_simulate(int64_t n1, const uint8_t *type, const int32_t *fanin0,
                         const int32_t *fanin1, const uint64_t *pi_words, uint64_t *word)
{
    int64_t next_pi = 0;
    for (int64_t v = 0; v < n1; ++v) {
        if (type[v] == 0) { word[v] = pi_words[next_pi++]; continue; }
        int32_t l0 = fanin0[v], l1 = fanin1[v];
        if (l0 < 0 || l1 < 0 || (l0 >> 1) >= v || (l1 >> 1) >= v) return -1;
        uint64_t w0 = word[l0 >> 1] ^ ((l0 & 1) ? ~0ULL : 0ULL);
        uint64_t w1 = word[l1 >> 1] ^ ((l1 & 1) ? ~0ULL : 0ULL);
        word[v] = (type[v] == 1) ? (w0 & w1) : w0;
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Adjacency (Section "Node Features and Node Label creation": G = (V,E),
 * adjacency A in R^{NxN}, degree D_ii = sum_j A_ij; aggregation by GraphSAGE
 * mean, i.e. A_hat = D^-1 A with D counted on the stored row).
 *
 * Every fanin record (driver u, inverted?) of a non-PI node v is an edge
 * u -> v.  Entries: (v,u) always; (u,v) too when ORC_SYMMETRIC; (v,v) when
 * ORC_SELF_LOOPS.  Duplicate entries are merged (A is binary).  Each stored
 * entry carries a byte: bit0 = the edge is inverted, bit1 = the column is a
 * driver of the row, bit2 = self-loop.  Copies of a batch are block-diagonal:
 * copy c shifts every id by c*n1.
 * ------------------------------------------------------------------------ */
typedef struct { int64_t row; int32_t col; uint8_t pol; } entry_t;

static int entry_cmp(const void *a, const void *b)
{
    const entry_t *x = (const entry_t *)a, *y = (const entry_t *)b;
    if (x->row != y->row) return (x->row > y->row) - (x->row < y->row);
    return (x->col > y->col) - (x->col < y->col);
}

/* sorted, merged entry list of ONE copy; returns count or -1 */
static int64_t one_copy_entries(int64_t n1, const uint8_t *type, const int32_t *fanin0,
                                const int32_t *fanin1, uint32_t flags, entry_t **out)
{
    int64_t cap = 5 * n1 + 8, m = 0;
    entry_t *e = (entry_t *)malloc(sizeof(entry_t) * (size_t)cap);
    if (!e) return -1;
    for (int64_t v = 0; v < n1; ++v) {
        if (flags & ORC_SELF_LOOPS) { e[m].row = v; e[m].col = (int32_t)v; e[m].pol = 4; ++m; }
        if (type[v] == 0) continue;
        const int32_t lits[2] = { fanin0[v], fanin1[v] };
        for (int t = 0; t < 2; ++t) {
            int32_t u = lits[t] >> 1;
            uint8_t inv = (uint8_t)(lits[t] & 1);
            e[m].row = v; e[m].col = u; e[m].pol = (uint8_t)(inv | 2); ++m;
            if (flags & ORC_SYMMETRIC) { e[m].row = u; e[m].col = (int32_t)v; e[m].pol = inv; ++m; }
        }
    }
    qsort(e, (size_t)m, sizeof(entry_t), entry_cmp);
    int64_t w = 0;
    for (int64_t t = 0; t < m; ++t) {
        if (w > 0 && e[w - 1].row == e[t].row && e[w - 1].col == e[t].col) e[w - 1].pol |= e[t].pol;
        else e[w++] = e[t];
    }
    *out = e;
    return w;
}

int64_t orc_csr_nnz(int64_t n1, const uint8_t *type, const int32_t *fanin0, const int32_t *fanin1,
                    int32_t batch, uint32_t flags)
{
    entry_t *e = NULL;
    int64_t m = one_copy_entries(n1, type, fanin0, fanin1, flags, &e);
    free(e);
    return m < 0 ? -1 : m * batch;
}

int32_t orc_csr_build(int64_t n1, const uint8_t *type, const int32_t *fanin0, const int32_t *fanin1,
                      int32_t batch, uint32_t flags, int64_t *rowptr, int32_t *col, float *val,
                      uint8_t *pol)
{
    entry_t *e = NULL;
    int64_t m = one_copy_entries(n1, type, fanin0, fanin1, flags, &e);
    if (m < 0) return -1;
    int64_t n = n1 * batch;
    for (int64_t i = 0; i <= n; ++i) rowptr[i] = 0;
    for (int32_t c = 0; c < batch; ++c)
        for (int64_t t = 0; t < m; ++t) {
            int64_t p = (int64_t)c * m + t;
            rowptr[(int64_t)c * n1 + e[t].row + 1] += 1;
            col[p] = (int32_t)((int64_t)c * n1 + e[t].col);
            pol[p] = e[t].pol;
        }
    for (int64_t i = 0; i < n; ++i) rowptr[i + 1] += rowptr[i];
    for (int64_t i = 0; i < n; ++i) {
        int64_t deg = rowptr[i + 1] - rowptr[i];           /* D_ii of the stored row */
        float w = (flags & ORC_NORM_MEAN) ? 1.0f / (float)deg : 1.0f;
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) val[p] = w;
    }
    free(e);
    return 0;
}

/* ------------------------------------------------------------------------
 * Aggregation Y = A_hat X (the sparse product both of the paper's kernels
 * compute, Section "Kernel Design - GROOT-GPU"), one row at a time in fp64 on
 * the fp32 weights and features as given.  S (optional) receives the sum of
 * absolute terms, the scale of the accepted rounding error.
 * ------------------------------------------------------------------------ */
void orc_spmm_f64(int64_t n, const int64_t *rowptr, const int32_t *col, const float *val,
                  const float *X, int32_t F, double *Y, double *S)
{
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        for (int32_t k = 0; k < F; ++k) {
            double y = 0.0, s = 0.0;
            for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
                double term = (double)val[p] * (double)X[(int64_t)col[p] * F + k];
                y += term;
                s += fabs(term);
            }
            Y[i * F + k] = y;
            if (S) S[i * F + k] = s;
        }
    }
}

/* ------------------------------------------------------------------------
 * Degree classes and degree sort (Section "Kernel Design - GROOT-GPU":
 * high-degree rows go to the HD kernel, the rest to the LD kernel, whose
 * step B computes each row's degree from the row pointer and stably sorts
 * rows by degree).  One threshold T: HD iff deg >= T.  by_degree lists LD
 * rows by ascending degree, ties by ascending id (what a stable sort of the
 * id-ordered rows gives); deg_offsets[d] = number of LD rows of degree < d,
 * for d = 0..T.
 * ------------------------------------------------------------------------ */
int32_t orc_plan(int64_t n, const int64_t *rowptr, int32_t T, uint8_t *row_class,
                 int32_t *hd_rows, int32_t *ld_rows, int32_t *by_degree, int64_t *deg_offsets,
                 int64_t *n_hd_out, int64_t *n_ld_out)
{
    if (T < 1) return -1;
    int64_t n_hd = 0, n_ld = 0;
    for (int64_t i = 0; i < n; ++i) {
        int64_t deg = rowptr[i + 1] - rowptr[i];
        row_class[i] = deg >= T;
        if (deg >= T) hd_rows[n_hd++] = (int32_t)i; else ld_rows[n_ld++] = (int32_t)i;
    }
    int64_t w = 0;
    for (int32_t d = 0; d < T; ++d) {
        deg_offsets[d] = w;
        for (int64_t i = 0; i < n; ++i)
            if (rowptr[i + 1] - rowptr[i] == d) by_degree[w++] = (int32_t)i;
    }
    deg_offsets[T] = w;
    *n_hd_out = n_hd;
    *n_ld_out = n_ld;
    return w == n_ld ? 0 : -1;
}

/* ------------------------------------------------------------------------
 * Partition rule used in place of METIS (Section "GNN and Edge Re-growth
 * After Partition"): the p-th contiguous slice of every copy's emission
 * order, part(v) = min(P-1, floor((v mod n1) * P / n1)).
 * ------------------------------------------------------------------------ */
void orc_part_of_default(int64_t n, int64_t n1, int32_t P, int32_t *part_of)
{
    for (int64_t v = 0; v < n; ++v) {
        int64_t q = ((v % n1) * P) / n1;
        part_of[v] = (int32_t)(q < P - 1 ? q : P - 1);
    }
}

/* ------------------------------------------------------------------------
 * Boundary edge re-growth for ONE part p (Eq. (1), Eq. (2), Algorithm 1):
 *   N(S_p) = union of one-hop neighbours of S_p,   B_p = N(S_p) \ S_p,
 *   C_p    = edges with one end in S_p and the other in B_p (either direction),
 *   S_p+   = S_p u B_p,    E_p+ = E[S_p] u C_p.
 * E is the stored pattern of the graph: (i,j) in E iff row i holds column j;
 * a node's one-hop neighbours are the other columns of its row.  Edges
 * between two boundary nodes belong to neither E[S_p] nor C_p and are left
 * out; a stored self-loop of a boundary node is kept so that its row is never
 * empty.  Local ids: S_p ascending, then B_p ascending.  Local weights are
 * 1/(local row length) when norm_mean, else 1.
 *
 * orc_regrow_sizes reports the sizes; orc_regrow_fill writes global_id and
 * the local CSR (columns ascending in local id).  n_crossing counts unordered
 * pairs {i,j}, i in S_p, j in B_p, joined by an entry in either direction.
 * With regrow = 0 (the paper's ablation without re-growth) B_p is empty and
 * only E[S_p] is kept.
 * ------------------------------------------------------------------------ */
static int has_entry(const int64_t *rowptr, const int32_t *col, int64_t i, int64_t j)
{
    for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) if (col[p] == j) return 1;
    return 0;
}

/* local_of[v] = local id of v in part p, or -1.  Returns n_owned via pointer. */
static int64_t label_part(int64_t n, const int64_t *rowptr, const int32_t *col,
                          const int32_t *part_of, int32_t p, uint32_t flags,
                          int64_t *local_of, int64_t *n_owned_out)
{
    uint8_t *in_N = (uint8_t *)calloc((size_t)n + 1, 1);
    if (!in_N) return -1;
    for (int64_t u = 0; u < n; ++u) {
        if (part_of[u] != p) continue;
        for (int64_t q = rowptr[u]; q < rowptr[u + 1]; ++q)
            if (col[q] != u) in_N[col[q]] = 1;               /* N(S_p), Eq. (1) */
    }
    int64_t next = 0;
    for (int64_t v = 0; v < n; ++v) local_of[v] = -1;
    for (int64_t v = 0; v < n; ++v) if (part_of[v] == p) local_of[v] = next++;
    *n_owned_out = next;
    if (flags & ORC_REGROW)
        for (int64_t v = 0; v < n; ++v)
            if (in_N[v] && part_of[v] != p) local_of[v] = next++;   /* B_p = N(S_p) \ S_p */
    free(in_N);
    return next;
}

int32_t orc_regrow_sizes(int64_t n, const int64_t *rowptr, const int32_t *col,
                         const int32_t *part_of, int32_t p, uint32_t flags,
                         int64_t *n_owned, int64_t *n_halo, int64_t *n_crossing, int64_t *nnz_local)
{
    int64_t *local_of = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    if (!local_of) return -1;
    int64_t owned = 0;
    int64_t total = label_part(n, rowptr, col, part_of, p, flags, local_of, &owned);
    if (total < 0) { free(local_of); return -1; }
    int64_t cross = 0, nnz = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (local_of[i] < 0) continue;
        int i_owned = part_of[i] == p;
        for (int64_t q = rowptr[i]; q < rowptr[i + 1]; ++q) {
            int64_t j = col[q];
            if (local_of[j] < 0) continue;
            int j_owned = part_of[j] == p;
            int keep = (i_owned && j_owned)                     /* E[S_p]            */
                    || (i_owned != j_owned)                     /* C_p               */
                    || (i == j);                                /* halo self-loop    */
            if (!keep) continue;
            ++nnz;
            if (i_owned && !j_owned) ++cross;                                     /* pair seen from S_p */
            if (!i_owned && j_owned && !has_entry(rowptr, col, j, i)) ++cross;    /* one-way edge       */
        }
    }
    *n_owned = owned; *n_halo = total - owned; *n_crossing = cross; *nnz_local = nnz;
    free(local_of);
    return 0;
}

typedef struct { int32_t col; float val; } cv_t;

static int cv_cmp(const void *a, const void *b)
{
    int32_t x = ((const cv_t *)a)->col, y = ((const cv_t *)b)->col;
    return (x > y) - (x < y);
}

/* weight_mode: 0 = all ones, 1 = 1/(local row length), 2 = keep the weight the
   entry has in the full graph (val must be given). */
int32_t orc_regrow_fill(int64_t n, const int64_t *rowptr, const int32_t *col, const float *val,
                        const int32_t *part_of, int32_t p, uint32_t flags, int32_t weight_mode,
                        int64_t *global_id, int64_t *sub_rowptr, int32_t *sub_col, float *sub_val)
{
    int64_t *local_of = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    if (!local_of) return -1;
    int64_t owned = 0;
    int64_t total = label_part(n, rowptr, col, part_of, p, flags, local_of, &owned);
    if (total < 0) { free(local_of); return -1; }
    for (int64_t v = 0; v < n; ++v) if (local_of[v] >= 0) global_id[local_of[v]] = v;
    int64_t w = 0;
    sub_rowptr[0] = 0;
    for (int64_t li = 0; li < total; ++li) {
        int64_t i = global_id[li];
        int i_owned = part_of[i] == p;
        int64_t len = rowptr[i + 1] - rowptr[i], m = 0;
        cv_t *row = (cv_t *)malloc(sizeof(cv_t) * (size_t)(len + 1));
        if (!row) { free(local_of); return -1; }
        for (int64_t q = rowptr[i]; q < rowptr[i + 1]; ++q) {
            int64_t j = col[q];
            if (local_of[j] < 0) continue;
            int j_owned = part_of[j] == p;
            if ((i_owned && j_owned) || (i_owned != j_owned) || i == j) {
                row[m].col = (int32_t)local_of[j];
                row[m].val = (weight_mode == 2) ? val[q] : 1.0f;
                ++m;
            }
        }
        qsort(row, (size_t)m, sizeof(cv_t), cv_cmp);
        for (int64_t t = 0; t < m; ++t) {
            sub_col[w] = row[t].col;
            sub_val[w] = (weight_mode == 1) ? 1.0f / (float)m : row[t].val;
            ++w;
        }
        free(row);
        sub_rowptr[li + 1] = w;
    }
    free(local_of);
    return 0;
}

/* ------------------------------------------------------------------------
 * Transposed aggregation (the backward pass of a GNN layer applies the
 * transpose of the forward aggregation; the paper motivates its kernels by
 * training time, Section "Accuracy and Accuracy Recovery of Various
 * Multipliers"):  (A_hat^T G)[j,k] = sum_i a_hat_ij * G[i,k].
 * orc_spmm_t_f64 is that definition as a scatter over the rows of A_hat, in
 * fp64, serially.  orc_csr_transpose writes A_hat^T as a CSR (entry (j,i)
 * carries the weight of (i,j); rows of the result list i ascending).
 * ------------------------------------------------------------------------ */
void orc_spmm_t_f64(int64_t n, const int64_t *rowptr, const int32_t *col, const float *val,
                    const float *G, int32_t F, double *out, double *S)
{
    for (int64_t t = 0; t < n * F; ++t) { out[t] = 0.0; if (S) S[t] = 0.0; }
    for (int64_t i = 0; i < n; ++i)
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            const int64_t j = col[p];
            for (int32_t k = 0; k < F; ++k) {
                double term = (double)val[p] * (double)G[i * F + k];
                out[j * F + k] += term;
                if (S) S[j * F + k] += fabs(term);
            }
        }
}

void orc_csr_transpose(int64_t n, const int64_t *rowptr, const int32_t *col, const float *val,
                       int64_t *t_rowptr, int32_t *t_col, float *t_val)
{
    for (int64_t j = 0; j <= n; ++j) t_rowptr[j] = 0;
    for (int64_t p = 0; p < rowptr[n]; ++p) t_rowptr[col[p] + 1] += 1;
    for (int64_t j = 0; j < n; ++j) t_rowptr[j + 1] += t_rowptr[j];
    int64_t *cursor = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    for (int64_t j = 0; j < n; ++j) cursor[j] = t_rowptr[j];
    for (int64_t i = 0; i < n; ++i)                        /* i ascending => each result row ascending */
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            int64_t q = cursor[col[p]]++;
            t_col[q] = (int32_t)i;
            t_val[q] = val[p];
        }
    free(cursor);
}
