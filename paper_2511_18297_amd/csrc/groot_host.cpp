// Host side of libgroot: graph construction, degree plan, partition with
// boundary edge re-growth, argument checking and the C ABI.  No HIP headers
// here; device work goes through the launchers in groot_kernels.hip.
#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <limits>
#include <memory>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "groot_internal.h"

namespace groot {

static thread_local std::string g_error;

void set_error(const std::string &msg) { g_error = msg; }

groot_status fail(groot_status st, const std::string &msg)
{
    g_error = msg;
    return st;
}

Tuning &tuning()
{
    static Tuning t;
    return t;
}

// Static split of [0,n) over the host threads.
static void parallel_for(int64_t n, int64_t min_per_thread,
                         const std::function<void(int64_t, int64_t)> &body)
{
    unsigned hw = std::thread::hardware_concurrency();
    int64_t nt = std::max<int64_t>(1, std::min<int64_t>(hw ? hw : 1, n / std::max<int64_t>(1, min_per_thread)));
    nt = std::min<int64_t>(nt, 32);
    if (nt <= 1) { body(0, n); return; }
    std::vector<std::thread> th;
    int64_t per = (n + nt - 1) / nt;
    for (int64_t t = 0; t < nt; ++t) {
        int64_t lo = t * per, hi = std::min(n, lo + per);
        if (lo >= hi) break;
        th.emplace_back([=, &body] { body(lo, hi); });
    }
    for (auto &t : th) t.join();
}

}  // namespace groot

using namespace groot;

// ---------------------------------------------------------------------------
// objects
// ---------------------------------------------------------------------------
struct groot_graph {
    int64_t n = 0, nnz = 0;
    int64_t n1 = 0;                 // nodes per copy (partition rule); == n for CSR graphs
    WeightMode weight_mode = WeightMode::Explicit;
    std::vector<int64_t> rowptr;
    std::vector<int32_t> col;
    std::vector<float> val;
    std::vector<uint8_t> pol;       // empty for graphs not built from an AIG
    bool symmetric = false;         // built with GROOT_SYMMETRIC: entry (i, j) is stored iff (j, i) is
};

struct groot_plan {
    const groot_graph *g = nullptr;
    int32_t threshold = 0;
    std::vector<uint8_t> row_class;
    std::vector<int32_t> hd_rows, ld_rows, ld_rows_by_degree;
    std::vector<int64_t> ld_deg_offsets;
    // kernel schedule
    std::vector<HdChunk> chunks;
    std::vector<HdSplitRow> split_rows;
    int64_t n_partials = 0;
    int32_t max_F = 0;
    bool resident = false;
    DevicePlan dev;
};

struct groot_parts {
    struct Part {
        int64_t n_owned = 0, n_halo = 0, n_crossing = 0;
        std::vector<int64_t> global_id;
        groot_graph sub;
    };
    std::vector<Part> parts;
};

struct groot_dev_part {
    DevicePart d;
    WeightMode weight_mode = WeightMode::Explicit;
    bool csr_moved = false;         // the CSR arrays now belong to a plan
};

// ---------------------------------------------------------------------------
// graph construction
// ---------------------------------------------------------------------------
namespace {

// Adjacency of one AIG copy.  Row v is assembled as [drivers..., self,
// fanouts in ascending id], so only the (at most two) drivers can be out of
// order or repeated; a short insertion pass puts the row in order and merges
// repeats.
groot_status build_one_copy(int64_t n1, const uint8_t *type, const int32_t *f0, const int32_t *f1,
                            uint32_t flags, std::vector<int64_t> &rowptr, std::vector<int32_t> &col,
                            std::vector<uint8_t> &pol)
{
    const bool sym = flags & GROOT_SYMMETRIC, loops = flags & GROOT_SELF_LOOPS;
    for (int64_t v = 0; v < n1; ++v) {
        if (type[v] > 2) return fail(GROOT_EINVAL, "node " + std::to_string(v) + ": unknown type");
        if (type[v] == 0) {
            if (f0[v] != -1 || f1[v] != -1)
                return fail(GROOT_EINVAL, "primary input " + std::to_string(v) + " has fanins");
            continue;
        }
        for (int32_t lit : {f0[v], f1[v]})
            if (lit < 0 || (int64_t)(lit >> 1) >= v)
                return fail(GROOT_EINVAL, "node " + std::to_string(v) + ": fanin literal " + std::to_string(lit) +
                                              " is negative or not before its node (AIG must be topological)");
        if (type[v] == 2 && f0[v] != f1[v])
            return fail(GROOT_EINVAL, "primary output " + std::to_string(v) + ": the two fanin slots differ");
    }
    // upper bound of each row's length, then a prefix sum gives write cursors
    std::vector<int64_t> cursor(n1 + 1, 0);
    for (int64_t v = 0; v < n1; ++v) {
        if (loops) cursor[v + 1] += 1;
        if (type[v] == 0) continue;
        cursor[v + 1] += 2;
        if (sym) { cursor[(f0[v] >> 1) + 1] += 1; cursor[(f1[v] >> 1) + 1] += 1; }
    }
    for (int64_t v = 0; v < n1; ++v) cursor[v + 1] += cursor[v];
    std::vector<int64_t> start(cursor.begin(), cursor.end() - 1);
    std::vector<int32_t> tcol(cursor[n1]);
    std::vector<uint8_t> tpol(cursor[n1]);
    std::vector<int64_t> fill(start);
    auto put = [&](int64_t row, int32_t c, uint8_t bits) {
        int64_t p = fill[row]++;
        tcol[p] = c;
        tpol[p] = bits;
    };
    for (int64_t v = 0; v < n1; ++v) {
        if (type[v] != 0) {
            put(v, f0[v] >> 1, (uint8_t)((f0[v] & 1) | 2));
            put(v, f1[v] >> 1, (uint8_t)((f1[v] & 1) | 2));
        }
        if (loops) put(v, (int32_t)v, 4);
        if (type[v] != 0 && sym) {
            put(f0[v] >> 1, (int32_t)v, (uint8_t)(f0[v] & 1));
            put(f1[v] >> 1, (int32_t)v, (uint8_t)(f1[v] & 1));
        }
    }
    // order + merge each row in place, then compact
    rowptr.assign(n1 + 1, 0);
    std::vector<int64_t> len(n1);
    parallel_for(n1, 1 << 16, [&](int64_t lo, int64_t hi) {
        for (int64_t v = lo; v < hi; ++v) {
            int64_t b = start[v], e = fill[v];
            for (int64_t i = b + 1; i < e; ++i) {          // insertion sort (rows are nearly sorted)
                int32_t c = tcol[i];
                uint8_t q = tpol[i];
                int64_t j = i;
                while (j > b && tcol[j - 1] > c) { tcol[j] = tcol[j - 1]; tpol[j] = tpol[j - 1]; --j; }
                tcol[j] = c;
                tpol[j] = q;
            }
            int64_t w = b;
            for (int64_t i = b; i < e; ++i) {
                if (w > b && tcol[w - 1] == tcol[i]) tpol[w - 1] |= tpol[i];
                else { tcol[w] = tcol[i]; tpol[w] = tpol[i]; ++w; }
            }
            len[v] = w - b;
        }
    });
    for (int64_t v = 0; v < n1; ++v) rowptr[v + 1] = rowptr[v] + len[v];
    col.resize(rowptr[n1]);
    pol.resize(rowptr[n1]);
    parallel_for(n1, 1 << 16, [&](int64_t lo, int64_t hi) {
        for (int64_t v = lo; v < hi; ++v) {
            std::memcpy(&col[rowptr[v]], &tcol[start[v]], sizeof(int32_t) * len[v]);
            std::memcpy(&pol[rowptr[v]], &tpol[start[v]], len[v]);
        }
    });
    return GROOT_OK;
}

void fill_uniform_weights(groot_graph &g)
{
    g.val.resize(g.nnz);
    const bool mean = g.weight_mode == WeightMode::Mean;
    parallel_for(g.n, 1 << 16, [&](int64_t lo, int64_t hi) {
        for (int64_t i = lo; i < hi; ++i) {
            int64_t b = g.rowptr[i], e = g.rowptr[i + 1];
            float w = mean ? 1.0f / (float)(e - b) : 1.0f;
            for (int64_t p = b; p < e; ++p) g.val[p] = w;
        }
    });
}

}  // namespace

extern "C" groot_status groot_graph_build(int64_t n1, const uint8_t *type, const int32_t *fanin0,
                                          const int32_t *fanin1, int32_t batch, uint32_t flags,
                                          groot_graph **out)
{
    if (!type || !fanin0 || !fanin1 || !out) return fail(GROOT_EINVAL, "groot_graph_build: NULL argument");
    if (n1 < 1 || batch < 1) return fail(GROOT_EINVAL, "groot_graph_build: n1 and batch must be >= 1");
    if (flags & ~(GROOT_SYMMETRIC | GROOT_SELF_LOOPS | GROOT_NORM_MEAN))
        return fail(GROOT_EINVAL, "groot_graph_build: unknown flag bits");
    if (n1 > (int64_t)std::numeric_limits<int32_t>::max() / batch)
        return fail(GROOT_ERANGE, "groot_graph_build: n1*batch does not fit int32 node ids");
    try {
        std::unique_ptr<groot_graph> g(new groot_graph);
        std::vector<int64_t> rp1;
        std::vector<int32_t> col1;
        std::vector<uint8_t> pol1;
        groot_status st = build_one_copy(n1, type, fanin0, fanin1, flags, rp1, col1, pol1);
        if (st != GROOT_OK) return st;
        const int64_t nnz1 = rp1[n1];
        g->n1 = n1;
        g->n = n1 * batch;
        g->nnz = nnz1 * batch;
        g->weight_mode = (flags & GROOT_NORM_MEAN) ? WeightMode::Mean : WeightMode::Ones;
        g->symmetric = (flags & GROOT_SYMMETRIC) != 0;
        g->rowptr.resize(g->n + 1);
        g->col.resize(g->nnz);
        g->pol.resize(g->nnz);
        for (int32_t c = 0; c < batch; ++c) {
            const int64_t row0 = (int64_t)c * n1, p0 = (int64_t)c * nnz1;
            const int32_t shift = (int32_t)row0;
            parallel_for(n1, 1 << 18, [&](int64_t lo, int64_t hi) {
                for (int64_t v = lo; v < hi; ++v) g->rowptr[row0 + v] = p0 + rp1[v];
            });
            parallel_for(nnz1, 1 << 18, [&](int64_t lo, int64_t hi) {
                for (int64_t p = lo; p < hi; ++p) g->col[p0 + p] = col1[p] + shift;
                std::memcpy(&g->pol[p0 + lo], &pol1[lo], (size_t)(hi - lo));
            });
        }
        g->rowptr[g->n] = g->nnz;
        fill_uniform_weights(*g);
        *out = g.release();
        return GROOT_OK;
    } catch (const std::bad_alloc &) {
        return fail(GROOT_ENOMEM, "groot_graph_build: out of host memory");
    }
}

extern "C" groot_status groot_graph_from_csr(int64_t n, const int64_t *rowptr, const int32_t *col,
                                             const float *val, groot_graph **out)
{
    if (!rowptr || !out) return fail(GROOT_EINVAL, "groot_graph_from_csr: NULL argument");
    if (n < 1) return fail(GROOT_EINVAL, "groot_graph_from_csr: n must be >= 1");
    if (n > std::numeric_limits<int32_t>::max()) return fail(GROOT_ERANGE, "groot_graph_from_csr: n >= 2^31");
    if (rowptr[0] != 0) return fail(GROOT_EINVAL, "groot_graph_from_csr: rowptr[0] != 0");
    for (int64_t i = 0; i < n; ++i)
        if (rowptr[i + 1] < rowptr[i]) return fail(GROOT_EINVAL, "groot_graph_from_csr: rowptr decreases");
    const int64_t nnz = rowptr[n];
    if (nnz > 0 && (!col || !val)) return fail(GROOT_EINVAL, "groot_graph_from_csr: NULL col/val");
    std::atomic<int64_t> bad_row{-1};
    parallel_for(n, 1 << 16, [&](int64_t lo, int64_t hi) {
        for (int64_t i = lo; i < hi; ++i)
            for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p)
                if (col[p] < 0 || col[p] >= n || (p > rowptr[i] && col[p - 1] >= col[p])) {
                    bad_row.store(i);
                    return;
                }
    });
    if (bad_row.load() >= 0)
        return fail(GROOT_EINVAL, "groot_graph_from_csr: row " + std::to_string(bad_row.load()) +
                                      " has a column out of range or not strictly ascending");
    try {
        std::unique_ptr<groot_graph> g(new groot_graph);
        g->n = g->n1 = n;
        g->nnz = nnz;
        g->weight_mode = WeightMode::Explicit;
        g->rowptr.assign(rowptr, rowptr + n + 1);
        g->col.assign(col, col + nnz);
        g->val.assign(val, val + nnz);
        *out = g.release();
        return GROOT_OK;
    } catch (const std::bad_alloc &) {
        return fail(GROOT_ENOMEM, "groot_graph_from_csr: out of host memory");
    }
}

extern "C" groot_status groot_graph_transpose(const groot_graph *g, groot_graph **out)
{
    if (!g || !out) return fail(GROOT_EINVAL, "groot_graph_transpose: NULL argument");
    try {
        std::unique_ptr<groot_graph> t(new groot_graph);
        const int64_t n = g->n;
        t->n = n;
        t->n1 = g->n1;
        t->nnz = g->nnz;
        t->weight_mode = WeightMode::Explicit;
        t->rowptr.assign(n + 1, 0);
        t->col.resize(g->nnz);
        t->val.resize(g->nnz);
        for (int64_t p = 0; p < g->nnz; ++p) ++t->rowptr[g->col[p] + 1];
        for (int64_t j = 0; j < n; ++j) t->rowptr[j + 1] += t->rowptr[j];
        std::vector<int64_t> cursor(t->rowptr.begin(), t->rowptr.end() - 1);
        // rows of g are visited in ascending order, so every row of the transpose fills in ascending column order
        for (int64_t i = 0; i < n; ++i)
            for (int64_t p = g->rowptr[i]; p < g->rowptr[i + 1]; ++p) {
                const int64_t q = cursor[g->col[p]]++;
                t->col[q] = (int32_t)i;
                t->val[q] = g->val[p];
            }
        *out = t.release();
        return GROOT_OK;
    } catch (const std::bad_alloc &) {
        return fail(GROOT_ENOMEM, "groot_graph_transpose: out of host memory");
    }
}

extern "C" groot_status groot_graph_view(const groot_graph *g, int64_t *n, int64_t *nnz,
                                         const int64_t **rowptr, const int32_t **col, const float **val,
                                         const uint8_t **pol)
{
    if (!g) return fail(GROOT_EINVAL, "groot_graph_view: NULL graph");
    if (n) *n = g->n;
    if (nnz) *nnz = g->nnz;
    if (rowptr) *rowptr = g->rowptr.data();
    if (col) *col = g->col.data();
    if (val) *val = g->val.data();
    if (pol) *pol = g->pol.empty() ? nullptr : g->pol.data();
    return GROOT_OK;
}

extern "C" void groot_graph_free(groot_graph *g) { delete g; }

// ---------------------------------------------------------------------------
// plan
// ---------------------------------------------------------------------------
namespace {

// HD schedule: every high-degree row is cut into balanced pieces of at most hd_chunk non-zeros.
// begin_of(k) / degree_of(k): first non-zero and stored length of the k-th high-degree row.
template <class Begin, class Degree>
groot_status hd_schedule(int64_t n_hd, const int32_t *hd_rows, Begin begin_of, Degree degree_of,
                         std::vector<HdChunk> &chunks, std::vector<HdSplitRow> &split_rows, int64_t &n_partials)
{
    const int64_t chunk = std::max(64, tuning().hd_chunk.load());
    int64_t slots = 0;
    for (int64_t k = 0; k < n_hd; ++k) {
        const int32_t row = hd_rows[k];
        const int64_t b = begin_of(k), d = degree_of(k);
        const int64_t pieces = std::max<int64_t>(1, (d + chunk - 1) / chunk);
        if (slots + pieces > std::numeric_limits<int32_t>::max() / 2)
            return fail(GROOT_ERANGE, "groot_spmm_plan: too many high-degree pieces");
        const int64_t per = (d + pieces - 1) / pieces;
        if (pieces > 1) split_rows.push_back(HdSplitRow{row, (int32_t)slots, (int32_t)pieces, 0});
        for (int64_t c = 0; c < pieces; ++c) {
            const int64_t lo = c * per, hi = std::min(d, lo + per);
            HdChunk ch;
            ch.begin = b + lo;
            ch.len = (int32_t)std::max<int64_t>(0, hi - lo);
            ch.row = row;
            ch.slot = pieces > 1 ? (int32_t)(slots + c) : -1;
            ch.row_nnz = (int32_t)std::min<int64_t>(d, std::numeric_limits<int32_t>::max());
            chunks.push_back(ch);
        }
        if (pieces > 1) slots += pieces;
    }
    n_partials = slots;
    return GROOT_OK;
}

// Pieces run in the order of their first column (key[c] of piece c): pieces of different rows that read the
// same stretch of feature rows (in an array multiplier: the a_j and b_i rows over the same partial products)
// then run close together, and the second reader finds the rows in the last-level cache.
void sort_hd_schedule(std::vector<HdChunk> &chunks, const std::vector<int32_t> &key)
{
    std::vector<int64_t> order(chunks.size());
    for (size_t c = 0; c < order.size(); ++c) order[c] = (int64_t)c;
    std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) { return key[a] < key[b]; });
    std::vector<HdChunk> sorted(chunks.size());
    for (size_t c = 0; c < order.size(); ++c) sorted[c] = chunks[order[c]];
    chunks.swap(sorted);
}

}  // namespace

extern "C" groot_status groot_spmm_plan(const groot_graph *g, int32_t degree_threshold, groot_plan **out)
{
    if (!g || !out) return fail(GROOT_EINVAL, "groot_spmm_plan: NULL argument");
    if (degree_threshold < 1) return fail(GROOT_EINVAL, "groot_spmm_plan: degree_threshold must be >= 1");
    try {
        std::unique_ptr<groot_plan> pl(new groot_plan);
        const int64_t n = g->n;
        const int32_t T = degree_threshold;
        pl->g = g;
        pl->threshold = T;
        pl->row_class.resize(n);
        // histogram of low degrees and class of every row
        std::vector<int64_t> hist(T + 1, 0);
        int64_t n_hd = 0;
        for (int64_t i = 0; i < n; ++i) {
            int64_t d = g->rowptr[i + 1] - g->rowptr[i];
            bool hd = d >= T;
            pl->row_class[i] = hd;
            if (hd) ++n_hd; else ++hist[d];
        }
        const int64_t n_ld = n - n_hd;
        pl->hd_rows.resize(n_hd);
        pl->ld_rows.resize(n_ld);
        pl->ld_rows_by_degree.resize(n_ld);
        pl->ld_deg_offsets.assign(T + 1, 0);
        for (int32_t d = 0; d < T; ++d) pl->ld_deg_offsets[d + 1] = pl->ld_deg_offsets[d] + hist[d];
        // counting sort: walking ids upward keeps equal degrees in id order (stable)
        std::vector<int64_t> cursor(pl->ld_deg_offsets.begin(), pl->ld_deg_offsets.end() - 1);
        int64_t ih = 0, il = 0;
        for (int64_t i = 0; i < n; ++i) {
            if (pl->row_class[i]) { pl->hd_rows[ih++] = (int32_t)i; continue; }
            pl->ld_rows[il++] = (int32_t)i;
            pl->ld_rows_by_degree[cursor[g->rowptr[i + 1] - g->rowptr[i]]++] = (int32_t)i;
        }
        groot_status hs = hd_schedule(n_hd, pl->hd_rows.data(), [&](int64_t k) { return g->rowptr[pl->hd_rows[k]]; },
                                      [&](int64_t k) { return g->rowptr[pl->hd_rows[k] + 1] - g->rowptr[pl->hd_rows[k]]; },
                                      pl->chunks, pl->split_rows, pl->n_partials);
        if (hs != GROOT_OK) return hs;
        std::vector<int32_t> key(pl->chunks.size());
        for (size_t c = 0; c < key.size(); ++c)
            key[c] = pl->chunks[c].len > 0 ? g->col[pl->chunks[c].begin] : std::numeric_limits<int32_t>::max();
        sort_hd_schedule(pl->chunks, key);
        *out = pl.release();
        return GROOT_OK;
    } catch (const std::bad_alloc &) {
        return fail(GROOT_ENOMEM, "groot_spmm_plan: out of host memory");
    }
}

extern "C" groot_status groot_plan_view(const groot_plan *plan, int64_t *n_hd, int64_t *n_ld,
                                        const uint8_t **row_class, const int32_t **hd_rows,
                                        const int32_t **ld_rows, const int32_t **ld_rows_by_degree,
                                        const int64_t **ld_deg_offsets)
{
    if (!plan) return fail(GROOT_EINVAL, "groot_plan_view: NULL plan");
    if (!plan->g) return fail(GROOT_EINVAL, "groot_plan_view: the plan was built on the device (use groot_plan_lists_device)");
    if (n_hd) *n_hd = (int64_t)plan->hd_rows.size();
    if (n_ld) *n_ld = (int64_t)plan->ld_rows.size();
    if (row_class) *row_class = plan->row_class.data();
    if (hd_rows) *hd_rows = plan->hd_rows.data();
    if (ld_rows) *ld_rows = plan->ld_rows.data();
    if (ld_rows_by_degree) *ld_rows_by_degree = plan->ld_rows_by_degree.data();
    if (ld_deg_offsets) *ld_deg_offsets = plan->ld_deg_offsets.data();
    return GROOT_OK;
}

namespace {
void release_device(groot_plan *pl)
{
    DevicePlan &d = pl->dev;
    dev_free(d.rowptr); dev_free(d.col); dev_free(d.val);
    dev_free(d.chunks); dev_free(d.split_rows); dev_free(d.partials); dev_free(d.zero_row); dev_free(d.mid_rows);
    dev_free(d.rp32); dev_free(d.col16); dev_free(d.hot_cols);
    dev_free(d.hd_rows); dev_free(d.hd_agg); dev_free(d.chunks_rank); dev_free(d.split_rows_rank);
    d = DevicePlan{};
    pl->resident = false;
}

template <class T>
groot_status to_device(T **dst, const T *src, size_t count, const char *what)
{
    *dst = nullptr;
    if (count == 0) return GROOT_OK;
    void *p = nullptr;
    int err = dev_alloc(&p, count * sizeof(T));
    if (err) return fail(GROOT_ENOMEM, std::string("groot_plan_upload: device allocation of ") + what +
                                           " failed: " + hip_error_text(err));
    *dst = (T *)p;
    if (src) {
        err = dev_upload(p, src, count * sizeof(T));
        if (err) return fail(GROOT_EHIP, std::string("groot_plan_upload: copy of ") + what +
                                             " failed: " + hip_error_text(err));
    }
    return GROOT_OK;
}
}  // namespace

namespace {
// Which LD kernel an uploaded plan uses.  The pipelined kernel gives every row D gather slots and always issues
// all D (a slot past the row's end reads a row of zeros), and a gather costs the same whether it hits a cache or
// not (it is the per-CU return path of the vector memory unit that it occupies): so D should be as small as the
// rows allow.  A low-degree row with more than D entries is masked there and computed by a row-list kernel (one
// lane group per row, nothing overlapped), which is fine as long as such rows are few.  Rule: the smallest D in
// kPipeMinDepth .. kPipeMaxDepth that leaves at most 2 low-degree rows in 100 to the row list; none does: the
// plain kernel (or D = kPipeMaxDepth when the knob insists).  at_most(d) = low-degree rows with at most d entries.
// -> DevicePlan::ld_pipelined (0 / 2), and the slot count
struct PipeChoice {
    int pipelined;
    int depth;
};
template <class AtMost>
PipeChoice choose_ld_kernel(int knob, int64_t n_ld, AtMost at_most)
{
    if (knob == 0 || n_ld <= 0) return {0, kPipeMaxDepth};
    const int forced = tuning().pipe_depth;
    if (forced >= kPipeMinDepth && forced <= kPipeMaxDepth) return {2, forced};
    for (int d = kPipeMinDepth; d <= kPipeMaxDepth; ++d)
        if ((n_ld - at_most(d)) * 50 <= n_ld) return {2, d};
    return {knob > 0 ? 2 : 0, kPipeMaxDepth};
}
}  // namespace

namespace {
// The fused layer's side of the high-degree rows (see DevicePlan) for a plan made on the host: the HD schedule
// with rows renamed to their place in hd_rows (ascending ids), and the buffer their aggregated features go to.
groot_status upload_layer_hd_side(groot_plan *pl, const int32_t *hd_rows_host, int64_t n_hd, int32_t max_F)
{
    DevicePlan &d = pl->dev;
    d.n_hd_rows = n_hd;
    if (n_hd == 0) return GROOT_OK;
    auto rank_of = [&](int32_t row) {
        return (int32_t)(std::lower_bound(hd_rows_host, hd_rows_host + n_hd, row) - hd_rows_host);
    };
    std::vector<HdChunk> chunks(pl->chunks);
    for (HdChunk &ch : chunks) ch.row = rank_of(ch.row);
    std::vector<HdSplitRow> split(pl->split_rows);
    for (HdSplitRow &sr : split) sr.row = rank_of(sr.row);
    groot_status st;
    if ((st = to_device(&d.chunks_rank, chunks.data(), chunks.size(), "HD schedule of the fused layer")) != GROOT_OK ||
        (st = to_device(&d.split_rows_rank, split.data(), split.size(), "HD split rows of the fused layer")) != GROOT_OK ||
        (st = to_device<float>(&d.hd_agg, nullptr, (size_t)n_hd * max_F, "high-degree sums of the fused layer")) != GROOT_OK ||
        (st = to_device(&d.hd_rows, hd_rows_host, (size_t)n_hd, "high-degree row list")) != GROOT_OK)
        return st;
    return GROOT_OK;
}
}  // namespace

extern "C" groot_status groot_plan_upload(groot_plan *plan, int32_t max_F)
{
    if (!plan) return fail(GROOT_EINVAL, "groot_plan_upload: NULL plan");
    if (max_F < 4 || max_F > 512 || max_F % 4) return fail(GROOT_EINVAL, "groot_plan_upload: max_F must be a multiple of 4 in [4,512]");
    if (!plan->g) {
        if (max_F <= plan->max_F) return GROOT_OK;
        return fail(GROOT_EINVAL, "groot_plan_upload: the plan was built on the device with a smaller max_F");
    }
    if (plan->resident) release_device(plan);
    const groot_graph *g = plan->g;
    DevicePlan &d = plan->dev;
    d.n = d.n_cols = g->n;
    d.nnz = g->nnz;
    d.threshold = plan->threshold;
    d.xcd_remap = tuning().xcd_remap;
    d.weight_mode = d.graph_weight_mode = (int)g->weight_mode;
    const bool need_val = g->weight_mode == WeightMode::Explicit;   // row-uniform weights are recomputed on the device
    if (need_val && tuning().uniform_detect && g->nnz > 0) {
        // Weights given entry by entry are often the mean normalisation all the same (a mapped netlist that
        // comes in as a CSR matrix): if every entry is bit for bit fl(1 / row length), or every entry is 1,
        // the kernels recompute the weight from the row pointer and never read the array (4 bytes per entry),
        // and the kernels for row-uniform weights apply.
        std::atomic<bool> mean{true}, ones{true};
        parallel_for(g->n, 1 << 16, [&](int64_t lo, int64_t hi) {
            bool m = true, o = true;
            for (int64_t i = lo; i < hi && (m || o); ++i) {
                const int64_t b = g->rowptr[i], e = g->rowptr[i + 1];
                const float w = e > b ? 1.0f / (float)(e - b) : 0.0f;
                for (int64_t q = b; q < e; ++q) {
                    uint32_t bits, want, one;
                    const float f1 = 1.0f;
                    std::memcpy(&bits, &g->val[q], 4);
                    std::memcpy(&want, &w, 4);
                    std::memcpy(&one, &f1, 4);
                    m = m && bits == want;
                    o = o && bits == one;
                }
            }
            if (!m) mean = false;
            if (!o) ones = false;
        });
        if (ones) d.weight_mode = (int)WeightMode::Ones;
        else if (mean) d.weight_mode = (int)WeightMode::Mean;
    }
    groot_status st;
    const std::vector<float> zeros(kZeroRowFloats + kTrashFloats, 0.0f);
    if ((st = to_device(&d.zero_row, zeros.data(), zeros.size(), "zero row")) != GROOT_OK ||
        (st = to_device(&d.rowptr, g->rowptr.data(), g->rowptr.size(), "rowptr")) != GROOT_OK ||
        (st = to_device(&d.col, g->col.data(), g->col.size(), "col")) != GROOT_OK ||
        (st = to_device(&d.val, g->val.data(), need_val ? g->val.size() : 0, "val")) != GROOT_OK ||
        (st = to_device(&d.chunks, plan->chunks.data(), plan->chunks.size(), "HD schedule")) != GROOT_OK ||
        (st = to_device(&d.split_rows, plan->split_rows.data(), plan->split_rows.size(), "HD split rows")) != GROOT_OK ||
        (st = to_device<float>(&d.partials, nullptr, (size_t)plan->n_partials * max_F, "HD partial sums")) != GROOT_OK) {
        std::string keep = groot_last_error();
        release_device(plan);
        set_error(keep);
        return st;
    }
    // LD kernel choice; the low-degree rows with more entries than the pipelined kernel has slots are the tail
    // of the degree-sorted list
    {
        const int64_t n_ld = (int64_t)plan->ld_rows.size();
        const std::vector<int64_t> &offs = plan->ld_deg_offsets;        // [d]: low-degree rows with fewer than d entries
        auto at_most = [&](int32_t len) { return offs.empty() ? 0 : offs[std::min<int32_t>(len + 1, plan->threshold)]; };
        const PipeChoice ch = choose_ld_kernel(tuning().ld_pipeline, n_ld, at_most);
        d.ld_pipelined = ch.pipelined;
        d.pipe_depth = ch.depth;
        // the fused layer kernel completes a longer row inside the tile's turn, unoverlapped: 5 slots only when
        // at most one low-degree row in 2000 has 6 entries or more
        d.sage_depth = (n_ld - at_most(5)) * 2000 <= n_ld ? 5 : 6;
        const int64_t first_mid = at_most(ch.depth);
        d.n_mid_rows = ch.pipelined ? n_ld - first_mid : 0;
        if (d.n_mid_rows &&
            (st = to_device(&d.mid_rows, plan->ld_rows_by_degree.data() + first_mid, (size_t)d.n_mid_rows, "long low-degree rows")) != GROOT_OK) {
            std::string keep = groot_last_error();
            release_device(plan);
            set_error(keep);
            return st;
        }
    }
    // compact CSR for the pipelined kernel (4-byte row pointers, 2-byte column codes), when the graph allows it
    if (d.ld_pipelined && tuning().csr_compress) {
        int32_t *hd_dev = nullptr;
        if ((st = to_device(&hd_dev, plan->hd_rows.data(), plan->hd_rows.size(), "high-degree row list")) != GROOT_OK) {
            std::string keep = groot_last_error();
            release_device(plan);
            set_error(keep);
            return st;
        }
        int err = launch_csr_compress(d, hd_dev, (int64_t)plan->hd_rows.size(), nullptr);
        dev_free(hd_dev);
        if (!err && d.compressed) err = pipe_compact_prepare();
        if (err) {
            release_device(plan);
            return fail(GROOT_EHIP, std::string("groot_plan_upload: compact CSR: ") + hip_error_text(err));
        }
    }
    if ((st = upload_layer_hd_side(plan, plan->hd_rows.data(), (int64_t)plan->hd_rows.size(), max_F)) != GROOT_OK) {
        std::string keep = groot_last_error();
        release_device(plan);
        set_error(keep);
        return st;
    }
    d.n_chunks = (int64_t)plan->chunks.size();
    d.nnz_hd = 0;
    for (const HdChunk &ch : plan->chunks) d.nnz_hd += ch.len;
    d.n_tiles = (g->n + kRowsPerLdTile - 1) / kRowsPerLdTile;
    d.n_split_rows = (int64_t)plan->split_rows.size();
    d.n_partials = plan->n_partials;
    plan->max_F = max_F;
    plan->resident = true;
    return GROOT_OK;
}

namespace {
groot_status check_features(const char *who, const void *a, const void *b, int32_t F)
{
    if (!a || !b) return fail(GROOT_EINVAL, std::string(who) + ": NULL device pointer");
    if (((uintptr_t)a | (uintptr_t)b) & 15) return fail(GROOT_EINVAL, std::string(who) + ": pointers must be 16-byte aligned");
    if (F < 4 || F > 512 || F % 4) return fail(GROOT_EINVAL, std::string(who) + ": F must be a multiple of 4 in [4,512]");
    return GROOT_OK;
}
}  // namespace

extern "C" groot_status groot_spmm_execute_phases(const groot_plan *plan, const float *X_dev, float *Y_dev,
                                                  int32_t F, uint32_t phases, void *hip_stream)
{
    if (!plan) return fail(GROOT_EINVAL, "groot_spmm_execute: NULL plan");
    groot_status st = check_features("groot_spmm_execute", X_dev, Y_dev, F);
    if (st != GROOT_OK) return st;
    if (!plan->resident) return fail(GROOT_EINVAL, "groot_spmm_execute: plan is not on the device (call groot_plan_upload)");
    if (F > plan->max_F) return fail(GROOT_EINVAL, "groot_spmm_execute: F exceeds the max_F given to groot_plan_upload");
    if (phases & ~GROOT_PHASE_ALL) return fail(GROOT_EINVAL, "groot_spmm_execute: unknown phase bits");
    const char *a = (const char *)X_dev, *b = (const char *)Y_dev;
    const int64_t x_bytes = plan->dev.n_cols * (int64_t)F * 4, y_bytes = plan->dev.n * (int64_t)F * 4;
    if (a < b + y_bytes && b < a + x_bytes) return fail(GROOT_EINVAL, "groot_spmm_execute: X and Y overlap");
    int err = 0;
    if (!err && (phases & GROOT_PHASE_LD)) err = launch_ld(plan->dev, X_dev, Y_dev, F, hip_stream);
    if (!err && (phases & GROOT_PHASE_HD) && plan->dev.n_chunks) err = launch_hd(plan->dev, X_dev, Y_dev, F, hip_stream);
    if (!err && (phases & GROOT_PHASE_FINISH) && plan->dev.n_split_rows) err = launch_hd_finish(plan->dev, Y_dev, F, hip_stream);
    if (err) return fail(GROOT_EHIP, std::string("groot_spmm_execute: launch failed: ") + hip_error_text(err));
    return GROOT_OK;
}

extern "C" groot_status groot_spmm_execute_rows(const groot_plan *plan, const float *X_dev, float *Y_dev, int32_t F,
                                                int64_t n_rows, const int64_t *out_ids_dev, void *hip_stream)
{
    if (!plan) return fail(GROOT_EINVAL, "groot_spmm_execute_rows: NULL plan");
    groot_status st = check_features("groot_spmm_execute_rows", X_dev, Y_dev, F);
    if (st != GROOT_OK) return st;
    if (!plan->resident) return fail(GROOT_EINVAL, "groot_spmm_execute_rows: plan is not on the device (call groot_plan_upload)");
    if (F > plan->max_F) return fail(GROOT_EINVAL, "groot_spmm_execute_rows: F exceeds the max_F given to groot_plan_upload");
    if (n_rows < 0 || n_rows > plan->dev.n) return fail(GROOT_EINVAL, "groot_spmm_execute_rows: n_rows outside [0, N]");
    if (n_rows == 0) return GROOT_OK;
    const RowOut out{out_ids_dev, n_rows};
    int err = launch_ld(plan->dev, X_dev, Y_dev, F, hip_stream, &out);
    if (!err && plan->dev.n_chunks) err = launch_hd(plan->dev, X_dev, Y_dev, F, hip_stream, &out);
    if (!err && plan->dev.n_split_rows) err = launch_hd_finish(plan->dev, Y_dev, F, hip_stream, &out);
    if (err) return fail(GROOT_EHIP, std::string("groot_spmm_execute_rows: launch failed: ") + hip_error_text(err));
    return GROOT_OK;
}

extern "C" groot_status groot_spmm_execute(const groot_plan *plan, const float *X_dev, float *Y_dev,
                                           int32_t F, void *hip_stream)
{
    return groot_spmm_execute_phases(plan, X_dev, Y_dev, F, GROOT_PHASE_ALL, hip_stream);
}

namespace {
struct PlacementTry {
    const groot_plan *plan;
    const float *X;
    float *Y;
    int32_t F;
    void *stream;
    groot_status status;
};
int placement_step(void *ctx)
{
    PlacementTry *t = (PlacementTry *)ctx;
    t->status = groot_spmm_execute(t->plan, t->X, t->Y, t->F, t->stream);
    return t->status == GROOT_OK ? 0 : -1;
}
}  // namespace

extern "C" groot_status groot_feature_placement(const groot_plan *plan, void *arena_dev, size_t arena_bytes, int32_t F,
                                                void *hip_stream, size_t *x_offset, size_t *y_offset, float *best_ms,
                                                float *first_ms)
{
    const char *who = "groot_feature_placement: ";
    if (!plan || !arena_dev || !x_offset || !y_offset) return fail(GROOT_EINVAL, std::string(who) + "NULL argument");
    if (!plan->resident) return fail(GROOT_EINVAL, std::string(who) + "plan is not on the device (call groot_plan_upload)");
    if (F < 4 || F > 512 || F % 4) return fail(GROOT_EINVAL, std::string(who) + "F must be a multiple of 4 in [4,512]");
    if (((uintptr_t)arena_dev & 15) != 0) return fail(GROOT_EINVAL, std::string(who) + "the arena must be 16-byte aligned");
    const size_t rows = (size_t)std::max(plan->dev.n, plan->dev.n_cols);
    const size_t size = rows * (size_t)F * 4;                 // one matrix
    const size_t step = std::max<size_t>(4096, size / 4 / 4096 * 4096);   // a quarter of it, in whole 4 KB units
    const int64_t apart = (int64_t)((size + step - 1) / step);      // steps between two matrices that do not overlap
    if (arena_bytes < size + (size_t)apart * step)
        return fail(GROOT_EINVAL, std::string(who) + "the arena must hold two matrices (the second starts at a multiple of a quarter matrix, in whole 4 KB units)");
    const int64_t last = (int64_t)((arena_bytes - size) / step);   // offsets 0 .. last steps
    char *base = (char *)arena_dev;
    PlacementTry t{plan, nullptr, nullptr, F, hip_stream, GROOT_OK};
    auto time_pair = [&](int64_t qx, int64_t qy, float *ms) -> groot_status {
        t.X = (const float *)(base + (size_t)qx * step);
        t.Y = (float *)(base + (size_t)qy * step);
        const int err = device_time_ms(hip_stream, 3, placement_step, &t, ms);
        if (err < 0) return t.status;                          // groot_spmm_execute has set the error text
        if (err) return fail(GROOT_EHIP, std::string(who) + hip_error_text(err));
        return GROOT_OK;
    };
    groot_status st;
    float first = 0.f;
    if ((st = time_pair(0, apart, &first)) != GROOT_OK) return st;   // the two matrices back to back, as first allocated
    float best = first;
    int64_t bx = 0, by = apart;
    // every pair of half-matrix offsets that does not overlap (the fast pairs are those in which both matrices
    // straddle a boundary between the two classes of address ranges, which a search along one coordinate at a time
    // does not find), then the quarter-matrix neighbours of the best pair, twice
    int64_t hop = 2;                                           // at most 16 offsets per matrix: 256 pairs whatever the arena's size
    while (last / hop + 1 > 16) hop += 2;
    for (int64_t qx = 0; qx <= last; qx += hop)
        for (int64_t qy = 0; qy <= last; qy += hop) {
            if (std::llabs(qx - qy) < apart || (qx == 0 && qy == apart)) continue;
            float ms = 0.f;
            if ((st = time_pair(qx, qy, &ms)) != GROOT_OK) return st;
            if (ms < best) { best = ms; bx = qx; by = qy; }
        }
    for (int round = 0; round < 2; ++round) {
        const int64_t cx = bx, cy = by;
        for (int64_t dx = -1; dx <= 1; ++dx)
            for (int64_t dy = -1; dy <= 1; ++dy) {
                const int64_t qx = cx + dx, qy = cy + dy;
                if ((dx == 0 && dy == 0) || qx < 0 || qy < 0 || qx > last || qy > last || std::llabs(qx - qy) < apart) continue;
                float ms = 0.f;
                if ((st = time_pair(qx, qy, &ms)) != GROOT_OK) return st;
                if (ms < best) { best = ms; bx = qx; by = qy; }
            }
        if (bx == cx && by == cy) break;
    }
    *x_offset = (size_t)bx * step;
    *y_offset = (size_t)by * step;
    if (best_ms) *best_ms = best;
    if (first_ms) *first_ms = first;
    return GROOT_OK;
}

extern "C" groot_status groot_rows_over_degree(const groot_plan *plan, const float *Z_dev, float *out_dev, int32_t F,
                                               void *hip_stream)
{
    const char *who = "groot_rows_over_degree: ";
    if (!plan || !Z_dev || !out_dev) return fail(GROOT_EINVAL, std::string(who) + "NULL argument");
    if (F < 4 || F > 512 || F % 4) return fail(GROOT_EINVAL, std::string(who) + "F must be a multiple of 4 in [4,512]");
    if ((((uintptr_t)Z_dev) | ((uintptr_t)out_dev)) & 15) return fail(GROOT_EINVAL, std::string(who) + "pointers must be 16-byte aligned");
    if (!plan->resident) return fail(GROOT_EINVAL, std::string(who) + "plan is not on the device (call groot_plan_upload)");
    const int err = launch_rows_over_degree(plan->dev, Z_dev, out_dev, F, hip_stream);
    if (err) return fail(GROOT_EHIP, std::string(who) + "launch failed: " + hip_error_text(err));
    return GROOT_OK;
}

extern "C" groot_status groot_sage_layer_backward_data(const groot_plan *plan, const float *dZ_over_deg_dev,
                                                       const float *WnT_dev, const float *WsT_dev, float *dX_dev,
                                                       int32_t F_out, int32_t F_in, void *hip_stream)
{
    const char *who = "groot_sage_layer_backward_data: ";
    if (!plan) return fail(GROOT_EINVAL, std::string(who) + "NULL plan");
    if ((F_out != 64 && F_out != 32) || (F_in != 64 && F_in != 32 && F_in != 16))
        return fail(GROOT_EINVAL, std::string(who) + "the layer's output width (the width of dZ) must be 32 or 64, its input width (of dX) 16, 32 or 64");
    groot_status st = check_features("groot_sage_layer_backward_data", dZ_over_deg_dev, dX_dev, F_out);
    if (st != GROOT_OK) return st;
    if (!WnT_dev || !WsT_dev) return fail(GROOT_EINVAL, std::string(who) + "NULL weight pointer");
    if (!plan->resident) return fail(GROOT_EINVAL, std::string(who) + "plan is not on the device (call groot_plan_upload)");
    if (!plan->g || !plan->g->symmetric || plan->g->weight_mode != WeightMode::Mean ||
        plan->dev.weight_mode != (int)WeightMode::Mean)
        return fail(GROOT_EINVAL, std::string(who) + "needs the plan of a graph built symmetric with mean weights (groot_graph_build with its default flags)");
    if (F_out > plan->max_F) return fail(GROOT_EINVAL, std::string(who) + "the width of dZ exceeds the max_F given to groot_plan_upload");
    if (plan->dev.n_cols != plan->dev.n)
        return fail(GROOT_EINVAL, std::string(who) + "the plan's columns were renamed to global rows (groot_plan_use_global_columns)");
    const char *a = (const char *)dZ_over_deg_dev, *b = (const char *)dX_dev;
    const int64_t z_bytes = plan->dev.n * (int64_t)F_out * 4, x_bytes = plan->dev.n * (int64_t)F_in * 4;
    if (a < b + x_bytes && b < a + z_bytes) return fail(GROOT_EINVAL, std::string(who) + "dZ and dX overlap");
    // unit-weight sums of the high-degree rows into the plan's side buffer, then the layer kernel in its gradient form
    DevicePlan hd = plan->dev;
    hd.chunks = plan->dev.chunks_rank;
    hd.split_rows = plan->dev.split_rows_rank;
    hd.weight_mode = (int)WeightMode::Ones;
    int err = 0;
    if (hd.n_chunks) err = launch_hd(hd, dZ_over_deg_dev, hd.hd_agg, F_out, hip_stream);
    if (!err && hd.n_split_rows) err = launch_hd_finish(hd, hd.hd_agg, F_out, hip_stream);
    if (!err) err = launch_sage_pipe(plan->dev, dZ_over_deg_dev, dX_dev, WnT_dev, WsT_dev, nullptr, 0, F_out, F_in,
                                     tuning().sage_pieces.load(), 1, hip_stream);
    if (err) return fail(GROOT_EHIP, std::string(who) + "launch failed: " + hip_error_text(err));
    return GROOT_OK;
}

namespace {
bool wgrad_widths_ok(int32_t F_in, int32_t F_out)
{
    return (F_in == 64 || F_in == 32) && (F_out == 64 || F_out == 32 || F_out == 16);
}
}  // namespace

extern "C" groot_status groot_sage_layer_backward_weights_workspace(const groot_plan *plan, int32_t F_in, int32_t F_out,
                                                                    size_t *bytes)
{
    const char *who = "groot_sage_layer_backward_weights_workspace: ";
    if (!plan || !bytes) return fail(GROOT_EINVAL, std::string(who) + "NULL argument");
    if (!wgrad_widths_ok(F_in, F_out)) return fail(GROOT_EINVAL, std::string(who) + "F_in must be 32 or 64, F_out 16, 32 or 64");
    const size_t b = sage_wgrad_workspace_bytes(F_in, F_out);
    if (b == 0) return fail(GROOT_EHIP, std::string(who) + "no device");
    *bytes = b;
    return GROOT_OK;
}

extern "C" groot_status groot_sage_layer_backward_weights(const groot_plan *plan, const float *X_dev, const float *dZ_dev,
                                                          float *dWn_dev, float *dWs_dev, int32_t F_in, int32_t F_out,
                                                          void *workspace_dev, size_t workspace_bytes, void *hip_stream)
{
    const char *who = "groot_sage_layer_backward_weights: ";
    if (!plan) return fail(GROOT_EINVAL, std::string(who) + "NULL plan");
    if (!wgrad_widths_ok(F_in, F_out)) return fail(GROOT_EINVAL, std::string(who) + "F_in must be 32 or 64, F_out 16, 32 or 64");
    groot_status st = check_features("groot_sage_layer_backward_weights", X_dev, dZ_dev, F_in);
    if (st != GROOT_OK) return st;
    if (!dWn_dev || !dWs_dev || !workspace_dev) return fail(GROOT_EINVAL, std::string(who) + "NULL output or workspace pointer");
    if ((((uintptr_t)dWn_dev) | ((uintptr_t)dWs_dev) | ((uintptr_t)workspace_dev)) & 15)
        return fail(GROOT_EINVAL, std::string(who) + "pointers must be 16-byte aligned");
    if (!plan->resident) return fail(GROOT_EINVAL, std::string(who) + "plan is not on the device (call groot_plan_upload)");
    if (plan->dev.weight_mode == (int)WeightMode::Explicit)
        return fail(GROOT_EINVAL, std::string(who) + "needs row-uniform weights (a graph built from an AIG, or one whose weights are 1 / row length)");
    if (F_in > plan->max_F) return fail(GROOT_EINVAL, std::string(who) + "F_in exceeds the max_F given to groot_plan_upload");
    if (plan->dev.n_cols != plan->dev.n)
        return fail(GROOT_EINVAL, std::string(who) + "the plan's columns were renamed to global rows (groot_plan_use_global_columns)");
    const size_t need = sage_wgrad_workspace_bytes(F_in, F_out);
    if (need == 0) return fail(GROOT_EHIP, std::string(who) + "no device");
    if (workspace_bytes < need)
        return fail(GROOT_EINVAL, std::string(who) + "workspace too small (ask groot_sage_layer_backward_weights_workspace)");
    // sums of the high-degree rows into the plan's side buffer, as for the forward layer
    DevicePlan hd = plan->dev;
    hd.chunks = plan->dev.chunks_rank;
    hd.split_rows = plan->dev.split_rows_rank;
    int err = 0;
    if (hd.n_chunks) err = launch_hd(hd, X_dev, hd.hd_agg, F_in, hip_stream);
    if (!err && hd.n_split_rows) err = launch_hd_finish(hd, hd.hd_agg, F_in, hip_stream);
    if (!err) err = launch_sage_wgrad(plan->dev, X_dev, dZ_dev, dWn_dev, dWs_dev, F_in, F_out, tuning().sage_pieces.load(),
                                      workspace_dev, hip_stream);
    if (err) return fail(GROOT_EHIP, std::string(who) + "launch failed: " + hip_error_text(err));
    return GROOT_OK;
}

extern "C" groot_status groot_sage_layer_forward_io(const groot_plan *plan, const float *X_dev, const float *Wn_dev,
                                                    const float *Ws_dev, const float *bias_dev, int32_t relu,
                                                    float *H_dev, int32_t F_in, int32_t F_out, void *hip_stream)
{
    const char *who = "groot_sage_layer_forward: ";
    if (!plan) return fail(GROOT_EINVAL, std::string(who) + "NULL plan");
    if ((F_in != 64 && F_in != 32) || (F_out != 64 && F_out != 32 && F_out != 16))
        return fail(GROOT_EINVAL, std::string(who) + "input width must be 32 or 64, output width 16, 32 or 64");
    const bool wavefronts = plan->resident && tuning().sage_kernel && plan->dev.weight_mode != (int)WeightMode::Explicit;
    if ((F_in != 64 || F_out != 64) && plan->resident && !wavefronts)
        return fail(GROOT_EINVAL, std::string(who) + "widths other than 64 -> 64 need row-uniform weights (and the default layer kernel)");
    groot_status st = check_features("groot_sage_layer_forward", X_dev, H_dev, F_in);
    if (st != GROOT_OK) return st;
    if (!Wn_dev || !Ws_dev) return fail(GROOT_EINVAL, std::string(who) + "NULL weight pointer");
    if (!plan->resident) return fail(GROOT_EINVAL, std::string(who) + "plan is not on the device (call groot_plan_upload)");
    if (F_in > plan->max_F) return fail(GROOT_EINVAL, std::string(who) + "the input width exceeds the max_F given to groot_plan_upload");
    if (plan->dev.n_cols != plan->dev.n)
        return fail(GROOT_EINVAL, std::string(who) + "the plan's columns were renamed to global rows (groot_plan_use_global_columns)");
    const char *a = (const char *)X_dev, *b = (const char *)H_dev;
    const int64_t x_bytes = plan->dev.n * (int64_t)F_in * 4, h_bytes = plan->dev.n * (int64_t)F_out * 4;
    if (a < b + h_bytes && b < a + x_bytes) return fail(GROOT_EINVAL, std::string(who) + "X and H overlap");
    int err = 0;
    if (wavefronts) {
        // high-degree rows: their aggregation goes to the plan's side buffer, the layer kernel picks it up there
        DevicePlan hd = plan->dev;
        hd.chunks = plan->dev.chunks_rank;
        hd.split_rows = plan->dev.split_rows_rank;
        if (hd.n_chunks) err = launch_hd(hd, X_dev, hd.hd_agg, F_in, hip_stream);
        if (!err && hd.n_split_rows) err = launch_hd_finish(hd, hd.hd_agg, F_in, hip_stream);
        if (!err) err = launch_sage_pipe(plan->dev, X_dev, H_dev, Wn_dev, Ws_dev, bias_dev, relu ? 1 : 0, F_in, F_out,
                                         tuning().sage_pieces.load(), 0, hip_stream);
    } else {
        // the kernel for explicit weights (64 -> 64): high-degree sums go to H first and are picked up from there
        if (plan->dev.n_chunks) err = launch_hd(plan->dev, X_dev, H_dev, F_in, hip_stream);
        if (!err && plan->dev.n_split_rows) err = launch_hd_finish(plan->dev, H_dev, F_in, hip_stream);
        if (!err) err = launch_sage(plan->dev, X_dev, H_dev, Wn_dev, Ws_dev, bias_dev, relu ? 1 : 0, hip_stream);
    }
    if (err) return fail(GROOT_EHIP, std::string(who) + "launch failed: " + hip_error_text(err));
    return GROOT_OK;
}

extern "C" groot_status groot_sage_layer_forward(const groot_plan *plan, const float *X_dev, const float *Wn_dev,
                                                 const float *Ws_dev, const float *bias_dev, int32_t relu,
                                                 float *H_dev, int32_t F, void *hip_stream)
{
    if (F != 64 && F != 32) return fail(GROOT_EINVAL, "groot_sage_layer_forward: F must be 64 or 32");
    return groot_sage_layer_forward_io(plan, X_dev, Wn_dev, Ws_dev, bias_dev, relu, H_dev, F, F, hip_stream);
}

extern "C" groot_status groot_plan_lists_device(const groot_plan *plan, uint8_t *row_class_dev, int32_t *hd_rows_dev,
                                                int32_t *ld_rows_dev, int32_t *ld_rows_by_degree_dev,
                                                int64_t *ld_deg_offsets_dev, int64_t *counts_dev, void *hip_stream)
{
    if (!plan) return fail(GROOT_EINVAL, "groot_plan_lists_device: NULL plan");
    if (!row_class_dev || !hd_rows_dev || !ld_rows_dev || !ld_rows_by_degree_dev || !ld_deg_offsets_dev || !counts_dev)
        return fail(GROOT_EINVAL, "groot_plan_lists_device: NULL output pointer");
    if (!plan->resident) return fail(GROOT_EINVAL, "groot_plan_lists_device: plan is not on the device (call groot_plan_upload)");
    if (plan->threshold > kPlanDeviceMaxThreshold)
        return fail(GROOT_ERANGE, "groot_plan_lists_device: degree threshold above " + std::to_string(kPlanDeviceMaxThreshold));
    int err = launch_plan_device(plan->dev.rowptr, plan->dev.n, plan->threshold, row_class_dev, hd_rows_dev, ld_rows_dev,
                                 ld_rows_by_degree_dev, ld_deg_offsets_dev, counts_dev, hip_stream);
    if (err == kErrOutOfDeviceMemory) return fail(GROOT_ENOMEM, "groot_plan_lists_device: scratch allocation failed");
    if (err) return fail(GROOT_EHIP, std::string("groot_plan_lists_device: ") + hip_error_text(err));
    return GROOT_OK;
}

extern "C" groot_status groot_plan_lists_device_static(const groot_plan *plan, uint8_t *row_class_dev,
                                                       int32_t *hd_rows_dev, int32_t *ld_rows_dev,
                                                       int32_t *ld_rows_by_degree_dev, int64_t *ld_deg_offsets_dev,
                                                       int64_t *counts_dev, void *hip_stream)
{
    if (!plan) return fail(GROOT_EINVAL, "groot_plan_lists_device_static: NULL plan");
    if (!row_class_dev || !hd_rows_dev || !ld_rows_dev || !ld_rows_by_degree_dev || !ld_deg_offsets_dev || !counts_dev)
        return fail(GROOT_EINVAL, "groot_plan_lists_device_static: NULL output pointer");
    if (!plan->resident)
        return fail(GROOT_EINVAL, "groot_plan_lists_device_static: plan is not on the device (call groot_plan_upload)");
    if (plan->threshold > kPlanDeviceMaxThreshold)
        return fail(GROOT_ERANGE, "groot_plan_lists_device_static: degree threshold above " + std::to_string(kPlanDeviceMaxThreshold));
    const size_t need = plan_static_scratch_needed(plan->dev.n, plan->threshold);
    if (need > kPlanStaticScratchBytes)
        return fail(GROOT_ERANGE, "groot_plan_lists_device_static: " + std::to_string(plan->dev.n) + " rows at threshold " +
                                      std::to_string(plan->threshold) + " need " + std::to_string(need) +
                                      " bytes of scratch, the built-in array holds " + std::to_string(kPlanStaticScratchBytes) +
                                      " (use groot_plan_lists_device)");
    int err = launch_plan_device_static(plan->dev.rowptr, plan->dev.n, plan->threshold, row_class_dev, hd_rows_dev,
                                        ld_rows_dev, ld_rows_by_degree_dev, ld_deg_offsets_dev, counts_dev, hip_stream);
    if (err) return fail(GROOT_EHIP, std::string("groot_plan_lists_device_static: ") + hip_error_text(err));
    return GROOT_OK;
}

extern "C" groot_status groot_plan_use_global_columns(groot_plan *plan, const int64_t *global_id_dev, int64_t n_global,
                                                      void *hip_stream)
{
    if (!plan || !global_id_dev) return fail(GROOT_EINVAL, "groot_plan_use_global_columns: NULL argument");
    if (!plan->resident) return fail(GROOT_EINVAL, "groot_plan_use_global_columns: plan is not on the device (call groot_plan_upload)");
    if (plan->dev.n_cols != plan->dev.n) return fail(GROOT_EINVAL, "groot_plan_use_global_columns: the columns were renamed before");
    if (n_global < plan->dev.n) return fail(GROOT_EINVAL, "groot_plan_use_global_columns: n_global is smaller than the plan's own row count");
    if (n_global > std::numeric_limits<int32_t>::max()) return fail(GROOT_ERANGE, "groot_plan_use_global_columns: n_global does not fit int32 columns");
    // the compact column codes name local rows: the plan goes back to the plain arrays
    plan->dev.compressed = 0;
    int err = launch_col_map(plan->dev.col, plan->dev.nnz, global_id_dev, hip_stream);
    if (err) return fail(GROOT_EHIP, std::string("groot_plan_use_global_columns: launch failed: ") + hip_error_text(err));
    plan->dev.n_cols = n_global;
    return GROOT_OK;
}

extern "C" void groot_plan_free(groot_plan *plan)
{
    if (!plan) return;
    if (plan->resident) release_device(plan);
    delete plan;
}

// ---------------------------------------------------------------------------
// partition + boundary edge re-growth
// ---------------------------------------------------------------------------
namespace {

// Sub-graph of one part.  local_of is a scratch array of n entries, all -1 on
// entry and on exit.
void build_part(const groot_graph &g, const int32_t *part_of, int32_t p, bool regrow,
                const std::vector<int32_t> &owned, std::vector<int32_t> &local_of,
                groot_parts::Part &out)
{
    const int64_t n_owned = (int64_t)owned.size();
    for (int64_t k = 0; k < n_owned; ++k) local_of[owned[k]] = (int32_t)k;
    // boundary nodes: columns of owned rows that live in another part
    std::vector<int32_t> halo;
    if (regrow) {
        for (int32_t v : owned)
            for (int64_t q = g.rowptr[v]; q < g.rowptr[v + 1]; ++q) {
                int32_t u = g.col[q];
                if (part_of[u] != p && local_of[u] == -1) { local_of[u] = -2; halo.push_back(u); }
            }
        std::sort(halo.begin(), halo.end());
        for (size_t k = 0; k < halo.size(); ++k) local_of[halo[k]] = (int32_t)(n_owned + (int64_t)k);
    }
    const int64_t n_halo = (int64_t)halo.size(), n_loc = n_owned + n_halo;
    out.n_owned = n_owned;
    out.n_halo = n_halo;
    out.global_id.resize(n_loc);
    for (int64_t k = 0; k < n_owned; ++k) out.global_id[k] = owned[k];
    for (int64_t k = 0; k < n_halo; ++k) out.global_id[n_owned + k] = halo[k];

    groot_graph &s = out.sub;
    s.n = s.n1 = n_loc;
    s.weight_mode = g.weight_mode;
    s.rowptr.assign(n_loc + 1, 0);
    // row lengths
    int64_t crossing = 0;
    for (int64_t k = 0; k < n_owned; ++k) {
        int32_t v = owned[k];
        int64_t len = 0;
        for (int64_t q = g.rowptr[v]; q < g.rowptr[v + 1]; ++q) {
            int32_t lu = local_of[g.col[q]];
            if (lu >= 0) { ++len; if (lu >= n_owned) ++crossing; }
        }
        s.rowptr[k + 1] = len;
    }
    for (int64_t k = 0; k < n_halo; ++k) {
        int32_t u = halo[k];
        int64_t len = 0;
        for (int64_t q = g.rowptr[u]; q < g.rowptr[u + 1]; ++q) {
            int32_t v = g.col[q];
            if (v == u) { ++len; continue; }
            int32_t lv = local_of[v];
            if (lv >= 0 && lv < n_owned) {
                ++len;
                // an edge stored only in this direction is a crossing pair not yet counted
                const int32_t *b = &g.col[g.rowptr[v]], *e = &g.col[g.rowptr[v + 1]];
                if (!std::binary_search(b, e, u)) ++crossing;
            }
        }
        s.rowptr[n_owned + k + 1] = len;
    }
    for (int64_t k = 0; k < n_loc; ++k) s.rowptr[k + 1] += s.rowptr[k];
    s.nnz = s.rowptr[n_loc];
    s.col.resize(s.nnz);
    s.val.resize(s.nnz);
    out.n_crossing = crossing;
    const bool explicit_w = g.weight_mode == WeightMode::Explicit;
    // Local ids are monotone in the global id inside the owned block and inside
    // the boundary block, so a row sorted by global column becomes sorted by
    // local column by writing its owned columns first and its boundary columns after.
    for (int64_t k = 0; k < n_loc; ++k) {
        int32_t v = (int32_t)out.global_id[k];
        const bool row_owned = k < n_owned;
        int64_t w = s.rowptr[k];
        for (int pass = 0; pass < 2; ++pass)
            for (int64_t q = g.rowptr[v]; q < g.rowptr[v + 1]; ++q) {
                int32_t c = g.col[q], lc = local_of[c];
                if (lc < 0) continue;
                bool col_owned = lc < n_owned;
                if (col_owned != (pass == 0)) continue;
                if (!row_owned && !col_owned && c != v) continue;   // boundary-boundary edge: not in E_p+
                s.col[w] = lc;
                if (explicit_w) s.val[w] = g.val[q];
                ++w;
            }
    }
    if (!explicit_w) fill_uniform_weights(s);
    for (int32_t v : owned) local_of[v] = -1;
    for (int32_t u : halo) local_of[u] = -1;
}

}  // namespace

extern "C" groot_status groot_partition_regrow(const groot_graph *g, int32_t num_parts,
                                               const int32_t *part_of, uint32_t flags, groot_parts **out)
{
    if (!g || !out) return fail(GROOT_EINVAL, "groot_partition_regrow: NULL argument");
    if (num_parts < 1 || num_parts > g->n) return fail(GROOT_EINVAL, "groot_partition_regrow: num_parts must be in [1,N]");
    if (flags & ~GROOT_REGROW) return fail(GROOT_EINVAL, "groot_partition_regrow: unknown flag bits");
    try {
        const int64_t n = g->n;
        const int32_t P = num_parts;
        std::vector<int32_t> rule;
        if (!part_of) {
            rule.resize(n);
            const int64_t n1 = g->n1;
            parallel_for(n, 1 << 18, [&](int64_t lo, int64_t hi) {
                for (int64_t v = lo; v < hi; ++v) {
                    int64_t q = ((v % n1) * P) / n1;
                    rule[v] = (int32_t)std::min<int64_t>(q, P - 1);
                }
            });
            part_of = rule.data();
        } else {
            for (int64_t v = 0; v < n; ++v)
                if (part_of[v] < 0 || part_of[v] >= P)
                    return fail(GROOT_EINVAL, "groot_partition_regrow: part_of[" + std::to_string(v) + "] outside [0,P)");
        }
        // owned lists by counting
        std::vector<int64_t> count(P + 1, 0);
        for (int64_t v = 0; v < n; ++v) ++count[part_of[v] + 1];
        std::vector<std::vector<int32_t>> owned(P);
        for (int32_t p = 0; p < P; ++p) owned[p].reserve(count[p + 1]);
        for (int64_t v = 0; v < n; ++v) owned[part_of[v]].push_back((int32_t)v);

        std::unique_ptr<groot_parts> res(new groot_parts);
        res->parts.resize(P);
        // parts are independent: a few worker threads, each with its own scratch map
        unsigned hw = std::thread::hardware_concurrency();
        int workers = (int)std::max(1u, std::min<unsigned>({hw ? hw : 1u, (unsigned)P, 8u}));
        if (n < (1 << 20)) workers = 1;
        std::atomic<int32_t> next{0};
        std::atomic<bool> oom{false};
        auto work = [&] {
            try {
                std::vector<int32_t> local_of(n, -1);
                for (int32_t p = next++; p < P; p = next++)
                    build_part(*g, part_of, p, flags & GROOT_REGROW, owned[p], local_of, res->parts[p]);
            } catch (const std::bad_alloc &) {
                oom = true;
            }
        };
        if (workers == 1) work();
        else {
            std::vector<std::thread> th;
            for (int t = 0; t < workers; ++t) th.emplace_back(work);
            for (auto &t : th) t.join();
        }
        if (oom) return fail(GROOT_ENOMEM, "groot_partition_regrow: out of host memory");
        *out = res.release();
        return GROOT_OK;
    } catch (const std::bad_alloc &) {
        return fail(GROOT_ENOMEM, "groot_partition_regrow: out of host memory");
    }
}

extern "C" int32_t groot_parts_count(const groot_parts *parts) { return parts ? (int32_t)parts->parts.size() : 0; }

extern "C" groot_status groot_parts_view(const groot_parts *parts, int32_t p, int64_t *n_owned, int64_t *n_halo,
                                         int64_t *n_crossing, const int64_t **global_id, const groot_graph **sub)
{
    if (!parts) return fail(GROOT_EINVAL, "groot_parts_view: NULL parts");
    if (p < 0 || p >= (int32_t)parts->parts.size()) return fail(GROOT_EINVAL, "groot_parts_view: part index out of range");
    const groot_parts::Part &pt = parts->parts[p];
    if (n_owned) *n_owned = pt.n_owned;
    if (n_halo) *n_halo = pt.n_halo;
    if (n_crossing) *n_crossing = pt.n_crossing;
    if (global_id) *global_id = pt.global_id.data();
    if (sub) *sub = &pt.sub;
    return GROOT_OK;
}

extern "C" void groot_parts_free(groot_parts *parts) { delete parts; }

// ---------------------------------------------------------------------------
// partition + boundary edge re-growth on the device
// ---------------------------------------------------------------------------
extern "C" groot_status groot_partition_regrow_device(const groot_plan *plan, int32_t num_parts,
                                                      const int32_t *part_of_dev, uint32_t flags, int32_t p,
                                                      void *hip_stream, groot_dev_part **out)
{
    if (!plan || !out) return fail(GROOT_EINVAL, "groot_partition_regrow_device: NULL argument");
    if (!plan->resident) return fail(GROOT_EINVAL, "groot_partition_regrow_device: plan is not on the device (call groot_plan_upload)");
    const int64_t n = plan->dev.n;
    if (plan->dev.n_cols != n)
        return fail(GROOT_EINVAL, "groot_partition_regrow_device: the plan's columns were renamed to global rows (groot_plan_use_global_columns)");
    if (num_parts < 1 || num_parts > n) return fail(GROOT_EINVAL, "groot_partition_regrow_device: num_parts must be in [1,N]");
    if (p < 0 || p >= num_parts) return fail(GROOT_EINVAL, "groot_partition_regrow_device: part index outside [0,P)");
    if (flags & ~GROOT_REGROW) return fail(GROOT_EINVAL, "groot_partition_regrow_device: unknown flag bits");
    std::unique_ptr<groot_dev_part> part(new (std::nothrow) groot_dev_part);
    if (!part) return fail(GROOT_ENOMEM, "groot_partition_regrow_device: out of host memory");
    part->weight_mode = (WeightMode)plan->dev.graph_weight_mode;
    const int64_t n1 = plan->g ? plan->g->n1 : n;
    int err = launch_regrow_device(plan->dev, n1, num_parts, part_of_dev, p, (flags & GROOT_REGROW) ? 1 : 0, hip_stream,
                                   &part->d);
    if (err == kErrOutOfDeviceMemory) return fail(GROOT_ENOMEM, "groot_partition_regrow_device: device allocation failed");
    if (err == kErrBadPartId) return fail(GROOT_EINVAL, "groot_partition_regrow_device: a part_of entry lies outside [0,P)");
    if (err) return fail(GROOT_EHIP, std::string("groot_partition_regrow_device: ") + hip_error_text(err));
    *out = part.release();
    return GROOT_OK;
}

extern "C" groot_status groot_dev_part_view(const groot_dev_part *part, int64_t *n_owned, int64_t *n_halo,
                                            int64_t *n_crossing, int64_t *nnz, const int64_t **global_id_dev,
                                            const int64_t **rowptr_dev, const int32_t **col_dev, const float **val_dev)
{
    if (!part) return fail(GROOT_EINVAL, "groot_dev_part_view: NULL part");
    if (n_owned) *n_owned = part->d.n_owned;
    if (n_halo) *n_halo = part->d.n_halo;
    if (n_crossing) *n_crossing = part->d.n_crossing;
    if (nnz) *nnz = part->d.nnz;
    if (global_id_dev) *global_id_dev = part->d.global_id;
    if (rowptr_dev) *rowptr_dev = part->d.rowptr;
    if (col_dev) *col_dev = part->d.col;
    if (val_dev) *val_dev = part->d.val;
    return GROOT_OK;
}

extern "C" groot_status groot_dev_part_download(const groot_dev_part *part, int64_t *global_id_host,
                                                int64_t *rowptr_host, int32_t *col_host, float *val_host,
                                                void *hip_stream)
{
    if (!part) return fail(GROOT_EINVAL, "groot_dev_part_download: NULL part");
    const DevicePart &d = part->d;
    const int64_t n = d.n_owned + d.n_halo;
    if ((rowptr_host || col_host || val_host) && part->csr_moved)
        return fail(GROOT_EINVAL, "groot_dev_part_download: the part's sub-graph has moved into a plan");
    if (val_host && !d.val) return fail(GROOT_EINVAL, "groot_dev_part_download: the sub-graph has no weight array (row-uniform weights)");
    int err = 0;
    if (!err && global_id_host) err = device_download(global_id_host, d.global_id, (size_t)n * 8, hip_stream);
    if (!err && rowptr_host) err = device_download(rowptr_host, d.rowptr, (size_t)(n + 1) * 8, hip_stream);
    if (!err && col_host) err = device_download(col_host, d.col, (size_t)d.nnz * 4, hip_stream);
    if (!err && val_host) err = device_download(val_host, d.val, (size_t)d.nnz * 4, hip_stream);
    if (err) return fail(GROOT_EHIP, std::string("groot_dev_part_download: ") + hip_error_text(err));
    return GROOT_OK;
}

extern "C" void groot_dev_part_free(groot_dev_part *part)
{
    if (!part) return;
    free_device_part(part->d);
    delete part;
}

namespace {
// frees device memory on scope exit unless released
struct DevBuf {
    void *p = nullptr;
    ~DevBuf() { dev_free(p); }
    int alloc(size_t bytes) { return dev_alloc(&p, bytes ? bytes : 1); }
    template <class T> T *as() const { return (T *)p; }
    void *release() { void *q = p; p = nullptr; return q; }
};
}  // namespace

extern "C" groot_status groot_dev_part_plan(groot_dev_part *part, int32_t degree_threshold, int32_t max_F,
                                            void *hip_stream, groot_plan **out)
{
    const char *who = "groot_dev_part_plan: ";
    if (!part || !out) return fail(GROOT_EINVAL, std::string(who) + "NULL argument");
    if (part->csr_moved) return fail(GROOT_EINVAL, std::string(who) + "the part's sub-graph already belongs to a plan");
    if (degree_threshold < 1) return fail(GROOT_EINVAL, std::string(who) + "degree_threshold must be >= 1");
    if (degree_threshold > kPlanDeviceMaxThreshold)
        return fail(GROOT_ERANGE, std::string(who) + "degree threshold above " + std::to_string(kPlanDeviceMaxThreshold));
    if (max_F < 4 || max_F > 512 || max_F % 4) return fail(GROOT_EINVAL, std::string(who) + "max_F must be a multiple of 4 in [4,512]");
    const int32_t T = degree_threshold;
    const int64_t n = part->d.n_owned + part->d.n_halo;
    if (n < 1) return fail(GROOT_EINVAL, std::string(who) + "the part has no rows");
    try {
        std::unique_ptr<groot_plan> pl(new groot_plan);
        // lists on the device; only the high-degree rows and the degree offsets are needed here
        DevBuf row_class, hd_rows, ld_rows, by_degree, deg_offsets, counts;
        if (row_class.alloc((size_t)n) || hd_rows.alloc((size_t)n * 4) || ld_rows.alloc((size_t)n * 4) ||
            by_degree.alloc((size_t)n * 4) || deg_offsets.alloc((size_t)(T + 1) * 8) || counts.alloc(16))
            return fail(GROOT_ENOMEM, std::string(who) + "device allocation of the plan lists failed");
        int err = launch_plan_device(part->d.rowptr, n, T, row_class.as<uint8_t>(), hd_rows.as<int32_t>(),
                                     ld_rows.as<int32_t>(), by_degree.as<int32_t>(), deg_offsets.as<int64_t>(),
                                     counts.as<int64_t>(), hip_stream);
        if (err == kErrOutOfDeviceMemory) return fail(GROOT_ENOMEM, std::string(who) + "scratch allocation failed");
        if (err) return fail(GROOT_EHIP, std::string(who) + hip_error_text(err));
        int64_t h_counts[2] = {0, 0};
        std::vector<int64_t> offs(T + 1, 0);
        if ((err = device_download(h_counts, counts.p, sizeof h_counts, hip_stream)) ||
            (err = device_download(offs.data(), deg_offsets.p, offs.size() * 8, hip_stream)))
            return fail(GROOT_EHIP, std::string(who) + hip_error_text(err));
        const int64_t n_hd = h_counts[0], n_ld = h_counts[1];
        if (n_hd < 0 || n_ld < 0 || n_hd + n_ld != n) return fail(GROOT_EHIP, std::string(who) + "inconsistent row counts from the device");
        // the schedule of the high-degree rows, cut and ordered on the device too: only four sizes come back
        DeviceHdSchedule sched;
        err = launch_hd_schedule_device(part->d.rowptr, part->d.col, hd_rows.as<int32_t>(), n_hd, tuning().hd_chunk,
                                        hip_stream, &sched);
        if (err == kErrOutOfDeviceMemory) return fail(GROOT_ENOMEM, std::string(who) + "device allocation of the HD schedule failed");
        if (err == kErrTooManyPieces) return fail(GROOT_ERANGE, std::string(who) + "too many high-degree pieces");
        if (err) return fail(GROOT_EHIP, std::string(who) + hip_error_text(err));
        DevicePlan &d = pl->dev;
        d.chunks = sched.chunks;                         // the plan owns them from here on (release_device)
        d.chunks_rank = sched.chunks_rank;
        d.split_rows = sched.split_rows;
        d.split_rows_rank = sched.split_rows_rank;
        pl->n_partials = sched.n_partials;
        const std::vector<float> zeros(kZeroRowFloats + kTrashFloats, 0.0f);
        groot_status st;
        if ((st = to_device(&d.zero_row, zeros.data(), zeros.size(), "zero row")) != GROOT_OK ||
            (st = to_device<float>(&d.partials, nullptr, (size_t)sched.n_partials * max_F, "HD partial sums")) != GROOT_OK ||
            (st = to_device<float>(&d.hd_agg, nullptr, (size_t)n_hd * max_F, "high-degree sums of the fused layer")) != GROOT_OK ||
            (st = to_device<int32_t>(&d.hd_rows, nullptr, (size_t)n_hd, "high-degree row list")) != GROOT_OK) {
            std::string keep = groot_last_error();
            release_device(pl.get());
            set_error(keep);
            return st;
        }
        if (n_hd && (err = device_copy(d.hd_rows, hd_rows.p, (size_t)n_hd * 4, hip_stream))) {
            release_device(pl.get());
            return fail(GROOT_EHIP, std::string(who) + hip_error_text(err));
        }
        d.n_hd_rows = n_hd;
        d.n = d.n_cols = n;
        d.nnz = part->d.nnz;
        d.threshold = T;
        d.xcd_remap = tuning().xcd_remap;
        d.weight_mode = d.graph_weight_mode = (int)part->weight_mode;
        d.n_tiles = (n + kRowsPerLdTile - 1) / kRowsPerLdTile;
        d.n_chunks = sched.n_chunks;
        d.nnz_hd = sched.nnz_hd;
        d.n_split_rows = sched.n_split_rows;
        d.n_partials = sched.n_partials;
        {
            auto at_most = [&](int32_t len) { return offs[std::min<int32_t>(len + 1, T)]; };
            const PipeChoice ch = choose_ld_kernel(tuning().ld_pipeline, n_ld, at_most);
            d.ld_pipelined = ch.pipelined;
            d.pipe_depth = ch.depth;
            d.sage_depth = (n_ld - at_most(5)) * 2000 <= n_ld ? 5 : 6;
            const int64_t first_mid = at_most(ch.depth);
            d.n_mid_rows = ch.pipelined ? n_ld - first_mid : 0;
            if (d.n_mid_rows) {             // the tail of the degree-sorted list, which is on the device already
                if ((st = to_device<int32_t>(&d.mid_rows, nullptr, (size_t)d.n_mid_rows, "long low-degree rows")) != GROOT_OK ||
                    (err = device_copy(d.mid_rows, by_degree.as<int32_t>() + first_mid, (size_t)d.n_mid_rows * 4, hip_stream))) {
                    std::string keep = err ? std::string(who) + hip_error_text(err) : std::string(groot_last_error());
                    release_device(pl.get());
                    set_error(keep);
                    return err ? GROOT_EHIP : st;
                }
            }
        }
        // the sub-graph moves into the plan
        d.rowptr = part->d.rowptr;
        d.col = part->d.col;
        d.val = part->d.val;
        part->d.rowptr = nullptr;
        part->d.col = nullptr;
        part->d.val = nullptr;
        part->csr_moved = true;
        if (d.ld_pipelined && tuning().csr_compress) {
            err = launch_csr_compress(d, hd_rows.as<int32_t>(), n_hd, hip_stream);
            if (!err && d.compressed) err = pipe_compact_prepare();
            if (err) {
                release_device(pl.get());               // the sub-graph's arrays are the plan's by now
                return fail(GROOT_EHIP, std::string(who) + "compact CSR: " + hip_error_text(err));
            }
        }
        pl->g = nullptr;
        pl->threshold = T;
        pl->max_F = max_F;
        pl->resident = true;
        *out = pl.release();
        return GROOT_OK;
    } catch (const std::bad_alloc &) {
        return fail(GROOT_ENOMEM, std::string(who) + "out of host memory");
    }
}

// ---------------------------------------------------------------------------
// row gather / scatter, tuning, errors
// ---------------------------------------------------------------------------
extern "C" groot_status groot_rows_gather(const int64_t *ids_dev, int64_t n, const float *X_dev, float *out_dev,
                                          int32_t F, void *hip_stream)
{
    if (n < 0) return fail(GROOT_EINVAL, "groot_rows_gather: negative n");
    if (n == 0) return GROOT_OK;
    if (!ids_dev) return fail(GROOT_EINVAL, "groot_rows_gather: NULL ids");
    groot_status st = check_features("groot_rows_gather", X_dev, out_dev, F);
    if (st != GROOT_OK) return st;
    int err = launch_rows_gather(ids_dev, n, X_dev, out_dev, F, hip_stream);
    if (err) return fail(GROOT_EHIP, std::string("groot_rows_gather: launch failed: ") + hip_error_text(err));
    return GROOT_OK;
}

extern "C" groot_status groot_rows_scatter(const int64_t *ids_dev, int64_t n, const float *in_dev, float *Y_dev,
                                           int32_t F, void *hip_stream)
{
    if (n < 0) return fail(GROOT_EINVAL, "groot_rows_scatter: negative n");
    if (n == 0) return GROOT_OK;
    if (!ids_dev) return fail(GROOT_EINVAL, "groot_rows_scatter: NULL ids");
    groot_status st = check_features("groot_rows_scatter", in_dev, Y_dev, F);
    if (st != GROOT_OK) return st;
    int err = launch_rows_scatter(ids_dev, n, in_dev, Y_dev, F, hip_stream);
    if (err) return fail(GROOT_EHIP, std::string("groot_rows_scatter: launch failed: ") + hip_error_text(err));
    return GROOT_OK;
}

extern "C" groot_status groot_plan_hd_pieces(const groot_plan *plan, int64_t capacity, int64_t *begin_host,
                                             int32_t *len_host, int32_t *row_host, int32_t *slot_host)
{
    const char *who = "groot_plan_hd_pieces: ";
    if (!plan) return fail(GROOT_EINVAL, std::string(who) + "NULL plan");
    if (!plan->resident && !plan->g) return fail(GROOT_EINVAL, std::string(who) + "the plan is not uploaded");
    const int64_t n = plan->resident ? plan->dev.n_chunks : (int64_t)plan->chunks.size();
    if (capacity < n) return fail(GROOT_EINVAL, std::string(who) + "capacity below the number of pieces");
    if (n == 0) return GROOT_OK;
    try {
        std::vector<HdChunk> chunks((size_t)n);
        if (plan->resident) {
            const int err = device_download(chunks.data(), plan->dev.chunks, (size_t)n * sizeof(HdChunk), nullptr);
            if (err) return fail(GROOT_EHIP, std::string(who) + hip_error_text(err));
        } else {
            chunks = plan->chunks;                      // a host plan before its upload: the list it will upload
        }
        for (int64_t c = 0; c < n; ++c) {
            if (begin_host) begin_host[c] = chunks[c].begin;
            if (len_host) len_host[c] = chunks[c].len;
            if (row_host) row_host[c] = chunks[c].row;
            if (slot_host) slot_host[c] = chunks[c].slot;
        }
    } catch (const std::bad_alloc &) {
        return fail(GROOT_ENOMEM, std::string(who) + "out of host memory");
    }
    return GROOT_OK;
}

extern "C" groot_status groot_plan_query(const groot_plan *plan, const char *what, int64_t *value)
{
    if (!plan || !what || !value) return fail(GROOT_EINVAL, "groot_plan_query: NULL argument");
    const std::string k(what);
    if (!plan->resident && plan->g && (k == "hd_pieces" || k == "hd_partials")) {
        *value = k == "hd_pieces" ? (int64_t)plan->chunks.size() : plan->n_partials;
        return GROOT_OK;                                  // the schedule of a host plan, before its upload
    }
    if (!plan->resident) return fail(GROOT_EINVAL, "groot_plan_query: plan is not on the device (call groot_plan_upload)");
    if (k == "ld_pipelined") *value = plan->dev.ld_pipelined;
    else if (k == "weight_mode") *value = plan->dev.weight_mode;
    else if (k == "hd_pieces") *value = plan->dev.n_chunks;
    else if (k == "hd_partials") *value = plan->dev.n_partials;
    else if (k == "nnz_hd") *value = plan->dev.nnz_hd;
    else if (k == "pipe_depth") *value = plan->dev.pipe_depth;
    else if (k == "csr_compressed") *value = plan->dev.compressed;
    else if (k == "uncoded_rows") *value = plan->dev.n_bad_rows;
    else if (k == "mid_rows") *value = plan->dev.n_mid_rows;
    else if (k == "csr_bytes" || k == "csr_bytes_ld" || k == "csr_bytes_hd") {
        // what the kernels read of the graph per execute: every row pointer and every entry's column index, the
        // entry's weight only when the kernels take the weights from the array; the HD kernel reads its pieces'
        // descriptors instead of row pointers
        const DevicePlan &d = plan->dev;
        const int64_t w_bytes = d.weight_mode == (int)WeightMode::Explicit ? 4 : 0;
        const int64_t per_entry = 4 + w_bytes;
        // the pipelined LD kernel (feature widths 32, 64, 128) reads the compact form when the plan has one
        const bool compact = d.ld_pipelined && d.compressed;
        const int64_t ld = compact ? 4 * (d.n + 1) + (2 + w_bytes) * (d.nnz - d.nnz_hd)
                                   : 8 * (d.n + 1) + per_entry * (d.nnz - d.nnz_hd);
        const int64_t hd = per_entry * d.nnz_hd + (int64_t)sizeof(HdChunk) * d.n_chunks;
        *value = k == "csr_bytes_ld" ? ld : k == "csr_bytes_hd" ? hd : ld + hd;
    }
    else return fail(GROOT_EINVAL, "groot_plan_query: unknown name '" + k + "'");
    return GROOT_OK;
}

extern "C" groot_status groot_set_tuning(const char *name, int64_t value)
{
    if (!name) return fail(GROOT_EINVAL, "groot_set_tuning: NULL name");
    std::string k(name);
    if (k == "xcd_remap") { tuning().xcd_remap = value ? 1 : 0; return GROOT_OK; }
    if (k == "pipe_depth") {
        if (value != 0 && (value < kPipeMinDepth || value > kPipeMaxDepth))
            return fail(GROOT_EINVAL, "groot_set_tuning: pipe_depth must be 0 or 5..8");
        tuning().pipe_depth = (int)value;
        return GROOT_OK;
    }
    if (k == "ld_pipeline") {
        if (value < -1 || value > 1) return fail(GROOT_EINVAL, "groot_set_tuning: ld_pipeline must be -1, 0 or 1");
        tuning().ld_pipeline = (int)value;
        return GROOT_OK;
    }
    if (k == "csr_compress") {
        if (value < 0 || value > 1) return fail(GROOT_EINVAL, "groot_set_tuning: csr_compress must be 0 or 1");
        tuning().csr_compress = (int)value;
        return GROOT_OK;
    }
    if (k == "sage_split" || k == "sage_kernel" || k == "uniform_detect") {
        if (value < 0 || value > 1) return fail(GROOT_EINVAL, "groot_set_tuning: " + k + " must be 0 or 1");
        (k == "sage_split" ? tuning().sage_split : k == "sage_kernel" ? tuning().sage_kernel : tuning().uniform_detect).store((int)value);
        return GROOT_OK;
    }
    if (k == "sage_pieces") {
        if (value != 2 && value != 3) return fail(GROOT_EINVAL, "groot_set_tuning: sage_pieces must be 2 or 3");
        tuning().sage_pieces = (int)value;
        return GROOT_OK;
    }
    if (k == "sage_gap") {
        if (value < 0 || value > 4) return fail(GROOT_EINVAL, "groot_set_tuning: sage_gap must be in [0,4]");
        tuning().sage_gap = (int)value;
        return GROOT_OK;
    }
    if (k == "hd_chunk") {
        if (value < 64 || value > 4096) return fail(GROOT_EINVAL, "groot_set_tuning: hd_chunk must be in [64,4096]");
        tuning().hd_chunk = (int)value;
        return GROOT_OK;
    }
    return fail(GROOT_EINVAL, "groot_set_tuning: unknown knob '" + k + "'");
}

extern "C" const char *groot_last_error(void) { return g_error.c_str(); }
