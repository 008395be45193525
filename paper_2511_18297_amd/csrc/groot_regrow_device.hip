// Device-side partition with boundary edge re-growth for gfx950 (paper: Section "GNN and Edge Re-growth
// After Partition", Eq. (1), Eq. (2), Algorithm 1), one part per call, from the CSR that an uploaded plan
// keeps on the device.  All integer work; the result is bit-identical to the host's groot_partition_regrow.
//
// For part p with node set S_p:
//   rg_mark      every owned row flags the columns that live in another part: B_p (Eq. (1))
//   rg_count / rg_scan_counts / rg_scatter
//                stable compaction of the owned ids and of the flagged ids, both ascending: the local
//                numbering S_p first, B_p after (global_id), and its inverse (local_of)
//   rg_row_len (+ rg_row_len_long for rows of many entries, one wavefront per row)
//                stored length of every local row: an owned row keeps its whole neighbourhood, a boundary
//                row keeps its self-loop and its edges into S_p (the crossing edges C_p of Eq. (2));
//                crossing pairs are counted on the way
//   rg_len_sums / rg_scan_sums / rg_len_write
//                exclusive prefix of the lengths: the sub-graph's row pointer
//   rg_fill (+ rg_fill_long)
//                the sub-graph's columns (and weights): local ids are monotone in the global id inside
//                S_p and inside B_p, so a row sorted by global column becomes sorted by local column by
//                writing its owned columns first and its boundary columns after
//   plus gather helpers for the high-degree schedule of a plan that is built from device arrays.
#include "groot_device.h"

namespace groot {

constexpr int kRgRowsPerWave = 1024;
constexpr int kRgRowsPerBlock = kRgRowsPerWave * kWavesPerBlock;   // 4096
constexpr int kRgItems = kRgRowsPerBlock / kBlock;                 // 16 consecutive items per thread in the scans
constexpr int32_t kRgNone = -1, kRgHalo = -2;
constexpr int kRgShort = 16;                                       // longest row that one lane walks alone
constexpr int kRgUnroll = 4;                                       // 64-entry chunks of a long row in flight
constexpr int kRgLongBlocks = 2048;                                // workgroups that share the long rows
constexpr int kRgCrossSlots = 64;                                  // counters that share the crossing-pair atomics

// adds the workgroup's sum of cross to one of kRgCrossSlots counters (every thread of the workgroup calls)
__device__ __forceinline__ void rg_add_crossing(int64_t cross, unsigned long long *__restrict__ slots)
{
    __shared__ int64_t s_cross[kWavesPerBlock];
    for (int off = kWave / 2; off > 0; off >>= 1) cross += __shfl_down(cross, off);
    if (threadIdx.x % kWave == 0) s_cross[threadIdx.x / kWave] = cross;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t t = 0;
        for (int w = 0; w < kWavesPerBlock; ++w) t += s_cross[w];
        if (t) atomicAdd(&slots[blockIdx.x % kRgCrossSlots], (unsigned long long)t);
    }
}

struct RgGraph {
    const int64_t *rowptr;
    const int32_t *col;
    const float *val;          // NULL unless the weights are explicit
    int64_t n, n1;
    const int32_t *part_of;    // NULL: the built-in rule
    int32_t p;
    uint32_t lo, hi;           // built-in rule: part p owns the nodes with lo <= (v mod n1) < hi
};

// Is node v in part p?  The caller's array, or the p-th contiguous slice of every copy:
// floor(r P / n1) = p  <=>  ceil(p n1 / P) <= r < ceil((p + 1) n1 / P)  for r = v mod n1 (n < 2^31).
__device__ __forceinline__ bool rg_owned(const RgGraph &g, int64_t v)
{
    if (g.part_of) return g.part_of[v] == g.p;
    const uint32_t r = (uint32_t)v % (uint32_t)g.n1;
    return r >= g.lo && r < g.hi;
}

// flag[0] |= 1 when a caller-supplied part id lies outside [0, P)
__global__ __launch_bounds__(kBlock) void rg_check_parts(const int32_t *__restrict__ part_of, int64_t n, int32_t P,
                                                         int32_t *__restrict__ flag)
{
    const int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (v < n) {
        const int32_t q = part_of[v];
        if (q < 0 || q >= P) atomicOr(flag, 1);
    }
}

__global__ __launch_bounds__(kBlock) void rg_fill_i32(int32_t *__restrict__ a, int64_t n, int32_t value)
{
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n) a[i] = value;
}

// Every owned row flags its columns of other parts.  Several rows may flag the same node: all of them
// store the same value.
__global__ __launch_bounds__(kBlock) void rg_mark(RgGraph g, int32_t *__restrict__ local_of)
{
    const int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= g.n || !rg_owned(g, v)) return;
    const int64_t b = g.rowptr[v], e = g.rowptr[v + 1];
    for (int64_t q = b; q < e; ++q) {
        const int32_t u = g.col[q];
        if (!rg_owned(g, u)) local_of[u] = kRgHalo;
    }
}

// cnt[2 b] = owned rows of block b, cnt[2 b + 1] = flagged rows of block b
__global__ __launch_bounds__(kBlock) void rg_count(RgGraph g, const int32_t *__restrict__ local_of,
                                                   int32_t *__restrict__ cnt)
{
    __shared__ int32_t s_cnt[2];
    if (threadIdx.x < 2) s_cnt[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kRgRowsPerBlock;
    int own = 0, halo = 0;
    for (int k = 0; k < kRgItems; ++k) {
        const int64_t v = base + (int64_t)k * kBlock + threadIdx.x;
        if (v < g.n) {
            if (rg_owned(g, v)) ++own;
            else if (local_of[v] == kRgHalo) ++halo;
        }
    }
    if (own) atomicAdd(&s_cnt[0], own);
    if (halo) atomicAdd(&s_cnt[1], halo);
    __syncthreads();
    if (threadIdx.x < 2) cnt[2 * (int64_t)blockIdx.x + threadIdx.x] = s_cnt[threadIdx.x];
}

// One workgroup per column c of cnt[., c] (cols columns): exclusive prefix over the blocks, total[c] = sum.
__global__ __launch_bounds__(kBlock) void rg_scan_counts(int32_t *__restrict__ cnt, int64_t n_blocks, int32_t cols,
                                                         int64_t *__restrict__ total)
{
    __shared__ int64_t s_part[kBlock];
    const int c = blockIdx.x;
    const int64_t seg = (n_blocks + kBlock - 1) / kBlock;
    const int64_t b0 = (int64_t)threadIdx.x * seg < n_blocks ? (int64_t)threadIdx.x * seg : n_blocks;
    const int64_t b1 = b0 + seg < n_blocks ? b0 + seg : n_blocks;
    int64_t sum = 0;
    for (int64_t b = b0; b < b1; ++b) sum += cnt[b * cols + c];
    s_part[threadIdx.x] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t run = 0;
        for (int t = 0; t < kBlock; ++t) { const int64_t v = s_part[t]; s_part[t] = run; run += v; }
        total[c] = run;
    }
    __syncthreads();
    int64_t run = s_part[threadIdx.x];
    for (int64_t b = b0; b < b1; ++b) {
        const int32_t v = cnt[b * cols + c];
        cnt[b * cols + c] = (int32_t)run;
        run += v;
    }
}

// Stable compaction: position of a row = rows of its kind in earlier blocks + in earlier wavefronts of the
// block + earlier in its own wavefront (ballot ranks in lane order).  total = {n_owned, n_halo}.
__global__ __launch_bounds__(kBlock) void rg_scatter(RgGraph g, const int32_t *__restrict__ prefix,
                                                     const int64_t *__restrict__ total, int32_t *__restrict__ local_of,
                                                     int64_t *__restrict__ global_id)
{
    __shared__ int32_t s_pos[kWavesPerBlock][2];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const uint64_t lt_mask = lane ? (~0ULL >> (64 - lane)) : 0ULL;
    const int64_t wbase = (int64_t)blockIdx.x * kRgRowsPerBlock + (int64_t)wave * kRgRowsPerWave;
    const int64_t n_owned = total[0];

    int own = 0, halo = 0;
    for (int k = 0; k < kRgRowsPerWave / kWave; ++k) {
        const int64_t v = wbase + (int64_t)k * kWave + lane;
        bool o = false, h = false;
        if (v < g.n) {
            o = rg_owned(g, v);
            h = !o && local_of[v] == kRgHalo;
        }
        own += __popcll(__ballot(o));
        halo += __popcll(__ballot(h));
    }
    if (lane == 0) { s_pos[wave][0] = own; s_pos[wave][1] = halo; }
    __syncthreads();
    if (threadIdx.x < 2) {
        int64_t run = prefix[2 * (int64_t)blockIdx.x + threadIdx.x];
        for (int w = 0; w < kWavesPerBlock; ++w) {
            const int32_t c = s_pos[w][threadIdx.x];
            s_pos[w][threadIdx.x] = (int32_t)run;
            run += c;
        }
    }
    __syncthreads();
    int64_t pos_o = s_pos[wave][0], pos_h = s_pos[wave][1];
    for (int k = 0; k < kRgRowsPerWave / kWave; ++k) {
        const int64_t v = wbase + (int64_t)k * kWave + lane;
        bool o = false, h = false;
        if (v < g.n) {
            o = rg_owned(g, v);
            h = !o && local_of[v] == kRgHalo;
        }
        const uint64_t m_o = __ballot(o), m_h = __ballot(h);
        if (o) {
            const int64_t k_loc = pos_o + __popcll(m_o & lt_mask);
            global_id[k_loc] = v;
            local_of[v] = (int32_t)k_loc;
        }
        if (h) {
            const int64_t k_loc = n_owned + pos_h + __popcll(m_h & lt_mask);
            global_id[k_loc] = v;
            local_of[v] = (int32_t)k_loc;
        }
        pos_o += __popcll(m_o);
        pos_h += __popcll(m_h);
    }
}

// is u a stored column of row v (columns ascending)?
__device__ __forceinline__ bool rg_row_has(const RgGraph &g, int64_t v, int32_t u)
{
    int64_t lo = g.rowptr[v], hi = g.rowptr[v + 1];
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        const int32_t c = g.col[mid];
        if (c == u) return true;
        if (c < u) lo = mid + 1; else hi = mid;
    }
    return false;
}

// Does entry (column c) of local row k (global v) belong to the sub-graph?  cross: it also is one crossing
// pair that no other entry counts.
__device__ __forceinline__ bool rg_keep(const RgGraph &g, const int32_t *__restrict__ local_of, int64_t n_owned,
                                        bool row_owned, int64_t v, int32_t c, bool &cross)
{
    cross = false;
    const int32_t lc = local_of[c];
    if (row_owned) {
        if (lc < 0) return false;
        cross = lc >= n_owned;
        return true;
    }
    if (c == v) return true;                                     // stored self-loop of a boundary node
    if (lc < 0 || lc >= n_owned) return false;                   // boundary-boundary edge: not in E_p+
    // an edge stored only in this direction is a crossing pair that its owned end did not count
    cross = !rg_row_has(g, c, (int32_t)v);
    return true;
}

// rg_keep without the crossing bookkeeping
__device__ __forceinline__ bool rg_keep_fast(const int32_t *__restrict__ local_of, int64_t n_owned, bool row_owned,
                                             int64_t v, int32_t c)
{
    const int32_t lc = local_of[c];
    if (row_owned) return lc >= 0;
    return c == v || (lc >= 0 && lc < n_owned);
}

// len[k] = stored length of local row k; the kRgCrossSlots counters of crossing together receive the number of
// unordered pairs {i in S_p, j in B_p} joined by an edge.
// A lane walks a short row alone; a row above kRgShort entries (the primary inputs of a multiplier have
// thousands) is put on long_list (n_long[0] entries, any order) and left to rg_row_len_long.
__global__ __launch_bounds__(kBlock) void rg_row_len(RgGraph g, const int32_t *__restrict__ local_of,
                                                     const int64_t *__restrict__ global_id, int64_t n_owned,
                                                     int64_t n_loc, int32_t *__restrict__ len,
                                                     unsigned long long *__restrict__ crossing,
                                                     int32_t *__restrict__ long_list, int32_t *__restrict__ n_long)
{
    const int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    int64_t cross = 0;
    if (k < n_loc) {
        const int64_t v = global_id[k];
        const int64_t b = g.rowptr[v], e = g.rowptr[v + 1];
        if (e - b > kRgShort) {
            long_list[atomicAdd(n_long, 1)] = (int32_t)k;
        } else {
            int32_t count = 0;
            for (int64_t q = b; q < e; ++q) {
                bool x;
                if (rg_keep(g, local_of, n_owned, k < n_owned, v, g.col[q], x)) ++count;
                if (x) ++cross;
            }
            len[k] = count;
        }
    }
    rg_add_crossing(cross, crossing);
}

// The rows of long_list, one wavefront per row at a time (kRgUnroll x 64 entries in flight).
__global__ __launch_bounds__(kBlock) void rg_row_len_long(RgGraph g, const int32_t *__restrict__ local_of,
                                                          const int64_t *__restrict__ global_id, int64_t n_owned,
                                                          int32_t *__restrict__ len,
                                                          unsigned long long *__restrict__ crossing,
                                                          const int32_t *__restrict__ long_list,
                                                          const int32_t *__restrict__ n_long)
{
    const int lane = threadIdx.x % kWave;
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerBlock;
    const int32_t n_rows = n_long[0];
    int64_t cross = 0;
    for (int64_t i = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave; i < n_rows; i += n_waves) {
        const int64_t k = long_list[i];
        const int64_t v = global_id[k];
        const int64_t b = g.rowptr[v], e = g.rowptr[v + 1];
        const bool row_owned = k < n_owned;
        int32_t count = 0;
        for (int64_t q0 = b; q0 < e; q0 += kRgUnroll * kWave) {
            int32_t c[kRgUnroll];
#pragma unroll
            for (int u = 0; u < kRgUnroll; ++u) {
                const int64_t q = q0 + u * kWave + lane;
                c[u] = q < e ? g.col[q] : -1;
            }
#pragma unroll
            for (int u = 0; u < kRgUnroll; ++u) {
                bool keep = false, x = false;
                if (c[u] >= 0) keep = rg_keep(g, local_of, n_owned, row_owned, v, c[u], x);
                count += __popcll(__ballot(keep));
                cross += x ? 1 : 0;
            }
        }
        if (lane == 0) len[k] = count;
    }
    rg_add_crossing(cross, crossing);
}

// sums[b] = sum of len over block b (4096 items)
__global__ __launch_bounds__(kBlock) void rg_len_sums(const int32_t *__restrict__ len, int64_t n,
                                                      int64_t *__restrict__ sums)
{
    __shared__ int64_t s_w[kWavesPerBlock];
    const int64_t base = (int64_t)blockIdx.x * kRgRowsPerBlock;
    int64_t sum = 0;
    for (int k = 0; k < kRgItems; ++k) {
        const int64_t i = base + (int64_t)k * kBlock + threadIdx.x;
        if (i < n) sum += len[i];
    }
    for (int off = kWave / 2; off > 0; off >>= 1) sum += __shfl_down(sum, off);
    if (threadIdx.x % kWave == 0) s_w[threadIdx.x / kWave] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t t = 0;
        for (int w = 0; w < kWavesPerBlock; ++w) t += s_w[w];
        sums[blockIdx.x] = t;
    }
}

// One workgroup: sums -> exclusive prefix, total[0] = sum of all, rowptr_end[0] = the same;
// cross_total[0] = sum of the crossing-pair counters
__global__ __launch_bounds__(kBlock) void rg_scan_sums(int64_t *__restrict__ sums, int64_t n_blocks,
                                                       int64_t *__restrict__ total, int64_t *__restrict__ rowptr_end,
                                                       const unsigned long long *__restrict__ cross_slots,
                                                       int64_t *__restrict__ cross_total)
{
    __shared__ int64_t s_part[kBlock];
    if (threadIdx.x == 0) {
        unsigned long long t = 0;
        for (int i = 0; i < kRgCrossSlots; ++i) t += cross_slots[i];
        cross_total[0] = (int64_t)t;
    }
    const int64_t seg = (n_blocks + kBlock - 1) / kBlock;
    const int64_t b0 = (int64_t)threadIdx.x * seg < n_blocks ? (int64_t)threadIdx.x * seg : n_blocks;
    const int64_t b1 = b0 + seg < n_blocks ? b0 + seg : n_blocks;
    int64_t sum = 0;
    for (int64_t b = b0; b < b1; ++b) sum += sums[b];
    s_part[threadIdx.x] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t run = 0;
        for (int t = 0; t < kBlock; ++t) { const int64_t v = s_part[t]; s_part[t] = run; run += v; }
        total[0] = run;
        rowptr_end[0] = run;
    }
    __syncthreads();
    int64_t run = s_part[threadIdx.x];
    for (int64_t b = b0; b < b1; ++b) {
        const int64_t v = sums[b];
        sums[b] = run;
        run += v;
    }
}

// rowptr[i] = sums[block of i] + lengths before i inside the block (thread t owns 16 consecutive items)
__global__ __launch_bounds__(kBlock) void rg_len_write(const int32_t *__restrict__ len, int64_t n,
                                                       const int64_t *__restrict__ sums, int64_t *__restrict__ rowptr)
{
    __shared__ int64_t s_w[kWavesPerBlock];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int64_t first = (int64_t)blockIdx.x * kRgRowsPerBlock + (int64_t)threadIdx.x * kRgItems;
    int32_t v[kRgItems];
    int64_t mine = 0;
    for (int k = 0; k < kRgItems; ++k) {
        v[k] = first + k < n ? len[first + k] : 0;
        mine += v[k];
    }
    int64_t incl = mine;                                     // inclusive prefix over the wavefront's lanes
    for (int off = 1; off < kWave; off <<= 1) {
        const int64_t up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
    }
    if (lane == kWave - 1) s_w[wave] = incl;
    __syncthreads();
    int64_t run = sums[blockIdx.x] + incl - mine;
    for (int w = 0; w < wave; ++w) run += s_w[w];
    for (int k = 0; k < kRgItems; ++k) {
        if (first + k < n) rowptr[first + k] = run;
        run += v[k];
    }
}

// Columns (and weights) of the sub-graph: per row the kept entries with an owned column, in order, then those
// with a boundary column.  Short rows here, one lane each; the rows of long_list in rg_fill_long.
__global__ __launch_bounds__(kBlock) void rg_fill(RgGraph g, const int32_t *__restrict__ local_of,
                                                  const int64_t *__restrict__ global_id, int64_t n_owned,
                                                  int64_t n_loc, const int64_t *__restrict__ sub_rowptr,
                                                  int32_t *__restrict__ sub_col, float *__restrict__ sub_val)
{
    const int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (k >= n_loc) return;
    const int64_t v = global_id[k];
    const int64_t b = g.rowptr[v], e = g.rowptr[v + 1];
    if (e - b > kRgShort) return;
    int64_t w = sub_rowptr[k];
    const int64_t w_end = sub_rowptr[k + 1];
    for (int pass = 0; pass < 2; ++pass)
        for (int64_t q = b; q < e; ++q) {
            const int32_t c = g.col[q];
            if (!rg_keep_fast(local_of, n_owned, k < n_owned, v, c)) continue;
            const int32_t lc = local_of[c];
            if ((lc < n_owned) != (pass == 0)) continue;
            if (w < w_end) {                                     // always true when the lengths match this walk
                sub_col[w] = lc;
                if (sub_val) sub_val[w] = g.val[q];
            }
            ++w;
        }
}

// One wavefront per long row at a time; positions inside a row by ballot ranks in lane order.
__global__ __launch_bounds__(kBlock) void rg_fill_long(RgGraph g, const int32_t *__restrict__ local_of,
                                                       const int64_t *__restrict__ global_id, int64_t n_owned,
                                                       const int64_t *__restrict__ sub_rowptr,
                                                       int32_t *__restrict__ sub_col, float *__restrict__ sub_val,
                                                       const int32_t *__restrict__ long_list,
                                                       const int32_t *__restrict__ n_long)
{
    const int lane = threadIdx.x % kWave;
    const uint64_t lt_mask = lane ? (~0ULL >> (64 - lane)) : 0ULL;
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerBlock;
    const int32_t n_rows = n_long[0];
    for (int64_t i = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave; i < n_rows; i += n_waves) {
        const int64_t k = long_list[i];
        const int64_t v = global_id[k];
        const int64_t b = g.rowptr[v], e = g.rowptr[v + 1];
        const bool row_owned = k < n_owned;
        int64_t w = sub_rowptr[k];
        const int64_t w_end = sub_rowptr[k + 1];
        for (int pass = 0; pass < 2; ++pass)
            for (int64_t q0 = b; q0 < e; q0 += kRgUnroll * kWave) {
                int32_t c[kRgUnroll], lc[kRgUnroll];
#pragma unroll
                for (int u = 0; u < kRgUnroll; ++u) {
                    const int64_t q = q0 + u * kWave + lane;
                    c[u] = q < e ? g.col[q] : -1;
                }
#pragma unroll
                for (int u = 0; u < kRgUnroll; ++u) lc[u] = c[u] >= 0 ? local_of[c[u]] : -1;
#pragma unroll
                for (int u = 0; u < kRgUnroll; ++u) {
                    bool keep = false;
                    if (c[u] >= 0) {
                        keep = row_owned ? lc[u] >= 0 : (c[u] == v || (lc[u] >= 0 && lc[u] < n_owned));
                        keep = keep && ((lc[u] < n_owned) == (pass == 0));
                    }
                    const uint64_t m = __ballot(keep);
                    const int64_t at = w + __popcll(m & lt_mask);
                    if (keep && at < w_end) {
                        sub_col[at] = lc[u];
                        if (sub_val) sub_val[at] = g.val[q0 + u * kWave + lane];
                    }
                    w += __popcll(m);
                }
            }
    }
}

namespace {

inline unsigned rg_grid(int64_t items, int per_block) { return (unsigned)((items + per_block - 1) / per_block); }

struct Scratch {
    void *p[8] = {};
    int used = 0;
    ~Scratch() { for (int i = 0; i < used; ++i) (void)hipFree(p[i]); }
    template <class T>
    bool get(T **out, size_t count)
    {
        void *q = nullptr;
        if (used >= 8 || hipMalloc(&q, (count ? count : 1) * sizeof(T)) != hipSuccess) return false;
        p[used++] = q;
        *out = (T *)q;
        return true;
    }
};

}  // namespace

void free_device_part(DevicePart &part)
{
    (void)hipFree(part.global_id);
    (void)hipFree(part.rowptr);
    (void)hipFree(part.col);
    (void)hipFree(part.val);
    part = DevicePart{};
}

// Returns 0, a hipError_t, kErrOutOfDeviceMemory, or kErrBadPartId (a part id outside [0, P)).
int launch_regrow_device(const DevicePlan &dp, int64_t n1, int32_t P, const int32_t *part_of_dev, int32_t p,
                         int regrow, void *stream, DevicePart *out)
{
    hipStream_t st = (hipStream_t)stream;
    const int64_t n = dp.n;
    *out = DevicePart{};
    if (n < 1 || n > 0x7fffffffLL || n1 < 1 || n1 > n || P < 1 || p < 0 || p >= P) return (int)hipErrorInvalidValue;
    // slice of the built-in rule: ceil(p n1 / P) .. ceil((p + 1) n1 / P), exact in 64 bits (n1, P < 2^31)
    const uint32_t lo = (uint32_t)(((int64_t)p * n1 + P - 1) / P), hi = (uint32_t)(((int64_t)(p + 1) * n1 + P - 1) / P);
    RgGraph g{dp.rowptr, dp.col, dp.graph_weight_mode == kExplicit ? dp.val : nullptr, n, n1, part_of_dev, p, lo, hi};
    const int64_t n_blocks = (n + kRgRowsPerBlock - 1) / kRgRowsPerBlock;

    Scratch scratch;
    int32_t *local_of = nullptr, *cnt = nullptr, *flag = nullptr, *len = nullptr, *long_list = nullptr;
    int64_t *total = nullptr, *sums = nullptr;
    if (!scratch.get(&local_of, (size_t)n) || !scratch.get(&cnt, (size_t)n_blocks * 2) || !scratch.get(&flag, 2) ||
        !scratch.get(&total, 4 + kRgCrossSlots))
        return kErrOutOfDeviceMemory;

    DevicePart part;
    hipError_t e = hipSuccess;
    auto done = [&](int code) {
        (void)hipStreamSynchronize(st);                          // scratch and partial results are freed next
        free_device_part(part);
        return code;
    };

    rg_fill_i32<<<dim3(1), dim3(kBlock), 0, st>>>(flag, 2, 0);
    rg_fill_i32<<<dim3(1), dim3(kBlock), 0, st>>>((int32_t *)total, 2 * (4 + kRgCrossSlots), 0);
    unsigned long long *cross_slots = (unsigned long long *)(total + 4);
    rg_fill_i32<<<dim3(rg_grid(n, kBlock)), dim3(kBlock), 0, st>>>(local_of, n, kRgNone);
    if (part_of_dev) rg_check_parts<<<dim3(rg_grid(n, kBlock)), dim3(kBlock), 0, st>>>(part_of_dev, n, P, flag);
    if (regrow) rg_mark<<<dim3(rg_grid(n, kBlock)), dim3(kBlock), 0, st>>>(g, local_of);
    rg_count<<<dim3((unsigned)n_blocks), dim3(kBlock), 0, st>>>(g, local_of, cnt);
    rg_scan_counts<<<dim3(2), dim3(kBlock), 0, st>>>(cnt, n_blocks, 2, total);
    if ((e = hipGetLastError()) != hipSuccess) return done((int)e);
    int64_t h_total[4] = {0, 0, 0, 0};
    int32_t h_flag = 0;
    if ((e = hipMemcpyAsync(h_total, total, 2 * sizeof(int64_t), hipMemcpyDeviceToHost, st)) != hipSuccess ||
        (e = hipMemcpyAsync(&h_flag, flag, sizeof(int32_t), hipMemcpyDeviceToHost, st)) != hipSuccess ||
        (e = hipStreamSynchronize(st)) != hipSuccess)
        return done((int)e);
    if (h_flag) return done(kErrBadPartId);
    part.n_owned = h_total[0];
    part.n_halo = h_total[1];
    const int64_t n_loc = part.n_owned + part.n_halo;
    if (part.n_owned < 0 || part.n_halo < 0 || n_loc > n) return done((int)hipErrorUnknown);

    if (hipMalloc((void **)&part.global_id, (size_t)(n_loc ? n_loc : 1) * sizeof(int64_t)) != hipSuccess ||
        hipMalloc((void **)&part.rowptr, (size_t)(n_loc + 1) * sizeof(int64_t)) != hipSuccess)
        return done(kErrOutOfDeviceMemory);
    const int64_t loc_blocks = (n_loc + kRgRowsPerBlock - 1) / kRgRowsPerBlock;
    if (!scratch.get(&len, (size_t)n_loc) || !scratch.get(&sums, (size_t)loc_blocks) ||
        !scratch.get(&long_list, (size_t)n_loc))
        return done(kErrOutOfDeviceMemory);
    int32_t *n_long = flag + 1;

    rg_scatter<<<dim3((unsigned)n_blocks), dim3(kBlock), 0, st>>>(g, cnt, total, local_of, part.global_id);
    if (n_loc) {
        rg_row_len<<<dim3(rg_grid(n_loc, kBlock)), dim3(kBlock), 0, st>>>(g, local_of, part.global_id, part.n_owned, n_loc,
                                                                          len, cross_slots, long_list, n_long);
        rg_row_len_long<<<dim3(kRgLongBlocks), dim3(kBlock), 0, st>>>(g, local_of, part.global_id, part.n_owned, len,
                                                                      cross_slots, long_list, n_long);
        rg_len_sums<<<dim3((unsigned)loc_blocks), dim3(kBlock), 0, st>>>(len, n_loc, sums);
    }
    rg_scan_sums<<<dim3(1), dim3(kBlock), 0, st>>>(sums, loc_blocks, total + 3, part.rowptr + n_loc, cross_slots, total + 2);
    if (n_loc) rg_len_write<<<dim3((unsigned)loc_blocks), dim3(kBlock), 0, st>>>(len, n_loc, sums, part.rowptr);
    if ((e = hipGetLastError()) != hipSuccess) return done((int)e);
    if ((e = hipMemcpyAsync(h_total + 2, total + 2, 2 * sizeof(int64_t), hipMemcpyDeviceToHost, st)) != hipSuccess ||
        (e = hipStreamSynchronize(st)) != hipSuccess)
        return done((int)e);
    part.n_crossing = h_total[2];
    part.nnz = h_total[3];
    if (part.nnz < 0 || part.nnz > dp.nnz) return done((int)hipErrorUnknown);

    if (hipMalloc((void **)&part.col, (size_t)(part.nnz ? part.nnz : 1) * sizeof(int32_t)) != hipSuccess)
        return done(kErrOutOfDeviceMemory);
    if (g.val && hipMalloc((void **)&part.val, (size_t)(part.nnz ? part.nnz : 1) * sizeof(float)) != hipSuccess)
        return done(kErrOutOfDeviceMemory);
    if (n_loc) {
        rg_fill<<<dim3(rg_grid(n_loc, kBlock)), dim3(kBlock), 0, st>>>(g, local_of, part.global_id, part.n_owned, n_loc,
                                                                       part.rowptr, part.col, part.val);
        rg_fill_long<<<dim3(kRgLongBlocks), dim3(kBlock), 0, st>>>(g, local_of, part.global_id, part.n_owned, part.rowptr,
                                                                   part.col, part.val, long_list, n_long);
    }
    if ((e = hipGetLastError()) != hipSuccess) return done((int)e);
    if ((e = hipStreamSynchronize(st)) != hipSuccess) return done((int)e);   // the scratch is freed on return
    *out = part;
    return 0;
}

// Milliseconds per call of fn(ctx), which enqueues work on the stream: one untimed call, then `reps` calls between two
// events.  Synchronises the stream.  0, or the first HIP error (fn returns 0 or an error of its own).
int device_time_ms(void *stream, int reps, int (*fn)(void *ctx), void *ctx, float *ms)
{
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t a = nullptr, b = nullptr;
    hipError_t e = hipEventCreate(&a);
    if (e == hipSuccess) e = hipEventCreate(&b);
    int err = (int)e;
    if (!err) err = fn(ctx);
    if (!err) err = (int)hipEventRecord(a, st);
    for (int r = 0; r < reps && !err; ++r) err = fn(ctx);
    if (!err) err = (int)hipEventRecord(b, st);
    if (!err) err = (int)hipEventSynchronize(b);
    float t = 0.f;
    if (!err) err = (int)hipEventElapsedTime(&t, a, b);
    if (a) (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
    if (err) (void)hipStreamSynchronize(st);
    *ms = reps > 0 ? t / (float)reps : 0.f;
    return err;
}

int device_download(void *dst_host, const void *src_dev, size_t bytes, void *stream)
{
    if (!bytes) return 0;
    hipStream_t st = (hipStream_t)stream;
    hipError_t err = hipMemcpyAsync(dst_host, src_dev, bytes, hipMemcpyDeviceToHost, st);
    hipError_t err2 = hipStreamSynchronize(st);
    return (int)(err != hipSuccess ? err : err2);
}

int device_copy(void *dst_dev, const void *src_dev, size_t bytes, void *stream)
{
    if (!bytes) return 0;
    hipStream_t st = (hipStream_t)stream;
    hipError_t err = hipMemcpyAsync(dst_dev, src_dev, bytes, hipMemcpyDeviceToDevice, st);
    hipError_t err2 = hipStreamSynchronize(st);
    return (int)(err != hipSuccess ? err : err2);
}

}  // namespace groot
