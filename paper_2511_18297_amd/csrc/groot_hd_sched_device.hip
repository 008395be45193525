// Schedule of the high-degree rows built on the device (gfx950), for plans whose matrix lives there.
// Section "Kernel Design - GROOT-GPU": the non-zeros of a high-degree row are partitioned statically; here a
// row of d entries is cut into ceil(d / hd_chunk) balanced pieces, a row with more than one piece gets a run of
// partial-sum slots, and the pieces run in the order of their first column (pieces of different rows that read
// the same stretch of feature rows then run close together).  Integer work; the arrays are bit-identical to what
// the host builds from the same rows (groot_spmm_plan): pieces in row order, then a stable sort by first column.
#include <cstring>

#include <hip/hip_runtime.h>
#include <rocprim/device/device_radix_sort.hpp>

#include "groot_device.h"

namespace groot {

namespace {

struct HsTotals {
    unsigned long long n_chunks, n_slots, n_split, nnz_hd;
};

__device__ __forceinline__ int64_t hs_pieces(int64_t d, int64_t chunk)
{
    const int64_t p = (d + chunk - 1) / chunk;
    return p < 1 ? 1 : p;
}

// per high-degree row k: number of pieces, of partial-sum slots (0 for a single piece), 1 if it is split
__global__ __launch_bounds__(kBlock) void hs_count(const int64_t *__restrict__ rowptr, const int32_t *__restrict__ hd_rows,
                                                   int64_t n_hd, int64_t chunk, int64_t *__restrict__ pieces,
                                                   int64_t *__restrict__ slots, int64_t *__restrict__ split)
{
    const int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (k >= n_hd) return;
    const int64_t r = hd_rows[k], d = rowptr[r + 1] - rowptr[r];
    const int64_t p = hs_pieces(d < 0 ? 0 : d, chunk);
    pieces[k] = p;
    slots[k] = p > 1 ? p : 0;
    split[k] = p > 1 ? 1 : 0;
}

// Exclusive prefix sums of the three arrays in place (one workgroup walks them in runs of its size), the totals and
// the number of entries of all high-degree rows.
__global__ __launch_bounds__(1024) void hs_scan(const int64_t *__restrict__ rowptr, const int32_t *__restrict__ hd_rows,
                                                int64_t n_hd, int64_t *__restrict__ pieces, int64_t *__restrict__ slots,
                                                int64_t *__restrict__ split, HsTotals *__restrict__ totals)
{
    __shared__ int64_t s_part[3][16];                    // per wavefront
    __shared__ int64_t s_carry[4];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    if (threadIdx.x < 4) s_carry[threadIdx.x] = 0;
    __syncthreads();
    int64_t nnz = 0;
    for (int64_t base = 0; base < n_hd; base += 1024) {
        const int64_t k = base + threadIdx.x;
        int64_t v[3] = {0, 0, 0};
        if (k < n_hd) {
            v[0] = pieces[k]; v[1] = slots[k]; v[2] = split[k];
            const int64_t r = hd_rows[k];
            nnz += rowptr[r + 1] - rowptr[r];
        }
        int64_t incl[3];
#pragma unroll
        for (int a = 0; a < 3; ++a) {                    // inclusive scan inside the wavefront
            int64_t x = v[a];
#pragma unroll
            for (int off = 1; off < kWave; off *= 2) {
                const int64_t y = __shfl_up(x, off);
                if (lane >= off) x += y;
            }
            incl[a] = x;
            if (lane == kWave - 1) s_part[a][wave] = x;
        }
        __syncthreads();
        int64_t before[3];
#pragma unroll
        for (int a = 0; a < 3; ++a) {
            int64_t b = s_carry[a];
            for (int w2 = 0; w2 < wave; ++w2) b += s_part[a][w2];
            before[a] = b;
        }
        if (k < n_hd) {
            pieces[k] = before[0] + incl[0] - v[0];
            slots[k] = before[1] + incl[1] - v[1];
            split[k] = before[2] + incl[2] - v[2];
        }
        __syncthreads();
        if (threadIdx.x == 1023) {
#pragma unroll
            for (int a = 0; a < 3; ++a) s_carry[a] = before[a] + incl[a];
        }
        __syncthreads();
    }
    // entries of the high-degree rows: per-thread sums -> one number (integer, order-free)
#pragma unroll
    for (int off = kWave / 2; off > 0; off /= 2) nnz += __shfl_down(nnz, off);
    if (lane == 0) s_part[0][wave] = nnz;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t t = 0;
        for (int w2 = 0; w2 < 16; ++w2) t += s_part[0][w2];
        totals->n_chunks = (unsigned long long)s_carry[0];
        totals->n_slots = (unsigned long long)s_carry[1];
        totals->n_split = (unsigned long long)s_carry[2];
        totals->nnz_hd = (unsigned long long)t;
    }
}

// One thread per high-degree row writes its pieces (in row order), its split-row record, the sort keys and the
// identity permutation; the *_rank arrays name the row by its place k in hd_rows instead of its id.
__global__ __launch_bounds__(kBlock) void hs_fill(const int64_t *__restrict__ rowptr, const int32_t *__restrict__ col,
                                                  const int32_t *__restrict__ hd_rows, int64_t n_hd, int64_t chunk,
                                                  const int64_t *__restrict__ piece_off, const int64_t *__restrict__ slot_off,
                                                  const int64_t *__restrict__ split_off, HdChunk *__restrict__ chunks,
                                                  HdChunk *__restrict__ chunks_rank, int32_t *__restrict__ keys,
                                                  int32_t *__restrict__ order, HdSplitRow *__restrict__ split_rows,
                                                  HdSplitRow *__restrict__ split_rows_rank)
{
    const int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (k >= n_hd) return;
    const int32_t row = hd_rows[k];
    const int64_t b = rowptr[row];
    int64_t d = rowptr[row + 1] - b;
    if (d < 0) d = 0;
    const int64_t pieces = hs_pieces(d, chunk), per = (d + pieces - 1) / pieces;
    const int64_t o = piece_off[k], sl = slot_off[k];
    if (pieces > 1) {
        split_rows[split_off[k]] = HdSplitRow{row, (int32_t)sl, (int32_t)pieces, 0};
        split_rows_rank[split_off[k]] = HdSplitRow{(int32_t)k, (int32_t)sl, (int32_t)pieces, 0};
    }
    for (int64_t c = 0; c < pieces; ++c) {
        const int64_t lo = c * per, hi = d < lo + per ? d : lo + per;
        HdChunk ch;
        ch.begin = b + lo;
        ch.len = (int32_t)(hi > lo ? hi - lo : 0);
        ch.row = row;
        ch.slot = pieces > 1 ? (int32_t)(sl + c) : -1;
        ch.row_nnz = (int32_t)(d < 0x7fffffffLL ? d : 0x7fffffffLL);
        chunks[o + c] = ch;
        ch.row = (int32_t)k;
        chunks_rank[o + c] = ch;
        keys[o + c] = ch.len > 0 ? col[ch.begin] : 0x7fffffff;
        order[o + c] = (int32_t)(o + c);
    }
}

__global__ __launch_bounds__(kBlock) void hs_permute(const HdChunk *__restrict__ in, const HdChunk *__restrict__ in_rank,
                                                     const int32_t *__restrict__ order, int64_t n,
                                                     HdChunk *__restrict__ out, HdChunk *__restrict__ out_rank)
{
    const int64_t c = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (c >= n) return;
    out[c] = in[order[c]];
    out_rank[c] = in_rank[order[c]];
}

struct Tmp {                                             // device memory freed on scope exit
    void *p[12] = {};
    int used = 0;
    ~Tmp() { for (int i = 0; i < used; ++i) (void)hipFree(p[i]); }
    template <class T>
    bool get(T **out, size_t count)
    {
        void *q = nullptr;
        if (used >= 12 || hipMalloc(&q, (count ? count : 1) * sizeof(T)) != hipSuccess) { (void)hipGetLastError(); return false; }
        p[used++] = q;
        *out = (T *)q;
        return true;
    }
};

}  // namespace

void free_device_hd_schedule(DeviceHdSchedule &s)
{
    (void)hipFree(s.chunks); (void)hipFree(s.chunks_rank); (void)hipFree(s.split_rows); (void)hipFree(s.split_rows_rank);
    s = DeviceHdSchedule{};
}

// hd_rows_dev: the n_hd high-degree rows, ascending.  Synchronises the stream (sizes are read back between the
// passes).  kErrOutOfDeviceMemory when an allocation fails, kErrTooManyPieces when the slots do not fit 31 bits.
int launch_hd_schedule_device(const int64_t *rowptr_dev, const int32_t *col_dev, const int32_t *hd_rows_dev, int64_t n_hd,
                              int32_t hd_chunk, void *stream, DeviceHdSchedule *out)
{
    *out = DeviceHdSchedule{};
    if (n_hd <= 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    const int64_t chunk = hd_chunk < 64 ? 64 : hd_chunk;
    Tmp tmp;
    int64_t *pieces = nullptr, *slots = nullptr, *split = nullptr;
    HsTotals *totals = nullptr;
    if (!tmp.get(&pieces, (size_t)n_hd) || !tmp.get(&slots, (size_t)n_hd) || !tmp.get(&split, (size_t)n_hd) ||
        !tmp.get(&totals, 1))
        return kErrOutOfDeviceMemory;
    const unsigned grid_rows = (unsigned)((n_hd + kBlock - 1) / kBlock);
    hs_count<<<dim3(grid_rows), dim3(kBlock), 0, st>>>(rowptr_dev, hd_rows_dev, n_hd, chunk, pieces, slots, split);
    hs_scan<<<dim3(1), dim3(1024), 0, st>>>(rowptr_dev, hd_rows_dev, n_hd, pieces, slots, split, totals);
    hipError_t e = hipGetLastError();
    HsTotals h = {};
    if (e == hipSuccess) e = hipMemcpyAsync(&h, totals, sizeof h, hipMemcpyDeviceToHost, st);
    hipError_t e2 = hipStreamSynchronize(st);
    if (e != hipSuccess || e2 != hipSuccess) return (int)(e != hipSuccess ? e : e2);
    if (h.n_slots > 0x3fffffffULL || h.n_chunks > 0x7fffffffULL) return kErrTooManyPieces;
    const int64_t n_chunks = (int64_t)h.n_chunks, n_split = (int64_t)h.n_split;

    HdChunk *raw = nullptr, *raw_rank = nullptr;
    int32_t *keys = nullptr, *keys_sorted = nullptr, *order = nullptr, *order_sorted = nullptr;
    DeviceHdSchedule s;
    if (!tmp.get(&raw, (size_t)n_chunks) || !tmp.get(&raw_rank, (size_t)n_chunks) || !tmp.get(&keys, (size_t)n_chunks) ||
        !tmp.get(&keys_sorted, (size_t)n_chunks) || !tmp.get(&order, (size_t)n_chunks) || !tmp.get(&order_sorted, (size_t)n_chunks))
        return kErrOutOfDeviceMemory;
    auto own = [&](auto **p, size_t count) {
        return hipMalloc((void **)p, (count ? count : 1) * sizeof(**p)) == hipSuccess;
    };
    if (!own(&s.chunks, (size_t)n_chunks) || !own(&s.chunks_rank, (size_t)n_chunks) || !own(&s.split_rows, (size_t)n_split) ||
        !own(&s.split_rows_rank, (size_t)n_split)) {
        (void)hipGetLastError();
        free_device_hd_schedule(s);
        return kErrOutOfDeviceMemory;
    }
    hs_fill<<<dim3(grid_rows), dim3(kBlock), 0, st>>>(rowptr_dev, col_dev, hd_rows_dev, n_hd, chunk, pieces, slots, split, raw,
                                                      raw_rank, keys, order, s.split_rows, s.split_rows_rank);
    e = hipGetLastError();
    // stable sort of the pieces by their first column: radix sort of (key, position) pairs
    size_t sort_bytes = 0;
    void *sort_tmp = nullptr;
    if (e == hipSuccess)
        e = rocprim::radix_sort_pairs(nullptr, sort_bytes, keys, keys_sorted, order, order_sorted, (size_t)n_chunks, 0, 32, st);
    if (e == hipSuccess && !tmp.get((char **)&sort_tmp, sort_bytes)) {
        free_device_hd_schedule(s);
        return kErrOutOfDeviceMemory;
    }
    if (e == hipSuccess)
        e = rocprim::radix_sort_pairs(sort_tmp, sort_bytes, keys, keys_sorted, order, order_sorted, (size_t)n_chunks, 0, 32, st);
    if (e == hipSuccess) {
        hs_permute<<<dim3((unsigned)((n_chunks + kBlock - 1) / kBlock)), dim3(kBlock), 0, st>>>(raw, raw_rank, order_sorted,
                                                                                            n_chunks, s.chunks, s.chunks_rank);
        e = hipGetLastError();
    }
    e2 = hipStreamSynchronize(st);                       // the temporaries are freed on return
    if (e != hipSuccess || e2 != hipSuccess) {
        free_device_hd_schedule(s);
        return (int)(e != hipSuccess ? e : e2);
    }
    s.n_chunks = n_chunks;
    s.n_split_rows = n_split;
    s.n_partials = (int64_t)h.n_slots;
    s.nnz_hd = (int64_t)h.nnz_hd;
    *out = s;
    return 0;
}

}  // namespace groot
