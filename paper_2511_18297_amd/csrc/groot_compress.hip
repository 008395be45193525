// Compact form of the device CSR for the pipelined LD kernel (gfx950): 4-byte row pointers and 2-byte column
// codes, built on the device from the resident CSR.  The aggregation is bound by the bytes it moves, and for
// the short rows of an EDA graph (Section "Kernel Design - GROOT-GPU": the low-degree class) the matrix
// itself is 5 % of them: 8 bytes of row pointer per row and 4 bytes per entry.  Nearly every entry of a
// low-degree row points either at a row close by (the gates of the same and of the neighbouring cells) or
// at one of the few high-degree rows (the primary inputs), which is what the two code ranges cover:
//     code <  0x8000:  column = row + code - 0x4000          (within -16384 .. +16383 rows)
//     code >= 0x8000:  column = hot[code - 0x8000]           (one of up to 32767 high-degree rows)
//     code == 0xFFFF:  neither (a primary output and its driver, say): the whole row is left to the row-list
//                      kernel, which reads the plain arrays
// Only rows that the pipelined kernel can serve are encoded (no more entries than it has slots, not
// high-degree); if more than one row in 50 cannot be encoded the plan keeps using the plain arrays.
#include "groot_device.h"

namespace groot {

// rp32[i] = low 32 bits of rowptr[i]; the caller has checked that the last row pointer fits
__global__ __launch_bounds__(kBlock) void rp32_kernel(const int64_t *__restrict__ rowptr, int64_t count,
                                                      uint32_t *__restrict__ out)
{
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < count; i += (int64_t)gridDim.x * kBlock)
        out[i] = (uint32_t)rowptr[i];
}

// One thread per row.  An entry that fits neither range gets kCodeBad and its row is appended to bad_rows (in no
// particular order): the pipelined kernel masks such a row and the row-list kernel computes it.
__global__ __launch_bounds__(kBlock) void col16_kernel(const int64_t *__restrict__ rowptr, const int32_t *__restrict__ col,
                                                       int64_t n, int32_t T, int32_t depth, const int32_t *__restrict__ hot,
                                                       int32_t n_hot, uint16_t *__restrict__ out, int32_t *__restrict__ bad_rows,
                                                       int32_t bad_cap, int32_t *__restrict__ n_bad)
{
    for (int64_t row = (int64_t)blockIdx.x * kBlock + threadIdx.x; row < n; row += (int64_t)gridDim.x * kBlock) {
        const int64_t s = rowptr[row], e = rowptr[row + 1];
        if (e - s > depth || e - s >= T) continue;                  // never read in compact form
        bool bad = false;
        for (int64_t p = s; p < e; ++p) {
            const int64_t c = col[p], delta = c - row;
            uint32_t code = kCodeBad;
            if (delta >= -kCodeNear && delta < kCodeNear) {
                code = (uint32_t)(delta + kCodeNear);
            } else {
                int32_t lo = 0, hi = n_hot;                         // first hot row >= c
                while (lo < hi) {
                    const int32_t mid = (lo + hi) / 2;
                    if (hot[mid] < c) lo = mid + 1; else hi = mid;
                }
                if (lo < n_hot && hot[lo] == c) code = kCodeHot + (uint32_t)lo;
                else bad = true;
            }
            out[p] = (uint16_t)code;
        }
        if (bad) {
            const int32_t k = atomicAdd(n_bad, 1);
            if (k < bad_cap) bad_rows[k] = (int32_t)row;
        }
    }
}

// Builds dp.rp32 / dp.col16 / dp.hot_cols from the resident CSR and the (device) list of high-degree rows,
// ascending, and appends the rows it cannot encode to dp.mid_rows.  Synchronises the stream.  On return
// dp.compressed says whether the compact form is usable; when it is not (too many entries for 32-bit row
// pointers, more than one low-degree row in 50 not encodable, no memory) its arrays are released and 0 is
// returned all the same: the plain arrays serve.
int launch_csr_compress(DevicePlan &dp, const int32_t *hd_rows_dev, int64_t n_hd, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    dp.compressed = 0;
    if (dp.n <= 0 || dp.nnz <= 0 || dp.nnz >= ((int64_t)1 << 32)) return 0;
    const int32_t n_hot = (int32_t)(n_hd < kCodeMaxHot ? n_hd : kCodeMaxHot);
    const int32_t bad_cap = (int32_t)(dp.n / 50 + 1024);
    int32_t *n_bad = nullptr, *bad_rows = nullptr, *merged = nullptr;
    auto give_up = [&](int err) {
        (void)hipFree(dp.rp32); (void)hipFree(dp.col16); (void)hipFree(dp.hot_cols); (void)hipFree(n_bad);
        (void)hipFree(bad_rows); (void)hipFree(merged);
        dp.rp32 = nullptr; dp.col16 = nullptr; dp.hot_cols = nullptr; dp.n_hot = 0;
        return err;
    };
    if (hipMalloc((void **)&dp.rp32, (size_t)(dp.n + 1) * 4) != hipSuccess ||
        hipMalloc((void **)&dp.col16, (size_t)dp.nnz * 2) != hipSuccess ||
        hipMalloc((void **)&dp.hot_cols, (size_t)(n_hot ? n_hot : 1) * 4) != hipSuccess ||
        hipMalloc((void **)&bad_rows, (size_t)bad_cap * 4) != hipSuccess ||
        hipMalloc((void **)&n_bad, 4) != hipSuccess) {
        (void)hipGetLastError();
        return give_up(0);                                           // out of device memory: not an error, the plain arrays serve
    }
    hipError_t e = hipMemsetAsync(n_bad, 0, 4, st);
    if (e == hipSuccess) e = hipMemsetAsync(dp.hot_cols, 0, (size_t)(n_hot ? n_hot : 1) * 4, st);
    if (e == hipSuccess && n_hot)
        e = hipMemcpyAsync(dp.hot_cols, hd_rows_dev, (size_t)n_hot * 4, hipMemcpyDeviceToDevice, st);
    if (e != hipSuccess) return give_up((int)e);
    const unsigned grid = 16384;
    rp32_kernel<<<dim3(grid), dim3(kBlock), 0, st>>>(dp.rowptr, dp.n + 1, dp.rp32);
    col16_kernel<<<dim3(grid), dim3(kBlock), 0, st>>>(dp.rowptr, dp.col, dp.n, dp.threshold, dp.pipe_depth, dp.hot_cols, n_hot, dp.col16,
                                                      bad_rows, bad_cap, n_bad);
    e = hipGetLastError();
    int32_t h_bad = bad_cap + 1;
    if (e == hipSuccess) e = hipMemcpyAsync(&h_bad, n_bad, 4, hipMemcpyDeviceToHost, st);
    hipError_t e2 = hipStreamSynchronize(st);
    if (e != hipSuccess || e2 != hipSuccess) return give_up((int)(e != hipSuccess ? e : e2));
    if (h_bad > bad_cap || (int64_t)h_bad * 50 > dp.n) return give_up(0);
    if (h_bad > 0) {
        // the rows that could not be encoded join the list of rows that the row-list kernel computes
        if (hipMalloc((void **)&merged, (size_t)(dp.n_mid_rows + h_bad) * 4) != hipSuccess) {
            (void)hipGetLastError();
            return give_up(0);
        }
        e = hipSuccess;
        if (dp.n_mid_rows) e = hipMemcpyAsync(merged, dp.mid_rows, (size_t)dp.n_mid_rows * 4, hipMemcpyDeviceToDevice, st);
        if (e == hipSuccess) e = hipMemcpyAsync(merged + dp.n_mid_rows, bad_rows, (size_t)h_bad * 4, hipMemcpyDeviceToDevice, st);
        e2 = hipStreamSynchronize(st);
        if (e != hipSuccess || e2 != hipSuccess) return give_up((int)(e != hipSuccess ? e : e2));
        (void)hipFree(dp.mid_rows);
        dp.mid_rows = merged;
        merged = nullptr;
        dp.n_mid_rows += h_bad;
    }
    (void)hipFree(n_bad);
    (void)hipFree(bad_rows);
    dp.n_hot = n_hot;
    dp.n_bad_rows = h_bad;
    dp.compressed = 1;
    return 0;
}

}  // namespace groot
