// HIP kernels of libgroot for gfx950 (wave64): the low-degree and high-degree
// aggregation kernels, the reduction of split high-degree rows, and the row
// gather / scatter of the partitioned mode.
//
// Feature rows are handled as float4 slices: a row of F floats is covered by
// a "lane group" of L lanes (L = smallest power of two >= F/4, at most 64), so
// one wavefront works on 64/L rows at a time and every load/store of a group
// is one contiguous F*4-byte segment.
#include "groot_device.h"

namespace groot {

// ---------------------------------------------------------------------------
// LD part.  A wavefront owns 64 consecutive rows.  When none of them is
// high-degree and the tile's non-zeros fit, the wavefront first copies the
// tile's column indices (and weights) to LDS with fully coalesced loads; lane
// groups then walk their rows (group g takes rows g, g+G, g+2G, ...), gather
// the feature slices of all neighbours of a row before accumulating them in
// registers, and store the finished slice.  The G groups of a wavefront always
// store G consecutive rows, i.e. one contiguous G*F*4-byte area per store.
// High-degree rows are skipped (HD pieces write them).
// ---------------------------------------------------------------------------
constexpr int kLdsBytes = kWavesPerBlock * (2 * kLdTileCap + kLdTileRows + 1) * 4;

template <int L, int W>
__device__ __forceinline__ void ld_tile(char *smem, int64_t tile, const int64_t *__restrict__ rowptr,
                                        const int32_t *__restrict__ col, const float *__restrict__ val,
                                        const v4f *__restrict__ X, v4f *__restrict__ Y, int64_t n,
                                        int32_t F4, int32_t T, const int64_t *__restrict__ out_ids, int64_t n_out)
{
    constexpr int G = kWave / L;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    int32_t *s_col = (int32_t *)smem + wave * kLdTileCap;
    float *s_val = (float *)smem + (kWavesPerBlock + wave) * kLdTileCap;
    int32_t *s_rel = (int32_t *)smem + 2 * kWavesPerBlock * kLdTileCap + wave * (kLdTileRows + 1);
    const int64_t base = (tile * kWavesPerBlock + wave) * kLdTileRows;   // may lie beyond n: empty tile

    const int64_t r = base + lane;
    int64_t rp0 = 0, rp1 = 0;
    if (r < n) { rp0 = rowptr[r]; rp1 = rowptr[r + 1]; }
    const int64_t tile_begin = rowptr[base < n ? base : n];
    const int64_t tile_end = rowptr[base + kLdTileRows < n ? base + kLdTileRows : n];
    const bool any_hd = __ballot(rp1 - rp0 >= T) != 0;
    const bool staged = !any_hd && (tile_end - tile_begin) <= kLdTileCap;

    if (staged) {
        const int m = (int)(tile_end - tile_begin);
        s_rel[lane] = (r < n) ? (int32_t)(rp0 - tile_begin) : m;
        if (lane == 0) s_rel[kLdTileRows] = m;
        for (int p = lane; p < m; p += kWave) {
            s_col[p] = __builtin_nontemporal_load(&col[tile_begin + p]);
            if (W == kExplicit) s_val[p] = __builtin_nontemporal_load(&val[tile_begin + p]);
        }
    }
    __syncthreads();

    const int g = lane / L, f = lane % L;
    for (int it = 0; it < kLdTileRows / G; ++it) {
        const int lr = it * G + g;
        const int64_t row = base + lr;
        if (row >= n_out) break;                         // n_out <= n: rows past it are not wanted
        const int64_t orow = out_ids ? out_ids[row] : row;
        if (staged) {
            const int64_t s = s_rel[lr], e = s_rel[lr + 1];
            for (int32_t ff = f; ff < F4; ff += L) {
                v4f acc = ld_row_sum<W, true>(s, e, s_col, s_val, X, F4, ff);
                __builtin_nontemporal_store(acc, &Y[orow * F4 + ff]);
            }
        } else {
            const int64_t s = rowptr[row], e = rowptr[row + 1];
            if (e - s >= T) continue;
            for (int32_t ff = f; ff < F4; ff += L) {
                v4f acc = ld_row_sum<W, false>(s, e, col, val, X, F4, ff);
                __builtin_nontemporal_store(acc, &Y[orow * F4 + ff]);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// HD part.  One workgroup per piece of a high-degree row (the plan cuts a row
// into balanced pieces).  The 256/L lane groups of the workgroup stride over
// the piece's non-zeros, each keeping a register accumulator for its float4
// slice; the group sums meet in LDS and are added by a tree.  The result goes
// to Y (single-piece rows) or to the row's slot of partial sums.
// ---------------------------------------------------------------------------
template <int L, int W>
__device__ __forceinline__ void hd_piece(char *smem, const HdChunk ch, const int32_t *__restrict__ col,
                                         const float *__restrict__ val, const v4f *__restrict__ X,
                                         v4f *__restrict__ Y, v4f *__restrict__ partials, int32_t F4,
                                         const int64_t *__restrict__ out_ids)
{
    constexpr int G = kBlock / L;
    v4f(*s_red)[L] = (v4f(*)[L])smem;                    // [G][L]
    const int g = threadIdx.x / L, f = threadIdx.x % L;
    const int64_t end = ch.begin + ch.len;
    const float rw = row_weight<W>(ch.row_nnz);

    for (int32_t fb = 0; fb < F4; fb += L) {
        const int32_t ff = fb + f;
        const bool live = ff < F4;
        v4f acc = {0.f, 0.f, 0.f, 0.f};
        if (live) {
            int64_t p = ch.begin + g;
            for (; p + 3 * G < end; p += 4 * G) {
                int32_t c0 = col[p], c1 = col[p + G], c2 = col[p + 2 * G], c3 = col[p + 3 * G];
                v4f x0 = X[(int64_t)c0 * F4 + ff], x1 = X[(int64_t)c1 * F4 + ff];
                v4f x2 = X[(int64_t)c2 * F4 + ff], x3 = X[(int64_t)c3 * F4 + ff];
                if (W == kExplicit) {
                    acc += val[p] * x0;
                    acc += val[p + G] * x1;
                    acc += val[p + 2 * G] * x2;
                    acc += val[p + 3 * G] * x3;
                } else {
                    acc += (x0 + x1) + (x2 + x3);
                }
            }
            for (; p < end; p += G) {
                v4f x = X[(int64_t)col[p] * F4 + ff];
                if (W == kExplicit) acc += val[p] * x;
                else acc += x;
            }
            if (W != kExplicit) acc *= rw;
        }
        s_red[g][f] = acc;
        __syncthreads();
#pragma unroll
        for (int stride = G / 2; stride > 0; stride /= 2) {
            if (g < stride) s_red[g][f] += s_red[g + stride][f];
            __syncthreads();
        }
        if (g == 0 && live) {
            v4f sum = s_red[0][f];
            if (ch.slot < 0) Y[(out_ids ? out_ids[ch.row] : (int64_t)ch.row) * F4 + ff] = sum;
            else partials[(int64_t)ch.slot * F4 + ff] = sum;
        }
        __syncthreads();
    }
}

// Block t of the LD launch computes the tile of rows [256 t, 256 t + 256).
template <int L, int W>
__global__ __launch_bounds__(kBlock) void ld_kernel(const int64_t *__restrict__ rowptr,
                                                    const int32_t *__restrict__ col,
                                                    const float *__restrict__ val,
                                                    const v4f *__restrict__ X, v4f *__restrict__ Y,
                                                    int64_t n, int32_t F4, int32_t T, int64_t n_tiles,
                                                    int64_t blocks_per_xcd, int remap,
                                                    const int64_t *__restrict__ out_ids, int64_t n_out)
{
    __shared__ __align__(16) char smem[kLdsBytes];
    const int64_t tile = logical_block(blocks_per_xcd, remap);
    if (tile >= n_tiles) return;
    ld_tile<L, W>(smem, tile, rowptr, col, val, X, Y, n, F4, T, out_ids, n_out);
}

// Block k of the HD launch computes piece k.
template <int L, int W>
__global__ __launch_bounds__(kBlock) void hd_kernel(const HdChunk *__restrict__ chunks,
                                                    const int32_t *__restrict__ col,
                                                    const float *__restrict__ val,
                                                    const v4f *__restrict__ X, v4f *__restrict__ Y,
                                                    v4f *__restrict__ partials, int32_t F4,
                                                    const int64_t *__restrict__ out_ids, int64_t n_out)
{
    __shared__ __align__(16) char smem[kBlock * sizeof(v4f)];
    const HdChunk ch = chunks[blockIdx.x];
    if (ch.row >= n_out) return;                         // the whole workgroup: a row that is not wanted
    hd_piece<L, W>(smem, ch, col, val, X, Y, partials, F4, out_ids);
}

// Y[row] = partials[first] + ... + partials[first+count-1], in that order.
template <int L>
__global__ __launch_bounds__(kBlock) void hd_finish_kernel(const HdSplitRow *__restrict__ rows,
                                                           int64_t n_rows,
                                                           const v4f *__restrict__ partials,
                                                           v4f *__restrict__ Y, int32_t F4,
                                                           const int64_t *__restrict__ out_ids, int64_t n_out)
{
    constexpr int G = kBlock / L;
    const int64_t k = (int64_t)blockIdx.x * G + threadIdx.x / L;
    if (k >= n_rows) return;
    const HdSplitRow sr = rows[k];
    if (sr.row >= n_out) return;
    const int64_t orow = out_ids ? out_ids[sr.row] : (int64_t)sr.row;
    for (int32_t ff = threadIdx.x % L; ff < F4; ff += L) {
        v4f acc = {0.f, 0.f, 0.f, 0.f};
        for (int32_t c = 0; c < sr.count; ++c) acc += partials[(int64_t)(sr.first + c) * F4 + ff];
        Y[orow * F4 + ff] = acc;
    }
}

// out[i] = X[ids[i]]  (kScatter = false)   or   Y[ids[i]] = in[i]  (kScatter = true)
template <int L, bool kScatter>
__global__ __launch_bounds__(kBlock) void rows_move_kernel(const int64_t *__restrict__ ids, int64_t n,
                                                           const v4f *__restrict__ src,
                                                           v4f *__restrict__ dst, int32_t F4)
{
    constexpr int G = kBlock / L;
    const int64_t i = (int64_t)blockIdx.x * G + threadIdx.x / L;
    if (i >= n) return;
    const int64_t id = ids[i];
    for (int32_t ff = threadIdx.x % L; ff < F4; ff += L) {
        if (kScatter) dst[id * F4 + ff] = src[i * F4 + ff];
        else dst[i * F4 + ff] = src[id * F4 + ff];
    }
}

// col[p] = ids[col[p]]: the columns of a part's sub-graph renamed from local ids to rows of the whole graph
__global__ __launch_bounds__(kBlock) void col_map_kernel(int32_t *__restrict__ col, int64_t nnz,
                                                         const int64_t *__restrict__ ids)
{
    for (int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x; p < nnz; p += (int64_t)gridDim.x * kBlock)
        col[p] = (int32_t)ids[col[p]];
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
static int lanes_for(int32_t F4)
{
    int L = 1;
    while (L < F4 && L < kWave) L *= 2;
    return L;
}

#define GROOT_DISPATCH_LW(L, W, CALL)                                  \
    switch (W) {                                                       \
    case kOnes: { constexpr int kW = kOnes; GROOT_DISPATCH_L(L, CALL) } break; \
    case kMean: { constexpr int kW = kMean; GROOT_DISPATCH_L(L, CALL) } break; \
    default: { constexpr int kW = kExplicit; GROOT_DISPATCH_L(L, CALL) } break; \
    }

int launch_ld(const DevicePlan &dp, const float *X, float *Y, int32_t F, void *stream, const RowOut *out)
{
    const int32_t F4 = F / 4;
    const int64_t *out_ids = out ? out->ids : nullptr;
    const int64_t n_out = out ? out->n_out : dp.n;
    // the pipelined kernel serves whole graphs at F = 32, 64 and 128 (ld_pipelined: 2 all three widths, 1 only the two wider)
    if (dp.zero_row && ((dp.ld_pipelined == 2 && F4 == 8) || (dp.ld_pipelined && (F4 == 16 || F4 == 32))))
        return launch_ld_pipelined(dp, X, Y, F, stream, out);
    const int64_t n_tiles = (n_out + kRowsPerLdTile - 1) / kRowsPerLdTile;
    if (n_tiles == 0) return 0;
    const int64_t per_xcd = (n_tiles + kXcds - 1) / kXcds;
    const int remap = dp.xcd_remap && n_tiles >= 4 * kXcds;
    const int64_t grid = remap ? per_xcd * kXcds : n_tiles;
    if (!grid_ok(grid)) return (int)hipErrorInvalidConfiguration;
    if (!weights_ok(dp)) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    GROOT_DISPATCH_LW(lanes_for(F4), dp.weight_mode,
                      (ld_kernel<kL, kW><<<dim3((unsigned)grid), dim3(kBlock), 0, st>>>(
                          dp.rowptr, dp.col, dp.val, (const v4f *)X, (v4f *)Y, dp.n, F4, dp.threshold, n_tiles,
                          per_xcd, remap, out_ids, n_out)));
    return (int)hipGetLastError();
}

int launch_hd(const DevicePlan &dp, const float *X, float *Y, int32_t F, void *stream, const RowOut *out)
{
    const int32_t F4 = F / 4;
    const int64_t *out_ids = out ? out->ids : nullptr;
    const int64_t n_out = out ? out->n_out : dp.n;
    if (!grid_ok(dp.n_chunks)) return (int)hipErrorInvalidConfiguration;
    if (!weights_ok(dp)) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    GROOT_DISPATCH_LW(lanes_for(F4), dp.weight_mode,
                      (hd_kernel<kL, kW><<<dim3((unsigned)dp.n_chunks), dim3(kBlock), 0, st>>>(
                          dp.chunks, dp.col, dp.val, (const v4f *)X, (v4f *)Y, (v4f *)dp.partials, F4, out_ids, n_out)));
    return (int)hipGetLastError();
}

int launch_hd_finish(const DevicePlan &dp, float *Y, int32_t F, void *stream, const RowOut *out)
{
    const int32_t F4 = F / 4;
    const int64_t *out_ids = out ? out->ids : nullptr;
    const int64_t n_out = out ? out->n_out : dp.n;
    const int L = lanes_for(F4);
    const int64_t grid = (dp.n_split_rows + kBlock / L - 1) / (kBlock / L);
    if (!grid_ok(grid)) return (int)hipErrorInvalidConfiguration;
    hipStream_t st = (hipStream_t)stream;
    GROOT_DISPATCH_L(L, (hd_finish_kernel<kL><<<dim3((unsigned)grid), dim3(kBlock), 0, st>>>(
                            dp.split_rows, dp.n_split_rows, (const v4f *)dp.partials, (v4f *)Y, F4, out_ids, n_out)));
    return (int)hipGetLastError();
}

int launch_col_map(int32_t *col, int64_t nnz, const int64_t *ids, void *stream)
{
    if (nnz <= 0) return 0;
    int64_t grid = (nnz + kBlock - 1) / kBlock;
    if (grid > 65536) grid = 65536;                      // grid-stride loop
    col_map_kernel<<<dim3((unsigned)grid), dim3(kBlock), 0, (hipStream_t)stream>>>(col, nnz, ids);
    return (int)hipGetLastError();
}

int launch_rows_gather(const int64_t *ids, int64_t n, const float *X, float *out, int32_t F, void *stream)
{
    const int32_t F4 = F / 4;
    const int L = lanes_for(F4);
    const int64_t grid = (n + kBlock / L - 1) / (kBlock / L);
    if (!grid_ok(grid)) return (int)hipErrorInvalidConfiguration;
    hipStream_t st = (hipStream_t)stream;
    GROOT_DISPATCH_L(L, (rows_move_kernel<kL, false><<<dim3((unsigned)grid), dim3(kBlock), 0, st>>>(
                            ids, n, (const v4f *)X, (v4f *)out, F4)));
    return (int)hipGetLastError();
}

int launch_rows_scatter(const int64_t *ids, int64_t n, const float *in, float *Y, int32_t F, void *stream)
{
    const int32_t F4 = F / 4;
    const int L = lanes_for(F4);
    const int64_t grid = (n + kBlock / L - 1) / (kBlock / L);
    if (!grid_ok(grid)) return (int)hipErrorInvalidConfiguration;
    hipStream_t st = (hipStream_t)stream;
    GROOT_DISPATCH_L(L, (rows_move_kernel<kL, true><<<dim3((unsigned)grid), dim3(kBlock), 0, st>>>(
                            ids, n, (const v4f *)in, (v4f *)Y, F4)));
    return (int)hipGetLastError();
}

const char *hip_error_text(int err) { return hipGetErrorString((hipError_t)err); }

int dev_alloc(void **p, size_t bytes) { return (int)hipMalloc(p, bytes); }

void dev_free(void *p)
{
    if (p) (void)hipFree(p);
}

int dev_upload(void *dst, const void *src, size_t bytes)
{
    return (int)hipMemcpy(dst, src, bytes, hipMemcpyHostToDevice);
}

}  // namespace groot
