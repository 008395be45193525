// Fused GraphSAGE-mean layer for gfx950:  H = act((A_hat X) Wn + X Ws + b),  F_in = F_out = 64.
//
// The aggregation of a tile of rows never goes to HBM: a workgroup computes the
// 64 aggregated rows of its tile exactly like the LD kernel (lane groups of 16
// lanes, float4 gathers, register sums), parks them with the rows' own features
// in LDS as a 64 x 128 fp32 tile [A_hat X | X], and multiplies that tile with
// the stacked weights [Wn; Ws] (128 x 64) on the matrix cores
// (v_mfma_f32_16x16x4_f32).  Wavefront w owns output columns 16w..16w+15: its
// 128 x 16 slice of the weights lives in 32 registers for the whole launch
// (workgroups are persistent and walk a contiguous range of tiles), so the only
// matrix operand read per tile is the LDS tile.  The 64 x 64 result goes back
// through LDS to be stored as full 256-byte rows.
// High-degree rows are aggregated beforehand by the HD kernel into H itself;
// the layer kernel picks those sums up from H instead of recomputing them.
#include "groot_device.h"

namespace groot {

constexpr int kSgRows = 64;                 // rows per workgroup tile (16 per wavefront)
constexpr int kSgF4 = 16;                   // 64 features = 16 float4
constexpr int kSgAStride = 132;             // floats per LDS row of [agg | self] (128 + 4: conflict-free MFMA operand reads)
constexpr int kSgOStride = 68;              // floats per LDS row of the output tile
constexpr int kSgCap = 128;                 // staged non-zeros per wavefront (16 rows)

// Held to 128 registers (4 wavefronts per SIMD, i.e. 4 resident workgroups per CU): the aggregation phase of
// one workgroup overlaps the matrix phase of the others.
template <int W>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(4, 4))) void sage_kernel(const int64_t *__restrict__ rowptr,
                                                      const int32_t *__restrict__ col,
                                                      const float *__restrict__ val,
                                                      const v4f *__restrict__ X, v4f *H,
                                                      const float *__restrict__ Wn,
                                                      const float *__restrict__ Ws,
                                                      const float *__restrict__ bias, int relu,
                                                      int64_t n, int32_t T, int64_t n_tiles,
                                                      int64_t tiles_per_wg, int64_t wgs_per_xcd, int remap)
{
    __shared__ __align__(16) float s_A[kSgRows * kSgAStride];
    __shared__ int32_t s_col[kWavesPerBlock][kSgCap];
    __shared__ float s_val[kWavesPerBlock][kSgCap];
    __shared__ int32_t s_rel[kWavesPerBlock][17];

    const int tid = threadIdx.x, w = tid / kWave, l = tid % kWave;
    const int g = l / 16, f = l % 16;            // lane group / float4 slice in the aggregation phase
    const int kq = l / 16, jcol = 16 * w + l % 16;   // k offset / output column in the matrix phase

    // this wavefront's slice of [Wn; Ws]: bfrag[kk] = Wcat[4 kk + kq][jcol]
    float bfrag[32];
#pragma unroll
    for (int kk = 0; kk < 32; ++kk) {
        const int k = 4 * kk + kq;
        bfrag[kk] = k < 64 ? Wn[k * 64 + jcol] : Ws[(k - 64) * 64 + jcol];
    }
    const float bias_v = bias ? bias[jcol] : 0.0f;

    const int64_t lw = logical_block(wgs_per_xcd, remap);
    const int64_t tile_begin = lw * tiles_per_wg;
    const int64_t tile_end = tile_begin + tiles_per_wg < n_tiles ? tile_begin + tiles_per_wg : n_tiles;

    // The row pointers and column indices of a tile are fetched one tile ahead and wait in registers
    // while the previous tile is aggregated and multiplied: two dependent memory latencies leave the
    // critical path of every tile.
    int64_t rp = 0, t_begin = 0;
    int32_t m = 0, c0 = 0, c1 = 0;
    float v0 = 0.f, v1 = 0.f;
    bool staged = false;
    auto fetch_csr = [&](int64_t tile) {
        const int64_t ri = tile * kSgRows + 16 * w + (l < 16 ? l : 16);
        rp = rowptr[ri < n ? ri : n];
        t_begin = __shfl(rp, 0);
        const int64_t t_end = __shfl(rp, 16), rp_next = __shfl_down(rp, 1);
        const bool any_hd = __ballot(l < 16 && rp_next - rp >= T) != 0;
        staged = !any_hd && (t_end - t_begin) <= kSgCap;
        m = staged ? (int32_t)(t_end - t_begin) : 0;
        if (l < m) {
            c0 = __builtin_nontemporal_load(&col[t_begin + l]);
            if (W == kExplicit) v0 = __builtin_nontemporal_load(&val[t_begin + l]);
        }
        if (l + kWave < m) {
            c1 = __builtin_nontemporal_load(&col[t_begin + kWave + l]);
            if (W == kExplicit) v1 = __builtin_nontemporal_load(&val[t_begin + kWave + l]);
        }
    };
    if (tile_begin < tile_end) fetch_csr(tile_begin);

    for (int64_t tile = tile_begin; tile < tile_end; ++tile) {
        const int64_t base = tile * kSgRows;
        const int64_t wbase = base + 16 * w;              // first of this wavefront's 16 rows
        // ---- aggregation: 16 rows per wavefront, 4 at a time
        const bool staged_now = staged;
        if (staged_now) {
            if (l < 17) s_rel[w][l] = (int32_t)(rp - t_begin);
            if (l < m) { s_col[w][l] = c0; if (W == kExplicit) s_val[w][l] = v0; }
            if (l + kWave < m) { s_col[w][l + kWave] = c1; if (W == kExplicit) s_val[w][l + kWave] = v1; }
        }
        __syncthreads();
        if (tile + 1 < tile_end) fetch_csr(tile + 1);     // lands while this tile is being worked on
#pragma unroll 1
        for (int it = 0; it < 4; ++it) {
            const int lr = it * 4 + g;
            const int64_t row = wbase + lr;
            v4f agg = {0.f, 0.f, 0.f, 0.f}, self = {0.f, 0.f, 0.f, 0.f};
            if (row < n) {
                self = X[row * kSgF4 + f];
                if (staged_now) {
                    agg = ld_row_sum<W, true, 6>(s_rel[w][lr], s_rel[w][lr + 1], s_col[w], s_val[w], X, kSgF4, f);
                } else {
                    const int64_t s = rowptr[row], e = rowptr[row + 1];
                    if (e - s >= T) agg = H[row * kSgF4 + f];       // aggregated by the HD kernel
                    else agg = ld_row_sum<W, false, 6>(s, e, col, val, X, kSgF4, f);
                }
            }
            float *dst = &s_A[(16 * w + lr) * kSgAStride + 4 * f];
            *(v4f *)dst = agg;
            *(v4f *)(dst + 64) = self;
        }
        __syncthreads();
        // ---- [agg | self] (64 x 128) times this wavefront's 128 x 16 weight slice
        v4f acc[4];
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) acc[rb] = (v4f){bias_v, bias_v, bias_v, bias_v};
#pragma unroll
        for (int kk = 0; kk < 32; ++kk) {
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) {
                const float a = s_A[(rb * 16 + l % 16) * kSgAStride + 4 * kk + kq];
                acc[rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, bfrag[kk], acc[rb], 0, 0, 0);
            }
        }
        __syncthreads();                                  // every wavefront is done reading the tile
        // ---- result tile to LDS (lane holds rows 4 kq + r of its column), then full-row stores
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float v = acc[rb][r];
                if (relu) v = v > 0.0f ? v : 0.0f;
                s_A[(rb * 16 + 4 * kq + r) * kSgOStride + jcol] = v;
            }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int idx = tid + kBlock * q;
            const int orow = idx / kSgF4, c4 = idx % kSgF4;
            const int64_t row = base + orow;
            if (row < n) __builtin_nontemporal_store(*(const v4f *)&s_A[orow * kSgOStride + 4 * c4], &H[row * kSgF4 + c4]);
        }
        __syncthreads();                                  // the tile buffer is free for the next tile
    }
}

int launch_sage(const DevicePlan &dp, const float *X, float *H, const float *Wn, const float *Ws, const float *bias,
                int relu, void *stream)
{
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return (int)e;
    const int64_t n_tiles = (dp.n + kSgRows - 1) / kSgRows;
    // persistent workgroups: exactly as many as the device keeps resident, so that all of them run at once
    int per_cu = 0;
    GROOT_DISPATCH_W(dp.weight_mode, (e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, sage_kernel<kW>, kBlock, 0)));
    if (e != hipSuccess) return (int)e;
    if (per_cu < 1) per_cu = 1;
    int64_t n_wg = (int64_t)cus * per_cu;
    n_wg = (n_wg + kXcds - 1) / kXcds * kXcds;
    if (n_wg > n_tiles) n_wg = n_tiles;
    const int remap = dp.xcd_remap && n_wg % kXcds == 0 && n_wg >= 4 * kXcds;
    const int64_t tiles_per_wg = (n_tiles + n_wg - 1) / n_wg;
    if (!grid_ok(n_wg)) return (int)hipErrorInvalidConfiguration;
    if (!weights_ok(dp)) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    GROOT_DISPATCH_W(dp.weight_mode, (sage_kernel<kW><<<dim3((unsigned)n_wg), dim3(kBlock), 0, st>>>(
                                         dp.rowptr, dp.col, dp.val, (const v4f *)X, (v4f *)H, Wn, Ws, bias, relu, dp.n,
                                         dp.threshold, n_tiles, tiles_per_wg, n_wg / kXcds, remap)));
    return (int)hipGetLastError();
}

}  // namespace groot
