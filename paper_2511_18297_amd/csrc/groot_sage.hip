// Fused GraphSAGE-mean layer for gfx950:  H = act((A_hat X) Wn + X Ws + b),  F_in = F_out = 64.
//
// The aggregation of a tile of 64 rows never goes to HBM: it is formed like in the LD kernel (lane
// groups of 16 lanes, float4 gathers, register sums), parked with the rows' own features in LDS as a
// 64 x 128 fp32 tile [A_hat X | X], and multiplied with the stacked weights [Wn; Ws] (128 x 64) on the
// matrix cores (v_mfma_f32_16x16x4_f32).
//
// The two halves are bound by different units (the gathers by memory, the products by the matrix
// cores), and a wavefront that issues vector memory instructions into a saturated memory pipeline is
// held at the issue, where it cannot feed the matrix cores either.  So the wavefronts are specialised.
// One persistent workgroup of 12 wavefronts per CU walks a contiguous range of tiles:
//   * 4 consumer wavefronts (one per SIMD) never touch global memory after loading their weights.
//     Consumer w owns output columns 16w..16w+15; its 128 x 16 slice of [Wn; Ws] lives in 32 registers.
//     Per tile it runs 128 matrix instructions on the LDS tile and writes its 64 x 16 result to an LDS
//     output tile.
//   * 8 producer wavefronts (two per SIMD) each aggregate 8 rows of the next tile into the other LDS
//     tile and store 8 rows of the previous result from the LDS output tile as full 256-byte rows.
//     Their gathers run one tile ahead in two register sets, across the barrier, so the memory
//     pipeline never drains; row pointers are fetched three tiles ahead and column indices two.
// Both roles meet at one barrier per tile.  The barrier orders LDS traffic only (no global fence):
// nothing is exchanged through global memory, and the producers' loads stay in flight across it.
// High-degree rows are aggregated beforehand by the HD kernel into H itself; the producers pick those
// sums up from H instead of recomputing them.
//
// kSplit: the dense products run on the bf16 matrix instruction (v_mfma_f32_16x16x32_bf16, a sixteenth of the
// fp32 instruction's time per multiply-add) without giving up fp32 accuracy.  Every fp32 operand is cut into
// three bf16 pieces, x = hi + mid + lo exactly up to 2^-24 |x| (8 significant bits each); a product keeps the
// six piece products down to 2^-16 relative size (hi hi, hi mid, mid hi, hi lo, lo hi, mid mid; the dropped
// ones are below 2^-24) and sums them in fp32 in the instruction's accumulator.  The producers cut their rows
// when they park them in LDS (three bf16 planes instead of one fp32 tile), the consumers cut their weights
// once, so the cutting costs each SIMD 11 vector instructions per pair of tile elements, once.
#include "groot_device.h"

namespace groot {

constexpr int kSgRows = 64;                 // rows per tile
constexpr int kSgF4 = 16;                   // 64 features = 16 float4
constexpr int kSgAStride = 132;             // floats per LDS row of [agg | self] (128 + 4: conflict-free operand reads)
constexpr int kSgOStride = 68;              // floats per LDS row of the output tile (conflict-free result writes)
constexpr int kSgBRow = 272;                // bytes per LDS row of one bf16 plane of [agg | self] (256 + 16: conflict-free)
constexpr int kSgPlane = kSgRows * kSgBRow; // bytes of one plane; a split tile is three planes: hi, mid, lo
typedef __bf16 sg_bf2 __attribute__((ext_vector_type(2)));
typedef __bf16 sg_bf8 __attribute__((ext_vector_type(8)));
typedef unsigned int sg_u4 __attribute__((ext_vector_type(4)));
typedef unsigned int sg_u2 __attribute__((ext_vector_type(2)));
typedef float sg_f2 __attribute__((ext_vector_type(2)));
#ifndef GROOT_SAGE_PRODUCERS
#define GROOT_SAGE_PRODUCERS 8      // 4 (one per SIMD, 16 rows each, four register sets) measured 30.3 ms against 29.2
#endif
constexpr int kSgConsumers = 4, kSgProducers = GROOT_SAGE_PRODUCERS;
constexpr int kSgThreads = (kSgConsumers + kSgProducers) * kWave;   // 768
constexpr int kSgProdRows = kSgRows / kSgProducers;                 // rows of a tile per producer
constexpr int kSgGroups = kSgProdRows / 4;                          // lane-group sweeps (4 rows each) per producer and tile
constexpr int kSgD = 6;                     // entries of a row on the pipelined path (AIG rows with a self-loop: 2 to 6)
constexpr int kSgSlots = kSgProdRows * kSgD;                        // slots of a producer's rows
constexpr int kSgH = (kSgSlots + kWave - 1) / kWave;                // column indices per lane
static_assert(kSgProdRows + 1 <= kWave, "row pointers of a producer fit one wavefront");

__device__ __forceinline__ void sage_wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also fences global memory, which
// makes every wavefront wait for all of its loads and stores in flight.
__device__ __forceinline__ void sage_lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// A wavefront that issues matrix instructions back to back keeps the SIMD's vector issue to itself: the
// other wavefronts of that SIMD (here two producers) do not get a single instruction in, whatever their
// priority.  The consumers therefore pause for a few cycles after every four matrix instructions (kGap
// selects the pause), which is when the producers' address arithmetic, loads and sums are issued.
template <int kGap>
__device__ __forceinline__ void sage_consumer_pause()
{
    if (kGap == 1) asm volatile("s_nop 7");
    if (kGap == 2) asm volatile("s_nop 15");
    if (kGap == 3) asm volatile("s_nop 15\n\ts_nop 7");
    if (kGap == 4) asm volatile("s_nop 15\n\ts_nop 15");
}

// two fp32 values -> their bf16 roundings (nearest even), packed: a in the low half
__device__ __forceinline__ unsigned sage_pack2(float a, float b)
{
    const sg_f2 x = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(x, sg_bf2));
}

// (a, b) = hi + mid + lo, three packed bf16 pairs; the remainders are exact in fp32
__device__ __forceinline__ void sage_split3(float a, float b, unsigned &hi, unsigned &mid, unsigned &lo)
{
    hi = sage_pack2(a, b);
    float ra = a - __builtin_bit_cast(float, hi << 16), rb = b - __builtin_bit_cast(float, hi & 0xffff0000u);
    mid = sage_pack2(ra, rb);
    ra -= __builtin_bit_cast(float, mid << 16);
    rb -= __builtin_bit_cast(float, mid & 0xffff0000u);
    lo = sage_pack2(ra, rb);
}

// four consecutive elements k..k+3 of tile row `row` into the three planes of a split tile
__device__ __forceinline__ void sage_park_split(char *tile, int row, int k, v4f x)
{
    unsigned h0, m0, l0, h1, m1, l1;
    sage_split3(x[0], x[1], h0, m0, l0);
    sage_split3(x[2], x[3], h1, m1, l1);
    char *p = tile + row * kSgBRow + k * 2;
    *(sg_u2 *)p = (sg_u2){h0, h1};
    *(sg_u2 *)(p + kSgPlane) = (sg_u2){m0, m1};
    *(sg_u2 *)(p + 2 * kSgPlane) = (sg_u2){l0, l1};
}

template <int W, int kGap, bool kSplit>
__global__ __launch_bounds__(kSgThreads) __attribute__((amdgpu_waves_per_eu(kSgThreads / 256, kSgThreads / 256))) void sage_kernel(
    const int64_t *__restrict__ rowptr, const int32_t *__restrict__ col, const float *__restrict__ val,
    const v4f *__restrict__ X, v4f *H, int64_t zero_off, const float *__restrict__ Wn,
    const float *__restrict__ Ws, const float *__restrict__ bias, int relu, int64_t n, int32_t T, int64_t n_tiles, int64_t tiles_per_wg,
    int64_t wgs_per_xcd, int remap)
{
    constexpr int kABytes = kSplit ? 3 * kSgPlane : kSgRows * kSgAStride * 4;   // 52,224 or 33,792 B per tile
    __shared__ __align__(16) char s_Araw[2][kABytes];
    __shared__ __align__(16) float s_O[2][kSgRows * kSgOStride];       // 34,816 B
    __shared__ __align__(8) int64_t s_slot[kSgProducers][kSgSlots];  // byte offset (from X) of slot k of row r at [6 r + k]
    __shared__ __align__(8) float s_slotw[kSgProducers][kSgSlots];   // its weight (explicit weights only)
    __shared__ float s_inv[kSgProducers][kSgProdRows];

    const int wv = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int64_t lw = logical_block(wgs_per_xcd, remap);
    const int64_t tile_begin = lw * tiles_per_wg;
    const int64_t tile_end = tile_begin + tiles_per_wg < n_tiles ? tile_begin + tiles_per_wg : n_tiles;
    if (tile_begin >= tile_end) return;                          // the whole workgroup leaves

    if (wv < kSgConsumers) {
        // =================================== consumer ===================================
        const int w = wv;
        const int kq = l / 16, jcol = 16 * w + l % 16;           // k slot / output column
        const float bias_v = bias ? bias[jcol] : 0.0f;
        // Split path: matrix instruction (ks, pieces) contracts k = 32 ks + 8 kq + e, e = 0..7; a lane's B operand
        // is the eight weights Wcat[32 ks + 8 kq + e][jcol], cut once into bw[ks][piece].
        // fp32 path: a lane reads four consecutive k of a tile row at once (k = 16 j + 4 kq + i, i = 0..3); matrix
        // instruction (j, i) contracts the four k slots kq = 0..3, so its B operand is
        // bfrag[4 j + i] = Wcat[16 j + 4 kq + i][jcol].
        sg_u4 bw[kSplit ? 4 : 1][3];
        float bfrag[kSplit ? 1 : 32];
        if constexpr (kSplit) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    const int k = 32 * ks + 8 * kq + e;
                    const float w0 = k < 64 ? Wn[k * 64 + jcol] : Ws[(k - 64) * 64 + jcol];
                    const float w1 = k + 1 < 64 ? Wn[(k + 1) * 64 + jcol] : Ws[(k + 1 - 64) * 64 + jcol];
                    unsigned h, m, lo_;
                    sage_split3(w0, w1, h, m, lo_);
                    bw[ks][0][e / 2] = h;
                    bw[ks][1][e / 2] = m;
                    bw[ks][2][e / 2] = lo_;
                }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int k = 16 * j + 4 * kq + i;
                    bfrag[4 * j + i] = k < 64 ? Wn[k * 64 + jcol] : Ws[(k - 64) * 64 + jcol];
                }
        }
        sage_lds_barrier();                                      // the first tile is in s_A[0]
        int cur = 0;
        for (int64_t tile = tile_begin; tile < tile_end; ++tile) {
            float *o_tile = s_O[cur];
            v4f acc[4];
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) acc[rb] = (v4f){bias_v, bias_v, bias_v, bias_v};
            if constexpr (kSplit) {
                const char *a_base = s_Araw[cur] + (l % 16) * kSgBRow + 16 * kq;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    sg_u4 a[3][4];
#pragma unroll
                    for (int pc = 0; pc < 3; ++pc)
#pragma unroll
                        for (int rb = 0; rb < 4; ++rb)
                            a[pc][rb] = *(const sg_u4 *)(a_base + pc * kSgPlane + rb * 16 * kSgBRow + 64 * ks);
                    // the six piece products, smallest first; four independent accumulators per product
                    constexpr int kPa[6] = {1, 2, 0, 1, 0, 0}, kPb[6] = {1, 0, 2, 0, 1, 0};
#pragma unroll
                    for (int t = 0; t < 6; ++t) {
#pragma unroll
                        for (int rb = 0; rb < 4; ++rb)
                            acc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(sg_bf8, a[kPa[t]][rb]),
                                                                              __builtin_bit_cast(sg_bf8, bw[ks][kPb[t]]),
                                                                              acc[rb], 0, 0, 0);
                        sage_consumer_pause<kGap>();
                    }
                }
            } else {
            const float *a_tile = (const float *)s_Araw[cur];
            // operands of step j+1 are read while the 16 matrix instructions of step j run
            v4f a[2][4];
#pragma unroll
            for (int rb = 0; rb < 4; ++rb)
                a[0][rb] = *(const v4f *)&a_tile[(rb * 16 + l % 16) * kSgAStride + 4 * kq];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (j + 1 < 8) {
#pragma unroll
                    for (int rb = 0; rb < 4; ++rb)
                        a[(j + 1) & 1][rb] = *(const v4f *)&a_tile[(rb * 16 + l % 16) * kSgAStride + 16 * (j + 1) + 4 * kq];
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
#pragma unroll
                    for (int rb = 0; rb < 4; ++rb)
                        acc[rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[j & 1][rb][i], bfrag[4 * j + i], acc[rb], 0, 0, 0);
                    sage_consumer_pause<kGap>();
                }
            }
            }
            // result (lane holds rows 4 kq + r of its column) to the output tile
#pragma unroll
            for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float v = acc[rb][r];
                    if (relu) v = v > 0.0f ? v : 0.0f;
                    o_tile[(rb * 16 + 4 * kq + r) * kSgOStride + jcol] = v;
                }
            sage_lds_barrier();
            cur ^= 1;
        }
        return;
    }

    // =================================== producer ===================================
    const int p = wv - kSgConsumers;             // rows 8p .. 8p+7 of every tile
    const int g = l / 16, f = l % 16;            // lane group / float4 slice

    // ---- CSR pipeline for the producer's 8 rows of a tile
    // rp_a: row pointers of the tile whose column indices are in cc (the next tile to be staged);
    // rp_b: row pointers of the tile after that.
    int64_t rp_a = 0, rp_b = 0;
    int32_t cc[kSgH];
    float vv[kSgH];
#pragma unroll
    for (int h = 0; h < kSgH; ++h) { cc[h] = 0; vv[h] = 0.f; }
    bool simple_a = false;
    auto load_rp = [&](int64_t tile) -> int64_t {
        const int64_t ri = tile * kSgRows + kSgProdRows * p + (l < kSgProdRows ? l : kSgProdRows);
        return rowptr[ri < n ? ri : n];          // lanes 0..kSgProdRows hold the pointers; rows past the end read rowptr[n]
    };
    // The producer's rows are "simple" when every row has at most kSgD entries and none is high-degree:
    // they go through the pipelined path.
    auto load_cols = [&]() {                     // from rp_a
        const int64_t begin = __shfl(rp_a, 0), t_end = __shfl(rp_a, kSgProdRows), rp_next = __shfl_down(rp_a, 1);
        const int64_t len = rp_next - rp_a;
        simple_a = __ballot(l < kSgProdRows && (len > kSgD || len >= T)) == 0;
        const int32_t m = simple_a ? (int32_t)(t_end - begin) : 0;
        // unconditional loads (lanes past the end read entry 0): the number of loads in flight stays known
#pragma unroll
        for (int h = 0; h < kSgH; ++h) {
            const int64_t i = l + kWave * h < m ? begin + l + kWave * h : 0;
            cc[h] = __builtin_nontemporal_load(&col[i]);
            if (W == kExplicit) vv[h] = __builtin_nontemporal_load(&val[i]);
        }
    };
    // rp_a, cc -> LDS as a slot table: every row gets exactly kSgD slots, lane s (and s + 64) prepares slot
    // k of row r, s = 6 r + k, as the byte offset of the gathered row from X.  A slot past the row's end
    // points at a row of zeros outside X, so the sum of a row is the plain sum of its kSgD slots.  Rows of
    // a tile that is not simple are staged as empty.  All index arithmetic of the gathers is done here,
    // once per tile and in parallel over the lanes, not per gathered row.
    bool simple_iss = false;                     // whether the tile now in the slot table is simple
    auto stage = [&]() {
        simple_iss = simple_a;
        const int32_t rel = simple_a ? (int32_t)(rp_a - __shfl(rp_a, 0)) : 0;
#pragma unroll
        for (int h = 0; h < kSgH; ++h) {
            const int s_ = l + kWave * h;
            const int r = s_ / kSgD, k = s_ - r * kSgD;
            const int32_t lo = __shfl(rel, r), hi = __shfl(rel, r + 1);
            const int src = lo + k;
            int32_t c = 0;
            float wv_ = 0.f;
#pragma unroll
            for (int q = 0; q < kSgH; ++q) {
                const int32_t cq = __shfl(cc[q], src - kWave * q);
                c = (src >> 6) == q ? cq : c;
                if (W == kExplicit) {
                    const float wq = __shfl(vv[q], src - kWave * q);
                    wv_ = (src >> 6) == q ? wq : wv_;
                }
            }
            const bool live = k < hi - lo;
            if (s_ < kSgSlots) {
                s_slot[p][s_] = live ? ((int64_t)c << 8) : zero_off;
                if (W == kExplicit) s_slotw[p][s_] = live ? wv_ : 0.f;
            }
        }
        const int32_t len = __shfl_down(rel, 1) - rel;           // all lanes take part in the exchange
        if (l < kSgProdRows) s_inv[p][l] = row_weight<W>(len);   // lane r: weight of row r
        sage_wave_sync();
    };

    // ---- aggregation of four simple rows (one per lane group) in two halves, a whole tile apart: the
    //      loads of a group of tile t+2 are issued right after the same group of tile t+1 has been
    //      summed.  The issue does not branch and every lane issues all kSgD + 1 loads, so the number
    //      of loads in flight is known at compile time and the wait before a group's sum lets the
    //      younger loads fly on.
    struct RowRegs {
        v4f xs[kSgD], self;
        float ws[kSgD];
        float inv;
    };
    RowRegs rr[kSgGroups];
    const char *Xf = (const char *)X + 16 * f;                   // this lane's float4 slice of row 0
    auto issue = [&](RowRegs &q, int64_t tile, int grp) {
        const int lr = grp * 4 + g;
        int64_t row = tile * kSgRows + kSgProdRows * p + lr;
        row = row < n ? row : n - 1;
        q.inv = s_inv[p][lr];
        q.self = *(const v4f *)(Xf + (row << 8));
#pragma unroll
        for (int k = 0; k < kSgD; ++k) {
            const int64_t off = s_slot[p][lr * kSgD + k];
            if (W == kExplicit) q.ws[k] = s_slotw[p][lr * kSgD + k];
            q.xs[k] = *(const v4f *)(Xf + off);
        }
    };
    // a row's [agg | self] slice of this lane into the LDS tile: fp32, or cut into the three bf16 planes
    auto park = [&](char *buf, int row_in_tile, v4f agg, v4f self) {
        if constexpr (kSplit) {
            sage_park_split(buf, row_in_tile, 4 * f, agg);
            sage_park_split(buf, row_in_tile, 64 + 4 * f, self);
        } else {
            float *dst = (float *)buf + row_in_tile * kSgAStride + 4 * f;
            *(v4f *)dst = agg;
            *(v4f *)(dst + 64) = self;
        }
    };
    auto finish = [&](RowRegs &q, int grp, char *buf) {
        const int lr = grp * 4 + g;
        v4f agg = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < kSgD; ++k) {
            if (W == kExplicit) agg += q.ws[k] * q.xs[k];
            else agg += q.xs[k];
        }
        if (W != kExplicit) agg *= q.inv;
        park(buf, kSgProdRows * p + lr, agg, q.self);            // rows past the end are never stored
    };
    // Any other row (long, high-degree, or next to one): straight from global memory, not overlapped.
    auto slow_rows = [&](int64_t tile, int grp, char *buf) {
        const int lr = grp * 4 + g;
        const int64_t row = tile * kSgRows + kSgProdRows * p + lr;
        v4f agg = {0.f, 0.f, 0.f, 0.f}, self = {0.f, 0.f, 0.f, 0.f};
        if (row < n) {
            self = X[row * kSgF4 + f];
            const int64_t s = rowptr[row], e = rowptr[row + 1];
            if (e - s >= T) agg = H[row * kSgF4 + f];            // aggregated by the HD kernel
            else agg = ld_row_sum<W, false, kSgD>(s, e, col, val, X, kSgF4, f);
        }
        park(buf, kSgProdRows * p + lr, agg, self);
    };
    // The producer's 8 rows of a finished tile: LDS output tile -> H, full rows.
    auto store_rows = [&](int64_t tile, const float *o_tile) {
#pragma unroll
        for (int grp = 0; grp < kSgGroups; ++grp) {
            const int lr = grp * 4 + g;
            const int64_t row = tile * kSgRows + kSgProdRows * p + lr;
            if (row < n)
                __builtin_nontemporal_store(*(const v4f *)&o_tile[(kSgProdRows * p + lr) * kSgOStride + 4 * f],
                                            &H[row * kSgF4 + f]);
        }
    };

    // ---- prologue: the first tile is aggregated on its own, the second one is put in flight
#pragma unroll 1
    for (int grp = 0; grp < kSgGroups; ++grp) slow_rows(tile_begin, grp, s_Araw[0]);
    rp_a = load_rp(tile_begin + 1);
    load_cols();
    stage();
    bool simple_fin = simple_iss;                                // tile_begin + 1: summed during the first phase
    rp_a = load_rp(tile_begin + 2);                              // same order of loads as in the loop: CSR, then rows
    load_cols();
    rp_b = load_rp(tile_begin + 3);
#pragma unroll
    for (int grp = 0; grp < kSgGroups; ++grp) issue(rr[grp], tile_begin + 1, grp);
    sage_lds_barrier();

    int cur = 0;
    for (int64_t tile = tile_begin; tile < tile_end; ++tile) {
        // While the consumers multiply `tile` (s_A[cur] -> s_O[cur]): store the result of tile-1, finish
        // tile+1 into s_A[cur^1], put tile+2 in flight.  Past the workgroup's last tile the pipeline runs
        // on empty: the loads still go to valid addresses, the sums land in the LDS tile nobody reads.
        char *a_next = s_Araw[cur ^ 1];
        stage();                                                 // CSR of tile+2 -> slot table
        rp_a = rp_b;
        load_cols();                                             // column indices of tile+3
        rp_b = load_rp(tile + 4);
        if (tile > tile_begin) store_rows(tile - 1, s_O[cur ^ 1]);
#pragma unroll
        for (int grp = 0; grp < kSgGroups; ++grp) {
            finish(rr[grp], grp, a_next);
            issue(rr[grp], tile + 2, grp);
        }
        if (!simple_fin) {                                       // rare: redo the producer's rows of tile+1
#pragma unroll 1
            for (int grp = 0; grp < kSgGroups; ++grp) slow_rows(tile + 1, grp, a_next);
        }
        simple_fin = simple_iss;
        sage_lds_barrier();
        cur ^= 1;
    }
    store_rows(tile_end - 1, s_O[cur ^ 1]);
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
    // persistent workgroups: one per CU (its 12 wavefronts fill three of a SIMD's wavefront slots each)
    int64_t n_wg = (cus + kXcds - 1) / kXcds * kXcds;
    if (n_wg > n_tiles) n_wg = n_tiles;
    const int remap = dp.xcd_remap && n_wg % kXcds == 0 && n_wg >= 4 * kXcds;
    const int64_t tiles_per_wg = (n_tiles + n_wg - 1) / n_wg;
    if (!grid_ok(n_wg)) return (int)hipErrorInvalidConfiguration;
    if (!weights_ok(dp) || !dp.zero_row) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    // the kernel reads entry 0 of the index (and weight) array from idle lanes: give it something to read
    // when the matrix has no entries, or no weight array
    const int32_t *col_arg = dp.col ? dp.col : (const int32_t *)dp.rowptr;
    const float *val_arg = dp.val ? dp.val : (const float *)dp.rowptr;
#define GROOT_SAGE_LAUNCH2(GAP, SPLIT)                                                                               \
    GROOT_DISPATCH_W(dp.weight_mode, (sage_kernel<kW, GAP, SPLIT><<<dim3((unsigned)n_wg), dim3(kSgThreads), 0, st>>>(    \
                                         dp.rowptr, col_arg, val_arg, (const v4f *)X, (v4f *)H, byte_distance(X, dp.zero_row), Wn, Ws, bias, \
                                         relu, dp.n, dp.threshold, n_tiles, tiles_per_wg, n_wg / kXcds, remap)))
#define GROOT_SAGE_LAUNCH(GAP)                                  \
    if (tuning().sage_split) { GROOT_SAGE_LAUNCH2(GAP, true); } \
    else { GROOT_SAGE_LAUNCH2(GAP, false); }
    switch (tuning().sage_gap.load()) {
    case 0: GROOT_SAGE_LAUNCH(0); break;
    case 1: GROOT_SAGE_LAUNCH(1); break;
    case 3: GROOT_SAGE_LAUNCH(3); break;
    case 4: GROOT_SAGE_LAUNCH(4); break;
    default: GROOT_SAGE_LAUNCH(2); break;
    }
#undef GROOT_SAGE_LAUNCH
#undef GROOT_SAGE_LAUNCH2
    return (int)hipGetLastError();
}

}  // namespace groot
