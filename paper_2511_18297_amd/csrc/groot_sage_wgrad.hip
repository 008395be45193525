// Weight gradients of the fused GraphSAGE-mean layer for gfx950:
//     dWn = (A_hat X)^T dZ,   dWs = X^T dZ,   X [N, FI], dZ [N, FO], dWn and dWs [FI, FO], FI = 32 or 64, FO = 16, 32 or 64
//     (described below for FI = FO = F = 64),
// for the layer Z = (A_hat X) Wn + X Ws + b with dZ the gradient of the loss at Z (Section "GNN and Edge
// Re-growth After Partition": the model is trained).  Two products with N as the contraction length: as plain
// matrix products over [N, 64] operands they take 58 ms each on 134 M rows with the vendor library, and the
// first needs A_hat X in memory.  Here one pass does both with the aggregation kept on chip.
//
// The aggregation is the fused layer kernel's (groot_sage_pipe.hip: a persistent workgroup per CU, every
// wavefront walks its own 16-row tiles and keeps the next tile's gathers in flight; slot table in LDS, a row of
// zeros for dead slots, a plain path for the tiles that hold a row the slots do not serve).  For every tile the
// wavefront has [A_hat X | X] (16 x 2F) and dZ (16 x F) in registers and adds [A_hat X | X]^T dZ (2F x F) to
// accumulators that it keeps for its whole sweep: 8 x 4 blocks of v_mfma_f32_16x16x16_bf16 at F = 64, the
// tile's 16 rows being the contraction length of one instruction.  fp32 accuracy as in the forward layer:
// every operand is cut into three bf16 pieces and six piece products are kept (two pieces and three products
// with the library's sage_pieces knob at 2).
//
// The matrix instruction wants, per lane, four consecutive contraction indices of one column of an operand, and
// here the contraction runs over rows, of which a lane holds one per sweep.  So the tile goes through LDS
// transposed, [column][row], and the rows are numbered so that the ones a lane holds are neighbours: row
// r = grp * kRpg + g of the tile (sweep grp, lane group g) is contraction index g * kG + grp, for both operands.
// A lane then writes its kG rows of one column as one 8-byte (F = 32: 4-byte) word, cut into pieces pairwise
// (the pair of rows of a word's half is what one cut of two values packs).
//
// Every wavefront ends by writing its 2F x F sums to its own slice of a workspace; a second kernel adds the
// slices in a fixed order in fp64.  No atomics: the result is the same on every run.
#include <type_traits>

#include "groot_device.h"

namespace groot {

constexpr int kWgRows = 16;                  // rows per tile: the contraction length of one matrix instruction
// wavefronts per workgroup (one workgroup per CU): one per SIMD at F = 64, where the accumulators alone take 128
// registers; two per SIMD at F = 32 (32 accumulator registers), so that one's vector work overlaps the other's matrix work
constexpr int wg_waves(int FI) { return FI == 64 ? 4 : 8; }
constexpr int kWgTRow = kWgRows * 2 + 8;     // bytes per column of a transposed bf16 plane (8 B of padding)

typedef float wg_f2 __attribute__((ext_vector_type(2)));
typedef __bf16 wg_bf2 __attribute__((ext_vector_type(2)));
typedef short wg_s4 __attribute__((ext_vector_type(4)));
typedef unsigned int wg_u2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void wg_wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// two fp32 values -> their bf16 roundings (nearest even), packed: a in the low half
__device__ __forceinline__ unsigned wg_pack2(float a, float b)
{
    const wg_f2 x = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(x, wg_bf2));
}

// (a, b) = hi + mid + lo, three packed bf16 pairs; the remainders are exact in fp32
__device__ __forceinline__ void wg_split3(float a, float b, unsigned (&pc)[3])
{
    pc[0] = wg_pack2(a, b);
    float ra = a - __builtin_bit_cast(float, pc[0] << 16), rb = b - __builtin_bit_cast(float, pc[0] & 0xffff0000u);
    pc[1] = wg_pack2(ra, rb);
    ra -= __builtin_bit_cast(float, pc[1] << 16);
    rb -= __builtin_bit_cast(float, pc[1] & 0xffff0000u);
    pc[2] = wg_pack2(ra, rb);
}

// The kG rows that one lane holds of columns c0 .. c0 + 3, into the P transposed planes: v[grp][j] is the value of
// row grp * kRpg + g, column c0 + j; the word of column c0 + j starts at contraction index g * kG.
template <int kG, int P, int kPlane>
__device__ __forceinline__ void wg_park(char *planes, int c0, int g, const v4f (&v)[kG])
{
    static_assert(kG == 4 || kG == 2, "four or two rows per lane");
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        char *p = planes + (c0 + j) * kWgTRow + g * kG * 2;
        unsigned lo[3], hi[3];
        wg_split3(v[0][j], v[1][j], lo);
        if constexpr (kG == 4) {
            wg_split3(v[2][j], v[3][j], hi);
#pragma unroll
            for (int q = 0; q < P; ++q) *(wg_u2 *)(p + q * kPlane) = (wg_u2){lo[q], hi[q]};
        } else {
#pragma unroll
            for (int q = 0; q < P; ++q) *(unsigned *)(p + q * kPlane) = lo[q];
        }
    }
}

// W: kOnes or kMean; FI: width of X; FO: width of dZ; D: gather slots per row on the pipelined path; P: bf16 pieces per
// operand.  The rows of dZ are loaded by the lane groups that load the rows of X (FI / 4 lanes per row): FO / FI float4
// per lane, or one with the lanes past the row's end idle.
template <int W, int FI, int FO, int D, int P>
__global__ __launch_bounds__(wg_waves(FI) * kWave) __attribute__((amdgpu_waves_per_eu(wg_waves(FI) / 4, wg_waves(FI) / 4))) void sage_wgrad_kernel(
    const int64_t *__restrict__ rowptr, const int32_t *__restrict__ col, const float *__restrict__ val,
    const char *__restrict__ X, const char *__restrict__ dZ, int64_t zero_off, int64_t n, int32_t T, int64_t n_tiles,
    int64_t tiles_per_part, int64_t waves_per_part, int32_t parts, const int32_t *__restrict__ hd_rows, int32_t n_hd,
    const char *__restrict__ hd_agg, float *__restrict__ partials)
{
    static_assert(FI == 64 || FI == 32, "width of X");
    static_assert(FO == 64 || FO == 32 || FO == 16, "width of dZ");
    static_assert(P == 3 || P == 2, "pieces per operand");
    static_assert(W == kOnes || W == kMean, "row-uniform weights");
    constexpr int F = FI;
    constexpr int kWgWaves = wg_waves(FI);
    constexpr int kL = F / 4, kRpg = kWave / kL, kG = kWgRows / kRpg, kRowShift = F == 64 ? 8 : 7;
    constexpr int kZShift = FO == 64 ? 8 : FO == 32 ? 7 : 6;             // log2 of a row of dZ in bytes
    constexpr int kZ = (FO / 4 + kL - 1) / kL;                           // float4 of a row of dZ per lane
    constexpr int kM = 2 * F, kMb = kM / 16, kNb = FO / 16;
    constexpr int kPlaneA = kM * kWgTRow, kPlaneB = FO * kWgTRow;
    constexpr int kSlots = kWgRows * D, kH = (kSlots + kWave - 1) / kWave;
    __shared__ __align__(16) int64_t s_slot[kWgWaves][kSlots];
    __shared__ float s_inv[kWgWaves][kWgRows];
    __shared__ __align__(16) char s_A[kWgWaves][P * kPlaneA];            // F = 64, P = 3: 15,360 B per wavefront
    __shared__ __align__(16) char s_B[kWgWaves][P * kPlaneB];            //                  7,680 B

    const int w = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int g = l / kL, f = l % kL;
    const int kq = l / 16, jl = l % 16;                  // matrix instruction: contraction quarter / row of A, column of B and D
    const int64_t part = blockIdx.x % parts, j = (blockIdx.x / parts) * kWgWaves + w;
    const int64_t x_begin = part * tiles_per_part;
    const int64_t x_end = x_begin + tiles_per_part < n_tiles ? x_begin + tiles_per_part : n_tiles;
    const int64_t t_first = x_begin + j, stride = waves_per_part;
    const char *Xf = X + 16 * f;
    const bool z_lane = 4 * f < FO;                      // kZ == 1: this lane holds four columns of dZ
    const char *Zf = dZ + 16 * (z_lane ? f : 0);         // an idle lane reads the row's first columns and parks nothing

    v4f acc[kMb][kNb];
#pragma unroll
    for (int mb = 0; mb < kMb; ++mb)
#pragma unroll
        for (int nb = 0; nb < kNb; ++nb) acc[mb][nb] = (v4f){0.f, 0.f, 0.f, 0.f};

    if (t_first < x_end) {
        // ---- CSR pipeline: rp_a and cc belong to the next tile to be staged, rp_b to the one after
        int64_t rp_a = 0, rp_b = 0;
        int32_t cc[kH];
#pragma unroll
        for (int h = 0; h < kH; ++h) cc[h] = 0;
        bool fix_a = true;                               // the tile has rows that the slots do not serve (or is ragged)
        int32_t len_a = 0;                               // lanes 0..15: stored length of the tile's row
        uint32_t live_a = 0;                             // bit h: slot l + 64 h holds an entry
        auto load_rp = [&](int64_t tile) -> int64_t {
            const int64_t ri = tile * kWgRows + (l < kWgRows ? l : kWgRows);
            return rowptr[ri < n ? ri : n];              // lanes 0..16 hold the pointers; rows past the end read rowptr[n]
        };
        auto load_cols = [&](int64_t tile) {             // from rp_a: every slot fetches its own entry
            const bool full = (tile + 1) * kWgRows <= n && tile < x_end;
            const int64_t begin = __shfl(rp_a, 0);
            const int32_t rel = full ? (int32_t)(rp_a - begin) : 0;
            len_a = __shfl_down(rel, 1) - rel;
            fix_a = !full || __ballot(l < kWgRows && (len_a > D || len_a >= T)) != 0;
            live_a = 0;
#pragma unroll
            for (int h = 0; h < kH; ++h) {               // unconditional loads (a dead slot reads entry 0)
                const int s = l + kWave * h;             // slot s: row r, entry k
                const int r = s / D, k = s - r * D;
                const int32_t lo = __shfl(rel, r), len = __shfl(rel, r + 1) - lo;
                const bool live = s < kSlots && k < len && len <= D && len < T;
                live_a |= (uint32_t)live << h;
                cc[h] = __builtin_nontemporal_load(&col[live ? begin + lo + k : 0]);
            }
        };
        auto stage = [&]() -> bool {                     // cc, live_a, len_a -> slot table and row weights; -> fix_a
#pragma unroll
            for (int h = 0; h < kH; ++h) {
                const int s = l + kWave * h;
                if (s < kSlots) s_slot[w][s] = ((live_a >> h) & 1) ? ((int64_t)cc[h] << kRowShift) : zero_off;
            }
            if (W == kMean && l < kWgRows) s_inv[w][l] = row_weight<kMean>(len_a);
            wg_wave_sync();
            return fix_a;
        };
        // ---- one sweep: kRpg rows, one per lane group: the row's D slots, its own features and its row of dZ
        struct Regs {
            v4f xs[D], self, dz[kZ];
            float inv;
        };
        Regs rr[kG];
        auto issue = [&](Regs &q, int64_t tile, int grp) {
            const int lr = grp * kRpg + g;
            int64_t row = tile * kWgRows + lr;
            row = row < n ? row : n - 1;                 // past the end: any valid row, the values are replaced by zeros
            if (W == kMean) q.inv = s_inv[w][lr];
#pragma unroll
            for (int k = 0; k < D; ++k) q.xs[k] = *(const v4f *)(Xf + s_slot[w][lr * D + k]);
            q.self = *(const v4f *)(Xf + (row << kRowShift));
#pragma unroll
            for (int i = 0; i < kZ; ++i) q.dz[i] = *(const v4f *)(Zf + (row << kZShift) + 16 * kL * i);
        };
        auto sum = [&](const Regs &q) -> v4f {
            v4f a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int k = 0; k < D; ++k) a += q.xs[k];
            if (W == kMean) a *= q.inv;
            return a;
        };

        // ---- prologue: the first tile is staged and put in flight, the CSR of the next two is on its way
        rp_a = load_rp(t_first);
        load_cols(t_first);
        bool fix_cur = stage();
        rp_a = load_rp(t_first + stride);
        load_cols(t_first + stride);
        rp_b = load_rp(t_first + 2 * stride);
#pragma unroll
        for (int grp = 0; grp < kG; ++grp) issue(rr[grp], t_first, grp);
        __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0): the loop's own order of loads is the only one from here on

        char *const a_t = s_A[w], *const b_t = s_B[w];
        for (int64_t tile = t_first; tile < x_end; tile += stride) {
            const bool fix_next = stage();               // CSR of the next tile -> slot table (this tile's sweeps are all issued)
            rp_a = rp_b;
            load_cols(tile + 2 * stride);
            rp_b = load_rp(tile + 3 * stride);
            const int64_t base = tile * kWgRows;
            // this tile's values out of the register sets, which take the rows of the next tile
            v4f av[kG], sv[kG], zv[kZ][kG];
#pragma unroll
            for (int grp = 0; grp < kG; ++grp) {
                const bool in = base + grp * kRpg + g < n;
                const v4f zero = {0.f, 0.f, 0.f, 0.f};
                av[grp] = sum(rr[grp]);                  // a ragged tile has no live slot: zeros
                sv[grp] = in ? rr[grp].self : zero;
#pragma unroll
                for (int i = 0; i < kZ; ++i) zv[i][grp] = in ? rr[grp].dz[i] : zero;
                issue(rr[grp], tile + stride, grp);
            }
            if (fix_cur) {
                // plain path: the rows of this tile that had no live slots (more entries than slots, high-degree, or
                // every row of the ragged last tile), straight from global memory; high-degree sums from the side buffer
#pragma unroll
                for (int grp = 0; grp < kG; ++grp) {
                    const int64_t row = base + grp * kRpg + g;
                    const bool full = base + kWgRows <= n;
                    if (row < n) {
                        const int64_t s = rowptr[row], e = rowptr[row + 1];
                        if (e - s >= T) {
                            int32_t lo = 0, hi = n_hd;   // the row's place in the list of high-degree rows
                            while (lo < hi) {
                                const int32_t mid = (lo + hi) / 2;
                                if (hd_rows[mid] < row) lo = mid + 1; else hi = mid;
                            }
                            av[grp] = *(const v4f *)(hd_agg + ((int64_t)lo << kRowShift) + 16 * f);
                        } else if (!full || e - s > D) {
                            av[grp] = ld_row_sum<W, false, 8>(s, e, col, val, (const v4f *)X, kL, f);
                        }
                    }
                }
            }
            // transposed into LDS, cut into pieces: [A_hat X | X] and dZ
            wg_park<kG, P, kPlaneA>(a_t, 4 * f, g, av);
            wg_park<kG, P, kPlaneA>(a_t, F + 4 * f, g, sv);
            if (z_lane) {
#pragma unroll
                for (int i = 0; i < kZ; ++i) wg_park<kG, P, kPlaneB>(b_t, 4 * (f + kL * i), g, zv[i]);
            }
            wg_wave_sync();
            // ---- [A_hat X | X]^T (2F x 16) times dZ (16 x F): lane (jl, kq) reads column jl of a block, rows 4 kq .. 4 kq + 3
            wg_u2 bop[kNb][P];
#pragma unroll
            for (int nb = 0; nb < kNb; ++nb)
#pragma unroll
                for (int pb = 0; pb < P; ++pb)
                    bop[nb][pb] = *(const wg_u2 *)(b_t + pb * kPlaneB + (16 * nb + jl) * kWgTRow + 8 * kq);
#pragma unroll
            for (int mb = 0; mb < kMb; ++mb) {
                wg_u2 aop[P];
#pragma unroll
                for (int pa = 0; pa < P; ++pa)
                    aop[pa] = *(const wg_u2 *)(a_t + pa * kPlaneA + (16 * mb + jl) * kWgTRow + 8 * kq);
                // the piece products that are kept: pa + pb < P, the smallest first
#pragma unroll
                for (int pb = P - 1; pb >= 0; --pb)
#pragma unroll
                    for (int pa = P - 1 - pb; pa >= 0; --pa)
#pragma unroll
                        for (int nb = 0; nb < kNb; ++nb)
                            acc[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(
                                __builtin_bit_cast(wg_s4, aop[pa]), __builtin_bit_cast(wg_s4, bop[nb][pb]), acc[mb][nb], 0, 0, 0);
            }
            wg_wave_sync();                              // all reads of the parked tile are done
            fix_cur = fix_next;
        }
    }
    // ---- this wavefront's sums to its slice of the workspace (zeros if it had no tile): lane holds rows
    //      16 mb + 4 kq + r of column 16 nb + jl
    float *mine = partials + ((int64_t)blockIdx.x * kWgWaves + w) * (kM * FO);
#pragma unroll
    for (int mb = 0; mb < kMb; ++mb)
#pragma unroll
        for (int nb = 0; nb < kNb; ++nb)
#pragma unroll
            for (int r = 0; r < 4; ++r) mine[(16 * mb + 4 * kq + r) * FO + 16 * nb + jl] = acc[mb][nb][r];
}

// dWn[m][n] (m < FI) and dWs[m - FI][n] = sum over the slices, in slice order, in fp64; half = FI * FO
__global__ __launch_bounds__(kBlock) void sage_wgrad_reduce_kernel(const float *__restrict__ partials, int64_t slices,
                                                                   int32_t half, float *__restrict__ dWn,
                                                                   float *__restrict__ dWs)
{
    const int32_t e = blockIdx.x * kBlock + threadIdx.x, count = 2 * half;
    if (e >= count) return;
    double s = 0.0;
#pragma unroll 8
    for (int64_t k = 0; k < slices; ++k) s += (double)partials[k * count + e];
    if (e < half) dWn[e] = (float)s;
    else dWs[e - half] = (float)s;
}

static int64_t wgrad_workgroups()
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return -1;
    int64_t n_wg = cus / kXcds * kXcds;                  // one workgroup per CU; consecutive workgroup ids land on different XCDs
    return n_wg < kXcds ? kXcds : n_wg;
}

// bytes of workspace that launch_sage_wgrad needs for these widths on the current device (0 on failure)
size_t sage_wgrad_workspace_bytes(int32_t FI, int32_t FO)
{
    const int64_t n_wg = wgrad_workgroups();
    return n_wg < 0 ? 0 : (size_t)n_wg * wg_waves(FI) * 2 * (size_t)FI * (size_t)FO * sizeof(float);
}

int launch_sage_wgrad(const DevicePlan &dp, const float *X, const float *dZ, float *dWn, float *dWs, int32_t FI, int32_t FO,
                      int pieces, void *workspace, void *stream)
{
    if (!weights_ok(dp) || !dp.zero_row || (FI != 64 && FI != 32) || (FO != 64 && FO != 32 && FO != 16) ||
        (pieces != 2 && pieces != 3) || !workspace)
        return (int)hipErrorInvalidValue;
    if (dp.weight_mode == kExplicit) return (int)hipErrorInvalidValue;
    if (dp.n_hd_rows && (!dp.hd_rows || !dp.hd_agg)) return (int)hipErrorInvalidValue;
    const int64_t n_wg = wgrad_workgroups();
    if (n_wg < 0) return (int)hipErrorInvalidDevice;
    const int64_t n_tiles = (dp.n + kWgRows - 1) / kWgRows;
    const int32_t parts = dp.xcd_remap ? kXcds : 1;
    const int64_t tiles_per_part = (n_tiles + parts - 1) / parts;
    const int64_t waves_per_part = n_wg / parts * wg_waves(FI);
    if (!grid_ok(n_wg) || n_tiles <= 0) return (int)hipErrorInvalidConfiguration;
    // the kernel reads entry 0 of the index array from idle lanes: give it something to read when the matrix has no entries
    const int32_t *col_arg = dp.col ? dp.col : (const int32_t *)dp.rowptr;
    const float *val_arg = dp.val ? dp.val : (const float *)dp.rowptr;
    hipStream_t st = (hipStream_t)stream;
#define GROOT_WGRAD_LAUNCH(WM, FFI, FFO, DD, PP)                                                                         \
    sage_wgrad_kernel<WM, FFI, FFO, DD, PP><<<dim3((unsigned)n_wg), dim3(wg_waves(FFI) * kWave), 0, st>>>(                 \
        dp.rowptr, col_arg, val_arg, (const char *)X, (const char *)dZ, byte_distance(X, dp.zero_row), dp.n, dp.threshold, \
        n_tiles, tiles_per_part, waves_per_part, parts, dp.hd_rows, (int32_t)dp.n_hd_rows, (const char *)dp.hd_agg,    \
        (float *)workspace)
#define GROOT_WGRAD_P(WM, FFI, FFO, DD)                        \
    if (pieces == 2) GROOT_WGRAD_LAUNCH(WM, FFI, FFO, DD, 2);  \
    else GROOT_WGRAD_LAUNCH(WM, FFI, FFO, DD, 3)
#define GROOT_WGRAD_D(WM, FFI, FFO)                                  \
    if (dp.sage_depth == 5) { GROOT_WGRAD_P(WM, FFI, FFO, 5); }      \
    else { GROOT_WGRAD_P(WM, FFI, FFO, 6); }
#define GROOT_WGRAD_FO(WM, FFI)                          \
    if (FO == 64) { GROOT_WGRAD_D(WM, FFI, 64); }        \
    else if (FO == 32) { GROOT_WGRAD_D(WM, FFI, 32); }   \
    else { GROOT_WGRAD_D(WM, FFI, 16); }
    if (FI == 64) {
        if (dp.weight_mode == kMean) { GROOT_WGRAD_FO(kMean, 64); }
        else { GROOT_WGRAD_FO(kOnes, 64); }
    } else {
        if (dp.weight_mode == kMean) { GROOT_WGRAD_FO(kMean, 32); }
        else { GROOT_WGRAD_FO(kOnes, 32); }
    }
#undef GROOT_WGRAD_FO
#undef GROOT_WGRAD_D
#undef GROOT_WGRAD_P
#undef GROOT_WGRAD_LAUNCH
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return (int)err;
    const int32_t count = 2 * FI * FO;
    sage_wgrad_reduce_kernel<<<dim3((unsigned)((count + kBlock - 1) / kBlock)), dim3(kBlock), 0, st>>>(
        (const float *)workspace, n_wg * wg_waves(FI), FI * FO, dWn, dWs);
    return (int)hipGetLastError();
}

}  // namespace groot
