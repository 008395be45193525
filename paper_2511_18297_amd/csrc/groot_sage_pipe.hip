// Fused GraphSAGE-mean layer for gfx950, self-contained wavefronts (two per SIMD):
//     H = act((A_hat X) Wn + X Ws + b),   X [N, FI], Wn and Ws [FI, FO], H [N, FO], FI = 32 or 64, FO = 16, 32 or 64
//     (described below for FI = FO = 64).
//
// The aggregation is the software-pipelined LD kernel's (a persistent workgroup per CU, every wavefront walks
// its own tiles and keeps a whole tile of gathers in flight; slot table in LDS, zero row for dead slots, no
// workgroup barrier after the start).  A tile here is 16 rows, the height of a matrix instruction.  Instead
// of storing the 16 sums, the wavefront parks [A_hat X | X] of its tile in its own LDS region, multiplies it
// with the stacked weights [Wn; Ws] (128 x 64) on the matrix cores, passes the 16 x 64 result through LDS once
// more to get whole rows per lane group, and stores them.  Nothing is shared between wavefronts, so nothing
// waits for another wavefront; while a wavefront multiplies, the gathers of its next tile are in flight, and
// the second wavefront of its SIMD issues whenever the first one waits (with one wavefront per SIMD, which
// could keep the weights in registers, every wait of that wavefront idles the SIMD: 25.9 against 24.5 ms of
// the 12-wavefront kernel).
//
// The dense product keeps fp32 accuracy on the bf16 matrix instruction (v_mfma_f32_16x16x32_bf16, a sixteenth
// of the fp32 instruction's time per multiply-add): every fp32 operand is cut into three bf16 pieces,
// x = hi + mid + lo up to 2^-24 |x|, and a product keeps the six piece products down to 2^-16 relative size
// (hi hi, hi mid, mid hi, hi lo, lo hi, mid mid; the dropped ones are below 2^-24), summed in fp32 in the
// instruction's accumulator.  The weights are cut once per workgroup into LDS, in the operand layout of the
// instruction (48 KB, one 16-byte read per lane and operand); the tile is cut when it is parked.
// With two pieces instead of three (template argument P; a knob of the library, off by default) a product keeps
// hi hi, hi mid and mid hi: what is dropped and what the two pieces do not represent stays below 3 x 2^-18 of
// |x| |w| per product, a bar twice as wide as fp32's for half the matrix instructions.
//
// The layer's gradient with respect to its input runs through the same kernel (template argument SD).  With
// dZ the gradient at the layer's pre-activation output, dX = A_hat^T (dZ Wn^T) + dZ Ws^T = (A_hat^T dZ) Wn^T + dZ Ws^T,
// and for a symmetric adjacency with mean weights A_hat^T = A D^-1: the aggregation is the plain (unit-weight)
// sum of the rows of dZ / deg, which the caller hands over, and the row's own part is that row times its length
// again.  So SD is the layer with unit weights whose own-row operand is scaled by the row's stored length.
//
// High-degree rows are aggregated beforehand by the HD kernel into a side buffer of the plan, one row per
// high-degree row in ascending order of their ids; a tile that contains one (or a row with more than kSpD entries,
// or the ragged end) is redone by a plain path that picks those sums up (the row's place in the buffer by binary
// search in the list of high-degree rows).
#include <type_traits>

#include "groot_device.h"

namespace groot {

constexpr int kSpRows = 16;                  // rows per tile: the height of a matrix instruction
static_assert(kSpRows * 64 <= kTrashFloats, "rows past the end of the matrix are stored to the trash area");

// Shapes for FI input and FO output features and NW wavefronts per workgroup (one workgroup per CU).
template <int FI, int FO, int NW>
struct SpCfg {
    static constexpr int kWaves = NW;
    static constexpr int kL = FI / 4;                // lanes per input row, one float4 each
    static constexpr int kRpg = kWave / kL;          // input rows per lane-group sweep
    static constexpr int kG = kSpRows / kRpg;        // sweeps per tile
    static constexpr int kRowShift = FI == 64 ? 8 : 7;   // log2 of an input row's bytes
    static constexpr int kK = 2 * FI;                // contraction length: [agg | self]
    static constexpr int kKs = kK / 32;              // k blocks of a matrix instruction
    static constexpr int kNb = FO / 16;              // blocks of 16 output columns
    static constexpr int kBRow = kK * 2 + 16;        // bytes per LDS row of one bf16 plane (16 B of padding: conflict-free)
    static constexpr int kPlane = kSpRows * kBRow;
    static constexpr int kOStride = FO + 4;          // floats per LDS row of the result tile
    static constexpr int kLo = FO / 4;               // lanes per output row
    static constexpr int kRo = kWave / kLo;          // output rows per store instruction
    static constexpr int kGo = kSpRows / kRo;        // store sweeps per tile
    static constexpr int kORowShift = FO == 64 ? 8 : FO == 32 ? 7 : 6;   // log2 of an output row's bytes
    static_assert(FI == 64 || FI == 32, "input width");
    static_assert(FO == 64 || FO == 32 || FO == 16, "output width");
    static_assert(kSpRows * kOStride * 4 <= 2 * kPlane, "the result tile fits the parked tile's space (two planes at least)");
};

typedef __bf16 sp_bf2 __attribute__((ext_vector_type(2)));
typedef __bf16 sp_bf8 __attribute__((ext_vector_type(8)));
typedef unsigned int sp_u4 __attribute__((ext_vector_type(4)));
typedef unsigned int sp_u2 __attribute__((ext_vector_type(2)));
typedef float sp_f2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void sp_wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// two fp32 values -> their bf16 roundings (nearest even), packed: a in the low half
__device__ __forceinline__ unsigned sp_pack2(float a, float b)
{
    const sp_f2 x = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(x, sp_bf2));
}

// (a, b) = hi + mid + lo, three packed bf16 pairs; the remainders are exact in fp32
__device__ __forceinline__ void sp_split3(float a, float b, unsigned &hi, unsigned &mid, unsigned &lo)
{
    hi = sp_pack2(a, b);
    float ra = a - __builtin_bit_cast(float, hi << 16), rb = b - __builtin_bit_cast(float, hi & 0xffff0000u);
    mid = sp_pack2(ra, rb);
    ra -= __builtin_bit_cast(float, mid << 16);
    rb -= __builtin_bit_cast(float, mid & 0xffff0000u);
    lo = sp_pack2(ra, rb);
}

// four consecutive elements k..k+3 of tile row `row` into the P planes (row stride kBRow, plane size kPlane)
template <int kBRow, int kPlane, int P>
__device__ __forceinline__ void sp_park(char *tile, int row, int k, v4f x)
{
    unsigned h0, m0, l0, h1, m1, l1;
    sp_split3(x[0], x[1], h0, m0, l0);                   // P = 2: the third piece is never used and is not computed
    sp_split3(x[2], x[3], h1, m1, l1);
    char *p = tile + row * kBRow + k * 2;
    *(sp_u2 *)p = (sp_u2){h0, h1};
    *(sp_u2 *)(p + kPlane) = (sp_u2){m0, m1};
    if constexpr (P == 3) *(sp_u2 *)(p + 2 * kPlane) = (sp_u2){l0, l1};
}

// W: kOnes or kMean; D: gather slots per row on the pipelined path; P: bf16 pieces per fp32 operand, 3 or 2
template <int W, int FI, int FO, int NW, int D, int P, bool SD = false>
__global__ __launch_bounds__(NW * kWave) __attribute__((amdgpu_waves_per_eu(NW / 4, NW / 4))) void sage_pipe_kernel(
    const int64_t *__restrict__ rowptr, const int32_t *__restrict__ col, const float *__restrict__ val,
    const char *__restrict__ X, char *H, int64_t zero_off, char *trash,
    const float *__restrict__ Wn, const float *__restrict__ Ws, const float *__restrict__ bias, int relu, int64_t n,
    int32_t T, int64_t n_tiles, int64_t tiles_per_part, int64_t waves_per_part, int32_t parts,
    const int32_t *__restrict__ hd_rows, int32_t n_hd, const char *__restrict__ hd_agg)
{
    static_assert(P == 3 || P == 2, "pieces per operand");
    static_assert(!SD || W == kOnes, "the own-row operand is scaled by the row length in the unit-weight form only");
    using C = SpCfg<FI, FO, NW>;
    constexpr int F = FI;
    constexpr int kSpD = D, kSpSlots = kSpRows * kSpD, kSpH = (kSpSlots + kWave - 1) / kWave;
    constexpr int kSpWaves = C::kWaves, kSpL = C::kL, kSpRpg = C::kRpg, kSpG = C::kG, kRowShift = C::kRowShift;
    constexpr int kKs = C::kKs, kNb = C::kNb, kSpBRow = C::kBRow, kSpPlane = C::kPlane, kSpOStride = C::kOStride;
    struct SlotW { int64_t off; float w; float pad; };
    using Slot = typename std::conditional<W == kExplicit, SlotW, int64_t>::type;
    __shared__ __align__(16) Slot s_slot[kSpWaves][kSpSlots];
    __shared__ float s_inv[kSpWaves][kSpRows];
    __shared__ __align__(16) char s_A[kSpWaves][P * kSpPlane];           // F = 64, P = 3: 13,056 B per wavefront; the result tile reuses it
    __shared__ __align__(16) sp_u4 s_W[kNb][kKs][P][kWave];              // F = 64, P = 3: 49,152 B: [nb][ks][piece][lane] B operands
    __shared__ float s_bias[FO];

    const int w = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int g = l / kSpL, f = l % kSpL;
    const int kq = l / 16, jl = l % 16;                  // matrix instruction: k block / row (A), column (B, D)
    const int64_t part = blockIdx.x % parts, j = (blockIdx.x / parts) * kSpWaves + w;
    const int64_t x_begin = part * tiles_per_part;
    const int64_t x_end = x_begin + tiles_per_part < n_tiles ? x_begin + tiles_per_part : n_tiles;
    const int64_t t_first = x_begin + j, stride = waves_per_part;
    const char *Xf = X + 16 * f;

    // ---- the weights, cut once per workgroup: s_W[nb][ks][piece][lane] is the B operand of output columns
    //      16 nb .. 16 nb + 15 for k = 32 ks + 8 kq + e, e = 0..7.  The wavefronts share the (nb, ks) pairs.
    //      Every wavefront reaches this barrier (none has left yet, nothing is in flight).
    {
        for (int c = w; c < kNb * kKs; c += kSpWaves) {
            const int nb = c / kKs, ks = c % kKs, jcol = 16 * nb + jl;
            sp_u4 pc[3];
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const int k = 32 * ks + 8 * kq + e;
                const float w0 = k < F ? Wn[k * FO + jcol] : Ws[(k - F) * FO + jcol];
                const float w1 = k + 1 < F ? Wn[(k + 1) * FO + jcol] : Ws[(k + 1 - F) * FO + jcol];
                unsigned h, m, lo_;
                sp_split3(w0, w1, h, m, lo_);
                pc[0][e / 2] = h;
                pc[1][e / 2] = m;
                pc[2][e / 2] = lo_;
            }
#pragma unroll
            for (int q = 0; q < P; ++q) s_W[nb][ks][q][l] = pc[q];
        }
    }
    if (threadIdx.x < FO) s_bias[threadIdx.x] = bias ? bias[threadIdx.x] : 0.0f;
    __syncthreads();
    if (t_first >= x_end) return;

    // ---- CSR pipeline: rp_a and cc/vv belong to the next tile to be staged, rp_b to the one after
    int64_t rp_a = 0, rp_b = 0;
    int32_t cc[kSpH];
    float vv[kSpH];
#pragma unroll
    for (int h = 0; h < kSpH; ++h) { cc[h] = 0; vv[h] = 0.f; }
    bool fix_a = true;                                   // the tile has rows that the slots do not serve (or is ragged)
    int32_t len_a = 0;                                   // lanes 0..kSpRows-1: stored length of the tile's row
    uint32_t live_a = 0;                                 // bit h: slot l + 64 h holds an entry
    auto load_rp = [&](int64_t tile) -> int64_t {
        const int64_t ri = tile * kSpRows + (l < kSpRows ? l : kSpRows);
        return rowptr[ri < n ? ri : n];                  // lanes 0..kSpRows hold the pointers; rows past the end read rowptr[n]
    };
    auto load_cols = [&](int64_t tile) {                 // from rp_a: every slot fetches its own entry
        const bool full = (tile + 1) * kSpRows <= n && tile < x_end;
        const int64_t begin = __shfl(rp_a, 0);
        const int32_t rel = full ? (int32_t)(rp_a - begin) : 0;
        len_a = __shfl_down(rel, 1) - rel;
        // a row with more entries than slots, or a high-degree row, has no live slot: the tile is completed by the
        // plain path below, row by row
        fix_a = !full || __ballot(l < kSpRows && (len_a > kSpD || len_a >= T)) != 0;
        live_a = 0;
        // unconditional loads (a dead slot reads entry 0): the number of loads in flight stays known
#pragma unroll
        for (int h = 0; h < kSpH; ++h) {
            const int s = l + kWave * h;                 // slot s: row r, entry k
            const int r = s / kSpD, k = s - r * kSpD;
            const int32_t lo = __shfl(rel, r), len = __shfl(rel, r + 1) - lo;
            const bool live = s < kSpSlots && k < len && len <= kSpD && len < T;
            live_a |= (uint32_t)live << h;
            const int64_t i = live ? begin + lo + k : 0;
            cc[h] = __builtin_nontemporal_load(&col[i]);
            if (W == kExplicit) vv[h] = __builtin_nontemporal_load(&val[i]);
        }
    };
    auto stage = [&]() -> bool {                         // cc, vv, live_a, len_a -> slot table and row weights; -> fix_a
#pragma unroll
        for (int h = 0; h < kSpH; ++h) {
            const int s = l + kWave * h;
            const bool live = (live_a >> h) & 1;
            if (s < kSpSlots) {
                const int64_t off = live ? ((int64_t)cc[h] << kRowShift) : zero_off;
                if constexpr (W == kExplicit) s_slot[w][s] = SlotW{off, live ? vv[h] : 0.f, 0.f};
                else s_slot[w][s] = off;
            }
        }
        if (W == kMean && l < kSpRows) s_inv[w][l] = row_weight<kMean>(len_a);
        if (SD && l < kSpRows) s_inv[w][l] = (float)len_a;   // exact: a row that the slots serve has few entries, and
                                                             // a longer one has fewer than 2^24 (the plain path redoes ragged tiles)
        sp_wave_sync();
        return fix_a;
    };

    // ---- one group: kSpRpg rows, one per lane group: the row's own features and its kSpD slots
    struct Regs {
        v4f xs[kSpD], self;
        float ws[W == kExplicit ? kSpD : 1];
        float inv;
    };
    Regs rr[kSpG];
    auto issue = [&](Regs &q, int64_t tile, int grp) {
        const int lr = grp * kSpRpg + g;
        int64_t row = tile * kSpRows + lr;
        row = row < n ? row : n - 1;                     // past the end: any valid row, the result is not kept
        if (W == kMean || SD) q.inv = s_inv[w][lr];
#pragma unroll
        for (int k = 0; k < kSpD; ++k) {
            if constexpr (W == kExplicit) {
                const SlotW sl = s_slot[w][lr * kSpD + k];
                q.xs[k] = *(const v4f *)(Xf + sl.off);
                q.ws[k] = sl.w;
            } else {
                q.xs[k] = *(const v4f *)(Xf + s_slot[w][lr * kSpD + k]);
            }
        }
        q.self = *(const v4f *)(Xf + (row << kRowShift));
    };
    auto sum = [&](const Regs &q) -> v4f {
        v4f a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < kSpD; ++k) {
            if (W == kExplicit) a += q.ws[k] * q.xs[k];
            else a += q.xs[k];
        }
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
    for (int grp = 0; grp < kSpG; ++grp) issue(rr[grp], t_first, grp);
    __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): the loop's own order of loads is the only one from here on

    char *const a_tile = s_A[w];
    float *const o_tile = (float *)s_A[w];               // after the products the parked tile is dead
    for (int64_t tile = t_first; tile < x_end; tile += stride) {
        const bool fix_next = stage();                   // CSR of the next tile -> slot table (this tile's groups are all issued)
        rp_a = rp_b;
        load_cols(tile + 2 * stride);
        rp_b = load_rp(tile + 3 * stride);
        const int64_t base = tile * kSpRows;
        // sums of this tile -> LDS, cut into bf16 pieces; the same register set takes the rows of the next tile
#pragma unroll
        for (int grp = 0; grp < kSpG; ++grp) {
            const v4f a = sum(rr[grp]);
            sp_park<kSpBRow, kSpPlane, P>(a_tile, grp * kSpRpg + g, 4 * f, a);
            sp_park<kSpBRow, kSpPlane, P>(a_tile, grp * kSpRpg + g, F + 4 * f, SD ? rr[grp].self * rr[grp].inv : rr[grp].self);
            issue(rr[grp], tile + stride, grp);
        }
        if (fix_cur) {
            // plain path: the rows of this tile that had no live slots (more entries than slots, high-degree, or
            // every row of the ragged last tile), straight from global memory; high-degree sums from the side buffer
#pragma unroll 1
            for (int grp = 0; grp < kSpG; ++grp) {
                const int64_t row = base + grp * kSpRpg + g;
                const bool full = base + kSpRows <= n;
                v4f a = {0.f, 0.f, 0.f, 0.f};
                bool redo = false;
                if (row < n) {
                    const int64_t s = rowptr[row], e = rowptr[row + 1];
                    redo = !full || e - s > kSpD || e - s >= T;
                    if (e - s >= T) {
                        int32_t lo = 0, hi = n_hd;       // the row's place in the list of high-degree rows
                        while (lo < hi) {
                            const int32_t mid = (lo + hi) / 2;
                            if (hd_rows[mid] < row) lo = mid + 1; else hi = mid;
                        }
                        a = *(const v4f *)(hd_agg + ((int64_t)lo << kRowShift) + 16 * f);
                    } else if (redo) {
                        a = ld_row_sum<W, false, 8>(s, e, col, val, (const v4f *)X, kSpL, f);
                    }
                }
                if (redo) sp_park<kSpBRow, kSpPlane, P>(a_tile, grp * kSpRpg + g, 4 * f, a);
                if (SD && !full && row < n) {            // a ragged tile carries no row lengths: the own-row operand again
                    const v4f own = *(const v4f *)(Xf + (row << kRowShift));
                    sp_park<kSpBRow, kSpPlane, P>(a_tile, grp * kSpRpg + g, F + 4 * f,
                                                  own * (float)(rowptr[row + 1] - rowptr[row]));
                }
            }
        }
        sp_wave_sync();
        // ---- [agg | self] (16 x 2F) times [Wn; Ws] (2F x F): lane (jl, kq) reads row jl, k = 32 ks + 8 kq + 0..7
        v4f acc[kNb];
#pragma unroll
        for (int nb = 0; nb < kNb; ++nb) {
            const float bv = s_bias[16 * nb + jl];
            acc[nb] = (v4f){bv, bv, bv, bv};
        }
        const char *a_lane = a_tile + jl * kSpBRow + 16 * kq;
        // P kKs steps (ks, weight piece pb = hi, mid, lo), each against the tile pieces whose product is kept
        // (P = 3: hi with lo, mid, hi; mid with mid, hi; lo with hi.  P = 2: hi with mid, hi; mid with hi), on kNb
        // independent accumulators.  The weight operands of step s + 1 are read from LDS while step s runs; a tile
        // piece of the next ks is read as soon as its register is dead (the last piece after the first step, the one
        // before it after the second, hi after the last step, where the first matrix instructions of the next ks do
        // not need it yet).
        sp_u4 aop[P], bop[2][kNb];
        auto read_a = [&](int ks, int pc) { aop[pc] = *(const sp_u4 *)(a_lane + pc * kSpPlane + 64 * ks); };
        auto read_b = [&](int s_) {
            const int ks = s_ / P, pb = s_ % P;
#pragma unroll
            for (int nb = 0; nb < kNb; ++nb) bop[s_ & 1][nb] = s_W[nb][ks][pb][l];
        };
#pragma unroll
        for (int pc = P - 1; pc >= 0; --pc) read_a(0, pc);
        read_b(0);
#pragma unroll
        for (int s_ = 0; s_ < P * kKs; ++s_) {
            const int ks = s_ / P, pb = s_ % P;
            if (s_ + 1 < P * kKs) read_b(s_ + 1);
            if (ks + 1 < kKs && pb >= 1) read_a(ks + 1, P - pb);     // piece P - pb was last used in the step before this one
            __builtin_amdgcn_sched_barrier(0);                       // the reads stay ahead of this step's matrix instructions
#pragma unroll
            for (int pa = P - 1 - pb; pa >= 0; --pa)
#pragma unroll
                for (int nb = 0; nb < kNb; ++nb)
                    acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(sp_bf8, aop[pa]),
                                                                      __builtin_bit_cast(sp_bf8, bop[s_ & 1][nb]),
                                                                      acc[nb], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (ks + 1 < kKs && pb == P - 1) read_a(ks + 1, 0);      // hi after the last step
        }
        sp_wave_sync();                                  // all reads of the parked tile are done: its space takes the result
        // ---- result: lane holds rows 4 kq + r of column 16 nb + jl; through LDS to whole rows per lane group
#pragma unroll
        for (int nb = 0; nb < kNb; ++nb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float v = acc[nb][r];
                if (relu) v = v > 0.0f ? v : 0.0f;
                o_tile[(4 * kq + r) * kSpOStride + 16 * nb + jl] = v;
            }
        sp_wave_sync();
#pragma unroll
        for (int go = 0; go < C::kGo; ++go) {
            const int lr = go * C::kRo + l / C::kLo, fo = l % C::kLo;
            const int64_t row = base + lr;
            const v4f v = *(const v4f *)&o_tile[lr * kSpOStride + 4 * fo];
            char *dst = row < n ? H + (row << C::kORowShift) : trash + (lr << C::kORowShift);
            __builtin_nontemporal_store(v, (v4f *)(dst + 16 * fo));
        }
        sp_wave_sync();                                  // the tiles in LDS are free for the next round
        fix_cur = fix_next;
    }
}

// out[i, :] = Z[i, :] / (stored length of row i), one lane per float4; out may be Z
__global__ __launch_bounds__(kBlock) void rows_over_degree_kernel(const int64_t *__restrict__ rowptr, const v4f *Z, v4f *out,
                                                                  int64_t n, int32_t F4)
{
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n * F4) return;
    const int64_t row = i / F4;
    const float d = (float)(rowptr[row + 1] - rowptr[row]);
    const v4f z = Z[i];
    out[i] = d > 0.f ? (v4f){z[0] / d, z[1] / d, z[2] / d, z[3] / d} : (v4f){0.f, 0.f, 0.f, 0.f};
}

int launch_rows_over_degree(const DevicePlan &dp, const float *Z, float *out, int32_t F, void *stream)
{
    const int64_t total = dp.n * (int64_t)(F / 4), grid = (total + kBlock - 1) / kBlock;
    if (total == 0) return 0;
    if (!grid_ok(grid)) return (int)hipErrorInvalidConfiguration;
    rows_over_degree_kernel<<<dim3((unsigned)grid), dim3(kBlock), 0, (hipStream_t)stream>>>(dp.rowptr, (const v4f *)Z, (v4f *)out,
                                                                                          dp.n, F / 4);
    return (int)hipGetLastError();
}

int launch_sage_pipe(const DevicePlan &dp, const float *X, float *H, const float *Wn, const float *Ws, const float *bias,
                     int relu, int32_t FI, int32_t FO, int pieces, int self_times_degree, void *stream)
{
    if (!weights_ok(dp) || !dp.zero_row || (FI != 64 && FI != 32) || (FO != 64 && FO != 32 && FO != 16) ||
        (pieces != 2 && pieces != 3))
        return (int)hipErrorInvalidValue;
    // row-uniform weights only: with explicit weights the slot table is twice as large and LDS does not hold it
    if (dp.weight_mode == kExplicit) return (int)hipErrorInvalidValue;
    const int wm = self_times_degree ? (int)kOnes : dp.weight_mode;
    if (dp.n_hd_rows && (!dp.hd_rows || !dp.hd_agg)) return (int)hipErrorInvalidValue;
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return (int)e;
    // wavefronts per workgroup: two per SIMD (at F = 32 three fit and are slower: 11.4 against 10.2 ms)
    constexpr int kNwRun = 8;
    const int64_t n_tiles = (dp.n + kSpRows - 1) / kSpRows;
    // one workgroup per CU; consecutive workgroup ids land on different XCDs
    int64_t n_wg = cus / kXcds * kXcds;
    if (n_wg < kXcds) n_wg = kXcds;
    const int32_t parts = dp.xcd_remap ? kXcds : 1;
    const int64_t tiles_per_part = (n_tiles + parts - 1) / parts;
    const int64_t waves_per_part = n_wg / parts * kNwRun;
    if (!grid_ok(n_wg) || n_tiles <= 0) return (int)hipErrorInvalidConfiguration;
    // the kernel reads entry 0 of the index (and weight) array from idle lanes: give it something to read
    // when the matrix has no entries, or no weight array
    const int32_t *col_arg = dp.col ? dp.col : (const int32_t *)dp.rowptr;
    const float *val_arg = dp.val ? dp.val : (const float *)dp.rowptr;
    char *trash = (char *)(dp.zero_row + kZeroRowFloats);
    hipStream_t st = (hipStream_t)stream;
#define GROOT_SAGE_PIPE_LAUNCH(WM, FFI, FFO, DD, PP)                                                                   \
    sage_pipe_kernel<WM, FFI, FFO, kNwRun, DD, PP, SDV><<<dim3((unsigned)n_wg), dim3(kNwRun * kWave), 0, st>>>(        \
        dp.rowptr, col_arg, val_arg, (const char *)X, (char *)H, byte_distance(X, dp.zero_row), trash, Wn, Ws, bias, relu, \
        dp.n, dp.threshold, n_tiles, tiles_per_part, waves_per_part, parts, dp.hd_rows, (int32_t)dp.n_hd_rows,         \
        (const char *)dp.hd_agg)
#define GROOT_SAGE_PIPE_P(WM, FFI, FFO, DD)                               \
    if (pieces == 2) GROOT_SAGE_PIPE_LAUNCH(WM, FFI, FFO, DD, 2);         \
    else GROOT_SAGE_PIPE_LAUNCH(WM, FFI, FFO, DD, 3)
#define GROOT_SAGE_PIPE_D(WM, FFI, FFO)                                   \
    if (dp.sage_depth == 5) { GROOT_SAGE_PIPE_P(WM, FFI, FFO, 5); }       \
    else { GROOT_SAGE_PIPE_P(WM, FFI, FFO, 6); }
#define GROOT_SAGE_PIPE_FO(WM, FFI)                            \
    if (FO == 64) { GROOT_SAGE_PIPE_D(WM, FFI, 64); }          \
    else if (FO == 32) { GROOT_SAGE_PIPE_D(WM, FFI, 32); }     \
    else { GROOT_SAGE_PIPE_D(WM, FFI, 16); }
    if (self_times_degree) {
        constexpr bool SDV = true;
        if (FI == 64) { GROOT_SAGE_PIPE_FO(kOnes, 64); }
        else { GROOT_SAGE_PIPE_FO(kOnes, 32); }
    } else {
        constexpr bool SDV = false;
        if (FI == 64) {
            if (wm == kMean) { GROOT_SAGE_PIPE_FO(kMean, 64); }
            else { GROOT_SAGE_PIPE_FO(kOnes, 64); }
        } else {
            if (wm == kMean) { GROOT_SAGE_PIPE_FO(kMean, 32); }
            else { GROOT_SAGE_PIPE_FO(kOnes, 32); }
        }
    }
#undef GROOT_SAGE_PIPE_D
#undef GROOT_SAGE_PIPE_P
#undef GROOT_SAGE_PIPE_FO
#undef GROOT_SAGE_PIPE_LAUNCH
    return (int)hipGetLastError();
}

}  // namespace groot
