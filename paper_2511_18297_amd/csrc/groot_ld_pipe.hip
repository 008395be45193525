// Software-pipelined LD kernel for gfx950: the low-degree rows of graphs whose rows are short (an AIG
// with self-loops has 2 to 6 entries per low-degree row), F = 32, 64 or 128.
//
// One persistent workgroup of four wavefronts per CU, i.e. one wavefront per SIMD.  Every wavefront walks
// its own tiles of G lane groups x (64 / L) rows (L = F / 4 lanes per row) and keeps a whole tile in
// flight: G register sets of D gathered float4 each (D = 5 to 8 slots per row, chosen per plan).  Right
// after the rows of a group of tile t have been summed and stored, the same register set is loaded with
// the group's rows of tile t+1, so the wavefront never waits with nothing in flight.  Compared with the
// plain LD kernel (32 wavefronts per CU, four rows in flight each, all of them drained at every tile) this
// keeps fewer requests in flight per CU (measured to be what the memory system of this chip prefers for
// this access pattern) and never lets the stream of requests stop.
//
// What makes the pipeline work (each item was a measured dead end without it):
//  * All address arithmetic is done once per tile, lane-parallel: lane s owns slot s = D r + k of a
//    wavefront-private table in LDS (byte offset of the k-th neighbour of row r); it fetches that entry's
//    column index itself, two tiles ahead, from the row pointers that arrived three tiles ahead (register
//    shuffles hand every slot its row's extent).  A slot past a row's end points at a row of zeros outside
//    X: the sum of a row is the plain sum of its D slots, in CSR order.
//  * The steady state has no branch and no conditional load or store, so the compiler's vmcnt waits are
//    exact: the wait before a group's sum leaves the G-1 younger groups in flight.  A row that does not
//    fit (more than D entries, or a high-degree row) is masked: all its slots point at the zero row and
//    its sum is stored to a trash area instead of Y (an address select, not a branch); the high-degree
//    kernel, or the row-list kernel below for low-degree rows longer than D, computes it.  Only the ragged
//    last tile is masked as a whole and redone by a plain, unoverlapped path.
//  * No workgroup barrier after the start (the list of hot rows is copied to LDS once): wavefronts share
//    nothing else.
#include <type_traits>

#include "groot_device.h"

namespace groot {

constexpr int kPipeWaves = 4;                // wavefronts per workgroup, one workgroup per CU
// lane-group sweeps (register sets) in flight per wavefront, by lanes per row.  Measured on the headline graph:
// 16 lanes (F = 64), LD kernels with X and Y where they run fastest: 13.08 / 12.75 / 12.94 / 12.63 / 12.75 ms for
// 4 / 5 / 6 / 7 / 8 (with both matrices in one class of address ranges 5 was the best: 16.9 / 14.4 / 14.2 / 13.7 /
// 14.0 / 13.8 / 13.9 ms for 2..8); 8 lanes (F = 32): 6.46 / 6.36 ms for 5 / 7; 32 lanes (F = 128): 31.0 / 30.5 /
// 31.3 ms per step for 5 / 7 / 8
constexpr int pipe_groups(int) { return 7; }

__device__ __forceinline__ void pipe_wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The compact form of the CSR (C = true: 4-byte row pointers, 2-byte column codes, the list of high-degree
// rows that a code can name; see groot_compress.hip) replaces the loads of the pipeline; the plain path and the
// row-list kernel keep reading the full arrays.
struct CompactCsr {
    const uint32_t *rp32;
    const uint16_t *col16;
    const int32_t *hot;
    int32_t n_hot;
};

// M: the sum of row r goes to row out_ids[r] of Y (the owned rows of a part written into place in the matrix of
// the whole graph); n is then the number of leading rows that are wanted.  Only without the compact matrix.
template <int L, int W, int G, int D, bool C, bool M = false>
__global__ __launch_bounds__(kPipeWaves * kWave) __attribute__((amdgpu_waves_per_eu(1, 2))) void ld_pipe_kernel(
    const int64_t *__restrict__ rowptr, const int32_t *__restrict__ col, const float *__restrict__ val,
    const CompactCsr cz, const char *__restrict__ X, char *__restrict__ Y, int64_t zero_off, char *trash, int64_t n,
    int32_t T, int64_t n_tiles, int64_t tiles_per_part, int64_t waves_per_part, int32_t parts,
    const int64_t *__restrict__ out_ids)
{
    static_assert(!(C && M), "the row-mapped form reads the plain arrays");
    constexpr int kRpg = kWave / L;                      // rows per lane group sweep
    constexpr int kTileRows = G * kRpg;
    constexpr int kPipeD = D;                            // slots per row
    constexpr int kSlots = kTileRows * kPipeD, kH = (kSlots + kWave - 1) / kWave;
    constexpr int kRowShift = L == 8 ? 7 : L == 16 ? 8 : 9;   // log2 of a feature row's bytes
    static_assert(L == 8 || L == 16 || L == 32, "one float4 per lane");
    static_assert(kTileRows + 1 <= kWave, "row pointers of a tile fit one wavefront");
    // a slot: byte offset of the gathered row from X; with explicit weights the entry's weight rides in the
    // same 16-byte slot, so that one LDS read per slot serves both
    struct SlotW { int64_t off; float w; float pad; };
    using Slot = typename std::conditional<W == kExplicit, SlotW, int64_t>::type;
    __shared__ __align__(16) Slot s_slot[kPipeWaves][kSlots];
    __shared__ float s_inv[kPipeWaves][kTileRows];       // row weight (1 unless W == kMean), or -1: the row is masked
    __shared__ int64_t s_oid[M ? kPipeWaves : 1][M ? kTileRows : 1];   // M: byte offset of the row's place in Y

    const int w = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int g = l / L, f = l % L;
    // Part x (an XCD) owns tiles [x TP, (x+1) TP); its wavefronts take them round-robin, so that the
    // part sweeps a narrow window of rows at any time.
    const int64_t part = blockIdx.x % parts, j = (blockIdx.x / parts) * kPipeWaves + w;
    const int64_t x_begin = part * tiles_per_part;
    const int64_t x_end = x_begin + tiles_per_part < n_tiles ? x_begin + tiles_per_part : n_tiles;
    const int64_t t_first = x_begin + j, stride = waves_per_part;
    extern __shared__ int32_t s_hot[];                   // C: the hot list (at least one element)
    if constexpr (C) {
        for (int i = threadIdx.x; i < cz.n_hot; i += kPipeWaves * kWave) s_hot[i] = cz.hot[i];
        if (threadIdx.x == 0 && cz.n_hot == 0) s_hot[0] = 0;
        __syncthreads();                                 // every wavefront gets here: none has left, nothing is in flight
    }
    if (t_first >= x_end) return;
    const char *Xf = X + 16 * f;

    // ---- CSR pipeline: rp_a and cc/vv belong to the next tile to be staged, rp_b to the one after
    int64_t rp_a = 0, rp_b = 0;
    int32_t cc[kH];
    float vv[kH];
#pragma unroll
    for (int h = 0; h < kH; ++h) { cc[h] = 0; vv[h] = 0.f; }
    bool ok_a = false;
    int32_t len_a = 0;                                   // lanes 0..kTileRows-1: stored length of the tile's row
    uint32_t live_a = 0;                                 // bit h: slot l + 64 h holds an entry
    int32_t base_a = 0;                                  // C: first row of the tile that cc belongs to
    int64_t oid_a = 0, oid_b = 0;                        // M: out_ids of the rows that rp_a / rp_b belong to
    auto load_oid = [&](int64_t tile) -> int64_t {
        if constexpr (!M) return 0;
        const int64_t ri = tile * kTileRows + (l < kTileRows ? l : 0);
        return out_ids[ri < n ? ri : 0];                 // rows past the end: any valid entry, never used
    };
    auto load_rp = [&](int64_t tile) -> int64_t {
        const int64_t ri = tile * kTileRows + (l < kTileRows ? l : kTileRows);
        // lanes 0..kTileRows hold the pointers; rows past the end read rowptr[n]
        if constexpr (C) return (int64_t)cz.rp32[ri < n ? ri : n];       // all of them below 2^32
        else return rowptr[ri < n ? ri : n];
    };
    auto load_cols = [&](int64_t tile) {                 // from rp_a: every slot fetches its own entry
        // a tile takes part in the pipeline when all its rows exist; a row that does not fit its slots (too long,
        // or high-degree) has no live slot, whatever its length: it does not disturb the rows around it
        ok_a = (tile + 1) * kTileRows <= n && tile < x_end;
        base_a = ok_a ? (int32_t)(tile * kTileRows) : 0;
        const int64_t begin = __shfl(rp_a, 0);
        const int32_t rel = ok_a ? (int32_t)(rp_a - begin) : 0;
        len_a = __shfl_down(rel, 1) - rel;
        live_a = 0;
        // unconditional loads (a dead slot reads entry 0): the number of loads in flight stays known
#pragma unroll
        for (int h = 0; h < kH; ++h) {
            const int s = l + kWave * h;                 // slot s: row r, entry k
            const int r = s / kPipeD, k = s - r * kPipeD;
            const int32_t lo = __shfl(rel, r), len = __shfl(rel, r + 1) - lo;
            const bool live = s < kSlots && k < len && len <= kPipeD && len < T;
            live_a |= (uint32_t)live << h;
            const int64_t i = live ? begin + lo + k : 0;
            // (plain loads, no streaming hint: the cache line a tile's entries end in is the one the next tile's
            // begin in, and that tile belongs to another wavefront of the same XCD, a moment later; 1.7 % of a step)
            if constexpr (C) cc[h] = cz.col16[i];
            else cc[h] = col[i];
            if (W == kExplicit) vv[h] = val[i];
        }
    };
    auto stage = [&]() -> bool {                         // cc, vv, live_a, len_a -> slot table and row weights
        uint64_t badm[kH];                               // C: slots whose entry no code expresses
#pragma unroll
        for (int h = 0; h < kH; ++h) {
            const int s = l + kWave * h;
            bool live = (live_a >> h) & 1;
            int32_t c = cc[h];
            if constexpr (C) {                           // code -> column: near the row, or one of the hot rows
                const bool bad = live && c == kCodeBad;
                badm[h] = __ballot(bad);
                live = live && !bad;
                const int32_t hot_c = s_hot[live && c >= kCodeHot ? c - kCodeHot : 0];
                c = c >= kCodeHot ? hot_c : base_a + s / kPipeD + c - kCodeNear;
            }
            if (s < kSlots) {
                const int64_t off = live ? ((int64_t)c << kRowShift) : zero_off;
                if constexpr (W == kExplicit) s_slot[w][s] = SlotW{off, live ? vv[h] : 0.f, 0.f};
                else s_slot[w][s] = off;
            }
        }
        bool row_ok = ok_a && len_a <= kPipeD && len_a < T;
        if constexpr (C) {                               // a row with a bad slot is masked as a whole: slots l D .. l D + D - 1
            const int sb = l * kPipeD, sh = sb & 63;
            uint64_t w0 = 0, w1 = 0;
#pragma unroll
            for (int q = 0; q < kH; ++q) {
                w0 = (sb >> 6) == q ? badm[q] : w0;
                w1 = (sb >> 6) + 1 == q ? badm[q] : w1;
            }
            const uint64_t bits = (w0 >> sh) | (sh ? w1 << (64 - sh) : 0);
            row_ok = row_ok && (bits & ((1u << kPipeD) - 1)) == 0;
        }
        if (l < kTileRows) s_inv[w][l] = row_ok ? row_weight<W == kMean ? kMean : kOnes>(len_a) : -1.0f;
        if constexpr (M) {
            if (l < kTileRows) s_oid[w][l] = oid_a << kRowShift;
        }
        pipe_wave_sync();
        return ok_a;
    };

    // ---- one group: kRpg rows, one per lane group
    struct Regs {
        v4f xs[kPipeD];
        float ws[W == kExplicit ? kPipeD : 1];
        float inv;
        int64_t oid;                                     // M: where the row's sum goes
    };
    Regs rr[G];
    auto issue = [&](Regs &q, int grp) {
        const int lr = grp * kRpg + g;
        q.inv = s_inv[w][lr];
        if constexpr (M) q.oid = s_oid[w][lr];
#pragma unroll
        for (int k = 0; k < kPipeD; ++k) {
            if constexpr (W == kExplicit) {
                const SlotW sl = s_slot[w][lr * kPipeD + k];
                q.xs[k] = *(const v4f *)(Xf + sl.off);
                q.ws[k] = sl.w;
            } else {
                q.xs[k] = *(const v4f *)(Xf + s_slot[w][lr * kPipeD + k]);
            }
        }
    };
    auto sum = [&](const Regs &q) -> v4f {
        v4f a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < kPipeD; ++k) {
            if (W == kExplicit) a += q.ws[k] * q.xs[k];
            else a += q.xs[k];
        }
        if (W == kMean) a *= q.inv;
        return a;
    };

    char *const tbase = trash + 16 * f;
    // ---- prologue: the first tile is staged and put in flight, the CSR of the next two is on its way
    rp_a = load_rp(t_first);
    oid_a = load_oid(t_first);
    load_cols(t_first);
    bool ok_cur = stage();
    rp_a = load_rp(t_first + stride);
    oid_a = load_oid(t_first + stride);
    load_cols(t_first + stride);
    rp_b = load_rp(t_first + 2 * stride);
    oid_b = load_oid(t_first + 2 * stride);
#pragma unroll
    for (int grp = 0; grp < G; ++grp) issue(rr[grp], grp);
    // Everything above has arrived before the loop starts: the loop's own order of loads is then the
    // only one the compiler has to account for at the loop head, and its waits stay exact.
    __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0)

    for (int64_t tile = t_first; tile < x_end; tile += stride) {
        const bool ok_next = stage();                    // CSR of the next tile -> slot table (this tile's groups are all issued)
        rp_a = rp_b;
        oid_a = oid_b;
        load_cols(tile + 2 * stride);
        rp_b = load_rp(tile + 3 * stride);
        oid_b = load_oid(tile + 3 * stride);
        const int64_t base = tile * kTileRows;
        char *const ybase = Y + (base << kRowShift) + 16 * f;
#pragma unroll
        for (int grp = 0; grp < G; ++grp) {
            const v4f a = sum(rr[grp]);
            const int roff = (grp * kRpg + g) << kRowShift;
            // a masked row (every row of a tile that is not ok) goes to the trash area: a select, no branch
            char *const yrow = M ? Y + rr[grp].oid + 16 * f : ybase + roff;
            char *const dst = rr[grp].inv >= 0.f ? yrow : tbase + roff;
            __builtin_nontemporal_store(a, (v4f *)dst);
            issue(rr[grp], grp);                         // the same rows of the next tile
        }
        if (!ok_cur) {
            // plain path: the rows of this tile that the pipeline serves elsewhere, straight from global memory
#pragma unroll 1
            for (int grp = 0; grp < G; ++grp) {
                const int64_t row = base + grp * kRpg + g;
                if (row < n) {
                    const int64_t s = rowptr[row], e = rowptr[row + 1];
                    if (e - s < T && e - s <= kPipeD)
                        __builtin_nontemporal_store(ld_row_sum<W, false>(s, e, col, val, (const v4f *)X, L, f),
                                                    (v4f *)(Y + ((M ? out_ids[row] : row) << kRowShift) + 16 * f));
                }
            }
        }
        ok_cur = ok_next;
    }
}

// Low-degree rows that are longer than the pipeline's slots, by list: one lane group per row.
template <int L, int W>
__global__ __launch_bounds__(kBlock) void ld_rows_kernel(const int32_t *__restrict__ rows, int64_t n_rows,
                                                         const int64_t *__restrict__ rowptr,
                                                         const int32_t *__restrict__ col, const float *__restrict__ val,
                                                         const v4f *__restrict__ X, v4f *__restrict__ Y, int32_t F4,
                                                         const int64_t *__restrict__ out_ids, int64_t n_out)
{
    constexpr int G = kBlock / L;
    const int64_t k = (int64_t)blockIdx.x * G + threadIdx.x / L;
    if (k >= n_rows) return;
    const int64_t row = rows[k];
    if (row >= n_out) return;                            // a row that is not wanted (row-mapped calls: boundary rows)
    const int64_t s = rowptr[row], e = rowptr[row + 1];
    const int64_t orow = out_ids ? out_ids[row] : row;
    for (int32_t ff = threadIdx.x % L; ff < F4; ff += L)
        __builtin_nontemporal_store(ld_row_sum<W, false>(s, e, col, val, X, F4, ff), &Y[orow * F4 + ff]);
}

struct PipeArgs {
    const int64_t *rowptr;
    const int32_t *col;
    const float *val;
    CompactCsr cz;
    bool compact;
    const char *X;
    char *Y;
    int64_t zero_off;                        // byte distance from X to the plan's row of zeros
    char *trash;
    int64_t n;
    int32_t T;
    int64_t n_tiles, tiles_per_part, waves_per_part;
    int32_t parts;
    int64_t n_wg;
    hipStream_t st;
    const int64_t *out_ids;                  // row-mapped form, else NULL
};

template <int L, int W, int G, int D>
static void pipe_launch(const PipeArgs &a)
{
    if (a.out_ids) {
        ld_pipe_kernel<L, W, G, D, false, true><<<dim3((unsigned)a.n_wg), dim3(kPipeWaves * kWave), 0, a.st>>>(
            a.rowptr, a.col, a.val, a.cz, a.X, a.Y, a.zero_off, a.trash, a.n, a.T, a.n_tiles, a.tiles_per_part,
            a.waves_per_part, a.parts, a.out_ids);
    } else if (a.compact) {
        const size_t lds = (size_t)(a.cz.n_hot ? a.cz.n_hot : 1) * sizeof(int32_t);
        ld_pipe_kernel<L, W, G, D, true><<<dim3((unsigned)a.n_wg), dim3(kPipeWaves * kWave), lds, a.st>>>(
            a.rowptr, a.col, a.val, a.cz, a.X, a.Y, a.zero_off, a.trash, a.n, a.T, a.n_tiles, a.tiles_per_part,
            a.waves_per_part, a.parts, nullptr);
    } else {
        ld_pipe_kernel<L, W, G, D, false><<<dim3((unsigned)a.n_wg), dim3(kPipeWaves * kWave), 0, a.st>>>(
            a.rowptr, a.col, a.val, a.cz, a.X, a.Y, a.zero_off, a.trash, a.n, a.T, a.n_tiles, a.tiles_per_part,
            a.waves_per_part, a.parts, nullptr);
    }
}

template <int W, int D>
static void pipe_dispatch_l(int32_t F4, const PipeArgs &a)
{
    if (F4 == 8) pipe_launch<8, W, pipe_groups(8), D>(a);
    else if (F4 == 16) pipe_launch<16, W, pipe_groups(16), D>(a);
    else pipe_launch<32, W, pipe_groups(32), D>(a);
}

template <int W>
static void pipe_dispatch_d(int depth, int32_t F4, const PipeArgs &a)
{
    switch (depth) {
    case 5: pipe_dispatch_l<W, 5>(F4, a); break;
    case 6: pipe_dispatch_l<W, 6>(F4, a); break;
    case 7: pipe_dispatch_l<W, 7>(F4, a); break;
    default: pipe_dispatch_l<W, 8>(F4, a); break;
    }
}

// The compact form keeps the hot list in dynamic LDS, up to 128 KB: the runtime wants to be told once per
// kernel that more than its default limit may be asked for.  Called when a plan gets its compact CSR (not at
// launch, which may be under stream capture).
template <int L, int W, int D>
static int pipe_allow_lds()
{
    return (int)hipFuncSetAttribute((const void *)&ld_pipe_kernel<L, W, pipe_groups(L), D, true>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kCodeMaxHot * (int)sizeof(int32_t));
}
template <int W, int D>
static int pipe_allow_lds_l()
{
    int err = pipe_allow_lds<8, W, D>();
    if (!err) err = pipe_allow_lds<16, W, D>();
    if (!err) err = pipe_allow_lds<32, W, D>();
    return err;
}
template <int W>
static int pipe_allow_lds_d()
{
    int err = pipe_allow_lds_l<W, 5>();
    if (!err) err = pipe_allow_lds_l<W, 6>();
    if (!err) err = pipe_allow_lds_l<W, 7>();
    if (!err) err = pipe_allow_lds_l<W, 8>();
    return err;
}
int pipe_compact_prepare()
{
    static std::atomic<int> state{-1};                   // -1 not tried, else the result
    int s = state.load();
    if (s >= 0) return s;
    int err = pipe_allow_lds_d<kOnes>();
    if (!err) err = pipe_allow_lds_d<kMean>();
    if (!err) err = pipe_allow_lds_d<kExplicit>();
    state.store(err);
    return err;
}

// out: the leading out->n_out rows only, row r written to row out->ids[r] of Y (ids NULL: to row r)
int launch_ld_pipelined(const DevicePlan &dp, const float *X, float *Y, int32_t F, void *stream, const RowOut *out)
{
    const int64_t n_rows = out ? out->n_out : dp.n;
    const int64_t *out_ids = out ? out->ids : nullptr;
    if (n_rows < 0 || n_rows > dp.n) return (int)hipErrorInvalidValue;
    if (n_rows == 0) return 0;
    const int32_t F4 = F / 4;
    if (F4 != 8 && F4 != 16 && F4 != 32) return (int)hipErrorInvalidValue;
    if (!weights_ok(dp) || !dp.zero_row) return (int)hipErrorInvalidValue;
    if (dp.pipe_depth < kPipeMinDepth || dp.pipe_depth > kPipeMaxDepth) return (int)hipErrorInvalidValue;
    if (dp.n_mid_rows && !dp.mid_rows) return (int)hipErrorInvalidValue;
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return (int)e;
    const int tile_rows = pipe_groups(F4) * (kWave / F4);
    const int64_t n_tiles = (n_rows + tile_rows - 1) / tile_rows;
    // one workgroup per CU; consecutive workgroup ids land on different XCDs
    int64_t n_wg = cus / kXcds * kXcds;
    if (n_wg < kXcds) n_wg = kXcds;
    const int32_t parts = dp.xcd_remap ? kXcds : 1;
    const int64_t tiles_per_part = (n_tiles + parts - 1) / parts;
    const int64_t waves_per_part = n_wg / parts * kPipeWaves;
    if (!grid_ok(n_wg) || n_tiles <= 0) return (int)hipErrorInvalidConfiguration;
    // the kernel reads entry 0 of the index (and weight) array from idle lanes: give it something to read
    // when the matrix has no entries, or no weight array
    const int32_t *col_arg = dp.col ? dp.col : (const int32_t *)dp.rowptr;
    const float *val_arg = dp.val ? dp.val : (const float *)dp.rowptr;
    char *trash = (char *)(dp.zero_row + kZeroRowFloats);
    static_assert(pipe_groups(8) <= 8 && pipe_groups(16) <= 8 && pipe_groups(32) <= 8 && 8 * kWave * 16 <= kTrashFloats * 4,
                  "a tile's masked sums fit the trash area");
    hipStream_t st = (hipStream_t)stream;
    // the compact matrix codes rows that the row list serves as uncoded, which only holds for whole-graph calls
    const bool compact = !out && dp.compressed && dp.rp32 && dp.col16 && dp.hot_cols;
    const PipeArgs a{dp.rowptr, col_arg, val_arg, CompactCsr{dp.rp32, dp.col16, dp.hot_cols, dp.n_hot}, compact,
                     (const char *)X, (char *)Y, byte_distance(X, dp.zero_row), trash, n_rows,
                     dp.threshold, n_tiles, tiles_per_part, waves_per_part, parts, n_wg, st, out_ids};
    GROOT_DISPATCH_W(dp.weight_mode, (pipe_dispatch_d<kW>(dp.pipe_depth, F4, a)));
    hipError_t err = hipGetLastError();
    // the low-degree rows with more entries than the pipeline has slots; the rows that the compact matrix cannot
    // code stand at the end of the list and are the pipeline's own whenever it reads the plain arrays
    const int64_t n_mid = compact ? dp.n_mid_rows : dp.n_mid_rows - dp.n_bad_rows;
    if (err != hipSuccess || n_mid <= 0) return (int)err;
    const int64_t grid = (n_mid + kBlock / F4 - 1) / (kBlock / F4);
    if (!grid_ok(grid)) return (int)hipErrorInvalidConfiguration;
    GROOT_DISPATCH_W(dp.weight_mode,
                     (F4 == 8 ? ld_rows_kernel<8, kW><<<dim3((unsigned)grid), dim3(kBlock), 0, st>>>(
                                    dp.mid_rows, n_mid, dp.rowptr, col_arg, val_arg, (const v4f *)X, (v4f *)Y, F4, out_ids, n_rows)
                      : F4 == 16 ? ld_rows_kernel<16, kW><<<dim3((unsigned)grid), dim3(kBlock), 0, st>>>(
                                       dp.mid_rows, n_mid, dp.rowptr, col_arg, val_arg, (const v4f *)X, (v4f *)Y, F4, out_ids, n_rows)
                                 : ld_rows_kernel<32, kW><<<dim3((unsigned)grid), dim3(kBlock), 0, st>>>(
                                       dp.mid_rows, n_mid, dp.rowptr, col_arg, val_arg, (const v4f *)X, (v4f *)Y, F4, out_ids, n_rows)));
    return (int)hipGetLastError();
}

}  // namespace groot
