// Software-pipelined LD kernel for gfx950: the low-degree rows of graphs whose rows are short (an AIG
// with self-loops has 2 to 6 entries per low-degree row), F = 32, 64 or 128.
//
// One persistent workgroup of four wavefronts per CU, i.e. one wavefront per SIMD.  Every wavefront walks
// its own tiles of G lane groups x (64 / L) rows (L = F / 4 lanes per row) and keeps a whole tile in
// flight: G register sets of kPipeD gathered float4 each.  Right after the rows of a group of tile t have
// been summed and stored, the same register set is loaded with the group's rows of tile t+1, so the
// wavefront never waits with nothing in flight.  Compared with the plain LD kernel (32 wavefronts per CU,
// four rows in flight each, all of them drained at every tile) this keeps fewer requests in flight per CU
// (measured to be what the memory system of this chip prefers for this access pattern) and never lets
// the stream of requests stop.
//
// What makes the pipeline work (each item was a measured dead end without it):
//  * All address arithmetic is done once per tile, lane-parallel: lane s prepares slot s = 6 r + k of a
//    wavefront-private table in LDS (byte offset of the k-th neighbour of row r) from register shuffles of
//    the CSR, which was loaded two tiles ahead (row pointers three).  A slot past a row's end points at a
//    row of zeros outside X: the sum of a row is the plain sum of its kPipeD slots, in CSR order.
//  * The steady state has no branch and no conditional load or store, so the compiler's vmcnt waits are
//    exact: the wait before a group's sum leaves the G-1 younger groups in flight.  The sums of a tile
//    that is not "simple" (a row with more than kPipeD entries, a high-degree row, the ragged last tile)
//    are stored to a trash area instead of Y, and the tile is then redone by a plain, unoverlapped path.
//  * No workgroup barrier anywhere: wavefronts share nothing.
#include <type_traits>

#include "groot_device.h"

namespace groot {

constexpr int kPipeD = 6;                    // slots per row
constexpr int kPipeWaves = 4;                // wavefronts per workgroup, one workgroup per CU

__device__ __forceinline__ void pipe_wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int L, int W, int G>
__global__ __launch_bounds__(kPipeWaves * kWave) __attribute__((amdgpu_waves_per_eu(1, 2))) void ld_pipe_kernel(
    const int64_t *__restrict__ rowptr, const int32_t *__restrict__ col, const float *__restrict__ val,
    const char *__restrict__ X, char *__restrict__ Y, int64_t zero_off, char *trash, int64_t n,
    int32_t T, int64_t n_tiles, int64_t tiles_per_part, int64_t waves_per_part, int32_t parts)
{
    constexpr int kRpg = kWave / L;                      // rows per lane group sweep
    constexpr int kTileRows = G * kRpg;
    constexpr int kSlots = kTileRows * kPipeD, kH = (kSlots + kWave - 1) / kWave;
    constexpr int kRowShift = L == 8 ? 7 : L == 16 ? 8 : 9;   // log2 of a feature row's bytes
    static_assert(L == 8 || L == 16 || L == 32, "one float4 per lane");
    static_assert(kTileRows + 1 <= kWave, "row pointers of a tile fit one wavefront");
    // a slot: byte offset of the gathered row from X; with explicit weights the entry's weight rides in the
    // same 16-byte slot, so that one LDS read per slot serves both
    struct SlotW { int64_t off; float w; float pad; };
    using Slot = typename std::conditional<W == kExplicit, SlotW, int64_t>::type;
    __shared__ __align__(16) Slot s_slot[kPipeWaves][kSlots];
    __shared__ float s_inv[kPipeWaves][kTileRows];

    const int w = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int g = l / L, f = l % L;
    // Part x (an XCD) owns tiles [x TP, (x+1) TP); its wavefronts take them round-robin, so that the
    // part sweeps a narrow window of rows at any time.
    const int64_t part = blockIdx.x % parts, j = (blockIdx.x / parts) * kPipeWaves + w;
    const int64_t x_begin = part * tiles_per_part;
    const int64_t x_end = x_begin + tiles_per_part < n_tiles ? x_begin + tiles_per_part : n_tiles;
    const int64_t t_first = x_begin + j, stride = waves_per_part;
    if (t_first >= x_end) return;
    const char *Xf = X + 16 * f;

    // ---- CSR pipeline: rp_a and cc/vv belong to the next tile to be staged, rp_b to the one after
    int64_t rp_a = 0, rp_b = 0;
    int32_t cc[kH];
    float vv[kH];
#pragma unroll
    for (int h = 0; h < kH; ++h) { cc[h] = 0; vv[h] = 0.f; }
    bool simple_a = false;
    auto load_rp = [&](int64_t tile) -> int64_t {
        const int64_t ri = tile * kTileRows + (l < kTileRows ? l : kTileRows);
        return rowptr[ri < n ? ri : n];                  // lanes 0..kTileRows hold the pointers; rows past the end read rowptr[n]
    };
    auto load_cols = [&](int64_t tile) {                 // from rp_a
        const int64_t begin = __shfl(rp_a, 0), t_end = __shfl(rp_a, kTileRows), rp_next = __shfl_down(rp_a, 1);
        const int64_t len = rp_next - rp_a;
        const bool full = (tile + 1) * kTileRows <= n && tile < x_end;
        simple_a = full && __ballot(l < kTileRows && (len > kPipeD || len >= T)) == 0;
        const int32_t m = simple_a ? (int32_t)(t_end - begin) : 0;          // <= kSlots
        // unconditional loads (lanes past the end read entry 0): the number of loads in flight stays known
#pragma unroll
        for (int h = 0; h < kH; ++h) {
            const int64_t i = l + kWave * h < m ? begin + l + kWave * h : 0;
            cc[h] = __builtin_nontemporal_load(&col[i]);
            if (W == kExplicit) vv[h] = __builtin_nontemporal_load(&val[i]);
        }
    };
    auto stage = [&]() -> bool {                         // rp_a, cc, vv -> slot table; a tile that is not simple is staged as empty
        const int32_t rel = simple_a ? (int32_t)(rp_a - __shfl(rp_a, 0)) : 0;
#pragma unroll
        for (int h = 0; h < kH; ++h) {
            const int s = l + kWave * h;                 // slot s: row r, entry k
            const int r = s / kPipeD, k = s - r * kPipeD;
            const int32_t lo = __shfl(rel, r), hi = __shfl(rel, r + 1);
            const int src = lo + k;
            int32_t c = 0;
            float wt = 0.f;
#pragma unroll
            for (int q = 0; q < kH; ++q) {
                const int32_t cq = __shfl(cc[q], src - kWave * q);
                c = (src >> 6) == q ? cq : c;
                if (W == kExplicit) {
                    const float wq = __shfl(vv[q], src - kWave * q);
                    wt = (src >> 6) == q ? wq : wt;
                }
            }
            const bool live = k < hi - lo;
            if (s < kSlots) {
                const int64_t off = live ? ((int64_t)c << kRowShift) : zero_off;
                if constexpr (W == kExplicit) s_slot[w][s] = SlotW{off, live ? wt : 0.f, 0.f};
                else s_slot[w][s] = off;
            }
        }
        const int32_t len = __shfl_down(rel, 1) - rel;   // all lanes take part in the exchange
        if (W == kMean && l < kTileRows) s_inv[w][l] = row_weight<kMean>(len);
        pipe_wave_sync();
        return simple_a;
    };

    // ---- one group: kRpg rows, one per lane group
    struct Regs {
        v4f xs[kPipeD];
        float ws[W == kExplicit ? kPipeD : 1];
        float inv;
    };
    Regs rr[G];
    auto issue = [&](Regs &q, int grp) {
        const int lr = grp * kRpg + g;
        if (W == kMean) q.inv = s_inv[w][lr];
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

    // ---- prologue: the first tile is staged and put in flight, the CSR of the next two is on its way
    rp_a = load_rp(t_first);
    load_cols(t_first);
    bool simple_cur = stage();
    rp_a = load_rp(t_first + stride);
    load_cols(t_first + stride);
    rp_b = load_rp(t_first + 2 * stride);
#pragma unroll
    for (int grp = 0; grp < G; ++grp) issue(rr[grp], grp);
    // Everything above has arrived before the loop starts: the loop's own order of loads is then the
    // only one the compiler has to account for at the loop head, and its waits stay exact.
    __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0)

    for (int64_t tile = t_first; tile < x_end; tile += stride) {
        const bool simple_next = stage();                // CSR of the next tile -> slot table (this tile's groups are all issued)
        rp_a = rp_b;
        load_cols(tile + 2 * stride);
        rp_b = load_rp(tile + 3 * stride);
        const int64_t base = tile * kTileRows;
        char *const ybase = (simple_cur ? Y + (base << kRowShift) : trash) + 16 * f;
#pragma unroll
        for (int grp = 0; grp < G; ++grp) {
            const v4f a = sum(rr[grp]);
            __builtin_nontemporal_store(a, (v4f *)(ybase + ((grp * kRpg + g) << kRowShift)));
            issue(rr[grp], grp);                         // the same rows of the next tile
        }
        if (!simple_cur) {
            // plain path: the low-degree rows of this tile straight from global memory
#pragma unroll 1
            for (int grp = 0; grp < G; ++grp) {
                const int64_t row = base + grp * kRpg + g;
                if (row < n) {
                    const int64_t s = rowptr[row], e = rowptr[row + 1];
                    if (e - s < T)
                        __builtin_nontemporal_store(ld_row_sum<W, false>(s, e, col, val, (const v4f *)X, L, f),
                                                    (v4f *)(Y + (row << kRowShift) + 16 * f));
                }
            }
        }
        simple_cur = simple_next;
    }
}

struct PipeArgs {
    const int64_t *rowptr;
    const int32_t *col;
    const float *val;
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
};

template <int L, int W, int G>
static void pipe_launch(const PipeArgs &a)
{
    ld_pipe_kernel<L, W, G><<<dim3((unsigned)a.n_wg), dim3(kPipeWaves * kWave), 0, a.st>>>(
        a.rowptr, a.col, a.val, a.X, a.Y, a.zero_off, a.trash, a.n, a.T, a.n_tiles, a.tiles_per_part, a.waves_per_part,
        a.parts);
}

template <int W, int G>
static void pipe_dispatch_l(int32_t F4, const PipeArgs &a)
{
    if (F4 == 8) pipe_launch<8, W, G>(a);
    else if (F4 == 16) pipe_launch<16, W, G>(a);
    else pipe_launch<32, W, G>(a);
}

int launch_ld_pipelined(const DevicePlan &dp, const float *X, float *Y, int32_t F, void *stream)
{
    constexpr int kG = 5;                                // groups in flight per wavefront (13.7 / 14.0 / 13.8 ms for 5 / 6 / 7)
    const int32_t F4 = F / 4;
    if (F4 != 8 && F4 != 16 && F4 != 32) return (int)hipErrorInvalidValue;
    if (!weights_ok(dp) || !dp.zero_row) return (int)hipErrorInvalidValue;
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return (int)e;
    const int tile_rows = kG * (kWave / F4);
    const int64_t n_tiles = (dp.n + tile_rows - 1) / tile_rows;
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
    hipStream_t st = (hipStream_t)stream;
    const PipeArgs a{dp.rowptr, col_arg, val_arg, (const char *)X, (char *)Y, byte_distance(X, dp.zero_row), trash, dp.n,
                     dp.threshold, n_tiles, tiles_per_part, waves_per_part, parts, n_wg, st};
    GROOT_DISPATCH_W(dp.weight_mode, (pipe_dispatch_l<kW, kG>(F4, a)));
    return (int)hipGetLastError();
}

}  // namespace groot
