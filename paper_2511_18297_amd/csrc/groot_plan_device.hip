// Device-side degree plan for gfx950: the LD kernel's "step B" of the paper on the GPU -- every row's
// degree from the row pointer, its class, and a stable counting sort of the low-degree rows by degree
// (linear time, as the paper notes for count sort).  All integer work; the lists are bit-identical to
// the host plan's.
//
// Three launches over blocks of 4096 consecutive rows (256 threads; a wavefront owns 1024 consecutive rows):
//   plan_count    per block: number of low-degree rows of every degree < T, of LD rows, of HD rows
//   plan_scan     per column of that table: exclusive prefix over the blocks (+ totals); then the
//                 degree offsets are the exclusive prefix of the per-degree totals
//   plan_scatter  per block again: every row gets its position = column start + rows of the same
//                 column in earlier blocks + in earlier wavefronts of the block + earlier in its own
//                 wavefront (ballot ranks in lane order), which is exactly the stable order
#include <mutex>

#include "groot_device.h"

namespace groot {

constexpr int kPlanRowsPerWave = 1024;
constexpr int kPlanRowsPerBlock = kPlanRowsPerWave * kWavesPerBlock;   // 4096
constexpr int kPlanMaxCols = kPlanDeviceMaxThreshold + 2;              // degrees 0..T-1, LD count, HD count
static_assert(kErrOutOfDeviceMemory == (int)hipErrorOutOfMemory, "error code shared with the host side");

// stored length of row i; a row pointer that runs backwards counts as an empty row
__device__ __forceinline__ int64_t plan_degree(const int64_t *__restrict__ rowptr, int64_t i)
{
    const int64_t d = rowptr[i + 1] - rowptr[i];
    return d < 0 ? 0 : d;
}

__device__ __forceinline__ void plan_wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// hist[block * cols + c]
__global__ __launch_bounds__(kBlock) void plan_count(const int64_t *__restrict__ rowptr, int64_t n, int32_t T,
                                                     int32_t cols, int32_t *__restrict__ hist,
                                                     uint8_t *__restrict__ row_class)
{
    __shared__ int32_t s_cnt[kPlanMaxCols];
    for (int c = threadIdx.x; c < cols; c += kBlock) s_cnt[c] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kPlanRowsPerBlock;
    for (int k = 0; k < kPlanRowsPerBlock / kBlock; ++k) {
        const int64_t i = base + (int64_t)k * kBlock + threadIdx.x;
        if (i < n) {
            const int64_t d = plan_degree(rowptr, i);
            const bool hd = d >= T;
            row_class[i] = hd ? 1 : 0;
            atomicAdd(&s_cnt[hd ? T + 1 : (int)d], 1);
            if (!hd) atomicAdd(&s_cnt[T], 1);
        }
    }
    __syncthreads();
    for (int c = threadIdx.x; c < cols; c += kBlock) hist[(int64_t)blockIdx.x * cols + c] = s_cnt[c];
}

// One workgroup per column: hist[., c] -> exclusive prefix over the blocks, total[c] = column sum.
__global__ __launch_bounds__(kBlock) void plan_scan(int32_t *__restrict__ hist, int64_t n_blocks, int32_t cols,
                                                    int64_t *__restrict__ total)
{
    __shared__ int64_t s_part[kBlock];
    const int c = blockIdx.x;
    const int64_t seg = (n_blocks + kBlock - 1) / kBlock;
    const int64_t b0 = (int64_t)threadIdx.x * seg, b1 = b0 + seg < n_blocks ? b0 + seg : n_blocks;
    int64_t sum = 0;
    for (int64_t b = b0; b < b1; ++b) sum += hist[b * cols + c];
    s_part[threadIdx.x] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t run = 0;
        for (int t = 0; t < kBlock; ++t) { int64_t v = s_part[t]; s_part[t] = run; run += v; }
        total[c] = run;
    }
    __syncthreads();
    int64_t run = s_part[threadIdx.x];
    for (int64_t b = b0; b < b1; ++b) {
        const int32_t v = hist[b * cols + c];
        hist[b * cols + c] = (int32_t)run;
        run += v;
    }
}

// deg_offsets[d] = number of LD rows of degree < d (d = 0..T); counts = {n_hd, n_ld}
__global__ void plan_offsets(const int64_t *__restrict__ total, int32_t T, int64_t *__restrict__ deg_offsets,
                             int64_t *__restrict__ counts)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        int64_t run = 0;
        for (int d = 0; d < T; ++d) { deg_offsets[d] = run; run += total[d]; }
        deg_offsets[T] = run;
        counts[0] = total[T + 1];
        counts[1] = total[T];
    }
}

__global__ __launch_bounds__(kBlock) void plan_scatter(const int64_t *__restrict__ rowptr, int64_t n, int32_t T,
                                                       int32_t cols, const int32_t *__restrict__ prefix,
                                                       const int64_t *__restrict__ deg_offsets,
                                                       int32_t *__restrict__ hd_rows, int32_t *__restrict__ ld_rows,
                                                       int32_t *__restrict__ by_degree)
{
    __shared__ int32_t s_pos[kWavesPerBlock][kPlanMaxCols];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const uint64_t lt_mask = lane ? (~0ULL >> (64 - lane)) : 0ULL;
    const int64_t wbase = (int64_t)blockIdx.x * kPlanRowsPerBlock + (int64_t)wave * kPlanRowsPerWave;

    for (int c = lane; c < cols; c += kWave) s_pos[wave][c] = 0;
    plan_wave_sync();
    // per-wavefront counts of every column
    for (int k = 0; k < kPlanRowsPerWave / kWave; ++k) {
        const int64_t i = wbase + (int64_t)k * kWave + lane;
        if (i < n) {
            const int64_t d = plan_degree(rowptr, i);
            const bool hd = d >= T;
            atomicAdd(&s_pos[wave][hd ? T + 1 : (int)d], 1);
            if (!hd) atomicAdd(&s_pos[wave][T], 1);
        }
    }
    __syncthreads();
    // start position of every (wavefront, column): earlier blocks + earlier wavefronts (+ the degree's offset)
    for (int c = threadIdx.x; c < cols; c += kBlock) {
        int64_t run = prefix[(int64_t)blockIdx.x * cols + c] + (c < T ? deg_offsets[c] : 0);
        for (int w = 0; w < kWavesPerBlock; ++w) {
            const int32_t v = s_pos[w][c];
            s_pos[w][c] = (int32_t)run;
            run += v;
        }
    }
    __syncthreads();
    // rows in order: 64 at a time, rank among equal columns by ballot in lane order
    for (int k = 0; k < kPlanRowsPerWave / kWave; ++k) {
        const int64_t i = wbase + (int64_t)k * kWave + lane;
        const bool valid = i < n;
        int64_t d = 0;
        if (valid) d = plan_degree(rowptr, i);
        const bool hd = valid && d >= T, ld = valid && d < T;
        const uint64_t m_hd = __ballot(hd), m_ld = __ballot(ld);
        if (hd) hd_rows[s_pos[wave][T + 1] + __popcll(m_hd & lt_mask)] = (int32_t)i;
        if (ld) ld_rows[s_pos[wave][T] + __popcll(m_ld & lt_mask)] = (int32_t)i;
        plan_wave_sync();
        if (lane == 0) { s_pos[wave][T + 1] += __popcll(m_hd); s_pos[wave][T] += __popcll(m_ld); }
        uint64_t remaining = m_ld;
        while (remaining) {                                  // one turn per distinct degree in this chunk
            const int leader = __ffsll((unsigned long long)remaining) - 1;
            const int dl = (int)__shfl((int)d, leader);
            const uint64_t peers = __ballot(ld && (int)d == dl);
            if (ld && (int)d == dl) by_degree[s_pos[wave][dl] + __popcll(peers & lt_mask)] = (int32_t)i;
            plan_wave_sync();
            if (lane == leader) s_pos[wave][dl] += __popcll(peers);
            plan_wave_sync();
            remaining &= ~peers;
        }
        plan_wave_sync();
    }
}

namespace {

// the four launches on the caller's stream, with the block table and the column totals where the caller says
int plan_launches(const int64_t *rowptr_dev, int64_t n, int32_t T, int32_t cols, int64_t n_blocks, int32_t *hist,
                  int64_t *total, uint8_t *row_class, int32_t *hd_rows, int32_t *ld_rows, int32_t *by_degree,
                  int64_t *deg_offsets, int64_t *counts, hipStream_t st)
{
    if (n_blocks)
        plan_count<<<dim3((unsigned)n_blocks), dim3(kBlock), 0, st>>>(rowptr_dev, n, T, cols, hist, row_class);
    plan_scan<<<dim3((unsigned)cols), dim3(kBlock), 0, st>>>(hist, n_blocks, cols, total);   // an empty graph: all totals 0
    plan_offsets<<<dim3(1), dim3(64), 0, st>>>(total, T, deg_offsets, counts);
    if (n_blocks)
        plan_scatter<<<dim3((unsigned)n_blocks), dim3(kBlock), 0, st>>>(rowptr_dev, n, T, cols, hist, deg_offsets,
                                                                      hd_rows, ld_rows, by_degree);
    return (int)hipGetLastError();
}

// Scratch of the entry point that may not allocate: the column totals (int64 [cols]) at offset 0 and the
// block table (int32 [n_blocks][cols]) behind them.  One copy per GPU, held until the process ends; every
// call on a GPU uses the same bytes.  In host code `scratch` is only a handle for hipGetSymbolAddress: the
// device address it yields is what kernels, copies and clears are given.
static __device__ __align__(256) unsigned char scratch[kPlanStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char *g_scratch_ptr[kMaxDevices] = {};

// device address of the current device's copy of `scratch` (looked up once per device)
int static_scratch(unsigned char **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return (int)e;
        if (!p) return (int)hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = (unsigned char *)p;
    }
    *out = g_scratch_ptr[dev];
    return 0;
}

constexpr size_t plan_totals_bytes(int32_t cols) { return ((size_t)cols * sizeof(int64_t) + 255) / 256 * 256; }

}  // namespace

int launch_plan_device(const int64_t *rowptr_dev, int64_t n, int32_t T, uint8_t *row_class, int32_t *hd_rows,
                       int32_t *ld_rows, int32_t *by_degree, int64_t *deg_offsets, int64_t *counts, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const int32_t cols = T + 2;
    const int64_t n_blocks = (n + kPlanRowsPerBlock - 1) / kPlanRowsPerBlock;
    if (T < 1 || cols > kPlanMaxCols || n < 0 || n > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    int32_t *hist = nullptr;
    int64_t *total = nullptr;
    hipError_t e = hipMalloc((void **)&hist, (size_t)(n_blocks ? n_blocks : 1) * cols * sizeof(int32_t));
    if (e != hipSuccess) return (int)hipErrorOutOfMemory;
    e = hipMalloc((void **)&total, (size_t)cols * sizeof(int64_t));
    if (e != hipSuccess) { (void)hipFree(hist); return (int)hipErrorOutOfMemory; }
    const int err = plan_launches(rowptr_dev, n, T, cols, n_blocks, hist, total, row_class, hd_rows, ld_rows, by_degree,
                                  deg_offsets, counts, st);
    hipError_t e2 = hipStreamSynchronize(st);               // the scratch is freed below
    (void)hipFree(hist);
    (void)hipFree(total);
    return err ? err : (int)e2;
}

size_t plan_static_scratch_needed(int64_t n, int32_t T)
{
    const int64_t n_blocks = (n + kPlanRowsPerBlock - 1) / kPlanRowsPerBlock;
    return plan_totals_bytes(T + 2) + (size_t)n_blocks * (size_t)(T + 2) * sizeof(int32_t);
}

int launch_plan_device_static(const int64_t *rowptr_dev, int64_t n, int32_t T, uint8_t *row_class, int32_t *hd_rows,
                              int32_t *ld_rows, int32_t *by_degree, int64_t *deg_offsets, int64_t *counts,
                              void *stream)
{
    const int32_t cols = T + 2;
    const int64_t n_blocks = (n + kPlanRowsPerBlock - 1) / kPlanRowsPerBlock;
    if (T < 1 || cols > kPlanMaxCols || n < 0 || n > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    if (plan_static_scratch_needed(n, T) > kPlanStaticScratchBytes) return (int)hipErrorInvalidValue;
    unsigned char *base = nullptr;
    const int err = static_scratch(&base);
    if (err) return err;
    // Nothing in the scratch has to start at zero: plan_count writes every column of every block's table
    // entry, plan_scan every total, before anything reads them.
    int64_t *total = (int64_t *)base;
    int32_t *hist = (int32_t *)(base + plan_totals_bytes(cols));
    return plan_launches(rowptr_dev, n, T, cols, n_blocks, hist, total, row_class, hd_rows, ld_rows, by_degree,
                         deg_offsets, counts, (hipStream_t)stream);
}

}  // namespace groot
