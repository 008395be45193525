// Internal declarations shared by the host side and the HIP kernels of libgroot.
#pragma once

#include <atomic>
#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "groot.h"

namespace groot {

enum class WeightMode : int { Ones = 0, Mean = 1, Explicit = 2 };

void set_error(const std::string &msg);
groot_status fail(groot_status st, const std::string &msg);

// One piece of a high-degree row: nnz range [begin, begin+len) of row `row`.
// slot >= 0: the partial sum goes to partials[slot]; slot < 0: the row has a
// single piece and its sum goes straight to Y.
struct HdChunk {
    int64_t begin;
    int32_t len;
    int32_t row;
    int32_t slot;
    int32_t row_nnz;   // stored length of the whole row (row-uniform weights are 1/row_nnz)
};

// A high-degree row that was split: Y[row] = sum of partials[first .. first+count)
struct HdSplitRow {
    int32_t row;
    int32_t first;
    int32_t count;
    int32_t pad;
};

// Process-wide launch-shape knobs (groot_set_tuning).  Every knob is an atomic integer: a call that reads one
// sees either the old or the new value, never a torn one; which of two racing calls wins is up to the caller.
struct Tuning {
    std::atomic<int> xcd_remap{1};
    std::atomic<int> hd_chunk{512};
    std::atomic<int> sage_gap{2};          // pacing of the fused layer's matrix wavefronts, see launch_sage
    std::atomic<int> sage_split{1};        // 12-wavefront fused layer: 1 dense products as six bf16 piece products, 0 fp32 matrix instructions
    std::atomic<int> sage_kernel{1};       // fused layer: 1 one self-contained wavefront per SIMD, 0 the 12-wavefront kernel
    std::atomic<int> sage_pieces{3};       // fused layer (sage_kernel 1): bf16 pieces per fp32 operand of the dense products, 3 or 2
    std::atomic<int> uniform_detect{1};    // groot_plan_upload looks whether explicit weights are row-uniform (see DevicePlan)
    std::atomic<int> csr_compress{1};      // groot_plan_upload builds the compact CSR for the pipelined LD kernel when it can
    std::atomic<int> pipe_depth{0};        // gather slots per row of the pipelined LD kernel: 0 the smallest that fits, or 5..8
    std::atomic<int> ld_pipeline{-1};      // pipelined LD kernel: 1 always (where it applies), 0 never, -1 by the row lengths
};
Tuning &tuning();

// Device-resident part of a plan.
struct DevicePlan {
    int64_t n = 0, nnz = 0;
    int32_t threshold = 0;
    int64_t *rowptr = nullptr;
    int32_t *col = nullptr;
    float *val = nullptr;
    int weight_mode = 0;            // WeightMode the kernels run in; explicit weights that turn out to be 1/row length
                                    // (or all 1) run as row-uniform weights and their array is not read
    int graph_weight_mode = 0;      // WeightMode of the graph itself; val is NULL unless this is Explicit
    int64_t n_tiles = 0;            // LD tiles of kRowsPerLdTile rows
    HdChunk *chunks = nullptr;
    int64_t n_chunks = 0;
    HdSplitRow *split_rows = nullptr;
    int64_t n_split_rows = 0;
    float *partials = nullptr;      // [n_partials, partial_stride]
    int64_t n_partials = 0;
    int64_t nnz_hd = 0;             // stored entries of the high-degree rows (sum of the pieces' lengths)
    int xcd_remap = 1;
    float *zero_row = nullptr;      // kZeroRowFloats zeros (the gather target of unused slots in the pipelined
                                    // kernels), followed by kTrashFloats that those kernels may overwrite
    // the fused layer's view of the high-degree rows: their ids (ascending), a buffer that takes their aggregated
    // features, one row per high-degree row in that order, and the HD schedule with every row named by its place
    // in the list instead of its id (so that the HD kernels write into the buffer)
    int32_t *hd_rows = nullptr;     // [n_hd_rows]
    int64_t n_hd_rows = 0;
    float *hd_agg = nullptr;        // [n_hd_rows, max_F]
    HdChunk *chunks_rank = nullptr; // [n_chunks]
    HdSplitRow *split_rows_rank = nullptr;   // [n_split_rows]
    // compact CSR for the pipelined LD kernel (groot_compress.hip); all NULL / 0 unless compressed
    uint32_t *rp32 = nullptr;       // [n+1] low 32 bits of rowptr (nnz < 2^32)
    uint16_t *col16 = nullptr;      // [nnz] column codes of the rows the pipelined kernel serves
    int32_t *hot_cols = nullptr;    // [n_hot] the high-degree rows that a code can name, ascending
    int32_t n_hot = 0;
    int64_t n_bad_rows = 0;         // rows with an entry that no code expresses (they are part of mid_rows)
    int compressed = 0;
    int64_t n_cols = 0;             // rows of the feature matrix the columns index: n, or the whole graph's row
                                    // count once a part's plan reads the global matrix in place
    int ld_pipelined = 0;           // pipelined LD kernel: 0 never, 1 for F = 64 and 128, 2 for F = 32 as well
    int sage_depth = 6;             // gather slots per row of the fused layer kernel: 5 when rows of 6 entries are rare, else 6
    int pipe_depth = 6;             // slots per row of the pipelined LD kernel: kPipeMinDepth .. kPipeMaxDepth
    int32_t *mid_rows = nullptr;    // low-degree rows with more than pipe_depth entries (the pipelined kernel
    int64_t n_mid_rows = 0;         // masks them; a row-list kernel computes them), ordered by (length, id)
};

constexpr int kCodeNear = 0x4000;     // column codes below kCodeHot: row + code - kCodeNear
constexpr int kCodeHot = 0x8000;      // codes from here on: index into the hot list
constexpr int kCodeBad = 0xFFFF;      // an entry that no code can express: its row is not served in compact form
constexpr int kCodeMaxHot = 0x7FFF;
constexpr int kPipeMinDepth = 5, kPipeMaxDepth = 8;   // gather slots per row the pipelined LD kernel is built for
constexpr int kZeroRowFloats = 128;
constexpr int kTrashFloats = 2048;
constexpr int kRowsPerLdTile = 256;   // rows of one LD block (4 wavefronts x 64 rows)

// Optional restriction and redirection of the output rows: only rows [0, n_out) are computed, and row r is
// written to Y[ids[r]] (ids == NULL: to Y[r]).  Device pointer.
struct RowOut {
    const int64_t *ids;
    int64_t n_out;
};

// Kernel launchers (groot_kernels.hip).  Return hipError_t as int (0 = success).
int launch_ld(const DevicePlan &dp, const float *X, float *Y, int32_t F, void *stream, const RowOut *out = nullptr);
int launch_ld_pipelined(const DevicePlan &dp, const float *X, float *Y, int32_t F, void *stream,
                        const RowOut *out = nullptr);   // F = 32, 64, 128
int launch_hd(const DevicePlan &dp, const float *X, float *Y, int32_t F, void *stream, const RowOut *out = nullptr);
int launch_hd_finish(const DevicePlan &dp, float *Y, int32_t F, void *stream, const RowOut *out = nullptr);
int launch_sage(const DevicePlan &dp, const float *X, float *H, const float *Wn, const float *Ws, const float *bias,
                int relu, void *stream);
int launch_sage_pipe(const DevicePlan &dp, const float *X, float *H, const float *Wn, const float *Ws, const float *bias,
                     int relu, int32_t F_in, int32_t F_out, int pieces, int self_times_degree,
                     void *stream);   // F_in 32 / 64, F_out 16 / 32 / 64, row-uniform weights; pieces 3 (fp32 accuracy) or 2;
                                      // self_times_degree: unit weights and the own-row operand times the row length (input gradient)
// Weight gradients of the fused layer (groot_sage_wgrad.hip): dWn = (A_hat X)^T dZ, dWs = X^T dZ, X of width F_in = 32
// or 64, dZ of width F_out = 16, 32 or 64, row-uniform weights; workspace of sage_wgrad_workspace_bytes bytes (0: no device).
size_t sage_wgrad_workspace_bytes(int32_t F_in, int32_t F_out);
int launch_sage_wgrad(const DevicePlan &dp, const float *X, const float *dZ, float *dWn, float *dWs, int32_t F_in,
                      int32_t F_out, int pieces, void *workspace, void *stream);
int launch_rows_over_degree(const DevicePlan &dp, const float *Z, float *out, int32_t F, void *stream);   // out may be Z
// Schedule of the high-degree rows built on the device (groot_hd_sched_device.hip): the pieces in execution order,
// once with rows named by id and once by their place in the list of high-degree rows, and the split rows likewise.
struct DeviceHdSchedule {
    HdChunk *chunks = nullptr, *chunks_rank = nullptr;
    HdSplitRow *split_rows = nullptr, *split_rows_rank = nullptr;
    int64_t n_chunks = 0, n_split_rows = 0, n_partials = 0, nnz_hd = 0;
};
constexpr int kErrTooManyPieces = -3;
int launch_hd_schedule_device(const int64_t *rowptr_dev, const int32_t *col_dev, const int32_t *hd_rows_dev, int64_t n_hd,
                              int32_t hd_chunk, void *stream, DeviceHdSchedule *out);   // synchronises the stream
void free_device_hd_schedule(DeviceHdSchedule &s);
// Compact CSR for the pipelined LD kernel, built on the device (groot_compress.hip); synchronises the stream.
int launch_csr_compress(DevicePlan &dp, const int32_t *hd_rows_dev, int64_t n_hd, void *stream);
int pipe_compact_prepare();   // once per process, before the first launch with a compact CSR; hipError_t as int
// col[p] = ids[col[p]] for p < nnz, in place (a part's local columns -> rows of the whole graph's feature matrix)
int launch_col_map(int32_t *col, int64_t nnz, const int64_t *ids, void *stream);
int launch_rows_gather(const int64_t *ids, int64_t n, const float *X, float *out, int32_t F, void *stream);
int launch_rows_scatter(const int64_t *ids, int64_t n, const float *in, float *Y, int32_t F, void *stream);
// Device-side plan lists (groot_plan_device.hip).  Synchronises the stream; kErrOutOfDeviceMemory when its
// scratch cannot be allocated.
constexpr int kPlanDeviceMaxThreshold = 1024;
constexpr int kErrOutOfDeviceMemory = 2;   // hipErrorOutOfMemory
int launch_plan_device(const int64_t *rowptr_dev, int64_t n, int32_t T, uint8_t *row_class, int32_t *hd_rows,
                       int32_t *ld_rows, int32_t *by_degree, int64_t *deg_offsets, int64_t *counts, void *stream);
// The same lists with the block table in a fixed array inside the library instead of allocated memory: no
// allocation, no synchronisation; hipErrorInvalidValue when plan_static_scratch_needed exceeds the array.
constexpr size_t kPlanStaticScratchBytes = (size_t)8 << 20;
size_t plan_static_scratch_needed(int64_t n, int32_t T);
int launch_plan_device_static(const int64_t *rowptr_dev, int64_t n, int32_t T, uint8_t *row_class, int32_t *hd_rows,
                              int32_t *ld_rows, int32_t *by_degree, int64_t *deg_offsets, int64_t *counts,
                              void *stream);
// One part of a partition with re-grown boundary, built on the device (groot_regrow_device.hip).  All pointers
// are device memory owned by the struct's holder; val is NULL unless the source graph has explicit weights.
struct DevicePart {
    int64_t n_owned = 0, n_halo = 0, n_crossing = 0, nnz = 0;
    int64_t *global_id = nullptr;   // [n_owned + n_halo]
    int64_t *rowptr = nullptr;      // [n_owned + n_halo + 1]
    int32_t *col = nullptr;         // [nnz] local ids
    float *val = nullptr;           // [nnz] or NULL
};
constexpr int kErrBadPartId = -2;   // a caller-supplied part id outside [0, P)
// Synchronises the stream.  part_of_dev may be NULL (built-in rule with n1 nodes per copy).
int launch_regrow_device(const DevicePlan &dp, int64_t n1, int32_t P, const int32_t *part_of_dev, int32_t p,
                         int regrow, void *stream, DevicePart *out);
void free_device_part(DevicePart &part);
// Small synchronous device reads and copies (sizes and lists of a plan built from device arrays).
int device_time_ms(void *stream, int reps, int (*fn)(void *ctx), void *ctx, float *ms);
int device_download(void *dst_host, const void *src_dev, size_t bytes, void *stream);
int device_copy(void *dst_dev, const void *src_dev, size_t bytes, void *stream);   // device to device, synchronous
const char *hip_error_text(int err);

// Device memory helpers (groot_kernels.hip, so that the host file needs no HIP headers).
int dev_alloc(void **p, size_t bytes);
void dev_free(void *p);
int dev_upload(void *dst, const void *src, size_t bytes);

}  // namespace groot
