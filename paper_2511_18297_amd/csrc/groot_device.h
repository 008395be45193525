// Device-side helpers shared by the HIP sources of libgroot (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>

#include "groot_internal.h"

namespace groot {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kBlock = 256;                  // threads per workgroup (4 wavefronts)
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kLdTileRows = 64;              // consecutive rows per wavefront tile
constexpr int kLdTileCap = 512;              // non-zeros of a tile that are staged in LDS
constexpr int kXcds = 8;                     // workgroups are dealt round-robin over 8 XCDs

// Each XCD has its own L2.  Consecutive hardware workgroup ids land on
// different XCDs, so the logical block index is transposed: XCD x walks the
// x-th contiguous eighth of the tiles in ascending order.
__device__ __forceinline__ int64_t logical_block(int64_t blocks_per_xcd, int remap)
{
    int64_t b = blockIdx.x;
    return remap ? (b % kXcds) * blocks_per_xcd + b / kXcds : b;
}

// Weight of the entries of a row: kExplicit reads val[]; kMean and kOnes are
// the row-uniform weights of graphs built from an AIG and need no weight array
// (1/row length is recomputed in registers, correctly rounded, from the row
// pointer; this saves 4 bytes of HBM traffic per non-zero).
enum : int { kOnes = (int)WeightMode::Ones, kMean = (int)WeightMode::Mean, kExplicit = (int)WeightMode::Explicit };

template <int W>
__device__ __forceinline__ float row_weight(int64_t row_nnz)
{
    return W == kMean ? (row_nnz > 0 ? 1.0f / (float)row_nnz : 0.0f) : 1.0f;
}

// Sum of one row for one float4 slice: the feature slices of up to D neighbours are gathered
// before the first add (kStaged: indices/weights come from the tile's copy in LDS, else from
// global memory), accumulated in registers in CSR order, and scaled by the row weight.
template <int W, bool kStaged, int D = 8>
__device__ __forceinline__ v4f ld_row_sum(int64_t s, int64_t e, const int32_t *__restrict__ cols,
                                          const float *__restrict__ vals, const v4f *__restrict__ X,
                                          int32_t F4, int32_t ff)
{
    v4f acc = {0.f, 0.f, 0.f, 0.f};
    for (int64_t p = s; p < e; p += D) {
        v4f x[D];
        float w[D];
#pragma unroll
        for (int k = 0; k < D; ++k) {
            if (p + k < e) {
                int32_t c = kStaged ? cols[p + k] : __builtin_nontemporal_load(&cols[p + k]);
                if (W == kExplicit) w[k] = kStaged ? vals[p + k] : __builtin_nontemporal_load(&vals[p + k]);
                x[k] = X[(int64_t)c * F4 + ff];
            }
        }
#pragma unroll
        for (int k = 0; k < D; ++k)
            if (p + k < e) {
                if (W == kExplicit) acc += w[k] * x[k];
                else acc += x[k];
            }
    }
    if (W != kExplicit) acc *= row_weight<W>(e - s);
    return acc;
}


#define GROOT_DISPATCH_L(L, CALL)        \
    switch (L) {                         \
    case 1: { constexpr int kL = 1; CALL; } break;   \
    case 2: { constexpr int kL = 2; CALL; } break;   \
    case 4: { constexpr int kL = 4; CALL; } break;   \
    case 8: { constexpr int kL = 8; CALL; } break;   \
    case 16: { constexpr int kL = 16; CALL; } break; \
    case 32: { constexpr int kL = 32; CALL; } break; \
    default: { constexpr int kL = 64; CALL; } break; \
    }

#define GROOT_DISPATCH_W(W, CALL)                           \
    switch (W) {                                            \
    case kOnes: { constexpr int kW = kOnes; CALL; } break;  \
    case kMean: { constexpr int kW = kMean; CALL; } break;  \
    default: { constexpr int kW = kExplicit; CALL; } break; \
    }

// Signed byte distance between two device addresses that belong to different allocations (the row of zeros
// of a plan, seen from a feature matrix): integer arithmetic on the addresses, not a pointer difference.
inline int64_t byte_distance(const void *from, const void *to)
{
    return (int64_t)((uintptr_t)to - (uintptr_t)from);
}

inline bool grid_ok(int64_t blocks) { return blocks > 0 && blocks <= 0x7fffffffLL; }

// explicit weights need the weight array on the device; the other modes never touch it
inline bool weights_ok(const DevicePlan &dp)
{
    return dp.weight_mode == kOnes || dp.weight_mode == kMean || dp.val != nullptr || dp.nnz == 0;
}

}  // namespace groot
