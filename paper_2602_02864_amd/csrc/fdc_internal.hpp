// Internal declarations shared by the host-only and the HIP translation units.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "fdc.h"

namespace fdc {

int32_t fail(int32_t code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

int32_t build_plan(int32_t F, const int32_t* slot_len, int32_t E, const int32_t* src,
                   const int32_t* dst, int32_t prefix_len, uint64_t* anc, int32_t* slot_start,
                   int32_t* level, int32_t* total_len);

constexpr int kMaxFields = 64;      // one 64-bit ancestor word per field in the kernels
constexpr int kMaxRowsDense = 16;   // rows per step the streaming projections take; more go to the tiled ones
constexpr int kMaxRowsStep = 1024;  // rows per step overall
constexpr int kStageSlots = 8;      // pinned staging ring for per-step metadata
constexpr int kMaxChunkTiles = 128; // 32-key tiles one attention workgroup walks at most (LDS-shared tiles)
constexpr int kMaxChunkTilesReg = 512;  // ... with tiles in registers
constexpr int kMaxChunkTilesWide = 64;  // ... in the many-row kernel (one tile list entry per lane)
constexpr int kMaxMaskedTiles = 32; // ... of which this many may reach into the slots
constexpr int kF16Default = 16;     // projections that take the fp16 path when fp16 weights exist: the LM head

// How one projection y = x W^T is cut: S splits of the reduction dimension,
// each handled by workgroups of `nw` wavefronts that keep their slice of the
// activations in registers and stream `nt` 16-row weight tiles per task.
struct GemmPlan {
    int KT = 0;        // 32-wide k tiles
    int n_tiles = 0;   // 16-row output tiles
    int S = 1;         // splits of K (partials summed by the consumer)
    int kt_split = 0;  // k tiles per split
    int nw = 8;        // wavefronts per workgroup
    int ktw = 16;      // compile-time bound on k tiles per wavefront
    int nt = 1;        // n tiles per task
    int n_tasks = 0;
    int grid = 0;
};

GemmPlan plan_gemm(int64_t n_out, int64_t k_in, bool swiglu);

// The same projection for more than 16 rows: workgroups of 2 x 2 wavefronts own
// 128 rows x (2 * ntw) 16-feature tiles, S splits of K.
struct TiledPlan {
    int KT = 0;        // 32-wide k tiles
    int n_tiles = 0;   // 16-feature tiles (padded weight rows included)
    int m_tiles = 0;   // 16-row tiles
    int S = 1;
    int kt_split = 0;
    int ntw = 8;       // feature tiles per wavefront
    int n_groups = 0;  // workgroup columns
    int m_blocks = 0;  // workgroup rows
    int grid = 0;
};

TiledPlan plan_tiled(int M, int64_t n_out, int64_t k_in, bool swiglu, int max_splits = 16);

}  // namespace fdc
