// Internal declarations shared by the host boundary and the kernel launchers.
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

#include "decentlam.h"

namespace dl {

// One phase of W, small enough to travel in the kernel-argument segment (4 KiB with the other
// arguments).  Two encodings of the entries:
//   direct   up to DL_MAX_NNZ entries, each a column index and its fp32 weight;
//   palette  up to DL_MAX_NNZ_PALETTE entries, each a column index and an index into a table of at
//            most DL_MAX_WEIGHT_VALUES distinct fp32 weights (every built-in topology has a handful);
//   rows     up to DL_MAX_NNZ_ROW_WEIGHTS entries, each a column index only: every row carries a single
//            weight value (an index into the same kind of table per row).
constexpr int kMaxNnzPalette = DL_MAX_NNZ_PALETTE;
constexpr int kMaxNnzRowWeights = DL_MAX_NNZ_ROW_WEIGHTS;
constexpr int kMaxWeightValues = DL_MAX_WEIGHT_VALUES;
struct PhaseArgs {
    int32_t n;
    int32_t palette;                     // 0: direct, 1: palette, 2: rows
    union {
        uint16_t row_ptr[DL_MAX_NODES + 1];       // offsets relative to this phase
        uint32_t row_ptr_pairs[DL_MAX_NODES / 2 + 1];   // the same, two per word: what the kernel's scalar loads fetch
    };
    union {
        struct {
            uint8_t col[DL_MAX_NNZ];
            float w[DL_MAX_NNZ];
        } direct;
        struct {
            uint8_t col[kMaxNnzPalette];
            uint8_t widx[kMaxNnzPalette];
            float value[kMaxWeightValues];
        } pal;
        struct {
            uint8_t col[kMaxNnzRowWeights];
            union {
                uint8_t widx[DL_MAX_NODES];          // per row
                uint32_t widx_words[DL_MAX_NODES / 4];   // the same, four per word: what the kernel's scalar loads fetch
            };
            float value[kMaxWeightValues];
        } rows;
    };
};
static_assert(sizeof(PhaseArgs) <= 4096 - 128, "kernel-argument segment is 4 KiB");
static_assert(offsetof(PhaseArgs, pal.value) == offsetof(PhaseArgs, rows.value) &&
              offsetof(PhaseArgs, pal.col) == offsetof(PhaseArgs, rows.col) &&
              offsetof(PhaseArgs, direct.col) == offsetof(PhaseArgs, rows.col),
              "the kernels read the column bytes and the palette of any encoding through one member");

enum Algo { ALGO_DECENTLAM = 0, ALGO_DMSGD = 1, ALGO_DSGD = 2, ALGO_DECENTLAM_XPREV = 3, ALGO_AWC_DMSGD = 4,
            ALGO_DA_DMSGD = 5 };

int set_error(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
int check_hip(hipError_t e, const char* what);
void clear_error();

// The gradient operand of a step: fp32, or a 16-bit format that is widened exactly on load.
struct GradArg {
    const void* p;
    int format;   // dl_grad_format
    int64_t ld;   // row stride in elements of that format
};
inline size_t grad_elem_bytes(int format) { return format == DL_GRAD_F32 ? 4 : 2; }

// Per-tensor sums of squares fused into a step.  Tensor t is the column range
// [offsets[t], offsets[t + 1]) of the caller's arrays.  Every workgroup of a step launch owns one
// tile of columns and writes, for every node, a record of 3 doubles (sums of squares of g, new m,
// new x) with plain stores: one per tile, or with 16-byte lanes one per half tile, so that a record
// always covers one range of `tc` columns and is numbered by it, whatever the column order of the
// launch.  The records of one node are contiguous (node i's record q sits at (i * capacity + q) * 3),
// so that the final pass, one workgroup per tensor and node, reads consecutive memory.
// A final pass adds, for every tensor, the records of the ranges that lie wholly inside it and sums
// the remaining edge columns directly from the arrays.
constexpr int kMaxNormGrids = 4;   // aligned body (in two launches when it starts off a 64 KiB boundary), peeled head, peeled tail
struct NormGrid {
    int64_t col0;    // first column of the launch, relative to the first column of the step
    int64_t cols;    // columns covered by the launch
    int64_t tile0;   // index of the launch's first record in `partial`
    int32_t tc;      // columns per record (a tile; half a tile with 16-byte lanes)
};
struct NormPlan {
    const int64_t* offsets;   // host, num_tensors + 1; offsets[0] is the first column of the step
    int32_t num_tensors;
    double* partial;          // device, room for n x capacity records of 3 doubles
    int64_t capacity;         // records per node: norm_tiles_bound(d)
    double* norms;            // device, [num_tensors][n][3]
    NormGrid grid[kMaxNormGrids];   // appended to by every launch_step call of one iteration
    int grids;
    int64_t tiles_used;       // records written so far
    int64_t col_base;         // logical column of the next launch_step call's column 0
    int64_t bw;               // 0: row-major arrays; > 0: blocked layout with this block width
};
// Upper bound on the number of tile records a step over d columns writes, at any alignment.
inline int64_t norm_tiles_bound(int64_t d) { return (d + 63) / 64 + 3; }

// Enqueue one fused iteration over columns [0, d) of x, m, g (already validated).
// `beta` is a double so that the momentum-free form can pass beta * gamma / gamma_prev unrounded.
// With `norms` the launches also write their tile records and append their grids to it (a batched
// launch must then cover whole blocks: it is recorded as one grid over batches * d logical columns).
// With batches > 1 the launches cover `batches` equally shaped problems whose arrays start
// batch_stride (x, m) and batch_stride_g (g) elements apart -- the full blocks of the blocked layout.
int launch_step(Algo algo, float* x, float* m, GradArg g, int32_t n, int64_t d, int64_t ld,
                const PhaseArgs& topo, float gamma, double beta, hipStream_t stream,
                NormPlan* norms = nullptr, int64_t batches = 1, int64_t batch_stride = 0,
                int64_t batch_stride_g = 0);
// After launch_step with `norms`: x, m, g as passed there.
int launch_norms_finish(const NormPlan& plan, const float* x, const float* m, GradArg g, int64_t ld, int32_t n,
                        hipStream_t stream);

// Device-resident topology (topology_pack_device), 32-bit words: header {magic, n, period, 0}, `period` phase
// offsets (in words from the start of the buffer, each even), then per phase n + 1 row offsets into the phase's
// entries (padded to an even count) followed by the entries as (column, fp32 weight bits) pairs.
constexpr uint32_t kDeviceTopoMagic = 0x444C4454u;   // "DLDT"
constexpr int kDeviceTopoHeaderWords = 4;
__host__ __device__ constexpr int device_topo_row_ptr_words(int n) { return (n + 2) & ~1; }
// Enqueue one iteration with the lists of phase `phase` read from `device_topology` (already validated).
int launch_step_wide(Algo algo, float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld, float gamma,
                     double beta, const void* device_topology, int32_t phase, hipStream_t stream);

// Least-squares gradient (already validated).
size_t lsq_workspace_bytes(int32_t n, int32_t b, int64_t d);
// What the kernels that launch_lsq picks for this shape and alignment actually use (<= lsq_workspace_bytes).
bool lsq_wide_accesses(const float* A, const float* x, int64_t d, int64_t ldA, int64_t ld);
int lsq_path(int32_t bs, int64_t d, bool wide_accesses, bool sampled = false);
size_t lsq_workspace_bytes_path(int32_t n, int32_t b, int64_t d, int path);
// Polls after which a wave of the column-split sweep stops waiting for the others (negative: the default); returns the old value.
int lsq_poll_limit(int polls);
// rows == nullptr: full-batch gradient over all b rows; otherwise bs sampled rows per node.
int launch_lsq(const float* A, const float* y, const float* x, float* g, float* loss, int32_t n,
               int32_t b, int64_t d, int64_t ldA, int64_t ld, const int32_t* rows, int32_t bs, float scale,
               void* workspace, hipStream_t stream);

// The boundary of local_grad_lsq / local_grad_lsq_rows: validates every argument (status codes as the
// header documents them), then calls launch_lsq.  `fn` names the entry point in error messages.
int lsq_entry(const char* fn, const float* A, const float* y, const float* x, float* g, float* loss, int32_t n,
              int32_t b, int64_t d, int64_t ldA, int64_t ld, const int32_t* rows, int32_t bs, bool sampled,
              float scale, void* workspace, size_t workspace_bytes, void* stream, bool exact_need = false);

// Diagnostics (already validated).
size_t stats_workspace_bytes(int64_t d);
int launch_stats(const float* x, const float* m, const float* ref, int32_t n, int64_t d, int64_t ld,
                 double* out, void* workspace, hipStream_t stream);

}  // namespace dl
