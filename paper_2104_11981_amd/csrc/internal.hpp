// Internal declarations shared by the host boundary and the kernel launchers.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "decentlam.h"

namespace dl {

// One phase of W, small enough to travel in the kernel-argument segment (4 KiB with the other
// arguments).  Two encodings of the entries:
//   direct   up to DL_MAX_NNZ entries, each a column index and its fp32 weight;
//   palette  up to DL_MAX_NNZ_PALETTE entries, each a column index and an index into a table of at
//            most DL_MAX_WEIGHT_VALUES distinct fp32 weights (every built-in topology has a handful).
constexpr int kMaxNnzPalette = DL_MAX_NNZ_PALETTE;
constexpr int kMaxWeightValues = DL_MAX_WEIGHT_VALUES;
struct PhaseArgs {
    int32_t n;
    int32_t palette;                     // 0: direct, 1: palette
    uint16_t row_ptr[DL_MAX_NODES + 1];  // offsets relative to this phase
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
    };
};
static_assert(sizeof(PhaseArgs) <= 4096 - 128, "kernel-argument segment is 4 KiB");

enum Algo { ALGO_DECENTLAM = 0, ALGO_DMSGD = 1, ALGO_DSGD = 2, ALGO_DECENTLAM_XPREV = 3 };

int set_error(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
int check_hip(hipError_t e, const char* what);
void clear_error();

// Enqueue one fused iteration over columns [0, d) of x, m, g (already validated).
// `beta` is a double so that the momentum-free form can pass beta * gamma / gamma_prev unrounded.
int launch_step(Algo algo, float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
                const PhaseArgs& topo, float gamma, double beta, hipStream_t stream);

// Least-squares gradient (already validated).
size_t lsq_workspace_bytes(int32_t n, int32_t b, int64_t d);
// rows == nullptr: full-batch gradient over all b rows; otherwise bs sampled rows per node.
int launch_lsq(const float* A, const float* y, const float* x, float* g, float* loss, int32_t n,
               int32_t b, int64_t d, int64_t ldA, int64_t ld, const int32_t* rows, int32_t bs, float scale,
               void* workspace, hipStream_t stream);

// Diagnostics (already validated).
size_t stats_workspace_bytes(int64_t d);
int launch_stats(const float* x, const float* m, const float* ref, int32_t n, int64_t d, int64_t ld,
                 double* out, void* workspace, hipStream_t stream);

}  // namespace dl
