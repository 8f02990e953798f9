// Internal declarations shared by the host boundary and the kernel launchers.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "decentlam.h"

namespace dl {

// One phase of W, small enough to travel in the kernel-argument segment, where a
// wavefront reads it with scalar loads (row index is wave-uniform).
struct PhaseArgs {
    int32_t n;
    uint16_t row_ptr[DL_MAX_NODES + 1];  // offsets relative to this phase
    uint8_t col[DL_MAX_NNZ];
    float w[DL_MAX_NNZ];
};
static_assert(sizeof(PhaseArgs) <= 3200, "kernel-argument segment is 4 KiB");

enum Algo { ALGO_DECENTLAM = 0, ALGO_DMSGD = 1, ALGO_DSGD = 2 };

int set_error(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
int check_hip(hipError_t e, const char* what);
void clear_error();

// Enqueue one fused iteration over columns [0, d) of x, m, g (already validated).
int launch_step(Algo algo, float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
                const PhaseArgs& topo, float gamma, float beta, hipStream_t stream);

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
