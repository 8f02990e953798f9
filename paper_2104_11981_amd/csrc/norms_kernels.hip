// Per-tensor sums of squares, final pass: adds the per-tile records the step launches wrote and sums
// the edge pieces of every tensor directly from the arrays (see NormPlan).
#include "device_util.hpp"
#include "internal.hpp"

namespace dl {

namespace {

using namespace dev;

// Small workgroups (most tensors are short and eight of these share a CU) with many loads in flight each
// (a long tensor is one workgroup's stream).  Measured on the 160-tensor ragged workload at 16 nodes:
// 256 threads x 8 records 26 us, x 4 records 28 us; 1024 threads x 4 records 43 us; records kept per tile
// instead of per node (strided reads) 59-75 us, though the step itself is then 1 % faster (a tile's
// records for all nodes are one contiguous write): 1.33 against 1.35 ms for step and final pass together.
constexpr int kFinishThreads = 256;
constexpr int kFinishUnroll = 8;
constexpr int kChunk = 440;   // tensors per final-pass launch (their offsets travel as kernel arguments)
struct OffsetChunk {
    int64_t v[kChunk + 1];    // column offsets relative to the first column of the step
};
struct FinishArgs {
    NormGrid grid[kMaxNormGrids];
    int grids;
};

// One workgroup per (tensor, node).  For every step launch ("grid" of tiles) the tensor's columns
// split into whole tiles, whose records the step launches wrote, and at most two edge pieces that
// share a tile with other tensors; the edge pieces are summed from g and from the m and x the step
// stored.  Fixed order of additions: same inputs, same bits.
template <int GF>
__global__ __launch_bounds__(kFinishThreads) void k_norms_finish(const float* __restrict__ x, const float* __restrict__ m,
                                                      const typename GradElem<GF>::type* __restrict__ g,
                                                      int64_t ld, int64_t ldg, int64_t bw, int n,
                                                      const double* __restrict__ partial, int64_t capacity,
                                                      double* __restrict__ norms, const FinishArgs fa,
                                                      const OffsetChunk chunk) {
    const int t = blockIdx.x, i = blockIdx.y;
    const int64_t lo = chunk.v[t], hi = chunk.v[t + 1];
    double s[3] = {0.0, 0.0, 0.0};
    auto columns = [&](int64_t a, int64_t b) {   // element-wise over [a, b)
        for (int64_t c = a + threadIdx.x; c < b; c += kFinishThreads) {
            // element (i, c): row-major i * ld + c, blocked ((c / bw) * n + i) * bw + c % bw
            const int64_t blk = bw > 0 ? c / bw : 0;
            const int64_t at = bw > 0 ? (blk * n + i) * bw + (c - blk * bw) : static_cast<int64_t>(i) * ld + c;
            const int64_t at_g = bw > 0 ? at : static_cast<int64_t>(i) * ldg + c;
            float gv[1];
            load_grad<1, GF>(g + at_g, gv);
            const double g1 = static_cast<double>(gv[0]);
            const double m1 = static_cast<double>(m[at]);
            const double x1 = static_cast<double>(x[at]);
            s[0] = __builtin_fma(g1, g1, s[0]);
            s[1] = __builtin_fma(m1, m1, s[1]);
            s[2] = __builtin_fma(x1, x1, s[2]);
        }
    };
    for (int k = 0; k < fa.grids; ++k) {
        const NormGrid gd = fa.grid[k];
        const int64_t a = lo > gd.col0 ? lo : gd.col0;                          // the tensor inside this grid
        const int64_t b = hi < gd.col0 + gd.cols ? hi : gd.col0 + gd.cols;
        if (a >= b) continue;
        const int64_t tiles = (gd.cols + gd.tc - 1) / gd.tc;
        const int64_t b0 = (a - gd.col0 + gd.tc - 1) / gd.tc;                   // first tile that starts at or after a
        const int64_t b1 = b == gd.col0 + gd.cols ? tiles : (b - gd.col0) / gd.tc;  // tiles [b0, b1) lie inside [a, b)
        if (b0 >= b1) {
            columns(a, b);
            continue;
        }
        columns(a, gd.col0 + b0 * gd.tc);
        const int64_t tail = gd.col0 + b1 * gd.tc;
        if (tail < b) columns(tail, b);
        // this node's records of the launch are consecutive; kFinishUnroll per thread in flight
        const double* mine = partial + (static_cast<int64_t>(i) * capacity + gd.tile0) * 3;
        int64_t q = b0 + threadIdx.x;
        for (; q + (kFinishUnroll - 1) * kFinishThreads < b1; q += kFinishUnroll * kFinishThreads) {
            double r[kFinishUnroll][3];
#pragma unroll
            for (int u = 0; u < kFinishUnroll; ++u) {
#pragma unroll
                for (int v = 0; v < 3; ++v) r[u][v] = mine[(q + u * kFinishThreads) * 3 + v];
            }
#pragma unroll
            for (int u = 0; u < kFinishUnroll; ++u) {   // same order of additions as one record at a time
                s[0] += r[u][0]; s[1] += r[u][1]; s[2] += r[u][2];
            }
        }
        for (; q < b1; q += kFinishThreads) {
            const double* rec = mine + q * 3;
            s[0] += rec[0]; s[1] += rec[1]; s[2] += rec[2];
        }
    }
    __shared__ double red[3][kFinishThreads];
#pragma unroll
    for (int q = 0; q < 3; ++q) red[q][threadIdx.x] = s[q];
    __syncthreads();
    for (int half = kFinishThreads / 2; half >= 1; half >>= 1) {
        if (static_cast<int>(threadIdx.x) < half) {
#pragma unroll
            for (int q = 0; q < 3; ++q) red[q][threadIdx.x] += red[q][threadIdx.x + half];
        }
        __syncthreads();
    }
    if (threadIdx.x < 3) norms[(static_cast<int64_t>(t) * n + i) * 3 + threadIdx.x] = red[threadIdx.x][0];
}

template <int GF>
int finish_chunks(const NormPlan& plan, const float* x, const float* m, const void* g, int64_t ld, int64_t ldg,
                  int32_t n, hipStream_t stream) {
    FinishArgs fa;
    fa.grids = plan.grids;
    for (int k = 0; k < kMaxNormGrids; ++k) fa.grid[k] = k < plan.grids ? plan.grid[k] : NormGrid{0, 0, 0, 64};
    for (int32_t t0 = 0; t0 < plan.num_tensors; t0 += kChunk) {
        const int32_t count = plan.num_tensors - t0 < kChunk ? plan.num_tensors - t0 : kChunk;
        OffsetChunk chunk;
        for (int j = 0; j <= kChunk; ++j)
            chunk.v[j] = plan.offsets[t0 + (j <= count ? j : count)] - plan.offsets[0];
        hipLaunchKernelGGL(k_norms_finish<GF>, dim3(static_cast<unsigned>(count), static_cast<unsigned>(n)),
                           dim3(kFinishThreads), 0, stream, x, m, static_cast<const typename GradElem<GF>::type*>(g), ld, ldg,
                           plan.bw, n, plan.partial, plan.capacity, plan.norms + static_cast<int64_t>(t0) * n * 3, fa,
                           chunk);
        if (int rc = check_hip(hipGetLastError(), "per-tensor sums, final pass")) return rc;
    }
    return DL_OK;
}

}  // namespace

int launch_norms_finish(const NormPlan& plan, const float* x, const float* m, GradArg g, int64_t ld, int32_t n,
                        hipStream_t stream) {
    if (g.format == DL_GRAD_BF16) return finish_chunks<DL_GRAD_BF16>(plan, x, m, g.p, ld, g.ld, n, stream);
    if (g.format == DL_GRAD_F16) return finish_chunks<DL_GRAD_F16>(plan, x, m, g.p, ld, g.ld, n, stream);
    return finish_chunks<DL_GRAD_F32>(plan, x, m, g.p, ld, g.ld, n, stream);
}

}  // namespace dl
