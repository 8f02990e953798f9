// Per-node least-squares gradient g_i = scale * A_i^T (A_i x_i - y_i) for gfx950.
//
// Every node has its own A_i and its own x_i, so this is a batch of n independent
// matrix-vector products with no shared operand: 1 flop per byte of A at best.
// The bound is HBM, and the kernels are organised around streaming A with wide
// coalesced loads; products are exact in fp64 (two fp32 factors) and sums are fp64.
//
//   k_residual   one wave per row r of A_i: res[i][r] = A_i[r,:] . x_i - y_i[r]
//                (lane-strided 16-byte loads, fp64 accumulators, wavefront-shuffle reduction)
//   k_transpose  one thread per 4 columns, one workgroup per (column block, row split, node):
//                partial[i][s][c] = sum_{r in split s} A_i[r,c] * res[i][r]
//   k_finish     g[i][c] = scale * sum_s partial[i][s][c] in fixed order (deterministic),
//                loss[i] = (scale/2) * sum_r res[i][r]^2
#include "internal.hpp"

namespace dl {
namespace {

constexpr int kThreads = 256;
typedef float vf4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Row splits of the transposed product: enough workgroups to fill 256 CUs several times over.
int row_splits(int32_t n, int32_t b, int64_t d) {
    const int64_t col_blocks = (d + 4 * kThreads - 1) / (4 * kThreads);
    int64_t s = (4096 + col_blocks * n - 1) / (col_blocks * n);
    if (s > b) s = b;
    if (s > 64) s = 64;
    if (s < 1) s = 1;
    return static_cast<int>(s);
}

template <bool VEC4>
__global__ __launch_bounds__(kThreads) void k_residual(const float* __restrict__ A,
                                                        const float* __restrict__ y,
                                                        const float* __restrict__ x,
                                                        double* __restrict__ res, int b, int64_t d,
                                                        int64_t ldA, int64_t ld) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i = blockIdx.y;
    const int r = blockIdx.x * (kThreads / 64) + wave;
    if (r >= b) return;
    const float* __restrict__ a = A + (static_cast<int64_t>(i) * b + r) * ldA;
    const float* __restrict__ xi = x + static_cast<int64_t>(i) * ld;
    double acc0 = 0.0, acc1 = 0.0, acc2 = 0.0, acc3 = 0.0;
    if constexpr (VEC4) {
        for (int64_t c = lane * 4; c < d; c += 256) {  // d % 4 == 0 here
            const vf4 av = *reinterpret_cast<const vf4*>(a + c);
            const vf4 xv = *reinterpret_cast<const vf4*>(xi + c);
            acc0 = __builtin_fma(static_cast<double>(av.x), static_cast<double>(xv.x), acc0);
            acc1 = __builtin_fma(static_cast<double>(av.y), static_cast<double>(xv.y), acc1);
            acc2 = __builtin_fma(static_cast<double>(av.z), static_cast<double>(xv.z), acc2);
            acc3 = __builtin_fma(static_cast<double>(av.w), static_cast<double>(xv.w), acc3);
        }
    } else {
        for (int64_t c = lane; c < d; c += 64)
            acc0 = __builtin_fma(static_cast<double>(a[c]), static_cast<double>(xi[c]), acc0);
    }
    const double dot = wave_sum((acc0 + acc1) + (acc2 + acc3));
    if (lane == 0) res[static_cast<int64_t>(i) * b + r] = dot - static_cast<double>(y[static_cast<int64_t>(i) * b + r]);
}

template <bool VEC4>
__global__ __launch_bounds__(kThreads) void k_transpose(const float* __restrict__ A,
                                                         const double* __restrict__ res,
                                                         double* __restrict__ partial, int b, int64_t d,
                                                         int64_t ldA, int splits) {
    constexpr int V = VEC4 ? 4 : 1;
    const int i = blockIdx.z, s = blockIdx.y;
    const int64_t c = (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x) * V;
    if (c >= d) return;
    const int r0 = static_cast<int>(static_cast<int64_t>(b) * s / splits);
    const int r1 = static_cast<int>(static_cast<int64_t>(b) * (s + 1) / splits);
    const float* __restrict__ a = A + static_cast<int64_t>(i) * b * ldA + c;
    const double* __restrict__ ri = res + static_cast<int64_t>(i) * b;
    double acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.0;
#pragma unroll 8
    for (int r = r0; r < r1; ++r) {
        const double rr = ri[r];
        if constexpr (VEC4) {
            const vf4 av = *reinterpret_cast<const vf4*>(a + static_cast<int64_t>(r) * ldA);
            acc[0] = __builtin_fma(static_cast<double>(av.x), rr, acc[0]);
            acc[1] = __builtin_fma(static_cast<double>(av.y), rr, acc[1]);
            acc[2] = __builtin_fma(static_cast<double>(av.z), rr, acc[2]);
            acc[3] = __builtin_fma(static_cast<double>(av.w), rr, acc[3]);
        } else {
            acc[0] = __builtin_fma(static_cast<double>(a[static_cast<int64_t>(r) * ldA]), rr, acc[0]);
        }
    }
    double* out = partial + (static_cast<int64_t>(i) * splits + s) * d + c;
#pragma unroll
    for (int v = 0; v < V; ++v) out[v] = acc[v];
}

__global__ __launch_bounds__(kThreads) void k_finish(const double* __restrict__ partial,
                                                      const double* __restrict__ res,
                                                      float* __restrict__ g, float* __restrict__ loss,
                                                      int b, int64_t d, int64_t ld, int splits,
                                                      double scale) {
    __shared__ double red[kThreads];
    const int i = blockIdx.y;
    const int64_t c = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (c < d) {
        const double* p = partial + static_cast<int64_t>(i) * splits * d + c;
        double acc = 0.0;
        for (int s = 0; s < splits; ++s) acc += p[static_cast<int64_t>(s) * d];
        g[static_cast<int64_t>(i) * ld + c] = static_cast<float>(scale * acc);
    }
    if (loss != nullptr && blockIdx.x == 0) {  // whole workgroup takes this branch together
        const double* ri = res + static_cast<int64_t>(i) * b;
        double sq = 0.0;
        for (int r = threadIdx.x; r < b; r += kThreads) sq = __builtin_fma(ri[r], ri[r], sq);
        red[threadIdx.x] = sq;
        __syncthreads();
        for (int half = kThreads / 2; half > 0; half >>= 1) {
            if (static_cast<int>(threadIdx.x) < half) red[threadIdx.x] += red[threadIdx.x + half];
            __syncthreads();
        }
        if (threadIdx.x == 0) loss[i] = static_cast<float>(0.5 * scale * red[0]);
    }
}

}  // namespace

size_t lsq_workspace_bytes(int32_t n, int32_t b, int64_t d) {
    const size_t res = static_cast<size_t>(n) * static_cast<size_t>(b);
    const size_t partial = static_cast<size_t>(n) * static_cast<size_t>(row_splits(n, b, d)) * static_cast<size_t>(d);
    return (res + partial) * sizeof(double) + 16;
}

int launch_lsq(const float* A, const float* y, const float* x, float* g, float* loss, int32_t n,
               int32_t b, int64_t d, int64_t ldA, int64_t ld, float scale, void* workspace,
               hipStream_t stream) {
    double* res = static_cast<double*>(workspace);
    double* partial = res + ((static_cast<size_t>(n) * b + 1) & ~size_t{1});  // keep 16-byte alignment
    const int splits = row_splits(n, b, d);
    const bool vec4 = d % 4 == 0 && ldA % 4 == 0 && ld % 4 == 0 &&
                      ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(x)) & 15u) == 0;
    if (n > 65535 || splits > 65535) return set_error(DL_EINVAL, "local_grad_lsq: n too large for the launch grid");

    const dim3 block(kThreads);
    const dim3 grid_r(static_cast<unsigned>((b + 3) / 4), static_cast<unsigned>(n));
    if (vec4)
        hipLaunchKernelGGL(k_residual<true>, grid_r, block, 0, stream, A, y, x, res, b, d, ldA, ld);
    else
        hipLaunchKernelGGL(k_residual<false>, grid_r, block, 0, stream, A, y, x, res, b, d, ldA, ld);
    if (int rc = check_hip(hipGetLastError(), "residual kernel launch")) return rc;

    if (d > 0) {
        const int V = vec4 ? 4 : 1;
        const dim3 grid_t(static_cast<unsigned>((d + static_cast<int64_t>(V) * kThreads - 1) / (static_cast<int64_t>(V) * kThreads)),
                          static_cast<unsigned>(splits), static_cast<unsigned>(n));
        if (vec4)
            hipLaunchKernelGGL(k_transpose<true>, grid_t, block, 0, stream, A, res, partial, b, d, ldA, splits);
        else
            hipLaunchKernelGGL(k_transpose<false>, grid_t, block, 0, stream, A, res, partial, b, d, ldA, splits);
        if (int rc = check_hip(hipGetLastError(), "transpose kernel launch")) return rc;
    }

    const dim3 grid_f(static_cast<unsigned>(d > 0 ? (d + kThreads - 1) / kThreads : 1), static_cast<unsigned>(n));
    hipLaunchKernelGGL(k_finish, grid_f, block, 0, stream, partial, res, g, loss, b, d, ld, splits,
                       static_cast<double>(scale));
    return check_hip(hipGetLastError(), "finish kernel launch");
}

}  // namespace dl
