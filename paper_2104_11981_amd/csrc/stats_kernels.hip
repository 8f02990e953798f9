// Diagnostics of the stacked state: consensus distance sum_i ||x_i - xbar||^2, ||xbar||^2,
// error against a reference vector (the relative-error metric of the appendix "Experimental
// setting for linear regression" is out[2] / (n * out[3])), and ||m||_F^2.
//
// HBM-bound, one pass: a thread owns VEC columns and walks down the n rows (a wave reads
// 64*VEC contiguous columns of one row per access).  Per column it keeps shifted sums around
// the first row's value p: s1 = sum_i (x_i - p), s2 = sum_i (x_i - p)^2, so that
// sum_i (x_i - xbar)^2 = s2 - s1^2 / n without the cancellation of the raw-moment formula.
// Partial sums go wave shuffle -> LDS -> one slot per workgroup; k_stats_finish adds the
// slots in a fixed order, so results are reproducible bit for bit.
#include <type_traits>

#include "internal.hpp"

namespace dl {
namespace {

constexpr int kThreads = 256;
constexpr int kOut = 5;
constexpr int64_t kMaxBlocks = 32768;          // workgroups per launch (see blocks_for)
constexpr int64_t kSlotPitch = 2 * kMaxBlocks;  // partial sums in the workspace: [output][slot], body launch then tail launch
typedef float vf4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

template <int VEC>
__device__ __forceinline__ void load_cols(const float* __restrict__ p, float (&v)[VEC]) {
    if constexpr (VEC == 4) {
        const vf4 t = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(p));   // streamed once
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        v[0] = __builtin_nontemporal_load(p);
    }
}

// HAS_M, HAS_REF: whether m and ref are given (compile-time, so that no load sits behind a test).
// Rows are taken kRows at a time: all their loads go out before the first one is used (rows past the
// last are clamped to it for the load and skipped in the sums).
constexpr int kRows = 8;
template <int VEC, bool HAS_M, bool HAS_REF>
__global__ __launch_bounds__(kThreads) void k_stats(const float* __restrict__ x, const float* __restrict__ m,
                                                     const float* __restrict__ ref, int n, int64_t d,
                                                     int64_t ld, double* __restrict__ slots) {
    __shared__ double red[kThreads / 64][kOut];
    double acc[kOut] = {0.0, 0.0, 0.0, 0.0, 0.0};
    // a workgroup walks over every gridDim.x-th block of kThreads * VEC columns: the number of
    // partial-sum slots stays small whatever d is, and the mapping is fixed, so sums are reproducible
    for (int64_t c = (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x) * VEC; c < d;
         c += static_cast<int64_t>(gridDim.x) * kThreads * VEC) {  // d is a multiple of VEC for this launch
        float pv[VEC], rv[VEC];
        load_cols<VEC>(x + c, pv);
        if constexpr (HAS_REF) load_cols<VEC>(ref + c, rv);
        double s1[VEC], s2[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) s1[v] = s2[v] = 0.0;
        for (int i0 = 0; i0 < n; i0 += kRows) {
            float xv[kRows][VEC], mv[kRows][VEC];
#pragma unroll
            for (int r = 0; r < kRows; ++r) {
                const int64_t i = i0 + r < n ? i0 + r : n - 1;
                load_cols<VEC>(x + i * ld + c, xv[r]);
                if constexpr (HAS_M) load_cols<VEC>(m + i * ld + c, mv[r]);
            }
#pragma unroll
            for (int r = 0; r < kRows; ++r) {
                if (i0 + r < n) {   // uniform
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        const double dev = static_cast<double>(xv[r][v]) - static_cast<double>(pv[v]);
                        s1[v] += dev;
                        s2[v] = __builtin_fma(dev, dev, s2[v]);
                        if constexpr (HAS_REF) {
                            const double e = static_cast<double>(xv[r][v]) - static_cast<double>(rv[v]);
                            acc[2] = __builtin_fma(e, e, acc[2]);
                        }
                    }
                    if constexpr (HAS_M) {
#pragma unroll
                        for (int v = 0; v < VEC; ++v)
                            acc[4] = __builtin_fma(static_cast<double>(mv[r][v]), static_cast<double>(mv[r][v]), acc[4]);
                    }
                }
            }
        }
        const double inv_n = 1.0 / static_cast<double>(n);
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            acc[0] += s2[v] - s1[v] * s1[v] * inv_n;
            const double mean = static_cast<double>(pv[v]) + s1[v] * inv_n;
            acc[1] = __builtin_fma(mean, mean, acc[1]);
            if constexpr (HAS_REF) acc[3] = __builtin_fma(static_cast<double>(rv[v]), static_cast<double>(rv[v]), acc[3]);
        }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int q = 0; q < kOut; ++q) {
        const double s = wave_sum(acc[q]);
        if (lane == 0) red[wave][q] = s;
    }
    __syncthreads();
    if (threadIdx.x < kOut) {
        const int q = threadIdx.x;
        slots[q * kSlotPitch + blockIdx.x] = (red[0][q] + red[1][q]) + (red[2][q] + red[3][q]);   // one array per output
    }
}

// One workgroup per output adds that output's slots in a fixed order: four slots per thread in flight,
// then wave shuffles, then the sixteen wave sums.
constexpr int kFinishThreads = 1024;
__global__ __launch_bounds__(kFinishThreads) void k_stats_finish(const double* __restrict__ slots, int64_t count,
                                                                  double* __restrict__ out) {
    __shared__ double red[kFinishThreads / 64];
    const double* mine = slots + blockIdx.x * kSlotPitch;
    double acc = 0.0;
    int64_t s = threadIdx.x;
    for (; s + 3 * kFinishThreads < count; s += 4 * kFinishThreads) {
        double v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = mine[s + u * kFinishThreads];
#pragma unroll
        for (int u = 0; u < 4; ++u) acc += v[u];
    }
    for (; s < count; s += kFinishThreads) acc += mine[s];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const double w = wave_sum(acc);
    if (lane == 0) red[wave] = w;
    __syncthreads();
    if (threadIdx.x == 0) {
        double total = 0.0;
        for (int k = 0; k < kFinishThreads / 64; ++k) total += red[k];
        out[blockIdx.x] = total;
    }
}

// Many more workgroups than fit the chip at once, each with one block of columns while d allows: with
// 8192 workgroups of three or four blocks each (25.6 M columns) the last of them ran on a nearly empty
// chip and the kernel took 1.07 instead of 1.01 ms.
int64_t blocks_for(int64_t cols, int vec) {
    const int64_t blocks = (cols + static_cast<int64_t>(kThreads) * vec - 1) / (static_cast<int64_t>(kThreads) * vec);
    return blocks < kMaxBlocks ? blocks : kMaxBlocks;
}

}  // namespace

size_t stats_workspace_bytes(int64_t d) {
    (void)d;   // the launches are capped at kMaxBlocks workgroups each, whatever d
    return static_cast<size_t>(kSlotPitch) * kOut * sizeof(double);
}

int launch_stats(const float* x, const float* m, const float* ref, int32_t n, int64_t d, int64_t ld,
                 double* out, void* workspace, hipStream_t stream) {
    double* slots = static_cast<double*>(workspace);
    const bool vec4 = (ld % 4 == 0) && ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(m) |
                                          reinterpret_cast<uintptr_t>(ref)) & 15u) == 0;
    const int64_t body = vec4 ? (d / 4) * 4 : 0;
    const int64_t tail = d - body;
    const int64_t nb_body = blocks_for(body, 4), nb_tail = blocks_for(tail, 1);
    auto launch = [&](auto vec_tag, int64_t blocks, const float* xp, const float* mp, const float* rp, int64_t cols,
                      double* out_slots) {
        constexpr int V = decltype(vec_tag)::value;
        const dim3 grid(static_cast<unsigned>(blocks)), block(kThreads);
        if (mp && rp) hipLaunchKernelGGL((k_stats<V, true, true>), grid, block, 0, stream, xp, mp, rp, n, cols, ld, out_slots);
        else if (mp) hipLaunchKernelGGL((k_stats<V, true, false>), grid, block, 0, stream, xp, mp, rp, n, cols, ld, out_slots);
        else if (rp) hipLaunchKernelGGL((k_stats<V, false, true>), grid, block, 0, stream, xp, mp, rp, n, cols, ld, out_slots);
        else hipLaunchKernelGGL((k_stats<V, false, false>), grid, block, 0, stream, xp, mp, rp, n, cols, ld, out_slots);
        return check_hip(hipGetLastError(), "stats kernel launch");
    };
    if (nb_body > 0) {
        if (int rc = launch(std::integral_constant<int, 4>(), nb_body, x, m, ref, body, slots)) return rc;
    }
    if (nb_tail > 0) {
        if (int rc = launch(std::integral_constant<int, 1>(), nb_tail, x + body, m ? m + body : nullptr,
                            ref ? ref + body : nullptr, tail, slots + nb_body))
            return rc;
    }
    hipLaunchKernelGGL(k_stats_finish, dim3(kOut), dim3(kFinishThreads), 0, stream, slots, nb_body + nb_tail, out);
    return check_hip(hipGetLastError(), "stats finish kernel launch");
}

}  // namespace dl
