// Diagnostics of the stacked state: consensus distance sum_i ||x_i - xbar||^2, ||xbar||^2,
// error against a reference vector (the relative-error metric of the appendix "Experimental
// setting for linear regression" is out[2] / (n * out[3])), and ||m||_F^2.
//
// HBM-bound, one pass: a thread owns VEC columns and walks down the n rows (a wave reads
// 64*VEC contiguous columns of one row per access; in large calls two runs of 128 columns 32 KiB
// apart, see SPLIT below).  Per column it keeps shifted sums around
// the first row's value p: s1 = sum_i (x_i - p), s2 = sum_i (x_i - p)^2, so that
// sum_i (x_i - xbar)^2 = s2 - s1^2 / n without the cancellation of the raw-moment formula.
// Partial sums go wave shuffle -> LDS -> one slot per workgroup; k_stats_finish adds the
// slots in a fixed order, so results are reproducible bit for bit.
#include <type_traits>

#include "internal.hpp"
#include "step_impl.hpp"

namespace dl {
namespace {

constexpr int kThreads = 256;
constexpr int kOut = 5;
constexpr int64_t kSplitMinColumns = 1 << 20;   // below this a call keeps the plain order (as the step kernel does)
constexpr int64_t kMaxBlocks = 32768;          // workgroups per launch (see blocks_for)
// partial sums in the workspace: [output][slot]; the launches of one call follow one another: the body (in the
// split order or not), a short plain launch for what precedes the first 64 KiB unit, the tail
constexpr int64_t kSlotPitch = 2 * kMaxBlocks + 64;
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
// Rows are taken ROWS at a time: all their loads go out before the first one is used (rows past the
// last are clamped to it for the load and skipped in the sums).
// SPLIT (VEC = 4, the first split_cols columns, a multiple of 16384, with x on a 64 KiB boundary): a wave's
// 256 columns are the two 512-byte segments 32 KiB apart of the step kernel's split tiles (step::split_column)
// instead of one run of 1 KiB: the order in which this GPU's memory streams at the same rate on every machine.
//
// Two shapes: 256 threads with 8 rows in flight, and for the launches over a million columns and more 1024 threads
// with 4 (the same bytes in flight per CU, a quarter of the workgroups and partial sums: 0.975 against 0.99 ms on
// 32 x 25.6 M).
template <int VEC, bool HAS_M, bool HAS_REF, bool SPLIT, int THREADS, int ROWS>
__global__ __launch_bounds__(THREADS) void k_stats(const float* __restrict__ x, const float* __restrict__ m,
                                                     const float* __restrict__ ref, int n, int64_t d,
                                                     int64_t ld, double* __restrict__ slots, int64_t split_cols) {
    __shared__ double red[THREADS / 64][kOut];
    double acc[kOut] = {0.0, 0.0, 0.0, 0.0, 0.0};
    // a workgroup walks over every gridDim.x-th block of THREADS * VEC columns: the number of
    // partial-sum slots stays small whatever d is, and the mapping is fixed, so sums are reproducible
    for (int64_t c0 = (static_cast<int64_t>(blockIdx.x) * THREADS + threadIdx.x) * VEC; c0 < d;
         c0 += static_cast<int64_t>(gridDim.x) * THREADS * VEC) {  // d is a multiple of VEC for this launch
        // SPLIT: the first split_cols columns (whole 64 KiB units) in the split order, the rest as they come
        const int64_t c = SPLIT && c0 < split_cols ? step::split_column(static_cast<uint32_t>(c0 >> 8), static_cast<int>(threadIdx.x & 63)) : c0;
        float pv[VEC], rv[VEC];
        load_cols<VEC>(x + c, pv);
        if constexpr (HAS_REF) load_cols<VEC>(ref + c, rv);
        double s1[VEC], s2[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) s1[v] = s2[v] = 0.0;
        for (int i0 = 0; i0 < n; i0 += ROWS) {
            float xv[ROWS][VEC], mv[ROWS][VEC];
#pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                const int64_t i = i0 + r < n ? i0 + r : n - 1;
                load_cols<VEC>(x + i * ld + c, xv[r]);
                if constexpr (HAS_M) load_cols<VEC>(m + i * ld + c, mv[r]);
            }
#pragma unroll
            for (int r = 0; r < ROWS; ++r) {
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
        double total = 0.0;
#pragma unroll
        for (int w = 0; w < THREADS / 64; w += 4) total += (red[w][q] + red[w + 1][q]) + (red[w + 2][q] + red[w + 3][q]);
        slots[q * kSlotPitch + blockIdx.x] = total;   // one array per output
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
// With few rows a block of columns is little work for the sums across the workgroup that end it: up to eight blocks
// per workgroup then, as long as 512 workgroups remain (4 nodes x 16.8 M columns: 105 -> 87 us).
int64_t blocks_for(int64_t cols, int vec, int threads, int n) {
    const int64_t one = static_cast<int64_t>(threads) * vec;
    int64_t blocks = (cols + one - 1) / one;
    int64_t share = n >= 24 ? 1 : n >= 12 ? 2 : n >= 6 ? 4 : 8;
    while (share > 1 && blocks / share < 512) share /= 2;
    blocks = (blocks + share - 1) / share;
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
    int64_t used = 0;   // slots handed out so far
    // columns [first, first + cols) in one launch; split: the first split_cols of them (a multiple of 16384) in the
    // split order
    auto launch = [&](auto vec_tag, auto split_tag, int64_t first, int64_t cols, int64_t split_cols) {
        constexpr int V = decltype(vec_tag)::value;
        constexpr bool S = decltype(split_tag)::value;
        const bool big = V == 4 && (S || cols >= kSplitMinColumns);   // every split launch is a big one
        const int64_t blocks = blocks_for(cols, V, big ? 1024 : kThreads, n);
        if (blocks == 0) return 0;
        const float* xp = x + first;
        const float* mp = m ? m + first : nullptr;
        const float* rp = ref ? ref + first : nullptr;
        double* out_slots = slots + used;
        used += blocks;
        const dim3 grid(static_cast<unsigned>(blocks));
        auto go = [&](auto has_m, auto has_ref) {
            constexpr bool M = decltype(has_m)::value, R = decltype(has_ref)::value;
            if constexpr (V == 4) {
                if (big) {
                    hipLaunchKernelGGL((k_stats<4, M, R, S, 1024, 4>), grid, dim3(1024), 0, stream, xp, mp, rp, n, cols, ld, out_slots, split_cols);
                    return;
                }
            }
            if constexpr (!S)   // the split order is for the big launches only
                hipLaunchKernelGGL((k_stats<V, M, R, false, kThreads, 8>), grid, dim3(kThreads), 0, stream, xp, mp, rp, n, cols, ld, out_slots, split_cols);
        };
        if (mp && rp) go(std::true_type(), std::true_type());
        else if (mp) go(std::true_type(), std::false_type());
        else if (rp) go(std::false_type(), std::true_type());
        else go(std::false_type(), std::false_type());
        return check_hip(hipGetLastError(), "stats kernel launch");
    };
    const std::integral_constant<int, 4> wide;
    const std::integral_constant<int, 1> narrow;
    // Large states whose rows share their offset inside a 128-byte line: the whole 64 KiB units of x go out in
    // the split order and the columns after them ride along in plain order (a launch of their own, eight
    // workgroups, took 11 us after the 1.04 ms of the units on 32 x 25.6 M); the columns before the first unit
    // are a launch of their own.
    int64_t pre = 0, units = 0;
    if (body >= kSplitMinColumns && ld % 32 == 0) {
        const uintptr_t at = reinterpret_cast<uintptr_t>(x) % (4u * step::kSplitUnit);
        pre = at ? static_cast<int64_t>((4u * step::kSplitUnit - at) / 4) : 0;
        units = (body - pre) / step::kSplitUnit;
    }
    if (units > 0) {
        if (int rc = launch(wide, std::true_type(), pre, body - pre, units * step::kSplitUnit)) return rc;
        if (int rc = launch(wide, std::false_type(), 0, pre, 0)) return rc;
    } else if (int rc = launch(wide, std::false_type(), 0, body, 0)) {
        return rc;
    }
    if (int rc = launch(narrow, std::false_type(), body, tail, 0)) return rc;
    hipLaunchKernelGGL(k_stats_finish, dim3(kOut), dim3(kFinishThreads), 0, stream, slots, used, out);
    return check_hip(hipGetLastError(), "stats finish kernel launch");
}

}  // namespace dl
