// The step for graphs that do not travel in kernel arguments: up to 1024 nodes, neighbour lists of any
// length with arbitrary weights, read from device memory (topology_pack_device).
//
// Same plan as k_step -- a workgroup owns a tile of columns for ALL n rows, parks the local pre-step in LDS as
// fp64, meets at one barrier, gathers, finishes in fp64, rounds once, stores in place: 20 bytes per
// node-element, race-free because no other workgroup touches these columns -- but built for reach, not for
// speed: the fp64 tile of n rows must fit 128 KiB of LDS, so a tile is 64 columns up to 256 nodes, 32 up to 512
// and 16 up to 1024 (rows of 256, 128 and 64 bytes per access: far from what the memory likes), 1024 threads
// take 1024 / TC rows at a time with up to 16 rows per thread, and every thread walks its rows' lists
// straight from device memory (row offsets and (column, weight) pairs; the lanes of a row read the same
// words).  Graphs that fit the kernel-argument encodings should use the ordinary calls.
#include "internal.hpp"

namespace dl {
namespace {

constexpr int kThreads = 1024;
constexpr int kRowsPerThread = 16;   // n * TC <= 16384

template <int ALGO, int TC>
__global__ __launch_bounds__(kThreads) void k_step_wide(float* __restrict__ x, float* __restrict__ m,
                                                         const float* __restrict__ g, int n, int64_t d, int64_t ld,
                                                         double gamma, double inv_gamma, double beta,
                                                         const uint32_t* __restrict__ topo, int phase) {
    extern __shared__ __attribute__((aligned(16))) double tile[];   // [n][TC]
    constexpr int RG = kThreads / TC;
    const int col = threadIdx.x % TC, rg = threadIdx.x / TC;
    const int64_t c = static_cast<int64_t>(blockIdx.x) * TC + col;
    const bool live = c < d;
    const uint32_t* ph = topo + topo[kDeviceTopoHeaderWords + phase];
    const uint32_t* row_ptr = ph;
    const uint2* entries = reinterpret_cast<const uint2*>(ph + device_topo_row_ptr_words(n));

    float xr[kRowsPerThread], mr[kRowsPerThread];
#pragma unroll
    for (int r = 0; r < kRowsPerThread; ++r) {
        const int i = rg + r * RG;
        xr[r] = mr[r] = 0.f;
        if (i < n) {
            float gv = 0.f;
            if (live) {
                const int64_t at = static_cast<int64_t>(i) * ld + c;
                xr[r] = __builtin_nontemporal_load(x + at);
                gv = __builtin_nontemporal_load(g + at);
                if constexpr (ALGO != ALGO_DSGD) mr[r] = __builtin_nontemporal_load(m + at);
            }
            double u;
            if constexpr (ALGO == ALGO_DMSGD) {
                const double m_new = beta * static_cast<double>(mr[r]) + static_cast<double>(gv);
                mr[r] = static_cast<float>(m_new);
                u = static_cast<double>(xr[r]) - gamma * m_new;
            } else {
                u = static_cast<double>(xr[r]) - gamma * static_cast<double>(gv);
            }
            tile[i * TC + col] = u;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRowsPerThread; ++r) {
        const int i = rg + r * RG;
        if (i < n) {
            double z = 0.0;
            const uint32_t e1 = row_ptr[i + 1];
            for (uint32_t e = row_ptr[i]; e < e1; ++e) {   // list order, one fused multiply-add per term
                const uint2 en = entries[e];
                z = __builtin_fma(static_cast<double>(__builtin_bit_cast(float, en.y)), tile[en.x * TC + col], z);
            }
            if (live) {
                const int64_t at = static_cast<int64_t>(i) * ld + c;
                if constexpr (ALGO == ALGO_DECENTLAM) {
                    const double xi = static_cast<double>(xr[r]);
                    const double gt = (xi - z) * inv_gamma;
                    const double m_new = __builtin_fma(beta, static_cast<double>(mr[r]), gt);
                    const float m_out = static_cast<float>(m_new);
                    __builtin_nontemporal_store(m_out, m + at);
                    __builtin_nontemporal_store(static_cast<float>(xi - gamma * m_new), x + at);
                } else {
                    if constexpr (ALGO == ALGO_DMSGD) __builtin_nontemporal_store(mr[r], m + at);
                    __builtin_nontemporal_store(static_cast<float>(z), x + at);
                }
            }
        }
    }
}

template <int ALGO, int TC>
int launch_tc(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld, double gamma, double beta,
              const uint32_t* topo, int phase, hipStream_t stream) {
    const size_t lds_bytes = static_cast<size_t>(n) * TC * sizeof(double);
    auto kernel = k_step_wide<ALGO, TC>;
    if (lds_bytes > 48 * 1024) {   // a driver attribute, set at every launch: no state is kept for this path
        if (int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024),
                               "hipFuncSetAttribute(max dynamic LDS)"))
            return rc;
    }
    const int64_t blocks = (d + TC - 1) / TC;
    if (blocks > 0x7fffffffLL) return set_error(DL_EINVAL, "step: d too large for one launch");
    hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), lds_bytes, stream, x, m, g, n, d, ld,
                       gamma, 1.0 / gamma, beta, topo, phase);
    return check_hip(hipGetLastError(), "step kernel launch (device-resident lists)");
}

template <int ALGO>
int launch_algo(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld, double gamma, double beta,
                const uint32_t* topo, int phase, hipStream_t stream) {
    if (n <= 256) return launch_tc<ALGO, 64>(x, m, g, n, d, ld, gamma, beta, topo, phase, stream);
    if (n <= 512) return launch_tc<ALGO, 32>(x, m, g, n, d, ld, gamma, beta, topo, phase, stream);
    return launch_tc<ALGO, 16>(x, m, g, n, d, ld, gamma, beta, topo, phase, stream);
}

}  // namespace

int launch_step_wide(Algo algo, float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld, float gamma,
                     double beta, const void* device_topology, int32_t phase, hipStream_t stream) {
    if (d <= 0) return DL_OK;
    if (n > DL_MAX_NODES_DEVICE) return set_error(DL_ETOPO, "step: n = %d exceeds DL_MAX_NODES_DEVICE = %d", n, DL_MAX_NODES_DEVICE);
    const uint32_t* topo = static_cast<const uint32_t*>(device_topology);
    const double gm = static_cast<double>(gamma);
    switch (algo) {
        case ALGO_DECENTLAM: return launch_algo<ALGO_DECENTLAM>(x, m, g, n, d, ld, gm, beta, topo, phase, stream);
        case ALGO_DMSGD: return launch_algo<ALGO_DMSGD>(x, m, g, n, d, ld, gm, beta, topo, phase, stream);
        case ALGO_DSGD: return launch_algo<ALGO_DSGD>(x, m, g, n, d, ld, gm, beta, topo, phase, stream);
        default: return set_error(DL_EINVAL, "step: this method has no kernel for device-resident lists");
    }
}

}  // namespace dl
