// Fused decentralized-update kernels for gfx950 (CDNA4).
//
// Mixing acts along the node axis only (matrix forms of Algorithms 1 and 2 in the
// appendix "Preliminary"), so every column of the stacked n x d arrays is an
// independent n-vector problem.  A workgroup owns a tile of TC = 64*VEC columns
// for ALL n rows:
//
//   phase 1  every wave streams whole rows of the tile (row index is wave-uniform):
//            x_j, g_j, m_j come in with VEC*4-byte loads, the local pre-step
//            (u_j = x_j - gamma g_j for DecentLaM, h_j = x_j - gamma (beta m_j + g_j)
//            for DmSGD) is evaluated in fp64 and parked in LDS as fp64;
//   phase 2  after one barrier, row i gathers its |N_i| neighbour rows from LDS
//            (weights and indices arrive through scalar loads from the kernel
//            arguments), finishes the update in fp64 and stores fp32 in place.
//
// HBM traffic is exactly read x, m, g + write x, m = 20 bytes per node-element,
// independent of the node degree; updating in place is race-free because no
// other workgroup touches these columns.
#include "internal.hpp"

namespace dl {
namespace {

constexpr int kWaves = 4;             // waves per workgroup
constexpr int kThreads = 64 * kWaves;

typedef float vf2 __attribute__((ext_vector_type(2)));
typedef float vf4 __attribute__((ext_vector_type(4)));

template <int VEC>
__device__ __forceinline__ void load_vec(const float* __restrict__ p, float (&v)[VEC]) {
    if constexpr (VEC == 4) {
        const vf4 t = *reinterpret_cast<const vf4*>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else if constexpr (VEC == 2) {
        const vf2 t = *reinterpret_cast<const vf2*>(p);
        v[0] = t.x; v[1] = t.y;
    } else {
        v[0] = *p;
    }
}

template <int VEC>
__device__ __forceinline__ void store_vec(float* __restrict__ p, const float (&v)[VEC]) {
    if constexpr (VEC == 4) {
        vf4 t; t.x = v[0]; t.y = v[1]; t.z = v[2]; t.w = v[3];
        *reinterpret_cast<vf4*>(p) = t;
    } else if constexpr (VEC == 2) {
        vf2 t; t.x = v[0]; t.y = v[1];
        *reinterpret_cast<vf2*>(p) = t;
    } else {
        *p = v[0];
    }
}

// VEC   columns per lane (width of the global accesses: 4, 8 or 16 bytes)
// RPT   rows per thread: the kernel covers n <= kWaves * RPT nodes
// ALGO  ALGO_DECENTLAM or ALGO_DMSGD
template <int VEC, int RPT, int ALGO>
__global__ __launch_bounds__(kThreads) void k_step(float* __restrict__ x, float* __restrict__ m,
                                                    const float* __restrict__ g, int64_t d, int64_t ld,
                                                    double gamma, double inv_gamma, double beta,
                                                    const PhaseArgs topo) {
    constexpr int TC = 64 * VEC;
    extern __shared__ double lds[];  // [n][TC]: u_j (DecentLaM) or h_j (DmSGD)

    const int n = topo.n;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t c = static_cast<int64_t>(blockIdx.x) * TC + lane * VEC;
    const bool live = c < d;  // d is a multiple of VEC for this launch

    float xr[RPT][VEC], mr[RPT][VEC], gr[RPT][VEC];

    // ---- phase 1: stream rows in, park the local pre-step in LDS
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int i = wave + kWaves * r;
        if (i < n && live) {
            const int64_t at = static_cast<int64_t>(i) * ld + c;
            load_vec<VEC>(x + at, xr[r]);
            load_vec<VEC>(g + at, gr[r]);
            load_vec<VEC>(m + at, mr[r]);
        }
    }
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int i = wave + kWaves * r;
        if (i < n && live) {
            double* slot = lds + i * TC + lane * VEC;
            if constexpr (ALGO == ALGO_DECENTLAM) {
#pragma unroll
                for (int v = 0; v < VEC; ++v)
                    slot[v] = static_cast<double>(xr[r][v]) - gamma * static_cast<double>(gr[r][v]);
            } else {
                float mn[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const double m_new = beta * static_cast<double>(mr[r][v]) + static_cast<double>(gr[r][v]);
                    mn[v] = static_cast<float>(m_new);
                    slot[v] = static_cast<double>(xr[r][v]) - gamma * m_new;
                }
                store_vec<VEC>(m + static_cast<int64_t>(i) * ld + c, mn);
            }
        }
    }
    __syncthreads();

    // ---- phase 2: gather-mix from LDS, finish the update, store in place
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int i = wave + kWaves * r;
        if (i < n && live) {
            double z[VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) z[v] = 0.0;
            const int e0 = topo.row_ptr[i], e1 = topo.row_ptr[i + 1];
            for (int e = e0; e < e1; ++e) {
                const double wij = static_cast<double>(topo.w[e]);
                const double* nb = lds + static_cast<int>(topo.col[e]) * TC + lane * VEC;
#pragma unroll
                for (int v = 0; v < VEC; ++v) z[v] = __builtin_fma(wij, nb[v], z[v]);
            }
            const int64_t at = static_cast<int64_t>(i) * ld + c;
            float xo[VEC];
            if constexpr (ALGO == ALGO_DECENTLAM) {
                float mo[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const double xi = static_cast<double>(xr[r][v]);
                    const double gt = (xi - z[v]) * inv_gamma;
                    const double m_new = __builtin_fma(beta, static_cast<double>(mr[r][v]), gt);
                    mo[v] = static_cast<float>(m_new);
                    xo[v] = static_cast<float>(xi - gamma * m_new);
                }
                store_vec<VEC>(m + at, mo);
            } else {
#pragma unroll
                for (int v = 0; v < VEC; ++v) xo[v] = static_cast<float>(z[v]);
            }
            store_vec<VEC>(x + at, xo);
        }
    }
}

template <int VEC, int RPT, int ALGO>
int launch_variant(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
                   const PhaseArgs& topo, double gamma, double beta, hipStream_t stream) {
    constexpr int TC = 64 * VEC;
    const size_t lds_bytes = static_cast<size_t>(n) * TC * sizeof(double);
    auto kernel = k_step<VEC, RPT, ALGO>;
    if (lds_bytes > 48 * 1024) {
        if (int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize,
                                                   static_cast<int>(lds_bytes)),
                               "hipFuncSetAttribute(max dynamic LDS)"))
            return rc;
    }
    const int64_t blocks = (d + TC - 1) / TC;
    if (blocks > 0x7fffffffLL) return set_error(DL_EINVAL, "step: d too large for one launch");
    hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), lds_bytes, stream, x,
                       m, g, d, ld, gamma, 1.0 / gamma, beta, topo);
    return check_hip(hipGetLastError(), "step kernel launch");
}

template <int VEC, int ALGO>
int launch_rows(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
                const PhaseArgs& topo, double gamma, double beta, hipStream_t stream) {
    const int rpt = (n + kWaves - 1) / kWaves;
    // widest_vec_for() keeps VEC * RPT <= 32 for VEC > 1, so wider variants are never built
#define DL_CASE(R)                                                                                 \
    if constexpr (VEC == 1 || VEC * R <= 32) {                                                               \
        if (rpt <= R) return launch_variant<VEC, R, ALGO>(x, m, g, n, d, ld, topo, gamma, beta, stream); \
    }
    DL_CASE(1) DL_CASE(2) DL_CASE(4) DL_CASE(8) DL_CASE(16) DL_CASE(32) DL_CASE(64)
#undef DL_CASE
    return set_error(DL_ETOPO, "step: n = %d has no kernel variant at vector width %d", n, VEC);
}

template <int ALGO>
int launch_cols(int vec, float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
                const PhaseArgs& topo, double gamma, double beta, hipStream_t stream) {
    if (d <= 0) return DL_OK;
    switch (vec) {
        case 4: return launch_rows<4, ALGO>(x, m, g, n, d, ld, topo, gamma, beta, stream);
        case 2: return launch_rows<2, ALGO>(x, m, g, n, d, ld, topo, gamma, beta, stream);
        default: return launch_rows<1, ALGO>(x, m, g, n, d, ld, topo, gamma, beta, stream);
    }
}

// Widest access for which the fp64 tile of n rows fits a 64 KiB LDS share (two workgroups per CU).
int widest_vec_for(int32_t n) {
    if (n <= 32) return 4;
    if (n <= 64) return 2;
    return 1;
}

}  // namespace

int launch_step(Algo algo, float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
                const PhaseArgs& topo, float gamma_f, float beta_f, hipStream_t stream) {
    const double gamma = static_cast<double>(gamma_f), beta = static_cast<double>(beta_f);

    // Pick the widest access all three arrays can share: same misalignment (in elements)
    // modulo the vector width and a row stride that preserves it.
    int vec = widest_vec_for(n);
    int64_t head = 0;
    for (; vec > 1; vec >>= 1) {
        const uintptr_t mask = static_cast<uintptr_t>(vec) - 1;
        const uintptr_t ax = (reinterpret_cast<uintptr_t>(x) >> 2) & mask;
        const uintptr_t am = (reinterpret_cast<uintptr_t>(m) >> 2) & mask;
        const uintptr_t ag = (reinterpret_cast<uintptr_t>(g) >> 2) & mask;
        if (ax == am && ax == ag && (ld & static_cast<int64_t>(mask)) == 0) {
            head = static_cast<int64_t>((vec - ax) & mask);
            break;
        }
    }
    if (vec == 1) head = 0;
    if (head > d) head = d;
    const int64_t body = ((d - head) / vec) * vec;
    const int64_t tail = d - head - body;

    auto run = [&](int v, int64_t c0, int64_t cols) {
        if (algo == ALGO_DECENTLAM)
            return launch_cols<ALGO_DECENTLAM>(v, x + c0, m + c0, g + c0, n, cols, ld, topo, gamma, beta, stream);
        return launch_cols<ALGO_DMSGD>(v, x + c0, m + c0, g + c0, n, cols, ld, topo, gamma, beta, stream);
    };
    if (int rc = run(vec, head, body)) return rc;   // aligned body first: it is the bulk
    if (int rc = run(1, 0, head)) return rc;        // columns are independent, so the peeled
    if (int rc = run(1, head + body, tail)) return rc;  // head and tail are separate launches
    return DL_OK;
}

}  // namespace dl
