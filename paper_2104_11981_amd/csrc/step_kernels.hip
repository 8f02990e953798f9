// Fused decentralized-update kernels for gfx950 (CDNA4).
//
// Mixing acts along the node axis only (matrix forms of Algorithms 1 and 2 in the
// appendix "Preliminary"), so every column of the stacked n x d arrays is an
// independent n-vector problem.  A workgroup of WAVES wavefronts owns a tile of
// TC = 64*VEC columns for ALL n rows:
//
//   phase 1  every wave streams whole rows of the tile (row index is wave-uniform):
//            x_j, g_j, m_j come in with VEC*4-byte non-temporal loads, the local
//            pre-step (u_j = x_j - gamma g_j for DecentLaM, h_j = x_j - gamma (beta m_j + g_j)
//            for DmSGD) is evaluated in fp64 and parked in LDS as fp64; meanwhile the
//            neighbour list of W is unpacked from the kernel arguments into an LDS
//            table of (fp64 weight, LDS row offset) pairs;
//   phase 2  after one barrier, row i gathers its |N_i| neighbour rows from LDS in
//            list order, a few neighbours at a time so that the table and tile reads of
//            a group are in flight together, finishes the update in
//            fp64 and stores fp32 in place with non-temporal stores.
//
// HBM traffic is exactly read x, m, g + write x, m = 20 bytes per node-element,
// independent of the node degree; updating in place is race-free because no
// other workgroup touches these columns.  The gather costs no time next to the
// streaming (measured: replacing it by a copy of the own row does not speed the
// kernel up), and the non-temporal accesses are worth about 5 %.
#include "internal.hpp"

namespace dl {
namespace {

typedef float vf2 __attribute__((ext_vector_type(2)));
typedef float vf4 __attribute__((ext_vector_type(4)));

// Streaming accesses: every byte is touched once per launch, so mark them non-temporal.
template <int VEC>
__device__ __forceinline__ void load_vec(const float* __restrict__ p, float (&v)[VEC]) {
    if constexpr (VEC == 4) {
        const vf4 t = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(p));
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else if constexpr (VEC == 2) {
        const vf2 t = __builtin_nontemporal_load(reinterpret_cast<const vf2*>(p));
        v[0] = t.x; v[1] = t.y;
    } else {
        v[0] = __builtin_nontemporal_load(p);
    }
}

template <int VEC>
__device__ __forceinline__ void store_vec(float* __restrict__ p, const float (&v)[VEC]) {
    if constexpr (VEC == 4) {
        vf4 t; t.x = v[0]; t.y = v[1]; t.z = v[2]; t.w = v[3];
        __builtin_nontemporal_store(t, reinterpret_cast<vf4*>(p));
    } else if constexpr (VEC == 2) {
        vf2 t; t.x = v[0]; t.y = v[1];
        __builtin_nontemporal_store(t, reinterpret_cast<vf2*>(p));
    } else {
        __builtin_nontemporal_store(v[0], p);
    }
}

// One neighbour in the LDS table.
struct alignas(16) Neighbour {
    double w;     // w_ij, promoted exactly from fp32
    int offset;   // j * TC: start of row j in the LDS tile, in doubles
    int unused;
};

// z += sum over K consecutive table entries; all K table reads, then all K tile reads, are
// issued before the first multiply-add so their latencies overlap.
template <int VEC, int K>
__device__ __forceinline__ void gather(const Neighbour* __restrict__ entry, const double* __restrict__ tile_at_lane,
                                       double (&z)[VEC]) {
    Neighbour nb[K];
#pragma unroll
    for (int t = 0; t < K; ++t) nb[t] = entry[t];
    double u[K][VEC];
#pragma unroll
    for (int t = 0; t < K; ++t) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) u[t][v] = tile_at_lane[nb[t].offset + v];
    }
#pragma unroll
    for (int t = 0; t < K; ++t) {   // list order, one fused multiply-add per term
#pragma unroll
        for (int v = 0; v < VEC; ++v) z[v] = __builtin_fma(nb[t].w, u[t][v], z[v]);
    }
}

// VEC    columns per lane (width of the global accesses: 4, 8 or 16 bytes)
// RPT    rows per thread; WAVES wavefronts per workgroup: the kernel covers n <= WAVES * RPT nodes
// ALGO   ALGO_DECENTLAM, ALGO_DMSGD, ALGO_DSGD (x <- W (x - gamma g); m is not touched) or
//        ALGO_DECENTLAM_XPREV: DecentLaM in its momentum-free form (appendix "Reformulation of
//        DecentLaM"), x_next = W (x - gamma g) + beta' (x - x_prev); here `m` is the buffer that
//        holds x_prev on entry and x_next on exit, x is only read, and `beta` carries
//        beta' = beta * gamma / gamma_prev: 16 bytes per node-element, one written array
template <int VEC, int RPT, int WAVES, int ALGO>
__global__ __launch_bounds__(64 * WAVES) void k_step(float* __restrict__ x, float* __restrict__ m,
                                                      const float* __restrict__ g, int64_t d, int64_t ld,
                                                      double gamma, double inv_gamma, double beta,
                                                      const PhaseArgs topo) {
    constexpr int TC = 64 * VEC;
    extern __shared__ double lds[];  // tile [n][TC] of u_j (DecentLaM) or h_j (DmSGD), then the table
    const int n = topo.n;
    Neighbour* table = reinterpret_cast<Neighbour*>(lds + n * TC);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t c = static_cast<int64_t>(blockIdx.x) * TC + lane * VEC;
    const bool live = c < d;  // d is a multiple of VEC for this launch

    // ---- phase 1: stream rows in
    float xr[RPT][VEC], mr[RPT][VEC], gr[RPT][VEC];
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int i = wave + WAVES * r;
        if (i < n && live) {
            const int64_t at = static_cast<int64_t>(i) * ld + c;
            load_vec<VEC>(x + at, xr[r]);
            load_vec<VEC>(g + at, gr[r]);
            if constexpr (ALGO != ALGO_DSGD) load_vec<VEC>(m + at, mr[r]);
        }
    }
    // neighbour list: kernel arguments -> LDS table (one entry per thread and round)
    const int nnz = topo.row_ptr[n];
    for (int e = threadIdx.x; e < nnz; e += 64 * WAVES) {
        Neighbour t;
        if (topo.palette) {  // uniform over the grid
            t.w = static_cast<double>(topo.pal.value[topo.pal.widx[e]]);
            t.offset = static_cast<int>(topo.pal.col[e]) * TC;
        } else {
            t.w = static_cast<double>(topo.direct.w[e]);
            t.offset = static_cast<int>(topo.direct.col[e]) * TC;
        }
        t.unused = 0;
        table[e] = t;
    }
    // local pre-step, parked in LDS
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int i = wave + WAVES * r;
        if (i < n && live) {
            double* slot = lds + i * TC + lane * VEC;
            if constexpr (ALGO != ALGO_DMSGD) {
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
    const double* tile_at_lane = lds + lane * VEC;
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int i = wave + WAVES * r;
        if (i < n && live) {
            double z[VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) z[v] = 0.0;
            int e = topo.row_ptr[i];
            const int e1 = topo.row_ptr[i + 1];
            // groups of 4 (2 for 16-byte lanes: eight fp64 values in flight keep the kernel at
            // 64 VGPRs, i.e. two 1024-thread workgroups per CU), then 2, then 1
            if constexpr (VEC < 4) {
                for (; e + 4 <= e1; e += 4) gather<VEC, 4>(table + e, tile_at_lane, z);
                if (e + 2 <= e1) {
                    gather<VEC, 2>(table + e, tile_at_lane, z);
                    e += 2;
                }
            } else {
                for (; e + 2 <= e1; e += 2) gather<VEC, 2>(table + e, tile_at_lane, z);
            }
            if (e < e1) gather<VEC, 1>(table + e, tile_at_lane, z);

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
            } else if constexpr (ALGO == ALGO_DECENTLAM_XPREV) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const double diff = static_cast<double>(xr[r][v]) - static_cast<double>(mr[r][v]);
                    xo[v] = static_cast<float>(__builtin_fma(beta, diff, z[v]));
                }
            } else {
#pragma unroll
                for (int v = 0; v < VEC; ++v) xo[v] = static_cast<float>(z[v]);
            }
            store_vec<VEC>((ALGO == ALGO_DECENTLAM_XPREV ? m : x) + at, xo);
        }
    }
}

size_t lds_bytes_for(int32_t n, int vec, int nnz) {
    return static_cast<size_t>(n) * 64 * vec * sizeof(double) + static_cast<size_t>(nnz) * sizeof(Neighbour);
}

template <int VEC, int RPT, int WAVES, int ALGO>
int launch_variant(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
                   const PhaseArgs& topo, double gamma, double beta, hipStream_t stream) {
    constexpr int TC = 64 * VEC;
    const size_t lds_bytes = lds_bytes_for(n, VEC, topo.row_ptr[n]);
    auto kernel = k_step<VEC, RPT, WAVES, ALGO>;
    if (lds_bytes > 48 * 1024) {
        if (int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize,
                                                   static_cast<int>(lds_bytes)),
                               "hipFuncSetAttribute(max dynamic LDS)"))
            return rc;
    }
    const int64_t blocks = (d + TC - 1) / TC;
    if (blocks > 0x7fffffffLL) return set_error(DL_EINVAL, "step: d too large for one launch");
    hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(blocks)), dim3(64 * WAVES), lds_bytes, stream,
                       x, m, g, d, ld, gamma, 1.0 / gamma, beta, topo);
    return check_hip(hipGetLastError(), "step kernel launch");
}

// Workgroup shape by node count: as many waves as rows up to 16, then more rows per thread.
template <int VEC, int ALGO>
int launch_rows(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
                const PhaseArgs& topo, double gamma, double beta, hipStream_t stream) {
#define DL_SHAPE(MAXN, W, R)                                                                        \
    if constexpr (VEC == 1 || VEC * (MAXN) <= 128) {                                                \
        if (n <= (MAXN)) return launch_variant<VEC, R, W, ALGO>(x, m, g, n, d, ld, topo, gamma, beta, stream); \
    }
    DL_SHAPE(4, 4, 1) DL_SHAPE(8, 8, 1) DL_SHAPE(16, 16, 1) DL_SHAPE(32, 16, 2)
    DL_SHAPE(64, 16, 4) DL_SHAPE(128, 16, 8) DL_SHAPE(256, 16, 16)
#undef DL_SHAPE
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

// Widest access for which the fp64 tile of n rows takes 64 KiB of LDS, so that two workgroups
// share a CU (VEC * n <= 128); beyond n = 128 the 4-byte variant uses up to 128 KiB.
int widest_vec_for(int32_t n) {
    if (n <= 32) return 4;
    if (n <= 64) return 2;
    return 1;
}

}  // namespace
int launch_step(Algo algo, float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
                const PhaseArgs& topo, float gamma_f, double beta, hipStream_t stream) {
    const double gamma = static_cast<double>(gamma_f);

    // Pick the widest access all three arrays can share: same misalignment (in elements)
    // modulo the vector width and a row stride that preserves it.
    int vec = widest_vec_for(n);
    int64_t head = 0;
    for (; vec > 1; vec >>= 1) {
        const uintptr_t mask = static_cast<uintptr_t>(vec) - 1;
        const uintptr_t ax = (reinterpret_cast<uintptr_t>(x) >> 2) & mask;
        const uintptr_t am = m ? (reinterpret_cast<uintptr_t>(m) >> 2) & mask : ax;
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
        if (algo == ALGO_DSGD)
            return launch_cols<ALGO_DSGD>(v, x + c0, nullptr, g + c0, n, cols, ld, topo, gamma, beta, stream);
        if (algo == ALGO_DECENTLAM_XPREV)
            return launch_cols<ALGO_DECENTLAM_XPREV>(v, x + c0, m + c0, g + c0, n, cols, ld, topo, gamma, beta, stream);
        return launch_cols<ALGO_DMSGD>(v, x + c0, m + c0, g + c0, n, cols, ld, topo, gamma, beta, stream);
    };
    if (int rc = run(vec, head, body)) return rc;   // aligned body first: it is the bulk
    if (int rc = run(1, 0, head)) return rc;        // columns are independent, so the peeled
    if (int rc = run(1, head + body, tail)) return rc;  // head and tail are separate launches
    return DL_OK;
}

}  // namespace dl
