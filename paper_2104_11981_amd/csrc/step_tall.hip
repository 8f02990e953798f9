// The fused step for 33-128 nodes on row-major arrays whose rows start on 64 KiB boundaries.
//
// What limits k_step there: its fp64 tile holds every row of a tile's columns.  Beyond 64 nodes that leaves room
// for 128 columns in a CU's LDS, and 128 columns are 8 bytes per lane, one 512-byte piece per row and tile; this
// GPU's memory wants 16-byte lanes that cover both 512-byte halves of an address pair (A, A + 32 KiB), the split
// tiles of step_impl.hpp.  Bare 3-read/2-write streams over 128 rows: 5.05-5.15 TB/s for every shape of a
// 128-column tile (one 512-byte piece; two 256-byte pieces 32 KiB apart; 16-byte lanes over two rows at a
// time), 6.0 TB/s for the split tile of 256 columns.  At 33-64 nodes the 16-byte lanes fit, but their tile of
// 96-128 KiB leaves one workgroup per CU, which has nothing to overlap its gathers with (a pause of 1.7 us between
// the loads and the stores of a bare stream costs 7 % with one workgroup per CU, 2.5 % with two).
//
// Here the global accesses are those of a split tile (16 bytes per lane, 256 columns) and an LDS tile of half that
// width is used twice: first for columns 0 and 1 of every lane, then, when every wave has finished gathering, for
// columns 2 and 3.  Each pass is the 8-byte-lane kernel's second phase on half of the columns, so the tile takes
// n x 128 x 8 bytes, and the results of the first pass wait in the registers of the inputs they replace until
// the row is stored whole.  All twelve values per row (x, g, m) are in registers at once: up to 96 of a thread's
// 128 registers at eight rows per thread, which a workgroup of 1024 threads alone on its CU can have; the shapes
// with three and four rows per thread (33-64 nodes, 10 to 16 waves, tile of at most 64 KiB) are built for 64
// registers, so that two or three workgroups share a CU.  Measured at 819 M node-elements (ring, DecentLaM): 48 / 64 nodes 6.4 TB/s (0.80) where
// k_step ran 5.95 / 6.2; 96 / 128 nodes 5.5 where it ran 5.2 / 5.0.
//
// Arithmetic, order of the sums and results are those of k_step: same bits.
#define DL_STEP_KERNEL_IMPL
#include "step_impl.hpp"

namespace dl {
namespace step {
namespace {

// GF: gradient format (fp32, or bf16 / fp16 widened on load: 8 bytes per lane)
template <int ALGO, int RPT, int WAVES, int GF>
__global__ __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(RPT <= 4 ? 8 : 4, RPT <= 4 ? 8 : 4))) void k_step_tall(float* __restrict__ x, float* __restrict__ m,
                                                    const typename GradElem<GF>::type* __restrict__ g, int64_t ld, int64_t ldg,
                                                    double gamma, double inv_gamma, double beta,
                                                    uint32_t batch_tiles, int64_t batch_stride, const PhaseArgs topo) {
    constexpr int TC = 128;   // columns of the LDS tile: two per lane and pass
    static_assert(ALGO != ALGO_DA_DMSGD, "one gather per iteration");
    constexpr bool kHasM = ALGO != ALGO_DSGD;
    // neighbours per gather: four as in k_step with 8-byte lanes, two where the registers end (64 for the shapes that
    // share a CU between two workgroups, 128 for the others)
    constexpr int GROUP = (RPT == 4 || (RPT == 3 && ALGO == ALGO_AWC_DMSGD) || (RPT > 7 && ALGO != ALGO_DMSGD && ALGO != ALGO_DSGD)) ? 2 : 4;
    extern __shared__ __attribute__((aligned(16))) double lds[];
    const int n = topo.n;
    using Entry = NeighbourCompact;
    Entry* table = reinterpret_cast<Entry*>(lds + n * TC);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Which columns: a split tile of a single row-major problem, or (batch_tiles != 0: the blocked layout) tile
    // blockIdx.x % batch_tiles, 256 consecutive columns, of sub-problem blockIdx.x / batch_tiles; all uniform.
    int64_t tile_col = split_column(blockIdx.x, 0);
    int lane_col = static_cast<int>(split_column(0, lane));
    if (batch_tiles) {
        const uint32_t sub = blockIdx.x / batch_tiles;
        x += sub * batch_stride;
        if constexpr (kHasM) m += sub * batch_stride;
        g += sub * batch_stride;
        tile_col = static_cast<int64_t>(blockIdx.x - sub * batch_tiles) * 256;
        lane_col = lane * 4;
    }

    // ---- all loads of the tile, what the first pre-step needs first: the rest may still be on its way while the
    // first pass runs (loads return in order)
    constexpr bool kEarlyM = ALGO == ALGO_DMSGD, kEarlyG = ALGO != ALGO_AWC_DMSGD;
    float xr[RPT][4], gr[RPT][4], mr[RPT][4];
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int i = wave + WAVES * r;
        const int64_t row = i < n ? i : 0;   // uniform; rows beyond the problem read row 0 and store nothing
        load_vec<4>(x + (row * ld + tile_col) + lane_col, xr[r]);
        if constexpr (kEarlyG) load_grad<4, GF>(g + (row * ldg + tile_col) + lane_col, gr[r]);
        if constexpr (kHasM && kEarlyM) load_vec<4>(m + (row * ld + tile_col) + lane_col, mr[r]);
    }
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int i = wave + WAVES * r;
        const int64_t row = i < n ? i : 0;
        if constexpr (!kEarlyG) load_grad<4, GF>(g + (row * ldg + tile_col) + lane_col, gr[r]);
        if constexpr (kHasM && !kEarlyM) load_vec<4>(m + (row * ld + tile_col) + lane_col, mr[r]);
    }

    // ---- neighbour list: kernel arguments -> LDS table (as in k_step)
    const uint32_t last_pair = topo.row_ptr_pairs[n >> 1];
    const int nnz = (n & 1) ? last_pair >> 16 : last_pair & 0xffffu;
    int e_begin[RPT], e_end[RPT];
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int i = wave + WAVES * r;
        const int row = i < n ? i : 0;
        const uint32_t lo = topo.row_ptr_pairs[row >> 1], hi = topo.row_ptr_pairs[(row + 1) >> 1];
        e_begin[r] = (row & 1) ? lo >> 16 : lo & 0xffffu;
        e_end[r] = (row & 1) ? hi & 0xffffu : hi >> 16;
    }
    if (topo.palette == 2) {   // one weight per row: every wave writes the entries of its rows
#pragma unroll
        for (int r = 0; r < RPT; ++r) {
            const int i = wave + WAVES * r;
            if (i < n) {
                const float w_row = topo.rows.value[row_palette_index(topo, i)];
                for (int e = e_begin[r] + lane; e < e_end[r]; e += 64) table[e].set(w_row, static_cast<int>(topo.rows.col[e]) * TC);
            }
        }
    } else {
        for (int e = threadIdx.x; e < nnz; e += 64 * WAVES) {
            if (topo.palette == 0) table[e].set(topo.direct.w[e], static_cast<int>(topo.direct.col[e]) * TC);
            else table[e].set(topo.pal.value[topo.pal.widx[e]], static_cast<int>(topo.pal.col[e]) * TC);
        }
    }

    const double* tile_at_lane = lds + lane * 2;
#pragma unroll
    for (int p = 0; p < 2; ++p) {   // columns 2p and 2p + 1 of every lane
        if (p == 1) {
            // Every load has long returned: said explicitly before the pass that stores, or the compiler, unsure
            // about paths that skipped a row, makes a row's stores wait for those of the row before it (loads and
            // stores share one in-order counter).
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), nothing else
            __syncthreads();   // every wave has finished gathering the first pass
        }
        // local pre-step into the tile
#pragma unroll
        for (int r = 0; r < RPT; ++r) {
            const int i = wave + WAVES * r;
            if (i < n) {   // uniform
                vd2 u;
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int v = 2 * p + q;
                    double uv;
                    if constexpr (ALGO == ALGO_AWC_DMSGD) {
                        uv = static_cast<double>(xr[r][v]);
                    } else if constexpr (ALGO == ALGO_DMSGD) {
                        const double m_new = beta * static_cast<double>(mr[r][v]) + static_cast<double>(gr[r][v]);
                        mr[r][v] = static_cast<float>(m_new);   // the new m waits here and is stored with x
                        uv = static_cast<double>(xr[r][v]) - gamma * m_new;
                    } else {
                        uv = static_cast<double>(xr[r][v]) - gamma * static_cast<double>(gr[r][v]);
                    }
                    if (q == 0) u.x = uv;
                    else u.y = uv;
                }
                *reinterpret_cast<vd2*>(lds + i * TC + lane * 2) = u;
                // x is wanted as a double again after the gather: widen it again there (one instruction) instead of
                // keeping sixteen doubles alive across the gather, which this kernel has no registers for
                if constexpr (ALGO == ALGO_DECENTLAM || ALGO == ALGO_DECENTLAM_XPREV) {
#pragma unroll
                    for (int q = 0; q < 2; ++q) asm volatile("" : "+v"(xr[r][2 * p + q]));
                }
            }
        }
        __syncthreads();

        // gather-mix, finish the update of the two columns; the second pass stores the row
#pragma unroll
        for (int r = 0; r < RPT; ++r) {
            const int i = wave + WAVES * r;
            if (i < n) {
                double z[2] = {0.0, 0.0};
                int e = e_begin[r];
                const int e1 = e_end[r];
                // groups of GROUP neighbours: four where the registers allow it, as in k_step with 8-byte lanes
                if constexpr (GROUP == 4) {
                    for (; e + 4 <= e1; e += 4) gather<2, 4>(table + e, tile_at_lane, z);
                    if (e + 2 <= e1) {
                        gather<2, 2>(table + e, tile_at_lane, z);
                        e += 2;
                    }
                } else {
                    for (; e + 2 <= e1; e += 2) gather<2, 2>(table + e, tile_at_lane, z);
                }
                for (; e < e1; ++e) gather<2, 1>(table + e, tile_at_lane, z);
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int v = 2 * p + q;
                    if constexpr (ALGO == ALGO_DECENTLAM) {
                        const double xi = static_cast<double>(xr[r][v]);
                        const double gt = (xi - z[q]) * inv_gamma;
                        const double m_new = __builtin_fma(beta, static_cast<double>(mr[r][v]), gt);
                        mr[r][v] = static_cast<float>(m_new);
                        xr[r][v] = static_cast<float>(xi - gamma * m_new);
                    } else if constexpr (ALGO == ALGO_DECENTLAM_XPREV) {   // m holds x_prev and receives x_next
                        const double diff = static_cast<double>(xr[r][v]) - static_cast<double>(mr[r][v]);
                        mr[r][v] = static_cast<float>(__builtin_fma(beta, diff, z[q]));
                    } else if constexpr (ALGO == ALGO_AWC_DMSGD) {
                        const double m_new = beta * static_cast<double>(mr[r][v]) + static_cast<double>(gr[r][v]);
                        mr[r][v] = static_cast<float>(m_new);
                        xr[r][v] = static_cast<float>(z[q] - gamma * m_new);
                    } else {   // DSGD, DmSGD
                        xr[r][v] = static_cast<float>(z[q]);
                    }
                }
                if (p == 1) {
                    // the lane's columns, worked out afresh from the lane number (two instructions) rather than kept
                    // in a register through both passes, which the four-row shape has none left for
                    const int lane_again = static_cast<int>(__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)));
                    const int64_t at = (static_cast<int64_t>(i) * ld + tile_col) +
                                       (batch_tiles ? static_cast<int64_t>(lane_again) * 4 : split_column(0, lane_again));
                    if constexpr (kHasM) store_vec<4>(m + at, mr[r]);
                    if constexpr (ALGO != ALGO_DECENTLAM_XPREV) store_vec<4>(x + at, xr[r]);
                }
            }
        }
    }
}

template <int ALGO, int GF, int RPT, int WAVES = 16>
int launch_tall_shape(const StepCall& s, uint32_t tiles, uint32_t batch_tiles) {
    const size_t lds_bytes = lds_bytes_for(s.n, 2, s.topo->row_ptr[s.n], 1);
    if (lds_bytes > 160 * 1024) return set_error(DL_ETOPO, "step: the two-pass kernel's tile does not fit");
    auto kernel = k_step_tall<ALGO, RPT, WAVES, GF>;
    if (lds_bytes > 48 * 1024) {
        static std::atomic<uint64_t> configured{0};   // per instantiation; see allow_large_lds
        if (int rc = allow_large_lds(reinterpret_cast<const void*>(kernel), configured)) return rc;
    }
    hipLaunchKernelGGL(kernel, dim3(tiles), dim3(64 * WAVES), lds_bytes, s.stream, s.x, s.m,
                       static_cast<const typename GradElem<GF>::type*>(s.g), s.ld, s.ldg, s.gamma, 1.0 / s.gamma, s.beta, batch_tiles,
                       s.batch_stride, *s.topo);
    return check_hip(hipGetLastError(), "step kernel launch (two-pass tiles)");
}

template <int ALGO, int GF = DL_GRAD_F32>
int launch_tall_algo(const StepCall& s, uint32_t tiles, uint32_t batch_tiles) {
    // waves x rows per thread.  Up to 64 nodes a shape without empty row slots is worth 2-4 % (36 / 40 / 56 nodes:
    // 6.5 / 6.45 / 6.3 TB/s with 12 x 3 / 10 x 4 / 14 x 4 against 6.2 / 6.25 / 6.2 with 16 x 3 / 16 x 3 / 16 x 4)
    if (s.n <= 36) return launch_tall_shape<ALGO, GF, 3, 12>(s, tiles, batch_tiles);
    if constexpr (ALGO != ALGO_AWC_DMSGD) {
        if (s.n <= 40) return launch_tall_shape<ALGO, GF, 4, 10>(s, tiles, batch_tiles);
    }
    if (s.n <= 48) return launch_tall_shape<ALGO, GF, 3>(s, tiles, batch_tiles);
    if constexpr (ALGO != ALGO_AWC_DMSGD) {
        if (s.n <= 56) return launch_tall_shape<ALGO, GF, 4, 14>(s, tiles, batch_tiles);
        if (s.n <= 64) return launch_tall_shape<ALGO, GF, 4>(s, tiles, batch_tiles);
    }
    if (s.n <= 80) return launch_tall_shape<ALGO, GF, 5>(s, tiles, batch_tiles);
    if (s.n <= 96) return launch_tall_shape<ALGO, GF, 6>(s, tiles, batch_tiles);
    if (s.n <= 112) return launch_tall_shape<ALGO, GF, 7>(s, tiles, batch_tiles);
    return launch_tall_shape<ALGO, GF, 8>(s, tiles, batch_tiles);
}

}  // namespace

bool tall_serves(int algo, int32_t n, int nnz, int gformat) {
    if (n <= 32 || n > 128 || algo == ALGO_DA_DMSGD || mixes_on_matrix_cores(n, nnz)) return false;
    // 16-bit gradients: the methods that have entry points of their own for them
    if (gformat != DL_GRAD_F32 && algo != ALGO_DECENTLAM && algo != ALGO_DMSGD && algo != ALGO_DECENTLAM_XPREV) return false;
    if (n > 48 && n <= 64 && algo == ALGO_AWC_DMSGD) return false;   // four rows per thread of x, g and m: 4 registers short
    return lds_bytes_for(n, 2, nnz, 1) <= 160 * 1024;
}

int launch_tall(int algo, const StepCall& s, uint32_t units, int gformat) {
    uint32_t tiles, batch_tiles = 0;
    if (s.batches > 1 || s.batch_stride != 0) {   // blocked layout: s.d columns per sub-problem, whole tiles only
        const int64_t per = s.d / 256, all = per * s.batches;
        if (s.d % 256 != 0 || per < 1 || all > 0x7fffffffLL || s.batch_stride_g != s.batch_stride)
            return set_error(DL_EINVAL, "step: the two-pass kernel takes blocks of whole 256-column tiles");
        tiles = static_cast<uint32_t>(all);
        batch_tiles = static_cast<uint32_t>(per);
    } else {
        if (units > 0x7fffffffu / kSplitTilesPerUnit) return set_error(DL_EINVAL, "step: d too large for one launch");
        tiles = units * kSplitTilesPerUnit;
    }
    if (gformat != DL_GRAD_F32) {
        const bool bf = gformat == DL_GRAD_BF16;
        switch (algo) {
            case ALGO_DECENTLAM:
                return bf ? launch_tall_algo<ALGO_DECENTLAM, DL_GRAD_BF16>(s, tiles, batch_tiles)
                          : launch_tall_algo<ALGO_DECENTLAM, DL_GRAD_F16>(s, tiles, batch_tiles);
            case ALGO_DMSGD:
                return bf ? launch_tall_algo<ALGO_DMSGD, DL_GRAD_BF16>(s, tiles, batch_tiles)
                          : launch_tall_algo<ALGO_DMSGD, DL_GRAD_F16>(s, tiles, batch_tiles);
            case ALGO_DECENTLAM_XPREV:
                return bf ? launch_tall_algo<ALGO_DECENTLAM_XPREV, DL_GRAD_BF16>(s, tiles, batch_tiles)
                          : launch_tall_algo<ALGO_DECENTLAM_XPREV, DL_GRAD_F16>(s, tiles, batch_tiles);
            default: return set_error(DL_EINVAL, "step: this method has no two-pass kernel for 16-bit gradients");
        }
    }
    switch (algo) {
        case ALGO_DECENTLAM: return launch_tall_algo<ALGO_DECENTLAM>(s, tiles, batch_tiles);
        case ALGO_DMSGD: return launch_tall_algo<ALGO_DMSGD>(s, tiles, batch_tiles);
        case ALGO_DSGD: return launch_tall_algo<ALGO_DSGD>(s, tiles, batch_tiles);
        case ALGO_AWC_DMSGD: return launch_tall_algo<ALGO_AWC_DMSGD>(s, tiles, batch_tiles);
        case ALGO_DECENTLAM_XPREV: return launch_tall_algo<ALGO_DECENTLAM_XPREV>(s, tiles, batch_tiles);
        default: return set_error(DL_EINVAL, "step: this method has no two-pass kernel");
    }
}

}  // namespace step
}  // namespace dl
