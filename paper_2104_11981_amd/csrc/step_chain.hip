// The fused step for row-major arrays whose rows alternate between starting on a 64 KiB boundary and
// starting 32 KiB after one (ld * 4 an odd multiple of 32 KiB: a contiguous 32 x 25.6 M array is the case
// that matters, 25.6 M * 4 = 3125 * 32 KiB).
//
// What this GPU's memory wants (measured with bare streams over 32 rows, 3 reads + 2 writes per element):
// every wave-wide access should cover both 512-byte halves of one "page", the addresses A and A + 32 KiB
// inside one 64 KiB-aligned unit.  Of all pairs of 512-byte segments at multiples of 32 KiB inside a
// 256 KiB block only those three pairs stream at 6.2 TB/s; every other pair, the neighbouring
// (A + 32 KiB, A + 64 KiB) included, gives 5.1.  The split tiles of step_impl.hpp arrange that for rows that
// start on 64 KiB boundaries: tile u of unit U (16384 columns) owns columns [128 u, 128 u + 128) of the unit
// and the same columns 8192 further on.  For a row that starts 32 KiB off, those two segments are the upper
// half of one page and the lower half of the next page: nothing a tile can do about it on its own, since all
// rows of a tile must share its columns (the mixing runs down the columns).
//
// Here a workgroup walks a chain of tiles, the same u in consecutive units, and treats its rows of the two
// kinds differently.  The launch starts where row 0 sits on a 64 KiB boundary, so the even rows are the
// aligned kind.  Thread slot 0 holds an even row and works as the ordinary kernel does.
// Slot 1 holds an odd row, whose pages pair the upper segment of unit U with the lower segment
// of unit U + 1:
//   * its lanes 0-31 (lower segment) load one unit ahead, together with lanes 32-63 loading the upper
//     segment of the current unit: one access, one page; the values loaded ahead wait in registers;
//   * its lanes 32-63 keep their results for one iteration and store them together with what lanes 0-31
//     compute for the next unit: again one access, one page.
// The same twelve registers serve both halves of the wave (inputs waiting in lanes 0-31, results waiting in
// lanes 32-63).  Only the first lower and the last upper segment of a chain go out as half pages.  Bare
// streams with this access pattern measured 2.65-2.67 ms on 32 x 25.6 M with ld = d against 2.82-2.89 ms
// with plain split tiles and 2.58-2.63 ms on rows that all start on 64 KiB boundaries (holding only the
// stores back: 2.75; both are needed).  This kernel on the same arrays: 2.63-2.65 ms (0.775-0.78 of the HBM
// peak) where the split tiles took 2.83 (0.72); rows on 64 KiB boundaries remain the fastest layout (2.51).
// Tried without gain: the next unit's loads issued ahead of the barrier that frees the tile (the other
// workgroup on the CU already covers that gap), a pause of the odd-numbered waves after the barrier.
//
// Arithmetic, order of the sums and results are those of k_step: same bits.
#define DL_STEP_KERNEL_IMPL
#include "step_impl.hpp"

namespace dl {
namespace step {
namespace {

// Which units a workgroup walks.  Long chains have few half pages (two per chain and odd row), but a launch
// of few, long workgroups ends with most of the chip idle while the last ones finish.  So the chains get
// shorter towards the end of the launch: up to kChainSegments runs of chains, each run with its own length.
constexpr int kChainSegments = 8;
struct ChainArgs {
    uint32_t units;                         // 64 KiB units (16384 columns) covered by the launch
    uint32_t segments;
    uint32_t first_group[kChainSegments];   // first chain (workgroup index / 64) of the run
    uint32_t first_unit[kChainSegments];    // its first unit
    uint32_t len[kChainSegments];           // units per chain in this run
};

template <int ALGO>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_step_chain(float* __restrict__ x, float* __restrict__ m,
                                                      const float* __restrict__ g, int64_t ld,
                                                      double gamma, double inv_gamma, double beta,
                                                      const ChainArgs chain, const PhaseArgs topo) {
    constexpr int VEC = 4, TC = 256, WAVES = 16;
    static_assert(ALGO == ALGO_DECENTLAM || ALGO == ALGO_DMSGD || ALGO == ALGO_AWC_DMSGD,
                  "methods that update (x, m) with one gather per iteration");
    extern __shared__ __attribute__((aligned(16))) double lds[];
    const int n = topo.n;
    Neighbour* table = reinterpret_cast<Neighbour*>(lds + n * TC);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool lower = lane < 32;
    const uint32_t u = blockIdx.x % kSplitTilesPerUnit, group = blockIdx.x / kSplitTilesPerUnit;
    uint32_t run = 0;   // uniform
#pragma unroll
    for (uint32_t k = 1; k < kChainSegments; ++k)
        if (k < chain.segments && group >= chain.first_group[k]) run = k;
    const uint32_t unit0 = chain.first_unit[run] + (group - chain.first_group[run]) * chain.len[run];
    const uint32_t unit1 = unit0 + chain.len[run] < chain.units ? unit0 + chain.len[run] : chain.units;
    const int lane_col = static_cast<int>(split_column(0, lane));

    // neighbour list: kernel arguments -> LDS table (as in k_step; once per chain)
    const uint32_t last_pair = topo.row_ptr_pairs[n >> 1];
    const int nnz = (n & 1) ? last_pair >> 16 : last_pair & 0xffffu;
    int rows[2], e_begin[2], e_end[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int i = 2 * wave + r;
        rows[r] = i;
        const int row = i < n ? i : 0;
        const uint32_t lo = topo.row_ptr_pairs[row >> 1], hi = topo.row_ptr_pairs[(row + 1) >> 1];
        e_begin[r] = (row & 1) ? lo >> 16 : lo & 0xffffu;
        e_end[r] = (row & 1) ? hi & 0xffffu : hi >> 16;
    }
    if (topo.palette == 2) {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            if (rows[r] < n) {
                const float w_row = topo.rows.value[row_palette_index(topo, rows[r])];
                for (int e = e_begin[r] + lane; e < e_end[r]; e += 64) table[e].set(w_row, static_cast<int>(topo.rows.col[e]) * TC);
            }
        }
    } else {
        for (int e = threadIdx.x; e < nnz; e += 64 * WAVES) {
            if (topo.palette == 0) table[e].set(topo.direct.w[e], static_cast<int>(topo.direct.col[e]) * TC);
            else table[e].set(topo.pal.value[topo.pal.widx[e]], static_cast<int>(topo.pal.col[e]) * TC);
        }
    }

    // row bases (uniform); rows beyond the problem read row 0 and store nothing
    const float* xrow[2];
    const float* grow[2];
    float* mrow[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int64_t at = static_cast<int64_t>(rows[r] < n ? rows[r] : 0) * ld;
        xrow[r] = x + at;
        grow[r] = g + at;
        mrow[r] = m + at;
    }
    const bool shifted_row = rows[1] < n;   // uniform

    // Slot 1's waiting values.  Lanes 0-31: the inputs x, g, m of the next unit's lower segment.  Lanes 32-63:
    // the results for the previous unit's upper segment (new x in wait_a, new m in wait_b).
    float wait_a[VEC] = {0.f, 0.f, 0.f, 0.f}, wait_b[VEC] = {0.f, 0.f, 0.f, 0.f}, wait_c[VEC] = {0.f, 0.f, 0.f, 0.f};
    if (lower && unit0 < unit1) {   // the chain's first lower segment has no partner: a half page
        const int64_t c = static_cast<int64_t>(unit0) * kSplitUnit + u * kSplitSegment + lane_col;
        load_vec<VEC>(xrow[1] + c, wait_a);
        load_vec<VEC>(grow[1] + c, wait_b);
        load_vec<VEC>(mrow[1] + c, wait_c);
    }

    double* slot[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) slot[r] = lds + (rows[r] < n ? rows[r] : 0) * TC + lane * 2;
    const double* tile_at_lane = lds + lane * 2;
    int64_t c = 0;
    for (uint32_t unit = unit0; unit < unit1; ++unit) {
        c = static_cast<int64_t>(unit) * kSplitUnit + u * kSplitSegment + lane_col;
        // ---- phase 1: all six loads, then the local pre-step into LDS
        float xr[2][VEC], gr[2][VEC], mr[2][VEC];
        load_vec<VEC>(xrow[0] + c, xr[0]);
        load_vec<VEC>(grow[0] + c, gr[0]);
        load_vec<VEC>(mrow[0] + c, mr[0]);
        // slot 1: lanes 0-31 one unit ahead; in the chain's last unit they have nothing left to fetch and
        // read what lanes 32-63 read (same lines: no traffic of their own)
        const int64_t c1 = lower ? (unit + 1 < unit1 ? c + kSplitUnit : c + kSplitDistance) : c;
        load_vec<VEC>(xrow[1] + c1, xr[1]);
        load_vec<VEC>(grow[1] + c1, gr[1]);
        load_vec<VEC>(mrow[1] + c1, mr[1]);
#pragma unroll
        for (int v = 0; v < VEC; ++v) {   // lanes 0-31: what waited is this unit's; what came in waits
            const float fx = xr[1][v], fg = gr[1][v], fm = mr[1][v];
            xr[1][v] = lower ? wait_a[v] : fx;
            gr[1][v] = lower ? wait_b[v] : fg;
            mr[1][v] = lower ? wait_c[v] : fm;
            if (lower) {   // a select per register; lanes 32-63 keep their waiting results
                wait_a[v] = fx;
                wait_b[v] = fg;
                wait_c[v] = fm;
            }
        }
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            if (rows[r] < n) {   // uniform
                if constexpr (ALGO == ALGO_AWC_DMSGD) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) slot[r][lds_col(v)] = static_cast<double>(xr[r][v]);
                } else if constexpr (ALGO != ALGO_DMSGD) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v)
                        slot[r][lds_col(v)] = static_cast<double>(xr[r][v]) - gamma * static_cast<double>(gr[r][v]);
                } else {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        const double m_new = beta * static_cast<double>(mr[r][v]) + static_cast<double>(gr[r][v]);
                        mr[r][v] = static_cast<float>(m_new);   // the new m waits here and is stored with x
                        slot[r][lds_col(v)] = static_cast<double>(xr[r][v]) - gamma * m_new;
                    }
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): nothing is outstanding on any path
        __syncthreads();

        // ---- phase 2: gather-mix from LDS, finish the update, store
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            if (rows[r] < n) {
                double z[VEC] = {0.0, 0.0, 0.0, 0.0};
                int e = e_begin[r];
                const int e1 = e_end[r];
                // two neighbours at a time only where the registers allow it: the kernel must stay within 64
                // (two workgroups per CU), and the twelve waiting registers are spoken for
                if constexpr (ALGO == ALGO_DMSGD) {
                    for (; e + 2 <= e1; e += 2) gather<VEC, 2>(table + e, tile_at_lane, z);
                }
                for (; e < e1; ++e) gather<VEC, 1>(table + e, tile_at_lane, z);
                float xo[VEC], mo[VEC];
                if constexpr (ALGO == ALGO_DECENTLAM) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        const double xi = static_cast<double>(xr[r][v]);
                        const double gt = (xi - z[v]) * inv_gamma;
                        const double m_new = __builtin_fma(beta, static_cast<double>(mr[r][v]), gt);
                        mo[v] = static_cast<float>(m_new);
                        xo[v] = static_cast<float>(xi - gamma * m_new);
                    }
                } else if constexpr (ALGO == ALGO_AWC_DMSGD) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        const double m_new = beta * static_cast<double>(mr[r][v]) + static_cast<double>(gr[r][v]);
                        mo[v] = static_cast<float>(m_new);
                        xo[v] = static_cast<float>(z[v] - gamma * m_new);
                    }
                } else {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        mo[v] = mr[r][v];
                        xo[v] = static_cast<float>(z[v]);
                    }
                }
                if (r == 0) {
                    store_vec<VEC>(mrow[0] + c, mo);
                    store_vec<VEC>(const_cast<float*>(xrow[0]) + c, xo);
                } else {
                    // lanes 0-31 store this unit's lower segment, lanes 32-63 the previous unit's upper one
                    float sx[VEC], sm[VEC];
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        sx[v] = lower ? xo[v] : wait_a[v];
                        sm[v] = lower ? mo[v] : wait_b[v];
                        if (!lower) {
                            wait_a[v] = xo[v];
                            wait_b[v] = mo[v];
                        }
                    }
                    const int64_t cs = lower ? c : c - kSplitUnit;
                    if (lower || unit > unit0) {
                        store_vec<VEC>(mrow[1] + cs, sm);
                        store_vec<VEC>(const_cast<float*>(xrow[1]) + cs, sx);
                    }
                }
            }
        }
        if (unit + 1 < unit1) __syncthreads();   // the tile is free for the next unit
    }
    if (shifted_row && !lower && unit0 < unit1) {   // the chain's last upper segment: a half page
        store_vec<VEC>(mrow[1] + c, wait_b);
        store_vec<VEC>(const_cast<float*>(xrow[1]) + c, wait_a);
    }
}

template <int ALGO>
int launch_chain_algo(const StepCall& s, uint32_t units, uint32_t len) {
    const size_t lds_bytes = lds_bytes_for(s.n, 4, s.topo->row_ptr[s.n], 1);
    if (lds_bytes > 80 * 1024) return set_error(DL_ETOPO, "step: the chain kernel's tile does not fit");
    auto kernel = k_step_chain<ALGO>;
    if (lds_bytes > 48 * 1024) {
        static std::atomic<uint64_t> configured{0};   // per instantiation; see allow_large_lds
        if (int rc = allow_large_lds(reinterpret_cast<const void*>(kernel), configured)) return rc;
    }
    // chains of `len` units while at least 16 chains of that length remain, then half as long, and so on
    ChainArgs chain{};
    chain.units = units;
    uint32_t groups = 0, unit = 0;
    for (uint32_t l = len; unit < units; l = l > 1 ? l / 2 : 1) {
        const uint32_t left = units - unit;
        const bool last = l == 1 || chain.segments + 1 == kChainSegments;
        uint32_t count = last ? (left + l - 1) / l : (left > 16 * l ? (left - 16 * l + l - 1) / l : 0);
        if (count == 0) continue;
        const uint32_t k = chain.segments++;
        chain.first_group[k] = groups;
        chain.first_unit[k] = unit;
        chain.len[k] = l;
        groups += count;
        unit += count * l;   // may pass `units` in the last run: the kernel clamps
    }
    hipLaunchKernelGGL(kernel, dim3(groups * kSplitTilesPerUnit), dim3(1024), lds_bytes, s.stream, s.x, s.m,
                       static_cast<const float*>(s.g), s.ld, s.gamma, 1.0 / s.gamma, s.beta, chain, *s.topo);
    return check_hip(hipGetLastError(), "step kernel launch (chained tiles)");
}

}  // namespace

bool chain_serves(int algo, int32_t n, int nnz) {
    if (n <= 16 || n > 32 || mixes_on_matrix_cores(n, nnz)) return false;
    return algo == ALGO_DECENTLAM || algo == ALGO_DMSGD || algo == ALGO_AWC_DMSGD;
}

int launch_chain(int algo, const StepCall& s, uint32_t units, uint32_t len) {
    switch (algo) {
        case ALGO_DECENTLAM: return launch_chain_algo<ALGO_DECENTLAM>(s, units, len);
        case ALGO_DMSGD: return launch_chain_algo<ALGO_DMSGD>(s, units, len);
        case ALGO_AWC_DMSGD: return launch_chain_algo<ALGO_AWC_DMSGD>(s, units, len);
        default: return set_error(DL_EINVAL, "step: this method has no chained-tile kernel");
    }
}

}  // namespace step
}  // namespace dl
