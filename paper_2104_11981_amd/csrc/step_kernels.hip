// Fused decentralized-update kernels for gfx950 (CDNA4).
//
// Mixing acts along the node axis only (matrix forms of Algorithms 1 and 2 in the
// appendix "Preliminary"), so every column of the stacked n x d arrays is an
// independent n-vector problem.  A workgroup of WAVES wavefronts owns a tile of
// TC = 64*VEC columns for ALL n rows:
//
//   phase 1  every wave streams whole rows of the tile (row index is wave-uniform):
//            x_j, g_j, m_j come in with VEC*4-byte non-temporal loads, all issued before anything
//            waits for one; the local pre-step (u_j = x_j - gamma g_j for DecentLaM,
//            h_j = x_j - gamma (beta m_j + g_j) for DmSGD) is evaluated in fp64 and parked in LDS
//            as fp64 (each tile row as planes of 64 pairs of doubles: 16-byte accesses, no bank
//            conflicts); meanwhile
//            the neighbour list of W is unpacked from the kernel arguments into an LDS table of
//            (fp64 weight, LDS row offset) pairs and every wave fetches the bounds of its rows'
//            slices of that list with scalar loads;
//   phase 2  after one barrier (and, for some shapes, a short pause of the odd-numbered waves
//            that spreads the workgroup's stores), row i gathers its |N_i| neighbour rows from
//            LDS in list order, finishes the update in fp64 and stores fp32 in place with
//            non-temporal stores.
//
// HBM traffic is exactly read x, m, g + write x, m = 20 bytes per node-element,
// independent of the node degree; updating in place is race-free because no
// other workgroup touches these columns.  Which columns a tile owns is free: large row-major
// launches use "split tiles" (step_impl.hpp), the column order this GPU's write path prefers.
//
// Dense graphs on 17-32 nodes take a different phase 2: the tile is multiplied by W on the matrix cores
// (fp64 MFMA; mix_dense in step_impl.hpp), a second barrier, and every row reads its sum with one access.
//
// The same template serves DSGD, the momentum-free form of DecentLaM, AWC-DmSGD and DA-DmSGD, bf16 or
// fp16 gradients (widened exactly on load), per-tile sums of squares of g, the new m and the new x
// (per-tensor norms are finished in norms_kernels.hip), and launches over "batches" (the blocks of the
// blocked layout).
#include "step_impl.hpp"

namespace dl {
namespace {

using namespace step;

// Below this a launch keeps plain tiles.  Measured with rows on 64 KiB boundaries, exponential graph, split tiles from
// 2^16 instead of 2^20 columns on: 32 nodes x 262144 / 524288 columns 0.66 / 0.71 -> 0.71 / 0.74 of the HBM peak, 48 nodes
// x 131072 / 524288 0.64 / 0.69 -> 0.73 / 0.74, 64 nodes x 131072 / 524288 0.59 / 0.67 -> 0.70 / 0.76.
constexpr int64_t kSplitMinColumns = 1 << 16;
constexpr int64_t kChainMinColumns = 1 << 20;   // the chained-tile kernel walks runs of units: long rows only

// Widest access by node count.  Up to 32 nodes the fp64 tile of 16-byte lanes takes 64 KiB of LDS and
// two workgroups share a CU.  Beyond that the wide lanes are kept and the tile grows to 128 KiB, one
// workgroup per CU: measured better than halving the lanes to keep two (64 nodes: 6.2 against 5.3 TB/s
// row-major, 6.5 against 6.4 blocked; 128 nodes with 8-byte lanes: 6.4 against 5.5 blocked), because
// the 16-byte lanes bring full 512-byte segments and their pairing (split tiles) with them.  (Large launches on
// 64 KiB-aligned rows of 33-128 nodes go to the two-pass kernel of step_tall.hip, which has 16-byte lanes at all of
// these node counts; this table is for everything else.)
// Longest chain of the chained-tile kernel, in units (the chains get shorter towards the end of a launch).
// Measured on 32 x 25.6 M, ld = d: 2.70 / 2.67 / 2.68 / 2.71 ms with every chain 2 / 4 / 8 / 16 units long (long
// chains leave the chip half idle at the end of the launch), 2.63 / 2.65 / 2.65 / 2.66 ms with chains of at
// most 8 / 16 / 32 / 64 units that shorten towards the end.
constexpr uint32_t kChainLength = 8;

int widest_vec_for(int32_t n, Algo /*algo*/) {
    if (n <= 64) return 4;
    if (n <= 128) return 2;
    return 1;
}

}  // namespace
int launch_step(Algo algo, float* x, float* m, GradArg g, int32_t n, int64_t d, int64_t ld,
                const PhaseArgs& topo, float gamma_f, double beta, hipStream_t stream, NormPlan* norms,
                int64_t batches, int64_t batch_stride, int64_t batch_stride_g) {
    const double gamma = static_cast<double>(gamma_f);
    const size_t gbytes = grad_elem_bytes(g.format);
    const unsigned gshift = gbytes == 4 ? 2 : 1;

    // 33-128 nodes, rows on 64 KiB boundaries, all arrays alike modulo 16 bytes: the whole 64 KiB units of a large
    // launch go to the kernel that keeps 16-byte lanes and split tiles by using its LDS tile twice (step_tall.hip);
    // the columns before and after them are short launches of their own.  Up to 64 nodes that kernel's second
    // workgroup per CU is worth more than the alignment: rows on any 512-byte boundary take it too (48 / 64 nodes,
    // rows alternating between 64 KiB boundaries and their midpoints: 6.15 / 6.0 TB/s against 5.7 with k_step; rows
    // on other 512-byte boundaries 6.1 / 5.8 against 5.7; at 96 and 128 nodes the comparison went either way).
    if (n > 32 && batches == 1 && !norms && d >= kSplitMinColumns && ld % (n <= 64 ? kSplitSegment : kSplitUnit) == 0 &&
        g.ld % 4 == 0 && tall_serves(algo, n, topo.row_ptr[n], g.format)) {
        const uintptr_t ax = (reinterpret_cast<uintptr_t>(x) >> 2) & 3;
        const uintptr_t am = m ? (reinterpret_cast<uintptr_t>(m) >> 2) & 3 : ax;
        const uintptr_t ag = (reinterpret_cast<uintptr_t>(g.p) >> gshift) & 3;
        const float* written = algo == ALGO_DECENTLAM_XPREV ? m : x;
        const int64_t first = static_cast<int64_t>((kSplitUnit - ((reinterpret_cast<uintptr_t>(written) >> 2) % kSplitUnit)) % kSplitUnit);
        const int64_t units = first <= d ? (d - first) / kSplitUnit : 0;
        if (ax == am && ax == ag && units > 0) {
            StepCall s;
            s.x = x + first;
            s.m = m ? m + first : nullptr;
            s.g = static_cast<const char*>(g.p) + static_cast<size_t>(first) * gbytes;
            s.n = n; s.d = units * kSplitUnit; s.ld = ld; s.ldg = g.ld;
            s.gamma = gamma; s.beta = beta; s.topo = &topo; s.stream = stream;
            s.na = NormArgs{nullptr, 0, 0};
            s.batches = 1; s.batch_stride = 0; s.batch_stride_g = 0; s.split_tiles = 0; s.by_xcd = false;
            if (int rc = launch_tall(algo, s, static_cast<uint32_t>(units), g.format)) return rc;
            const int64_t after = first + units * kSplitUnit;   // fewer than kSplitUnit columns on either side
            GradArg g_after = g;
            g_after.p = static_cast<const char*>(g.p) + static_cast<size_t>(after) * gbytes;
            if (first > 0) {
                if (int rc = launch_step(algo, x, m, g, n, first, ld, topo, gamma_f, beta, stream, nullptr, 1, 0, 0)) return rc;
            }
            if (after == d) return DL_OK;
            return launch_step(algo, x + after, m ? m + after : nullptr, g_after, n, d - after, ld, topo, gamma_f, beta,
                               stream, nullptr, 1, 0, 0);
        }
    }

    // The blocked layout on 33-40 and 49-56 nodes (blocks of whole 256-column tiles, everything 16-byte aligned, a
    // launch of 4096 tiles and more): the same kernel in its shapes of 10 to 14 waves, two or three workgroups per CU
    // where k_step has one whose gathers nothing overlaps.  Ring / exponential graph, TB/s: 36 nodes 6.4 / 6.4 against
    // 6.25 / 6.25, 40 nodes 6.25 / 6.3 against 6.2 / 5.8, 56 nodes 6.3 / 6.3 against 6.4 / 6.05; with the 16-wave
    // shapes (48, 64 nodes) 6.4 / 6.05 either way, so those stay with k_step.
    if (n > 32 && (n <= 40 || (n > 48 && n <= 56)) && batch_stride != 0 && !norms && d % 256 == 0 && ld == d && g.ld == d &&
        batch_stride % 4 == 0 && batch_stride_g == batch_stride && batches * (d / 256) >= kSplitMinColumns / 256 &&
        ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(m)) & 15u) == 0 &&
        (reinterpret_cast<uintptr_t>(g.p) & (4 * gbytes - 1)) == 0 && tall_serves(algo, n, topo.row_ptr[n], g.format)) {
        StepCall s;
        s.x = x; s.m = m; s.g = g.p;
        s.n = n; s.d = d; s.ld = ld; s.ldg = g.ld;
        s.gamma = gamma; s.beta = beta; s.topo = &topo; s.stream = stream;
        s.na = NormArgs{nullptr, 0, 0};
        s.batches = batches; s.batch_stride = batch_stride; s.batch_stride_g = batch_stride_g; s.split_tiles = 0; s.by_xcd = false;
        return launch_tall(algo, s, 0, g.format);
    }

    // Pick the widest access all three arrays can share: same misalignment (in elements)
    // modulo the vector width and row strides that preserve it.
    int vec = widest_vec_for(n, algo);
    int64_t head = 0;
    for (; vec > 1; vec >>= 1) {
        const uintptr_t mask = static_cast<uintptr_t>(vec) - 1;
        const uintptr_t ax = (reinterpret_cast<uintptr_t>(x) >> 2) & mask;
        const uintptr_t am = m ? (reinterpret_cast<uintptr_t>(m) >> 2) & mask : ax;
        const uintptr_t ag = (reinterpret_cast<uintptr_t>(g.p) >> gshift) & mask;
        const int64_t strides = ld | g.ld | (batches > 1 ? (batch_stride | batch_stride_g) : 0);
        if (ax == am && ax == ag && (strides & static_cast<int64_t>(mask)) == 0) {
            head = static_cast<int64_t>((vec - ax) & mask);
            break;
        }
    }
    // The fp64 tile and the LDS table of neighbours must fit a CU's 160 KiB: 59-64 nodes with their 118-128 KiB
    // tile take 16-byte lanes only up to about 2000 entries (16 bytes each); beyond, narrower lanes (half the
    // tile, 8 bytes per entry) serve every list the encodings accept.
    if (!mixes_on_matrix_cores(n, topo.row_ptr[n])) {
        while (vec > 1 && static_cast<size_t>(n) * 64 * vec * sizeof(double) +
                              static_cast<size_t>(topo.row_ptr[n]) * (vec == 4 ? 16 : 8) > 160 * 1024)
            vec >>= 1;
    }
    if (vec == 1) head = 0;
    else head = static_cast<int64_t>((vec - ((reinterpret_cast<uintptr_t>(x) >> 2) & (vec - 1))) & (vec - 1));
    if (head > d) head = d;
    const int64_t body = ((d - head) / vec) * vec;
    const int64_t tail = d - head - body;

    auto run = [&](int v, int64_t c0, int64_t cols, uint32_t split_tiles = 0, bool by_xcd = false) {
        if (cols <= 0) return static_cast<int>(DL_OK);
        StepCall s;
        s.split_tiles = split_tiles;
        s.by_xcd = by_xcd;
        s.x = x + c0;
        s.m = m ? m + c0 : nullptr;
        s.g = static_cast<const char*>(g.p) + static_cast<size_t>(c0) * gbytes;
        s.n = n; s.d = cols; s.ld = ld; s.ldg = g.ld;
        s.gamma = gamma; s.beta = beta; s.topo = &topo; s.stream = stream;
        s.na = NormArgs{nullptr, 0, 0};
        s.batches = batches; s.batch_stride = batch_stride; s.batch_stride_g = batch_stride_g;
        if (norms) {
            // records: one per tile, with 16-byte lanes one per half tile (128 columns)
            const int tile_cols = 64 * v;
            const int tc = v == 4 ? 128 : tile_cols;
            if (norms->grids >= kMaxNormGrids) return set_error(DL_EINVAL, "step: too many launches for the per-tensor sums");
            NormGrid& gr = norms->grid[norms->grids++];
            gr.col0 = norms->col_base + c0; gr.cols = cols * batches; gr.tile0 = norms->tiles_used; gr.tc = tc;
            s.na = NormArgs{norms->partial, gr.tile0, norms->capacity};
            norms->tiles_used += (cols + tile_cols - 1) / tile_cols * (tile_cols / tc) * batches;
        }
        switch (algo) {
            case ALGO_DECENTLAM: return launch_method<ALGO_DECENTLAM>(v, g.format, norms != nullptr, s);
            case ALGO_DMSGD: return launch_method<ALGO_DMSGD>(v, g.format, norms != nullptr, s);
            case ALGO_DSGD: return launch_method<ALGO_DSGD>(v, g.format, norms != nullptr, s);
            case ALGO_AWC_DMSGD: return launch_method<ALGO_AWC_DMSGD>(v, g.format, norms != nullptr, s);
            case ALGO_DA_DMSGD: return launch_method<ALGO_DA_DMSGD>(v, g.format, norms != nullptr, s);
            default: return launch_method<ALGO_DECENTLAM_XPREV>(v, g.format, norms != nullptr, s);
        }
    };
    // Large single problems with 16-byte lanes: split tiles (see split_column) from the first column at
    // which the written array is 64 KiB-aligned, whole 64 KiB units only; what precedes is a launch
    // of its own, what follows rides along as ordinary tiles of the same launch.  (The per-tensor sums
    // need tiles that are column ranges.)  Rows that start at different offsets inside a 128-byte line
    // cannot be paired up; their launch goes out in the per-XCD order instead (step_impl.hpp).
    // (with per-tensor sums only from 2^20 columns on: where the tiles start decides the order of those sums, and below
    // that it does not depend on where the arrays lie)
    const bool large = vec == 4 && batches == 1 && body >= (norms ? kChainMinColumns : kSplitMinColumns);
    if (large && ld % 32 != 0) {
        if (int rc = run(vec, head, body, 0, true)) return rc;
    } else if (large) {
        const float* written = algo == ALGO_DECENTLAM_XPREV ? m : x;
        const uintptr_t at = reinterpret_cast<uintptr_t>(written + head) % (4u * kSplitUnit);
        const int64_t pre = at ? static_cast<int64_t>((4u * kSplitUnit - at) / 4) : 0;
        const int64_t units = (body - pre) / kSplitUnit;
        // Rows that alternate between 64 KiB boundaries and their midpoints (ld * 4 an odd multiple of
        // 32 KiB), all three arrays alike: the whole units go to the chained-tile kernel (step_chain.hip).
        const auto on_unit = [&](const void* p, size_t elem) {
            return p && (reinterpret_cast<uintptr_t>(p) + static_cast<size_t>(head + pre) * elem) % (4u * kSplitUnit) == 0;
        };
        const bool chained = ld % kSplitUnit == kSplitDistance && units > 0 && body >= kChainMinColumns && !norms && g.format == DL_GRAD_F32 &&
                             g.ld == ld && on_unit(x, 4) && on_unit(m, 4) && on_unit(g.p, 4) &&
                             chain_serves(algo, n, topo.row_ptr[n]);
        if (chained) {
            StepCall s;
            s.x = x + head + pre;
            s.m = m + head + pre;
            s.g = static_cast<const float*>(g.p) + head + pre;
            s.n = n; s.d = units * kSplitUnit; s.ld = ld; s.ldg = ld;
            s.gamma = gamma; s.beta = beta; s.topo = &topo; s.stream = stream;
            s.na = NormArgs{nullptr, 0, 0};
            s.batches = 1; s.batch_stride = 0; s.batch_stride_g = 0; s.split_tiles = 0; s.by_xcd = false;
            if (int rc = launch_chain(algo, s, static_cast<uint32_t>(units), kChainLength)) return rc;
            if (int rc = run(vec, head + pre + units * kSplitUnit, body - pre - units * kSplitUnit)) return rc;
        } else if (int rc = run(vec, head + pre, body - pre, static_cast<uint32_t>(units * kSplitTilesPerUnit))) {
            return rc;
        }
        if (int rc = run(vec, head, pre)) return rc;
    } else if (int rc = run(vec, head, body)) {   // aligned body first: it is the bulk
        return rc;
    }
    if (int rc = run(1, 0, head)) return rc;        // columns are independent, so the peeled
    if (int rc = run(1, head + body, tail)) return rc;  // head and tail are separate launches
    return DL_OK;
}

}  // namespace dl
