// Implementation shared by the translation units that instantiate the step kernel, one per method
// (the instantiations are split over several files only so that they compile in parallel).
#pragma once

#include <atomic>
#include <type_traits>

#include "device_util.hpp"
#include "internal.hpp"

namespace dl {
namespace step {

using namespace dev;

// A launch may cover `count` equally shaped sub-problems ("batches": the blocks of the blocked
// layout): consecutive workgroups walk the tiles of batch 0, then batch 1, ...
struct BatchArgs {
    int64_t stride;        // elements between consecutive batches of x and m
    int64_t stride_g;      // the same for g, in its elements
    uint32_t tiles;        // tiles per batch; 0: the launch is a single problem
    uint32_t split_tiles;  // 16-byte lanes, single problem: the first split_tiles tiles are split tiles (below)
    uint32_t by_xcd;       // single problem: workgroups of one XCD take neighbouring tiles (below)
};

// Split tiles.  Stores reach HBM fastest when a workgroup fills, row by row, both 512-byte halves of a
// pair of addresses A and A + 32 KiB inside one 64 KiB-aligned unit.  Measured with a 3-read/2-write
// stream over 32 rows about 100 MiB apart: 6.5 TB/s that way, 5.4 TB/s when a tile's 1 KiB per row is
// one piece (loads alone run at 7 TB/s either way; segments of 128 or 256 bytes, and every other
// distance from 4 KiB to 1 MiB, are slower than one piece).  Columns are independent, so a tile may
// be any set of columns: the first split_tiles tiles of a launch cover the launch's 64 KiB units
// (16384 columns) one after the other, 64 tiles per unit, tile u of a unit taking columns
// [128 u, 128 u + 128) and the same columns 8192 further on.  The launch code starts such a launch
// where the written array is 64 KiB-aligned; the rows keep that alignment if ld * 4 is a multiple of
// 64 KiB.
//
// Rows that do not all start at the same offset inside a 128-byte line (ld not a multiple of 32) cannot
// be served that way: every row piece of every tile then ends inside a line, which the neighbouring
// tile completes.  Such launches keep one piece per row and tile (half as many shared lines) and give
// the workgroups of one XCD (workgroup id mod 8) a contiguous share of the tiles, so that the two
// writers of a shared line sit behind the same L2.  Measured on 32 x 25.6 M with ld = d + 8 / d + 1000:
// 3.43 / 3.39 ms against 3.82 / 3.89 ms in the split order (aligned rows: 2.51 ms; the header recommends them).
constexpr int kSplitSegment = 128;    // columns per segment (512 bytes)
constexpr int kSplitDistance = 8192;  // columns between the two segments of a tile (32 KiB)
constexpr int kSplitUnit = 2 * kSplitDistance;
constexpr int kSplitTilesPerUnit = kSplitDistance / kSplitSegment;
__host__ __device__ inline int64_t split_column(uint32_t tile, int lane) {   // first of the lane's 4 columns
    const uint32_t unit = tile / kSplitTilesPerUnit, u = tile % kSplitTilesPerUnit;
    return static_cast<int64_t>(unit) * kSplitUnit + (lane >> 5) * kSplitDistance + u * kSplitSegment + (lane & 31) * 4;
}

// Per-launch arguments of the per-tensor sums (see NormPlan): where the tile records go.
struct NormArgs {
    double* partial;
    int64_t tile0;      // record index of this launch's tile 0
    int64_t capacity;   // records per node: node i's records start at partial + i * capacity * 3
};

// Everything a launch needs besides its template parameters.
struct StepCall {
    float* x;
    float* m;
    const void* g;
    int32_t n;
    int64_t d, ld, ldg;
    double gamma, beta;
    const PhaseArgs* topo;
    hipStream_t stream;
    NormArgs na;
    int64_t batches, batch_stride, batch_stride_g;   // batches == 1: a single problem
    uint32_t split_tiles;                            // see BatchArgs
    bool by_xcd;                                     // see BatchArgs
};


// Dense mixing on the matrix cores (mix_dense below): constants and the two host-checkable functions.
constexpr int kDensePad = 16;
constexpr int kDenseRows = 32;   // rows of the padded problem: two 16-row blocks, eight groups of four ...
constexpr int kDenseRowsMax = 48;   // ... or three blocks and twelve groups (33-48 nodes, three rows per thread)
// Where element (i, k) of W sits in its LDS array, in doubles: per block of 16 rows, sixteen slabs (one
// per pair of columns) of 16 rows x 2 columns, two doubles of padding after each.  With the padding
// both access patterns are free of bank conflicts: a wave that writes one row of W (lane = column)
// touches 32 different 8-byte banks, and so does a half-wave that reads an A operand (16 rows x
// 2 columns of one slab).  (Without it the row writes were 16-way conflicts: 42 % of the kernel's LDS
// cycles, measured.)
constexpr int kDenseSlab = 2 * 16 + 2;
__host__ __device__ constexpr int dense_w_doubles(int rows) { return (rows / 16) * (rows / 2) * kDenseSlab; }
__host__ __device__ constexpr int dense_w_at(int i, int k, int rows = kDenseRows) {
    return (i >> 4) * (rows / 2) * kDenseSlab + (k >> 1) * kDenseSlab + (i & 15) * 2 + (k & 1);
}
constexpr int kDenseWDoubles = dense_w_doubles(kDenseRows);
// Where the matrix cores (mix_dense) beat the gather, measured with DecentLaM on c3-sized arrays
// (n x d = 819 M elements) and circulant graphs: the product costs the same at any density but more
// per byte the fewer rows a tile has (32 / 28 / 24 / 20 nodes: 2.70 / 2.95 / 3.22 / 3.32 ms), the
// gather grows with the entries per row (32 nodes: 2.61 / 2.74 / 2.93 / 3.50 ms at 13 / 14 / 20 / 32;
// 28 nodes: 2.89 / 3.00 / 3.53 at 16 / 18 / 28; 24 nodes: 3.22 / 3.34 / 3.46 at 20 / 22 / 24; 20 nodes:
// 3.21 at 20).  The two cross at about 46 - n entries per row: 14 at 32 nodes, 18 at 28, 22 at 24,
// never below 23 nodes.
// Three row blocks (33-48 nodes, one workgroup per CU), same arrays: the product takes 4.25 / 4.0 / 3.6 ms
// at 36 / 40 / 48 nodes, the gather 3.85 / 3.75 / 3.5 ms at 23 entries per row, 4.2 / 4.1 / 3.9 at 28 and
// 4.9 / 5.2 / 5.5 at all-to-all: they cross at about 38 - n / 4 entries per row (26 at 48 nodes, 28 at 40,
// 29 at 36).
inline bool mixes_on_matrix_cores(int n, int nnz) {
    if (n > kDenseRows) return n <= kDenseRowsMax && 4 * nnz >= (152 - n) * n;
    return n > 16 && nnz >= (46 - n) * n;
}

// Launch the kernel of one method for the given vector width, gradient format and sums option
// (defined in step_<method>.hip).
template <int ALGO>
int launch_method(int vec, int format, bool norms, const StepCall& s);

// Chained split tiles for rows that alternate between 64 KiB boundaries and their midpoints (step_chain.hip):
// whether that kernel serves this method, node count and graph, and its launch over `units` whole 64 KiB
// units of columns starting at s.x / s.m / s.g (row 0 of each on a 64 KiB boundary, fp32 gradients with the
// row stride of x), `len` units per workgroup.
bool chain_serves(int algo, int32_t n, int nnz);
int launch_chain(int algo, const StepCall& s, uint32_t units, uint32_t len);

// Two LDS passes under split tiles for 33-128 nodes (step_tall.hip): whether that kernel serves this method, node
// count and graph, and its launch over `units` whole 64 KiB units of columns starting at s.x / s.m / s.g (row 0 of
// x on a 64 KiB boundary, s.ld a multiple of 128, every array 16-byte aligned, fp32 gradients); or, with
// s.batch_stride != 0 (blocked layout), over s.batches sub-problems of s.d columns each (s.d a multiple of 256,
// `units` unused).
bool tall_serves(int algo, int32_t n, int nnz, int gformat);
int launch_tall(int algo, const StepCall& s, uint32_t units, int gformat);

#ifdef DL_STEP_KERNEL_IMPL
namespace {

// Position of a lane's v-th column inside a row of the LDS tile, in doubles, relative to the lane's
// base (lane * 2 with two or more columns per lane, else lane): a row is kept as VEC / 2 planes of 64
// pairs of doubles (columns 2p and 2p + 1 of every lane side by side), so that a lane reads and writes
// 16 bytes at a time (ds_read_b128 / ds_write_b128) and a wave's access is 1 KiB of consecutive
// addresses: free of bank conflicts.  With a lane's VEC columns all side by side (32-byte groups per
// lane) 71 % of the LDS cycles were bank conflicts (measured) and the kernel was LDS-bound at 2.6 ms on
// the headline workload whatever the traffic.  Planes of single doubles (8-byte accesses) are equally
// conflict-free but issue twice the instructions: from about ten neighbours per row on, where the LDS
// reads start to show, the 16-byte form measured 2-15 % faster (32 nodes, 10 / 16 / 32 entries per row:
// 2.57 / 2.78 / 3.53 ms against 2.62 / 2.91 / 4.14).
__device__ __forceinline__ constexpr int lds_col(int v) { return (v >> 1) * 128 + (v & 1); }
typedef double vd2 __attribute__((ext_vector_type(2)));

// The palette index of a row in the one-weight-per-row form of the neighbour list, for a uniform row: a
// word load and a shift, because there are no scalar byte loads and a vector load from the kernel
// arguments would be waited for together with every row load before it.
__device__ __forceinline__ unsigned row_palette_index(const PhaseArgs& topo, int row) {
    return (topo.rows.widx_words[row >> 2] >> (8 * (row & 3))) & 0xffu;
}

// One neighbour in the LDS table.  Lanes of 16 bytes (up to 64 nodes) read the 16-byte form with one
// access; the narrower lanes (65 nodes and more, where the fp64 tile already takes 128 KiB) use the
// 8-byte form and widen the weight when they use it, so that graphs of up to DL_MAX_NNZ_ROW_WEIGHTS
// entries still fit the LDS beside the tile.
struct alignas(16) Neighbour {
    double w;     // w_ij, promoted exactly from fp32
    int offset;   // j * TC: start of row j in the LDS tile, in doubles
    int unused;
    __device__ __forceinline__ void set(float weight, int at) { w = static_cast<double>(weight); offset = at; unused = 0; }
    __device__ __forceinline__ double weight() const { return w; }
};
struct alignas(8) NeighbourCompact {
    float w;
    int offset;
    __device__ __forceinline__ void set(float weight, int at) { w = weight; offset = at; }
    __device__ __forceinline__ double weight() const { return static_cast<double>(w); }
};
template <int VEC>
using NeighbourFor = typename std::conditional<VEC == 4, Neighbour, NeighbourCompact>::type;

// z += sum over K consecutive table entries; all K table reads, then all K tile reads, are
// issued before the first multiply-add so their latencies overlap.
template <int VEC, int K>
__device__ __forceinline__ void gather(const NeighbourFor<VEC>* __restrict__ entry,
                                       const double* __restrict__ tile_at_lane, double (&z)[VEC]) {
    NeighbourFor<VEC> nb[K];
#pragma unroll
    for (int t = 0; t < K; ++t) nb[t] = entry[t];
    double u[K][VEC];
#pragma unroll
    for (int t = 0; t < K; ++t) {
        if constexpr (VEC >= 2) {
#pragma unroll
            for (int v = 0; v < VEC; v += 2) {
                const vd2 pair = *reinterpret_cast<const vd2*>(tile_at_lane + nb[t].offset + lds_col(v));
                u[t][v] = pair.x;
                u[t][v + 1] = pair.y;
            }
        } else {
            u[t][0] = tile_at_lane[nb[t].offset];
        }
    }
#pragma unroll
    for (int t = 0; t < K; ++t) {   // list order, one fused multiply-add per term
#pragma unroll
        for (int v = 0; v < VEC; ++v) z[v] = __builtin_fma(nb[t].weight(), u[t][v], z[v]);
    }
}

// Dense W (up to 48 nodes, most pairs neighbours; see mixes_on_matrix_cores): the mixing of a tile is the fp64 contraction
// Z[32 x TC] = W[32 x 32] * U[32 x TC] (48 x 48 for 33-48 nodes: three blocks of 16 rows where this text says
// two), and it runs on the matrix cores (v_mfma_f64_16x16x4_f64)
// instead of |N_i| LDS gathers per row.  Wave w owns the 16 positions [16 w, 16 w + 16) of every
// tile row: for each of the eight groups of four rows it reads its 4 x 16 block of U as the B
// operand (lane l: row l / 16 of the group, position l % 16), multiplies it with the two 16 x 4
// blocks of W kept in LDS (lane l: row l % 16, column l / 16 of the block; see dense_w_at) and, when
// all products are in, writes its 32 x 16 block of Z over U: it alone read those positions, so no
// barrier separates the two.  The result registers of the instruction hold rows l / 16 + 4 r
// (r = 0..3) of column l % 16 (layout checked on the device).  Tile rows are kDensePad doubles longer than
// the tile is wide so that the four rows of an operand read fall into different LDS banks.
// Sums run in the instruction's order, not in list order: fp64 rounding differs in the last bits, far
// inside the fp32 rounding of the result.  A zero weight multiplies its node's value like any other,
// so a non-finite value in one node's column reaches every node of that column, neighbour or not.
typedef double vd4 __attribute__((ext_vector_type(4)));
template <int STRIDE, int RB>
__device__ __forceinline__ void mix_dense(double* __restrict__ tile, const double* __restrict__ w_operands, int n, int wave,
                                          int lane) {
    constexpr int ROWS = 16 * RB;
    double* mine = tile + (lane >> 4) * STRIDE + 16 * wave + (lane & 15);
    const double* a_at = w_operands + dense_w_at(lane & 15, lane >> 4, ROWS);   // + dense_w_at(16 rb, 4 s) per operand
    // one named accumulator per row block (an array of them made the compiler copy all of them after
    // every step, each copy waiting for its instruction to finish: 2.88 instead of 2.66 ms at 32 nodes)
    vd4 acc0 = {0.0, 0.0, 0.0, 0.0}, acc1 = {0.0, 0.0, 0.0, 0.0}, acc2 = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int s = 0; s < ROWS / 4; ++s) {
        if (4 * s < n) {   // uniform; rows from n on hold zeros, whole groups of them are skipped
            const double b = mine[4 * s * STRIDE];
            acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a_at[dense_w_at(0, 4 * s, ROWS)], b, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a_at[dense_w_at(16, 4 * s, ROWS)], b, acc1, 0, 0, 0);
            if constexpr (RB == 3)
                acc2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a_at[dense_w_at(32, 4 * s, ROWS)], b, acc2, 0, 0, 0);
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        mine[4 * r * STRIDE] = acc0[r];
        mine[(16 + 4 * r) * STRIDE] = acc1[r];
        if constexpr (RB == 3) mine[(32 + 4 * r) * STRIDE] = acc2[r];
    }
}

// After the barrier all waves of a workgroup gather, compute and store at the same moment, and the
// memory system sees the workgroup's 64 KiB of stores as one burst.  Letting the odd-numbered waves
// (SIMDs 1 and 3) begin that phase 32-48 x 64 cycles later measured 4-8 % faster while the kernel
// still stalled on vector loads after the barrier; since it does not, the pause is worth about 1 %
// (2.50 against 2.52 ms on the 32-node headline workload, both layouts) and is kept where it was
// measured: 16-byte lanes up to 32 nodes, every form that moves 14 B per node-element or more.  Off
// where it measured neutral or harmful: DSGD (12 B), 64 nodes and more, the 16-wave single-row shape
// with less than 20 B, the variants with per-tensor sums.
template <int VEC, int RPT, int WAVES, int ALGO, int GF, bool NORMS, bool DENSE>
constexpr int stagger_units() {
    if (DENSE || NORMS || VEC != 4 || ALGO == ALGO_DSGD || ALGO == ALGO_DA_DMSGD) return 0;
    const bool twenty_bytes = ALGO != ALGO_DECENTLAM_XPREV && GF == DL_GRAD_F32;
    if (RPT == 2 && WAVES == 16) return twenty_bytes ? 48 : 32;
    if (RPT == 1 && WAVES == 16) return twenty_bytes ? 32 : 0;
    if (RPT == 1 && WAVES <= 8) return 32;
    return 0;
}

// VEC    columns per lane (width of the global accesses: 4, 8 or 16 bytes)
// RPT    rows per thread; WAVES wavefronts per workgroup: the kernel covers n <= WAVES * RPT nodes
// ALGO   ALGO_DECENTLAM, ALGO_DMSGD, ALGO_DSGD (x <- W (x - gamma g); m is not touched) or
//        ALGO_DECENTLAM_XPREV: DecentLaM in its momentum-free form (appendix "Reformulation of
//        DecentLaM"), x_next = W (x - gamma g) + beta' (x - x_prev); here `m` is the buffer that
//        holds x_prev on entry and x_next on exit, x is only read, and `beta` carries
//        beta' = beta * gamma / gamma_prev: 16 bytes per node-element, one written array;
//        ALGO_AWC_DMSGD (m <- beta m + g; x <- W x - gamma m: the tile holds x) and ALGO_DA_DMSGD
//        (mh = beta m + g; x <- W (x - gamma mh); m <- W mh: the tile holds h, then mh, each gathered)
// GF     dl_grad_format of g;  NORMS: accumulate the per-tensor sums of squares
// DENSE  mix on the matrix cores (see mix_dense): 16-byte lanes, 16 waves with two rows per thread
//        (17-32 nodes, used from 23 on) or three (33-48 nodes)
template <int VEC, int RPT, int WAVES, int ALGO, int GF, bool NORMS, bool DENSE = false>
__global__ __launch_bounds__(64 * WAVES) void k_step(float* __restrict__ x, float* __restrict__ m,
                                                      const typename GradElem<GF>::type* __restrict__ g,
                                                      int64_t d, int64_t ld, int64_t ldg,
                                                      double gamma, double inv_gamma, double beta,
                                                      const BatchArgs batch, const NormArgs na,
                                                      const PhaseArgs topo) {
    constexpr int TC = 64 * VEC;
    static_assert(!DENSE || (VEC == 4 && (RPT == 2 || RPT == 3) && WAVES == 16), "dense mixing: two shapes");
    constexpr int DROWS = 16 * RPT;   // DENSE: rows of the padded problem
    constexpr int STRIDE = DENSE ? TC + kDensePad : TC;   // doubles from one tile row to the next
    // tile [n][TC] of u_j (DecentLaM) or h_j (DmSGD), then the table; DENSE: [32][STRIDE], then W as operands
    extern __shared__ __attribute__((aligned(16))) double lds[];
    const int n = topo.n;
    using Entry = NeighbourFor<VEC>;
    Entry* table = reinterpret_cast<Entry*>(lds + n * TC);
    double* w_operands = lds + DROWS * STRIDE;   // DENSE: W, laid out by dense_w_at

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t tile = blockIdx.x;
    if (batch.by_xcd) {   // XCD x = workgroup id mod 8 walks its own contiguous share of the tiles
        const uint32_t q = gridDim.x / 8, r = gridDim.x % 8, xcd = blockIdx.x % 8;
        tile = xcd * q + (xcd < r ? xcd : r) + blockIdx.x / 8;
    }
    if (batch.tiles) {   // uniform: which sub-problem, which of its tiles
        const uint32_t b = tile / batch.tiles;
        tile -= b * batch.tiles;
        x += b * batch.stride;
        if constexpr (ALGO != ALGO_DSGD) m += b * batch.stride;
        g += b * batch.stride_g;
    }
    // First column of the tile (uniform) and the lane's offset inside it; see split_column.
    int64_t tile_col = static_cast<int64_t>(tile) * TC;
    int lane_col = lane * VEC;
    if constexpr (VEC == 4) {
        if (tile < batch.split_tiles) {   // uniform over the workgroup
            tile_col = split_column(tile, 0);
            lane_col = static_cast<int>(split_column(0, lane));
        }
    }
    const int64_t c = tile_col + lane_col;
    const bool live = c < d;  // d is a multiple of VEC for this launch

    // Neighbour list: kernel arguments -> LDS table, one entry per thread and round.  In the direct
    // form the first round's two loads go out here, ahead of the rows, and are used once the rows
    // are on their way.
    const uint32_t last_pair = topo.row_ptr_pairs[n >> 1];   // uniform: a scalar load
    const int nnz = (n & 1) ? last_pair >> 16 : last_pair & 0xffffu;
    const bool direct = topo.palette == 0;   // uniform over the grid
    const int e_mine = threadIdx.x;
    // (no branch around these two loads, or they would be waited for at its end; in the palette form
    // they read bytes of the other encoding, which nobody uses)
    const int e_safe = !DENSE && e_mine < nnz && e_mine < DL_MAX_NNZ ? e_mine : 0;
    const unsigned col_mine = topo.direct.col[e_safe];
    const float w_mine = topo.direct.w[e_safe];
    // DENSE: lane l of a wave takes entry l of each of the wave's rows; the palette rides along, one
    // value per lane
    const float palette_mine = topo.pal.value[DENSE ? lane : 0];
    // ---- phase 1: stream rows in.  Every load is issued before anything waits for one: rows and
    // lanes beyond the problem read the tile's first column of row 0 instead (in bounds, never used),
    // so that no load sits inside a branch, and the row bases are uniform (scalar address
    // arithmetic, one vector register of offsets for all loads).
    float xr[RPT][VEC], mr[RPT][VEC], gr[RPT][VEC];
    // NORMS: sums of squares that are complete before the barrier (g; the new m of DmSGD), reduced
    // over the wave right away and kept as scalars so that they cost no vector registers later
    // With 16-byte lanes the sums are kept per half of the tile (lanes 0-31 and 32-63: 128 columns each,
    // contiguous also in a split tile), so a record always covers one 128-column range.
    constexpr int H = (NORMS && VEC == 4) ? 2 : 1;
    double early[RPT][H][2];
    const int safe_col = live ? lane_col : 0;
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int i = wave + WAVES * r;
        const int64_t row = i < n ? i : 0;   // uniform
        load_vec<VEC>(x + (row * ld + tile_col) + safe_col, xr[r]);
        load_grad<VEC, GF>(g + (row * ldg + tile_col) + safe_col, gr[r]);
        if constexpr (ALGO != ALGO_DSGD) load_vec<VEC>(m + (row * ld + tile_col) + safe_col, mr[r]);
    }
    // This wave's slices of the neighbour list (uniform, hence scalar loads): fetched now, used
    // after the barrier, where a vector load from the kernel arguments would first wait for the
    // stores of the row before it (loads and stores share one in-order counter).
    int e_begin[RPT], e_end[RPT];
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int i = wave + WAVES * r;
        const int row = i < n ? i : 0;
        const uint32_t lo = topo.row_ptr_pairs[row >> 1], hi = topo.row_ptr_pairs[(row + 1) >> 1];   // two offsets per word
        e_begin[r] = (row & 1) ? lo >> 16 : lo & 0xffffu;
        e_end[r] = (row & 1) ? hi & 0xffffu : hi >> 16;
    }
    // DENSE: a wave writes rows i and i + 16 of W into the operand array, zeros first, then its
    // entries (LDS writes of one wave land in program order).
    unsigned dense_col[RPT], dense_widx[RPT];
    float dense_w[RPT];
    if constexpr (DENSE) {
#pragma unroll
        for (int r = 0; r < RPT; ++r) {
            const int e = e_begin[r] + lane;
            const int e_row = e < e_end[r] ? e : 0;   // all encodings keep their columns in the same bytes
            dense_col[r] = topo.rows.col[e_row];
            dense_widx[r] = topo.pal.widx[topo.palette == 1 ? e_row : 0];
            dense_w[r] = topo.direct.w[direct ? e_row : 0];
        }
    }
    if (!DENSE && direct && e_mine < nnz) {
        Entry t;
        t.set(w_mine, static_cast<int>(col_mine) * TC);
        table[e_mine] = t;
    }
    if (!DENSE && topo.palette == 2) {   // one weight per row: every wave writes the entries of its rows
#pragma unroll
        for (int r = 0; r < RPT; ++r) {
            const int i = wave + WAVES * r;
            if (i < n) {
                const float w_row = topo.rows.value[row_palette_index(topo, i)];
                for (int e = e_begin[r] + lane; e < e_end[r]; e += 64) {
                    Entry t;
                    t.set(w_row, static_cast<int>(topo.rows.col[e]) * TC);
                    table[e] = t;
                }
            }
        }
    }
    const int e_first = (DENSE || topo.palette == 2) ? nnz : (direct ? e_mine + 64 * WAVES : e_mine);
    for (int e = e_first; e < nnz; e += 64 * WAVES) {   // later rounds of the direct form; palette form
        Entry t;
        if (direct) t.set(topo.direct.w[e], static_cast<int>(topo.direct.col[e]) * TC);
        else t.set(topo.pal.value[topo.pal.widx[e]], static_cast<int>(topo.pal.col[e]) * TC);
        table[e] = t;
    }
    // local pre-step, parked in LDS
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int i = wave + WAVES * r;
        double sq_g = 0.0, sq_m = 0.0;   // this lane's share (NORMS)
        if constexpr (DENSE) {
            // row i of W: zeros, then the entries of the list
            double* w_row = w_operands + dense_w_at(i, 0, DROWS);
            if (lane < DROWS) w_row[dense_w_at(0, lane, DROWS)] = 0.0;
            // the weight: its own (direct), by the entry's palette index, or by the row's (the palettes of the
            // two forms sit in the same bytes)
            unsigned widx = dense_widx[r];
            if (topo.palette == 2) widx = row_palette_index(topo, i < n ? i : 0);   // uniform
            const float from_palette = __shfl(palette_mine, static_cast<int>(widx & 63u));
            if (i < n && e_begin[r] + lane < e_end[r]) {
                const unsigned k = dense_col[r];
                w_row[dense_w_at(0, static_cast<int>(k), DROWS)] = static_cast<double>(direct ? dense_w[r] : from_palette);
            }
            if (i >= n) {   // uniform: a row of the padding, all zeros
                double* pad = lds + i * STRIDE + lane * 2;
#pragma unroll
                for (int v = 0; v < VEC; ++v) pad[lds_col(v)] = 0.0;
            }
        }
        if (i < n) {   // uniform; lanes beyond the problem work on the stand-in column and store nothing
            double* slot = lds + i * STRIDE + lane * (VEC >= 2 ? 2 : 1);
            if constexpr (NORMS) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const double gv = static_cast<double>(gr[r][v]);
                    sq_g = __builtin_fma(gv, gv, sq_g);
                }
            }
            if constexpr (ALGO == ALGO_AWC_DMSGD) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) slot[lds_col(v)] = static_cast<double>(xr[r][v]);
            } else if constexpr (ALGO == ALGO_DA_DMSGD) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) {   // h_j now; mh_j takes the tile over later
                    const double mh = beta * static_cast<double>(mr[r][v]) + static_cast<double>(gr[r][v]);
                    slot[lds_col(v)] = static_cast<double>(xr[r][v]) - gamma * mh;
                }
            } else if constexpr (ALGO != ALGO_DMSGD) {
#pragma unroll
                for (int v = 0; v < VEC; ++v)
                    slot[lds_col(v)] = static_cast<double>(xr[r][v]) - gamma * static_cast<double>(gr[r][v]);
            } else {
                float mn[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const double m_new = beta * static_cast<double>(mr[r][v]) + static_cast<double>(gr[r][v]);
                    mn[v] = static_cast<float>(m_new);
                    slot[lds_col(v)] = static_cast<double>(xr[r][v]) - gamma * m_new;
                    if constexpr (NORMS) {
                        const double mv = static_cast<double>(mn[v]);
                        sq_m = __builtin_fma(mv, mv, sq_m);
                    }
                }
                // the new m waits in the registers of the old one and is stored together with x
                // after the barrier: one burst of stores per row measures faster than two
#pragma unroll
                for (int v = 0; v < VEC; ++v) mr[r][v] = mn[v];
            }
        }
        if constexpr (NORMS) {
            if (!live) sq_g = sq_m = 0.0;
            if (i < n) {   // wave-uniform: all 64 lanes take part
                if constexpr (ALGO == ALGO_DMSGD) {
                    const double both = H == 2 ? half_sum2(sq_g, sq_m, lane) : wave_sum2(sq_g, sq_m, lane);   // even lanes: g, odd: m
                    const double other = dpp_f64<0xB1>(both);
                    early[r][0][0] = uniform_f64(both);
                    early[r][0][1] = uniform_f64(other);
                    if constexpr (H == 2) {
                        early[r][1][0] = lane_f64<32>(both);
                        early[r][1][1] = lane_f64<32>(other);
                    }
                } else {
                    const double sg = H == 2 ? half_sum(sq_g) : wave_sum(sq_g);
                    early[r][0][0] = uniform_f64(sg);
                    if constexpr (H == 2) early[r][1][0] = lane_f64<32>(sg);
                }
            }
        }
    }
    // Every load has returned on every path from here on: said explicitly, or the compiler, unsure
    // about paths that skipped a row, makes the second row's stores wait for the first row's
    // (loads and stores share one in-order counter).
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), nothing else
    __syncthreads();
    // Odd waves start their second phase a little later (see stagger_units).
    constexpr int kStagger = stagger_units<VEC, RPT, WAVES, ALGO, GF, NORMS, DENSE>();
    if constexpr (kStagger > 0) {
        if (wave & 1) __builtin_amdgcn_s_sleep(kStagger);
    }

    // ---- phase 2: gather-mix from LDS, finish the update, store in place
    const double* tile_at_lane = lds + lane * (VEC >= 2 ? 2 : 1);
    if constexpr (DENSE) {
        mix_dense<STRIDE, RPT>(lds, w_operands, n, wave, lane);
        __syncthreads();   // the tile now holds Z = W U
    }
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int i = wave + WAVES * r;
        double sq_m = 0.0, sq_x = 0.0;   // this lane's share (NORMS)
        if (i < n) {
            double z[VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) z[v] = 0.0;
            int e = e_begin[r];
            const int e1 = e_end[r];
            if constexpr (DENSE) {   // the tile already holds z
#pragma unroll
                for (int v = 0; v < VEC; v += 2) {
                    const vd2 pair = *reinterpret_cast<const vd2*>(tile_at_lane + i * STRIDE + lds_col(v));
                    z[v] = pair.x;
                    z[v + 1] = pair.y;
                }
                e = e1;
            }
            // groups of 4 (2 for 16-byte lanes: eight fp64 values in flight; the kernel must stay within
            // 64 VGPRs for two 1024-thread workgroups per CU; groups of 3 measured the same, of 4 slower),
            // then 2, then 1
            else if constexpr (VEC < 4) {
                for (; e + 4 <= e1; e += 4) gather<VEC, 4>(table + e, tile_at_lane, z);
                if (e + 2 <= e1) {
                    gather<VEC, 2>(table + e, tile_at_lane, z);
                    e += 2;
                }
            } else {
                for (; e + 2 <= e1; e += 2) gather<VEC, 2>(table + e, tile_at_lane, z);
            }
            for (; e < e1; ++e) gather<VEC, 1>(table + e, tile_at_lane, z);

            const int64_t at = (static_cast<int64_t>(i) * ld + tile_col) + lane_col;   // uniform base + lane offset
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
                    if constexpr (NORMS) {
                        const double mv = static_cast<double>(mo[v]);
                        sq_m = __builtin_fma(mv, mv, sq_m);
                    }
                }
                if (live) store_vec<VEC>(m + at, mo);
            } else if constexpr (ALGO == ALGO_DECENTLAM_XPREV) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const double diff = static_cast<double>(xr[r][v]) - static_cast<double>(mr[r][v]);
                    xo[v] = static_cast<float>(__builtin_fma(beta, diff, z[v]));
                }
            } else if constexpr (ALGO == ALGO_AWC_DMSGD) {
                float mo[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const double m_new = beta * static_cast<double>(mr[r][v]) + static_cast<double>(gr[r][v]);
                    mo[v] = static_cast<float>(m_new);
                    xo[v] = static_cast<float>(z[v] - gamma * m_new);
                    if constexpr (NORMS) {
                        const double mv = static_cast<double>(mo[v]);
                        sq_m = __builtin_fma(mv, mv, sq_m);
                    }
                }
                if (live) store_vec<VEC>(m + at, mo);
            } else {   // DSGD, DmSGD; DA-DmSGD: x is done, its momentum follows below
#pragma unroll
                for (int v = 0; v < VEC; ++v) xo[v] = static_cast<float>(z[v]);
                if constexpr (ALGO == ALGO_DMSGD) {
                    if (live) store_vec<VEC>(m + at, mr[r]);
                }
            }
            if (live) store_vec<VEC>((ALGO == ALGO_DECENTLAM_XPREV ? m : x) + at, xo);
            if constexpr (NORMS) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const double xv = static_cast<double>(xo[v]);
                    sq_x = __builtin_fma(xv, xv, sq_x);
                }
            }
        }
        // sums of squares: one record of 3 doubles (g, new m, new x) per row and tile, with 16-byte
        // lanes per row and half tile; records are numbered by the columns they cover (column / 128
        // of the launch, or tile index); lanes beyond the launch contribute zeros
        if constexpr (NORMS) {
            if (!live) sq_m = sq_x = 0.0;
            if (i < n) {
                int64_t record = blockIdx.x;
                if constexpr (H == 2) {
                    record = batch.tiles ? 2 * static_cast<int64_t>(blockIdx.x) : tile_col / 128;
                    if (lane >= 32) record += lane_col >= kSplitDistance ? kSplitDistance / 128 : 1;
                }
                double* rec = na.partial + (i * na.capacity + na.tile0 + record) * 3;
                const bool upper = H == 2 && lane >= 32;
                const int hl = H == 2 ? lane & 31 : lane;
                const double e0 = upper ? early[r][H - 1][0] : early[r][0][0];
                if constexpr (ALGO == ALGO_DMSGD) {
                    const double e1 = upper ? early[r][H - 1][1] : early[r][0][1];
                    const double sx = H == 2 ? half_sum(sq_x) : wave_sum(sq_x);
                    if (hl < 3) rec[hl] = hl == 0 ? e0 : (hl == 1 ? e1 : sx);
                } else {
                    const double mx = H == 2 ? half_sum2(sq_m, sq_x, lane) : wave_sum2(sq_m, sq_x, lane);   // even lanes: m, odd: x
                    if (hl < 3) rec[(hl + 1) % 3] = hl == 2 ? e0 : mx;
                }
            }
        }
    }
    // DA-DmSGD, second partial average: the same tile is used again for mh_j = beta m_j + g_j (recomputed
    // from the registers), so that the fp64 tile stays at 64 KiB and two workgroups share a CU.
    if constexpr (ALGO == ALGO_DA_DMSGD) {
        __syncthreads();   // every wave has finished gathering h
#pragma unroll
        for (int r = 0; r < RPT; ++r) {
            const int i = wave + WAVES * r;
            if (i < n) {
                double* slot = lds + i * STRIDE + lane * (VEC >= 2 ? 2 : 1);
#pragma unroll
                for (int v = 0; v < VEC; ++v)
                    slot[lds_col(v)] = beta * static_cast<double>(mr[r][v]) + static_cast<double>(gr[r][v]);
            } else if constexpr (DENSE) {   // a row of the padding: zeros again
                double* pad = lds + i * STRIDE + lane * 2;
#pragma unroll
                for (int v = 0; v < VEC; ++v) pad[lds_col(v)] = 0.0;
            }
        }
        __syncthreads();
        if constexpr (DENSE) {
            mix_dense<STRIDE, RPT>(lds, w_operands, n, wave, lane);
            __syncthreads();
        }
#pragma unroll
        for (int r = 0; r < RPT; ++r) {
            const int i = wave + WAVES * r;
            if (i < n) {
                double zm[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) zm[v] = 0.0;
                int e = e_begin[r];
                const int e1 = e_end[r];
                if constexpr (DENSE) {
#pragma unroll
                    for (int v = 0; v < VEC; v += 2) {
                        const vd2 pair = *reinterpret_cast<const vd2*>(tile_at_lane + i * STRIDE + lds_col(v));
                        zm[v] = pair.x;
                        zm[v + 1] = pair.y;
                    }
                    e = e1;
                }
                for (; e + 2 <= e1; e += 2) gather<VEC, 2>(table + e, tile_at_lane, zm);
                for (; e < e1; ++e) gather<VEC, 1>(table + e, tile_at_lane, zm);
                float mo[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) mo[v] = static_cast<float>(zm[v]);
                if (live) store_vec<VEC>(m + ((static_cast<int64_t>(i) * ld + tile_col) + lane_col), mo);
                if constexpr (NORMS) {   // the record's second slot, left at zero by the first gather: the sum of the new m
                    double sq = 0.0;
#pragma unroll
                    for (int v = 0; v < VEC; ++v) sq = __builtin_fma(static_cast<double>(mo[v]), static_cast<double>(mo[v]), sq);
                    if (!live) sq = 0.0;
                    const double sm = H == 2 ? half_sum(sq) : wave_sum(sq);
                    int64_t record = blockIdx.x;
                    if constexpr (H == 2) {
                        record = batch.tiles ? 2 * static_cast<int64_t>(blockIdx.x) : tile_col / 128;
                        if (lane >= 32) record += lane_col >= kSplitDistance ? kSplitDistance / 128 : 1;
                    }
                    if ((H == 2 ? lane & 31 : lane) == 0) na.partial[(i * na.capacity + na.tile0 + record) * 3 + 1] = sm;
                }
            }
        }
    }
}

// More than 48 KiB of dynamic LDS takes a function attribute: set once per kernel instantiation and device to the
// most this chip has (the call costs about 2 us, a fifth of a small step).  The one thing the library remembers
// between calls is that this has been done (a bit per kernel variant and device, the header says so: `configured`
// is a static of the calling instantiation); devices with ordinal 64 and up set it at every launch.
inline int allow_large_lds(const void* kernel, std::atomic<uint64_t>& configured) {
    int device = 0;
    if (int rc = check_hip(hipGetDevice(&device), "hipGetDevice")) return rc;
    const uint64_t bit = device >= 0 && device < 64 ? uint64_t{1} << device : uint64_t{0};
    if (!(configured.load(std::memory_order_relaxed) & bit) || bit == 0) {
        if (int rc = check_hip(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024),
                               "hipFuncSetAttribute(max dynamic LDS)"))
            return rc;
        configured.fetch_or(bit, std::memory_order_relaxed);
    }
    return DL_OK;
}

size_t lds_bytes_for(int32_t n, int vec, int nnz, int tiles) {
    const size_t entry = vec == 4 ? sizeof(Neighbour) : sizeof(NeighbourCompact);
    return static_cast<size_t>(tiles) * n * 64 * vec * sizeof(double) + static_cast<size_t>(nnz) * entry;
}

template <int VEC, int RPT, int WAVES, int ALGO, int GF, bool NORMS, bool DENSE = false>
int launch_variant(const StepCall& s) {
    constexpr int TC = 64 * VEC;
    const size_t lds_bytes = DENSE ? (static_cast<size_t>(16 * RPT) * (TC + kDensePad) + dense_w_doubles(16 * RPT)) * sizeof(double)
                                   : lds_bytes_for(s.n, VEC, s.topo->row_ptr[s.n], 1);
    auto kernel = k_step<VEC, RPT, WAVES, ALGO, GF, NORMS, DENSE>;
    if (lds_bytes > 160 * 1024)
        return set_error(DL_ETOPO, "step: n = %d with %d entries needs %zu bytes of LDS, a CU has 163840", s.n,
                         static_cast<int>(s.topo->row_ptr[s.n]), lds_bytes);
    if (lds_bytes > 48 * 1024) {
        static std::atomic<uint64_t> configured{0};   // one bit per device ordinal below 64
        if (int rc = allow_large_lds(reinterpret_cast<const void*>(kernel), configured)) return rc;
    }
    const int64_t tiles = (s.d + TC - 1) / TC;
    const int64_t blocks = tiles * s.batches;
    if (blocks > 0x7fffffffLL) return set_error(DL_EINVAL, "step: d too large for one launch");
    const BatchArgs batch{s.batch_stride, s.batch_stride_g, s.batches > 1 ? static_cast<uint32_t>(tiles) : 0u,
                          VEC == 4 && s.batches == 1 ? s.split_tiles : 0u, s.batches == 1 && s.by_xcd ? 1u : 0u};
    hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(blocks)), dim3(64 * WAVES), lds_bytes, s.stream,
                       s.x, s.m, static_cast<const typename GradElem<GF>::type*>(s.g), s.d, s.ld, s.ldg,
                       s.gamma, 1.0 / s.gamma, s.beta, batch, s.na, *s.topo);
    return check_hip(hipGetLastError(), "step kernel launch");
}

// Workgroup shape by node count: as many waves as rows up to 8 nodes, two rows per thread up to 32, then
// more rows per thread.  The fp64 tile may take up to 128 KiB of LDS, see widest_vec_for.  Measured on
// arrays of 819 M elements (DecentLaM, ring, 16-byte lanes), TB/s of the 20 B per node-element:
//   9-16 nodes    8 waves x 2 rows (four workgroups per CU) against 16 x 1 (two, with idle waves below 16
//                 nodes): 6.1 / 6.3 / 6.5 against 5.5 / 5.9 / 6.05 at 9 / 12 / 16 nodes
//   17-24 nodes   10 x 2 and 12 x 2 against 16 x 2: 6.2 / 6.4 / 6.3 / 6.5 against 5.65 / 5.8 / 6.0 / 6.0 at
//                 17 / 20 / 22 / 24 nodes (14 x 2 for 25-28 nodes measured worse than 16 x 2: 14 waves do
//                 not spread evenly over four SIMDs)
//   33-48 nodes   16 x 3 against 16 x 4 (whose fourth row slot loads a stand-in row): 6.1 / 5.9 / 6.05 against
//                 5.8 / 5.6 / 5.75 at 36 / 40 / 48 nodes
//   65-96, 129-192 nodes   16 x 6 and 16 x 12 against 16 x 8 and 16 x 16: 5.0 / 5.3 / 4.7 / 4.85 against 4.7 / 5.05 /
//                 4.3 / 4.5 at 80 / 96 / 160 / 192 nodes
//   1-8 nodes     two rows per thread (1 x 2, 2 x 2, 4 x 2) measured equal or worse than one (6.4-6.6)
template <int VEC, int ALGO, int GF, bool NORMS>
int launch_rows(const StepCall& s) {
    if constexpr (VEC == 4) {
        if (mixes_on_matrix_cores(s.n, s.topo->row_ptr[s.n])) {
            if (s.n <= kDenseRows) return launch_variant<4, 2, 16, ALGO, GF, NORMS, true>(s);
            return launch_variant<4, 3, 16, ALGO, GF, NORMS, true>(s);
        }
    }
#define DL_SHAPE(MAXN, W, R)                                                             \
    if constexpr (VEC == 1 || VEC * (MAXN) <= 256) {                                     \
        if (s.n <= (MAXN)) return launch_variant<VEC, R, W, ALGO, GF, NORMS>(s);         \
    }
    DL_SHAPE(1, 1, 1) DL_SHAPE(2, 2, 1) DL_SHAPE(4, 4, 1) DL_SHAPE(8, 8, 1) DL_SHAPE(16, 8, 2) DL_SHAPE(20, 10, 2) DL_SHAPE(24, 12, 2) DL_SHAPE(32, 16, 2) DL_SHAPE(48, 16, 3)
    DL_SHAPE(64, 16, 4) DL_SHAPE(96, 16, 6) DL_SHAPE(128, 16, 8) DL_SHAPE(192, 16, 12) DL_SHAPE(256, 16, 16)
#undef DL_SHAPE
    return set_error(DL_ETOPO, "step: n = %d has no kernel variant at vector width %d", s.n, VEC);
}

template <int ALGO, int GF, bool NORMS>
int launch_cols(int vec, const StepCall& s) {
    if (s.d <= 0) return DL_OK;
    switch (vec) {
        case 4: return launch_rows<4, ALGO, GF, NORMS>(s);
        case 2: return launch_rows<2, ALGO, GF, NORMS>(s);
        default: return launch_rows<1, ALGO, GF, NORMS>(s);
    }
}

// 16-bit gradients exist for every method but DSGD, per-tensor sums for the methods that keep (x, m).
template <int ALGO>
int launch_extras(int vec, int format, bool norms, const StepCall& s) {
    if constexpr (ALGO == ALGO_DECENTLAM || ALGO == ALGO_DMSGD || ALGO == ALGO_AWC_DMSGD || ALGO == ALGO_DA_DMSGD) {
        if (norms) {
            if (format == DL_GRAD_BF16) return launch_cols<ALGO, DL_GRAD_BF16, true>(vec, s);
            if (format == DL_GRAD_F16) return launch_cols<ALGO, DL_GRAD_F16, true>(vec, s);
            return launch_cols<ALGO, DL_GRAD_F32, true>(vec, s);
        }
    }
    if constexpr (ALGO != ALGO_DSGD) {
        if (!norms) {
            if (format == DL_GRAD_BF16) return launch_cols<ALGO, DL_GRAD_BF16, false>(vec, s);
            if (format == DL_GRAD_F16) return launch_cols<ALGO, DL_GRAD_F16, false>(vec, s);
        }
    }
    if (norms || format != DL_GRAD_F32)
        return set_error(DL_EINVAL, "step: this method has no variant with 16-bit gradients / per-tensor sums");
    return launch_cols<ALGO, DL_GRAD_F32, false>(vec, s);
}


}  // namespace
#endif  // DL_STEP_KERNEL_IMPL

}  // namespace step
}  // namespace dl
