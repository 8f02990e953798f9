// Per-node least-squares gradient g_i = scale * A_i^T (A_i x_i - y_i) for gfx950.
//
// Every node has its own A_i and its own x_i, so this is a batch of n independent
// matrix-vector products with no shared operand: 1 flop per byte of A at best.
// The bound is HBM, and the kernels are organised around streaming A with wide
// coalesced loads; products are exact in fp64 (two fp32 factors) and sums are fp64.
//
// Single sweep (rows of A on 16-byte boundaries, 1024 < d <= 32768; 256 threads up to d = 8192, 1024 beyond; rows of
// A on other boundaries: k_fused_narrow below, d <= 16384; rows of up to 1024 columns: k_fused_rows below, a wave
// per row):
// k_fused keeps a tile of R rows of A_i in
// registers, split by columns over the 256 threads of a workgroup; the R residuals are reduced
// with wavefront shuffles plus one LDS hop, then the same registers feed the transposed
// product, so A is read from HBM exactly once (4*b*d bytes per node).  The next tile's loads are
// issued before the current tile's reduction.  Each workgroup owns a block of rows of one node
// and leaves a partial gradient; k_finish_fused adds the partials in fixed order.  (Folding that sum into
// k_fused -- the block that finds all blocks of its node done adds them up -- was built and measured and is
// not used: the chip has eight L2 caches, a device-wide fence writes back and invalidates a whole one, and one
// fencing thread per block took workload 5 from 0.65 to 0.69 ms and 8 nodes of 1024 x 1024 from 31 to 73 us;
// without fences, with device-scope atomic accesses for everything that crosses blocks, the final sum of one
// block is a chain of uncached loads: 0.64 ms and 54 us.  The second launch costs less than either.)
//
// Single sweep for wider rows (32768 < d <= 262144, d a multiple of 4, rows of A on 16-byte boundaries):
// k_fused_split, the columns of a row block split over waves that exchange one number per wave and row
// through device memory; see there.
//
// Small problems (bs * d <= 4096 elements per node, any alignment): k_small, one launch,
// one workgroup per node with A_i, x_i and the residuals in LDS; such sizes are bound by launch
// latency, and this is one launch instead of two or three.
//
// Two sweeps (any shape and alignment):
//   k_residual   one wave per row r of A_i: res[i][r] = A_i[r,:] . x_i - y_i[r]
//                (lane-strided 16-byte loads, fp64 accumulators, wavefront-shuffle reduction)
//   k_transpose  one thread per 4 columns, one workgroup per (column block, row split, node):
//                partial[i][s][c] = sum_{r in split s} A_i[r,c] * res[i][r]
//   k_finish     g[i][c] = scale * sum_s partial[i][s][c] in fixed order (deterministic),
//                loss[i] = (scale/2) * sum_r res[i][r]^2
#include <atomic>

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

// Mini-batch gradients: logical row r of node i is physical row rows[i*bs + r] of A_i and y_i
// (clamped into [0, b) so that a bad index can never leave the arrays).
__device__ __forceinline__ int physical_row(const int32_t* __restrict__ rows_i, int r, int b) {
    const int p = rows_i[r];
    return p < 0 ? 0 : (p >= b ? b - 1 : p);
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

// rows == nullptr: all b rows (bs == b); otherwise bs sampled rows per node.
// WIDE: a whole workgroup per row instead of one wave (few, long rows: a wave per row would leave
// most of the GPU idle).
template <bool VEC4, bool WIDE>
__global__ __launch_bounds__(kThreads) void k_residual(const float* __restrict__ A,
                                                        const float* __restrict__ y,
                                                        const float* __restrict__ x,
                                                        double* __restrict__ res, int b, int64_t d,
                                                        int64_t ldA, int64_t ld,
                                                        const int32_t* __restrict__ rows, int bs) {
    __shared__ double part[kThreads / 64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i = blockIdx.y;
    const int r = WIDE ? blockIdx.x : blockIdx.x * (kThreads / 64) + wave;
    if (r >= bs) return;   // WIDE: the whole workgroup leaves together
    const int t = WIDE ? static_cast<int>(threadIdx.x) : lane;   // position in the row's team of threads
    constexpr int kTeam = WIDE ? kThreads : 64;
    const int pr = rows ? physical_row(rows + static_cast<int64_t>(i) * bs, r, b) : r;
    const float* __restrict__ a = A + (static_cast<int64_t>(i) * b + pr) * ldA;
    const float* __restrict__ xi = x + static_cast<int64_t>(i) * ld;
    double acc0 = 0.0, acc1 = 0.0, acc2 = 0.0, acc3 = 0.0;
    if constexpr (VEC4) {
#pragma unroll 4
        for (int64_t c = t * 4; c < d; c += kTeam * 4) {  // d % 4 == 0 here
            const vf4 av = *reinterpret_cast<const vf4*>(a + c);
            const vf4 xv = *reinterpret_cast<const vf4*>(xi + c);
            acc0 = __builtin_fma(static_cast<double>(av.x), static_cast<double>(xv.x), acc0);
            acc1 = __builtin_fma(static_cast<double>(av.y), static_cast<double>(xv.y), acc1);
            acc2 = __builtin_fma(static_cast<double>(av.z), static_cast<double>(xv.z), acc2);
            acc3 = __builtin_fma(static_cast<double>(av.w), static_cast<double>(xv.w), acc3);
        }
    } else {
        for (int64_t c = t; c < d; c += kTeam)
            acc0 = __builtin_fma(static_cast<double>(a[c]), static_cast<double>(xi[c]), acc0);
    }
    double dot = wave_sum((acc0 + acc1) + (acc2 + acc3));
    if constexpr (WIDE) {
        if (lane == 0) part[wave] = dot;
        __syncthreads();
        dot = (part[0] + part[1]) + (part[2] + part[3]);
        if (threadIdx.x != 0) return;
    } else {
        if (lane != 0) return;
    }
    res[static_cast<int64_t>(i) * bs + r] = dot - static_cast<double>(y[static_cast<int64_t>(i) * b + pr]);
}

template <bool VEC4>
__global__ __launch_bounds__(kThreads) void k_transpose(const float* __restrict__ A,
                                                         const double* __restrict__ res,
                                                         double* __restrict__ partial, int b, int64_t d,
                                                         int64_t ldA, int splits,
                                                         const int32_t* __restrict__ rows, int bs) {
    constexpr int V = VEC4 ? 4 : 1;
    const int i = blockIdx.z, s = blockIdx.y;
    const int64_t c = (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x) * V;
    if (c >= d) return;
    const int r0 = static_cast<int>(static_cast<int64_t>(bs) * s / splits);
    const int r1 = static_cast<int>(static_cast<int64_t>(bs) * (s + 1) / splits);
    const float* __restrict__ a = A + static_cast<int64_t>(i) * b * ldA + c;
    const double* __restrict__ ri = res + static_cast<int64_t>(i) * bs;
    const int32_t* __restrict__ rows_i = rows ? rows + static_cast<int64_t>(i) * bs : nullptr;
    double acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.0;
#pragma unroll 8
    for (int r = r0; r < r1; ++r) {
        const double rr = ri[r];
        const int pr = rows_i ? physical_row(rows_i, r, b) : r;
        if constexpr (VEC4) {
            const vf4 av = *reinterpret_cast<const vf4*>(a + static_cast<int64_t>(pr) * ldA);
            acc[0] = __builtin_fma(static_cast<double>(av.x), rr, acc[0]);
            acc[1] = __builtin_fma(static_cast<double>(av.y), rr, acc[1]);
            acc[2] = __builtin_fma(static_cast<double>(av.z), rr, acc[2]);
            acc[3] = __builtin_fma(static_cast<double>(av.w), rr, acc[3]);
        } else {
            acc[0] = __builtin_fma(static_cast<double>(a[static_cast<int64_t>(pr) * ldA]), rr, acc[0]);
        }
    }
    double* out = partial + (static_cast<int64_t>(i) * splits + s) * d + c;
#pragma unroll
    for (int v = 0; v < V; ++v) out[v] = acc[v];
}

// Sum of the `splits` partial gradients of one node for 64 consecutive columns per workgroup: wave w adds the
// w-th quarter of the partials for its lane's column, eight loads in flight at a time, and wave 0 adds the four
// quarters; every sum in a fixed order.  (One thread per column adding all partials one after the other was a
// chain of dependent loads in a grid of d / 256 workgroups per node: 18 us of the 31 us that 8 nodes of
// 1024 x 1024 took, more than the sweep over A itself.)
constexpr int kFinishColumns = 64;
__device__ __forceinline__ void finish_columns(const double* __restrict__ partial_i, float* __restrict__ g_i,
                                               int64_t d, int splits, double scale, double (&quarter)[4][kFinishColumns],
                                               bool poisoned = false) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t c = static_cast<int64_t>(blockIdx.x) * kFinishColumns + lane;
    const int per = (splits + 3) / 4;
    const int s0 = w * per < splits ? w * per : splits, s1 = s0 + per < splits ? s0 + per : splits;
    double acc = 0.0;
    if (c < d) {
        const double* p = partial_i + c;
        int s = s0;
        for (; s + 8 <= s1; s += 8) {
            double v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = p[static_cast<int64_t>(s + k) * d];
#pragma unroll
            for (int k = 0; k < 8; ++k) acc += v[k];
        }
        for (; s < s1; ++s) acc += p[static_cast<int64_t>(s) * d];
    }
    quarter[w][lane] = acc;
    __syncthreads();
    if (w == 0 && c < d)
        g_i[c] = poisoned ? __builtin_nanf("")
                          : static_cast<float>(scale * (((quarter[0][lane] + quarter[1][lane]) + quarter[2][lane]) + quarter[3][lane]));
}

__global__ __launch_bounds__(kThreads) void k_finish(const double* __restrict__ partial,
                                                      const double* __restrict__ res,
                                                      float* __restrict__ g, float* __restrict__ loss,
                                                      int b, int64_t d, int64_t ld, int splits,
                                                      double scale) {
    __shared__ double red[kThreads];
    static_assert(kThreads == 4 * kFinishColumns, "four waves per workgroup");
    const int i = blockIdx.y;
    finish_columns(partial + static_cast<int64_t>(i) * splits * d, g + static_cast<int64_t>(i) * ld, d, splits, scale,
                   *reinterpret_cast<double (*)[4][kFinishColumns]>(red));
    if (loss != nullptr && blockIdx.x == 0) {  // whole workgroup takes this branch together
        __syncthreads();   // the column sums are out of `red`
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


// ---------------------------------------------------------------- single sweep
// A value that is the same in every lane, moved to a scalar register (it then costs no vector register).
__device__ __forceinline__ float uniform_f32(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, v)));
}

// CPT  16-byte column chunks per thread (thread t owns columns 4t + 4 THREADS q .. +3, q < CPT)
// R    rows of A per register tile
template <int CPT, int R>
struct Tile {
    vf4 a[R][CPT];
    float tl[R][3];   // TAIL: the row's last d % 4 elements (uniform over the workgroup), zeros after them
    float y[R];       // the rows' entries of y_i (uniform): fetched with the tile, not after the barrier that follows it
};

// The physical rows of a tile (uniform): rows past the block's end are clamped to its last row, sampled rows are looked
// up.  Called one tile ahead of the loads that use the result, so that the look-up is not waited for when the loads
// should go out (with the look-up inside load_tile a sampled sweep ran at 0.65 of the HBM peak where the plain one
// runs at 0.85).
template <int R>
__device__ __forceinline__ void tile_rows(int (&prow)[R], int r, int r_last, const int32_t* __restrict__ rows_i, int b) {
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const int row = (r + rr < r_last) ? r + rr : r_last;
        prow[rr] = rows_i ? physical_row(rows_i, row, b) : row;
    }
}

// The same with the look-ups of 128 consecutive logical rows kept in two registers per lane (lane j: rows base + j and
// base + 64 + j), fetched by vector loads 64 rows or more ahead of their use and handed out with readlane: a scalar
// look-up per tile shares its counter with the tile's LDS traffic, and waiting for one means waiting for the other
// (64 nodes, 4096 sampled rows of 4096 columns: see launch_lsq).  Requests must come in non-decreasing row order and
// advance by less than 64 rows at a time; the form with x_i in LDS has no registers for this and looks up row by row.
// off, stride: request r stands for logical row off + r * stride (0, 1: r itself; s, splits: the interleaved rows of row
// block s, see k_fused).
struct RowWindow {
    const int32_t* rows_i;
    int b, r_last, base;
    int lo, hi;
    int off, stride;
    __device__ __forceinline__ int fetch(int first) const {
        const int row = first + static_cast<int>(threadIdx.x & 63);
        return physical_row(rows_i, off + (row < r_last ? row : r_last) * stride, b);
    }
    __device__ __forceinline__ void init(const int32_t* __restrict__ rows, int b_, int r0, int r_last_, int off_ = 0, int stride_ = 1) {
        off = off_; stride = stride_;
        rows_i = rows; b = b_; r_last = r_last_; base = r0;
        lo = hi = 0;
        if (rows_i) {
            lo = fetch(r0);
            hi = fetch(r0 + 64);
        }
    }
    template <int R>
    __device__ __forceinline__ void tile(int (&prow)[R], int r) {
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            const int row = (r + rr < r_last) ? r + rr : r_last;   // uniform
            if (rows_i) {
                if (row - base >= 64) {   // uniform; the window moves on by 64 rows, the next 64 look-ups go out
                    base += 64;
                    lo = hi;
                    hi = fetch(base + 64);
                }
                prow[rr] = __builtin_amdgcn_readlane(lo, row - base);
            } else {
                prow[rr] = off + row * stride;
            }
        }
    }
};

// Loads never need a predicate: rows past the block's end are clamped to its last row (their
// residual is forced to zero below) and column chunks past d are clamped to the last chunk
// (their x is zero and their accumulators are never stored).
// TAIL (d not a multiple of 4): the 16-byte chunks cover the first dm = d - d % 4 columns and the last dt = d % 4
// elements of a row are read one by one from an address that is the same for the whole workgroup, so that no access
// reaches past column d of any row.
template <int CPT, int R, bool TAIL = false>
__device__ __forceinline__ void load_tile(Tile<CPT, R>& t, const float* __restrict__ a_node, int64_t ldA,
                                          const int (&prow)[R], const int (&col)[CPT],
                                          const float* __restrict__ yi, int64_t dm = 0, int dt = 0) {
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const int row = prow[rr];
        const float* __restrict__ a_row = a_node + static_cast<int64_t>(row) * ldA;
        t.y[rr] = yi[row];
#pragma unroll
        for (int q = 0; q < CPT; ++q)
            t.a[rr][q] = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(a_row + col[q]));
        if constexpr (TAIL) {
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                const float v = a_row[dm + (k < dt ? k : 0)];
                t.tl[rr][k] = k < dt ? uniform_f32(v) : 0.f;
            }
        }
    }
}

// XL: the thread's chunks of x_i wait in LDS (xl[q * 64 * WAVES], written by this thread) instead of in registers
template <int CPT, int R, int WAVES, bool XL = false, bool TAIL = false>
__device__ __forceinline__ void consume_tile(const Tile<CPT, R>& t, const float (&xs)[CPT][4], const vf4* xl,
                                             double (&acc)[CPT][4], double& sq, double (*red)[R],
                                             int r, int r1, int lane, int wave, const float (&xt)[3],
                                             double (&acc_tail)[3], double* tail_sums) {
    double p[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        double s0 = 0.0, s1 = 0.0;
#pragma unroll
        for (int q = 0; q < CPT; ++q) {
            vf4 xv;
            if constexpr (XL) {
                xv = xl[q * 64 * WAVES];
            } else {
                xv.x = xs[q][0]; xv.y = xs[q][1]; xv.z = xs[q][2]; xv.w = xs[q][3];
            }
            s0 = __builtin_fma(static_cast<double>(t.a[rr][q].x), static_cast<double>(xv.x), s0);
            s1 = __builtin_fma(static_cast<double>(t.a[rr][q].y), static_cast<double>(xv.y), s1);
            s0 = __builtin_fma(static_cast<double>(t.a[rr][q].z), static_cast<double>(xv.z), s0);
            s1 = __builtin_fma(static_cast<double>(t.a[rr][q].w), static_cast<double>(xv.w), s1);
        }
        p[rr] = wave_sum(s0 + s1);
    }
    if (lane == 0) {
#pragma unroll
        for (int rr = 0; rr < R; ++rr) red[wave][rr] = p[rr];
    }
    __syncthreads();
    // The transposed product re-converts the tile from fp32: keeping the forward pass's fp64
    // copies alive across the barrier would double the register footprint of the tile.
    Tile<CPT, R> u = t;
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
#pragma unroll
        for (int q = 0; q < CPT; ++q) asm volatile("" : "+v"(u.a[rr][q]));
    }
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        double res = 0.0;
        if (r + rr < r1) {  // uniform over the workgroup
            double dot = 0.0;   // the waves' shares in a fixed order
#pragma unroll
            for (int w4 = 0; w4 < WAVES; w4 += 4)
                dot += (red[w4][rr] + red[w4 + 1][rr]) + (red[w4 + 2][rr] + red[w4 + 3][rr]);
            if constexpr (TAIL) {   // the last d % 4 columns: the same values in every thread
#pragma unroll
                for (int k = 0; k < 3; ++k) {
                    float xk = xt[k];
                    asm volatile("" : "+s"(xk));   // widened here, row by row: three doubles kept across the loop are registers the wide forms lack
                    dot = __builtin_fma(static_cast<double>(t.tl[rr][k]), static_cast<double>(xk), dot);
                }
            }
            res = dot - static_cast<double>(t.y[rr]);
        }
        sq = __builtin_fma(res, res, sq);
        if constexpr (TAIL) {
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                if constexpr (WAVES > 4) {   // the 1024-thread forms have no registers to spare: thread 0 keeps the sums in LDS
                    if (threadIdx.x == 0) tail_sums[k] = __builtin_fma(static_cast<double>(t.tl[rr][k]), res, tail_sums[k]);
                } else {
                    acc_tail[k] = __builtin_fma(static_cast<double>(t.tl[rr][k]), res, acc_tail[k]);
                }
            }
        }
#pragma unroll
        for (int q = 0; q < CPT; ++q) {
            acc[q][0] = __builtin_fma(static_cast<double>(u.a[rr][q].x), res, acc[q][0]);
            acc[q][1] = __builtin_fma(static_cast<double>(u.a[rr][q].y), res, acc[q][1]);
            acc[q][2] = __builtin_fma(static_cast<double>(u.a[rr][q].z), res, acc[q][2]);
            acc[q][3] = __builtin_fma(static_cast<double>(u.a[rr][q].w), res, acc[q][3]);
        }
    }
}

// THREADS: 256 up to d = 8192; 1024 threads with four column chunks each carry the single sweep to d = 16384, with
// eight chunks each and x_i in LDS (XL) to d = 32768 (8 nodes of 2048 x 32768: 0.36 ms, 0.74 of the HBM peak, where
// the two sweeps take 0.83 ms)
// (one workgroup per CU within 128 registers, no prefetch; 512 threads with eight chunks each measured 2-3 % slower:
// 16 nodes of 1024 x 16384 5.75 against 5.94 TB/s, 8 nodes of 4096 x 16384 6.31 against 6.44; up to d = 8192, 512
// threads with four chunks, with or without prefetch, are slower than 256 with eight: 64 nodes of 1024 x 6144
// 5.6-5.8 against 6.2 TB/s)
template <int CPT, int R, bool PF, int THREADS, bool XL = false, bool TAIL = false>
__global__ __launch_bounds__(THREADS, THREADS > 256 ? 4 : 2) void k_fused(const float* __restrict__ A, const float* __restrict__ y,
                                                     const float* __restrict__ x, double* __restrict__ partial,
                                                     double* __restrict__ sq_partial, int b, int64_t d,
                                                     int64_t ldA, int64_t ld, int splits,
                                                     const int32_t* __restrict__ rows, int bs) {
    constexpr int WAVES = THREADS / 64;
    __shared__ double red[2][WAVES][R];  // two buffers: one barrier per tile is enough
    const int i = blockIdx.y, s = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // The forms with one row per tile and 256 threads (2048 < d <= 8192) give row block s the rows s, s + splits, ...: the
    // blocks of a node, which run side by side, then read neighbouring rows of A_i, one window that moves through the
    // matrix, instead of `splits` places far apart (same box, same calls: 32 nodes of 4096 x 6144 0.83 -> 0.89 of the HBM
    // peak, 16 of 4096 x 8192 0.82 -> 0.85, 64 of 4096 x 4096 0.86 either way; the 1024-thread forms, whose workgroups read
    // rows of 64-128 KiB, gain nothing).  There r counts the block's own rows and the row window turns it into the row it
    // stands for.
    constexpr bool kInterleaved = R == 1 && THREADS == 256;
    const int r0 = kInterleaved ? 0 : static_cast<int>(static_cast<int64_t>(bs) * s / splits);
    const int r1 = kInterleaved ? (bs - s + splits - 1) / splits
                                : static_cast<int>(static_cast<int64_t>(bs) * (s + 1) / splits);  // r1 > r0: splits <= bs
    const int row_off = kInterleaved ? s : 0, row_stride = kInterleaved ? splits : 1;
    const int32_t* __restrict__ rows_i = rows ? rows + static_cast<int64_t>(i) * bs : nullptr;

    extern __shared__ vf4 x_chunks[];   // XL: CPT * THREADS chunks of x_i, each read only by the thread that wrote it
    const vf4* xl = x_chunks + threadIdx.x;
    // TAIL: the chunks cover the first dm columns (dm >= 4), the remaining dt = d % 4 are handled element by element
    const int64_t dm = TAIL ? (d & ~int64_t{3}) : d;
    const int dt = static_cast<int>(d - dm);
    float xt[3] = {0.f, 0.f, 0.f};
    double acc_tail[3] = {0.0, 0.0, 0.0};
    __shared__ double tail_sums[3];   // TAIL with 1024 threads: thread 0's sums (nobody else touches them)
    if (TAIL && WAVES > 4 && threadIdx.x == 0) tail_sums[0] = tail_sums[1] = tail_sums[2] = 0.0;
    if constexpr (TAIL) {
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            const float v = x[static_cast<int64_t>(i) * ld + dm + (k < dt ? k : 0)];
            xt[k] = k < dt ? uniform_f32(v) : 0.f;
        }
    }
    int col[CPT];
    float xs[CPT][4];
    double acc[CPT][4];
    // x_i is read once per workgroup: its rows need not be on 16-byte boundaries, only A's
    const bool x_wide = ((reinterpret_cast<uintptr_t>(x) & 15u) | (static_cast<uint64_t>(ld) & 3u)) == 0;
#pragma unroll
    for (int q = 0; q < CPT; ++q) {
        const int c = 4 * static_cast<int>(threadIdx.x) + 4 * THREADS * q;
        const bool inside = c < dm;
        col[q] = inside ? c : static_cast<int>(dm) - 4;
        const float* xp = x + static_cast<int64_t>(i) * ld + col[q];
        const vf4 xv = x_wide ? *reinterpret_cast<const vf4*>(xp) : vf4{xp[0], xp[1], xp[2], xp[3]};
        if constexpr (XL) {
            x_chunks[q * THREADS + threadIdx.x] = inside ? xv : vf4{0.f, 0.f, 0.f, 0.f};
        } else {
            xs[q][0] = inside ? xv.x : 0.f; xs[q][1] = inside ? xv.y : 0.f;
            xs[q][2] = inside ? xv.z : 0.f; xs[q][3] = inside ? xv.w : 0.f;
        }
        acc[q][0] = acc[q][1] = acc[q][2] = acc[q][3] = 0.0;
    }
    double sq = 0.0;
    const float* __restrict__ a_node = A + static_cast<int64_t>(i) * b * ldA;
    const float* __restrict__ yi = y + static_cast<int64_t>(i) * b;

    if constexpr (PF) {
        Tile<CPT, R> t0, t1;
        int p0[R], p1[R];   // physical rows of the tile that is loaded next into t0 / t1
        RowWindow win;
        win.init(rows_i, b, r0, r1 - 1, row_off, row_stride);
        win.tile<R>(p0, r0);
        load_tile<CPT, R, TAIL>(t0, a_node, ldA, p0, col, yi, dm, dt);
        win.tile<R>(p1, r0 + R);
        for (int r = r0; r < r1; r += 2 * R) {
            load_tile<CPT, R, TAIL>(t1, a_node, ldA, p1, col, yi, dm, dt);
            win.tile<R>(p0, r + 2 * R);
            consume_tile<CPT, R, WAVES, XL, TAIL>(t0, xs, xl, acc, sq, red[0], r, r1, lane, wave, xt, acc_tail, tail_sums);
            load_tile<CPT, R, TAIL>(t0, a_node, ldA, p0, col, yi, dm, dt);
            win.tile<R>(p1, r + 3 * R);
            consume_tile<CPT, R, WAVES, XL, TAIL>(t1, xs, xl, acc, sq, red[1], r + R, r1, lane, wave, xt, acc_tail, tail_sums);
        }
    } else {
        Tile<CPT, R> t0;
        int buf = 0;
        int p0[R];   // physical rows of the next tile
        constexpr bool kWindow = !XL;   // see RowWindow; the form with x_i in LDS has no register left for it
        RowWindow win;
        if constexpr (kWindow) {
            win.init(rows_i, b, r0, r1 - 1, row_off, row_stride);
            win.tile<R>(p0, r0);
        } else {
            tile_rows<R>(p0, r0, r1 - 1, rows_i, b);
        }
        for (int r = r0; r < r1; r += R, buf ^= 1) {
            if constexpr (XL) {   // the column offsets are worked out per row here: eight registers the kernel lacks
                int c0 = 4 * static_cast<int>(threadIdx.x);
                asm volatile("" : "+v"(c0));
#pragma unroll
                for (int q = 0; q < CPT; ++q) {
                    const int c = c0 + 4 * THREADS * q;
                    col[q] = c < static_cast<int>(dm) ? c : static_cast<int>(dm) - 4;
                }
            }
            if constexpr (XL) tile_rows<R>(p0, r, r1 - 1, rows_i, b);   // (no register to carry a row number through the tile)
            load_tile<CPT, R, TAIL>(t0, a_node, ldA, p0, col, yi, dm, dt);
            if constexpr (kWindow) win.tile<R>(p0, r + R);
            else if constexpr (!XL) tile_rows<R>(p0, r + R, r1 - 1, rows_i, b);
            consume_tile<CPT, R, WAVES, XL, TAIL>(t0, xs, xl, acc, sq, red[buf], r, r1, lane, wave, xt, acc_tail, tail_sums);
        }
    }

    double* out = partial + (static_cast<int64_t>(i) * splits + s) * d;
    int c_first = 4 * static_cast<int>(threadIdx.x);
    if constexpr (THREADS > 256) asm volatile("" : "+v"(c_first));   // worked out again here, not carried through the loop
#pragma unroll
    for (int q = 0; q < CPT; ++q) {
        const int c = c_first + 4 * THREADS * q;
        if (c < dm) {
            out[c + 0] = acc[q][0]; out[c + 1] = acc[q][1]; out[c + 2] = acc[q][2]; out[c + 3] = acc[q][3];
        }
    }
    if constexpr (TAIL) {
        if (threadIdx.x == 0) {
#pragma unroll
            for (int k = 0; k < 3; ++k)
                if (k < dt) out[dm + k] = WAVES > 4 ? tail_sums[k] : acc_tail[k];
        }
    }
    if (threadIdx.x == 0) sq_partial[static_cast<int64_t>(i) * splits + s] = sq;
}

// The single sweep for short rows (d <= 1024): a wave owns whole rows, so a row's residual is a sum over lanes -- no
// LDS hop and no barrier inside the loop, which is what holds k_fused back on short rows (one barrier per 4 rows of
// 4 KiB at d = 1024, and a workgroup of 256 threads with most of its lanes idle below that).  L lanes share a row
// (64: the wave reads one row per access with CPW chunks per lane; 8, 16, 32: one chunk per lane and 64 / L
// consecutive rows per access), R accesses are in flight per lane.  A chunk is V columns: 4 (rows of A on 16-byte
// boundaries, d a multiple of 4), 2 (rows on 8-byte boundaries, d even) or 1 (anything).  The four waves of a
// workgroup take consecutive groups of rows, so that a contiguous A is read in contiguous pieces, and add their sums
// up through LDS once, at the end of the row block.
template <int V, int CPW, int L, int R>
__global__ __launch_bounds__(256) void k_fused_rows(const float* __restrict__ A, const float* __restrict__ y,
                                                    const float* __restrict__ x, double* __restrict__ partial,
                                                    double* __restrict__ sq_partial, int b, int64_t d,
                                                    int64_t ldA, int64_t ld, int splits,
                                                    const int32_t* __restrict__ rows, int bs) {
    static_assert(L == 64 || CPW == 1, "several chunks per lane only when a row fills the wave");
    typedef float vfv __attribute__((ext_vector_type(V)));
    constexpr int G = 64 / L;       // rows per wave-wide access
    constexpr int STEP = 4 * G;     // rows per workgroup-wide access
    constexpr int QG = CPW < 4 ? CPW : 4;   // chunks per lane that pass through LDS together at the end
    constexpr int COLS = V * L * QG;
    __shared__ double sums[STEP][COLS];
    __shared__ double sq_wave[4];
    const int i = blockIdx.y, s = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int sub = lane & (L - 1), slot = wave * G + lane / L;
    const int r0 = static_cast<int>(static_cast<int64_t>(bs) * s / splits);
    const int r1 = static_cast<int>(static_cast<int64_t>(bs) * (s + 1) / splits);
    const int32_t* __restrict__ rows_i = rows ? rows + static_cast<int64_t>(i) * bs : nullptr;

    // chunk q of this lane: columns V (sub + q L) .. + V - 1; chunks past d read column 0 with x = 0, never stored
    int col[CPW];
    float xs[CPW][V];
    double acc[CPW][V];
#pragma unroll
    for (int q = 0; q < CPW; ++q) {
        const int c = V * (sub + q * L);
        const bool inside = c < d;   // d is a multiple of V
        col[q] = inside ? c : 0;
        const float* xp = x + static_cast<int64_t>(i) * ld + col[q];   // x_i is read once: element by element
#pragma unroll
        for (int v = 0; v < V; ++v) {
            xs[q][v] = inside ? xp[v] : 0.f;
            acc[q][v] = 0.0;
        }
    }
    double sq = 0.0;
    const float* __restrict__ a_node = A + static_cast<int64_t>(i) * b * ldA;
    const float* __restrict__ yi = y + static_cast<int64_t>(i) * b;

    // the lane's physical rows of an iteration: rows past the block's end read its last row and count for nothing;
    // sampled rows are looked up one iteration ahead, so that the loads of A never wait for the look-up
    int pr[R];
    const auto rows_of = [&](int r) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int row = r + j * STEP + slot;
            pr[j] = row < r1 ? row : r1 - 1;
            if (rows_i) pr[j] = physical_row(rows_i, pr[j], b);
        }
    };
    rows_of(r0);
    for (int r = r0; r < r1; r += STEP * R) {
        vfv a[R][CPW];
        float yv[R];
        // all loads first
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const float* __restrict__ a_row = a_node + static_cast<int64_t>(pr[j]) * ldA;
#pragma unroll
            for (int q = 0; q < CPW; ++q) a[j][q] = __builtin_nontemporal_load(reinterpret_cast<const vfv*>(a_row + col[q]));
            yv[j] = yi[pr[j]];
        }
        rows_of(r + STEP * R);
#pragma unroll
        for (int j = 0; j < R; ++j) {
            double s0 = 0.0, s1 = 0.0;
#pragma unroll
            for (int q = 0; q < CPW; ++q) {
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    double& sv = ((q * V + v) & 1) ? s1 : s0;
                    sv = __builtin_fma(static_cast<double>(a[j][q][v]), static_cast<double>(xs[q][v]), sv);
                }
            }
            double dot = s0 + s1;
#pragma unroll
            for (int off = L / 2; off > 0; off >>= 1) dot += __shfl_xor(dot, off, 64);   // every lane of the row has the sum
            const double res = r + j * STEP + slot < r1 ? dot - static_cast<double>(yv[j]) : 0.0;
            if (sub == 0) sq = __builtin_fma(res, res, sq);
#pragma unroll
            for (int q = 0; q < CPW; ++q) {
#pragma unroll
                for (int v = 0; v < V; ++v) acc[q][v] = __builtin_fma(static_cast<double>(a[j][q][v]), res, acc[q][v]);
            }
        }
    }

    // the STEP row slots of the workgroup hold sums over disjoint rows for the same columns: add them in slot order,
    // up to four chunks per lane (COLS columns) at a time
    sq = wave_sum(sq);
    if (lane == 0) sq_wave[wave] = sq;
    double* out = partial + (static_cast<int64_t>(i) * splits + s) * d;
#pragma unroll
    for (int q0 = 0; q0 < CPW; q0 += QG) {
        if (q0 > 0) __syncthreads();   // the previous group has been read
#pragma unroll
        for (int q = q0; q < q0 + QG && q < CPW; ++q) {
#pragma unroll
            for (int v = 0; v < V; ++v) sums[slot][V * (sub + (q - q0) * L) + v] = acc[q][v];
        }
        __syncthreads();
        const int first = V * L * q0;   // first column of the group
        for (int c = threadIdx.x; c < COLS && first + c < d; c += 256) {
            double total = 0.0;
#pragma unroll
            for (int k = 0; k < STEP; ++k) total += sums[k][c];
            out[first + c] = total;
        }
    }
    if (threadIdx.x == 0) sq_partial[static_cast<int64_t>(i) * splits + s] = (sq_wave[0] + sq_wave[1]) + (sq_wave[2] + sq_wave[3]);
}

// The single sweep for rows of A that are not on 16-byte boundaries (ldA not a multiple of 4, or a base that is
// not 16-byte aligned): the same structure as k_fused with 8-byte (V = 2: rows on 8-byte boundaries) or 4-byte
// (V = 1: any rows) accesses, K columns per thread in K / V chunks, R rows per tile, no prefetch.  A is still read
// once; what the narrow accesses cost is rate (8 nodes of 4096 x 7850, contiguous: 0.19 ms, 0.67 of the HBM peak,
// against 0.17 ms with ldA = 7852 in k_fused and 0.49 ms in two sweeps; 64 nodes of 4096 x 4095 with ldA = 4095:
// 1.05 ms, 0.51, against 1.93 ms), not a second pass.  V = 2 with an odd d: thread 0 takes the last column by itself.
template <int V, int K, int R, int THREADS>
__global__ __launch_bounds__(THREADS) void k_fused_narrow(const float* __restrict__ A, const float* __restrict__ y,
                                                           const float* __restrict__ x, double* __restrict__ partial,
                                                           double* __restrict__ sq_partial, int b, int64_t d,
                                                           int64_t ldA, int64_t ld, int splits,
                                                           const int32_t* __restrict__ rows, int bs) {
    constexpr int CPT = K / V, WAVES = THREADS / 64;
    typedef float vfv __attribute__((ext_vector_type(V)));
    __shared__ double red[2][WAVES][R];
    const int i = blockIdx.y, s = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r0 = static_cast<int>(static_cast<int64_t>(bs) * s / splits);
    const int r1 = static_cast<int>(static_cast<int64_t>(bs) * (s + 1) / splits);
    const int32_t* __restrict__ rows_i = rows ? rows + static_cast<int64_t>(i) * bs : nullptr;
    const int dm = static_cast<int>(d - d % V);            // columns covered by whole chunks
    const bool tail = V == 2 && dm < d && threadIdx.x == 0;   // one more column, thread 0's

    // chunk q of this thread: columns column_of(q) .. + V - 1, clamped to the last whole chunk (whose x is zero here and
    // whose sums are never stored); worked out where it is used rather than kept: CPT registers the wide forms lack
    const int last_chunk = dm >= V ? dm - V : 0;
    const auto column_of = [&](int q) {
        int c0 = V * static_cast<int>(threadIdx.x);
        asm volatile("" : "+v"(c0));
        const int c = c0 + V * THREADS * q;
        return c < dm ? c : last_chunk;
    };
    float xs[CPT][V];
    double acc[CPT][V];
    const float* __restrict__ xi = x + static_cast<int64_t>(i) * ld;
#pragma unroll
    for (int q = 0; q < CPT; ++q) {
        const int c = V * static_cast<int>(threadIdx.x) + V * THREADS * q;
        const bool inside = c < dm;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const float xv = dm >= V ? xi[(inside ? c : last_chunk) + v] : 0.f;
            xs[q][v] = inside ? xv : 0.f;
            acc[q][v] = 0.0;
        }
    }
    const float x_tail = tail ? xi[dm] : 0.f;
    double acc_tail = 0.0, sq = 0.0;
    const float* __restrict__ a_node = A + static_cast<int64_t>(i) * b * ldA;
    const float* __restrict__ yi = y + static_cast<int64_t>(i) * b;

    int buf = 0;
    for (int r = r0; r < r1; r += R, buf ^= 1) {
        float a[R][CPT][V], a_tail[R];
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            int row = (r + rr < r1 - 1) ? r + rr : r1 - 1;
            if (rows_i) row = physical_row(rows_i, row, b);
            const float* __restrict__ a_row = a_node + static_cast<int64_t>(row) * ldA;
#pragma unroll
            for (int q = 0; q < CPT; ++q) {
                if (dm >= V) {   // uniform
                    const vfv t = __builtin_nontemporal_load(reinterpret_cast<const vfv*>(a_row + column_of(q)));
#pragma unroll
                    for (int v = 0; v < V; ++v) a[rr][q][v] = t[v];
                } else {
#pragma unroll
                    for (int v = 0; v < V; ++v) a[rr][q][v] = 0.f;
                }
            }
            a_tail[rr] = tail ? a_row[dm] : 0.f;
        }
        double p[R];
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            double s0 = 0.0;
#pragma unroll
            for (int q = 0; q < CPT; ++q) {
#pragma unroll
                for (int v = 0; v < V; ++v) s0 = __builtin_fma(static_cast<double>(a[rr][q][v]), static_cast<double>(xs[q][v]), s0);
            }
            s0 = __builtin_fma(static_cast<double>(a_tail[rr]), static_cast<double>(x_tail), s0);   // zero but in thread 0
            p[rr] = wave_sum(s0);
        }
        if (lane == 0) {
#pragma unroll
            for (int rr = 0; rr < R; ++rr) red[buf][wave][rr] = p[rr];
        }
        __syncthreads();
        // the transposed product widens the tile again: keeping the first product's fp64 copies alive across the
        // barrier would double the tile's registers
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
#pragma unroll
            for (int q = 0; q < CPT; ++q) {
#pragma unroll
                for (int v = 0; v < V; ++v) asm volatile("" : "+v"(a[rr][q][v]));
            }
        }
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            double res = 0.0;
            if (r + rr < r1) {   // uniform over the workgroup
                const int pr = rows_i ? physical_row(rows_i, r + rr, b) : r + rr;
                double dot = 0.0;   // the waves' shares in a fixed order
#pragma unroll
                for (int w = 0; w < WAVES; ++w) dot += red[buf][w][rr];
                res = dot - static_cast<double>(yi[pr]);
            }
            sq = __builtin_fma(res, res, sq);
#pragma unroll
            for (int q = 0; q < CPT; ++q) {
#pragma unroll
                for (int v = 0; v < V; ++v) acc[q][v] = __builtin_fma(static_cast<double>(a[rr][q][v]), res, acc[q][v]);
            }
            acc_tail = __builtin_fma(static_cast<double>(a_tail[rr]), res, acc_tail);
        }
    }
    double* out = partial + (static_cast<int64_t>(i) * splits + s) * d;
#pragma unroll
    for (int q = 0; q < CPT; ++q) {
        const int c = V * static_cast<int>(threadIdx.x) + V * THREADS * q;
        if (c < dm) {
#pragma unroll
            for (int v = 0; v < V; ++v) out[c + v] = acc[q][v];
        }
    }
    if (tail) out[dm] = acc_tail;
    if (threadIdx.x == 0) sq_partial[static_cast<int64_t>(i) * splits + s] = sq;
}

// ---------------------------------------------------------------- single sweep, rows wider than a workgroup's registers
// Beyond 32768 columns one workgroup cannot hold a row's accumulators (d fp64 sums), so the columns of a row block are
// split over several waves, each with its own 2048 columns, its accumulators and no shared memory, and what crosses
// waves is one number per wave and row: the wave's share of the row's dot product.  Every wave writes its share to
// its slot of the row (an 8-byte device-scope atomic store, the value is the message), reads the row's slots of all
// waves (one device-scope atomic load per lane), adds them with the fixed-order wave sum -- the same bits in every wave --
// and multiplies its tile by that residual.  No fence anywhere: a device-wide fence writes back a whole L2, eight of
// which this chip has.  A slot that has not been written yet holds kSlotEmpty, a NaN whose low mantissa bits no sum
// of products of fp32 numbers can have (k_fill_slots writes it before every call).  A row's share is published
// L iterations before it is collected and its loads are issued LA iterations before that.  The row blocks of a node take
// interleaved rows (see the kernel), so that side by side they move one window through A_i.
// Measured (fraction of the HBM peak for 4 n b d bytes; the two sweeps: 0.33-0.35): 8 nodes of 1024 x 65536 0.76, 8 of
// 2048 x 49152 0.78, 8 of 1024 x 57344 0.76, 4 of 1024 x 131072 0.75, 4 of 1024 x 98304 0.73, 2 of 4096 x 100000 0.72,
// 64 of 128 x 65536 0.69, 16 of 1024 x 36864 0.68 (the four-chunk shape, see split_shape), 8 of 1024 x 33000 0.61; beyond
// 131072 columns (two slots per lane, SL = 2) 2 of 1024 x 262144 0.67, 2 of 1024 x 200000 0.59.
// Tried without gain:
// L = 2 (four tiles of eight chunks do not fit 256 registers; with six or seven chunks per lane they do and shapes
// that are whole multiples of 1536 or 1792 columns gain 0.03-0.06, but 65536 columns fall to 0.55), the slots read at
// the top of the iteration (with L = 1 the others' shares are not there yet and the second read costs more than the
// first saved), one wave per workgroup (0.57-0.71), the rows read through buffer descriptors (same rates).  Not what
// holds it back: the waiting itself -- with the poll limit at zero (nobody waits, the numbers are then wrong) the same
// launches run slower, 0.56-0.62 where they run 0.67-0.73: waves that keep pace read a row together, and the memory
// likes that better than 32 waves each at its own row -- nor the loads in flight (the four-chunk shape with the loads two
// iterations ahead: 0.63 where one iteration gives 0.67).
// The waves of a row block wait for one another, so all of them must be on the chip together: the launch never has
// more workgroups than the chip holds at once (launch_fused_split checks the occupancy the runtime reports), and
// every wait is bounded: a wave that polls max_polls times in vain raises `failed`, stops waiting for the rest of
// its rows and runs to its end; k_finish_fused then writes NaN for g and loss of that launch's nodes.
// Two shapes.  Eight 16-byte chunks per lane (2048 columns per wave), two waves per SIMD, L = LA = 1: the faster one where
// a row is whole workgroups of such waves (multiples of 8192 columns) and the only one beyond 65536 columns (a lane reads
// one slot of a row up to 131072 columns, two up to 262144).
// Four chunks per lane (1024 columns per wave), three waves per SIMD, L = 2: for the other widths up to 65536, where the
// first leaves waves idle or half empty (36864 columns 0.55 -> 0.68 of the peak, 40000 0.57 -> 0.66; but 65536 columns
// 0.75 -> 0.70 and 64 nodes of them 0.69 -> 0.61, hence not everywhere; beyond 65536 columns, with two slots per lane, it
// gained nothing: 100000 columns 0.56 either way, 120000 0.53).
struct SplitShape {
    int cpt;        // 16-byte chunks per lane
    int resident;   // workgroups per launch at most: 256 CUs x 2, or x 3
    int wave_cols() const { return 256 * cpt; }
};
constexpr int kSplitNarrowMaxD = 64 * 1024;
SplitShape split_shape(int64_t d) {
    return (d <= kSplitNarrowMaxD && d % 8192 != 0) ? SplitShape{4, 768} : SplitShape{8, 512};
}
constexpr int kSplitWaves = 4;                        // waves per workgroup (they share nothing; neighbours in a row, they read a contiguous piece of it)
constexpr int64_t kMaxSplitD = 128 * 2048;   // 128 slots per row: two loads per lane beyond 131072 columns
constexpr unsigned long long kSlotEmpty = 0x7ff8dec0de5107e1ull;
constexpr int kSplitPolls = 1 << 21;   // seconds; local_grad_lsq_poll_limit sets another number

// The sum over a wave without the LDS crossbar, the same value in every lane: two butterfly steps inside the quads and
// two rotations inside the rows of 16 lanes as data-parallel moves, then lane 0 of each row read into scalar
// registers and added in a fixed order.  (wave_sum's six permutes through LDS and the waits on them are about 600
// cycles; a row of k_fused_split has two such sums on the path that paces the waves of a row block.)
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
    const unsigned long long bits = __builtin_bit_cast(unsigned long long, v);
    const int lo = __builtin_amdgcn_update_dpp(0, static_cast<int>(bits), CTRL, 0xf, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, static_cast<int>(bits >> 32), CTRL, 0xf, 0xf, false);
    return __builtin_bit_cast(double, (static_cast<unsigned long long>(static_cast<unsigned>(hi)) << 32) | static_cast<unsigned>(lo));
}
__device__ __forceinline__ double lane_value(double v, int lane) {   // uniform result
    const unsigned long long bits = __builtin_bit_cast(unsigned long long, v);
    const unsigned lo = static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(bits), lane));
    const unsigned hi = static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(bits >> 32), lane));
    return __builtin_bit_cast(double, (static_cast<unsigned long long>(hi) << 32) | lo);
}
__device__ __forceinline__ double wave_sum_uniform(double v) {
    v += dpp_move<0xB1>(v);    // quad_perm [1, 0, 3, 2]: lane ^ 1
    v += dpp_move<0x4E>(v);    // quad_perm [2, 3, 0, 1]: lane ^ 2
    v += dpp_move<0x124>(v);   // row_ror 4: the next quad of the row
    v += dpp_move<0x128>(v);   // row_ror 8: the other half of the row
    return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}

__device__ __forceinline__ unsigned long long slot_load(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(kThreads) void k_fill_slots(unsigned long long* __restrict__ slots, int64_t count,
                                                        unsigned* __restrict__ failed) {
    for (int64_t k = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; k < count;
         k += static_cast<int64_t>(gridDim.x) * kThreads)
        slots[k] = kSlotEmpty;
    if (blockIdx.x == 0 && threadIdx.x == 0) *failed = 0u;
}

template <int CPT>
struct SplitTile {
    vf4 a[CPT];
    float y;
};

template <int CPT, int WPE, int L, int LA, int SL>   // chunks per lane, waves per SIMD, iterations ahead: publishing, loads; slots read per lane
__global__ __launch_bounds__(64 * kSplitWaves, WPE) void k_fused_split(const float* __restrict__ A, const float* __restrict__ y,
                                                                    const float* __restrict__ x, double* __restrict__ partial,
                                                                    double* __restrict__ sq_partial,
                                                                    unsigned long long* __restrict__ slots,
                                                                    unsigned* __restrict__ failed, int b, int64_t d,
                                                                    int64_t ldA, int64_t ld, int splits, int nslots, int node0,
                                                                    int max_polls, const int32_t* __restrict__ rows, int bs) {
    constexpr int NB = L + LA + 1;   // register tiles in rotation
    constexpr int kWaveCols = 256 * CPT;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int gw = static_cast<int>(blockIdx.x) * kSplitWaves + wave;   // this wave's slot; its columns start at 2048 gw
    if (gw >= nslots) return;   // whole waves only; nothing in this kernel is shared within a workgroup
    const int s = blockIdx.y, i = node0 + static_cast<int>(blockIdx.z);
    // bs logical rows per node: all b rows, or (rows != nullptr) the sampled ones, looked up as they come
    // Row block s takes the logical rows s, s + splits, s + 2 splits, ...: the blocks of a node, which run side by side,
    // then read neighbouring rows of A_i at any moment, one window that moves through the matrix, instead of `splits`
    // places far apart.  Below, r counts the block's own rows (0 .. r1 - 1) and logical(r) is the row it stands for.
    const int r0 = 0;
    const int r1 = (bs - s + splits - 1) / splits;   // r1 >= 1: splits <= bs
    auto logical = [&](int r) -> int { return s + r * splits; };
    const int32_t* __restrict__ rows_i = rows ? rows + static_cast<int64_t>(i) * bs : nullptr;

    // a thread's chunks of x_i wait in LDS (xl[256 q], written and read by this thread alone), not in 32 registers
    __shared__ vf4 x_chunks[CPT * 64 * kSplitWaves];
    vf4* xl = x_chunks + threadIdx.x;
    int col[CPT];   // chunks past column d are clamped to the last one: their x is zero and their sums are never stored
    double acc[CPT][4];
    const bool x_wide = ((reinterpret_cast<uintptr_t>(x) & 15u) | (static_cast<uint64_t>(ld) & 3u)) == 0;
#pragma unroll
    for (int q = 0; q < CPT; ++q) {
        const int64_t c = static_cast<int64_t>(gw) * kWaveCols + 256 * q + 4 * lane;
        const bool inside = c < d;   // d is a multiple of 4: chunks are inside or outside as a whole
        col[q] = static_cast<int>(inside ? c : d - 4);
        const float* xp = x + static_cast<int64_t>(i) * ld + col[q];
        const vf4 xv = x_wide ? *reinterpret_cast<const vf4*>(xp) : vf4{xp[0], xp[1], xp[2], xp[3]};
        xl[64 * kSplitWaves * q] = inside ? xv : vf4{0.f, 0.f, 0.f, 0.f};
        acc[q][0] = acc[q][1] = acc[q][2] = acc[q][3] = 0.0;
    }
    const float* __restrict__ a_node = A + static_cast<int64_t>(i) * b * ldA;
    const float* __restrict__ yi = y + static_cast<int64_t>(i) * b;
    unsigned long long* slots_i = slots + static_cast<int64_t>(i) * bs * nslots;

    // The physical row of logical row r (uniform), asked for one iteration before the loads that need it.
    auto physical = [&](int r) -> int {
        const int row = logical(r < r1 ? r : r1 - 1);   // rows past the block's end read its last row again (never used)
        return rows_i ? physical_row(rows_i, row, b) : row;
    };
    auto load = [&](SplitTile<CPT>& t, int row) {
        const float* __restrict__ a_row = a_node + static_cast<int64_t>(row) * ldA;
        t.y = yi[row];
#pragma unroll
        for (int q = 0; q < CPT; ++q)
            t.a[q] = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(a_row + col[q]));
    };
    auto publish = [&](const SplitTile<CPT>& t, int r) {   // this wave's share of row r's dot product
        if (r >= r1) return;   // uniform
        double s0 = 0.0, s1 = 0.0;
#pragma unroll
        for (int q = 0; q < CPT; ++q) {
            const vf4 xv = xl[64 * kSplitWaves * q];
            s0 = __builtin_fma(static_cast<double>(t.a[q].x), static_cast<double>(xv.x), s0);
            s1 = __builtin_fma(static_cast<double>(t.a[q].y), static_cast<double>(xv.y), s1);
            s0 = __builtin_fma(static_cast<double>(t.a[q].z), static_cast<double>(xv.z), s0);
            s1 = __builtin_fma(static_cast<double>(t.a[q].w), static_cast<double>(xv.w), s1);
        }
        const double p = wave_sum_uniform(s0 + s1);
        unsigned long long bits = __builtin_bit_cast(unsigned long long, p);
        if (bits == kSlotEmpty) bits ^= 1ull;   // (cannot happen with fp32 inputs; the mark stays unique anyway)
        if (lane == 0)
            __hip_atomic_store(slots_i + static_cast<int64_t>(logical(r)) * nslots + gw, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    bool gave_up = false;   // uniform
    double sq = 0.0;
    // The row's slots, SL per lane: lane l reads slots l, l + 64, ... (beyond the last slot: slot 0, counting for nothing).
    struct Slots {
        unsigned long long v[SL];
    };
    auto peek = [&](int r) -> Slots {
        const int row = logical(r < r1 ? r : r1 - 1);
        Slots got;
#pragma unroll
        for (int j = 0; j < SL; ++j)
            got.v[j] = slot_load(slots_i + static_cast<int64_t>(row) * nslots + (lane + 64 * j < nslots ? lane + 64 * j : 0));
        return got;
    };
    auto any_empty = [&](const Slots& got) -> bool {   // uniform
        bool empty = false;
#pragma unroll
        for (int j = 0; j < SL; ++j) empty |= got.v[j] == kSlotEmpty;
        return __builtin_amdgcn_ballot_w64(empty) != 0ull;
    };
    auto consume = [&](const SplitTile<CPT>& t, int r, Slots got) {
        if (r >= r1) return;   // uniform
        if (!gave_up) {
            int polls = 0;
            while (any_empty(got)) {   // until every wave of the block has published
                if (++polls > max_polls) {
                    gave_up = true;
                    if (lane == 0) __hip_atomic_store(failed, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
                got = peek(r);
            }
        }
        double share = 0.0;   // the lane's slots in ascending order, then the wave sum: one order for every wave
#pragma unroll
        for (int j = 0; j < SL; ++j) share += lane + 64 * j < nslots ? __builtin_bit_cast(double, got.v[j]) : 0.0;
        const double res = wave_sum_uniform(share) - static_cast<double>(t.y);   // the same bits in every wave of the block
        sq = __builtin_fma(res, res, sq);
#pragma unroll
        for (int q = 0; q < CPT; ++q) {
            vf4 a = t.a[q];
            asm volatile("" : "+v"(a));   // widened here again: fp64 copies kept since publish() would double the tile's footprint
            acc[q][0] = __builtin_fma(static_cast<double>(a.x), res, acc[q][0]);
            acc[q][1] = __builtin_fma(static_cast<double>(a.y), res, acc[q][1]);
            acc[q][2] = __builtin_fma(static_cast<double>(a.z), res, acc[q][2]);
            acc[q][3] = __builtin_fma(static_cast<double>(a.w), res, acc[q][3]);
        }
    };

    SplitTile<CPT> t[NB];
    // Row rho waits in t[(rho - r0) % NB]: rows r0 .. r0 + L + LA - 1 on their way, the first L of them published.
#pragma unroll
    for (int k = 0; k < L + LA; ++k) load(t[k], physical(r0 + k));
#pragma unroll
    for (int k = 0; k < L; ++k) publish(t[k], r0 + k);
    int prow = physical(r0 + L + LA);
    for (int r = r0; r < r1; r += NB) {
#pragma unroll
        for (int k = 0; k < NB; ++k) {   // row r + k waits in t[k]
            load(t[(k + L + LA) % NB], prow);
            prow = physical(r + k + L + LA + 1);
            publish(t[(k + L) % NB], r + k + L);
            consume(t[k], r + k, peek(r + k));
        }
    }

    // (partial and sq_partial belong to this launch: its first node is their node 0)
    double* out = partial + (static_cast<int64_t>(blockIdx.z) * splits + s) * d;
#pragma unroll
    for (int q = 0; q < CPT; ++q) {
        const int64_t c = static_cast<int64_t>(gw) * kWaveCols + 256 * q + 4 * lane;
        if (c < d) {
            out[c + 0] = acc[q][0]; out[c + 1] = acc[q][1]; out[c + 2] = acc[q][2]; out[c + 3] = acc[q][3];
        }
    }
    if (gw == 0 && lane == 0) sq_partial[static_cast<int64_t>(blockIdx.z) * splits + s] = sq;
}

__global__ __launch_bounds__(kThreads) void k_finish_fused(const double* __restrict__ partial,
                                                            const double* __restrict__ sq_partial,
                                                            float* __restrict__ g, float* __restrict__ loss,
                                                            int64_t d, int64_t ld, int splits, double scale,
                                                            const unsigned* __restrict__ failed) {
    __shared__ double quarter[4][kFinishColumns];
    const int i = blockIdx.y;
    // k_fused_split only: a wave that gave up waiting for the others has used an incomplete residual; the launch's
    // results (and those of the launches after it in the same call) then read NaN
    const bool poisoned = failed != nullptr && *failed != 0u;
    finish_columns(partial + static_cast<int64_t>(i) * splits * d, g + static_cast<int64_t>(i) * ld, d, splits, scale, quarter, poisoned);
    if (loss != nullptr && blockIdx.x == 0 && threadIdx.x < 64) {   // one wave: lane-strided, then the fixed-order wave sum
        double sq = 0.0;
        for (int s = threadIdx.x; s < splits; s += 64) sq += sq_partial[static_cast<int64_t>(i) * splits + s];
        sq = wave_sum(sq);
        if (threadIdx.x == 0) loss[i] = poisoned ? __builtin_nanf("") : static_cast<float>(0.5 * scale * sq);
    }
}

// ---------------------------------------------------------------- small problems
constexpr int kSmallElements = 4096;   // floats of A_i kept in LDS; beyond, one workgroup per node is too little parallelism
constexpr int kSmallD = 2048;
constexpr int kSmallRows = 1024;

bool small_problem(int32_t bs, int64_t d) {
    return d >= 1 && d <= kSmallD && bs <= kSmallRows && static_cast<int64_t>(bs) * d <= kSmallElements;
}
size_t small_lds_bytes(int32_t bs, int64_t d) {
    return static_cast<size_t>(bs) * sizeof(double) + (static_cast<size_t>(bs) * d + d) * sizeof(float);
}

// One workgroup per node.  LDS: res[bs] (fp64), then A_i as bs x d floats, then x_i.  Residuals: a
// wave per row, lanes strided over the columns, fixed-order wave sum.  Gradient: a thread per column,
// rows in order.  Everything in a fixed order: same inputs, same bits.
__global__ __launch_bounds__(kThreads) void k_small(const float* __restrict__ A, const float* __restrict__ y,
                                                     const float* __restrict__ x, float* __restrict__ g,
                                                     float* __restrict__ loss, int b, int d, int64_t ldA,
                                                     int64_t ld, const int32_t* __restrict__ rows, int bs,
                                                     double scale) {
    extern __shared__ double small_lds[];
    double* res = small_lds;
    float* As = reinterpret_cast<float*>(small_lds + bs);
    float* xs = As + static_cast<size_t>(bs) * d;
    const int i = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int32_t* __restrict__ rows_i = rows ? rows + static_cast<int64_t>(i) * bs : nullptr;
    const float* __restrict__ a_node = A + static_cast<int64_t>(i) * b * ldA;
    for (int c = threadIdx.x; c < d; c += kThreads) xs[c] = x[static_cast<int64_t>(i) * ld + c];
    for (int r = wave; r < bs; r += kThreads / 64) {   // a wave copies a row: coalesced along the columns
        const int pr = rows_i ? physical_row(rows_i, r, b) : r;
        const float* __restrict__ a_row = a_node + static_cast<int64_t>(pr) * ldA;
        for (int c = lane; c < d; c += 64) As[r * d + c] = a_row[c];
    }
    __syncthreads();
    for (int r = wave; r < bs; r += kThreads / 64) {
        double acc = 0.0;
        for (int c = lane; c < d; c += 64)
            acc = __builtin_fma(static_cast<double>(As[r * d + c]), static_cast<double>(xs[c]), acc);
        const double dot = wave_sum(acc);
        if (lane == 0) {
            const int pr = rows_i ? physical_row(rows_i, r, b) : r;
            res[r] = dot - static_cast<double>(y[static_cast<int64_t>(i) * b + pr]);
        }
    }
    __syncthreads();
    for (int c = threadIdx.x; c < d; c += kThreads) {
        double acc = 0.0;
        for (int r = 0; r < bs; ++r) acc = __builtin_fma(static_cast<double>(As[r * d + c]), res[r], acc);
        g[static_cast<int64_t>(i) * ld + c] = static_cast<float>(scale * acc);
    }
    if (loss != nullptr && wave == 0) {   // one wave, fixed order
        double sq = 0.0;
        for (int r = lane; r < bs; r += 64) sq = __builtin_fma(res[r], res[r], sq);
        sq = wave_sum(sq);
        if (lane == 0) loss[i] = static_cast<float>(0.5 * scale * sq);
    }
}

// Row blocks per node for the single sweep: as many workgroups as are resident at once -- two per CU, 512 (one per
// CU, 256, for the 1024-thread kernel beyond d = 8192); more, shorter ones lose up to 15 % -- but at least one double
// tile and at least eight rows each: every workgroup writes a partial gradient of d doubles, which the final pass
// reads again, as much traffic as four rows of A each way.  Measured, workgroups in total 128 / 256 / 512 / 1024:
// 8 nodes of 1024 x 1024: 26.7 / 16.5 / 14.8 / 17.4 us; 8 nodes of 256 x 4096: 17.0 / 14.8 / 21.0 / 24.7 us;
// 64 nodes of 4096 x 4096: 1312 / 747 / 624 / 691 us; 16 nodes of 1024 x 16384: 292 / 185 / 201 / 231 us.
// Short rows (k_fused_rows) have fewer bytes in flight per workgroup and want more of them: 64 nodes of
// 32768 x 128 with 512 / 1024 / 2048 / 4096 workgroups 224 / 175 / 173 / 175 us, of 16384 x 256 216 / 172 / 170 / 179,
// 4 nodes of 100000 x 300 115 / 86 / 86 / 86, but 64 nodes of 8192 x 512 165 / 166 / 172 / 183 and of 4096 x 1024
// 158 / 182 / 182 / 194.
int fused_splits(int32_t n, int32_t b, int64_t d, int rows_per_iteration) {
    const int64_t resident = d > 8192 ? 256 : d > 384 ? 512 : d > 256 ? 1024 : 2048;
    int64_t s = (resident + n / 2) / n;
    const int64_t rows_each = rows_per_iteration > 8 ? rows_per_iteration : 8;
    const int64_t most = (b + rows_each - 1) / rows_each;
    if (s > most) s = most;
    const int64_t cap = d > 4096 ? 256 : 512;   // the final pass adds a node's partials a quarter per wave, one after the other
    if (s > cap) s = cap;
    if (s < 1) s = 1;
    return static_cast<int>(s);
}

// rows consumed per loop iteration: by a workgroup of k_fused_rows in its 16-byte shapes up to d = 1024, then two
// register tiles of R rows, or one without prefetch
int fused_rows(int64_t d) {
    return d <= 32 ? 256 : d <= 64 ? 128 : d <= 128 ? 64 : d <= 256 ? 32 : d <= 512 ? 16 : d <= 1024 ? 8 : d <= 2048 ? 4 : d <= 4096 ? 2 : 1;
}
constexpr int kMaxNarrowD = 16384;  // rows off the 16-byte boundaries: 1024 threads x 16 columns
constexpr int kMaxFusedD = 32768;   // 1024 threads x 8 chunks of 4 columns (from 16385 on with x_i in LDS)

// Short rows: a wave per row (or per 2, 4, 8 rows); V columns per access and lane.
constexpr int kMaxRowsKernelD = 1024;   // any alignment
// With rows on 16-byte boundaries and d a multiple of 4 the wave-per-row kernel also beats k_fused where k_fused's
// shapes fit badly, its steps being 256 columns where k_fused's are 1024 (16 nodes, 256 M elements of A, fraction
// of the HBM peak, k_fused_rows / k_fused): d = 1028 0.85 / 0.42, 1540 0.82 / 0.72, 1792 0.80, 1900 - / 0.69,
// 2000 - / 0.80, 2048 0.79 / 0.82, 2052 0.76 / 0.61, 2560 0.77 / 0.65, 2564 - / 0.83, 2600 0.68 / -, 3000 0.73 / 0.83
// (k_fused with three chunks per thread from 2561 on).
// Rows off the 16-byte boundaries, or a d that is not a multiple of 4 with aligned rows above 1024: a wave per row up to
// 2048 columns (k_fused_narrow there, with its barrier per tile of a few short rows: 0.31-0.62 of the peak).
bool rows_kernel_serves(int64_t d, bool aligned_rows) {
    if (d <= kMaxRowsKernelD) return true;
    if (!aligned_rows) return d <= 3072;
    return d % 4 == 0 && (d <= 1960 || (d > 2048 && d <= 2560));
}
template <int V>
int launch_fused_rows(dim3 grid, hipStream_t stream, const float* A, const float* y, const float* x, double* fpartial,
                      double* sq_partial, int32_t b, int64_t d, int64_t ldA, int64_t ld, int fs, const int32_t* rows,
                      int32_t bs) {
    const dim3 block(256);
    const int64_t chunks = (d + V - 1) / V;
#define DL_ROWS_KERNEL(CPW, L, R) \
    hipLaunchKernelGGL((k_fused_rows<V, CPW, L, R>), grid, block, 0, stream, A, y, x, fpartial, sq_partial, b, d, ldA, ld, fs, rows, bs)
    if (chunks <= 8) DL_ROWS_KERNEL(1, 8, 8);
    else if (chunks <= 16) DL_ROWS_KERNEL(1, 16, 8);
    else if (chunks <= 32) DL_ROWS_KERNEL(1, 32, 8);
    else if (chunks <= 64) DL_ROWS_KERNEL(1, 64, 8);
    else if (chunks <= 128) DL_ROWS_KERNEL(2, 64, 4);
    else if (chunks <= 192) DL_ROWS_KERNEL(3, 64, 2);
    else if (chunks <= 256) DL_ROWS_KERNEL(4, 64, 2);
    else if constexpr (V == 4) {   // 1025-1960 and 2049-2560 columns on 16-byte boundaries, see rows_kernel_serves
        if (chunks <= 320) DL_ROWS_KERNEL(5, 64, 1);
        else if (chunks <= 384) DL_ROWS_KERNEL(6, 64, 1);
        else if (chunks <= 448) DL_ROWS_KERNEL(7, 64, 1);
        else if (chunks <= 512) DL_ROWS_KERNEL(8, 64, 1);
        else DL_ROWS_KERNEL(10, 64, 1);
    } else if constexpr (V == 2) {   // rows on 8-byte boundaries: up to 2048 columns
        if (chunks <= 512) DL_ROWS_KERNEL(8, 64, 1);
        else if (chunks <= 640) DL_ROWS_KERNEL(10, 64, 1);
        else if (chunks <= 768) DL_ROWS_KERNEL(12, 64, 1);
        else if (chunks <= 1024) DL_ROWS_KERNEL(16, 64, 1);
        else if (chunks <= 1280) DL_ROWS_KERNEL(20, 64, 1);
        else DL_ROWS_KERNEL(24, 64, 1);
    } else {                         // any rows: up to 2048 columns
        if (chunks <= 512) DL_ROWS_KERNEL(8, 64, 1);
        else if (chunks <= 1024) DL_ROWS_KERNEL(16, 64, 1);
        else if (chunks <= 1536) DL_ROWS_KERNEL(24, 64, 1);
        else if (chunks <= 2048) DL_ROWS_KERNEL(32, 64, 1);
        else if (chunks <= 2560) DL_ROWS_KERNEL(40, 64, 1);
        else DL_ROWS_KERNEL(48, 64, 1);
    }
#undef DL_ROWS_KERNEL
    return check_hip(hipGetLastError(), "fused gradient kernel launch (short rows)");
}

// The single sweep's kernel by columns per row (TAIL: d is not a multiple of 4).
// One chunk column of 1024 (256 threads) or 4096 (1024 threads) columns more per shape: a shape made for twice the
// columns loads, and throws away, up to as much again as it uses (16 nodes, 256 M elements of A: d = 2500 / 5000 /
// 10000 / 20000 ran at 0.64 / 0.65 / 0.59 / 0.64 of the HBM peak with the shapes of 4096 / 8192 / 16384 / 32768 columns).
template <bool TAIL>
int launch_fused(dim3 grid, hipStream_t stream, const float* A, const float* y, const float* x, double* fpartial,
                 double* sq_partial, int32_t b, int64_t d, int64_t ldA, int64_t ld, int fs, const int32_t* rows, int32_t bs) {
#define DL_FUSED(CPT, R, PF, THREADS) \
    hipLaunchKernelGGL((k_fused<CPT, R, PF, THREADS, false, TAIL>), grid, dim3(THREADS), 0, stream, A, y, x, fpartial, sq_partial, b, d, ldA, ld, fs, rows, bs)
    // more than 16384 columns: eight chunks per thread would be a row of A (32 registers) and the accumulators (64)
    // filling the thread's 128 registers, so its chunks of x_i wait in LDS (16 KiB per chunk column, one workgroup per CU)
    auto wide = [&](auto chunks) -> int {
        constexpr int CPT = decltype(chunks)::value;
        auto kernel = k_fused<CPT, 1, false, 1024, true, TAIL>;
        static std::atomic<uint64_t> configured{0};   // per instantiation: one bit per device ordinal below 64
        int device = 0;
        if (int rc = check_hip(hipGetDevice(&device), "hipGetDevice")) return rc;
        const uint64_t bit = device >= 0 && device < 64 ? uint64_t{1} << device : uint64_t{0};
        if (!(configured.load(std::memory_order_relaxed) & bit) || bit == 0) {
            if (int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, CPT * 16 * 1024),
                                   "hipFuncSetAttribute(max dynamic LDS)"))
                return rc;
            configured.fetch_or(bit, std::memory_order_relaxed);
        }
        hipLaunchKernelGGL(kernel, grid, dim3(1024), CPT * 16 * 1024, stream, A, y, x, fpartial, sq_partial, b, d, ldA, ld, fs, rows, bs);
        return 0;
    };
    if (d <= 1024) {   // a handful of rows per node, see launch_lsq
        if constexpr (!TAIL) DL_FUSED(1, 4, true, 256);
    }
    else if (d <= 2048) DL_FUSED(2, 2, true, 256);
    else if (d <= 3072) DL_FUSED(3, 1, true, 256);
    else if (d <= 4096) DL_FUSED(4, 1, true, 256);
    else if (d <= 5120) DL_FUSED(5, 1, true, 256);
    else if (d <= 6144) DL_FUSED(6, 1, false, 256);   // (with prefetch: 0.76-0.78 against 0.82)
    else if (d <= 7168) DL_FUSED(7, 1, false, 256);
    else if (d <= 8192) DL_FUSED(8, 1, false, 256);
    else if (d <= 12288) DL_FUSED(3, 1, false, 1024);   // (with prefetch, or as five or six chunks of 512 threads, it does not fit 128 registers)
    else if (d <= 16384) DL_FUSED(4, 1, false, 1024);
    else if (d <= 20480) { if (int rc = wide(std::integral_constant<int, 5>())) return rc; }
    else if (d <= 24576) { if (int rc = wide(std::integral_constant<int, 6>())) return rc; }
    else if (d <= 28672) { if (int rc = wide(std::integral_constant<int, 7>())) return rc; }
    else { if (int rc = wide(std::integral_constant<int, 8>())) return rc; }
#undef DL_FUSED
    return check_hip(hipGetLastError(), "fused gradient kernel launch");
}

// The single sweep with narrow accesses, by columns per row (V = 2: rows on 8-byte boundaries, V = 1: any).
template <int V>
int launch_fused_narrow(dim3 grid, hipStream_t stream, const float* A, const float* y, const float* x, double* fpartial,
                        double* sq_partial, int32_t b, int64_t d, int64_t ldA, int64_t ld, int fs, const int32_t* rows,
                        int32_t bs) {
#define DL_NARROW(K, R, THREADS) \
    hipLaunchKernelGGL((k_fused_narrow<V, K, R, THREADS>), grid, dim3(THREADS), 0, stream, A, y, x, fpartial, sq_partial, b, d, ldA, ld, fs, rows, bs)
    // K columns per thread: a shape per 512 or 1024 columns (256 threads), per 4096 beyond 8192; two or four rows per
    // tile where the columns are few (2502 columns, 8-byte accesses: 0.43 / 0.50 / 0.61 of the peak with 1 / 2 / 4)
    if (d <= 2560) DL_NARROW(10, 4, 256);   // (up to 2048: k_fused_rows)
    else if (d <= 3072) DL_NARROW(12, 4, 256);
    else if (d <= 4096) DL_NARROW(16, 2, 256);
    else if (d <= 5120) DL_NARROW(20, 2, 256);
    else if (d <= 6144) DL_NARROW(24, 2, 256);
    else if (d <= 7168) DL_NARROW(28, 1, 256);
    else if (d <= 8192) DL_NARROW(32, 1, 256);
    else if (d <= 12288) DL_NARROW(12, 1, 1024);
    else DL_NARROW(16, 1, 1024);
#undef DL_NARROW
    return check_hip(hipGetLastError(), "fused gradient kernel launch (narrow accesses)");
}

// How a call over rows wider than kMaxFusedD is cut up for k_fused_split: launches of `nodes` nodes with `splits` row
// blocks each, a wave per 2048 or 1024 columns of a row block, so that no launch has more workgroups than the chip
// holds at once (split_shape).  A pure
// function of the shape (no device query): the workspace size depends on it.  Few nodes per launch allow more row
// blocks per node and so fill the chip better where nodes x slots divides the chip badly (8 nodes of 65536 columns,
// 43 slots: one launch of 8 x 5 blocks uses 1720 of 2048 waves, two launches of 4 x 11 blocks 1892); every launch
// costs its pipeline's fill and drain and the gap to the next, priced at 24 rows' time.
struct SplitChunk {
    int nodes, splits;
};
int split_slots(int64_t d) { return static_cast<int>((d + split_shape(d).wave_cols() - 1) / split_shape(d).wave_cols()); }
SplitChunk split_chunk(int n_left, int32_t b, int nslots, int resident) {
    const int blocks = resident / ((nslots + kSplitWaves - 1) / kSplitWaves);   // row blocks per launch: 32 or more up to kMaxSplitD
    const int most = b >= 32 ? b / 16 : 1;        // a row block has 16 rows or more
    SplitChunk best{1, 1};
    int64_t best_cost = INT64_MAX;
    for (int m = n_left < blocks ? n_left : blocks; m >= 1; --m) {
        int s = blocks / m;
        if (s > most) s = most;
        const int64_t launches = (n_left + m - 1) / m;
        const int64_t cost = launches * ((b + s - 1) / s + 24);
        if (cost < best_cost) {
            best_cost = cost;
            best = SplitChunk{m, s};
        }
    }
    return best;
}
// The plan is made for b rounded down to a power of two, and the workspace holds the largest plan of all such values
// up to b: its size then never shrinks when b grows (a workspace sized for b rows serves every smaller batch).
int split_plan_rows(int32_t b) {
    int q = 1;
    while (2 * static_cast<int64_t>(q) <= b) q *= 2;
    return q;
}
size_t split_sums_doubles(int32_t n, int32_t plan_rows, int64_t d, int nslots) {
    const int resident = split_shape(d).resident;
    size_t doubles = 0;
    for (int node0 = 0; node0 < n;) {
        const SplitChunk c = split_chunk(n - node0, plan_rows, nslots, resident);
        const size_t blocks = static_cast<size_t>(c.nodes) * c.splits;
        doubles += ((blocks + 1) & ~size_t{1}) + blocks * static_cast<size_t>(d);
        node0 += c.nodes;
    }
    return doubles;
}
// bytes: the slots and the failure word, then every launch's sums of squares and partial gradients
size_t split_workspace_bytes(int32_t n, int32_t b, int64_t d) {
    const int nslots = split_slots(d);
    size_t sums = 0;
    for (int64_t q = 1; q <= b; q *= 2) {
        const size_t v = split_sums_doubles(n, static_cast<int32_t>(q), d, nslots);
        if (v > sums) sums = v;
    }
    return (static_cast<size_t>(n) * static_cast<size_t>(b) * nslots + 2 + sums) * sizeof(double);
}

// Workgroups of k_fused_split the current device holds at once (asked once per device); 0 on error.
template <int CPT, int WPE, int L, int LA, int SL>
int split_resident_workgroups() {
    static std::atomic<int> known[64];
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return 0;
    if (device >= 0 && device < 64) {
        const int v = known[device].load(std::memory_order_relaxed);
        if (v) return v;
    }
    int per_cu = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_fused_split<CPT, WPE, L, LA, SL>, 64 * kSplitWaves, 0) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) return 0;
    const int total = per_cu * cus;
    if (device >= 0 && device < 64 && total > 0) known[device].store(total, std::memory_order_relaxed);
    return total;
}

std::atomic<int> g_split_polls{kSplitPolls};

// Returns DL_OK after launching, a status on error, or -1 when the device cannot hold a launch at once (the caller
// then takes the two sweeps).
int launch_fused_split(hipStream_t stream, const float* A, const float* y, const float* x, float* g, float* loss,
                       int32_t n, int32_t b, int64_t d, int64_t ldA, int64_t ld, const int32_t* rows, int32_t bs,
                       double scale, void* workspace) {
    const int nslots = split_slots(d);
    const SplitShape shape = split_shape(d);
    const bool narrow = shape.cpt == 4, two_slots = nslots > 64;
    const int resident = narrow ? split_resident_workgroups<4, 3, 2, 1, 1>()
                         : two_slots ? split_resident_workgroups<8, 2, 1, 1, 2>() : split_resident_workgroups<8, 2, 1, 1, 1>();
    if (resident < shape.resident) return -1;
    unsigned long long* slots = static_cast<unsigned long long*>(workspace);
    const int64_t slot_count = static_cast<int64_t>(n) * bs * nslots;
    unsigned* failed = reinterpret_cast<unsigned*>(slots + slot_count);
    double* sums = reinterpret_cast<double*>(slots + slot_count + 2);
    const int64_t fill_blocks = (slot_count + 4 * kThreads - 1) / (4 * kThreads);
    hipLaunchKernelGGL(k_fill_slots, dim3(static_cast<unsigned>(fill_blocks < 2048 ? (fill_blocks < 1 ? 1 : fill_blocks) : 2048)),
                       dim3(kThreads), 0, stream, slots, slot_count, failed);
    if (int rc = check_hip(hipGetLastError(), "slot fill kernel launch")) return rc;
    for (int node0 = 0; node0 < n;) {
        const SplitChunk c = split_chunk(n - node0, split_plan_rows(bs), nslots, shape.resident);
        const size_t blocks = static_cast<size_t>(c.nodes) * c.splits;
        double* sq_partial = sums;
        double* fpartial = sums + ((blocks + 1) & ~size_t{1});
        sums = fpartial + blocks * static_cast<size_t>(d);
        const dim3 grid(static_cast<unsigned>((nslots + kSplitWaves - 1) / kSplitWaves), static_cast<unsigned>(c.splits), static_cast<unsigned>(c.nodes));
        const int polls = g_split_polls.load(std::memory_order_relaxed);
        if (narrow)
            hipLaunchKernelGGL((k_fused_split<4, 3, 2, 1, 1>), grid, dim3(64 * kSplitWaves), 0, stream, A, y, x, fpartial, sq_partial,
                               slots, failed, b, d, ldA, ld, c.splits, nslots, node0, polls, rows, bs);
        else if (two_slots)
            hipLaunchKernelGGL((k_fused_split<8, 2, 1, 1, 2>), grid, dim3(64 * kSplitWaves), 0, stream, A, y, x, fpartial, sq_partial,
                               slots, failed, b, d, ldA, ld, c.splits, nslots, node0, polls, rows, bs);
        else
            hipLaunchKernelGGL((k_fused_split<8, 2, 1, 1, 1>), grid, dim3(64 * kSplitWaves), 0, stream, A, y, x, fpartial, sq_partial,
                               slots, failed, b, d, ldA, ld, c.splits, nslots, node0, polls, rows, bs);
        if (int rc = check_hip(hipGetLastError(), "fused gradient kernel launch (columns split over waves)")) return rc;
        const dim3 grid_ff(static_cast<unsigned>((d + kFinishColumns - 1) / kFinishColumns), static_cast<unsigned>(c.nodes));
        hipLaunchKernelGGL(k_finish_fused, grid_ff, dim3(kThreads), 0, stream, fpartial, sq_partial, g + static_cast<int64_t>(node0) * ld,
                           loss ? loss + node0 : nullptr, d, ld, c.splits, scale, static_cast<const unsigned*>(failed));
        if (int rc = check_hip(hipGetLastError(), "finish kernel launch")) return rc;
        node0 += c.nodes;
    }
    return DL_OK;
}

}  // namespace

bool lsq_wide_accesses(const float* A, const float* x, int64_t d, int64_t ldA, int64_t ld) {
    (void)x; (void)d; (void)ld;   // the single sweep reads x_i once per workgroup, at whatever alignment it has
    return ldA % 4 == 0 && (reinterpret_cast<uintptr_t>(A) & 15u) == 0;
}

// b = rows actually used per node.  path: 0 the two-sweep kernels, 1 the single sweep, 2 the small-problem kernel,
// 3 the single sweep with a row's columns split over waves (launch_lsq picks by shape and alignment), -1 the largest.
size_t lsq_workspace_bytes_path(int32_t n, int32_t b, int64_t d, int path) {
    // two-sweep layout: res[n*b], partial[n*splits*d]; single-sweep layout: sq[n*splits], partial[n*splits*d]
    const size_t res = static_cast<size_t>(n) * static_cast<size_t>(b);
    const size_t partial = static_cast<size_t>(n) * static_cast<size_t>(row_splits(n, b, d)) * static_cast<size_t>(d);
    const size_t two_sweeps = (res + partial) * sizeof(double) + 16;
    size_t fused = 0;
    if (d > 0 && d <= kMaxFusedD) {
        const size_t fs = static_cast<size_t>(fused_splits(n, b, d, fused_rows(d)));
        fused = (static_cast<size_t>(n) * fs * (static_cast<size_t>(d) + 1)) * sizeof(double) + 16;
    }
    // the column-split sweep falls back to the two sweeps on a device that cannot hold its launch at once
    size_t split = 0;
    if (d > kMaxFusedD && d <= kMaxSplitD && d % 4 == 0) {
        split = split_workspace_bytes(n, b, d);
        if (split < two_sweeps) split = two_sweeps;
    }
    if (path == 0) return two_sweeps;
    if (path == 1) return fused;
    if (path == 2) return 0;
    if (path == 3) return split;
    const size_t most = fused > two_sweeps ? fused : two_sweeps;
    return split > most ? split : most;
}

size_t lsq_workspace_bytes(int32_t n, int32_t b, int64_t d) { return lsq_workspace_bytes_path(n, b, d, -1); }

int lsq_poll_limit(int polls) { return g_split_polls.exchange(polls < 0 ? kSplitPolls : polls, std::memory_order_relaxed); }

// wide_accesses: rows of A on 16-byte boundaries (lsq_wide_accesses).  The single sweep also takes a d that is
// not a multiple of 4 (its last d % 4 columns element by element), from d = 8 on, and, up to d = 16384 and with
// narrower accesses, rows that are not on such boundaries.
int lsq_path(int32_t bs, int64_t d, bool wide_accesses, bool sampled) {
    if (small_problem(bs, d)) return 2;
    if (d <= 0) return 0;
    if (d <= kMaxRowsKernelD) return 1;                     // a wave per row, any alignment
    if (!wide_accesses) return d <= kMaxNarrowD ? 1 : 0;   // narrow accesses, same workspace layout
    if (d <= kMaxFusedD) return 1;
    (void)sampled;
    return (d <= kMaxSplitD && d % 4 == 0) ? 3 : 0;   // columns split over waves
}

int launch_lsq(const float* A, const float* y, const float* x, float* g, float* loss, int32_t n,
               int32_t b, int64_t d, int64_t ldA, int64_t ld, const int32_t* rows, int32_t bs, float scale,
               void* workspace, hipStream_t stream) {
    if (rows == nullptr) bs = b;
    double* res = static_cast<double*>(workspace);
    double* partial = res + ((static_cast<size_t>(n) * bs + 1) & ~size_t{1});  // keep 16-byte alignment
    const int splits = row_splits(n, bs, d);
    const bool aligned_rows = lsq_wide_accesses(A, x, d, ldA, ld);
    // the two sweeps' 16-byte loads need whole chunks, of x_i too
    const bool vec4 = aligned_rows && d % 4 == 0 && ld % 4 == 0 && (reinterpret_cast<uintptr_t>(x) & 15u) == 0;
    int path = lsq_path(bs, d, aligned_rows, rows != nullptr);
    if (n > 65535 || splits > 65535) return set_error(DL_EINVAL, "local_grad_lsq: n too large for the launch grid");
    if (path == 3) {
        const int rc = launch_fused_split(stream, A, y, x, g, loss, n, b, d, ldA, ld, rows, bs, static_cast<double>(scale), workspace);
        if (rc >= 0) return rc;
        path = 0;   // this device does not hold the launch at once
    }

    const dim3 block(kThreads);
    if (path == 2) {
        const size_t lds = small_lds_bytes(bs, d);
        if (lds > 48 * 1024) {
            if (int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(k_small),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)),
                                   "hipFuncSetAttribute(max dynamic LDS)"))
                return rc;
        }
        hipLaunchKernelGGL(k_small, dim3(static_cast<unsigned>(n)), block, lds, stream, A, y, x, g, loss, b,
                           static_cast<int>(d), ldA, ld, rows, bs, static_cast<double>(scale));
        return check_hip(hipGetLastError(), "small gradient kernel launch");
    }
    if (path == 1) {
        const int fs = fused_splits(n, bs, d, fused_rows(d));
        double* sq_partial = static_cast<double*>(workspace);
        double* fpartial = sq_partial + ((static_cast<size_t>(n) * fs + 1) & ~size_t{1});
        const dim3 grid(static_cast<unsigned>(fs), static_cast<unsigned>(n));
        int rc;
        const bool even = ldA % 2 == 0 && (reinterpret_cast<uintptr_t>(A) & 7u) == 0;
        // (up to 64 rows per node of 513-1024 columns on 16-byte boundaries keep k_fused with one chunk per thread: such
        // calls are bound by latency, and its 5.5 us against 6.2 are 5 % of the small least-squares workload's iteration)
        const bool few_rows = bs <= 64 && d > 512 && aligned_rows && d % 4 == 0;
        if (rows_kernel_serves(d, aligned_rows) && !few_rows) {
            if (aligned_rows && d % 4 == 0)
                rc = launch_fused_rows<4>(grid, stream, A, y, x, fpartial, sq_partial, b, d, ldA, ld, fs, rows, bs);
            else if (even && d % 2 == 0)
                rc = launch_fused_rows<2>(grid, stream, A, y, x, fpartial, sq_partial, b, d, ldA, ld, fs, rows, bs);
            else
                rc = launch_fused_rows<1>(grid, stream, A, y, x, fpartial, sq_partial, b, d, ldA, ld, fs, rows, bs);
        } else if (!aligned_rows) {
            rc = even ? launch_fused_narrow<2>(grid, stream, A, y, x, fpartial, sq_partial, b, d, ldA, ld, fs, rows, bs)
                      : launch_fused_narrow<1>(grid, stream, A, y, x, fpartial, sq_partial, b, d, ldA, ld, fs, rows, bs);
        } else {
            rc = d % 4 == 0 ? launch_fused<false>(grid, stream, A, y, x, fpartial, sq_partial, b, d, ldA, ld, fs, rows, bs)
                            : launch_fused<true>(grid, stream, A, y, x, fpartial, sq_partial, b, d, ldA, ld, fs, rows, bs);
        }
        if (rc) return rc;
        const dim3 grid_ff(static_cast<unsigned>((d + kFinishColumns - 1) / kFinishColumns), static_cast<unsigned>(n));
        hipLaunchKernelGGL(k_finish_fused, grid_ff, block, 0, stream, fpartial, sq_partial, g, loss, d, ld, fs,
                           static_cast<double>(scale), static_cast<const unsigned*>(nullptr));
        return check_hip(hipGetLastError(), "finish kernel launch");
    }

    // few long rows: a workgroup per row (a wave per row would occupy n * bs / 4 workgroups only)
    const bool wide = static_cast<int64_t>(n) * bs <= 4096 && d >= 4096;
    const dim3 grid_r(static_cast<unsigned>(wide ? bs : (bs + 3) / 4), static_cast<unsigned>(n));
    if (vec4 && wide)
        hipLaunchKernelGGL((k_residual<true, true>), grid_r, block, 0, stream, A, y, x, res, b, d, ldA, ld, rows, bs);
    else if (vec4)
        hipLaunchKernelGGL((k_residual<true, false>), grid_r, block, 0, stream, A, y, x, res, b, d, ldA, ld, rows, bs);
    else if (wide)
        hipLaunchKernelGGL((k_residual<false, true>), grid_r, block, 0, stream, A, y, x, res, b, d, ldA, ld, rows, bs);
    else
        hipLaunchKernelGGL((k_residual<false, false>), grid_r, block, 0, stream, A, y, x, res, b, d, ldA, ld, rows, bs);
    if (int rc = check_hip(hipGetLastError(), "residual kernel launch")) return rc;

    if (d > 0) {
        const int V = vec4 ? 4 : 1;
        const dim3 grid_t(static_cast<unsigned>((d + static_cast<int64_t>(V) * kThreads - 1) / (static_cast<int64_t>(V) * kThreads)),
                          static_cast<unsigned>(splits), static_cast<unsigned>(n));
        if (vec4)
            hipLaunchKernelGGL(k_transpose<true>, grid_t, block, 0, stream, A, res, partial, b, d, ldA, splits, rows, bs);
        else
            hipLaunchKernelGGL(k_transpose<false>, grid_t, block, 0, stream, A, res, partial, b, d, ldA, splits, rows, bs);
        if (int rc = check_hip(hipGetLastError(), "transpose kernel launch")) return rc;
    }

    const dim3 grid_f(static_cast<unsigned>(d > 0 ? (d + kFinishColumns - 1) / kFinishColumns : 1), static_cast<unsigned>(n));
    hipLaunchKernelGGL(k_finish, grid_f, block, 0, stream, partial, res, g, loss, bs, d, ld, splits,
                       static_cast<double>(scale));
    return check_hip(hipGetLastError(), "finish kernel launch");
}

}  // namespace dl

// ---------------------------------------------------------------- local_grad_lsq_static
// The same gradient for callers that cannot hand over (or allocate) a workspace: the partial sums go
// to an array that is part of the library's device image.  Every GPU that loads the library holds its
// own copy at its own address until the process ends; in host code the array's name is only a handle,
// so the address is asked for once per device and that pointer is what the kernels get.
namespace dl {
namespace {

static __device__ __align__(256) unsigned char scratch[DL_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];   // per device ordinal; zero-initialised

// Address of the current device's copy of `scratch` (resolved on the first call on that device).
int static_scratch(void** out) {
    int device = 0;
    if (int rc = check_hip(hipGetDevice(&device), "hipGetDevice")) return rc;
    if (device < 0 || device >= kMaxDevices)
        return set_error(DL_EINVAL, "local_grad_lsq_static: device ordinal %d, at most %d devices are supported", device,
                         kMaxDevices);
    void* p = g_scratch_ptr[device].load(std::memory_order_acquire);
    if (p == nullptr) {
        if (int rc = check_hip(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)")) return rc;
        if (p == nullptr) return set_error(DL_EHIP, "local_grad_lsq_static: the scratch array has no device address");
        g_scratch_ptr[device].store(p, std::memory_order_release);   // two threads racing store the same value
    }
    *out = p;
    return DL_OK;
}

}  // namespace
}  // namespace dl

extern "C" int local_grad_lsq_static(const float* A, const float* y, const float* x, float* g, float* loss, int32_t n,
                                     int32_t b, int64_t d, int64_t ldA, int64_t ld, float scale, void* stream) {
    using namespace dl;
    clear_error();
    // sizes first: a problem beyond the array is refused before anything touches the device
    if (n >= 1 && b >= 1 && d >= 0) {
        const size_t need = lsq_workspace_bytes_path(n, b, d, lsq_path(b, d, lsq_wide_accesses(A, x, d, ldA, ld)));
        if (need > static_cast<size_t>(DL_STATIC_SCRATCH_BYTES))
            return set_error(DL_ECAP, "local_grad_lsq_static: n = %d, b = %d, d = %lld needs %zu bytes of scratch, the "
                             "library's array holds DL_STATIC_SCRATCH_BYTES = %zu; use local_grad_lsq with a workspace",
                             n, b, static_cast<long long>(d), need, static_cast<size_t>(DL_STATIC_SCRATCH_BYTES));
    }
    void* ws = nullptr;
    if (int rc = static_scratch(&ws)) return rc;
    return lsq_entry("local_grad_lsq_static", A, y, x, g, loss, n, b, d, ldA, ld, nullptr, b, false, scale, ws,
                     static_cast<size_t>(DL_STATIC_SCRATCH_BYTES), stream, /*exact_need=*/true);
}
