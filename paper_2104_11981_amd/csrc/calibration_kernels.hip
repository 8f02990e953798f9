// Bare streams with the step kernel's access pattern: the achievable-bandwidth denominator of the
// benchmark.  No arithmetic of the method, no LDS tile, no neighbour list: a workgroup of 16 waves owns
// the same 256 columns of all n <= 32 rows that a tile of the step kernel owns (wave w takes rows w and
// w + 16), issues the same non-temporal 16-byte loads of x, g, m up front, meets at one barrier and
// issues the same stores of m and x.  What such a stream reaches is what this GPU's memory gives a
// kernel that reads three arrays and writes two in this tile order; the step kernel is priced against
// it beside the 8 TB/s figure.
//
// Tile orders: plain (tile t owns columns [256 t, 256 t + 256)) and split (tile u of every 64 KiB unit
// owns columns [128 u, 128 u + 128) of the unit and the same columns 8192 further on: the order of the
// step kernel's large launches, see split_column in step_impl.hpp).
#include "internal.hpp"
#include "step_impl.hpp"

namespace dl {
namespace {

typedef float vf4 __attribute__((ext_vector_type(4)));

// KIND 0: x <- x + c g, m <- c m + g (3 reads, 2 writes); 1: the three reads only; 2: the two writes only
template <int KIND>
__global__ __launch_bounds__(1024) void k_stream(float* __restrict__ x, float* __restrict__ m,
                                                  const float* __restrict__ g, int n, int64_t ld, int split, float c) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t col = split ? step::split_column(blockIdx.x, lane) : static_cast<int64_t>(blockIdx.x) * 256 + lane * 4;
    vf4 xv[2], gv[2], mv[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int i = wave + 16 * r;
        const int64_t at = static_cast<int64_t>(i < n ? i : 0) * ld + col;   // rows beyond n: row 0, in bounds, unused
        if constexpr (KIND != 2) {
            xv[r] = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(x + at));
            gv[r] = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(g + at));
            mv[r] = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(m + at));
        } else {
            xv[r] = gv[r] = mv[r] = vf4{c, c, c, c};
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int i = wave + 16 * r;
        const vf4 x_new = xv[r] + c * gv[r], m_new = c * mv[r] + gv[r];
        if constexpr (KIND == 1) {
            asm volatile("" : : "v"(x_new), "v"(m_new));   // the loads must happen; nothing is stored
        } else if (i < n) {
            const int64_t at = static_cast<int64_t>(i) * ld + col;
            __builtin_nontemporal_store(m_new, reinterpret_cast<vf4*>(m + at));
            __builtin_nontemporal_store(x_new, reinterpret_cast<vf4*>(x + at));
        }
    }
}

}  // namespace
}  // namespace dl

extern "C" int dl_calibration_stream(int kind, int split, float* x, float* m, const float* g, int32_t n, int64_t d,
                                     int64_t ld, int64_t* columns_out, void* stream) {
    using namespace dl;
    const char* fn = "dl_calibration_stream";
    clear_error();
    if (kind < 0 || kind > 2 || (split != 0 && split != 1)) return set_error(DL_EINVAL, "%s: kind in 0..2, split in 0..1", fn);
    if (n < 1 || n > 32) return set_error(DL_EINVAL, "%s: n = %d, need 1 <= n <= 32", fn, n);
    if (d < 0 || ld < d) return set_error(DL_EINVAL, "%s: need 0 <= d <= ld", fn);
    if (!x || !m || !g || !columns_out) return set_error(DL_EINVAL, "%s: x, m, g and columns_out must not be NULL", fn);
    if (((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(m) | reinterpret_cast<uintptr_t>(g)) & 15u) || ld % 4)
        return set_error(DL_EINVAL, "%s: x, m, g must be 16-byte aligned and ld a multiple of 4", fn);
    // whole tiles only (whole 64 KiB units in the split order); the remaining columns are left alone
    const int64_t cols = split ? d / step::kSplitUnit * step::kSplitUnit : d / 256 * 256;
    *columns_out = cols;
    const int64_t tiles = cols / 256;
    if (tiles > 0x7fffffffLL) return set_error(DL_EINVAL, "%s: d too large for one launch", fn);
    if (tiles == 0) return DL_OK;
    const dim3 grid(static_cast<unsigned>(tiles)), block(1024);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (kind == 0) hipLaunchKernelGGL(k_stream<0>, grid, block, 0, s, x, m, g, n, ld, split, 0.5f);
    else if (kind == 1) hipLaunchKernelGGL(k_stream<1>, grid, block, 0, s, x, m, g, n, ld, split, 0.5f);
    else hipLaunchKernelGGL(k_stream<2>, grid, block, 0, s, x, m, g, n, ld, split, 0.5f);
    return check_hip(hipGetLastError(), "calibration stream launch");
}
