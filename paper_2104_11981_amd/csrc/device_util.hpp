// Device-side helpers shared by the step kernels and the per-tensor final pass: streaming vector
// accesses, the gradient storage formats, wave-level sums.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "decentlam.h"

namespace dl {
namespace dev {

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

// Gradient element types by dl_grad_format; 16-bit values widen to fp32 exactly.
template <int GF> struct GradElem { using type = float; };
template <> struct GradElem<DL_GRAD_BF16> { using type = uint16_t; };
template <> struct GradElem<DL_GRAD_F16> { using type = _Float16; };

template <int VEC, int GF>
__device__ __forceinline__ void load_grad(const typename GradElem<GF>::type* __restrict__ p, float (&v)[VEC]) {
    if constexpr (GF == DL_GRAD_F32) {
        load_vec<VEC>(p, v);
    } else {
        using E = typename GradElem<GF>::type;
        E raw[VEC];
        if constexpr (VEC == 1) {
            raw[0] = __builtin_nontemporal_load(p);
        } else {
            typedef E vec_t __attribute__((ext_vector_type(VEC)));
            const vec_t t = __builtin_nontemporal_load(reinterpret_cast<const vec_t*>(p));
#pragma unroll
            for (int k = 0; k < VEC; ++k) raw[k] = t[k];
        }
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            if constexpr (GF == DL_GRAD_BF16)   // bf16 is the upper half of the fp32 pattern
                v[k] = __builtin_bit_cast(float, static_cast<uint32_t>(raw[k]) << 16);
            else
                v[k] = static_cast<float>(raw[k]);
        }
    }
}

// Cross-lane exchange of a double on the data-parallel-primitive network (no LDS traffic).
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    const int lo = __builtin_amdgcn_update_dpp(0, static_cast<int>(b), CTRL, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, static_cast<int>(b >> 32), CTRL, 0xF, 0xF, true);
    return __builtin_bit_cast(double, (static_cast<uint64_t>(static_cast<uint32_t>(hi)) << 32) |
                                          static_cast<uint32_t>(lo));
}

// Sums over the 64 lanes in a fixed order, the result in every lane: butterfly steps inside each
// row of 16 lanes on the primitive network (swap inside pairs, swap pairs inside quads, mirror
// inside 8, mirror inside 16), then two exchanges between the four rows.
__device__ __forceinline__ double wave_sum(double v) {
    v += dpp_f64<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_f64<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_f64<0x141>(v);   // row_half_mirror
    v += dpp_f64<0x140>(v);   // row_mirror
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    return v;
}
// Two sums for little more than the price of one: after the first step even lanes carry on with a,
// odd lanes with b, and every later step (swap pairs inside quads, rotate a row by 4 and by 8,
// exchange rows) keeps the parity of the lane.  Even lanes return sum(a), odd lanes sum(b).
__device__ __forceinline__ double wave_sum2(double a, double b, int lane) {
    a += dpp_f64<0xB1>(a);
    b += dpp_f64<0xB1>(b);
    double v = (lane & 1) ? b : a;
    v += dpp_f64<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_f64<0x124>(v);   // row_ror:4
    v += dpp_f64<0x128>(v);   // row_ror:8
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    return v;
}
// The same sums over each half of the wave (lanes 0-31, lanes 32-63): the last exchange is left out.
__device__ __forceinline__ double half_sum(double v) {
    v += dpp_f64<0xB1>(v);
    v += dpp_f64<0x4E>(v);
    v += dpp_f64<0x141>(v);
    v += dpp_f64<0x140>(v);
    v += __shfl_xor(v, 16, 64);
    return v;
}
__device__ __forceinline__ double half_sum2(double a, double b, int lane) {
    a += dpp_f64<0xB1>(a);
    b += dpp_f64<0xB1>(b);
    double v = (lane & 1) ? b : a;
    v += dpp_f64<0x4E>(v);
    v += dpp_f64<0x124>(v);
    v += dpp_f64<0x128>(v);
    v += __shfl_xor(v, 16, 64);
    return v;
}
template <int LANE>
__device__ __forceinline__ double lane_f64(double v) {   // the value of one lane as a scalar
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = __builtin_amdgcn_readlane(static_cast<int>(b), LANE);
    const uint32_t hi = __builtin_amdgcn_readlane(static_cast<int>(b >> 32), LANE);
    return __builtin_bit_cast(double, (static_cast<uint64_t>(hi) << 32) | lo);
}
__device__ __forceinline__ double uniform_f64(double v) {   // lane 0's value as a scalar
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<int>(b));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<int>(b >> 32));
    return __builtin_bit_cast(double, (static_cast<uint64_t>(hi) << 32) | lo);
}

}  // namespace dev
}  // namespace dl
