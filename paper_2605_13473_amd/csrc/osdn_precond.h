// Shared pieces of the phase-1 kernels (preconditioner sweep and its reverse).
#pragma once
#include "osdn_kernels.h"

namespace osdn {

constexpr int P1_MAX_SWEEPS = 66;       // 64 guarantee exactness
constexpr float P1_TOL = 1e-6f;         // relative agreement of the inner products between sweeps
constexpr int PB = 8;                   // tokens per LDS prefetch block in the sequential loops

// projection onto [lo, hi] as one median-of-three (lo = -inf, hi = +inf when there is none)
__device__ __forceinline__ float clip3(float x, float lo, float hi) { return __builtin_amdgcn_fmed3f(x, lo, hi); }
// the affine step before projection, written once so that forward and replay round identically
template <bool HAS_RET>
__device__ __forceinline__ float d_bar(float r, float d, float step, float s) {
    return HAS_RET ? __builtin_fmaf(step, s, r * d) : __builtin_fmaf(step, s, d);
}
__device__ __forceinline__ void store_vec(float *dst, const float (&v)[4]) {
    *reinterpret_cast<f32x4 *>(dst) = f32x4{v[0], v[1], v[2], v[3]};
}
__device__ __forceinline__ void store_vec(bf16 *dst, const float (&v)[8]) {
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (bf16)v[e];
    *reinterpret_cast<bf16x8 *>(dst) = o;
}
__device__ __forceinline__ void store_vec(bf16 *dst, const float (&v)[4]) {
    bf16x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (bf16)v[e];
    *reinterpret_cast<bf16x4 *>(dst) = o;
}
__device__ __forceinline__ float wave_max(float x) {      // x >= 0
    x = fmaxf(x, dpp_f32<0xB1>(x));
    x = fmaxf(x, dpp_f32<0x4E>(x));
    x = fmaxf(x, dpp_f32<0x141>(x));
    x = fmaxf(x, dpp_f32<0x140>(x));
    x = fmaxf(x, dpp_f32<0x142, 0xA>(x));      // rows that are not written keep old = 0 <= x
    x = fmaxf(x, dpp_f32<0x143, 0xC>(x));
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}
// One workgroup = 16 wavefronts: the sequential loops run on K/64 of them, the parallel
// phases (row dots, tile conversion, outputs) on all, four per SIMD, to hide LDS latency.
constexpr int P1T = 512, P1W = P1T / 64;
// sum of the per-wave partials of row i (fixed order)
__device__ __forceinline__ float sumw(const float *part, int i) {
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < P1W; ++w) s += part[w * C + i];
    return s;
}

}  // namespace osdn
