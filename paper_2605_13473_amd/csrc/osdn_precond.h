// Shared pieces of the phase-1 kernels (preconditioner sweep and its reverse).
#pragma once
#include "osdn_kernels.h"

namespace osdn {

constexpr int P1_MAX_SWEEPS = 66;       // 64 guarantee exactness
constexpr float P1_TOL = 1e-6f;         // relative agreement of the inner products between sweeps (forward)
constexpr float P1_TOL_BWD = 1e-7f;     // ... of sigma in the reverse sweep, whose errors add up in the adjoint of d
constexpr int PB = 8;                   // tokens per LDS prefetch block in the sequential loops

// projection onto [lo, hi] as one median-of-three (lo = -inf, hi = +inf when there is none)
__device__ __forceinline__ float clip3(float x, float lo, float hi) { return __builtin_amdgcn_fmed3f(x, lo, hi); }
// the affine step before projection, written once so that forward and replay round identically
template <bool HAS_RET>
__device__ __forceinline__ float d_bar(float r, float d, float step, float s) {
    return HAS_RET ? __builtin_fmaf(step, s, r * d) : __builtin_fmaf(step, s, d);
}
// Did the step land inside the box (the projection's gradient mask)?  Decided from the signs
// of (r d - face) + step s, each evaluated with a single rounding at its own scale, rather
// than by comparing the rounded sum with the face: a coordinate that sits on a face, or
// comes within an ulp of it, is then told apart from one pushed across it by less than an ulp.
template <bool HAS_RET>
__device__ __forceinline__ bool lands_inside(float r, float d, float step, float s, float lo, float hi) {
    const float above_lo = HAS_RET ? __builtin_fmaf(r, d, -lo) : d - lo;
    const float above_hi = HAS_RET ? __builtin_fmaf(r, d, -hi) : d - hi;
    return __builtin_fmaf(step, s, above_lo) >= 0.f && __builtin_fmaf(step, s, above_hi) <= 0.f;
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
// One workgroup = 8 wavefronts, two per SIMD.
constexpr int P1T = 512, P1W = P1T / 64;
// sum of the per-wave partials of row i (fixed order)
__device__ __forceinline__ float sumw(const float *part, int i) {
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < P1W; ++w) s += part[w * C + i];
    return s;
}

// partner lane ^ 4 inside a row of 16 lanes: two DPP moves (row_shl:4 into lanes 0-3 and 8-11 of
// every row, row_shr:4 into the others)
__device__ __forceinline__ float lane_xor4(float x) {
    const int xi = __builtin_bit_cast(int, x);
    int t = __builtin_amdgcn_update_dpp(0, xi, 0x104, 0xF, 0x5, false);
    t = __builtin_amdgcn_update_dpp(t, xi, 0x114, 0xF, 0xA, false);
    return __builtin_bit_cast(float, t);
}
// Every lane holds TS values v[0..TS); returns to lane l the sum of v[l % TS] over the group of
// TS lanes it belongs to (the 64 / TS partial sums per value are left to the caller).
template <int TS>
__device__ __forceinline__ float lane_fold(const float (&v)[TS], int lane) {
    static_assert(TS == 16 || TS == 8, "run length");
    // after the step with lane bit b, a lane keeps the values whose index has bit b equal to
    // its own and adds the partner lane's copy of them: the count halves, the group doubles
    float w[TS / 2], x[TS / 4], y[TS / 8];
    const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4, b3 = lane & 8;
#pragma unroll
    for (int m = 0; m < TS / 2; ++m)
        w[m] = (b0 ? v[2 * m + 1] : v[2 * m]) + dpp_f32<0xB1>(b0 ? v[2 * m] : v[2 * m + 1]);     // lane ^ 1
#pragma unroll
    for (int m = 0; m < TS / 4; ++m)
        x[m] = (b1 ? w[2 * m + 1] : w[2 * m]) + dpp_f32<0x4E>(b1 ? w[2 * m] : w[2 * m + 1]);     // lane ^ 2
#pragma unroll
    for (int m = 0; m < TS / 8; ++m)
        y[m] = (b2 ? x[2 * m + 1] : x[2 * m]) + lane_xor4(b2 ? x[2 * m] : x[2 * m + 1]);         // lane ^ 4
    if (TS == 8) return y[0];                  // value lane % 8, summed over its 8 lanes
    return (b3 ? y[TS / 8 - 1] : y[0]) + dpp_f32<0x128>(b3 ? y[0] : y[TS / 8 - 1]);   // lane ^ 8 (row_ror:8)
}
// the same for 8 values, carried on to the sum over the whole wavefront: every lane gets the
// total of v[lane % 8] (fixed order of additions)
__device__ __forceinline__ float lane_fold8_all(const float (&v)[8], int lane) {
    float y = lane_fold<8>(v, lane);
    y += dpp_f32<0x128>(y);
    y += __shfl_xor(y, 16, 64);
    y += __shfl_xor(y, 32, 64);
    return y;
}
// ---- a chunk of the recurrence in solved form ---------------------------------------------
// Where a chunk of 64 tokens has no retention and no coordinate meets the box, both sweeps are
// linear in the K-vector they carry (d forward, its adjoint backward) and couple the tokens only
// through 64 scalars (the inner products <d_t, s_t>, resp. sigma_t = <s_t, abar_t>), which solve a
// unit triangular 64 x 64 system built from the Gram matrix of the squared keys.  That system is
// inverted for all chunks side by side; what stays sequential per chunk is
//     x = S v + r0 ;  y = M x ;  w = w(y) ;  v' = v + t0 +- S^T w
// (S = the 64 x K tile of squared keys, v the carried vector): two matrix-vector products with
// S and one with the 64 x 64 inverse M.  Thread layouts of a 512-thread workgroup:
//   rows   : thread (i = tid / 8, part = tid % 8) owns coordinates [part * EPT, (part + 1) * EPT) of token i
//            (resp. columns [8 part, 8 part + 8) of row i of M); sums over the 8 lanes of a token
//   columns: thread (c = tid / NG, tg = tid % NG) owns tokens u * NG + tg of coordinate c; sums over NG lanes
template <int K> struct Lin {
    static constexpr int EPT = K / 8;
    static constexpr int NG = P1T / K;
    static constexpr int LD = K + (K == 128 ? 8 : 4);     // row stride of the s tile: column reads of a half-wave hit 32 banks
    static constexpr int VSTR = EPT + 4;                  // a thread's slice of a K-vector: slices start 16 bytes off a bank period
    static constexpr int XSTR = 12;                       // ... of a 64-vector (8 entries per slice)
    static __device__ __forceinline__ int vidx(int c) { return (c / EPT) * VSTR + c % EPT; }
    // Position of coordinate c inside a row of the s tile: the 16-byte groups of a 16-coordinate
    // slice are rotated by half the slice index, so that the 8 threads that write one group each
    // for 8 adjacent slices (128 bytes apart) cover all 32 banks; column reads stay conflict-free.
    static __device__ __forceinline__ int swz(int c) { return (c & ~12) | ((((c >> 2) + (c >> 5)) & 3) << 2); }
    static __device__ __forceinline__ int xidx(int i) { return (i >> 3) * XSTR + (i & 7); }
};
// sum over the 8 (4) adjacent lanes of an aligned group, returned to all of them
__device__ __forceinline__ float sum_lanes8(float x) {
    x += dpp_f32<0xB1>(x);
    x += dpp_f32<0x4E>(x);
    x += lane_xor4(x);
    return x;
}
__device__ __forceinline__ float sum_lanes4(float x) {
    x += dpp_f32<0xB1>(x);
    x += dpp_f32<0x4E>(x);
    return x;
}

__device__ __forceinline__ float lane_bcast(float x, int src_lane) {     // src_lane uniform
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), src_lane));
}

}  // namespace osdn
