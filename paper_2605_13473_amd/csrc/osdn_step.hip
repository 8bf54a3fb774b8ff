// Recurrent (token-by-token) form of the OSDN update for short inputs: the decode step of
// Appendix K (gate, preconditioner update with the clip, rank-one write, read) for 1..64
// tokens in one launch, with the state slice of a workgroup held in registers throughout.
//
//   k~_t = d_t (.) k_t
//   S   <- alpha_t S ;  e = beta_t (v_t - S k_t) ;  S <- S + e k~_t^T ;  o_t = scale S q_t
//   (alpha_t a scalar, or one gate per key channel: S <- S Diag(alpha_t), the online-scaled
//   KDA recurrence in this library's V x K orientation of the state)
//   d_{t+1} = clip(r_t d_t + eta b'(1 - b' p)/n s),  s = k_t^2, n = max(sum s, eps), p = <d_t, s>
//
// A workgroup of four wavefronts owns 16 rows of S of one (batch, head); a wavefront owns 4 of
// them, a lane K / 64 adjacent coordinates.  Every wavefront keeps its own copy of d (the
// update needs two sums over the coordinates, like the two inner products per row).
#include "osdn_precond.h"

namespace osdn {

constexpr int STEP_T = 256, STEP_RPW = 4, STEP_ROWS = (STEP_T / 64) * STEP_RPW;   // 16 rows per workgroup

// RET: 0 = no retention, 1 = one gate per (token, head), 2 = one per coordinate; GV: one state
// gate per key channel
template <typename T, int K, int RET, bool GV>
__global__ __launch_bounds__(STEP_T) void step_kernel(StepArgs a) {
    constexpr bool HAS_RET = RET != 0, RET_VEC = RET == 2;
    constexpr int CPT = K / 64;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int nslice = a.V / STEP_ROWS;
    const int slice = blockIdx.x % nslice, chain = blockIdx.x / nslice;
    const int b = chain / a.H, h = chain % a.H;
    const size_t bh = (size_t)b * a.H + h;
    const int v0 = slice * STEP_ROWS + wave * STEP_RPW;
    const int c0 = lane * CPT;
    const bool project = a.d_min <= a.d_max;
    const float lo = project ? a.d_min : -INFINITY, hi = project ? a.d_max : INFINITY;

    float d[CPT], Sr[STEP_RPW][CPT];
#pragma unroll
    for (int e = 0; e < CPT; ++e) d[e] = a.d_in ? a.d_in[bh * K + c0 + e] : 1.f;
#pragma unroll
    for (int r = 0; r < STEP_RPW; ++r)
#pragma unroll
        for (int e = 0; e < CPT; ++e) Sr[r][e] = a.S_in ? a.S_in[(bh * a.V + v0 + r) * K + c0 + e] : 0.f;

    const T *qg = static_cast<const T *>(a.q), *kg = static_cast<const T *>(a.k), *vg = static_cast<const T *>(a.v);
    T *og = static_cast<T *>(a.o);
    for (int t = 0; t < a.T; ++t) {
        const size_t th = ((size_t)b * a.T + t) * a.H + h;
        float kf[CPT], qf[CPT], kt[CPT];
#pragma unroll
        for (int e = 0; e < CPT; ++e) {
            kf[e] = to_f32(kg[th * K + c0 + e]);
            qf[e] = to_f32(qg[th * K + c0 + e]);
            kt[e] = d[e] * kf[e];
        }
        const float bet = a.beta[th];
        float alpha[CPT];                           // one state gate per (token, head), or one per key channel
#pragma unroll
        for (int e = 0; e < CPT; ++e)
            alpha[e] = a.log_alpha ? __expf(GV ? a.log_alpha[th * K + c0 + e] : a.log_alpha[th]) : 1.f;
        float ret[CPT];                             // one gate per (token, head), or one per coordinate
#pragma unroll
        for (int e = 0; e < CPT; ++e)
            ret[e] = HAS_RET ? (RET_VEC ? a.retention[th * K + c0 + e] : a.retention[th]) : 1.f;
        float orow = 0.f;                           // lane r < 4 ends with the output of row v0 + r
#pragma unroll
        for (int r = 0; r < STEP_RPW; ++r) {
            float dot = 0.f;
#pragma unroll
            for (int e = 0; e < CPT; ++e) { Sr[r][e] *= alpha[e]; dot = __builtin_fmaf(Sr[r][e], kf[e], dot); }
            dot = wave_sum(dot);
            const float ev = bet * (to_f32(vg[th * a.V + v0 + r]) - dot);
            float od = 0.f;
#pragma unroll
            for (int e = 0; e < CPT; ++e) { Sr[r][e] = __builtin_fmaf(ev, kt[e], Sr[r][e]); od = __builtin_fmaf(Sr[r][e], qf[e], od); }
            od = wave_sum(od);
            if (lane == r) orow = od;
        }
        if (lane < STEP_RPW) og[th * a.V + v0 + lane] = from_f32<T>(a.scale * orow);
        // the preconditioner moves after the token has used it
        float sn = 0.f, sp = 0.f, sv[CPT];
#pragma unroll
        for (int e = 0; e < CPT; ++e) { sv[e] = kf[e] * kf[e]; sn += sv[e]; sp = __builtin_fmaf(sv[e], d[e], sp); }
        sn = wave_sum(sn);
        sp = wave_sum(sp);
        const float nn = fmaxf(sn, a.eps);
        const float bp = a.beta_aware ? bet : 1.f;
        const float cb = a.eta * bp / nn;
        const float step = cb - cb * bp * sp;
#pragma unroll
        for (int e = 0; e < CPT; ++e) d[e] = clip3(d_bar<HAS_RET>(ret[e], d[e], step, sv[e]), lo, hi);
    }
#pragma unroll
    for (int r = 0; r < STEP_RPW; ++r)
#pragma unroll
        for (int e = 0; e < CPT; ++e) a.S_out[(bh * a.V + v0 + r) * K + c0 + e] = Sr[r][e];
    if (slice == 0 && wave == 0) {
#pragma unroll
        for (int e = 0; e < CPT; ++e) a.d_out[bh * K + c0 + e] = d[e];
    }
}

template <typename T, int RET, bool GV>
static int launch_step_t(const StepArgs &a, hipStream_t st) {
    dim3 grid(a.B * a.H * (a.V / STEP_ROWS)), block(STEP_T);
    if (a.K == 64) hipLaunchKernelGGL((step_kernel<T, 64, RET, GV>), grid, block, 0, st, a);
    else if (a.K == 128) hipLaunchKernelGGL((step_kernel<T, 128, RET, GV>), grid, block, 0, st, a);
    else return -1;
    return 0;
}
template <typename T>
static int launch_step_io(const StepArgs &a, hipStream_t st) {
    const int ret = a.retention ? (a.ret_vec ? 2 : 1) : 0;
    const bool gv = a.log_alpha && a.gate_vec;
    if (ret == 2) return gv ? launch_step_t<T, 2, true>(a, st) : launch_step_t<T, 2, false>(a, st);
    if (ret == 1) return gv ? launch_step_t<T, 1, true>(a, st) : launch_step_t<T, 1, false>(a, st);
    return gv ? launch_step_t<T, 0, true>(a, st) : launch_step_t<T, 0, false>(a, st);
}
int launch_step(const StepArgs &a, bool bf16_io, hipStream_t st) {
    return bf16_io ? launch_step_io<bf16>(a, st) : launch_step_io<float>(a, st);
}

}  // namespace osdn
