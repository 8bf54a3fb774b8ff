// Phase 1 of OSDN: the online preconditioner sweep (Algorithm 1, Eq. (dt_update) and its
// retention form Eq. (dt_update_apf)), and its reverse sweep (Section 4.5).
//
// The recurrence over d is sequential in t with O(K) work per token, so one wavefront
// owns one (batch, head) chain: lane l keeps K/64 consecutive coordinates of d in
// registers, the two inner products per token are wave reductions over DPP, and key rows
// are fetched several tokens ahead so that only the d-dependent part sits on the critical
// path.  All arithmetic is fp32; k~ is rounded once, from fp32 d * k, to the I/O type.
#include "osdn_kernels.h"

namespace osdn {

template <typename T, int EPL> struct alignas(sizeof(T) * EPL) Row { T v[EPL]; };

constexpr int P1_UNROLL = 8;

template <typename T, int EPL>
__global__ __launch_bounds__(64) void precond_fwd_kernel(PrecondArgs a) {
    const int lane = threadIdx.x;
    const int b = blockIdx.x / a.H, h = blockIdx.x % a.H;
    const int K = 64 * EPL;
    const int j0 = lane * EPL;
    const T *k = static_cast<const T *>(a.k);
    T *kt = static_cast<T *>(a.k_tilde);
    const size_t bh = (size_t)b * a.H + h;
    const bool project = a.d_min <= a.d_max;

    float d[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) d[e] = a.d_in ? a.d_in[bh * K + j0 + e] : 1.f;

    for (int t0 = 0; t0 < a.T; t0 += P1_UNROLL) {
        // ---- everything that does not depend on d, for P1_UNROLL tokens ----
        Row<T, EPL> kr[P1_UNROLL];
        float bet[P1_UNROLL], ret[P1_UNROLL];
#pragma unroll
        for (int u = 0; u < P1_UNROLL; ++u) {
            const int t = min(t0 + u, a.T - 1);
            const size_t th = ((size_t)b * a.T + t) * a.H + h;
            kr[u] = *reinterpret_cast<const Row<T, EPL> *>(k + th * K + j0);
            bet[u] = a.beta[th];
            ret[u] = a.retention ? a.retention[th] : 1.f;
        }
        float s[P1_UNROLL][EPL], ca[P1_UNROLL], cb[P1_UNROLL];
#pragma unroll
        for (int u = 0; u < P1_UNROLL; ++u) {
            float part = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const float kv = to_f32(kr[u].v[e]);
                s[u][e] = kv * kv;
                part += s[u][e];
            }
            const float n = fmaxf(wave_sum(part), a.eps);
            const float bp = a.beta_aware ? bet[u] : 1.f;
            // step = cb - ca * p  with p = <d, s>
            cb[u] = a.eta * bp / n;
            ca[u] = cb[u] * bp;
        }
        // ---- the sequential part ----
#pragma unroll
        for (int u = 0; u < P1_UNROLL; ++u) {
            const int t = t0 + u;
            if (t < a.T) {
                const size_t th = ((size_t)b * a.T + t) * a.H + h;
                if (a.d_ckpt && (t % C) == 0) {
#pragma unroll
                    for (int e = 0; e < EPL; ++e)
                        a.d_ckpt[(bh * (a.T / C) + t / C) * K + j0 + e] = d[e];
                }
                Row<T, EPL> out;
                float part = 0.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    out.v[e] = from_f32<T>(d[e] * to_f32(kr[u].v[e]));
                    part += d[e] * s[u][e];
                }
                *reinterpret_cast<Row<T, EPL> *>(kt + th * K + j0) = out;
                const float p = wave_sum(part);
                const float step = cb[u] - ca[u] * p;
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    float dn = ret[u] * d[e] + step * s[u][e];
                    if (project) dn = fminf(fmaxf(dn, a.d_min), a.d_max);
                    d[e] = dn;
                }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < EPL; ++e) a.d_out[bh * K + j0 + e] = d[e];
}

// Reverse sweep (Section 4.5; the projection passes gradient where the unprojected value
// lies in [d_min, d_max]).  One wavefront per chain, chunk by chunk from the right: the
// chunk's d trajectory is replayed from the stored chunk-start value into LDS, then the
// tokens are visited in reverse carrying the adjoint of d.
//   in : k, beta, retention, d_ckpt, dkt (dL/dk~, fp32), dk_read (dL/dk read side, fp32),
//        dbeta (partial, from phase 2), dd_out
//   out: dk (io type) = dk_read + d_t . dkt + phase-1 terms ; dbeta += ; dretention ; dd_in
template <typename T, int EPL>
__global__ __launch_bounds__(64) void precond_bwd_kernel(PrecondBwdArgs a) {
    constexpr int K = 64 * EPL;
    __shared__ float d_traj[C][K];      // d_t for the tokens of the current chunk
    const int lane = threadIdx.x;
    const int b = blockIdx.x / a.H, h = blockIdx.x % a.H;
    const int j0 = lane * EPL;
    const size_t bh = (size_t)b * a.H + h;
    const T *k = static_cast<const T *>(a.k);
    T *dk = static_cast<T *>(a.dk);
    const bool project = a.d_min <= a.d_max;
    const int N = a.T / C;

    float gd[EPL];                      // adjoint of d_{t+1}
#pragma unroll
    for (int e = 0; e < EPL; ++e) gd[e] = a.dd_out ? a.dd_out[bh * K + j0 + e] : 0.f;

    for (int n = N - 1; n >= 0; --n) {
        // replay the chunk forward: same arithmetic, same order as precond_fwd_kernel
        float d[EPL];
#pragma unroll
        for (int e = 0; e < EPL; ++e) d[e] = a.d_ckpt[(bh * N + n) * K + j0 + e];
        for (int i = 0; i < C; ++i) {
            const size_t th = ((size_t)b * a.T + n * C + i) * a.H + h;
            Row<T, EPL> kr = *reinterpret_cast<const Row<T, EPL> *>(k + th * K + j0);
            float s[EPL], part_n = 0.f, part_p = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                d_traj[i][j0 + e] = d[e];
                const float kv = to_f32(kr.v[e]);
                s[e] = kv * kv;
                part_n += s[e];
                part_p += d[e] * s[e];
            }
            const float nn = fmaxf(wave_sum(part_n), a.eps);
            const float bp = a.beta_aware ? a.beta[th] : 1.f;
            const float cb = a.eta * bp / nn, ca = cb * bp;
            const float step = cb - ca * wave_sum(part_p);
            const float r = a.retention ? a.retention[th] : 1.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                float dn = r * d[e] + step * s[e];
                if (project) dn = fminf(fmaxf(dn, a.d_min), a.d_max);
                d[e] = dn;
            }
        }
        // reverse over the chunk (d_traj is private to this wave: no barrier needed,
        // each lane reads back only what it wrote)
        for (int i = C - 1; i >= 0; --i) {
            const size_t th = ((size_t)b * a.T + n * C + i) * a.H + h;
            Row<T, EPL> kr = *reinterpret_cast<const Row<T, EPL> *>(k + th * K + j0);
            const float beta = a.beta[th];
            const float r = a.retention ? a.retention[th] : 1.f;
            float kv[EPL], s[EPL], dt[EPL], part_n = 0.f, part_p = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                kv[e] = to_f32(kr.v[e]);
                s[e] = kv[e] * kv[e];
                dt[e] = d_traj[i][j0 + e];
                part_n += s[e];
                part_p += dt[e] * s[e];
            }
            const float n_raw = wave_sum(part_n);
            const float nn = fmaxf(n_raw, a.eps);
            const float p = wave_sum(part_p);
            const float bp = a.beta_aware ? beta : 1.f;
            const float cb = a.eta * bp / nn, ca = cb * bp;
            const float step = cb - ca * p;
            // mask by the projection, then the two inner products with the masked adjoint
            float part_r = 0.f, part_c = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const float dbar = r * dt[e] + step * s[e];
                if (project && !(dbar >= a.d_min && dbar <= a.d_max)) gd[e] = 0.f;
                part_r += gd[e] * dt[e];
                part_c += gd[e] * s[e];
            }
            const float g_r = wave_sum(part_r);
            const float g_c = wave_sum(part_c);
            const float g_p = -g_c * ca;
            const float g_nraw = (n_raw >= a.eps) ? -g_c * step / nn : 0.f;
            const float g_bp = g_c * a.eta * (1.f - 2.f * bp * p) / nn;
            const size_t off = th * K + j0;
            Row<T, EPL> out;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const float gkt = a.dkt[off + e];
                const float gs = step * gd[e] + g_p * dt[e] + g_nraw;
                const float gk = a.dk_read[off + e] + dt[e] * gkt + 2.f * kv[e] * gs;
                out.v[e] = from_f32<T>(gk);
                gd[e] = r * gd[e] + g_p * s[e] + kv[e] * gkt;
            }
            *reinterpret_cast<Row<T, EPL> *>(dk + off) = out;
            if (lane == 0) {
                if (a.beta_aware) a.dbeta[th] += g_bp;
                if (a.dretention) a.dretention[th] = g_r;
            }
        }
    }
#pragma unroll
    for (int e = 0; e < EPL; ++e) a.dd_in[bh * K + j0 + e] = gd[e];
}

template <typename T>
static int launch_precond_fwd_t(const PrecondArgs &a, hipStream_t st) {
    dim3 grid(a.B * a.H), block(64);
    if (a.K == 64) hipLaunchKernelGGL((precond_fwd_kernel<T, 1>), grid, block, 0, st, a);
    else if (a.K == 128) hipLaunchKernelGGL((precond_fwd_kernel<T, 2>), grid, block, 0, st, a);
    else return -1;
    return 0;
}
int launch_precond_fwd(const PrecondArgs &a, bool bf16_io, hipStream_t st) {
    return bf16_io ? launch_precond_fwd_t<bf16>(a, st) : launch_precond_fwd_t<float>(a, st);
}

template <typename T>
static int launch_precond_bwd_t(const PrecondBwdArgs &a, hipStream_t st) {
    dim3 grid(a.B * a.H), block(64);
    if (a.K == 64) hipLaunchKernelGGL((precond_bwd_kernel<T, 1>), grid, block, 0, st, a);
    else if (a.K == 128) hipLaunchKernelGGL((precond_bwd_kernel<T, 2>), grid, block, 0, st, a);
    else return -1;
    return 0;
}
int launch_precond_bwd(const PrecondBwdArgs &a, bool bf16_io, hipStream_t st) {
    return bf16_io ? launch_precond_bwd_t<bf16>(a, st) : launch_precond_bwd_t<float>(a, st);
}

}  // namespace osdn
