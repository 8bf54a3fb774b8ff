// Phase 1 of OSDN: the online preconditioner sweep (Algorithm 1, Eq. (dt_update) and its
// retention form Eq. (dt_update_apf)), and its reverse sweep (Section 4.5).
//
// The recurrence  d_{t+1} = clip(r_t d_t + c_t s_t),  s_t = k_t (.) k_t,
//                 c_t = eta b'(1 - b' p_t)/n_t,  p_t = <d_t, s_t>
// couples the K coordinates only through the scalar p_t.  One workgroup owns one
// (batch, head) chain and walks it in chunks of 64 tokens held in LDS.  Inside a chunk it
// solves for the 64 scalars p by fixed-point sweeps: given p (first guess: <d_0, s_t>), the
// recurrence separates into K independent scalar recurrences (one thread per coordinate,
// 64 steps of fma + median-of-three, clip included); from the resulting trajectory the 64
// inner products are recomputed in parallel; the sweep repeats until they reproduce
// themselves.  Sweep m fixes at least the first m tokens exactly, so 64 sweeps always
// suffice; because the coupling is O(eta) two do in practice (also when coordinates sit on a
// face of the box, which the scalar recurrences handle by themselves).  No per-token
// cross-lane reduction is left on the sequential path.  All arithmetic is fp32; k~ is
// rounded once, from fp32 d * k.
//
// The reverse sweep has the same structure: with sigma_t = <s_t, abar_t> known, the adjoint
// recurrence  abar_t = mask_t (.) a_{t+1},  a_t = k_t (.) dL/dk~_t + r_t abar_t - ca_t sigma_t s_t
// separates per coordinate; sigma is found by the same kind of sweeps.
#include "osdn_precond.h"

namespace osdn {

template <typename T, int K, bool HAS_RET>
__global__ __launch_bounds__(P1T) void precond_fwd_kernel(PrecondArgs a) {
    constexpr int LD = K + 1;                    // odd stride: rows and columns both conflict-free
    constexpr int VN = 4;                        // a thread moves groups of 4 consecutive columns
    constexpr int NW = C * K / VN / P1T;         // groups per thread for a [64 x K] tile
    static_assert(NW >= 1, "tile smaller than the workgroup");
    constexpr int KQ = K / P1W;                   // columns per thread in a row dot
    __shared__ float ss[C * LD];                 // s = k^2 of the chunk
    __shared__ float Dt[C * LD];                 // d_i for the tokens of the chunk
    __shared__ float d0[K], dnew[K];
    __shared__ float cbs[C], cas[C], nraws[C], ps[C];
    __shared__ __attribute__((aligned(16))) float cs[C];
    __shared__ __attribute__((aligned(16))) float rs[C];
    __shared__ float part[P1W * C], part2[P1W * C];
    __shared__ int done;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int b = blockIdx.x / a.H, h = blockIdx.x % a.H;
    const size_t bh = (size_t)b * a.H + h;
    const T *k = static_cast<const T *>(a.k);
    T *kt = static_cast<T *>(a.k_tilde);
    const bool project = a.d_min <= a.d_max;
    const float lo = project ? a.d_min : -INFINITY, hi = project ? a.d_max : INFINITY;
    const int N = (a.T + C - 1) / C;

    if (tid < K) d0[tid] = a.d_in ? a.d_in[bh * K + tid] : 1.f;

    u32x4 kreg[NW];                              // (bf16: only .x, .y are used)
    float betreg = 0.f, retreg = 1.f;
#define OSDN_P1_LOAD(n_)                                                                         \
    {                                                                                            \
        const int t0_ = (n_) * C;                                                                \
        _Pragma("unroll") for (int m = 0; m < NW; ++m) {                                         \
            const int i = tid + m * P1T, r = i / (K / VN), c = (i % (K / VN)) * VN;               \
            const int t = min(t0_ + r, a.T - 1);                                                 \
            const T *src_ = k + (((size_t)b * a.T + t) * a.H + h) * K + c;                       \
            if (sizeof(T) == 2) { const u32x2 v_ = *reinterpret_cast<const u32x2 *>(src_); kreg[m] = u32x4{v_[0], v_[1], 0u, 0u}; } \
            else kreg[m] = *reinterpret_cast<const u32x4 *>(src_);                               \
        }                                                                                        \
        if (tid < C) {                                                                           \
            const int t = min(t0_ + tid, a.T - 1);                                               \
            const size_t th = ((size_t)b * a.T + t) * a.H + h;                                   \
            betreg = a.beta[th];                                                                 \
            if (HAS_RET) retreg = a.retention[th];                                               \
        }                                                                                        \
    }
    OSDN_P1_LOAD(a.n0)

#ifdef OSDN_DIAG
    long long tph[6] = {0, 0, 0, 0, 0, 0}, tlast = clock64();
#define OSDN_TICK(j) { const long long now_ = clock64(); tph[j] += now_ - tlast; tlast = now_; }
#else
#define OSDN_TICK(j)
#endif
    for (int n = a.n0; n < a.n1; ++n) {
        const int t0 = n * C;
        const int nvalid = min(C, a.T - t0);
        // ---- registers -> LDS (rows past the end of the sequence become no-op tokens) ----
        u32x4 kcur[NW];
#pragma unroll
        for (int m = 0; m < NW; ++m) {
            kcur[m] = kreg[m];
            const int i = tid + m * P1T, r = i / (K / VN), c = (i % (K / VN)) * VN;
#pragma unroll
            for (int e = 0; e < VN; ++e) {
                const float kv = r < nvalid ? vec_get<T>(kcur[m], e) : 0.f;
                ss[r * LD + c + e] = kv * kv;
            }
        }
        const float bet = betreg, ret = retreg;
        __syncthreads();
        OSDN_TICK(0)
        if (n + 1 < a.n1) OSDN_P1_LOAD(n + 1)
        if (a.d_ckpt && tid < K) a.d_ckpt[(bh * N + n) * K + tid] = d0[tid];
        // ---- per token: n_raw = sum s, and the first guess p = <d_0, s> ----
        {
            const int i = lane, q0 = wave * KQ;
            float sn = 0.f, sp = 0.f;
#pragma unroll 8
            for (int c = 0; c < KQ; ++c) {
                const float s = ss[i * LD + q0 + c];
                sn += s;
                sp = __builtin_fmaf(s, d0[q0 + c], sp);
            }
            part[wave * C + i] = sn;
            part2[wave * C + i] = sp;
        }
        __syncthreads();
        if (tid < C) {
            const int i = tid;
            const float nraw = sumw(part, i), p = sumw(part2, i);
            const bool valid = i < nvalid;
            const float nn = fmaxf(nraw, a.eps);
            const float bp = a.beta_aware ? bet : 1.f;
            const float cb = valid ? a.eta * bp / nn : 0.f;
            const float ca = cb * bp;
            nraws[i] = nraw; cbs[i] = cb; cas[i] = ca; rs[i] = valid ? ret : 1.f;
            ps[i] = p;
            cs[i] = cb - ca * p;
        }
        __syncthreads();
        OSDN_TICK(1)
        // ---- fixed-point sweeps ----
        int sweeps_used = 0;
        for (int sweep = 0; sweep < P1_MAX_SWEEPS; ++sweep) {
            ++sweeps_used;
            if (tid < K) {                      // K independent scalar recurrences
                float d = d0[tid];
                // LDS operands are fetched one block of PB tokens ahead of their use
                float sb[2][PB], cb_[2][PB], rb[2][PB];
#define OSDN_QLOAD(buf, i0_)                                                                     \
    _Pragma("unroll") for (int u = 0; u < PB; ++u) {                                             \
        sb[buf][u] = ss[((i0_) + u) * LD + tid]; cb_[buf][u] = cs[(i0_) + u];                     \
        if (HAS_RET) rb[buf][u] = rs[(i0_) + u];                                                 \
    }
                OSDN_QLOAD(0, 0)
#pragma unroll
                for (int blk = 0; blk < C / PB; ++blk) {
                    if (blk + 1 < C / PB) OSDN_QLOAD((blk + 1) & 1, (blk + 1) * PB)
#pragma unroll
                    for (int u = 0; u < PB; ++u) {
                        const int i = blk * PB + u;
                        Dt[i * LD + tid] = d;
                        d = clip3(d_bar<HAS_RET>(rb[blk & 1][u], d, cb_[blk & 1][u], sb[blk & 1][u]), lo, hi);
                    }
                }
                dnew[tid] = d;
            }
            __syncthreads();
            OSDN_TICK(2)
            {                                   // recompute p_i = <d_i, s_i> from the trajectory
                const int i = lane, q0 = wave * KQ;
                float sp = 0.f;
#pragma unroll 8
                for (int c = 0; c < KQ; ++c) sp = __builtin_fmaf(ss[i * LD + q0 + c], Dt[i * LD + q0 + c], sp);
                part2[wave * C + i] = sp;
            }
            __syncthreads();
            if (tid < C) {
                const int i = tid;
                const float p = sumw(part2, i);
                const bool ok = fabsf(p - ps[i]) <= P1_TOL * fabsf(p);
                const bool all_ok = __all(ok);
                if (all_ok) {
                    if (tid == 0) done = 1;
                } else {
                    if (tid == 0) done = 0;
                    ps[i] = p;
                    cs[i] = cbs[i] - cas[i] * p;
                }
            }
            __syncthreads();
            OSDN_TICK(3)
            if (done) break;
        }
        // ---- accepted: (cs, ps) generated Dt and dnew ----
#pragma unroll
        for (int m = 0; m < NW; ++m) {
            const int i = tid + m * P1T, r = i / (K / VN), c = (i % (K / VN)) * VN;
            if (r < nvalid) {
                float out[VN];
#pragma unroll
                for (int e = 0; e < VN; ++e) out[e] = Dt[r * LD + c + e] * vec_get<T>(kcur[m], e);
                store_vec(kt + (((size_t)b * a.T + t0 + r) * a.H + h) * K + c, out);
            }
        }
        if (a.tok_scalars && tid < nvalid) {
            const size_t th = ((size_t)b * a.T + t0 + tid) * a.H + h;
            *reinterpret_cast<float4 *>(a.tok_scalars + th * 4) = make_float4(cs[tid], ps[tid], nraws[tid], (float)sweeps_used);
        }
        if (tid < K) d0[tid] = dnew[tid];
        __syncthreads();
        OSDN_TICK(4)
    }
#ifdef OSDN_DIAG
    if (a.tok_scalars && tid == 0 && blockIdx.x == 0)
        for (int j = 0; j < 5; ++j) a.tok_scalars[(((size_t)b * a.T + 2 + j) * a.H + h) * 4 + 3] = (float)tph[j];
#endif
    if (tid < K) a.d_out[bh * K + tid] = d0[tid];
}

template <typename T, bool HAS_RET>
static int launch_precond_fwd_t(const PrecondArgs &a, hipStream_t st) {
    dim3 grid(a.B * a.H), block(P1T);
    if (a.K == 64) hipLaunchKernelGGL((precond_fwd_kernel<T, 64, HAS_RET>), grid, block, 0, st, a);
    else if (a.K == 128) hipLaunchKernelGGL((precond_fwd_kernel<T, 128, HAS_RET>), grid, block, 0, st, a);
    else return -1;
    return 0;
}
int launch_precond_fwd(const PrecondArgs &a, bool bf16_io, hipStream_t st) {
    if (a.retention)
        return bf16_io ? launch_precond_fwd_t<bf16, true>(a, st) : launch_precond_fwd_t<float, true>(a, st);
    return bf16_io ? launch_precond_fwd_t<bf16, false>(a, st) : launch_precond_fwd_t<float, false>(a, st);
}

}  // namespace osdn
