// Reverse sweep over the projected affine recurrence of the preconditioner (Section 4.5),
// split so that only what is sequential stays on the sequential path.
//
// With  abar_t = mask_t (.) a_{t+1},  sigma_t = <s_t, abar_t>,  s_t = k_t (.) k_t,
//       a_t    = k_t (.) dL/dk~_t + r_t abar_t - ca_t sigma_t s_t        (ca_t = eta b'^2 / n_t)
// the only coupling between chunks is the K-vector a at the chunk boundary, and inside a chunk
// the only coupling between coordinates is the scalar sigma_t.  Three kernels:
//   precond_mask   one workgroup per (chain, chunk), all chunks in parallel: replays d from the
//                  stored chunk-start value and step scalars and records, per coordinate, the
//                  64-bit mask of tokens whose unprojected update stayed inside the box
//   precond_chain  one workgroup per chain, chunks right to left: finds sigma by fixed-point
//                  sweeps (as the forward kernel finds <d, s>), keeps the adjoint at every chunk
//                  boundary and the 64 sigmas of every chunk, nothing else
//   precond_post   one workgroup per (chain, chunk), all chunks in parallel, one thread per
//                  coordinate: replays d, re-runs the adjoint recurrence of its chunk from the
//                  stored boundary value, sigmas and masks, and writes dk, dbeta, dretention
// The retention gate is absent, one value per (token, head), or one per coordinate (RET).
//
// Without retention, on a chunk in which no coordinate met the box (every mask bit set), the
// recurrence is linear with constant coefficients:  abar_i = g + sum_{j>i} (lambda_j - ca_j
// sigma_j s_j)  (g = the adjoint at the chunk's right end, lambda_j = k_j (.) dL/dk~_j), hence
//     (I + U) sigma = S g + rho0,   U_ij = <s_i, s_j> ca_j (j > i),   rho0_i = <s_i, sum_{j>i} lambda_j>,
//     a_left = g + sum_j lambda_j - S^T (ca (.) sigma).
//   precond_lin_m  one workgroup per (chain, chunk), all chunks in parallel, needs the forward
//                  pass only: writes the chunk's masks (in place of precond_mask, which is not
//                  launched when this form is on), decides whether the chunk qualifies and, if
//                  so, leaves (I + U)^-1 (Gram matrix and blocked inverse on the fp32 MFMA), kept
//                  in the I/O type;
//   precond_lin_r  the same grid, once dL/dk~ of the chunk is there: rho0 and sum_j lambda_j;
// on such a chunk precond_chain only has the three matrix-vector products left (osdn_precond.h,
// "a chunk of the recurrence in solved form"); on any other chunk it runs its sweeps.
#include "osdn_precond.h"

namespace osdn {

// ---------------------------------------------------------------- precond_mask ----
// RET (all three kernels): 0 = no retention, 1 = one gate per (token, head), 2 = one per coordinate
template <typename T, int K, int RET>
__global__ __launch_bounds__(K) void precond_mask_kernel(PrecondBwdArgs a) {
    constexpr bool HAS_RET = RET != 0, RET_VEC = RET == 2;
    __shared__ __attribute__((aligned(16))) float steps[C];
    __shared__ __attribute__((aligned(16))) float rs[C];
    const int n = a.n0 + blockIdx.x, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int N = a.T / C;
    const size_t bh = (size_t)b * a.H + h;
    const size_t tokc = ((size_t)b * a.T + (size_t)n * C) * a.H + h;
    const bool project = a.d_min <= a.d_max;
    const float lo = project ? a.d_min : -INFINITY, hi = project ? a.d_max : INFINITY;
    if (tid < C) {
        const size_t th = tokc + (size_t)tid * a.H;
        steps[tid] = a.tok_scalars[th * 4];
        rs[tid] = (HAS_RET && !RET_VEC) ? a.retention[th] : 1.f;
    }
    const T *kp = static_cast<const T *>(a.k) + tokc * K;
    const float *rp = RET_VEC ? a.retention + tokc * K : nullptr;
    const uint32_t kstride = (uint32_t)a.H * K;
    float kv[C], rvv[RET_VEC ? C : 1];
#pragma unroll
    for (int i = 0; i < C; ++i) {
        kv[i] = to_f32(kp[(uint32_t)tid + (uint32_t)i * kstride]);
        if (RET_VEC) rvv[RET_VEC ? i : 0] = rp[(uint32_t)tid + (uint32_t)i * kstride];
    }
    float d = a.d_ckpt[(bh * N + n) * K + tid];
    __syncthreads();
    uint32_t mlo = 0u, mhi = 0u;
#pragma unroll
    for (int i = 0; i < C; ++i) {
        const float sq = kv[i] * kv[i];
        const float r = RET_VEC ? rvv[RET_VEC ? i : 0] : rs[i];
        const uint32_t in = lands_inside<HAS_RET>(r, d, steps[i], sq, lo, hi) ? (1u << (i & 31)) : 0u;
        d = clip3(d_bar<HAS_RET>(r, d, steps[i], sq), lo, hi);
        if (i < 32) mlo |= in; else mhi |= in;
    }
    a.masks[(bh * N + n) * K + tid] = make_uint2(mlo, mhi);
}

// ----------------------------------------------------------------- precond_lin ----
// Two kernels, both one workgroup per (chain, chunk).  precond_lin_m needs the forward pass only
// (keys, step scalars, d at the chunk start): it replays d over the chunk for the box masks (what
// precond_mask does when this form is off: the same arithmetic, from the s tile it builds anyway),
// decides from them whether the chunk qualifies, and inverts the system.
// precond_lin_r needs dL/dk~ of the chunk as well: rho0 and the sum of lambda.
template <typename T, int K>
__global__ __launch_bounds__(P1T) void precond_lin_m_kernel(PrecondBwdArgs a) {
    typedef Lin<K> LN;
    constexpr int EPT = LN::EPT, VN = 16 / sizeof(T), NVK = EPT / VN;
    constexpr int LDT = K + 4;                   // s tile: MFMA fragment reads (row = lane % 16, k = lane / 16) spread over the banks
    constexpr int LDF = C + 1;
    constexpr int TI_F = C * LDF + 3 * 16 * 17;  // (I + A)^-1 and the block products: in the s tile's space once A is built
    static_assert(TI_F <= C * LDT || K == 64, "the inverse reuses the s tile");
    __shared__ __attribute__((aligned(16))) float Ss[C * LDT > TI_F ? C * LDT : TI_F];
    __shared__ __attribute__((aligned(16))) float Af[C * LDF];
    __shared__ float cas[C];
    __shared__ float steps[C];
    float *Ti = Ss, *Xs = Ss + C * LDF;

    const int n = a.n0 + blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int N = a.T / C;
    const size_t bhn = ((size_t)b * a.H + h) * N + n;
    const size_t tokc = ((size_t)b * a.T + (size_t)n * C) * a.H + h;
    const int i = tid >> 3, part = tid & 7;
    const uint32_t kstride = (uint32_t)a.H * K;
    u32x4 kv[NVK];
    {
        const uint32_t off = ((uint32_t)i * kstride + (uint32_t)(part * EPT)) * (uint32_t)sizeof(T);
        const u32x4 *kp = reinterpret_cast<const u32x4 *>(static_cast<const T *>(a.k) + tokc * K);
#pragma unroll
        for (int m = 0; m < NVK; ++m) kv[m] = at_byte(kp, off + 16 * m);
    }
    const bool project = a.d_min <= a.d_max;
    float nraw = 1.f, bet = 0.f, d = 1.f;
    if (tid < C) {
        const size_t th = tokc + (size_t)tid * a.H;
        const float4 sc = *reinterpret_cast<const float4 *>(a.tok_scalars + th * 4);
        steps[tid] = sc.x;
        nraw = sc.z;
        bet = a.beta[th];
    }
    if (project && tid < K) d = a.d_ckpt[bhn * K + tid];
#pragma unroll
    for (int m = 0; m < NVK; ++m)
#pragma unroll
        for (int e4 = 0; e4 < VN; e4 += 4) {
            float sq[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float kf = vec_get<T>(kv[m], e4 + e);
                sq[e] = kf * kf;
            }
            store_vec(Ss + i * LDT + part * EPT + m * VN + e4, sq);
        }
    __syncthreads();
    // ---- the box masks of the chunk; does it qualify?  (no coordinate met the box at any token) ----
    bool ok = true;
    if (project && tid < K) {
        uint32_t mlo = 0u, mhi = 0u;
#pragma unroll 8
        for (int t = 0; t < C; ++t) {
            const float sq = Ss[t * LDT + tid], st = steps[t];
            const uint32_t in = lands_inside<false>(1.f, d, st, sq, a.d_min, a.d_max) ? (1u << (t & 31)) : 0u;
            d = clip3(d_bar<false>(1.f, d, st, sq), a.d_min, a.d_max);
            if (t < 32) mlo |= in; else mhi |= in;
        }
        a.masks[bhn * K + tid] = make_uint2(mlo, mhi);
        ok = (mlo & mhi) == 0xffffffffu;
    }
    const int clean = __syncthreads_and(ok ? 1 : 0);
    if (tid == 0) a.lin_clean[bhn] = clean;
    if (!clean) return;
    if (tid < C) {
        const float nn = fmaxf(nraw, a.eps);
        const float bp = a.beta_aware ? bet : 1.f;
        cas[tid] = a.eta * bp / nn * bp;
    }
    __syncthreads();
    // ---- A = tril(ca_i <s_i, s_j>, -1): the transpose of U; (I + A)^-1 = ((I + U)^-1)^T ----
    for (int idx = wave; idx < 10; idx += P1W) {
        const int ib = idx < 1 ? 0 : idx < 3 ? 1 : idx < 6 ? 2 : 3;
        const int jb = idx - (ib * (ib + 1)) / 2;
        const f32x4 acc = mma_tile0<float, true, true>(Ss + ib * 16 * LDT, LDT, Ss + jb * 16 * LDT, LDT, K, lane);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int ii = ib * 16 + acc_row(lane, r), jj = jb * 16 + acc_col(lane);
            Af[ii * LDF + jj] = (jj < ii) ? cas[ii] * acc[r] : 0.f;
        }
    }
    __syncthreads();                                             // the s tile is dead: its space takes the inverse
    ut_inverse64<LDF>(Af, Ti, Xs, wave, lane);
    // ---- (I + U)^-1, row i: entries j >= i are column i of the lower inverse ----
    // (kept in the I/O type: its diagonal is 1 and the rest is of the size of the step, so with
    // bf16 I/O the rounding is far inside what that I/O type's other operands carry)
    {
        T *mg = static_cast<T *>(a.lin_M) + bhn * C * C + i * C + part * 8;
        constexpr int VNM = 16 / sizeof(T);
#pragma unroll
        for (int e4 = 0; e4 < 8; e4 += VNM) {
            float o[VNM];
#pragma unroll
            for (int e = 0; e < VNM; ++e) {
                const int j = part * 8 + e4 + e;
                o[e] = j >= i ? Ti[j * LDF + i] : 0.f;
            }
            store_vec(mg + e4, o);
        }
    }
}

// rho0_i = <s_i, sum_{j > i} lambda_j> and sum_j lambda_j, lambda_j = k_j (.) dL/dk~_j: thread
// (c = tid % K, tg = tid / K) keeps TS consecutive tokens of coordinate c in registers; the suffix
// sums run down its tokens and across the runs through LDS; the row dots are folded over the lanes
// as in the sweeps of precond_chain.
template <typename T, int K>
__global__ __launch_bounds__(P1T) void precond_lin_r_kernel(PrecondBwdArgs a) {
    constexpr int NSEG = P1T / K, TS = C / NSEG, WPS = K / 64, NPART = K / TS;
    __shared__ float tot[NSEG * K];
    __shared__ float part[P1W * 64];
    const int n = a.n0 + blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c = tid % K, sg = tid / K;
    const int N = a.T / C;
    const size_t bhn = ((size_t)b * a.H + h) * N + n;
    if (!a.lin_clean[bhn]) return;                               // (uniform)
    const size_t tokc = ((size_t)b * a.T + (size_t)n * C) * a.H + h;
    const uint32_t kstride = (uint32_t)a.H * K;
    const T *kp = static_cast<const T *>(a.k) + tokc * K, *gp = static_cast<const T *>(a.dkt) + tokc * K;
    float sv[TS], lam[TS];
#pragma unroll
    for (int u = 0; u < TS; ++u) {
        const uint32_t o = (uint32_t)(sg * TS + u) * kstride + (uint32_t)c;
        const float kf = to_f32(lane_elem(kp, o));
        sv[u] = kf * kf;
        lam[u] = kf * to_f32(lane_elem(gp, o));
    }
    float acc = 0.f;
#pragma unroll
    for (int u = TS - 1; u >= 0; --u) {                          // exclusive suffix sums inside the run
        const float t = lam[u];
        lam[u] = acc;
        acc += t;
    }
    tot[sg * K + c] = acc;
    __syncthreads();
    float offs = 0.f;
#pragma unroll
    for (int g2 = NSEG - 1; g2 > 0; --g2)
        if (g2 > sg) offs += tot[g2 * K + c];
    if (sg == 0) a.lin_t0[bhn * K + c] = acc + offs;
    float prod[TS];
#pragma unroll
    for (int u = 0; u < TS; ++u) prod[u] = sv[u] * (lam[u] + offs);
    part[wave * 64 + lane] = lane_fold<TS>(prod, lane);
    __syncthreads();
    if (tid < C) {
        const int w0 = (tid / TS) * WPS, u = tid % TS;
        float r = 0.f;
#pragma unroll
        for (int j = 0; j < NPART; ++j) r += part[(w0 + j / (64 / TS)) * 64 + (j % (64 / TS)) * TS + u];
        a.lin_r0[bhn * C + tid] = r;
    }
}

// --------------------------------------------------------------- precond_chain ----
// The adjoint recurrence is linear in a (the masks are data of the forward pass), so a chunk
// is cut into NSEG = 512 / K runs of TS tokens and every thread owns one coordinate of one
// run, all in registers: it runs the recurrence over its TS tokens from a zero right-hand
// value, keeping abar_i = L_i + P_i * carry in the two parts L_i, P_i; the runs are chained
// through LDS (one fma per run); the TS products s_i abar_i of a thread are folded over the
// lanes of the wavefront (each lane ends with the sum of one token over a group of lanes) and
// the sigma of a token is the sum of K / TS such partials.  No tile of the chunk is ever in LDS.
// LINK: chunks that qualify take the solved form (no retention only; see the top of this file)
template <typename T, int K, int RET, bool LINK>
__global__ __launch_bounds__(P1T) void precond_chain_kernel(PrecondBwdArgs a) {
    static_assert(!LINK || RET == 0, "the solved form has no retention");
    constexpr bool HAS_RET = RET != 0, RET_VEC = RET == 2;
    constexpr int NSEG = P1T / K;                 // runs per chunk
    constexpr int TS = C / NSEG;                  // tokens per run
    constexpr int WPS = K / 64;                   // wavefronts per run
    constexpr int NPART = K / TS;                 // partial sums per token
    __shared__ float ga[K];                      // adjoint of d at the right end of the chunk
    __shared__ float segL[NSEG * K], segP[NSEG * K];
    __shared__ float cas[C], sig[C];
    __shared__ __attribute__((aligned(16))) float rs[C];
    __shared__ __attribute__((aligned(16))) float casig[C];
    __shared__ float part[P1W * 64];
    __shared__ int done;
    // chunks in solved form (see the top of this file)
    typedef Lin<K> LN;
    constexpr int EPT = LN::EPT, VN = 16 / sizeof(T), NVK = EPT / VN, NG = LN::NG;
    __shared__ __attribute__((aligned(16))) float Sl[C * LN::LD];       // s = k^2 of the chunk
    __shared__ __attribute__((aligned(16))) float gp[8 * LN::VSTR];     // copy of ga, sliced per thread of the row layout
    __shared__ __attribute__((aligned(16))) float xs[8 * LN::XSTR];     // S g + rho0
    __shared__ float ws[C];                                             // ca (.) sigma

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c = tid % K, sg = tid / K;          // coordinate and run of this thread
    const int li = tid >> 3, lpart = tid & 7;     // row layout of the solved form: token, slice
    const int lc = tid / NG, ltg = tid % NG;      // column layout: coordinate, token group
    const int b = blockIdx.x / a.H, h = blockIdx.x % a.H;     // b: batch entry, or packed sequence
    const size_t bh = (size_t)b * a.H + h;                    // the chain: indexes dd_out / dd_in
    int bt = b;                                               // batch entry of the token tensors
    if (a.seq_chunks) {
        bool begins, ends;
        if (!clip_to_sequence(a.seq_chunks, b, a.n0, a.n1, begins, ends)) return;
        a.dd_out = ends ? a.dd_last : a.dd_in;
        bt = 0;
    }
    const size_t bth = (size_t)bt * a.H + h;                  // indexes the per-chunk buffers
    const bool project = a.d_min <= a.d_max;
    const int N = a.T / C;
    const uint32_t kstride = (uint32_t)a.H * K;   // elements between consecutive tokens

    if (tid < K) {
        const float g0 = a.dd_out ? a.dd_out[bh * K + tid] : 0.f;
        ga[tid] = g0;
        gp[LN::vidx(tid)] = g0;
    }

    T kreg[TS], greg[TS];
    float rreg[RET_VEC ? TS : 1];               // per-coordinate retention of the next chunk
    float nrawreg = 1.f, betreg = 0.f, retreg = 1.f;
    uint2 mreg = make_uint2(0xffffffffu, 0xffffffffu);
#define OSDN_P1_BLOAD(n_)                                                                        \
    {                                                                                            \
        const size_t tokc_ = ((size_t)bt * a.T + (size_t)(n_) * C) * a.H + h;                    \
        const T *kp_ = static_cast<const T *>(a.k) + tokc_ * K;                                  \
        const T *gp_ = static_cast<const T *>(a.dkt) + tokc_ * K;                                \
        _Pragma("unroll") for (int u = 0; u < TS; ++u) {                                         \
            const uint32_t o_ = (uint32_t)(sg * TS + u) * kstride + (uint32_t)c;                 \
            kreg[u] = lane_elem(kp_, o_); greg[u] = lane_elem(gp_, o_);                          \
            if (RET_VEC) rreg[RET_VEC ? u : 0] = lane_elem(a.retention + tokc_ * K, o_);         \
        }                                                                                        \
        if (tid < C) {                                                                           \
            const size_t th = tokc_ + (size_t)tid * a.H;                                         \
            nrawreg = a.tok_scalars[th * 4 + 2];                                                 \
            betreg = a.beta[th];                                                                 \
            if (HAS_RET && !RET_VEC) retreg = a.retention[th];                                   \
        }                                                                                        \
        if (project) mreg = a.masks[(bth * N + (n_)) * K + c];                                   \
    }
    // Registers of a chunk in solved form: the thread's slice of its key row and of its row of
    // the inverse, the token's scalars (slice 0 only), the coordinate's sum of lambda (group 0 only).
    struct LinRegs {
        u32x4 kq[NVK];
        u32x4 mq[8 * sizeof(T) / 16];
        float rho, nraw, beta, t0;
    };
#define OSDN_P1_LLOAD(n_, R)                                                                     \
    {                                                                                            \
        __builtin_amdgcn_sched_barrier(0);     /* the sets are requested in program order */     \
        const size_t tokc_ = ((size_t)bt * a.T + (size_t)(n_) * C) * a.H + h;                    \
        const size_t bhn_ = bth * N + (n_);                                                      \
        const uint32_t off_ = ((uint32_t)li * kstride + (uint32_t)(lpart * EPT)) * (uint32_t)sizeof(T); \
        const u32x4 *kp_ = reinterpret_cast<const u32x4 *>(static_cast<const T *>(a.k) + tokc_ * K); \
        _Pragma("unroll") for (int m_ = 0; m_ < NVK; ++m_) R.kq[m_] = at_byte(kp_, off_ + 16 * m_); \
        const u32x4 *mp_ = reinterpret_cast<const u32x4 *>(static_cast<const T *>(a.lin_M) + bhn_ * C * C + li * C + lpart * 8); \
        _Pragma("unroll") for (int m_ = 0; m_ < (int)(8 * sizeof(T) / 16); ++m_) R.mq[m_] = mp_[m_]; \
        const size_t th = tokc_ + (size_t)li * a.H;      /* (every lane of a token loads its scalars) */ \
        R.nraw = a.tok_scalars[th * 4 + 2];                                                      \
        R.beta = a.beta[th];                                                                     \
        R.rho = a.lin_r0[bhn_ * C + li];                                                         \
        R.t0 = a.lin_t0[bhn_ * K + lc];                                                          \
        __builtin_amdgcn_sched_barrier(0);                                                       \
    }
    // One chunk in solved form from the registers R (a step outside the run [m_lo, n_hi] does
    // nothing but the refill); when they have been read, they are refilled with the chunk three
    // further on (clamped to the run: past its end a harmless reload of its last chunk).  No load or store of the step sits under a branch, and lanes that hold the
    // same value all store it: the loads of the other two register sets then stay in flight
    // across the step (behind a branch the compiler can no longer count what is outstanding and
    // waits for everything).
#define OSDN_P1_LSTEP(n_, R, m_lo, n_hi)                                                         \
    {                                                                                            \
        const bool act_ = (n_) <= (n_hi) && (n_) >= (m_lo);       /* uniform */                  \
        float pre_ = 0.f;                                                                        \
        if (act_) {                                                                              \
        const size_t tokc_s = ((size_t)bt * a.T + (size_t)(n_) * C) * a.H + h;                   \
        a.a_ckpt[(bth * N + (n_)) * K + c] = ga[c];                                              \
        /* x = S g + rho0, and the s tile into LDS for the product with S^T */                   \
        float y = 0.f;                                                                           \
        _Pragma("unroll") for (int m_ = 0; m_ < NVK; ++m_)                                       \
            _Pragma("unroll") for (int e4 = 0; e4 < VN; e4 += 4) {                               \
                const f32x4 gv = *reinterpret_cast<const f32x4 *>(gp + lpart * LN::VSTR + m_ * VN + e4); \
                float sq[4];                                                                     \
                _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                  \
                    const float kf = vec_get<T>(R.kq[m_], e4 + e);                               \
                    sq[e] = kf * kf;                                                             \
                    y = __builtin_fmaf(sq[e], gv[e], y);                                         \
                }                                                                                \
                store_vec(Sl + li * LN::LD + LN::swz(lpart * EPT + m_ * VN + e4), sq);                    \
            }                                                                                    \
        y = sum_lanes8(y);                                                                       \
        const float nn_ = fmaxf(R.nraw, a.eps);                                                  \
        const float bp_ = a.beta_aware ? R.beta : 1.f;                                           \
        const float ca_i = a.eta * bp_ / nn_ * bp_;                                              \
        xs[LN::xidx(li)] = y + R.rho;                                                            \
        __syncthreads();                                                                         \
        /* sigma = (I + U)^-1 x */                                                               \
        float sgm = 0.f;                                                                         \
        _Pragma("unroll") for (int h4 = 0; h4 < 2; ++h4) {                                       \
            const f32x4 xv = *reinterpret_cast<const f32x4 *>(xs + lpart * LN::XSTR + 4 * h4);   \
            _Pragma("unroll") for (int e = 0; e < 4; ++e)                                        \
                sgm = __builtin_fmaf(vec_get<T>(R.mq[(4 * h4 + e) / VN], (4 * h4 + e) % VN), xv[e], sgm); \
        }                                                                                        \
        sgm = sum_lanes8(sgm);                                                                   \
        ws[li] = ca_i * sgm;                                                                     \
        a.tok_scalars[(tokc_s + (size_t)li * a.H) * 4 + 3] = sgm;                                \
        pre_ = ga[lc] + R.t0;                   /* (no loaded value is kept past the refill, */  \
        asm volatile("" : "+v"(pre_));          /*  and this sum is not moved behind it)     */  \
        }                                                                                        \
        OSDN_P1_LLOAD(min(max((n_) - 3, (m_lo)), (n_hi)), R)                                     \
        if (act_) {                                                                              \
        __syncthreads();                                                                         \
        /* a_left = g + sum lambda - S^T (ca (.) sigma) */                                       \
        float acc_ = 0.f;                                                                        \
        _Pragma("unroll") for (int u = 0; u < C / NG; ++u)                                       \
            acc_ = __builtin_fmaf(Sl[(u * NG + ltg) * LN::LD + LN::swz(lc)], ws[u * NG + ltg], acc_);     \
        acc_ = NG == 4 ? sum_lanes4(acc_) : sum_lanes8(acc_);                                    \
        const float gn = pre_ - acc_;                                                            \
        ga[lc] = gn;                                                                             \
        gp[LN::vidx(lc)] = gn;                                                                   \
        __syncthreads();                                                                         \
        }                                                                                        \
    }
    // Which chunks take the solved form: the flags precond_lin left, as bits in LDS (bit n - n0;
    // chunks past the table's reach sweep).  With LINK only the solved form prefetches (three
    // chunks deep, inside a run of such chunks); a chunk that has to sweep fetches its operands
    // when it starts: keeping both sets of registers alive across the loop would spill.
    constexpr int FLAG_WORDS = 512;
    __shared__ uint32_t flagw[LINK ? FLAG_WORDS : 1];
    const bool lin = LINK && a.lin_clean != nullptr;
    if (lin) {
        for (int base = 0; base < a.n1 - a.n0 && base < FLAG_WORDS * 32; base += P1T) {
            const int nn = a.n0 + base + tid;
            const int f = nn < a.n1 ? a.lin_clean[bth * N + nn] : 0;
            const unsigned long long bits = __ballot(f != 0);
            if (lane == 0) {
                flagw[(base >> 5) + 2 * wave] = (uint32_t)bits;
                flagw[(base >> 5) + 2 * wave + 1] = (uint32_t)(bits >> 32);
            }
        }
    }
    if (!LINK) OSDN_P1_BLOAD(a.n1 - 1)
    __syncthreads();
    auto solved = [&](int nn) -> bool {            // uniform
        const int r = nn - a.n0;
        return lin && r < FLAG_WORDS * 32 && ((flagw[LINK ? r >> 5 : 0] >> (r & 31)) & 1u) != 0;
    };

    for (int n = a.n1 - 1; n >= a.n0; --n) {
        const size_t tokc = ((size_t)bt * a.T + (size_t)n * C) * a.H + h;
        if (LINK && solved(n)) {
            // the run [m, n] of chunks in solved form, three chunks in flight
            int m = n;
            while (m > a.n0 && solved(m - 1)) --m;
            // (the first three steps only request operands: with nothing requested ahead of the
            // loop, the compiler's count of what is outstanding at the top of the loop is exact)
            LinRegs r0, r1, r2;
            for (int j = n + 3; j >= m; j -= 3) {
                OSDN_P1_LSTEP(j, r0, m, n)
                OSDN_P1_LSTEP(j - 1, r1, m, n)
                OSDN_P1_LSTEP(j - 2, r2, m, n)
            }
            n = m;                                  // (the loop's own decrement moves past the run)
            continue;
        }
        // ---- this thread's (s, lambda) = (k^2, k . dL/dk~) and mask bits ----
        if (LINK) OSDN_P1_BLOAD(n)
        float sv[TS], lam[TS];
#pragma unroll
        for (int u = 0; u < TS; ++u) {
            const float kv = to_f32(kreg[u]);
            sv[u] = kv * kv;
            lam[u] = kv * to_f32(greg[u]);
        }
        const uint32_t mword = (sg * TS) < 32 ? mreg.x : mreg.y;
        const uint32_t mbits = (mword >> ((sg * TS) & 31)) & ((1u << TS) - 1u);
        if (tid < C) {
            const float nn = fmaxf(nrawreg, a.eps);
            const float bp = a.beta_aware ? betreg : 1.f;
            rs[tid] = retreg; cas[tid] = a.eta * bp / nn * bp; sig[tid] = 0.f; casig[tid] = 0.f;
        }
        if (tid < K) a.a_ckpt[(bth * N + n) * K + tid] = ga[tid];
        __syncthreads();
        float rv[TS];                           // retention of this thread's coordinate, token by token
        if (HAS_RET) {
#pragma unroll
            for (int u = 0; u < TS; ++u) rv[u] = RET_VEC ? rreg[RET_VEC ? u : 0] : rs[sg * TS + u];
        }
        if (!LINK && n > a.n0) OSDN_P1_BLOAD(n - 1)      // next chunk: in flight during the sweeps
        // a wavefront whose coordinates never touched the box in this run, without retention:
        // P stays 1 and L is a plain running sum
        const bool plain = !HAS_RET && __all(mbits == ((1u << TS) - 1u));
        // ---- sweeps for sigma_i = <s_i, abar_i> ----
        float dprev = 0.f, a_left = 0.f;
        for (int sweep = 0; sweep < P1_MAX_SWEEPS; ++sweep) {
            float abL[TS], abP[TS];
            float loc = 0.f, P = 1.f;
            if (plain) {
#pragma unroll
                for (int u = TS - 1; u >= 0; --u) {
                    abL[u] = loc;
                    loc += __builtin_fmaf(-casig[sg * TS + u], sv[u], lam[u]);
                }
            } else {
#pragma unroll
                for (int u = TS - 1; u >= 0; --u) {
                    const bool in = (mbits >> u) & 1u;
                    abL[u] = in ? loc : 0.f;
                    abP[u] = in ? P : 0.f;
                    const float src = __builtin_fmaf(-casig[sg * TS + u], sv[u], lam[u]);
                    loc = HAS_RET ? __builtin_fmaf(rv[u], abL[u], src) : abL[u] + src;
                    P = HAS_RET ? rv[u] * abP[u] : abP[u];
                }
            }
            segL[sg * K + c] = loc;
            segP[sg * K + c] = P;
            __syncthreads();
            // value of a at the right end of this run: chain the runs to its right
            float carry = ga[c];
#pragma unroll
            for (int s2 = NSEG - 1; s2 > 0; --s2)
                if (s2 > sg) carry = __builtin_fmaf(segP[s2 * K + c], carry, segL[s2 * K + c]);
            a_left = __builtin_fmaf(P, carry, loc);      // (meaningful in run 0: left end of the chunk)
            float prod[TS];
            if (plain) {
#pragma unroll
                for (int u = 0; u < TS; ++u) prod[u] = sv[u] * (abL[u] + carry);
            } else {
#pragma unroll
                for (int u = 0; u < TS; ++u) prod[u] = sv[u] * __builtin_fmaf(abP[u], carry, abL[u]);
            }
            part[wave * 64 + lane] = lane_fold<TS>(prod, lane);
            __syncthreads();
            if (tid < C) {
                const int i = tid, w0 = (i / TS) * WPS, u = i % TS;
                float sg_ = 0.f;
#pragma unroll
                for (int j = 0; j < NPART; ++j)     // fixed order: wavefronts of the run, lane groups
                    sg_ += part[(w0 + j / (64 / TS)) * 64 + (j % (64 / TS)) * TS + u];
                const float mx = wave_max(fabsf(sg_));
                const float dcur = wave_max(fabsf(sg_ - sig[i]));
                // converged, or (from the second pass on) the observed contraction ratio says
                // that the next difference would be below the tolerance
                const bool all_ok = dcur <= P1_TOL_BWD * mx ||
                                    (sweep >= 1 && dcur <= 0.1f * dprev && dcur * dcur <= P1_TOL_BWD * mx * dprev);
                dprev = dcur;
                sig[i] = sg_;
                casig[i] = cas[i] * sg_;
                if (tid == 0) done = all_ok ? 1 : 0;
            }
            __syncthreads();
            if (done) break;
        }
        // ---- accepted: sig generated a_left ----
        if (tid < C) a.tok_scalars[(tokc + (size_t)tid * a.H) * 4 + 3] = sig[tid];
        if (sg == 0) { ga[c] = a_left; gp[LN::vidx(c)] = a_left; }
        __syncthreads();
    }
    if (tid < K) a.dd_in[bh * K + tid] = ga[tid];
}

// ---------------------------------------------------------------- precond_post ----
//   in : k, beta, retention, d_ckpt, tok_scalars (step, <d,s>, sum s, sigma per token),
//        a_ckpt (adjoint of d at the right end of every chunk), dkt (dL/dk~),
//        dk_read (read-side dL/dk), dbeta (partial, from phase 2)
//   out: dk (io type) = dk_read + d_t . dkt + 2 k_t (step_t abar_t + g_p d_t + g_nraw),
//        dbeta += sigma_t eta (1 - 2 b' p_t)/n_t,  dretention_t = <abar_t, d_t>
template <typename T, int K, int RET>
__global__ __launch_bounds__(K) __attribute__((amdgpu_waves_per_eu(2, 8))) void precond_post_kernel(PrecondBwdArgs a) {
    constexpr bool HAS_RET = RET != 0, RET_VEC = RET == 2;
    constexpr int LD = K + 1;
    __shared__ __attribute__((aligned(16))) float st_s[C];
    __shared__ __attribute__((aligned(16))) float r_s[C];
    __shared__ __attribute__((aligned(16))) float casig_s[C];
    __shared__ __attribute__((aligned(16))) float gp_s[C];
    __shared__ __attribute__((aligned(16))) float gn_s[C];
    // the scalar gate's dL/dr_i = sum over the coordinates of abar_i d_i: folded over the lanes of a
    // wavefront eight tokens at a time, one partial per wavefront and token here
    __shared__ float rpart[(HAS_RET && !RET_VEC) ? (K / 64) * C : 1];
    static_assert(PB == 8, "the fold takes eight values per lane");
    const int n = a.n0 + blockIdx.x, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int N = a.T / C;
    const size_t bh = (size_t)b * a.H + h;
    const size_t tokc = ((size_t)b * a.T + (size_t)n * C) * a.H + h;
    const bool project = a.d_min <= a.d_max;
    const float lo = project ? a.d_min : -INFINITY, hi = project ? a.d_max : INFINITY;
    if (tid < C) {
        const size_t th = tokc + (size_t)tid * a.H;
        const float4 sc = *reinterpret_cast<const float4 *>(a.tok_scalars + th * 4);
        const float step = sc.x, p = sc.y, n_raw = sc.z, sg = sc.w;
        const float bet = a.beta[th];
        const float nn = fmaxf(n_raw, a.eps);
        const float bp = a.beta_aware ? bet : 1.f;
        const float ca = a.eta * bp / nn * bp;
        st_s[tid] = step;
        r_s[tid] = (HAS_RET && !RET_VEC) ? a.retention[th] : 1.f;
        casig_s[tid] = ca * sg;
        gp_s[tid] = -sg * ca;
        gn_s[tid] = (n_raw >= a.eps) ? -sg * step / nn : 0.f;
        if (a.beta_aware) a.dbeta[th] += sg * a.eta * (1.f - 2.f * bp * p) / nn;
    }
    // uniform bases + 32-bit per-thread offsets (64 rows of H*K elements: below 2^31)
    const T *kp = static_cast<const T *>(a.k) + tokc * K;
    const T *gp = static_cast<const T *>(a.dkt) + tokc * K, *rp = static_cast<const T *>(a.dk_read) + tokc * K;
    T *op = static_cast<T *>(a.dk) + tokc * K;
    const float *retp = RET_VEC ? a.retention + tokc * K : nullptr;     // per-coordinate retention and its gradient
    float *dretp = (RET_VEC && a.dretention) ? a.dretention + tokc * K : nullptr;
    const uint32_t kstride = (uint32_t)a.H * K;
    float Dv[C];
    // which steps landed inside the box: decided once, by precond_mask (or precond_lin_m)
    const uint2 mbits = project ? a.masks[(bh * N + n) * K + tid] : make_uint2(0xffffffffu, 0xffffffffu);
    const uint32_t mlo = mbits.x, mhi = mbits.y;
    {   // ---- replay d over the chunk (same arithmetic as the forward kernel) ----
        float kv[C];
#pragma unroll
        for (int i = 0; i < C; ++i) kv[i] = to_f32(lane_elem(kp + (size_t)i * kstride, tid));
        float d = a.d_ckpt[(bh * N + n) * K + tid];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < C; ++i) {
            Dv[i] = d;
            const float r = RET_VEC ? lane_elem(retp + (size_t)i * kstride, tid) : r_s[i];
            d = clip3(d_bar<HAS_RET>(r, d, st_s[i], kv[i] * kv[i]), lo, hi);
        }
    }
    // ---- the chunk's adjoint recurrence, right to left, and the elementwise outputs ----
    float av = a.a_ckpt[(bh * N + n) * K + tid];
    // (the per-token scalars are read again through pointers the compiler cannot identify with
    // the arrays, so that it does not keep the replay's 128 values in registers)
    const float *st_p = st_s, *r_p = r_s, *casig_p = casig_s, *gp_p = gp_s, *gn_p = gn_s;
    asm volatile("" : "+v"(st_p), "+v"(r_p), "+v"(casig_p), "+v"(gp_p), "+v"(gn_p));
    float kb[2][PB], gb[2][PB], rb[2][PB], rrb[RET_VEC ? 2 : 1][RET_VEC ? PB : 1];
    // byte offsets (in units of T) of the next row to fetch and of the next row to write
    constexpr uint32_t FS = sizeof(float) / sizeof(T);
    const uint32_t rowb = kstride * (uint32_t)sizeof(T);
    uint32_t lofs = ((uint32_t)tid + (uint32_t)(C - 1) * kstride) * (uint32_t)sizeof(T);
    asm volatile("" : "+v"(lofs));
    uint32_t sofs = lofs;
#define OSDN_PLOAD(buf, ih_)                                                                     \
    _Pragma("unroll") for (int u = 0; u < PB; ++u) {                                             \
        kb[buf][u] = to_f32(at_byte(kp, lofs)); gb[buf][u] = to_f32(at_byte(gp, lofs));          \
        rb[buf][u] = to_f32(at_byte(rp, lofs));                                                  \
        if (RET_VEC) rrb[RET_VEC ? buf : 0][RET_VEC ? u : 0] = at_byte(retp, lofs * FS);         \
        lofs -= rowb;                                                                            \
    }
    OSDN_PLOAD(0, C - 1)
#pragma unroll
    for (int blk = 0; blk < C / PB; ++blk) {
        const int ih = C - 1 - blk * PB;
        if (blk + 1 < C / PB) OSDN_PLOAD((blk + 1) & 1, ih - PB)
        float pr[PB];
#pragma unroll
        for (int u = 0; u < PB; ++u) {
            const int i = ih - u;
            const uint32_t bit = (i < 32 ? mlo : mhi) & (1u << (i & 31));
            const float ab = bit ? av : 0.f;
            const float kv = kb[blk & 1][u], g = gb[blk & 1][u], Di = Dv[i];
            const float gsum = st_p[i] * ab + gp_p[i] * Di + gn_p[i];
            at_byte(op, sofs) = from_f32<T>(rb[blk & 1][u] + Di * g + 2.f * kv * gsum);
            if (RET_VEC) { if (dretp) at_byte(dretp, sofs * FS) = ab * Di; }
            pr[u] = ab * Di;
            sofs -= rowb;
            const float src = __builtin_fmaf(-casig_p[i], kv * kv, kv * g);
            const float r = RET_VEC ? rrb[RET_VEC ? blk & 1 : 0][RET_VEC ? u : 0] : r_p[i];
            av = HAS_RET ? __builtin_fmaf(r, ab, src) : ab + src;
        }
        if (HAS_RET && !RET_VEC) {
            const int lane = tid & 63;
            const float tot = lane_fold8_all(pr, lane);     // lane l: token ih - l % 8, summed over the wavefront
            if (lane < PB) rpart[(HAS_RET && !RET_VEC) ? (tid >> 6) * C + ih - lane : 0] = tot;
        }
    }
    if (HAS_RET && !RET_VEC) {
        __syncthreads();
        if (tid < C && a.dretention) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < K / 64; ++w) s += rpart[(HAS_RET && !RET_VEC) ? w * C + tid : 0];
            a.dretention[tokc + (size_t)tid * a.H] = s;
        }
    }
}

// -------------------------------------------------------------------- launchers ----
template <typename T, int K, int RET>
static void launch_chain_k(const PrecondBwdArgs &a, int nchains, hipStream_t st) {
    if constexpr (RET == 0) {
        if (a.lin_clean) {
            hipLaunchKernelGGL((precond_chain_kernel<T, K, 0, true>), dim3(nchains), dim3(P1T), 0, st, a);
            return;
        }
    }
    hipLaunchKernelGGL((precond_chain_kernel<T, K, RET, false>), dim3(nchains), dim3(P1T), 0, st, a);
}
template <typename T, int RET>
static int launch_precond_bwd_t(const PrecondBwdArgs &a, int which, hipStream_t st) {
    const dim3 per_chunk(a.n1 - a.n0, a.H, a.B);
    const int nchains = (a.seq_chunks ? a.n_seqs : a.B) * a.H;
    if (a.K == 64) {
        if (which == 0) hipLaunchKernelGGL((precond_mask_kernel<T, 64, RET>), per_chunk, dim3(64), 0, st, a);
        else if (which == 1) launch_chain_k<T, 64, RET>(a, nchains, st);
        else hipLaunchKernelGGL((precond_post_kernel<T, 64, RET>), per_chunk, dim3(64), 0, st, a);
    } else if (a.K == 128) {
        if (which == 0) hipLaunchKernelGGL((precond_mask_kernel<T, 128, RET>), per_chunk, dim3(128), 0, st, a);
        else if (which == 1) launch_chain_k<T, 128, RET>(a, nchains, st);
        else hipLaunchKernelGGL((precond_post_kernel<T, 128, RET>), per_chunk, dim3(128), 0, st, a);
    } else {
        return -1;
    }
    return 0;
}
static int launch_precond_bwd_any(const PrecondBwdArgs &a, bool bf16_io, int which, hipStream_t st) {
    const int ret = a.retention ? (a.ret_vec ? 2 : 1) : 0;
    if (ret == 2)
        return bf16_io ? launch_precond_bwd_t<bf16, 2>(a, which, st) : launch_precond_bwd_t<float, 2>(a, which, st);
    if (ret == 1)
        return bf16_io ? launch_precond_bwd_t<bf16, 1>(a, which, st) : launch_precond_bwd_t<float, 1>(a, which, st);
    return bf16_io ? launch_precond_bwd_t<bf16, 0>(a, which, st) : launch_precond_bwd_t<float, 0>(a, which, st);
}
template <typename T>
static int launch_precond_lin_t(const PrecondBwdArgs &a, bool m_part, hipStream_t st) {
    const dim3 per_chunk(a.n1 - a.n0, a.H, a.B);
    if (a.K == 64) {
        if (m_part) hipLaunchKernelGGL((precond_lin_m_kernel<T, 64>), per_chunk, dim3(P1T), 0, st, a);
        else hipLaunchKernelGGL((precond_lin_r_kernel<T, 64>), per_chunk, dim3(P1T), 0, st, a);
    } else if (a.K == 128) {
        if (m_part) hipLaunchKernelGGL((precond_lin_m_kernel<T, 128>), per_chunk, dim3(P1T), 0, st, a);
        else hipLaunchKernelGGL((precond_lin_r_kernel<T, 128>), per_chunk, dim3(P1T), 0, st, a);
    } else {
        return -1;
    }
    return 0;
}
// only without retention.  m_part: flags and inverses of the chunks [n0, n1) (needs the masks when
// there is a box); else rho0 and the sums of lambda (needs the flags and dL/dk~ of those chunks)
int launch_precond_lin_bwd(const PrecondBwdArgs &a, bool bf16_io, bool m_part, hipStream_t st) {
    if (a.retention || !a.lin_clean || !a.lin_M || !a.lin_r0 || !a.lin_t0) return -1;
    return bf16_io ? launch_precond_lin_t<bf16>(a, m_part, st) : launch_precond_lin_t<float>(a, m_part, st);
}
int launch_precond_mask(const PrecondBwdArgs &a, bool bf16_io, hipStream_t st) { return launch_precond_bwd_any(a, bf16_io, 0, st); }
int launch_precond_chain(const PrecondBwdArgs &a, bool bf16_io, hipStream_t st) { return launch_precond_bwd_any(a, bf16_io, 1, st); }
int launch_precond_post(const PrecondBwdArgs &a, bool bf16_io, hipStream_t st) { return launch_precond_bwd_any(a, bf16_io, 2, st); }

}  // namespace osdn
