// Reverse sweep over the preconditioner's recurrence (Section 4.5) in solved form, general case:
// one retention value per (token, head) and any box masks.
//
// With  abar_t = m_t (.) a_{t+1},  sigma_t = <s_t, abar_t>,  a_t = lambda_t + r_t abar_t - ca_t sigma_t s_t
// (s_t = k_t (.) k_t, lambda_t = k_t (.) dL/dk~_t, m_t the 0/1 box mask of token t per coordinate,
// a_64 = g the adjoint that arrives at the chunk's right end) everything is linear in (g, lambda)
// once the masks are known, and they are data of the forward pass.  Writing W(p..q) for the
// per-coordinate indicator "the mask bits p..q are all set" and R(p..q) for the product of r_p..r_q,
// the 64 unknowns sigma of a chunk solve the unit triangular system
//     (I + U) sigma = S~ g + rho0,
//     U_tj  = ca_j R(t+1..j-1) sum_c s_tc s_jc W_c(t..j-1)            (j > t)
//     S~_tc = s_tc R(t+1..63) W_c(t..63)
//     rho0_t = <s_t (.) m_t, b_t>,  b_63 = 0,  b_{t-1} = lambda_t + r_t m_t (.) b_t
// and the adjoint that leaves the chunk on the left is
//     a_0 = D (.) g + t0 - S-^T (ca (.) sigma),   D_c = R(0..63) W_c(0..63),   t0 = b_{-1},
//     S-_tc = s_tc R(0..t-1) W_c(0..t-1).
// A coordinate contributes to U_tj only while its mask bits t..j-1 form one run of ones, so the
// sum over c is not a Gram matrix; but the coordinates whose 64 bits are all set do form one (on
// the fp32 MFMA), those with no bit set contribute nothing, and the few in between are added pair
// by pair.  Three kernels, as for the plain form: precond_gen_m (forward data only: masks, U, its
// inverse, the indicators and retention products the chain needs), precond_gen_r (rho0, t0 once
// dL/dk~ is there) and precond_gen_chain (three matrix-vector products per chunk).
#include "osdn_precond.h"

namespace osdn {

// per-chunk record of the indicators and retention products (bytes)
//   [0, 1024)            u16 rowbits[64][8]: bit e of entry (t, p): W_c(t..63), c = p * EPT + e
//   [1024, 1024 + K)     u8  z0[c]: lowest mask bit of coordinate c that is not set (64: none)
//   [1152, 1408)         f32 rsuf[t] = R(t+1..63)
//   [1408, 1664)         f32 rpre[t] = R(0..t-1)
//   [1664, 1668)         f32 R(0..63)
constexpr int GEN_AUX = 2048, GA_Z0 = 1024, GA_RSUF = 1152, GA_RPRE = 1408, GA_RALL = 1664;

__device__ __forceinline__ uint64_t mask64(uint2 w) { return ((uint64_t)w.y << 32) | w.x; }
// first bit at or above t that is not set in w (64: none)
__device__ __forceinline__ int next_zero(uint64_t w, int t) {
    const uint64_t z = (~w) >> t;
    return z ? t + __builtin_ctzll(z) : 64;
}

// ------------------------------------------------------------------ precond_gen_m ----
template <typename T, int K, bool HAS_RET>
__global__ __launch_bounds__(P1T) void precond_gen_m_kernel(PrecondBwdArgs a) {
    typedef Lin<K> LN;
    constexpr int EPT = LN::EPT, VN = 16 / sizeof(T), NVK = EPT / VN;
    constexpr int LDT = K + 4, LDF = C + 1;
    constexpr int TI_F = C * LDF + 3 * 16 * 17;
    constexpr int NG8 = 8;                       // coordinates staged per round of the pair sums
    static_assert(TI_F <= C * LDT || K == 64, "the inverse reuses the s tile");
    __shared__ __attribute__((aligned(16))) float Ss[C * LDT > TI_F ? C * LDT : TI_F];
    __shared__ __attribute__((aligned(16))) float Af[C * LDF];
    __shared__ float cas[C], steps[C], rs[C];
    __shared__ float rpre_s[C + 1];              // R(0..t-1), t = 0..64
    __shared__ uint2 mw[K];
    __shared__ int mixl[K];
    __shared__ int wcnt[K / 64];
    __shared__ uint32_t cleanw[K / 32];
    __shared__ float colv[NG8][C];
    __shared__ unsigned char nzv[NG8][C];
    float *Ti = Ss, *Xs = Ss + C * LDF;

    const int n = a.n0 + blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int N = a.T / C;
    const size_t bhn = ((size_t)b * a.H + h) * N + n;
    const size_t tokc = ((size_t)b * a.T + (size_t)n * C) * a.H + h;
    const int i = tid >> 3, part = tid & 7;
    const uint32_t kstride = (uint32_t)a.H * K;
    unsigned char *aux = a.lin_aux + bhn * GEN_AUX;
    const bool project = a.d_min <= a.d_max;
    const float lo = project ? a.d_min : -INFINITY, hi = project ? a.d_max : INFINITY;

    u32x4 kv[NVK];
    {
        const uint32_t off = ((uint32_t)i * kstride + (uint32_t)(part * EPT)) * (uint32_t)sizeof(T);
        const u32x4 *kp = reinterpret_cast<const u32x4 *>(static_cast<const T *>(a.k) + tokc * K);
#pragma unroll
        for (int m = 0; m < NVK; ++m) kv[m] = at_byte(kp, off + 16 * m);
    }
    float d = 1.f;
    if (tid < C) {
        const size_t th = tokc + (size_t)tid * a.H;
        const float4 sc = *reinterpret_cast<const float4 *>(a.tok_scalars + th * 4);
        const float bet = a.beta[th];
        const float nn = fmaxf(sc.z, a.eps);
        const float bp = a.beta_aware ? bet : 1.f;
        steps[tid] = sc.x;
        cas[tid] = a.eta * bp / nn * bp;
        rs[tid] = HAS_RET ? a.retention[th] : 1.f;
    }
    if (project && tid < K) d = a.d_ckpt[bhn * K + tid];
    if (tid < K / 32) cleanw[tid] = 0u;
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
    // ---- the box masks (replay of d, the arithmetic of precond_mask); the coordinates sorted into
    //      all bits set / no bit set / in between; the retention products ----
    if (tid < K) {
        uint32_t mlo = 0xffffffffu, mhi = 0xffffffffu;
        if (project) {
            mlo = 0u; mhi = 0u;
#pragma unroll 8
            for (int t = 0; t < C; ++t) {
                const float sq = Ss[t * LDT + tid], st = steps[t], r = rs[t];
                const uint32_t in = lands_inside<HAS_RET>(r, d, st, sq, lo, hi) ? (1u << (t & 31)) : 0u;
                d = clip3(d_bar<HAS_RET>(r, d, st, sq), lo, hi);
                if (t < 32) mlo |= in; else mhi |= in;
            }
            a.masks[bhn * K + tid] = make_uint2(mlo, mhi);
        }
        mw[tid] = make_uint2(mlo, mhi);
        const uint64_t w = mask64(make_uint2(mlo, mhi));
        aux[GA_Z0 + tid] = (unsigned char)next_zero(w, 0);
        const bool clean = w == ~0ull, mixed = !clean && w != 0ull;
        const unsigned long long cb = __ballot(clean), mb = __ballot(mixed);
        if (lane == 0) {
            cleanw[2 * wave] = (uint32_t)cb;
            cleanw[2 * wave + 1] = (uint32_t)(cb >> 32);
            wcnt[wave] = __builtin_popcountll(mb);
        }
        // (position inside this wavefront's part of the list; the offset of the part follows below)
        if (mixed) mixl[wave * 64 + __builtin_popcountll(mb & ((1ull << lane) - 1ull))] = tid;
    } else if (tid >= P1T - C) {
        // prefix and suffix products of the retention over the 64 tokens (one wavefront, lane = token)
        const int t = lane;
        float inc = HAS_RET ? rs[t] : 1.f, dec = inc;            // inclusive scans from the left / from the right
        if (HAS_RET) {
#pragma unroll
            for (int sft = 1; sft < C; sft <<= 1) {
                const float up = __shfl_up(inc, sft, 64), dn = __shfl_down(dec, sft, 64);
                if (t >= sft) inc *= up;
                if (t + sft < C) dec *= dn;
            }
        }
        float pre = __shfl_up(inc, 1, 64), suf = __shfl_down(dec, 1, 64);
        if (t == 0) pre = 1.f;
        if (t == C - 1) suf = 1.f;
        rpre_s[t] = pre;
        if (t == C - 1) rpre_s[C] = inc;
        *reinterpret_cast<float *>(aux + GA_RPRE + 4 * t) = pre;
        *reinterpret_cast<float *>(aux + GA_RSUF + 4 * t) = suf;
        if (t == C - 1) *reinterpret_cast<float *>(aux + GA_RALL) = inc;
    }
    __syncthreads();
    // ---- W_c(t..63) for this thread's token and coordinates ----
    {
        uint32_t bits = 0u;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const uint64_t w = mask64(mw[part * EPT + e]);
            bits |= (((~w) >> i) == 0ull) ? (1u << e) : 0u;
        }
        reinterpret_cast<uint16_t *>(aux)[i * 8 + part] = (uint16_t)bits;
    }
    // ---- pair sums over the coordinates in between: thread (t = i, j = t + 1 + 8 q + part) ----
    float acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = 0.f;
    int nmix = 0;
#pragma unroll
    for (int w = 0; w < K / 64; ++w) nmix += wcnt[w];
    for (int base = 0; base < nmix; base += NG8) {
        const int cnt = min(NG8, nmix - base);
        if (wave < cnt) {
            // entry base + wave of the list (the parts of the wavefronts one after the other)
            int idx = base + wave, w = 0;
            while (idx >= wcnt[w]) { idx -= wcnt[w]; ++w; }
            const int c = mixl[w * 64 + idx];
            colv[wave][lane] = Ss[lane * LDT + c];
            nzv[wave][lane] = (unsigned char)next_zero(mask64(mw[c]), lane);
        }
        __syncthreads();
        for (int g = 0; g < cnt; ++g) {
            const float st = colv[g][i];
            const int nz = nzv[g][i];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int j = i + 1 + 8 * q + part;
                const float sj = colv[g][j & (C - 1)];
                acc[q] = (j <= nz && j < C) ? __builtin_fmaf(st, sj, acc[q]) : acc[q];
            }
        }
        __syncthreads();
    }
    // ---- Gram matrix of the coordinates whose bits are all set (if there are any), on the MFMA ----
    bool anyclean = false;
#pragma unroll
    for (int w = 0; w < K / 32; ++w) anyclean = anyclean || cleanw[w] != 0u;     // (uniform)
    if (anyclean) {
        const uint32_t cw = cleanw[(part * EPT) >> 5] >> ((part * EPT) & 31);
#pragma unroll
        for (int m = 0; m < NVK; ++m)
#pragma unroll
            for (int e4 = 0; e4 < VN; e4 += 4) {
                float sq[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float kf = vec_get<T>(kv[m], e4 + e);
                    sq[e] = ((cw >> (m * VN + e4 + e)) & 1u) ? kf * kf : 0.f;
                }
                store_vec(Ss + i * LDT + part * EPT + m * VN + e4, sq);
            }
        __syncthreads();
        for (int idx = wave; idx < 10; idx += P1W) {
            const int ib = idx < 1 ? 0 : idx < 3 ? 1 : idx < 6 ? 2 : 3;
            const int jb = idx - (ib * (ib + 1)) / 2;
            const f32x4 g4 = mma_tile0<float, true, true>(Ss + ib * 16 * LDT, LDT, Ss + jb * 16 * LDT, LDT, K, lane);
#pragma unroll
            for (int r = 0; r < 4; ++r) Af[(ib * 16 + acc_row(lane, r)) * LDF + jb * 16 + acc_col(lane)] = g4[r];
        }
        __syncthreads();
    }
    // ---- A = U^T, strictly lower triangular: A_jt = ca_j R(t+1..j-1) (Gram part + pair sums), by the
    //      thread that owns the pair.  R(t+1..j-1) = R(0..j-1) / R(0..t); where that prefix has run
    //      to zero, the product term by term. ----
    {
        const float den = HAS_RET ? rpre_s[i + 1] : 1.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int j = i + 1 + 8 * q + part;
            if (j < C) {
                float P = 1.f;
                if (HAS_RET) {
                    if (den > 1e-30f) P = rpre_s[j] / den;
                    else for (int l = i + 1; l < j; ++l) P *= rs[l];
                }
                const float gram = anyclean ? Af[j * LDF + i] : 0.f;
                Af[j * LDF + i] = cas[j] * P * (gram + acc[q]);
            }
        }
    }
    __syncthreads();                                             // the s tile is dead: its space takes the inverse
    ut_inverse64<LDF>(Af, Ti, Xs, wave, lane);
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
    if (tid == 0) a.lin_clean[bhn] = 1;
}

// ------------------------------------------------------------------ precond_gen_r ----
// rho0 and t0: the adjoint recurrence of the chunk with sigma = 0 and g = 0, in the run layout of
// the sweeps (thread = coordinate c of run sg, TS tokens in registers, the runs chained through LDS).
template <typename T, int K, bool HAS_RET>
__global__ __launch_bounds__(P1T) void precond_gen_r_kernel(PrecondBwdArgs a) {
    constexpr int NSEG = P1T / K, TS = C / NSEG, WPS = K / 64, NPART = K / TS;
    __shared__ float segL[NSEG * K], segP[NSEG * K];
    __shared__ float rs[C];
    __shared__ float part[P1W * 64];
    const int n = a.n0 + blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c = tid % K, sg = tid / K;
    const int N = a.T / C;
    const size_t bhn = ((size_t)b * a.H + h) * N + n;
    const size_t tokc = ((size_t)b * a.T + (size_t)n * C) * a.H + h;
    const uint32_t kstride = (uint32_t)a.H * K;
    const bool project = a.d_min <= a.d_max;
    const T *kp = static_cast<const T *>(a.k) + tokc * K, *gp = static_cast<const T *>(a.dkt) + tokc * K;
    float sv[TS], lam[TS];
#pragma unroll
    for (int u = 0; u < TS; ++u) {
        const uint32_t o = (uint32_t)(sg * TS + u) * kstride + (uint32_t)c;
        const float kf = to_f32(lane_elem(kp, o));
        sv[u] = kf * kf;
        lam[u] = kf * to_f32(lane_elem(gp, o));
    }
    if (tid < C) rs[tid] = HAS_RET ? a.retention[tokc + (size_t)tid * a.H] : 1.f;
    const uint2 mreg = project ? a.masks[bhn * K + c] : make_uint2(0xffffffffu, 0xffffffffu);
    const uint32_t mword = (sg * TS) < 32 ? mreg.x : mreg.y;
    const uint32_t mbits = (mword >> ((sg * TS) & 31)) & ((1u << TS) - 1u);
    __syncthreads();
    float abL[TS], abP[TS];
    float loc = 0.f, P = 1.f;
#pragma unroll
    for (int u = TS - 1; u >= 0; --u) {
        const bool in = (mbits >> u) & 1u;
        const float r = rs[sg * TS + u];
        abL[u] = in ? loc : 0.f;
        abP[u] = in ? P : 0.f;
        loc = __builtin_fmaf(r, abL[u], lam[u]);
        P = r * abP[u];
    }
    segL[sg * K + c] = loc;
    segP[sg * K + c] = P;
    __syncthreads();
    float carry = 0.f;                              // (nothing arrives from the right)
#pragma unroll
    for (int s2 = NSEG - 1; s2 > 0; --s2)
        if (s2 > sg) carry = __builtin_fmaf(segP[s2 * K + c], carry, segL[s2 * K + c]);
    if (sg == 0) a.lin_t0[bhn * K + c] = __builtin_fmaf(P, carry, loc);
    float prod[TS];
#pragma unroll
    for (int u = 0; u < TS; ++u) prod[u] = sv[u] * __builtin_fmaf(abP[u], carry, abL[u]);
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

// -------------------------------------------------------------- precond_gen_chain ----
// One workgroup per chain, chunks right to left, every chunk in solved form:
//     x = R~ (.) (S W~ g) + rho0 ;  sigma = M x ;  g <- D (.) g + t0 - S-^T (ca (.) sigma)
// with the operands of three chunks in flight (three register sets used in turn; no load or
// store sits under a branch, so the loads of the other two sets stay in flight across a step).
template <typename T, int K>
__global__ __launch_bounds__(P1T) void precond_gen_chain_kernel(PrecondBwdArgs a) {
    typedef Lin<K> LN;
    constexpr int EPT = LN::EPT, VN = 16 / sizeof(T), NVK = EPT / VN, NG = LN::NG;
    constexpr int MQ = 8 * sizeof(T) / 16;
    __shared__ float ga[K];
    __shared__ __attribute__((aligned(16))) float Sl[C * LN::LD];
    __shared__ __attribute__((aligned(16))) float gp[8 * LN::VSTR];
    __shared__ __attribute__((aligned(16))) float xs[8 * LN::XSTR];
    __shared__ float ws[C];

    const int tid = threadIdx.x;
    const int c = tid % K;
    const int li = tid >> 3, lpart = tid & 7;
    const int lc = tid / NG, ltg = tid % NG;
    const int b = blockIdx.x / a.H, h = blockIdx.x % a.H;
    const size_t bh = (size_t)b * a.H + h;
    int bt = b;
    if (a.seq_chunks) {
        bool begins, ends;
        if (!clip_to_sequence(a.seq_chunks, b, a.n0, a.n1, begins, ends)) return;
        a.dd_out = ends ? a.dd_last : a.dd_in;
        bt = 0;
    }
    const size_t bth = (size_t)bt * a.H + h;
    const int N = a.T / C;
    const uint32_t kstride = (uint32_t)a.H * K;

    if (tid < K) {
        const float g0 = a.dd_out ? a.dd_out[bh * K + tid] : 0.f;
        ga[tid] = g0;
        gp[LN::vidx(tid)] = g0;
    }
    struct Regs {
        u32x4 kq[NVK];
        u32x4 mq[MQ];
        float rho, ca, rsuf, rpre, t0, rall;
        uint32_t rowbits, z0;
    };
#define OSDN_PG_LOAD(n_, R)                                                                      \
    {                                                                                            \
        __builtin_amdgcn_sched_barrier(0);                                                       \
        const size_t tokc_ = ((size_t)bt * a.T + (size_t)(n_) * C) * a.H + h;                    \
        const size_t bhn_ = bth * N + (n_);                                                      \
        const uint32_t off_ = ((uint32_t)li * kstride + (uint32_t)(lpart * EPT)) * (uint32_t)sizeof(T); \
        const u32x4 *kp_ = reinterpret_cast<const u32x4 *>(static_cast<const T *>(a.k) + tokc_ * K); \
        _Pragma("unroll") for (int m_ = 0; m_ < NVK; ++m_) R.kq[m_] = at_byte(kp_, off_ + 16 * m_); \
        const u32x4 *mp_ = reinterpret_cast<const u32x4 *>(static_cast<const T *>(a.lin_M) + bhn_ * C * C + li * C + lpart * 8); \
        _Pragma("unroll") for (int m_ = 0; m_ < MQ; ++m_) R.mq[m_] = mp_[m_];                    \
        const size_t th = tokc_ + (size_t)li * a.H;                                              \
        const float nraw_ = a.tok_scalars[th * 4 + 2];                                           \
        const float bet_ = a.beta[th];                                                           \
        const unsigned char *aux_ = a.lin_aux + bhn_ * GEN_AUX;                                  \
        R.rho = a.lin_r0[bhn_ * C + li];                                                         \
        R.rsuf = *reinterpret_cast<const float *>(aux_ + GA_RSUF + 4 * li);                      \
        R.rpre = *reinterpret_cast<const float *>(aux_ + GA_RPRE + 4 * li);                      \
        R.rall = *reinterpret_cast<const float *>(aux_ + GA_RALL);                               \
        R.rowbits = reinterpret_cast<const uint16_t *>(aux_)[li * 8 + lpart];                    \
        R.z0 = aux_[GA_Z0 + lc];                                                                 \
        R.t0 = a.lin_t0[bhn_ * K + lc];                                                          \
        const float nn_ = fmaxf(nraw_, a.eps);                                                   \
        const float bp_ = a.beta_aware ? bet_ : 1.f;                                             \
        R.ca = a.eta * bp_ / nn_ * bp_;                                                          \
        __builtin_amdgcn_sched_barrier(0);                                                       \
    }
#define OSDN_PG_STEP(n_, R, m_lo, n_hi)                                                          \
    {                                                                                            \
        const bool act_ = (n_) <= (n_hi) && (n_) >= (m_lo);       /* uniform */                  \
        float pre_ = 0.f;                                                                        \
        uint32_t z0_ = 0u;                                                                       \
        if (act_) {                                                                              \
        const size_t tokc_s = ((size_t)bt * a.T + (size_t)(n_) * C) * a.H + h;                   \
        a.a_ckpt[(bth * N + (n_)) * K + c] = ga[c];                                              \
        float y = 0.f;                                                                           \
        _Pragma("unroll") for (int m_ = 0; m_ < NVK; ++m_)                                       \
            _Pragma("unroll") for (int e4 = 0; e4 < VN; e4 += 4) {                               \
                const f32x4 gv = *reinterpret_cast<const f32x4 *>(gp + lpart * LN::VSTR + m_ * VN + e4); \
                float sq[4];                                                                     \
                _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                  \
                    const float kf = vec_get<T>(R.kq[m_], e4 + e);                               \
                    sq[e] = kf * kf;                                                             \
                    const float gm = ((R.rowbits >> (m_ * VN + e4 + e)) & 1u) ? gv[e] : 0.f;     \
                    y = __builtin_fmaf(sq[e], gm, y);                                            \
                }                                                                                \
                store_vec(Sl + li * LN::LD + LN::swz(lpart * EPT + m_ * VN + e4), sq);           \
            }                                                                                    \
        y = sum_lanes8(y);                                                                       \
        xs[LN::xidx(li)] = __builtin_fmaf(R.rsuf, y, R.rho);                                     \
        __syncthreads();                                                                         \
        float sgm = 0.f;                                                                         \
        _Pragma("unroll") for (int h4 = 0; h4 < 2; ++h4) {                                       \
            const f32x4 xv = *reinterpret_cast<const f32x4 *>(xs + lpart * LN::XSTR + 4 * h4);   \
            _Pragma("unroll") for (int e = 0; e < 4; ++e)                                        \
                sgm = __builtin_fmaf(vec_get<T>(R.mq[(4 * h4 + e) / VN], (4 * h4 + e) % VN), xv[e], sgm); \
        }                                                                                        \
        sgm = sum_lanes8(sgm);                                                                   \
        ws[li] = R.ca * R.rpre * sgm;                                                            \
        a.tok_scalars[(tokc_s + (size_t)li * a.H) * 4 + 3] = sgm;                                \
        pre_ = __builtin_fmaf(R.z0 == 64u ? R.rall : 0.f, ga[lc], R.t0);                         \
        z0_ = R.z0;                                                                              \
        asm volatile("" : "+v"(pre_), "+v"(z0_));                                                \
        }                                                                                        \
        OSDN_PG_LOAD(min(max((n_) - 3, (m_lo)), (n_hi)), R)                                      \
        if (act_) {                                                                              \
        __syncthreads();                                                                         \
        float acc_ = 0.f;                                                                        \
        _Pragma("unroll") for (int u = 0; u < C / NG; ++u) {                                     \
            const int j_ = u * NG + ltg;                                                         \
            const float sv_ = Sl[j_ * LN::LD + LN::swz(lc)];                                     \
            acc_ = __builtin_fmaf((uint32_t)j_ <= z0_ ? sv_ : 0.f, ws[j_], acc_);                \
        }                                                                                        \
        acc_ = NG == 4 ? sum_lanes4(acc_) : sum_lanes8(acc_);                                    \
        const float gn = pre_ - acc_;                                                            \
        ga[lc] = gn;                                                                             \
        gp[LN::vidx(lc)] = gn;                                                                   \
        __syncthreads();                                                                         \
        }                                                                                        \
    }
    __syncthreads();
    {
        const int m = a.n0, n = a.n1 - 1;
        Regs r0, r1, r2;
        for (int j = n + 3; j >= m; j -= 3) {
            OSDN_PG_STEP(j, r0, m, n)
            OSDN_PG_STEP(j - 1, r1, m, n)
            OSDN_PG_STEP(j - 2, r2, m, n)
        }
    }
    if (tid < K) a.dd_in[bh * K + tid] = ga[tid];
#undef OSDN_PG_LOAD
#undef OSDN_PG_STEP
}

// -------------------------------------------------------------------- launchers ----
template <typename T>
static int launch_gen_t(const PrecondBwdArgs &a, int which, hipStream_t st) {
    const dim3 per_chunk(a.n1 - a.n0, a.H, a.B);
    const int nchains = (a.seq_chunks ? a.n_seqs : a.B) * a.H;
    const bool ret = a.retention != nullptr;
#define OSDN_GEN_LAUNCH(K_)                                                                      \
    if (which == 0) {                                                                            \
        if (ret) hipLaunchKernelGGL((precond_gen_m_kernel<T, K_, true>), per_chunk, dim3(P1T), 0, st, a);  \
        else hipLaunchKernelGGL((precond_gen_m_kernel<T, K_, false>), per_chunk, dim3(P1T), 0, st, a);     \
    } else if (which == 1) {                                                                     \
        if (ret) hipLaunchKernelGGL((precond_gen_r_kernel<T, K_, true>), per_chunk, dim3(P1T), 0, st, a);  \
        else hipLaunchKernelGGL((precond_gen_r_kernel<T, K_, false>), per_chunk, dim3(P1T), 0, st, a);     \
    } else {                                                                                     \
        hipLaunchKernelGGL((precond_gen_chain_kernel<T, K_>), dim3(nchains), dim3(P1T), 0, st, a);         \
    }
    if (a.K == 64) { OSDN_GEN_LAUNCH(64) }
    else if (a.K == 128) { OSDN_GEN_LAUNCH(128) }
    else return -1;
#undef OSDN_GEN_LAUNCH
    return 0;
}
// which: 0 = precond_gen_m, 1 = precond_gen_r, 2 = precond_gen_chain (chunks [n0, n1))
int launch_precond_gen(const PrecondBwdArgs &a, bool bf16_io, int which, hipStream_t st) {
    if (a.ret_vec || !a.lin_clean || !a.lin_M || !a.lin_r0 || !a.lin_t0 || !a.lin_aux) return -1;
    return bf16_io ? launch_gen_t<bf16>(a, which, st) : launch_gen_t<float>(a, which, st);
}

}  // namespace osdn
