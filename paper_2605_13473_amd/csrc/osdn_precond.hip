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
    OSDN_P1_LOAD(0)

#ifdef OSDN_DIAG
    long long tph[6] = {0, 0, 0, 0, 0, 0}, tlast = clock64();
#define OSDN_TICK(j) { const long long now_ = clock64(); tph[j] += now_ - tlast; tlast = now_; }
#else
#define OSDN_TICK(j)
#endif
    for (int n = 0; n < N; ++n) {
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
        if (n + 1 < N) OSDN_P1_LOAD(n + 1)
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

// Reverse sweep.  Per chunk, right to left: replay the chunk's d trajectory from the stored
// chunk-start value with the per-token step the forward pass kept (recording, per
// coordinate, a 64-bit mask of the tokens whose unprojected value stayed inside the box);
// find sigma by sweeps; then every output of the chunk is elementwise.
//   in : k, beta, retention, d_ckpt, tok_scalars (step, p, n_raw per token), dkt (dL/dk~,
//        fp32), dk_read (dL/dk read side, fp32), dbeta (partial, from phase 2), dd_out
//   out: dk (io type) = dk_read + d_t . dkt + phase-1 terms ; dbeta += ; dretention ; dd_in
template <typename T, int K, bool HAS_RET>
__global__ __launch_bounds__(P1T) void precond_bwd_kernel(PrecondBwdArgs a) {
    constexpr int LD = K + 1;
    constexpr int NF = C * K / 4 / P1T;           // groups of 4 columns per thread for a [64 x K] tile
    constexpr int KQ = K / P1W;
    __shared__ float ks[C * LD];                 // k
    __shared__ float gs[C * LD];                 // dL/dk~
    __shared__ float Dt[C * LD];                 // d_i
    __shared__ float At[C * LD];                 // masked adjoint abar_i
    __shared__ float ga[K], ganew[K];            // adjoint of d at the right / left end of the chunk
    __shared__ float cas[C], sig[C];
    __shared__ __attribute__((aligned(16))) float steps[C];
    __shared__ __attribute__((aligned(16))) float rs[C];
    __shared__ __attribute__((aligned(16))) float casig[C];
    __shared__ float part[P1W * C], part2[P1W * C];
    __shared__ int done;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int b = blockIdx.x / a.H, h = blockIdx.x % a.H;
    const size_t bh = (size_t)b * a.H + h;
    const T *k = static_cast<const T *>(a.k);
    T *dk = static_cast<T *>(a.dk);
    const bool project = a.d_min <= a.d_max;
    const float lo = project ? a.d_min : -INFINITY, hi = project ? a.d_max : INFINITY;
    const int N = a.T / C;

    if (tid < K) ga[tid] = a.dd_out ? a.dd_out[bh * K + tid] : 0.f;

    // the [64 x K] tiles are walked as groups of 4 columns: thread -> (row r, columns c..c+3)
    u32x2 kreg2[NF];        // bf16: 4 elements = 8 bytes ; fp32 uses kreg4
    u32x4 kreg4[NF];
    float4 greg[NF];
    float4 screg = make_float4(0.f, 0.f, 0.f, 0.f);
    float betreg = 0.f, retreg = 1.f, dbreg = 0.f;
#define OSDN_P1_BLOAD(n_)                                                                        \
    {                                                                                            \
        const size_t tokc_ = ((size_t)b * a.T + (size_t)(n_) * C) * a.H + h;                     \
        _Pragma("unroll") for (int m = 0; m < NF; ++m) {                                         \
            const int i = tid + m * P1T, r = i / (K / 4), c = (i % (K / 4)) * 4;                  \
            const size_t off = (tokc_ + (size_t)r * a.H) * K + c;                                \
            if (sizeof(T) == 2) kreg2[m] = *reinterpret_cast<const u32x2 *>(k + off);            \
            else kreg4[m] = *reinterpret_cast<const u32x4 *>(k + off);                           \
            greg[m] = *reinterpret_cast<const float4 *>(a.dkt + off);                            \
        }                                                                                        \
        if (tid < C) {                                                                           \
            const size_t th = tokc_ + (size_t)tid * a.H;                                         \
            screg = *reinterpret_cast<const float4 *>(a.tok_scalars + th * 4);                   \
            betreg = a.beta[th];                                                                 \
            dbreg = a.dbeta[th];                                                                 \
            if (HAS_RET) retreg = a.retention[th];                                               \
        }                                                                                        \
    }
    OSDN_P1_BLOAD(N - 1)

#ifdef OSDN_DIAG
    long long tph[6] = {0, 0, 0, 0, 0, 0}, tlast = clock64();
#endif
    for (int n = N - 1; n >= 0; --n) {
        const size_t tokc = ((size_t)b * a.T + (size_t)n * C) * a.H + h;
        // ---- registers -> LDS ----
#pragma unroll
        for (int m = 0; m < NF; ++m) {
            const int i = tid + m * P1T, r = i / (K / 4), c = (i % (K / 4)) * 4;
            const u32x4 kv4 = sizeof(T) == 2 ? u32x4{kreg2[m][0], kreg2[m][1], 0u, 0u} : kreg4[m];
            const float g4[4] = {greg[m].x, greg[m].y, greg[m].z, greg[m].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                ks[r * LD + c + e] = vec_get<T>(kv4, e);
                gs[r * LD + c + e] = g4[e];
            }
        }
        // per-token scalars of this chunk (threads < 64 keep theirs in registers as well)
        const float step = screg.x, p = screg.y, n_raw = screg.z, bet = betreg, ret = retreg, dbeta_in = dbreg;
        const float nn = fmaxf(n_raw, a.eps);
        const float bp = a.beta_aware ? bet : 1.f;
        const float ca = a.eta * bp / nn * bp;
        if (tid < C) { steps[tid] = step; rs[tid] = ret; cas[tid] = ca; sig[tid] = 0.f; casig[tid] = 0.f; }
        float d = 0.f;
        if (tid < K) d = a.d_ckpt[(bh * N + n) * K + tid];
        __syncthreads();
        OSDN_TICK(0)
        float4 rc[NF];                          // read-side dL/dk of this chunk, needed at the end
#pragma unroll
        for (int m = 0; m < NF; ++m) {
            const int i = tid + m * P1T, r = i / (K / 4), c = (i % (K / 4)) * 4;
            rc[m] = *reinterpret_cast<const float4 *>(a.dk_read + (tokc + (size_t)r * a.H) * K + c);
        }
        // ---- replay the chunk forward (same arithmetic as the forward kernel); bit i of the
        //      mask: the unprojected d_{i+1} of this coordinate lies inside the box ----
        uint32_t mlo = 0u, mhi = 0u;
        if (tid < K) {
            float kb[2][PB], sb_[2][PB], rb[2][PB];
#define OSDN_RLOAD(buf, i0_)                                                                     \
    _Pragma("unroll") for (int u = 0; u < PB; ++u) {                                             \
        kb[buf][u] = ks[((i0_) + u) * LD + tid]; sb_[buf][u] = steps[(i0_) + u];                  \
        if (HAS_RET) rb[buf][u] = rs[(i0_) + u];                                                 \
    }
            OSDN_RLOAD(0, 0)
#pragma unroll
            for (int blk = 0; blk < C / PB; ++blk) {
                if (blk + 1 < C / PB) OSDN_RLOAD((blk + 1) & 1, (blk + 1) * PB)
#pragma unroll
                for (int u = 0; u < PB; ++u) {
                    const int i = blk * PB + u;
                    Dt[i * LD + tid] = d;
                    const float kv = kb[blk & 1][u];
                    const float db = d_bar<HAS_RET>(rb[blk & 1][u], d, sb_[blk & 1][u], kv * kv);
                    d = clip3(db, lo, hi);
                    const uint32_t in = (d == db) ? (1u << (i & 31)) : 0u;
                    if (i < 32) mlo |= in; else mhi |= in;
                }
            }
        }
        const bool all_in = __all(mlo == 0xffffffffu && mhi == 0xffffffffu);    // per wave
        // ---- sweeps for sigma_i = <s_i, abar_i> ----
        OSDN_TICK(1)
        float dprev = 0.f;
        int sweeps_used = 0;
        for (int sweep = 0; sweep < P1_MAX_SWEEPS; ++sweep) {
            ++sweeps_used;
            // source term of the adjoint recurrence, all threads: At <- lambda_i - ca_i sigma_i s_i
#pragma unroll
            for (int j = 0; j < C * K / P1T; ++j) {      // consecutive lanes -> consecutive columns
                const int e = tid + j * P1T, r = e / K, x = r * LD + e % K;
                const float kv = ks[x];
                At[x] = __builtin_fmaf(-casig[r] * kv, kv, kv * gs[x]);
            }
            __syncthreads();
            if (tid < K) {
                float av = ga[tid];
                float sb[2][PB], rb[2][PB];
#define OSDN_VLOAD(buf, ih_)                                                                     \
    _Pragma("unroll") for (int u = 0; u < PB; ++u) {                                             \
        sb[buf][u] = At[((ih_) - u) * LD + tid];                                                 \
        if (HAS_RET) rb[buf][u] = rs[(ih_) - u];                                                 \
    }
                OSDN_VLOAD(0, C - 1)
                if (all_in) {       // no coordinate of this wave touched the box in this chunk
#pragma unroll
                    for (int blk = 0; blk < C / PB; ++blk) {
                        const int ih = C - 1 - blk * PB;
                        if (blk + 1 < C / PB) OSDN_VLOAD((blk + 1) & 1, ih - PB)
#pragma unroll
                        for (int u = 0; u < PB; ++u) {
                            At[(ih - u) * LD + tid] = av;
                            av = HAS_RET ? __builtin_fmaf(rb[blk & 1][u], av, sb[blk & 1][u]) : av + sb[blk & 1][u];
                        }
                    }
                } else {
#pragma unroll
                    for (int blk = 0; blk < C / PB; ++blk) {
                        const int ih = C - 1 - blk * PB;
                        if (blk + 1 < C / PB) OSDN_VLOAD((blk + 1) & 1, ih - PB)
#pragma unroll
                        for (int u = 0; u < PB; ++u) {
                            const int i = ih - u;
                            const uint32_t bit = (i < 32 ? mlo : mhi) & (1u << (i & 31));
                            const float ab = bit ? av : 0.f;
                            At[i * LD + tid] = ab;  // the source of token i was fetched a block ahead
                            av = HAS_RET ? __builtin_fmaf(rb[blk & 1][u], ab, sb[blk & 1][u]) : ab + sb[blk & 1][u];
                        }
                    }
                }
                ganew[tid] = av;
            }
            __syncthreads();
            OSDN_TICK(2)
            {
                const int i = lane, q0 = wave * KQ;
                float sp = 0.f;
#pragma unroll 8
                for (int c = 0; c < KQ; ++c) {
                    const float kv = ks[i * LD + q0 + c];
                    sp = __builtin_fmaf(kv * kv, At[i * LD + q0 + c], sp);
                }
                part[wave * C + i] = sp;
            }
            __syncthreads();
            if (tid < C) {
                const int i = tid;
                const float sg = sumw(part, i);
                const float mx = wave_max(fabsf(sg));
                const float dcur = wave_max(fabsf(sg - sig[i]));
                // converged, or (from the second pass on) the observed contraction ratio says
                // that the next difference would be below the tolerance
                const bool all_ok = dcur <= P1_TOL * mx ||
                                    (sweep >= 1 && dcur <= 0.1f * dprev && dcur * dcur <= P1_TOL * mx * dprev);
                dprev = dcur;
                sig[i] = sg;
                casig[i] = cas[i] * sg;
                if (tid == 0) done = all_ok ? 1 : 0;
            }
            __syncthreads();
            OSDN_TICK(3)
            if (done) break;
        }
        // ---- accepted: sig generated At and ganew ----
        if (n > 0) OSDN_P1_BLOAD(n - 1)         // next chunk: in flight during the output phase
        // g_r = <abar_i, d_i> if it is asked for
        if (a.dretention) {
            const int i = lane, q0 = wave * KQ;
            float sp = 0.f;
#pragma unroll 8
            for (int c = 0; c < KQ; ++c) sp = __builtin_fmaf(At[i * LD + q0 + c], Dt[i * LD + q0 + c], sp);
            part2[wave * C + i] = sp;
        }
        // per-token scalars that enter the elementwise outputs: g_p, g_nraw -> part[0..2*64)
        if (tid < C) {
            const float g_c = sig[tid];
            const float g_p = -g_c * ca;
            const float g_nraw = (n_raw >= a.eps) ? -g_c * step / nn : 0.f;
            const float g_bp = g_c * a.eta * (1.f - 2.f * bp * p) / nn;
            part[tid] = g_p;
            part[C + tid] = g_nraw;
            const size_t th = tokc + (size_t)tid * a.H;
            if (a.beta_aware) a.dbeta[th] = dbeta_in + g_bp;
        }
        __syncthreads();
        OSDN_TICK(4)
        if (a.dretention && tid < C) a.dretention[tokc + (size_t)tid * a.H] = sumw(part2, tid);
        // dk = dk_read + d_i . dkt + 2 k (step abar + g_p d_i + g_nraw)
#pragma unroll
        for (int m = 0; m < NF; ++m) {
            const int i = tid + m * P1T, r = i / (K / 4), c = (i % (K / 4)) * 4;
            const size_t off = (tokc + (size_t)r * a.H) * K + c;
            const float rdv[4] = {rc[m].x, rc[m].y, rc[m].z, rc[m].w};
            const float st = steps[r], g_p = part[r], g_nraw = part[C + r];
            float out[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int x = r * LD + c + e;
                const float gsum = st * At[x] + g_p * Dt[x] + g_nraw;
                out[e] = rdv[e] + Dt[x] * gs[x] + 2.f * ks[x] * gsum;
            }
            store_vec(dk + off, out);
        }
        if (tid < K) ga[tid] = ganew[tid];
#ifdef OSDN_DIAG
        if (tid == 0) const_cast<float *>(a.tok_scalars)[(tokc + a.H) * 4 + 3] = (float)sweeps_used;
#endif
        __syncthreads();
        OSDN_TICK(5)
    }
#ifdef OSDN_DIAG
    if (tid == 0 && blockIdx.x == 0)
        for (int j = 0; j < 6; ++j) const_cast<float *>(a.tok_scalars)[(((size_t)b * a.T + 10 + j) * a.H + h) * 4 + 3] = (float)tph[j];
#endif
    if (tid < K) a.dd_in[bh * K + tid] = ga[tid];
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

template <typename T, bool HAS_RET>
static int launch_precond_bwd_t(const PrecondBwdArgs &a, hipStream_t st) {
    dim3 grid(a.B * a.H), block(P1T);
    if (a.K == 64) hipLaunchKernelGGL((precond_bwd_kernel<T, 64, HAS_RET>), grid, block, 0, st, a);
    else if (a.K == 128) hipLaunchKernelGGL((precond_bwd_kernel<T, 128, HAS_RET>), grid, block, 0, st, a);
    else return -1;
    return 0;
}
int launch_precond_bwd(const PrecondBwdArgs &a, bool bf16_io, hipStream_t st) {
    if (a.retention)
        return bf16_io ? launch_precond_bwd_t<bf16, true>(a, st) : launch_precond_bwd_t<float, true>(a, st);
    return bf16_io ? launch_precond_bwd_t<bf16, false>(a, st) : launch_precond_bwd_t<float, false>(a, st);
}

}  // namespace osdn
