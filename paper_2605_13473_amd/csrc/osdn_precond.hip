// Phase 1 of OSDN: the online preconditioner sweep (Algorithm 1, Eq. (dt_update) and its
// retention form Eq. (dt_update_apf)).
//
// The recurrence  d_{t+1} = clip(r_t d_t + c_t s_t),  s_t = k_t (.) k_t,
//                 c_t = eta b'(1 - b' p_t)/n_t,  p_t = <d_t, s_t>
// couples the K coordinates only through the scalar p_t.  One workgroup owns one
// (batch, head) chain and walks it in chunks of 64 tokens.  Inside a chunk it solves for the
// 64 scalars p by fixed-point sweeps: given p (first guess: <d_0, s_t>) the recurrence
// separates into K independent scalar recurrences; from the resulting trajectory the 64 inner
// products are recomputed; the sweep repeats until they reproduce themselves.  Sweep m fixes
// at least the first m tokens exactly, so 64 sweeps always suffice; because the coupling is
// O(eta) two do in practice, also when coordinates sit on a face of the box.
//
// A sweep does not walk the 64 tokens one after the other.  The chunk is cut into 8 runs of
// 8 tokens, one wavefront per run, a lane per coordinate (pair): everything a thread needs of
// the chunk (its k, s, d) stays in registers.  One token maps d to clip(r d + c s), and maps
// of that form compose to x -> clip3(A x + B, L, H) with
//     A' = r A,  B' = r B + c s,  L' = clip(r L + c s),  H' = clip(r H + c s)      (r >= 0),
// so a thread first composes the map of its run, the runs are chained through LDS (one
// fma + median-of-three per run), and with its run's starting value known the thread replays
// its 8 tokens.  The products s d are folded over the lanes of the wavefront and the p of a
// token is the sum of 8 partials.  All arithmetic is fp32; k~ is rounded once, from fp32 d k.
//
// For few long chains the same composition is taken one level up: the chain is cut into pieces,
// one workgroup per piece walks its chunks from a start value it is given and also composes the
// accepted run maps into one map for the piece; the next sweep carries the chain's start value
// through those maps to get its start values, and the sweeps over all pieces repeat until no
// start value of a chain moves (the caller launches them ahead of time; the workgroups of a
// settled chain return at once).
#include "osdn_precond.h"

#include <cfloat>

namespace osdn {

constexpr int RUN = 8;                           // tokens per run; C / RUN runs = wavefronts

// CPT adjacent elements of type T <-> floats, as one memory access
template <typename T, int CPT> struct Pack;
template <> struct Pack<bf16, 2> {
    typedef uint32_t Raw;
    static __device__ __forceinline__ void unpack(Raw w, float (&o)[2]) {
        o[0] = __builtin_bit_cast(float, w << 16);
        o[1] = __builtin_bit_cast(float, w & 0xffff0000u);
    }
    static __device__ __forceinline__ Raw pack(const float (&v)[2]) {
        const uint32_t lo = __builtin_bit_cast(unsigned short, (bf16)v[0]);
        const uint32_t hi = __builtin_bit_cast(unsigned short, (bf16)v[1]);
        return lo | (hi << 16);
    }
};
template <> struct Pack<bf16, 1> {
    typedef bf16 Raw;
    static __device__ __forceinline__ void unpack(Raw w, float (&o)[1]) { o[0] = (float)w; }
    static __device__ __forceinline__ Raw pack(const float (&v)[1]) { return (bf16)v[0]; }
};
template <> struct Pack<float, 2> {
    typedef float2 Raw;
    static __device__ __forceinline__ void unpack(Raw w, float (&o)[2]) { o[0] = w.x; o[1] = w.y; }
    static __device__ __forceinline__ Raw pack(const float (&v)[2]) { return make_float2(v[0], v[1]); }
};
template <> struct Pack<float, 1> {
    typedef float Raw;
    static __device__ __forceinline__ void unpack(Raw w, float (&o)[1]) { o[0] = w; }
    static __device__ __forceinline__ Raw pack(const float (&v)[1]) { return v[0]; }
};

// RET: 0 = no retention, 1 = one gate per (token, head), 2 = one per coordinate (diag(r_t))
// PIECES: one workgroup per piece of a chain (sweeps over the whole sequence) instead of one per chain
template <typename T, int K, int RET, bool PIECES>
__global__ __launch_bounds__(P1T) void precond_fwd_kernel(PrecondArgs a) {
    constexpr bool HAS_RET = RET != 0, RET_VEC = RET == 2;
    constexpr int RE = RET_VEC ? K / 64 : 1;      // retention values a thread keeps per token
    constexpr int CPT = K / 64;                   // coordinates per thread (adjacent)
    constexpr int NRUN = C / RUN;                 // = wavefronts of the workgroup
    static_assert(NRUN == P1W && RUN == 8, "one wavefront per run of 8 tokens");
    typedef Pack<T, CPT> Pk;
    __shared__ float dcur[K];                    // d at the start of the chunk
    // (A, B, L, H) per run and coordinate, [run][e][lane] for coordinate lane * CPT + e: the 16-byte
    // accesses of adjacent lanes are then adjacent (a lane's own coordinates 32 bytes apart made
    // every such access a two-way bank conflict)
    __shared__ __attribute__((aligned(16))) float4 maps[NRUN * K];
    __shared__ int okflag[NRUN];

    const int tid = threadIdx.x, run = tid >> 6, lane = tid & 63;
    const int c0 = lane * CPT;                    // first coordinate of this thread
    const int u_own = lane & (RUN - 1);           // the token of the run whose scalars this lane keeps
    const int piece = PIECES ? blockIdx.x % a.pieces : 0;
    const int chain = PIECES ? blockIdx.x / a.pieces : blockIdx.x;
    const int b = chain / a.H, h = chain % a.H;               // b: batch entry, or packed sequence
    if (a.settled && !(PIECES && a.sweep == 0) && a.settled[chain]) return;
    if (PIECES) {
        a.n0 += piece * a.piece_chunks;
        a.n1 = min(a.n1, a.n0 + a.piece_chunks);
        if (a.n0 >= a.n1) return;
    }
    const size_t bh = (size_t)b * a.H + h;                    // the chain: indexes d_in / d_out
    int bt = b;                                               // batch entry of the token tensors
    if (a.seq_chunks) {
        bool begins, ends;
        if (!clip_to_sequence(a.seq_chunks, b, a.n0, a.n1, begins, ends)) return;
        a.d_in = begins ? a.d_first : a.d_out;
        bt = 0;
    }
    const size_t bth = (size_t)bt * a.H + h;                  // indexes the per-chunk buffers
    const bool project = a.d_min <= a.d_max;
    const float lo = project ? a.d_min : -INFINITY, hi = project ? a.d_max : INFINITY;
    const int N = (a.T + C - 1) / C;
    const uint32_t kstride = (uint32_t)a.H * K;   // elements between consecutive tokens

    if (!PIECES) {
        if (tid < K) dcur[tid] = a.d_in ? a.d_in[bh * K + tid] : 1.f;
    } else {
        // The start value of this piece: the chain's own start value carried through the maps
        // that the previous sweep left for the pieces before this one (first sweep: the chain's
        // start value itself, as a guess).  Every workgroup of the chain walks all its pieces and
        // so sees whether any start value moved by more than the tolerance of the sweeps; if
        // none did, what the previous sweep wrote stands and the chain is settled.
        const size_t buf = (size_t)gridDim.x * K;                 // elements of one buffer
        const size_t cur = (a.sweep & 1) * buf, prev = buf - cur;
        float x = 1.f, xs = 1.f;
        bool moved = a.sweep == 0;
        if (tid < K) {
            x = xs = a.d_in ? a.d_in[bh * K + tid] : 1.f;
            if (a.sweep > 0)
                for (int q = 0; q < a.pieces; ++q) {
                    const size_t i = (bh * a.pieces + q) * K + tid;
                    const float old = a.piece_start[prev + i];
                    if (q == piece) xs = x;
                    if (!(fabsf(x - old) <= P1_TOL * fmaxf(fabsf(x), fabsf(old)))) moved = true;
                    const float4 m = a.piece_map[prev + i];
                    x = clip3(__builtin_fmaf(m.x, x, m.y), m.z, m.w);
                }
        }
        const bool any = __syncthreads_or(moved);
        if (piece == 0 && tid == 0) a.settled[chain] = any ? 0 : 1;
        if (!any) return;
        if (tid < K) {
            dcur[tid] = xs;
            a.piece_start[cur + (bh * a.pieces + piece) * K + tid] = xs;
        }
        a.piece_map += cur;
    }
    float PA = 1.f, PB = 0.f, PL = -FLT_MAX, PH = FLT_MAX;    // thread c < K: the piece so far, as a map of coordinate c

    typedef Pack<float, CPT> Pr;
    typename Pk::Raw kreg[RUN];                  // this thread's k of the next chunk
    typename Pr::Raw rreg[RET_VEC ? RUN : 1];    // ... and its per-coordinate retention
    float betreg = 0.f, retreg = 1.f;            // gates of token (run, u_own) of the next chunk
#define OSDN_P1_LOAD(n_)                                                                         \
    {                                                                                            \
        const int t0_ = (n_) * C;                                                                \
        const T *kp_ = static_cast<const T *>(a.k) + (((size_t)bt * a.T + t0_) * a.H + h) * K;   \
        _Pragma("unroll") for (int u = 0; u < RUN; ++u) {                                        \
            const int i_ = min(run * RUN + u, a.T - 1 - t0_);    /* rows past the end: reread */ \
            kreg[u] = *reinterpret_cast<const typename Pk::Raw *>(kp_ + (uint32_t)i_ * kstride + c0); \
            if (RET_VEC)                                                                         \
                rreg[u] = *reinterpret_cast<const typename Pr::Raw *>(                           \
                    a.retention + (((size_t)bt * a.T + t0_) * a.H + h) * K + (uint32_t)i_ * kstride + c0); \
        }                                                                                        \
        const int t = min(t0_ + run * RUN + u_own, a.T - 1);                                     \
        const size_t th = ((size_t)bt * a.T + t) * a.H + h;                                      \
        betreg = a.beta[th];                                                                     \
        if (HAS_RET && !RET_VEC) retreg = a.retention[th];                                       \
    }
    OSDN_P1_LOAD(a.n0)

    __syncthreads();
    for (int n = a.n0; n < a.n1; ++n) {
        const int t0 = n * C;
        const int nvalid = min(C, a.T - t0);
        // ---- this thread's k and s = k^2 (rows past the end of the sequence: no-op tokens) ----
        float kf[RUN][CPT], sv[RUN][CPT];
#pragma unroll
        for (int u = 0; u < RUN; ++u) {
            Pk::unpack(kreg[u], kf[u]);
#pragma unroll
            for (int e = 0; e < CPT; ++e) {
                if (run * RUN + u >= nvalid) kf[u][e] = 0.f;
                sv[u][e] = kf[u][e] * kf[u][e];
            }
        }
        const float bet = betreg, ret = retreg;
        // ---- the scalars of token (run, u_own): n_raw = sum s, first guess p = <d_0, s> ----
        float nraw, cb, ca, p_cur, c_cur;
        {
            float dst[CPT];
#pragma unroll
            for (int e = 0; e < CPT; ++e) dst[e] = dcur[c0 + e];
            if (a.d_ckpt && run == 0) {
#pragma unroll
                for (int e = 0; e < CPT; ++e) a.d_ckpt[(bth * N + n) * K + c0 + e] = dst[e];
            }
            float vn[RUN], vp[RUN];
#pragma unroll
            for (int u = 0; u < RUN; ++u) {
                vn[u] = 0.f; vp[u] = 0.f;
#pragma unroll
                for (int e = 0; e < CPT; ++e) { vn[u] += sv[u][e]; vp[u] = __builtin_fmaf(sv[u][e], dst[e], vp[u]); }
            }
            nraw = lane_fold8_all(vn, lane);
            p_cur = lane_fold8_all(vp, lane);
            const bool valid = run * RUN + u_own < nvalid;
            const float nn = fmaxf(nraw, a.eps);
            const float bp = a.beta_aware ? bet : 1.f;
            cb = valid ? a.eta * bp / nn : 0.f;
            ca = cb * bp;
            c_cur = cb - ca * p_cur;
        }
        float rv[RUN][RE];                      // retention of this thread's coordinates (no-op tokens: 1)
#pragma unroll
        for (int u = 0; u < RUN; ++u) {
            if (RET_VEC) {
                float r2[CPT];
                Pr::unpack(rreg[RET_VEC ? u : 0], r2);
#pragma unroll
                for (int e = 0; e < RE; ++e) rv[u][e] = run * RUN + u < nvalid ? r2[e] : 1.f;
            } else {
                rv[u][0] = HAS_RET ? lane_bcast(run * RUN + u < nvalid ? ret : 1.f, u) : 1.f;
            }
        }
        if (n + 1 < a.n1) OSDN_P1_LOAD(n + 1)
        // ---- fixed-point sweeps ----
        int sweeps_used = 0;
        float dtr[RUN][CPT], dend[CPT];
        for (int sweep = 0; sweep < P1_MAX_SWEEPS; ++sweep) {
            ++sweeps_used;
            float cv[RUN];
#pragma unroll
            for (int u = 0; u < RUN; ++u) cv[u] = lane_bcast(c_cur, u);
            // the map of this run, x -> clip3(A x + B, L, H), per coordinate
#pragma unroll
            for (int e = 0; e < CPT; ++e) {
                float A = 1.f, B = 0.f, L = -FLT_MAX, H = FLT_MAX;
#pragma unroll
                for (int u = 0; u < RUN; ++u) {
                    const float bs = cv[u] * sv[u][e];
                    if (HAS_RET) {
                        const float r = rv[u][RET_VEC ? e : 0];
                        A *= r;
                        B = __builtin_fmaf(r, B, bs);
                        L = clip3(__builtin_fmaf(r, L, bs), lo, hi);
                        H = clip3(__builtin_fmaf(r, H, bs), lo, hi);
                    } else {
                        B += bs;
                        L = clip3(L + bs, lo, hi);
                        H = clip3(H + bs, lo, hi);
                    }
                }
                maps[(run * CPT + e) * 64 + lane] = make_float4(A, B, L, H);
            }
            __syncthreads();
            float vp[RUN];
#pragma unroll
            for (int u = 0; u < RUN; ++u) vp[u] = 0.f;
#pragma unroll
            for (int e = 0; e < CPT; ++e) {
                // d at the start of this run: the runs to its left applied to d at the chunk start
                float d = dcur[c0 + e];
#pragma unroll
                for (int j = 0; j < NRUN - 1; ++j)
                    if (j < run) {
                        const float4 m = maps[(j * CPT + e) * 64 + lane];
                        d = clip3(__builtin_fmaf(m.x, d, m.y), m.z, m.w);
                    }
                // replay of the run's tokens (the same arithmetic as the reverse sweep's replay)
#pragma unroll
                for (int u = 0; u < RUN; ++u) {
                    dtr[u][e] = d;
                    vp[u] = __builtin_fmaf(sv[u][e], d, vp[u]);
                    d = clip3(d_bar<HAS_RET>(rv[u][RET_VEC ? e : 0], d, cv[u], sv[u][e]), lo, hi);
                }
                dend[e] = d;
            }
            const float p_new = lane_fold8_all(vp, lane);
            const bool ok = fabsf(p_new - p_cur) <= P1_TOL * fabsf(p_new);
            const bool wave_ok = __all(ok);
            if (lane == 0) okflag[run] = wave_ok ? 1 : 0;
            __syncthreads();
            bool all_ok = true;
#pragma unroll
            for (int w = 0; w < NRUN; ++w) all_ok = all_ok && okflag[w] != 0;
            if (all_ok) break;
            p_cur = p_new;
            c_cur = cb - ca * p_new;
        }
        // ---- accepted: (c_cur, p_cur) generated dtr and dend ----
        {
            T *ktp = static_cast<T *>(a.k_tilde) + (((size_t)bt * a.T + t0) * a.H + h) * K;
#pragma unroll
            for (int u = 0; u < RUN; ++u) {
                const int i = run * RUN + u;
                if (i < nvalid) {
                    float out[CPT];
#pragma unroll
                    for (int e = 0; e < CPT; ++e) out[e] = dtr[u][e] * kf[u][e];
                    *reinterpret_cast<typename Pk::Raw *>(ktp + (uint32_t)i * kstride + c0) = Pk::pack(out);
                }
            }
        }
        if (a.tok_scalars && lane < RUN && run * RUN + lane < nvalid) {
            const size_t th = ((size_t)bt * a.T + t0 + run * RUN + lane) * a.H + h;
            *reinterpret_cast<float4 *>(a.tok_scalars + th * 4) = make_float4(c_cur, p_cur, nraw, (float)sweeps_used);
        }
        if (run == NRUN - 1) {
#pragma unroll
            for (int e = 0; e < CPT; ++e) dcur[c0 + e] = dend[e];
        }
        if (PIECES && tid < K) {                 // the accepted run maps, applied after the piece so far
#pragma unroll
            for (int j = 0; j < NRUN; ++j) {
                const float4 m = maps[(j * CPT + tid % CPT) * 64 + tid / CPT];
                PA *= m.x;
                PB = __builtin_fmaf(m.x, PB, m.y);
                PL = clip3(__builtin_fmaf(m.x, PL, m.y), m.z, m.w);
                PH = clip3(__builtin_fmaf(m.x, PH, m.y), m.z, m.w);
            }
        }
        __syncthreads();
    }
    if (PIECES && tid < K) a.piece_map[(bh * a.pieces + piece) * K + tid] = make_float4(PA, PB, PL, PH);
    if (tid < K && (!PIECES || piece == a.pieces - 1)) a.d_out[bh * K + tid] = dcur[tid];
}

template <typename T, int RET, bool PIECES>
static int launch_precond_fwd_tp(const PrecondArgs &a, hipStream_t st) {
    dim3 grid((a.seq_chunks ? a.n_seqs : a.B) * a.H * (PIECES ? a.pieces : 1)), block(P1T);
    if (a.K == 64) hipLaunchKernelGGL((precond_fwd_kernel<T, 64, RET, PIECES>), grid, block, 0, st, a);
    else if (a.K == 128) hipLaunchKernelGGL((precond_fwd_kernel<T, 128, RET, PIECES>), grid, block, 0, st, a);
    else return -1;
    return 0;
}
template <typename T, int RET>
static int launch_precond_fwd_t(const PrecondArgs &a, hipStream_t st) {
    return a.pieces ? launch_precond_fwd_tp<T, RET, true>(a, st) : launch_precond_fwd_tp<T, RET, false>(a, st);
}
int launch_precond_fwd(const PrecondArgs &a, bool bf16_io, hipStream_t st) {
    const int ret = a.retention ? (a.ret_vec ? 2 : 1) : 0;
    if (ret == 2) return bf16_io ? launch_precond_fwd_t<bf16, 2>(a, st) : launch_precond_fwd_t<float, 2>(a, st);
    if (ret == 1) return bf16_io ? launch_precond_fwd_t<bf16, 1>(a, st) : launch_precond_fwd_t<float, 1>(a, st);
    return bf16_io ? launch_precond_fwd_t<bf16, 0>(a, st) : launch_precond_fwd_t<float, 0>(a, st);
}

}  // namespace osdn
