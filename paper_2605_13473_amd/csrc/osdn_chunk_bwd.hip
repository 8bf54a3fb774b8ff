// Phase 2 backward of OSDN in chunkwise form.  The paper prints only the chain rule through
// k~ = d . k (Section 4.5); the chunk-level adjoints below are plain matrix calculus on the
// forward formulas (Appendix A.2 / B.1), per chunk, with S the state at the start of the
// chunk, dS' the adjoint of the state at its end, G the in-chunk cumulative log-decay,
// gamma = e^G, rho = e^{G_C - G}, Gamma_ij = e^{G_i - G_j}:
//
//   forward:  A = tril(beta_i Gamma_ij <k_i,k~_j>, -1), T = (I+A)^-1, R0 = V - gamma.(K S^T),
//             E = T (beta . R0), P = tril(Gamma . Q K~^T), O = scale[gamma.(Q S^T) + P E],
//             S' = gamma_C S + E^T (rho . K~)
//   bwd_chain (sequential, right to left, per (b, h, slice of V)):
//             dE = scale P^T dO + (rho . K~) dS'^T ;  dS = gamma_C dS' + scale dO^T (gamma . Q) - dE^T W
//             (P is the tile output_fwd left; q and dO are read where the caller put them)
//   bwd_post  (parallel):  dR = T^T dE ; dV = beta . dR ; dA = -tril(dR E^T, -1) ;
//             dP = scale tril(dO E^T) ; cA = dA . beta_i Gamma ; cP = dP . Gamma ;
//             dQ = cP K~ + scale gamma . (dO S) ; dK = cA K~ - gamma beta . (dR S) ;
//             dK~ = cA^T K + cP^T Q + rho . (E dS') ;
//             dbeta_i = <dR_i, R0_i> + sum_j dA_ij Gamma_ij <k_i,k~_j> ;
//             dG from every place G enters; dlog_alpha = suffix sums of dG inside the chunk.
//
// With one state gate per key channel (GV) the same kernels run, ungated, on the operands in
// which the forward pass folded the channel decays (Gamma . Q, Gamma . K, K~ / Gamma); the
// state adjoint decays per channel between chunks, the write rows carry the chunk's decay per
// channel in place of rho, and the unfold kernel at the end of this file maps the gradients
// back to q, k, k~ and log alpha.
#include "osdn_kernels.h"

namespace osdn {


// sum over the 16 lanes of a DPP row (lanes sharing lane>>4), returned to all of them
__device__ __forceinline__ float row16_sum(float x) {
    x += dpp_f32<0xB1>(x);
    x += dpp_f32<0x4E>(x);
    x += dpp_f32<0x141>(x);
    x += dpp_f32<0x140>(x);
    return x;
}

// a one-value (fp32) MFMA fragment times a scalar; the 8-value bf16 fragments are never scaled
__device__ __forceinline__ float scale_frag(float f, float s) { return f * s; }
__device__ __forceinline__ bf16x8 scale_frag(bf16x8 f, float) { return f; }

// ------------------------------------------------------------- bwd_chain ----
// Mirror image of state_fwd, right to left: wavefronts 0-3 carry dS (transposed, fp32, in
// MFMA accumulators), wavefronts 4-7 bring the next chunk's operand tiles into the other LDS
// buffer and write the dS' checkpoint and dE^T back.  The operands come as the forward pass and
// the caller left them: (rho . K~)^T and -W^T from chunk_prep, P from output_fwd, q and the
// slice of dO in their natural [token][feature] layout (operands whose contraction index runs
// along the rows are fetched with the LDS transpose read), so no kernel has to run ahead of this
// one.  The local part of dE, scale P^T dO, is formed here as well.  The loader wavefronts move
// the three [64 x K] tiles; the small ones (P, the slice of dO) are fetched by the compute
// wavefronts themselves, a chunk ahead, into registers they have to spare.
constexpr int CT_ = 512, CL_ = 256;

// GV: one state gate per key channel (the chunk's decay per channel comes from chunk_prep).
// VS: rows of S (values) owned by one workgroup, 32 or 16 (the narrow slice when the chains are few:
// twice the workgroups, each with half the work on the dependent path per chunk).
template <typename T, int K, bool GV, int VS>
__global__ __launch_bounds__(CT_) void bwd_chain_kernel(ChunkArgs a) {
    constexpr int NVT = VS / 16;                    // value tiles per compute wave
    constexpr int PAD = Pad<T>::v, LDK = K + PAD, LDC = C + PAD, LDS_ = VS + PAD;
    constexpr int VN = 16 / sizeof(T);
    constexpr int NKT = K / 64;
    constexpr int KS = Mfma<T>::KSTEP;
    constexpr bool BF = sizeof(T) == 2;
    constexpr int NB = BF ? 2 : 1;
    constexpr int LTN = NB == 2 ? CL_ / 2 : CL_;    // two loader groups (one per chunk parity) when double-buffered
    constexpr int NWV = C * K / VN / LTN;           // vectors per loader thread: a [64 x K] or [K x 64] tile
    constexpr int NCW = CT_ - CL_;                  // compute threads
    constexpr int NPV = C * C / VN / NCW;           // vectors per compute thread: the [64 x 64] tile P
    constexpr int NOV = C * VS / VN;                // vectors of the [64 x VS] slice of dO
    constexpr int NUV = (NOV + NCW - 1) / NCW;      // ... per compute thread (NOV < NCW: the upper threads repeat the lower ones' vectors)
    static_assert(C * K / VN % LTN == 0 && (NOV % NCW == 0 || NCW % NOV == 0) && C * C / VN % NCW == 0, "tiles must split evenly");
    __shared__ __attribute__((aligned(16))) T Krt[NB][K * LDC];     // (rho . K~)^T   [kf][i], as chunk_prep left it
    __shared__ __attribute__((aligned(16))) T Wtt[NB][K * LDC];     // -W^T           [kf][i]
    __shared__ __attribute__((aligned(16))) T Qn[NB][C * LDK];      // q              [i][kf]
    __shared__ __attribute__((aligned(16))) T Pn[NB][C * LDC];      // P              [i][j]
    __shared__ __attribute__((aligned(16))) T dOn[NB][C * LDS_];    // dO slice       [i][v]
    __shared__ __attribute__((aligned(16))) T dOg[BF ? NB : 1][BF ? C * LDS_ : 1];   // scale gamma_i dO (bf16: a tile of its own)
    __shared__ __attribute__((aligned(16))) T dSb[VS * LDK];        // dS' in the I/O type [v][kf]
    __shared__ __attribute__((aligned(16))) T dEt[VS * LDC];        // dE^T [v][i]
    __shared__ float gCs[NB];
    __shared__ float sgam[NB][C];                                   // scale gamma_i

    int chain, slice;
    chain_slice_of(blockIdx.x, a.V / VS, (a.seq_chunks ? a.n_seqs : a.B) * a.H, chain, slice);
    const int vs = slice * VS, h = chain % a.H, b = chain / a.H;   // b: batch entry, or packed sequence
    int bt = b;                                 // batch entry of the token tensors
    if (a.seq_chunks) {
        bool begins, ends;
        if (!clip_to_sequence(a.seq_chunks, b, a.n0, a.n1, begins, ends)) return;
        a.dS_out = ends ? a.dS_last : a.dS_in;
        bt = 0;
    }
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const bool loader = wave >= 4;
    const int lt = tid - CL_;
    const int lgrp = NB == 2 ? (lt >> 7) & 1 : 0;
    const int lti = NB == 2 ? lt & 127 : lt;
    const size_t bh = (size_t)b * a.H + h;      // the chain: indexes dS_out / dS_in
    const size_t bth = (size_t)bt * a.H + h;    // indexes the per-chunk buffers
    const size_t tstride = a.H;

    f32x4 dSt[NVT][NKT];                  // rows = features, cols = values
    if (!loader) {
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
            for (int q = 0; q < NKT; ++q) {
                const int v = vs + vt * 16 + acc_col(lane), c0 = (wave * NKT + q) * 16 + acc_row(lane, 0);
                if (a.dS_out) dSt[vt][q] = *reinterpret_cast<const f32x4 *>(a.dS_out + (bh * a.V + v) * K + c0);
                else dSt[vt][q] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
    }
    u32x4 kreg[NWV], wreg[NWV], qreg[NWV];          // loaders
    u32x4 preg[NPV], oreg[NUV];                     // compute wavefronts
    float greg = 0.f;
#define OSDN_BC_LOAD(n_)                                                                         \
    {                                                                                            \
        const size_t bhn_ = bth * a.N + (n_);                                                    \
        const size_t tok_ = ((size_t)bt * a.T + (size_t)(n_) * C) * a.H + h;                     \
        const T *kg = static_cast<const T *>(a.Ktr) + bhn_ * K * C;                              \
        const T *wg = static_cast<const T *>(a.Wt) + bhn_ * K * C;                               \
        const T *qg = static_cast<const T *>(a.q) + tok_ * K;                                    \
        _Pragma("unroll") for (int m = 0; m < NWV; ++m) {                                        \
            const int i = lti + m * LTN;                                                          \
            kreg[m] = *reinterpret_cast<const u32x4 *>(kg + (size_t)i * VN);                     \
            wreg[m] = *reinterpret_cast<const u32x4 *>(wg + (size_t)i * VN);                     \
            qreg[m] = *tile_vec(qg, tstride * K, i / (K / VN), (i % (K / VN)) * VN);             \
        }                                                                                        \
        greg = a.log_alpha ? a.log_alpha[tok_ + (size_t)lane * tstride] : 0.f;                   \
    }
#define OSDN_BC_STORE(buf_)                                                                      \
    {                                                                                            \
        const float G_ = wave_cumsum(greg, lane);                                                \
        const float GC_ = __shfl(G_, 63, 64);                                                    \
        const float sg_ = a.scale * __expf(G_);              /* scale gamma of token `lane` */   \
        _Pragma("unroll") for (int m = 0; m < NWV; ++m) {                                        \
            const int i = lti + m * LTN;                                                          \
            { const int r = i / (C / VN), c = (i % (C / VN)) * VN;                               \
              *reinterpret_cast<u32x4 *>(&Krt[buf_][r * LDC + c]) = kreg[m];                     \
              *reinterpret_cast<u32x4 *>(&Wtt[buf_][r * LDC + c]) = wreg[m]; }                   \
            { const int r = i / (K / VN), c = (i % (K / VN)) * VN;                               \
              *reinterpret_cast<u32x4 *>(&Qn[buf_][r * LDK + c]) = qreg[m]; }                    \
        }                                                                                        \
        if (lti < C) sgam[buf_][lti] = sg_;              /* (the first wave of the group: lane = lti) */ \
        if (lti == 0) gCs[buf_] = __expf(GC_);                                                   \
    }
    // the compute wavefronts' own operands: P and the slice of dO of chunk n_ into registers, and
    // from there into the LDS buffer of that chunk (bf16: also dO with its rows scaled by scale gamma)
#define OSDN_BC_CLOAD(n_)                                                                        \
    {                                                                                            \
        const size_t bhn_ = bth * a.N + (n_);                                                    \
        const size_t tok_ = ((size_t)bt * a.T + (size_t)(n_) * C) * a.H + h;                     \
        const T *pg = static_cast<const T *>(a.Pm) + bhn_ * C * C;                               \
        const T *og = static_cast<const T *>(a.dO) + tok_ * a.V + vs;                            \
        _Pragma("unroll") for (int m = 0; m < NPV; ++m)                                          \
            preg[m] = *reinterpret_cast<const u32x4 *>(pg + (size_t)(tid + m * NCW) * VN);       \
        _Pragma("unroll") for (int m = 0; m < NUV; ++m) {                                        \
            const int i = (tid + m * NCW) % NOV;                                                  \
            oreg[m] = *tile_vec(og, tstride * a.V, i / (VS / VN), (i % (VS / VN)) * VN);         \
        }                                                                                        \
    }
#define OSDN_BC_CSTORE(buf_)                                                                     \
    {                                                                                            \
        _Pragma("unroll") for (int m = 0; m < NPV; ++m) {                                        \
            const int i = tid + m * NCW, r = i / (C / VN), c = (i % (C / VN)) * VN;               \
            *reinterpret_cast<u32x4 *>(&Pn[buf_][r * LDC + c]) = preg[m];                        \
        }                                                                                        \
        _Pragma("unroll") for (int m = 0; m < NUV; ++m) {                                        \
            const int i = (tid + m * NCW) % NOV, r = i / (VS / VN), c = (i % (VS / VN)) * VN;     \
            *reinterpret_cast<u32x4 *>(&dOn[buf_][r * LDS_ + c]) = oreg[m];                      \
            if (BF) {                                                                            \
                const float f_ = sgam[buf_][r];                                                  \
                float o_[VN];                                                                    \
                _Pragma("unroll") for (int e = 0; e < VN; ++e) o_[e] = f_ * vec_get<T>(oreg[m], e); \
                store_vec_t(&dOg[BF ? buf_ : 0][BF ? r * LDS_ + c : 0], o_);                     \
            }                                                                                    \
        }                                                                                        \
    }
    if (!loader) OSDN_BC_CLOAD(a.n1 - 1)
    if (loader) {
        if (NB == 2) {
            if (lgrp == ((a.n1 - 1) & 1)) {
                OSDN_BC_LOAD(a.n1 - 1)
                OSDN_BC_STORE((a.n1 - 1) & 1)
                OSDN_BC_LOAD(max(a.n1 - 3, a.n0))
            } else {
                OSDN_BC_LOAD(max(a.n1 - 2, a.n0))
            }
        } else {
            OSDN_BC_LOAD(a.n1 - 1)
            OSDN_BC_STORE(0)
            OSDN_BC_LOAD(max(a.n1 - 2, a.n0))
        }
    }

    __syncthreads();                    // (scale gamma of the first chunk is in LDS)
    if (!loader) {
        OSDN_BC_CSTORE(NB == 2 ? (a.n1 - 1) & 1 : 0)
        OSDN_BC_CLOAD(max(a.n1 - 2, a.n0))
    }

    for (int n = a.n1 - 1; n >= a.n0; --n) {
        const int buf = NB == 2 ? (n & 1) : 0;
        const size_t bhn = bth * a.N + n;
        // ---- phase A (compute): dS', rounded, into LDS ----
        f32x4 gch[GV ? NKT : 1];                                    // channel decays of this lane's state rows
        if (!loader) {
#pragma unroll
            for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
                for (int q = 0; q < NKT; ++q)
                    store_tile_t(dSb + vt * 16 * LDK + (wave * NKT + q) * 16, LDK, dSt[vt][q], lane);
            if (GV) {
#pragma unroll
                for (int q = 0; q < NKT; ++q)
                    gch[GV ? q : 0] = *reinterpret_cast<const f32x4 *>(
                        a.gamC + bhn * K + (wave * NKT + q) * 16 + acc_row(lane, 0));
            }
        }
        __syncthreads();                                            // barrier 1
        if (loader) {
            if (NB == 2) {
                if (lgrp == ((n + 1) & 1)) {                        // this group's chunk (n - 1) comes next
                    if (n > a.n0) {
                        OSDN_BC_STORE((n - 1) & 1)
                        OSDN_BC_LOAD(max(n - 3, a.n0))              // (past the start: a harmless reload)
                    }
                } else {
                    store_tile_global(static_cast<T *>(a.dS_ckpt) + (bhn * a.V + vs) * K, (size_t)K, dSb, LDK, VS, K, lti, LTN);
                }
            } else {
                store_tile_global(static_cast<T *>(a.dS_ckpt) + (bhn * a.V + vs) * K, (size_t)K, dSb, LDK, VS, K, lt, CL_);
            }
        } else {
            // ---- phase B: dE = scale P^T dO + (rho . K~) dS'^T (rows 16*wave ..), kept transposed ----
            const int k0 = (wave * 16) / KS * KS;                   // P[i'][i] = 0 for i' < i
#pragma unroll
            for (int vt = 0; vt < NVT; ++vt) {
                f32x4 acc = mma_tile0<T, false, true>(&Krt[buf][wave * 16], LDC, dSb + vt * 16 * LDK, LDK, K, lane);
                const f32x4 loc = mma_tile0<T, false, false>(&Pn[buf][k0 * LDC + wave * 16], LDC,
                                                             &dOn[buf][k0 * LDS_ + vt * 16], LDS_, C - k0, lane);
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[r] = __builtin_fmaf(a.scale, loc[r], acc[r]);
                store_tile_t(dEt + vt * 16 * LDC + wave * 16, LDC, acc, lane);
            }
        }
        __syncthreads();                                            // barrier 2
        if (loader) {
            if (NB == 2) {
                if (lgrp == ((n + 1) & 1))                          // the group with no load wait ahead
                    store_tile_global(static_cast<T *>(a.dEt) + (bhn * a.V + vs) * C, (size_t)C, dEt, LDC, VS, C, lti, LTN);
            } else {
                store_tile_global(static_cast<T *>(a.dEt) + (bhn * a.V + vs) * C, (size_t)C, dEt, LDC, VS, C, lt, CL_);
            }
        } else {
            // ---- phase C: dS <- gamma_C dS' + (scale gamma . dO)^T Q - dE^T W, transposed ----
            const float gC = gCs[buf];
#pragma unroll
            for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
                for (int q = 0; q < NKT; ++q) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) dSt[vt][q][r] *= GV ? gch[GV ? q : 0][r] : gC;
                    const int ct = (wave * NKT + q) * 16;
                    if (BF) {
                        mma_tile<T, false, false>(dSt[vt][q], &Qn[buf][ct], LDK, &dOg[BF ? buf : 0][BF ? vt * 16 : 0], LDS_, C, lane);
                    } else {
                        // fp32: one value per lane and operand, scaled on the way (no second tile)
                        for (int kk = 0; kk < C; kk += KS) {
                            typename Mfma<T>::Frag fa = Mfma<T>::template load<false>(&Qn[buf][kk * LDK + ct], LDK, lane);
                            typename Mfma<T>::Frag fb = Mfma<T>::template load<false>(&dOn[buf][kk * LDS_ + vt * 16], LDS_, lane);
                            fb = scale_frag(fb, sgam[buf][kk + (lane >> 4)]);
                            dSt[vt][q] = Mfma<T>::mma(fa, fb, dSt[vt][q]);
                        }
                    }
                    mma_tile<T, true, true>(dSt[vt][q], &Wtt[buf][ct * LDC], LDC, dEt + vt * 16 * LDC, LDC, C, lane);
                }
        }
        if (NB == 1) __syncthreads();                               // single buffer: everyone is through with it
        if (n > a.n0) {
            if (NB == 1 && loader) {
                OSDN_BC_STORE(0)
                OSDN_BC_LOAD(max(n - 2, a.n0))
            }
            if (!loader) {
                // the next chunk's small tiles into its buffer (free since barrier 1 of this chunk;
                // its scale gamma table was written before barrier 2), then the request for the one after
                OSDN_BC_CSTORE(NB == 2 ? (n - 1) & 1 : 0)
                OSDN_BC_CLOAD(max(n - 2, a.n0))
            }
        }
    }
    if (!loader) {
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
            for (int q = 0; q < NKT; ++q) {
                const int v = vs + vt * 16 + acc_col(lane), c0 = (wave * NKT + q) * 16 + acc_row(lane, 0);
                *reinterpret_cast<f32x4 *>(a.dS_in + (bh * a.V + v) * K + c0) = dSt[vt][q];
            }
    }
}

// -------------------------------------------------------------- bwd_post ----
// One workgroup of 8 wavefronts per chunk and head (two per SIMD, so that LDS and MFMA
// latencies of one overlap with the other's issue).  V is walked in slabs of VB columns; the
// slab buffers are reused for Q and K~ once the walk is over.
// PW_ wavefronts per workgroup (a parameter of the work split below; 8 is what is launched).

// GV: one state gate per key channel.  The kernel then runs on the folded operands with no
// scalar gate (log_alpha null); the write rows carry the chunk's decay per channel instead of
// rho, and dL/d(that decay) is collected per channel.
template <typename T, int K, bool GV, int PW_, bool PAIR>
__global__ __launch_bounds__(PW_ * 64) void bwd_post_kernel(ChunkArgs a) {
    constexpr int PT_ = PW_ * 64;
    constexpr int PAD = sizeof(T) == 2 ? 16 : Pad<T>::v, LDK = K + PAD, LDC = C + PAD;   // bf16: rows 32 bytes apart modulo 128
    constexpr int VB = sizeof(T) == 2 ? 64 : 32;        // slab width
    constexpr int LDV = VB + PAD;
    constexpr int NVT = VB / 16;                         // column tiles of a slab
    constexpr int WPR = PW_ / 4;                         // wavefronts that share a row block in steps (1), (2)
    constexpr int NVW = NVT / WPR;                       // column tiles of a slab per wavefront there
    static_assert(NVT % WPR == 0 && NVW >= 1, "slab too narrow for this many wavefronts");
    constexpr int NCT = K / 16;                          // column tiles of the [64 x K] results
    constexpr int WPC = PW_ / NCT > 0 ? PW_ / NCT : 1;   // wavefronts per column tile ...
    constexpr int IBN = 4 / WPC;                         // ... and row blocks per wavefront
    static_assert(WPC <= 4 && 4 % WPC == 0, "column tiles / wavefronts");
    constexpr int NLT = (10 + PW_ - 1) / PW_;            // lower 16x16 tiles per wavefront
    constexpr int KS = Mfma<T>::KSTEP;
    // persistent
    __shared__ __attribute__((aligned(16))) T Ks[C * LDK];
    __shared__ __attribute__((aligned(16))) T Tt[C * LDC];       // T; after the walk: cA
    __shared__ float Gs[C], Bs[C];
    __shared__ float Egs[C], Ers[C];                     // gamma_i = e^{G_i} and rho_i = e^{G_C - G_i}, once per row
    __shared__ float red[4 * C];                         // [4][64] partial sums across tiles
    __shared__ float red2[4 * C];
    __shared__ float red3[4 * C];
    __shared__ float dbeta_s[WPR * C];
    __shared__ float sdot[PW_], trsum_s[PW_];
    __shared__ float colss[GV ? PT_ : 1];                // <dS', S> column by column (partials)
    __shared__ float dgam_s[GV ? (PW_ / (K / 16) > 0 ? PW_ / (K / 16) : 1) * K : 1];   // sum_i (K~/Gamma)_ic (E dS')_ic, per row-block group
    // slab buffers, later Q / K~ / cP and the row-dot partials
    constexpr int SLAB_ELEMS = 3 * C * LDV + 2 * VB * LDC + 2 * VB * LDK;
    constexpr int POST_ELEMS = 2 * C * LDK + C * LDC + (PW_ * C * 4) / (int)sizeof(T);
    constexpr int POOL = SLAB_ELEMS > POST_ELEMS ? SLAB_ELEMS : POST_ELEMS;
    __shared__ __attribute__((aligned(16))) T pool[POOL];
    T *dOs = pool;                      // [64][LDV]  dO slab (natural), later dV staging
    T *Vs = dOs + C * LDV;              // [64][LDV]  V slab
    T *dRs = Vs + C * LDV;              // [64][LDV]  dR slab (natural)
    T *Ets = dRs + C * LDV;             // [VB][LDC]  E^T slab
    T *dEts = Ets + VB * LDC;           // [VB][LDC]  dE^T slab
    T *Ss = dEts + VB * LDC;            // [VB][LDK]  S slab
    T *dSs = Ss + VB * LDK;             // [VB][LDK]  dS' slab
    T *Qs = pool;                       // after the walk
    T *Kts = Qs + C * LDK;
    T *cPs = Kts + C * LDK;             // [64][LDC]
    float *pq = reinterpret_cast<float *>(cPs + C * LDC);        // [PW_][64]
    T *cAs = Tt;                        // [64][LDC]

    // PAIR (large launches, bf16): a workgroup does two adjacent chunks one after the other (the
    // launcher halves the grid): the first loads of the second chunk (gates, K, T, the first slab)
    // are issued when the walk of the first is over and arrive while its results are finished.
    constexpr int tasks = PAIR ? 2 : 1;
    const int n_first = a.n0 + blockIdx.x * tasks, h = blockIdx.y, b = blockIdx.z;
    const int ntask = min(tasks, a.n1 - n_first);
    int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const size_t tstride = a.H;
    // the slab tiles travel through registers: the next slab (after the last one: Q and K~) is
    // fetched while the workgroup computes on the current one
    TileRegs<T, C, VB, PT_> r_dO, r_V;
    TileRegs<T, VB, C, PT_> r_Et, r_dEt;
    TileRegs<T, VB, K, PT_> r_S, r_dS;
    TileRegs<T, C, K, PT_> r_Q, r_Kt, r_Kn;
    TileRegs<T, C, C, PT_> r_Tn;
    float r_g = 0.f, r_b = 0.f;
#define OSDN_BP_FETCH(tok_, bhn_, v0_)                                                           \
    {                                                                                            \
        r_dO.fetch(static_cast<const T *>(a.dO) + (tok_) * a.V + (v0_), tstride * a.V, tid);     \
        r_V.fetch(static_cast<const T *>(a.v) + (tok_) * a.V + (v0_), tstride * a.V, tid);       \
        r_Et.fetch(static_cast<const T *>(a.Et) + ((bhn_) * a.V + (v0_)) * C, (size_t)C, tid);   \
        r_dEt.fetch(static_cast<const T *>(a.dEt) + ((bhn_) * a.V + (v0_)) * C, (size_t)C, tid); \
        r_S.fetch(static_cast<const T *>(a.S_ckpt) + ((bhn_) * a.V + (v0_)) * K, (size_t)K, tid); \
        r_dS.fetch(static_cast<const T *>(a.dS_ckpt) + ((bhn_) * a.V + (v0_)) * K, (size_t)K, tid); \
    }
    // gates, K and T of a chunk, then its first slab
#define OSDN_BP_ISSUE(n_)                                                                        \
    {                                                                                            \
        const size_t bhn_i = ((size_t)b * a.H + h) * a.N + (n_);                                 \
        const size_t tok_i = ((size_t)b * a.T + (size_t)(n_) * C) * a.H + h;                     \
        if (wave == 0) {                                                                         \
            const size_t th = tok_i + (size_t)lane * tstride;                                    \
            r_g = a.log_alpha ? a.log_alpha[th] : 0.f;                                           \
            r_b = a.beta[th];                                                                    \
        }                                                                                        \
        r_Kn.fetch(static_cast<const T *>(a.k) + tok_i * K, tstride * K, tid);                   \
        r_Tn.fetch(static_cast<const T *>(a.Tm) + bhn_i * C * C, (size_t)C, tid);                \
        OSDN_BP_FETCH(tok_i, bhn_i, 0)                                                           \
    }
    OSDN_BP_ISSUE(n_first)
#pragma unroll 1
    for (int task = 0; task < ntask; ++task) {
    // (the thread index is made opaque once per chunk, so that the lane addresses of the body
    // are not all computed ahead of the loop and kept in registers)
    asm volatile("" : "+v"(tid));
    wave = __builtin_amdgcn_readfirstlane(tid >> 6); lane = tid & 63;
    const int n = n_first + task;
    const size_t bhn = ((size_t)b * a.H + h) * a.N + n;
    const size_t tok0 = ((size_t)b * a.T + (size_t)n * C) * a.H + h;
    const int ct = (wave % NCT) * 16;   // this wave's column tile of the [64 x K] results ...
    const int ib0 = (wave / NCT) * IBN; // ... and its first row block
    const bool has_ct = wave < NCT * WPC;

    if (task > 0) __syncthreads();      // the previous chunk is through with every LDS tile
    if (wave == 0) {
        const float G = wave_cumsum(r_g, lane);
        Gs[lane] = G;
        Egs[lane] = __expf(G);
        Ers[lane] = __expf(lane_bcast63(G) - G);
        Bs[lane] = r_b;
    }
    r_Kn.put(Ks, LDK, tid);
    r_Tn.put(Tt, LDC, tid);

    // accumulators over the walk
    f32x4 dP[NLT], dA[NLT];             // the lower tiles idx = wave, wave + PW_ (< 10)
    f32x4 dQg[IBN], dKg[IBN], dKr[IBN]; // [row block ib0 + .], column tile ct
    float dbeta_part[4] = {0.f, 0.f, 0.f, 0.f};     // rows 16*(wave/2) + acc_row(lane, r), this wave's columns
    float ss_part = 0.f;                // <dS', S>
#pragma unroll
    for (int t = 0; t < NLT; ++t) { dP[t] = f32x4{0.f, 0.f, 0.f, 0.f}; dA[t] = f32x4{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
    for (int ib = 0; ib < IBN; ++ib) {
        dQg[ib] = f32x4{0.f, 0.f, 0.f, 0.f};
        dKg[ib] = f32x4{0.f, 0.f, 0.f, 0.f};
        dKr[ib] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const int rb = wave / WPR;          // row block of steps (1), (2)
    float gam_rb[4] = {1.f, 1.f, 1.f, 1.f};   // gamma of this lane's four rows there (set once G is in LDS)

    for (int v0 = 0; v0 < a.V; v0 += VB) {
        __syncthreads();
        r_dO.put(dOs, LDV, tid); r_V.put(Vs, LDV, tid);
        r_Et.put(Ets, LDC, tid); r_dEt.put(dEts, LDC, tid);
        r_S.put(Ss, LDK, tid); r_dS.put(dSs, LDK, tid);
        if (v0 + VB < a.V) {
            OSDN_BP_FETCH(tok0, bhn, v0 + VB)
        } else {
            r_Q.fetch(static_cast<const T *>(a.q) + tok0 * K, tstride * K, tid);
            r_Kt.fetch(static_cast<const T *>(a.kt) + tok0 * K, tstride * K, tid);
        }
        __syncthreads();
        if (v0 == 0) {
#pragma unroll
            for (int r = 0; r < 4; ++r) gam_rb[r] = Egs[rb * 16 + acc_row(lane, r)];
        }
        // <dS', S> over this slab (with per-channel gates: column by column, thread tid keeps column tid % K)
        if (GV) {
            for (int idx = tid; idx < VB * K; idx += PT_) {
                const int r = idx / K, c = idx % K;
                ss_part += to_f32(Ss[r * LDK + c]) * to_f32(dSs[r * LDK + c]);
            }
        } else {
            constexpr int VN = 16 / sizeof(T);
            for (int v = tid; v < VB * K / VN; v += PT_) {
                const int r = v / (K / VN), c = (v % (K / VN)) * VN;
                ss_part = dot_vec<T>(*reinterpret_cast<const u32x4 *>(Ss + r * LDK + c),
                                     *reinterpret_cast<const u32x4 *>(dSs + r * LDK + c), ss_part);
            }
        }
        // (1) dR = T^T dE, rows j = 16*rb.. ; (2) R0 = V - gamma . (K S^T), same rows
        {
            const int k0 = (rb * 16) / KS * KS;         // T[i][j] = 0 for i < j
            f32x4 dr[NVW], ks[NVW];             // the first product of each takes 0 as its addend
            {
                typename Mfma<T>::Frag ft = Mfma<T>::template load<false>(Tt + k0 * LDC + rb * 16, LDC, lane);
#pragma unroll
                for (int q = 0; q < NVW; ++q) {
                    const int vt = (wave % WPR) * NVW + q;
                    typename Mfma<T>::Frag fe = Mfma<T>::template load<true>(dEts + vt * 16 * LDC + k0, LDC, lane);
                    dr[q] = Mfma<T>::mma(ft, fe, f32x4{0.f, 0.f, 0.f, 0.f});
                }
            }
            for (int kk = k0 + KS; kk < C; kk += KS) {
                typename Mfma<T>::Frag ft = Mfma<T>::template load<false>(Tt + kk * LDC + rb * 16, LDC, lane);
#pragma unroll
                for (int q = 0; q < NVW; ++q) {
                    const int vt = (wave % WPR) * NVW + q;
                    typename Mfma<T>::Frag fe = Mfma<T>::template load<true>(dEts + vt * 16 * LDC + kk, LDC, lane);
                    dr[q] = Mfma<T>::mma(ft, fe, dr[q]);
                }
            }
#pragma unroll
            for (int kk = 0; kk < K; kk += KS) {
                typename Mfma<T>::Frag fk = Mfma<T>::template load<true>(Ks + rb * 16 * LDK + kk, LDK, lane);
#pragma unroll
                for (int q = 0; q < NVW; ++q) {
                    const int vt = (wave % WPR) * NVW + q;
                    typename Mfma<T>::Frag fs = Mfma<T>::template load<true>(Ss + vt * 16 * LDK + kk, LDK, lane);
                    ks[q] = Mfma<T>::mma(fk, fs, kk == 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : ks[q]);
                }
            }
#pragma unroll
            for (int q = 0; q < NVW; ++q) {
                const int vt = (wave % WPR) * NVW + q;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int i = rb * 16 + acc_row(lane, r), c = vt * 16 + acc_col(lane);
                    const float r0 = to_f32(Vs[i * LDV + c]) - gam_rb[r] * ks[q][r];
                    dbeta_part[r] += dr[q][r] * r0;
                }
                store_tile(dRs + rb * 16 * LDV + vt * 16, LDV, dr[q], lane);
            }
        }
        __syncthreads();
        // (3,4) dP += dO E^T, dA -= dR E^T on the lower tiles
#pragma unroll
        for (int t = 0; t < NLT; ++t) {
            const int idx = wave + PW_ * t;
            if (idx < 10) {
                const int ib = idx < 1 ? 0 : idx < 3 ? 1 : idx < 6 ? 2 : 3;
                const int jb = idx - (ib * (ib + 1)) / 2;
                for (int kk = 0; kk < VB; kk += KS) {
                    typename Mfma<T>::Frag fb = Mfma<T>::template load<false>(Ets + kk * LDC + jb * 16, LDC, lane);
                    typename Mfma<T>::Frag fo = Mfma<T>::template load<true>(dOs + ib * 16 * LDV + kk, LDV, lane);
                    typename Mfma<T>::Frag fr = Mfma<T>::template load<true>(dRs + ib * 16 * LDV + kk, LDV, lane);
                    dP[t] = Mfma<T>::mma(fo, fb, dP[t]);
                    dA[t] = Mfma<T>::mma(fr, fb, dA[t]);
                }
            }
        }
        // (5,6,7) dQg += dO S ; dKg += dR S ; dKr += E dS'   (column tile ct)
        if (has_ct) {
            for (int kk = 0; kk < VB; kk += KS) {
                typename Mfma<T>::Frag fs = Mfma<T>::template load<false>(Ss + kk * LDK + ct, LDK, lane);
                typename Mfma<T>::Frag fd = Mfma<T>::template load<false>(dSs + kk * LDK + ct, LDK, lane);
#pragma unroll
                for (int iq = 0; iq < IBN; ++iq) {
                    const int ib = ib0 + iq;
                    typename Mfma<T>::Frag fo = Mfma<T>::template load<true>(dOs + ib * 16 * LDV + kk, LDV, lane);
                    typename Mfma<T>::Frag fr = Mfma<T>::template load<true>(dRs + ib * 16 * LDV + kk, LDV, lane);
                    typename Mfma<T>::Frag fe = Mfma<T>::template load<false>(Ets + kk * LDC + ib * 16, LDC, lane);
                    dQg[iq] = Mfma<T>::mma(fo, fs, dQg[iq]);
                    dKg[iq] = Mfma<T>::mma(fr, fs, dKg[iq]);
                    dKr[iq] = Mfma<T>::mma(fe, fd, dKr[iq]);
                }
            }
        }
        __syncthreads();
        // dV = beta . dR for this slab, staged through the dO buffer
        {
            constexpr int VN = 16 / sizeof(T);
            for (int v = tid; v < C * VB / VN; v += PT_) {
                const int r = v / (VB / VN), c = (v % (VB / VN)) * VN;
                const u32x4 in = *reinterpret_cast<const u32x4 *>(dRs + r * LDV + c);
                float o[VN];
#pragma unroll
                for (int e = 0; e < VN; ++e) o[e] = Bs[r] * vec_get<T>(in, e);
                store_vec_t(dOs + r * LDV + c, o);
            }
        }
        __syncthreads();
        store_tile_global(static_cast<T *>(a.dv) + tok0 * a.V + v0, tstride * a.V, dOs, LDV, C, VB, tid, PT_);
    }
    __syncthreads();
    // ---- after the walk: Q, K~ into the pool ----
    r_Q.put(Qs, LDK, tid);
    r_Kt.put(Kts, LDK, tid);
    if (task + 1 < ntask) OSDN_BP_ISSUE(n + 1)
    {                                                   // upper triangle of cA, cP is zero
        constexpr int VN = 16 / sizeof(T);
        for (int v = tid; v < C * C / VN; v += PT_) {
            const int i = v / (C / VN), j = (v % (C / VN)) * VN;
            *reinterpret_cast<u32x4 *>(cAs + i * LDC + j) = u32x4{0u, 0u, 0u, 0u};
            *reinterpret_cast<u32x4 *>(cPs + i * LDC + j) = u32x4{0u, 0u, 0u, 0u};
        }
    }
    if (GV) colss[GV ? tid : 0] = ss_part;               // thread tid summed rows of column tid % K
    ss_part = wave_sum(ss_part);
    if (lane == 0) sdot[wave] = ss_part;
    for (int idx = tid; idx < 4 * C; idx += PT_) { red[idx] = 0.f; red2[idx] = 0.f; red3[idx] = 0.f; }
    for (int idx = tid; idx < PW_ * C; idx += PT_) pq[idx] = 0.f;          // row-dot partials: a wavefront fills its own row blocks
    // dbeta: the walk's part, reduced over the 16 lanes of a row; two waves share a row block
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const float sred = row16_sum(dbeta_part[r]);
        if (acc_col(lane) == 0) dbeta_s[(wave % WPR) * C + rb * 16 + acc_row(lane, r)] = sred;
    }
    __syncthreads();
    // ---- lower tiles: A0, P, X, cA, cP ----
#pragma unroll
    for (int t = 0; t < NLT; ++t) {
        const int idx = wave + PW_ * t;
        if (idx < 10) {
            const int ib = idx < 1 ? 0 : idx < 3 ? 1 : idx < 6 ? 2 : 3;
            const int jb = idx - (ib * (ib + 1)) / 2;
            const f32x4 kk = mma_tile0<T, true, true>(Ks + ib * 16 * LDK, LDK, Kts + jb * 16 * LDK, LDK, K, lane);
            const f32x4 qk = mma_tile0<T, true, true>(Qs + ib * 16 * LDK, LDK, Kts + jb * 16 * LDK, LDK, K, lane);
            f32x4 ca, cp;
            float colx = 0.f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = ib * 16 + acc_row(lane, r), j = jb * 16 + acc_col(lane);
                const float gam = (j <= i) ? __expf(Gs[i] - Gs[j]) : 0.f;
                const float da = (j < i) ? -dA[t][r] : 0.f;             // dA_ij
                const float dp = (j <= i) ? a.scale * dP[t][r] : 0.f;   // dP_ij
                const float a0 = gam * kk[r];                            // A_ij / beta_i
                const float x = da * Bs[i] * a0 + dp * gam * qk[r];      // dA.A + dP.P
                ca[r] = da * Bs[i] * gam;
                cp[r] = dp * gam;
                const float rs_a = row16_sum(da * a0);
                const float rs_x = row16_sum(x);
                if (acc_col(lane) == 0) {
                    red[jb * C + i] = rs_a;          // each (jb, i) is written by exactly one lane
                    red2[jb * C + i] = rs_x;
                }
                colx += x;
            }
            colx += __shfl_xor(colx, 16, 64);
            colx += __shfl_xor(colx, 32, 64);
            if (lane < 16) red3[ib * C + jb * 16 + lane] = colx;     // each (ib, j) written once
            store_tile(cAs + ib * 16 * LDC + jb * 16, LDC, ca, lane);
            store_tile(cPs + ib * 16 * LDC + jb * 16, LDC, cp, lane);
        }
    }
    __syncthreads();
    // ---- dQ, dK (read side), dK~ and the inner products that enter dG (column tile ct) ----
    // dG_i takes <d(gamma Q)_i, gamma_i Q_i> + <d(gamma K)_i, gamma_i K_i> - <d(rho K~)_i, rho_i K~_i>
    // as one number per row; the last term, summed over all rows, goes to the chunk's last token
    float tc[IBN][4];                             // [row block][r]: that combination over this wave's columns
    float trs = 0.f;                              // the last term over this lane's elements
#pragma unroll
    for (int ib = 0; ib < IBN; ++ib)
#pragma unroll
        for (int r = 0; r < 4; ++r) tc[ib][r] = 0.f;
    T *dq_g = static_cast<T *>(a.dq) + tok0 * K;
    T *dk_g = static_cast<T *>(a.dk_read) + tok0 * K;
    T *dkt_g = static_cast<T *>(a.dkt) + tok0 * K;
    const float gcv = (GV && has_ct) ? a.gamC[bhn * K + ct + acc_col(lane)] : 1.f;   // this lane's channel
    float dgc = 0.f;
    if (has_ct) {
#pragma unroll
        for (int iq = 0; iq < IBN; ++iq) {
            const int ib = ib0 + iq;
            f32x4 aq, ak, at;                   // the first product of each takes 0 as its addend
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            // cP K~ and cA K~: contraction over j <= i
            const int kd = min(C, ((ib + 1) * 16 + KS - 1) / KS * KS);
            for (int kk = 0; kk < kd; kk += KS) {
                typename Mfma<T>::Frag fk = Mfma<T>::template load<false>(Kts + kk * LDK + ct, LDK, lane);
                typename Mfma<T>::Frag fp = Mfma<T>::template load<true>(cPs + ib * 16 * LDC + kk, LDC, lane);
                typename Mfma<T>::Frag fa = Mfma<T>::template load<true>(cAs + ib * 16 * LDC + kk, LDC, lane);
                if (kk == 0) { aq = Mfma<T>::mma(fp, fk, zero); ak = Mfma<T>::mma(fa, fk, zero); }
                else { aq = Mfma<T>::mma(fp, fk, aq); ak = Mfma<T>::mma(fa, fk, ak); }
            }
            // cA^T K + cP^T Q: rows j = 16*ib.., contraction over i >= j
            const int k0 = (ib * 16) / KS * KS;
            {
                typename Mfma<T>::Frag fat = Mfma<T>::template load<false>(cAs + k0 * LDC + ib * 16, LDC, lane);
                typename Mfma<T>::Frag fpt = Mfma<T>::template load<false>(cPs + k0 * LDC + ib * 16, LDC, lane);
                typename Mfma<T>::Frag fkk = Mfma<T>::template load<false>(Ks + k0 * LDK + ct, LDK, lane);
                typename Mfma<T>::Frag fqq = Mfma<T>::template load<false>(Qs + k0 * LDK + ct, LDK, lane);
                at = Mfma<T>::mma(fat, fkk, zero);
                at = Mfma<T>::mma(fpt, fqq, at);
            }
            for (int kk = k0 + KS; kk < C; kk += KS) {
                typename Mfma<T>::Frag fat = Mfma<T>::template load<false>(cAs + kk * LDC + ib * 16, LDC, lane);
                typename Mfma<T>::Frag fpt = Mfma<T>::template load<false>(cPs + kk * LDC + ib * 16, LDC, lane);
                typename Mfma<T>::Frag fkk = Mfma<T>::template load<false>(Ks + kk * LDK + ct, LDK, lane);
                typename Mfma<T>::Frag fqq = Mfma<T>::template load<false>(Qs + kk * LDK + ct, LDK, lane);
                at = Mfma<T>::mma(fat, fkk, at);
                at = Mfma<T>::mma(fpt, fqq, at);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = ib * 16 + acc_row(lane, r), c = ct + acc_col(lane);
                const float gam = Egs[i], rho = Ers[i];
                const float gq = a.scale * gam * dQg[iq][r];         // gamma . d(gamma Q)
                const float gk = -Bs[i] * gam * dKg[iq][r];           // gamma . d(gamma K)
                const float gr = (GV ? gcv : rho) * dKr[iq][r];       // rho . d(rho K~)
                const float qv = to_f32(Qs[i * LDK + c]), kv = to_f32(Ks[i * LDK + c]),
                            ktv = to_f32(Kts[i * LDK + c]);
                if (GV) dgc = __builtin_fmaf(ktv, dKr[iq][r], dgc);
                tc[iq][r] = __builtin_fmaf(gq, qv, __builtin_fmaf(gk, kv, -(gr * ktv)));
                trs = __builtin_fmaf(gr, ktv, trs);
                const uint32_t go = ((uint32_t)i * (uint32_t)(tstride * K) + (uint32_t)c) * (uint32_t)sizeof(T);
                *reinterpret_cast<T *>(reinterpret_cast<char *>(dq_g) + go) = from_f32<T>(aq[r] + gq);
                *reinterpret_cast<T *>(reinterpret_cast<char *>(dk_g) + go) = from_f32<T>(ak[r] + gk);
                *reinterpret_cast<T *>(reinterpret_cast<char *>(dkt_g) + go) = from_f32<T>(at[r] + gr);
            }
        }
    }
    if (GV && has_ct) {                 // column sums over the rows: lanes 16 apart share a column
        dgc += __shfl_xor(dgc, 16, 64);
        dgc += __shfl_xor(dgc, 32, 64);
        if (lane < 16) dgam_s[GV ? (wave / NCT) * K + ct + lane : 0] = dgc;
    }
    // per-row sums across the 16 lanes of a row, then across waves through LDS
    if (has_ct) {
#pragma unroll
        for (int iq = 0; iq < IBN; ++iq)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float sc = row16_sum(tc[iq][r]);
                if (acc_col(lane) == 0) pq[wave * C + (ib0 + iq) * 16 + acc_row(lane, r)] = sc;
            }
    }
    trs = wave_sum(trs);
    if (lane == 0) trsum_s[wave] = trs;
    __syncthreads();
    if (GV && tid < K) {                // dL/d(decay of channel tid over the chunk)
        float sd = 0.f;
#pragma unroll
        for (int j = 0; j < WPC; ++j) sd += dgam_s[GV ? j * K + tid : 0];
#pragma unroll
        for (int j = 0; j < PT_ / K; ++j) sd += colss[GV ? tid + j * K : 0];
        a.dgamC[bhn * K + tid] = sd;
    }
    if (wave == 0) {
        const int i = lane;
        float t_c = 0.f;
#pragma unroll
        for (int w = 0; w < PW_; ++w) t_c += pq[w * C + i];
        const float rowa = red[i] + red[C + i] + red[2 * C + i] + red[3 * C + i];
        const float rowx = red2[i] + red2[C + i] + red2[2 * C + i] + red2[3 * C + i];
        const float colx = red3[i] + red3[C + i] + red3[2 * C + i] + red3[3 * C + i];
        const size_t th = tok0 + (size_t)i * tstride;
        float dbw = rowa;
#pragma unroll
        for (int w = 0; w < WPR; ++w) dbw += dbeta_s[w * C + i];
        a.dbeta[th] = dbw;
        if (a.dlog_alpha) {
            float dG = rowx - colx + t_c;
            float ssum = 0.f, tr_sum = 0.f;
#pragma unroll
            for (int w = 0; w < PW_; ++w) { ssum += sdot[w]; tr_sum += trsum_s[w]; }
            if (i == C - 1) dG += tr_sum + __expf(Gs[C - 1]) * ssum;
            a.dlog_alpha[th] = wave_suffix_sum(dG, lane);
        }
    }
    }   // task
}

// -------------------------------------------------------------- launchers ----
template <typename T, bool GV, int VS>
static int launch_chain_t(const ChunkArgs &a, hipStream_t st) {
    dim3 grid((a.V / VS) * a.H * (a.seq_chunks ? a.n_seqs : a.B)), block(CT_);
    if ((GV && !a.gamC) || !a.Pm || !a.q || !a.dO) return -1;
    if (a.K == 64) hipLaunchKernelGGL((bwd_chain_kernel<T, 64, GV, VS>), grid, block, 0, st, a);
    else if (a.K == 128) hipLaunchKernelGGL((bwd_chain_kernel<T, 128, GV, VS>), grid, block, 0, st, a);
    else return -1;
    return 0;
}
// Slices of 16 values when the caller asks for them (few chains: see ChunkArgs::narrow_slices).
template <typename T, bool GV>
static int launch_chain_v(const ChunkArgs &a, hipStream_t st) {
    return a.narrow_slices ? launch_chain_t<T, GV, 16>(a, st) : launch_chain_t<T, GV, 32>(a, st);
}
int launch_bwd_chain(const ChunkArgs &a, bool bf16_io, hipStream_t st) {
    if (a.gate_vec) return bf16_io ? launch_chain_v<bf16, true>(a, st) : launch_chain_v<float, true>(a, st);
    return bf16_io ? launch_chain_v<bf16, false>(a, st) : launch_chain_v<float, false>(a, st);
}
constexpr int BP_MIN_WGS = 2048;
template <typename T, bool GV>
static int launch_post_t(const ChunkArgs &a, hipStream_t st) {
    constexpr int PW = 8;           // wavefronts per workgroup (16 was measured for bf16: the kernel then
                                    // has to fit 128 registers, spills, and takes twice as long)
    // two chunks per workgroup when the launch still fills the chip many times over (one workgroup per CU)
    const int chunks = a.n1 - a.n0;
    constexpr bool PAIRABLE = sizeof(T) == 2 && !GV;     // elsewhere the prefetch registers would spill
    const bool pairs = PAIRABLE && chunks >= 2 && (long long)chunks * a.H * a.B >= BP_MIN_WGS;
    dim3 grid(pairs ? (chunks + 1) / 2 : chunks, a.H, a.B), block(PW * 64);
    if (GV && (!a.gamC || !a.dgamC || a.log_alpha || a.dlog_alpha)) return -1;
    if (pairs) {
        if (a.K == 64) hipLaunchKernelGGL((bwd_post_kernel<T, 64, GV, PW, PAIRABLE>), grid, block, 0, st, a);
        else if (a.K == 128) hipLaunchKernelGGL((bwd_post_kernel<T, 128, GV, PW, PAIRABLE>), grid, block, 0, st, a);
        else return -1;
        return 0;
    }
    if (a.K == 64) hipLaunchKernelGGL((bwd_post_kernel<T, 64, GV, PW, false>), grid, block, 0, st, a);
    else if (a.K == 128) hipLaunchKernelGGL((bwd_post_kernel<T, 128, GV, PW, false>), grid, block, 0, st, a);
    else return -1;
    return 0;
}
int launch_bwd_post(const ChunkArgs &a, bool bf16_io, hipStream_t st) {
    if (a.gate_vec) return bf16_io ? launch_post_t<bf16, true>(a, st) : launch_post_t<float, true>(a, st);
    return bf16_io ? launch_post_t<bf16, false>(a, st) : launch_post_t<float, false>(a, st);
}

// ---------------------------------------------------------------- unfold ----
// One state gate per key channel: phase 2 worked on Qg = Gamma . Q, Kg = Gamma . K and
// Kd = K~ / Gamma (Gamma = e^{G}, G the cumulative log-decay of every channel inside the
// chunk), and on gamma_C = Gamma's last row.  Per chunk this kernel rebuilds G and maps
//     dq = Gamma . dQg,   dk_read = Gamma . dKg,   dk~ = dKd / Gamma             (in place)
//     dG = dq . q + dk_read . k - dk~ . k~   (elementwise: G reaches the loss through the three
//          folded operands only),  dG[last token] += gamma_C . dgamma_C,
//     dlog_alpha = suffix sum of dG over the tokens of the chunk, channel by channel.
template <typename T, int K>
__global__ __launch_bounds__(NT) void unfold_kernel(UnfoldArgs a) {
    constexpr int GLD = K + 4, VN = 16 / sizeof(T);
    __shared__ __attribute__((aligned(16))) float Gt[C * GLD];     // G, then dG, then dlog_alpha
    const int n = a.n0 + blockIdx.x, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const size_t bhn = ((size_t)b * a.H + h) * a.N + n;
    const size_t tok0 = ((size_t)b * a.T + (size_t)n * C) * a.H + h;
    const size_t rs = (size_t)a.H * K;                              // elements between consecutive tokens
    const float *gp = a.log_alpha + tok0 * K;
    for (int v = tid; v < C * K / 4; v += NT) {
        const int i = v / (K / 4), c = (v % (K / 4)) * 4;
        *reinterpret_cast<f32x4 *>(Gt + i * GLD + c) = *reinterpret_cast<const f32x4 *>(gp + (size_t)i * rs + c);
    }
    __syncthreads();
    if (tid < K) {
        float G = 0.f;
#pragma unroll 16
        for (int i = 0; i < C; ++i) {
            G += Gt[i * GLD + tid];
            Gt[i * GLD + tid] = G;
        }
    }
    __syncthreads();
    const T *qp = static_cast<const T *>(a.q) + tok0 * K, *kp = static_cast<const T *>(a.k) + tok0 * K,
            *tp = static_cast<const T *>(a.kt) + tok0 * K;
    T *dqp = static_cast<T *>(a.dq) + tok0 * K, *dkp = static_cast<T *>(a.dk_read) + tok0 * K,
      *dtp = static_cast<T *>(a.dkt) + tok0 * K;
    for (int v = tid; v < C * K / VN; v += NT) {
        const int i = v / (K / VN), c = (v % (K / VN)) * VN;
        const size_t o = (size_t)i * rs + c;
        const u32x4 qv = *reinterpret_cast<const u32x4 *>(qp + o), kv = *reinterpret_cast<const u32x4 *>(kp + o),
                    tv = *reinterpret_cast<const u32x4 *>(tp + o);
        const u32x4 gq = *reinterpret_cast<const u32x4 *>(dqp + o), gk = *reinterpret_cast<const u32x4 *>(dkp + o),
                    gt = *reinterpret_cast<const u32x4 *>(dtp + o);
        float oq[VN], ok[VN], ot[VN];
#pragma unroll
        for (int e = 0; e < VN; ++e) {
            const float G = Gt[i * GLD + c + e];
            const float gam = __expf(G), inv = __expf(-G);
            oq[e] = vec_get<T>(gq, e) * gam;
            ok[e] = vec_get<T>(gk, e) * gam;
            ot[e] = vec_get<T>(gt, e) * inv;
            Gt[i * GLD + c + e] = oq[e] * vec_get<T>(qv, e) + ok[e] * vec_get<T>(kv, e) - ot[e] * vec_get<T>(tv, e);
        }
        store_vec_t(dqp + o, oq);
        store_vec_t(dkp + o, ok);
        store_vec_t(dtp + o, ot);
    }
    __syncthreads();
    if (tid < K) {
        float acc = a.gamC[bhn * K + tid] * a.dgamC[bhn * K + tid];
#pragma unroll 16
        for (int i = C - 1; i >= 0; --i) {
            acc += Gt[i * GLD + tid];
            Gt[i * GLD + tid] = acc;
        }
    }
    __syncthreads();
    float *dg = a.dlog_alpha + tok0 * K;
    for (int v = tid; v < C * K / 4; v += NT) {
        const int i = v / (K / 4), c = (v % (K / 4)) * 4;
        *reinterpret_cast<f32x4 *>(dg + (size_t)i * rs + c) = *reinterpret_cast<const f32x4 *>(Gt + i * GLD + c);
    }
}

template <typename T>
static int launch_unfold_t(const UnfoldArgs &a, hipStream_t st) {
    dim3 grid(a.n1 - a.n0, a.H, a.B), block(NT);
    if (a.K == 64) hipLaunchKernelGGL((unfold_kernel<T, 64>), grid, block, 0, st, a);
    else if (a.K == 128) hipLaunchKernelGGL((unfold_kernel<T, 128>), grid, block, 0, st, a);
    else return -1;
    return 0;
}
int launch_unfold(const UnfoldArgs &a, bool bf16_io, hipStream_t st) {
    if (!a.log_alpha || !a.q || !a.k || !a.kt || !a.dq || !a.dk_read || !a.dkt || !a.gamC || !a.dgamC || !a.dlog_alpha)
        return -1;
    return bf16_io ? launch_unfold_t<bf16>(a, st) : launch_unfold_t<float>(a, st);
}

}  // namespace osdn
