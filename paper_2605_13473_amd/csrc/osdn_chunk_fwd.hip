// Phase 2 forward of OSDN in chunkwise WY/UT form (Appendix A.2; gated, decay-ratio gauge
// of Appendix B.1), chunk length C = 64.  With G the in-chunk cumulative log-decay,
// gamma_i = e^{G_i}, rho_i = e^{G_C - G_i}, Gamma_ij = e^{G_i - G_j} (only j <= i is formed):
//
//   chunk_prep   (parallel over chunks):  A = tril(beta_i Gamma_ij <k_i, k~_j>, -1),
//                T = (I + A)^-1 in fp32,  W = T (beta gamma . K),  U = T (beta . V)
//   state_fwd    (sequential over chunks, parallel over (b, h, slice of V)):
//                E = U - W S^T ;  S <- gamma_C S + E^T (rho . K~)      (S fp32 in registers)
//   output_fwd   (parallel over chunks):  O = scale [ gamma . (Q S^T) + P E ],  P = tril(Gamma . Q K~^T)
//                (P is also written out when a backward pass follows)
//
// All contractions run on MFMA with fp32 accumulation; operands are staged in LDS in the
// I/O element type.
#include "osdn_kernels.h"

namespace osdn {

// ------------------------------------------------------------ chunk_prep ----
// Besides T it leaves the tiles the chain kernels consume in exactly the layout their MFMA
// operands want, so that those kernels only copy: -W^T, (rho . K~)^T and U^T (transposes come
// for free from the accumulator layout, or from a 0/1 selector product for K~).
// The row scalings of the right-hand sides move into T: W = (T diag(beta gamma)) K and
// U = (T diag(beta)) V, so that K and V enter the products as they come from memory.
//
// GV: one state gate per key channel (the chunkwise UT form of online-scaled KDA, appendix
// section on Kimi Delta Attention with online scaling).  The cumulative channel decays
// Gamma [64 x K] do not factor out of the Gram matrix as a 64 x 64 mask, so they are folded
// into the operands: K <- Gamma . K and K~ <- K~ / Gamma in LDS before anything else, after
// which the kernel runs as with no gate at all; it also leaves Gamma . Q, K~ / Gamma and the
// chunk's total decay per channel for the state and output kernels.  1 / Gamma grows like
// e^{|G|}: the cumulative log-decay of a channel inside a chunk has to stay above about -80.
constexpr int CP_ = 512;        // threads of a chunk_prep workgroup (8 wavefronts)
constexpr int CP_TASKS = 2;     // chunks per workgroup of a large launch
constexpr int CP_MIN_WGS = 2048;  // ... large: at least this many workgroups of one chunk each (four rounds of two per CU)
template <typename T, int K, bool GV>
__global__ __launch_bounds__(CP_) void chunk_prep_kernel(ChunkArgs a) {
    // K and K~ are read 16 bytes per lane along k (Gram matrix, transposes): 32 bytes of padding
    // for bf16 (not with per-channel gates, where two workgroups would no longer fit a CU); the
    // tiles that are written transposed keep 16
    constexpr int PAD = Pad<T>::v, LDK = K + (sizeof(T) == 2 && !GV ? 16 : PAD), LDC = C + PAD, LDF = C + 1;
    constexpr int NW = CP_ / 64;
    __shared__ __attribute__((aligned(16))) T X1[C * LDK];      // K, then V slabs
    __shared__ __attribute__((aligned(16))) T X2[C * LDK];      // K~, then W staging
    __shared__ __attribute__((aligned(16))) T Tu[C * LDC];      // T diag(beta)
    // scratch: A (fp32) | (I + A)^-1 (fp32).  A's space later holds
    // T diag(beta gamma); the rest doubles as the staging tile for the transposed outputs.
    constexpr int STAGE_F = (K * LDC * (int)sizeof(T) + 3) / 4;
    constexpr int TI_F = C * LDF + C;               // (I + A)^-1 and one row of column scalars
    constexpr int TW_F = C * LDC * (int)sizeof(T) / 4;
    constexpr int AF_F = ((C * LDF > TW_F ? C * LDF : TW_F) + 3) & ~3;
    __shared__ __attribute__((aligned(16))) float scratch[AF_F + (TI_F > STAGE_F ? TI_F : STAGE_F)];
    float *Af = scratch;                                        // A (fp32)
    float *Ti = scratch + AF_F;                                 // (I + A)^-1 (fp32), 16-byte aligned
    float *Xs = reinterpret_cast<float *>(Tu);                  // [3][16][17] block products of the inverse: T diag(beta) comes after it
    T *Tw = reinterpret_cast<T *>(Af);                          // [64][LDC], once A is dead
    T *stage = reinterpret_cast<T *>(Ti);                       // [K][LDC] / [64][LDC], while Ti is not live
    __shared__ float Gs[C], Bs[C];
    __shared__ float gCs[GV ? K : 1];                           // per-channel decay over the whole chunk

    // A workgroup builds `tasks` adjacent chunks one after the other: while it works on one, the
    // K, K~ tiles and gates of the next are already on their way (a third of a chunk's time is the
    // wait for its first loads otherwise).  The launcher asks for two only when the launch still
    // fills the chip several times over: on a short segment the longer workgroups would only
    // lengthen the time to its last chunk.
    const int tasks = (int)gridDim.x < a.n1 - a.n0 ? CP_TASKS : 1;
    const int n_first = a.n0 + blockIdx.x * tasks, h = blockIdx.y, b = blockIdx.z;
    const int ntask = min(tasks, a.n1 - n_first);
    int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const size_t tstride = a.H;                                           // tokens are H rows apart
    TileRegs<T, C, K, CP_> r_K, r_Kt;
    TileRegs<T, C, C, CP_> r_V;
    float r_g = 0.f, r_b = 0.f;
#define OSDN_CP_ISSUE(n_, with_v_)                                                               \
    {                                                                                            \
        const size_t tok_ = ((size_t)b * a.T + (size_t)(n_) * C) * a.H + h;                      \
        r_K.fetch(static_cast<const T *>(a.k) + tok_ * K, tstride * K, tid);                     \
        r_Kt.fetch(static_cast<const T *>(a.kt) + tok_ * K, tstride * K, tid);                   \
        if (with_v_) r_V.fetch(static_cast<const T *>(a.v) + tok_ * a.V, tstride * a.V, tid);    \
        if (wave == 0) {                                                                         \
            const size_t th = tok_ + (size_t)lane * tstride;                                     \
            r_g = (!GV && a.log_alpha) ? a.log_alpha[th] : 0.f;   /* GV: the gates go into the operands */ \
            r_b = a.beta[th];                                                                    \
        }                                                                                        \
    }
    OSDN_CP_ISSUE(n_first, true)
#pragma unroll 1
    for (int task = 0; task < ntask; ++task) {
    // (the thread index is made opaque once per chunk: otherwise every lane address of the body is
    // computed ahead of the loop and kept in registers, three times the registers of one chunk)
    asm volatile("" : "+v"(tid));
    wave = __builtin_amdgcn_readfirstlane(tid >> 6); lane = tid & 63;
    const int n = n_first + task;
    const size_t bhn = ((size_t)b * a.H + h) * a.N + n;
    const size_t tok0 = ((size_t)b * a.T + (size_t)n * C) * a.H + h;      // (b, first token, h)

    if (task > 0) __syncthreads();      // the previous chunk is through with every LDS tile
    if (wave == 0) {
        Gs[lane] = wave_cumsum(r_g, lane);
        Bs[lane] = r_b;
    }
    r_K.put(X1, LDK, tid);
    r_Kt.put(X2, LDK, tid);
    // the first slab of V stays in registers while the chunk's T is being built
    const T *vg = static_cast<const T *>(a.v) + tok0 * a.V;
    if (task + 1 < ntask) OSDN_CP_ISSUE(n + 1, false)
    __syncthreads();
    if (GV) {
        // cumulative log-decay of every channel, G [64 x K] in fp32, in the scratch space (not
        // yet in use): loaded with vector reads, summed down the columns by one thread per
        // channel, then K <- e^{G} K and K~ <- e^{-G} K~ in LDS and Gamma . Q straight to memory,
        // all threads on 16-byte vectors
        constexpr int GLD = K + 4, VN = 16 / sizeof(T);
        static_assert(C * GLD <= AF_F + (TI_F > STAGE_F ? TI_F : STAGE_F), "G must fit the scratch space");
        float *Gt = scratch;
        const size_t rs = tstride * K;
        const float *gp = a.log_alpha + tok0 * K;
        for (int v = tid; v < C * K / 4; v += CP_) {
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
            gCs[GV ? tid : 0] = __expf(G);
            a.gamC[bhn * K + tid] = __expf(G);
        }
        __syncthreads();
        const T *qp = static_cast<const T *>(a.q) + tok0 * K;
        T *qg = static_cast<T *>(a.Qg) + tok0 * K;
        for (int v = tid; v < C * K / VN; v += CP_) {
            const int i = v / (K / VN), c = (v % (K / VN)) * VN;
            const u32x4 kv = *reinterpret_cast<const u32x4 *>(X1 + i * LDK + c);
            const u32x4 tv = *reinterpret_cast<const u32x4 *>(X2 + i * LDK + c);
            const u32x4 qv = *reinterpret_cast<const u32x4 *>(qp + (size_t)i * rs + c);
            float ko[VN], to[VN], qo[VN];
#pragma unroll
            for (int e = 0; e < VN; ++e) {
                const float G = Gt[i * GLD + c + e];
                const float gam = __expf(G), inv = __expf(-G);
                ko[e] = vec_get<T>(kv, e) * gam;
                to[e] = vec_get<T>(tv, e) * inv;
                qo[e] = vec_get<T>(qv, e) * gam;
            }
            store_vec_t(X1 + i * LDK + c, ko);
            store_vec_t(X2 + i * LDK + c, to);
            store_vec_t(qg + (size_t)i * rs + c, qo);
        }
        __syncthreads();
        store_tile_global(static_cast<T *>(a.Kg) + tok0 * K, tstride * K, X1, LDK, C, K, tid, CP_);
        store_tile_global(static_cast<T *>(a.Kd) + tok0 * K, tstride * K, X2, LDK, C, K, tid, CP_);
        __syncthreads();            // the scratch space is handed over to A
    }

    // ---- A = tril(beta_i Gamma_ij <k_i, k~_j>, -1): the ten lower 16x16 tiles ----
    for (int idx = wave; idx < 10; idx += NW) {
        const int ib = idx < 1 ? 0 : idx < 3 ? 1 : idx < 6 ? 2 : 3;
        const int jb = idx - (ib * (ib + 1)) / 2;
        const f32x4 acc = mma_tile0<T, true, true>(X1 + ib * 16 * LDK, LDK, X2 + jb * 16 * LDK, LDK, K, lane);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = ib * 16 + acc_row(lane, r), j = jb * 16 + acc_col(lane);
            Af[i * LDF + j] = (j < i) ? Bs[i] * __expf(Gs[i] - Gs[j]) * acc[r] : 0.f;
        }
    }
    // ---- (rho . K~)^T: pick 16x16 blocks of K~, scale rows by rho_j, store transposed ----
    {
        const float GC = Gs[C - 1];
        for (int t = wave; t < (K / 16) * 4; t += NW) {
            const int nb = t >> 2, jb = t & 3;                  // 16 features of K~, 16 tokens
            {
                f32x4 acc = pick16<T>(X2 + jb * 16 * LDK, LDK, nb * 16, lane);
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[r] *= __expf(GC - Gs[jb * 16 + acc_row(lane, r)]);
                if (GV) {                       // (gamma_C / Gamma) . K~ = gamma_C . (K~ / Gamma), channel by channel
                    const float gc = gCs[GV ? nb * 16 + acc_col(lane) : 0];
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[r] *= gc;
                }
                store_tile_t(stage + nb * 16 * LDC + jb * 16, LDC, acc, lane);
            }
        }
    }
    __syncthreads();
    store_tile_global(static_cast<T *>(a.Ktr) + bhn * K * C, (size_t)C, stage, LDC, K, C, tid, CP_);
    __syncthreads();                // the staging tile is free again: (I + A)^-1 is built in its place

    // beta_j gamma_j, once per column (behind (I + A)^-1)
    float *BGs = Ti + C * LDF;
    if (wave == NW - 1) BGs[lane] = Bs[lane] * __expf(Gs[lane]);
    // ---- T = (I + A)^-1 in fp32, blocked ----
    ut_inverse64<LDF>(Af, Ti, Xs, wave, lane);
    // ---- T in the I/O type, three times: as it is (straight to memory), with the columns scaled
    //      by beta (for U) and by beta gamma (for W); the upper triangle is exactly zero ----
    {
        constexpr int VN = 16 / sizeof(T);
        T *tg = a.Tm ? static_cast<T *>(a.Tm) + bhn * C * C : nullptr;      // (kept for the backward pass only)
        for (int v = tid; v < C * C / VN; v += CP_) {
            const int i = v / (C / VN), j0 = (v % (C / VN)) * VN;
            float plain[VN], tu[VN], tw[VN];
#pragma unroll
            for (int e = 0; e < VN; ++e) {
                const int j = j0 + e;
                const float t = j <= i ? Ti[i * LDF + j] : 0.f;
                plain[e] = t;
                tu[e] = t * Bs[j];
                tw[e] = t * BGs[j];
            }
            if (tg) store_vec_t(tg + i * C + j0, plain);
            store_vec_t(Tu + i * LDC + j0, tu);
            store_vec_t(Tw + i * LDC + j0, tw);
        }
    }
    __syncthreads();                // Ti is dead from here on: its space is the staging tile again

    // ---- -W^T, W = (T diag(beta gamma)) K (the chain kernels fetch it with transpose reads) ----
    {
        for (int t = wave; t < (K / 16) * 4; t += NW) {
            const int nb = t >> 2, ib = t & 3;
            {
                const int kdim = min(C, ((ib + 1) * 16 + Mfma<T>::KSTEP - 1) / Mfma<T>::KSTEP * Mfma<T>::KSTEP);
                f32x4 acc = mma_tile0<T, true, false>(Tw + ib * 16 * LDC, LDC, X1 + nb * 16, LDK, kdim, lane);
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[r] = -acc[r];
                store_tile_t(stage + nb * 16 * LDC + ib * 16, LDC, acc, lane);
            }
        }
    }
    __syncthreads();
    store_tile_global(static_cast<T *>(a.Wt) + bhn * K * C, (size_t)C, stage, LDC, K, C, tid, CP_);

    // ---- U^T = ((T diag(beta)) V)^T, 64 columns of V at a time ----
    for (int v0 = 0; v0 < a.V; v0 += C) {
        __syncthreads();
        r_V.put(X1, LDC, tid);
        if (v0 + C < a.V) r_V.fetch(vg + v0 + C, tstride * a.V, tid);
        else if (task + 1 < ntask)          // the next chunk's first slab
            r_V.fetch(static_cast<const T *>(a.v) + (tok0 + (size_t)C * a.H) * a.V, tstride * a.V, tid);
        __syncthreads();
#pragma unroll
        for (int iq = 0; iq < 2; ++iq) {
            const int ib = (wave >> 2) * 2 + iq, wb = wave & 3;        // 16 columns of V (wb), two row blocks
            const int kdim = min(C, ((ib + 1) * 16 + Mfma<T>::KSTEP - 1) / Mfma<T>::KSTEP * Mfma<T>::KSTEP);
            const f32x4 acc = mma_tile0<T, true, false>(Tu + ib * 16 * LDC, LDC, X1 + wb * 16, LDC, kdim, lane);
            store_tile_t(stage + wb * 16 * LDC + ib * 16, LDC, acc, lane);
        }
        __syncthreads();
        store_tile_global(static_cast<T *>(a.Ut) + (bhn * a.V + v0) * C, (size_t)C, stage, LDC, C, C, tid, CP_);
    }
    }   // task
}

// ------------------------------------------------------------- state_fwd ----
// Sequential over the chunks of one (batch, head), one workgroup per slice of VS rows of S.
// Wavefronts 0-3 carry the dependent chain  S_n -> E_n -> S_{n+1}: the state slice lives
// transposed in their MFMA accumulators (fp32), so that its rounding to the I/O type lands in
// LDS with vector stores.  Wavefronts 4-7 only move data: they bring the next chunk's W,
// (rho . K~)^T and U^T tiles (already in operand layout) into the other LDS buffer and write
// the state checkpoint and E^T back, off the chain.  Two barriers per chunk.
constexpr int CT_ = 512;        // threads of a chain workgroup
constexpr int CL_ = 256;        // ... of which loaders

// GV: one state gate per key channel; the chunk's decay per channel comes from chunk_prep.
// VS: rows of S (values) owned by one workgroup, 32 or 16.  With few chains the narrow slice
// gives twice the workgroups, each with half the work on the dependent path per chunk.
template <typename T, int K, bool GV, int VS>
__global__ __launch_bounds__(CT_) void state_fwd_kernel(ChunkArgs a) {
    constexpr int NVT = VS / 16;                // value tiles per compute wave
    constexpr int PAD = Pad<T>::v, LDK = K + PAD, LDC = C + PAD;
    constexpr int VN = 16 / sizeof(T);
    constexpr int NKT = K / 64;                 // state row tiles (features) per compute wave
    constexpr int NB = sizeof(T) == 2 ? 2 : 1;  // LDS operand buffers (fp32 tiles are too big for two)
    // With two buffers the loaders work as two groups of two wavefronts, one per chunk parity:
    // a group fetches chunk c + 2 right after it has put chunk c into LDS, so every global
    // load has two chunk times to arrive.
    constexpr int LTN = NB == 2 ? CL_ / 2 : CL_;    // threads that share one chunk's tiles
    constexpr int NWV = C * K / VN / LTN;       // 16-byte vectors per loader thread, [64 x K] tile
    constexpr int NUV = VS * C / VN / LTN;
    static_assert(VS * C / VN % LTN == 0 && C * K / VN % LTN == 0, "tiles must split evenly over the loaders");
    __shared__ __attribute__((aligned(16))) T Wts[NB][K * LDC];      // -W^T  [kf][i], as chunk_prep left it
    __shared__ __attribute__((aligned(16))) T Ktr[NB][K * LDC];
    __shared__ __attribute__((aligned(16))) T Uts[NB][VS * LDC];
    __shared__ __attribute__((aligned(16))) T Sb[VS * LDK];     // S in the I/O type
    __shared__ __attribute__((aligned(16))) T Et[VS * LDC];     // E^T
    __shared__ float gCs[NB];

    int chain, slice;
    chain_slice_of(blockIdx.x, a.V / VS, (a.seq_chunks ? a.n_seqs : a.B) * a.H, chain, slice);
    const int vs = slice * VS, h = chain % a.H, b = chain / a.H;   // b: batch entry, or packed sequence
    int bt = b;                                 // batch entry of the token tensors
    if (a.seq_chunks) {
        bool begins, ends;
        if (!clip_to_sequence(a.seq_chunks, b, a.n0, a.n1, begins, ends)) return;
        a.S_in = begins ? a.S_first : a.S_out;
        bt = 0;
    }
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const bool loader = wave >= 4;
    const int lt = tid - CL_;                   // loader thread index
    const int lgrp = NB == 2 ? (lt >> 7) & 1 : 0;   // loader group (chunk parity it serves)
    const int lti = NB == 2 ? lt & 127 : lt;    // index inside the group
    const bool gwave = NB == 2 ? (wave & 1) == 0 : wave == 4;   // the group's wave that handles the gate
    const size_t bh = (size_t)b * a.H + h;      // the chain: indexes S_in / S_out
    const size_t bth = (size_t)bt * a.H + h;    // indexes the per-chunk buffers
    const size_t tstride = a.H;

    // ---- compute waves: state slice, transposed: St[vt][q] rows = features, cols = values ----
    f32x4 St[NVT][NKT];
    if (!loader) {
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
            for (int q = 0; q < NKT; ++q) {
                const int v = vs + vt * 16 + acc_col(lane), c0 = (wave * NKT + q) * 16 + acc_row(lane, 0);
                if (a.S_in) St[vt][q] = *reinterpret_cast<const f32x4 *>(a.S_in + (bh * a.V + v) * K + c0);
                else St[vt][q] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
    }
    // ---- loader waves: registers for one chunk ----
    u32x4 wreg[NWV], kreg[NWV], ureg[NUV];
    float greg = 0.f;
#define OSDN_SF_LOAD(n_)                                                                         \
    {                                                                                            \
        const size_t bhn_ = bth * a.N + (n_);                                                    \
        const T *wg = static_cast<const T *>(a.Wt) + bhn_ * K * C;                               \
        const T *kg = static_cast<const T *>(a.Ktr) + bhn_ * K * C;                              \
        const T *ug = static_cast<const T *>(a.Ut) + (bhn_ * a.V + vs) * C;                      \
        _Pragma("unroll") for (int m = 0; m < NWV; ++m) {                                        \
            const int i = lti + m * LTN;                                                          \
            wreg[m] = *reinterpret_cast<const u32x4 *>(wg + (size_t)i * VN);                     \
            kreg[m] = *reinterpret_cast<const u32x4 *>(kg + (size_t)i * VN);                     \
        }                                                                                        \
        _Pragma("unroll") for (int m = 0; m < NUV; ++m) {                                        \
            const int i = lti + m * LTN;                                                          \
            ureg[m] = *reinterpret_cast<const u32x4 *>(ug + (size_t)i * VN);                     \
        }                                                                                        \
        if (gwave)                                                                               \
            greg = a.log_alpha ? a.log_alpha[((size_t)bt * a.T + (size_t)(n_) * C + lane) * a.H + h] : 0.f; \
    }
#define OSDN_SF_STORE(buf_)                                                                      \
    {                                                                                            \
        _Pragma("unroll") for (int m = 0; m < NWV; ++m) {                                        \
            const int i = lti + m * LTN;                                                          \
            { const int r = i / (C / VN), c = (i % (C / VN)) * VN;                               \
              *reinterpret_cast<u32x4 *>(&Wts[buf_][r * LDC + c]) = wreg[m];                     \
              *reinterpret_cast<u32x4 *>(&Ktr[buf_][r * LDC + c]) = kreg[m]; }                   \
        }                                                                                        \
        _Pragma("unroll") for (int m = 0; m < NUV; ++m) {                                        \
            const int i = lti + m * LTN, r = i / (C / VN), c = (i % (C / VN)) * VN;               \
            *reinterpret_cast<u32x4 *>(&Uts[buf_][r * LDC + c]) = ureg[m];                       \
        }                                                                                        \
        if (gwave) {                                                                             \
            const float G_ = wave_cumsum(greg, lane);                                            \
            if (lane == 63) gCs[buf_] = __expf(G_);                                              \
        }                                                                                        \
    }
    if (loader) {
        if (NB == 2) {
            if (lgrp == (a.n0 & 1)) {
                OSDN_SF_LOAD(a.n0)
                OSDN_SF_STORE(a.n0 & 1)
                OSDN_SF_LOAD(min(a.n0 + 2, a.n1 - 1))
            } else {
                OSDN_SF_LOAD(min(a.n0 + 1, a.n1 - 1))
            }
        } else {
            OSDN_SF_LOAD(a.n0)
            OSDN_SF_STORE(0)
            OSDN_SF_LOAD(min(a.n0 + 1, a.n1 - 1))
        }
    }

    for (int n = a.n0; n < a.n1; ++n) {
        const int buf = NB == 2 ? (n & 1) : 0;
        const size_t bhn = bth * a.N + n;
        // ---- phase A (compute): S, rounded, into LDS ----
        f32x4 gch[GV ? NKT : 1];                                    // channel decays of this lane's state rows
        if (!loader) {
#pragma unroll
            for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
                for (int q = 0; q < NKT; ++q)
                    store_tile_t(Sb + vt * 16 * LDK + (wave * NKT + q) * 16, LDK, St[vt][q], lane);
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
                if (lgrp == ((n + 1) & 1)) {                        // this group's chunk comes next
                    if (n + 1 < a.n1) {
                        OSDN_SF_STORE((n + 1) & 1)                  // free since barrier 1
                        OSDN_SF_LOAD(min(n + 3, a.n1 - 1))          // (past the end: a harmless reload)
                    }
                } else if (a.S_ckpt) {
                    // checkpoint of the chunk-start state (read between barrier 1 and barrier 2)
                    store_tile_global(static_cast<T *>(a.S_ckpt) + (bhn * a.V + vs) * K, (size_t)K, Sb, LDK, VS, K, lti, LTN);
                }
            } else if (a.S_ckpt) {
                store_tile_global(static_cast<T *>(a.S_ckpt) + (bhn * a.V + vs) * K, (size_t)K, Sb, LDK, VS, K, lt, CL_);
            }
        } else {
            // ---- phase B: E = U - W S^T (rows 16*wave ..), kept transposed ----
#pragma unroll
            for (int vt = 0; vt < NVT; ++vt) {
                f32x4 acc = mma_tile0<T, false, true>(&Wts[buf][wave * 16], LDC, Sb + vt * 16 * LDK, LDK, K, lane);
                const T *up = &Uts[buf][(vt * 16 + acc_col(lane)) * LDC + wave * 16 + acc_row(lane, 0)];
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[r] += to_f32(up[r]);         // U + (-W) S^T
                store_tile_t(Et + vt * 16 * LDC + wave * 16, LDC, acc, lane);
            }
        }
        __syncthreads();                                            // barrier 2
        if (loader) {
            if (NB == 2) {
                if (lgrp == ((n + 1) & 1))                          // the group with no load wait ahead
                    store_tile_global(static_cast<T *>(a.Et) + (bhn * a.V + vs) * C, (size_t)C, Et, LDC, VS, C, lti, LTN);
            } else {
                store_tile_global(static_cast<T *>(a.Et) + (bhn * a.V + vs) * C, (size_t)C, Et, LDC, VS, C, lt, CL_);
            }
        } else {
            // ---- phase C: S <- gamma_C S + E^T (rho . K~), transposed ----
            const float gC = gCs[buf];
#pragma unroll
            for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
                for (int q = 0; q < NKT; ++q) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) St[vt][q][r] *= GV ? gch[GV ? q : 0][r] : gC;
                    mma_tile<T, true, true>(St[vt][q], &Ktr[buf][(wave * NKT + q) * 16 * LDC], LDC,
                                            Et + vt * 16 * LDC, LDC, C, lane);
                }
        }
        if (NB == 1) {                                              // single buffer: refill it now
            __syncthreads();
            if (loader && n + 1 < a.n1) {
                OSDN_SF_STORE(0)
                OSDN_SF_LOAD(min(n + 2, a.n1 - 1))
            }
        }
    }
    if (!loader) {
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
            for (int q = 0; q < NKT; ++q) {
                const int v = vs + vt * 16 + acc_col(lane), c0 = (wave * NKT + q) * 16 + acc_row(lane, 0);
                *reinterpret_cast<f32x4 *>(a.S_out + (bh * a.V + v) * K + c0) = St[vt][q];
            }
    }
}

// ------------------------------------------------------------ output_fwd ----
constexpr int OT_ = 512;        // threads of an output_fwd workgroup: 8 wavefronts, (row block, half of the value tiles)
template <typename T, int K>
__global__ __launch_bounds__(OT_) void output_fwd_kernel(ChunkArgs a) {
    constexpr int PAD = sizeof(T) == 2 ? 16 : Pad<T>::v, LDK = K + PAD, LDC = C + PAD;   // bf16: rows 32 bytes apart modulo 128 (every operand read here is 16 bytes per lane along k)
    constexpr int NW = OT_ / 64;
    __shared__ __attribute__((aligned(16))) T Qs[C * LDK];
    __shared__ __attribute__((aligned(16))) T Kts[C * LDK];     // K~, later the output staging tile
    __shared__ __attribute__((aligned(16))) T Ss[C * LDK];      // 64 rows of the chunk-start state
    __shared__ __attribute__((aligned(16))) T Ps[C * LDC];      // tril(Gamma . Q K~^T)
    __shared__ __attribute__((aligned(16))) T Ets[C * LDC];     // 64 rows of E^T
    __shared__ float Gs[C];

    const int n = a.n0 + blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const size_t bhn = ((size_t)b * a.H + h) * a.N + n;
    const size_t tok0 = ((size_t)b * a.T + (size_t)n * C) * a.H + h;
    const size_t tstride = a.H;

    if (wave == 0) {
        const float g = a.log_alpha ? a.log_alpha[tok0 + (size_t)lane * tstride] : 0.f;
        Gs[lane] = wave_cumsum(g, lane);
    }
    load_tile(Qs, LDK, static_cast<const T *>(a.q) + tok0 * K, tstride * K, C, K, tid, OT_);
    load_tile(Kts, LDK, static_cast<const T *>(a.kt) + tok0 * K, tstride * K, C, K, tid, OT_);
    // the slabs of S and E^T travel through registers, one slab ahead of the products
    TileRegs<T, C, K, OT_> r_S;
    TileRegs<T, C, C, OT_> r_E;
    r_S.fetch(static_cast<const T *>(a.S_ckpt) + bhn * a.V * K, (size_t)K, tid);
    r_E.fetch(static_cast<const T *>(a.Et) + bhn * a.V * C, (size_t)C, tid);
    __syncthreads();
    // P^T tiles (rows j, columns i) so that the store lands k-contiguous in Ps[i][j]
    for (int idx = wave; idx < 16; idx += NW) {
        const int ib = idx >> 2, jb = idx & 3;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        if (jb <= ib) {
            mma_tile<T, true, true>(acc, Kts + jb * 16 * LDK, LDK, Qs + ib * 16 * LDK, LDK, K, lane);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int j = jb * 16 + acc_row(lane, r), i = ib * 16 + acc_col(lane);
                acc[r] = (j <= i) ? __expf(Gs[i] - Gs[j]) * acc[r] : 0.f;
            }
        }
        store_tile_t(Ps + ib * 16 * LDC + jb * 16, LDC, acc, lane);
    }
    T *Os = Kts;
    for (int v0 = 0; v0 < a.V; v0 += C) {
        __syncthreads();
        // P is kept for the backward pass (its chain kernel forms scale P^T dO from it)
        if (v0 == 0 && a.Pm) store_tile_global(static_cast<T *>(a.Pm) + bhn * C * C, (size_t)C, Ps, LDC, C, C, tid, OT_);
        r_S.put(Ss, LDK, tid);
        r_E.put(Ets, LDC, tid);
        if (v0 + C < a.V) {
            r_S.fetch(static_cast<const T *>(a.S_ckpt) + (bhn * a.V + v0 + C) * K, (size_t)K, tid);
            r_E.fetch(static_cast<const T *>(a.Et) + (bhn * a.V + v0 + C) * C, (size_t)C, tid);
        }
        __syncthreads();
        const int rb = wave & 3;                    // row block of this wavefront; the other bit: which value tiles
        const int kdim = min(C, ((rb + 1) * 16 + Mfma<T>::KSTEP - 1) / Mfma<T>::KSTEP * Mfma<T>::KSTEP);
#pragma unroll
        for (int vq = 0; vq < 4 / (NW / 4); ++vq) {
            const int vt = (wave >> 2) * (4 / (NW / 4)) + vq;
            f32x4 a1 = {0.f, 0.f, 0.f, 0.f}, a2 = {0.f, 0.f, 0.f, 0.f};
            mma_tile<T, true, true>(a1, Qs + rb * 16 * LDK, LDK, Ss + vt * 16 * LDK, LDK, K, lane);
            mma_tile<T, true, true>(a2, Ps + rb * 16 * LDC, LDC, Ets + vt * 16 * LDC, LDC, kdim, lane);
#pragma unroll
            for (int r = 0; r < 4; ++r)
                a1[r] = a.scale * (__expf(Gs[rb * 16 + acc_row(lane, r)]) * a1[r] + a2[r]);
            store_tile(Os + rb * 16 * LDC + vt * 16, LDC, a1, lane);
        }
        __syncthreads();
        store_tile_global(static_cast<T *>(a.o) + tok0 * a.V + v0, tstride * a.V, Os, LDC, C, C, tid, OT_);
    }
}

// -------------------------------------------------------------- launchers ----
template <typename T, bool GV>
static int launch_prep_t(const ChunkArgs &a, hipStream_t st) {
    const int chunks = a.n1 - a.n0;
    const bool pairs = chunks >= 2 && (long long)chunks * a.H * a.B >= CP_MIN_WGS;
    dim3 grid(pairs ? (chunks + CP_TASKS - 1) / CP_TASKS : chunks, a.H, a.B), block(CP_);
    if (GV && (!a.log_alpha || !a.Qg || !a.Kg || !a.Kd || !a.gamC)) return -1;
    if (a.K == 64) hipLaunchKernelGGL((chunk_prep_kernel<T, 64, GV>), grid, block, 0, st, a);
    else if (a.K == 128) hipLaunchKernelGGL((chunk_prep_kernel<T, 128, GV>), grid, block, 0, st, a);
    else return -1;
    return 0;
}
int launch_chunk_prep(const ChunkArgs &a, bool bf16_io, hipStream_t st) {
    if (a.gate_vec) return bf16_io ? launch_prep_t<bf16, true>(a, st) : launch_prep_t<float, true>(a, st);
    return bf16_io ? launch_prep_t<bf16, false>(a, st) : launch_prep_t<float, false>(a, st);
}
template <typename T, bool GV, int VS>
static int launch_state_t(const ChunkArgs &a, hipStream_t st) {
    dim3 grid((a.V / VS) * a.H * (a.seq_chunks ? a.n_seqs : a.B)), block(CT_);
    if (GV && !a.gamC) return -1;
    if (a.K == 64) hipLaunchKernelGGL((state_fwd_kernel<T, 64, GV, VS>), grid, block, 0, st, a);
    else if (a.K == 128) hipLaunchKernelGGL((state_fwd_kernel<T, 128, GV, VS>), grid, block, 0, st, a);
    else return -1;
    return 0;
}
// Slices of 16 values when the caller asks for them (few chains: see ChunkArgs::narrow_slices).
template <typename T, bool GV>
static int launch_state_v(const ChunkArgs &a, hipStream_t st) {
    return a.narrow_slices ? launch_state_t<T, GV, 16>(a, st) : launch_state_t<T, GV, 32>(a, st);
}
int launch_state_fwd(const ChunkArgs &a, bool bf16_io, hipStream_t st) {
    if (a.gate_vec) return bf16_io ? launch_state_v<bf16, true>(a, st) : launch_state_v<float, true>(a, st);
    return bf16_io ? launch_state_v<bf16, false>(a, st) : launch_state_v<float, false>(a, st);
}
template <typename T>
static int launch_output_t(const ChunkArgs &a, hipStream_t st) {
    dim3 grid(a.n1 - a.n0, a.H, a.B), block(OT_);
    if (a.K == 64) hipLaunchKernelGGL((output_fwd_kernel<T, 64>), grid, block, 0, st, a);
    else if (a.K == 128) hipLaunchKernelGGL((output_fwd_kernel<T, 128>), grid, block, 0, st, a);
    else return -1;
    return 0;
}
int launch_output_fwd(const ChunkArgs &a, bool bf16_io, hipStream_t st) {
    return bf16_io ? launch_output_t<bf16>(a, st) : launch_output_t<float>(a, st);
}

}  // namespace osdn
