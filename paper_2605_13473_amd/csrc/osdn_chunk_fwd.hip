// Phase 2 forward of OSDN in chunkwise WY/UT form (Appendix A.2; gated, decay-ratio gauge
// of Appendix B.1), chunk length C = 64.  With G the in-chunk cumulative log-decay,
// gamma_i = e^{G_i}, rho_i = e^{G_C - G_i}, Gamma_ij = e^{G_i - G_j} (only j <= i is formed):
//
//   chunk_prep   (parallel over chunks):  A = tril(beta_i Gamma_ij <k_i, k~_j>, -1),
//                T = (I + A)^-1 in fp32,  W = T (beta gamma . K),  U = T (beta . V)
//   state_fwd    (sequential over chunks, parallel over (b, h, slice of V)):
//                E = U - W S^T ;  S <- gamma_C S + E^T (rho . K~)      (S fp32 in registers)
//   output_fwd   (parallel over chunks):  O = scale [ gamma . (Q S^T) + tril(Gamma . Q K~^T) E ]
//
// All contractions run on MFMA with fp32 accumulation; operands are staged in LDS in the
// I/O element type.
#include "osdn_kernels.h"

namespace osdn {

// ------------------------------------------------------------ chunk_prep ----
template <typename T, int K>
__global__ __launch_bounds__(NT) void chunk_prep_kernel(ChunkArgs a) {
    constexpr int PAD = Pad<T>::v, LDK = K + PAD, LDC = C + PAD, LDF = C + 1;
    __shared__ __attribute__((aligned(16))) T X1[C * LDK];      // K, then beta gamma K, then V slabs
    __shared__ __attribute__((aligned(16))) T X2[C * LDK];      // K~, then output staging
    __shared__ __attribute__((aligned(16))) T Tt[C * LDC];      // T in the I/O type
    __shared__ float Af[C * LDF];                               // A (fp32)
    __shared__ float Ti[C * LDF];                               // (I + A)^-1 (fp32)
    __shared__ float Xs[3 * 16 * 17];                           // block-product scratch
    __shared__ float Gs[C], Bs[C];

    const int n = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const size_t bhn = ((size_t)b * a.H + h) * a.N + n;
    const size_t tok0 = ((size_t)b * a.T + (size_t)n * C) * a.H + h;      // (b, first token, h)
    const size_t tstride = a.H;                                           // tokens are H rows apart

    if (wave == 0) {
        const size_t th = tok0 + (size_t)lane * tstride;
        const float g = a.log_alpha ? a.log_alpha[th] : 0.f;
        Gs[lane] = wave_cumsum(g, lane);
        Bs[lane] = a.beta[th];
    }
    load_tile(X1, LDK, static_cast<const T *>(a.k) + tok0 * K, tstride * K, C, K, tid, NT);
    load_tile(X2, LDK, static_cast<const T *>(a.kt) + tok0 * K, tstride * K, C, K, tid, NT);
    __syncthreads();

    // ---- A = tril(beta_i Gamma_ij <k_i, k~_j>, -1): the ten lower 16x16 tiles ----
    for (int idx = wave; idx < 10; idx += 4) {
        const int ib = idx < 1 ? 0 : idx < 3 ? 1 : idx < 6 ? 2 : 3;
        const int jb = idx - (ib * (ib + 1)) / 2;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        mma_tile<T, true, true>(acc, X1 + ib * 16 * LDK, LDK, X2 + jb * 16 * LDK, LDK, K, lane);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = ib * 16 + acc_row(lane, r), j = jb * 16 + acc_col(lane);
            Af[i * LDF + j] = (j < i) ? Bs[i] * __expf(Gs[i] - Gs[j]) * acc[r] : 0.f;
        }
    }
    __syncthreads();

    // ---- T = (I + A)^-1, 16x16 blocks.  Diagonal blocks: forward substitution, one
    //      column per lane.  Block (i,j), i > j: T_ij = -T_ii sum_{m=j}^{i-1} A_im T_mj. ----
    if (lane < 16) {
        const int o = wave * 16;
        float x[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            float v = (i == lane) ? 1.f : 0.f;
#pragma unroll
            for (int j = 0; j < i; ++j) v -= Af[(o + i) * LDF + o + j] * x[j];
            x[i] = v;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) Ti[(o + i) * LDF + o + lane] = x[i];
    }
    __syncthreads();
    for (int s = 1; s <= 3; ++s) {
        const int nblk = 4 - s;
        for (int task = tid; task < nblk * 256; task += NT) {
            const int bi = task >> 8, e = task & 255, r = e >> 4, c = e & 15;
            const int i = s + bi, j = bi;
            float acc = 0.f;
            for (int m = j; m < i; ++m)
#pragma unroll
                for (int l = 0; l < 16; ++l)
                    acc += Af[(i * 16 + r) * LDF + m * 16 + l] * Ti[(m * 16 + l) * LDF + j * 16 + c];
            Xs[(bi * 16 + r) * 17 + c] = acc;
        }
        __syncthreads();
        for (int task = tid; task < nblk * 256; task += NT) {
            const int bi = task >> 8, e = task & 255, r = e >> 4, c = e & 15;
            const int i = s + bi, j = bi;
            float acc = 0.f;
            for (int l = 0; l <= r; ++l) acc += Ti[(i * 16 + r) * LDF + i * 16 + l] * Xs[(bi * 16 + l) * 17 + c];
            Ti[(i * 16 + r) * LDF + j * 16 + c] = -acc;
        }
        __syncthreads();
    }
    // T in the I/O type (upper triangle exactly zero), and beta gamma . K in place
    for (int idx = tid; idx < C * C; idx += NT) {
        const int i = idx >> 6, j = idx & 63;
        Tt[i * LDC + j] = from_f32<T>(j <= i ? Ti[i * LDF + j] : 0.f);
    }
    for (int idx = tid; idx < C * K; idx += NT) {
        const int j = idx / K, c = idx % K;
        X1[j * LDK + c] = from_f32<T>(Bs[j] * __expf(Gs[j]) * to_f32(X1[j * LDK + c]));
    }
    __syncthreads();
    store_tile_global(static_cast<T *>(a.Tm) + bhn * C * C, C, Tt, LDC, C, C, tid, NT);

    // ---- W = T (beta gamma . K) ----
    {
        constexpr int NKT = K / 64;     // column tiles per wave
#pragma unroll
        for (int qn = 0; qn < NKT; ++qn) {
            const int nb = wave * NKT + qn;
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                const int kdim = min(C, ((ib + 1) * 16 + Mfma<T>::KSTEP - 1) / Mfma<T>::KSTEP * Mfma<T>::KSTEP);
                mma_tile<T, true, false>(acc, Tt + ib * 16 * LDC, LDC, X1 + nb * 16, LDK, kdim, lane);
                store_tile(X2 + ib * 16 * LDK + nb * 16, LDK, acc, lane);
            }
        }
    }
    __syncthreads();
    store_tile_global(static_cast<T *>(a.W) + bhn * C * K, K, X2, LDK, C, K, tid, NT);

    // ---- U = T (beta . V), 64 columns of V at a time ----
    const T *vg = static_cast<const T *>(a.v) + tok0 * a.V;
    for (int v0 = 0; v0 < a.V; v0 += C) {
        __syncthreads();
        constexpr int VN = 16 / sizeof(T);
        for (int i = tid; i < C * (C / VN); i += NT) {
            const int r = i / (C / VN), c = (i % (C / VN)) * VN;
            uint4 raw = *reinterpret_cast<const uint4 *>(vg + (size_t)r * tstride * a.V + v0 + c);
            const float br = Bs[r];
#pragma unroll
            for (int e = 0; e < VN; ++e) X1[r * LDC + c + e] = from_f32<T>(br * vec_get<T>(raw, e));
        }
        __syncthreads();
#pragma unroll
        for (int ib = 0; ib < 4; ++ib) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            const int kdim = min(C, ((ib + 1) * 16 + Mfma<T>::KSTEP - 1) / Mfma<T>::KSTEP * Mfma<T>::KSTEP);
            mma_tile<T, true, false>(acc, Tt + ib * 16 * LDC, LDC, X1 + wave * 16, LDC, kdim, lane);
            store_tile(X2 + ib * 16 * LDC + wave * 16, LDC, acc, lane);
        }
        __syncthreads();
        store_tile_global(static_cast<T *>(a.U) + bhn * C * a.V + v0, a.V, X2, LDC, C, C, tid, NT);
    }
}

// ------------------------------------------------------------- state_fwd ----
constexpr int VS = 32;      // rows of S (values) owned by one workgroup

// (one workgroup per CU is the intended residency: let the register allocator use the file)
template <typename T, int K>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(1, 2))) void state_fwd_kernel(ChunkArgs a) {
    constexpr int PAD = Pad<T>::v, LDK = K + PAD, LDC = C + PAD, LDU = VS + PAD;
    constexpr int VN = 16 / sizeof(T);
    constexpr int NKT = K / 64;                 // S column tiles per wave
    constexpr int NW = C * K / VN / NT;         // 16-byte vectors per thread for a [64 x K] tile
    constexpr int NU = C * VS / VN / NT;          // (exact: C*VS/VN is a multiple of NT)
    static_assert(C * VS / VN % NT == 0, "U slab must split evenly over the workgroup");
    __shared__ __attribute__((aligned(16))) T Ws[C * LDK];
    __shared__ __attribute__((aligned(16))) T Ktt[K * LDC];     // (rho . K~)^T
    __shared__ __attribute__((aligned(16))) T Us[C * LDU];
    __shared__ __attribute__((aligned(16))) T Sb[VS * LDK];     // S in the I/O type
    __shared__ __attribute__((aligned(16))) T Et[VS * LDC];     // E^T

    int chain, slice;
    chain_slice_of(blockIdx.x, a.V / VS, a.B * a.H, chain, slice);
    const int vs = slice * VS, h = chain % a.H, b = chain / a.H;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const size_t bh = (size_t)b * a.H + h;
    const size_t tstride = a.H;

    f32x4 S[2][NKT];
#pragma unroll
    for (int vt = 0; vt < 2; ++vt)
#pragma unroll
        for (int qn = 0; qn < NKT; ++qn)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int v = vs + vt * 16 + acc_row(lane, r), c = (wave * NKT + qn) * 16 + acc_col(lane);
                S[vt][qn][r] = a.S_in ? a.S_in[(bh * a.V + v) * K + c] : 0.f;
            }

    uint4 wreg[NW], kreg[NW], ureg[NU];
    float greg;
#define OSDN_STATE_PREFETCH(n_)                                                                  \
    {                                                                                            \
        const size_t bhn_ = bh * a.N + (n_);                                                     \
        const size_t tok_ = ((size_t)b * a.T + (size_t)(n_) * C) * a.H + h;                      \
        const T *wg = static_cast<const T *>(a.W) + bhn_ * C * K;                                \
        const T *kg = static_cast<const T *>(a.kt) + tok_ * K;                                   \
        const T *ug = static_cast<const T *>(a.U) + bhn_ * C * a.V + vs;                         \
        _Pragma("unroll") for (int m = 0; m < NW; ++m) {                                         \
            const int i = tid + m * NT, r = i / (K / VN), c = (i % (K / VN)) * VN;               \
            wreg[m] = *reinterpret_cast<const uint4 *>(wg + (size_t)r * K + c);                  \
            kreg[m] = *reinterpret_cast<const uint4 *>(kg + (size_t)r * tstride * K + c);        \
        }                                                                                        \
        _Pragma("unroll") for (int m = 0; m < NU; ++m) {                                         \
            const int i = tid + m * NT, r = i / (VS / VN), c = (i % (VS / VN)) * VN;             \
            ureg[m] = *reinterpret_cast<const uint4 *>(ug + (size_t)r * a.V + c);                \
        }                                                                                        \
        greg = a.log_alpha ? a.log_alpha[tok_ + (size_t)lane * tstride] : 0.f;                   \
    }
    OSDN_STATE_PREFETCH(0)

    for (int n = 0; n < a.N; ++n) {
        const size_t bhn = bh * a.N + n;
        // ---- 1. registers -> LDS ----
        const float G = wave_cumsum(greg, lane);
        const float GC = __shfl(G, 63, 64);
#pragma unroll
        for (int m = 0; m < NW; ++m) {
            const int i = tid + m * NT, r = i / (K / VN), c = (i % (K / VN)) * VN;
            *reinterpret_cast<uint4 *>(Ws + r * LDK + c) = wreg[m];
            const float rho = __expf(GC - __shfl(G, r, 64));
#pragma unroll
            for (int e = 0; e < VN; ++e) Ktt[(c + e) * LDC + r] = from_f32<T>(rho * vec_get<T>(kreg[m], e));
        }
#pragma unroll
        for (int m = 0; m < NU; ++m) {
            const int i = tid + m * NT, r = i / (VS / VN), c = (i % (VS / VN)) * VN;
            *reinterpret_cast<uint4 *>(Us + r * LDU + c) = ureg[m];
        }
#pragma unroll
        for (int vt = 0; vt < 2; ++vt)
#pragma unroll
            for (int qn = 0; qn < NKT; ++qn)
                store_tile(Sb + vt * 16 * LDK + (wave * NKT + qn) * 16, LDK, S[vt][qn], lane);
        __syncthreads();
        if (a.S_ckpt)
            store_tile_global(static_cast<T *>(a.S_ckpt) + (bhn * a.V + vs) * K, K, Sb, LDK, VS, K, tid, NT);
        // ---- 2. fetch the next chunk while this one is computed ----
        if (n + 1 < a.N) OSDN_STATE_PREFETCH(n + 1)
        // ---- 3. E = U - W S^T (rows 16*wave .. +16), kept transposed ----
#pragma unroll
        for (int vt = 0; vt < 2; ++vt) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            mma_tile<T, true, true>(acc, Ws + wave * 16 * LDK, LDK, Sb + vt * 16 * LDK, LDK, K, lane);
#pragma unroll
            for (int r = 0; r < 4; ++r)
                acc[r] = to_f32(Us[(wave * 16 + acc_row(lane, r)) * LDU + vt * 16 + acc_col(lane)]) - acc[r];
            store_tile_t(Et + vt * 16 * LDC + wave * 16, LDC, acc, lane);
        }
        __syncthreads();
        store_tile_global(static_cast<T *>(a.Et) + (bhn * a.V + vs) * C, C, Et, LDC, VS, C, tid, NT);
        // ---- 4. S <- gamma_C S + E^T (rho . K~) ----
        const float gC = __expf(GC);
#pragma unroll
        for (int vt = 0; vt < 2; ++vt)
#pragma unroll
            for (int qn = 0; qn < NKT; ++qn) {
#pragma unroll
                for (int r = 0; r < 4; ++r) S[vt][qn][r] *= gC;
                mma_tile<T, true, true>(S[vt][qn], Et + vt * 16 * LDC, LDC,
                                        Ktt + (wave * NKT + qn) * 16 * LDC, LDC, C, lane);
            }
        __syncthreads();
    }
#pragma unroll
    for (int vt = 0; vt < 2; ++vt)
#pragma unroll
        for (int qn = 0; qn < NKT; ++qn)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int v = vs + vt * 16 + acc_row(lane, r), c = (wave * NKT + qn) * 16 + acc_col(lane);
                a.S_out[(bh * a.V + v) * K + c] = S[vt][qn][r];
            }
}

// ------------------------------------------------------------ output_fwd ----
template <typename T, int K>
__global__ __launch_bounds__(NT) void output_fwd_kernel(ChunkArgs a) {
    constexpr int PAD = Pad<T>::v, LDK = K + PAD, LDC = C + PAD;
    __shared__ __attribute__((aligned(16))) T Qs[C * LDK];
    __shared__ __attribute__((aligned(16))) T Kts[C * LDK];     // K~, later the output staging tile
    __shared__ __attribute__((aligned(16))) T Ss[C * LDK];      // 64 rows of the chunk-start state
    __shared__ __attribute__((aligned(16))) T Ps[C * LDC];      // tril(Gamma . Q K~^T)
    __shared__ __attribute__((aligned(16))) T Ets[C * LDC];     // 64 rows of E^T
    __shared__ float Gs[C];

    const int n = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const size_t bhn = ((size_t)b * a.H + h) * a.N + n;
    const size_t tok0 = ((size_t)b * a.T + (size_t)n * C) * a.H + h;
    const size_t tstride = a.H;

    if (wave == 0) {
        const float g = a.log_alpha ? a.log_alpha[tok0 + (size_t)lane * tstride] : 0.f;
        Gs[lane] = wave_cumsum(g, lane);
    }
    load_tile(Qs, LDK, static_cast<const T *>(a.q) + tok0 * K, tstride * K, C, K, tid, NT);
    load_tile(Kts, LDK, static_cast<const T *>(a.kt) + tok0 * K, tstride * K, C, K, tid, NT);
    __syncthreads();
    // P^T tiles (rows j, columns i) so that the store lands k-contiguous in Ps[i][j]
    for (int idx = wave; idx < 16; idx += 4) {
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
        load_tile(Ss, LDK, static_cast<const T *>(a.S_ckpt) + (bhn * a.V + v0) * K, (size_t)K, C, K, tid, NT);
        load_tile(Ets, LDC, static_cast<const T *>(a.Et) + (bhn * a.V + v0) * C, (size_t)C, C, C, tid, NT);
        __syncthreads();
        const int kdim = min(C, ((wave + 1) * 16 + Mfma<T>::KSTEP - 1) / Mfma<T>::KSTEP * Mfma<T>::KSTEP);
#pragma unroll
        for (int vt = 0; vt < 4; ++vt) {
            f32x4 a1 = {0.f, 0.f, 0.f, 0.f}, a2 = {0.f, 0.f, 0.f, 0.f};
            mma_tile<T, true, true>(a1, Qs + wave * 16 * LDK, LDK, Ss + vt * 16 * LDK, LDK, K, lane);
            mma_tile<T, true, true>(a2, Ps + wave * 16 * LDC, LDC, Ets + vt * 16 * LDC, LDC, kdim, lane);
#pragma unroll
            for (int r = 0; r < 4; ++r)
                a1[r] = a.scale * (__expf(Gs[wave * 16 + acc_row(lane, r)]) * a1[r] + a2[r]);
            store_tile(Os + wave * 16 * LDC + vt * 16, LDC, a1, lane);
        }
        __syncthreads();
        store_tile_global(static_cast<T *>(a.o) + tok0 * a.V + v0, tstride * a.V, Os, LDC, C, C, tid, NT);
    }
}

// -------------------------------------------------------------- launchers ----
template <typename T>
static int launch_prep_t(const ChunkArgs &a, hipStream_t st) {
    dim3 grid(a.N, a.H, a.B), block(NT);
    if (a.K == 64) hipLaunchKernelGGL((chunk_prep_kernel<T, 64>), grid, block, 0, st, a);
    else if (a.K == 128) hipLaunchKernelGGL((chunk_prep_kernel<T, 128>), grid, block, 0, st, a);
    else return -1;
    return 0;
}
int launch_chunk_prep(const ChunkArgs &a, bool bf16_io, hipStream_t st) {
    return bf16_io ? launch_prep_t<bf16>(a, st) : launch_prep_t<float>(a, st);
}
template <typename T>
static int launch_state_t(const ChunkArgs &a, hipStream_t st) {
    dim3 grid((a.V / VS) * a.H * a.B), block(NT);
    if (a.K == 64) hipLaunchKernelGGL((state_fwd_kernel<T, 64>), grid, block, 0, st, a);
    else if (a.K == 128) hipLaunchKernelGGL((state_fwd_kernel<T, 128>), grid, block, 0, st, a);
    else return -1;
    return 0;
}
int launch_state_fwd(const ChunkArgs &a, bool bf16_io, hipStream_t st) {
    return bf16_io ? launch_state_t<bf16>(a, st) : launch_state_t<float>(a, st);
}
template <typename T>
static int launch_output_t(const ChunkArgs &a, hipStream_t st) {
    dim3 grid(a.N, a.H, a.B), block(NT);
    if (a.K == 64) hipLaunchKernelGGL((output_fwd_kernel<T, 64>), grid, block, 0, st, a);
    else if (a.K == 128) hipLaunchKernelGGL((output_fwd_kernel<T, 128>), grid, block, 0, st, a);
    else return -1;
    return 0;
}
int launch_output_fwd(const ChunkArgs &a, bool bf16_io, hipStream_t st) {
    return bf16_io ? launch_output_t<bf16>(a, st) : launch_output_t<float>(a, st);
}

}  // namespace osdn
