// Device-side building blocks shared by the OSDN kernels (gfx950 / CDNA4, wave64).
//
//  - element types: float and __bf16; all accumulation is fp32
//  - MFMA 16x16 tiles: v_mfma_f32_16x16x32_bf16 (8 bf16 per lane and operand) and
//    v_mfma_f32_16x16x4_f32 (1 float per lane and operand).  Both leave the 16x16
//    result in the same place: lane l holds rows 4*(l/16)+r, r=0..3, of column l%16,
//    so every kernel is written once and instantiated for both element types.
//  - wave-level sums and scans by DPP / shuffles
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace osdn {

typedef __bf16 bf16;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16))) uint32_t u32x4;      // 16 raw bytes (a native vector: stays in registers)
typedef __attribute__((__vector_size__(8))) uint32_t u32x2;

constexpr int C = 64;          // chunk length
constexpr int NT = 256;        // threads per workgroup of the chunk kernels (4 waves)

// Default padding of an LDS row: 16 bytes.  Measured per access pattern on bf16 tiles (LDS active
// and bank-conflict cycles per wavefront instruction): a fragment read of 16 bytes per lane along
// k takes 8 cycles at this padding and 4 at 32 bytes; the transpose read 4 per pair at either;
// the 8-byte transposed tile store 8 against 15; the 2-byte tile store 2 against 4.  Kernels whose
// tiles are almost only read along k, and that have the LDS to spare, use 32 bytes instead.
template <typename T> struct Pad { static constexpr int v = 16 / sizeof(T); };

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16 x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float x) { return (bf16)x; }  // RNE

// ------------------------------------------------------------------ MFMA ----
// Operand conventions: an operand tile is addressed as X(row, k) where `row` is the
// M index (A operand) or the N index (B operand) and k the contraction index.
// KCONTIG = true : X(row,k) = base[row*ld + k]   (k contiguous)
// KCONTIG = false: X(row,k) = base[k*ld + row]   (stored transposed)
template <typename T> struct Mfma;

template <> struct Mfma<float> {
    static constexpr int KSTEP = 4;
    typedef float Frag;
    template <bool KCONTIG>
    static __device__ __forceinline__ Frag load(const float *base, int ld, int lane) {
        const int row = lane & 15, kk = lane >> 4;
        return KCONTIG ? base[row * ld + kk] : base[kk * ld + row];
    }
    static __device__ __forceinline__ f32x4 mma(Frag a, Frag b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
};

template <> struct Mfma<bf16> {
    static constexpr int KSTEP = 32;
    typedef bf16x8 Frag;
    template <bool KCONTIG>
    static __device__ __forceinline__ Frag load(const bf16 *base, int ld, int lane) {
        const int row = lane & 15, kk = (lane >> 4) * 8;
        if (KCONTIG) {
            return *reinterpret_cast<const bf16x8 *>(base + row * ld + kk);   // 16-byte aligned by layout
        } else {
            // LDS transpose read (ds_read_b64_tr_b16): inside a group of 16 lanes, lane j passes the
            // address of 4 contiguous 16-bit values, (row j/4, columns 4(j%4)..) of a 4 x 16 block,
            // and receives column j of that block, i.e. 4 consecutive k for its own row index.
            // Two of them give the 8 values of the fragment.  base must be an LDS address with
            // 8-byte aligned rows (ld a multiple of 4).
            typedef short v4s __attribute__((ext_vector_type(4)));
            typedef short v8s __attribute__((ext_vector_type(8)));
            typedef __attribute__((address_space(3))) v4s *lds_v4s;
            const bf16 *p = base + (kk + (row >> 2)) * ld + 4 * (row & 3);
            const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p));
            const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p + 4 * ld));
            return __builtin_bit_cast(Frag, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
    }
    static __device__ __forceinline__ f32x4 mma(Frag a, Frag b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};

// A(16 x kdim) * B(16 x kdim)^T, kdim >= one MFMA step: the first product takes the constant 0
// as its addend (an operand of the instruction), so no accumulator has to be cleared
template <typename T, bool A_KC, bool B_KC>
__device__ __forceinline__ f32x4 mma_tile0(const T *A, int lda, const T *B, int ldb, int kdim, int lane) {
    constexpr int KS = Mfma<T>::KSTEP;
    f32x4 acc = Mfma<T>::mma(Mfma<T>::template load<A_KC>(A, lda, lane), Mfma<T>::template load<B_KC>(B, ldb, lane),
                             f32x4{0.f, 0.f, 0.f, 0.f});
    for (int k0 = KS; k0 < kdim; k0 += KS) {
        typename Mfma<T>::Frag a = Mfma<T>::template load<A_KC>(A_KC ? A + k0 : A + k0 * lda, lda, lane);
        typename Mfma<T>::Frag b = Mfma<T>::template load<B_KC>(B_KC ? B + k0 : B + k0 * ldb, ldb, lane);
        acc = Mfma<T>::mma(a, b, acc);
    }
    return acc;
}

// acc(16x16) += A(16 x kdim) * B(16 x kdim)^T ; A, B point at (row 0, k 0) of their tiles
template <typename T, bool A_KC, bool B_KC>
__device__ __forceinline__ void mma_tile(f32x4 &acc, const T *A, int lda, const T *B, int ldb,
                                         int kdim, int lane) {
    constexpr int KS = Mfma<T>::KSTEP;
    for (int k0 = 0; k0 < kdim; k0 += KS) {
        typename Mfma<T>::Frag a = Mfma<T>::template load<A_KC>(A_KC ? A + k0 : A + k0 * lda, lda, lane);
        typename Mfma<T>::Frag b = Mfma<T>::template load<B_KC>(B_KC ? B + k0 : B + k0 * ldb, ldb, lane);
        acc = Mfma<T>::mma(a, b, acc);
    }
}

// (I + A)^-1 for a strictly lower triangular 64 x 64 A, in fp32 in LDS, in 16 x 16 blocks; only the
// lower blocks of Ti are written (the rest is zero by definition and never stored).  Diagonal
// blocks: forward substitution, one column per lane.  Block (i,j), i > j:
// T_ij = -T_ii sum_{m=j}^{i-1} A_im T_mj, both products on the fp32 MFMA, one wavefront per block.
// Af, Ti: [64][LDF]; Xs: scratch of 3 x 16 x 17 floats.  Every thread of a workgroup of at least
// four wavefronts calls it (it synchronises the workgroup); A must be complete before the call.
template <int LDF>
__device__ __forceinline__ void ut_inverse64(const float *Af, float *Ti, float *Xs, int wave, int lane);

// position of accumulator element r of this lane inside its 16x16 tile
__device__ __forceinline__ int acc_row(int lane, int r) { return ((lane >> 4) << 2) + r; }
__device__ __forceinline__ int acc_col(int lane) { return lane & 15; }

// store a 16x16 accumulator tile into LDS as dst[row*ld + col]  (four scalar stores)
template <typename T>
__device__ __forceinline__ void store_tile(T *dst, int ld, f32x4 acc, int lane) {
#pragma unroll
    for (int r = 0; r < 4; ++r) dst[acc_row(lane, r) * ld + acc_col(lane)] = from_f32<T>(acc[r]);
}
// store transposed, dst[col*ld + row]: the four rows of a lane are contiguous
template <typename T>
__device__ __forceinline__ void store_tile_t(T *dst, int ld, f32x4 acc, int lane);
template <>
__device__ __forceinline__ void store_tile_t<float>(float *dst, int ld, f32x4 acc, int lane) {
    *reinterpret_cast<f32x4 *>(dst + acc_col(lane) * ld + acc_row(lane, 0)) = acc;
}
template <>
__device__ __forceinline__ void store_tile_t<bf16>(bf16 *dst, int ld, f32x4 acc, int lane) {
    bf16x4 v;
#pragma unroll
    for (int r = 0; r < 4; ++r) v[r] = (bf16)acc[r];
    *reinterpret_cast<bf16x4 *>(dst + acc_col(lane) * ld + acc_row(lane, 0)) = v;
}

// acc(row m, col c) = X[m][c0 + c], a 16x16 block of a row-major LDS tile (X points at its
// first row), obtained by multiplying with a 0/1 selector on the MFMA unit (exact).  Followed
// by store_tile_t this transposes a block with vector LDS accesses only.
template <typename T> __device__ __forceinline__ f32x4 pick16(const T *X, int ld, int c0, int lane);
template <> __device__ __forceinline__ f32x4 pick16<float>(const float *X, int ld, int c0, int lane) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const int n = lane & 15, kq = lane >> 4;
#pragma unroll
    for (int s = 0; s < 4; ++s)
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(X[n * ld + c0 + 4 * s + kq], (n == 4 * s + kq) ? 1.f : 0.f,
                                                   acc, 0, 0, 0);
    return acc;
}
template <> __device__ __forceinline__ f32x4 pick16<bf16>(const bf16 *X, int ld, int c0, int lane) {
    const int n = lane & 15, k8 = (lane >> 4) * 8;
    const int kk = c0 & ~31, half = (c0 >> 4) & 1;
    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(X + n * ld + kk + k8);
    bf16x8 sel;
#pragma unroll
    for (int e = 0; e < 8; ++e) sel[e] = (bf16)((k8 + e == n + 16 * half) ? 1.f : 0.f);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, sel, acc, 0, 0, 0);
}

// ------------------------------------------------------- global <-> LDS ----
// element e (compile-time after unrolling) of a 16-byte vector of T held in a u32x4, as fp32
__device__ __forceinline__ uint32_t vec_word(const u32x4 &v, int w) { return v[w]; }
template <typename T> __device__ __forceinline__ float vec_get(const u32x4 &v, int e);
template <> __device__ __forceinline__ float vec_get<float>(const u32x4 &v, int e) {
    return __builtin_bit_cast(float, vec_word(v, e));
}
template <> __device__ __forceinline__ float vec_get<bf16>(const u32x4 &v, int e) {
    const uint32_t w = vec_word(v, e >> 1);
    return __builtin_bit_cast(float, (e & 1) ? (w & 0xffff0000u) : (w << 16));
}

// A tile in global memory is addressed as a wavefront-uniform base pointer plus a 32-bit byte
// offset per lane (one address register per access instead of a 64-bit computation each; the
// library only accepts shapes whose tiles span less than 4 GB).
template <typename T>
__device__ __forceinline__ const u32x4 *tile_vec(const T *g, size_t g_ld, int r, int c) {
    const uint32_t off = ((uint32_t)r * (uint32_t)g_ld + (uint32_t)c) * (uint32_t)sizeof(T);
    return reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(g) + off);
}
template <typename T>
__device__ __forceinline__ u32x4 *tile_vec(T *g, size_t g_ld, int r, int c) {
    const uint32_t off = ((uint32_t)r * (uint32_t)g_ld + (uint32_t)c) * (uint32_t)sizeof(T);
    return reinterpret_cast<u32x4 *>(reinterpret_cast<char *>(g) + off);
}

// The same for single elements: element at a 32-bit byte offset from a wavefront-uniform base,
// and element `lane` of a wavefront-uniform row.
template <typename U>
__device__ __forceinline__ U &at_byte(U *base, uint32_t byte_off) {
    using B = typename std::conditional<std::is_const<U>::value, const char, char>::type;
    return *reinterpret_cast<U *>(reinterpret_cast<B *>(base) + byte_off);
}
template <typename U>
__device__ __forceinline__ U &lane_elem(U *row, int lane_index) {
    return at_byte(row, (uint32_t)lane_index * (uint32_t)sizeof(U));
}

// copy a [rows x cols] tile of T from global (row stride g_ld elements) into LDS (row
// stride s_ld), 16 bytes per thread and step; cols must be a multiple of 16/sizeof(T)
template <typename T>
__device__ __forceinline__ void load_tile(T *s, int s_ld, const T *g, size_t g_ld, int rows,
                                          int cols, int tid, int nthreads) {
    constexpr int VN = 16 / sizeof(T);
    const int vpr = cols / VN;
    for (int i = tid; i < rows * vpr; i += nthreads) {
        const int r = i / vpr, c = (i % vpr) * VN;
        *reinterpret_cast<u32x4 *>(s + r * s_ld + c) = *tile_vec(g, g_ld, r, c);
    }
}
template <typename T>
__device__ __forceinline__ void store_tile_global(T *g, size_t g_ld, const T *s, int s_ld, int rows,
                                                  int cols, int tid, int nthreads) {
    constexpr int VN = 16 / sizeof(T);
    const int vpr = cols / VN;
    for (int i = tid; i < rows * vpr; i += nthreads) {
        const int r = i / vpr, c = (i % vpr) * VN;
        *tile_vec(g, g_ld, r, c) = *reinterpret_cast<const u32x4 *>(s + r * s_ld + c);
    }
}

// 16 bytes of T from floats (4 fp32 or 8 bf16), one vector store
__device__ __forceinline__ void store_vec_t(float *dst, const float (&v)[4]) {
    *reinterpret_cast<f32x4 *>(dst) = f32x4{v[0], v[1], v[2], v[3]};
}
__device__ __forceinline__ void store_vec_t(bf16 *dst, const float (&v)[8]) {
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (bf16)v[e];
    *reinterpret_cast<bf16x8 *>(dst) = o;
}

// acc + <a, b> over 16 bytes of T held in u32x4 (bf16: four two-element dot products in fp32)
template <typename T> __device__ __forceinline__ float dot_vec(const u32x4 &a, const u32x4 &b, float acc);
template <> __device__ __forceinline__ float dot_vec<float>(const u32x4 &a, const u32x4 &b, float acc) {
#pragma unroll
    for (int e = 0; e < 4; ++e) acc = __builtin_fmaf(vec_get<float>(a, e), vec_get<float>(b, e), acc);
    return acc;
}
template <> __device__ __forceinline__ float dot_vec<bf16>(const u32x4 &a, const u32x4 &b, float acc) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int w = 0; w < 4; ++w)
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, vec_word(a, w)),
                                              __builtin_bit_cast(bf16x2, vec_word(b, w)), acc, false);
    return acc;
}

// The same copy in two halves, so that the global loads of a tile can be in flight while the
// workgroup computes on the previous one: tile_fetch issues them into registers, tile_put
// writes the registers into LDS.  NT threads share a [ROWS x COLS] tile.
template <typename T, int ROWS, int COLS, int NT_>
struct TileRegs {
    static constexpr int VN = 16 / sizeof(T), VPR = COLS / VN, TOTAL = ROWS * VPR, NV = (TOTAL + NT_ - 1) / NT_;
    static_assert(TOTAL % NT_ == 0 || NT_ % TOTAL == 0, "tile must split evenly over (some of) the threads");
    u32x4 v[NV];
    __device__ __forceinline__ void fetch(const T *g, size_t g_ld, int tid) {
#pragma unroll
        for (int m = 0; m < NV; ++m) {
            const int i = tid + m * NT_, r = i / VPR, c = (i % VPR) * VN;
            if (TOTAL % NT_ == 0 || i < TOTAL) v[m] = *tile_vec(g, g_ld, r, c);
        }
    }
    __device__ __forceinline__ void put(T *s, int s_ld, int tid) const {
#pragma unroll
        for (int m = 0; m < NV; ++m) {
            const int i = tid + m * NT_, r = i / VPR, c = (i % VPR) * VN;
            if (TOTAL % NT_ == 0 || i < TOTAL) *reinterpret_cast<u32x4 *>(s + r * s_ld + c) = v[m];
        }
    }
};

template <int LDF>
__device__ __forceinline__ void ut_inverse64(const float *Af, float *Ti, float *Xs, int wave, int lane) {
    if (wave < 4 && lane < 16) {
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
        if (wave < 4 - s) {
            const int i = s + wave, j = wave;
            float *xw = Xs + wave * 16 * 17;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            for (int m = j; m < i; ++m)
                mma_tile<float, true, false>(acc, Af + i * 16 * LDF + m * 16, LDF, Ti + m * 16 * LDF + j * 16, LDF, 16, lane);
            store_tile(xw, 17, acc, lane);
            f32x4 t = {0.f, 0.f, 0.f, 0.f};
            mma_tile<float, true, false>(t, Ti + i * 16 * LDF + i * 16, LDF, xw, 17, 16, lane);
#pragma unroll
            for (int r = 0; r < 4; ++r) t[r] = -t[r];
            store_tile(Ti + i * 16 * LDF + j * 16, LDF, t, lane);
        }
        __syncthreads();
    }
}

// --------------------------------------------------------- wave helpers ----
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_f32(float src, float old = 0.f) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, old),
                                                                 __builtin_bit_cast(int, src), CTRL,
                                                                 ROW_MASK, 0xF, false));
}
// sum over the 64 lanes, returned to every lane (fixed reduction tree => deterministic)
__device__ __forceinline__ float wave_sum(float x) {
    x += dpp_f32<0xB1>(x);         // quad_perm [1,0,3,2]
    x += dpp_f32<0x4E>(x);         // quad_perm [2,3,0,1]
    x += dpp_f32<0x141>(x);        // row_half_mirror
    x += dpp_f32<0x140>(x);        // row_mirror: every lane of a row of 16 holds the row sum
    x += dpp_f32<0x142, 0xA>(x);   // row_bcast:15 into rows 1 and 3
    x += dpp_f32<0x143, 0xC>(x);   // row_bcast:31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}

// the value of lane 63, in every lane
__device__ __forceinline__ float lane_bcast63(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}
// inclusive prefix sum over the 64 lanes of a wave
__device__ __forceinline__ float wave_cumsum(float x, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        float y = __shfl_up(x, off, 64);
        if (lane >= off) x += y;
    }
    return x;
}
// exclusive-from-the-right ("suffix") inclusive sum: out[l] = sum_{m >= l} x[m]
__device__ __forceinline__ float wave_suffix_sum(float x, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        float y = __shfl_down(x, off, 64);
        if (lane + off < 64) x += y;
    }
    return x;
}

// offsets into the caller's [B,T,H,D] tensors and the library's per-chunk tiles
__device__ __forceinline__ size_t tok_off(int b, int t, int h, int T, int H, int D) {
    return (((size_t)b * T + t) * H + h) * (size_t)D;
}

// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  The chain kernels
// run V/VS workgroups per (batch, head) chain that all read the same W / K~ / Q tiles: this
// maps a 1-D workgroup id so that the slices of one chain share an XCD (and its L2).
constexpr int NUM_XCD = 8;
__device__ __forceinline__ void chain_slice_of(int wg, int nslices, int nchains, int &chain, int &slice) {
    if (nchains % NUM_XCD == 0) {
        const int xcd = wg % NUM_XCD, j = wg / NUM_XCD;
        slice = j % nslices;
        chain = xcd + NUM_XCD * (j / nslices);
    } else {
        slice = wg % nslices;
        chain = wg / nslices;
    }
}


// Packed sequences: clip the chunk range [n0, n1) of a launch to the chunks of sequence s.
// begins / ends: the sequence starts / stops inside the launch's range.  False: nothing left.
__device__ __forceinline__ bool clip_to_sequence(const int *seq_chunks, int s, int &n0, int &n1, bool &begins,
                                                 bool &ends) {
    const int cb = seq_chunks[s], ce = seq_chunks[s + 1];
    begins = cb >= n0;
    ends = ce <= n1;
    n0 = max(n0, cb);
    n1 = min(n1, ce);
    return n0 < n1;
}

}  // namespace osdn
