// Sequences whose length is not a multiple of the chunk length are padded on the way in and
// cut on the way out: the pad tokens (k = q = v = dO = 0, beta = 0, log alpha = 0, retention = 1)
// leave d and S, and every adjoint that passes through them, exactly as they are.
#include "osdn_kernels.h"

namespace osdn {

// Rows are moved in 16-byte words when the row length and both base addresses allow it, else
// in 4-byte words (W = uint4 or uint32_t; the fill value is a 32-bit pattern either way).
__device__ __forceinline__ void splat(uint32_t &w, uint32_t fill) { w = fill; }
__device__ __forceinline__ void splat(uint4 &w, uint32_t fill) { w = make_uint4(fill, fill, fill, fill); }
inline bool wide_ok(const void *a, const void *b, size_t row_bytes) {
    return row_bytes % 16 == 0 && (reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b)) % 16 == 0;
}
inline dim3 copy_grid(size_t total) {
    const size_t blocks = (total + 255) / 256;
    return dim3((unsigned)(blocks < 65535 * 16 ? blocks : 65535 * 16));
}

// dst[b][t][:] = t < Ts ? src[b][t][:] : fill, for t < Td; rows of wpr words
template <typename W>
__global__ __launch_bounds__(256) void copy_rows_kernel(const W *src, int Ts, W *dst, int Td, uint32_t wpr,
                                                         uint32_t fill, size_t total) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const size_t row = i / wpr;
        const uint32_t w = (uint32_t)(i % wpr);
        const size_t b = row / Td;
        const int t = (int)(row % Td);
        W val;
        splat(val, fill);
        if (t < Ts) val = src[(b * Ts + t) * wpr + w];
        dst[i] = val;
    }
}

int launch_copy_rows(const void *src, int Ts, void *dst, int Td, int B, size_t row_bytes, uint32_t fill,
                     hipStream_t st) {
    if (row_bytes % 4 != 0) return -1;
    if (wide_ok(src, dst, row_bytes)) {
        const uint32_t wpr = (uint32_t)(row_bytes / 16);
        const size_t total = (size_t)B * Td * wpr;
        hipLaunchKernelGGL(copy_rows_kernel<uint4>, copy_grid(total), dim3(256), 0, st, static_cast<const uint4 *>(src),
                           Ts, static_cast<uint4 *>(dst), Td, wpr, fill, total);
    } else {
        const uint32_t wpr = (uint32_t)(row_bytes / 4);
        const size_t total = (size_t)B * Td * wpr;
        hipLaunchKernelGGL(copy_rows_kernel<uint32_t>, copy_grid(total), dim3(256), 0, st,
                           static_cast<const uint32_t *>(src), Ts, static_cast<uint32_t *>(dst), Td, wpr, fill, total);
    }
    return 0;
}

// ---- packed sequences -------------------------------------------------------------------
// Sequences packed back to back on one token axis are moved so that each starts on a chunk
// boundary.  Two small tables, one entry per chunk of the padded axis, describe the move:
// chunk_row[c] = packed row of the chunk's first token, chunk_len[c] = its tokens (1..64).

// small host arrays reach the device as kernel arguments: nothing to keep alive, no copy engine
constexpr int UPLOAD_INTS = 512;
struct IntBlock { int v[UPLOAD_INTS]; };
__global__ __launch_bounds__(256) void upload_ints_kernel(IntBlock blk, int count, int *dst) {
    for (int i = threadIdx.x; i < count; i += blockDim.x) dst[i] = blk.v[i];
}

int launch_upload_ints(const int *host, size_t count, int *dst, hipStream_t st) {
    for (size_t at = 0; at < count; at += UPLOAD_INTS) {
        IntBlock blk;
        const int n = (int)(count - at < (size_t)UPLOAD_INTS ? count - at : (size_t)UPLOAD_INTS);
        for (int i = 0; i < UPLOAD_INTS; ++i) blk.v[i] = i < n ? host[at + i] : 0;
        hipLaunchKernelGGL(upload_ints_kernel, dim3(1), dim3(256), 0, st, blk, n, dst + at);
    }
    return 0;
}

// to_padded: padded[c*64 + t][:] = t < chunk_len[c] ? packed[chunk_row[c] + t][:] : fill
// otherwise: packed[chunk_row[c] + t][:] = padded[c*64 + t][:] for t < chunk_len[c]
template <typename W, bool TO_PADDED>
__global__ __launch_bounds__(256) void move_chunk_rows_kernel(const W *src, W *dst, const int *chunk_row,
                                                               const int *chunk_len, uint32_t wpr, uint32_t fill,
                                                               size_t total) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const size_t row = i / wpr;
        const uint32_t w = (uint32_t)(i % wpr);
        const size_t c = row / C;
        const int t = (int)(row % C);
        const bool valid = t < chunk_len[c];
        const size_t packed = ((size_t)chunk_row[c] + t) * wpr + w;
        if (TO_PADDED) {
            W val;
            splat(val, fill);
            if (valid) val = src[packed];
            dst[i] = val;
        } else if (valid) {
            dst[packed] = src[i];
        }
    }
}

template <typename W>
static void launch_move_t(const void *src, void *dst, const int *chunk_row, const int *chunk_len, int n_chunks,
                          size_t row_bytes, bool to_padded, uint32_t fill, hipStream_t st) {
    const uint32_t wpr = (uint32_t)(row_bytes / sizeof(W));
    const size_t total = (size_t)n_chunks * C * wpr;
    if (to_padded)
        hipLaunchKernelGGL((move_chunk_rows_kernel<W, true>), copy_grid(total), dim3(256), 0, st,
                           static_cast<const W *>(src), static_cast<W *>(dst), chunk_row, chunk_len, wpr, fill, total);
    else
        hipLaunchKernelGGL((move_chunk_rows_kernel<W, false>), copy_grid(total), dim3(256), 0, st,
                           static_cast<const W *>(src), static_cast<W *>(dst), chunk_row, chunk_len, wpr, fill, total);
}

int launch_move_chunk_rows(const void *src, void *dst, const int *chunk_row, const int *chunk_len, int n_chunks,
                           size_t row_bytes, bool to_padded, uint32_t fill, hipStream_t st) {
    if (row_bytes % 4 != 0) return -1;
    if (wide_ok(src, dst, row_bytes))
        launch_move_t<uint4>(src, dst, chunk_row, chunk_len, n_chunks, row_bytes, to_padded, fill, st);
    else
        launch_move_t<uint32_t>(src, dst, chunk_row, chunk_len, n_chunks, row_bytes, to_padded, fill, st);
    return 0;
}

}  // namespace osdn
