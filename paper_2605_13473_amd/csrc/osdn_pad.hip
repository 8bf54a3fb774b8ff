// Sequences whose length is not a multiple of the chunk length are padded on the way in and
// cut on the way out: the pad tokens (k = q = v = dO = 0, beta = 0, log alpha = 0, retention = 1)
// leave d and S, and every adjoint that passes through them, exactly as they are.
#include "osdn_kernels.h"

namespace osdn {

// dst[b][t][:] = t < Ts ? src[b][t][:] : fill, for t < Td; rows of wpr 32-bit words
__global__ __launch_bounds__(256) void copy_rows_kernel(const uint32_t *src, int Ts, uint32_t *dst, int Td,
                                                         uint32_t wpr, uint32_t fill, size_t total) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const size_t row = i / wpr;
        const uint32_t w = (uint32_t)(i % wpr);
        const size_t b = row / Td;
        const int t = (int)(row % Td);
        dst[i] = t < Ts ? src[(b * Ts + t) * wpr + w] : fill;
    }
}

int launch_copy_rows(const void *src, int Ts, void *dst, int Td, int B, size_t row_bytes, uint32_t fill,
                     hipStream_t st) {
    if (row_bytes % 4 != 0) return -1;
    const uint32_t wpr = (uint32_t)(row_bytes / 4);
    const size_t total = (size_t)B * Td * wpr;
    const size_t blocks = (total + 255) / 256;
    hipLaunchKernelGGL(copy_rows_kernel, dim3((unsigned)(blocks < 65535 * 16 ? blocks : 65535 * 16)), dim3(256), 0, st,
                       static_cast<const uint32_t *>(src), Ts, static_cast<uint32_t *>(dst), Td, wpr, fill, total);
    return 0;
}

}  // namespace osdn
