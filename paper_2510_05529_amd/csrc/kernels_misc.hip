// Small utility kernels: block-table publication and the calibration copy.
#include "internal.h"

namespace h1bkv {

namespace {

// New (sequence, page slot) -> page assignments travel as a kernel argument and are written into the
// device block table in stream order, so the append/decode kernels behind it see them.
__global__ void publish_kernel(TablePairs tp, int32_t *block_table) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < tp.n) block_table[tp.index[i]] = tp.page[i];
}

// Grid-stride copy, 16 bytes per lane per step.
__global__ __launch_bounds__(256) void stream_copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

hipError_t launch_publish(const TablePairs &pairs, int32_t *block_table, hipStream_t st) {
    hipLaunchKernelGGL(publish_kernel, dim3(1), dim3(256), 0, st, pairs, block_table);
    return hipGetLastError();
}

hipError_t launch_stream_copy(void *dst, const void *src, size_t n_bytes, hipStream_t st) {
    const size_t n16 = n_bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(stream_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<uint4 *>(dst),
                       static_cast<const uint4 *>(src), n16);
    return hipGetLastError();
}

}  // namespace h1bkv
