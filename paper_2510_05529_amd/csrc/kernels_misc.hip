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

// Grid-stride read, 4 independent 16-byte loads per lane per step, XOR-folded so the loads cannot be elided.
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4 *__restrict__ src, size_t n16, uint4 *__restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        acc.x ^= a.x ^ b.x ^ c.x ^ d.x;
        acc.y ^= a.y ^ b.y ^ c.y ^ d.y;
        acc.z ^= a.z ^ b.z ^ c.z ^ d.z;
        acc.w ^= a.w ^ b.w ^ c.w ^ d.w;
    }
    for (; i < n16; i += stride) {
        const uint4 a = src[i];
        acc.x ^= a.x; acc.y ^= a.y; acc.z ^= a.z; acc.w ^= a.w;
    }
    // one store per workgroup: fold the lanes through the first lane of each wave
    for (int off = 32; off > 0; off >>= 1) {
        acc.x ^= __shfl_xor(acc.x, off); acc.y ^= __shfl_xor(acc.y, off);
        acc.z ^= __shfl_xor(acc.z, off); acc.w ^= __shfl_xor(acc.w, off);
    }
    __shared__ uint4 part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0)
        sink[blockIdx.x] = make_uint4(part[0].x ^ part[1].x ^ part[2].x ^ part[3].x, part[0].y ^ part[1].y ^ part[2].y ^ part[3].y,
                                      part[0].z ^ part[1].z ^ part[2].z ^ part[3].z, part[0].w ^ part[1].w ^ part[2].w ^ part[3].w);
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

hipError_t launch_stream_read(const void *src, size_t n_bytes, void *sink, hipStream_t st) {
    const size_t n16 = n_bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 8192) blocks = 8192;                     // sink holds 8192 x 16 bytes
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<const uint4 *>(src), n16,
                       static_cast<uint4 *>(sink));
    return hipGetLastError();
}

}  // namespace h1bkv
