// Small memory kernels: arena clear, per-sequence metadata upload, and the prefill cache
// writer that stores K/V rows (text rows only in a lazy layer) and the Q Cache rows.
#include "qc_device.h"

namespace qc {

__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* p, size_t n16, unsigned char* tail, int ntail) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const uint4 z = {0u, 0u, 0u, 0u};
  for (; i < n16; i += stride) p[i] = z;
  if (blockIdx.x == 0 && (int)threadIdx.x < ntail) tail[threadIdx.x] = 0;
}

hipError_t launch_fill_zero(void* dev, size_t bytes, hipStream_t stream) {
  if (bytes == 0) return hipSuccess;
  size_t n16 = bytes / 16;
  int ntail = (int)(bytes % 16);
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  if (blocks == 0) blocks = 1;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (uint4*)dev, n16,
                     (unsigned char*)dev + n16 * 16, ntail);
  return hipGetLastError();
}

// *counter = add ? *counter + value : value (one lane): the decode-step counter a replayed graph reads.
__global__ void counter_update_kernel(int32_t* counter, int32_t value, int32_t add) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *counter = add ? *counter + value : value;
}

hipError_t launch_counter_update(int32_t* counter, int32_t value, int32_t add, hipStream_t stream) {
  hipLaunchKernelGGL(counter_update_kernel, dim3(1), dim3(64), 0, stream, counter, value, add);
  return hipGetLastError();
}

__global__ void meta_upload_kernel(int32_t* meta, int32_t max_batch, int32_t first, int32_t count, int32_t rows, MetaChunk c) {
  int i = threadIdx.x;
  if (i < count)
    for (int r = 0; r < rows; ++r) meta[r * max_batch + first + i] = c.v[r][i];
}

hipError_t launch_meta_upload(int32_t* meta_dev, int32_t max_batch, int32_t first, int32_t count, int32_t rows,
                              const MetaChunk& chunk, hipStream_t stream) {
  hipLaunchKernelGGL(meta_upload_kernel, dim3(1), dim3(MetaChunk::N), 0, stream, meta_dev, max_batch, first,
                     count, rows, chunk);
  return hipGetLastError();
}

}  // namespace qc
