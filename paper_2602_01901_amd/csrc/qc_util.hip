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

__global__ void table_upload_kernel(int32_t* tables, int32_t count, TableChunk c) {
  const int i = threadIdx.x;
  if (i < count) tables[c.at[i]] = c.page[i];
}

hipError_t launch_table_upload(int32_t* tables, int32_t count, const TableChunk& chunk, hipStream_t stream) {
  if (count == 0) return hipSuccess;
  hipLaunchKernelGGL(table_upload_kernel, dim3(1), dim3(TableChunk::N), 0, stream, tables, count, chunk);
  return hipGetLastError();
}

// Moves the rows of one sequence inside up to MoveChunk::N regions (qc_seq_grow): region i holds, per
// head, `rows[i]` rows of row_bytes at src[i] + h*src_stride[i] that go to dst[i] + h*dst_stride[i]
// (byte offsets from `base`).  One workgroup per (region, head), 16 bytes per lane.  Source and
// destination never overlap.
__global__ __launch_bounds__(256) void move_rows_kernel(char* base0, char* base1, int32_t row_bytes, MoveChunk c) {
  const int i = blockIdx.x, h = blockIdx.y;
  char* base = c.arena[i] ? base1 : base0;
  const int64_t n16 = (int64_t)c.rows[i] * row_bytes / 16;
  const uint4* src = (const uint4*)(base + c.src[i] + (int64_t)h * c.src_stride[i]);
  uint4* dst = (uint4*)(base + c.dst[i] + (int64_t)h * c.dst_stride[i]);
  for (int64_t j = threadIdx.x; j < n16; j += 256) dst[j] = src[j];
}

hipError_t launch_move_rows(void* arena0, void* arena1, int32_t row_bytes, int32_t n_heads, int32_t count,
                            const MoveChunk& chunk, hipStream_t stream) {
  if (count == 0) return hipSuccess;
  hipLaunchKernelGGL(move_rows_kernel, dim3(count, n_heads), dim3(256), 0, stream, (char*)arena0, (char*)arena1,
                     row_bytes, chunk);
  return hipGetLastError();
}

}  // namespace qc
