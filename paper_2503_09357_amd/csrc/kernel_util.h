// Small helper kernels: layout conversion and counter reset.
#pragma once

#include "device_common.h"

namespace dagsched_dev {

// [rows][cols] int32 -> [cols][rows], 64x64 tiles through LDS (both sides coalesced)
__global__ __launch_bounds__(256) void transpose_i32_kernel(const int32_t *__restrict__ in, int32_t *__restrict__ out,
                                                             int64_t rows, int64_t cols) {
  __shared__ int32_t tile[64][65];
  const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4) {
    int64_t r = r0 + i, cc = c0 + tx;
    if (r < rows && cc < cols) tile[i][tx] = in[r * cols + cc];
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    int64_t cc = c0 + i, r = r0 + tx;
    if (r < rows && cc < cols) out[cc * rows + r] = tile[tx][i];
  }
}

// A fill kernel instead of a memset node: safe to record into a captured graph.
__global__ void reset_counter_kernel(int32_t *counter) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *counter = 0;
}

}  // namespace dagsched_dev
