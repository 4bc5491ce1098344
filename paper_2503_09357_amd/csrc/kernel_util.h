// Small helper kernels: layout conversion, counter reset, missing-channel flags.
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
__global__ void reset_counter_kernel(int32_t *counter) {        // two words: the lists of the first and second fallback
  if (threadIdx.x == 0 && blockIdx.x == 0) { counter[0] = 0; counter[1] = 0; }
}

// Missing channels (Sec. III eqs. (9)-(10)), run after the evaluation when the cluster graph lacks some pair: one
// workgroup per candidate copies the candidate's placement into LDS as bytes (one coalesced pass over the row) and
// walks the edge list (u | v << 16, one coalesced dword per edge); an edge whose ends sit on machines a != b with
// bit b of no_channel[a] set makes the candidate NO_CHANNEL, unless it is malformed already (then its placement
// may not even be in range).  placement is candidate-major, N entries per candidate.  Dynamic LDS: 512 + N bytes;
// any workgroup size that is a multiple of 64.
__global__ __launch_bounds__(1024) void channel_flag_kernel(int32_t N, int32_t E, int32_t P,
                                                            const uint32_t *__restrict__ edges,
                                                            const uint64_t *__restrict__ no_channel,
                                                            const int32_t *__restrict__ placement, OutPtrs out) {
  extern __shared__ __align__(16) unsigned char channel_lds[];
  uint64_t *mask = reinterpret_cast<uint64_t *>(channel_lds);
  uint8_t *machine = channel_lds + DAGSCHED_MAX_DEVICES * sizeof(uint64_t);
  const int64_t c = blockIdx.x;
  const int32_t before = out.flags[c];
  if (before == DAGSCHED_FLAG_BAD_PLACEMENT || before == DAGSCHED_FLAG_BAD_RANK) return;   // uniform over the workgroup
  if ((int)threadIdx.x < DAGSCHED_MAX_DEVICES) mask[threadIdx.x] = (int)threadIdx.x < P ? no_channel[threadIdx.x] : 0;
  const int32_t *pl = placement + c * N;
  for (int32_t v = threadIdx.x; v < N; v += blockDim.x) machine[v] = (uint8_t)pl[v];
  __syncthreads();
  int found = 0;
#pragma unroll 4
  for (int32_t k = threadIdx.x; k < E; k += blockDim.x) {
    const uint32_t e = edges[k];
    const uint32_t a = machine[e & 0xFFFFu], b = machine[e >> 16];
    found |= (a != b) && ((mask[a] >> b) & 1u);
  }
  if (!__syncthreads_or(found)) return;
  if (threadIdx.x == 0) {
    out.flags[c] = DAGSCHED_FLAG_NO_CHANNEL;
    out.makespan[c] = -1;
    out.bubble[c] = -1;
  }
  if ((int)threadIdx.x < P) out.peak_mem[c * out.peak_stride_c + threadIdx.x * out.peak_stride_j] = -1;
}

}  // namespace dagsched_dev
