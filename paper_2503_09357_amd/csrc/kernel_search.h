// Helpers for a planner that searches with the evaluator in its loop (the part a MIP solver plays in
// Sec. IV-V): a one-move neighbourhood of a base schedule, the choice of the best feasible candidate,
// and the start/end times of one schedule for a Gantt chart (cf. the charts of Sec. V).
#pragma once

#include "device_common.h"

namespace dagsched_dev {

// operations per machine of the base schedule (placements outside [0, P) are not counted)
__global__ __launch_bounds__(256) void machine_count_kernel(int32_t N, int32_t P, const int32_t *__restrict__ pl,
                                                             int32_t *__restrict__ cnt) {
  __shared__ int32_t h[DAGSCHED_MAX_DEVICES];
  if (threadIdx.x < DAGSCHED_MAX_DEVICES) h[threadIdx.x] = 0;
  __syncthreads();
  for (int i = threadIdx.x; i < N; i += blockDim.x) {
    const int32_t m = pl[i];
    if ((uint32_t)m < (uint32_t)P) atomicAdd(&h[m], 1);
  }
  __syncthreads();
  if (threadIdx.x < DAGSCHED_MAX_DEVICES) cnt[threadIdx.x] = h[threadIdx.x];
}

struct ProposeParams {
  int32_t N, P, C;
  const int32_t *base_pl, *base_rk;    // [N]
  const uint32_t *rnd;                 // [4 * C]
  const int32_t *cnt;                  // [P] operations per machine of the base
  int32_t *out_pl, *out_rk;            // entry (c, i) at c * stride_c + i * stride_n
  int64_t stride_c, stride_n;
  int32_t orders_only;                 // 1: moves stay on the operation's machine
};

// Candidate 0 = the base.  Candidate c >= 1 = the base with one move, (r0, r1, r2, r3) = rnd[4c .. 4c+3],
// v = r1 mod N on machine m at rank r:
//   r0 even: v trades places with the operation after it on m (nothing if it is the last);
//   r0 odd:  m2 = r2 mod P; m2 == m: v is re-inserted at position r3 mod n_m of m;
//            m2 != m: v is inserted at position r3 mod (n_m2 + 1) of m2.
// orders_only: m2 = m whatever r2 is (the candidates keep the base's placement).
// One workgroup per candidate; the move is the same for every thread, each thread rewrites some operations.
__global__ __launch_bounds__(256) void propose_kernel(ProposeParams p) {
  const int c = blockIdx.x;
  const int N = p.N;
  enum { kNone, kSwap, kWithin, kAcross };
  int mode = kNone;
  int32_t v = 0, m = 0, r = 0, m2 = 0, r_new = 0;
  if (c > 0) {
    const uint32_t r0 = p.rnd[4 * (int64_t)c], r1 = p.rnd[4 * (int64_t)c + 1], r2 = p.rnd[4 * (int64_t)c + 2],
                   r3 = p.rnd[4 * (int64_t)c + 3];
    v = (int32_t)(r1 % (uint32_t)N);
    m = p.base_pl[v];
    r = p.base_rk[v];
    if ((uint32_t)m < (uint32_t)p.P) {                      // a base outside the model is copied unchanged
      const int32_t n_m = p.cnt[m];
      if ((r0 & 1u) == 0u) {
        if (r + 1 < n_m) mode = kSwap;
      } else {
        m2 = p.orders_only ? m : (int32_t)(r2 % (uint32_t)p.P);
        if (m2 == m) {
          r_new = (int32_t)(r3 % (uint32_t)n_m);
          mode = kWithin;
        } else {
          r_new = (int32_t)(r3 % (uint32_t)(p.cnt[m2] + 1));
          mode = kAcross;
        }
      }
    }
  }
  for (int i = threadIdx.x; i < N; i += blockDim.x) {
    int32_t pl = p.base_pl[i], rk = p.base_rk[i];
    if (mode == kSwap) {
      if (i == v) rk = r + 1;
      else if (pl == m && rk == r + 1) rk = r;
    } else if (mode == kWithin) {
      if (i == v) rk = r_new;
      else if (pl == m) {
        if (r_new > r && rk > r && rk <= r_new) --rk;
        else if (r_new < r && rk >= r_new && rk < r) ++rk;
      }
    } else if (mode == kAcross) {
      if (i == v) { pl = m2; rk = r_new; }
      else if (pl == m && rk > r) --rk;
      else if (pl == m2 && rk >= r_new) ++rk;
    }
    const int64_t at = (int64_t)c * p.stride_c + (int64_t)i * p.stride_n;
    p.out_pl[at] = pl;
    p.out_rk[at] = rk;
  }
}

// best[0] = index of the feasible (flag 0) candidate with the least makespan, the lowest index among
// equals; best[1] = its makespan; (-1, -1) when none is feasible.  One workgroup.
__global__ __launch_bounds__(1024) void select_kernel(int32_t C, const int32_t *__restrict__ makespan,
                                                       const int32_t *__restrict__ flags, int32_t *__restrict__ best) {
  __shared__ unsigned long long s_key[16];
  unsigned long long key = ~0ull;                          // makespan << 32 | index: one unsigned min does both
  for (int c = threadIdx.x; c < C; c += blockDim.x)
    if (flags[c] == 0) key = min(key, ((unsigned long long)(uint32_t)makespan[c] << 32) | (uint32_t)c);
  for (int d = 1; d < kWave; d <<= 1) {
    const unsigned long long o = __shfl_xor(key, d, kWave);
    key = min(key, o);
  }
  if ((threadIdx.x & 63) == 0) s_key[threadIdx.x >> 6] = key;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < (int)(blockDim.x >> 6); ++w) key = min(key, s_key[w]);
    best[0] = (key == ~0ull) ? -1 : (int32_t)(uint32_t)key;
    best[1] = (key == ~0ull) ? -1 : (int32_t)(key >> 32);
  }
}

// start / end times of one evaluated schedule from the end-time array the general kernel left in its
// workspace; -1 everywhere when the schedule carries a flag.
__global__ __launch_bounds__(256) void schedule_out_kernel(int32_t N, const int32_t *__restrict__ dur,
                                                            const int32_t *__restrict__ end_ws,
                                                            const int32_t *__restrict__ flag_in, int32_t *__restrict__ start,
                                                            int32_t *__restrict__ end, int32_t *__restrict__ flag_out) {
  const int flag = *flag_in;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < N; i += gridDim.x * blockDim.x) {
    const int32_t e = end_ws[i];
    start[i] = flag ? -1 : e - dur[i];
    end[i] = flag ? -1 : e;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) *flag_out = flag;
}

}  // namespace dagsched_dev
