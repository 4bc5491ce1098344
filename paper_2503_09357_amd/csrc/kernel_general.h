// General evaluation kernel: any N, any time range (int32 end times).  It is the fallback of the
// ring kernel (candidates whose 16-bit state saturated or stalled) and the main path for problems
// the ring kernel does not take.  End-time state in LDS when it fits, else in a global workspace.
//
// One wavefront per workgroup, G = 64 / Pseg candidates per wavefront, lane = (candidate, machine).
// Edge-granular polling: per round a lane consumes at most one DAG predecessor of the head operation
// of its machine's order list and completes the operation once all predecessors have ended:
//   s_v = max(0, e_chainpred, max_u e_u + delta(u,v)), e_v = s_v + D^o_v   (eqs. (3),(7),(11)-(13), Sec. III)
#pragma once

#include "device_common.h"

namespace dagsched_dev {

struct GeneralParams {
  int32_t N, P, Pseg, G, C;
  int64_t row_stride;          // elements between consecutive candidates in list / end workspaces
  const int32_t *pred_ptr;     // [N+1] predecessor CSR of B
  const int32_t *pred_idx;     // [E]
  const int32_t *dur;          // [N]
  const int32_t *comm;         // [P*P]
  const int64_t *mem_delta;    // [N]
  const int64_t *weight;       // [N] static memory per operation (eq. (16)), or NULL
  const int64_t *mem_limit;    // [P] memory limit per machine, or NULL
  int64_t sum_dur;
  const int32_t *placement;    // [C][N] candidate-major
  const int32_t *rank;         // [C][N]
  int32_t *ws_list;            // [C][row_stride] order lists, machine after machine
  int32_t *ws_end;             // [C][row_stride] end times (global-state variant)
  const int32_t *cand_list;    // optional: evaluate only candidates cand_list[0 .. *cand_count)
  const int32_t *cand_count;
  OutPtrs out;
};

template <bool LDS_STATE>
__global__ __launch_bounds__(kWave) void relax_general_kernel(GeneralParams p) {
  extern __shared__ int32_t smem[];
  __shared__ int32_t s_cnt[kWave];
  __shared__ int32_t s_off[kWave];
  __shared__ int32_t s_flag[kWave];
  __shared__ int32_t s_cand[kWave];

  const int lane = threadIdx.x;
  const int N = p.N, P = p.P, Pseg = p.Pseg, G = p.G;
  const int64_t total = p.cand_list ? (int64_t)*p.cand_count : (int64_t)p.C;
  const int64_t first = (int64_t)blockIdx.x * G;
  if (first >= total) return;
  const int ng = (int)min((int64_t)G, total - first);
  const int g = lane / Pseg, j = lane % Pseg;

  s_cnt[lane] = 0;
  s_flag[lane] = 0;
  if (lane < ng) s_cand[lane] = p.cand_list ? p.cand_list[first + lane] : (int32_t)(first + lane);
  __syncthreads();

  // placement in range (eq. (6)); count operations per machine; reset the end-time state
  for (int gg = 0; gg < ng; ++gg) {
    const int64_t c = s_cand[gg];
    const int32_t *pl = p.placement + c * N;
    int32_t *end_g = LDS_STATE ? (smem + (size_t)gg * N) : (p.ws_end + c * p.row_stride);
    for (int v = lane; v < N; v += kWave) {
      int32_t pi = pl[v];
      if ((uint32_t)pi >= (uint32_t)P) atomicOr(&s_flag[gg], kBitBadPlacement);
      else atomicAdd(&s_cnt[gg * Pseg + pi], 1);
      if (LDS_STATE) end_g[v] = -1; else st_agent(end_g + v, -1);
    }
  }
  __syncthreads();
  // exclusive prefix over the machines of each candidate: start of machine j inside the list
  {
    int my = s_cnt[lane], incl = my;
    for (int d = 1; d < Pseg; d <<= 1) {
      int t = __shfl_up(incl, d, Pseg);
      if (j >= d) incl += t;
    }
    s_off[lane] = incl - my;
  }
  __syncthreads();
  // order lists list_j[rank] = operation (the fixed disjunctive arcs u of eqs. (7),(17)-(18))
  for (int gg = 0; gg < ng; ++gg) {
    if (s_flag[gg] & kBitBadPlacement) continue;
    const int64_t c = s_cand[gg];
    const int32_t *pl = p.placement + c * N;
    const int32_t *rk = p.rank + c * N;
    int32_t *list = p.ws_list + c * p.row_stride;
    for (int v = lane; v < N; v += kWave) {
      int32_t pi = pl[v], r = rk[v];
      if ((uint32_t)r >= (uint32_t)s_cnt[gg * Pseg + pi]) atomicOr(&s_flag[gg], kBitBadRank);
      else st_agent(list + s_off[gg * Pseg + pi] + r, v);
    }
  }
  __syncthreads();                   // workgroup scope is enough: one wavefront writes and reads these lists
  // every (machine, rank) slot must be hit exactly once: a slot written twice keeps one writer only
  for (int gg = 0; gg < ng; ++gg) {
    if (s_flag[gg]) continue;
    const int64_t c = s_cand[gg];
    const int32_t *pl = p.placement + c * N;
    const int32_t *rk = p.rank + c * N;
    const int32_t *list = p.ws_list + c * p.row_stride;
    for (int v = lane; v < N; v += kWave) {
      if (ld_agent(list + s_off[gg * Pseg + pl[v]] + rk[v]) != v) atomicOr(&s_flag[gg], kBitBadRank);
    }
  }
  __syncthreads();

  // relaxation, lane = (candidate g, machine j)
  const bool lane_valid = (g < ng) && (j < P);
  const int64_t c = lane_valid ? s_cand[g] : s_cand[0];
  const int32_t *pl = p.placement + c * N;
  const int32_t *list = p.ws_list + c * p.row_stride;
  int32_t *end_g = LDS_STATE ? (smem + (size_t)(lane_valid ? g : 0) * N) : (p.ws_end + c * p.row_stride);
  int k = 0, kend = 0;
  if (lane_valid && s_flag[g] == 0) {
    k = s_off[lane];
    kend = k + s_cnt[lane];
  }
  bool active = k < kend;
  int v = 0, pp = 0, pe = 0;
  if (active) {
    v = ld_agent(list + k);
    pp = p.pred_ptr[v];
    pe = p.pred_ptr[v + 1];
  }
  int32_t acc = 0;              // time at which machine j becomes free (end of its previous operation)
  int64_t level = 0, peak = 0;  // running memory level on machine j above its base level, and its maximum
  int64_t base = 0;             // static memory of everything placed on machine j (eq. (16))
  const uint64_t segmask = ((Pseg == kWave) ? ~0ull : ((1ull << Pseg) - 1ull)) << (g * Pseg);
  const int64_t max_rounds = (int64_t)N + p.pred_ptr[N] + 4;

  for (int64_t round = 0; round < max_rounds; ++round) {
    bool progressed = false;
    if (active) {
      if (pp < pe) {
        int u = p.pred_idx[pp];
        int32_t eu = LDS_STATE ? end_g[u] : ld_agent(end_g + u);
        if (eu >= 0) {   // predecessor has ended: s_v >= e_u + delta(u, v), eqs. (11)-(13)
          int pu = pl[u];
          int32_t d = (pu != j) ? p.comm[pu * P + j] : 0;
          acc = max(acc, eu + d);
          ++pp;
          progressed = true;
        }
      }
      if (pp == pe) {      // all inputs have arrived and the machine is free: run v (eq. (3))
        int32_t e = acc + p.dur[v];
        if (LDS_STATE) end_g[v] = e; else st_agent(end_g + v, e);
        acc = e;
        level += p.mem_delta[v];      // eq. (19); the next operation starts from this level (eqs. (17)-(18))
        peak = max(peak, level);
        if (p.weight) base += p.weight[v];
        ++k;
        progressed = true;
        if (k < kend) {
          v = ld_agent(list + k);
          pp = p.pred_ptr[v];
          pe = p.pred_ptr[v + 1];
        } else {
          active = false;
        }
      }
    }
    __syncthreads();                 // orders this round's end-time stores before the next round's loads
    const uint64_t bal_prog = __ballot(progressed);
    if (active && (bal_prog & segmask) == 0) {
      // nothing of this candidate moved although operations remain: the combined graph is cyclic
      s_flag[g] = kBitCyclic;
      active = false;
    }
    if (__ballot(active) == 0) break;
  }
  if (p.mem_limit && lane_valid && s_flag[g] == 0 && base + peak > p.mem_limit[j]) atomicOr(&s_flag[g], kBitOverMemory);
  __syncthreads();

  // reductions and outputs
  int32_t z = acc;
  for (int d = 1; d < Pseg; d <<= 1) z = max(z, __shfl_xor(z, d, Pseg));
  if (lane_valid) {
    const int flag = flag_from_bits(s_flag[g]);
    p.out.peak_mem[c * p.out.peak_stride_c + j * p.out.peak_stride_j] = flag ? -1 : base + peak;
    if (j == 0) {
      p.out.makespan[c] = flag ? -1 : z;
      p.out.bubble[c] = flag ? -1 : (int64_t)P * z - p.sum_dur;
      p.out.flags[c] = flag;
    }
  }
}

}  // namespace dagsched_dev
