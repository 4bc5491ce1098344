// Evaluation with channel contention (Sec. III, eqs. (11)-(15)), a placement per candidate.
//
// The message of an edge (u, x) of B whose ends sit on different machines a, b is a transfer that occupies the
// channel (a, b) for comm[a][b] time units: it starts once u has ended and the transfer before it on the channel
// has ended (eqs. (13), (14)-(15)), and x starts after it has ended (eq. (12)).  The order of the transfers of a
// channel comes with the candidate (edge_rank, dense per channel), like the order of the operations of a machine.
// With every binary fixed the schedule is a longest path on operations and transfers:
//   c_k = max(e_u, d_prev(k)),  d_k = c_k + comm[a][b]
//   s_x = max(0, e_chainpred(x), max over in-edges k: same machine ? e_u : d_k),  e_x = s_x + D^o_x
//
// One workgroup per candidate, round-synchronous (one barrier per round).  Thread j < P walks machine j's order
// list and completes its head operation once every in-edge has delivered (the producer's end time for an edge
// inside the machine, the transfer's end time otherwise; one word polled per round).  Every thread also owns the
// channels t, t + T, t + 2T, ... of the P * P ordered pairs (T threads) and completes the head transfer of each once
// its producer has ended.  Channels are not polled blindly: a machine that completes an operation rings the bell
// of every channel the operation feeds (a counter in LDS), and a channel looks at its head transfer's producer
// only when its bell has rung since it last looked (or right after it completed a transfer).  A round in which
// nothing completes although something is left is a deadlock: a cycle through operations and transfers.
// A workgroup takes one candidate after the other; its order lists, end times and channel tables live in a
// workspace row of its own (indexed by the workgroup, not by the candidate), read and written at the L2.
#pragma once

#include "device_common.h"

namespace dagsched_dev {

constexpr int kContendedThreads = 512;                    // largest workgroup; the host launches fewer threads for few machines
constexpr int kChannelsPerThread = 8;                     // P * P <= 8 * (threads launched)
static_assert(DAGSCHED_MAX_DEVICES * DAGSCHED_MAX_DEVICES <= kChannelsPerThread * kContendedThreads, "every channel needs an owner");
// threads per workgroup for P machines: a multiple of 64, enough owners for the P * P channels
constexpr int contended_threads(int P) {
  const int need = (P * P + kChannelsPerThread - 1) / kChannelsPerThread;
  const int t = ((need < 128 ? 128 : need) + kWave - 1) / kWave * kWave;
  return t > kContendedThreads ? kContendedThreads : t;
}
// dynamic LDS: the bell of every channel
constexpr size_t contended_lds(int P) { return (size_t)P * (size_t)P * sizeof(int32_t); }

struct ContendedParams {
  int32_t N, E, P, C;
  const int32_t *pred_ptr, *pred_idx;   // [N + 1], [E] predecessor CSR of B: producer of every in-edge
  const int32_t *pred_eid;              // [E] the in-edge's index k in successor-CSR order (the index edge_rank uses)
  const int32_t *edge_src, *edge_dst;   // [E] ends of edge k
  const int32_t *succ_ptr;              // [N + 1] successor CSR of B: the out-edges of u are k = succ_ptr[u] .. succ_ptr[u + 1] - 1
  const int32_t *dur;                   // [N]
  const int32_t *comm;                  // [P * P] (0 where the pair has no channel: those candidates are flagged afterwards)
  const int64_t *mem_delta, *weight, *mem_limit;
  int64_t sum_dur;
  const int32_t *placement, *rank;      // [C][N]
  const int32_t *edge_rank;             // [C][E]
  int32_t *ws_list, *ws_end;            // [grid][row_n] order lists machine after machine; end times of the operations
  int32_t *ws_tlist, *ws_tend;          // [grid][row_e] transfers channel after channel; end times of the transfers
  int32_t *ws_ccnt, *ws_coff;           // [grid][row_c] transfers per channel; start of the channel in ws_tlist
  int32_t *ws_echan;                    // [grid][row_e] channel a * P + b of edge k under this candidate, -1 inside a machine
  int64_t row_n, row_e, row_c;
  OutPtrs out;
};

// (four wavefronts per SIMD: the kernel waits on the L2 most of the time, and candidates in flight are what hides it)
__global__ __launch_bounds__(kContendedThreads) __attribute__((amdgpu_waves_per_eu(4, 8))) void relax_contended_kernel(ContendedParams p) {
  __shared__ int32_t s_cnt[kWave], s_off[kWave + 1];
  __shared__ int32_t s_flag, s_z;
  __shared__ int32_t s_part[kContendedThreads];
  extern __shared__ int32_t s_bell[];                       // [P * P] how often a producer of the channel has completed an operation
  const int t = threadIdx.x, T = (int)blockDim.x;
  const int N = p.N, E = p.E, P = p.P, PP = P * P;
  int32_t *list = p.ws_list + (int64_t)blockIdx.x * p.row_n, *end = p.ws_end + (int64_t)blockIdx.x * p.row_n;
  int32_t *tlist = p.ws_tlist + (int64_t)blockIdx.x * p.row_e, *tend = p.ws_tend + (int64_t)blockIdx.x * p.row_e;
  int32_t *ccnt = p.ws_ccnt + (int64_t)blockIdx.x * p.row_c, *coff = p.ws_coff + (int64_t)blockIdx.x * p.row_c;
  int32_t *echan = p.ws_echan + (int64_t)blockIdx.x * p.row_e;

  for (int64_t c = blockIdx.x; c < p.C; c += gridDim.x) {
    const int32_t *pl = p.placement + c * N, *rk = p.rank + c * N, *er = p.edge_rank + c * E;
    if (t < kWave) s_cnt[t] = 0;
    if (t == 0) { s_flag = 0; s_z = 0; }
    for (int ch = t; ch < PP; ch += T) st_agent(&ccnt[ch], 0);
    __syncthreads();
    // x in range (eq. (6)), operations per machine
    for (int v = t; v < N; v += T) {
      const int32_t pi = pl[v];
      if ((uint32_t)pi >= (uint32_t)P) atomicOr(&s_flag, kBitBadPlacement);
      else atomicAdd(&s_cnt[pi], 1);
      st_agent(&end[v], -1);
    }
    __syncthreads();
    bool bad = s_flag != 0;                                 // the same for every thread
    if (!bad) {
      if (t == 0) {
        int at = 0;
        for (int j = 0; j < P; ++j) { s_off[j] = at; at += s_cnt[j]; }
        s_off[P] = at;
      }
      __syncthreads();
      // a total order per machine (eqs. (7)-(8)): list_j[rank] = operation, every slot hit exactly once
      for (int v = t; v < N; v += T) {
        const int32_t pi = pl[v], r = rk[v];
        if ((uint32_t)r >= (uint32_t)s_cnt[pi]) atomicOr(&s_flag, kBitBadRank);
        else st_agent(&list[s_off[pi] + r], v);
      }
      // transfers per channel
      for (int k = t; k < E; k += T) {
        const int32_t a = pl[p.edge_src[k]], b = pl[p.edge_dst[k]];
        if (a != b) atomicAdd(&ccnt[a * P + b], 1);
        st_agent(&echan[k], a != b ? a * P + b : -1);
        st_agent(&tend[k], -1);
      }
      __syncthreads();
      for (int v = t; v < N; v += T) {
        const int32_t pi = pl[v], r = rk[v];
        if ((uint32_t)r < (uint32_t)s_cnt[pi] && ld_agent(&list[s_off[pi] + r]) != v) atomicOr(&s_flag, kBitBadRank);
      }
      // start of every channel in the transfer list: each thread sums a block of consecutive channels, thread 0 scans
      const int per = (PP + T - 1) / T;
      int mine = 0;
      for (int i = 0; i < per; ++i) {
        const int ch = t * per + i;
        if (ch < PP) mine += ld_agent(&ccnt[ch]);
      }
      s_part[t] = mine;
      __syncthreads();
      if (t == 0) {
        int at = 0;
        for (int i = 0; i < T; ++i) { const int x = s_part[i]; s_part[i] = at; at += x; }
      }
      __syncthreads();
      {
        int at = s_part[t];
        for (int i = 0; i < per; ++i) {
          const int ch = t * per + i;
          if (ch < PP) { st_agent(&coff[ch], at); at += ld_agent(&ccnt[ch]); }
        }
      }
      __syncthreads();
      // a total order per channel (eqs. (14)-(15))
      for (int k = t; k < E; k += T) {
        const int32_t a = pl[p.edge_src[k]], b = pl[p.edge_dst[k]];
        if (a == b) continue;
        const int ch = a * P + b;
        const int32_t r = er[k];
        if ((uint32_t)r >= (uint32_t)ld_agent(&ccnt[ch])) atomicOr(&s_flag, kBitBadRank);
        else st_agent(&tlist[ld_agent(&coff[ch]) + r], k);
      }
      __syncthreads();
      for (int k = t; k < E; k += T) {
        const int32_t a = pl[p.edge_src[k]], b = pl[p.edge_dst[k]];
        if (a == b) continue;
        const int ch = a * P + b;
        const int32_t r = er[k];
        if ((uint32_t)r < (uint32_t)ld_agent(&ccnt[ch]) && ld_agent(&tlist[ld_agent(&coff[ch]) + r]) != k) atomicOr(&s_flag, kBitBadRank);
      }
      __syncthreads();
      bad = s_flag != 0;
    }

    int32_t free_at = 0;                                     // machine t: end of its previous operation
    int64_t level = 0, peak = 0, base = 0;
    if (!bad) {
      // Machine state (threads below P): the head operation v, its in-edges q .. qend of which those before q have
      // delivered (acc = latest delivery so far), and where the next one delivers: the producer's end time for an
      // edge inside the machine, the transfer's end time otherwise.  Only that one word is polled per round.
      int k = 0, kend = 0, v = 0, q = 0, qend = 0;
      int32_t acc = 0;
      const int32_t *poll = end;
      auto next_edge = [&]() {                                // where in-edge q of v delivers
        const int u = p.pred_idx[q];
        poll = (pl[u] == t) ? &end[u] : &tend[p.pred_eid[q]];   // eq. (12)
      };
      auto next_op = [&]() {
        v = ld_agent(&list[k]);
        q = p.pred_ptr[v]; qend = p.pred_ptr[v + 1];
        acc = free_at;
        if (q < qend) next_edge();
      };
      if (t < P) { k = s_off[t]; kend = s_off[t + 1]; if (k < kend) next_op(); }
      // Channel state: head transfer c_k of each owned channel, its producer c_u, and the bell count last acted on
      // (-1: look at the head without waiting for a bell)
      int32_t c_at[kChannelsPerThread], c_end[kChannelsPerThread], c_free[kChannelsPerThread];
      int32_t c_u[kChannelsPerThread], c_seen[kChannelsPerThread];
      for (int ch = t; ch < PP; ch += T) s_bell[ch] = 0;
#pragma unroll
      for (int i = 0; i < kChannelsPerThread; ++i) {
        const int ch = t + i * T;
        c_at[i] = c_end[i] = c_free[i] = c_u[i] = 0;
        c_seen[i] = -1;
        if (ch < PP) {
          c_at[i] = ld_agent(&coff[ch]);
          c_end[i] = c_at[i] + ld_agent(&ccnt[ch]);
          if (c_at[i] < c_end[i]) c_u[i] = p.edge_src[ld_agent(&tlist[c_at[i]])];
        }
      }
      __syncthreads();
      const int64_t max_rounds = (int64_t)N + E + 2;          // every round but the last completes something
      for (int64_t round = 0; round < max_rounds; ++round) {
        bool progressed = false;
        if (k < kend) {
          while (q < qend) {                                  // in-edges deliver in any order; they are waited for in turn
            const int32_t at = ld_agent(poll);
            if (at < 0) break;
            acc = max(acc, at);
            ++q;
            progressed = true;
            if (q < qend) next_edge();
          }
          if (q == qend) {
            const int32_t e = acc + p.dur[v];                 // eq. (3); acc >= free_at: one operation at a time, eq. (7)
            st_agent(&end[v], e);
            free_at = e;
            level += p.mem_delta[v];                          // eq. (19)
            peak = max(peak, level);
            if (p.weight) base += p.weight[v];                // eq. (16)
            // (the end time must have arrived at the L2 before a bell is rung: the wavefront waits for its stores)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            for (int kq = p.succ_ptr[v]; kq < p.succ_ptr[v + 1]; ++kq) {   // the channels v feeds hear of it
              const int ch = ld_agent(&echan[kq]);
              if (ch >= 0) atomicAdd(&s_bell[ch], 1);
            }
            ++k;
            if (k < kend) next_op();
            progressed = true;
          }
        }
        // A bell rung in this round is acted on in this round or the next: the count is read before the producer's end
        // time is, and the end time was written before the bell was rung.
#pragma unroll
        for (int i = 0; i < kChannelsPerThread; ++i) {
          if (c_at[i] < c_end[i]) {
            const int32_t bell = *(volatile int32_t *)&s_bell[t + i * T];
            if (bell != c_seen[i]) {
              const int32_t eu = ld_agent(&end[c_u[i]]);
              if (eu >= 0) {                                   // eq. (13); the channel is free from c_free on, eqs. (14)-(15)
                const int32_t d = max(c_free[i], eu) + p.comm[t + i * T];   // eq. (11)
                st_agent(&tend[ld_agent(&tlist[c_at[i]])], d);
                c_free[i] = d;
                ++c_at[i];
                if (c_at[i] < c_end[i]) c_u[i] = p.edge_src[ld_agent(&tlist[c_at[i]])];
                c_seen[i] = -1;                                // the next head's producer may have ended long ago
                progressed = true;
              } else {
                c_seen[i] = bell;
              }
            }
          }
        }
        if (!__syncthreads_or(progressed)) break;
      }
      bool left = k < kend;
#pragma unroll
      for (int i = 0; i < kChannelsPerThread; ++i) left = left || c_at[i] < c_end[i];
      const bool unfinished = left;
      if (__syncthreads_or(unfinished)) { if (t == 0) s_flag = kBitCyclic; }
      else {
        if (t < P) {
          atomicMax(&s_z, free_at);
          if (p.mem_limit && base + peak > p.mem_limit[t]) atomicOr(&s_flag, kBitOverMemory);
        }
      }
      __syncthreads();
    }
    const int flag = flag_from_bits(s_flag);
    if (t < P) p.out.peak_mem[c * p.out.peak_stride_c + t * p.out.peak_stride_j] = flag ? -1 : base + peak;
    if (t == 0) {
      const int32_t z = s_z;
      p.out.makespan[c] = flag ? -1 : z;
      p.out.bubble[c] = flag ? -1 : (int64_t)P * z - p.sum_dur;
      p.out.flags[c] = flag;
    }
    __syncthreads();                                         // the shared words are reset for the next candidate
  }
}

}  // namespace dagsched_dev
