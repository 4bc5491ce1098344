// Shared-placement kernel: the evaluation path for batches whose candidates all place the operations alike (a
// pipeline with its stage -> machine map fixed, as in the experiments of Sec. V) and differ in the order only.
//
// With the allocation x (eq. (6)) known when the handle is made, everything the ring kernel's feeder wavefronts
// work out per candidate is a constant of the problem: the delay on every DAG edge (eqs. (11)-(13): the channel
// delay when the two machines differ, else 0), the operations of every machine and hence where its part of the
// order list starts.  The host builds one op per operation, in the ring kernel's format, and the kernel keeps
// that table in LDS next to the candidates' end times and order lists.  No feeders, no ring, no wavefront waits
// for another one:
//
//   waves 0..W-1, RELAXERS     lane (g, j) walks machine j's list of candidate g: looks up the op of the list's
//                              next entry, reads the end times of its predecessors, and, once all have ended,
//                              s_v = max(0, e_chainpred, max_u e_u + delta(u,v)), e_v = s_v + D^o_v
//                              (eqs. (3),(7),(11)-(13)).  One trip = at most one operation per lane; the op after
//                              the current one and the list entry after that are fetched a trip ahead.
//   waves W..2W-1, ACCOUNTANTS lane (g, j) takes the peak of machine j's running memory level (eqs. (17)-(19)).
//   further waves              only help with ingest, so that one round of loads covers a candidate's rows.
//
// A candidate whose placement differs from the shared one is left to the general int32 kernel (the caller's
// promise is a hint, never trusted).  End times are 16-bit (the host proves that they fit).
//
// Cycle test: every lane that is not through holds an operation in every trip, so a trip in which no lane of a
// candidate completes one changes nothing and neither will any later trip: the combined graph has a cycle
// (eqs. (5),(7),(8) cannot hold together).  Looked for once per window of 8 trips; every window either completes
// an operation or retires its candidates, so the loop ends after at most N * G + G windows.
#pragma once

#include "device_common.h"
#include "kernel_ring.h"   // LDS pointer types

namespace dagsched_dev {

constexpr int kBitOtherPlacement = 64;   // internal: the candidate does not use the shared placement

struct StaticParams {
  int32_t N, P, Pseg, log_pseg, G, W, C;   // G candidates per relaxer wavefront, W relaxers per workgroup
  const uint4 *ops;          // [N] x = o(pred0) | o(pred1) << 16, y = o(pred2) | o(pred3) << 16, z = four 8-bit delays,
                             //     w = duration | o(v) << 16; o(u) = 2u, the byte offset of u's cell in a candidate's
                             //     cell array; unused predecessors name cell N (always 0) with delay 0
  const uint8_t *machine;    // [N rounded up to 4] the shared placement
  const int32_t *off;        // [Pseg + 1] start of machine j in every order list (N from machine P on)
  const int64_t *mem_delta;  // [N]
  const int64_t *base;       // [P] static memory on each machine under the shared placement (eq. (16)), or NULL
  const int64_t *mem_limit;  // [P] or NULL
  int64_t sum_dur;           // original units
  int32_t time_scale;
  const int32_t *placement, *rank;   // [C][N]
  int32_t *fb_count, *fb_list;       // candidates with another placement
  uint32_t o_mem, o_cand, cand_stride, o_list, o_book, total;   // LDS: ops at 0, memory adjustments; per candidate cells then list; bookkeeping
  OutPtrs out;
};

// PR: DAG predecessors looked at per op (2 or 4)
template <int PR>
__global__ __launch_bounds__(1024) void relax_static_kernel(StaticParams p) {
  extern __shared__ __align__(16) unsigned char lds[];
  const int kThreads = (int)blockDim.x;                     // at least 128 * W; further wavefronts only help with ingest
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int N = p.N, P = p.P, Pseg = p.Pseg, G = p.G, W = p.W;
  const int GW = G * W;                                     // candidates per workgroup, at most 64
  const int64_t c0 = (int64_t)blockIdx.x * GW;
  const int ng = (int)min((int64_t)GW, (int64_t)p.C - c0);
  lds_byte_t *const ldsb = (lds_byte_t *)lds;
  uint4 *opsw = (uint4 *)lds;
  int64_t *memw = (int64_t *)(lds + p.o_mem);               // [N] A_i
  int32_t *flagw = (int32_t *)(lds + p.o_book);             // [64]
  int32_t *offw = (int32_t *)(lds + p.o_book + 256);        // [Pseg + 1]
  int64_t *peakw = (int64_t *)(lds + p.o_book + 1024);      // [W][64]
  constexpr uint32_t kNever = 0xFFFFu;

  // ---------------------------------------------------------------- ingest (all wavefronts)
  const int tpc = kThreads / GW;                            // a team of consecutive threads per candidate (at least 2)
  const int team = tid / tpc, tt = tid - team * tpc;
  // The candidate's rows are read four nodes per load, kChunk loads of each row in flight per thread; the first
  // chunk is requested before the tables and the LDS are set up, which hides its latency.
  constexpr int kChunk = 8;
  const bool vec_ok = ((N & 3) == 0) && ((((uintptr_t)p.placement) | ((uintptr_t)p.rank)) & 15) == 0;
  const int nq = N >> 2;
  const int4 *pl4 = (const int4 *)(p.placement + (c0 + (team < ng ? team : 0)) * N);
  const int4 *rk4 = (const int4 *)(p.rank + (c0 + (team < ng ? team : 0)) * N);
  const uint32_t *m4 = (const uint32_t *)p.machine;
  int4 a4[kChunk], r4[kChunk];
  uint32_t mq[kChunk];
  auto request = [&](int q0) {
#pragma unroll
    for (int u = 0; u < kChunk; ++u) {
      const int q = q0 + u * tpc;
      a4[u] = q < nq ? pl4[q] : make_int4(0, 0, 0, 0);
      r4[u] = q < nq ? rk4[q] : make_int4(0, 0, 0, 0);
      mq[u] = q < nq ? m4[q] : 0u;
    }
  };
  if (vec_ok && team < ng) request(tt);
  for (int i = tid; i < N; i += kThreads) { opsw[i] = p.ops[i]; memw[i] = p.mem_delta[i]; }
  if (tid < kWave) flagw[tid] = 0;
  if (tid <= Pseg) offw[tid] = p.off[tid];
  // cells 0..N-1 "not ended", cell N = 0 (stands for absent predecessors), N+1 trash, N+2 never ends;
  // list entries 0..N-1 "unwritten", four entries of padding that name operation 0.  Every candidate slot of the
  // workgroup is initialised, also those beyond the end of the batch: their lanes read it like the others.
  if (team < GW) {
    uint32_t *cw = (uint32_t *)(lds + p.o_cand + team * p.cand_stride);
    uint32_t *lw = (uint32_t *)(lds + p.o_cand + team * p.cand_stride + p.o_list);
    auto cell0 = [&](int k) -> uint32_t { return (k < N || k == N + 2) ? kNever : 0u; };
    for (int i = tt; i < (N + 4) / 2; i += tpc) cw[i] = cell0(2 * i) | (cell0(2 * i + 1) << 16);
    for (int i = tt; i < (N + 5) / 2; i += tpc) lw[i] = (2 * i < N ? kNever : 0u) | ((2 * i + 1 < N ? kNever : 0u) << 16);
  }
  __syncthreads();
  // x as promised (else: another kernel's candidate), ranks inside the machine's range (eqs. (6)-(8))
  if (team < ng) {
    const int32_t *pl = p.placement + (c0 + team) * N, *rk = p.rank + (c0 + team) * N;
    uint16_t *list = (uint16_t *)(lds + p.o_cand + team * p.cand_stride + p.o_list);
    int bits = 0;
    auto place = [&](int v, int32_t a, int32_t r, int m) {
      if ((uint32_t)a >= (uint32_t)P) {
        bits |= kBitBadPlacement;
      } else if (a != m) {
        bits |= kBitOtherPlacement;
      } else {
        const int o0 = offw[m], n = offw[m + 1] - o0;
        if ((uint32_t)r >= (uint32_t)n) bits |= kBitBadRank;
        else list[o0 + r] = (uint16_t)v;
      }
    };
    if (vec_ok) {
      for (int q0 = tt; q0 < nq; q0 += kChunk * tpc) {
        if (q0 != tt) request(q0);
#pragma unroll
        for (int u = 0; u < kChunk; ++u) {
          const int q = q0 + u * tpc;
          if (q < nq) {
            place(4 * q + 0, a4[u].x, r4[u].x, mq[u] & 0xFF);
            place(4 * q + 1, a4[u].y, r4[u].y, (mq[u] >> 8) & 0xFF);
            place(4 * q + 2, a4[u].z, r4[u].z, (mq[u] >> 16) & 0xFF);
            place(4 * q + 3, a4[u].w, r4[u].w, mq[u] >> 24);
          }
        }
      }
    } else {
      for (int v = tt; v < N; v += tpc) place(v, pl[v], rk[v], p.machine[v]);
    }
    if (bits) atomicOr(&flagw[team], bits);
  }
  __syncthreads();
  // N operations into N slots: no slot left unwritten <=> every (machine, rank) slot hit exactly once
  if (team < ng && !(flagw[team] & (kBitBadPlacement | kBitOtherPlacement))) {
    const uint32_t *lw = (const uint32_t *)(lds + p.o_cand + team * p.cand_stride + p.o_list);
    bool hole = false;
    for (int i = tt; i < (N + 1) / 2; i += tpc) {
      const uint32_t w = lw[i];
      hole |= (w & 0xFFFFu) == kNever || (2 * i + 1 < N && (w >> 16) == kNever);
    }
    if (hole) atomicOr(&flagw[team], kBitBadRank);
  }
  __syncthreads();

  // ---------------------------------------------------------------- roles
  const bool lane_on = lane < G * Pseg;
  const int ql = lane_on ? lane : 0;
  const int g = ql >> p.log_pseg, j = ql & (Pseg - 1);
  const int role_wave = wave < W ? wave : wave - W;
  const int gi = role_wave * G + g;                         // candidate slot in the workgroup
  const bool ok = lane_on && gi < ng && flagw[gi] == 0 && j < P;
  const uint32_t n_ops = ok ? (uint32_t)(offw[j + 1] - offw[j]) : 0u;
  const uint32_t cbase = (uint32_t)(uintptr_t)(ldsb + p.o_cand + (uint32_t)gi * p.cand_stride);
  // lanes without operations look at the list's padding (operation 0, which they never run)
  const uint32_t lbase = cbase + p.o_list + 2u * (n_ops ? (uint32_t)offw[j] : (uint32_t)N);
  uint32_t x_acc = 0;                                       // the machine is free from time 0 on

  if (wave < W) {
    // ------------------------------------------------------------ relaxer
    auto ld16 = [](uint32_t a) -> uint32_t { return (uint32_t)*(lds_vu16_t *)(uintptr_t)a; };
    const uint32_t ops_base = (uint32_t)(uintptr_t)ldsb;
    const uint32_t trash = cbase + 2u * ((uint32_t)N + 1u);
    const uint64_t seg0 = (Pseg == kWave) ? ~0ull : ((1ull << Pseg) - 1ull);
    const uint32_t seg_shift = (uint32_t)(g * Pseg);
    uint32_t cnt = n_ops;                                    // operations this lane still has to see through (0: retired)
    uint32_t done = 0;                                       // operations completed
    uint32_t idn = ld16(lbase + 2);                          // list entry after the current one
    uint32_t lp = lbase + 4;                                 // address of the entry after that
    u32x4_t cur = *(lds_vu32x4_t *)(uintptr_t)(ops_base + ld16(lbase) * 16u);
    uint32_t e0 = ld16(cbase + (cur.x & 0xFFFFu)), e1 = ld16(cbase + (cur.x >> 16)), e2 = 0, e3 = 0;
    if (PR == 4) { e2 = ld16(cbase + (cur.y & 0xFFFFu)); e3 = ld16(cbase + (cur.y >> 16)); }
    __builtin_amdgcn_s_setprio(3);
    const uint32_t max_windows = (uint32_t)N * (uint32_t)G + (uint32_t)G + 2u;
    for (uint32_t win = 0; win < max_windows; ++win) {
      uint64_t ran_acc = 0;
#pragma unroll
      for (int sub = 0; sub < 8; ++sub) {
        const u32x4_t nxt = *(lds_vu32x4_t *)(uintptr_t)(ops_base + idn * 16u);
        const uint32_t idnn = ld16(lp);
        uint32_t x = max(max(x_acc, e0 + (cur.z & 0xFFu)), e1 + ((cur.z >> 8) & 0xFFu));
        if (PR == 4) x = max(max(x, e2 + ((cur.z >> 16) & 0xFFu)), e3 + (cur.z >> 24));
        const bool ran = x < kNever && done < cnt;
        x += cur.w & 0xFFFFu;
        *(lds_vu16_t *)(uintptr_t)(ran ? cbase + (cur.w >> 16) : trash) = (uint16_t)x;
        x_acc = ran ? x : x_acc;
        cur.x = ran ? nxt.x : cur.x; cur.y = ran ? nxt.y : cur.y; cur.z = ran ? nxt.z : cur.z; cur.w = ran ? nxt.w : cur.w;
        idn = ran ? idnn : idn;
        lp += ran ? 2u : 0u;
        done += ran ? 1u : 0u;
        ran_acc |= __ballot(ran);
        e0 = ld16(cbase + (cur.x & 0xFFFFu)); e1 = ld16(cbase + (cur.x >> 16));
        if (PR == 4) { e2 = ld16(cbase + (cur.y & 0xFFFFu)); e3 = ld16(cbase + (cur.y >> 16)); }
      }
      const bool unfinished = done < cnt;
      if (__ballot(unfinished) == 0) break;
      if (unfinished && ((ran_acc >> seg_shift) & seg0) == 0) {   // nothing moved in this candidate: a cycle
        atomicOr(&flagw[gi], kBitCyclic);
        cnt = 0;
      }
    }
    if (done < cnt) atomicOr(&flagw[gi], kBitInternal);      // the window bound ran out: never expected
    __builtin_amdgcn_s_setprio(0);
  } else if (wave < 2 * W) {
    // ------------------------------------------------------------ accountant
    const uint16_t *list = (const uint16_t *)(lds + p.o_cand + (uint32_t)gi * p.cand_stride + p.o_list) + (n_ops ? offw[j] : N);
    int64_t level = 0, peak = 0;
    for (uint32_t k = 0; __ballot(k < n_ops) != 0; k += 4) {
      int64_t m[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) m[u] = (k + u < n_ops) ? memw[list[k + u]] : 0;
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (k + u < n_ops) { level += m[u]; peak = max(peak, level); }   // eq. (19) along the chain
    }
    if (ok && p.base) peak += p.base[j];
    if (ok && p.mem_limit && peak > p.mem_limit[j]) atomicOr(&flagw[gi], kBitOverMemory);
    if (lane_on) peakw[role_wave * kWave + ql] = peak;
  }
  __syncthreads();

  // ---------------------------------------------------------------- reductions and outputs (relaxer wavefronts)
  if (wave < W) {
    int32_t z = (int32_t)x_acc;
    for (int d = 1; d < Pseg; d <<= 1) z = max(z, __shfl_xor(z, d, Pseg));
    if (lane_on && gi < ng && j < P) {
      const int64_t c = c0 + gi;
      const int bits = flagw[gi];
      if ((bits & kBitOtherPlacement) && !(bits & kBitBadPlacement)) {
        if (j == 0) { const int slot = atomicAdd(p.fb_count, 1); p.fb_list[slot] = (int32_t)c; }
        return;                                              // the general kernel writes this candidate
      }
      const int flag = flag_from_bits(bits);
      const int64_t zz = (int64_t)z * p.time_scale;
      p.out.peak_mem[c * p.out.peak_stride_c + j * p.out.peak_stride_j] = flag ? -1 : peakw[wave * kWave + ql];
      if (j == 0) {
        p.out.makespan[c] = flag ? -1 : (int32_t)zz;
        p.out.bubble[c] = flag ? -1 : (int64_t)P * zz - p.sum_dur;
        p.out.flags[c] = flag;
      }
    }
  }
}

}  // namespace dagsched_dev
