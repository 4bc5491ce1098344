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
// A workgroup stays on its CU and takes one batch of G * W candidates after the other.  While the relaxers work on
// a batch, the other wavefronts request the rows of the workgroup's next batch into registers, so that the read
// from HBM runs behind the relaxation instead of before it and ingest is a scatter out of registers.
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
  uint32_t o_mem, o_mach, o_cand, cand_stride, o_list, o_book, total;   // LDS: ops at 0, memory adjustments, machines; per candidate cells then list; bookkeeping
  OutPtrs out;
};

// PR: DAG predecessors looked at per op (2 or 4)
template <int PR>
__global__ __launch_bounds__(1024) void relax_static_kernel(StaticParams p) {
  extern __shared__ __align__(16) unsigned char lds[];
  const int kThreads = (int)blockDim.x;                     // at least 128 * W
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int N = p.N, P = p.P, Pseg = p.Pseg, G = p.G, W = p.W;
  const int GW = G * W;                                     // candidates per batch, at most 64
  const int n_batches = (int)(((int64_t)p.C + GW - 1) / GW);
  lds_byte_t *const ldsb = (lds_byte_t *)lds;
  uint4 *opsw = (uint4 *)lds;
  int64_t *memw = (int64_t *)(lds + p.o_mem);               // [N] A_i
  int32_t *flagw = (int32_t *)(lds + p.o_book);             // [64]
  int32_t *offw = (int32_t *)(lds + p.o_book + 256);        // [Pseg + 1]
  uint32_t *pairw = (uint32_t *)(lds + p.o_book + 640);     // [Pseg] start | end << 16 of machine j in every order list
  // [64] 1 = some machine of the candidate is over its memory limit; apart from flagw, which the relaxers read when
  // they start on a batch while the accountants may already have found a limit exceeded
  uint8_t *overb = lds + p.o_book + 896;
  int64_t *peakw = (int64_t *)(lds + p.o_book + 1024);      // [W][64]
  constexpr uint32_t kNever = 0xFFFFu;

  // Ingest is the work of the wavefronts that do not relax: a team of consecutive threads per candidate slot.
  // A candidate's rows are read four nodes per load, kChunk loads of each row per thread and round.
  const int n_help = kThreads - W * kWave;                  // at least 64 * W >= G * W
  const int tpc = n_help / GW;
  const int ht = tid - W * kWave;
  const int team = ht >= 0 ? ht / tpc : GW;                 // GW: no team (relaxers, left-over threads)
  const int tt = ht >= 0 ? ht - team * tpc : 0;
  constexpr int kChunk = 8;
  const bool vec_ok = ((N & 3) == 0) && ((((uintptr_t)p.placement) | ((uintptr_t)p.rank)) & 15) == 0;
  const int nq = N >> 2;
  uint32_t *machw = (uint32_t *)(lds + p.o_mach);           // [N / 4 rounded up] the shared placement, four machines per word
  int4 a4[kChunk], r4[kChunk];
  // kChunk quads of this thread's share of candidate `team` of batch b, from quad q0 on.  One base per batch and
  // row (the same for the whole workgroup) plus a 32-bit offset per thread: the rows of a batch span less than 4 GB.
  auto request = [&](int b, int q0) {
    const int64_t c = (int64_t)b * GW + team;
    if (!vec_ok || team >= GW || b >= n_batches || c >= p.C) return;
    // (the batch number through readfirstlane: the bases stay in scalar registers and are worked out here, not
    // carried along as per-thread pointers from batch to batch, which cost more registers than there are)
    const int64_t bs = __builtin_amdgcn_readfirstlane(b);
    const char *base_pl = (const char *)(p.placement + bs * GW * N);
    const char *base_rk = (const char *)(p.rank + bs * GW * N);
    // (an offset the compiler cannot see through: the eight offsets are worked out here, at the loads, instead of
    // being kept from batch to batch and spilled, with a wait for every load behind each reload)
    const uint32_t row = (uint32_t)team * (uint32_t)N * 4u;
    asm volatile("" : "+v"(q0));
#pragma unroll
    for (int u = 0; u < kChunk; ++u) {
      const int q = q0 + u * tpc;
      const uint32_t off = row + (uint32_t)(q < nq ? q : 0) * 16u;
      a4[u] = *(const int4 *)(base_pl + off);
      r4[u] = *(const int4 *)(base_rk + off);
    }
  };
  request((int)blockIdx.x, tt);
  for (int i = tid; i < N; i += kThreads) { opsw[i] = p.ops[i]; memw[i] = p.mem_delta[i]; }
  for (int i = tid; i < (N + 3) / 4; i += kThreads) machw[i] = ((const uint32_t *)p.machine)[i];
  if (tid <= Pseg) offw[tid] = p.off[tid];
  if (tid < Pseg) pairw[tid] = (uint32_t)p.off[tid] | ((uint32_t)p.off[tid + 1] << 16);

  const bool lane_on = lane < G * Pseg;
  const int ql = lane_on ? lane : 0;
  const int g = ql >> p.log_pseg, j = ql & (Pseg - 1);
  const int role_wave = wave < W ? wave : wave - W;
  const int gi = role_wave * G + g;                         // candidate slot of this lane (roles only)
  const uint32_t cbase = (uint32_t)(uintptr_t)(ldsb + p.o_cand + (uint32_t)(gi < GW ? gi : 0) * p.cand_stride);

  // cells 0..N-1 "not ended", cell N = 0 (stands for absent predecessors), two cells of padding; list entries
  // 0..N-1 "unwritten", four entries of padding that name operation 0.  Every candidate slot is set up, also
  // those beyond the end of the batch: their lanes read it like the others.
  const int tpa = kThreads / GW;                            // threads per candidate slot when all wavefronts take part
  const int slot_a = tid / tpa, ta = tid - slot_a * tpa;
  auto init_batch = [&]() {
    if (tid < kWave) { flagw[tid] = 0; overb[tid] = 0; }
    if (slot_a >= GW) return;
    const int cwords = (N + 4) / 2, lwords = (N + 5) / 2;   // the list follows the cells
    uint32_t *w = (uint32_t *)(lds + p.o_cand + slot_a * p.cand_stride);
    for (int i = ta; i < cwords + lwords; i += tpa) {
      const int k = i < cwords ? i : i - cwords;
      w[i] = (2 * k < N ? kNever : 0u) | ((2 * k + 1 < N ? kNever : 0u) << 16);
    }
  };

  // Relaxers and the other wavefronts run loops of their own over the workgroup's batches and meet at the same
  // five barriers per batch (the rows in flight for the next batch then cost the relaxers no registers).
  if (wave < W) {
    for (int b = (int)blockIdx.x; b < n_batches; b += (int)gridDim.x) {
      const int64_t c0 = (int64_t)b * GW;
      const int ng = (int)min((int64_t)GW, (int64_t)p.C - c0);
      init_batch();
      __syncthreads();                                       // the others scatter the rows into the lists ...
      __syncthreads();                                       // ... and look for unwritten slots
      __syncthreads();
      // ---------------------------------------------------------- relaxer
      const bool ok = lane_on && gi < ng && flagw[gi] == 0 && j < P;
      const uint32_t n_ops = ok ? (uint32_t)(offw[j + 1] - offw[j]) : 0u;
      // lanes without operations look at the list's padding (operation 0, which they never run)
      const uint32_t lbase = cbase + p.o_list + 2u * (n_ops ? (uint32_t)offw[j] : (uint32_t)N);
      uint32_t x_acc = 0;                                    // the machine is free from time 0 on
      auto ld16 = [](uint32_t a) -> uint32_t { return (uint32_t)*(lds_vu16_t *)(uintptr_t)a; };
      const uint32_t ops_base = (uint32_t)(uintptr_t)ldsb;
      const uint32_t trash = cbase + 2u * ((uint32_t)N + 1u);
      const uint64_t seg0 = (Pseg == kWave) ? ~0ull : ((1ull << Pseg) - 1ull);
      const uint32_t seg_shift = (uint32_t)(g * Pseg);
      uint32_t cnt = n_ops;                                  // operations this lane still has to see through (0: retired)
      uint32_t done = 0;                                     // operations completed
      uint32_t idn = ld16(lbase + 2);                        // list entry after the current one
      uint32_t lp = lbase + 4;                               // address of the entry after that
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
      if (done < cnt) atomicOr(&flagw[gi], kBitInternal);    // the window bound ran out: never expected
      __builtin_amdgcn_s_setprio(0);
      __syncthreads();
      // ---------------------------------------------------------- reductions and outputs
      int32_t z = (int32_t)x_acc;
      for (int d = 1; d < Pseg; d <<= 1) z = max(z, __shfl_xor(z, d, Pseg));
      if (lane_on && gi < ng && j < P) {
        const int64_t c = c0 + gi;
        const int bits = flagw[gi] | (overb[gi] ? kBitOverMemory : 0);
        if ((bits & kBitOtherPlacement) && !(bits & kBitBadPlacement)) {
          if (j == 0) { const int slot = atomicAdd(p.fb_count, 1); p.fb_list[slot] = (int32_t)c; }   // the general kernel writes this candidate
        } else {
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
      __syncthreads();                                       // the flags and peaks are reset by the next batch
    }
  } else {
    for (int b = (int)blockIdx.x; b < n_batches; b += (int)gridDim.x) {
      const int64_t c0 = (int64_t)b * GW;
      const int ng = (int)min((int64_t)GW, (int64_t)p.C - c0);
      // ---------------------------------------------------------- ingest
      init_batch();
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
          // Branch-free, so that the LDS reads of a round are all in flight together: a node that cannot be put
          // into its list is written to the last padding entry of the list, which nobody reads.
          const uint32_t dump = (uint32_t)N + 3u;
          for (int q0 = tt; q0 < nq; q0 += kChunk * tpc) {
            if (q0 != tt) request(b, q0);                    // (the first round was requested a batch ago)
            uint32_t mw[kChunk];
#pragma unroll
            for (int u = 0; u < kChunk; ++u) mw[u] = machw[min(q0 + u * tpc, nq - 1)];
#pragma unroll
            for (int half = 0; half < kChunk; half += 4) {
              uint32_t pr[4][4];
#pragma unroll
              for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e) pr[u][e] = pairw[(mw[half + u] >> (8 * e)) & 0xFF];
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                const int q = q0 + (half + u) * tpc;
                const int32_t av[4] = {a4[half + u].x, a4[half + u].y, a4[half + u].z, a4[half + u].w};
                const int32_t rv[4] = {r4[half + u].x, r4[half + u].y, r4[half + u].z, r4[half + u].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  const uint32_t m = (mw[half + u] >> (8 * e)) & 0xFF;
                  const uint32_t o0 = pr[u][e] & 0xFFFFu, n = (pr[u][e] >> 16) - o0;
                  const bool live = q < nq;
                  const bool bad_pl = (uint32_t)av[e] >= (uint32_t)P, other = (uint32_t)av[e] != m, bad_rk = (uint32_t)rv[e] >= n;
                  bits |= (live && bad_pl) ? kBitBadPlacement : 0;
                  bits |= (live && !bad_pl && other) ? kBitOtherPlacement : 0;
                  bits |= (live && !bad_pl && !other && bad_rk) ? kBitBadRank : 0;
                  const bool put = live && !other && !bad_rk;   // (a placement out of range is another placement too)
                  list[put ? o0 + (uint32_t)rv[e] : dump] = (uint16_t)(4 * q + e);
                }
              }
            }
          }
        } else {
          for (int v = tt; v < N; v += tpc) place(v, pl[v], rk[v], (machw[v >> 2] >> ((v & 3) << 3)) & 0xFF);
        }
        if (bits) atomicOr(&flagw[team], bits);
      }
      __syncthreads();
      // N operations into N slots: no slot left unwritten <=> every (machine, rank) slot hit exactly once
      if (team < ng && !(flagw[team] & (kBitBadPlacement | kBitOtherPlacement))) {
        const uint32_t *lw = (const uint32_t *)(lds + p.o_cand + team * p.cand_stride + p.o_list);
        bool hole = false;
        const int nw = (N + 1) / 2;
        for (int i0 = tt; i0 < nw; i0 += 8 * tpc) {
          uint32_t w[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) w[u] = lw[min(i0 + u * tpc, nw - 1)];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int i = min(i0 + u * tpc, nw - 1);
            hole |= (w[u] & 0xFFFFu) == kNever || (2 * i + 1 < N && (w[u] >> 16) == kNever);
          }
        }
        if (hole) atomicOr(&flagw[team], kBitBadRank);
      }
      __syncthreads();
      // the rows of this workgroup's next batch: on their way while the relaxers work
      request(b + (int)gridDim.x, tt);
      if (wave < 2 * W) {
        // -------------------------------------------------------- accountant
        const bool ok = lane_on && gi < ng && flagw[gi] == 0 && j < P;
        const uint32_t n_ops = ok ? (uint32_t)(offw[j + 1] - offw[j]) : 0u;
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
        if (ok && p.mem_limit && peak > p.mem_limit[j]) overb[gi] = 1;
        if (lane_on) peakw[role_wave * kWave + ql] = peak;
      }
      __syncthreads();                                       // the relaxers write the outputs ...
      __syncthreads();                                       // ... before the next batch resets flags and peaks
    }
  }
}

}  // namespace dagsched_dev
