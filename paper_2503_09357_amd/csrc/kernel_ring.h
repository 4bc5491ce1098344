// Ring kernel: the fast evaluation path.
//
// Workgroup = 2 + FEEDERS wavefronts with a role, which never meet at a barrier while the schedule is being
// relaxed (further wavefronts, if launched, only help with ingest); lane (g, j) of every wavefront stands for
// machine j of candidate g:
//
//   wave 0, the RELAXER   pops compact "ops" from a per-lane ring in LDS and runs the max-plus
//                         recurrence
//                           s_v = max(0, e_chainpred, max_u e_u + delta(u,v)),  e_v = s_v + D^o_v
//                         (eqs. (3),(7),(11)-(13), Sec. III) against the end-time array of its
//                         candidate in LDS.  Its loop touches LDS only and is branch-free.
//   waves 1..FEEDERS, the FEEDERS  walk machine j's order list, fetch the shared operator records from
//                         L2, look up the placement of every DAG predecessor (one byte or four bits per
//                         node in LDS, or one byte in L2) and the channel delay (LDS), and push the
//                         resulting op into the relaxer's ring.
//   wave FEEDERS + 1, the ACCOUNTANT  walks the order lists and takes the peak of each machine's running
//                         memory level (eqs. (17)-(19)), which depends on the order only.
//
// The feeders run ahead and absorb every global-memory latency.  A lone wavefront issues an instruction
// every few cycles at best and waits out every LDS round trip, so the relaxer's trip is kept short and
// its critical path (end times arrive -> add, max -> compare -> select next op -> next end-time reads)
// carries no scalar instruction.  The CUs are LDS-capacity bound on the large configurations (only a
// few candidates fit), so the other wavefronts run on SIMDs that would otherwise idle.
//
// End times are kept as 16-bit unsigned values (sentinel 0xFFFF = not yet ended), which halves the
// LDS footprint (template HALF = 0 or 1).  HALF = 2 keeps them in 32 bits (sentinel 0x80000000) for problems whose
// times cannot stay below 0xFFFF: the same kernel with half the candidates resident, always exact.  HALF = 3 does
// so too and also lifts the limits of the op format on delays (255) and durations (65534): an op then names the
// machines of its predecessors instead of the delays (six bits each), the relaxer looks the delays up in a 32-bit
// table in LDS together with the end times, and the duration is low + 65535 * high with eight more bits for high.  When the host cannot prove that every end time stays below 0xFFFF the kernel runs
// "optimistically": an operation whose end time would reach 0xFFFF is never completed, its candidate
// stalls exactly like a cyclic one; the two are told apart at the deadlock (does some held op have all its
// predecessors ended?) and the candidates stopped by the range are handed to the general int32 kernel.
//
// Ring protocol (single consumer per lane, no atomics, no counters): a lane's ring has RING slots of
// 16 bytes; op i of the lane's stream goes to slot i mod RING.  The last dword of a slot is either
// "duration | address << 16" of a delivered op (duration < 0xFFFF) or "0xFFFF | i << 16": free, op i
// was the last one copied out of it (the ring starts as if ops -RING .. -1 had been).  A feeder
// delivers op i once the slot says that op i - RING is out, writing the last dword last; the relaxer
// copies a delivered slot into registers and writes the free mark.  LDS executes one wavefront's
// accesses in order, so a delivered last dword proves that the rest of the slot is complete.
#pragma once

#include "device_common.h"

namespace dagsched_dev {

// Op layout (one 16-byte slot).  ha(x) is the 16-bit address of the end-time cell of x: its LDS byte
// address when the end-time arrays of the workgroup fit 64 KB (template HALF = 0), else the byte
// address / 2 (HALF = 1); with 32-bit end times (HALF = 2, see below) the byte address / 4.  The arrays come first in
// the workgroup's LDS.  Unused predecessor slots name the
// candidate's dummy cell (end time 0, delay 0); a part that does not end its operation names the
// candidate's trash cell instead of v and has duration 0.
//   x = ha(pred0) | ha(pred1) << 16
//   y = ha(pred2) | ha(pred3) << 16
//   z = delta0 | delta1 << 8 | delta2 << 16 | delta3 << 24
//   w = duration | ha(v) << 16
constexpr uint32_t kNotDone16 = 0xFFFFu;
constexpr uint32_t kNotDone32 = 0x80000000u;          // above every time the library accepts (INT32_MAX bounds them)
constexpr int ring_threads(int feeders) { return (2 + feeders) * kWave; }   // relaxer, feeders, accountant

// One shared record per operation part: up to four DAG predecessors (unused slots name the dummy
// node N).  Part i of operation v sits at rec[i * rec_plane + v]; only the last part carries the
// duration.
//   x = u0 | u1 << 16, y = u2 | u3 << 16, z = dur (30 bits) | first_part << 30 | has_more << 31, w = v << 16
struct LdsLayout {
  uint32_t s_stride, pi_stride;                       // bytes per candidate; the state array starts at 0
  uint32_t o_pi, o_ring, o_scr, o_total, o_peak, o_cnt, o_off, o_flag, o_abort, o_over, o_comm, total;
  uint32_t pib_mode;                                  // where the placement bytes are: 0 L2 workspace, 1 LDS, 2 LDS as nibbles
  uint32_t cell_bytes;                                // 2: 16-bit end times, 4: 32-bit
  uint32_t wide;                                      // 1: wide ops (machines instead of delays, durations below 256 * 65535)
  uint32_t win_log2;                                  // window mode: log2 of the cells per candidate (0: one cell per operation)
};

struct RingParams {
  int32_t N, P, Pseg, log_pseg, G, C;
  int32_t optimistic;                  // 1: candidates stopped by the 16-bit range go to fb_list, 0: a deadlock is always a cycle
  int64_t list_stride;                 // uint16 elements per candidate in ws_list
  const uint4 *rec;                    // [parts][rec_plane] shared operator records (times divided by time_scale)
  int32_t rec_plane;                   // records per part plane (>= N)
  int32_t id_bits;                     // order-list entry = node | (parts - 1) << id_bits
  const uint8_t *nparts;               // [N] parts per node, or NULL when every node has one part
  const int32_t *comm;                 // [P*P] channel delays divided by time_scale (all <= 255)
  const int64_t *mem_delta;            // [N]
  const int64_t *weight;               // [N] static memory per operation (eq. (16)), or NULL
  const int64_t *mem_limit;            // [P] memory limit per machine, or NULL
  int64_t sum_dur;                     // in original units
  int32_t time_scale;                  // gcd of every duration and delay
  const int32_t *placement, *rank;     // [C][N]
  uint16_t *ws_list;                   // [C][list_stride]
  uint8_t *ws_pib;                     // [C][pib_stride] placement as one byte per node; entry N = P (the dummy node's machine)
  int64_t pib_stride;
  int32_t *fb_count, *fb_list;         // candidates left to the fallback (the 32-bit form of this kernel, or the general kernel)
  const int32_t *cand_list, *cand_count;   // not NULL: evaluate the candidates cand_list[0 .. *cand_count) instead of 0 .. C-1
  uint32_t spin_cap;                   // bound on relaxer / feeder loop trips
  uint32_t win_magic;                  // window mode: ceil(2^32 / (cells - 3)), for node -> cell name
  int32_t *ws_meta;                    // window mode: [workgroups][4][64] what ingest hands to relaxation: operations per
                                       // lane, start of the lane's list, op parts per lane, flag bits per candidate
  LdsLayout lds;
  OutPtrs out;
};

// FEEDERS feeder wavefronts share a lane's stream: feeder f owns the parts with seq % FEEDERS == f.
// PIBL = 1: the placement bytes of the workgroup's candidates sit in LDS (fastest feeders); PIBL = 0: in an
// L2-resident workspace, which leaves the LDS to more candidates or a deeper ring; PIBL = 2 (P <= 16): in LDS,
// four bits per node.  A nibble cannot name the dummy machine P, so in that mode time starts at kOrigin = 255
// instead of 0: the dummy cell still holds 0, and 0 + any delay <= 255 never exceeds a machine-free time, which
// makes the dummy's placement irrelevant.  The origin is subtracted from the makespan at the end.
// KIND: 0 general; 1 every operation is a single part (at most four DAG predecessors each): the feeders walk
// the order lists directly; 2 at most two DAG predecessors each (single parts as well): the second pair of
// every record and op is the dummy and neither the feeders nor the relaxer look at it; 3 at most one (what is
// left of a pipeline's DAG once the edges that other paths imply are dropped): one end-time read per trip, one
// placement byte and one delay per op.  Chosen by the host.
//
// HALF = 4, the WINDOW mode, for graphs whose edges are short in the order of the node ids (layered graphs): a
// candidate then gets K cells instead of one per operation, K a power of two chosen by the host, and operation v
// uses the cell of its NAME c(v) = (v div (K-3)) * K + 1 + v mod (K-3), slot c mod K; the slots 0, K-2 and K-1 of
// every period stay free for "nothing yet" (name 0), the trash cell and the dummy.  A cell is a 32-bit word, name
// in the upper half, 16-bit end time in the lower one, written with an LDS maximum, so that a later name is never
// replaced by an earlier one.  A reader that finds the name it expects has the end time; an earlier name means
// "not ended yet"; a later name means that the window has moved past an operation somebody still waits for: that
// operation's readers never run, the candidate deadlocks, and at the deadlock the later name tells the miss from a
// cycle: the candidate goes to the int32 kernel like one stopped by the 16-bit range.  Nothing else changes: node
// ids stay what they are in the lists, the records and the placement bytes; only the feeders turn them into names
// when they pack an op.  The end-time state shrinks from 2 N bytes to 4 K per candidate, and with it the LDS a
// workgroup needs while it relaxes; the order lists, which need 2 N bytes of LDS while they are built, are then
// built by a launch of their own (PHASE = 1: ingest only, hands cnt / off / total / flags over through ws_meta)
// and the relaxation (PHASE = 2) runs with several workgroups per CU.  PHASE = 0 is the fused kernel.
// HALF = 5 is the window mode for end times that need 32 bits: a cell is 64 bits, name above and end time below,
// written with a 64-bit LDS maximum; names, ops and the ingest launch are the same.
template <int RING, int FEEDERS, int HALF, int PIBL, int KIND = 0, int PHASE = 0>
__global__ __launch_bounds__(1024) void relax_ring_kernel(RingParams p) {
  // ring_threads(FEEDERS) threads have a role while the schedule is relaxed; the host may launch more (a
  // multiple of 64): the extra wavefronts only help with ingest and then wait at the final barrier.
  const int kThreads = (int)blockDim.x;
  constexpr int kFeeders = FEEDERS;
  extern __shared__ __align__(16) unsigned char lds[];
  static_assert((RING & (RING - 1)) == 0, "RING must be a power of two");
  static_assert(RING >= FEEDERS, "every feeder needs a slot of its own");
  static_assert(KIND >= 0 && KIND <= 3, "general, single parts, two predecessors, one predecessor");
  static_assert(KIND != 3 || HALF <= 1, "the one-predecessor kind is built for the 16-bit cells only");
  static_assert(HALF >= 0 && HALF <= 5, "byte, half or quarter addresses; 3: quarter addresses and delays looked up by the relaxer; 4, 5: window");
  static_assert(PHASE >= 0 && PHASE <= 2, "fused, ingest only, relaxation only");
  constexpr bool kWin = HALF == 4 || HALF == 5;             // a window of named cells per candidate
  constexpr bool kWin32 = HALF == 5;                        // ... of 64 bits: name above, 32-bit end time below
  static_assert(!kWin || PIBL == 0, "window mode keeps the placement bytes in the workspace row");
  static_assert(kWin || PHASE == 0, "only the window mode is split into two launches");
  constexpr bool kCell32 = HALF == 2 || HALF == 3;          // 32-bit end times
  constexpr bool kWide = HALF == 3;                         // ops name machines, not delays; durations below 256 * 65535
  constexpr int kAsh = kCell32 ? 2 : kWin ? 0 : HALF;       // 16-bit address -> LDS byte address
  static_assert(!(kWide && PIBL == 2), "wide ops need the dummy machine, which a nibble cannot name");
  constexpr uint32_t kNotDone = (kCell32 || kWin32) ? kNotDone32 : kNotDone16;
  constexpr int kNodeShift = (kCell32 || kWin) ? 0 : 1 - HALF;   // node -> offset of its cell in the units of the 16-bit addresses
  constexpr int PR = KIND == 3 ? 1 : KIND == 2 ? 2 : 4;     // DAG predecessors per op
  constexpr uint32_t kOrigin = PIBL == 2 ? 255u : 0u;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int N = p.N, P = p.P, Pseg = p.Pseg, G = p.G;
  const int L = G * Pseg;                                   // lanes in use per wavefront
  const int64_t c0 = (int64_t)blockIdx.x * G;
  // (a launch over a list of candidates is sized for the longest list possible: the workgroups beyond its end leave)
  const int64_t n_todo = p.cand_list ? (int64_t)*p.cand_count : (int64_t)p.C;
  if (c0 >= n_todo) return;
  const int ng = (int)min((int64_t)G, n_todo - c0);
  auto cid = [&](int gg) -> int64_t { return p.cand_list ? (int64_t)p.cand_list[c0 + gg] : c0 + gg; };
  const LdsLayout &o = p.lds;
  lds_byte_t *const ldsb = (lds_byte_t *)lds;

  uint32_t *ringw = (uint32_t *)(lds + o.o_ring);
  uint32_t *totalw = (uint32_t *)(lds + o.o_total);        // [64] ops (operation parts) in the lane's stream
  int64_t *peakw = (int64_t *)(lds + o.o_peak);            // [64]
  int32_t *cntw = (int32_t *)(lds + o.o_cnt);              // [64] operations per (candidate, machine)
  int32_t *offw = (int32_t *)(lds + o.o_off);              // [64] start of the machine inside the list
  int32_t *flagw = (int32_t *)(lds + o.o_flag);            // [64] (G used)
  int32_t *abortw = (int32_t *)(lds + o.o_abort);          // [64] (G used) 0, 1 = stopped by the 16-bit range (or internal), 2 = cycle
  // [64] (G used) 1 = some machine of the candidate is over its memory limit.  Kept apart from flagw, which every
  // wavefront reads when it takes up its role: the accountant finds this out while the others are already relaxing.
  uint8_t *overb = lds + o.o_over;
  uint8_t *commb = (uint8_t *)(lds + o.o_comm);            // [(P+1)][Pseg], diagonal and dummy row zero

  // window mode: names of the dummy node and of the trash cell, cells per candidate
  const uint32_t win_mask = kWin ? (1u << o.win_log2) - 1u : 0u;
  const uint32_t win_dummy = win_mask, win_trash = win_mask - 1u;
  int32_t *const meta = kWin ? p.ws_meta + (int64_t)blockIdx.x * 4 * kWave : nullptr;
  // window mode: the name of a node's cell (the dummy node N has the dummy's name)
  auto name_of = [&](uint32_t v) -> uint32_t {
    return v == (uint32_t)p.N ? win_dummy : v + 3u * __umulhi(v, p.win_magic) + 1u;
  };
  // ---------------------------------------------------------------- ingest (all wavefronts)
  if (tid < kWave) {
    if (PHASE != 2) { cntw[tid] = 0; totalw[tid] = 0; flagw[tid] = 0; }
    else { cntw[tid] = meta[tid]; offw[tid] = meta[kWave + tid]; totalw[tid] = (uint32_t)meta[2 * kWave + tid]; flagw[tid] = meta[3 * kWave + tid]; }
    abortw[tid] = 0; peakw[tid] = 0; overb[tid] = 0;
  }
  if (PHASE != 1)
  for (int i = tid; i < RING * kWave; i += kThreads) {     // every slot free, as if ops -RING .. -1 had been taken
    // (a free slot is copied and looked at like an op: some cell of the workgroup, no delay)
    ringw[4 * i + 0] = ringw[4 * i + 1] = kWin ? win_dummy * 0x10001u : ((uint32_t)(uintptr_t)ldsb >> kAsh) * 0x10001u;
    ringw[4 * i + 2] = 0;
    ringw[4 * i + 3] = kNotDone16 | ((uint32_t)((i >> 6) - RING) << 16);
  }
  if (PHASE == 1) {
  } else if (kWide) {                                       // 64 rows of Pseg dwords (any six-bit machine id stays inside)
    uint32_t *commw = (uint32_t *)(lds + o.o_comm);
    for (int i = tid; i < kWave * Pseg; i += kThreads) {
      const int a = i >> p.log_pseg, b = i & (Pseg - 1);
      commw[i] = (a < P && b < P && a != b) ? (uint32_t)p.comm[a * P + b] : 0u;
    }
  } else {
    for (int i = tid; i < (P + 1) * Pseg; i += kThreads) {  // rows of Pseg bytes: [source machine][destination]
      const int a = i >> p.log_pseg, b = i & (Pseg - 1);
      commb[i] = (a < P && b < P && a != b) ? (uint8_t)p.comm[a * P + b] : (uint8_t)0;
    }
  }
  // The candidates of the workgroup are ingested side by side, a team of kThreads / G consecutive threads
  // each, so that small problems do not pay one round of load latency per candidate.
  const int n_teams = G;
  const int tpc = kThreads / n_teams;
  const int team = tid / tpc, tt = tid - team * tpc;        // this thread's team and its place in it
  if (PHASE != 2) {
  // The order lists are first built in LDS, over the (not yet used) end-time arrays: every entry starts as
  // "unwritten" (0xFFFF, which no list entry equals: the host checks that)
  for (int gg = team; gg < ng; gg += n_teams) {
    uint32_t *lw = (uint32_t *)(lds + gg * o.s_stride);
    for (int i = tt; i < (N + 1) / 2; i += tpc) lw[i] = 0xFFFFFFFFu;
  }
  __syncthreads();

  // 16-byte loads a thread keeps in flight per row pass (measured: eight instead of four 5 % on config 2, 2 % on
  // config 5; with the general kind's register needs 2 % slower on config 4)
  constexpr int kIn = KIND == 0 ? 4 : 8;
  const bool vec_ok = ((N & 3) == 0) && ((((uintptr_t)p.placement) | ((uintptr_t)p.rank)) & 15) == 0;
  const int nq = N >> 2;

  // placement in range (eq. (6)), operations per machine
  for (int gg = team; gg < ng; gg += n_teams) {
    const int32_t *pl = p.placement + cid(gg) * N;
    uint8_t *pib = PIBL ? lds + o.o_pi + gg * o.pi_stride : p.ws_pib + cid(gg) * p.pib_stride;
    int32_t *cnt_g = cntw + gg * Pseg;
    if (PIBL == 2) { if (tt == 0 && !(N & 1)) pib[N >> 1] = 0; }   // the dummy's nibble: any machine will do
    else if (tt == 0) pib[N] = (uint8_t)P;                  // the dummy node sits on a dummy machine whose delays are all zero
    if (vec_ok) {
      const int4 *pl4 = (const int4 *)pl;
      uint32_t *piw = (uint32_t *)pib;
      uint16_t *pih = (uint16_t *)pib;
      for (int q0 = tt; q0 < nq; q0 += kIn * tpc) {
        int4 a[kIn];
#pragma unroll
        for (int u = 0; u < kIn; ++u) {
          const int q = q0 + u * tpc;
          a[u] = (q < nq) ? pl4[q] : make_int4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < kIn; ++u) {
          const int q = q0 + u * tpc;
          if (q < nq) {
            const uint32_t hi = (uint32_t)a[u].x | (uint32_t)a[u].y | (uint32_t)a[u].z | (uint32_t)a[u].w;
            const bool bad = hi >= 64u || a[u].x >= P || a[u].y >= P || a[u].z >= P || a[u].w >= P;
            if (bad) {
              atomicOr(&flagw[gg], kBitBadPlacement);
            } else {
              if (PIBL == 2) pih[q] = (uint16_t)((uint32_t)a[u].x | ((uint32_t)a[u].y << 4) | ((uint32_t)a[u].z << 8) | ((uint32_t)a[u].w << 12));
              else piw[q] = (uint32_t)a[u].x | ((uint32_t)a[u].y << 8) | ((uint32_t)a[u].z << 16) | ((uint32_t)a[u].w << 24);
              atomicAdd(&cnt_g[a[u].x], 1); atomicAdd(&cnt_g[a[u].y], 1);
              atomicAdd(&cnt_g[a[u].z], 1); atomicAdd(&cnt_g[a[u].w], 1);
            }
          }
        }
      }
    } else if (PIBL == 2) {
      for (int h = tt; 2 * h < N; h += tpc) {               // two nodes per thread: one byte of nibbles (node N is the dummy)
        const int32_t pa = pl[2 * h], pb = (2 * h + 1 < N) ? pl[2 * h + 1] : 0;
        if ((uint32_t)pa >= (uint32_t)P || (uint32_t)pb >= (uint32_t)P) {
          atomicOr(&flagw[gg], kBitBadPlacement);
        } else {
          pib[h] = (uint8_t)(pa | (pb << 4));
          atomicAdd(&cnt_g[pa], 1);
          if (2 * h + 1 < N) atomicAdd(&cnt_g[pb], 1);
        }
      }
    } else {
      for (int v = tt; v < N; v += tpc) {
        const int32_t pi = pl[v];
        if ((uint32_t)pi >= (uint32_t)P) {
          atomicOr(&flagw[gg], kBitBadPlacement);
        } else {
          pib[v] = (uint8_t)pi;
          atomicAdd(&cnt_g[pi], 1);
        }
      }
    }
  }
  __syncthreads();
  if (wave == 0) {                                          // exclusive prefix over the machines of each candidate
    const int my = lane < L ? cntw[lane] : 0;
    int incl = my;
    const int jj = lane & (Pseg - 1);
    for (int d = 1; d < Pseg; d <<= 1) {
      const int t = __shfl_up(incl, d, Pseg);
      if (jj >= d) incl += t;
    }
    if (lane < L) offw[lane] = incl - my;
  }
  __syncthreads();
  // dense ranks (eqs. (7)-(8)): every rank inside its machine's range and, after N writes into N slots,
  // no slot left unwritten <=> every (machine, rank) slot hit exactly once
  for (int gg = team; gg < ng; gg += n_teams) {
    if (flagw[gg] & kBitBadPlacement) continue;
    const int32_t *rk = p.rank + cid(gg) * N;
    const uint8_t *pib = PIBL ? lds + o.o_pi + gg * o.pi_stride
                              : p.ws_pib + cid(gg) * p.pib_stride;   // written by this workgroup before the barrier above
    uint16_t *lds_list = (uint16_t *)(lds + gg * o.s_stride);
    const int32_t *cnt_g = cntw + gg * Pseg, *off_g = offw + gg * Pseg;
    int32_t *flag_g = flagw + gg;
    // list entry: node | (parts - 1) << id_bits
    uint32_t *extra_g = totalw + gg * Pseg;                 // parts beyond the first, per machine
    auto place = [&](int v, int pi, int32_t r, uint32_t np1) {
      if ((uint32_t)r >= (uint32_t)cnt_g[pi]) {
        atomicOr(flag_g, kBitBadRank);
      } else {
        lds_list[off_g[pi] + r] = (uint16_t)((uint32_t)v | (np1 << p.id_bits));
        if (KIND == 0 && np1) atomicAdd(&extra_g[pi], np1);
      }
    };
    if (vec_ok) {
      const int4 *rk4 = (const int4 *)rk;
      const uint32_t *piw = (const uint32_t *)pib;
      const uint16_t *pih = (const uint16_t *)pib;
      const uint32_t *np4 = (const uint32_t *)p.nparts;     // four part counts per load (N % 4 == 0 here)
      for (int q0 = tt; q0 < nq; q0 += kIn * tpc) {
        int4 a[kIn];
        uint32_t npw[kIn];
#pragma unroll
        for (int u = 0; u < kIn; ++u) {
          const int q = q0 + u * tpc;
          a[u] = (q < nq) ? rk4[q] : make_int4(0, 0, 0, 0);
          npw[u] = (np4 && q < nq) ? np4[q] - 0x01010101u : 0u;   // every count is at least 1: no borrow between bytes
        }
#pragma unroll
        for (int u = 0; u < kIn; ++u) {
          const int q = q0 + u * tpc;
          if (q < nq) {
            uint32_t pw;
            if (PIBL == 2) {                                  // four nibbles, spread to four bytes
              const uint32_t h = pih[q];
              pw = (h & 0xFu) | ((h & 0xF0u) << 4) | ((h & 0xF00u) << 8) | ((h & 0xF000u) << 12);
            } else {
              pw = piw[q];
            }
            place(4 * q + 0, pw & 0xFF, a[u].x, npw[u] & 0xFF);
            place(4 * q + 1, (pw >> 8) & 0xFF, a[u].y, (npw[u] >> 8) & 0xFF);
            place(4 * q + 2, (pw >> 16) & 0xFF, a[u].z, (npw[u] >> 16) & 0xFF);
            place(4 * q + 3, pw >> 24, a[u].w, npw[u] >> 24);
          }
        }
      }
    } else {
      for (int v = tt; v < N; v += tpc)
        place(v, PIBL == 2 ? (pib[v >> 1] >> ((v & 1) << 2)) & 0xF : pib[v], rk[v], p.nparts ? (uint32_t)p.nparts[v] - 1u : 0u);
    }
  }
  __syncthreads();
  // order lists to HBM (coalesced), looking for unwritten slots on the way
  for (int gg = team; gg < ng; gg += n_teams) {
    if (flagw[gg] & kBitBadPlacement) continue;
    const uint32_t *lw = (const uint32_t *)(lds + gg * o.s_stride);
    uint32_t *gw = (uint32_t *)(p.ws_list + cid(gg) * p.list_stride);       // rows are 128-byte aligned
    bool hole = false;
    for (int i = tt; i < (N + 1) / 2; i += tpc) {
      const uint32_t w = lw[i];
      hole |= (w & 0xFFFFu) == 0xFFFFu || (2 * i + 1 < N && (w >> 16) == 0xFFFFu);
      gw[i] = w;
    }
    if (hole) atomicOr(&flagw[gg], kBitBadRank);
  }
  __syncthreads();                                          // workgroup scope: the lists are read by this workgroup only
  if (tid < kWave) totalw[tid] += (uint32_t)cntw[tid];      // ops per lane: its operations plus their further parts
  if (PHASE == 1) {                                         // the relaxation is a launch of its own
    if (tid < kWave) { meta[tid] = cntw[tid]; meta[kWave + tid] = offw[tid]; meta[2 * kWave + tid] = (int32_t)totalw[tid]; meta[3 * kWave + tid] = flagw[tid]; }
    return;
  }
  }
  // end-time state: every operation "not ended"; the dummy node N has ended at time 0 on a dummy
  // machine P whose delays are all zero; cell N+1 is a trash cell for parts that do not end an operation
  for (int gg = team; gg < ng; gg += n_teams) {
    uint32_t *sw = (uint32_t *)(lds + gg * o.s_stride);
    if (kWin) {                                             // no name anywhere, but the dummy's in its slot, ended at 0
      if (kWin32) {
        for (uint32_t i = (uint32_t)tt; i <= win_mask; i += (uint32_t)tpc) { sw[2 * i] = 0u; sw[2 * i + 1] = i == win_dummy ? win_dummy : 0u; }
      } else {
        for (uint32_t i = (uint32_t)tt; i <= win_mask; i += (uint32_t)tpc) sw[i] = i == win_dummy ? win_dummy << 16 : 0u;
      }
    } else if (kCell32) {
      for (int i = tt; i < N + 2; i += tpc) sw[i] = i < N ? kNotDone32 : 0u;
    } else {
      for (int i = tt; i < (N + 3) / 2; i += tpc) {
        const uint32_t lo = (2 * i < N) ? kNotDone16 : 0u, hi = (2 * i + 1 < N) ? kNotDone16 : 0u;
        sw[i] = lo | (hi << 16);
      }
    }
  }
  __syncthreads();

  // ---------------------------------------------------------------- roles
  const bool lane_on = lane < L;
  const int ql = lane_on ? lane : 0;
  const int g = ql >> p.log_pseg, j = ql & (Pseg - 1);
  const bool cand_ok = lane_on && g < ng && flagw[g] == 0;
  const bool has_ops = cand_ok && j < P && cntw[ql] > 0;
  // 16-bit address of this candidate's cell 0: LDS addresses (halved when HALF), so that the relaxer uses them as they are
  const uint32_t sbase = ((uint32_t)(uintptr_t)ldsb >> kAsh) + (uint32_t)g * (o.s_stride >> kAsh);
  // window mode: LDS byte address of the cell of a name (sbase is then the byte address of the candidate's cells)
  auto win_addr = [&](uint32_t name) -> uint32_t { return sbase + ((name & win_mask) << (kWin32 ? 3 : 2)); };

  int32_t acc = 0;
  bool stalled = false;

  if (wave == 0) {
    // ------------------------------------------------------------ relaxer
    lds_byte_t *const ring_lane = ldsb + o.o_ring + (uint32_t)lane * 16u;   // ring layout: [slot][lane] of 16 bytes
    // the lane is through when it has taken this many ops (counted at ingest) and holds none: tm then equals this
    const uint32_t tm_end = (totalw[lane] << 16) | kNotDone16;
    lds_vi32_t *const abort_p = (lds_vi32_t *)(ldsb + o.o_abort) + g;
    const uint64_t segmask = ((Pseg == kWave) ? ~0ull : ((1ull << Pseg) - 1ull)) << (g * Pseg);
    auto cell = [&](uint32_t a16) -> uint32_t {
      if (kWin) return *(lds_vu32_t *)(uintptr_t)win_addr(a16);     // name << 16 | end time
      return kCell32 ? *(lds_vu32_t *)(uintptr_t)(a16 << 2) : (uint32_t)*(lds_vu16_t *)(uintptr_t)(a16 << kAsh);
    };
    // window mode: where a lane that ran nothing (or a part that ends no operation) leaves its value: a dword of its
    // own.  The cells are written with an LDS maximum, and lanes that aim one at the same address are served one
    // after the other, unlike plain stores: a shared trash cell cost 40 % of the LDS pipe's time.
    const uint32_t own_trash = (uint32_t)(uintptr_t)(ldsb + o.o_scr) + (uint32_t)lane * (kWin32 ? 8u : 4u);
    auto set_cell = [&](uint32_t a16, uint32_t v) {
      // (window: the maximum keeps a later name from being replaced by an earlier one)
      if (kWin32) (void)__hip_atomic_fetch_max((DAGSCHED_LDS uint64_t *)(uintptr_t)(a16 == win_trash ? own_trash : win_addr(a16)),
                                              ((uint64_t)a16 << 32) | v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      else if (kWin) (void)__hip_atomic_fetch_max((DAGSCHED_LDS uint32_t *)(uintptr_t)(a16 == win_trash ? own_trash : win_addr(a16)),
                                            (a16 << 16) | v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      else if (kCell32) *(lds_vu32_t *)(uintptr_t)(a16 << 2) = v;
      else *(lds_vu16_t *)(uintptr_t)(a16 << kAsh) = (uint16_t)v;
    };
    const uint32_t dummy = kWin ? win_dummy : sbase + ((uint32_t)N << kNodeShift);
    // The loop body is branch-free: every trip stores x somewhere (the trash cell unless an op ran).
    const uint32_t trash = kWin ? win_trash : sbase + (((uint32_t)N + 1u) << kNodeShift);
    __builtin_amdgcn_s_setprio(3);                          // the relaxer's trip is the critical path of the workgroup:
                                                            // it goes first wherever it shares a SIMD (measured: 4-5 % on the MoE workload)
    bool idle = true, dead = !has_ops;                      // idle: the registers hold a free slot's content, not an op
    uint32_t x_acc = kOrigin;                               // the machine is free from the time origin on
    // ops taken from the ring, as t << 16 | 0xFFFF: the free mark that the slot of op t gets when op t is taken
    // (the host sends a problem with 65536 op parts or more to the general kernel)
    uint32_t tm = kNotDone16;
    constexpr uint32_t kSlotMask = (uint32_t)(RING - 1) << 10;
    // where lanes that take nothing write their "slot free" mark (the store adds 12, the place of a slot's last dword)
    lds_byte_t *const scr_m12 = ldsb + o.o_scr + (uint32_t)lane * (kWin32 ? 8u : 4u) - 12u;
    // "This lane holds no op": the registers hold the content of a free slot, whose "duration" 0xFFFF can never
    // run; such a lane copies slot t again in every trip until an op is there.
    const uint32_t z0 = dummy | (dummy << 16);
    uint32_t w0 = z0, w1 = z0, w2 = 0, w3 = kNotDone16;     // current op, in ring format
    uint64_t prog_acc = 0;
    bool expired = true;
    lds_byte_t *slot_p = ring_lane;                         // ring slot of op t
    u32x4_t r = *(lds_vu32x4_t *)slot_p;                    // ... as read during the previous trip
    // end times of the current op's predecessors, read at the end of the previous trip
    // (64-bit window cells: the time in e, the name in n)
    uint32_t n0 = 0, n1 = 0, n2 = 0, n3 = 0;
    auto read_cell = [&](uint32_t a16, uint32_t &e, uint32_t &n) {
      if (kWin32) { const uint64_t c = *(lds_vu64_t *)(uintptr_t)win_addr(a16); e = (uint32_t)c; n = (uint32_t)(c >> 32); }
      else e = cell(a16);
    };
    uint32_t e0, e1, e2, e3;
    read_cell(dummy, e0, n0);
    e1 = e2 = e3 = e0; n1 = n2 = n3 = n0;
    // wide ops: the delays of the current op's predecessors, looked up together with the end times
    lds_vu32_t *const commw = (lds_vu32_t *)(ldsb + o.o_comm) + j;
    const uint32_t lps = (uint32_t)p.log_pseg;
    uint32_t d0 = 0, d1 = 0, d2 = 0, d3 = 0;
    // The test for deadlocks costs about as much as a trip and the jump back to the top of the loop a little less, so
    // the loop is unrolled 32 times with the deadlock test once per pass (1.22 -> 1.09 ms on the MoE workload against
    // 8 times); "all through" is looked for every 8 trips with two predecessors per op (the pipelines: short lists),
    // else every 16 (1-2 % either way).
    constexpr int kEndMask = KIND >= 2 ? 7 : 15;
    for (uint32_t it = 0; it < p.spin_cap; it += 32) {
#pragma unroll
      for (int sub = 0; sub < 32; ++sub) {
        const bool empty = (r.w & 0xFFFFu) == kNotDone16;   // slot t does not hold op t yet
        uint32_t x;
        bool ran;
        if (kWide) {
          // (the sentinel plus a delay stays below 2^32; whatever ended, plus delay and duration, below 2^31: the
          // library accepts no problem whose times could pass INT32_MAX)
          x = max(max(x_acc, e0 + d0), e1 + d1);
          if (PR == 4) x = max(max(x, e2 + d2), e3 + d3);
          ran = x < kNotDone && !idle;
          // duration = low + 65535 * high: the low part, which shares the slot's last dword with the free mark, is
          // then never 0xFFFF
          const uint32_t hi = w2 >> 24;
          x += (w3 & 0xFFFFu) + (hi << 16) - hi;
        } else if (kWin32) {
          bool named = (n0 == (w0 & 0xFFFFu)) & (n1 == (w0 >> 16));
          if (PR == 4) named = named & (n2 == (w1 & 0xFFFFu)) & (n3 == (w1 >> 16));
          x = max(max(x_acc, e0 + (w2 & 0xFFu)), e1 + (PR == 4 ? (w2 >> 8) & 0xFFu : w2 >> 8));
          if (PR == 4) x = max(max(x, e2 + ((w2 >> 16) & 0xFFu)), e3 + (w2 >> 24));
          x += w3 & 0xFFFFu;
          ran = named && !idle;                               // (the library accepts no problem whose times could pass INT32_MAX)
        } else if (kWin) {
          // a predecessor has ended when its cell carries its name; the end time is the cell's lower half
          // (no short-circuit: the trip stays free of branches)
          bool named = ((e0 >> 16) == (w0 & 0xFFFFu)) & ((e1 >> 16) == (w0 >> 16));
          if (PR == 4) named = named & ((e2 >> 16) == (w1 & 0xFFFFu)) & ((e3 >> 16) == (w1 >> 16));
          x = max(max(x_acc, (e0 & 0xFFFFu) + (w2 & 0xFFu)), (e1 & 0xFFFFu) + (PR == 4 ? (w2 >> 8) & 0xFFu : w2 >> 8));
          if (PR == 4) x = max(max(x, (e2 & 0xFFFFu) + ((w2 >> 16) & 0xFFu)), (e3 & 0xFFFFu) + (w2 >> 24));
          x += w3 & 0xFFFFu;
          ran = named && x < kNotDone;                        // (a free slot's "duration" 0xFFFF lifts x over the range)
        } else {
          if (PR == 1) x = max(x_acc, e0 + w2);
          else x = max(max(x_acc, e0 + (w2 & 0xFFu)), e1 + (PR == 4 ? (w2 >> 8) & 0xFFu : w2 >> 8));
          if (PR == 4) x = max(max(x, e2 + ((w2 >> 16) & 0xFFu)), e3 + (w2 >> 24));
          x += w3 & 0xFFFFu;
          // an op, every predecessor ended and no 16-bit overflow (a free slot's "duration" 0xFFFF lifts x over the
          // 16-bit sentinel, not over the 32-bit one: there the lane's state is asked)
          ran = kCell32 ? (x < kNotDone && !idle) : x < kNotDone;
        }
        x_acc = ran ? x : x_acc;                            // the machine is busy until x (chain edge, eq. (7))
        set_cell(ran ? (w3 >> 16) : trash, x);
        const bool next = ran || idle;                      // the registers take the content of slot t
        const bool idle_next = next && empty;               // ... which is still free: nothing held (not next: an op is held)
        const bool take = next ^ idle_next;                 // ... which is op t
        // The ring slot for the next trip.  With four predecessors per op it is requested before the end times
        // (it arrives first, and what depends on it is done while they are on their way: 1-5 %); with two, where
        // the feeders are what limits, after everything else (a delivery is then seen a little earlier: 1-3 %).
        const uint32_t mark = tm;                           // "free, op t was the last one taken from here"
        tm += take ? 0x10000u : 0u;
        lds_byte_t *const next_p = ring_lane + ((tm >> 6) & kSlotMask);
        const uint32_t c0 = r.x, c1 = r.y, c2 = r.z, c3 = r.w;
        if (PR == 4) r = *(lds_vu32x4_t *)next_p;
        w0 = next ? c0 : w0;
        if (PR == 4) w1 = next ? c1 : w1;
        // The end-time reads of the next trip (LDS accesses keep their program order, so everything below
        // overlaps with their latency).
        read_cell(w0 & 0xFFFFu, e0, n0);
        if (PR >= 2) read_cell(w0 >> 16, e1, n1);
        if (PR == 4) { read_cell(w1 & 0xFFFFu, e2, n2); read_cell(w1 >> 16, e3, n3); }
        if (kWide) {
          const uint32_t m = next ? c2 : w2;                // (w2 itself is updated below)
          d0 = commw[(m & 63u) << lps]; d1 = commw[((m >> 6) & 63u) << lps];
          if (PR == 4) { d2 = commw[((m >> 12) & 63u) << lps]; d3 = commw[((m >> 18) & 63u) << lps]; }
        }
        // One trip without progress while every unfinished machine holds an op is already a deadlock
        // (end times only change when some op runs), so progress is sampled once per window.
        if (sub == 31) prog_acc = __ballot(ran || take);    // an op taken now has not been tested yet
        idle = idle_next;
        w2 = next ? c2 : w2;
        w3 = next ? c3 : w3;
        // the slot just copied is free again: its last dword says so (and which op left it) to the feeders
        *(lds_vu32_t *)((take ? slot_p : scr_m12) + 12) = mark;
        slot_p = next_p;
        if (PR != 4) r = *(lds_vu32x4_t *)next_p;
        if ((sub & kEndMask) == kEndMask && sub != 31 && __ballot(!(dead || (idle && tm == tm_end))) == 0) { expired = false; goto relaxed; }
      }
      const bool fin = dead || (idle && tm == tm_end);
      const uint64_t open = __ballot(!fin);
      if (open == 0) { expired = false; break; }
      // Deadlock: every unfinished machine of a candidate holds an op and none of its machines ran or took an op
      // in the sampled trip.  The test is kept cheap (it runs once per window for every lane); what follows a
      // deadlock is rare and sits behind a branch that the whole wavefront takes or skips.
      const uint64_t stuck = (__ballot(!idle) | ~open) & ~prog_acc;
      const bool deadlock = !fin && (stuck & segmask) == segmask;
      if (__ballot(deadlock) != 0) {
        // If one of the held ops has all its predecessors ended, only the 16-bit range stopped it (optimistic
        // mode: the int32 kernel takes the candidate); otherwise every held op waits for an op that can never
        // run, i.e. the combined graph has a cycle.
        // (window mode: likewise when every predecessor's cell carries its name; and a cell that carries a LATER name
        // says that the window moved past a predecessor this op still waits for: the int32 kernel's candidate, too)
        bool win_stop = false;
        if (kWin) {
          const uint32_t m0 = kWin32 ? n0 : e0 >> 16, m1 = kWin32 ? n1 : e1 >> 16, i0 = w0 & 0xFFFFu, i1 = w0 >> 16;
          bool named = m0 == i0 && m1 == i1, later = m0 > i0 || m1 > i1;
          if (PR == 4) {
            const uint32_t m2 = kWin32 ? n2 : e2 >> 16, m3 = kWin32 ? n3 : e3 >> 16, i2 = w1 & 0xFFFFu, i3 = w1 >> 16;
            named = named && m2 == i2 && m3 == i3;
            later = later || m2 > i2 || m3 > i3;
          }
          win_stop = named || later;
        }
        const bool range_stop = deadlock && !idle && (kWin ? win_stop : max(max(e0, PR >= 2 ? e1 : 0u), PR == 4 ? max(e2, e3) : 0u) < kNotDone);
        const bool overflow = (__ballot(range_stop) & segmask) != 0;
        if (deadlock) *abort_p = overflow ? 1 : 2;
        stalled = stalled || deadlock;
        dead = dead || deadlock;
      }
      prog_acc = 0;
    }
  relaxed:
    if (expired) {                                          // bounded wait ran out: report, release the feeder
      const bool fin = dead || (idle && tm == tm_end);
      if (!fin) { flagw[g] = kBitInternal; *abort_p = 1; }
    }
    acc = (int32_t)(x_acc - kOrigin);
  } else if (wave <= kFeeders) {
    // ------------------------------------------------------------ feeders
    // Per lane the op parts of machine j form a stream (the parts of one operation are consecutive;
    // the order-list entry of a node carries its part count, so the stream is known from the ids
    // alone).  Feeder f owns every kFeeders-th part.  A part is ADMITTED when the relaxer has copied the
    // previous part out of its ring slot, then moves through a fixed pipeline without ever stalling:
    //   trip t    record requested from L2
    //   trip t+1  placement bytes of its predecessors requested (L2), or read from LDS
    //   trip t+2  (trip t+1 when the placement bytes are in LDS) channel delays read from LDS, op packed
    //             and written to the ring
    // The loop is unrolled by the pipeline depth so that the registers rotate by renaming, not by moves.
    const int f = wave - 1;
    const uint8_t *const pib_g = p.ws_pib + cid(cand_ok ? g : 0) * p.pib_stride;   // L2-resident: this workgroup wrote it
    lds_cu8_t *const pib_l = (lds_cu8_t *)(ldsb + o.o_pi + g * o.pi_stride);
    auto pib = [&](uint32_t u) -> uint32_t {
      if (PIBL == 2) return ((uint32_t)pib_l[u >> 1] >> ((u & 1u) << 2)) & 0xFu;
      return PIBL ? (uint32_t)pib_l[u] : (uint32_t)pib_g[u];
    };
    lds_cu8_t *const commr = (lds_cu8_t *)(ldsb + o.o_comm) + j;
    lds_byte_t *const ring_lane = ldsb + o.o_ring + (uint32_t)lane * 16u;
    lds_vi32_t *const abort_p = (lds_vi32_t *)(ldsb + o.o_abort) + g;
    const uint16_t *list = p.ws_list + cid(cand_ok ? g : 0) * p.list_stride;
    const uint32_t base2 = sbase | (sbase << 16);
    const uint32_t trash = kWin ? win_trash : sbase + (((uint32_t)N + 1u) << kNodeShift);
    const uint32_t vbits = (uint32_t)p.id_bits, vmask = (1u << vbits) - 1u;
    const uint32_t n_plane = (uint32_t)p.rec_plane;
    const uint32_t lps = (uint32_t)p.log_pseg;
    const uint32_t k0 = has_ops ? (uint32_t)offw[ql] : 1u;
    const uint32_t klast = has_ops ? k0 + (uint32_t)cntw[ql] - 1u : 0u;   // list position of the lane's last node
    bool pending = false;
    uint32_t admitted = 0, written = 0;
    uint32_t aseq = (uint32_t)f;                            // index in the lane's stream of the next part to admit
    uint32_t wseq = (uint32_t)f;                            // ... of the next part to write
    // cursor: the next part to admit is the record at `addr`; `rem` more parts of the same node follow;
    // the node sits at list position k, and k > klast means the stream is exhausted
    // When every operation is a single part, feeder f simply owns the nodes at list positions k0 + f,
    // k0 + f + kFeeders, ... and looks one of them ahead.
    constexpr bool kSingle = KIND != 0;
    uint32_t k = kSingle ? k0 + (uint32_t)f : k0;
    const uint32_t w0 = has_ops ? (uint32_t)list[min(k, klast)] : 0u;
    uint32_t addr = w0 & vmask, rem = kSingle ? 0u : w0 >> vbits;
    // list entries of the next kFeeders nodes: one trip moves the cursor by kFeeders parts, so it can
    // enter at most that many nodes
    uint32_t ids[kFeeders];
#pragma unroll
    for (int i = 0; i < kFeeders; ++i) ids[i] = has_ops ? (uint32_t)list[min(k0 + 1u + (uint32_t)i, klast)] : 0u;
    // move the cursor one part ahead
    auto advance = [&]() {
      const bool in_node = rem != 0;
      addr = in_node ? addr + n_plane : (ids[0] & vmask);
      rem = in_node ? rem - 1u : (ids[0] >> vbits);
      k += in_node ? 0u : 1u;
#pragma unroll
      for (int i = 0; i + 1 < kFeeders; ++i) ids[i] = in_node ? ids[i] : ids[i + 1];
    };
    if (kSingle) {
      ids[0] = has_ops ? (uint32_t)list[min(k + (uint32_t)kFeeders, klast)] : 0u;
    } else {
      for (int i = 0; i < f; ++i) advance();                // feeder f starts at its first own part
#pragma unroll
      for (int i = 0; i < kFeeders; ++i) ids[i] = has_ops ? (uint32_t)list[min(k + 1u + (uint32_t)i, klast)] : 0u;
    }
    struct Entry { uint4 rec; uint32_t q0, q1, q2, q3, fl; };   // fl: 1 valid
    constexpr int kStages = PIBL ? 2 : 3;
    Entry E[kStages];
#pragma unroll
    for (int i = 0; i < kStages; ++i) { E[i].rec = make_uint4(0, 0, 0, 0); E[i].q0 = E[i].q1 = E[i].q2 = E[i].q3 = 0; E[i].fl = 0; }

    // The look at the relaxer's "given up" flag and the end test wait for LDS and cost a dozen instructions: once
    // per kRounds turns of the pipeline.  Four turns where the relaxer limits (the general kind: 2 % on the MoE
    // workload); one where the feeders do and a workgroup's last ops are waited for (3 % on the pipelines).
    constexpr int kRounds = KIND == 0 ? 4 : 1;
    for (uint32_t it = 0; it < p.spin_cap; it += kStages * kRounds) {
      if (*abort_p) { k = klast + 1u; written = admitted; }   // the relaxer gave this candidate up
      if (__ballot(!(k > klast && written == admitted)) == 0) break;
#pragma unroll
      for (int s_ = 0; s_ < kStages * kRounds; ++s_) {
        const int s = s_ % kStages;
        Entry &e0 = E[s];                             // admitted in this trip
        Entry &e1 = E[(s + kStages - 1) % kStages];   // admitted one trip ago: its record has arrived
        Entry &e2 = E[(s + 1) % kStages];             // the oldest: written in this trip (e1 itself when the depth is two)
        if (kStages == 2) {
          e1.q0 = pib(e1.rec.x & 0xFFFFu);
          if (PR >= 2) e1.q1 = pib(e1.rec.x >> 16);
          if (PR == 4) { e1.q2 = pib(e1.rec.y & 0xFFFFu); e1.q3 = pib(e1.rec.y >> 16); }
        }
        // (A) channel delays of e2
        // (wide ops carry the machines themselves; the dummy node's machine P becomes this lane's own: no delay)
        const uint32_t d0 = kWide ? (e2.q0 == (uint32_t)P ? (uint32_t)j : e2.q0) : commr[e2.q0 << lps];
        const uint32_t d1 = PR < 2 ? 0u : kWide ? (e2.q1 == (uint32_t)P ? (uint32_t)j : e2.q1) : commr[e2.q1 << lps];
        const uint32_t d2 = PR != 4 ? 0u : kWide ? (e2.q2 == (uint32_t)P ? (uint32_t)j : e2.q2) : commr[e2.q2 << lps];
        const uint32_t d3 = PR != 4 ? 0u : kWide ? (e2.q3 == (uint32_t)P ? (uint32_t)j : e2.q3) : commr[e2.q3 << lps];
        // (1) move the cursor past the part admitted in the previous trip and the other feeders' parts
        // (2) entries of the next nodes (consumed one trip later at the earliest).  Lanes whose cursor stayed
        // keep theirs and all read the same entry instead, which costs the vector cache one line, not one per lane.
        const bool moved = pending;
        if (kSingle) {
          addr = moved ? ids[0] & vmask : addr;
          k += moved ? (uint32_t)kFeeders : 0u;
          aseq += moved ? (uint32_t)kFeeders : 0u;
          const uint32_t t = list[moved ? min(k + (uint32_t)kFeeders, klast) : 0u];
          ids[0] = moved ? t : ids[0];
        } else {
          if (pending) {
#pragma unroll
            for (int a = 0; a < kFeeders; ++a) advance();
            aseq += kFeeders;
          }
#pragma unroll
          for (int i = 0; i < kFeeders; ++i) {
            const uint32_t t = list[moved ? min(k + 1u + (uint32_t)i, klast) : 0u];
            ids[i] = moved ? t : ids[i];
          }
        }
        // (3) admission
        // (measured: with two predecessors per op a branch around the read for exhausted lanes pays, 3 %; else not, 1 %)
        lds_vu32_t *const mark_p = (lds_vu32_t *)(ring_lane + ((aseq & (uint32_t)(RING - 1)) << 10) + 12);
        const uint32_t mark_free = ((aseq - (uint32_t)RING) << 16) | kNotDone16;
        if (KIND >= 2) {
          pending = (k <= klast) && *mark_p == mark_free;
        } else {
          const uint32_t mark = *mark_p;
          pending = (k <= klast) & (mark == mark_free);
        }
        e0.fl = pending ? 1u : 0u;
        e0.rec = p.rec[pending ? addr : 0u];                 // lanes that admit nothing share one record
        admitted += pending ? 1u : 0u;
        // (B) placement bytes of e1's predecessors (its record was requested one trip ago)
        if (kStages == 3) {
          if (!(e1.fl & 1u)) e1.rec.x = e1.rec.y = (uint32_t)N | ((uint32_t)N << 16);   // nothing admitted: the dummy node's byte
          e1.q0 = pib(e1.rec.x & 0xFFFFu);
          if (PR >= 2) e1.q1 = pib(e1.rec.x >> 16);
          if (PR == 4) { e1.q2 = pib(e1.rec.y & 0xFFFFu); e1.q3 = pib(e1.rec.y >> 16); }
        }
        // (D) pack e2 and publish it
        if (e2.fl & 1u) {
          const bool more = !kSingle && (e2.rec.z >> 31) != 0;
          const uint32_t dst = more ? trash : kWin ? name_of(e2.rec.w >> 16) : sbase + ((e2.rec.w >> 16) << kNodeShift);
          const uint32_t dur = e2.rec.z & 0xFFFFu;
          lds_byte_t *const sp = ring_lane + ((wseq & (uint32_t)(RING - 1)) << 10);
          // node ids below 32768 whenever they are shifted, so shifting both halves at once cannot carry over;
          // the whole slot first with its free mark unchanged, then the last dword
          const u32x4_t val = {kWin ? name_of(e2.rec.x & 0xFFFFu) | (name_of(e2.rec.x >> 16) << 16) : (e2.rec.x << kNodeShift) + base2,
                               kWin ? (PR == 4 ? name_of(e2.rec.y & 0xFFFFu) | (name_of(e2.rec.y >> 16) << 16) : win_dummy * 0x10001u)
                                    : (e2.rec.y << kNodeShift) + base2,
                               kWide ? d0 | (d1 << 6) | (d2 << 12) | (d3 << 18) | (((e2.rec.z >> 16) & 0xFFu) << 24)
                                     : d0 | (d1 << 8) | (d2 << 16) | (d3 << 24),
                               ((wseq - (uint32_t)RING) << 16) | kNotDone16};
          *(lds_vu32x4_t *)sp = val;
          *(lds_vu32_t *)(sp + 12) = dur | (dst << 16);
          wseq += kFeeders;
          ++written;
        }
      }
    }
  } else if (wave == kFeeders + 1) {
    // ------------------------------------------------------------ accountant
    // Peak of the running memory level of machine j (eqs. (17)-(19)): it depends on the order only,
    // so one wavefront walks the order lists on its own, four operations per trip.
    const uint16_t *list = p.ws_list + cid(cand_ok ? g : 0) * p.list_stride;
    const uint32_t vmask = (1u << p.id_bits) - 1u;
    const int k0 = has_ops ? offw[ql] : 0;
    const int kend = has_ops ? k0 + cntw[ql] : 0;
    int64_t level = 0, peak = 0, base = 0;                  // level above the machine's base; base = static memory on it (eq. (16))
    for (int k = k0; __ballot(k < kend) != 0; k += 4) {
      uint32_t id[4];
      int64_t m[4], wt[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) id[u] = (k + u < kend) ? ((uint32_t)list[k + u] & vmask) : 0u;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        m[u] = p.mem_delta[id[u]];
        wt[u] = p.weight ? p.weight[id[u]] : 0;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (k + u < kend) { level += m[u]; peak = max(peak, level); base += wt[u]; }   // eq. (19) along the chain
    }
    peak += base;
    if (p.mem_limit && cand_ok && j < P && peak > p.mem_limit[j]) overb[g] = 1;   // an empty machine has peak 0
    if (lane_on) peakw[ql] = peak;
  }
  __syncthreads();

  // ---------------------------------------------------------------- reductions and outputs (wave 0)
  if (wave == 0) {
    int32_t z = acc;
    for (int d = 1; d < Pseg; d <<= 1) z = max(z, __shfl_xor(z, d, Pseg));
    if (lane_on && g < ng && j < P) {
      const int64_t c = cid(g);
      int bits = flagw[g] | (overb[g] ? kBitOverMemory : 0);
      if (stalled || abortw[g]) {
        if (p.optimistic && !(bits & kBitInternal) && abortw[g] != 2) {
          if (j == 0) { const int slot = atomicAdd(p.fb_count, 1); p.fb_list[slot] = (int32_t)c; }
          return;                                            // the general kernel writes this candidate
        }
        bits |= kBitCyclic;
      }
      const int flag = flag_from_bits(bits);
      const int64_t zz = (int64_t)z * p.time_scale;
      p.out.peak_mem[c * p.out.peak_stride_c + j * p.out.peak_stride_j] = flag ? -1 : peakw[ql];
      if (j == 0) {
        p.out.makespan[c] = flag ? -1 : (int32_t)zz;
        p.out.bubble[c] = flag ? -1 : (int64_t)P * zz - p.sum_dur;
        p.out.flags[c] = flag;
      }
    }
  }
}

}  // namespace dagsched_dev
