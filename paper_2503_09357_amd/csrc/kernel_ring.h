// Ring kernel: the fast evaluation path.
//
// Workgroup = two wavefronts that never meet at a barrier while the schedule is being relaxed:
//
//   wave 0, the RELAXER  lane (g, j) owns machine j of candidate g.  It pops compact "ops" from a
//                        per-lane ring in LDS and runs the max-plus recurrence
//                          s_v = max(0, e_chainpred, max_u e_u + delta(u,v)),  e_v = s_v + D^o_v
//                        (eqs. (3),(7),(11)-(13), Sec. III) against the end-time array of its
//                        candidate in LDS.  Its loop touches LDS only.
//   wave 1, the FEEDER   lane (g, j) walks machine j's order list, chases the shared operator
//                        records in L2, looks up the placement of every DAG predecessor and the
//                        channel delay, and pushes the resulting op into the relaxer's ring.  It
//                        also accumulates the machine's memory level and peak (eqs. (17)-(19)),
//                        which depend on the order only.
//
// The feeder runs ahead and absorbs every global-memory latency; the relaxer's critical loop is one
// LDS round trip, a few integer ops and one LDS write per operation.  A lone wavefront issues at most
// one instruction every four cycles, so the relaxer loop is written to be as short as possible.  The
// CUs are LDS-capacity bound on the large configurations (only a few candidates fit), so the second
// wavefront runs on a SIMD that would otherwise idle.
//
// End times are kept as 16-bit unsigned values (sentinel 0xFFFF = not yet ended), which halves the
// LDS footprint.  When the host cannot prove that every end time stays below 0xFFFF the kernel runs
// "optimistically": an operation whose end time would reach 0xFFFF is never completed, its candidate
// stalls exactly like a cyclic one, and every stalled candidate is handed to the general int32 kernel.
//
// Ring protocol (single producer, single consumer per lane, no atomics): a lane's ring has RING
// slots of kOpWords dwords; the last dword carries the op's sequence number.  The feeder writes the
// payload first and the tagged dword last; the relaxer reads the tagged dword first.  LDS executes
// one wavefront's accesses in order, so a matching tag proves the payload is complete.  The relaxer
// publishes how many ops it has copied into registers (tail); the feeder only overwrites a slot
// when fewer than RING ops are outstanding.
#pragma once

#include "device_common.h"

namespace dagsched_dev {

// LDS pointers with an explicit address space: volatile accesses through generic pointers would be
// compiled to flat loads, these compile to ds_read/ds_write.
#define DAGSCHED_LDS __attribute__((address_space(3)))
typedef DAGSCHED_LDS unsigned char lds_byte_t;
typedef DAGSCHED_LDS volatile uint32_t lds_vu32_t;
typedef DAGSCHED_LDS volatile uint16_t lds_vu16_t;
typedef DAGSCHED_LDS volatile int32_t lds_vi32_t;
typedef DAGSCHED_LDS const uint8_t lds_cu8_t;

// Op layouts.  ha(x) is the 16-bit address of the end-time cell of x: its LDS byte address when the
// end-time arrays of the workgroup fit 64 KB (template HALF = 0), else the byte address / 2 (HALF = 1);
// the arrays start at LDS offset 0.  Unused predecessor slots name the candidate's dummy cell (end time
// 0, delay 0); a part that does not end its operation names the candidate's trash cell instead of v.
// seq = index of the op in its lane, modulo (SeqMask + 1); ring tags start as all ones, which no op
// matches before its slot has been rewritten.
//   PREDS = 4, five dwords                           PREDS = 3, four dwords
//     w0 = ha(pred0) | ha(pred1) << 16                 w0 = ha(pred0) | ha(pred1) << 16
//     w1 = ha(pred2) | ha(pred3) << 16                 w1 = ha(pred2) | ha(v) << 16
//     w2 = delta0 | delta1 << 8 | delta2 << 16         w2 = duration
//          | delta3 << 24                              w3 = delta0 | delta1 << 8 | delta2 << 16
//     w3 = duration                                         | seq << 24                    (tag word)
//     w4 = ha(v) | seq << 16               (tag word)
// The duration is 0 for every part but the last of an operation.
template <int PREDS> struct OpFormat;
template <> struct OpFormat<4> {
  static constexpr int kWords = 5, kTagWord = 4, kSeqShift = 16;
  static constexpr uint32_t kSeqMask = 0xFFFFu;
};
template <> struct OpFormat<3> {
  static constexpr int kWords = 4, kTagWord = 3, kSeqShift = 24;
  static constexpr uint32_t kSeqMask = 0xFFu;
};
constexpr uint32_t kNotDone16 = 0xFFFFu;
constexpr int ring_threads(int feeders) { return (2 + feeders) * kWave; }   // relaxer, feeders, accountant

// One shared record per operation part: up to PREDS DAG predecessors (unused slots name the dummy
// node N).  Part i of operation v sits at rec[i * rec_plane + v]; only the last part carries the
// duration.
//   x = u0 | u1 << 16, y = u2 | u3 << 16, z = dur (30 bits) | first_part << 30 | has_more << 31, w = v << 16
struct LdsLayout {
  uint32_t s_stride, pi_stride;                       // bytes per candidate; the state array starts at 0
  uint32_t o_pi, o_ring, o_tail, o_total, o_peak, o_cnt, o_off, o_flag, o_abort, o_comm, total;
};

struct RingParams {
  int32_t N, P, Pseg, log_pseg, G, C;
  int32_t optimistic;                  // 1: stalled candidates go to fb_list, 0: a stall is a cycle
  int64_t list_stride;                 // uint16 elements per candidate in ws_list
  const uint4 *rec;                    // [parts][rec_plane] shared operator records (times divided by time_scale)
  int32_t rec_plane;                   // records per part plane (>= N)
  int32_t id_bits;                     // order-list entry = node | (parts - 1) << id_bits
  const uint8_t *nparts;               // [N] parts per node, or NULL when every node has one part
  const int32_t *comm;                 // [P*P] channel delays divided by time_scale (all <= 255)
  const int64_t *mem_delta;            // [N]
  int64_t sum_dur;                     // in original units
  int32_t time_scale;                  // gcd of every duration and delay
  const int32_t *placement, *rank;     // [C][N]
  uint16_t *ws_list;                   // [C][list_stride]
  int32_t *fb_count, *fb_list;         // candidates left to the general kernel
  uint32_t spin_cap;                   // bound on relaxer / feeder loop trips
  LdsLayout lds;
  OutPtrs out;
};

// FEEDERS feeder wavefronts share a lane's stream: feeder f owns the parts with (seq - 1) % FEEDERS == f.
template <int RING, int PREDS, int FEEDERS, int HALF>
__global__ __launch_bounds__(ring_threads(FEEDERS)) void relax_ring_kernel(RingParams p) {
  using Fmt = OpFormat<PREDS>;
  constexpr int kOpWords = Fmt::kWords;
  constexpr int kThreads = ring_threads(FEEDERS);
  constexpr int kFeeders = FEEDERS;
  extern __shared__ __align__(16) unsigned char lds[];
  static_assert((RING & (RING - 1)) == 0, "RING must be a power of two");
  constexpr uint32_t kPlaneBytes = RING * kWave * 4;        // ring layout: [word][slot][lane]
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int N = p.N, P = p.P, Pseg = p.Pseg, G = p.G;
  const int L = G * Pseg;                                   // lanes in use per wavefront
  const int64_t c0 = (int64_t)blockIdx.x * G;
  const int ng = (int)min((int64_t)G, (int64_t)p.C - c0);
  const LdsLayout &o = p.lds;
  lds_byte_t *const ldsb = (lds_byte_t *)lds;

  uint32_t *ringw = (uint32_t *)(lds + o.o_ring);
  uint32_t *tailw = (uint32_t *)(lds + o.o_tail);          // [64] ops the relaxer has taken
  uint32_t *totalw = (uint32_t *)(lds + o.o_total);        // [64] ops in the lane's stream, once a feeder knows
  int64_t *peakw = (int64_t *)(lds + o.o_peak);            // [64]
  int32_t *cntw = (int32_t *)(lds + o.o_cnt);              // [64] operations per (candidate, machine)
  int32_t *offw = (int32_t *)(lds + o.o_off);              // [64] start of the machine inside the list
  int32_t *flagw = (int32_t *)(lds + o.o_flag);            // [64] (G used)
  int32_t *abortw = (int32_t *)(lds + o.o_abort);          // [64] (G used)
  uint8_t *commb = (uint8_t *)(lds + o.o_comm);            // [(P+1)][Pseg], diagonal and dummy row zero

  // ---------------------------------------------------------------- ingest (both wavefronts)
  if (tid < kWave) { cntw[tid] = 0; tailw[tid] = 0; totalw[tid] = 0xFFFFFFFFu; flagw[tid] = 0; abortw[tid] = 0; peakw[tid] = 0; }
  for (int i = tid; i < kOpWords * RING * kWave; i += kThreads) ringw[i] = 0xFFFFFFFFu;
  for (int i = tid; i < (P + 1) * Pseg; i += kThreads) {    // rows of Pseg bytes: [source machine][destination]
    const int a = i >> p.log_pseg, b = i & (Pseg - 1);
    commb[i] = (a < P && b < P && a != b) ? (uint8_t)p.comm[a * P + b] : (uint8_t)0;
  }
  const int bm_words = (N + 31) >> 5;                       // rank bitmap, aliased over the state array
  for (int gg = 0; gg < ng; ++gg) {
    uint32_t *bm = (uint32_t *)(lds + gg * o.s_stride);
    for (int i = tid; i < bm_words; i += kThreads) bm[i] = 0;
  }
  __syncthreads();

  const bool vec_ok = ((N & 3) == 0) && ((((uintptr_t)p.placement) | ((uintptr_t)p.rank)) & 15) == 0;
  const int nq = N >> 2;

  // placement in range (eq. (6)), operations per machine
  for (int gg = 0; gg < ng; ++gg) {
    const int32_t *pl = p.placement + (c0 + gg) * N;
    uint8_t *pib = lds + o.o_pi + gg * o.pi_stride;
    int32_t *cnt_g = cntw + gg * Pseg;
    if (vec_ok) {
      const int4 *pl4 = (const int4 *)pl;
      uint32_t *piw = (uint32_t *)pib;
      for (int q0 = tid; q0 < nq; q0 += 4 * kThreads) {
        int4 a[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int q = q0 + u * kThreads;
          a[u] = (q < nq) ? pl4[q] : make_int4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int q = q0 + u * kThreads;
          if (q < nq) {
            const uint32_t hi = (uint32_t)a[u].x | (uint32_t)a[u].y | (uint32_t)a[u].z | (uint32_t)a[u].w;
            const bool bad = hi >= 64u || a[u].x >= P || a[u].y >= P || a[u].z >= P || a[u].w >= P;
            if (bad) {
              atomicOr(&flagw[gg], kBitBadPlacement);
            } else {
              piw[q] = (uint32_t)a[u].x | ((uint32_t)a[u].y << 8) | ((uint32_t)a[u].z << 16) | ((uint32_t)a[u].w << 24);
              atomicAdd(&cnt_g[a[u].x], 1); atomicAdd(&cnt_g[a[u].y], 1);
              atomicAdd(&cnt_g[a[u].z], 1); atomicAdd(&cnt_g[a[u].w], 1);
            }
          }
        }
      }
    } else {
      for (int v = tid; v < N; v += kThreads) {
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
  // dense ranks (eqs. (7)-(8)): every (machine, rank) slot hit exactly once; order lists to HBM
  for (int gg = 0; gg < ng; ++gg) {
    if (flagw[gg] & kBitBadPlacement) continue;
    const int32_t *rk = p.rank + (c0 + gg) * N;
    const uint8_t *pib = lds + o.o_pi + gg * o.pi_stride;
    uint32_t *bm = (uint32_t *)(lds + gg * o.s_stride);
    uint16_t *list = p.ws_list + (c0 + gg) * p.list_stride;
    const int32_t *cnt_g = cntw + gg * Pseg, *off_g = offw + gg * Pseg;
    int32_t *flag_g = flagw + gg;
    auto place = [&](int v, int pi, int32_t r) {
      if ((uint32_t)r >= (uint32_t)cnt_g[pi]) {
        atomicOr(flag_g, kBitBadRank);
      } else {
        const uint32_t pos = (uint32_t)(off_g[pi] + r);
        const uint32_t bit = 1u << (pos & 31);
        if (atomicOr(&bm[pos >> 5], bit) & bit) atomicOr(flag_g, kBitBadRank);
        else list[pos] = (uint16_t)(p.nparts ? (uint32_t)v | ((uint32_t)(p.nparts[v] - 1) << p.id_bits) : (uint32_t)v);
      }
    };
    if (vec_ok) {
      const int4 *rk4 = (const int4 *)rk;
      const uint32_t *piw = (const uint32_t *)pib;
      for (int q0 = tid; q0 < nq; q0 += 4 * kThreads) {
        int4 a[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int q = q0 + u * kThreads;
          a[u] = (q < nq) ? rk4[q] : make_int4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int q = q0 + u * kThreads;
          if (q < nq) {
            const uint32_t pw = piw[q];
            place(4 * q + 0, pw & 0xFF, a[u].x);
            place(4 * q + 1, (pw >> 8) & 0xFF, a[u].y);
            place(4 * q + 2, (pw >> 16) & 0xFF, a[u].z);
            place(4 * q + 3, pw >> 24, a[u].w);
          }
        }
      }
    } else {
      for (int v = tid; v < N; v += kThreads) place(v, pib[v], rk[v]);
    }
  }
  __syncthreads();                                          // workgroup scope: the lists are read by this workgroup only
  // end-time state: every operation "not ended"; the dummy node N has ended at time 0 on a dummy
  // machine P whose delays are all zero; cell N+1 is a trash cell for parts that do not end an operation
  for (int gg = 0; gg < ng; ++gg) {
    uint32_t *sw = (uint32_t *)(lds + gg * o.s_stride);
    for (int i = tid; i < (N + 3) / 2; i += kThreads) {
      const uint32_t lo = (2 * i < N) ? kNotDone16 : 0u, hi = (2 * i + 1 < N) ? kNotDone16 : 0u;
      sw[i] = lo | (hi << 16);
    }
    if (tid == 0) (lds + o.o_pi + gg * o.pi_stride)[N] = (uint8_t)P;
  }
  __syncthreads();

  // ---------------------------------------------------------------- roles
  const bool lane_on = lane < L;
  const int ql = lane_on ? lane : 0;
  const int g = ql >> p.log_pseg, j = ql & (Pseg - 1);
  const bool cand_ok = lane_on && g < ng && flagw[g] == 0;
  const bool has_ops = cand_ok && j < P && cntw[ql] > 0;
  const uint32_t sbase = (uint32_t)g * (o.s_stride >> HALF);   // 16-bit address of this candidate's cell 0

  int32_t acc = 0;
  bool stalled = false;

  if (wave == 0) {
    // ------------------------------------------------------------ relaxer
    lds_byte_t *const ring_lane = ldsb + o.o_ring + (uint32_t)lane * 4u;    // this lane's column of the ring
    lds_vu32_t *const tail_p = (lds_vu32_t *)(ldsb + o.o_tail) + lane;
    lds_vu32_t *const total_p = (lds_vu32_t *)(ldsb + o.o_total) + lane;
    lds_vi32_t *const abort_p = (lds_vi32_t *)(ldsb + o.o_abort) + g;
    const uint64_t segmask = ((Pseg == kWave) ? ~0ull : ((1ull << Pseg) - 1ull)) << (g * Pseg);
    auto cell = [&](uint32_t a16) -> lds_vu16_t & { return *(lds_vu16_t *)(ldsb + (a16 << HALF)); };
    const uint32_t dummy = sbase + ((uint32_t)N << (1 - HALF));
    // The loop body is branch-free: "this lane holds no op" is an op that can never run (duration
    // 0xFFFF) and every trip stores x somewhere (the trash cell unless the op ran).
    const uint32_t trash = sbase + (((uint32_t)N + 1u) << (1 - HALF));
    bool idle = true, dead = !has_ops;
    uint32_t t = 0, x_acc = 0;
    // current op: predecessor addresses (two words), packed delays, duration, destination address
    uint32_t ca = dummy | (dummy << 16), cb = ca, cd = 0, cdur = kNotDone16, cdst = trash;
    uint64_t prog_acc = 0;
    bool expired = true;
    uint32_t rt = 0xFFFFFFFFu, r0 = 0, r1 = 0, r2 = 0, r3 = 0;   // ring slot t as read at the end of the previous trip
    for (uint32_t it = 0; it < p.spin_cap; it += 8) {
#pragma unroll
      for (int sub = 0; sub < 8; ++sub) {
        // end times of the current op's predecessors (the critical reads go first)
        const uint32_t e0 = cell(ca & 0xFFFFu), e1 = cell(ca >> 16), e2 = cell(cb & 0xFFFFu);
        const uint32_t e3 = (PREDS == 4) ? (uint32_t)cell(cb >> 16) : 0u;
        uint32_t x = max(max(x_acc, e0 + (cd & 0xFFu)), e1 + ((cd >> 8) & 0xFFu));
        x = max(x, e2 + ((cd >> 16) & 0xFFu));
        if (PREDS == 4) x = max(x, e3 + (cd >> 24));
        x += cdur;
        const bool ready = x < kNotDone16;                  // every predecessor ended, no 16-bit overflow, not idle
        x_acc = ready ? x : x_acc;                          // the machine is busy until x (chain edge, eq. (7))
        cell(ready ? cdst : trash) = (uint16_t)x;
        const bool take = (ready || idle) && ((rt >> Fmt::kSeqShift) == (t & Fmt::kSeqMask));
        prog_acc |= __ballot(ready || take);                // an op taken now has not been tested yet
        idle = take ? false : (ready || idle);
        ca = take ? r0 : ca;
        if (PREDS == 4) {
          cb = take ? r1 : cb;
          cd = take ? r2 : cd;
          cdur = take ? r3 : (ready ? kNotDone16 : cdur);
          cdst = take ? (rt & 0xFFFFu) : cdst;
        } else {
          cb = take ? (r1 & 0xFFFFu) : cb;                  // the upper half is the destination, not a predecessor
          cd = take ? (rt & 0xFFFFFFu) : cd;
          cdur = take ? r2 : (ready ? kNotDone16 : cdur);
          cdst = take ? (r1 >> 16) : cdst;
        }
        t += take ? 1u : 0u;
        *tail_p = t;
        // next op of this lane (tagged word first), read now and looked at in the next trip: its LDS
        // latency hides behind the next trip's end-time reads
        {
          lds_byte_t *const sp = ring_lane + ((t & (uint32_t)(RING - 1)) << 8);
          rt = *(lds_vu32_t *)(sp + Fmt::kTagWord * kPlaneBytes);
          r0 = *(lds_vu32_t *)(sp);
          r1 = *(lds_vu32_t *)(sp + kPlaneBytes);
          r2 = *(lds_vu32_t *)(sp + 2 * kPlaneBytes);
          if (PREDS == 4) r3 = *(lds_vu32_t *)(sp + 3 * kPlaneBytes);
        }
      }
      const bool fin = dead || (idle && t == *total_p);
      if (__ballot(!fin) == 0) { expired = false; break; }
      const uint64_t hold = __ballot(!idle || fin);
      if (!fin && (prog_acc & segmask) == 0 && (hold & segmask) == segmask) {
        // every unfinished machine of this candidate holds an op and none could run for a whole
        // window: deadlock, i.e. a cycle of the combined graph (or a 16-bit overflow when optimistic)
        stalled = true;
        dead = true;
        *abort_p = 1;
      }
      if (prog_acc == 0) __builtin_amdgcn_s_sleep(4);       // nothing could run: leave the issue slots to the feeders
      prog_acc = 0;
    }
    if (expired) {                                          // bounded wait ran out: report, release the feeder
      const bool fin = dead || (idle && t == *total_p);
      if (!fin) { flagw[g] = kBitInternal; *abort_p = 1; }
    }
    acc = (int32_t)x_acc;
  } else if (wave <= kFeeders) {
    // ------------------------------------------------------------ feeders
    // Per lane the op parts of machine j form a stream (the parts of one operation are consecutive;
    // the order-list entry of a node carries its part count, so the stream is known from the ids
    // alone).  Feeder f owns every kFeeders-th part.  A part is ADMITTED when its ring slot is free
    // (fewer than RING parts between it and the relaxer's tail), then moves through a fixed pipeline
    // without ever stalling:
    //   trip t    record requested from L2
    //   trip t+1  placement bytes of its predecessors read from LDS
    //   trip t+2  channel delays read from LDS, op packed and written to the ring
    // The loop is unrolled by three so that the pipeline registers rotate by renaming, not by moves.
    const int f = wave - 1;
    __builtin_amdgcn_s_setprio(2);                          // the relaxer only polls; feeding must not wait behind it
    lds_cu8_t *const pib = (lds_cu8_t *)(ldsb + o.o_pi + g * o.pi_stride);
    lds_cu8_t *const commr = (lds_cu8_t *)(ldsb + o.o_comm) + j;
    lds_byte_t *const ring_lane = ldsb + o.o_ring + (uint32_t)lane * 4u;
    lds_vu32_t *const tail_p = (lds_vu32_t *)(ldsb + o.o_tail) + lane;
    lds_vi32_t *const abort_p = (lds_vi32_t *)(ldsb + o.o_abort) + g;
    const uint16_t *list = p.ws_list + (c0 + (cand_ok ? g : 0)) * p.list_stride;
    lds_vu32_t *const total_p = (lds_vu32_t *)(ldsb + o.o_total) + lane;
    const uint32_t base2 = sbase | (sbase << 16);
    const uint32_t trash = sbase + (((uint32_t)N + 1u) << (1 - HALF));
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
    uint32_t k = k0;
    const uint32_t w0 = has_ops ? (uint32_t)list[k0] : 0u;
    uint32_t addr = w0 & vmask, rem = w0 >> vbits;
    uint32_t id1 = has_ops ? (uint32_t)list[min(k0 + 1u, klast)] : 0u;
    uint32_t id2 = has_ops ? (uint32_t)list[min(k0 + 2u, klast)] : 0u;
    // move the cursor one part ahead; returns true when it entered the next node (or left the list)
    auto advance = [&](uint32_t next_id) -> bool {
      const bool in_node = rem != 0;
      addr = in_node ? addr + n_plane : (next_id & vmask);
      rem = in_node ? rem - 1u : (next_id >> vbits);
      k += in_node ? 0u : 1u;
      return !in_node;
    };
    for (int i = 0; i < f; ++i) {                           // feeder f starts at its first own part
      const bool crossed = advance(id1);
      id1 = crossed ? id2 : id1;
    }
    struct Entry { uint4 rec; uint32_t q0, q1, q2, q3, fl; };   // fl: 1 valid, 2 last part of the lane
    Entry E[3];
#pragma unroll
    for (int i = 0; i < 3; ++i) { E[i].rec = make_uint4(0, 0, 0, 0); E[i].q0 = E[i].q1 = E[i].q2 = E[i].q3 = 0; E[i].fl = 0; }

    for (uint32_t it = 0; it < p.spin_cap; it += 3) {
      if (*abort_p) { k = klast + 1u; written = admitted; }   // the relaxer gave this candidate up
      if (__ballot(!(k > klast && written == admitted)) == 0) break;
#pragma unroll
      for (int s = 0; s < 3; ++s) {
        Entry &e0 = E[s];                 // admitted in this trip
        Entry &e1 = E[(s + 2) % 3];       // admitted one trip ago
        Entry &e2 = E[(s + 1) % 3];       // admitted two trips ago
        // (A) channel delays of e2 (its placement bytes were read one trip ago)
        const uint32_t d0 = commr[e2.q0 << lps], d1 = commr[e2.q1 << lps], d2 = commr[e2.q2 << lps];
        const uint32_t d3 = (PREDS == 4) ? (uint32_t)commr[e2.q3 << lps] : 0u;
        // (1) move the cursor past the part admitted in the previous trip and the other feeders' parts
        if (pending) {
#pragma unroll
          for (int a = 0; a < kFeeders; ++a) {
            const bool crossed = advance(id1);
            id1 = crossed ? id2 : id1;
          }
          aseq += kFeeders;
        }
        // (2) ids of the next two nodes (reloaded every trip; consumed one trip later at the earliest)
        id1 = list[min(k + 1u, klast)];
        id2 = list[min(k + 2u, klast)];
        // (3) admission
        pending = (k <= klast) && (aseq - *tail_p) < (uint32_t)RING;
        e0.fl = pending ? (1u | ((k == klast && rem == 0u) ? 2u : 0u)) : 0u;
        e0.rec = p.rec[addr];
        admitted += pending ? 1u : 0u;
        // (B) placement bytes of e1's predecessors (its record was requested one trip ago)
        e1.q0 = pib[e1.rec.x & 0xFFFFu]; e1.q1 = pib[e1.rec.x >> 16];
        e1.q2 = pib[e1.rec.y & 0xFFFFu];
        if (PREDS == 4) e1.q3 = pib[e1.rec.y >> 16];
        // (D) pack e2 and publish it
        if (e2.fl & 1u) {
          const bool more = (e2.rec.z >> 31) != 0;
          const uint32_t dst = more ? trash : sbase + ((e2.rec.w >> 16) << (1 - HALF));
          const uint32_t tagbits = (wseq & Fmt::kSeqMask) << Fmt::kSeqShift;
          lds_byte_t *const sp = ring_lane + ((wseq & (uint32_t)(RING - 1)) << 8);
          // node ids below 32768 whenever HALF == 0, so shifting both halves at once cannot carry over
          *(lds_vu32_t *)(sp) = (e2.rec.x << (1 - HALF)) + base2;
          if (PREDS == 4) {
            *(lds_vu32_t *)(sp + kPlaneBytes) = (e2.rec.y << (1 - HALF)) + base2;
            *(lds_vu32_t *)(sp + 2 * kPlaneBytes) = d0 | (d1 << 8) | (d2 << 16) | (d3 << 24);
            *(lds_vu32_t *)(sp + 3 * kPlaneBytes) = e2.rec.z & 0x3FFFFFFFu;
            *(lds_vu32_t *)(sp + 4 * kPlaneBytes) = dst | tagbits;
          } else {
            *(lds_vu32_t *)(sp + kPlaneBytes) = (((e2.rec.y & 0xFFFFu) << (1 - HALF)) + sbase) | (dst << 16);
            *(lds_vu32_t *)(sp + 2 * kPlaneBytes) = e2.rec.z & 0x3FFFFFFFu;
            *(lds_vu32_t *)(sp + 3 * kPlaneBytes) = d0 | (d1 << 8) | (d2 << 16) | tagbits;
          }
          if (e2.fl & 2u) *total_p = wseq + 1;              // the lane's stream ends with this op
          wseq += kFeeders;
          ++written;
        }
      }
    }
  } else {
    // ------------------------------------------------------------ accountant
    // Peak of the running memory level of machine j (eqs. (17)-(19)): it depends on the order only,
    // so one wavefront walks the order lists on its own, four operations per trip.
    const uint16_t *list = p.ws_list + (c0 + (cand_ok ? g : 0)) * p.list_stride;
    const uint32_t vmask = (1u << p.id_bits) - 1u;
    const int k0 = has_ops ? offw[ql] : 0;
    const int kend = has_ops ? k0 + cntw[ql] : 0;
    int64_t level = 0, peak = 0;
    for (int k = k0; __ballot(k < kend) != 0; k += 4) {
      uint32_t id[4];
      int64_t m[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) id[u] = (k + u < kend) ? ((uint32_t)list[k + u] & vmask) : 0u;
#pragma unroll
      for (int u = 0; u < 4; ++u) m[u] = p.mem_delta[id[u]];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (k + u < kend) { level += m[u]; peak = max(peak, level); }   // eq. (19) along the chain
    }
    if (lane_on) peakw[ql] = peak;
  }
  __syncthreads();

  // ---------------------------------------------------------------- reductions and outputs (wave 0)
  if (wave == 0) {
    int32_t z = acc;
    for (int d = 1; d < Pseg; d <<= 1) z = max(z, __shfl_xor(z, d, Pseg));
    if (lane_on && g < ng && j < P) {
      const int64_t c = c0 + g;
      int bits = flagw[g];
      if (stalled || abortw[g]) {
        if (p.optimistic && !(bits & kBitInternal)) {
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
