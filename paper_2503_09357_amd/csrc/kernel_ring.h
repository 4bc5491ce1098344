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

// Op layout (five dwords).  "Half-address" = LDS byte address / 2 of a 16-bit end-time cell; the
// end-time arrays start at LDS offset 0, so every half-address fits 16 bits.
//   w0 = ha(pred0) | ha(pred1) << 16       unused predecessor slots name the candidate's dummy cell
//   w1 = ha(pred2) | ha(pred3) << 16       (end time 0, delay 0)
//   w2 = delta0 | delta1 << 8 | delta2 << 16 | delta3 << 24
//   w3 = duration (0 for every part but the last of an operation)
//   w4 = ha(v) | FINAL << 16 | LAST << 17 | seq << 18         seq = (index of the op in its lane + 1) mod 2^14
constexpr int kOpWords = 5;
constexpr uint32_t kOpFinal = 1u << 16;   // completes its operation: add D^o, write the end time
constexpr uint32_t kOpLast = 1u << 17;    // last op of this lane's order list
constexpr int kOpSeqShift = 18;
constexpr uint32_t kOpSeqMask = 0x3FFFu;
constexpr uint32_t kNotDone16 = 0xFFFFu;
constexpr int kThreads = 2 * kWave;

// One shared record per operation part: up to four DAG predecessors (unused slots name the dummy
// node N).  Part i of operation v sits at rec[i * rec_plane + v]; only the last part carries the
// duration.
//   x = u0 | u1 << 16, y = u2 | u3 << 16, z = dur (30 bits) | first_part << 30 | has_more << 31, w = v << 16
struct LdsLayout {
  uint32_t s_stride, pi_stride;                       // bytes per candidate; the state array starts at 0
  uint32_t o_pi, o_ring, o_tail, o_peak, o_cnt, o_off, o_flag, o_abort, o_comm, total;
};

struct RingParams {
  int32_t N, P, Pseg, log_pseg, G, C;
  int32_t optimistic;                  // 1: stalled candidates go to fb_list, 0: a stall is a cycle
  int64_t list_stride;                 // uint16 elements per candidate in ws_list
  const uint4 *rec;                    // [parts][rec_plane] shared operator records (times divided by time_scale)
  int32_t rec_plane;                   // records per part plane (>= N)
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

template <int RING>
__global__ __launch_bounds__(kThreads) void relax_ring_kernel(RingParams p) {
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
  int64_t *peakw = (int64_t *)(lds + o.o_peak);            // [64]
  int32_t *cntw = (int32_t *)(lds + o.o_cnt);              // [64] operations per (candidate, machine)
  int32_t *offw = (int32_t *)(lds + o.o_off);              // [64] start of the machine inside the list
  int32_t *flagw = (int32_t *)(lds + o.o_flag);            // [64] (G used)
  int32_t *abortw = (int32_t *)(lds + o.o_abort);          // [64] (G used)
  uint8_t *commb = (uint8_t *)(lds + o.o_comm);            // [(P+1)*P], diagonal and dummy row zero

  // ---------------------------------------------------------------- ingest (both wavefronts)
  if (tid < kWave) { cntw[tid] = 0; tailw[tid] = 0; flagw[tid] = 0; abortw[tid] = 0; peakw[tid] = 0; }
  for (int i = tid; i < kOpWords * RING * kWave; i += kThreads) ringw[i] = 0;
  for (int i = tid; i < (P + 1) * P; i += kThreads)
    commb[i] = (i < P * P && (i / P) != (i % P)) ? (uint8_t)p.comm[i] : (uint8_t)0;
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
        else list[pos] = (uint16_t)v;
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
  __threadfence();
  __syncthreads();
  // end-time state: every operation "not ended"; the dummy node N has ended at time 0 on a dummy
  // machine P whose delays are all zero
  for (int gg = 0; gg < ng; ++gg) {
    uint32_t *sw = (uint32_t *)(lds + gg * o.s_stride);
    for (int i = tid; i < (N + 2) / 2; i += kThreads) {
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
  const uint32_t sbase_half = (uint32_t)g * (o.s_stride >> 1);   // half-address of this candidate's cell 0

  int32_t acc = 0;
  bool stalled = false;

  if (wave == 0) {
    // ------------------------------------------------------------ relaxer
    lds_vu16_t *const cells = (lds_vu16_t *)ldsb;                           // indexed by half-address
    lds_byte_t *const ring_lane = ldsb + o.o_ring + (uint32_t)lane * 4u;    // this lane's column of the ring
    lds_vu32_t *const tail_p = (lds_vu32_t *)(ldsb + o.o_tail) + lane;
    lds_vi32_t *const abort_p = (lds_vi32_t *)(ldsb + o.o_abort) + g;
    const uint64_t segmask = ((Pseg == kWave) ? ~0ull : ((1ull << Pseg) - 1ull)) << (g * Pseg);
    const uint32_t dummy = sbase_half + (uint32_t)N;
    bool all_taken = !has_ops, have_cur = false;
    uint32_t t = 0, want = 1, x_acc = 0;
    uint32_t cw0 = dummy | (dummy << 16), cw1 = cw0, cw2 = 0, cw3 = 0, cw4 = dummy;
    uint64_t prog_acc = 0;
    bool expired = true;
    for (uint32_t it = 0; it < p.spin_cap; it += 8) {
#pragma unroll
      for (int sub = 0; sub < 8; ++sub) {
        // next op of this lane, read speculatively every trip (tagged word first)
        lds_byte_t *const sp = ring_lane + ((t & (uint32_t)(RING - 1)) << 8);
        const uint32_t r4 = *(lds_vu32_t *)(sp + 4 * kPlaneBytes);
        const uint32_t r0 = *(lds_vu32_t *)(sp);
        const uint32_t r1 = *(lds_vu32_t *)(sp + kPlaneBytes);
        const uint32_t r2 = *(lds_vu32_t *)(sp + 2 * kPlaneBytes);
        const uint32_t r3 = *(lds_vu32_t *)(sp + 3 * kPlaneBytes);
        // end times of the current op's predecessors
        const uint32_t e0 = cells[cw0 & 0xFFFFu], e1 = cells[cw0 >> 16];
        const uint32_t e2 = cells[cw1 & 0xFFFFu], e3 = cells[cw1 >> 16];
        uint32_t x = max(max(x_acc, e0 + (cw2 & 0xFFu)), e1 + ((cw2 >> 8) & 0xFFu));
        x = max(max(x, e2 + ((cw2 >> 16) & 0xFFu)), e3 + (cw2 >> 24));
        x += cw3;
        const bool ready = have_cur && x < kNotDone16;      // every predecessor ended and no 16-bit overflow
        if (ready) {
          x_acc = x;                                        // the machine is busy until x (chain edge, eq. (7))
          if (cw4 & kOpFinal) cells[cw4 & 0xFFFFu] = (uint16_t)x;
        }
        const bool take = !all_taken && (ready || !have_cur) && ((r4 >> kOpSeqShift) == want);
        prog_acc |= __ballot(ready || take);                // an op taken now has not been tested yet
        have_cur = take || (have_cur && !ready);
        if (take) {
          cw0 = r0; cw1 = r1; cw2 = r2; cw3 = r3; cw4 = r4;
          ++t;
          want = (t + 1) & kOpSeqMask;
          *tail_p = t;
          all_taken = (r4 & kOpLast) != 0;
        }
      }
      const bool fin = all_taken && !have_cur;
      if (__ballot(!fin) == 0) { expired = false; break; }
      const uint64_t hold = __ballot(have_cur || fin);
      if (!fin && (prog_acc & segmask) == 0 && (hold & segmask) == segmask) {
        // every unfinished machine of this candidate holds an op and none could run for a whole
        // window: deadlock, i.e. a cycle of the combined graph (or a 16-bit overflow when optimistic)
        stalled = true;
        all_taken = true;
        have_cur = false;
        *abort_p = 1;
      }
      prog_acc = 0;
    }
    if (expired) {                                          // bounded wait ran out: report, release the feeder
      const bool fin = all_taken && !have_cur;
      if (!fin) { flagw[g] = kBitInternal; *abort_p = 1; }
    }
    acc = (int32_t)x_acc;
  } else {
    // ------------------------------------------------------------ feeder
    // Per lane the op parts of machine j form a stream (parts of one operation are consecutive).  A
    // three-stage register pipeline rc -> r1 -> r2 holds the next three parts; the part after them is
    // (re)loaded into a temporary every trip and accepted into r2 one trip later, so a global load
    // always has a full trip to land.  Two sets of temporaries alternate (the loop is unrolled by
    // two) so that a freshly loaded register is never copied in the trip that issued it.
    lds_cu8_t *const pib = (lds_cu8_t *)(ldsb + o.o_pi + g * o.pi_stride);
    lds_cu8_t *const commr = (lds_cu8_t *)(ldsb + o.o_comm) + j;
    lds_byte_t *const ring_lane = ldsb + o.o_ring + (uint32_t)lane * 4u;
    lds_vu32_t *const tail_p = (lds_vu32_t *)(ldsb + o.o_tail) + lane;
    lds_vi32_t *const abort_p = (lds_vi32_t *)(ldsb + o.o_abort) + g;
    const uint16_t *list = p.ws_list + (c0 + (cand_ok ? g : 0)) * p.list_stride;
    const uint32_t base2 = sbase_half | (sbase_half << 16);
    const int k0 = has_ops ? offw[ql] : 0;
    const int kend = has_ops ? k0 + cntw[ql] : 1;
    bool fin = !has_ops;
    uint32_t head = 0, tail_seen = 0;
    int64_t level = 0, peak = 0;
    constexpr uint32_t kStValid = 1u, kStLastNode = 2u;    // dynamic flags in the low half of rec.w
    uint4 rc = make_uint4(0, 0, 0, 0), r1 = rc, r2 = rc;
    int64_t m0 = 0, m1 = 0, m2 = 0;
    // loader: identity of the part the temporaries are loading
    int npos = k0;
    uint32_t nv = has_ops ? (uint32_t)list[k0] : 0u;
    uint32_t naddr = nv;
    uint32_t idq1 = (has_ops && k0 + 1 < kend) ? (uint32_t)list[k0 + 1] : 0u;
    bool stream_end = !has_ops;
    uint4 tra = p.rec[naddr], trb = tra;
    int64_t tma = p.mem_delta[nv], tmb = tma;
    uint32_t tia = has_ops ? (uint32_t)list[min(npos + 2, kend - 1)] : 0u, tib = tia;
    uint32_t q0 = pib[0], q1 = q0, q2 = q0, q3 = q0;       // placement bytes of rc's predecessors
    const uint32_t n_plane = (uint32_t)p.rec_plane;

    auto trip = [&](uint4 &tr, int64_t &tm, uint32_t &ti, uint4 &tr_new, int64_t &tm_new, uint32_t &ti_new) {
      bool full = (head - tail_seen) >= (uint32_t)RING;
      if (!fin && full) {
        tail_seen = *tail_p;
        full = (head - tail_seen) >= (uint32_t)RING;
        if (full && *abort_p) fin = true;
      }
      const bool rc_valid = (rc.w & kStValid) != 0;
      const bool produce = !fin && !full && rc_valid;
      // channel delays of rc (its placement bytes were read one trip ago); placement bytes of r1
      const uint32_t d0 = commr[q0 * P], d1 = commr[q1 * P], d2 = commr[q2 * P], d3 = commr[q3 * P];
      const uint32_t n0 = pib[r1.x & 0xFFFFu], n1 = pib[r1.x >> 16], n2 = pib[r1.y & 0xFFFFu], n3 = pib[r1.y >> 16];
      if (produce) {
        const bool more = (rc.z >> 31) != 0;
        const bool last = !more && (rc.w & kStLastNode);
        const uint32_t w4 = (sbase_half + (rc.w >> 16)) | (more ? 0u : kOpFinal) | (last ? kOpLast : 0u) |
                            (((head + 1) & kOpSeqMask) << kOpSeqShift);
        lds_byte_t *const sp = ring_lane + ((head & (uint32_t)(RING - 1)) << 8);
        *(lds_vu32_t *)(sp) = rc.x + base2;
        *(lds_vu32_t *)(sp + kPlaneBytes) = rc.y + base2;
        *(lds_vu32_t *)(sp + 2 * kPlaneBytes) = d0 | (d1 << 8) | (d2 << 16) | (d3 << 24);
        *(lds_vu32_t *)(sp + 3 * kPlaneBytes) = rc.z & 0x3FFFFFFFu;
        *(lds_vu32_t *)(sp + 4 * kPlaneBytes) = w4;
        ++head;
        if (rc.z & 0x40000000u) { level += m0; peak = max(peak, level); }   // first part: eq. (19) along the chain
        if (last) fin = true;
      }
      if (!fin && (produce || !rc_valid)) {                 // shift the pipeline, accept the temporary
        rc = r1; m0 = m1; q0 = n0; q1 = n1; q2 = n2; q3 = n3;
        r1 = r2; m1 = m2;
        if (!stream_end) {
          const bool t_more = (tr.z >> 31) != 0;
          r2 = make_uint4(tr.x, tr.y, tr.z, (tr.w & 0xFFFF0000u) | kStValid | ((npos == kend - 1) ? kStLastNode : 0u));
          m2 = tm;
          if (t_more) {
            naddr += n_plane;
          } else if (npos == kend - 1) {
            stream_end = true;
          } else {
            ++npos; nv = idq1; naddr = idq1; idq1 = ti;
          }
        } else {
          r2 = make_uint4(0, 0, 0, 0);
        }
      }
      if (!stream_end) {                                    // (re)load the part after r2
        tr_new = p.rec[naddr];
        tm_new = p.mem_delta[nv];
        ti_new = list[min(npos + 2, kend - 1)];
      }
    };
    for (uint32_t it = 0; it < p.spin_cap; it += 2) {
      if (__ballot(!fin) == 0) break;
      trip(tra, tma, tia, trb, tmb, tib);
      trip(trb, tmb, tib, tra, tma, tia);
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
