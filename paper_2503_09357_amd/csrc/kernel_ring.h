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
// LDS read, a few integer ops and one LDS write per operation.  The CUs are LDS-capacity bound on
// the large configurations (only a few candidates fit), so the second wavefront runs on a SIMD that
// would otherwise idle.
//
// End times are kept as 16-bit unsigned values (sentinel 0xFFFF = not yet ended), which halves the
// LDS footprint.  When the host cannot prove that every end time stays below 0xFFFF the kernel runs
// "optimistically": an operation whose end time would reach 0xFFFF is never completed, its candidate
// stalls exactly like a cyclic one, and every stalled candidate is handed to the general int32 kernel.
//
// Ring protocol (single producer, single consumer per lane, no atomics): slot i of a lane's ring
// holds kOpWords dwords; the last dword carries a generation bit that flips on every lap.  The
// feeder writes the payload first and the tagged dword last; the relaxer reads the tagged dword
// first.  LDS executes one wavefront's accesses in order, so a matching tag proves the payload is
// complete.  The relaxer publishes how many ops it has copied into registers (tail); the feeder only
// overwrites slot i when fewer than RING ops are outstanding.
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

constexpr int kOpWords = 5;
constexpr uint32_t kOpFinal = 1u << 16;   // completes its operation: add D^o, write the end time
constexpr uint32_t kOpLast = 1u << 17;    // last op of this lane's order list
constexpr int kOpGenShift = 18;
constexpr uint32_t kNotDone16 = 0xFFFFu;

// One shared record per operation part: up to four DAG predecessors (unused slots name the dummy
// node N whose end time is 0 and whose delay is 0).  An operation with more than four predecessors
// continues in the overflow area [N, n_rec); only the last part carries the duration.
//   x = u0 | u1 << 16, y = u2 | u3 << 16, z = dur (31 bits) | has_more << 31, w = next | v << 16
struct LdsLayout {
  uint32_t s_stride, pi_stride;                       // bytes per candidate
  uint32_t o_state, o_pi, o_ring, o_tail, o_peak, o_cnt, o_off, o_flag, o_abort, o_comm, total;
};

struct RingParams {
  int32_t N, P, Pseg, log_pseg, G, C;
  int32_t ring, log_ring;              // ring slots per lane (power of two)
  int32_t optimistic;                  // 1: stalled candidates go to fb_list, 0: a stall is a cycle
  int64_t list_stride;                 // uint16 elements per candidate in ws_list
  const uint4 *rec;                    // [n_rec] shared operator records (times already divided by time_scale)
  const int32_t *comm;                 // [P*P] channel delays divided by time_scale (all <= 255)
  const int64_t *mem_delta;            // [N]
  int64_t sum_dur;                     // in original units
  int32_t time_scale;                  // gcd of every duration and delay
  const int32_t *placement, *rank;     // [C][N]
  uint16_t *ws_list;                   // [C][list_stride]
  int32_t *fb_count, *fb_list;         // candidates left to the general kernel
  uint32_t spin_cap;
  LdsLayout lds;
  OutPtrs out;
};

__global__ __launch_bounds__(2 * kWave) void relax_ring_kernel(RingParams p) {
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int N = p.N, P = p.P, Pseg = p.Pseg, G = p.G;
  const int L = G * Pseg;                                   // lanes in use per wavefront
  const int RING = p.ring;
  const int64_t c0 = (int64_t)blockIdx.x * G;
  const int ng = (int)min((int64_t)G, (int64_t)p.C - c0);
  const LdsLayout &o = p.lds;
  lds_byte_t *const ldsb = (lds_byte_t *)lds;

  uint32_t *ringw = (uint32_t *)(lds + o.o_ring);          // [(slot*kOpWords + d) * L + lane]
  uint32_t *tailw = (uint32_t *)(lds + o.o_tail);          // [L] ops the relaxer has taken
  int64_t *peakw = (int64_t *)(lds + o.o_peak);            // [L]
  int32_t *cntw = (int32_t *)(lds + o.o_cnt);              // [L] operations per (candidate, machine)
  int32_t *offw = (int32_t *)(lds + o.o_off);              // [L] start of the machine inside the list
  int32_t *flagw = (int32_t *)(lds + o.o_flag);            // [G]
  int32_t *abortw = (int32_t *)(lds + o.o_abort);          // [G]
  uint8_t *commb = (uint8_t *)(lds + o.o_comm);            // [(P+1)*P], diagonal and dummy row zero

  // ---------------------------------------------------------------- ingest (both wavefronts)
  for (int i = tid; i < L; i += 2 * kWave) {
    cntw[i] = 0; tailw[i] = 0; flagw[i] = 0; abortw[i] = 0; peakw[i] = 0;
  }
  for (int i = tid; i < kOpWords * RING * L; i += 2 * kWave) ringw[i] = 0;
  for (int i = tid; i < (P + 1) * P; i += 2 * kWave)
    commb[i] = (i < P * P && (i / P) != (i % P)) ? (uint8_t)p.comm[i] : (uint8_t)0;
  const int bm_words = (N + 31) >> 5;                       // rank bitmap, aliased over the state array
  for (int gg = 0; gg < ng; ++gg) {
    uint32_t *bm = (uint32_t *)(lds + o.o_state + gg * o.s_stride);
    for (int i = tid; i < bm_words; i += 2 * kWave) bm[i] = 0;
  }
  __syncthreads();

  // placement in range (eq. (6)), operations per machine
  for (int gg = 0; gg < ng; ++gg) {
    const int32_t *pl = p.placement + (c0 + gg) * N;
    uint8_t *pib = lds + o.o_pi + gg * o.pi_stride;
    for (int v = tid; v < N; v += 2 * kWave) {
      const int32_t pi = pl[v];
      if ((uint32_t)pi >= (uint32_t)P) {
        atomicOr(&flagw[gg], kBitBadPlacement);
      } else {
        pib[v] = (uint8_t)pi;
        atomicAdd(&cntw[gg * Pseg + pi], 1);
      }
    }
  }
  __syncthreads();
  if (wave == 0) {                                          // exclusive prefix over the machines of each candidate
    const int idx = lane < L ? lane : 0;
    const int my = lane < L ? cntw[idx] : 0;
    int incl = my;
    const int j = lane & (Pseg - 1);
    for (int d = 1; d < Pseg; d <<= 1) {
      const int t = __shfl_up(incl, d, Pseg);
      if (j >= d) incl += t;
    }
    if (lane < L) offw[lane] = incl - my;
  }
  __syncthreads();
  // dense ranks (eqs. (7)-(8)): every (machine, rank) slot hit exactly once; order lists to HBM
  for (int gg = 0; gg < ng; ++gg) {
    if (flagw[gg] & kBitBadPlacement) continue;
    const int32_t *rk = p.rank + (c0 + gg) * N;
    const uint8_t *pib = lds + o.o_pi + gg * o.pi_stride;
    uint32_t *bm = (uint32_t *)(lds + o.o_state + gg * o.s_stride);
    uint16_t *list = p.ws_list + (c0 + gg) * p.list_stride;
    for (int v = tid; v < N; v += 2 * kWave) {
      const int pi = pib[v];
      const int32_t r = rk[v];
      if ((uint32_t)r >= (uint32_t)cntw[gg * Pseg + pi]) {
        atomicOr(&flagw[gg], kBitBadRank);
      } else {
        const uint32_t pos = (uint32_t)(offw[gg * Pseg + pi] + r);
        const uint32_t bit = 1u << (pos & 31);
        if (atomicOr(&bm[pos >> 5], bit) & bit) atomicOr(&flagw[gg], kBitBadRank);
        else list[pos] = (uint16_t)v;
      }
    }
  }
  __threadfence();
  __syncthreads();
  // end-time state: every operation "not ended"; the dummy node N has ended at time 0 on a dummy
  // machine P whose delays are all zero
  for (int gg = 0; gg < ng; ++gg) {
    uint32_t *sw = (uint32_t *)(lds + o.o_state + gg * o.s_stride);
    for (int i = tid; i < (N + 2) / 2; i += 2 * kWave) {
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
  const uint32_t gen_mask = 1u << kOpGenShift;
  const uint32_t plane = (uint32_t)L;                       // dwords between the words of one op
  const uint32_t slot_words = (uint32_t)(kOpWords * L);

  int32_t acc = 0;
  bool stalled = false;

  if (wave == 0) {
    // ------------------------------------------------------------ relaxer
    lds_vu16_t *const state = (lds_vu16_t *)(ldsb + o.o_state + g * o.s_stride);
    lds_vu32_t *const ring_r = (lds_vu32_t *)(ldsb + o.o_ring) + ql;
    lds_vu32_t *const tail_p = (lds_vu32_t *)(ldsb + o.o_tail) + ql;
    lds_vi32_t *const abort_p = (lds_vi32_t *)(ldsb + o.o_abort) + g;
    const uint64_t segmask = ((Pseg == kWave) ? ~0ull : ((1ull << Pseg) - 1ull)) << (g * Pseg);
    bool fin = !has_ops, all_fetched = !has_ops, have_cur = false, have_nxt = false;
    uint32_t t = 0, x_acc = 0;
    uint32_t c0w = 0, c1w = 0, c2w = 0, c3w = 0, c4w = 0;
    uint32_t n0w = 0, n1w = 0, n2w = 0, n3w = 0, n4w = 0;
    uint64_t prog_acc = 0;
    bool expired = true;
    for (uint32_t it = 0; it < p.spin_cap; ++it) {
      if (!have_cur && have_nxt) {
        c0w = n0w; c1w = n1w; c2w = n2w; c3w = n3w; c4w = n4w;
        have_cur = true; have_nxt = false;
      }
      // speculative read of the next ring slot (tagged word first)
      const uint32_t slot = t & (uint32_t)(RING - 1);
      lds_vu32_t *const sp = ring_r + slot * slot_words;
      const uint32_t r4 = sp[4 * plane];
      const uint32_t r0 = sp[0], r1 = sp[plane], r2 = sp[2 * plane], r3 = sp[3 * plane];
      // end times of the current op's predecessors
      const uint32_t e0 = state[c0w & 0xFFFFu], e1 = state[c0w >> 16];
      const uint32_t e2 = state[c1w & 0xFFFFu], e3 = state[c1w >> 16];
      uint32_t x = max(max(x_acc, e0 + (c2w & 0xFFu)), e1 + ((c2w >> 8) & 0xFFu));
      x = max(max(x, e2 + ((c2w >> 16) & 0xFFu)), e3 + (c2w >> 24));
      x += c3w;
      const bool ready = have_cur && x < kNotDone16;        // every predecessor ended and no 16-bit overflow
      if (ready) {
        x_acc = x;                                          // the machine is busy until x (chain edge, eq. (7))
        if (c4w & kOpFinal) state[c4w & 0xFFFFu] = (uint16_t)x;
        if (c4w & kOpLast) fin = true;
        have_cur = false;
      }
      prog_acc |= __ballot(ready);
      const uint32_t want_gen = (((t >> p.log_ring) & 1u) ^ 1u) << kOpGenShift;
      const bool got = !have_nxt && !all_fetched && ((r4 & gen_mask) == want_gen);
      if (got) {
        n0w = r0; n1w = r1; n2w = r2; n3w = r3; n4w = r4;
        have_nxt = true;
        ++t;
        *tail_p = t;
        if (r4 & kOpLast) all_fetched = true;
      }
      if ((it & 7u) == 7u) {
        if (__ballot(!fin) == 0) { expired = false; break; }
        const uint64_t hold = __ballot(have_cur || fin);
        if (!fin && (prog_acc & segmask) == 0 && (hold & segmask) == segmask) {
          // every unfinished machine of this candidate holds an op and none could run for a whole
          // window: deadlock, i.e. a cycle of the combined graph (or a 16-bit overflow when optimistic)
          stalled = true;
          fin = true;
          *abort_p = 1;
        }
        prog_acc = 0;
      }
    }
    if (expired && __ballot(!fin) != 0) {                   // bounded wait ran out: report, release the feeder
      if (!fin) { flagw[g] = kBitInternal; *abort_p = 1; }
    }
    acc = (int32_t)x_acc;
  } else {
    // ------------------------------------------------------------ feeder
    lds_cu8_t *const pib = (lds_cu8_t *)(ldsb + o.o_pi + g * o.pi_stride);
    lds_cu8_t *const commr = (lds_cu8_t *)(ldsb + o.o_comm);
    lds_vu32_t *const ring_wp = (lds_vu32_t *)(ldsb + o.o_ring) + ql;
    lds_vu32_t *const tail_p = (lds_vu32_t *)(ldsb + o.o_tail) + ql;
    lds_vi32_t *const abort_p = (lds_vi32_t *)(ldsb + o.o_abort) + g;
    const uint16_t *list = p.ws_list + (c0 + (cand_ok ? g : 0)) * p.list_stride;
    int k = has_ops ? offw[ql] : 0;
    const int kend = has_ops ? k + cntw[ql] : 0;
    bool fin = !has_ops;
    uint32_t head = 0, tail_seen = 0;
    int64_t level = 0, peak = 0;
    uint4 rc = make_uint4(0, 0, 0, 0), rn = make_uint4(0, 0, 0, 0);
    int64_t mc = 0, mn = 0;
    uint32_t v2 = 0;
    bool first_part = true;
    if (!fin) {
      const uint32_t v0 = list[k];
      rc = p.rec[v0];
      mc = p.mem_delta[v0];
      if (k + 1 < kend) { const uint32_t v1 = list[k + 1]; rn = p.rec[v1]; mn = p.mem_delta[v1]; }
      if (k + 2 < kend) v2 = list[k + 2];
    }
    for (uint32_t it = 0; it < p.spin_cap; ++it) {
      if (__ballot(!fin) == 0) break;
      bool full = (head - tail_seen) >= (uint32_t)RING;
      if (!fin && full) {
        tail_seen = *tail_p;
        full = (head - tail_seen) >= (uint32_t)RING;
        if (full && *abort_p) fin = true;
      }
      if (!fin && !full) {
        const uint32_t u0 = rc.x & 0xFFFFu, u1 = rc.x >> 16, u2 = rc.y & 0xFFFFu, u3 = rc.y >> 16;
        const uint32_t d0 = commr[pib[u0] * P + j], d1 = commr[pib[u1] * P + j];
        const uint32_t d2 = commr[pib[u2] * P + j], d3 = commr[pib[u3] * P + j];
        const bool more = (rc.z >> 31) != 0;
        const bool last = !more && (k + 1 == kend);
        const uint32_t gen = (((head >> p.log_ring) & 1u) ^ 1u) << kOpGenShift;
        const uint32_t w4 = (rc.w >> 16) | (more ? 0u : kOpFinal) | (last ? kOpLast : 0u) | gen;
        lds_vu32_t *const sp = ring_wp + (head & (uint32_t)(RING - 1)) * slot_words;
        sp[0] = rc.x;
        sp[plane] = rc.y;
        sp[2 * plane] = d0 | (d1 << 8) | (d2 << 16) | (d3 << 24);
        sp[3 * plane] = rc.z & 0x7FFFFFFFu;
        sp[4 * plane] = w4;
        ++head;
        if (first_part) { level += mc; peak = max(peak, level); }   // eq. (19) along the chain
        if (more) {
          rc = p.rec[N + (rc.w & 0xFFFFu)];
          first_part = false;
        } else {
          first_part = true;
          ++k;
          if (k == kend) {
            fin = true;
          } else {
            rc = rn; mc = mn;
            if (k + 1 < kend) { rn = p.rec[v2]; mn = p.mem_delta[v2]; }
            if (k + 2 < kend) v2 = list[k + 2];
          }
        }
      }
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
