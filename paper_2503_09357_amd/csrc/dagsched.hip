// dagsched: batched evaluation of candidate operator schedules on gfx950 (MI355X) - host side and C-ABI.
//
// Per candidate (a placement x and dense per-machine ranks fixing y/u of the MIP in Sec. III of
// arxiv 2503.09357) the kernels compute the earliest-start schedule on the disjunctive graph
// (operator-DAG edges plus one chain edge between consecutive operations of a machine):
//   s_v = max(0, e_chainpred(v), max_{(u,v) in B} e_u + delta(u,v)),  e_v = s_v + D^o_v     eqs. (2),(3),(7),(11)-(13)
// and from it the makespan (eqs. (1)-(2)), the total idle time P*z - sum D^o, the per-machine peak of
// the running memory level (eqs. (17)-(19)) and a structural cycle flag (eqs. (5),(7),(8) infeasible).
//
// Mapping: one lane per (candidate, machine).  A machine's operations are totally ordered, so in a
// Kahn round at most one operation per machine becomes ready: lane (c, j) walks machine j's order
// list of candidate c and polls the end times of the DAG predecessors of its head operation.  All
// lanes of a candidate sit in one 64-wide wavefront (P <= 64), so "no lane of the candidate advanced"
// (a ballot) is an exact deadlock test, i.e. a cycle of the combined graph.
//
// Two kernels: the ring kernel (kernel_ring.h; 16-bit end times in LDS, relaxer + feeder wavefronts)
// is the fast path; the general kernel (kernel_general.h; int32 end times) takes what the ring kernel
// cannot prove or finish.  No MFMA anywhere: integer max/plus with data-dependent gathers is not a
// contraction.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <numeric>
#include <vector>

#include "dagsched.h"
#include "device_common.h"
#include "kernel_coarsen.h"
#include "kernel_contended.h"
#include "kernel_general.h"
#include "kernel_ring.h"
#include "kernel_search.h"
#include "kernel_static.h"
#include "kernel_util.h"

using namespace dagsched_dev;

// Scratch of dagsched_schedule_static, the entry point for callers that cannot allocate: one order-list row and one
// end-time row of kStaticMaxNodes int32 each, then the small output block of the one-candidate evaluation.  The
// array's name is a host-side stand-in only; host code uses the device address that hipGetSymbolAddress returns for
// the current device (every GPU holds a copy of its own), kept per device in g_scratch.
constexpr int kStaticMaxNodes = DAGSCHED_STATIC_MAX_NODES;
constexpr size_t kScratchOut = 2 * sizeof(int32_t) * (size_t)kStaticMaxNodes;
constexpr size_t kScratchBytes = kScratchOut + 32 + 8 * DAGSCHED_MAX_DEVICES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

constexpr int kMaxGpus = 64;
unsigned char *g_scratch[kMaxGpus] = {};   // device address of `scratch` on each GPU a handle was made on

thread_local char g_hip_error[256] = "";

bool hip_ok(hipError_t e, const char *what) {
  if (e == hipSuccess) return true;
  snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", what, hipGetErrorString(e));
  return false;
}

inline int next_pow2(int x) {
  int p = 1;
  while (p < x) p <<= 1;
  return p;
}
inline int ilog2(int x) {
  int l = 0;
  while ((1 << l) < x) ++l;
  return l;
}
inline uint32_t align_up(uint32_t x, uint32_t a) { return (x + a - 1) / a * a; }

enum { kVariantGeneralLds = 1, kVariantGeneralGlobal = 2, kVariantRingExact = 3, kVariantRingOptimistic = 4,
       kVariantRing32 = 5, kVariantStatic = 6 };

}  // namespace

struct dagsched {
  int32_t N = 0, E = 0, P = 0, Pseg = 0, max_cand = 0, layout = 0, device = 0;
  int64_t sum_dur = 0;
  int32_t variant = 0;
  // general kernel
  int32_t gen_G = 0, gen_lds = 0;
  bool gen_lds_state = false;
  int64_t row_stride = 0;
  int32_t *d_pred_ptr = nullptr, *d_pred_idx = nullptr, *d_dur = nullptr, *d_comm = nullptr;
  int64_t *d_mem = nullptr, *d_weight = nullptr, *d_limit = nullptr;
  int32_t *ws_list = nullptr, *ws_end = nullptr;
  // ring kernel
  int32_t ring_G = 0, ring_slots = 0, ring_feeders = 1, ring_kind = 0, ring_block = 256, rec_plane = 0, id_bits = 16, time_scale = 1;
  uint8_t *d_nparts = nullptr;
  int64_t list_stride = 0, pib_stride = 0;
  uint8_t *ws_pib = nullptr;
  LdsLayout lds{};
  // Fallback of the optimistic 16-bit run and of the window mode: the same problem in the 32-bit form of the ring
  // kernel (exact), launched over the list of candidates the first run left; fb_G == 0: the general kernel instead
  int32_t fb_G = 0, fb_slots = 0, fb_feeders = 1, fb_block = 256, fb_kind = 0;
  bool fb_optimistic = false;             // the fallback is itself a 16-bit run with the general kernel behind it (window mode on
                                          // a problem too large for 32-bit cells)
  LdsLayout fb_lds{};
  LdsLayout lds_ingest{};                 // window mode: layout of the ingest launch
  int32_t ingest_block = 1024;
  uint32_t win_magic = 0;
  int32_t *ws_meta = nullptr;             // window mode: what the ingest launch hands to the relaxation, per workgroup
  uint4 *d_rec = nullptr;
  int32_t *d_comm_scaled = nullptr;
  uint64_t *d_no_channel = nullptr;   // [P] bit b of word a: no channel a -> b (eq. (10)); null when every pair has one
  uint32_t *d_edges = nullptr;        // [E] u | v << 16 for the pass that flags candidates using such a pair
  uint16_t *ws_list16 = nullptr;
  int32_t *d_fb_count = nullptr, *d_fb_list = nullptr;
  uint32_t spin_cap = 0;
  // shared-placement kernel
  StaticParams st{};
  int32_t st_preds = 4, st_grid = 1;      // st_grid: workgroups that are resident at once (each loops over batches)
  uint4 *d_st_ops = nullptr;
  uint8_t *d_st_machine = nullptr;
  int32_t *d_st_off = nullptr;
  int64_t *d_st_base = nullptr;
  // search helpers: machine counts of a base schedule; one row of general-kernel workspace and outputs
  int32_t *ws_cnt = nullptr, *ws_sched_list = nullptr, *ws_sched_end = nullptr;
  unsigned char *ws_sched_out = nullptr;
  // candidate-minor input staging
  int32_t *ws_tp = nullptr, *ws_tr = nullptr, *ws_te = nullptr;
  // evaluation with channel contention: edge tables and one workspace row per resident workgroup
  bool contention = false;
  int32_t *d_pred_eid = nullptr, *d_edge_src = nullptr, *d_edge_dst = nullptr, *d_succ_ptr = nullptr;
  int32_t *wc_list = nullptr, *wc_end = nullptr, *wc_tlist = nullptr, *wc_tend = nullptr, *wc_ccnt = nullptr, *wc_coff = nullptr, *wc_echan = nullptr;
  int32_t wc_grid = 0;
  int64_t row_e = 0, row_c = 0;
};

namespace {

int validate_desc(const dagsched_desc_t *d, std::vector<int32_t> *pred_ptr, std::vector<int32_t> *pred_idx,
                  int64_t *sum_dur_out) {
  if (!d) return DAGSCHED_EINVAL;
  const int32_t N = d->n_nodes, E = d->n_edges, P = d->n_devices;
  if (N < 1 || N > DAGSCHED_MAX_NODES || E < 0 || P < 1 || P > DAGSCHED_MAX_DEVICES) return DAGSCHED_EINVAL;
  if (!d->row_ptr || !d->dur || !d->comm || !d->mem_delta || (E > 0 && !d->col_idx)) return DAGSCHED_EINVAL;
  if (d->max_candidates < 1) return DAGSCHED_EINVAL;
  if (d->layout != DAGSCHED_CAND_MAJOR && d->layout != DAGSCHED_CAND_MINOR) return DAGSCHED_EINVAL;
  if (const dagsched_shape_t *sh = d->shape) {
    const int32_t g = sh->cand_per_block, r = sh->ring_slots, b = sh->block_threads;
    if (g < 0 || g > kWave || (g & (g - 1))) return DAGSCHED_EINVAL;
    if (r != 0 && r != 4 && r != 8 && r != 16 && r != 32) return DAGSCHED_EINVAL;
    if (sh->feeders < 0 || sh->feeders > 4 || sh->placement_mode < -1 || sh->placement_mode > 2) return DAGSCHED_EINVAL;
    if (b < 0 || b > 1024 || b % kWave) return DAGSCHED_EINVAL;
    if (sh->state_bits != 0 && sh->state_bits != 16 && sh->state_bits != 32) return DAGSCHED_EINVAL;
    if (sh->preds_per_op != 0 && sh->preds_per_op != 2 && sh->preds_per_op != 4) return DAGSCHED_EINVAL;
    if (sh->kernel < 0 || sh->kernel > 1 || sh->static_waves < 0 || sh->static_waves > 8) return DAGSCHED_EINVAL;
    if (sh->ignore_shared_placement < 0 || sh->ignore_shared_placement > 1) return DAGSCHED_EINVAL;
    if (sh->window_cells < -1 || (sh->window_cells > 0 && (sh->window_cells < 8 || sh->window_cells > 32768 ||
                                                             (sh->window_cells & (sh->window_cells - 1)))))
      return DAGSCHED_EINVAL;
  }
  if (d->row_ptr[0] != 0 || d->row_ptr[N] != E) return DAGSCHED_EINVAL;
  for (int32_t u = 0; u < N; ++u)
    if (d->row_ptr[u + 1] < d->row_ptr[u]) return DAGSCHED_EINVAL;
  std::vector<int32_t> indeg(N, 0);
  for (int32_t u = 0; u < N; ++u)
    for (int32_t k = d->row_ptr[u]; k < d->row_ptr[u + 1]; ++k) {
      const int32_t w = d->col_idx[k];
      if (w < 0 || w >= N || w == u) return DAGSCHED_EINVAL;
      ++indeg[w];
    }
  int64_t sum_dur = 0, max_comm = 0;
  for (int32_t v = 0; v < N; ++v) {
    if (d->dur[v] < 0) return DAGSCHED_EINVAL;
    sum_dur += d->dur[v];
  }
  if (d->weight)
    for (int32_t v = 0; v < N; ++v)
      if (d->weight[v] < 0) return DAGSCHED_EINVAL;
  if (d->shared_placement)
    for (int32_t v = 0; v < N; ++v)
      if (d->shared_placement[v] < 0 || d->shared_placement[v] >= P) return DAGSCHED_EINVAL;
  for (int32_t a = 0; a < P; ++a)
    for (int32_t b = 0; b < P; ++b)
      if (a != b) {
        if (d->comm[a * P + b] < DAGSCHED_NO_CHANNEL) return DAGSCHED_EINVAL;
        max_comm = std::max<int64_t>(max_comm, d->comm[a * P + b]);
      }
  // predecessor CSR (edge multiplicity kept) and acyclicity of B by peeling sources
  std::vector<int32_t> pptr(N + 1, 0);
  for (int32_t v = 0; v < N; ++v) pptr[v + 1] = pptr[v] + indeg[v];
  std::vector<int32_t> pidx(E > 0 ? E : 1), fill(pptr.begin(), pptr.end() - 1);
  for (int32_t u = 0; u < N; ++u)
    for (int32_t k = d->row_ptr[u]; k < d->row_ptr[u + 1]; ++k) pidx[fill[d->col_idx[k]]++] = u;
  std::vector<int32_t> stack;
  stack.reserve(N);
  for (int32_t v = 0; v < N; ++v)
    if (indeg[v] == 0) stack.push_back(v);
  int32_t peeled = 0;
  while (!stack.empty()) {
    const int32_t u = stack.back();
    stack.pop_back();
    ++peeled;
    for (int32_t k = d->row_ptr[u]; k < d->row_ptr[u + 1]; ++k)
      if (--indeg[d->col_idx[k]] == 0) stack.push_back(d->col_idx[k]);
  }
  if (peeled != N) return DAGSCHED_ECYCLE;
  // a path visits each node once and pays at most one delay per edge: below this bound int32 is exact
  if (sum_dur + (int64_t)(N - 1) * max_comm > (int64_t)INT32_MAX) return DAGSCHED_EOVERFLOW;
  if (pred_ptr) pred_ptr->swap(pptr);
  if (pred_idx) pred_idx->swap(pidx);
  if (sum_dur_out) *sum_dur_out = sum_dur;
  return DAGSCHED_OK;
}

template <typename T>
bool upload(T **dst, const T *src, size_t n) {
  if (!hip_ok(hipMalloc((void **)dst, std::max<size_t>(n, 1) * sizeof(T)), "hipMalloc")) return false;
  if (n == 0) return true;
  return hip_ok(hipMemcpy(*dst, src, n * sizeof(T), hipMemcpyHostToDevice), "hipMemcpy");
}

template <typename T>
bool dev_alloc(T **dst, size_t n) {
  return hip_ok(hipMalloc((void **)dst, std::max<size_t>(n, 1) * sizeof(T)), "hipMalloc workspace");
}

void free_handle(dagsched *h) {
  if (!h) return;
  void *bufs[] = {h->d_pred_ptr, h->d_pred_idx, h->d_dur, h->d_comm, h->d_mem, h->d_weight, h->d_limit, h->ws_list, h->ws_end, h->d_rec,
                  h->d_comm_scaled, h->d_nparts, h->ws_list16, h->ws_pib, h->ws_cnt, h->ws_sched_list, h->ws_sched_end,
                  h->ws_sched_out, h->d_fb_count, h->d_fb_list, h->ws_meta, h->ws_tp, h->ws_tr, h->d_no_channel, h->d_edges,
                  h->d_st_ops, h->d_st_machine, h->d_st_off, h->d_st_base, h->ws_te, h->d_pred_eid, h->d_edge_src, h->d_edge_dst, h->d_succ_ptr,
                  h->wc_list, h->wc_end, h->wc_tlist, h->wc_tend, h->wc_ccnt, h->wc_coff, h->wc_echan};
  for (void *b : bufs)
    if (b) (void)hipFree(b);
  delete h;
}

// pib_lds: 0 placement bytes in L2, 1 in LDS, 2 in LDS as nibbles (P <= 16)
// cell_bytes: 2 (16-bit end times) or 4
// win_log2 > 0: window mode, 2^win_log2 named cells of four bytes per candidate instead of one cell per operation
LdsLayout ring_layout(int N, int P, int G, int ring, int pib_lds, int cell_bytes, bool wide, int win_log2 = 0) {
  LdsLayout o{};
  uint32_t at = 0;
  o.s_stride = win_log2 ? (cell_bytes == 4 ? 8u : 4u) << win_log2          // window: name and end time, 16 or 32 bits each
                        : align_up((uint32_t)cell_bytes * (uint32_t)(N + 2), 4);   // N cells + dummy + trash; the arrays start at LDS offset 0
  o.win_log2 = (uint32_t)win_log2;
  o.cell_bytes = (uint32_t)cell_bytes;
  at += (uint32_t)G * o.s_stride;
  o.pi_stride = pib_lds == 1 ? align_up((uint32_t)(N + 1), 4) : pib_lds == 2 ? align_up((uint32_t)(N + 2) / 2u, 4) : 0u;
  o.pib_mode = (uint32_t)pib_lds;
  o.o_pi = at;    at += (uint32_t)G * o.pi_stride;
  at = align_up(at, 16);
  o.o_ring = at;  at += (uint32_t)ring * kWave * 16u;
  o.o_scr = at;   at += kWave * ((win_log2 && cell_bytes == 4) ? 8u : 4u);
  o.o_total = at; at += kWave * 4u;
  at = align_up(at, 8);
  o.o_peak = at;  at += kWave * 8u;
  o.o_cnt = at;   at += kWave * 4u;
  o.o_off = at;   at += kWave * 4u;
  o.o_flag = at;  at += kWave * 4u;
  o.o_abort = at; at += kWave * 4u;
  o.o_over = at;  at += kWave;
  o.wide = wide ? 1u : 0u;
  // channel delays: a byte each, rows [source machine + the dummy's][destination]; wide ops: a dword each, 64 rows
  o.o_comm = at;  at += wide ? (uint32_t)kWave * (uint32_t)next_pow2(P) * 4u
                             : align_up((uint32_t)(P + 1) * (uint32_t)next_pow2(P), 4);
  o.total = align_up(at, 16);
  return o;
}

// Decide whether the ring kernel can take this problem and with which shape.
// Needs: every scaled delay <= 255, at most 65536 overflow records, the scaled lower bound on any
// makespan (critical path of B, heaviest possible average load) below the 16-bit range, and an LDS
// footprint that fits a workgroup.
using RingKernel = void (*)(RingParams);
template <int HALF>
RingKernel ring_kernel_pick(int ring, int feeders, int pib_lds, int kind);

struct RingPlan {
  bool ok = false, exact = false, cell32 = false;
  int G = 0, ring = 0, feeders = 1, kind = 0, block = 256;
  int32_t scale = 1;
  LdsLayout lds{};
  std::vector<uint4> rec;
  int rec_plane = 0, id_bits = 16;
  std::vector<uint8_t> nparts;
  std::vector<int32_t> comm_scaled;
  // window mode: cells per candidate (0: off), the layout and workgroup size of the ingest launch
  int win_log2 = 0, ingest_block = 1024;
  uint32_t win_magic = 0;
  LdsLayout lds_ingest{};
};

RingPlan plan_ring(const dagsched_desc_t *d, const std::vector<int32_t> &pred_ptr, const std::vector<int32_t> &pred_idx,
                   int64_t sum_dur, int lds_max, int n_cu) {
  RingPlan plan;
  const int N = d->n_nodes, P = d->n_devices, Pseg = next_pow2(P);
  int64_t g = 0, max_comm = 0;
  for (int v = 0; v < N; ++v) g = std::gcd<int64_t, int64_t>(g, d->dur[v]);
  for (int a = 0; a < P; ++a)
    for (int b = 0; b < P; ++b)
      if (a != b) {
        g = std::gcd<int64_t, int64_t>(g, d->comm[a * P + b]);
        max_comm = std::max<int64_t>(max_comm, d->comm[a * P + b]);
      }
  if (g == 0) g = 1;                                   // every duration and delay is zero
  // delays above 255 or durations above 65534 (in units of the gcd) do not fit the compact op: wide ops then
  bool wide = max_comm / g > 255;
  for (int v = 0; v < N; ++v) wide = wide || d->dur[v] / g >= (int64_t)kNotDone16;
  for (int v = 0; v < N; ++v)
    if (d->dur[v] / g >= 256 * 65535) return plan;       // ... whose durations are low + 65535 * high, high < 256
  // longest path of B alone in scaled units (no delays): a lower bound on every makespan
  std::vector<int64_t> fin(N, -1);
  {
    std::vector<int32_t> order;                        // topological order by repeated peeling on pred lists
    std::vector<int32_t> indeg(N);
    for (int v = 0; v < N; ++v) indeg[v] = pred_ptr[v + 1] - pred_ptr[v];
    order.reserve(N);
    for (int v = 0; v < N; ++v) if (indeg[v] == 0) order.push_back(v);
    for (size_t i = 0; i < order.size(); ++i) {
      const int u = order[i];
      int64_t best = 0;
      for (int k = pred_ptr[u]; k < pred_ptr[u + 1]; ++k) best = std::max(best, fin[pred_idx[k]]);
      fin[u] = best + d->dur[u] / g;
      for (int k = d->row_ptr[u]; k < d->row_ptr[u + 1]; ++k)
        if (--indeg[d->col_idx[k]] == 0) order.push_back(d->col_idx[k]);
    }
  }
  const int64_t crit = *std::max_element(fin.begin(), fin.end());
  const int64_t lower = std::max<int64_t>(crit, (sum_dur / g + P - 1) / P);
  const int64_t upper = sum_dur / g + (int64_t)(N - 1) * (max_comm / g);
  plan.scale = (int32_t)g;

  constexpr int PR = 4;                                // DAG predecessors per op part
  // Predecessor lists of the ops.  An edge (u, v) is left out when B has another path u -> w1 -> ... -> wk -> v
  // whose intermediate durations sum to at least the largest channel delay: then s_v >= e_wk >= ... >= e_u +
  // sum D^o_wi >= e_u + delta(u, v) whatever the candidate, so eqs. (11)-(13) for (u, v) are implied (and a cycle
  // through (u, v) also runs through that path).  Fewer parts mean fewer relaxer trips on the critical path, and
  // a pipeline's operations keep a single predecessor each (the forward -> backward edge of a stage is implied by
  // the path through the next stage), which selects a lighter kind of kernel.  Bounded search: six hops, 512
  // visits (four hops do for the plain pipelines, six for the bidirectional one with its transfer operations).
  std::vector<std::vector<int32_t>> op_preds(N);
  {
    struct Item { int32_t node, hops; int64_t sum; };
    std::vector<Item> stack;
    auto implied = [&](int32_t u, int32_t v) {
      stack.clear();
      stack.push_back({u, 0, 0});
      int visits = 0;
      while (!stack.empty()) {
        const Item it = stack.back();
        stack.pop_back();
        if (++visits > 512) return false;
        for (int32_t k = d->row_ptr[it.node]; k < d->row_ptr[it.node + 1]; ++k) {
          const int32_t y = d->col_idx[k];
          if (y == v) {
            if (it.hops >= 1 && it.sum >= max_comm) return true;
          } else if (it.hops + 1 < 6) {
            stack.push_back({y, it.hops + 1, it.sum + d->dur[y]});
          }
        }
      }
      return false;
    };
    for (int v = 0; v < N; ++v) {
      const int deg = pred_ptr[v + 1] - pred_ptr[v];
      for (int k = pred_ptr[v]; k < pred_ptr[v + 1]; ++k)
        if (deg < 2 || !implied(pred_idx[k], v)) op_preds[v].push_back(pred_idx[k]);
    }
  }
  // shared operator records, part i of node v at [i * plane + v]
  const uint32_t dummy = (uint32_t)N;
  int max_parts = 1;
  for (int v = 0; v < N; ++v) max_parts = std::max(max_parts, ((int)op_preds[v].size() + PR - 1) / PR);
  if (max_parts > 16) return plan;                     // very wide fan-in: leave it to the general kernel
  {                                                    // the kernel counts a lane's op parts in 16 bits
    int64_t total_parts = 0;
    for (int v = 0; v < N; ++v) total_parts += std::max(1, ((int)op_preds[v].size() + PR - 1) / PR);
    if (total_parts >= 65536) return plan;
  }
  // kernel kind: 2 when no operation has more than two DAG predecessors, 1 when none has more than four (every
  // operation is a single part), 0 otherwise (or when the caller's shape asks for four predecessors per op)
  size_t max_deg = 0;
  for (int v = 0; v < N; ++v) max_deg = std::max(max_deg, op_preds[v].size());
  plan.kind = (d->shape && d->shape->preds_per_op == 4) ? 0 : max_deg <= 1 ? 3 : max_deg <= 2 ? 2 : max_parts == 1 ? 1 : 0;
  if (d->shape && d->shape->preds_per_op == 2 && plan.kind == 3) plan.kind = 2;   // (the caller asks for the two-predecessor kind)
  const int plane = N;
  std::vector<uint4> rec((size_t)max_parts * plane, make_uint4(dummy | (dummy << 16), dummy | (dummy << 16), 0, 0));
  for (int v = 0; v < N; ++v) {
    const int deg = (int)op_preds[v].size();
    const int parts = std::max(1, (deg + PR - 1) / PR);
    // A part waits for its own predecessors and for the parts before it, so the operation ends one trip
    // later for every part that follows the one holding its last predecessor.  Predecessors that end late
    // on the critical path of B alone go last, and the first part takes the remainder.
    std::vector<int32_t> &ps = op_preds[v];
    std::stable_sort(ps.begin(), ps.end(), [&](int32_t a, int32_t b) { return fin[a] < fin[b]; });
    const int first = deg - PR * (parts - 1);
    for (int part = 0; part < parts; ++part) {
      uint32_t u[4] = {dummy, dummy, dummy, dummy};
      const int lo = part == 0 ? 0 : first + (part - 1) * PR, hi = part == 0 ? first : lo + PR;
      for (int k = lo; k < hi && k < deg; ++k) u[k - lo] = (uint32_t)ps[k];
      const bool more = part + 1 < parts;
      // (wide ops: low part below 0xFFFF, which marks a free ring slot, and the high part above it)
      const uint32_t dur = more ? 0u
                         : wide ? (uint32_t)((d->dur[v] / g) % 65535) | ((uint32_t)((d->dur[v] / g) / 65535) << 16)
                                : (uint32_t)std::min<int64_t>(d->dur[v] / g, kNotDone16);
      rec[(size_t)part * plane + v] = make_uint4(u[0] | (u[1] << 16), u[2] | (u[3] << 16),
                                                 dur | (part == 0 ? 0x40000000u : 0u) | (more ? 0x80000000u : 0u),
                                                 (uint32_t)v << 16);
    }
  }
  plan.rec.swap(rec);
  plan.rec_plane = plane;
  // the order-list entries are 16 bits: node id below, (parts - 1) above
  int part_bits = 0;
  while ((1 << part_bits) < max_parts) ++part_bits;
  plan.id_bits = 16 - part_bits;
  if (N > (1 << plan.id_bits)) return plan;            // ids and part counts do not fit: general kernel
  for (int v = 0; v < N; ++v) {                        // 0xFFFF marks an unwritten list slot during ingest
    const int parts = std::max(1, ((int)op_preds[v].size() + PR - 1) / PR);
    if (((uint32_t)v | ((uint32_t)(parts - 1) << plan.id_bits)) == 0xFFFFu) return plan;
  }
  if (max_parts > 1) {
    plan.nparts.resize(N);
    for (int v = 0; v < N; ++v) plan.nparts[v] = (uint8_t)std::max(1, ((int)op_preds[v].size() + PR - 1) / PR);
  }
  plan.comm_scaled.resize((size_t)P * P);
  for (int i = 0; i < P * P; ++i) plan.comm_scaled[i] = (i / P != i % P) ? (int32_t)(d->comm[i] / g) : 0;

  // shape: most candidates resident per CU first.  Placement bytes in LDS give the fastest feeders but cost
  // N bytes per candidate; in L2 they leave room for more candidates or a deeper ring.  Measured weights: a
  // four-slot ring counts 0.7 (hot lanes outrun it), placement bytes in L2 count 0.7 (0.85 with two predecessors
  // per op: half the gathers; a 36-layer MoE graph, N = 6912: four workgroups per CU with them in L2 0.179 us per
  // candidate, three with them in LDS 0.135), and workgroups beyond
  // five per CU count nothing, half-empty wavefronts count 0.65 (the feeders do the same work for half the
  // candidates); at equal counts, more workgroups of fewer candidates.
  // a shape given with the description wins, field by field
  const dagsched_shape_t *sh = d->shape;
  // Width of the end times.  16 bits when every end time provably fits, or when most candidates can be expected to
  // fit (the rest then go to the int32 kernel one by one); 32 bits (half the candidates resident, always exact)
  // when they cannot: makespans of list schedules lie around three times the lower bound.
  const int force_bits = sh ? sh->state_bits : 0;
  const bool fits16 = upper + 255 < (int64_t)kNotDone16;
  plan.cell32 = wide || force_bits == 32 || (force_bits != 16 && !fits16 && 3 * lower >= (int64_t)kNotDone16);
  if (!plan.cell32 && lower >= (int64_t)kNotDone16) return plan;   // 16 bits asked for, and no candidate could stay inside them
  const int cell_bytes = plan.cell32 ? 4 : 2;
  // Window mode: when the operations run roughly in the order of their ids (a layered graph numbered level by
  // level), a candidate needs only a window of K named cells instead of a cell per operation (see the kernel).
  // A candidate whose schedule does not fit the window is handed to the int32 kernel, never evaluated wrongly, but
  // that kernel is some seventy times slower, so K is chosen with a margin: operation x = u + m (K - 3) takes over
  // the cell of u, and it must lie at least 24 levels of B (edges on the longest path from a source) behind every
  // reader v of u, for every edge (u, v) and every m.  (The layered workload: margin 29 at 4096 cells, where a
  // trip-by-trip simulation of 48 list schedules found none that misses; 13 at 2048 cells, where 11 of 48 miss.
  // The MoE graph, numbered micro-batch by micro-batch: no K has a margin, although its edges are short once the
  // implied ones are dropped.)  The margin alone does not do: the MoE graph RENUMBERED level by level has a margin
  // of 53 levels at 1024 cells and 70 % of its list schedules miss there (6 of 4096 at 2048 cells, none at 4096,
  // where the mode is slower than a cell per operation anyway: 1.29 against 1.11 ms): its levels are narrow (19
  // operations for 32 machines), so the machines follow the chains of their micro-batches, not the levels.  Hence
  // the second condition: a level holds at least one operation per machine on average.  Taken when such a K
  // shrinks the end-time state at least 2.5 times on a problem large enough for that to matter, or when the
  // caller's shape names K.
  int win_log2 = 0;
  {
    const int want = sh ? sh->window_cells : 0;
    int64_t span = 0;
    bool topological = true;
    for (int v = 0; v < N; ++v)
      for (int32_t u : op_preds[v]) { topological = topological && u < v; span = std::max<int64_t>(span, v - u); }
    int K = 0;
    if (want > 0) {
      K = want;
    } else if (want == 0 && N >= 8192 && topological) {
      std::vector<int32_t> lvl(N, 0);                      // (ids are a topological order here)
      for (int v = 0; v < N; ++v)
        for (int32_t u : op_preds[v]) lvl[v] = std::max(lvl[v], lvl[u] + 1);
      const int64_t n_levels = (int64_t)*std::max_element(lvl.begin(), lvl.end()) + 1;
      for (int k = 1024; k <= 32768 && !K && (int64_t)N >= n_levels * P; k <<= 1) {
        if ((int64_t)k * 4 * 5 > (int64_t)(2 * N) * 2 || span >= k - 3) continue;
        int64_t margin = INT64_MAX;
        for (int v = 0; v < N && margin >= 24; ++v)
          for (int32_t u : op_preds[v])
            for (int64_t x = (int64_t)u + (k - 3); x < N; x += k - 3) margin = std::min<int64_t>(margin, (int64_t)lvl[x] - lvl[v]);
        if (margin >= 24) K = k;
      }
    }
    const bool fits_names = K >= 8 && K <= 32768 && (int64_t)N + 3 * ((int64_t)N / (K - 3)) + 1 <= 65535;
    const bool worth = want > 0 || (int64_t)K * 4 * 5 <= (int64_t)(2 * N) * 2;
    if (K && topological && fits_names && worth && !wide) win_log2 = ilog2(K);   // (32-bit end times: cells of 64 bits)
  }
  const int force_g = sh ? sh->cand_per_block : 0;
  const int force_ring = sh ? sh->ring_slots : 0;
  const int force_feeders = sh ? sh->feeders : 0;
  const int force_pib = sh ? sh->placement_mode : -1;
  int64_t best_score = -1;
  int best_wgs = 0;
  for (int G = kWave / Pseg; G >= 1; G >>= 1) {
    if (force_g && G != force_g) continue;
    for (int pib_lds : {1, 2, 0}) {
      if (force_pib >= 0 && pib_lds != force_pib) continue;
      if (win_log2 && pib_lds != 0) continue;             // window mode: the placement bytes stay in the workspace row
      if (pib_lds == 2 && (P > 16 || wide)) continue;     // a nibble per node; not with wide ops (see the kernel: time origin)
      for (int ring : {8, 16, 32, 4}) {
        if (force_ring && ring != force_ring) continue;
        if (pib_lds ? ring > 8 : ring < 8) continue;     // instantiated: LDS with 4 or 8 slots, L2 with 8, 16 or 32
        LdsLayout o = ring_layout(N, P, G, ring, pib_lds, cell_bytes, wide, win_log2);
        if ((int)o.total > lds_max) continue;
        if (!win_log2 && (uint64_t)G * (o.s_stride >> (plan.cell32 ? 2 : 1)) > 65536u) continue;   // half (quarter) addresses must fit 16 bits
        // window mode: the ingest launch builds the lists of the workgroup's G candidates in LDS, 2 N bytes each
        if (win_log2 && (int)ring_layout(N, P, G, 0, 0, 2, false).total > lds_max) continue;
        int wgs = std::min(5, lds_max / (int)align_up(o.total, 512));   // beyond ~20 wavefronts the CU is issue-bound
        if (wgs < 1) continue;
        // window mode relaxes every candidate of a full batch at once when it can: workgroups per CU beyond what the
        // batch fills count nothing, nor do those that leave the number of rounds as it is (four per CU needed: three
        // resident take two rounds like two); a deeper ring does count (config 5: 3 % for sixteen slots over eight,
        // 11 % with 32-bit end times)
        if (win_log2) {
          const int64_t need = std::max<int64_t>(1, ((d->max_candidates + G - 1) / G + n_cu - 1) / n_cu);
          const int64_t rounds = (need + wgs - 1) / wgs;
          wgs = (int)std::min<int64_t>(wgs, (need + rounds - 1) / rounds);
        }
        const int64_t score = (int64_t)wgs * G * (ring >= 8 ? 100 : 70) * (pib_lds == 1 ? 100 : pib_lds == 2 ? 99 : plan.kind == 2 ? 85 : 70) *
                                  (G * Pseg < kWave ? 65 : 100) + (ring == 16 ? 2 : 0) - G;
        if (score > best_score) { best_score = score; best_wgs = wgs; plan.G = G; plan.ring = ring; plan.lds = o; }
      }
    }
  }
  // feeders (measured): four when a single workgroup has the CU to itself and every placement byte comes from L2
  // (config 5: 3.6 % over two), three with one or two workgroups per CU (config 3: 13 % over two, config 4: 2.4 %),
  // two with more (config 2: three cost 16 %), one when the CU is full of wavefronts anyway
  plan.feeders = force_feeders ? force_feeders
               : (best_wgs == 1 && plan.lds.pib_mode == 0 && plan.ring == 16) ? 4
               : best_wgs <= 2 ? 3
               : (best_wgs * 4 <= 24 ? 2 : 1);
  auto built = [&](int feeders) {
    return win_log2    ? (plan.cell32 ? ring_kernel_pick<5>(plan.ring, feeders, (int)plan.lds.pib_mode, plan.kind) != nullptr
                                      : ring_kernel_pick<4>(plan.ring, feeders, (int)plan.lds.pib_mode, plan.kind) != nullptr)
         : wide        ? ring_kernel_pick<3>(plan.ring, feeders, (int)plan.lds.pib_mode, plan.kind) != nullptr
         : plan.cell32 ? ring_kernel_pick<2>(plan.ring, feeders, (int)plan.lds.pib_mode, plan.kind) != nullptr
                       : ring_kernel_pick<0>(plan.ring, feeders, (int)plan.lds.pib_mode, plan.kind) != nullptr;
  };
  // the one-predecessor kind exists for the 16-bit cells and the common shapes: else the two-predecessor kind does
  if (plan.kind == 3 && (win_log2 || wide || plan.cell32 || !built(plan.feeders))) plan.kind = 2;
  if (!force_feeders && !built(plan.feeders)) plan.feeders = 2;
  if (best_score < 0 || !built(plan.feeders)) return plan;   // shape not built
  // the nibble kernels start time at 255 (see the kernel), which the 16-bit range must hold as well
  // (a candidate that does not fit the window goes to the int32 kernel like one that leaves the 16-bit range: window
  // mode always runs with that kernel behind it)
  plan.exact = !win_log2 && (plan.cell32 || upper + (plan.lds.pib_mode == 2 ? 255 : 0) < (int64_t)kNotDone16);
  if (win_log2 && best_score >= 0) {
    plan.win_log2 = win_log2;
    plan.win_magic = (uint32_t)((1ull << 32) / (uint64_t)((1 << win_log2) - 3)) + 1u;
    plan.lds_ingest = ring_layout(N, P, plan.G, 0, 0, 2, false);
    const int ingest_wgs = std::max(1, lds_max / (int)align_up(plan.lds_ingest.total, 512));
    plan.ingest_block = ingest_wgs == 1 ? 1024 : ingest_wgs == 2 ? 512 : 256;
  }
  // workgroup size: the wavefronts with a role, plus helpers for the ingest phase when the LDS leaves the CU
  // nearly empty of wavefronts (one workgroup per CU: 1024 threads, two: 512)
  plan.block = ring_threads(plan.feeders);
  const int force_block = sh ? sh->block_threads : 0;
  if (force_block >= plan.block && force_block <= 1024 && force_block % kWave == 0) plan.block = force_block;
  else if (best_wgs == 1) plan.block = 1024;
  else if (best_wgs == 2) plan.block = std::max(plan.block, 512);
  plan.ok = best_score >= 0;
  return plan;
}

using RingKernel = void (*)(RingParams);
// The instantiated shapes: placement bytes in LDS with 4 or 8 ring slots, as nibbles in LDS likewise, in L2 with 8, 16
// or 32; one to four feeders where that was ever measured useful; each in the three kinds of the kernel.
#define DAGSCHED_RING_CASES(PIB, RING, F)                                                         \
  case 0 * 10000 + PIB * 1000 + RING * 10 + F: return relax_ring_kernel<RING, F, HALF, PIB, 0>;    \
  case 1 * 10000 + PIB * 1000 + RING * 10 + F: return relax_ring_kernel<RING, F, HALF, PIB, 1>;    \
  case 2 * 10000 + PIB * 1000 + RING * 10 + F: return relax_ring_kernel<RING, F, HALF, PIB, 2>;
// the one-predecessor kind: 16-bit cells only
#define DAGSCHED_RING_CASES_ONE(PIB, RING, F)                                                     \
  case 3 * 10000 + PIB * 1000 + RING * 10 + F: return relax_ring_kernel<RING, F, HALF, PIB, 3>;
// window mode: the relaxation launch (PHASE = 2) in the shapes that large layered problems get, and the ingest launch
#define DAGSCHED_WIN_CASES(RING, F)                                                               \
  case 0 * 10000 + RING * 10 + F: return relax_ring_kernel<RING, F, 4, 0, 0, 2>;                  \
  case 1 * 10000 + RING * 10 + F: return relax_ring_kernel<RING, F, 4, 0, 1, 2>;                  \
  case 2 * 10000 + RING * 10 + F: return relax_ring_kernel<RING, F, 4, 0, 2, 2>;
#define DAGSCHED_WIN32_CASES(RING, F)                                                             \
  case 0 * 10000 + RING * 10 + F: return relax_ring_kernel<RING, F, 5, 0, 0, 2>;                  \
  case 1 * 10000 + RING * 10 + F: return relax_ring_kernel<RING, F, 5, 0, 1, 2>;                  \
  case 2 * 10000 + RING * 10 + F: return relax_ring_kernel<RING, F, 5, 0, 2, 2>;
RingKernel ring_ingest_kernel(int kind) {
  return kind == 0 ? relax_ring_kernel<8, 2, 4, 0, 0, 1> : kind == 1 ? relax_ring_kernel<8, 2, 4, 0, 1, 1> : relax_ring_kernel<8, 2, 4, 0, 2, 1>;
}
template <int HALF>
RingKernel ring_kernel_pick(int ring, int feeders, int pib_lds, int kind) {
  if constexpr (HALF == 5) {                                    // window mode with 32-bit end times: fewer shapes
    if (pib_lds != 0) return nullptr;
    switch (kind * 10000 + ring * 10 + feeders) {
      DAGSCHED_WIN32_CASES(8, 2) DAGSCHED_WIN32_CASES(16, 2) DAGSCHED_WIN32_CASES(16, 3)
      default: return nullptr;
    }
  } else if constexpr (HALF == 4) {
    if (pib_lds != 0) return nullptr;
    switch (kind * 10000 + ring * 10 + feeders) {
      DAGSCHED_WIN_CASES(8, 1) DAGSCHED_WIN_CASES(8, 2) DAGSCHED_WIN_CASES(8, 3)
      DAGSCHED_WIN_CASES(16, 2) DAGSCHED_WIN_CASES(16, 3) DAGSCHED_WIN_CASES(16, 4)
      default: return nullptr;
    }
  } else if constexpr (HALF == 2) {                             // 32-bit end times: the shapes that large problems get
    switch (kind * 10000 + pib_lds * 1000 + ring * 10 + feeders) {
      DAGSCHED_RING_CASES(1, 8, 1) DAGSCHED_RING_CASES(1, 8, 2) DAGSCHED_RING_CASES(1, 8, 3)
      DAGSCHED_RING_CASES(2, 8, 2) DAGSCHED_RING_CASES(2, 8, 3)
      DAGSCHED_RING_CASES(0, 8, 2) DAGSCHED_RING_CASES(0, 16, 2) DAGSCHED_RING_CASES(0, 16, 3) DAGSCHED_RING_CASES(0, 16, 4)
      default: return nullptr;
    }
  } else if constexpr (HALF == 3) {                      // ... and wide ops (no nibbles)
    switch (kind * 10000 + pib_lds * 1000 + ring * 10 + feeders) {
      DAGSCHED_RING_CASES(1, 8, 1) DAGSCHED_RING_CASES(1, 8, 2) DAGSCHED_RING_CASES(1, 8, 3)
      DAGSCHED_RING_CASES(0, 8, 2) DAGSCHED_RING_CASES(0, 16, 2) DAGSCHED_RING_CASES(0, 16, 3) DAGSCHED_RING_CASES(0, 16, 4)
      default: return nullptr;
    }
  } else {
  switch (kind * 10000 + pib_lds * 1000 + ring * 10 + feeders) {
    DAGSCHED_RING_CASES(1, 4, 1) DAGSCHED_RING_CASES(1, 4, 2)
    DAGSCHED_RING_CASES(1, 8, 1) DAGSCHED_RING_CASES(1, 8, 2) DAGSCHED_RING_CASES(1, 8, 3) DAGSCHED_RING_CASES(1, 8, 4)
    DAGSCHED_RING_CASES(2, 4, 1) DAGSCHED_RING_CASES(2, 4, 2)
    DAGSCHED_RING_CASES(2, 8, 1) DAGSCHED_RING_CASES(2, 8, 2) DAGSCHED_RING_CASES(2, 8, 3)
    DAGSCHED_RING_CASES(0, 8, 1) DAGSCHED_RING_CASES(0, 8, 2) DAGSCHED_RING_CASES(0, 8, 3)
    DAGSCHED_RING_CASES(0, 16, 1) DAGSCHED_RING_CASES(0, 16, 2) DAGSCHED_RING_CASES(0, 16, 3) DAGSCHED_RING_CASES(0, 16, 4)
    DAGSCHED_RING_CASES(0, 32, 1) DAGSCHED_RING_CASES(0, 32, 2) DAGSCHED_RING_CASES(0, 32, 3)
    DAGSCHED_RING_CASES_ONE(1, 4, 1) DAGSCHED_RING_CASES_ONE(1, 4, 2)
    DAGSCHED_RING_CASES_ONE(1, 8, 1) DAGSCHED_RING_CASES_ONE(1, 8, 2) DAGSCHED_RING_CASES_ONE(1, 8, 3)
    DAGSCHED_RING_CASES_ONE(2, 8, 1) DAGSCHED_RING_CASES_ONE(2, 8, 2) DAGSCHED_RING_CASES_ONE(2, 8, 3)
    DAGSCHED_RING_CASES_ONE(0, 8, 2) DAGSCHED_RING_CASES_ONE(0, 8, 3) DAGSCHED_RING_CASES_ONE(0, 16, 2) DAGSCHED_RING_CASES_ONE(0, 16, 3)
    default: return nullptr;
  }
  }
}
#undef DAGSCHED_RING_CASES
#undef DAGSCHED_RING_CASES_ONE
RingKernel ring_kernel_for(const dagsched *h) {
  // byte addresses when the workgroup's end-time arrays fit 64 KB, half addresses otherwise
  const bool half = (uint64_t)h->ring_G * h->lds.s_stride > 65536u;
  const int pib_lds = (int)h->lds.pib_mode;
  if (h->lds.win_log2)
    return h->lds.cell_bytes == 4 ? ring_kernel_pick<5>(h->ring_slots, h->ring_feeders, pib_lds, h->ring_kind)
                                  : ring_kernel_pick<4>(h->ring_slots, h->ring_feeders, pib_lds, h->ring_kind);
  if (h->lds.wide) return ring_kernel_pick<3>(h->ring_slots, h->ring_feeders, pib_lds, h->ring_kind);
  if (h->lds.cell_bytes == 4) return ring_kernel_pick<2>(h->ring_slots, h->ring_feeders, pib_lds, h->ring_kind);
  return half ? ring_kernel_pick<1>(h->ring_slots, h->ring_feeders, pib_lds, h->ring_kind)
              : ring_kernel_pick<0>(h->ring_slots, h->ring_feeders, pib_lds, h->ring_kind);
}

// the kernel of the second run over the candidates the first one left (32-bit cells, or 16-bit ones behind a window)
RingKernel fallback_kernel(const dagsched *h) {
  const int pib_lds = (int)h->fb_lds.pib_mode;
  if (h->fb_lds.cell_bytes == 4) return ring_kernel_pick<2>(h->fb_slots, h->fb_feeders, pib_lds, h->fb_kind);
  const bool half = (uint64_t)h->fb_G * h->fb_lds.s_stride > 65536u;
  return half ? ring_kernel_pick<1>(h->fb_slots, h->fb_feeders, pib_lds, h->fb_kind)
              : ring_kernel_pick<0>(h->fb_slots, h->fb_feeders, pib_lds, h->fb_kind);
}

int static_threads(int relaxers) {                       // relaxers, accountants and as many wavefronts again for ingest
  return std::min(1024, 4 * relaxers * kWave);
}

// Plan of the shared-placement kernel: one op per operation with its delays resolved, the machines' list segments,
// and how many relaxing wavefronts share a workgroup.  Not taken (ok = false) when an operation has more than four
// distinct DAG predecessors, a time does not fit the op format or 16 bits, or the LDS is too small.
struct StaticPlan {
  bool ok = false;
  int G = 0, W = 0, preds = 4, scale = 1, wgs = 1;      // wgs: workgroups that fit a CU
  uint32_t o_mem = 0, o_mach = 0, o_cand = 0, cand_stride = 0, o_list = 0, o_book = 0, total = 0;
  std::vector<uint4> ops;
  std::vector<uint8_t> machine;
  std::vector<int32_t> off;
  std::vector<int64_t> base;
};

StaticPlan plan_static(const dagsched_desc_t *d, const std::vector<int32_t> &pred_ptr, const std::vector<int32_t> &pred_idx,
                       int64_t sum_dur, int lds_max, int n_cu) {
  StaticPlan plan;
  const int N = d->n_nodes, P = d->n_devices, Pseg = next_pow2(P);
  const int32_t *pi = d->shared_placement;
  if (2 * (N + 4) > 65535) return plan;                // cell offsets are 16-bit
  int64_t g = 0, max_delay = 0;
  for (int v = 0; v < N; ++v) g = std::gcd<int64_t, int64_t>(g, d->dur[v]);
  for (int v = 0; v < N; ++v)
    for (int k = pred_ptr[v]; k < pred_ptr[v + 1]; ++k) {
      const int u = pred_idx[k];
      if (pi[u] != pi[v]) {
        g = std::gcd<int64_t, int64_t>(g, d->comm[pi[u] * P + pi[v]]);
        max_delay = std::max<int64_t>(max_delay, d->comm[pi[u] * P + pi[v]]);
      }
    }
  if (g == 0) g = 1;
  if (max_delay / g > 255) return plan;
  if (sum_dur / g + (int64_t)(N - 1) * (max_delay / g) >= (int64_t)kNotDone16) return plan;   // every end time below 0xFFFF
  plan.ops.resize(N);
  int max_preds = 0;
  for (int v = 0; v < N; ++v) {
    // distinct predecessors; of two edges from one producer the delays are equal
    std::vector<int32_t> us(pred_idx.begin() + pred_ptr[v], pred_idx.begin() + pred_ptr[v + 1]);
    std::sort(us.begin(), us.end());
    us.erase(std::unique(us.begin(), us.end()), us.end());
    if (us.size() > 4) return plan;
    max_preds = std::max<int>(max_preds, (int)us.size());
    uint32_t o[4] = {2u * N, 2u * N, 2u * N, 2u * N}, dl[4] = {0, 0, 0, 0};
    for (size_t i = 0; i < us.size(); ++i) {
      o[i] = 2u * (uint32_t)us[i];
      dl[i] = pi[us[i]] != pi[v] ? (uint32_t)(d->comm[pi[us[i]] * P + pi[v]] / g) : 0u;
    }
    plan.ops[v] = make_uint4(o[0] | (o[1] << 16), o[2] | (o[3] << 16), dl[0] | (dl[1] << 8) | (dl[2] << 16) | (dl[3] << 24),
                             (uint32_t)(d->dur[v] / g) | ((2u * (uint32_t)v) << 16));
  }
  plan.preds = max_preds <= 2 ? 2 : 4;
  plan.scale = (int)g;
  plan.machine.assign((size_t)(N + 3) / 4 * 4, 0);
  std::vector<int32_t> cnt(Pseg + 1, 0);
  for (int v = 0; v < N; ++v) { plan.machine[v] = (uint8_t)pi[v]; ++cnt[pi[v]]; }
  plan.off.assign(Pseg + 1, N);
  for (int j = 0, at = 0; j <= Pseg; ++j) { plan.off[j] = at; at += j < Pseg ? cnt[j] : 0; }
  if (d->weight) {
    plan.base.assign(P, 0);
    for (int v = 0; v < N; ++v) plan.base[pi[v]] += d->weight[v];
  }
  // LDS: op table, memory adjustments, then per candidate the cells (N + 3, padded) and the list (N + 4 entries), then bookkeeping
  plan.G = kWave / Pseg;
  const uint32_t cells = align_up((uint32_t)((N + 4) / 2) * 4u, 4u), list = (uint32_t)((N + 5) / 2) * 4u;
  plan.o_mem = (uint32_t)N * 16u;
  plan.o_mach = plan.o_mem + (uint32_t)N * 8u;
  plan.o_cand = align_up(plan.o_mach + (uint32_t)(N + 3) / 4u * 4u, 16u);
  plan.o_list = cells;
  plan.cand_stride = align_up(cells + list, 16u);
  const int lds_cu = 160 * 1024;
  int best_w = 0, best_score = -1;
  const int forced_w = d->shape ? d->shape->static_waves : 0;
  for (int w = 1; w <= 8; ++w) {
    if (plan.G * w > kWave) break;                     // 64 flag words per workgroup
    if (forced_w && w != forced_w) continue;
    const uint32_t total = plan.o_cand + (uint32_t)(plan.G * w) * plan.cand_stride + 1024u + 512u * (uint32_t)w;
    if ((int)total > lds_max) break;
    const int wgs = std::min(lds_cu / (int)total, 32 / (static_threads(w) / kWave));
    // a handle for small batches is better off with the ring kernel: one launch instead of three, and workgroups of
    // this size would leave CUs idle (1F1B pipeline, 1024 candidates: 0.012 ms there, 0.015-0.019 ms here)
    if (!forced_w && (int64_t)d->max_candidates < (int64_t)2 * n_cu * std::max(1, wgs) * plan.G * w) continue;
    // one relaxer per SIMD is enough (measured on the zero-bubble pipeline: 1 x 4 relaxers 0.291 ms, 2 x 2 0.301 ms,
    // 1 x 5 0.309 ms, 3 x 1 0.359 ms); among equals the larger workgroup: fewer copies of the tables
    const int relaxers = std::min(wgs * w, 4);
    const int score = relaxers * 8 + w - (wgs * w > 4 ? 4 : 0);
    if (score > best_score) { best_score = score; best_w = w; plan.wgs = std::max(1, wgs); }
  }
  if (!best_w) return plan;
  plan.W = best_w;
  plan.o_book = plan.o_cand + (uint32_t)(plan.G * plan.W) * plan.cand_stride;
  plan.total = plan.o_book + 1024u + 512u * (uint32_t)plan.W;
  plan.ok = true;
  return plan;
}

// A kernel that asks for more than 48 KB of dynamic LDS must be allowed to.  The attribute belongs to the kernel
// function (per device), not to a handle: it is only ever raised, so that a handle made later with a smaller
// footprint never takes away what an earlier handle on the same kernel instantiation needs.
bool allow_large_lds(const void *kernel, int device, int bytes) {
  static std::mutex mu;
  static std::map<std::pair<const void *, int>, int> allowed;
  std::lock_guard<std::mutex> lock(mu);
  int &have = allowed[{kernel, device}];
  if (bytes <= have) return true;
  if (!hip_ok(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes), "hipFuncSetAttribute")) return false;
  have = bytes;
  return true;
}

size_t channel_flag_lds(int32_t n_nodes) {               // mask words + one byte per node
  return (size_t)DAGSCHED_MAX_DEVICES * sizeof(uint64_t) + (size_t)n_nodes;
}

OutPtrs make_out(const dagsched *h, int32_t n_cand, int32_t *makespan, int64_t *bubble, int64_t *peak_mem,
                 int32_t *flags) {
  OutPtrs o;
  o.makespan = makespan; o.bubble = bubble; o.peak_mem = peak_mem; o.flags = flags;
  if (h->layout == DAGSCHED_CAND_MAJOR) { o.peak_stride_c = h->P; o.peak_stride_j = 1; }
  else { o.peak_stride_c = 1; o.peak_stride_j = n_cand; }
  return o;
}

void launch_general(dagsched *h, int32_t n_cand, const int32_t *pl, const int32_t *rk, const OutPtrs &out,
                    const int32_t *cand_list, const int32_t *cand_count, hipStream_t stream) {
  GeneralParams p;
  p.N = h->N; p.P = h->P; p.Pseg = h->Pseg; p.G = h->gen_G; p.C = n_cand;
  p.row_stride = h->row_stride;
  p.pred_ptr = h->d_pred_ptr; p.pred_idx = h->d_pred_idx; p.dur = h->d_dur; p.comm = h->d_comm; p.mem_delta = h->d_mem;
  p.weight = h->d_weight; p.mem_limit = h->d_limit;
  p.sum_dur = h->sum_dur;
  p.placement = pl; p.rank = rk;
  p.ws_list = h->ws_list; p.ws_end = h->ws_end;
  p.cand_list = cand_list; p.cand_count = cand_count;
  p.out = out;
  const unsigned blocks = (unsigned)((n_cand + h->gen_G - 1) / h->gen_G);
  if (h->gen_lds_state)
    hipLaunchKernelGGL(relax_general_kernel<true>, dim3(blocks), dim3(kWave), (size_t)h->gen_lds, stream, p);
  else
    hipLaunchKernelGGL(relax_general_kernel<false>, dim3(blocks), dim3(kWave), 0, stream, p);
}

int launch_evaluate(dagsched *h, int32_t n_cand, const int32_t *placement, const int32_t *rank, int32_t *makespan,
                    int64_t *bubble, int64_t *peak_mem, int32_t *flags, hipStream_t stream) {
  const int32_t N = h->N;
  const int32_t *pl = placement, *rk = rank;
  if (h->layout == DAGSCHED_CAND_MINOR) {
    dim3 grid((unsigned)((n_cand + 63) / 64), (unsigned)((N + 63) / 64));
    hipLaunchKernelGGL(transpose_i32_kernel, grid, dim3(256), 0, stream, placement, h->ws_tp, (int64_t)N, (int64_t)n_cand);
    hipLaunchKernelGGL(transpose_i32_kernel, grid, dim3(256), 0, stream, rank, h->ws_tr, (int64_t)N, (int64_t)n_cand);
    pl = h->ws_tp;
    rk = h->ws_tr;
  }
  const OutPtrs out = make_out(h, n_cand, makespan, bubble, peak_mem, flags);
  if (h->variant == kVariantGeneralLds || h->variant == kVariantGeneralGlobal) {
    launch_general(h, n_cand, pl, rk, out, nullptr, nullptr, stream);
  } else if (h->variant == kVariantStatic) {
    hipLaunchKernelGGL(reset_counter_kernel, dim3(1), dim3(1), 0, stream, h->d_fb_count);
    StaticParams p = h->st;
    p.C = n_cand; p.placement = pl; p.rank = rk; p.out = out;
    const int per_wg = p.G * p.W;
    const unsigned blocks = (unsigned)std::min((n_cand + per_wg - 1) / per_wg, h->st_grid);
    hipLaunchKernelGGL(h->st_preds == 2 ? relax_static_kernel<2> : relax_static_kernel<4>, dim3(blocks),
                       dim3((unsigned)static_threads(p.W)), (size_t)p.total, stream, p);
    launch_general(h, n_cand, pl, rk, out, h->d_fb_list, h->d_fb_count, stream);   // candidates with another placement
  } else {
    const bool optimistic = h->variant == kVariantRingOptimistic;
    if (optimistic) hipLaunchKernelGGL(reset_counter_kernel, dim3(1), dim3(1), 0, stream, h->d_fb_count);
    RingParams p;
    p.N = N; p.P = h->P; p.Pseg = h->Pseg; p.log_pseg = ilog2(h->Pseg); p.G = h->ring_G; p.C = n_cand;
    p.optimistic = optimistic ? 1 : 0;
    p.list_stride = h->list_stride;
    p.rec = h->d_rec; p.rec_plane = h->rec_plane; p.id_bits = h->id_bits; p.nparts = h->d_nparts; p.comm = h->d_comm_scaled; p.mem_delta = h->d_mem;
    p.weight = h->d_weight; p.mem_limit = h->d_limit;
    p.sum_dur = h->sum_dur; p.time_scale = h->time_scale;
    p.placement = pl; p.rank = rk;
    p.ws_list = h->ws_list16; p.ws_pib = h->ws_pib; p.pib_stride = h->pib_stride;
    p.fb_count = h->d_fb_count; p.fb_list = h->d_fb_list;
    p.cand_list = nullptr; p.cand_count = nullptr;
    p.spin_cap = h->spin_cap;
    p.win_magic = h->win_magic; p.ws_meta = h->ws_meta;
    p.out = out;
    const unsigned blocks = (unsigned)((n_cand + h->ring_G - 1) / h->ring_G);
    if (h->lds.win_log2) {                                // window mode: the lists are built by a launch of their own
      p.lds = h->lds_ingest;
      p.lds.win_log2 = h->lds.win_log2;
      hipLaunchKernelGGL(ring_ingest_kernel(h->ring_kind), dim3(blocks), dim3((unsigned)h->ingest_block), (size_t)h->lds_ingest.total,
                         stream, p);
    }
    p.lds = h->lds;
    hipLaunchKernelGGL(ring_kernel_for(h), dim3(blocks), dim3((unsigned)h->ring_block), (size_t)h->lds.total,
                       stream, p);
    if (optimistic && h->fb_G) {
      // what the run above left: the same candidates again with 32-bit end times (exact), straight off the list
      RingParams q = p;
      q.G = h->fb_G; q.optimistic = h->fb_optimistic ? 1 : 0; q.lds = h->fb_lds;
      q.cand_list = h->d_fb_list; q.cand_count = h->d_fb_count;
      q.fb_list = h->d_fb_list + h->max_cand; q.fb_count = h->d_fb_count + 1;   // (what this run leaves in its turn)
      const unsigned blocks2 = (unsigned)((n_cand + h->fb_G - 1) / h->fb_G);   // as if every candidate were on the list
      hipLaunchKernelGGL(fallback_kernel(h), dim3(blocks2), dim3((unsigned)h->fb_block), (size_t)h->fb_lds.total, stream, q);
      if (h->fb_optimistic) launch_general(h, n_cand, pl, rk, out, h->d_fb_list + h->max_cand, h->d_fb_count + 1, stream);
    } else if (optimistic) {
      launch_general(h, n_cand, pl, rk, out, h->d_fb_list, h->d_fb_count, stream);
    }
  }
  // the evaluation ran with delay 0 on pairs without a channel; candidates that use one are flagged now
  if (h->d_no_channel)
    // few candidates: larger workgroups, or the chip's wavefront slots stay empty
    hipLaunchKernelGGL(channel_flag_kernel, dim3((unsigned)n_cand), dim3(n_cand < 2048 ? 1024 : 256), channel_flag_lds(N), stream, N, h->E,
                       h->P, h->d_edges, h->d_no_channel, pl, out);
  if (!hip_ok(hipGetLastError(), "kernel launch")) return DAGSCHED_EHIP;
  return DAGSCHED_OK;
}

int check_evaluate_args(dagsched *h, int32_t n_cand, const void *a, const void *b, const void *c, const void *d,
                        const void *e, const void *f) {
  if (!h || n_cand < 0 || n_cand > h->max_cand) return DAGSCHED_EINVAL;
  if (n_cand > 0 && (!a || !b || !c || !d || !e || !f)) return DAGSCHED_EINVAL;
  return DAGSCHED_OK;
}

}  // namespace

extern "C" {

int dagsched_validate(const dagsched_desc_t *desc) { return validate_desc(desc, nullptr, nullptr, nullptr); }

int dagsched_create(const dagsched_desc_t *caller_desc, dagsched_t **out) {
  if (!out) return DAGSCHED_EINVAL;
  std::vector<int32_t> pred_ptr, pred_idx;
  int64_t sum_dur = 0;
  int rc = validate_desc(caller_desc, &pred_ptr, &pred_idx, &sum_dur);
  if (rc != DAGSCHED_OK) return rc;
  if (caller_desc->contention != 0 && caller_desc->contention != 1) return DAGSCHED_EINVAL;
  if (caller_desc->contention) {                        // a path may pay one transfer per edge of B
    int64_t max_comm = 0;
    for (int a = 0; a < caller_desc->n_devices; ++a)
      for (int b = 0; b < caller_desc->n_devices; ++b)
        if (a != b) max_comm = std::max<int64_t>(max_comm, caller_desc->comm[a * caller_desc->n_devices + b]);
    if (sum_dur + (int64_t)caller_desc->n_edges * max_comm > (int64_t)INT32_MAX) return DAGSCHED_EOVERFLOW;
  }
  // pairs without a channel (eq. (10)) become a bit matrix for the flag pass; the evaluation itself sees delay 0
  dagsched_desc_t cleaned = *caller_desc;
  const dagsched_desc_t *desc = &cleaned;
  std::vector<int32_t> comm_present((size_t)cleaned.n_devices * cleaned.n_devices);
  std::vector<uint64_t> no_channel((size_t)cleaned.n_devices, 0);
  bool any_missing = false;
  for (int a = 0; a < cleaned.n_devices; ++a)
    for (int b = 0; b < cleaned.n_devices; ++b) {
      const int32_t d = caller_desc->comm[a * cleaned.n_devices + b];
      const bool missing = a != b && d == DAGSCHED_NO_CHANNEL;
      if (missing) no_channel[a] |= (uint64_t)1 << b;
      any_missing = any_missing || missing;
      comm_present[(size_t)a * cleaned.n_devices + b] = (a == b || missing) ? 0 : d;
    }
  cleaned.comm = comm_present.data();
  std::vector<uint32_t> edges;                         // node ids fit 16 bits (DAGSCHED_MAX_NODES)
  if (any_missing)
    for (int32_t u = 0; u < cleaned.n_nodes; ++u)
      for (int32_t k = cleaned.row_ptr[u]; k < cleaned.row_ptr[u + 1]; ++k)
        edges.push_back((uint32_t)u | ((uint32_t)cleaned.col_idx[k] << 16));
  int n_dev = 0;
  if (!hip_ok(hipGetDeviceCount(&n_dev), "hipGetDeviceCount")) return DAGSCHED_EHIP;
  if (desc->hip_device < 0 || desc->hip_device >= n_dev) return DAGSCHED_EINVAL;
  if (!hip_ok(hipSetDevice(desc->hip_device), "hipSetDevice")) return DAGSCHED_EHIP;
  if (desc->hip_device < kMaxGpus && !g_scratch[desc->hip_device]) {   // with the handle's device current
    unsigned char *ptr = nullptr;
    if (!hip_ok(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)), "hipGetSymbolAddress") || !ptr) return DAGSCHED_EHIP;
    g_scratch[desc->hip_device] = ptr;
  }
  int lds_max = 0, n_cu = 0;
  if (!hip_ok(hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, desc->hip_device),
              "hipDeviceGetAttribute") ||
      !hip_ok(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, desc->hip_device),
              "hipDeviceGetAttribute"))
    return DAGSCHED_EHIP;
  n_cu = std::max(1, n_cu);

  dagsched *h = new (std::nothrow) dagsched();
  if (!h) return DAGSCHED_ENOMEM;
  h->N = desc->n_nodes; h->E = desc->n_edges; h->P = desc->n_devices;
  h->Pseg = next_pow2(h->P);
  h->max_cand = desc->max_candidates; h->layout = desc->layout; h->device = desc->hip_device;
  h->sum_dur = sum_dur;
  h->row_stride = ((int64_t)h->N + 31) / 32 * 32;     // 128-byte rows: no cache line shared by two candidates
  h->list_stride = ((int64_t)h->N + 63) / 64 * 64;
  h->pib_stride = ((int64_t)h->N + 1 + 127) / 128 * 128;
  const size_t maxc = (size_t)h->max_cand;

  RingPlan plan;
  StaticPlan splan;
  const bool force_general = desc->shape && desc->shape->kernel == 1;
  if (!force_general && desc->shared_placement && !(desc->shape && desc->shape->ignore_shared_placement))
    splan = plan_static(desc, pred_ptr, pred_idx, sum_dur, lds_max, n_cu);
  if (!force_general && !splan.ok) plan = plan_ring(desc, pred_ptr, pred_idx, sum_dur, lds_max, n_cu);
  const bool need_general = splan.ok || !plan.ok || !plan.exact;

  bool ok = upload(&h->d_mem, desc->mem_delta, (size_t)h->N) &&
            (!desc->weight || upload(&h->d_weight, desc->weight, (size_t)h->N)) &&
            (!desc->mem_limit || upload(&h->d_limit, desc->mem_limit, (size_t)h->P));
  // the general kernel's view of the problem is always resident: dagsched_schedule runs it on one candidate
  ok = ok && upload(&h->d_pred_ptr, pred_ptr.data(), (size_t)h->N + 1) &&
       upload(&h->d_pred_idx, pred_idx.data(), (size_t)h->E) &&
       upload(&h->d_dur, desc->dur, (size_t)h->N) &&
       upload(&h->d_comm, desc->comm, (size_t)h->P * h->P) &&
       (!any_missing || (upload(&h->d_no_channel, no_channel.data(), no_channel.size()) &&
                         upload(&h->d_edges, edges.data(), edges.size()) &&
                         (channel_flag_lds(h->N) <= 48 * 1024 ||
                          allow_large_lds((const void *)channel_flag_kernel, h->device, (int)channel_flag_lds(h->N))))) &&
       dev_alloc(&h->ws_cnt, (size_t)DAGSCHED_MAX_DEVICES) &&
       dev_alloc(&h->ws_sched_list, (size_t)h->row_stride) && dev_alloc(&h->ws_sched_end, (size_t)h->row_stride) &&
       dev_alloc(&h->ws_sched_out, (size_t)(32 + 8 * DAGSCHED_MAX_DEVICES));
  if (ok && need_general) {
    h->gen_G = kWave / h->Pseg;
    const int64_t lds_need = (int64_t)h->gen_G * h->N * 4;
    h->gen_lds_state = lds_need + 1024 <= lds_max;
    h->gen_lds = h->gen_lds_state ? (int32_t)lds_need : 0;
    ok = dev_alloc(&h->ws_list, maxc * (size_t)h->row_stride);
    if (ok && !h->gen_lds_state) ok = dev_alloc(&h->ws_end, maxc * (size_t)h->row_stride);
    if (ok && h->gen_lds > 48 * 1024)
      ok = allow_large_lds((const void *)relax_general_kernel<true>, h->device, h->gen_lds);
    h->variant = h->gen_lds_state ? kVariantGeneralLds : kVariantGeneralGlobal;
  }
  if (ok && splan.ok) {
    h->variant = kVariantStatic;
    h->time_scale = splan.scale;
    h->st_preds = splan.preds;
    h->st_grid = n_cu * splan.wgs;
    ok = upload(&h->d_st_ops, splan.ops.data(), splan.ops.size()) &&
         upload(&h->d_st_machine, splan.machine.data(), splan.machine.size()) &&
         upload(&h->d_st_off, splan.off.data(), splan.off.size()) &&
         (splan.base.empty() || upload(&h->d_st_base, splan.base.data(), splan.base.size())) &&
         dev_alloc(&h->d_fb_count, 2) && dev_alloc(&h->d_fb_list, maxc);
    StaticParams &s = h->st;
    s.N = h->N; s.P = h->P; s.Pseg = h->Pseg; s.log_pseg = ilog2(h->Pseg); s.G = splan.G; s.W = splan.W;
    s.ops = h->d_st_ops; s.machine = h->d_st_machine; s.off = h->d_st_off; s.mem_delta = h->d_mem;
    s.base = h->d_st_base; s.mem_limit = h->d_limit;
    s.sum_dur = h->sum_dur; s.time_scale = splan.scale;
    s.fb_count = h->d_fb_count; s.fb_list = h->d_fb_list;
    s.o_mem = splan.o_mem; s.o_mach = splan.o_mach; s.o_cand = splan.o_cand; s.cand_stride = splan.cand_stride; s.o_list = splan.o_list; s.o_book = splan.o_book;
    s.total = splan.total;
    if (ok && s.total > 48 * 1024)
      ok = allow_large_lds(splan.preds == 2 ? (const void *)relax_static_kernel<2> : (const void *)relax_static_kernel<4>, h->device, (int)s.total);
  }
  if (ok && plan.ok) {
    h->variant = !plan.exact ? kVariantRingOptimistic : plan.cell32 ? kVariantRing32 : kVariantRingExact;   // (window mode is never exact)
    h->ring_G = plan.G; h->ring_slots = plan.ring; h->ring_feeders = plan.feeders; h->ring_kind = plan.kind; h->ring_block = plan.block; h->lds = plan.lds; h->time_scale = plan.scale;
    h->rec_plane = plan.rec_plane; h->id_bits = plan.id_bits;
    const int64_t cap = ((int64_t)h->N + h->E + 1024) * 64;
    h->spin_cap = (uint32_t)std::min<int64_t>(cap, 0x7FFFFFFF);
    ok = upload(&h->d_rec, plan.rec.data(), plan.rec.size()) &&
         upload(&h->d_comm_scaled, plan.comm_scaled.data(), plan.comm_scaled.size()) &&
         (plan.nparts.empty() || upload(&h->d_nparts, plan.nparts.data(), plan.nparts.size())) &&
         dev_alloc(&h->ws_list16, maxc * (size_t)h->list_stride) &&
         (plan.lds.pib_mode != 0 || dev_alloc(&h->ws_pib, maxc * (size_t)h->pib_stride));   // only read when the placement is not in LDS
    if (ok && !plan.exact) ok = dev_alloc(&h->d_fb_count, 2) && dev_alloc(&h->d_fb_list, 2 * maxc);   // (two lists)
    if (ok && !plan.exact && !plan.lds.wide) {
      // the candidates a 16-bit or window run leaves behind: 32-bit end times, a cell per operation, where that fits
      dagsched_shape_t fsh{};
      fsh.placement_mode = -1;
      fsh.state_bits = 32;
      fsh.window_cells = -1;
      dagsched_desc_t fd = *desc;
      fd.shape = &fsh;
      const RingPlan fp = plan_ring(&fd, pred_ptr, pred_idx, sum_dur, lds_max, n_cu);
      // (same records, part counts and delays: both plans divide by the same common factor and drop the same edges)
      if (fp.ok && fp.exact && fp.cell32 && !fp.lds.wide && fp.scale == plan.scale && fp.rec_plane == plan.rec_plane &&
          fp.id_bits == plan.id_bits && fp.rec.size() == plan.rec.size()) {
        h->fb_G = fp.G; h->fb_slots = fp.ring; h->fb_feeders = fp.feeders; h->fb_block = fp.block; h->fb_lds = fp.lds; h->fb_kind = fp.kind;
        if (fp.lds.pib_mode == 0 && !h->ws_pib) ok = dev_alloc(&h->ws_pib, maxc * (size_t)h->pib_stride);
        const void *fk = (const void *)ring_kernel_pick<2>(fp.ring, fp.feeders, (int)fp.lds.pib_mode, fp.kind);
        if (!fk) h->fb_G = 0;
        if (ok && fp.lds.total > 48 * 1024) ok = allow_large_lds(fk, h->device, (int)fp.lds.total);
      }
      if (ok && !h->fb_G && plan.win_log2) {
        // too large for that: the misses of the window go to the 16-bit kernel with a cell per operation (its own range
        // stops to a second list and the general kernel)
        fsh.state_bits = 0;
        const RingPlan gp = plan_ring(&fd, pred_ptr, pred_idx, sum_dur, lds_max, n_cu);
        if (gp.ok && !gp.cell32 && !gp.win_log2 && !gp.lds.wide && gp.scale == plan.scale && gp.rec_plane == plan.rec_plane &&
            gp.id_bits == plan.id_bits && gp.rec.size() == plan.rec.size()) {
          h->fb_G = gp.G; h->fb_slots = gp.ring; h->fb_feeders = gp.feeders; h->fb_block = gp.block; h->fb_lds = gp.lds; h->fb_kind = gp.kind;
          h->fb_optimistic = !gp.exact;
          if (gp.lds.pib_mode == 0 && !h->ws_pib) ok = dev_alloc(&h->ws_pib, maxc * (size_t)h->pib_stride);
          const void *gk = (const void *)fallback_kernel(h);
          if (!gk) h->fb_G = 0;
          if (ok && gk && gp.lds.total > 48 * 1024) ok = allow_large_lds(gk, h->device, (int)gp.lds.total);
        }
      }
    }
    if (ok && plan.win_log2) {
      h->lds_ingest = plan.lds_ingest; h->ingest_block = plan.ingest_block; h->win_magic = plan.win_magic;
      ok = dev_alloc(&h->ws_meta, ((maxc + plan.G - 1) / plan.G) * 4 * (size_t)kWave) &&
           (h->lds_ingest.total <= 48 * 1024 || allow_large_lds((const void *)ring_ingest_kernel(plan.kind), h->device, (int)h->lds_ingest.total));
    }
    if (ok && h->lds.total > 48 * 1024)
      ok = allow_large_lds((const void *)ring_kernel_for(h), h->device, (int)h->lds.total);
  }
  if (ok && h->layout == DAGSCHED_CAND_MINOR)
    ok = dev_alloc(&h->ws_tp, maxc * (size_t)h->N) && dev_alloc(&h->ws_tr, maxc * (size_t)h->N);
  if (ok && desc->contention) {
    // the edges by their index in successor-CSR order (the index edge_rank uses), and that index for every in-edge
    const int32_t E = h->E;
    std::vector<int32_t> peid((size_t)std::max(E, 1)), esrc((size_t)std::max(E, 1)), edst((size_t)std::max(E, 1));
    std::vector<int32_t> fill(pred_ptr.begin(), pred_ptr.end() - 1);
    for (int32_t u = 0; u < h->N; ++u)
      for (int32_t k = desc->row_ptr[u]; k < desc->row_ptr[u + 1]; ++k) {
        const int32_t v = desc->col_idx[k];
        peid[fill[v]++] = k; esrc[k] = u; edst[k] = v;
      }
    h->contention = true;
    // as many workgroups as fit the CUs' wavefront slots (32 per CU) and LDS, each with a workspace row of its own
    const int per_cu = std::min(std::min(16, 32 / (contended_threads(h->P) / kWave)), (int)(150 * 1024 / (contended_lds(h->P) + 4096)));
    h->wc_grid = (int32_t)std::min<int64_t>(h->max_cand, (int64_t)n_cu * std::max(1, per_cu));
    h->row_e = ((int64_t)std::max(E, 1) + 31) / 32 * 32;
    h->row_c = ((int64_t)h->P * h->P + 1 + 31) / 32 * 32;
    const size_t g = (size_t)h->wc_grid;
    ok = upload(&h->d_pred_eid, peid.data(), (size_t)E) && upload(&h->d_edge_src, esrc.data(), (size_t)E) &&
         upload(&h->d_edge_dst, edst.data(), (size_t)E) && upload(&h->d_succ_ptr, desc->row_ptr, (size_t)h->N + 1) &&
         dev_alloc(&h->wc_list, g * (size_t)h->row_stride) && dev_alloc(&h->wc_end, g * (size_t)h->row_stride) &&
         dev_alloc(&h->wc_tlist, g * (size_t)h->row_e) && dev_alloc(&h->wc_tend, g * (size_t)h->row_e) &&
         dev_alloc(&h->wc_echan, g * (size_t)h->row_e) &&
         dev_alloc(&h->wc_ccnt, g * (size_t)h->row_c) && dev_alloc(&h->wc_coff, g * (size_t)h->row_c) &&
         (h->layout != DAGSCHED_CAND_MINOR || dev_alloc(&h->ws_te, maxc * (size_t)std::max(E, 1)));
  }
  if (!ok) {
    const bool oom = strstr(g_hip_error, "memory") != nullptr;
    free_handle(h);
    return oom ? DAGSCHED_ENOMEM : DAGSCHED_EHIP;
  }
  *out = h;
  return DAGSCHED_OK;
}

int dagsched_evaluate(dagsched_t *h, int32_t n_cand, const int32_t *placement, const int32_t *rank, int32_t *makespan,
                      int64_t *bubble, int64_t *peak_mem, int32_t *flags, void *hip_stream) {
  int rc = check_evaluate_args(h, n_cand, placement, rank, makespan, bubble, peak_mem, flags);
  if (rc != DAGSCHED_OK || n_cand == 0) return rc;
  return launch_evaluate(h, n_cand, placement, rank, makespan, bubble, peak_mem, flags, (hipStream_t)hip_stream);
}

int dagsched_evaluate_contended(dagsched_t *h, int32_t n_cand, const int32_t *placement, const int32_t *rank,
                                const int32_t *edge_rank, int32_t *makespan, int64_t *bubble, int64_t *peak_mem,
                                int32_t *flags, void *hip_stream) {
  int rc = check_evaluate_args(h, n_cand, placement, rank, makespan, bubble, peak_mem, flags);
  if (rc != DAGSCHED_OK) return rc;
  if (!h->contention || (n_cand > 0 && h->E > 0 && !edge_rank)) return DAGSCHED_EINVAL;
  if (n_cand == 0) return DAGSCHED_OK;
  hipStream_t stream = (hipStream_t)hip_stream;
  const int32_t N = h->N, E = h->E;
  const int32_t *pl = placement, *rk = rank, *er = edge_rank;
  if (h->layout == DAGSCHED_CAND_MINOR) {
    dim3 grid((unsigned)((n_cand + 63) / 64), (unsigned)((N + 63) / 64));
    hipLaunchKernelGGL(transpose_i32_kernel, grid, dim3(256), 0, stream, placement, h->ws_tp, (int64_t)N, (int64_t)n_cand);
    hipLaunchKernelGGL(transpose_i32_kernel, grid, dim3(256), 0, stream, rank, h->ws_tr, (int64_t)N, (int64_t)n_cand);
    pl = h->ws_tp; rk = h->ws_tr;
    if (E > 0) {
      dim3 egrid((unsigned)((n_cand + 63) / 64), (unsigned)((E + 63) / 64));
      hipLaunchKernelGGL(transpose_i32_kernel, egrid, dim3(256), 0, stream, edge_rank, h->ws_te, (int64_t)E, (int64_t)n_cand);
      er = h->ws_te;
    }
  }
  ContendedParams p;
  p.N = N; p.E = E; p.P = h->P; p.C = n_cand;
  p.pred_ptr = h->d_pred_ptr; p.pred_idx = h->d_pred_idx; p.pred_eid = h->d_pred_eid;
  p.edge_src = h->d_edge_src; p.edge_dst = h->d_edge_dst; p.succ_ptr = h->d_succ_ptr;
  p.dur = h->d_dur; p.comm = h->d_comm; p.mem_delta = h->d_mem; p.weight = h->d_weight; p.mem_limit = h->d_limit;
  p.sum_dur = h->sum_dur;
  p.placement = pl; p.rank = rk; p.edge_rank = er;
  p.ws_list = h->wc_list; p.ws_end = h->wc_end; p.ws_tlist = h->wc_tlist; p.ws_tend = h->wc_tend;
  p.ws_ccnt = h->wc_ccnt; p.ws_coff = h->wc_coff; p.ws_echan = h->wc_echan;
  p.row_n = h->row_stride; p.row_e = h->row_e; p.row_c = h->row_c;
  p.out = make_out(h, n_cand, makespan, bubble, peak_mem, flags);
  hipLaunchKernelGGL(relax_contended_kernel, dim3((unsigned)std::min(n_cand, h->wc_grid)), dim3((unsigned)contended_threads(h->P)), contended_lds(h->P), stream, p);
  if (h->d_no_channel)
    hipLaunchKernelGGL(channel_flag_kernel, dim3((unsigned)n_cand), dim3(n_cand < 2048 ? 1024 : 256), channel_flag_lds(N), stream, N, E,
                       h->P, h->d_edges, h->d_no_channel, pl, p.out);
  if (!hip_ok(hipGetLastError(), "kernel launch")) return DAGSCHED_EHIP;
  return DAGSCHED_OK;
}

int dagsched_time_evaluate(dagsched_t *h, int32_t n_cand, const int32_t *placement, const int32_t *rank,
                           int32_t *makespan, int64_t *bubble, int64_t *peak_mem, int32_t *flags, void *hip_stream,
                           int32_t reps, float *ms_per_eval) {
  int rc = check_evaluate_args(h, n_cand, placement, rank, makespan, bubble, peak_mem, flags);
  if (rc != DAGSCHED_OK) return rc;
  if (reps < 1 || !ms_per_eval || n_cand == 0) return DAGSCHED_EINVAL;
  hipStream_t stream = (hipStream_t)hip_stream;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (!hip_ok(hipEventCreate(&e0), "hipEventCreate") || !hip_ok(hipEventCreate(&e1), "hipEventCreate")) {
    if (e0) (void)hipEventDestroy(e0);
    return DAGSCHED_EHIP;
  }
  rc = DAGSCHED_OK;
  if (!hip_ok(hipEventRecord(e0, stream), "hipEventRecord")) rc = DAGSCHED_EHIP;
  for (int i = 0; i < reps && rc == DAGSCHED_OK; ++i)
    rc = launch_evaluate(h, n_cand, placement, rank, makespan, bubble, peak_mem, flags, stream);
  if (rc == DAGSCHED_OK && !hip_ok(hipEventRecord(e1, stream), "hipEventRecord")) rc = DAGSCHED_EHIP;
  if (rc == DAGSCHED_OK && !hip_ok(hipEventSynchronize(e1), "hipEventSynchronize")) rc = DAGSCHED_EHIP;
  float ms = 0.f;
  if (rc == DAGSCHED_OK && !hip_ok(hipEventElapsedTime(&ms, e0, e1), "hipEventElapsedTime")) rc = DAGSCHED_EHIP;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc == DAGSCHED_OK) *ms_per_eval = ms / (float)reps;
  return rc;
}

void dagsched_destroy(dagsched_t *h) {
  if (!h) return;
  (void)hipSetDevice(h->device);
  (void)hipDeviceSynchronize();
  free_handle(h);
}

namespace {
int launch_propose(dagsched_t *h, int32_t n_cand, const int32_t *base_placement, const int32_t *base_rank,
                   const uint32_t *rnd, int32_t *placement, int32_t *rank, void *hip_stream, int orders_only) {
  if (!h || n_cand < 0 || n_cand > h->max_cand) return DAGSCHED_EINVAL;
  if (n_cand == 0) return DAGSCHED_OK;
  if (!base_placement || !base_rank || !rnd || !placement || !rank) return DAGSCHED_EINVAL;
  hipStream_t stream = (hipStream_t)hip_stream;
  hipLaunchKernelGGL(machine_count_kernel, dim3(1), dim3(256), 0, stream, h->N, h->P, base_placement, h->ws_cnt);
  ProposeParams p;
  p.N = h->N; p.P = h->P; p.C = n_cand;
  p.base_pl = base_placement; p.base_rk = base_rank; p.rnd = rnd; p.cnt = h->ws_cnt;
  p.out_pl = placement; p.out_rk = rank; p.orders_only = orders_only;
  if (h->layout == DAGSCHED_CAND_MAJOR) { p.stride_c = h->N; p.stride_n = 1; }
  else { p.stride_c = 1; p.stride_n = n_cand; }
  hipLaunchKernelGGL(propose_kernel, dim3((unsigned)n_cand), dim3(256), 0, stream, p);
  if (!hip_ok(hipGetLastError(), "kernel launch")) return DAGSCHED_EHIP;
  return DAGSCHED_OK;
}

}  // namespace

int dagsched_propose(dagsched_t *h, int32_t n_cand, const int32_t *base_placement, const int32_t *base_rank,
                     const uint32_t *rnd, int32_t *placement, int32_t *rank, void *hip_stream) {
  return launch_propose(h, n_cand, base_placement, base_rank, rnd, placement, rank, hip_stream, 0);
}

int dagsched_propose_orders(dagsched_t *h, int32_t n_cand, const int32_t *base_placement, const int32_t *base_rank,
                            const uint32_t *rnd, int32_t *placement, int32_t *rank, void *hip_stream) {
  return launch_propose(h, n_cand, base_placement, base_rank, rnd, placement, rank, hip_stream, 1);
}

int dagsched_select(dagsched_t *h, int32_t n_cand, const int32_t *makespan, const int32_t *flags, int32_t *best,
                    void *hip_stream) {
  if (!h || n_cand < 0 || !best || (n_cand > 0 && (!makespan || !flags))) return DAGSCHED_EINVAL;
  hipLaunchKernelGGL(select_kernel, dim3(1), dim3(1024), 0, (hipStream_t)hip_stream, n_cand, makespan, flags, best);
  if (!hip_ok(hipGetLastError(), "kernel launch")) return DAGSCHED_EHIP;
  return DAGSCHED_OK;
}

namespace {
// One candidate through the int32 kernel with its order list and end times in the given workspace rows (row_stride
// int32 each; the kernel writes every entry it later reads, so the rows need no clearing), its outputs in `o`
// (32 + 8 * DAGSCHED_MAX_DEVICES bytes), then start = end - duration.
int launch_schedule(dagsched_t *h, int32_t *list_row, int32_t *end_row, unsigned char *o, const int32_t *placement,
                    const int32_t *rank, int32_t *start, int32_t *end, int32_t *flag, hipStream_t stream) {
  GeneralParams p;
  p.N = h->N; p.P = h->P; p.Pseg = h->Pseg; p.G = 1; p.C = 1;
  p.row_stride = h->row_stride;
  p.pred_ptr = h->d_pred_ptr; p.pred_idx = h->d_pred_idx; p.dur = h->d_dur; p.comm = h->d_comm; p.mem_delta = h->d_mem;
  p.weight = h->d_weight; p.mem_limit = h->d_limit;
  p.sum_dur = h->sum_dur;
  p.placement = placement; p.rank = rank;
  p.ws_list = list_row; p.ws_end = end_row;
  p.cand_list = nullptr; p.cand_count = nullptr;
  p.out.makespan = (int32_t *)o; p.out.flags = (int32_t *)(o + 4); p.out.bubble = (int64_t *)(o + 8);
  p.out.peak_mem = (int64_t *)(o + 16); p.out.peak_stride_c = h->P; p.out.peak_stride_j = 1;
  hipLaunchKernelGGL(relax_general_kernel<false>, dim3(1), dim3(kWave), 0, stream, p);
  if (h->d_no_channel)
    hipLaunchKernelGGL(channel_flag_kernel, dim3(1), dim3(1024), channel_flag_lds(h->N), stream, h->N, h->E, h->P,
                       h->d_edges, h->d_no_channel, placement, p.out);
  hipLaunchKernelGGL(schedule_out_kernel, dim3((unsigned)std::min(256, (h->N + 255) / 256)), dim3(256), 0, stream, h->N,
                     h->d_dur, end_row, (const int32_t *)(o + 4), start, end, flag);
  if (!hip_ok(hipGetLastError(), "kernel launch")) return DAGSCHED_EHIP;
  return DAGSCHED_OK;
}
}  // namespace

int dagsched_schedule(dagsched_t *h, const int32_t *placement, const int32_t *rank, int32_t *start, int32_t *end,
                      int32_t *flag, void *hip_stream) {
  if (!h || !placement || !rank || !start || !end || !flag) return DAGSCHED_EINVAL;
  return launch_schedule(h, h->ws_sched_list, h->ws_sched_end, h->ws_sched_out, placement, rank, start, end, flag,
                         (hipStream_t)hip_stream);
}

int dagsched_schedule_static(dagsched_t *h, const int32_t *placement, const int32_t *rank, int32_t *start, int32_t *end,
                             int32_t *flag, void *hip_stream) {
  if (!h || !placement || !rank || !start || !end || !flag) return DAGSCHED_EINVAL;
  if (h->N > kStaticMaxNodes) return DAGSCHED_ESCRATCH;
  unsigned char *ptr = h->device < kMaxGpus ? g_scratch[h->device] : nullptr;
  if (!ptr) return DAGSCHED_EHIP;                          // (dagsched_create resolves it; a handle implies it is there)
  // rows of row_stride <= kStaticMaxNodes entries each (N rounded up to 32, and kStaticMaxNodes is a multiple of 32)
  int32_t *list_row = (int32_t *)ptr, *end_row = list_row + kStaticMaxNodes;
  return launch_schedule(h, list_row, end_row, ptr + kScratchOut, placement, rank, start, end, flag, (hipStream_t)hip_stream);
}

int dagsched_coarsen(int32_t n_nodes, int32_t n_edges, const int32_t *row_ptr, const int32_t *col_idx,
                     const int32_t *dur, const int64_t *mem_delta, const int64_t *mem_req,
                     const dagsched_coarsen_params_t *params, int32_t hip_device, int32_t *node_map,
                     int32_t *c_row_ptr, int32_t *c_col_idx, int32_t *c_dur, int64_t *c_mem_delta,
                     int64_t *c_mem_req, dagsched_coarsen_result_t *result) {
  const int32_t n = n_nodes, E = n_edges;
  if (n < 1 || n > DAGSCHED_MAX_NODES || E < 0 || !row_ptr || !dur || !mem_delta || (E > 0 && !col_idx)) return DAGSCHED_EINVAL;
  if (!params || params->target_nodes < 1 || !node_map || !c_row_ptr || (E > 0 && !c_col_idx) || !c_dur || !c_mem_delta ||
      !c_mem_req || !result)
    return DAGSCHED_EINVAL;
  if (row_ptr[0] != 0 || row_ptr[n] != E) return DAGSCHED_EINVAL;
  // the graph: CSR shape, no self-loops, acyclic (sources peeled until none is left)
  std::vector<int32_t> indeg(n, 0), stack;
  for (int32_t u = 0; u < n; ++u) {
    if (row_ptr[u + 1] < row_ptr[u]) return DAGSCHED_EINVAL;
    for (int32_t k = row_ptr[u]; k < row_ptr[u + 1]; ++k) {
      const int32_t v = col_idx[k];
      if (v < 0 || v >= n || v == u) return DAGSCHED_EINVAL;
      ++indeg[v];
    }
  }
  int64_t sum_dur = 0;
  for (int32_t v = 0; v < n; ++v) {
    if (dur[v] < 0 || (mem_req && mem_req[v] < 0)) return DAGSCHED_EINVAL;
    sum_dur += dur[v];
  }
  for (int32_t v = 0; v < n; ++v)
    if (indeg[v] == 0) stack.push_back(v);
  int32_t peeled = 0;
  while (!stack.empty()) {
    const int32_t u = stack.back();
    stack.pop_back();
    ++peeled;
    for (int32_t k = row_ptr[u]; k < row_ptr[u + 1]; ++k)
      if (--indeg[col_idx[k]] == 0) stack.push_back(col_idx[k]);
  }
  if (peeled != n) return DAGSCHED_ECYCLE;
  if (sum_dur > (int64_t)INT32_MAX) return DAGSCHED_EOVERFLOW;   // a group's duration is a sum of durations

  int n_dev = 0;
  if (!hip_ok(hipGetDeviceCount(&n_dev), "hipGetDeviceCount")) return DAGSCHED_EHIP;
  if (hip_device < 0 || hip_device >= n_dev) return DAGSCHED_EINVAL;
  if (!hip_ok(hipSetDevice(hip_device), "hipSetDevice")) return DAGSCHED_EHIP;

  CoarsenParams p{};
  p.n = n; p.n_edges = E; p.words = (n + 63) / 64; p.target = params->target_nodes;
  p.edge_dur_max = params->edge_dur_max; p.edge_mem_max = params->edge_mem_max;
  p.nonedge_dur_max = params->nonedge_dur_max; p.nonedge_mem_max = params->nonedge_mem_max;
  std::vector<int64_t> dur64(dur, dur + n), req64(n, 0);
  if (mem_req) req64.assign(mem_req, mem_req + n);
  const size_t matrix = (size_t)n * (size_t)p.words;
  std::vector<void *> owned;
  auto alloc = [&](auto **dst, size_t count) {
    if (!dev_alloc(dst, count)) return false;
    owned.push_back((void *)*dst);
    return true;
  };
  int32_t *d_row_ptr = nullptr, *d_col_idx = nullptr;
  bool ok = alloc(&d_row_ptr, (size_t)n + 1) && alloc(&d_col_idx, (size_t)E) && alloc(&p.succ, matrix) && alloc(&p.pred, matrix) && alloc(&p.kept, matrix) &&
            alloc(&p.dur, (size_t)n) && alloc(&p.mem, (size_t)n) && alloc(&p.req, (size_t)n) && alloc(&p.alive, (size_t)n) &&
            alloc(&p.parent, (size_t)n) && alloc(&p.outdeg, (size_t)n) && alloc(&p.indeg, (size_t)n) && alloc(&p.only, (size_t)n) &&
            alloc(&p.depth, (size_t)n) && alloc(&p.left, (size_t)n) && alloc(&p.index_of, (size_t)n) && alloc(&p.node_map, (size_t)n) &&
            alloc(&p.c_row_ptr, (size_t)n + 1) && alloc(&p.c_col_idx, (size_t)E) && alloc(&p.c_dur, (size_t)n) &&
            alloc(&p.c_mem, (size_t)n) && alloc(&p.c_req, (size_t)n) && alloc(&p.counts, 3);
  p.row_ptr = d_row_ptr; p.col_idx = d_col_idx;
  auto h2d = [&](void *dst, const void *src, size_t bytes) {
    return bytes == 0 || hip_ok(hipMemcpy(dst, src, bytes, hipMemcpyHostToDevice), "hipMemcpy");
  };
  ok = ok && h2d(d_row_ptr, row_ptr, sizeof(int32_t) * ((size_t)n + 1)) && h2d(d_col_idx, col_idx, sizeof(int32_t) * (size_t)E) &&
       h2d(p.dur, dur64.data(), sizeof(int64_t) * (size_t)n) && h2d(p.mem, mem_delta, sizeof(int64_t) * (size_t)n) &&
       h2d(p.req, req64.data(), sizeof(int64_t) * (size_t)n) &&
       hip_ok(hipMemset(p.succ, 0, matrix * sizeof(unsigned long long)), "hipMemset") &&
       hip_ok(hipMemset(p.pred, 0, matrix * sizeof(unsigned long long)), "hipMemset") &&
       hip_ok(hipMemset(p.kept, 0, matrix * sizeof(unsigned long long)), "hipMemset");
  int32_t counts[3] = {0, 0, 0};
  std::vector<int64_t> out_dur(n);
  if (ok) {
    hipLaunchKernelGGL(coarsen_kernel, dim3(1), dim3(1024), 0, (hipStream_t)nullptr, p);
    ok = hip_ok(hipGetLastError(), "kernel launch") && hip_ok(hipDeviceSynchronize(), "hipDeviceSynchronize");
  }
  auto d2h = [&](void *dst, const void *src, size_t bytes) {
    return bytes == 0 || hip_ok(hipMemcpy(dst, src, bytes, hipMemcpyDeviceToHost), "hipMemcpy");
  };
  ok = ok && d2h(counts, p.counts, sizeof(counts));
  const size_t k = ok ? (size_t)counts[0] : 0;
  int32_t coarse_edges = 0;
  ok = ok && d2h(node_map, p.node_map, sizeof(int32_t) * (size_t)n) && d2h(c_row_ptr, p.c_row_ptr, sizeof(int32_t) * (k + 1));
  if (ok) coarse_edges = c_row_ptr[k];
  ok = ok && d2h(c_col_idx, p.c_col_idx, sizeof(int32_t) * (size_t)coarse_edges) && d2h(out_dur.data(), p.c_dur, sizeof(int64_t) * k) &&
       d2h(c_mem_delta, p.c_mem, sizeof(int64_t) * k) && d2h(c_mem_req, p.c_req, sizeof(int64_t) * k);
  const bool oom = !ok && strstr(g_hip_error, "memory") != nullptr;
  for (void *b : owned) (void)hipFree(b);
  if (!ok) return oom ? DAGSCHED_ENOMEM : DAGSCHED_EHIP;
  for (size_t i = 0; i < k; ++i) c_dur[i] = (int32_t)out_dur[i];
  result->n_coarse = counts[0]; result->n_coarse_edges = coarse_edges;
  result->merges_edge = counts[1]; result->merges_nonedge = counts[2];
  return DAGSCHED_OK;
}

int dagsched_plan(const dagsched_desc_t *caller_desc, int32_t lds_bytes, int32_t n_cu, dagsched_info_t *info) {
  if (!info || lds_bytes < 1024 || n_cu < 1) return DAGSCHED_EINVAL;
  std::vector<int32_t> pred_ptr, pred_idx;
  int64_t sum_dur = 0;
  const int rc = validate_desc(caller_desc, &pred_ptr, &pred_idx, &sum_dur);
  if (rc != DAGSCHED_OK) return rc;
  // what dagsched_create does with the description, without the uploads: missing channels evaluate as delay 0
  dagsched_desc_t cleaned = *caller_desc;
  const int P = cleaned.n_devices;
  std::vector<int32_t> comm_present((size_t)P * P);
  for (int a = 0; a < P; ++a)
    for (int b = 0; b < P; ++b) {
      const int32_t d = caller_desc->comm[a * P + b];
      comm_present[(size_t)a * P + b] = (a == b || d == DAGSCHED_NO_CHANNEL) ? 0 : d;
    }
  cleaned.comm = comm_present.data();
  dagsched h;
  h.N = cleaned.n_nodes; h.E = cleaned.n_edges; h.P = P; h.Pseg = next_pow2(P);
  const bool force_general = cleaned.shape && cleaned.shape->kernel == 1;
  RingPlan plan;
  StaticPlan splan;
  if (!force_general && cleaned.shared_placement && !(cleaned.shape && cleaned.shape->ignore_shared_placement))
    splan = plan_static(&cleaned, pred_ptr, pred_idx, sum_dur, lds_bytes, n_cu);
  if (!force_general && !splan.ok) plan = plan_ring(&cleaned, pred_ptr, pred_idx, sum_dur, lds_bytes, n_cu);
  if (splan.ok || !plan.ok || !plan.exact) {
    h.gen_G = kWave / h.Pseg;
    const int64_t lds_need = (int64_t)h.gen_G * h.N * 4;
    h.gen_lds_state = lds_need + 1024 <= lds_bytes;
    h.gen_lds = h.gen_lds_state ? (int32_t)lds_need : 0;
    h.variant = h.gen_lds_state ? kVariantGeneralLds : kVariantGeneralGlobal;
  }
  if (splan.ok) {
    h.variant = kVariantStatic;
    h.time_scale = splan.scale; h.st_preds = splan.preds;
    h.st.G = splan.G; h.st.W = splan.W; h.st.total = splan.total;
  }
  if (plan.ok) {
    h.variant = !plan.exact ? kVariantRingOptimistic : plan.cell32 ? kVariantRing32 : kVariantRingExact;
    h.ring_G = plan.G; h.ring_slots = plan.ring; h.ring_feeders = plan.feeders; h.ring_kind = plan.kind; h.ring_block = plan.block;
    h.lds = plan.lds; h.time_scale = plan.scale;
  }
  return dagsched_get_info(&h, info);
}

int dagsched_get_info(const dagsched_t *h, dagsched_info_t *info) {
  if (!h || !info) return DAGSCHED_EINVAL;
  memset(info, 0, sizeof(*info));
  info->variant = h->variant;
  const bool ring = h->variant == kVariantRingExact || h->variant == kVariantRingOptimistic || h->variant == kVariantRing32;
  info->cand_per_block = ring ? h->ring_G : h->gen_G;
  info->block_threads = ring ? h->ring_block : kWave;
  info->lds_bytes = ring ? (int32_t)h->lds.total : h->gen_lds;
  info->state_bits = ring && h->lds.cell_bytes != 4 ? 16 : 32;
  if (h->variant == kVariantStatic) {
    info->cand_per_block = h->st.G * h->st.W;
    info->block_threads = static_threads(h->st.W);
    info->lds_bytes = (int32_t)h->st.total;
    info->state_bits = 16;
    info->time_scale = h->time_scale;
    info->preds_per_op = (int8_t)h->st_preds;
    return DAGSCHED_OK;
  }
  info->time_scale = h->time_scale;
  if (ring) {
    info->ring_slots = (int16_t)h->ring_slots;
    info->feeders = (int8_t)h->ring_feeders;
    info->placement_mode = (int8_t)h->lds.pib_mode;
    info->preds_per_op = (int8_t)(h->ring_kind == 3 ? 1 : h->ring_kind == 2 ? 2 : 4);
    info->kernel_kind = (int8_t)h->ring_kind;
    info->wide_ops = (int8_t)h->lds.wide;
    info->window_log2 = (int8_t)h->lds.win_log2;
  }
  return DAGSCHED_OK;
}

int dagsched_last_fallbacks(dagsched_t *h, void *hip_stream, int32_t *count) {
  if (!h || !count) return DAGSCHED_EINVAL;
  *count = 0;
  const bool has_list = h->d_fb_count && (h->variant == kVariantRingOptimistic || h->variant == kVariantStatic);
  if (!has_list) return DAGSCHED_OK;
  if (!hip_ok(hipMemcpyAsync(count, h->d_fb_count, sizeof(int32_t), hipMemcpyDeviceToHost, (hipStream_t)hip_stream),
              "hipMemcpyAsync") ||
      !hip_ok(hipStreamSynchronize((hipStream_t)hip_stream), "hipStreamSynchronize"))
    return DAGSCHED_EHIP;
  return DAGSCHED_OK;
}

const char *dagsched_strerror(int code) {
  static thread_local char buf[320];
  switch (code) {
    case DAGSCHED_OK: return "ok";
    case DAGSCHED_EINVAL: return "invalid argument";
    case DAGSCHED_ECYCLE: return "the operator graph is cyclic";
    case DAGSCHED_EOVERFLOW: return "sum(dur) + (N-1)*max(comm) exceeds INT32_MAX";
    case DAGSCHED_ENOMEM: return "out of memory";
    case DAGSCHED_ESCRATCH: return "the problem has more operations than the static scratch of the allocation-free entry point holds";
    case DAGSCHED_EHIP:
      snprintf(buf, sizeof(buf), "HIP runtime failure (%s)", g_hip_error[0] ? g_hip_error : "no detail recorded");
      return buf;
    default: return "unknown error code";
  }
}

}  // extern "C"
