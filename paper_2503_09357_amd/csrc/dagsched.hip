// dagsched: batched evaluation of candidate operator schedules on gfx950 (MI355X).
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
// lanes of a candidate sit in one 64-wide wavefront (P <= 64), so "no lane of the candidate advanced
// in a round" (a ballot) is an exact deadlock test, i.e. a cycle of the combined graph.
//
// No MFMA anywhere: the work is integer max/plus with data-dependent gathers, not a contraction.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "dagsched.h"

namespace {

constexpr int kWave = 64;
constexpr int kFlagCyclicBit = 1, kFlagBadPlacementBit = 2, kFlagBadRankBit = 4;

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

// ------------------------------------------------------------------------------------------------
// device helpers

// Loads/stores that must observe data written earlier in the same kernel by other lanes go to L2
// (agent scope) so that a stale line in the per-CU vector cache can never be returned.
__device__ __forceinline__ int32_t ld_agent(const int32_t *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(int32_t *p, int32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

struct GeneralParams {
  int32_t N, P, Pseg, G, C;
  int64_t row_stride;          // elements between consecutive candidates in list / end workspaces
  const int32_t *pred_ptr;     // [N+1] predecessor CSR of B
  const int32_t *pred_idx;     // [E]
  const int32_t *dur;          // [N]
  const int32_t *comm;         // [P*P]
  const int64_t *mem_delta;    // [N]
  int64_t sum_dur;
  const int32_t *placement;    // [C][N] candidate-major
  const int32_t *rank;         // [C][N]
  int32_t *ws_list;            // [C][row_stride] order lists, machine after machine
  int32_t *ws_end;             // [C][row_stride] end times (global-state variant)
  int32_t *makespan;
  int64_t *bubble;
  int64_t *peak_mem;
  int32_t *flags;
  int64_t peak_stride_c, peak_stride_j;   // peak_mem[c*peak_stride_c + j*peak_stride_j]
};

// ------------------------------------------------------------------------------------------------
// General kernel: any N, any time range (int32 end times), state in LDS when it fits, else in a
// global workspace.  One wavefront per workgroup, G = 64 / Pseg candidates per wavefront.
// Edge-granular polling: per round a lane consumes at most one DAG predecessor of its head
// operation and completes the operation once all of them have ended.
template <bool LDS_STATE>
__global__ __launch_bounds__(kWave) void relax_general_kernel(GeneralParams p) {
  extern __shared__ int32_t smem[];
  __shared__ int32_t s_cnt[kWave];
  __shared__ int32_t s_off[kWave];
  __shared__ int32_t s_flag[kWave];

  const int lane = threadIdx.x;
  const int N = p.N, P = p.P, Pseg = p.Pseg, G = p.G;
  const int64_t c0 = (int64_t)blockIdx.x * G;
  const int ng = (int)min((int64_t)G, (int64_t)p.C - c0);
  const int g = lane / Pseg, j = lane % Pseg;

  s_cnt[lane] = 0;
  s_flag[lane] = 0;
  __syncthreads();

  // a1: placement in range (eq. (6)); count operations per machine; reset the end-time state
  for (int gg = 0; gg < ng; ++gg) {
    const int32_t *pl = p.placement + (c0 + gg) * N;
    int32_t *end_g = LDS_STATE ? (smem + (size_t)gg * N) : (p.ws_end + (c0 + gg) * p.row_stride);
    for (int v = lane; v < N; v += kWave) {
      int32_t pi = pl[v];
      if ((uint32_t)pi >= (uint32_t)P) atomicOr(&s_flag[gg], kFlagBadPlacementBit);
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
  // a2: order lists list_j[rank] = operation (the fixed disjunctive arcs u of eqs. (7),(17)-(18))
  for (int gg = 0; gg < ng; ++gg) {
    if (s_flag[gg] & kFlagBadPlacementBit) continue;
    const int32_t *pl = p.placement + (c0 + gg) * N;
    const int32_t *rk = p.rank + (c0 + gg) * N;
    int32_t *list = p.ws_list + (c0 + gg) * p.row_stride;
    for (int v = lane; v < N; v += kWave) {
      int32_t pi = pl[v], r = rk[v];
      if ((uint32_t)r >= (uint32_t)s_cnt[gg * Pseg + pi]) atomicOr(&s_flag[gg], kFlagBadRankBit);
      else st_agent(list + s_off[gg * Pseg + pi] + r, v);
    }
  }
  __threadfence();
  __syncthreads();
  // every (machine, rank) slot must be hit exactly once: a slot written twice keeps one writer only
  for (int gg = 0; gg < ng; ++gg) {
    if (s_flag[gg]) continue;
    const int32_t *pl = p.placement + (c0 + gg) * N;
    const int32_t *rk = p.rank + (c0 + gg) * N;
    const int32_t *list = p.ws_list + (c0 + gg) * p.row_stride;
    for (int v = lane; v < N; v += kWave) {
      if (ld_agent(list + s_off[gg * Pseg + pl[v]] + rk[v]) != v) atomicOr(&s_flag[gg], kFlagBadRankBit);
    }
  }
  __syncthreads();

  // a3/a4/a7: relaxation, lane = (candidate g, machine j)
  const bool lane_valid = (g < ng) && (j < P);
  const int64_t c = c0 + g;
  const int32_t *pl = p.placement + (lane_valid ? c : 0) * N;
  const int32_t *list = p.ws_list + (lane_valid ? c : 0) * p.row_stride;
  int32_t *end_g = LDS_STATE ? (smem + (size_t)(lane_valid ? g : 0) * N)
                             : (p.ws_end + (lane_valid ? c : 0) * p.row_stride);
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
  int64_t level = 0, peak = 0;  // running memory level on machine j and its maximum
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
    if (!LDS_STATE) __threadfence();
    __syncthreads();
    const uint64_t bal_prog = __ballot(progressed);
    if (active && (bal_prog & segmask) == 0) {
      // nothing of this candidate moved although operations remain: the combined graph is cyclic
      s_flag[g] = kFlagCyclicBit;
      active = false;
    }
    if (__ballot(active) == 0) break;
  }
  __syncthreads();

  // a5/a6/a8: reductions and outputs
  int32_t z = acc;
  for (int d = 1; d < Pseg; d <<= 1) z = max(z, __shfl_xor(z, d, Pseg));
  if (lane_valid) {
    const int bits = s_flag[g];
    const int flag = (bits & kFlagBadPlacementBit) ? DAGSCHED_FLAG_BAD_PLACEMENT
                   : (bits & kFlagBadRankBit)      ? DAGSCHED_FLAG_BAD_RANK
                   : (bits & kFlagCyclicBit)       ? DAGSCHED_FLAG_CYCLIC
                                                   : DAGSCHED_FLAG_OK;
    p.peak_mem[c * p.peak_stride_c + j * p.peak_stride_j] = flag ? -1 : peak;
    if (j == 0) {
      p.makespan[c] = flag ? -1 : z;
      p.bubble[c] = flag ? -1 : (int64_t)P * z - p.sum_dur;
      p.flags[c] = flag;
    }
  }
}

// [rows][cols] int32 -> [cols][rows], 64x64 tiles through LDS (both sides coalesced)
__global__ __launch_bounds__(256) void transpose_i32_kernel(const int32_t *__restrict__ in, int32_t *__restrict__ out,
                                                             int64_t rows, int64_t cols) {
  __shared__ int32_t tile[64][65];
  const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4) {
    int64_t r = r0 + i, cc = c0 + tx;
    if (r < rows && cc < cols) tile[i][tx] = in[r * cols + cc];
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    int64_t cc = c0 + i, r = r0 + tx;
    if (r < rows && cc < cols) out[cc * rows + r] = tile[tx][i];
  }
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// host side

struct dagsched {
  int32_t N = 0, E = 0, P = 0, Pseg = 0, G = 0, max_cand = 0, layout = 0, device = 0;
  int64_t sum_dur = 0, row_stride = 0;
  int32_t variant = 0, lds_bytes = 0, state_bits = 32, block_threads = kWave;
  int32_t *d_pred_ptr = nullptr, *d_pred_idx = nullptr, *d_dur = nullptr, *d_comm = nullptr;
  int64_t *d_mem = nullptr;
  int32_t *ws_list = nullptr, *ws_end = nullptr, *ws_tp = nullptr, *ws_tr = nullptr;
};

namespace {

enum { kVariantGeneralLds = 1, kVariantGeneralGlobal = 2 };

int validate_desc(const dagsched_desc_t *d, std::vector<int32_t> *pred_ptr, std::vector<int32_t> *pred_idx,
                  int64_t *sum_dur_out) {
  if (!d) return DAGSCHED_EINVAL;
  const int32_t N = d->n_nodes, E = d->n_edges, P = d->n_devices;
  if (N < 1 || N > DAGSCHED_MAX_NODES || E < 0 || P < 1 || P > DAGSCHED_MAX_DEVICES) return DAGSCHED_EINVAL;
  if (!d->row_ptr || !d->dur || !d->comm || !d->mem_delta || (E > 0 && !d->col_idx)) return DAGSCHED_EINVAL;
  if (d->max_candidates < 1) return DAGSCHED_EINVAL;
  if (d->layout != DAGSCHED_CAND_MAJOR && d->layout != DAGSCHED_CAND_MINOR) return DAGSCHED_EINVAL;
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
  for (int32_t a = 0; a < P; ++a)
    for (int32_t b = 0; b < P; ++b)
      if (a != b) {
        if (d->comm[a * P + b] < 0) return DAGSCHED_EINVAL;
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

void free_handle(dagsched *h) {
  if (!h) return;
  void *bufs[] = {h->d_pred_ptr, h->d_pred_idx, h->d_dur, h->d_comm, h->d_mem, h->ws_list, h->ws_end, h->ws_tp, h->ws_tr};
  for (void *b : bufs)
    if (b) (void)hipFree(b);
  delete h;
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
  GeneralParams p;
  p.N = N; p.P = h->P; p.Pseg = h->Pseg; p.G = h->G; p.C = n_cand;
  p.row_stride = h->row_stride;
  p.pred_ptr = h->d_pred_ptr; p.pred_idx = h->d_pred_idx; p.dur = h->d_dur; p.comm = h->d_comm; p.mem_delta = h->d_mem;
  p.sum_dur = h->sum_dur;
  p.placement = pl; p.rank = rk;
  p.ws_list = h->ws_list; p.ws_end = h->ws_end;
  p.makespan = makespan; p.bubble = bubble; p.peak_mem = peak_mem; p.flags = flags;
  if (h->layout == DAGSCHED_CAND_MAJOR) { p.peak_stride_c = h->P; p.peak_stride_j = 1; }
  else { p.peak_stride_c = 1; p.peak_stride_j = n_cand; }
  const unsigned blocks = (unsigned)((n_cand + h->G - 1) / h->G);
  if (h->variant == kVariantGeneralLds)
    hipLaunchKernelGGL(relax_general_kernel<true>, dim3(blocks), dim3(kWave), (size_t)h->lds_bytes, stream, p);
  else
    hipLaunchKernelGGL(relax_general_kernel<false>, dim3(blocks), dim3(kWave), 0, stream, p);
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

int dagsched_create(const dagsched_desc_t *desc, dagsched_t **out) {
  if (!out) return DAGSCHED_EINVAL;
  std::vector<int32_t> pred_ptr, pred_idx;
  int64_t sum_dur = 0;
  int rc = validate_desc(desc, &pred_ptr, &pred_idx, &sum_dur);
  if (rc != DAGSCHED_OK) return rc;
  int n_dev = 0;
  if (!hip_ok(hipGetDeviceCount(&n_dev), "hipGetDeviceCount")) return DAGSCHED_EHIP;
  if (desc->hip_device < 0 || desc->hip_device >= n_dev) return DAGSCHED_EINVAL;
  if (!hip_ok(hipSetDevice(desc->hip_device), "hipSetDevice")) return DAGSCHED_EHIP;

  dagsched *h = new (std::nothrow) dagsched();
  if (!h) return DAGSCHED_ENOMEM;
  h->N = desc->n_nodes; h->E = desc->n_edges; h->P = desc->n_devices;
  h->Pseg = next_pow2(h->P);
  h->G = kWave / h->Pseg;
  h->max_cand = desc->max_candidates; h->layout = desc->layout; h->device = desc->hip_device;
  h->sum_dur = sum_dur;
  h->row_stride = ((int64_t)h->N + 31) / 32 * 32;     // 128-byte rows: no cache line shared by two candidates

  int lds_max = 0;
  if (!hip_ok(hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, h->device), "hipDeviceGetAttribute")) {
    delete h;
    return DAGSCHED_EHIP;
  }
  const int64_t lds_need = (int64_t)h->G * h->N * 4;
  if (lds_need + 1024 <= lds_max) { h->variant = kVariantGeneralLds; h->lds_bytes = (int32_t)lds_need; }
  else { h->variant = kVariantGeneralGlobal; h->lds_bytes = 0; }

  const size_t ws = (size_t)h->max_cand * (size_t)h->row_stride;
  bool ok = upload(&h->d_pred_ptr, pred_ptr.data(), (size_t)h->N + 1) &&
            upload(&h->d_pred_idx, pred_idx.data(), (size_t)h->E) &&
            upload(&h->d_dur, desc->dur, (size_t)h->N) &&
            upload(&h->d_comm, desc->comm, (size_t)h->P * h->P) &&
            upload(&h->d_mem, desc->mem_delta, (size_t)h->N) &&
            hip_ok(hipMalloc((void **)&h->ws_list, ws * sizeof(int32_t)), "hipMalloc workspace");
  if (ok && h->variant == kVariantGeneralGlobal)
    ok = hip_ok(hipMalloc((void **)&h->ws_end, ws * sizeof(int32_t)), "hipMalloc workspace");
  if (ok && h->layout == DAGSCHED_CAND_MINOR)
    ok = hip_ok(hipMalloc((void **)&h->ws_tp, (size_t)h->max_cand * h->N * sizeof(int32_t)), "hipMalloc workspace") &&
         hip_ok(hipMalloc((void **)&h->ws_tr, (size_t)h->max_cand * h->N * sizeof(int32_t)), "hipMalloc workspace");
  if (ok && h->variant == kVariantGeneralLds && h->lds_bytes > 48 * 1024)
    ok = hip_ok(hipFuncSetAttribute((const void *)relax_general_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    h->lds_bytes), "hipFuncSetAttribute");
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

int dagsched_get_info(const dagsched_t *h, dagsched_info_t *info) {
  if (!h || !info) return DAGSCHED_EINVAL;
  memset(info, 0, sizeof(*info));
  info->variant = h->variant;
  info->cand_per_block = h->G;
  info->block_threads = h->block_threads;
  info->lds_bytes = h->lds_bytes;
  info->state_bits = h->state_bits;
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
    case DAGSCHED_EHIP:
      snprintf(buf, sizeof(buf), "HIP runtime failure (%s)", g_hip_error[0] ? g_hip_error : "no detail recorded");
      return buf;
    default: return "unknown error code";
  }
}

}  // extern "C"
