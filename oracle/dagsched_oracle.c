/*
 * CPU oracle for batched evaluation of candidate operator schedules.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, serial, slow and meant to be checked against the paper by
 * eye.  It shares no code with the HIP library and must never be called from the product path;
 * only the tests, the smoke check and the benchmark's CPU-baseline leg load it.
 *
 * What it computes (Sec. III of arxiv 2503.09357).  A candidate fixes every binary of the MIP:
 * the allocation x (eq. (6)) as placement[i], and the per-machine total orders y (eqs. (7)-(8))
 * together with the immediate-precedence variables u (used by eqs. (17)-(18)) as dense ranks:
 * on machine j the ranks are exactly 0..n_j-1.  With the binaries fixed, eqs. (2), (3), (5), (7)
 * and (11)-(13) are difference constraints  s_v >= e_u + const  on the disjunctive graph
 * (operator DAG edges B plus one chain edge between consecutive operations of a machine), and
 * the optimum of eq. (1) is the longest path: the earliest-start schedule
 *
 *     s_v = max( 0,                                   all machines free at t = 0 (assumption 1)
 *                e_u               (u,v) chain edge,  one op per machine at a time (eq. (7))
 *                e_u + delta(u,v)  (u,v) in B  )      eqs. (13),(11),(12): c >= e_u, d >= c + D^c, s_v >= d
 *     e_v = s_v + D^o_v                               eq. (3), non-preemptive (assumption 3)
 *
 * with delta(u,v) = comm[placement[u]][placement[v]] when the two machines differ and 0 when they
 * coincide (machine-dimension form of D^c, footnote of Sec. III; co-located operations exchange
 * no message).  Results per candidate:
 *
 *     makespan  z = max_v e_v                                           eqs. (1)-(2)
 *     bubble      = P * z - sum_v D^o_v    idle time of all P machines inside [0, z]
 *     peak_mem[j] = max(0, max_k sum_{t<k} A_{list_j[t]})               eqs. (17)-(19): m+ = m- + A,
 *                   the level after an operation is the level before the next one on that machine;
 *                   the level starts at 0 and 0 takes part in the maximum
 *     flags       = 2 BAD_PLACEMENT | 4 BAD_RANK | 32 NO_CHANNEL | 1 CYCLIC | 16 OVER_MEMORY | 0 (exactly
 *                   one value, tested in that order); flagged candidates return -1 in every other output.
 *
 * Missing channels (eqs. (9)-(10)): an off-diagonal comm entry of -1 says that the cluster graph has
 * no channel from the row's machine to the column's.  z = x * x of eq. (9) is then forced to 0 by
 * eq. (10): a candidate that places the two ends of some edge of B on such a pair (in that
 * direction) violates it and is flagged NO_CHANNEL.  Machines talk to themselves without a channel
 * (the diagonal is never read).
 *
 * Optional static memory (eq. (16)): with weights W_i >= 0 the level of machine j starts at
 * base_j = sum of W_i over the operations placed on j (the least m- that eq. (16) allows for the
 * machine's first operation), so peak_mem[j] = base_j + max(0, max_k sum_{t<k} A).  With limits
 * M_j (the memory limit of a machine, Sec. III problem statement; the paper prints no inequality
 * for it) a candidate that is otherwise feasible and has peak_mem[j] > M_j for some j is flagged
 * OVER_MEMORY.
 *
 * A candidate is CYCLIC when DAG edges and chain edges together contain a directed cycle
 * (eqs. (5), (7), (8) cannot hold together).  The test is structural (Kahn's algorithm pops
 * fewer than N nodes), so zero-duration cycles are found as well.
 *
 * Algorithm: Kahn topological order on the combined graph, one candidate at a time.
 *
 * Pins (tests/test_oracle_*.py): 1F1B and GPipe closed forms, P = 1, one machine per node,
 * alternating path, critical-path and load lower bounds, an independent unit-time-step simulator,
 * brute-force enumeration of all linear extensions on tiny DAGs, the constraint system itself
 * (eqs. (2),(3),(7),(11)-(13),(17)-(19)) with tightness, scaling / relabelling / time-reversal
 * invariances, constructed cycles and malformed candidates; missing channels against the product
 * form of eqs. (9)-(10) over one-hot allocations, and against pipelines on a chain-shaped cluster.
 * Parity unpinned: the DualPipe bubble values and the random-graph speed-up of Sec. V (the
 * instances and the schedules found there are not published).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { OR_OK = 0, OR_EINVAL = -1, OR_ECYCLE = -2, OR_EOVERFLOW = -3, OR_ENOMEM = -4 };
enum { FLAG_CYCLIC = 1, FLAG_BAD_PLACEMENT = 2, FLAG_BAD_RANK = 4, FLAG_OVER_MEMORY = 16, FLAG_NO_CHANNEL = 32 };
enum { NO_CHANNEL = -1 };   /* comm entry of a machine pair outside C */
enum { LAYOUT_CAND_MAJOR = 0, LAYOUT_CAND_MINOR = 1 };

/*
 * Checks on the problem itself (not on a candidate):
 *   EINVAL     sizes out of range, CSR not monotone, index out of range, self-loop, negative
 *              duration, off-diagonal comm entry below -1 (-1 itself: no channel, eq. (10))
 *   ECYCLE     the operator graph is not a DAG (Sec. III requires one)
 *   EOVERFLOW  sum(dur) + (N-1) * max off-diagonal comm > INT32_MAX: a path visits every node at
 *              most once and pays at most one delay per edge, so below this bound int32 times
 *              are exact
 */
int dagsched_oracle_check_problem(int32_t N, int32_t E, int32_t P, const int32_t *row_ptr,
                                  const int32_t *col_idx, const int32_t *dur, const int32_t *comm,
                                  const int64_t *mem_delta) {
  if (N < 1 || E < 0 || P < 1 || P > 64) return OR_EINVAL;
  if (!row_ptr || !dur || !comm || !mem_delta || (E > 0 && !col_idx)) return OR_EINVAL;
  if (row_ptr[0] != 0 || row_ptr[N] != E) return OR_EINVAL;
  for (int32_t u = 0; u < N; ++u)
    if (row_ptr[u + 1] < row_ptr[u]) return OR_EINVAL;
  for (int32_t u = 0; u < N; ++u)
    for (int32_t k = row_ptr[u]; k < row_ptr[u + 1]; ++k)
      if (col_idx[k] < 0 || col_idx[k] >= N || col_idx[k] == u) return OR_EINVAL;
  int64_t sum_dur = 0, max_comm = 0;
  for (int32_t v = 0; v < N; ++v) {
    if (dur[v] < 0) return OR_EINVAL;
    sum_dur += dur[v];
  }
  for (int32_t a = 0; a < P; ++a)
    for (int32_t b = 0; b < P; ++b) {
      if (a == b) continue;
      if (comm[a * P + b] < NO_CHANNEL) return OR_EINVAL;
      if (comm[a * P + b] > max_comm) max_comm = comm[a * P + b];
    }
  /* the DAG must be acyclic: Kahn on B alone */
  int32_t *indeg = (int32_t *)calloc((size_t)N, sizeof(int32_t));
  int32_t *queue = (int32_t *)malloc((size_t)N * sizeof(int32_t));
  if (!indeg || !queue) { free(indeg); free(queue); return OR_ENOMEM; }
  for (int32_t k = 0; k < E; ++k) indeg[col_idx[k]]++;
  int32_t head = 0, tail = 0;
  for (int32_t v = 0; v < N; ++v) if (indeg[v] == 0) queue[tail++] = v;
  while (head < tail) {
    int32_t u = queue[head++];
    for (int32_t k = row_ptr[u]; k < row_ptr[u + 1]; ++k)
      if (--indeg[col_idx[k]] == 0) queue[tail++] = col_idx[k];
  }
  free(indeg); free(queue);
  if (tail != N) return OR_ECYCLE;
  if (sum_dur + (int64_t)(N - 1) * max_comm > (int64_t)INT32_MAX) return OR_EOVERFLOW;
  return OR_OK;
}

typedef struct {
  int32_t *cnt;     /* [P]   n_j                                   */
  int32_t *off;     /* [P+1] start of machine j in list            */
  int32_t *list;    /* [N]   list[off[j] + r] = node of rank r     */
  int32_t *indeg;   /* [N]   remaining predecessors (DAG + chain)  */
  int32_t *indeg_b; /* [N]   DAG in-degree (with multiplicity)     */
  int32_t *queue;   /* [N]                                         */
  int64_t *ready;   /* [N]   lower bound on s_v collected so far   */
  int64_t *start;   /* [N]                                         */
  int64_t *end;     /* [N]                                         */
} scratch_t;

static void scratch_free(scratch_t *w) {
  free(w->cnt); free(w->off); free(w->list); free(w->indeg); free(w->indeg_b);
  free(w->queue); free(w->ready); free(w->start); free(w->end);
}

static int scratch_alloc(scratch_t *w, int32_t N, int32_t P) {
  memset(w, 0, sizeof(*w));
  w->cnt = (int32_t *)malloc((size_t)P * sizeof(int32_t));
  w->off = (int32_t *)malloc((size_t)(P + 1) * sizeof(int32_t));
  w->list = (int32_t *)malloc((size_t)N * sizeof(int32_t));
  w->indeg = (int32_t *)malloc((size_t)N * sizeof(int32_t));
  w->indeg_b = (int32_t *)calloc((size_t)N, sizeof(int32_t));
  w->queue = (int32_t *)malloc((size_t)N * sizeof(int32_t));
  w->ready = (int64_t *)malloc((size_t)N * sizeof(int64_t));
  w->start = (int64_t *)malloc((size_t)N * sizeof(int64_t));
  w->end = (int64_t *)malloc((size_t)N * sizeof(int64_t));
  if (!w->cnt || !w->off || !w->list || !w->indeg || !w->indeg_b || !w->queue || !w->ready ||
      !w->start || !w->end) {
    scratch_free(w);
    return OR_ENOMEM;
  }
  return OR_OK;
}

/*
 * One candidate.  pl[v*stride], rk[v*stride] are placement and rank of node v.
 * Returns the flag; on flag 0 fills *makespan, *bubble, peak[j*peak_stride] and leaves
 * start/end times of every node in w->start / w->end.
 */
static int32_t evaluate_one(int32_t N, int32_t P, const int32_t *row_ptr, const int32_t *col_idx,
                            const int32_t *dur, const int32_t *comm, const int64_t *mem_delta,
                            const int64_t *weight, const int64_t *limit,
                            const int32_t *pl, const int32_t *rk, int64_t stride, scratch_t *w,
                            int32_t *makespan, int64_t *bubble, int64_t *peak, int64_t peak_stride) {
  /* 1. placement in range (eq. (6): exactly one machine of J) */
  for (int32_t v = 0; v < N; ++v) {
    int32_t j = pl[v * stride];
    if (j < 0 || j >= P) return FLAG_BAD_PLACEMENT;
  }
  /* 2. ranks dense per machine: a total order on each machine (eqs. (7)-(8)) */
  for (int32_t j = 0; j < P; ++j) w->cnt[j] = 0;
  for (int32_t v = 0; v < N; ++v) w->cnt[pl[v * stride]]++;
  w->off[0] = 0;
  for (int32_t j = 0; j < P; ++j) w->off[j + 1] = w->off[j] + w->cnt[j];
  for (int32_t i = 0; i < N; ++i) w->list[i] = -1;
  for (int32_t v = 0; v < N; ++v) {
    int32_t j = pl[v * stride], r = rk[v * stride];
    if (r < 0 || r >= w->cnt[j]) return FLAG_BAD_RANK;
    if (w->list[w->off[j] + r] != -1) return FLAG_BAD_RANK;
    w->list[w->off[j] + r] = v;
  }
  /* 3. every message has a channel: z_{u,x,ju,jx} = x_{u,ju} * x_{x,jx} must be 0 outside C (eqs. (9)-(10)) */
  for (int32_t u = 0; u < N; ++u)
    for (int32_t k = row_ptr[u]; k < row_ptr[u + 1]; ++k) {
      int32_t ju = pl[u * stride], jx = pl[col_idx[k] * stride];
      if (ju != jx && comm[ju * P + jx] == NO_CHANNEL) return FLAG_NO_CHANNEL;
    }
  /* 4. Kahn on the combined graph: DAG edges B plus chain edges list_j[k] -> list_j[k+1] */
  for (int32_t v = 0; v < N; ++v) {
    w->indeg[v] = w->indeg_b[v] + (rk[v * stride] > 0 ? 1 : 0);
    w->ready[v] = 0;                                   /* s_v >= 0 */
  }
  int32_t head = 0, tail = 0;
  for (int32_t v = 0; v < N; ++v) if (w->indeg[v] == 0) w->queue[tail++] = v;
  while (head < tail) {
    int32_t v = w->queue[head++];
    int32_t jv = pl[v * stride];
    int64_t s = w->ready[v];
    int64_t e = s + dur[v];                            /* eq. (3) */
    w->start[v] = s;
    w->end[v] = e;
    for (int32_t k = row_ptr[v]; k < row_ptr[v + 1]; ++k) {      /* data-dependent successors */
      int32_t x = col_idx[k];
      int32_t jx = pl[x * stride];
      int64_t delay = (jx != jv) ? comm[jv * P + jx] : 0;        /* eqs. (11)-(13) */
      if (e + delay > w->ready[x]) w->ready[x] = e + delay;
      if (--w->indeg[x] == 0) w->queue[tail++] = x;
    }
    int32_t r = rk[v * stride];
    if (r + 1 < w->cnt[jv]) {                                    /* next op on the same machine, eq. (7) */
      int32_t x = w->list[w->off[jv] + r + 1];
      if (e > w->ready[x]) w->ready[x] = e;
      if (--w->indeg[x] == 0) w->queue[tail++] = x;
    }
  }
  if (tail < N) return FLAG_CYCLIC;
  /* 5. reductions */
  int64_t z = 0, sum_dur = 0;
  for (int32_t v = 0; v < N; ++v) {
    if (w->end[v] > z) z = w->end[v];                  /* eq. (2) */
    sum_dur += dur[v];
  }
  *makespan = (int32_t)z;
  *bubble = (int64_t)P * z - sum_dur;
  int32_t over = 0;
  for (int32_t j = 0; j < P; ++j) {
    int64_t base = 0;                                  /* eq. (16): static memory of everything placed on j */
    if (weight)
      for (int32_t k = 0; k < w->cnt[j]; ++k) base += weight[w->list[w->off[j] + k]];
    int64_t level = base, top = base;                  /* eqs. (17)-(19) along the chain */
    for (int32_t k = 0; k < w->cnt[j]; ++k) {
      level += mem_delta[w->list[w->off[j] + k]];
      if (level > top) top = level;
    }
    peak[j * peak_stride] = top;
    if (limit && top > limit[j]) over = 1;
  }
  return over ? FLAG_OVER_MEMORY : 0;
}

/*
 * Evaluate candidates [first, first + count) of a batch of n_cand candidates.
 * layout 0: placement[c*N + v], peak_mem[c*P + j];  layout 1: placement[v*n_cand + c], peak_mem[j*n_cand + c].
 * All pointers are host memory; outputs are indexed by the absolute candidate number.
 */
int dagsched_oracle_evaluate_mem(int32_t N, int32_t E, int32_t P, const int32_t *row_ptr,
                                 const int32_t *col_idx, const int32_t *dur, const int32_t *comm,
                                 const int64_t *mem_delta, const int64_t *weight, const int64_t *mem_limit,
                                 int32_t layout, int64_t n_cand,
                                 const int32_t *placement, const int32_t *rank, int64_t first,
                                 int64_t count, int32_t *makespan, int64_t *bubble, int64_t *peak_mem,
                                 int32_t *flags) {
  int rc = dagsched_oracle_check_problem(N, E, P, row_ptr, col_idx, dur, comm, mem_delta);
  if (rc != OR_OK) return rc;
  if (weight)
    for (int32_t v = 0; v < N; ++v)
      if (weight[v] < 0) return OR_EINVAL;
  if (layout != LAYOUT_CAND_MAJOR && layout != LAYOUT_CAND_MINOR) return OR_EINVAL;
  if (n_cand < 0 || first < 0 || count < 0 || first + count > n_cand) return OR_EINVAL;
  if (count == 0) return OR_OK;
  if (!placement || !rank || !makespan || !bubble || !peak_mem || !flags) return OR_EINVAL;
  scratch_t w;
  rc = scratch_alloc(&w, N, P);
  if (rc != OR_OK) return rc;
  for (int32_t k = 0; k < E; ++k) w.indeg_b[col_idx[k]]++;
  for (int64_t c = first; c < first + count; ++c) {
    const int32_t *pl, *rk;
    int64_t stride, peak_stride;
    int64_t *peak;
    if (layout == LAYOUT_CAND_MAJOR) {
      pl = placement + c * N; rk = rank + c * N; stride = 1;
      peak = peak_mem + c * P; peak_stride = 1;
    } else {
      pl = placement + c; rk = rank + c; stride = n_cand;
      peak = peak_mem + c; peak_stride = n_cand;
    }
    int32_t z = -1;
    int64_t b = -1;
    int32_t f = evaluate_one(N, P, row_ptr, col_idx, dur, comm, mem_delta, weight, mem_limit, pl, rk, stride,
                             &w, &z, &b, peak, peak_stride);
    flags[c] = f;
    if (f != 0) {
      z = -1; b = -1;
      for (int32_t j = 0; j < P; ++j) peak[j * peak_stride] = -1;
    }
    makespan[c] = z;
    bubble[c] = b;
  }
  scratch_free(&w);
  return OR_OK;
}

/*
 * The full earliest-start schedule of ONE candidate (placement[N], rank[N]), for the constraint
 * checker: start/end times (eqs. (2),(3)) and memory level before/after every operation
 * (m-, m+ of eqs. (16)-(19); the base level of a machine is the static memory placed on it, 0
 * when weight is NULL).  Returns the problem code (<0) or the flag (>= 0); the arrays are filled
 * only when the result is 0.
 */
int dagsched_oracle_schedule_mem(int32_t N, int32_t E, int32_t P, const int32_t *row_ptr,
                                 const int32_t *col_idx, const int32_t *dur, const int32_t *comm,
                                 const int64_t *mem_delta, const int64_t *weight, const int32_t *placement,
                                 const int32_t *rank, int64_t *start, int64_t *end, int64_t *m_minus,
                                 int64_t *m_plus) {
  int rc = dagsched_oracle_check_problem(N, E, P, row_ptr, col_idx, dur, comm, mem_delta);
  if (rc != OR_OK) return rc;
  if (!placement || !rank || !start || !end || !m_minus || !m_plus) return OR_EINVAL;
  scratch_t w;
  rc = scratch_alloc(&w, N, P);
  if (rc != OR_OK) return rc;
  for (int32_t k = 0; k < E; ++k) w.indeg_b[col_idx[k]]++;
  int64_t *peak = (int64_t *)malloc((size_t)P * sizeof(int64_t));
  if (!peak) { scratch_free(&w); return OR_ENOMEM; }
  int32_t z;
  int64_t b;
  int32_t f = evaluate_one(N, P, row_ptr, col_idx, dur, comm, mem_delta, weight, NULL, placement, rank, 1, &w,
                           &z, &b, peak, 1);
  if (f == 0) {
    for (int32_t v = 0; v < N; ++v) { start[v] = w.start[v]; end[v] = w.end[v]; }
    for (int32_t j = 0; j < P; ++j) {
      int64_t level = 0;
      if (weight)
        for (int32_t k = 0; k < w.cnt[j]; ++k) level += weight[w.list[w.off[j] + k]];   /* eq. (16) */
      for (int32_t k = 0; k < w.cnt[j]; ++k) {
        int32_t v = w.list[w.off[j] + k];
        m_minus[v] = level;
        level += mem_delta[v];                         /* eq. (19) */
        m_plus[v] = level;
      }
    }
  }
  free(peak);
  scratch_free(&w);
  return f;
}

/*
 * ---------------------------------------------------------------------------------------------------
 * Channel contention (Sec. III, eqs. (11)-(15)).
 *
 * In the functions above a message is a pure delay.  The paper's model is stricter: the message of an edge
 * (u, x) of B whose ends sit on different machines a = placement[u], b = placement[x] is a transfer that
 * occupies the channel (a, b) from its start c to its end d, with c >= e_u (eq. (13)), d - c >= D^c
 * (eq. (11), D^c = comm[a][b] in the machine-dimension form) and s_x >= d (eq. (12)); two transfers on one
 * channel must not overlap, and the binaries w of eqs. (14)-(15) say which of the two goes first.  A candidate
 * fixes those binaries as well: edge_rank[k] is the dense rank of the transfer of edge k (k = position in
 * col_idx) among the transfers of its channel.  Edges inside a machine need no transfer; their edge_rank is
 * not looked at.  With every binary fixed the earliest-start schedule is again a longest path, now on the
 * graph whose nodes are the operations and the transfers:
 *
 *     c_k = max(e_u, d_prev(k)),  d_k = c_k + comm[a][b]       prev(k): the transfer before k on its channel
 *     s_x = max(0, e_chainpred(x), max over in-edges k: same machine ? e_u : d_k),  e_x = s_x + D^o_x
 *
 * Flags as above, with BAD_RANK also for a channel whose ranks are not exactly 0..n-1, and CYCLIC for a cycle
 * through operations and transfers.  The makespan is taken over the operations (eq. (2)); every transfer
 * ends before the operation it feeds starts.
 *
 * Pins (tests/test_contention_oracle.py): a hand-worked case with two transfers on one channel in both
 * orders (tests/golden/hand_contention.txt); a unit-time-step simulation of the model written from the
 * definition (tests/checkers.py); the cases that reduce to the functions above (zero delays, at most one
 * transfer per channel); for batches with one shared placement, the same model expressed as extra nodes on
 * channel-machines and evaluated without any notion of a transfer.
 */
typedef struct {
  int32_t *esrc;     /* [E] producer of edge k                                   */
  int32_t *ccnt;     /* [P*P] transfers per channel                               */
  int32_t *coff;     /* [P*P+1]                                                   */
  int32_t *clist;    /* [E] clist[coff[ch] + r] = edge of rank r on channel ch    */
  int32_t *tindeg;   /* [E] remaining predecessors of transfer k                  */
  int64_t *tready;   /* [E] lower bound on c_k collected so far                   */
  int64_t *tend;     /* [E] d_k (-1: the edge has no transfer)                    */
  int32_t *queue;    /* [N+E] operations v as v, transfers k as N + k             */
} cscratch_t;

static void cscratch_free(cscratch_t *c) {
  free(c->esrc); free(c->ccnt); free(c->coff); free(c->clist); free(c->tindeg); free(c->tready); free(c->tend); free(c->queue);
}

static int cscratch_alloc(cscratch_t *c, int32_t N, int32_t E, int32_t P) {
  memset(c, 0, sizeof(*c));
  size_t e = (size_t)(E > 0 ? E : 1), pp = (size_t)P * P;
  c->esrc = (int32_t *)malloc(e * sizeof(int32_t));
  c->ccnt = (int32_t *)malloc(pp * sizeof(int32_t));
  c->coff = (int32_t *)malloc((pp + 1) * sizeof(int32_t));
  c->clist = (int32_t *)malloc(e * sizeof(int32_t));
  c->tindeg = (int32_t *)malloc(e * sizeof(int32_t));
  c->tready = (int64_t *)malloc(e * sizeof(int64_t));
  c->tend = (int64_t *)malloc(e * sizeof(int64_t));
  c->queue = (int32_t *)malloc(((size_t)N + e) * sizeof(int32_t));
  if (!c->esrc || !c->ccnt || !c->coff || !c->clist || !c->tindeg || !c->tready || !c->tend || !c->queue) {
    cscratch_free(c);
    return OR_ENOMEM;
  }
  return OR_OK;
}

/* One candidate with channel contention; er[k*stride] is the rank of edge k's transfer on its channel. */
static int32_t evaluate_one_contended(int32_t N, int32_t E, int32_t P, const int32_t *row_ptr, const int32_t *col_idx,
                                      const int32_t *dur, const int32_t *comm, const int64_t *mem_delta,
                                      const int64_t *weight, const int64_t *limit, const int32_t *pl,
                                      const int32_t *rk, const int32_t *er, int64_t stride, scratch_t *w,
                                      cscratch_t *c, int32_t *makespan, int64_t *bubble, int64_t *peak,
                                      int64_t peak_stride) {
  /* 1., 2. as without contention: x in range (eq. (6)), a total order per machine (eqs. (7)-(8)) */
  for (int32_t v = 0; v < N; ++v) {
    int32_t j = pl[v * stride];
    if (j < 0 || j >= P) return FLAG_BAD_PLACEMENT;
  }
  for (int32_t j = 0; j < P; ++j) w->cnt[j] = 0;
  for (int32_t v = 0; v < N; ++v) w->cnt[pl[v * stride]]++;
  w->off[0] = 0;
  for (int32_t j = 0; j < P; ++j) w->off[j + 1] = w->off[j] + w->cnt[j];
  for (int32_t i = 0; i < N; ++i) w->list[i] = -1;
  for (int32_t v = 0; v < N; ++v) {
    int32_t j = pl[v * stride], r = rk[v * stride];
    if (r < 0 || r >= w->cnt[j]) return FLAG_BAD_RANK;
    if (w->list[w->off[j] + r] != -1) return FLAG_BAD_RANK;
    w->list[w->off[j] + r] = v;
  }
  /* ... and a total order per channel (eqs. (14)-(15)): the transfers of channel (a, b) have ranks 0..n-1 */
  for (int32_t ch = 0; ch < P * P; ++ch) c->ccnt[ch] = 0;
  for (int32_t k = 0; k < E; ++k) {
    int32_t a = pl[c->esrc[k] * stride], b = pl[col_idx[k] * stride];
    if (a != b) c->ccnt[a * P + b]++;
  }
  c->coff[0] = 0;
  for (int32_t ch = 0; ch < P * P; ++ch) c->coff[ch + 1] = c->coff[ch] + c->ccnt[ch];
  for (int32_t i = 0; i < E; ++i) c->clist[i] = -1;
  for (int32_t k = 0; k < E; ++k) {
    int32_t a = pl[c->esrc[k] * stride], b = pl[col_idx[k] * stride];
    if (a == b) continue;
    int32_t ch = a * P + b, r = er[k * stride];
    if (r < 0 || r >= c->ccnt[ch]) return FLAG_BAD_RANK;
    if (c->clist[c->coff[ch] + r] != -1) return FLAG_BAD_RANK;
    c->clist[c->coff[ch] + r] = k;
  }
  /* 3. every message has a channel (eqs. (9)-(10)) */
  for (int32_t k = 0; k < E; ++k) {
    int32_t a = pl[c->esrc[k] * stride], b = pl[col_idx[k] * stride];
    if (a != b && comm[a * P + b] == NO_CHANNEL) return FLAG_NO_CHANNEL;
  }
  /* 4. Kahn on operations and transfers */
  int32_t n_transfers = 0;
  for (int32_t v = 0; v < N; ++v) {
    w->indeg[v] = w->indeg_b[v] + (rk[v * stride] > 0 ? 1 : 0);   /* one per in-edge, direct or through its transfer */
    w->ready[v] = 0;
  }
  for (int32_t k = 0; k < E; ++k) {
    int32_t a = pl[c->esrc[k] * stride], b = pl[col_idx[k] * stride];
    c->tend[k] = -1;
    c->tready[k] = 0;
    c->tindeg[k] = 0;
    if (a != b) {
      c->tindeg[k] = 1 + (er[k * stride] > 0 ? 1 : 0);            /* its producer, and the transfer before it */
      ++n_transfers;
    }
  }
  int32_t head = 0, tail = 0;
  for (int32_t v = 0; v < N; ++v) if (w->indeg[v] == 0) c->queue[tail++] = v;
  while (head < tail) {
    int32_t q = c->queue[head++];
    if (q < N) {                                           /* an operation */
      int32_t v = q, jv = pl[v * stride];
      int64_t s = w->ready[v], e = s + dur[v];             /* eq. (3) */
      w->start[v] = s;
      w->end[v] = e;
      for (int32_t k = row_ptr[v]; k < row_ptr[v + 1]; ++k) {
        int32_t x = col_idx[k];
        if (pl[x * stride] == jv) {                        /* same machine: no message */
          if (e > w->ready[x]) w->ready[x] = e;
          if (--w->indeg[x] == 0) c->queue[tail++] = x;
        } else {                                           /* the transfer may start once v has ended, eq. (13) */
          if (e > c->tready[k]) c->tready[k] = e;
          if (--c->tindeg[k] == 0) c->queue[tail++] = N + k;
        }
      }
      int32_t r = rk[v * stride];
      if (r + 1 < w->cnt[jv]) {                            /* next operation on the machine, eq. (7) */
        int32_t x = w->list[w->off[jv] + r + 1];
        if (e > w->ready[x]) w->ready[x] = e;
        if (--w->indeg[x] == 0) c->queue[tail++] = x;
      }
    } else {                                               /* a transfer */
      int32_t k = q - N, x = col_idx[k];
      int32_t a = pl[c->esrc[k] * stride], b = pl[x * stride], ch = a * P + b;
      int64_t d = c->tready[k] + comm[ch];                 /* eq. (11) */
      c->tend[k] = d;
      if (d > w->ready[x]) w->ready[x] = d;                /* eq. (12) */
      if (--w->indeg[x] == 0) c->queue[tail++] = x;
      int32_t r = er[k * stride];
      if (r + 1 < c->ccnt[ch]) {                           /* next transfer on the channel, eqs. (14)-(15) */
        int32_t k2 = c->clist[c->coff[ch] + r + 1];
        if (d > c->tready[k2]) c->tready[k2] = d;
        if (--c->tindeg[k2] == 0) c->queue[tail++] = N + k2;
      }
    }
  }
  if (tail < N + n_transfers) return FLAG_CYCLIC;
  /* 5. reductions, as without contention */
  int64_t z = 0, sum_dur = 0;
  for (int32_t v = 0; v < N; ++v) {
    if (w->end[v] > z) z = w->end[v];                      /* eq. (2) */
    sum_dur += dur[v];
  }
  *makespan = (int32_t)z;
  *bubble = (int64_t)P * z - sum_dur;
  int32_t over = 0;
  for (int32_t j = 0; j < P; ++j) {
    int64_t base = 0;                                      /* eq. (16) */
    if (weight)
      for (int32_t k = 0; k < w->cnt[j]; ++k) base += weight[w->list[w->off[j] + k]];
    int64_t level = base, top = base;                      /* eqs. (17)-(19) */
    for (int32_t k = 0; k < w->cnt[j]; ++k) {
      level += mem_delta[w->list[w->off[j] + k]];
      if (level > top) top = level;
    }
    peak[j * peak_stride] = top;
    if (limit && top > limit[j]) over = 1;
  }
  return over ? FLAG_OVER_MEMORY : 0;
}

/*
 * Candidates [first, first + count) of a batch with channel contention.  edge_rank has E entries per
 * candidate, laid out like placement (layout 0: edge_rank[c*E + k]; layout 1: edge_rank[k*n_cand + c]).
 * Besides the checks of dagsched_oracle_check_problem: sum(dur) + E * max comm must not exceed INT32_MAX
 * (a path may pay one transfer per edge).  When t_end is not NULL (count == 1 only) it receives the end of
 * every edge's transfer, -1 for edges inside a machine, and start / end the operations' times.
 */
int dagsched_oracle_evaluate_contended(int32_t N, int32_t E, int32_t P, const int32_t *row_ptr, const int32_t *col_idx,
                                       const int32_t *dur, const int32_t *comm, const int64_t *mem_delta,
                                       const int64_t *weight, const int64_t *mem_limit, int32_t layout, int64_t n_cand,
                                       const int32_t *placement, const int32_t *rank, const int32_t *edge_rank,
                                       int64_t first, int64_t count, int32_t *makespan, int64_t *bubble,
                                       int64_t *peak_mem, int32_t *flags, int64_t *start, int64_t *end, int64_t *t_end) {
  int rc = dagsched_oracle_check_problem(N, E, P, row_ptr, col_idx, dur, comm, mem_delta);
  if (rc != OR_OK) return rc;
  if (weight)
    for (int32_t v = 0; v < N; ++v)
      if (weight[v] < 0) return OR_EINVAL;
  if (layout != LAYOUT_CAND_MAJOR && layout != LAYOUT_CAND_MINOR) return OR_EINVAL;
  if (n_cand < 0 || first < 0 || count < 0 || first + count > n_cand) return OR_EINVAL;
  if (t_end && count != 1) return OR_EINVAL;
  {
    int64_t sum_dur = 0, max_comm = 0;
    for (int32_t v = 0; v < N; ++v) sum_dur += dur[v];
    for (int32_t a = 0; a < P; ++a)
      for (int32_t b = 0; b < P; ++b)
        if (a != b && comm[a * P + b] > max_comm) max_comm = comm[a * P + b];
    if (sum_dur + (int64_t)E * max_comm > (int64_t)INT32_MAX) return OR_EOVERFLOW;
  }
  if (count == 0) return OR_OK;
  if (!placement || !rank || (E > 0 && !edge_rank) || !makespan || !bubble || !peak_mem || !flags) return OR_EINVAL;
  scratch_t w;
  cscratch_t c;
  rc = scratch_alloc(&w, N, P);
  if (rc != OR_OK) return rc;
  rc = cscratch_alloc(&c, N, E, P);
  if (rc != OR_OK) { scratch_free(&w); return rc; }
  for (int32_t k = 0; k < E; ++k) w.indeg_b[col_idx[k]]++;
  for (int32_t u = 0; u < N; ++u)
    for (int32_t k = row_ptr[u]; k < row_ptr[u + 1]; ++k) c.esrc[k] = u;
  for (int64_t cand = first; cand < first + count; ++cand) {
    const int32_t *pl, *rk, *er;
    int64_t stride, peak_stride;
    int64_t *peak;
    if (layout == LAYOUT_CAND_MAJOR) {
      pl = placement + cand * N; rk = rank + cand * N; er = edge_rank + cand * E; stride = 1;
      peak = peak_mem + cand * P; peak_stride = 1;
    } else {
      pl = placement + cand; rk = rank + cand; er = edge_rank + cand; stride = n_cand;
      peak = peak_mem + cand; peak_stride = n_cand;
    }
    int32_t z = -1;
    int64_t b = -1;
    int32_t f = evaluate_one_contended(N, E, P, row_ptr, col_idx, dur, comm, mem_delta, weight, mem_limit, pl, rk, er,
                                       stride, &w, &c, &z, &b, peak, peak_stride);
    flags[cand] = f;
    if (f != 0) {
      z = -1; b = -1;
      for (int32_t j = 0; j < P; ++j) peak[j * peak_stride] = -1;
    }
    makespan[cand] = z;
    bubble[cand] = b;
    if (t_end && (f == 0 || f == FLAG_OVER_MEMORY)) {
      for (int32_t k = 0; k < E; ++k) t_end[k] = c.tend[k];
      if (start && end)
        for (int32_t v = 0; v < N; ++v) { start[v] = w.start[v]; end[v] = w.end[v]; }
    }
  }
  cscratch_free(&c);
  scratch_free(&w);
  return OR_OK;
}
