/*
 * dagsched - batched evaluation of candidate operator schedules on one MI355X (gfx950).
 *
 * Problem statement (arxiv 2503.09357, Sec. III and its notation table).  An operator DAG
 * G_m(I, B) with durations D^o_i, a cluster of P machines with a channel-delay matrix (the
 * machine-dimension form of D^c, footnote of Sec. III) and memory adjustments A_i are fixed.
 * A *candidate* fixes every binary of the MIP: the allocation x (eq. (6)) as placement[i], and
 * the per-machine total order y / immediate precedence u (eqs. (7)-(8), (17)-(18)) as a dense
 * per-machine rank[i] (on machine j the ranks are exactly 0..n_j-1).  With the binaries fixed,
 * eqs. (2), (3), (5), (7), (11)-(13) are difference constraints on the disjunctive graph (DAG
 * edges plus one chain edge between consecutive operations of a machine) and the optimum of
 * eq. (1) is a longest path.  For every candidate the library returns
 *
 *   makespan   z = max_i e_i, where s_v = max(0, e_chainpred(v), max_{(u,v) in B} e_u + delta(u,v)),
 *              e_v = s_v + D^o_v, delta(u,v) = comm[placement[u]][placement[v]] if the machines
 *              differ, else 0                                    (eqs. (1)-(3), (7), (11)-(13))
 *   bubble     P * z - sum_i D^o_i  (idle time of all P machines inside [0, z])
 *   peak_mem   per machine, the maximum over prefixes of its order of the running sum of A_i,
 *              the empty prefix included, on top of the machine's base level: the static memory
 *              W_i of everything placed on it (eq. (16)), 0 when no weights are given
 *                                                                 (eqs. (16)-(19))
 *   flags      0, or exactly one of DAGSCHED_FLAG_*; a flagged candidate has makespan = bubble =
 *              every peak_mem entry = -1.
 *
 * All entry points are thread-compatible, not thread-safe per handle: one evaluate at a time per
 * handle; distinct handles are independent.
 */
#ifndef DAGSCHED_H
#define DAGSCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dagsched dagsched_t; /* opaque, owned by the library */

/* Return codes of create / validate / evaluate. */
enum {
  DAGSCHED_OK = 0,
  DAGSCHED_EINVAL = -1,    /* null pointer, size out of range, malformed CSR, negative dur / weight, comm entry
                              below -1, bad layout, n_cand > max_candidates */
  DAGSCHED_ECYCLE = -2,    /* the operator graph itself is cyclic (Sec. III requires a DAG) */
  DAGSCHED_EOVERFLOW = -3, /* sum(dur) + (N-1) * max off-diagonal comm > INT32_MAX: int32 times would not be exact */
  DAGSCHED_ENOMEM = -4,    /* host or device allocation failed */
  DAGSCHED_EHIP = -5,      /* any other HIP runtime failure */
  DAGSCHED_ESCRATCH = -6   /* dagsched_schedule_static: more than DAGSCHED_STATIC_MAX_NODES operations */
};

/* Per-candidate flags[c]: exactly one value, tested in this order. */
enum {
  DAGSCHED_FLAG_OK = 0,
  DAGSCHED_FLAG_BAD_PLACEMENT = 2, /* some placement[i] outside [0, P)                    (eq. (6))      */
  DAGSCHED_FLAG_BAD_RANK = 4,      /* some machine's ranks are not exactly {0..n_j-1}     (eqs. (7)-(8)) */
  DAGSCHED_FLAG_NO_CHANNEL = 32,   /* some edge (u, v) of B has its ends on machines a != b whose comm[a*P + b] is
                                      DAGSCHED_NO_CHANNEL: z = x * x of eq. (9) must be 0 there (eq. (10))      */
  DAGSCHED_FLAG_CYCLIC = 1,        /* DAG edges + chain edges contain a directed cycle: eqs. (5), (7), (8)
                                      cannot hold together.  Structural test, zero-duration cycles included. */
  DAGSCHED_FLAG_INTERNAL = 8,      /* a kernel's bounded wait expired; never expected, the candidate's other
                                      outputs are -1.  Reported instead of hanging the GPU. */
  DAGSCHED_FLAG_OVER_MEMORY = 16   /* tested last: otherwise feasible, but some peak_mem[j] > mem_limit[j]
                                      (the per-machine memory limit of the problem statement of Sec. III and of
                                      the bounds of Sec. V-A; the paper prints no inequality for it) */
};

/* Memory layout of placement, rank and peak_mem. */
enum {
  DAGSCHED_CAND_MAJOR = 0, /* placement[c*N + i], peak_mem[c*P + j] */
  DAGSCHED_CAND_MINOR = 1  /* placement[i*C + c], peak_mem[j*C + c]  (C = n_cand of the call) */
};

/* comm entry of an ordered machine pair that is not in the channel set C (eq. (10)). */
#define DAGSCHED_NO_CHANNEL (-1)

/* Limits of this implementation. */
#define DAGSCHED_MAX_DEVICES 64
#define DAGSCHED_MAX_NODES 65535

/*
 * Optional launch shape of the evaluation kernels.  dagsched_create chooses a shape by itself from the
 * problem's size; a caller that evaluates very many batches of one problem can time a few shapes on a batch of
 * its own (dagsched_time_evaluate) and keep the fastest.  Every field: 0 = chosen by the library
 * (placement_mode: -1).  A shape that is not built or does not fit the GPU's LDS makes the library fall back
 * to its general int32 kernel (dagsched_get_info tells); results never depend on the shape.  The library reads
 * no environment variable: this struct is the only way to steer the choice.
 */
typedef struct {
  int32_t cand_per_block;   /* candidates per workgroup: a power of two, at most 64 / (P rounded up to a power of two) */
  int32_t ring_slots;       /* 4 or 8 with the placement in LDS; 8, 16 or 32 with it in L2                  */
  int32_t feeders;          /* wavefronts that prepare operations for the relaxing wavefront: 1..4          */
  int32_t placement_mode;   /* -1 chosen by the library, 0 one byte per node in L2, 1 in LDS, 2 four bits per
                               node in LDS (P <= 16)                                                        */
  int32_t block_threads;    /* workgroup size: a multiple of 64, at least 64 * (2 + feeders), at most 1024  */
  int32_t state_bits;       /* width of the end times kept on chip: 16 (twice the candidates resident; candidates
                               whose end times leave the range are evaluated again with 32-bit end times) or 32 */
  int32_t preds_per_op;     /* 4: the kernel kind that reads four predecessors per op and splits operations with
                               more into parts, also where a leaner kind (single parts, two predecessors, one)
                               applies; 2: the two-predecessor kind also where the one-predecessor kind applies   */
  int32_t kernel;           /* 1: the general int32 kernel, whatever else would apply                        */
  int32_t static_waves;     /* relaxing wavefronts per workgroup of the shared-placement kernel (1..8); naming it
                               also makes small handles take that kernel                                     */
  int32_t ignore_shared_placement; /* 1: dagsched_desc_t.shared_placement is not used                        */
  int32_t window_cells;     /* end-time cells per candidate in the window mode of the ring kernel (16- or 32-bit end
                               times; for graphs whose
                               edges are short in the order of the node ids): a power of two from 8 to 32768 to ask
                               for that many, -1 to forbid the mode, 0 to let the library decide.  Candidates whose
                               schedule does not fit the window are evaluated again with a cell per operation   */
} dagsched_shape_t;

/*
 * The candidate-independent part of the problem.  Every pointer is HOST memory and is deep-copied
 * by dagsched_create; the caller may free it as soon as the call returns.
 */
typedef struct {
  int32_t n_nodes;          /* N = |I|, 1 <= N <= DAGSCHED_MAX_NODES                                        */
  int32_t n_edges;          /* E = |B| >= 0                                                                  */
  int32_t n_devices;        /* P = |J|, 1 <= P <= DAGSCHED_MAX_DEVICES                                       */
  const int32_t *row_ptr;   /* [N+1] successor CSR of B: edges u -> col_idx[k], k in [row_ptr[u], row_ptr[u+1]) */
  const int32_t *col_idx;   /* [E]   duplicates allowed, self-loops rejected                                 */
  const int32_t *dur;       /* [N]   D^o_i >= 0                                                              */
  const int32_t *comm;      /* [P*P] comm[src*P + dst] >= 0 off the diagonal, or DAGSCHED_NO_CHANNEL for a pair
                                     without a channel; may be asymmetric; the diagonal is never read        */
  const int64_t *mem_delta; /* [N]   A_i, any sign                                                           */
  int32_t max_candidates;   /* capacity of the per-handle device workspace, >= 1                             */
  int32_t layout;           /* DAGSCHED_CAND_MAJOR or DAGSCHED_CAND_MINOR                                     */
  int32_t hip_device;       /* ordinal of the GPU that owns the handle                                       */
  const int64_t *weight;    /* [N]   W_i >= 0, static memory of operation i (eq. (16)), or NULL: all zero    */
  const int64_t *mem_limit; /* [P]   memory limit of machine j, or NULL: no limit, OVER_MEMORY never set     */
  const dagsched_shape_t *shape; /* launch shape to use, or NULL: chosen by the library                      */
  const int32_t *shared_placement; /* [N] or NULL.  A hint: (nearly) every candidate of every batch will place
                                     operation i on machine shared_placement[i] (a pipeline with a fixed stage ->
                                     machine map, as in Sec. V) and only the orders differ.  The library may then
                                     resolve the delay of every edge once (eqs. (11)-(13)) and evaluate such
                                     candidates with a kernel of their own; candidates that place differently
                                     are still evaluated, one by one and slowly.  Results never depend on it.
                                     Entries outside [0, P): DAGSCHED_EINVAL                                   */
  int32_t contention;       /* 1: dagsched_evaluate_contended will be called on this handle; create then also
                               checks sum(dur) + E * max comm <= INT32_MAX (a path may pay one transfer per edge)
                               and allocates that call's workspace.  0 otherwise                               */
} dagsched_desc_t;

/*
 * Host-only check of a description (no GPU is touched): sizes, CSR shape, signs, acyclicity of B
 * (Sec. III: G_m is a DAG) and the int32 exactness bound.  Returns DAGSCHED_OK or the error
 * dagsched_create would return for the same description.
 */
int dagsched_validate(const dagsched_desc_t *desc);

/*
 * Validate, then upload the problem to desc->hip_device and allocate the workspace for
 * max_candidates candidates.  On success *out receives the handle; on error *out is untouched.
 * Synchronous; uses the device's default stream for the upload.
 */
int dagsched_create(const dagsched_desc_t *desc, dagsched_t **out);

/*
 * Evaluate n_cand candidates (0 <= n_cand <= max_candidates).  All six array arguments are DEVICE
 * pointers on the handle's GPU, owned by the caller and borrowed until the work enqueued on
 * hip_stream (a hipStream_t, or NULL for the default stream) has completed:
 *   placement, rank : int32, N * n_cand entries in the handle's layout       (inputs, read only)
 *   makespan        : int32 [n_cand]
 *   bubble          : int64 [n_cand]
 *   peak_mem        : int64, n_cand * P entries in the handle's layout
 *   flags           : int32 [n_cand]
 * Asynchronous: enqueues kernels only, performs no host synchronisation and no allocation.
 * Per-candidate problems are reported through flags, never through the return code.
 * Implements, per candidate, validation of x and y (eqs. (6)-(8)), of the channels used (eqs. (9)-(10)), the chain edges u, the
 * max-plus longest path (eqs. (2), (3), (5), (7), (11)-(13)), and the memory levels (eqs. (16)-(19)).
 */
int dagsched_evaluate(dagsched_t *h, int32_t n_cand, const int32_t *placement, const int32_t *rank,
                      int32_t *makespan, int64_t *bubble, int64_t *peak_mem, int32_t *flags,
                      void *hip_stream);

/*
 * dagsched_evaluate with channel contention (eqs. (11)-(15)): the message of an edge (u, x) of B whose ends sit on
 * different machines a, b is a transfer that occupies the channel (a, b) for comm[a*P + b] time units; it starts
 * once u has ended (eq. (13)) and the transfer before it on that channel has ended (eqs. (14)-(15)), and x starts
 * after it has ended (eqs. (11)-(12)).  The order of the transfers of a channel, i.e. the binaries w of eqs.
 * (14)-(15), comes with the candidate:
 *   edge_rank : int32 DEVICE, E * n_cand entries in the handle's layout (candidate-major edge_rank[c*E + k],
 *               candidate-minor edge_rank[k*C + c]); entry k belongs to the k-th edge of the description's CSR
 *               (u -> col_idx[k]) and is the rank of its transfer among the transfers of the same channel, which
 *               must be exactly 0..n-1 on every channel (else DAGSCHED_FLAG_BAD_RANK).  Entries of edges inside a
 *               machine are not looked at.
 * Everything else as dagsched_evaluate: same outputs, same flags (DAGSCHED_FLAG_CYCLIC now also for a cycle through
 * transfers), same asynchrony.  The makespan is taken over the operations (eq. (2)).  Only for handles made with
 * dagsched_desc_t.contention = 1 (else DAGSCHED_EINVAL).
 */
int dagsched_evaluate_contended(dagsched_t *h, int32_t n_cand, const int32_t *placement, const int32_t *rank,
                                const int32_t *edge_rank, int32_t *makespan, int64_t *bubble, int64_t *peak_mem,
                                int32_t *flags, void *hip_stream);

/* Release the handle and its device memory.  NULL is a no-op.  Synchronises the device first. */
void dagsched_destroy(dagsched_t *h);

/* Static, human-readable text for a return code; for DAGSCHED_EHIP it includes the last HIP error
 * recorded by this library on the calling thread. */
const char *dagsched_strerror(int code);

/*
 * Helpers for a planner that searches with dagsched_evaluate in its loop.  The paper hands the search over
 * the binaries x, y to a MIP solver (Sec. IV-V); these three calls are what a local search needs instead.
 * All pointers are DEVICE memory; all three calls are asynchronous on hip_stream and allocate nothing.
 *
 * dagsched_propose: the one-move neighbourhood of a base schedule (base_placement, base_rank: int32 [N], a
 * valid candidate).  Writes n_cand candidates (n_cand <= max_candidates) into placement / rank in the handle's
 * layout.  Candidate 0 is the base itself.  Candidate c >= 1 is the base with one move fixed by the four
 * words rnd[4c .. 4c+3] = (r0, r1, r2, r3) that the caller draws (rnd: uint32 [4 * n_cand]); with v = r1 mod N
 * the operation that moves, m its machine, n_j the operations on machine j in the base:
 *   r0 even  v trades places with the operation right after it on m (nothing when v is the last one there)
 *   r0 odd   m2 = r2 mod P;  m2 == m: v is re-inserted at position r3 mod n_m of m;
 *            m2 != m: v is inserted at position r3 mod (n_m2 + 1) of m2.
 * Every other operation keeps its relative order, so every candidate is dense; it may be cyclic.
 *
 * dagsched_propose_orders: the same with m2 = m whatever r2 is: every candidate keeps the allocation x of the
 * base and only the orders y change (the search of the pipeline experiments of Sec. V, where the stage ->
 * machine map is given).  With the base's placement as dagsched_desc_t.shared_placement the whole search runs
 * on the shared-placement kernel.
 *
 * dagsched_select: best[0] = index of the candidate with flags == 0 and the least makespan (lowest index
 * among equals), best[1] = that makespan; (-1, -1) when no candidate is feasible.  best: int32 [2].
 *
 * dagsched_schedule: start and end time of every operation of ONE candidate (placement, rank, start, end:
 * int32 [N], the earliest-start schedule of eqs. (2), (3), (7), (11)-(13)) and its flag (int32 [1]);
 * start = end = -1 everywhere when the flag is not 0.  For Gantt charts like those of Sec. V.
 */
int dagsched_propose(dagsched_t *h, int32_t n_cand, const int32_t *base_placement, const int32_t *base_rank,
                     const uint32_t *rnd, int32_t *placement, int32_t *rank, void *hip_stream);
int dagsched_propose_orders(dagsched_t *h, int32_t n_cand, const int32_t *base_placement, const int32_t *base_rank,
                            const uint32_t *rnd, int32_t *placement, int32_t *rank, void *hip_stream);
int dagsched_select(dagsched_t *h, int32_t n_cand, const int32_t *makespan, const int32_t *flags, int32_t *best,
                    void *hip_stream);
int dagsched_schedule(dagsched_t *h, const int32_t *placement, const int32_t *rank, int32_t *start, int32_t *end,
                      int32_t *flag, void *hip_stream);

/*
 * dagsched_schedule for callers that cannot allocate or have no workspace to give: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results and same asynchrony as
 * dagsched_schedule, but the per-call scratch (one order-list row, one end-time row, a small output block) lives in
 * a static device array of the library instead of the handle's workspace: about 257 KiB that every GPU a handle
 * was made on holds until the process ends.  The call allocates and frees nothing.  Problems with more than
 * DAGSCHED_STATIC_MAX_NODES operations are refused with DAGSCHED_ESCRATCH (nothing is enqueued).  All calls on
 * one GPU share that GPU's array, whatever the handle: calls that overlap in time on one GPU (different streams,
 * different threads) race; calls enqueued on one stream do not.  The array keeps the last call's contents, which
 * no call reads: every entry a call reads it has written before.
 */
#define DAGSCHED_STATIC_MAX_NODES 32768
int dagsched_schedule_static(dagsched_t *h, const int32_t *placement, const int32_t *rank, int32_t *start,
                             int32_t *end, int32_t *flag, void *hip_stream);

/*
 * Graph coarsening before the planning (Sec. IV, Alg. 1): merge operations greedily until at most target_nodes are
 * left, so that the planner works on a graph of manageable size.  Runs on the GPU hip_device (one persistent
 * workgroup; the merges are inherently sequential, each step is parallel over the graph), synchronously: every
 * pointer is HOST memory, device memory is allocated and released inside the call.
 *
 *   Redundant edges   (i1, i2) in B with some i3 such that (i1, i3) and (i3, i2) are in B (two hops, as the set
 *                     printed in Sec. IV) are left out while a candidate pair is looked for, never deleted.
 *   GetCandidateEdge  an edge (i1, i2) of the reduced graph whose head i2 has a single input and whose tail i1 has
 *                     a single output there, with dur[i1] + dur[i2] <= edge_dur_max and mem_req[i1] + mem_req[i2]
 *                     <= edge_mem_max; of several the lowest (i1, i2).
 *   GetCandidateNonEdge  two operations of equal depth (edges on the longest path of B from a source; they cannot
 *                     reach one another) with sums within nonedge_dur_max / nonedge_mem_max; of several the pair
 *                     with the least summed duration, then the lowest (i1, i2), i1 < i2.
 *   MergeNodes        duration, memory adjustment and memory requirement are summed, the edges of both operations
 *                     go to the new one, which keeps the smaller of the two names.
 *   Loop              as Alg. 1: edge merges while there is a candidate, then non-edge merges while there is one,
 *                     again from the top; it ends as soon as target_nodes is reached, or after a pass without a merge.
 * A negative threshold switches that kind of merge off.  What the paper leaves open (the thresholds, the choice
 * among several candidates, the rule for non-edges, the loop's exits) is fixed as stated here.
 *
 * Inputs: the successor CSR of B (as in dagsched_desc_t; duplicates allowed), dur [N] >= 0 with a sum of at most
 * INT32_MAX, mem_delta [N], mem_req [N] >= 0 or NULL (all zero).  Outputs, owned by the caller: node_map [N]
 * (operation -> index of its group; groups are numbered by their smallest member), the coarse graph c_row_ptr
 * [N + 1] / c_col_idx [E] (the first n_coarse + 1 and n_coarse_edges entries are written; columns ascending, no
 * duplicates), c_dur, c_mem_delta, c_mem_req [N] (the first n_coarse entries), and *result.
 * Returns DAGSCHED_OK, DAGSCHED_EINVAL (null pointer, sizes, malformed CSR, negative dur or mem_req, target_nodes
 * < 1), DAGSCHED_ECYCLE (B is cyclic), DAGSCHED_EOVERFLOW (sum of dur above INT32_MAX), DAGSCHED_ENOMEM, DAGSCHED_EHIP.
 */
typedef struct {
  int32_t target_nodes;     /* N of Alg. 1, >= 1 */
  int64_t edge_dur_max, edge_mem_max;        /* thresholds of GetCandidateEdge on the sums of a pair    */
  int64_t nonedge_dur_max, nonedge_mem_max;  /* thresholds of GetCandidateNonEdge (the stricter ones)   */
} dagsched_coarsen_params_t;

typedef struct {
  int32_t n_coarse;         /* operations left */
  int32_t n_coarse_edges;   /* edges of the coarse graph */
  int32_t merges_edge;      /* merges proposed by GetCandidateEdge */
  int32_t merges_nonedge;   /* merges proposed by GetCandidateNonEdge */
} dagsched_coarsen_result_t;

int dagsched_coarsen(int32_t n_nodes, int32_t n_edges, const int32_t *row_ptr, const int32_t *col_idx,
                     const int32_t *dur, const int64_t *mem_delta, const int64_t *mem_req,
                     const dagsched_coarsen_params_t *params, int32_t hip_device, int32_t *node_map,
                     int32_t *c_row_ptr, int32_t *c_col_idx, int32_t *c_dur, int64_t *c_mem_delta,
                     int64_t *c_mem_req, dagsched_coarsen_result_t *result);

/*
 * Introspection for benchmarks and tests: which kernel variant the handle selected and its launch
 * shape.  Fills the struct and returns DAGSCHED_OK, or DAGSCHED_EINVAL on NULL.
 */
typedef struct {
  int32_t variant;         /* 1, 2 general int32 kernel (end times in LDS / in HBM); 3 ring kernel, 16-bit times
                              proven to fit; 4 the same run optimistically (or in window mode) with a second, exact run behind it;
                              5 ring kernel with 32-bit times; 6 shared-placement kernel */
  int32_t cand_per_block;  /* candidates evaluated by one workgroup */
  int32_t block_threads;   /* workgroup size */
  int32_t lds_bytes;       /* dynamic LDS per workgroup */
  int32_t state_bits;      /* width of the per-node end-time state (16 or 32) */
  int16_t ring_slots;      /* ring kernel: slots per lane of the op ring, else 0 */
  int8_t kernel_kind;      /* ring kernel: 0 operations split into parts of four predecessors, 1 every operation a
                              single part, 2 at most two predecessors per operation, 3 at most one */
  int8_t wide_ops;         /* ring kernel: 1 when ops name machines instead of delays (delays above 255 or durations
                              above 65534 after the common factor is divided out) */
  int32_t time_scale;      /* common factor of every duration and delay, divided out inside the kernels */
  int8_t feeders;          /* ring kernel: feeder wavefronts per workgroup */
  int8_t placement_mode;   /* ring kernel: where the placement bytes sit (0 L2, 1 LDS, 2 LDS as four bits per node) */
  int8_t preds_per_op;     /* predecessors read per op: 1, 2 or 4 (ring and shared-placement kernels) */
  int8_t window_log2;      /* ring kernel in window mode: log2 of the end-time cells per candidate, else 0 */
} dagsched_info_t;
int dagsched_get_info(const dagsched_t *h, dagsched_info_t *info);

/*
 * Host-only (no GPU is touched): the kernel variant and launch shape dagsched_create would choose for this
 * description on a GPU with lds_bytes of LDS per workgroup and n_cu compute units (an MI355X has 163840 and 256).
 * Returns what dagsched_validate returns for the description, or DAGSCHED_EINVAL for a NULL info or sizes below
 * 1024 bytes / 1 unit.  For capacity planning, and for testing the planning code where no GPU is at hand.
 */
int dagsched_plan(const dagsched_desc_t *desc, int32_t lds_bytes, int32_t n_cu, dagsched_info_t *info);

/*
 * How many candidates of the handle's LAST evaluate needed a second, slower evaluation: those whose end times left
 * the 16-bit range of an optimistic run or whose schedule did not fit the window (variant 4: they are evaluated
 * again by the 32-bit form of the ring kernel, where a 32-bit end time per operation fits the GPU's LDS, else by
 * the general int32 kernel one by one, which is an order of magnitude slower per candidate), or that do not use
 * the shared placement (variant 6: the general kernel).  A caller who sees a large count should ask for 32-bit
 * state (dagsched_shape_t.state_bits), forbid the window (window_cells = -1) or drop the hint.  Synchronises hip_stream, the stream the
 * evaluate was enqueued on, and copies one word to the host: not for the asynchronous path.  *count = 0 for
 * variants without such a list.
 */
int dagsched_last_fallbacks(dagsched_t *h, void *hip_stream, int32_t *count);

/*
 * Timing aid: evaluate `reps` times back to back on hip_stream between two HIP events recorded on
 * that same stream and return the mean milliseconds per evaluate in *ms_per_eval.  Synchronises
 * hip_stream.  Same pointer contract as dagsched_evaluate.
 */
int dagsched_time_evaluate(dagsched_t *h, int32_t n_cand, const int32_t *placement, const int32_t *rank,
                           int32_t *makespan, int64_t *bubble, int64_t *peak_mem, int32_t *flags,
                           void *hip_stream, int32_t reps, float *ms_per_eval);

#ifdef __cplusplus
}
#endif
#endif /* DAGSCHED_H */
