/*
 * CPU oracle for the graph-coarsening heuristic of Sec. IV (Alg. 1) of arxiv 2503.09357.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, serial and slow: a byte adjacency matrix, every quantity recomputed
 * from scratch in every call of the two candidate functions, so that each step can be checked against the
 * text by eye.  It shares no code with the HIP library and is never called from the product path.
 *
 * What the section defines, and the reading taken where it leaves a choice:
 *
 *  - Topologically redundant edges: (i1, i2) in B such that some i3 has (i1, i3) in B and (i3, i2) in B
 *    (two hops, nothing longer).  They are removed only while a candidate is looked for; B' below is B
 *    without them.  Merging works on B itself.
 *  - GetCandidateEdge: an edge (i1, i2) of B' whose head i2 has a single input and whose tail i1 has a single
 *    output (degrees counted in B'), with D^o_i1 + D^o_i2 <= edge_dur_max and R_i1 + R_i2 <= edge_mem_max,
 *    R the operations' memory requirement.  Of several such edges the one with the lowest (i1, i2) is
 *    returned (reading: the paper does not say which).
 *  - GetCandidateNonEdge: two operations without an edge.  Reading (the paper gives no rule beyond "stricter
 *    thresholds"): two operations of equal depth, depth = number of edges on the longest path of B from a
 *    source; such operations cannot reach one another, so merging them keeps the graph acyclic.  Thresholds
 *    nonedge_dur_max, nonedge_mem_max on the sums.  Of several pairs the one with the least summed duration,
 *    then the lowest (i1, i2), i1 < i2.
 *  - MergeNodes: the new operation has the summed duration, memory adjustment and memory requirement, every
 *    edge into or out of either operation now ends at the new one, parallel edges collapse and the edge
 *    between the two disappears.  The new operation is named after the smaller of the two names (so an
 *    operation's name is always the smallest original index in its group).
 *  - The loop of Alg. 1.  The guard of its second inner loop is read as "GetCandidateNonEdge returns" (as
 *    printed it tests the other function); "Break if |I| <= N" ends the whole procedure, as does a pass of the
 *    outer loop in which neither inner loop merges anything (as printed the outer loop never ends).
 *
 * Output: node_map[v] = index of v's group, groups numbered in the order of their names; the coarse graph
 * as a successor CSR with ascending column indices; per group the three sums.
 *
 * Pins (tests/test_coarsen_oracle.py): hand-worked graphs for the two-hop rule, the single-input /
 * single-output rule and the equal-depth rule; the closed form of a chain under a duration threshold; the
 * invariants (sums preserved, acyclic, coarse edges = images of the original edges, critical path kept by
 * edge merges, stop exactly at the target); a 200-operation random graph of maximum degree 3 brought to 40
 * operations (the scale of Sec. V-B); a second evaluator written with Python sets from the definitions.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { CO_OK = 0, CO_EINVAL = -1, CO_ECYCLE = -2, CO_ENOMEM = -4 };

typedef struct {
  int32_t n;
  unsigned char *adj;     /* adj[u * n + v] = 1 iff (u, v) in B, u and v names of living operations */
  unsigned char *red;     /* B' of the current call */
  unsigned char *alive;
  int64_t *dur, *mem, *req;
  int32_t *outdeg, *indeg, *depth, *left;
} graph_t;

/* B' = B without the topologically redundant edges (two-hop rule). */
static void reduced_graph(graph_t *g) {
  const int32_t n = g->n;
  for (int32_t u = 0; u < n; ++u)
    for (int32_t v = 0; v < n; ++v) {
      unsigned char keep = 0;
      if (g->alive[u] && g->alive[v] && g->adj[(size_t)u * n + v]) {
        keep = 1;
        for (int32_t w = 0; w < n && keep; ++w)
          if (g->alive[w] && g->adj[(size_t)u * n + w] && g->adj[(size_t)w * n + v]) keep = 0;
      }
      g->red[(size_t)u * n + v] = keep;
    }
  for (int32_t u = 0; u < n; ++u) { g->outdeg[u] = 0; g->indeg[u] = 0; }
  for (int32_t u = 0; u < n; ++u)
    for (int32_t v = 0; v < n; ++v)
      if (g->red[(size_t)u * n + v]) { g->outdeg[u]++; g->indeg[v]++; }
}

static int get_candidate_edge(graph_t *g, int64_t dur_max, int64_t mem_max, int32_t *a, int32_t *b) {
  const int32_t n = g->n;
  reduced_graph(g);
  for (int32_t u = 0; u < n; ++u)
    for (int32_t v = 0; v < n; ++v)
      if (g->red[(size_t)u * n + v] && g->outdeg[u] == 1 && g->indeg[v] == 1 &&
          g->dur[u] + g->dur[v] <= dur_max && g->req[u] + g->req[v] <= mem_max) {
        *a = u; *b = v;
        return 1;
      }
  return 0;
}

/* depth[v] = edges on the longest path of B from a source to v, by peeling sources */
static void depths(graph_t *g) {
  const int32_t n = g->n;
  for (int32_t v = 0; v < n; ++v) {
    g->depth[v] = 0;
    g->left[v] = 0;
    if (g->alive[v])
      for (int32_t u = 0; u < n; ++u)
        if (g->alive[u] && g->adj[(size_t)u * n + v]) g->left[v]++;
  }
  for (int32_t round = 0; round < n; ++round) {          /* at most n rounds: one level per round */
    int any = 0;
    for (int32_t u = 0; u < n; ++u)
      if (g->alive[u] && g->left[u] == 0 && g->depth[u] == round) {
        /* u's depth is final (all its predecessors were peeled in earlier rounds) */
        for (int32_t v = 0; v < n; ++v)
          if (g->alive[v] && g->adj[(size_t)u * n + v]) {
            if (g->depth[v] < round + 1) g->depth[v] = round + 1;
            g->left[v]--;
            any = 1;
          }
      }
    if (!any) break;
  }
}

static int get_candidate_nonedge(graph_t *g, int64_t dur_max, int64_t mem_max, int32_t *a, int32_t *b) {
  const int32_t n = g->n;
  /* (the redundant edges need not be removed here: each is a shortcut of a two-edge path, so the longest
     paths, and with them the depths, are the same in B and in B') */
  depths(g);
  int found = 0;
  int64_t best = 0;
  for (int32_t u = 0; u < n; ++u)
    for (int32_t v = u + 1; v < n; ++v)
      if (g->alive[u] && g->alive[v] && g->depth[u] == g->depth[v] &&
          g->dur[u] + g->dur[v] <= dur_max && g->req[u] + g->req[v] <= mem_max) {
        const int64_t s = g->dur[u] + g->dur[v];
        if (!found || s < best) { found = 1; best = s; *a = u; *b = v; }   /* (u, v) ascending: ties keep the lowest pair */
      }
  return found;
}

static void merge_nodes(graph_t *g, int32_t a, int32_t b, int32_t *name_of) {
  const int32_t n = g->n;
  const int32_t m = a < b ? a : b, o = a < b ? b : a;
  g->dur[m] += g->dur[o];
  g->mem[m] += g->mem[o];
  g->req[m] += g->req[o];
  for (int32_t x = 0; x < n; ++x) {
    if (g->adj[(size_t)o * n + x]) g->adj[(size_t)m * n + x] = 1;
    if (g->adj[(size_t)x * n + o]) g->adj[(size_t)x * n + m] = 1;
  }
  for (int32_t x = 0; x < n; ++x) { g->adj[(size_t)o * n + x] = 0; g->adj[(size_t)x * n + o] = 0; }
  g->adj[(size_t)m * n + m] = 0;
  g->alive[o] = 0;
  for (int32_t v = 0; v < n; ++v)
    if (name_of[v] == o) name_of[v] = m;
}

/*
 * All pointers are host memory.  row_ptr / col_idx: successor CSR of B (duplicates allowed, self-loops and
 * cycles rejected).  mem_req may be NULL (all zero).  Outputs: *n_coarse, node_map[n], c_row_ptr[n + 1]
 * (the first *n_coarse + 1 entries are used), c_col_idx[n_edges] (the first c_row_ptr[*n_coarse] entries),
 * c_dur, c_mem_delta, c_mem_req [n] (the first *n_coarse entries), *n_merges_edge and *n_merges_nonedge.
 */
int coarsen_oracle(int32_t n, int32_t n_edges, const int32_t *row_ptr, const int32_t *col_idx, const int64_t *dur,
                   const int64_t *mem_delta, const int64_t *mem_req, int32_t target, int64_t edge_dur_max,
                   int64_t edge_mem_max, int64_t nonedge_dur_max, int64_t nonedge_mem_max, int32_t *n_coarse,
                   int32_t *node_map, int32_t *c_row_ptr, int32_t *c_col_idx, int64_t *c_dur, int64_t *c_mem_delta,
                   int64_t *c_mem_req, int32_t *n_merges_edge, int32_t *n_merges_nonedge) {
  if (n < 1 || n_edges < 0 || target < 1 || !row_ptr || !dur || !mem_delta || (n_edges > 0 && !col_idx)) return CO_EINVAL;
  if (row_ptr[0] != 0 || row_ptr[n] != n_edges) return CO_EINVAL;
  graph_t g;
  memset(&g, 0, sizeof(g));
  g.n = n;
  g.adj = (unsigned char *)calloc((size_t)n * n, 1);
  g.red = (unsigned char *)calloc((size_t)n * n, 1);
  g.alive = (unsigned char *)malloc((size_t)n);
  g.dur = (int64_t *)malloc((size_t)n * sizeof(int64_t));
  g.mem = (int64_t *)malloc((size_t)n * sizeof(int64_t));
  g.req = (int64_t *)malloc((size_t)n * sizeof(int64_t));
  g.outdeg = (int32_t *)malloc((size_t)n * sizeof(int32_t));
  g.indeg = (int32_t *)malloc((size_t)n * sizeof(int32_t));
  g.depth = (int32_t *)malloc((size_t)n * sizeof(int32_t));
  g.left = (int32_t *)malloc((size_t)n * sizeof(int32_t));
  int32_t *name_of = (int32_t *)malloc((size_t)n * sizeof(int32_t));
  int rc = CO_OK;
  if (!g.adj || !g.red || !g.alive || !g.dur || !g.mem || !g.req || !g.outdeg || !g.indeg || !g.depth || !g.left || !name_of)
    rc = CO_ENOMEM;
  for (int32_t u = 0; rc == CO_OK && u < n; ++u) {
    if (row_ptr[u + 1] < row_ptr[u]) { rc = CO_EINVAL; break; }
    for (int32_t k = row_ptr[u]; k < row_ptr[u + 1]; ++k) {
      const int32_t v = col_idx[k];
      if (v < 0 || v >= n || v == u) { rc = CO_EINVAL; break; }
      g.adj[(size_t)u * n + v] = 1;
    }
  }
  if (rc == CO_OK) {
    for (int32_t v = 0; v < n; ++v) {
      if (dur[v] < 0 || (mem_req && mem_req[v] < 0)) rc = CO_EINVAL;
      g.alive[v] = 1; g.dur[v] = dur[v]; g.mem[v] = mem_delta[v]; g.req[v] = mem_req ? mem_req[v] : 0; name_of[v] = v;
    }
  }
  if (rc == CO_OK) {                                       /* B must be a DAG (Sec. III): every operation gets peeled */
    depths(&g);
    for (int32_t v = 0; v < n; ++v)
      if (g.left[v] != 0) rc = CO_ECYCLE;
  }
  int32_t size = n, merges_e = 0, merges_n = 0;
  while (rc == CO_OK && size > target) {                   /* the outer loop of Alg. 1 */
    int merged = 0;
    int32_t a, b;
    while (size > target && get_candidate_edge(&g, edge_dur_max, edge_mem_max, &a, &b)) {
      merge_nodes(&g, a, b, name_of);
      --size; ++merges_e; merged = 1;
    }
    while (size > target && get_candidate_nonedge(&g, nonedge_dur_max, nonedge_mem_max, &a, &b)) {
      merge_nodes(&g, a, b, name_of);
      --size; ++merges_n; merged = 1;
    }
    if (!merged) break;
  }
  if (rc == CO_OK) {
    int32_t *index_of = g.left;                            /* name -> index of the group */
    int32_t k = 0;
    for (int32_t v = 0; v < n; ++v)
      if (g.alive[v]) {
        index_of[v] = k;
        c_dur[k] = g.dur[v]; c_mem_delta[k] = g.mem[v]; c_mem_req[k] = g.req[v];
        ++k;
      }
    *n_coarse = k;
    for (int32_t v = 0; v < n; ++v) node_map[v] = index_of[name_of[v]];
    int32_t at = 0;
    k = 0;
    for (int32_t u = 0; u < n; ++u)
      if (g.alive[u]) {
        c_row_ptr[k++] = at;
        for (int32_t v = 0; v < n; ++v)
          if (g.alive[v] && g.adj[(size_t)u * n + v]) c_col_idx[at++] = index_of[v];
      }
    c_row_ptr[k] = at;
    *n_merges_edge = merges_e;
    *n_merges_nonedge = merges_n;
  }
  free(g.adj); free(g.red); free(g.alive); free(g.dur); free(g.mem); free(g.req);
  free(g.outdeg); free(g.indeg); free(g.depth); free(g.left); free(name_of);
  return rc;
}
