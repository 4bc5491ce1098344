// Graph coarsening before the planning (Sec. IV, Alg. 1): operations are merged greedily until at most a target
// number is left.  One persistent workgroup holds the whole procedure, because every merge changes which edges are
// redundant and which pairs qualify, so the merges are inherently one after the other; inside a step everything is
// data-parallel over the graph:
//
//   B as two bit matrices in global memory (L2-resident): succ[u] and pred[v], n rows of W = ceil(n / 64) words; a
//   wavefront reads a row 64 words at a time.
//   Topologically redundant edge (u, v):  some w with (u, w) and (w, v) in B  <=>  succ[u] AND pred[v] != 0.  The
//   reduced graph B' is kept as a third bit matrix with its degrees.  A merge into m can change the status only of
//   edges that leave m or a predecessor of m (an edge (u, v) looks at succ[u] and at the rows of u's successors),
//   so after a merge only those rows are worked out again, a wavefront per row.
//   GetCandidateEdge:     a 64-bit atomic minimum over the rows with a single output in B' whose target has a single
//                         input there, key (u, v).
//   GetCandidateNonEdge:  depth = longest path in edges from a source, by peeling sources round by round.  Merging
//                         two operations of equal depth changes no depth (the new operation's predecessors are the
//                         union of theirs), so the depths are worked out once per run of non-edge merges.  Then a
//                         64-bit atomic minimum over pairs of equal depth, key (summed duration, u, v).
//   MergeNodes:           OR of the two rows in both matrices, the column of the vanishing operation rewritten
//                         row by row (one thread per neighbour), sums of duration, memory adjustment and memory
//                         requirement; the merged operation keeps the smaller name.
//
// Every loop either merges (at most n - 1 times in all) or ends, and no wavefront ever waits for another one
// except at barriers that all reach: the kernel always terminates.
#pragma once

#include "device_common.h"

namespace dagsched_dev {

struct CoarsenParams {
  int32_t n, n_edges, words, target;     // words = ceil(n / 64)
  int64_t edge_dur_max, edge_mem_max, nonedge_dur_max, nonedge_mem_max;
  const int32_t *row_ptr, *col_idx;      // successor CSR of B
  unsigned long long *succ, *pred;       // [n][words], zero on entry
  unsigned long long *kept;              // [n][words], zero on entry: the edges of the reduced graph B'
  int64_t *dur, *mem, *req;              // [n] in: the operations' attributes; out: the groups' sums at their names
  int32_t *alive, *parent;               // [n] work
  int32_t *outdeg, *indeg, *only, *depth, *left;   // [n] work
  int32_t *index_of;                     // [n] work: name -> index of the group
  // results
  int32_t *node_map;                     // [n]
  int32_t *c_row_ptr, *c_col_idx;        // [n + 1], [n_edges]
  int64_t *c_dur, *c_mem, *c_req;        // [n]
  int32_t *counts;                       // [3] groups, edge merges, non-edge merges
};

constexpr unsigned long long kNoCandidate = ~0ull;

// values that other wavefronts change with atomics are read at the L2, never from a line the CU may still hold
__device__ __forceinline__ int32_t ld_l2(const int32_t *p) { return ld_agent(p); }

// f(v) for every set bit v of a row of W words, ascending, with all lanes of the wavefront taking part (the row is
// read 64 words at a time, a word per lane); owner = the lane that holds v's word, base = first word of the chunk.
template <typename F>
__device__ __forceinline__ void for_each_bit(const unsigned long long *row, int W, int lane, F f) {
  for (int base = 0; base < W; base += kWave) {
    const unsigned long long word = (base + lane < W) ? row[base + lane] : 0ull;
    unsigned long long nz = __ballot(word != 0);
    while (nz) {
      const int owner = __builtin_ctzll(nz);
      nz &= nz - 1;
      unsigned long long bits = __shfl(word, owner, kWave);
      while (bits) {
        const int v = ((base + owner) << 6) + __builtin_ctzll(bits);
        bits &= bits - 1;
        f(v, base, owner);
      }
    }
  }
}

__global__ __launch_bounds__(1024) void coarsen_kernel(CoarsenParams p) {
  __shared__ unsigned long long s_best;
  __shared__ int s_any;
  const int tid = threadIdx.x, nthreads = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nwaves = nthreads >> 6;
  const int n = p.n, W = p.words;

  for (int v = tid; v < n; v += nthreads) { p.alive[v] = 1; p.parent[v] = v; p.indeg[v] = 0; p.outdeg[v] = 0; p.only[v] = -1; }
  for (int u = tid; u < n; u += nthreads)
    for (int k = p.row_ptr[u]; k < p.row_ptr[u + 1]; ++k) {
      const int v = p.col_idx[k];
      atomicOr(&p.succ[(size_t)u * W + (v >> 6)], 1ull << (v & 63));
      atomicOr(&p.pred[(size_t)v * W + (u >> 6)], 1ull << (u & 63));
    }
  __syncthreads();

  // Row u of the reduced graph B' (one wavefront): an edge (u, v) stays unless some operation lies between u and v.
  // The in-degrees of B' follow the bits that changed against the row as it was.
  auto reduce_row = [&](int u) {
    const unsigned long long *su = p.succ + (size_t)u * W;
    unsigned long long *ku = p.kept + (size_t)u * W;
    int kept_count = 0, last = -1;
    for (int base = 0; base < W; base += kWave) {
      const unsigned long long word = (base + lane < W) ? su[base + lane] : 0ull;
      unsigned long long keep = 0;
      unsigned long long nz = __ballot(word != 0);
      while (nz) {
        const int owner = __builtin_ctzll(nz);
        nz &= nz - 1;
        unsigned long long bits = __shfl(word, owner, kWave);
        while (bits) {
          const int b = __builtin_ctzll(bits);
          bits &= bits - 1;
          const int v = ((base + owner) << 6) + b;
          const unsigned long long *pv = p.pred + (size_t)v * W;
          bool hit = false;
          for (int x = lane; x < W; x += kWave) hit = hit || (su[x] & pv[x]) != 0;
          if (__ballot(hit) == 0) {                          // no operation between u and v
            ++kept_count;
            last = v;
            if (lane == owner) keep |= 1ull << b;
          }
        }
      }
      if (base + lane < W) {
        const unsigned long long old = ku[base + lane];
        unsigned long long diff = old ^ keep;
        while (diff) {
          const int b = __builtin_ctzll(diff);
          diff &= diff - 1;
          atomicAdd(&p.indeg[((base + lane) << 6) + b], ((keep >> b) & 1ull) ? 1 : -1);
        }
        ku[base + lane] = keep;
      }
    }
    if (lane == 0) { p.outdeg[u] = kept_count; p.only[u] = last; }
  };

  for (int u = wave; u < n; u += nwaves) reduce_row(u);
  __syncthreads();

  // MergeNodes(a, b): the operation with the larger name vanishes into the one with the smaller name
  auto merge_nodes = [&](int a, int b) {
    const int m = min(a, b), o = max(a, b);
    unsigned long long *sm = p.succ + (size_t)m * W, *so = p.succ + (size_t)o * W;
    unsigned long long *pm = p.pred + (size_t)m * W, *po = p.pred + (size_t)o * W;
    const unsigned long long bit_m = 1ull << (m & 63), bit_o = 1ull << (o & 63);
    const int wm = m >> 6, wo = o >> 6;
    // every neighbour of o now sees m instead (a neighbour's row is touched by the one thread that owns its bit)
    for (int w = tid; w < W; w += nthreads) {
      unsigned long long bits = so[w];
      while (bits) {
        const int x = (w << 6) + __builtin_ctzll(bits);
        bits &= bits - 1;
        if (x == m) continue;
        unsigned long long *px = p.pred + (size_t)x * W;
        px[wo] &= ~bit_o;
        px[wm] |= bit_m;
      }
      bits = po[w];
      while (bits) {
        const int x = (w << 6) + __builtin_ctzll(bits);
        bits &= bits - 1;
        if (x == m) continue;
        unsigned long long *sx = p.succ + (size_t)x * W;
        sx[wo] &= ~bit_o;
        sx[wm] |= bit_m;
      }
    }
    __syncthreads();
    for (int w = tid; w < W; w += nthreads) {
      unsigned long long s = sm[w] | so[w], q = pm[w] | po[w];
      if (w == wm) { s &= ~bit_m; q &= ~bit_m; }
      if (w == wo) { s &= ~bit_o; q &= ~bit_o; }
      sm[w] = s; pm[w] = q;
      so[w] = 0; po[w] = 0;
    }
    if (tid == 0) {
      p.dur[m] += p.dur[o]; p.mem[m] += p.mem[o]; p.req[m] += p.req[o];
      p.alive[o] = 0;
      p.parent[o] = m;
    }
    __syncthreads();
    // the reduced graph again, where it can have changed: the rows of m, of o (now empty) and of m's predecessors
    {
      int item = 0;
      if (wave == 0) reduce_row(m);
      if (wave == 1 % nwaves) reduce_row(o);
      for_each_bit(pm, W, lane, [&](int x, int, int) {
        if (item++ % nwaves == wave) reduce_row(x);
      });
    }
    __syncthreads();
  };

  int size = n, merges_edge = 0, merges_nonedge = 0;
  while (size > p.target) {                                 // the outer loop of Alg. 1
    bool merged = false;
    while (size > p.target) {                               // GetCandidateEdge / MergeNodes
      if (tid == 0) s_best = kNoCandidate;
      __syncthreads();
      for (int u = tid; u < n; u += nthreads) {
        if (!p.alive[u] || p.outdeg[u] != 1) continue;
        const int v = p.only[u];
        if (ld_l2(&p.indeg[v]) == 1 && p.dur[u] + p.dur[v] <= p.edge_dur_max && p.req[u] + p.req[v] <= p.edge_mem_max)
          atomicMin(&s_best, ((unsigned long long)(uint32_t)u << 32) | (uint32_t)v);
      }
      __syncthreads();
      const unsigned long long best = s_best;
      __syncthreads();
      if (best == kNoCandidate) break;
      merge_nodes((int)(best >> 32), (int)(best & 0xFFFFFFFFu));
      --size; ++merges_edge; merged = true;
    }
    bool have_depths = false;
    while (size > p.target) {                               // GetCandidateNonEdge / MergeNodes
      if (!have_depths) {
        // depth = edges on the longest path from a source: sources are peeled round by round; an operation whose last
        // predecessor is peeled in round r has depth r + 1 and is peeled in the next round
        for (int v = wave; v < n; v += nwaves) {
          int c = 0;
          if (p.alive[v]) {
            const unsigned long long *pv = p.pred + (size_t)v * W;
            for (int x = lane; x < W; x += kWave) c += __builtin_popcountll(pv[x]);
            for (int s = 1; s < kWave; s <<= 1) c += __shfl_xor(c, s, kWave);
          }
          if (lane == 0) { p.left[v] = c; p.depth[v] = 0; }
        }
        __syncthreads();
        // Per round first the operations to peel are marked (left = -1; what the marking reads is at rest since the
        // last barrier), then, behind a barrier, their successors are told; a peeled operation gets left = -2.
        for (int round = 0; round < n; ++round) {
          if (tid == 0) s_any = 0;
          for (int v = tid; v < n; v += nthreads)
            if (p.alive[v] && ld_l2(&p.left[v]) == 0 && ld_l2(&p.depth[v]) == round) st_agent(&p.left[v], -1);
          __syncthreads();
          for (int v = wave; v < n; v += nwaves) {
            if (!p.alive[v] || ld_l2(&p.left[v]) != -1) continue;   // wave-uniform
            for_each_bit(p.succ + (size_t)v * W, W, lane, [&](int x, int, int) {
              if (lane == 0) { atomicMax(&p.depth[x], round + 1); atomicSub(&p.left[x], 1); s_any = 1; }
            });
            if (lane == 0) st_agent(&p.left[v], -2);
          }
          __syncthreads();
          const int any = s_any;
          __syncthreads();
          if (!any) break;
        }
        have_depths = true;
      }
      if (tid == 0) s_best = kNoCandidate;
      __syncthreads();
      for (int u = tid; u < n; u += nthreads) {
        if (!p.alive[u]) continue;
        const int du = ld_l2(&p.depth[u]);
        const int64_t dur_u = p.dur[u], req_u = p.req[u];
        unsigned long long mine = kNoCandidate;
        for (int v = u + 1; v < n; ++v) {
          if (!p.alive[v] || ld_l2(&p.depth[v]) != du) continue;
          const int64_t s = dur_u + p.dur[v];
          if (s <= p.nonedge_dur_max && req_u + p.req[v] <= p.nonedge_mem_max)
            mine = min(mine, ((unsigned long long)s << 32) | ((unsigned long long)(uint32_t)u << 16) | (uint32_t)v);
        }
        if (mine != kNoCandidate) atomicMin(&s_best, mine);
      }
      __syncthreads();
      const unsigned long long best = s_best;
      __syncthreads();
      if (best == kNoCandidate) break;
      merge_nodes((int)((best >> 16) & 0xFFFFu), (int)(best & 0xFFFFu));
      --size; ++merges_nonedge; merged = true;
    }
    if (!merged) break;
  }

  // groups numbered in the order of their names; the coarse graph as a CSR with ascending columns
  for (int v = wave; v < n; v += nwaves) {                  // edges per row, kept in `left`
    int c = 0;
    if (p.alive[v]) {
      const unsigned long long *sv = p.succ + (size_t)v * W;
      for (int x = lane; x < W; x += kWave) c += __builtin_popcountll(sv[x]);
      for (int s = 1; s < kWave; s <<= 1) c += __shfl_xor(c, s, kWave);
    }
    if (lane == 0) p.left[v] = c;
  }
  __syncthreads();
  if (tid == 0) {
    int k = 0, at = 0;
    for (int v = 0; v < n; ++v)
      if (p.alive[v]) {
        p.index_of[v] = k;
        p.c_dur[k] = p.dur[v]; p.c_mem[k] = p.mem[v]; p.c_req[k] = p.req[v];
        p.c_row_ptr[k] = at;
        at += p.left[v];
        ++k;
      }
    p.c_row_ptr[k] = at;
    p.counts[0] = k; p.counts[1] = merges_edge; p.counts[2] = merges_nonedge;
  }
  __syncthreads();
  for (int v = tid; v < n; v += nthreads) {
    int r = v;
    while (p.parent[r] != r) r = p.parent[r];               // names only ever point to smaller names: the walk ends
    p.node_map[v] = p.index_of[r];
  }
  for (int v = wave; v < n; v += nwaves) {
    if (!p.alive[v]) continue;
    int at = p.c_row_ptr[p.index_of[v]];
    for_each_bit(p.succ + (size_t)v * W, W, lane, [&](int x, int, int) {
      if (lane == 0) p.c_col_idx[at] = p.index_of[x];
      ++at;
    });
  }
}

}  // namespace dagsched_dev
