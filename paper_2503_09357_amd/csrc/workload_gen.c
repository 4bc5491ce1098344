/*
 * Seeded synthetic candidate generator: random operator placements and
 * randomized list schedules over a fixed operator DAG.
 *
 * This file only draws inputs.  It holds none of the evaluator's arithmetic
 * (no start/end times, no makespan, no memory levels): a candidate is a
 * placement x (one machine per operation, Sec. III eq. (6)) and a total order
 * per machine (the y/u binaries of eqs. (7)-(8), (17)-(18)) written as dense
 * per-machine ranks.
 *
 * Recipe ("randomized list scheduling"): keep the set of operations whose DAG
 * predecessors have all been picked; pick one of them uniformly at random;
 * append it to the order of the machine it is placed on; repeat.  The pick
 * sequence is a linear extension of the DAG, so the per-machine orders it
 * induces are always jointly acyclic, and ranks are dense by construction.
 *
 * Random numbers: splitmix64 (seeding) + xoshiro256** (stream), both public
 * domain algorithms by Blackman and Vigna; one independent stream per
 * candidate so that results do not depend on how candidates are chunked.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct { uint64_t s[4]; } rng_t;

static uint64_t splitmix64(uint64_t *x) {
  uint64_t z = (*x += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

static inline uint64_t rotl64(uint64_t x, int k) { return (x << k) | (x >> (64 - k)); }

static uint64_t rng_next(rng_t *r) {
  uint64_t *s = r->s;
  const uint64_t result = rotl64(s[1] * 5, 7) * 9;
  const uint64_t t = s[1] << 17;
  s[2] ^= s[0]; s[3] ^= s[1]; s[1] ^= s[2]; s[0] ^= s[3];
  s[2] ^= t;
  s[3] = rotl64(s[3], 45);
  return result;
}

static void rng_seed(rng_t *r, uint64_t seed, uint64_t stream) {
  uint64_t x = seed ^ (0xD1B54A32D192ED03ull * (stream + 1));
  for (int i = 0; i < 4; ++i) r->s[i] = splitmix64(&x);
}

/* unbiased integer in [0, n), n >= 1 (multiply-shift with rejection) */
static uint32_t rng_below(rng_t *r, uint32_t n) {
  uint64_t m = (uint64_t)(uint32_t)(rng_next(r) >> 32) * (uint64_t)n;
  uint32_t lo = (uint32_t)m;
  if (lo < n) {
    uint32_t thresh = (uint32_t)(-n) % n;
    while (lo < thresh) {
      m = (uint64_t)(uint32_t)(rng_next(r) >> 32) * (uint64_t)n;
      lo = (uint32_t)m;
    }
  }
  return (uint32_t)(m >> 32);
}

/*
 * n_nodes, row_ptr[N+1], col_idx[E]: successor CSR of the operator DAG (must be acyclic).
 * n_devices: number of machines P.
 * first_cand, n_cand: candidates [first_cand, first_cand + n_cand) are generated;
 *                     candidate c uses stream (seed, c) whatever the chunking.
 * fixed_placement:    [N] machine per node used for every candidate, or NULL.
 * group, n_groups:    when fixed_placement is NULL, every candidate draws one machine
 *                     uniformly per group and node v goes to the machine of group[v].
 * placement_out, rank_out: [n_cand][N] int32, candidate-major.
 * Returns 0, or -1 on bad arguments / out of memory / a cyclic DAG.
 */
int dagsched_workload_list_schedules(int32_t n_nodes, const int32_t *row_ptr, const int32_t *col_idx,
                                     int32_t n_devices, int64_t first_cand, int64_t n_cand, uint64_t seed,
                                     const int32_t *fixed_placement, const int32_t *group, int32_t n_groups,
                                     int32_t *placement_out, int32_t *rank_out) {
  if (n_nodes < 1 || n_devices < 1 || n_cand < 0 || !row_ptr || !placement_out || !rank_out) return -1;
  if (!fixed_placement && (!group || n_groups < 1)) return -1;
  const int32_t N = n_nodes;
  int32_t *indeg0 = (int32_t *)calloc((size_t)N, sizeof(int32_t));
  int32_t *indeg = (int32_t *)malloc((size_t)N * sizeof(int32_t));
  int32_t *ready = (int32_t *)malloc((size_t)N * sizeof(int32_t));
  int32_t *count = (int32_t *)malloc((size_t)n_devices * sizeof(int32_t));
  int32_t *gdev = (int32_t *)malloc((size_t)(n_groups > 0 ? n_groups : 1) * sizeof(int32_t));
  int rc = 0;
  if (!indeg0 || !indeg || !ready || !count || !gdev) { rc = -1; goto done; }
  for (int32_t u = 0; u < N; ++u)
    for (int32_t k = row_ptr[u]; k < row_ptr[u + 1]; ++k) indeg0[col_idx[k]]++;

  for (int64_t ci = 0; ci < n_cand; ++ci) {
    rng_t r;
    rng_seed(&r, seed, (uint64_t)(first_cand + ci));
    int32_t *pl = placement_out + (size_t)ci * N;
    int32_t *rk = rank_out + (size_t)ci * N;
    if (fixed_placement) {
      memcpy(pl, fixed_placement, (size_t)N * sizeof(int32_t));
    } else {
      for (int32_t g = 0; g < n_groups; ++g) gdev[g] = (int32_t)rng_below(&r, (uint32_t)n_devices);
      for (int32_t v = 0; v < N; ++v) pl[v] = gdev[group[v]];
    }
    memcpy(indeg, indeg0, (size_t)N * sizeof(int32_t));
    memset(count, 0, (size_t)n_devices * sizeof(int32_t));
    int32_t n_ready = 0, picked = 0;
    for (int32_t v = 0; v < N; ++v) if (indeg[v] == 0) ready[n_ready++] = v;
    while (n_ready > 0) {
      uint32_t i = rng_below(&r, (uint32_t)n_ready);
      int32_t v = ready[i];
      ready[i] = ready[--n_ready];
      rk[v] = count[pl[v]]++;
      ++picked;
      for (int32_t k = row_ptr[v]; k < row_ptr[v + 1]; ++k) {
        int32_t w = col_idx[k];
        if (--indeg[w] == 0) ready[n_ready++] = w;
      }
    }
    if (picked != N) { rc = -1; goto done; }
  }
done:
  free(indeg0); free(indeg); free(ready); free(count); free(gdev);
  return rc;
}
