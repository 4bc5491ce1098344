// Host-side sanitizer run: the CPU oracles and the host half of the library (description checks and the planning
// of kernel variant and launch shape) over problem files written by tests/sanitize/run.py, built with
// -fsanitize=address,undefined for the host.  No GPU is touched.  Prints one line per problem; exits non-zero when
// a call returns what it should not (the sanitizers abort on their own findings).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "dagsched.h"

extern "C" {
int dagsched_oracle_check_problem(int32_t, int32_t, int32_t, const int32_t *, const int32_t *, const int32_t *, const int32_t *,
                                  const int64_t *);
int dagsched_oracle_evaluate_mem(int32_t, int32_t, int32_t, const int32_t *, const int32_t *, const int32_t *, const int32_t *,
                                 const int64_t *, const int64_t *, const int64_t *, int32_t, int64_t, const int32_t *,
                                 const int32_t *, int64_t, int64_t, int32_t *, int64_t *, int64_t *, int32_t *);
int dagsched_oracle_evaluate_contended(int32_t, int32_t, int32_t, const int32_t *, const int32_t *, const int32_t *,
                                       const int32_t *, const int64_t *, const int64_t *, const int64_t *, int32_t, int64_t,
                                       const int32_t *, const int32_t *, const int32_t *, int64_t, int64_t, int32_t *,
                                       int64_t *, int64_t *, int32_t *, int64_t *, int64_t *, int64_t *);
int coarsen_oracle(int32_t, int32_t, const int32_t *, const int32_t *, const int64_t *, const int64_t *, const int64_t *, int32_t,
                   int64_t, int64_t, int64_t, int64_t, int32_t *, int32_t *, int32_t *, int32_t *, int64_t *, int64_t *, int64_t *,
                   int32_t *, int32_t *);
}

template <typename T>
static std::vector<T> read_vec(FILE *f, size_t n) {
  std::vector<T> v(n);
  if (n && fread(v.data(), sizeof(T), n, f) != n) { fprintf(stderr, "short read\n"); exit(2); }
  return v;
}

int main(int argc, char **argv) {
  int bad = 0;
  for (int a = 1; a < argc; ++a) {
    FILE *f = fopen(argv[a], "rb");
    if (!f) { fprintf(stderr, "cannot open %s\n", argv[a]); return 2; }
    // header: N, E, P, C, shared (0/1), max_candidates
    const std::vector<int32_t> hd = read_vec<int32_t>(f, 6);
    const int32_t N = hd[0], E = hd[1], P = hd[2], C = hd[3], shared = hd[4], maxc = hd[5];
    auto row_ptr = read_vec<int32_t>(f, (size_t)N + 1);
    auto col_idx = read_vec<int32_t>(f, (size_t)E);
    auto dur = read_vec<int32_t>(f, (size_t)N);
    auto comm = read_vec<int32_t>(f, (size_t)P * P);
    auto mem = read_vec<int64_t>(f, (size_t)N);
    auto weight = read_vec<int64_t>(f, (size_t)N);
    auto limit = read_vec<int64_t>(f, (size_t)P);
    auto pl = read_vec<int32_t>(f, (size_t)C * N);
    auto rk = read_vec<int32_t>(f, (size_t)C * N);
    auto er = read_vec<int32_t>(f, (size_t)C * E);
    fclose(f);

    // the library's host half: description check and planning, with and without the optional fields and shapes
    dagsched_desc_t d{};
    d.n_nodes = N; d.n_edges = E; d.n_devices = P;
    d.row_ptr = row_ptr.data(); d.col_idx = col_idx.data(); d.dur = dur.data(); d.comm = comm.data(); d.mem_delta = mem.data();
    d.max_candidates = maxc; d.layout = DAGSCHED_CAND_MAJOR; d.hip_device = 0;
    const int v0 = dagsched_validate(&d);
    int plans = 0;
    dagsched_info_t info{};
    for (int variant = 0; variant < 12; ++variant) {
      dagsched_shape_t sh{};
      sh.placement_mode = -1;
      dagsched_desc_t dd = d;
      dd.weight = (variant & 1) ? weight.data() : nullptr;
      dd.mem_limit = (variant & 1) ? limit.data() : nullptr;
      dd.shared_placement = (shared && (variant & 2)) ? pl.data() : nullptr;
      if (variant >= 4) {
        sh.feeders = 1 + variant % 4; sh.ring_slots = (variant & 4) ? 8 : 16; sh.placement_mode = variant % 3;
        sh.state_bits = variant >= 10 ? 32 : 0; sh.preds_per_op = variant == 7 ? 4 : 0; sh.static_waves = variant == 6 ? 2 : 0;
        sh.kernel = variant == 11 ? 1 : 0;
        sh.window_cells = variant == 8 ? 64 : variant == 9 ? -1 : variant == 5 ? 4096 : 0;
        dd.shape = &sh;
      }
      const int rc = dagsched_plan(&dd, 160 * 1024, 256, &info);
      if (rc != v0) { fprintf(stderr, "%s: plan returned %d, validate %d\n", argv[a], rc, v0); ++bad; }
      if (rc == DAGSCHED_OK) { ++plans; if (info.variant < 1 || info.variant > 6 || info.lds_bytes > 160 * 1024) ++bad; }
      (void)dagsched_plan(&dd, 64 * 1024, 8, &info);        // a smaller GPU: other shapes, or the int32 kernel
    }

    // the oracles
    const int o0 = dagsched_oracle_check_problem(N, E, P, row_ptr.data(), col_idx.data(), dur.data(), comm.data(), mem.data());
    if ((o0 == 0) != (v0 == 0)) { fprintf(stderr, "%s: oracle check %d, library %d\n", argv[a], o0, v0); ++bad; }
    std::vector<int32_t> z(C), fl(C);
    std::vector<int64_t> bub(C), peak((size_t)C * P);
    long feasible = 0, feasible_c = 0;
    if (o0 == 0) {
      for (int layout = 0; layout < 1; ++layout) {
        int rc = dagsched_oracle_evaluate_mem(N, E, P, row_ptr.data(), col_idx.data(), dur.data(), comm.data(), mem.data(),
                                              weight.data(), limit.data(), layout, C, pl.data(), rk.data(), 0, C, z.data(),
                                              bub.data(), peak.data(), fl.data());
        if (rc != 0) ++bad;
        for (int c = 0; c < C; ++c) feasible += fl[c] == 0;
        rc = dagsched_oracle_evaluate_contended(N, E, P, row_ptr.data(), col_idx.data(), dur.data(), comm.data(), mem.data(),
                                                nullptr, nullptr, layout, C, pl.data(), rk.data(), er.data(), 0, C, z.data(),
                                                bub.data(), peak.data(), fl.data(), nullptr, nullptr, nullptr);
        if (rc != 0 && rc != -3) ++bad;
        for (int c = 0; c < C; ++c) feasible_c += rc == 0 && fl[c] == 0;
      }
    }
    int32_t n_coarse = -1, me = 0, mn = 0;
    if (o0 == 0 && N <= 1600) {
      std::vector<int64_t> d64(dur.begin(), dur.end()), cd(N), cm(N), cr(N);
      std::vector<int32_t> node_map(N), crp((size_t)N + 1), cci((size_t)E + 1);
      const int rc = coarsen_oracle(N, E, row_ptr.data(), col_idx.data(), d64.data(), mem.data(), weight.data(), N / 4 + 1, 60, 1000,
                                    25, 400, &n_coarse, node_map.data(), crp.data(), cci.data(), cd.data(), cm.data(), cr.data(),
                                    &me, &mn);
      if (rc != 0) ++bad;
    }
    printf("%s: N=%d E=%d P=%d C=%d validate=%d plans=%d feasible=%ld with-contention=%ld coarse=%d (%d+%d merges)\n", argv[a], N, E, P, C,
           v0, plans, feasible, feasible_c, n_coarse, me, mn);
    fflush(stdout);
  }
  if (bad) { fprintf(stderr, "%d unexpected results\n", bad); return 1; }
  return 0;
}
