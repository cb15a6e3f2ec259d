// Host-only entry points of the C ABI, run under AddressSanitizer and UndefinedBehaviorSanitizer (host code only;
// nothing here needs a GPU or launches a kernel).  Built by the package's build step into tests/native/host_san with
// the host half of dion_api.hip instrumented; tests/test_lib_host.py runs it and expects a clean exit.
// What it calls: the planning behind dion_workspace_bytes (shape grouping, Gram-matrix splits, the carving of the
// workspace) over a grid of shapes and batch sizes up to the limits the header allows, dion_cholesky_grid over
// compute-unit counts, batches and ranks, dion_strerror over all codes, and the argument checks that every other
// entry point makes before it touches the device; and the integer arithmetic that deals the output tiles of the
// triangular inverse out to its workgroups (csrc/inv_tree_order.hpp, the header the kernel itself includes): every
// tile of every level exactly once, for all tile counts up to r = 5120 and a range of workgroup counts, and no
// workgroup more than one tile's length above another.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <algorithm>
#include <vector>

#include "../../include/dion.h"
#include "../../paper_2504_05295_amd/csrc/inv_tree_order.hpp"

static int failures = 0;
#define EXPECT(cond)                                                   \
  do {                                                                 \
    if (!(cond)) {                                                     \
      fprintf(stderr, "line %d: expectation failed: %s\n", __LINE__, #cond); \
      ++failures;                                                      \
    }                                                                  \
  } while (0)

int main() {
  const int64_t dims[] = {1, 7, 63, 64, 65, 255, 256, 257, 1000, 2048, 3072, 8192, 16384, 53248, 1 << 20, 0x7fffff00LL};
  const int64_t ranks[] = {1, 2, 63, 64, 65, 128, 255, 256, 768, 1024, 4096, 32768};
  const int counts[] = {1, 2, 3, 28, 112, 128, 129, 196, 257, 1000};
  size_t calls = 0;
  for (int64_t m : dims)
    for (int64_t n : dims)
      for (int64_t r : ranks) {
        if (r > m || r > n) continue;
        for (int count : counts) {
          if ((double)m * (double)n * (double)count > 4e13) continue;   // stay below what size_t arithmetic is meant for
          std::vector<int64_t> ms(count, m), ns(count, n), rs(count, r);
          if (count > 2) { ms[1] = n; ns[1] = m; }                       // a second shape group
          for (int g = 0; g < 2; ++g)
            for (int math = 0; math < 2; ++math) {
              size_t bytes = 0;
              const int rc = dion_workspace_bytes(count, ms.data(), ns.data(), rs.data(), g, math, &bytes);
              EXPECT(rc == DION_OK);
              EXPECT(bytes % 256 == 0 && bytes > 0);
              ++calls;
            }
        }
      }
  // invalid shapes and arguments
  {
    size_t bytes = 0;
    const int64_t bad[][3] = {{0, 4, 1}, {4, 0, 1}, {4, 4, 0}, {4, 4, 5}, {8, 3, 4}, {-1, 4, 1}, {0x7fffff01LL, 8, 1}, {65536, 65536, 32769}};
    for (auto& b : bad) EXPECT(dion_workspace_bytes(1, &b[0], &b[1], &b[2], 0, 0, &bytes) == DION_EINVAL);
    const int64_t one = 8;
    EXPECT(dion_workspace_bytes(1, &one, &one, &one, 7, 0, &bytes) == DION_EINVAL);
    EXPECT(dion_workspace_bytes(1, &one, &one, &one, 0, 9, &bytes) == DION_EINVAL);
    EXPECT(dion_workspace_bytes(1, nullptr, nullptr, nullptr, 0, 0, &bytes) == DION_EINVAL);
    EXPECT(dion_workspace_bytes(-1, &one, &one, &one, 0, 0, &bytes) == DION_EINVAL);
    EXPECT(dion_workspace_bytes(1, &one, &one, &one, 0, 0, nullptr) == DION_EINVAL);
  }
  for (int cus : {0, 1, 2, 7, 64, 104, 228, 256, 304, 1024, 1 << 20})
    for (int batch : {0, 1, 2, 3, 5, 28, 112, 128, 129, 196, 257, 100000})
      for (int64_t r : {(int64_t)0, (int64_t)1, (int64_t)63, (int64_t)64, (int64_t)256, (int64_t)257, (int64_t)768, (int64_t)2048, (int64_t)8192, (int64_t)8193, (int64_t)32768, (int64_t)1 << 40}) {
        int w = -1;
        const int rc = dion_cholesky_grid(cus, batch, r, &w);
        if (rc == DION_OK) EXPECT(w >= 0 && (long long)w * batch <= cus);
        else EXPECT(rc == DION_EINVAL);
        ++calls;
      }
  EXPECT(dion_cholesky_grid(256, 1, 2048, nullptr) == DION_EINVAL);
  for (int code = -3; code < 40; ++code) EXPECT(dion_strerror(code) != nullptr);
  // every other entry point checks its state handle before anything else
  {
    int status = 0, bad = 0;
    float ms[8];
    EXPECT(dion_last_status(nullptr, &status, &bad) == DION_EINVAL);
    EXPECT(dion_set_orth_mode(nullptr, 0) == DION_EINVAL);
    EXPECT(dion_set_wait_limit(nullptr, 1) == DION_EINVAL);
    EXPECT(dion_set_stage_timing(nullptr, 1) == DION_EINVAL);
    EXPECT(dion_stage_times(nullptr, ms) == DION_EINVAL);
    EXPECT(dion_step(nullptr, nullptr, nullptr, nullptr, nullptr, 8, 8, 2, 0.9f, 0.1f, nullptr) == DION_EINVAL);
    EXPECT(dion_destroy_state(nullptr) == DION_OK || dion_destroy_state(nullptr) == DION_EINVAL);
  }
  // tile order of the triangular inverse
  size_t orders = 0;
  const int group_counts[] = {1, 2, 3, 4, 5, 7, 8, 15, 16, 35, 63, 64, 100, 255, 256};
  for (int nb = 2; nb <= 80; ++nb)
    for (int groups : group_counts)
      for (int S = 1; S < nb; S *= 2) {
        const int npairs = dion::inv_tree_pairs(nb, S), rounds = dion::inv_tree_rounds(nb, S, groups);
        for (int phase = 0; phase < 2; ++phase) {
          std::vector<int> taken((size_t)npairs * S * S, 0);
          std::vector<long> load(groups, 0);
          for (int wg = 0; wg < groups; ++wg)
            for (int round = 0; round < rounds; ++round) {
              int q = -1, ti = -1, tj = -1;
              if (!dion::inv_tree_tile(nb, S, phase, groups, wg, round, q, ti, tj)) continue;
              const int sd = std::min(S, nb - (2 * q * S + S));
              EXPECT(q >= 0 && q < npairs && ti >= 0 && ti < sd && tj >= 0 && tj < S);
              if (!(q >= 0 && q < npairs && ti >= 0 && ti < S && tj >= 0 && tj < S)) continue;
              ++taken[((size_t)q * S + ti) * S + tj];
              load[wg] += phase == 0 ? S - tj : ti + 1;
            }
          for (int q = 0; q < npairs; ++q) {
            const int sd = std::min(S, nb - (2 * q * S + S));
            for (int ti = 0; ti < S; ++ti)
              for (int tj = 0; tj < S; ++tj) EXPECT(taken[((size_t)q * S + ti) * S + tj] == (ti < sd ? 1 : 0));
          }
          long lo = load[0], hi = load[0];
          for (long l : load) { lo = std::min(lo, l); hi = std::max(hi, l); }
          EXPECT(hi - lo <= S);
          ++orders;
        }
      }
  printf("tile order of the triangular inverse: %zu (tile count, workgroups, level, product) cases\n", orders);
  printf("host entry points under the sanitizers: %zu calls, %d failed expectations\n", calls, failures);
  return failures == 0 ? 0 : 1;
}
