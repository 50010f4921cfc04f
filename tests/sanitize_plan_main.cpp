// Driver for the host twin of the decode partition rule, built with -fsanitize=address,undefined by
// tests/test_host_sanitizers.py.  stdin: rows_per_b workers batch, then batch context lengths.
// stdout: per total n_segments, then six integers per segment.
#include <cstdio>
#include <vector>

#include "host_plan.h"

int main() {
  int rows_per_b = 0, workers = 0, batch = 0;
  if (std::scanf("%d %d %d", &rows_per_b, &workers, &batch) != 3 || batch < 0) return 2;
  std::vector<int32_t> lens((size_t)batch);
  for (int b = 0; b < batch; ++b)
    if (std::scanf("%d", &lens[b]) != 1) return 2;
  const rollattn::HostPlan p = rollattn::host_plan(lens.data(), batch, rows_per_b, workers);
  // capacity exactly as the library sizes it: every worker boundary and every row end closes one segment
  const int64_t cap = (int64_t)workers + (int64_t)batch * rows_per_b;
  std::vector<int32_t> segs((size_t)(6 * cap));
  const int32_t n = rollattn::expand_segments(p, batch, rows_per_b, workers, segs.data(), cap);
  std::printf("%d %d %d\n", p.per, p.total, n);
  for (int32_t i = 0; i < n && i < cap; ++i)
    std::printf("%d %d %d %d %d %d\n", segs[6 * i], segs[6 * i + 1], segs[6 * i + 2], segs[6 * i + 3], segs[6 * i + 4], segs[6 * i + 5]);
  return 0;
}
