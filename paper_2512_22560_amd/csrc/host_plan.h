// Host twin of the decode partition rule (the arithmetic of plan_decode_kernel), in plain C++ with no GPU
// dependency, so that it can also be built and run on its own under the host sanitizers.
#pragma once

#include <stdint.h>

#include <algorithm>
#include <vector>

namespace rollattn {

constexpr int kPlanBlockTokens = 32;    // unit of the decode partition: two pages

// The partition rule on the host (same arithmetic as plan_decode_kernel).
struct HostPlan {
  int32_t per = 1, total = 0;
  std::vector<int32_t> prefix;   // [B + 1]
};

inline HostPlan host_plan(const int32_t* lens, int32_t batch, int32_t rows_per_b, int32_t workers) {
  HostPlan p;
  p.prefix.resize((size_t)batch + 1);
  int32_t run = 0;
  for (int32_t b = 0; b < batch; ++b) {
    p.prefix[b] = run;
    run += (lens[b] + kPlanBlockTokens - 1) / kPlanBlockTokens;
  }
  p.prefix[batch] = run;
  p.total = run * rows_per_b;
  p.per = std::max(1, (p.total + workers - 1) / workers);
  return p;
}

// Expands (per, total, prefix) into the row segments each worker walks: 6 int32 per segment,
// (worker, b, row, first block, block count, slot) with slot = -1 for a whole row (written
// directly), else the partial slot (0 or 1) the segment's result goes to.
inline int32_t expand_segments(const HostPlan& p, int32_t batch, int32_t rows_per_b, int32_t workers, int32_t* out,
                        int64_t cap_segments) {
  int64_t n_seg = 0;
  for (int32_t w = 0; w < workers; ++w) {
    const int64_t x0 = (int64_t)w * p.per;
    if (x0 >= p.total) break;
    int32_t left = (int32_t)std::min<int64_t>(p.per, p.total - x0);
    // largest b with rows_per_b * prefix[b] <= x0
    int32_t lo = 0, hi = batch;
    while (hi - lo > 1) {
      const int32_t mid = (lo + hi) >> 1;
      if ((int64_t)rows_per_b * p.prefix[mid] <= x0) lo = mid; else hi = mid;
    }
    int32_t b = lo, n = p.prefix[b + 1] - p.prefix[b];
    const int32_t rem = (int32_t)(x0 - (int64_t)rows_per_b * p.prefix[b]);
    int32_t r = rem / n, blk = rem % n;
    bool first = true;
    while (left > 0) {
      const int32_t cnt = std::min(left, n - blk);
      if (out && n_seg < cap_segments) {
        int32_t* o = out + 6 * n_seg;
        o[0] = w; o[1] = b; o[2] = r; o[3] = blk; o[4] = cnt;
        o[5] = (blk == 0 && cnt == n) ? -1 : (first ? 0 : 1);
      }
      ++n_seg;
      first = false;
      left -= cnt;
      if (left > 0) {
        blk = 0;
        if (++r == rows_per_b) {
          r = 0;
          do {
            ++b;
            n = p.prefix[b + 1] - p.prefix[b];
          } while (n == 0);
        }
      }
    }
  }
  return (int32_t)std::min<int64_t>(n_seg, INT32_MAX);
}

}  // namespace rollattn
