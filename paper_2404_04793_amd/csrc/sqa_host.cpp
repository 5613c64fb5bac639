// Host-only part of libsqa: status strings and the budget allocator
// (Algorithm 1 steps 5-11, Sec. 4.2.2, Appendix A.2).  No HIP calls here.
// Compiled with -ffp-contract=off: the cost sums below must be evaluated as
// written (sequential IEEE double) so that the choice between near-equal
// splits does not depend on the compiler.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <mutex>
#include <new>
#include <vector>
#include "sqa.h"

extern "C" const char* sqa_status_str(sqa_status s) {
  switch (s) {
    case SQA_OK: return "ok";
    case SQA_ERR_NULL: return "null pointer";
    case SQA_ERR_SHAPE: return "bad shape";
    case SQA_ERR_DTYPE: return "bad dtype";
    case SQA_ERR_POLICY: return "bad policy";
    case SQA_ERR_BUDGET: return "bad budget";
    case SQA_ERR_CAPACITY: return "capacity too small";
    case SQA_ERR_HIP: return "HIP error";
    case SQA_ERR_STATE: return "cache longer than its budget";
  }
  return "unknown status";
}

namespace {

// sum of squared deviations from the mean of v[lo..hi)
double run_cost(const std::vector<double>& v, int lo, int hi) {
  double s = 0.0;
  for (int t = lo; t < hi; ++t) s += v[t];
  const double mean = s / static_cast<double>(hi - lo);
  double e = 0.0;
  for (int t = lo; t < hi; ++t) { const double d = v[t] - mean; e += d * d; }
  return e;
}

}  // namespace

extern "C" sqa_status sqa_allocate_budgets(const float* cos, int n_layers, int64_t total_budget, double p,
                                           int32_t* budget_out, int8_t* group_out) {
  if (!cos || !budget_out) return SQA_ERR_NULL;
  if (n_layers < 1) return SQA_ERR_SHAPE;
  if (!(p > 0.0 && p <= 1.0) || total_budget < n_layers) return SQA_ERR_BUDGET;
  const int L = n_layers;
  for (int i = 0; i < L; ++i) if (std::isnan(cos[i])) return SQA_ERR_SHAPE;

  // layers in ascending (cosine, index) order
  std::vector<int> order(L);
  for (int i = 0; i < L; ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return cos[a] < cos[b]; });
  std::vector<double> v(L);
  for (int r = 0; r < L; ++r) v[r] = static_cast<double>(cos[order[r]]);
  std::vector<char> can_cut(L, 0);                 // a cut may sit just before rank r
  int n_cuts = 0;
  for (int r = 1; r < L; ++r) if (v[r - 1] < v[r]) { can_cut[r] = 1; ++n_cuts; }
  const int k = std::min(3, n_cuts + 1);

  std::vector<int8_t> group(L, 1);
  if (k == 2) {
    double best = 0.0; int best_c = -1;
    for (int c = 1; c < L; ++c) {
      if (!can_cut[c]) continue;
      const double cost = run_cost(v, 0, c) + run_cost(v, c, L);
      if (best_c < 0 || cost < best) { best = cost; best_c = c; }
    }
    for (int r = best_c; r < L; ++r) group[order[r]] = 2;
  } else if (k == 3) {
    double best = 0.0; int b1 = -1, b2 = -1;
    for (int c1 = 1; c1 < L - 1; ++c1) {
      if (!can_cut[c1]) continue;
      for (int c2 = c1 + 1; c2 < L; ++c2) {
        if (!can_cut[c2]) continue;
        const double cost = run_cost(v, 0, c1) + run_cost(v, c1, c2) + run_cost(v, c2, L);
        if (b1 < 0 || cost < best) { best = cost; b1 = c1; b2 = c2; }
      }
    }
    for (int r = 0; r < L; ++r) group[order[r]] = r < b1 ? 0 : (r < b2 ? 1 : 2);
  }

  std::vector<int32_t> budget(L);
  if (k == 1) {
    const int64_t base = total_budget / L, rem = total_budget % L;
    for (int i = 0; i < L; ++i) {
      const int64_t b = base + (i < rem ? 1 : 0);
      if (b > INT32_MAX) return SQA_ERR_BUDGET;
      budget[i] = static_cast<int32_t>(b);
    }
  } else {
    int n3 = 0;
    for (int i = 0; i < L; ++i) n3 += group[i] == 2;
    const int n12 = L - n3;
    const double low_d = std::floor(static_cast<double>(total_budget) * p / static_cast<double>(L));
    if (low_d < 1.0 || low_d > static_cast<double>(INT32_MAX)) return SQA_ERR_BUDGET;
    const int64_t b_low = static_cast<int64_t>(low_d);
    const int64_t rest = total_budget - static_cast<int64_t>(n3) * b_low;
    const int64_t b_high = rest / n12, rem = rest % n12;
    if (b_high + 1 > INT32_MAX) return SQA_ERR_BUDGET;
    int seen = 0;
    for (int i = 0; i < L; ++i) {
      if (group[i] == 2) budget[i] = static_cast<int32_t>(b_low);
      else { budget[i] = static_cast<int32_t>(b_high + (seen < rem ? 1 : 0)); ++seen; }
    }
  }
  for (int i = 0; i < L; ++i) budget_out[i] = budget[i];
  if (group_out) for (int i = 0; i < L; ++i) group_out[i] = group[i];
  return SQA_OK;
}

// ---- free list of block numbers for blocked K/V allocation (host book-keeping only) ----
struct sqa_block_pool {
  std::mutex mu;
  std::vector<int32_t> returned;     // blocks given back, reused last-in first-out
  std::vector<uint8_t> in_use;       // [n_blocks]
  int32_t next_fresh = 0;            // blocks next_fresh .. n_blocks-1 were never taken
  int32_t n_blocks = 0;
};

extern "C" sqa_block_pool* sqa_block_pool_create(int32_t n_blocks) {
  if (n_blocks < 1) return nullptr;
  sqa_block_pool* p = new (std::nothrow) sqa_block_pool;
  if (!p) return nullptr;
  try {
    p->in_use.assign(static_cast<size_t>(n_blocks), 0);
    p->returned.reserve(static_cast<size_t>(n_blocks));
  } catch (const std::bad_alloc&) {
    delete p;
    return nullptr;
  }
  p->n_blocks = n_blocks;
  return p;
}

extern "C" void sqa_block_pool_destroy(sqa_block_pool* pool) { delete pool; }

extern "C" int32_t sqa_block_pool_free_count(const sqa_block_pool* pool) {
  if (!pool) return -1;
  std::lock_guard<std::mutex> lock(const_cast<sqa_block_pool*>(pool)->mu);
  return static_cast<int32_t>(pool->returned.size()) + (pool->n_blocks - pool->next_fresh);
}

extern "C" sqa_status sqa_block_pool_take(sqa_block_pool* pool, int32_t n, int32_t* ids_out) {
  if (!pool || (n > 0 && !ids_out)) return SQA_ERR_NULL;
  if (n < 0) return SQA_ERR_SHAPE;
  std::lock_guard<std::mutex> lock(pool->mu);
  const int64_t free_now = static_cast<int64_t>(pool->returned.size()) + (pool->n_blocks - pool->next_fresh);
  if (n > free_now) return SQA_ERR_CAPACITY;
  for (int32_t i = 0; i < n; ++i) {
    int32_t id;
    if (pool->next_fresh < pool->n_blocks) id = pool->next_fresh++;
    else { id = pool->returned.back(); pool->returned.pop_back(); }
    pool->in_use[static_cast<size_t>(id)] = 1;
    ids_out[i] = id;
  }
  return SQA_OK;
}

extern "C" sqa_status sqa_block_pool_give(sqa_block_pool* pool, const int32_t* ids, int32_t n) {
  if (!pool || (n > 0 && !ids)) return SQA_ERR_NULL;
  if (n < 0) return SQA_ERR_SHAPE;
  std::lock_guard<std::mutex> lock(pool->mu);
  // check everything first (a block named twice in one call is caught by marking as we go and undoing)
  int32_t ok = 0;
  for (; ok < n; ++ok) {
    const int32_t id = ids[ok];
    if (id < 0 || id >= pool->n_blocks || pool->in_use[static_cast<size_t>(id)] != 1) break;
    pool->in_use[static_cast<size_t>(id)] = 2;           // seen in this call
  }
  if (ok < n) {
    for (int32_t i = 0; i < ok; ++i) pool->in_use[static_cast<size_t>(ids[i])] = 1;
    return SQA_ERR_SHAPE;
  }
  for (int32_t i = 0; i < n; ++i) {
    pool->in_use[static_cast<size_t>(ids[i])] = 0;
    pool->returned.push_back(ids[i]);
  }
  return SQA_OK;
}
