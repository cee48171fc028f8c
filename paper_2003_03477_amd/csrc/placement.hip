// Placement of embedding tables on parameter servers (host code only, no device work).
// Section 3.1, "Embedding PS": tables are spread over the embedding PSs so that every PS carries
// a similar look-up cost, the cost of each table being profiled beforehand and the assignment
// being a bin-packing problem; a table too large for one PS is partitioned (here: by rows) and
// its parts are placed like tables of their own, each pooling what it owns.
// The packing is the longest-processing-time rule: items by decreasing cost, each to the PS
// with the least load so far (makespan at most 4/3 - 1/(3m) of the optimum on m PSs).
#include <algorithm>
#include <vector>

#include "../../include/shadowsync.h"

extern "C" int ss_plan_placement(int32_t num_tables, const int64_t* rows, const double* cost,
                                 int32_t num_ps, int64_t max_rows_per_shard, ss_shard* out_shards,
                                 int32_t capacity, int32_t* out_num_shards, double* out_ps_cost) {
  if (num_tables < 1 || !rows || !cost || num_ps < 1 || !out_num_shards) return SS_EINVAL;
  std::vector<ss_shard> sh;
  for (int32_t t = 0; t < num_tables; ++t) {
    if (rows[t] < 1 || !(cost[t] >= 0.0)) return SS_EINVAL;
    int64_t parts = 1;
    if (max_rows_per_shard > 0) parts = (rows[t] + max_rows_per_shard - 1) / max_rows_per_shard;
    const int64_t per = (rows[t] + parts - 1) / parts;
    for (int64_t first = 0; first < rows[t]; first += per) {
      ss_shard s;
      s.table = t;
      s.first_row = first;
      s.rows = std::min(per, rows[t] - first);
      s.cost = cost[t] * (double)s.rows / (double)rows[t];   // look-ups spread evenly over rows
      s.ps = -1;
      sh.push_back(s);
    }
  }
  *out_num_shards = (int32_t)sh.size();
  if ((int64_t)sh.size() > capacity || !out_shards) return SS_ENOMEM;
  std::vector<int> order(sh.size());
  for (size_t i = 0; i < order.size(); ++i) order[i] = (int)i;
  // by decreasing cost; equal costs keep (table, first row) order, so the plan is unique
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return sh[a].cost > sh[b].cost; });
  std::vector<double> load((size_t)num_ps, 0.0);
  for (int i : order) {
    int best = 0;
    for (int p = 1; p < num_ps; ++p)
      if (load[p] < load[best]) best = p;
    sh[i].ps = best;
    load[best] += sh[i].cost;
  }
  for (size_t i = 0; i < sh.size(); ++i) out_shards[i] = sh[i];
  if (out_ps_cost)
    for (int p = 0; p < num_ps; ++p) out_ps_cost[p] = load[p];
  return SS_OK;
}
