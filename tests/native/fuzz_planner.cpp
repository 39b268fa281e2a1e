// Random batches through the host planner, built with AddressSanitizer and UBSan by
// tests/test_host_sanitizers.py: every (request, kv head, query row) must get each of its
// visible keys exactly once from the work items, whatever the knobs.
#include <cstdio>
#include <cstdlib>
#include <random>
#include "efim_internal.h"

using namespace efim;
int main() {
  std::mt19937 rng(7);
  long items_total = 0;
  for (int iter = 0; iter < 400; ++iter) {
    int batch = 1 + rng() % 12;
    std::vector<int32_t> c(batch), n(batch);
    for (int r = 0; r < batch; ++r) {
      int kind = rng() % 6;
      c[r] = kind == 0 ? 0 : (kind == 1 ? rng() % 70 : (kind == 2 ? rng() % 9000 : rng() % 40000));
      n[r] = (rng() % 5 == 0) ? 0 : (rng() % 3 == 0 ? 1 + rng() % 600 : 1 + rng() % 40);
    }
    static const int hq[] = {1, 4, 8, 28, 32, 14, 6}, hkv[] = {1, 4, 2, 4, 8, 2, 1};
    int h = rng() % 7;
    efim_batch_t b{};
    b.batch = batch; b.cached_len = c.data(); b.new_len = n.data();
    b.num_q_heads = hq[h]; b.num_kv_heads = hkv[h]; b.head_dim = (rng() & 1) ? 64 : 128;
    b.page_size = 8 << (rng() % 6);
    int maxp = 0; for (int r = 0; r < batch; ++r) maxp = std::max(maxp, (c[r] + n[r] + b.page_size - 1) / b.page_size);
    b.max_pages_per_req = std::max(1, maxp); b.num_pages = 1 << 24;
    b.block_table = reinterpret_cast<const int32_t*>(0x1000);
    static const int splits[] = {-1, -1, 0, 64, 128, 512}; static const int tiles[] = {0, 0, 128, 256};
    tuning().split_kv = splits[rng() % 6]; tuning().row_tile = tiles[rng() % 4]; tuning().xcd_grouping = rng() & 1;
    int64_t total = 0;
    int rc = validate_batch(&b, &total);
    if (rc != EFIM_OK) { printf("validate rc %d at iter %d\n", rc, iter); return 1; }
    Plan plan;
    int slots = (rng() & 1) ? 256 : 512;
    build_plan(&b, slots, &plan);
    items_total += (long)plan.items.size();
    // coverage: every (req, kv head, row) x key range is covered exactly once
    const int g = b.num_q_heads / b.num_kv_heads;
    for (int r = 0; r < batch; ++r) {
      if (n[r] == 0) continue;
      for (int kh = 0; kh < b.num_kv_heads; ++kh) {
        std::vector<int> rows(n[r] * g, 0);
        for (const WorkItem& w : plan.items) {
          if (w.row_count == 0 || w.req != r || w.kv_head != kh) continue;
          if (w.row_begin < 0 || w.row_begin + w.row_count > n[r] * g || w.key_begin < 0 || w.key_end <= w.key_begin) { printf("bad item iter %d\n", iter); return 1; }
          for (int i = 0; i < w.row_count; ++i) {
            int row = w.row_begin + i; int vis = c[r] + row / g + 1;
            int lo = std::min(w.key_begin, vis), hi = std::min(w.key_end, vis);
            rows[row] += hi - lo;
          }
        }
        for (int row = 0; row < n[r] * g; ++row)
          if (rows[row] != c[r] + row / g + 1) { printf("coverage iter %d req %d head %d row %d: %d vs %d\n", iter, r, kh, row, rows[row], c[r] + row / g + 1); return 1; }
      }
    }
  }
  printf("planner ok, %ld items\n", items_total);
  return 0;
}
