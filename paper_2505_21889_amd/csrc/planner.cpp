// Host-side planner: turns the ragged batch into a list of workgroup-sized work items.
//
// Row space of a (request, kv head) pair: row = token * g + head_in_group with g = Hq/Hkv,
// so rows of one token are adjacent and the causal limit C_r + token + 1 grows with the row.
// A query tile is a run of `rows_per_item` such rows; it needs keys [0, C_r + last_token + 1).
// When there are too few tiles to fill the device, or some are much longer than the average,
// the key range of a tile is cut into chunks (multiples of the 64-key LDS tile) whose partial
// results a merge pass combines in a fixed order.
#include <algorithm>
#include <cstring>
#include <functional>

#include "efim_internal.h"

namespace efim {

Tuning& tuning() {
  static Tuning t;
  return t;
}

int validate_batch(const efim_batch_t* b, int64_t* total_new) {
  if (!b) return EFIM_ERR_INVALID_ARG;
  if (b->batch < 0 || b->num_q_heads <= 0 || b->num_kv_heads <= 0 || b->head_dim <= 0 ||
      b->page_size <= 0 || b->max_pages_per_req < 0 || b->num_pages < 0)
    return EFIM_ERR_INVALID_ARG;
  if (b->num_q_heads % b->num_kv_heads != 0) return EFIM_ERR_INVALID_ARG;
  if (b->head_dim != 64 && b->head_dim != 128) return EFIM_ERR_UNSUPPORTED;
  // pages are powers of two; a 1 KB gather (4 or 8 tokens of one head) must not cross one
  if (b->page_size < kMinPageSize || b->page_size > kMaxPageSize || (b->page_size & (b->page_size - 1)) != 0)
    return EFIM_ERR_UNSUPPORTED;
  if (b->num_q_heads / b->num_kv_heads > 64) return EFIM_ERR_UNSUPPORTED;
  int64_t total = 0;
  if (b->batch > 0) {
    if (!b->cached_len || !b->new_len) return EFIM_ERR_INVALID_ARG;
    for (int r = 0; r < b->batch; ++r) {
      const int64_t c = b->cached_len[r], n = b->new_len[r];
      if (c < 0 || n < 0) return EFIM_ERR_INVALID_ARG;
      if (c + n > (int64_t)1 << 30) return EFIM_ERR_UNSUPPORTED;
      if (n > 0) {
        const int64_t pages = (c + n + b->page_size - 1) / b->page_size;
        if (pages > b->max_pages_per_req || pages > b->num_pages) return EFIM_ERR_INVALID_ARG;
      }
      total += n;
    }
    if (total * b->num_q_heads > (int64_t)1 << 31) return EFIM_ERR_UNSUPPORTED;
    if (total > 0 && !b->block_table) return EFIM_ERR_INVALID_ARG;
  }
  if (total_new) *total_new = total;
  return EFIM_OK;
}

namespace {

struct Tile {
  int32_t req, kv_head, row_begin, row_count, key_end;
  int32_t ktiles;  // ceil(key_end / kKeyTile)
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

void build_plan(const efim_batch_t* b, int num_slots, Plan* plan) {
  const int g = b->num_q_heads / b->num_kv_heads;
  const int D = b->head_dim;
  plan->reqs.clear();
  plan->items.clear();
  plan->merges.clear();
  plan->num_partial_slots = 0;

  int64_t row = 0;
  int64_t max_rows = 0;
  for (int r = 0; r < b->batch; ++r) {
    ReqInfo ri{b->cached_len[r], b->new_len[r], (int32_t)row, 0};
    plan->reqs.push_back(ri);
    row += b->new_len[r];
    max_rows = std::max<int64_t>(max_rows, (int64_t)g * b->new_len[r]);
  }
  // Query-row tile of a workgroup: 128 rows (each of the 4 waves owns 32; two workgroups per
  // compute unit, suits steps bound by HBM) or, when some kv head has more rows than that and
  // the step is therefore compute-heavy, 256 rows (8 waves of 32; one workgroup per unit).
  // "Compute-heavy" = arithmetic intensity (flop per K/V/Q/O byte) above the machine balance
  // of about 315 flop/byte (2.5 PFLOP/s over 8 TB/s).
  const Tuning& tn0 = tuning();
  double flops = 0.0, bytes = 0.0;
  for (int r = 0; r < b->batch; ++r) {
    const double n = b->new_len[r], c = b->cached_len[r];
    if (n == 0) continue;
    flops += 4.0 * D * b->num_q_heads * n * (c + 0.5 * (n + 1));
    bytes += 4.0 * D * ((c + n) * b->num_kv_heads + n * b->num_q_heads);
  }
  // A step bound by HBM also takes the 256-row configuration when it has at least two such
  // tiles per compute unit: the tiles then balance over the 256 slots without cutting key
  // ranges (no merge pass), and that configuration gathers two tiles ahead.
  int M = 128;
  if (tn0.row_tile == 256) {
    M = 256;
  } else if (tn0.row_tile == 0) {
    int64_t wide_tiles = 0;
    for (int r = 0; r < b->batch; ++r)
      wide_tiles += (int64_t)b->num_kv_heads * (((int64_t)g * b->new_len[r] + 255) / 256);
    if ((max_rows > 128 && flops > 315.0 * bytes) || wide_tiles >= num_slots) M = 256;
  }
  plan->rows_per_item = M;
  if (M == 256) num_slots = std::max(1, num_slots / 2);  // 8-wave workgroups: one per compute unit

  std::vector<Tile> tiles;
  int64_t total_cost = 0;
  int64_t max_cost = 0;
  for (int r = 0; r < b->batch; ++r) {
    const int64_t n = b->new_len[r], c = b->cached_len[r];
    if (n == 0) continue;
    const int64_t rows = n * g;
    for (int h = 0; h < b->num_kv_heads; ++h) {
      for (int64_t r0 = 0; r0 < rows; r0 += M) {
        Tile t;
        t.req = r;
        t.kv_head = h;
        t.row_begin = (int32_t)r0;
        t.row_count = (int32_t)std::min<int64_t>(M, rows - r0);
        const int64_t last_token = (r0 + t.row_count - 1) / g;
        t.key_end = (int32_t)(c + last_token + 1);
        t.ktiles = (t.key_end + kKeyTile - 1) / kKeyTile;
        tiles.push_back(t);
        total_cost += t.ktiles + 4;
        max_cost = std::max<int64_t>(max_cost, t.ktiles + 4);
      }
    }
  }

  // Split policy.  chunk = key tiles per work item (0 = no split).  A workgroup slot's fair
  // share of the whole step is `avg`; a tile much longer than that would finish last, so long
  // tiles are cut into pieces.  Which piece length is best depends on how the pieces pack
  // into the slots (one piece too many costs a whole extra round with most slots idle), so
  // for steps of moderate size the candidates are tried on a model of the device: pieces
  // handed out longest first to `num_slots` slots, a fixed start-up cost per piece.
  const Tuning& tn = tuning();
  constexpr int64_t kStartCost = 4;  // start-up of a work item, in units of one key tile
  auto pieces_of = [&](const Tile& t, int64_t chunk) {
    return (chunk > 0 && 10 * (int64_t)t.ktiles > 13 * chunk) ? (int)((t.ktiles + chunk - 1) / chunk) : 1;
  };
  int64_t chunk = 0;
  if (tn.split_kv > 0) {
    chunk = std::max(1, tn.split_kv / kKeyTile);
  } else if (tn.split_kv < 0 && !tiles.empty()) {
    const double avg = (double)total_cost / std::max(1, num_slots);
    if ((double)max_cost > 1.3 * avg) {
      chunk = (int64_t)std::max(4.0, avg);
      if (tiles.size() <= (size_t)4 * num_slots) {
        // Quick estimate of a candidate: the pieces run in rounds of `num_slots`, a round
        // lasts as long as the longest piece.  The most promising candidates are then played
        // through: pieces handed out longest first, each to the slot that is free first, the
        // step taking as long as the fullest slot.  (A finer model with bandwidth sharing
        // between busy slots was fitted to chunk sweeps on the device and picked worse plans.)
        auto estimate = [&](int64_t c) {
          int64_t pieces = 0, longest = 0;
          for (const Tile& t : tiles) {
            const int n = pieces_of(t, c);
            pieces += n;
            longest = std::max<int64_t>(longest, (t.ktiles + n - 1) / n);
          }
          const int64_t rounds = (pieces + num_slots - 1) / num_slots;
          return rounds * (longest + kStartCost);
        };
        std::vector<int64_t> costs, load;
        auto makespan = [&](int64_t c) {
          costs.clear();
          for (const Tile& t : tiles) {
            const int n = pieces_of(t, c);
            const int64_t per = (t.ktiles + n - 1) / n;
            for (int64_t done = 0; done < t.ktiles; done += per)
              costs.push_back(std::min<int64_t>(per, t.ktiles - done) + kStartCost);
          }
          std::sort(costs.begin(), costs.end(), std::greater<int64_t>());
          load.assign((size_t)num_slots, 0);  // min-heap of slot loads
          auto cmp = std::greater<int64_t>();
          for (int64_t w : costs) {
            std::pop_heap(load.begin(), load.end(), cmp);
            load.back() += w;
            std::push_heap(load.begin(), load.end(), cmp);
          }
          return *std::max_element(load.begin(), load.end());
        };
        const int64_t lo = std::max<int64_t>(4, (int64_t)(0.5 * avg));
        const int64_t hi = std::max<int64_t>(lo, max_cost - kStartCost);
        const int64_t step = std::max<int64_t>(1, (hi - lo) / 64);
        std::vector<std::pair<int64_t, int64_t>> ranked;  // (estimate, candidate)
        for (int64_t c = lo; c <= hi; c += step) ranked.push_back({estimate(c), c});
        std::sort(ranked.begin(), ranked.end());
        int64_t best = makespan(chunk), best_chunk = chunk;
        for (size_t i = 0; i < ranked.size() && i < 6; ++i) {
          const int64_t c = ranked[i].second;
          const int64_t m = makespan(c);
          if (m < best || (m == best && c > best_chunk)) { best = m; best_chunk = c; }
        }
        chunk = best_chunk;
      }
    }
  }

  struct Pending { WorkItem w; int64_t cost; int64_t group; };
  std::vector<Pending> pend;
  pend.reserve(tiles.size() * 2);
  int64_t slot = 0;
  for (const Tile& t : tiles) {
    const int nsplit = pieces_of(t, chunk);
    const int64_t group = (int64_t)t.req * b->num_kv_heads + t.kv_head;
    if (nsplit == 1) {
      WorkItem w{t.req, t.kv_head, t.row_begin, t.row_count, 0, t.key_end, -1, -1};
      pend.push_back({w, t.ktiles + 4, group});
    } else {
      const int per = (t.ktiles + nsplit - 1) / nsplit;  // key tiles per chunk
      MergeItem m{t.req, t.kv_head, t.row_begin, t.row_count, (int32_t)slot, 0, plan->reqs[t.req].row_start, 0};
      int made = 0;
      for (int s = 0; s < nsplit; ++s) {
        const int64_t kb = (int64_t)s * per * kKeyTile;
        if (kb >= t.key_end) break;
        const int64_t ke = std::min<int64_t>(t.key_end, kb + (int64_t)per * kKeyTile);
        WorkItem w{t.req, t.kv_head, t.row_begin, t.row_count, (int32_t)kb, (int32_t)ke,
                   (int32_t)(slot + made), (int32_t)plan->merges.size()};
        pend.push_back({w, (ke - kb + kKeyTile - 1) / kKeyTile + 4, group});
        ++made;
      }
      m.nsplit = made;
      slot += made;
      plan->merges.push_back(m);
    }
  }
  plan->num_partial_slots = slot;

  // Order: heaviest first.  With XCD grouping, items that read the same K/V (same request and
  // kv head) are given workgroup ids congruent modulo 8, so they run on one XCD and share its
  // L2; the groups are spread over the 8 XCDs by greedy load balancing.
  constexpr int kXcds = 8;
  auto by_cost = [](const Pending& a, const Pending& c) { return a.cost > c.cost; };
  const int64_t ngroups = (int64_t)b->batch * b->num_kv_heads;
  bool group_xcd = tn.xcd_grouping && pend.size() >= (size_t)4 * kXcds;
  if (group_xcd) {
    // only worthwhile when several items share a group
    group_xcd = pend.size() > (size_t)tiles.size() || tiles.size() > (size_t)ngroups;
  }
  if (!group_xcd) {
    std::stable_sort(pend.begin(), pend.end(), by_cost);
    plan->items.reserve(pend.size());
    for (auto& p : pend) plan->items.push_back(p.w);
  } else {
    std::vector<int64_t> gcost(ngroups, 0), gmax(ngroups, 0);
    for (auto& p : pend) {
      gcost[p.group] += p.cost;
      gmax[p.group] = std::max<int64_t>(gmax[p.group], p.cost);
    }
    std::vector<int64_t> order(ngroups);
    for (int64_t i = 0; i < ngroups; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t c) { return gcost[a] > gcost[c]; });
    std::vector<int> gx(ngroups, 0);
    int64_t load[kXcds] = {0};
    for (int64_t gi : order) {
      if (gcost[gi] == 0) continue;
      int best = 0;
      for (int x = 1; x < kXcds; ++x) if (load[x] < load[best]) best = x;
      gx[gi] = best;
      load[best] += gcost[gi];
    }
    // When a (request, kv head) pair has many query tiles (long new sequences), inside one XCD
    // the items run group after group (heaviest group first, and inside a group
    // heaviest item first): the workgroups resident at any time then read the K/V of only one
    // or two (request, kv head) pairs, which fits the 4 MB L2, instead of a slice of all of them.
    // With few query tiles per pair there is little to share and plain heaviest-first order
    // balances better.
    int64_t live_groups = 0;
    for (int64_t gi = 0; gi < ngroups; ++gi) live_groups += gcost[gi] > 0;
    const bool group_major = (int64_t)tiles.size() >= 4 * std::max<int64_t>(1, live_groups);
    std::vector<Pending> per[kXcds];
    for (auto& p : pend) per[gx[p.group]].push_back(p);
    size_t longest = 0;
    for (int x = 0; x < kXcds; ++x) {
      if (!group_major) {
        std::stable_sort(per[x].begin(), per[x].end(), by_cost);
        longest = std::max(longest, per[x].size());
        continue;
      }
      // (groups by their LONGEST item first, then by their whole cost: a request with a long
      // cached context and few new rows is a light group of one or two very long items, and an
      // item of 120 key tiles that starts last is a tenth of the whole step on its own)
      std::stable_sort(per[x].begin(), per[x].end(), [&](const Pending& a, const Pending& c) {
        if (a.group != c.group) {
          if (gmax[a.group] != gmax[c.group]) return gmax[a.group] > gmax[c.group];
          if (gcost[a.group] != gcost[c.group]) return gcost[a.group] > gcost[c.group];
          return a.group < c.group;
        }
        return a.cost > c.cost;
      });
      longest = std::max(longest, per[x].size());
    }
    plan->items.reserve(longest * kXcds);
    const WorkItem nothing{0, 0, 0, 0, 0, 0, -1, -1};
    for (size_t k = 0; k < longest; ++k)
      for (int x = 0; x < kXcds; ++x) plan->items.push_back(k < per[x].size() ? per[x][k].w : nothing);
    while (!plan->items.empty() && plan->items.back().row_count == 0) plan->items.pop_back();
  }

  plan->max_item_rows = 0;
  for (const WorkItem& w : plan->items) plan->max_item_rows = std::max(plan->max_item_rows, (int)w.row_count);

  // Layout of the staged header and of the device workspace.
  size_t off = 0;
  plan->off_items = off;
  off = align_up(off + plan->items.size() * sizeof(DevItem), 256);
  plan->off_merges = off;
  off = align_up(off + plan->merges.size() * sizeof(MergeItem), 256);
  plan->header_bytes = off;
  // A partial-result slot holds as many rows as the largest work item has (in steps of 32), not
  // a whole row tile: decode-like steps cut every key range and have a handful of rows per item.
  plan->partial_rows = std::min(M, (plan->max_item_rows + 31) / 32 * 32);
  if (plan->partial_rows < 32) plan->partial_rows = 32;
  const size_t prows = (size_t)plan->partial_rows;
  off = 0;
  plan->off_part_o = off;
  // per row: D binary16 values, then (max, sum, scale, unused) as fp32
  off = align_up(off + (size_t)plan->num_partial_slots * prows * D * sizeof(uint16_t), 256);
  plan->off_part_ml = off;
  off = align_up(off + (size_t)plan->num_partial_slots * prows * 4 * sizeof(float), 256);
  plan->total_bytes = off < 256 ? 256 : off;  // never zero, so callers always pass a real buffer
}

}  // namespace efim
