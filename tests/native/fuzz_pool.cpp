// Random request streams through the session pool, built with AddressSanitizer and UBSan by
// tests/test_host_sanitizers.py: lengths reported must be consistent and every prompt must
// hold the request's tokens plus the three markers.
#include <cstdio>
#include <random>
#include <vector>
#include "efim.h"
int main() {
  std::mt19937 rng(11);
  for (int variant = 0; variant < 4; ++variant) {
    efim_session_pool_t* pool = efim_session_pool_create(1, 2, 3, variant & 1 ? 16 : 1, variant >> 1);
    if (!pool) return 1;
    std::vector<std::vector<int32_t>> pre(8), suf(8);
    for (int step = 0; step < 20000; ++step) {
      uint64_t user = rng() % 8;
      int action = rng() % 10;
      auto tok = [&]() { return (int32_t)(4 + rng() % 50); };
      if (action < 5) { int k = rng() % 20; for (int i = 0; i < k; ++i) pre[user].push_back(tok()); }       // extend the prefix
      else if (action < 6) { suf[user].assign(rng() % 30, 0); for (auto& t : suf[user]) t = tok(); }        // new suffix
      else if (action < 7) { if (!pre[user].empty()) pre[user].resize(rng() % pre[user].size()); }          // shrink
      else if (action < 8) { if (!pre[user].empty()) pre[user][rng() % pre[user].size()] = tok(); }         // edit
      else if (action < 9) { efim_session_drop(pool, user); }
      efim_prompt_info_t info;
      int rc = efim_session_transform(pool, user, pre[user].empty() ? nullptr : pre[user].data(), (int64_t)pre[user].size(),
                                      suf[user].empty() ? nullptr : suf[user].data(), (int64_t)suf[user].size(), &info);
      if (rc != EFIM_OK) { printf("rc %d\n", rc); return 1; }
      if (info.prompt_len != info.common_len + info.suffix_len + info.inc_len + 3 || info.new_len < 1 ||
          info.cached_len + info.new_len != info.prompt_len) { printf("bad info at %d\n", step); return 1; }
      std::vector<int32_t> prompt((size_t)info.prompt_len + 2, -1);
      int64_t n = efim_session_prompt(pool, user, prompt.data(), (int64_t)prompt.size());
      if (n != info.prompt_len) { printf("prompt length\n"); return 1; }
      // the prompt holds exactly the prefix and suffix tokens plus the three markers
      if ((int64_t)(pre[user].size() + suf[user].size()) + 3 != n) { printf("token count\n"); return 1; }
      if (rng() % 50 == 0) { int64_t m = efim_session_prompt(pool, user, prompt.data(), 3); (void)m; }
    }
    if (efim_session_count(pool) > 8) return 1;
    efim_session_pool_destroy(pool);
  }
  // invalid arguments
  efim_prompt_info_t info;
  if (efim_session_transform(nullptr, 0, nullptr, 0, nullptr, 0, &info) == EFIM_OK) return 1;
  efim_session_pool_destroy(nullptr);
  printf("session pool ok\n");
  return 0;
}
