// Session pool: rewrites infilling requests from FIM (PSM) order to EFIM order and reports
// what a prefix-matching KV cache reuses (EFIM Sec. 3.1, steps 1-5).  Host code only.
#include <algorithm>
#include <cstdint>
#include <mutex>
#include <new>
#include <unordered_map>
#include <vector>

#include "efim.h"

namespace {

using Tokens = std::vector<int32_t>;

struct Session {
  Tokens prefix;  // the part between <P> and <S> of the layout in use
  Tokens suffix;
  Tokens prompt;  // last prompt built for this user
};

bool starts_with(const int32_t* seq, int64_t n, const Tokens& head) {
  return n >= (int64_t)head.size() && std::equal(head.begin(), head.end(), seq);
}

bool same(const int32_t* seq, int64_t n, const Tokens& t) {
  return n == (int64_t)t.size() && std::equal(t.begin(), t.end(), seq);
}

}  // namespace

struct efim_session_pool {
  int32_t tok_p, tok_s, tok_m;
  int32_t granularity;
  bool always_psm;
  std::mutex lock;
  std::unordered_map<uint64_t, Session> sessions;

  bool is_marker(int32_t t) const { return t == tok_p || t == tok_s || t == tok_m; }
  bool clean(const int32_t* seq, int64_t n) const {
    for (int64_t i = 0; i < n; ++i)
      if (is_marker(seq[i])) return false;
    return true;
  }
};

extern "C" {

efim_session_pool_t* efim_session_pool_create(int32_t tok_p, int32_t tok_s, int32_t tok_m,
                                              int32_t reuse_granularity, int32_t always_psm) {
  if (tok_p == tok_s || tok_p == tok_m || tok_s == tok_m || reuse_granularity < 1) return nullptr;
  efim_session_pool* pool = new (std::nothrow) efim_session_pool;
  if (!pool) return nullptr;
  pool->tok_p = tok_p;
  pool->tok_s = tok_s;
  pool->tok_m = tok_m;
  pool->granularity = reuse_granularity;
  pool->always_psm = always_psm != 0;
  return pool;
}

void efim_session_pool_destroy(efim_session_pool_t* pool) { delete pool; }

int efim_session_transform(efim_session_pool_t* pool, uint64_t user, const int32_t* prefix,
                           int64_t n_prefix, const int32_t* suffix, int64_t n_suffix,
                           efim_prompt_info_t* info) {
  if (!pool || !info || n_prefix < 0 || n_suffix < 0) return EFIM_ERR_INVALID_ARG;
  if ((n_prefix > 0 && !prefix) || (n_suffix > 0 && !suffix)) return EFIM_ERR_INVALID_ARG;
  if (!pool->clean(prefix, n_prefix) || !pool->clean(suffix, n_suffix)) return EFIM_ERR_INVALID_ARG;
  try {
    std::lock_guard<std::mutex> guard(pool->lock);
    auto found = pool->sessions.find(user);
    int64_t common_len = n_prefix;  // PSM: the whole prefix sits between <P> and <S>
    int32_t order = EFIM_ORDER_PSM;
    if (found == pool->sessions.end()) {
      Session fresh;
      fresh.prefix.assign(prefix, prefix + n_prefix);
      fresh.suffix.assign(suffix, suffix + n_suffix);
      found = pool->sessions.emplace(user, std::move(fresh)).first;
    } else {
      Session& s = found->second;
      const bool suffix_kept = same(suffix, n_suffix, s.suffix);
      const bool grew = n_prefix > (int64_t)s.prefix.size() && starts_with(prefix, n_prefix, s.prefix);
      if (suffix_kept && grew && !pool->always_psm) {
        order = EFIM_ORDER_EFIM;
        common_len = (int64_t)s.prefix.size();
      } else if (!(suffix_kept && same(prefix, n_prefix, s.prefix))) {
        s.prefix.assign(prefix, prefix + n_prefix);
        s.suffix.assign(suffix, suffix + n_suffix);
      }
    }
    Session& s = found->second;
    Tokens prompt;
    prompt.reserve((size_t)(n_prefix + n_suffix + 3));
    prompt.push_back(pool->tok_p);
    prompt.insert(prompt.end(), prefix, prefix + common_len);
    prompt.push_back(pool->tok_s);
    prompt.insert(prompt.end(), suffix, suffix + n_suffix);
    prompt.push_back(pool->tok_m);
    prompt.insert(prompt.end(), prefix + common_len, prefix + n_prefix);

    const int64_t limit = std::min<int64_t>((int64_t)s.prompt.size(), (int64_t)prompt.size() - 1);
    int64_t match = 0;
    while (match < limit && s.prompt[(size_t)match] == prompt[(size_t)match]) ++match;
    match -= match % pool->granularity;

    info->order = order;
    info->reserved = 0;
    info->common_len = common_len;
    info->inc_len = n_prefix - common_len;
    info->suffix_len = n_suffix;
    info->prompt_len = (int64_t)prompt.size();
    info->cached_len = match;
    info->new_len = (int64_t)prompt.size() - match;
    s.prompt.swap(prompt);
    return EFIM_OK;
  } catch (const std::bad_alloc&) {
    return EFIM_ERR_INVALID_ARG;
  }
}

int64_t efim_session_prompt(efim_session_pool_t* pool, uint64_t user, int32_t* dst, int64_t capacity) {
  if (!pool || capacity < 0 || (capacity > 0 && !dst)) return EFIM_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> guard(pool->lock);
  auto found = pool->sessions.find(user);
  if (found == pool->sessions.end()) return 0;
  const Tokens& prompt = found->second.prompt;
  const int64_t n = std::min<int64_t>(capacity, (int64_t)prompt.size());
  std::copy(prompt.begin(), prompt.begin() + n, dst);
  return (int64_t)prompt.size();
}

int efim_session_drop(efim_session_pool_t* pool, uint64_t user) {
  if (!pool) return EFIM_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> guard(pool->lock);
  return pool->sessions.erase(user) ? 1 : 0;
}

int64_t efim_session_count(efim_session_pool_t* pool) {
  if (!pool) return EFIM_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> guard(pool->lock);
  return (int64_t)pool->sessions.size();
}

}  // extern "C"
