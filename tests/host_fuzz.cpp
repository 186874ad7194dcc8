// Random allocator workload for a sanitizer build of the host half of the library
// (built and run by tests/test_host_sanitizers.py with -fsanitize=address,undefined).
// Exercises every host entry point, valid and invalid arguments alike, and checks the
// pool's own accounting after each batch of operations.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <utility>
#include <vector>

#include "jenga.h"

#define CHECK(c)                                                           \
  do {                                                                     \
    if (!(c)) {                                                            \
      std::fprintf(stderr, "host_fuzz: check failed at line %d: %s\n", __LINE__, #c); \
      return 1;                                                            \
    }                                                                      \
  } while (0)

int main(int argc, char** argv) {
  const unsigned seed = argc > 1 ? unsigned(std::atoi(argv[1])) : 1u;
  const int n_ops = argc > 2 ? std::atoi(argv[2]) : 200000;
  std::mt19937 rng(seed);
  jenga_kind_desc kinds[3] = {};
  kinds[0] = {JENGA_FULL, JENGA_BF16, 3, 2, 64, 16, 0, 0, 0};          // 3 * 8 KiB = 24 KiB
  kinds[1] = {JENGA_WINDOW, JENGA_BF16, 1, 2, 64, 16, 48, 0, 0};       // 8 KiB
  kinds[2] = {JENGA_OPAQUE, JENGA_F32, 1, 0, 0, 1, 0, 0, 16 * 1024};   // 16 KiB
  int64_t lcm = 0;
  CHECK(jenga_lcm_page_bytes(kinds, 3, &lcm) == JENGA_OK && lcm == 48 * 1024);
  jenga_pool* pool = nullptr;
  const int64_t n_large = 40;
  // an OPAQUE page is one unit: any other tokens_per_page (0 would divide by zero in the
  // request layer) is refused at creation
  for (int32_t bad_t : {0, -1, 16}) {
    jenga_kind_desc bad[3] = {kinds[0], kinds[1], kinds[2]};
    bad[2].tokens_per_page = bad_t;
    int64_t l = 0;
    CHECK(jenga_lcm_page_bytes(bad, 3, &l) == JENGA_ERR_INVALID);
    CHECK(jenga_pool_create(nullptr, n_large * lcm, lcm, bad, 3, &pool) == JENGA_ERR_INVALID && pool == nullptr);
  }
  CHECK(jenga_pool_create(nullptr, n_large * lcm + 100, lcm, kinds, 3, &pool) == JENGA_OK);

  std::vector<std::pair<int, int>> used, cached;
  std::vector<int64_t> requests;
  int64_t clock = 0;
  for (int op = 0; op < n_ops; ++op) {
    ++clock;
    const unsigned u = rng() % 100;
    // allocations made through the request layer may have evicted pages this driver kept as
    // cached: forget those
    for (size_t j = 0; j < cached.size();) {
      int32_t st = -1;
      CHECK(jenga_small_state(pool, cached[j].first, cached[j].second, &st) == JENGA_OK);
      if (st != JENGA_PAGE_EVICTABLE) cached.erase(cached.begin() + j); else ++j;
    }
    if (u < 30) {
      const int k = int(rng() % 3);
      int32_t sid = -1, n_ev = 0, ek[8], ei[8];
      const int rc = jenga_alloc_small_evict(pool, k, int64_t(rng() % 7), &sid, ek, ei, 8, &n_ev);
      if (rc == JENGA_OK) {
        for (int i = 0; i < n_ev && i < 8; ++i)
          for (size_t j = 0; j < cached.size(); ++j)
            if (cached[j] == std::make_pair(int(ek[i]), int(ei[i]))) { cached.erase(cached.begin() + j); break; }
        used.push_back({k, sid});
        CHECK(jenga_set_last_access(pool, k, sid, clock - int64_t(rng() % 5)) == JENGA_OK);
        CHECK(jenga_set_prefix_length(pool, k, sid, int64_t(rng() % 9)) == JENGA_OK);
      } else {
        CHECK(rc == JENGA_ERR_OOM);
      }
    } else if (u < 50 && !used.empty()) {
      const size_t j = rng() % used.size();
      const bool keep = rng() % 3 != 0;
      CHECK(jenga_release_small(pool, used[j].first, used[j].second, keep) == JENGA_OK);
      if (keep) cached.push_back(used[j]);
      used.erase(used.begin() + j);
    } else if (u < 58 && !cached.empty()) {
      const size_t j = rng() % cached.size();
      CHECK(jenga_acquire_cached(pool, cached[j].first, cached[j].second) == JENGA_OK);
      used.push_back(cached[j]);
      cached.erase(cached.begin() + j);
    } else if (u < 64 && !cached.empty()) {
      const size_t j = rng() % cached.size();
      CHECK(jenga_set_last_access(pool, cached[j].first, cached[j].second, int64_t(rng() % (clock + 1))) == JENGA_OK);
    } else if (u < 80) {
      // request layer: grow, share, finish
      const int64_t req = 1000 + int64_t(rng() % 12);
      const int k = int(rng() % 2);
      int32_t have = 0;
      CHECK(jenga_request_num_pages(pool, req, k, &have) == JENGA_OK);
      const int rc = jenga_request_extend(pool, req, k, int64_t(have) * 16 + int64_t(rng() % 70));
      CHECK(rc == JENGA_OK || rc == JENGA_ERR_OOM);
      bool known = false;
      for (int64_t r : requests) known = known || r == req;
      if (!known) requests.push_back(req);
      jenga_request_touch(pool, req, k, 0, 1 << 20, clock);
      jenga_request_set_prefix_lengths(pool, req, k);
      int32_t row[64];
      const int rc2 = jenga_request_block_table_row(pool, req, k, row, 64);
      CHECK(rc2 == JENGA_OK || rc2 == JENGA_ERR_INVALID);
    } else if (u < 84 && requests.size() >= 2) {
      const int64_t src = requests[rng() % requests.size()];
      const int64_t dst = 2000 + int64_t(rng() % 1000);
      int32_t have = 0;
      jenga_request_num_pages(pool, src, 0, &have);
      bool known = false;
      for (int64_t r : requests) known = known || r == dst;
      if (jenga_request_share_prefix(pool, src, dst, 0, int32_t(rng() % (have + 1))) == JENGA_OK && !known)
        requests.push_back(dst);
    } else if (u < 92 && !requests.empty()) {
      const size_t j = rng() % requests.size();
      const int rc = rng() % 2 ? jenga_request_free(pool, requests[j])
                               : jenga_request_release(pool, requests[j], 0);
      CHECK(rc == JENGA_OK);
      requests.erase(requests.begin() + j);
    } else {
      // invalid calls must be refused, not crash
      int32_t x = 0;
      int64_t y = 0;
      CHECK(jenga_free_small(pool, 5, 0) == JENGA_ERR_INVALID);
      CHECK(jenga_free_small(pool, 0, -3) == JENGA_ERR_INVALID);
      CHECK(jenga_acquire_cached(pool, 1, 1 << 30) == JENGA_ERR_INVALID);
      CHECK(jenga_small_refcount(pool, 2, -1, &x) == JENGA_ERR_INVALID);
      CHECK(jenga_large_page_owner(pool, n_large, &x, &y) == JENGA_ERR_INVALID);
      CHECK(jenga_kv_offset(pool, 2, 0, 0, 0, 0, 0, &y) == JENGA_ERR_INVALID);
      CHECK(jenga_request_free(pool, 999999) == JENGA_ERR_INVALID);
    }
    if (op % 512 == 0) {
      jenga_pool_info info;
      CHECK(jenga_pool_get_info(pool, &info) == JENGA_OK && info.n_large_pages == n_large);
      int64_t owned = 0;
      for (int k = 0; k < 3; ++k) {
        jenga_kind_stats st;
        CHECK(jenga_pool_kind_stats(pool, k, &st) == JENGA_OK);
        CHECK(st.used_small_pages >= 0 && st.unused_small_pages >= 0 && st.evictable_small_pages >= 0);
        CHECK(st.used_small_pages + st.unused_small_pages + st.evictable_small_pages ==
              st.owned_large_pages * st.small_per_large);
        owned += st.owned_large_pages;
      }
      CHECK(owned + info.free_large_pages == n_large);
    }
  }
  // drain: everything must come back
  for (auto& p : used) CHECK(jenga_release_small(pool, p.first, p.second, 0) == JENGA_OK);
  for (auto& p : cached) {
    int32_t st = -1;
    CHECK(jenga_small_state(pool, p.first, p.second, &st) == JENGA_OK);
    if (st != JENGA_PAGE_EVICTABLE) continue;
    CHECK(jenga_acquire_cached(pool, p.first, p.second) == JENGA_OK);
    CHECK(jenga_free_small(pool, p.first, p.second) == JENGA_OK);
  }
  for (int64_t r : requests) CHECK(jenga_request_free(pool, r) == JENGA_OK);
  // pages left evictable by request_release/touch paths above are none (release used keep = 0)
  jenga_pool_info info;
  CHECK(jenga_pool_get_info(pool, &info) == JENGA_OK);
  CHECK(info.free_large_pages == n_large);
  CHECK(jenga_pool_destroy(pool) == JENGA_OK);
  std::printf("host_fuzz ok: seed %u, %d ops\n", seed, n_ops);
  return 0;
}
