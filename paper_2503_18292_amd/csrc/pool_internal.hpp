// Internal layout of the host pool object, shared by the allocator (pool.cpp)
// and the kernel launchers (kernels.hip).  Not part of the C ABI.
#pragma once

#include <cstdint>
#include <set>
#include <tuple>
#include <unordered_map>
#include <vector>

#include "jenga.h"

namespace jenga {

struct Kind {
  jenga_kind_desc desc{};
  int64_t small_bytes = 0;   // S_k
  int64_t slice_bytes = 0;   // one layer's K+V for one page of tokens (0 for OPAQUE)
  int64_t per_large = 0;     // r_k
  int32_t elem_bytes = 0;
  int32_t t_log2 = 0;        // log2(tokens_per_page), or -tokens_per_page when that is no power of two

  // level 2 state.  A small page is used (bit in `used`: it has references), evictable
  // (bit in `cached`: valid contents, no references; Sec. 5.4) or empty (neither).
  // `extra_refs` holds (count - 1) for pages with more than one reference.
  std::vector<uint64_t> used;
  std::vector<uint64_t> cached;
  std::unordered_map<int32_t, int32_t> extra_refs;
  // LRU keys of Sec. 5.1, kept for used and evictable pages; allocated on first use
  std::vector<int64_t> last_access;
  std::vector<int64_t> prefix_length;
  // large pages of this kind that still have an empty slot: all of them, and grouped by
  // the request they are associated with.  Ordered: the lowest-numbered one is *begin().
  std::set<int64_t> with_room;
  std::unordered_map<int64_t, std::set<int64_t>> with_room_by_request;
  // evictable small pages ordered by (last access, -prefix length, id): *begin() goes first
  std::set<std::tuple<int64_t, int64_t, int32_t>> evictable;
  int64_t owned_large = 0;
  int64_t used_small = 0;
  int64_t cached_small = 0;
};

// Set by the kernel half of the library when it is linked in (the allocator also builds alone, for
// host-only checks): per-device set-up that should not wait for the first decode call, run by
// jenga_pool_create for a pool that lies in device memory.  Failures are left to that first call.
extern void (*device_setup_hook)() noexcept;

struct RequestPages {
  std::vector<std::vector<int32_t>> pages;   // [kind][logical page] -> small id or -1
  std::vector<int64_t> first_resident;       // [kind] every page below it is already -1
};

}  // namespace jenga

struct jenga_pool {
  char* base = nullptr;
  int64_t pool_bytes = 0;
  int64_t large_bytes = 0;
  int64_t n_large = 0;
  std::vector<jenga::Kind> kinds;
  // level 1 state
  std::vector<int32_t> large_kind;        // -1: free
  std::vector<int64_t> large_request;     // valid while large_kind >= 0
  std::vector<int32_t> large_empty;       // empty slots, valid while owned
  std::vector<int32_t> large_used;        // used slots, valid while owned
  std::vector<int32_t> large_cached;      // evictable slots, valid while owned
  std::set<int64_t> free_large;           // ordered: lowest-numbered first
  // large pages whose small pages are all evictable (Sec. 5.4), ordered by
  // (latest last access of their small pages, -largest prefix length, page number)
  std::set<std::tuple<int64_t, int64_t, int64_t>> evictable_large;
  std::vector<std::tuple<int64_t, int64_t, int64_t>> evictable_large_key;   // key while in the set
  std::unordered_map<int64_t, jenga::RequestPages> requests;
};
