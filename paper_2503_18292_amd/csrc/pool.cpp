// Host half of the library: the two-level page allocator (paper Sec. 4.1), its
// request-aware placement (Sec. 4.3) and the per-request page lists that become
// per-layer-type block tables (Sec. 4.2 item 2).  Pure host code: the device
// base pointer is stored and never dereferenced.
#include <algorithm>
#include <cstring>
#include <limits>
#include <memory>
#include <new>
#include <numeric>

#include "pool_internal.hpp"

using jenga::Kind;
using jenga::RequestPages;

namespace jenga {
void (*device_setup_hook)() noexcept = nullptr;
}

namespace {

bool is_attention(int32_t type) {
  return type == JENGA_FULL || type == JENGA_WINDOW || type == JENGA_CROSS;
}

bool is_pow2(int64_t x) { return x > 0 && (x & (x - 1)) == 0; }

// Fills the derived fields of a kind from its descriptor.  Returns a jenga_status.
int derive_kind(const jenga_kind_desc& d, Kind* k) {
  k->desc = d;
  if (d.type < JENGA_FULL || d.type > JENGA_OPAQUE) return JENGA_ERR_INVALID;
  if (d.n_layers < 1) return JENGA_ERR_INVALID;
  if (d.dtype != JENGA_F32 && d.dtype != JENGA_BF16) return JENGA_ERR_INVALID;
  k->elem_bytes = d.dtype == JENGA_F32 ? 4 : 2;
  if (is_attention(d.type)) {
    if (d.n_kv_heads < 1 || d.head_dim < 1) return JENGA_ERR_INVALID;
    // any page size (Sec. 4.1 footnote: the number of tokens per page is arbitrary) whose K rows
    // and V rows stay 16-byte aligned
    if (d.tokens_per_page < 1 || d.tokens_per_page > 4096) return JENGA_ERR_UNSUPPORTED;
    if (d.head_dim != 64 && d.head_dim != 128 && d.head_dim != 256) return JENGA_ERR_UNSUPPORTED;
    if (d.type == JENGA_WINDOW ? d.window <= 0 : d.window != 0) return JENGA_ERR_INVALID;
    k->slice_bytes = int64_t(2) * d.n_kv_heads * d.tokens_per_page * d.head_dim * k->elem_bytes;
    const int64_t need = k->slice_bytes * d.n_layers;
    k->small_bytes = d.small_page_bytes == 0 ? need : d.small_page_bytes;
    if (k->small_bytes < need) return JENGA_ERR_INVALID;
    if (is_pow2(d.tokens_per_page)) {
      k->t_log2 = 0;
      while ((1 << k->t_log2) < d.tokens_per_page) ++k->t_log2;
    } else {
      k->t_log2 = -d.tokens_per_page;        // the kernels divide
    }
    if ((int64_t(d.tokens_per_page) * d.head_dim * k->elem_bytes) % 16 != 0) return JENGA_ERR_ALIGN;
  } else {
    // an OPAQUE page is one unit: request lengths of such a kind count pages
    if (d.small_page_bytes <= 0 || d.window != 0 || d.tokens_per_page != 1) return JENGA_ERR_INVALID;
    k->slice_bytes = 0;
    k->small_bytes = d.small_page_bytes;
    k->t_log2 = 0;
  }
  if (k->small_bytes % 16 != 0) return JENGA_ERR_ALIGN;
  return JENGA_OK;
}

int lcm_of(const std::vector<Kind>& kinds, int64_t* out) {
  int64_t l = 1;
  for (const Kind& k : kinds) {
    const int64_t g = std::gcd(l, k.small_bytes);
    const int64_t f = k.small_bytes / g;
    if (l > std::numeric_limits<int64_t>::max() / f) return JENGA_ERR_UNSUPPORTED;
    l *= f;
  }
  *out = l;
  return JENGA_OK;
}

inline bool bit_get(const std::vector<uint64_t>& v, int64_t i) { return (v[i >> 6] >> (i & 63)) & 1; }
inline void bit_set(std::vector<uint64_t>& v, int64_t i) { v[i >> 6] |= uint64_t(1) << (i & 63); }
inline void bit_clear(std::vector<uint64_t>& v, int64_t i) { v[i >> 6] &= ~(uint64_t(1) << (i & 63)); }

// No exception may cross the C ABI: every entry point below runs its body through this.  The
// containers of the pool can only throw when host memory runs out, reported as JENGA_ERR_OOM.
template <class F>
int guarded(F&& body) noexcept {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return JENGA_ERR_OOM;
  } catch (...) {
    return JENGA_ERR_INVALID;
  }
}

bool kind_ok(const jenga_pool* p, int32_t kind) { return p && kind >= 0 && kind < int32_t(p->kinds.size()); }

// Lowest slot of an owned large page that is neither used nor evictable, or -1.
int64_t first_empty(const Kind& k, int64_t large) {
  const int64_t begin = large * k.per_large, end = (large + 1) * k.per_large;
  int64_t i = begin;
  while (i < end) {
    const int64_t w = i >> 6;
    uint64_t inv = ~(k.used[w] | k.cached[w]);
    inv &= ~uint64_t(0) << (i & 63);
    const int64_t word_end = (w + 1) << 6;
    if (word_end > end) inv &= (uint64_t(1) << (end & 63)) - 1;
    if (inv) return (w << 6) + __builtin_ctzll(inv);
    i = word_end;
  }
  return -1;
}

void ensure_keys(jenga_pool* p, Kind& k) {
  if (k.last_access.empty()) {
    k.last_access.assign(size_t(p->n_large * k.per_large), 0);
    k.prefix_length.assign(size_t(p->n_large * k.per_large), 0);
  }
}

std::tuple<int64_t, int64_t, int32_t> small_key(const Kind& k, int32_t sid) {
  if (k.last_access.empty()) return {0, 0, sid};
  return {k.last_access[sid], -k.prefix_length[sid], sid};
}

void drop_from_room_sets(jenga_pool* p, Kind& k, int64_t large) {
  k.with_room.erase(large);
  auto it = k.with_room_by_request.find(p->large_request[large]);
  if (it != k.with_room_by_request.end()) {
    it->second.erase(large);
    if (it->second.empty()) k.with_room_by_request.erase(it);
  }
}

// Keeps the large page's membership and key in the evictable-large set in step with its
// counters: member iff all its small pages are evictable (Sec. 5.4).  Its LRU time is the latest
// last access among all its small pages (Sec. 5.4 step 3); equal times go to the larger maximum
// prefix length (Sec. 5.1), then to the lower page number.
void refresh_evictable_large(jenga_pool* p, int64_t large) {
  auto& cur = p->evictable_large_key[large];
  if (std::get<2>(cur) >= 0) {
    p->evictable_large.erase(cur);
    std::get<2>(cur) = -1;
  }
  const int32_t kind = p->large_kind[large];
  if (kind < 0) return;
  const Kind& k = p->kinds[kind];
  if (int64_t(p->large_cached[large]) != k.per_large) return;
  int64_t ts = std::numeric_limits<int64_t>::min(), len = std::numeric_limits<int64_t>::min();
  for (int64_t s = large * k.per_large; s < (large + 1) * k.per_large; ++s) {
    ts = std::max(ts, k.last_access.empty() ? 0 : k.last_access[s]);
    len = std::max(len, k.prefix_length.empty() ? 0 : k.prefix_length[s]);
  }
  cur = {ts, -len, large};
  p->evictable_large.insert(cur);
}

// A free large page becomes `kind`'s, all its small pages associated with `request`.
void adopt_large(jenga_pool* p, int32_t kind, int64_t large, int64_t request) {
  Kind& k = p->kinds[kind];
  p->large_kind[large] = kind;
  p->large_request[large] = request;
  p->large_empty[large] = int32_t(k.per_large);
  p->large_used[large] = 0;
  p->large_cached[large] = 0;
  ++k.owned_large;
  k.with_room.insert(large);
  k.with_room_by_request[request].insert(large);
}

// An owned large page whose small pages are all empty goes back to level 1.
void return_large(jenga_pool* p, int64_t large) {
  Kind& k = p->kinds[p->large_kind[large]];
  drop_from_room_sets(p, k, large);
  p->large_kind[large] = -1;
  p->large_request[large] = 0;
  p->large_empty[large] = p->large_used[large] = p->large_cached[large] = 0;
  --k.owned_large;
  p->free_large.insert(large);
}

// Takes the lowest empty slot of an owned large page that is known to have one.
int32_t take_slot(jenga_pool* p, int32_t kind, int64_t large) {
  Kind& k = p->kinds[kind];
  const int64_t sid = first_empty(k, large);
  bit_set(k.used, sid);
  ++k.used_small;
  ++p->large_used[large];
  if (--p->large_empty[large] == 0) drop_from_room_sets(p, k, large);
  return int32_t(sid);      // (a page with an empty slot is not an evictable large page: no set to update)
}

struct Evicted {
  int32_t* kinds;
  int32_t* ids;
  int32_t cap;
  int32_t n;
  void add(int32_t kind, int32_t sid) {
    if (n < cap) {
      if (kinds) kinds[n] = kind;
      if (ids) ids[n] = sid;
    }
    ++n;
  }
};

// allocate() of Sec. 4.1 in the order of Sec. 4.3, extended by the eviction steps of
// Sec. 5.4.  With nothing evictable steps 3 and 5 find nothing and this is Sec. 4.3.
int alloc_small(jenga_pool* p, int32_t kind, int64_t request, int32_t* out, Evicted* ev) {
  Kind& k = p->kinds[kind];
  // step 1: an empty small page associated with this request
  auto mine = k.with_room_by_request.find(request);
  if (mine != k.with_room_by_request.end() && !mine->second.empty()) {
    *out = take_slot(p, kind, *mine->second.begin());
    return JENGA_OK;
  }
  // step 2: an empty large page; all its small pages become associated with the request
  if (!p->free_large.empty()) {
    const int64_t large = *p->free_large.begin();
    p->free_large.erase(p->free_large.begin());
    adopt_large(p, kind, large, request);
    *out = take_slot(p, kind, large);
    return JENGA_OK;
  }
  // step 3: evict the least recently used evictable large page, of whatever kind
  if (!p->evictable_large.empty()) {
    const int64_t large = std::get<2>(*p->evictable_large.begin());
    const int32_t old_kind = p->large_kind[large];
    Kind& ko = p->kinds[old_kind];
    for (int64_t s = large * ko.per_large; s < (large + 1) * ko.per_large; ++s) {   // all evictable
      ko.evictable.erase(small_key(ko, int32_t(s)));
      bit_clear(ko.cached, s);
      --ko.cached_small;
      if (ev) ev->add(old_kind, int32_t(s));
    }
    p->large_cached[large] = 0;
    refresh_evictable_large(p, large);          // leaves the set
    --ko.owned_large;                           // (it had no empty slot, so it is in no room set)
    p->large_kind[large] = -1;
    adopt_large(p, kind, large, request);
    *out = take_slot(p, kind, large);
    return JENGA_OK;
  }
  // step 4: an empty small page of this kind associated with another request
  if (!k.with_room.empty()) {
    *out = take_slot(p, kind, *k.with_room.begin());
    return JENGA_OK;
  }
  // step 5: evict the least recently used evictable small page of this kind
  if (!k.evictable.empty()) {
    const int32_t sid = std::get<2>(*k.evictable.begin());
    k.evictable.erase(k.evictable.begin());
    const int64_t large = sid / k.per_large;
    bit_clear(k.cached, sid);
    --k.cached_small;
    --p->large_cached[large];
    bit_set(k.used, sid);
    ++k.used_small;
    ++p->large_used[large];
    refresh_evictable_large(p, large);
    if (ev) ev->add(kind, sid);
    *out = sid;
    return JENGA_OK;
  }
  return JENGA_ERR_OOM;
}

bool small_in_range(const jenga_pool* p, int32_t kind, int32_t sid) {
  return sid >= 0 && int64_t(sid) < p->n_large * p->kinds[kind].per_large;
}

bool small_live(const jenga_pool* p, int32_t kind, int32_t sid) {
  return small_in_range(p, kind, sid) && bit_get(p->kinds[kind].used, sid);
}

// free(small_page_id) of Sec. 4.1 (keep_cached false) or the end of a request under prefix
// caching (keep_cached true: the page stays evictable, Sec. 5.4).
int release_small(jenga_pool* p, int32_t kind, int32_t sid, bool keep_cached) {
  if (!small_live(p, kind, sid)) return JENGA_ERR_INVALID;
  Kind& k = p->kinds[kind];
  auto extra = k.extra_refs.find(sid);
  if (extra != k.extra_refs.end()) {        // shared page: one sharer fewer
    if (--extra->second == 0) k.extra_refs.erase(extra);
    return JENGA_OK;
  }
  bit_clear(k.used, sid);
  --k.used_small;
  const int64_t large = sid / k.per_large;
  --p->large_used[large];
  if (keep_cached) {
    bit_set(k.cached, sid);
    ++k.cached_small;
    ++p->large_cached[large];
    k.evictable.insert(small_key(k, sid));
  } else {
    if (p->large_empty[large]++ == 0) {
      k.with_room.insert(large);
      k.with_room_by_request[p->large_request[large]].insert(large);
    }
  }
  if (p->large_used[large] == 0 && p->large_cached[large] == 0)
    return_large(p, large);                 // every small page empty (Sec. 4.1 free())
  else if (keep_cached)
    refresh_evictable_large(p, large);      // it may have been the last page not yet evictable
  return JENGA_OK;
}

int free_small(jenga_pool* p, int32_t kind, int32_t sid) { return release_small(p, kind, sid, false); }

}  // namespace

extern "C" {

int jenga_lcm_page_bytes(const jenga_kind_desc* kinds, int32_t n_kinds, int64_t* out_bytes) {
  return guarded([&]() -> int {
  if (!kinds || n_kinds < 1 || !out_bytes) return JENGA_ERR_INVALID;
  std::vector<Kind> ks(n_kinds);
  for (int32_t i = 0; i < n_kinds; ++i) {
    const int rc = derive_kind(kinds[i], &ks[i]);
    if (rc != JENGA_OK) return rc;
  }
  return lcm_of(ks, out_bytes);
  });
}

int jenga_pool_create(void* device_base, int64_t pool_bytes, int64_t large_page_bytes,
                      const jenga_kind_desc* kinds, int32_t n_kinds, jenga_pool** out) {
  return guarded([&]() -> int {
  if (!kinds || n_kinds < 1 || !out || pool_bytes < 0 || large_page_bytes <= 0) return JENGA_ERR_INVALID;
  *out = nullptr;
  if (reinterpret_cast<uintptr_t>(device_base) % 256 != 0) return JENGA_ERR_ALIGN;
  std::unique_ptr<jenga_pool> p(new (std::nothrow) jenga_pool());
  if (!p) return JENGA_ERR_OOM;
  p->kinds.resize(n_kinds);
  for (int32_t i = 0; i < n_kinds; ++i) {
    const int rc = derive_kind(kinds[i], &p->kinds[i]);
    if (rc != JENGA_OK) return rc;
  }
  int64_t lcm = 0;
  int rc = lcm_of(p->kinds, &lcm);
  if (rc != JENGA_OK) return rc;
  if (large_page_bytes % lcm != 0) return JENGA_ERR_INVALID;
  p->base = static_cast<char*>(device_base);
  p->pool_bytes = pool_bytes;
  p->large_bytes = large_page_bytes;
  p->n_large = pool_bytes / large_page_bytes;
  for (Kind& k : p->kinds) {
    k.per_large = large_page_bytes / k.small_bytes;
    if (k.per_large > std::numeric_limits<int32_t>::max() ||
        p->n_large * k.per_large > std::numeric_limits<int32_t>::max())
      return JENGA_ERR_UNSUPPORTED;      // small ids are int32
    k.used.assign(size_t((p->n_large * k.per_large + 63) / 64), 0);
    k.cached.assign(k.used.size(), 0);
  }
  p->large_kind.assign(size_t(p->n_large), -1);
  p->large_request.assign(size_t(p->n_large), 0);
  p->large_empty.assign(size_t(p->n_large), 0);
  p->large_used.assign(size_t(p->n_large), 0);
  p->large_cached.assign(size_t(p->n_large), 0);
  p->evictable_large_key.assign(size_t(p->n_large), std::make_tuple(int64_t(0), int64_t(0), int64_t(-1)));
  for (int64_t i = 0; i < p->n_large; ++i) p->free_large.insert(p->free_large.end(), i);
  if (device_base != nullptr && jenga::device_setup_hook != nullptr) jenga::device_setup_hook();
  *out = p.release();
  return JENGA_OK;
  });
}

int jenga_pool_destroy(jenga_pool* pool) {
  if (!pool) return JENGA_ERR_INVALID;
  delete pool;
  return JENGA_OK;
}

int jenga_alloc_small(jenga_pool* pool, int32_t kind, int64_t request, int32_t* out_small_id) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind) || !out_small_id) return JENGA_ERR_INVALID;
  return alloc_small(pool, kind, request, out_small_id, nullptr);
  });
}

int jenga_ref_small(jenga_pool* pool, int32_t kind, int32_t small_id) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind) || !small_live(pool, kind, small_id)) return JENGA_ERR_INVALID;
  ++pool->kinds[kind].extra_refs[small_id];
  return JENGA_OK;
  });
}

int jenga_free_small(jenga_pool* pool, int32_t kind, int32_t small_id) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind)) return JENGA_ERR_INVALID;
  return free_small(pool, kind, small_id);
  });
}

int jenga_pool_get_info(const jenga_pool* pool, jenga_pool_info* out) {
  return guarded([&]() -> int {
  if (!pool || !out) return JENGA_ERR_INVALID;
  out->large_page_bytes = pool->large_bytes;
  out->n_large_pages = pool->n_large;
  out->free_large_pages = int64_t(pool->free_large.size());
  out->n_kinds = int32_t(pool->kinds.size());
  out->reserved = 0;
  return JENGA_OK;
  });
}

int jenga_pool_kind_stats(const jenga_pool* pool, int32_t kind, jenga_kind_stats* out) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind) || !out) return JENGA_ERR_INVALID;
  const Kind& k = pool->kinds[kind];
  out->small_page_bytes = k.small_bytes;
  out->slice_bytes = k.slice_bytes;
  out->small_per_large = k.per_large;
  out->owned_large_pages = k.owned_large;
  out->used_small_pages = k.used_small;
  out->unused_small_pages = k.owned_large * k.per_large - k.used_small - k.cached_small;
  out->evictable_small_pages = k.cached_small;
  return JENGA_OK;
  });
}

int jenga_large_page_owner(const jenga_pool* pool, int64_t large_page, int32_t* out_kind,
                           int64_t* out_request) {
  return guarded([&]() -> int {
  if (!pool || large_page < 0 || large_page >= pool->n_large || !out_kind || !out_request)
    return JENGA_ERR_INVALID;
  *out_kind = pool->large_kind[large_page];
  *out_request = pool->large_request[large_page];
  return JENGA_OK;
  });
}

int jenga_small_refcount(const jenga_pool* pool, int32_t kind, int32_t small_id, int32_t* out) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind) || !out) return JENGA_ERR_INVALID;
  const Kind& k = pool->kinds[kind];
  if (small_id < 0 || int64_t(small_id) >= pool->n_large * k.per_large) return JENGA_ERR_INVALID;
  if (!bit_get(k.used, small_id)) { *out = 0; return JENGA_OK; }
  auto it = k.extra_refs.find(small_id);
  *out = 1 + (it == k.extra_refs.end() ? 0 : it->second);
  return JENGA_OK;
  });
}

int jenga_kv_offset(const jenga_pool* pool, int32_t kind, int32_t small_id, int32_t layer,
                    int32_t kv_head, int32_t is_v, int32_t token_in_page, int64_t* out_bytes) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind) || !out_bytes) return JENGA_ERR_INVALID;
  const Kind& k = pool->kinds[kind];
  if (!is_attention(k.desc.type)) return JENGA_ERR_INVALID;
  if (small_id < 0 || int64_t(small_id) >= pool->n_large * k.per_large) return JENGA_ERR_INVALID;
  if (layer < 0 || layer >= k.desc.n_layers || kv_head < 0 || kv_head >= k.desc.n_kv_heads ||
      token_in_page < 0 || token_in_page >= k.desc.tokens_per_page || (is_v != 0 && is_v != 1))
    return JENGA_ERR_INVALID;
  const int64_t row = int64_t(k.desc.head_dim) * k.elem_bytes;
  const int64_t plane = row * k.desc.tokens_per_page;
  *out_bytes = int64_t(small_id) * k.small_bytes + int64_t(layer) * k.slice_bytes +
               int64_t(kv_head) * 2 * plane + int64_t(is_v) * plane + int64_t(token_in_page) * row;
  return JENGA_OK;
  });
}

int jenga_request_extend(jenga_pool* pool, int64_t request, int32_t kind, int64_t new_len) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind) || new_len < 0) return JENGA_ERR_INVALID;
  const Kind& k = pool->kinds[kind];
  const int64_t T = k.desc.tokens_per_page;
  const int64_t need = (new_len + T - 1) / T;
  if (need > std::numeric_limits<int32_t>::max()) return JENGA_ERR_INVALID;
  RequestPages& rp = pool->requests[request];
  if (rp.pages.empty()) {
    rp.pages.resize(pool->kinds.size());
    rp.first_resident.assign(pool->kinds.size(), 0);
  }
  std::vector<int32_t>& lst = rp.pages[kind];
  while (int64_t(lst.size()) < need) {
    int32_t sid = -1;
    const int rc = alloc_small(pool, kind, request, &sid, nullptr);
    if (rc != JENGA_OK) return rc;
    lst.push_back(sid);
  }
  if (k.desc.type == JENGA_WINDOW) {
    // only the last `window` tokens are needed (Sec. 5.1): pages wholly before them go
    const int64_t lo = std::max<int64_t>(0, new_len - k.desc.window);
    int64_t& p = rp.first_resident[kind];
    while (p < int64_t(lst.size()) && T * (p + 1) <= lo) {
      if (lst[p] >= 0) {
        free_small(pool, kind, lst[p]);
        lst[p] = -1;
      }
      ++p;
    }
  }
  return JENGA_OK;
  });
}

int jenga_request_share_prefix(jenga_pool* pool, int64_t src_request, int64_t dst_request,
                               int32_t kind, int32_t n_pages) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind) || n_pages < 0 || src_request == dst_request) return JENGA_ERR_INVALID;
  auto src = pool->requests.find(src_request);
  if (src == pool->requests.end() || int64_t(src->second.pages[kind].size()) < n_pages)
    return JENGA_ERR_INVALID;
  RequestPages& dst = pool->requests[dst_request];       // may rehash: re-find src below
  src = pool->requests.find(src_request);
  if (dst.pages.empty()) {
    dst.pages.resize(pool->kinds.size());
    dst.first_resident.assign(pool->kinds.size(), 0);
  }
  if (!dst.pages[kind].empty()) return JENGA_ERR_INVALID;
  Kind& k = pool->kinds[kind];
  const std::vector<int32_t>& s = src->second.pages[kind];
  for (int32_t p = 0; p < n_pages; ++p) {
    if (s[p] >= 0) ++k.extra_refs[s[p]];
    dst.pages[kind].push_back(s[p]);
  }
  return JENGA_OK;
  });
}

int jenga_request_free(jenga_pool* pool, int64_t request) {
  return guarded([&]() -> int {
  if (!pool) return JENGA_ERR_INVALID;
  auto it = pool->requests.find(request);
  if (it == pool->requests.end()) return JENGA_ERR_INVALID;
  for (size_t kind = 0; kind < it->second.pages.size(); ++kind)
    for (int32_t sid : it->second.pages[kind])
      if (sid >= 0) free_small(pool, int32_t(kind), sid);
  pool->requests.erase(it);
  return JENGA_OK;
  });
}

int jenga_request_num_pages(const jenga_pool* pool, int64_t request, int32_t kind, int32_t* out) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind) || !out) return JENGA_ERR_INVALID;
  auto it = pool->requests.find(request);
  *out = it == pool->requests.end() ? 0 : int32_t(it->second.pages[kind].size());
  return JENGA_OK;
  });
}

int jenga_request_block_table_row(const jenga_pool* pool, int64_t request, int32_t kind,
                                  int32_t* row, int32_t width) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind) || !row || width < 0) return JENGA_ERR_INVALID;
  auto it = pool->requests.find(request);
  size_t n = 0;
  if (it != pool->requests.end()) {
    const std::vector<int32_t>& lst = it->second.pages[kind];
    if (lst.size() > size_t(width)) return JENGA_ERR_INVALID;
    n = lst.size();
    if (n) std::memcpy(row, lst.data(), n * sizeof(int32_t));
  }
  std::fill(row + n, row + width, -1);
  return JENGA_OK;
  });
}

int jenga_requests_extend(jenga_pool* pool, int32_t kind, const int64_t* requests,
                          const int64_t* new_lens, int32_t n) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind) || n < 0 || (n > 0 && (!requests || !new_lens))) return JENGA_ERR_INVALID;
  for (int32_t i = 0; i < n; ++i) {
    const int rc = jenga_request_extend(pool, requests[i], kind, new_lens[i]);
    if (rc != JENGA_OK) return rc;
  }
  return JENGA_OK;
  });
}

int jenga_block_table_fill(const jenga_pool* pool, int32_t kind, const int64_t* requests, int32_t n,
                           int32_t* table, int32_t width) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind) || n < 0 || width < 0 || (n > 0 && (!requests || !table)))
    return JENGA_ERR_INVALID;
  for (int32_t i = 0; i < n; ++i) {
    const int rc = jenga_request_block_table_row(pool, requests[i], kind, table + int64_t(i) * width, width);
    if (rc != JENGA_OK) return rc;
  }
  return JENGA_OK;
  });
}

int jenga_alloc_small_evict(jenga_pool* pool, int32_t kind, int64_t request, int32_t* out_small_id,
                            int32_t* evicted_kinds, int32_t* evicted_ids, int32_t capacity,
                            int32_t* out_n_evicted) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind) || !out_small_id || capacity < 0) return JENGA_ERR_INVALID;
  Evicted ev{evicted_kinds, evicted_ids, capacity, 0};
  const int rc = alloc_small(pool, kind, request, out_small_id, &ev);
  if (out_n_evicted) *out_n_evicted = ev.n;
  return rc;
  });
}

int jenga_release_small(jenga_pool* pool, int32_t kind, int32_t small_id, int32_t keep_cached) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind)) return JENGA_ERR_INVALID;
  return release_small(pool, kind, small_id, keep_cached != 0);
  });
}

int jenga_acquire_cached(jenga_pool* pool, int32_t kind, int32_t small_id) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind) || !small_in_range(pool, kind, small_id)) return JENGA_ERR_INVALID;
  Kind& k = pool->kinds[kind];
  if (!bit_get(k.cached, small_id)) return JENGA_ERR_INVALID;
  k.evictable.erase(small_key(k, small_id));
  bit_clear(k.cached, small_id);
  --k.cached_small;
  bit_set(k.used, small_id);
  ++k.used_small;
  const int64_t large = small_id / k.per_large;
  --pool->large_cached[large];
  ++pool->large_used[large];
  refresh_evictable_large(pool, large);
  return JENGA_OK;
  });
}

namespace {
// Changes one LRU key of a used or evictable page and keeps the ordered sets in step.
int set_key(jenga_pool* pool, int32_t kind, int32_t sid, bool is_time, int64_t value) {
  if (!kind_ok(pool, kind) || !small_in_range(pool, kind, sid)) return JENGA_ERR_INVALID;
  Kind& k = pool->kinds[kind];
  const bool cached = bit_get(k.cached, sid);
  if (!cached && !bit_get(k.used, sid)) return JENGA_ERR_INVALID;     // empty pages have no keys
  ensure_keys(pool, k);
  if (cached) k.evictable.erase(small_key(k, sid));
  (is_time ? k.last_access : k.prefix_length)[sid] = value;
  if (cached) {
    k.evictable.insert(small_key(k, sid));
    refresh_evictable_large(pool, sid / k.per_large);
  }
  return JENGA_OK;
}
}  // namespace

int jenga_set_last_access(jenga_pool* pool, int32_t kind, int32_t small_id, int64_t time) {
  return guarded([&]() -> int {
  return set_key(pool, kind, small_id, true, time);
  });
}

int jenga_set_prefix_length(jenga_pool* pool, int32_t kind, int32_t small_id, int64_t length) {
  return guarded([&]() -> int {
  return set_key(pool, kind, small_id, false, length);
  });
}

int jenga_small_state(const jenga_pool* pool, int32_t kind, int32_t small_id, int32_t* out_state) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind) || !small_in_range(pool, kind, small_id) || !out_state) return JENGA_ERR_INVALID;
  const Kind& k = pool->kinds[kind];
  *out_state = bit_get(k.used, small_id) ? JENGA_PAGE_USED
               : bit_get(k.cached, small_id) ? JENGA_PAGE_EVICTABLE : JENGA_PAGE_EMPTY;
  return JENGA_OK;
  });
}

int jenga_request_release(jenga_pool* pool, int64_t request, int32_t keep_cached) {
  return guarded([&]() -> int {
  if (!pool) return JENGA_ERR_INVALID;
  auto it = pool->requests.find(request);
  if (it == pool->requests.end()) return JENGA_ERR_INVALID;
  for (size_t kind = 0; kind < it->second.pages.size(); ++kind)
    for (int32_t sid : it->second.pages[kind])
      if (sid >= 0) release_small(pool, int32_t(kind), sid, keep_cached != 0);
  pool->requests.erase(it);
  return JENGA_OK;
  });
}

int jenga_request_touch(jenga_pool* pool, int64_t request, int32_t kind, int64_t first_token,
                        int64_t end_token, int64_t time) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind) || first_token < 0 || end_token < first_token) return JENGA_ERR_INVALID;
  auto it = pool->requests.find(request);
  if (it == pool->requests.end()) return JENGA_ERR_INVALID;
  const std::vector<int32_t>& lst = it->second.pages[kind];
  const int64_t T = pool->kinds[kind].desc.tokens_per_page;
  const int64_t p_end = std::min<int64_t>(int64_t(lst.size()), (end_token + T - 1) / T);
  for (int64_t pg = first_token / T; pg < p_end; ++pg)
    if (lst[pg] >= 0) set_key(pool, kind, lst[pg], true, time);
  return JENGA_OK;
  });
}

int jenga_request_set_prefix_lengths(jenga_pool* pool, int64_t request, int32_t kind) {
  return guarded([&]() -> int {
  if (!kind_ok(pool, kind)) return JENGA_ERR_INVALID;
  auto it = pool->requests.find(request);
  if (it == pool->requests.end()) return JENGA_ERR_INVALID;
  const std::vector<int32_t>& lst = it->second.pages[kind];
  const int64_t T = pool->kinds[kind].desc.tokens_per_page;
  for (size_t pg = 0; pg < lst.size(); ++pg)
    if (lst[pg] >= 0) set_key(pool, kind, lst[pg], false, int64_t(pg + 1) * T);
  return JENGA_OK;
  });
}

int jenga_possible_prefixes(int32_t rule, int32_t param, const uint8_t* is_hit, int32_t n_tokens,
                            uint8_t* out_valid) {
  return guarded([&]() -> int {
  if (n_tokens < 0 || (n_tokens > 0 && !is_hit) || !out_valid) return JENGA_ERR_INVALID;
  if ((rule == JENGA_HIT_WINDOW || rule == JENGA_HIT_EVERY) && param < 1) return JENGA_ERR_INVALID;
  out_valid[0] = 0;
  switch (rule) {
    case JENGA_HIT_FULL: {            // every token of the prefix cached
      bool ok = true;
      for (int32_t p = 1; p <= n_tokens; ++p) {
        ok = ok && is_hit[p - 1];
        out_valid[p] = ok;
      }
      return JENGA_OK;
    }
    case JENGA_HIT_WINDOW: {          // the last `param` tokens of the prefix cached
      int32_t run = 0;                // cached tokens ending at p
      for (int32_t p = 1; p <= n_tokens; ++p) {
        run = is_hit[p - 1] ? run + 1 : 0;
        out_valid[p] = run >= std::min(param, p);
      }
      return JENGA_OK;
    }
    case JENGA_HIT_EVERY:             // one cached state every `param` tokens
      for (int32_t p = 1; p <= n_tokens; ++p) out_valid[p] = (p % param == 0) && is_hit[p - 1];
      return JENGA_OK;
    default:
      return JENGA_ERR_INVALID;
  }
  });
}

int jenga_longest_common_prefix(const uint8_t* const* valid_sets, int32_t n_sets, int32_t n_tokens) {
  return guarded([&]() -> int {
  if (!valid_sets || n_sets < 1 || n_tokens < 0) return JENGA_ERR_INVALID;
  for (int32_t p = n_tokens; p >= 1; --p) {
    bool all = true;
    for (int32_t s = 0; s < n_sets && all; ++s) all = valid_sets[s] && valid_sets[s][p];
    if (all) return p;
  }
  return 0;
  });
}

const char* jenga_strerror(int status) {
  switch (status) {
    case JENGA_OK: return "ok";
    case JENGA_ERR_INVALID: return "invalid argument or state";
    case JENGA_ERR_OOM: return "out of pages";
    case JENGA_ERR_ALIGN: return "pointer or size not aligned";
    case JENGA_ERR_WORKSPACE: return "split-K workspace too small";
    case JENGA_ERR_HIP: return "HIP runtime error";
    case JENGA_ERR_UNSUPPORTED: return "unsupported shape";
    default: return "unknown status";
  }
}

int jenga_version(void) { return 0x000100; }

}  // extern "C"
