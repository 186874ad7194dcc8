// Host half of the library: the two-level page allocator (paper Sec. 4.1), its
// request-aware placement (Sec. 4.3) and the per-request page lists that become
// per-layer-type block tables (Sec. 4.2 item 2).  Pure host code: the device
// base pointer is stored and never dereferenced.
#include <algorithm>
#include <cstring>
#include <limits>
#include <new>
#include <numeric>

#include "pool_internal.hpp"

using jenga::Kind;
using jenga::RequestPages;

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
    if (!is_pow2(d.tokens_per_page) || d.tokens_per_page < 8 || d.tokens_per_page > 128)
      return JENGA_ERR_UNSUPPORTED;
    if (d.head_dim != 64 && d.head_dim != 128 && d.head_dim != 256) return JENGA_ERR_UNSUPPORTED;
    if (d.type == JENGA_WINDOW ? d.window <= 0 : d.window != 0) return JENGA_ERR_INVALID;
    k->slice_bytes = int64_t(2) * d.n_kv_heads * d.tokens_per_page * d.head_dim * k->elem_bytes;
    const int64_t need = k->slice_bytes * d.n_layers;
    k->small_bytes = d.small_page_bytes == 0 ? need : d.small_page_bytes;
    if (k->small_bytes < need) return JENGA_ERR_INVALID;
    k->t_log2 = 0;
    while ((1 << k->t_log2) < d.tokens_per_page) ++k->t_log2;
  } else {
    if (d.small_page_bytes <= 0 || d.window != 0) return JENGA_ERR_INVALID;
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

// Lowest clear bit in [begin, end), or -1.
int64_t first_clear(const std::vector<uint64_t>& v, int64_t begin, int64_t end) {
  int64_t i = begin;
  while (i < end) {
    const int64_t w = i >> 6;
    uint64_t inv = ~v[w];
    inv &= ~uint64_t(0) << (i & 63);
    const int64_t word_end = (w + 1) << 6;
    if (word_end > end) inv &= (uint64_t(1) << (end & 63)) - 1;
    if (inv) return (w << 6) + __builtin_ctzll(inv);
    i = word_end;
  }
  return -1;
}

bool kind_ok(const jenga_pool* p, int32_t kind) { return p && kind >= 0 && kind < int32_t(p->kinds.size()); }

// Takes the lowest unused slot of an owned large page that is known to have one.
int32_t take_slot(jenga_pool* p, int32_t kind, int64_t large) {
  Kind& k = p->kinds[kind];
  const int64_t sid = first_clear(k.used, large * k.per_large, (large + 1) * k.per_large);
  bit_set(k.used, sid);
  ++k.used_small;
  if (--p->large_unused[large] == 0) {
    k.with_room.erase(large);
    auto it = k.with_room_by_request.find(p->large_request[large]);
    if (it != k.with_room_by_request.end()) {
      it->second.erase(large);
      if (it->second.empty()) k.with_room_by_request.erase(it);
    }
  }
  return int32_t(sid);
}

int alloc_small(jenga_pool* p, int32_t kind, int64_t request, int32_t* out) {
  Kind& k = p->kinds[kind];
  // step 1 (Sec. 4.3): an unused small page associated with this request
  auto mine = k.with_room_by_request.find(request);
  if (mine != k.with_room_by_request.end() && !mine->second.empty()) {
    *out = take_slot(p, kind, *mine->second.begin());
    return JENGA_OK;
  }
  // step 2: a new large page; all its small pages become associated with the request
  if (!p->free_large.empty()) {
    const int64_t large = *p->free_large.begin();
    p->free_large.erase(p->free_large.begin());
    p->large_kind[large] = kind;
    p->large_request[large] = request;
    p->large_unused[large] = int32_t(k.per_large);
    ++k.owned_large;
    k.with_room.insert(large);
    k.with_room_by_request[request].insert(large);
    *out = take_slot(p, kind, large);
    return JENGA_OK;
  }
  // step 3: an unused small page of this kind associated with another request
  if (!k.with_room.empty()) {
    *out = take_slot(p, kind, *k.with_room.begin());
    return JENGA_OK;
  }
  return JENGA_ERR_OOM;
}

bool small_live(const jenga_pool* p, int32_t kind, int32_t sid) {
  const Kind& k = p->kinds[kind];
  return sid >= 0 && int64_t(sid) < p->n_large * k.per_large && bit_get(k.used, sid);
}

int free_small(jenga_pool* p, int32_t kind, int32_t sid) {
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
  const int64_t req = p->large_request[large];
  if (++p->large_unused[large] == k.per_large) {
    // every small page unused: back to the large-page allocator (Sec. 4.1 free())
    k.with_room.erase(large);
    auto it = k.with_room_by_request.find(req);
    if (it != k.with_room_by_request.end()) {
      it->second.erase(large);
      if (it->second.empty()) k.with_room_by_request.erase(it);
    }
    p->large_kind[large] = -1;
    p->large_request[large] = 0;
    p->large_unused[large] = 0;
    --k.owned_large;
    p->free_large.insert(large);
  } else {
    k.with_room.insert(large);
    k.with_room_by_request[req].insert(large);
  }
  return JENGA_OK;
}

}  // namespace

extern "C" {

int jenga_lcm_page_bytes(const jenga_kind_desc* kinds, int32_t n_kinds, int64_t* out_bytes) {
  if (!kinds || n_kinds < 1 || !out_bytes) return JENGA_ERR_INVALID;
  std::vector<Kind> ks(n_kinds);
  for (int32_t i = 0; i < n_kinds; ++i) {
    const int rc = derive_kind(kinds[i], &ks[i]);
    if (rc != JENGA_OK) return rc;
  }
  return lcm_of(ks, out_bytes);
}

int jenga_pool_create(void* device_base, int64_t pool_bytes, int64_t large_page_bytes,
                      const jenga_kind_desc* kinds, int32_t n_kinds, jenga_pool** out) {
  if (!kinds || n_kinds < 1 || !out || pool_bytes < 0 || large_page_bytes <= 0) return JENGA_ERR_INVALID;
  *out = nullptr;
  if (reinterpret_cast<uintptr_t>(device_base) % 256 != 0) return JENGA_ERR_ALIGN;
  jenga_pool* p = new (std::nothrow) jenga_pool();
  if (!p) return JENGA_ERR_OOM;
  p->kinds.resize(n_kinds);
  for (int32_t i = 0; i < n_kinds; ++i) {
    const int rc = derive_kind(kinds[i], &p->kinds[i]);
    if (rc != JENGA_OK) { delete p; return rc; }
  }
  int64_t lcm = 0;
  int rc = lcm_of(p->kinds, &lcm);
  if (rc != JENGA_OK) { delete p; return rc; }
  if (large_page_bytes % lcm != 0) { delete p; return JENGA_ERR_INVALID; }
  p->base = static_cast<char*>(device_base);
  p->pool_bytes = pool_bytes;
  p->large_bytes = large_page_bytes;
  p->n_large = pool_bytes / large_page_bytes;
  for (Kind& k : p->kinds) {
    k.per_large = large_page_bytes / k.small_bytes;
    if (k.per_large > std::numeric_limits<int32_t>::max() ||
        p->n_large * k.per_large > std::numeric_limits<int32_t>::max()) {
      delete p;
      return JENGA_ERR_UNSUPPORTED;      // small ids are int32
    }
    k.used.assign(size_t((p->n_large * k.per_large + 63) / 64), 0);
  }
  p->large_kind.assign(size_t(p->n_large), -1);
  p->large_request.assign(size_t(p->n_large), 0);
  p->large_unused.assign(size_t(p->n_large), 0);
  for (int64_t i = 0; i < p->n_large; ++i) p->free_large.insert(p->free_large.end(), i);
  *out = p;
  return JENGA_OK;
}

int jenga_pool_destroy(jenga_pool* pool) {
  if (!pool) return JENGA_ERR_INVALID;
  delete pool;
  return JENGA_OK;
}

int jenga_alloc_small(jenga_pool* pool, int32_t kind, int64_t request, int32_t* out_small_id) {
  if (!kind_ok(pool, kind) || !out_small_id) return JENGA_ERR_INVALID;
  return alloc_small(pool, kind, request, out_small_id);
}

int jenga_ref_small(jenga_pool* pool, int32_t kind, int32_t small_id) {
  if (!kind_ok(pool, kind) || !small_live(pool, kind, small_id)) return JENGA_ERR_INVALID;
  ++pool->kinds[kind].extra_refs[small_id];
  return JENGA_OK;
}

int jenga_free_small(jenga_pool* pool, int32_t kind, int32_t small_id) {
  if (!kind_ok(pool, kind)) return JENGA_ERR_INVALID;
  return free_small(pool, kind, small_id);
}

int jenga_pool_get_info(const jenga_pool* pool, jenga_pool_info* out) {
  if (!pool || !out) return JENGA_ERR_INVALID;
  out->large_page_bytes = pool->large_bytes;
  out->n_large_pages = pool->n_large;
  out->free_large_pages = int64_t(pool->free_large.size());
  out->n_kinds = int32_t(pool->kinds.size());
  out->reserved = 0;
  return JENGA_OK;
}

int jenga_pool_kind_stats(const jenga_pool* pool, int32_t kind, jenga_kind_stats* out) {
  if (!kind_ok(pool, kind) || !out) return JENGA_ERR_INVALID;
  const Kind& k = pool->kinds[kind];
  out->small_page_bytes = k.small_bytes;
  out->slice_bytes = k.slice_bytes;
  out->small_per_large = k.per_large;
  out->owned_large_pages = k.owned_large;
  out->used_small_pages = k.used_small;
  out->unused_small_pages = k.owned_large * k.per_large - k.used_small;
  return JENGA_OK;
}

int jenga_large_page_owner(const jenga_pool* pool, int64_t large_page, int32_t* out_kind,
                           int64_t* out_request) {
  if (!pool || large_page < 0 || large_page >= pool->n_large || !out_kind || !out_request)
    return JENGA_ERR_INVALID;
  *out_kind = pool->large_kind[large_page];
  *out_request = pool->large_request[large_page];
  return JENGA_OK;
}

int jenga_small_refcount(const jenga_pool* pool, int32_t kind, int32_t small_id, int32_t* out) {
  if (!kind_ok(pool, kind) || !out) return JENGA_ERR_INVALID;
  const Kind& k = pool->kinds[kind];
  if (small_id < 0 || int64_t(small_id) >= pool->n_large * k.per_large) return JENGA_ERR_INVALID;
  if (!bit_get(k.used, small_id)) { *out = 0; return JENGA_OK; }
  auto it = k.extra_refs.find(small_id);
  *out = 1 + (it == k.extra_refs.end() ? 0 : it->second);
  return JENGA_OK;
}

int jenga_kv_offset(const jenga_pool* pool, int32_t kind, int32_t small_id, int32_t layer,
                    int32_t kv_head, int32_t is_v, int32_t token_in_page, int64_t* out_bytes) {
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
}

int jenga_request_extend(jenga_pool* pool, int64_t request, int32_t kind, int64_t new_len) {
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
    const int rc = alloc_small(pool, kind, request, &sid);
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
}

int jenga_request_share_prefix(jenga_pool* pool, int64_t src_request, int64_t dst_request,
                               int32_t kind, int32_t n_pages) {
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
}

int jenga_request_free(jenga_pool* pool, int64_t request) {
  if (!pool) return JENGA_ERR_INVALID;
  auto it = pool->requests.find(request);
  if (it == pool->requests.end()) return JENGA_ERR_INVALID;
  for (size_t kind = 0; kind < it->second.pages.size(); ++kind)
    for (int32_t sid : it->second.pages[kind])
      if (sid >= 0) free_small(pool, int32_t(kind), sid);
  pool->requests.erase(it);
  return JENGA_OK;
}

int jenga_request_num_pages(const jenga_pool* pool, int64_t request, int32_t kind, int32_t* out) {
  if (!kind_ok(pool, kind) || !out) return JENGA_ERR_INVALID;
  auto it = pool->requests.find(request);
  *out = it == pool->requests.end() ? 0 : int32_t(it->second.pages[kind].size());
  return JENGA_OK;
}

int jenga_request_block_table_row(const jenga_pool* pool, int64_t request, int32_t kind,
                                  int32_t* row, int32_t width) {
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
}

int jenga_requests_extend(jenga_pool* pool, int32_t kind, const int64_t* requests,
                          const int64_t* new_lens, int32_t n) {
  if (!kind_ok(pool, kind) || n < 0 || (n > 0 && (!requests || !new_lens))) return JENGA_ERR_INVALID;
  for (int32_t i = 0; i < n; ++i) {
    const int rc = jenga_request_extend(pool, requests[i], kind, new_lens[i]);
    if (rc != JENGA_OK) return rc;
  }
  return JENGA_OK;
}

int jenga_block_table_fill(const jenga_pool* pool, int32_t kind, const int64_t* requests, int32_t n,
                           int32_t* table, int32_t width) {
  if (!kind_ok(pool, kind) || n < 0 || width < 0 || (n > 0 && (!requests || !table)))
    return JENGA_ERR_INVALID;
  for (int32_t i = 0; i < n; ++i) {
    const int rc = jenga_request_block_table_row(pool, requests[i], kind, table + int64_t(i) * width, width);
    if (rc != JENGA_OK) return rc;
  }
  return JENGA_OK;
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
