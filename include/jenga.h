/*
 * jenga.h -- C ABI of the MI355X paged-decode hot path behind a heterogeneous
 * (multi layer type) KV-cache memory manager.
 *
 * Two halves:
 *   host   a two-level page allocator over one device memory pool: equal large
 *          pages whose size is a common multiple (normally the least one) of
 *          every layer type's small-page size, split on demand into small pages
 *          of one type, placed request-aware (paper Sec. 4.1, 4.3), plus the
 *          per-request page lists that become per-layer-type block tables
 *          (Sec. 4.2 item 2).  Never touches device memory.
 *   device HIP kernels for gfx950 that append one token's K/V into its page and
 *          run batched single-token decode attention through a layer type's
 *          block table (the kernel view of Sec. 4.2: start pointer, page size,
 *          page ids).
 *
 * Conventions
 *   - every function returns JENGA_OK (0) or a negative jenga_status; nothing
 *     throws across the boundary; jenga_strerror() names a status;
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP
 *     device memory of the current device; the library never allocates, frees or
 *     copies device memory and never synchronises a stream;
 *   - host calls on one pool are not thread safe (the caller serialises them, as
 *     a serving engine's single scheduler thread does);
 *   - device calls validate what the host can see, enqueue their kernels on
 *     `stream` and return; the caller orders them (append before decode on the
 *     same stream) and keeps every buffer alive until the stream has run them.
 *
 * Address map (all sizes in bytes; e = element size of the kind's dtype)
 *   small page `sid` of kind k starts at   device_base + sid * small_page_bytes[k]
 *   layer `l` of the kind inside it at      + l * slice,  slice = 2 * n_kv_heads * T * D * e
 *   KV head h inside the layer slice at     + h * (2 * T * D * e)
 *   K rows first, then V rows               + (is_v ? T * D * e : 0)
 *   token t of the page, element d          + (t * D + d) * e
 *   (page-layer partition of Sec. 4.2; the order inside a layer slice is this
 *   library's choice, the paper leaves it open.)
 */
#ifndef JENGA_H
#define JENGA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct jenga_pool jenga_pool;   /* opaque host object */
typedef void* jenga_stream;             /* a hipStream_t, or NULL for the null stream */

typedef enum {
  JENGA_OK = 0,
  JENGA_ERR_INVALID = -1,    /* bad argument, unknown id, double free, wrong kind type */
  JENGA_ERR_OOM = -2,        /* no page: every allocation step failed; also host memory exhausted */
  JENGA_ERR_ALIGN = -3,      /* a pointer or size is not 16-byte aligned */
  JENGA_ERR_WORKSPACE = -4,  /* split-K workspace too small */
  JENGA_ERR_HIP = -5,        /* a HIP runtime call failed */
  JENGA_ERR_UNSUPPORTED = -6 /* shape outside what the kernels are built for */
} jenga_status;

typedef enum { JENGA_F32 = 0, JENGA_BF16 = 1 } jenga_dtype;

typedef enum {
  JENGA_FULL = 0,    /* attends to every cached token */
  JENGA_WINDOW = 1,  /* attends to the last `window` tokens, the newest included (Sec. 3.1 a, 5.1) */
  JENGA_CROSS = 2,   /* fixed encoder (image) K/V, written once, no append (Sec. 3.1 c) */
  JENGA_OPAQUE = 3   /* pages the kernels never read, e.g. a state-space layer's state (Sec. 3.1 b) */
} jenga_kind_type;

/* One layer type ("kind").  For attention kinds a small page holds tokens_per_page
 * tokens for all n_layers layers of the kind (Sec. 4.1 footnote, Sec. 4.2). */
typedef struct {
  int32_t type;             /* jenga_kind_type */
  int32_t dtype;            /* jenga_dtype of K/V (and of q, k_new, v_new) */
  int32_t n_layers;         /* >= 1 */
  int32_t n_kv_heads;       /* attention kinds: >= 1 */
  int32_t head_dim;         /* attention kinds: 64, 128 or 256 */
  int32_t tokens_per_page;  /* attention kinds: 1 .. 4096 (Sec. 4.1 footnote: arbitrary; 16, 32, 64, 128 and 8
                               run on the fast addressing paths); OPAQUE: 1 */
  int32_t window;           /* WINDOW kinds: > 0; others: 0 */
  int32_t reserved;         /* 0 */
  int64_t small_page_bytes; /* 0: n_layers * slice for attention kinds; otherwise at least that,
                               and a multiple of 16.  OPAQUE kinds must give it. */
} jenga_kind_desc;

typedef struct {
  int64_t large_page_bytes;
  int64_t n_large_pages;
  int64_t free_large_pages;
  int32_t n_kinds;
  int32_t reserved;
} jenga_pool_info;

typedef struct {
  int64_t small_page_bytes;
  int64_t slice_bytes;        /* one layer's part of a small page (0 for OPAQUE) */
  int64_t small_per_large;    /* r_k = large_page_bytes / small_page_bytes */
  int64_t owned_large_pages;  /* large pages currently split into pages of this kind */
  int64_t used_small_pages;   /* reference count > 0 */
  int64_t unused_small_pages; /* empty ones inside owned large pages: internal fragmentation (Sec. 4.3, 4.4) */
  int64_t evictable_small_pages; /* valid contents, no user (Sec. 5.4) */
} jenga_kind_stats;

/* State of a small page under prefix caching (Sec. 5.4). */
typedef enum { JENGA_PAGE_EMPTY = 0, JENGA_PAGE_EVICTABLE = 1, JENGA_PAGE_USED = 2 } jenga_page_state;
/* Customised hit rules of Sec. 5.2 / 5.3. */
typedef enum { JENGA_HIT_FULL = 0, JENGA_HIT_WINDOW = 1, JENGA_HIT_EVERY = 2 } jenga_hit_rule;

/* ------------------------------------------------------------------ host: pool */

/* Least common multiple of the kinds' small-page sizes: the compatible page size of
 * Sec. 1 / Sec. 4.1 (2 KB, 3 KB -> 6 KB; 256, 384 -> 768).  kinds: host array.
 * Errors: INVALID (bad descriptor), ALIGN, UNSUPPORTED (overflow of int64). */
int jenga_lcm_page_bytes(const jenga_kind_desc* kinds, int32_t n_kinds, int64_t* out_bytes);

/* Create the allocator over [device_base, device_base + pool_bytes).  The pool is cut
 * into floor(pool_bytes / large_page_bytes) large pages, all free (Sec. 4.1).
 * large_page_bytes must be a positive common multiple of every kind's small-page size
 * (pass jenga_lcm_page_bytes() for the paper's choice).  device_base is borrowed, must be
 * 256-byte aligned, and may be NULL for host-only use (device calls then fail INVALID).
 * The descriptors are copied.  *out is owned by the caller until jenga_pool_destroy. */
int jenga_pool_create(void* device_base, int64_t pool_bytes, int64_t large_page_bytes,
                      const jenga_kind_desc* kinds, int32_t n_kinds, jenga_pool** out);
int jenga_pool_destroy(jenga_pool* pool);

/* allocate() of Sec. 4.1 with the request-aware order of Sec. 4.3:
 *   1. an unused small page of this kind inside a large page associated with `request`;
 *   2. else a free large page: it becomes this kind's, all its small pages associated
 *      with `request`;
 *   3. else an unused small page of this kind associated with another request;
 *   else JENGA_ERR_OOM.
 * Ties: lowest-numbered large page, lowest slot in it.  The id returned is global for the
 * kind: id = large_page * small_per_large + slot, so id * small_page_bytes is its byte
 * offset from device_base (Sec. 4.1 last paragraph).  Its reference count starts at 1. */
int jenga_alloc_small(jenga_pool* pool, int32_t kind, int64_t request, int32_t* out_small_id);
/* One more reference to a live small page (prefix sharing). INVALID if it is unused. */
int jenga_ref_small(jenga_pool* pool, int32_t kind, int32_t small_id);
/* free(small_page_id) of Sec. 4.1: drop one reference; at zero the page is unused, and if
 * every small page of its large page is unused the large page returns to level 1 at once
 * and loses its kind and request.  INVALID on an unused page (double free). */
int jenga_free_small(jenga_pool* pool, int32_t kind, int32_t small_id);

int jenga_pool_get_info(const jenga_pool* pool, jenga_pool_info* out);
int jenga_pool_kind_stats(const jenga_pool* pool, int32_t kind, jenga_kind_stats* out);
/* Kind owning a large page (-1: free) and the request it is associated with (Sec. 4.3). */
int jenga_large_page_owner(const jenga_pool* pool, int64_t large_page, int32_t* out_kind,
                           int64_t* out_request);
int jenga_small_refcount(const jenga_pool* pool, int32_t kind, int32_t small_id, int32_t* out);
/* Byte offset from device_base of element 0 of (small page, layer, kv head, K or V, token). */
int jenga_kv_offset(const jenga_pool* pool, int32_t kind, int32_t small_id, int32_t layer,
                    int32_t kv_head, int32_t is_v, int32_t token_in_page, int64_t* out_bytes);

/* ------------------------------------------- host: per-request page lists / block tables */

/* Make kind `kind` of `request` hold tokens [0, new_len): logical pages are appended with
 * jenga_alloc_small until ceil(new_len / tokens_per_page) exist; then, for WINDOW kinds,
 * every resident page p with tokens_per_page * (p + 1) <= new_len - window is freed and its
 * entry becomes -1 (only the window is needed, Sec. 5.1).  For OPAQUE kinds new_len counts
 * pages.  On OOM the pages obtained so far are kept and the error returned. */
int jenga_request_extend(jenga_pool* pool, int64_t request, int32_t kind, int64_t new_len);
/* dst (which must have no pages of this kind) starts as a sharer of src's first n_pages
 * logical pages: each resident one gets one more reference. */
int jenga_request_share_prefix(jenga_pool* pool, int64_t src_request, int64_t dst_request,
                               int32_t kind, int32_t n_pages);
/* The request finished: drop its reference on every page of every kind, forget it. */
int jenga_request_free(jenga_pool* pool, int64_t request);
int jenga_request_num_pages(const jenga_pool* pool, int64_t request, int32_t kind, int32_t* out);
/* Row of kind `kind`'s block table for `request`: row[p] = small id of logical page p, -1 if
 * not resident; entries past the request's pages are -1.  row: host, `width` entries.
 * INVALID if the request has more than `width` pages. */
int jenga_request_block_table_row(const jenga_pool* pool, int64_t request, int32_t kind,
                                  int32_t* row, int32_t width);

/* Batched forms for a decode step over n requests (host arrays of n entries):
 * jenga_requests_extend == jenga_request_extend(requests[i], kind, new_lens[i]) for i in order,
 * stopping at the first error; jenga_block_table_fill writes row i of a host table
 * [n][width] as jenga_request_block_table_row does. */
int jenga_requests_extend(jenga_pool* pool, int32_t kind, const int64_t* requests,
                          const int64_t* new_lens, int32_t n);
int jenga_block_table_fill(const jenga_pool* pool, int32_t kind, const int64_t* requests, int32_t n,
                           int32_t* table, int32_t width);

/* ------------------------------------------------- host: prefix-cache side (paper Sec. 5) */

/* jenga_alloc_small is the five-step allocation of Sec. 5.4:
 *   1. an empty small page associated with the request;  2. an empty large page;
 *   3. evict the least recently used evictable large page (of any kind; it is re-typed);
 *   4. an empty small page of the kind associated with another request;
 *   5. evict the least recently used evictable small page of the kind.
 * With nothing evictable this is the three-step order of Sec. 4.3.  A large page is evictable
 * when all its small pages are evictable (Sec. 5.4: one used or one empty small page keeps it
 * out of step 3); its LRU time is the latest last access among all its small pages.  Among
 * equal times the larger prefix length goes first (Sec. 5.1), then the lower number.  After
 * step 3 every small page of the large page is empty.  This variant also reports what was evicted,
 * so the caller can drop it from its prefix index: up to `capacity` (kind, id) pairs are
 * written to the host arrays (either may be NULL), *out_n_evicted gets the full count. */
int jenga_alloc_small_evict(jenga_pool* pool, int32_t kind, int64_t request, int32_t* out_small_id,
                            int32_t* evicted_kinds, int32_t* evicted_ids, int32_t capacity,
                            int32_t* out_n_evicted);
/* Like jenga_free_small, but at reference count zero the page stays evictable (valid contents
 * kept for later prefix hits) when keep_cached != 0. */
int jenga_release_small(jenga_pool* pool, int32_t kind, int32_t small_id, int32_t keep_cached);
/* Prefix-cache hit: an evictable page is used again (reference count 1).  INVALID otherwise. */
int jenga_acquire_cached(jenga_pool* pool, int32_t kind, int32_t small_id);
/* LRU keys of Sec. 5.1 (update_last_access, set_prefix_length) for a used or evictable page. */
int jenga_set_last_access(jenga_pool* pool, int32_t kind, int32_t small_id, int64_t time);
int jenga_set_prefix_length(jenga_pool* pool, int32_t kind, int32_t small_id, int64_t length);
int jenga_small_state(const jenga_pool* pool, int32_t kind, int32_t small_id, int32_t* out_state);
/* Request-level forms: release every page of the request (evictable if keep_cached); stamp
 * the pages covering tokens [first_token, end_token) of one kind with `time` (the layer type
 * decides the range: everything for full attention, the window for sliding-window layers,
 * Sec. 5.1); give page p of the request prefix length (p + 1) * tokens_per_page. */
int jenga_request_release(jenga_pool* pool, int64_t request, int32_t keep_cached);
int jenga_request_touch(jenga_pool* pool, int64_t request, int32_t kind, int64_t first_token,
                        int64_t end_token, int64_t time);
int jenga_request_set_prefix_lengths(jenga_pool* pool, int64_t request, int32_t kind);

/* get_possible_prefix of Sec. 5.2: is_hit[t] != 0 when token t (0-based) is cached for the
 * layer type; out_valid (host, n_tokens + 1 bytes) gets out_valid[p] = 1 when the prefix of p
 * tokens is a valid hit.  JENGA_HIT_FULL: all p tokens cached.  JENGA_HIT_WINDOW: the last
 * min(param, p) tokens cached.  JENGA_HIT_EVERY: p is a multiple of param and token p - 1 is
 * cached (state-space layers cache one state every 512 tokens, Sec. 5.3). */
int jenga_possible_prefixes(int32_t rule, int32_t param, const uint8_t* is_hit, int32_t n_tokens,
                            uint8_t* out_valid);
/* Longest prefix valid for every layer type (Sec. 5.2): valid_sets[s] as written by
 * jenga_possible_prefixes.  Returns the length (0: none) or a negative status. */
int jenga_longest_common_prefix(const uint8_t* const* valid_sets, int32_t n_sets, int32_t n_tokens);

/* ------------------------------------------------------------------------ device: kernels */

/* Store the new token's K and V of one layer for every request of the batch ("store KV
 * cache for each token", Sec. 2): for request b with L = seq_lens[b] > 0 the token at
 * position L - 1 goes to page block_table[b][(L - 1) / T], row (L - 1) % T (address map
 * above).  k_new, v_new: device, [batch][n_kv_heads][head_dim] in the kind's dtype, 16-byte
 * aligned.  block_table: device int32 [batch][bt_stride]; seq_lens: device int32 [batch],
 * lengths *after* this append.  Requests with L <= 0 or a negative table entry are skipped.
 * Errors: INVALID for CROSS / OPAQUE kinds, bad layer, NULL pointers, batch < 0. */
int jenga_kv_append(const jenga_pool* pool, int32_t kind, int32_t layer,
                    const void* k_new, const void* v_new,
                    const int32_t* block_table, int32_t bt_stride,
                    const int32_t* seq_lens, int32_t batch, jenga_stream stream);

/* Bulk form of jenga_kv_append for a run of tokens per request (the write a chunked prefill
 * does just before decoding starts, Sec. 6.2): request b owns source rows
 * [cu_tokens[b], cu_tokens[b+1]) and its first row is the token at sequence position
 * start_pos[b]; row r of k_src / v_src is [n_kv_heads][head_dim] in the kind's dtype.  Tokens
 * whose page is not resident (negative table entry, e.g. a window page that already slid out)
 * are skipped.  k_src, v_src: device, [total_tokens][n_kv_heads][head_dim], 16-byte aligned;
 * cu_tokens: device int32 [batch + 1], non-decreasing, cu_tokens[batch] <= total_tokens;
 * start_pos: device int32 [batch]; block_table as for jenga_kv_append.  Works for FULL, WINDOW
 * and CROSS kinds (encoder K/V is written once this way).  Errors as jenga_kv_append. */
int jenga_kv_write_range(const jenga_pool* pool, int32_t kind, int32_t layer,
                         const void* k_src, const void* v_src, const int32_t* cu_tokens,
                         const int32_t* start_pos, const int32_t* block_table, int32_t bt_stride,
                         int32_t batch, int32_t total_tokens, jenga_stream stream);

/* Upper bound of the number of work partitions (wavefront tasks) the decode kernels use for
 * these arguments.  The visible K/V of all (request, KV head) pairs, cut into tiles and laid
 * end to end (each pair charged a few extra units for the cost of starting on it), is divided
 * into equal partitions; pages_per_split = 0 lets the library take one partition per
 * wavefront the device can hold at once (every wavefront then has the same amount of work
 * whatever the mix of lengths), pages_per_split > 0 fixes the partition size.
 * Returns the bound (>= 1) or a negative status. */
int jenga_decode_num_partitions(const jenga_pool* pool, int32_t kind, int32_t n_q_heads,
                                int32_t batch, int32_t max_seq_len, int32_t window,
                                int32_t pages_per_split);
/* Bytes of split-K workspace jenga_paged_decode needs for these arguments (> 0), or a
 * negative status: one (max, sum, accumulator) record per query head for each of
 * (partitions + batch * n_kv_heads) slots, plus 8 bytes per (request, KV head), plus 8 bytes per
 * request for batches above 1024 (whose per-request prefix sums a small kernel of its own leaves
 * there for the decode kernel; up to 1024 requests every block makes them for itself). */
int64_t jenga_decode_workspace_bytes(const jenga_pool* pool, int32_t kind, int32_t n_q_heads,
                                     int32_t batch, int32_t max_seq_len, int32_t window,
                                     int32_t pages_per_split);

/* Batched single-token decode attention of one layer through the kind's block table
 * (kernel interface of Sec. 4.2).  For request b and query head h (KV head h / G,
 * G = n_q_heads / n_kv_heads):
 *     out[b][h][:] = sum_{t in Vis_b} softmax_t(scale * <q[b][h], K_t>) * V_t
 * Vis_b = [max(0, L_b - window), L_b) if window > 0, else [0, L_b), L_b = seq_lens[b]
 * (for CROSS kinds L_b is the encoder length).  fp32 accumulation; out is fp32
 * [batch][n_q_heads][head_dim]; L_b <= 0 gives zeros.
 *   q            device, [batch][n_q_heads][head_dim] in the kind's dtype, 16-byte aligned
 *   k_new, v_new both NULL, or the new token's rows exactly as for jenga_kv_append (FULL and
 *                WINDOW kinds only): the append is then done inside the decode kernel -- the
 *                wavefront that reads a request's last page takes the row at position L - 1
 *                from k_new / v_new, stores it into the page, and attends to it -- which saves
 *                the separate jenga_kv_append launch (for very large batches of short requests
 *                the library still runs the append as a launch of its own in front, which is
 *                faster there).  Pool contents and results are identical either way.
 *   block_table  device int32 [batch][bt_stride]; every page overlapping Vis_b must be
 *                resident (>= 0); other entries are never read
 *   seq_lens     device int32 [batch], each <= max_seq_len.  A larger one (a caller error, e.g. a
 *                stale max_seq_len) is clamped in both kernels: the request is attended over its
 *                first max_seq_len tokens, and its k_new / v_new rows are NOT stored (their
 *                position lies outside what the launch was sized for)
 *   max_seq_len  host upper bound of seq_lens; sizes the grid; bt_stride * T >= max_seq_len
 *   window       0: none.  WINDOW kinds: the kind's window (a smaller positive one is allowed,
 *                0 or a larger one is INVALID: those pages are not resident).
 *   pages_per_split  0: automatic (balanced partitions); else the partition size in pages of K/V
 *   workspace    device, >= jenga_decode_workspace_bytes(...), 16-byte aligned, caller-owned;
 *                holds per-partition (max, sum, accumulator) between the two kernels
 * Runs the partial kernel and the split-K reduction on `stream`.
 * Errors: INVALID, ALIGN, WORKSPACE, UNSUPPORTED (G > 16; batch > 65535; more than 2^30 tiles
 * over all (request, KV head) pairs), HIP. */
int jenga_paged_decode(const jenga_pool* pool, int32_t kind, int32_t layer,
                       const void* q, int32_t n_q_heads,
                       const void* k_new, const void* v_new,
                       const int32_t* block_table, int32_t bt_stride,
                       const int32_t* seq_lens, int32_t batch, int32_t max_seq_len,
                       int32_t window, float scale, int32_t pages_per_split,
                       void* workspace, int64_t workspace_bytes,
                       float* out, jenga_stream stream);
/* The two kernels of jenga_paged_decode one at a time (same arguments, same checks):
 * the partial kernel fills `workspace`; the reduction merges it into `out` by the
 * log-sum-exp rule  m* = max m_i,  out = sum_i acc_i 2^(m_i - m*) / sum_i l_i 2^(m_i - m*). */
int jenga_paged_decode_partial(const jenga_pool* pool, int32_t kind, int32_t layer,
                               const void* q, int32_t n_q_heads,
                               const void* k_new, const void* v_new,
                               const int32_t* block_table, int32_t bt_stride,
                               const int32_t* seq_lens, int32_t batch, int32_t max_seq_len,
                               int32_t window, float scale, int32_t pages_per_split,
                               void* workspace, int64_t workspace_bytes, jenga_stream stream);
int jenga_splitk_reduce(const jenga_pool* pool, int32_t kind, int32_t n_q_heads,
                        const int32_t* seq_lens, int32_t batch, int32_t max_seq_len,
                        int32_t window, int32_t pages_per_split,
                        const void* workspace, int64_t workspace_bytes,
                        float* out, jenga_stream stream);

#define JENGA_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)
/* For callers that cannot allocate device memory -- code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc: jenga_paged_decode without the workspace arguments.
 * The records between the two kernels live in a buffer inside the library (a file-scope device
 * array of JENGA_STATIC_SCRATCH_BYTES = 32 MiB, which every GPU the library runs on holds
 * until the process ends); the call allocates and frees nothing, on the device or through any
 * allocating library routine.  Arguments, checks and results are those of jenga_paged_decode
 * (bit-identical output for pages_per_split = 0 and for any other value).
 * Limit: JENGA_ERR_WORKSPACE when the records of this launch need more than the buffer:
 *   (partitions + batch * n_kv_heads) * G * (head_dim + 2) * 4 + batch * n_kv_heads * 8  bytes,
 * partitions = wavefronts the device holds at once, 1024 on an MI355X (e.g. batch 1024 with 8 KV
 * heads, G = 4, head_dim 128 needs 19.2 MB; the Gemma-2-9B shape at batch 64 3.2 MB).
 * Every call on one GPU uses that GPU's buffer: calls that may overlap on one GPU (different
 * streams, or graphs replayed concurrently) race and must be serialised by the caller.  Nothing
 * in the buffer has to start at zero; each call overwrites what it reads.
 * The buffer's address on a GPU is looked up once, when the first pool is created with that GPU
 * current (else by the first call there, which should then not run under stream capture).
 * Further errors: HIP (no current device, or the buffer's address cannot be found). */
int jenga_paged_decode_static(const jenga_pool* pool, int32_t kind, int32_t layer,
                              const void* q, int32_t n_q_heads,
                              const void* k_new, const void* v_new,
                              const int32_t* block_table, int32_t bt_stride,
                              const int32_t* seq_lens, int32_t batch, int32_t max_seq_len,
                              int32_t window, float scale, int32_t pages_per_split,
                              float* out, jenga_stream stream);

/* Measurement aids (not on the hot path): a plain device copy and a plain device read of
 * `bytes` (multiple of 16) with 16-byte accesses, used to find the achievable HBM rate and
 * to calibrate profiler byte counters.  `sink`: device, >= 4 bytes. */
int jenga_stream_copy(void* dst, const void* src, int64_t bytes, jenga_stream stream);
int jenga_stream_read(const void* src, int64_t bytes, void* sink, jenga_stream stream);

const char* jenga_strerror(int status);
/* 0xMMmmpp */
int jenga_version(void);

#ifdef __cplusplus
}
#endif
#endif /* JENGA_H */
