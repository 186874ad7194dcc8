// Shared by the decode kernel's front end and engine (device code, gfx950): launch parameters,
// the flat work partitioning, element types and the page-id registers.
// Included by kernels.hip only; everything lives in that file's unnamed namespace.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

constexpr int kWave = 64;
constexpr int kMaxBatch = 1024;         // up to here the per-request prefix sums are made by every block, in LDS;
                                        // larger batches get them from a kernel of their own, through the workspace
constexpr int kMaxGridBatch = 65535;    // one row of reduction blocks per request: the grid's y limit
constexpr int kMaxPartitions = 8192;    // bound of the automatic grid (sizes the workspace)
// Starting on a segment (block-table row, query rows, first loads, final merge and store) costs a
// wavefront about as long as streaming two tiles (measured: 4.4 to 5 us against 2.5 us per
// tile); the flat space charges every segment a few units before its first tile, so that a
// chunk that spans a segment boundary gets fewer tiles and finishes with the others.  Measured
// with 1, 2, 3, 4 and 6 units on four workloads: 3 is best or equal to the best on each.
constexpr int kSegStartUnits = 3;
constexpr float kNegBig = -1.0e30f;     // finite stand-in for -inf: keeps exp2(m - m) well defined

struct DecodeParams {
  const char* layer_base;     // pool base + layer * slice_bytes
  int64_t small_bytes;        // page stride
  int32_t head_stride;        // bytes between KV heads inside a layer slice: 2 * T * D * e
  int32_t v_offset;           // bytes from a head's K rows to its V rows: T * D * e
  int32_t t_log2;             // log2 of the tokens per page, or minus the tokens per page if that is no power of two
  int32_t tokens_per_page;
  int32_t n_kv_heads;
  int32_t n_q_heads;
  int32_t group;           // query heads per KV head
  int32_t max_page_id;        // ids read from the block table are clamped to [0, max_page_id]
  const void* q;
  const int32_t* block_table;
  int32_t bt_stride;
  const int32_t* seq_lens;
  int32_t batch;
  int32_t max_seq_len;
  int32_t window;
  float scale_log2;           // softmax scale * log2(e): scores live in the base-2 domain
  int32_t chunk_tiles;        // > 0: tiles per partition; 0: ceil(W / gridDim.x)
  int32_t min_chunk_tiles;    // lower bound of the automatic chunk
  const void* k_new;          // fused append: [batch][n_kv_heads][D] rows of the token at L - 1, or NULL
  const void* v_new;
  float* ws_acc;              // [slot][G][D]
  float* ws_ml;               // [slot][G][2]  (running max, running sum)
  int32_t* ws_meta;           // [segment][2]  first and last chunk that hold tiles of the segment
  const int32_t* ws_incl;     // batch > kMaxBatch: [batch] inclusive prefix sums of the requests' flat units
  const int32_t* ws_len;      //                    [batch] clamped lengths, negated where the clamp took effect
  float* out;                 // [batch][n_q_heads][D] when the reduction of the same call follows, else NULL:
                              // a record that covers its whole segment is then written there, normalised
};

// Page of a token and first token of a page; t_log2 as in DecodeParams (negative: minus the page
// size, which is then no power of two and costs a division).
__device__ __forceinline__ int page_of_token(int t_log2, int t) { return t_log2 >= 0 ? t >> t_log2 : t / -t_log2; }
__device__ __forceinline__ int first_token_of(int t_log2, int page) { return t_log2 >= 0 ? page << t_log2 : page * -t_log2; }

// Visible pages [p_lo, p_hi) and first visible token of a request of length L.
__device__ __forceinline__ void visible_pages(int L, int window, int t_log2, int* lo_tok,
                                              int* p_lo, int* p_hi) {
  const int lo = window > 0 ? max(0, L - window) : 0;
  *lo_tok = lo;
  *p_lo = page_of_token(t_log2, lo);
  *p_hi = page_of_token(t_log2, L - 1) + 1;                 // L >= 1
}

// Units of the flat space one (request, KV head) segment takes: kSegStartUnits, then one per
// tile (of 2^tile_log2 tokens, counted from the first visible page).  0 for an empty request.
__device__ __forceinline__ int units_of(int L, int window, int t_log2, int tile_log2) {
  if (L <= 0) return 0;
  int lo_tok, p_lo, p_hi;
  visible_pages(L, window, t_log2, &lo_tok, &p_lo, &p_hi);
  return kSegStartUnits + ((first_token_of(t_log2, p_hi - p_lo) + (1 << tile_log2) - 1) >> tile_log2);
}

// R rounds of 64 requests (see scan_requests); rounds past the batch hold no request.
template <int R, class Units>
__device__ __forceinline__ int scan_rounds(const int32_t* seq_lens, int batch, int lane,
                                           int* s_incl, int* s_len, Units units) {
  int raw[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int i = r * kWave + lane;
    raw[r] = i < batch ? seq_lens[i] : 0;
  }
  int incl[R], enc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) incl[r] = units(raw[r], &enc[r]);
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int up = __shfl_up(incl[r], off);
      if (lane >= off) incl[r] += up;
    }
  }
  int carry = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int i = r * kWave + lane;
    incl[r] += carry;
    if (i < batch) {
      s_incl[i] = incl[r];
      s_len[i] = enc[r];
    }
    carry = __builtin_amdgcn_readlane(incl[r], kWave - 1);
  }
  __syncthreads();
  return carry;
}

// Inclusive prefix sums of units * n_kv_heads per request into LDS, lengths next to them: the
// length the kernels work with is min(seq_lens[i], max_seq_len), stored negated when the clamp
// took effect (such a request is attended over its first max_seq_len tokens, and its new row,
// whose position lies past what the caller sized the launch for, is not stored).
// Returns W.  All 64 lanes of the (single-wave) block take part.
__device__ __forceinline__ int scan_requests(const int32_t* seq_lens, int batch, int max_seq_len,
                                             int window, int t_log2, int tile_log2, int n_kv_heads,
                                             int lane, int* s_incl, int* s_len) {
  constexpr int kRounds = kMaxBatch / kWave;
  auto units = [&](int raw, int* enc) {
    const int Li = min(raw, max_seq_len);
    *enc = raw > max_seq_len ? -Li : Li;
    return units_of(Li, window, t_log2, tile_log2) * n_kv_heads;
  };
  if (batch <= kWave) {                        // one round: one load, one wave scan
    const int raw = lane < batch ? seq_lens[lane] : 0;
    int enc;
    int incl = units(raw, &enc);
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const int up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    if (lane < batch) {
      s_incl[lane] = incl;
      s_len[lane] = enc;
    }
    __syncthreads();
    return __builtin_amdgcn_readlane(incl, kWave - 1);
  }
  // Larger batches, 64 requests a round: lane l of round r takes request 64 r + l, so a round's
  // lengths are one coalesced 256-byte load.  All rounds are requested before any is used (one
  // memory round trip), each is scanned over the wavefront on its own (the scans do not depend on
  // one another, so they overlap), and the rounds' totals are carried along at the end.
  const int K = (batch + kWave - 1) / kWave;
  if (K <= 4) return scan_rounds<4>(seq_lens, batch, lane, s_incl, s_len, units);
  return scan_rounds<kRounds>(seq_lens, batch, lane, s_incl, s_len, units);
}

__device__ __forceinline__ int chunk_of(int chunk_tiles, int min_chunk_tiles, int W, int n_part) {
  return chunk_tiles > 0 ? chunk_tiles : max(min_chunk_tiles, (W + n_part - 1) / n_part);
}

// First request whose inclusive prefix exceeds flat position x (x < W).
static_assert(kMaxBatch <= kWave * kWave, "find_request searches the runs of 64 requests with one lane each");
__device__ __forceinline__ int find_request(const int* s_incl, int batch, int x, int lane) {
  // two rounds whatever the batch: which run of 64 requests, then which request in it
  // (s_incl is non-decreasing, so the first run whose last entry exceeds x holds the answer)
  int c0 = 0;
  if (batch > kWave) {
    const int n_runs = (batch + kWave - 1) / kWave;        // at most kMaxBatch / kWave = 16
    const int last = min((lane + 1) * kWave, batch) - 1;
    const bool past = lane < n_runs && s_incl[last] > x;
    const unsigned long long hit = __ballot(past);
    c0 = (hit ? __builtin_ctzll(hit) : n_runs - 1) * kWave;
  }
  const int i = c0 + lane;
  const bool past = i < batch && s_incl[i] > x;
  const unsigned long long hit = __ballot(past);
  return hit ? c0 + __builtin_ctzll(hit) : batch - 1;
}

// The same search in prefix sums that lie in global memory (batches above kMaxBatch): rounds of
// 64 probes, each cutting the range to a 64th, then the last 64 entries one per lane.
__device__ __forceinline__ int find_request_global(const int32_t* incl, int batch, int x, int lane) {
  int lo = 0, n = batch;
  while (n > kWave) {
    const int step = (n + kWave - 1) / kWave;
    const int first = lane * step;                          // this lane's part: [first, first + step) of the range
    const bool mine = first < n;
    const bool past = mine && incl[lo + min(first + step, n) - 1] > x;
    const unsigned long long hit = __ballot(past);
    const int f = hit ? __builtin_ctzll(hit) : (n - 1) / step;
    lo += f * step;
    n = min(step, n - f * step);
  }
  const bool past = lane < n && incl[lo + lane] > x;
  const unsigned long long hit = __ballot(past);
  return hit ? lo + __builtin_ctzll(hit) : batch - 1;
}

// ---- element types ---------------------------------------------------------------
struct F32 {
  static constexpr int kBytes = 4;
};
struct BF16 {
  static constexpr int kBytes = 2;
};

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));   // 16 bytes; a native vector, so it can be loaded non-temporally

// Page ids of the pages a wavefront is about to read, 128 at a time in two registers: lane j
// of register (c & 1) holds the id of page 64*c + j (relative to the first page).  A
// v_readlane turns one into a scalar, which makes the page's base address scalar too.  When
// the K and V requests of a tile enter run c of 64 pages, the register of run c+1 (== that of
// run c-1, which they have just left) is reloaded.
struct PageIds {
  const int32_t* row;   // block-table entry of relative page 0 (nullptr: nothing loaded yet)
  int n_pages;
  int n_loaded;         // pages the registers were loaded for (0 once a refill has replaced them)
  int lane;
  int max_id;
  int reg0, reg1;       // two scalars, not an array: an indexed member would live in scratch memory
  int next_run;         // k_stream_in: first page of the run whose entry triggers the next load

  // A table entry that is negative or past the pool (a caller error: pages of the visible
  // range must be resident) is clamped, so the kernel reads wrong data rather than faulting.
  __device__ __forceinline__ int fetch(int first) const {
    const int i = first + lane;
    return i < n_pages ? min(max(row[i], 0), max_id) : 0;
  }
  // The next (request, KV head) segment of a wavefront is usually the next head of the same
  // request, whose pages are the same ones: when the registers still hold the first 128 entries
  // of that very row, nothing is fetched (a segment start otherwise waits a memory round trip for
  // its page ids before it can request any K/V).
  __device__ __forceinline__ void init(const int32_t* r, int n, int l, int max_page_id) {
    if (r == row && n <= n_loaded) {
      n_pages = n;
      next_run = kWave;
      return;
    }
    row = r; n_pages = n; lane = l; max_id = max_page_id;
    n_loaded = n;
    next_run = kWave;
    reg0 = fetch(0);
    reg1 = fetch(kWave);
  }
  __device__ __forceinline__ int get(int page_rel) const {
    const int r = (page_rel & kWave) ? reg1 : reg0;
    return __builtin_amdgcn_readlane(r, page_rel & (kWave - 1));
  }
  // The id of a page that differs from lane to lane (pages of any size: a 16-token block then
  // takes its rows from several pages): two cross-lane reads, one per register.
  __device__ __forceinline__ int get_lane(int page_rel) const {
    const int a = __shfl(reg0, page_rel & (kWave - 1));
    const int b = __shfl(reg1, page_rel & (kWave - 1));
    return (page_rel & kWave) ? b : a;
  }
  // The same for pages of any size, where a run of 64 pages need not begin with a tile: called with
  // the page of the tile's first token, it loads run c+1 once the stream is in run c.
  __device__ __forceinline__ void k_stream_in(int page_rel) {
    if (page_rel >= next_run && next_run + kWave < n_pages) {
      const int next = fetch(next_run + kWave);
      if (next_run & kWave) reg0 = next;
      else reg1 = next;
      next_run += kWave;
      n_loaded = 0;
    }
  }
  // Call after the K stream has issued the loads of a tile starting at page_rel.
  __device__ __forceinline__ void k_stream_at(int page_rel) {
    if ((page_rel & (kWave - 1)) == 0 && page_rel > 0 && page_rel + kWave < n_pages) {
      const int next = fetch(page_rel + kWave);
      if (page_rel & kWave) reg0 = next;
      else reg1 = next;
      n_loaded = 0;       // the registers no longer hold the start of the row
    }
  }
};

}  // namespace
