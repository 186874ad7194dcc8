// Device half of the library, written for gfx950 (CDNA4, 64-wide wavefronts).
//
//   kv_append_kernel       stores the new token's K/V rows into their page
//   kv_write_range_kernel  stores a run of tokens per request (chunked prefill) the same way
//   decode_partial_kernel  streams K and V pages through a layer type's block table with
//                          16-byte non-temporal loads, fp32 online softmax, the G query heads
//                          of a KV head share every load; one wavefront per work partition
//   splitk_reduce_kernel   log-sum-exp merge of the partitions of each (request, query head)
//
// Decode attention is bandwidth-bound (G flop per byte of bf16 K/V).  What decides the speed
// is (1) that every wavefront always has KiB-sized loads in flight, (2) that no wavefront
// idles while others still work (work is cut into equal pieces, not into per-request pieces),
// and (3) that the arithmetic stays out of the way of the loads.  Three engines share the
// front end: the matrix-core engine (bf16 K/V, pages of 16 tokens or more: both products of
// a 16-token block are small dense contractions and go through MFMA, which leaves the vector
// ALUs almost idle and is what keeps 8 and 16 heads per KV head at the HBM rate), the quad
// engine (16-token pages on the vector ALUs: fp32 K/V, and 256-element bf16 rows with few
// heads, where it measures slightly faster), and the general row engine (the rest).
//
// The kernel view of the pool is the one of paper Sec. 4.2: a start pointer (pool base +
// layer offset), a page stride (the kind's small-page size) and page ids (the kind's block
// table).
//
// Work partitioning ("flat" split-K).  The visible K/V of request b is cut into tiles (a
// fixed number of tokens, one or a few pages).  All tiles of all (request, KV head) pairs are
// laid end to end, request-major then head then token order, each segment preceded by a few
// units that stand for the cost of starting on it, W units in total, and cut into equal chunks
// of C units; wavefront w owns units [w*C, (w+1)*C).  A chunk usually lies inside
// one (request, head) segment and sometimes spans the end of one and the start of the next;
// for every segment it touches, the wavefront writes one partial record (running max, running
// sum, un-normalised accumulator) to slot  segment_index + w  of the workspace: both terms
// are non-decreasing along the flat order and one of them increases from one record to the
// next, so slots never collide, and the records of a segment are consecutive.  With the
// automatic chunk size C = ceil(W / partitions) every wavefront has the same amount of work
// whatever the mix of sequence lengths, the grid is one resident wave of blocks, and
// consecutive blocks -- which the hardware deals round-robin to the 8 XCDs -- carry equal
// work.  W and the per-request offsets are recomputed by every block from seq_lens (one
// coalesced load and a wave scan per 64 requests), so the host needs no knowledge of the
// lengths and never synchronises.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <mutex>
#include <unordered_map>

#include "pool_internal.hpp"

namespace {

constexpr int kWave = 64;
constexpr int kMaxBatch = 1024;         // per-request prefix sums are kept in LDS
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
  int32_t t_log2;
  int32_t n_kv_heads;
  int32_t n_q_heads;
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
};

// Visible pages [p_lo, p_hi) and first visible token of a request of length L.
__device__ __forceinline__ void visible_pages(int L, int window, int t_log2, int* lo_tok,
                                              int* p_lo, int* p_hi) {
  const int lo = window > 0 ? max(0, L - window) : 0;
  *lo_tok = lo;
  *p_lo = lo >> t_log2;
  *p_hi = (L + (1 << t_log2) - 1) >> t_log2;
}

// Units of the flat space one (request, KV head) segment takes: kSegStartUnits, then one per
// tile (of 2^tile_log2 tokens, counted from the first visible page).  0 for an empty request.
__device__ __forceinline__ int units_of(int L, int window, int t_log2, int tile_log2) {
  if (L <= 0) return 0;
  int lo_tok, p_lo, p_hi;
  visible_pages(L, window, t_log2, &lo_tok, &p_lo, &p_hi);
  return kSegStartUnits + ((((p_hi - p_lo) << t_log2) + (1 << tile_log2) - 1) >> tile_log2);
}

// Inclusive prefix sums of units * n_kv_heads per request into LDS, lengths next to them.
// Returns W.  All 64 lanes of the (single-wave) block take part.
__device__ __forceinline__ int scan_requests(const int32_t* seq_lens, int batch, int max_seq_len,
                                             int window, int t_log2, int tile_log2, int n_kv_heads,
                                             int lane, int* s_incl, int* s_len) {
  int run = 0;
  for (int c0 = 0; c0 < batch; c0 += kWave) {
    const int i = c0 + lane;
    const int Li = i < batch ? min(seq_lens[i], max_seq_len) : 0;
    int incl = units_of(Li, window, t_log2, tile_log2) * n_kv_heads;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const int up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    if (i < batch) {
      s_incl[i] = run + incl;
      s_len[i] = Li;
    }
    run += __builtin_amdgcn_readlane(incl, kWave - 1);
  }
  __syncthreads();
  return run;
}

__device__ __forceinline__ int chunk_of(int chunk_tiles, int min_chunk_tiles, int W, int n_part) {
  return chunk_tiles > 0 ? chunk_tiles : max(min_chunk_tiles, (W + n_part - 1) / n_part);
}

// First request whose inclusive prefix exceeds flat position x (x < W).
__device__ __forceinline__ int find_request(const int* s_incl, int batch, int x, int lane) {
  for (int c0 = 0; c0 < batch; c0 += kWave) {
    const int i = c0 + lane;
    const bool past = i < batch && s_incl[i] > x;
    const unsigned long long hit = __ballot(past);
    if (hit) return c0 + __builtin_ctzll(hit);
  }
  return batch - 1;
}

// ---- cross-lane helpers ------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true);
  return x + __int_as_float(y);
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_max(float x) {
  const int y = __builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), CTRL, ROW_MASK, 0xf, false);
  return fmaxf(x, __int_as_float(y));
}

// Maximum over the wave, in an SGPR-uniform value.
__device__ __forceinline__ float wave_max(float x) {
  x = dpp_max<0xB1, 0xf>(x);    // lane ^ 1
  x = dpp_max<0x4E, 0xf>(x);    // lane ^ 2
  x = dpp_max<0x124, 0xf>(x);   // row_ror:4
  x = dpp_max<0x128, 0xf>(x);   // row_ror:8  -> every lane holds its row's maximum
  x = dpp_max<0x142, 0xa>(x);   // row_bcast:15 into rows 1 and 3
  x = dpp_max<0x143, 0xc>(x);   // row_bcast:31 into rows 2 and 3 -> lane 63 holds the maximum
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), kWave - 1));
}

// Sum over aligned groups of LANES lanes, result in every lane of the group.
template <int LANES>
__device__ __forceinline__ float group_sum(float x) {
  static_assert(LANES == 8 || LANES == 16 || LANES == 32 || LANES == 64, "group size");
  x = dpp_add<0xB1>(x);    // quad_perm [1,0,3,2]: lane ^ 1
  x = dpp_add<0x4E>(x);    // quad_perm [2,3,0,1]: lane ^ 2
  x = dpp_add<0x141>(x);   // row_half_mirror: the other quad of each 8 lanes
  if constexpr (LANES >= 16) x = dpp_add<0x140>(x);   // row_mirror: the other half of each 16 lanes
  if constexpr (LANES >= 32) {
    // v_permlane16_swap exchanges odd rows of the first operand with even rows of the second;
    // fed the same value twice, the two results hold each row and its neighbour row.
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  }
  if constexpr (LANES >= 64) {
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  }
  return x;
}

// ---- element types ---------------------------------------------------------------
struct F32 {
  static constexpr int kBytes = 4;
};
struct BF16 {
  static constexpr int kBytes = 2;
};

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));   // 16 bytes; a native vector, so it can be loaded non-temporally

// <k, q> over the 16 bytes a lane holds.
template <typename E>
__device__ __forceinline__ float dot16(const u32x4& k, const u32x4& q) {
  if constexpr (E::kBytes == 4) {
    float s = __uint_as_float(k.x) * __uint_as_float(q.x);
    s = fmaf(__uint_as_float(k.y), __uint_as_float(q.y), s);
    s = fmaf(__uint_as_float(k.z), __uint_as_float(q.z), s);
    s = fmaf(__uint_as_float(k.w), __uint_as_float(q.w), s);
    return s;
  } else {
    // v_dot2_f32_bf16: two bf16 products accumulated in fp32 per instruction.  The words are
    // copied to scalars first: a bit cast applied directly to a vector element read the
    // first element every time with this compiler.
    const unsigned kw[4] = {k.x, k.y, k.z, k.w};
    const unsigned qw[4] = {q.x, q.y, q.z, q.w};
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, kw[i]),
                                          __builtin_bit_cast(bf16x2_t, qw[i]), s, false);
    return s;
  }
}

// The 16 bytes of a lane as fp32 values (4 for fp32 storage, 8 for bf16).
template <typename E>
__device__ __forceinline__ void unpack16(const u32x4& v, float* f) {
  if constexpr (E::kBytes == 4) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  } else {
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
  }
}

// Page ids of the pages a wavefront is about to read, 128 at a time in two registers: lane j
// of register (c & 1) holds the id of page 64*c + j (relative to the first page).  A
// v_readlane turns one into a scalar, which makes the page's base address scalar too.  The
// K stream runs one tile ahead of the V stream, so when K enters chunk c the register of
// chunk c+1 (== that of chunk c-1, which V has just left) is reloaded.
struct PageIds {
  const int32_t* row;   // block-table entry of relative page 0
  int n_pages;
  int lane;
  int max_id;
  int reg0, reg1;       // two scalars, not an array: an indexed member would live in scratch memory

  // A table entry that is negative or past the pool (a caller error: pages of the visible
  // range must be resident) is clamped, so the kernel reads wrong data rather than faulting.
  __device__ __forceinline__ int fetch(int first) const {
    const int i = first + lane;
    return i < n_pages ? min(max(row[i], 0), max_id) : 0;
  }
  __device__ __forceinline__ void init(const int32_t* r, int n, int l, int max_page_id) {
    row = r; n_pages = n; lane = l; max_id = max_page_id;
    reg0 = fetch(0);
    reg1 = fetch(kWave);
  }
  // true when the table entry itself is a page of the pool (used before writing into it)
  __device__ __forceinline__ bool writable(int page_rel) const {
    const int raw = row[page_rel];
    return raw >= 0 && raw <= max_id;
  }
  __device__ __forceinline__ int get(int page_rel) const {
    const int r = (page_rel & kWave) ? reg1 : reg0;
    return __builtin_amdgcn_readlane(r, page_rel & (kWave - 1));
  }
  // Call after the K stream has issued the loads of a tile starting at page_rel.
  __device__ __forceinline__ void k_stream_at(int page_rel) {
    if ((page_rel & (kWave - 1)) == 0 && page_rel > 0) {
      const int next = fetch(page_rel + kWave);
      if (page_rel & kWave) reg0 = next;
      else reg1 = next;
    }
  }
};

// Writes one partial record.  acc lives in the V lane geometry: lanes [0, LPT) hold EPL
// consecutive output elements each.
template <int D, int G, int EPL>
__device__ __forceinline__ void store_partial(const DecodeParams& p, int64_t slot, int lane, int lpt,
                                              const float (&m)[G], const float (&l)[G],
                                              const float (&acc)[G][EPL]) {
  if (lane < lpt) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float* dst = p.ws_acc + (slot * G + g) * D + lane * EPL;
#pragma unroll
      for (int j = 0; j < EPL; j += 4)
        *reinterpret_cast<float4*>(dst + j) =
            make_float4(acc[g][j], acc[g][j + 1], acc[g][j + 2], acc[g][j + 3]);
      if (lane == 0) *reinterpret_cast<float2*>(p.ws_ml + (slot * G + g) * 2) = make_float2(m[g], l[g]);
    }
  }
}

// ---- engine for 16-token pages: one token per quad of lanes -----------------------------
//
// The two operands are read in two different lane geometries:
//   K  lane l reads token l/4 of the page: the (l%4)-th 16 bytes of every 64-byte piece of
//      that token's row (a quad of lanes reads 64 contiguous bytes).  A lane therefore sums
//      a quarter of ONE token's dot product in its own registers and the only cross-lane
//      work per score is a sum over 4 lanes.
//   V  lane l reads the 16 bytes at l*16 of every KiB of the page, i.e. it owns EPL output
//      elements and sees token (l / LPT) of each load.
// The softmax weights are produced in the K geometry (one token per quad) and consumed in
// the V geometry, so they cross lanes through a small LDS array (broadcast reads, no bank
// conflicts).  The running maximum is wave-uniform, which makes the final merge of the V
// lane groups a plain sum.
template <typename E_, int D_, int G_>
struct QuadEngine {
  using E = E_;
  static constexpr int D = D_, G = G_;
  static constexpr int T = 16;
  static constexpr int ROW = D * E::kBytes;            // bytes per token row (<= 512 here)
  static constexpr int EPL = 16 / E::kBytes;           // elements per 16 bytes
  static constexpr int KCH = ROW / 64;                 // 64-byte pieces per row == 1 KiB loads per page
  static constexpr int PPT = 8 / KCH;                  // pages per tile (1, 2 or 4)
  static constexpr int NLD = 8;                        // loads per tile, K and V alike
  static constexpr int LPT = ROW / 16;                 // V geometry: lanes per token row
  static constexpr int TPL = kWave / LPT;              // V geometry: tokens per load
  static constexpr int V_OFF = T * ROW;                // K rows come first in a (page, head) block
  static constexpr int kTileLog2 = PPT == 1 ? 4 : PPT == 2 ? 5 : 6;
  static constexpr int kLdsFloats = 2 * PPT * T * G;   // softmax weights of a tile, double buffered
  // Pipeline depth, see run().  Measured: with 4 query heads per KV head the deeper pipeline is
  // worth +6 % although some of its registers spill to accumulation registers; with 2 heads
  // both depths run at the same speed.
  static constexpr int kAhead = 1;
  static_assert(KCH >= 2 && KCH <= 8, "row size");

  __device__ __forceinline__ static void run(const DecodeParams& p, int lane, int b, int kvh, int L, int tile0,
                             int n_tiles, int append_tile, int64_t slot, float* lds) {
    int lo_tok, p_lo, p_hi;
    visible_pages(L, p.window, 4, &lo_tok, &p_lo, &p_hi);
    const int page0 = p_lo + tile0 * PPT;
    const int n_pages = min(n_tiles * PPT, p_hi - page0);
    const int tok0 = page0 * T;
    float (*s_prob)[PPT * T][G] = reinterpret_cast<float (*)[PPT * T][G]>(lds);

    PageIds ids;
    ids.init(p.block_table + int64_t(b) * p.bt_stride + page0, n_pages, lane, p.max_page_id);

    const char* kv_base = p.layer_base + int64_t(kvh) * p.head_stride;   // wave-uniform
    const unsigned k_voff = (lane >> 2) * ROW + (lane & 3) * 16;         // K geometry
    const unsigned v_voff = V_OFF + lane * 16;                           // V geometry
    const int k_tok = lane >> 2;
    const int v_grp = lane / LPT;

    // query rows in the K geometry: for every 64-byte piece, this lane's 16 bytes
    u32x4 qv[G][KCH];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const char* qp = static_cast<const char*>(p.q) +
                       (int64_t(b) * p.n_q_heads + kvh * G + g) * ROW + (lane & 3) * 16;
#pragma unroll
      for (int c = 0; c < KCH; ++c) qv[g][c] = *reinterpret_cast<const u32x4*>(qp + c * 64);
    }

    float m[G], l[G], acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      m[g] = kNegBig;
      l[g] = 0.f;
#pragma unroll
      for (int j = 0; j < EPL; ++j) acc[g][j] = 0.f;
    }

    auto load_pages = [&](int tile, unsigned voff, int step, u32x4* buf) {
#pragma unroll
      for (int pp = 0; pp < PPT; ++pp) {
        const int page_rel = tile * PPT + pp;
        if (PPT == 1 || page_rel < n_pages) {
          const char* pb = kv_base + int64_t(ids.get(page_rel)) * p.small_bytes;
#pragma unroll
          for (int c = 0; c < KCH; ++c)
            buf[pp * KCH + c] =
                __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pb + voff + c * step));
        } else {
#pragma unroll
          for (int c = 0; c < KCH; ++c) buf[pp * KCH + c] = u32x4{0, 0, 0, 0};
        }
      }
    };

    // Software pipeline.  AHEAD = 1 (two tiles deep): while tile t is computed, K(t+1), V(t+1)
    // and (after the scores) K(t+2) are in flight, 16 to 32 KiB per wavefront.  AHEAD = 0: V(t)
    // is issued at the start of tile t and K(t+1) after the scores, 8 to 16 KiB in flight (kept
    // for comparison; not the configuration that is built).
    // Loads return in order, so waiting for the oldest tile leaves the younger ones outstanding.
    constexpr int AHEAD = kAhead;
    u32x4 kb[1 + AHEAD][NLD], vb[1 + AHEAD][NLD];
    load_pages(0, k_voff, 64, kb[0]);
    if (AHEAD) {
      load_pages(0, v_voff, 1024, vb[0]);
      if (n_tiles > 1) {
        load_pages(1, k_voff, 64, kb[AHEAD]);
        ids.k_stream_at(PPT);
      }
    }

    auto step = [&](int tile, u32x4* kbuf, u32x4* vbuf, u32x4* v_next) {
      if (tile + AHEAD < n_tiles) load_pages(tile + AHEAD, v_voff, 1024, v_next);

      // Fused append: the wavefront whose chunk holds the tile of the newest token (position
      // L - 1) takes that token's rows from k_new / v_new instead of the pool and stores them
      // into the page.  The rows are fetched here, once per (request, head), rather than held
      // in registers through the whole loop.
      if (tile == append_tile) {
        const char* kn = static_cast<const char*>(p.k_new) + (int64_t(b) * p.n_kv_heads + kvh) * ROW;
        const char* vn = static_cast<const char*>(p.v_new) + (int64_t(b) * p.n_kv_heads + kvh) * ROW;
        u32x4 k_app[KCH];
#pragma unroll
        for (int c = 0; c < KCH; ++c)
          k_app[c] = *reinterpret_cast<const u32x4*>(kn + c * 64 + (lane & 3) * 16);
        const u32x4 v_app = *reinterpret_cast<const u32x4*>(vn + (lane % LPT) * 16);
        const int pos = L - 1;
        const int page_rel = (pos >> 4) - page0;
        const int pp_new = page_rel - tile * PPT;           // page of the tile that holds the new token
        const int t_new = pp_new * T + (pos & 15);          // its index inside the tile
        char* pb = const_cast<char*>(kv_base) + int64_t(ids.get(page_rel)) * p.small_bytes;
        const bool store = ids.writable(page_rel);
        if (k_tok == (pos & 15)) {
#pragma unroll
          for (int c = 0; c < KCH; ++c) {
            if (store) *reinterpret_cast<u32x4*>(pb + k_voff + c * 64) = k_app[c];
#pragma unroll
            for (int pp = 0; pp < PPT; ++pp)
              if (pp == pp_new) kbuf[pp * KCH + c] = k_app[c];
          }
        }
        bool mine = false;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
          if ((i / KCH) * T + (i % KCH) * TPL + v_grp == t_new) {
            vbuf[i] = v_app;
            mine = true;
          }
        }
        if (mine && store) *reinterpret_cast<u32x4*>(pb + V_OFF + (pos & 15) * ROW + (lane % LPT) * 16) = v_app;
      }

      // one score per (page of the tile, query head) and lane: token k_tok of that page
      float s[PPT][G];
#pragma unroll
      for (int pp = 0; pp < PPT; ++pp)
#pragma unroll
        for (int g = 0; g < G; ++g) {
          float x = 0.f;
#pragma unroll
          for (int c = 0; c < KCH; ++c) x += dot16<E>(kbuf[pp * KCH + c], qv[g][c]);
          x = dpp_add<0xB1>(x);      // lane ^ 1
          x = dpp_add<0x4E>(x);      // lane ^ 2: all four lanes of the quad hold the token's score
          s[pp][g] = x * p.scale_log2;
        }

      if (tile + 1 + AHEAD < n_tiles) {
        load_pages(tile + 1 + AHEAD, k_voff, 64, kbuf);
        ids.k_stream_at((tile + 1 + AHEAD) * PPT);
      }

      const int tile_tok = tok0 + tile * PPT * T;           // first token of the tile
      const bool clean = tile_tok >= lo_tok && tile_tok + PPT * T <= L;
      if (!clean) {
#pragma unroll
        for (int pp = 0; pp < PPT; ++pp) {
          const int t = tile_tok + pp * T + k_tok;
          if (t < lo_tok || t >= L) {
#pragma unroll
            for (int g = 0; g < G; ++g) s[pp][g] = kNegBig;
          }
        }
        // V rows outside the visible set may hold anything (even NaN): make them zero
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
          const int t = tile_tok + (i / KCH) * T + (i % KCH) * TPL + v_grp;
          if (t < lo_tok || t >= L) vbuf[i] = u32x4{0, 0, 0, 0};
        }
      }

      float (*prob)[G] = s_prob[tile & 1];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float mx = s[0][g];
#pragma unroll
        for (int pp = 1; pp < PPT; ++pp) mx = fmaxf(mx, s[pp][g]);
        const float m_new = fmaxf(m[g], wave_max(mx));
        const float alpha = __builtin_amdgcn_exp2f(m[g] - m_new);
        float sum = 0.f;
#pragma unroll
        for (int pp = 0; pp < PPT; ++pp) {
          float e = __builtin_amdgcn_exp2f(s[pp][g] - m_new);
          if (!clean) e = (s[pp][g] == kNegBig) ? 0.f : e;
          sum += e;
          if ((lane & 3) == 0) prob[pp * T + k_tok][g] = e;
        }
        l[g] = fmaf(l[g], alpha, sum);
        m[g] = m_new;
#pragma unroll
        for (int j = 0; j < EPL; ++j) acc[g][j] *= alpha;
      }
      __builtin_amdgcn_wave_barrier();

#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int t_in_tile = (i / KCH) * T + (i % KCH) * TPL + v_grp;
        float w[G];
#pragma unroll
        for (int g = 0; g < G; ++g) w[g] = prob[t_in_tile][g];
        float vf[EPL];
        unpack16<E>(vbuf[i], vf);
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int j = 0; j < EPL; ++j) acc[g][j] = fmaf(w[g], vf[j], acc[g][j]);
      }
      __builtin_amdgcn_wave_barrier();
    };

    if (AHEAD) {
      for (int tile = 0; tile < n_tiles; tile += 2) {
        step(tile, kb[0], vb[0], vb[AHEAD]);
        if (tile + 1 < n_tiles) step(tile + 1, kb[AHEAD], vb[AHEAD], vb[0]);
      }
    } else {
      for (int tile = 0; tile < n_tiles; ++tile) step(tile, kb[0], vb[0], vb[0]);
    }

    // every quad of lanes carried the same l; the V lane groups share m, so they just add up
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float lt = l[g];
#pragma unroll
      for (int off = 4; off < kWave; off <<= 1) lt += __shfl_xor(lt, off);
      l[g] = lt;
#pragma unroll
      for (int off = LPT; off < kWave; off <<= 1)
#pragma unroll
        for (int j = 0; j < EPL; ++j) acc[g][j] += __shfl_xor(acc[g][j], off);
    }
    store_partial<D, G, EPL>(p, slot, lane, LPT, m, l, acc);
  }
};

// ---- engine for any page size: rows spread over lanes -----------------------------------
//
// K and V are read alike: a token's row is LPT lanes x 16 bytes, one wave-wide load covers
// TPL = 64 / LPT consecutive tokens (1 KiB, contiguous in the page).  Every partial dot
// product is summed over LPT lanes, so this engine spends several times more vector-ALU
// work per byte than the one above; it covers what the other two are not built for (8-token
// pages; fp32 K/V in pages other than 16 tokens, with 8 query heads per KV head, or 1 KiB rows).  Each group of LPT lanes runs
// its own online softmax over the tokens it sees; the groups are merged once at the end.
template <typename E_, int D_, int G_>
struct RowEngine {
  using E = E_;
  static constexpr int D = D_, G = G_;
  static constexpr int ROW = D * E::kBytes;
  static constexpr int EPL = 16 / E::kBytes;
  static constexpr int LPT = ROW / 16;
  static constexpr int TPL = kWave / LPT;
  static constexpr int NL = 8;                 // loads per tile
  static constexpr int TT = NL * TPL;          // tokens per tile: 8, 16, 32 or 64
  static constexpr int kTileLog2 = TT == 8 ? 3 : TT == 16 ? 4 : TT == 32 ? 5 : 6;
  static constexpr int kLdsFloats = 0;

  __device__ __forceinline__ static void run(const DecodeParams& p, int lane, int b, int kvh, int L, int tile0,
                             int n_tiles, int append_tile, int64_t slot, float*) {
    int lo_tok, p_lo, p_hi;
    visible_pages(L, p.window, p.t_log2, &lo_tok, &p_lo, &p_hi);
    const int t_mask = (1 << p.t_log2) - 1;
    // tiles are counted from the first visible page; a tile may be a fraction of a page
    const int first_tok = tile0 * TT;                       // relative to page p_lo
    const int page0 = p_lo + (first_tok >> p.t_log2);
    const int tok_off0 = first_tok & t_mask;                // offset of the chunk inside page0
    const int n_pages = min((tok_off0 + n_tiles * TT + t_mask) >> p.t_log2, p_hi - page0);
    const int abs0 = (page0 << p.t_log2) + tok_off0;        // absolute index of the chunk's first token

    PageIds ids;
    ids.init(p.block_table + int64_t(b) * p.bt_stride + page0, n_pages, lane, p.max_page_id);

    const int sub = lane % LPT;
    const int grp = lane / LPT;
    const char* head_base = p.layer_base + int64_t(kvh) * p.head_stride + lane * 16;

    u32x4 qv[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const char* qp = static_cast<const char*>(p.q) +
                       (int64_t(b) * p.n_q_heads + kvh * G + g) * ROW + sub * 16;
      qv[g] = *reinterpret_cast<const u32x4*>(qp);
    }

    float m[G], l[G], acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      m[g] = kNegBig;
      l[g] = 0.f;
#pragma unroll
      for (int j = 0; j < EPL; ++j) acc[g][j] = 0.f;
    }

    auto load_tile = [&](int tile, int v_off, u32x4* buf) {
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        const int tokr = tok_off0 + tile * TT + i * TPL;     // relative to page0, wave-uniform
        const int page_rel = tokr >> p.t_log2;
        if (page_rel < n_pages) {
          const char* src = head_base + int64_t(ids.get(page_rel)) * p.small_bytes + v_off +
                            (tokr & t_mask) * ROW;
          buf[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src));
        } else {
          buf[i] = u32x4{0, 0, 0, 0};
        }
      }
    };

    u32x4 kbuf[NL], vbuf[NL];
    load_tile(0, 0, kbuf);

    for (int tile = 0; tile < n_tiles; ++tile) {
      load_tile(tile, p.v_offset, vbuf);

      // fused append (see the quad engine): rows of the token at L - 1 come from k_new / v_new
      if (tile == append_tile) {
        const int64_t off = (int64_t(b) * p.n_kv_heads + kvh) * ROW + sub * 16;
        const u32x4 k_app = *reinterpret_cast<const u32x4*>(static_cast<const char*>(p.k_new) + off);
        const u32x4 v_app = *reinterpret_cast<const u32x4*>(static_cast<const char*>(p.v_new) + off);
        const int pos = L - 1;
        const int page_rel = (pos >> p.t_log2) - page0;
        bool mine = false;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
          if (abs0 + tile * TT + i * TPL + grp == pos) {
            kbuf[i] = k_app;
            vbuf[i] = v_app;
            mine = true;
          }
        }
        char* dst = const_cast<char*>(head_base) + int64_t(ids.get(page_rel)) * p.small_bytes +
                    (pos & t_mask) * ROW - grp * ROW;     // head_base carries lane * 16 = grp * ROW + sub * 16
        if (mine && ids.writable(page_rel)) {
          *reinterpret_cast<u32x4*>(dst) = k_app;
          *reinterpret_cast<u32x4*>(dst + p.v_offset) = v_app;
        }
      }

      float s[NL][G];
#pragma unroll
      for (int i = 0; i < NL; ++i)
#pragma unroll
        for (int g = 0; g < G; ++g)
          s[i][g] = group_sum<LPT>(dot16<E>(kbuf[i], qv[g])) * p.scale_log2;

      if (tile + 1 < n_tiles) {
        load_tile(tile + 1, 0, kbuf);
        const int tokr = tok_off0 + (tile + 1) * TT;
        if ((tokr & t_mask) == 0) ids.k_stream_at(tokr >> p.t_log2);
      }

      const int t_abs0 = abs0 + tile * TT + grp;
      const bool clean = (abs0 + tile * TT >= lo_tok) && (abs0 + (tile + 1) * TT <= L);
      bool valid[NL];
#pragma unroll
      for (int i = 0; i < NL; ++i) valid[i] = true;
      if (!clean) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
          const int t = t_abs0 + i * TPL;
          valid[i] = (t >= lo_tok) && (t < L);
          if (!valid[i]) {
            vbuf[i] = u32x4{0, 0, 0, 0};             // masked rows may hold anything, even NaN
#pragma unroll
            for (int g = 0; g < G; ++g) s[i][g] = kNegBig;
          }
        }
      }

      float pr[NL][G];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float mx = s[0][g];
#pragma unroll
        for (int i = 1; i < NL; ++i) mx = fmaxf(mx, s[i][g]);
        const float m_new = fmaxf(m[g], mx);
        const float alpha = __builtin_amdgcn_exp2f(m[g] - m_new);
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
          float e = __builtin_amdgcn_exp2f(s[i][g] - m_new);
          if (!clean) e = valid[i] ? e : 0.f;
          pr[i][g] = e;
          sum += e;
        }
        l[g] = fmaf(l[g], alpha, sum);
        m[g] = m_new;
#pragma unroll
        for (int j = 0; j < EPL; ++j) acc[g][j] *= alpha;
      }

#pragma unroll
      for (int i = 0; i < NL; ++i) {
        float vf[EPL];
        unpack16<E>(vbuf[i], vf);
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int j = 0; j < EPL; ++j) acc[g][j] = fmaf(pr[i][g], vf[j], acc[g][j]);
      }
    }

    // merge the TPL token groups (lanes that hold the same elements of different tokens)
#pragma unroll
    for (int off = LPT; off < kWave; off <<= 1) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float m_o = __shfl_xor(m[g], off);
        const float l_o = __shfl_xor(l[g], off);
        const float m_new = fmaxf(m[g], m_o);
        const float a = __builtin_amdgcn_exp2f(m[g] - m_new);
        const float c = __builtin_amdgcn_exp2f(m_o - m_new);
        l[g] = l[g] * a + l_o * c;
        m[g] = m_new;
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
          const float acc_o = __shfl_xor(acc[g][j], off);
          acc[g][j] = acc[g][j] * a + acc_o * c;
        }
      }
    }
    store_partial<D, G, EPL>(p, slot, lane, LPT, m, l, acc);
  }
};

// ---- engine for bf16 K/V in pages of 16 tokens or more: both contractions on the matrix cores
//
// The work per 16-token block is a small dense contraction, scores = K[16 x D] . Q^T[D x G] and
// out += P[G x 16] . V[16 x D], and the matrix cores take it off the vector ALUs altogether:
// with 8 heads on every K/V byte those can no longer keep up with HBM (the quad engine would
// need about 70 vector instructions per KiB), and with fewer heads the loads still issue
// earlier and more evenly when so little else competes for the issue slots.  The G heads are
// padded to the 16 rows / columns of the instructions.  Operand layouts (lane l, n = l % 16,
// j = l / 16), checked on the device: A holds row n and B holds column n, each with
// consecutive k (8j .. 8j+7 for 16x16x32, 4j .. 4j+3 for 16x16x16); the result holds column n,
// rows 4j .. 4j+3.
//   scores  v_mfma_f32_16x16x32_bf16, A = K page (row = token, k = d): lane (n, j) reads the
//           16 bytes at d = 8j of each 64-byte piece of token n's row -- a plain 16-byte load,
//           64-byte runs per token as in the quad engine.  B = Q (column = head, zero for the
//           padding heads).  Result: lane (n, j) holds head n, tokens 4j .. 4j+3 of the page.
//   values  v_mfma_f32_16x16x16_bf16, A = P (row = head, k = token of the page): exactly the
//           four probabilities lane (n, j) holds after the softmax.  B = V (k = token,
//           column = d) wants four tokens of one column per lane, but V arrives row-major:
//           the rows go through LDS and come back through ds_read_b64_tr_b16, which hands
//           lane (n, j) column n of the 4 rows whose addresses lanes 4r .. 4r+3 of its 16-lane
//           group supplied.  Result: lane (n, j) holds output element 16 * block + n of heads
//           4j .. 4j+3.
// The instruction takes bf16 operands; a probability goes in as the sum of two bf16 numbers
// (its rounding and the rounding of the remainder, 16 significant bits together) in two
// products, so the result stays within fp32 rounding of an fp32 weighted sum -- the matrix
// cores are idle most of the time anyway.
template <int D_, int G_>
struct MatEngine {
  using E = BF16;
  static constexpr int D = D_, G = G_;
  static constexpr int T = 16;                 // tokens per block; a page holds 1, 2, 4 or 8 blocks
  static constexpr int ROW = D * 2;            // bytes per token row
  static constexpr int KCH = ROW / 64;         // k-steps of the score product == 1 KiB loads per page
  static constexpr int PPT = 8 / KCH;          // blocks per tile (1, 2 or 4)
  static constexpr int NLD = 8;                // 16-byte loads per lane and tile, K and V alike
  static constexpr int LPT = ROW / 16;         // V loads: lanes per token row
  static constexpr int TPL = kWave / LPT;      // V loads: token rows per load
  static constexpr int NBLK = D / 16;          // 16-wide blocks of the output row
  static constexpr int LROW = ROW + 32;        // LDS row pitch: 8 banks further per row
  static constexpr int kTileLog2 = PPT == 1 ? 4 : PPT == 2 ? 5 : 6;
  static constexpr int kLdsFloats = PPT * T * LROW / 4;
  static_assert(KCH == 2 || KCH == 4 || KCH == 8, "row size");
  static_assert(G <= 16, "heads are padded to 16");

  typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
  typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  typedef float f32x4 __attribute__((ext_vector_type(4)));

  // max / sum over the four lanes n, n + 16, n + 32, n + 48
  __device__ __forceinline__ static float across_groups_max(float x) {
    unsigned u = __float_as_uint(x);
    auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    u = __float_as_uint(x);
    r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  }
  __device__ __forceinline__ static float across_groups_sum(float x) {
    unsigned u = __float_as_uint(x);
    auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    u = __float_as_uint(x);
    r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
  }

  __device__ __forceinline__ static void run(const DecodeParams& p, int lane, int b, int kvh, int L, int tile0,
                             int n_tiles, int append_tile, int64_t slot, float* lds) {
    // Pages of 16, 32, 64 or 128 tokens are read as runs of 16-token blocks: block q (counted
    // from the first visible page) lies in page q >> sh at row offset (q & sub_mask) * 16.
    const int sh = p.t_log2 - 4;
    const int sub_mask = (1 << sh) - 1;
    int lo_tok, p_lo, p_hi;
    visible_pages(L, p.window, p.t_log2, &lo_tok, &p_lo, &p_hi);
    const int blk0 = tile0 * PPT;                              // first block of the chunk
    const int page0 = p_lo + (blk0 >> sh);
    const int off0 = blk0 & sub_mask;                          // its place inside page0
    const int n_blk = min(n_tiles * PPT, ((p_hi - p_lo) << sh) - blk0);
    const int n_pages = (off0 + n_blk + sub_mask) >> sh;
    const int tok0 = ((p_lo << sh) + blk0) * T;
    char* v_lds = reinterpret_cast<char*>(lds);

    PageIds ids;
    ids.init(p.block_table + int64_t(b) * p.bt_stride + page0, n_pages, lane, p.max_page_id);

    const int n = lane & 15, j = lane >> 4;
    const int v_row = lane / LPT;                                        // V loads: row v_row + TPL * c of the page
    const char* kv_base = p.layer_base + int64_t(kvh) * p.head_stride;   // wave-uniform
    const unsigned k_voff = n * ROW + j * 16;                            // A operand of the score product
    const unsigned v_voff = p.v_offset + lane * 16;
    const unsigned lds_wr = v_row * LROW + (lane % LPT) * 16;            // this lane's V bytes (+ row offset)
    const unsigned lds_rd = (4 * j + (n >> 2)) * LROW + (n & 3) * 8;     // transposed read (+ page, + block)

    // B operand of the score product: head n (zero rows for the padding heads)
    bf16x8 qb[KCH];
#pragma unroll
    for (int c = 0; c < KCH; ++c) {
      u32x4 w = u32x4{0, 0, 0, 0};
      if (n < G)
        w = *reinterpret_cast<const u32x4*>(static_cast<const char*>(p.q) +
                                           (int64_t(b) * p.n_q_heads + kvh * G + n) * ROW + j * 16 + c * 64);
      qb[c] = __builtin_bit_cast(bf16x8, w);
    }

    float m = kNegBig, l = 0.f;        // of head n; l is this lane's share (its tokens only)
    f32x4 acc[NBLK];
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) acc[blk] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto load_pages = [&](int tile, unsigned voff, int step, u32x4* buf) {
#pragma unroll
      for (int pp = 0; pp < PPT; ++pp) {
        const int r = tile * PPT + pp;
        if (PPT == 1 || r < n_blk) {
          const int q = off0 + r;
          const char* pb = kv_base + int64_t(ids.get(q >> sh)) * p.small_bytes + (q & sub_mask) * (T * ROW);
#pragma unroll
          for (int c = 0; c < KCH; ++c)
            buf[pp * KCH + c] =
                __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pb + voff + c * step));
        } else {
#pragma unroll
          for (int c = 0; c < KCH; ++c) buf[pp * KCH + c] = u32x4{0, 0, 0, 0};
        }
      }
    };

    // two tiles deep, as in the quad engine
    u32x4 kb[2][NLD], vb[2][NLD];
    load_pages(0, k_voff, 64, kb[0]);
    load_pages(0, v_voff, 1024, vb[0]);
    // the K stream tells the page-id registers when it enters a new page
    auto k_entered = [&](int tile) {
      const int q = off0 + tile * PPT;
      if ((q & sub_mask) == 0) ids.k_stream_at(q >> sh);
    };
    if (n_tiles > 1) {
      load_pages(1, k_voff, 64, kb[1]);
      k_entered(1);
    }

    auto step = [&](int tile, u32x4* kbuf, u32x4* vbuf, u32x4* v_next) {
      if (tile + 1 < n_tiles) load_pages(tile + 1, v_voff, 1024, v_next);

      // fused append: rows of the token at L - 1 come from k_new / v_new and are stored into the page
      if (tile == append_tile) {
        const char* kn = static_cast<const char*>(p.k_new) + (int64_t(b) * p.n_kv_heads + kvh) * ROW;
        const char* vn = static_cast<const char*>(p.v_new) + (int64_t(b) * p.n_kv_heads + kvh) * ROW;
        const int pos = L - 1;
        const int r_new = (pos >> 4) - ((p_lo << sh) + blk0);     // block of the new token, relative to the chunk
        const int pp_new = r_new - tile * PPT;
        const int page_rel = (off0 + r_new) >> sh;
        char* pb = const_cast<char*>(kv_base) + int64_t(ids.get(page_rel)) * p.small_bytes +
                   ((off0 + r_new) & sub_mask) * (T * ROW);
        const bool store = ids.writable(page_rel);
        if (n == (pos & 15)) {
#pragma unroll
          for (int c = 0; c < KCH; ++c) {
            const u32x4 k_app = *reinterpret_cast<const u32x4*>(kn + j * 16 + c * 64);
            if (store) *reinterpret_cast<u32x4*>(pb + k_voff + c * 64) = k_app;
#pragma unroll
            for (int pp = 0; pp < PPT; ++pp)
              if (pp == pp_new) kbuf[pp * KCH + c] = k_app;
          }
        }
        const u32x4 v_app = *reinterpret_cast<const u32x4*>(vn + (lane % LPT) * 16);
        bool mine = false;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
          if ((i / KCH) * T + (i % KCH) * TPL + v_row == pp_new * T + (pos & 15)) {
            vbuf[i] = v_app;
            mine = true;
          }
        }
        if (mine && store) *reinterpret_cast<u32x4*>(pb + p.v_offset + (pos & 15) * ROW + (lane % LPT) * 16) = v_app;
      }

      // scores: lane (n, j) gets head n, tokens 4j .. 4j+3 of each page
      f32x4 s[PPT];
#pragma unroll
      for (int pp = 0; pp < PPT; ++pp) {
        s[pp] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < KCH; ++c)
          s[pp] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kbuf[pp * KCH + c]), qb[c],
                                                          s[pp], 0, 0, 0);
      }

      if (tile + 2 < n_tiles) {
        load_pages(tile + 2, k_voff, 64, kbuf);
        k_entered(tile + 2);
      }

      const int tile_tok = tok0 + tile * PPT * T;
      const bool clean = tile_tok >= lo_tok && tile_tok + PPT * T <= L;
#pragma unroll
      for (int pp = 0; pp < PPT; ++pp)
#pragma unroll
        for (int i = 0; i < 4; ++i) s[pp][i] *= p.scale_log2;
      if (!clean) {
#pragma unroll
        for (int pp = 0; pp < PPT; ++pp)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int t = tile_tok + pp * T + 4 * j + i;
            if (t < lo_tok || t >= L) s[pp][i] = kNegBig;
          }
        // V rows outside the visible set may hold anything (even NaN): make them zero
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
          const int t = tile_tok + (i / KCH) * T + (i % KCH) * TPL + v_row;
          if (t < lo_tok || t >= L) vbuf[i] = u32x4{0, 0, 0, 0};
        }
      }

      // V rows into LDS, row-major
#pragma unroll
      for (int i = 0; i < NLD; ++i)
        *reinterpret_cast<u32x4*>(v_lds + ((i / KCH) * T + (i % KCH) * TPL) * LROW + lds_wr) = vbuf[i];

      // online softmax of head n
      float mx = s[0][0];
#pragma unroll
      for (int pp = 0; pp < PPT; ++pp)
#pragma unroll
        for (int i = 0; i < 4; ++i) mx = fmaxf(mx, s[pp][i]);
      const float m_new = fmaxf(m, across_groups_max(mx));
      const float alpha = __builtin_amdgcn_exp2f(m - m_new);
      bf16x4 prob_hi[PPT], prob_lo[PPT];
      float sum = 0.f;
#pragma unroll
      for (int pp = 0; pp < PPT; ++pp)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float e = __builtin_amdgcn_exp2f(s[pp][i] - m_new);
          if (!clean) e = (s[pp][i] == kNegBig) ? 0.f : e;
          const __bf16 hi = static_cast<__bf16>(e);
          prob_hi[pp][i] = hi;
          prob_lo[pp][i] = static_cast<__bf16>(e - static_cast<float>(hi));
          sum += e;
        }
      l = fmaf(l, alpha, sum);
      m = m_new;

      // The accumulator rows of this lane belong to heads 4j .. 4j+3: fetch their factors.  Once
      // the running maxima have settled every factor is exactly 1 and the step is skipped.
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
        float a[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
          a[i] = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (4 * j + i), __float_as_int(alpha)));
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk)
#pragma unroll
          for (int i = 0; i < 4; ++i) acc[blk][i] *= a[i];
      }

      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
#pragma unroll
      for (int pp = 0; pp < PPT; ++pp)
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk) {
          const s16x4 v4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (lds_s16x4_ptr)(v_lds + pp * T * LROW + lds_rd + blk * 32));
          const bf16x4 vt = __builtin_bit_cast(bf16x4, v4);
          acc[blk] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(prob_hi[pp], vt, acc[blk], 0, 0, 0);
          acc[blk] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(prob_lo[pp], vt, acc[blk], 0, 0, 0);
        }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    };

    for (int tile = 0; tile < n_tiles; tile += 2) {
      step(tile, kb[0], vb[0], vb[1]);
      if (tile + 1 < n_tiles) step(tile + 1, kb[1], vb[1], vb[0]);
    }

    l = across_groups_sum(l);
    // one partial record: lane (n, j) holds element 16 * blk + n of heads 4j .. 4j+3
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int h = 4 * j + i;
      if (h < G) {
        float* dst = p.ws_acc + (slot * G + h) * D + n;
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk) dst[blk * 16] = acc[blk][i];
      }
    }
    if (j == 0 && n < G) *reinterpret_cast<float2*>(p.ws_ml + (slot * G + n) * 2) = make_float2(m, l);
  }
};

// One wavefront per partition of the flat tile space (see the head of the file).
template <class Eng>
__global__ __launch_bounds__(kWave) void decode_partial_kernel(const DecodeParams p) {
  __shared__ int s_incl[kMaxBatch];
  __shared__ int s_len[kMaxBatch];
  __shared__ float s_eng[Eng::kLdsFloats > 0 ? Eng::kLdsFloats : 1];
  const int lane = threadIdx.x;
  const int W = scan_requests(p.seq_lens, p.batch, p.max_seq_len, p.window, p.t_log2, Eng::kTileLog2,
                              p.n_kv_heads, lane, s_incl, s_len);
  const int C = chunk_of(p.chunk_tiles, p.min_chunk_tiles, W, gridDim.x);
  const int64_t x0 = int64_t(blockIdx.x) * C;
  if (x0 >= W) return;
  int x = int(x0);
  const int x1 = int(min<int64_t>(W, x0 + C));
  while (x < x1) {
    const int b = find_request(s_incl, p.batch, x, lane);
    const int start_b = b > 0 ? s_incl[b - 1] : 0;
    const int units_b = (s_incl[b] - start_b) / p.n_kv_heads;     // start-up units + tiles, per head
    const int rem = x - start_b;
    const int kvh = rem / units_b;
    const int seg0 = start_b + kvh * units_b;                     // flat position of the segment
    const int xe = min(x1, seg0 + units_b);
    // tiles of the segment inside [x, xe): none if the chunk ends inside the start-up units
    const int tile0 = max(x - seg0 - kSegStartUnits, 0);
    const int n_tiles = xe - seg0 - kSegStartUnits - tile0;
    if (n_tiles > 0) {
      const int64_t slot = int64_t(b) * p.n_kv_heads + kvh + blockIdx.x;
      // fused append: the chunk that holds the tile of the newest token (position L - 1) writes it
      int append_tile = -1;
      if (p.k_new != nullptr) {
        const int L = s_len[b];
        int lo_tok, p_lo, p_hi;
        visible_pages(L, p.window, p.t_log2, &lo_tok, &p_lo, &p_hi);
        const int t_pos = ((L - 1) - (p_lo << p.t_log2)) >> Eng::kTileLog2;
        if (t_pos >= tile0 && t_pos < tile0 + n_tiles) append_tile = t_pos - tile0;
      }
      Eng::run(p, lane, b, kvh, s_len[b], tile0, n_tiles, append_tile, slot, s_eng);
    }
    x = xe;
  }
}

// One block (one wavefront) per (request, query head): merges the records of its segment,
//   m* = max m_i,  out = sum_i acc_i 2^(m_i - m*) / sum_i l_i 2^(m_i - m*).
// Thread i < D/4 owns output elements [4i, 4i+4); all 64 lanes take part in the scan.
template <int D>
__global__ __launch_bounds__(kWave) void splitk_reduce_kernel(
    const float* __restrict__ ws_acc, const float* __restrict__ ws_ml,
    const int32_t* __restrict__ seq_lens, int32_t batch, int32_t max_seq_len, int32_t window,
    int32_t t_log2, int32_t tile_log2, int32_t chunk_tiles, int32_t min_chunk_tiles, int32_t n_part,
    int32_t n_kv_heads, int32_t n_q_heads, float* __restrict__ out) {
  const int hq = blockIdx.x;
  const int b = blockIdx.y;
  const int lane = threadIdx.x;
  const int G = n_q_heads / n_kv_heads;
  // prefix of units * heads up to request b, and W
  int run = 0, start_b = 0, units_b = 0;
  for (int c0 = 0; c0 < batch; c0 += kWave) {
    const int i = c0 + lane;
    const int Li = i < batch ? min(seq_lens[i], max_seq_len) : 0;
    const int n = units_of(Li, window, t_log2, tile_log2);
    int incl = n * n_kv_heads;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const int up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    if (b >= c0 && b < c0 + kWave) {
      units_b = __builtin_amdgcn_readlane(n, b - c0);
      start_b = run + __builtin_amdgcn_readlane(incl, b - c0) - units_b * n_kv_heads;
    }
    run += __builtin_amdgcn_readlane(incl, kWave - 1);
  }
  const bool owner = lane < D / 4;
  float4* dst = reinterpret_cast<float4*>(out + (int64_t(b) * n_q_heads + hq) * D) + lane;
  if (units_b == 0) {
    if (owner) *dst = make_float4(0.f, 0.f, 0.f, 0.f);
    return;
  }
  const int C = chunk_of(chunk_tiles, min_chunk_tiles, run, n_part);
  const int kvh = hq / G;
  const int g = hq - kvh * G;
  const int S = start_b + kvh * units_b + kSegStartUnits;   // flat position of the segment's first tile
  const int c_lo = S / C;
  const int c_hi = (S + (units_b - kSegStartUnits) - 1) / C;
  const int64_t seg = int64_t(b) * n_kv_heads + kvh;
  // Four records at a time, all their loads issued before any is used (a segment rarely has
  // more than four); the running maximum is carried from one group to the next.
  float m_star = kNegBig, l_star = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int c0 = c_lo; c0 <= c_hi; c0 += 4) {
    float2 ml[4];
    float4 a[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t rec = (seg + min(c0 + i, c_hi)) * G + g;
      ml[i] = *reinterpret_cast<const float2*>(ws_ml + rec * 2);
      a[i] = owner ? *(reinterpret_cast<const float4*>(ws_acc + rec * D) + lane) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float m_new = m_star;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (c0 + i <= c_hi) m_new = fmaxf(m_new, ml[i].x);
    const float keep = __builtin_amdgcn_exp2f(m_star - m_new);
    l_star *= keep;
    acc.x *= keep; acc.y *= keep; acc.z *= keep; acc.w *= keep;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (c0 + i > c_hi) continue;
      const float w = __builtin_amdgcn_exp2f(ml[i].x - m_new);
      l_star = fmaf(ml[i].y, w, l_star);
      acc.x = fmaf(a[i].x, w, acc.x); acc.y = fmaf(a[i].y, w, acc.y);
      acc.z = fmaf(a[i].z, w, acc.z); acc.w = fmaf(a[i].w, w, acc.w);
    }
    m_star = m_new;
  }
  const float inv = l_star > 0.f ? 1.0f / l_star : 0.f;
  if (owner) *dst = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
}

// One thread per 16 bytes of the new K and V rows.
__global__ __launch_bounds__(256) void kv_append_kernel(
    char* __restrict__ layer_base, int64_t small_bytes, int32_t head_stride, int32_t v_offset,
    int32_t t_log2, int32_t n_kv_heads, int32_t row_bytes, const char* __restrict__ k_new,
    const char* __restrict__ v_new, const int32_t* __restrict__ block_table, int32_t bt_stride,
    const int32_t* __restrict__ seq_lens, int32_t batch, int32_t max_page_id) {
  const int chunks = row_bytes / 16;                       // 16-byte chunks per row
  const int64_t per_req = int64_t(n_kv_heads) * 2 * chunks;
  const int64_t idx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= per_req * batch) return;
  const int b = int(idx / per_req);
  int r = int(idx % per_req);
  const int h = r / (2 * chunks);
  r -= h * 2 * chunks;
  const int is_v = r / chunks;
  const int c = r - is_v * chunks;
  const int L = seq_lens[b];
  if (L <= 0) return;
  const int pos = L - 1;
  const int page = pos >> t_log2;
  if (page >= bt_stride) return;
  const int sid = block_table[int64_t(b) * bt_stride + page];
  if (sid < 0 || sid > max_page_id) return;
  const char* src = (is_v ? v_new : k_new) + (int64_t(b) * n_kv_heads + h) * row_bytes + c * 16;
  char* dst = layer_base + int64_t(sid) * small_bytes + int64_t(h) * head_stride +
              (is_v ? v_offset : 0) + (pos & ((1 << t_log2) - 1)) * row_bytes + c * 16;
  *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
}

// Bulk write of a run of tokens per request (chunked prefill).  One block per source token
// row: the request and page lookups are wave-uniform (scalar loads), the threads then copy the
// row's 2 * n_kv_heads * D * e bytes 16 at a time.  Source rows are token-major,
// [token][kv head][D]; request b owns rows [cu_tokens[b], cu_tokens[b+1]) and its first row is
// sequence position start_pos[b].
__global__ __launch_bounds__(256) void kv_write_range_kernel(
    char* __restrict__ layer_base, int64_t small_bytes, int32_t head_stride, int32_t v_offset,
    int32_t t_log2, int32_t n_kv_heads, int32_t row_bytes, const char* __restrict__ k_src,
    const char* __restrict__ v_src, const int32_t* __restrict__ cu_tokens,
    const int32_t* __restrict__ start_pos, const int32_t* __restrict__ block_table,
    int32_t bt_stride, int32_t batch, int32_t max_page_id) {
  const int tok = blockIdx.x;
  // request of this token: last b with cu_tokens[b] <= tok
  int lo = 0, hi = batch;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu_tokens[mid] <= tok) lo = mid; else hi = mid;
  }
  const int b = lo;
  if (tok >= cu_tokens[b + 1]) return;            // padding rows past the last request
  const int pos = start_pos[b] + (tok - cu_tokens[b]);
  const int page = pos >> t_log2;
  if (pos < 0 || page >= bt_stride) return;
  const int sid = block_table[int64_t(b) * bt_stride + page];
  if (sid < 0 || sid > max_page_id) return;       // page not resident (e.g. already slid out)
  const int chunks = row_bytes / 16;              // 16-byte pieces per (head, K or V) row
  char* page_base = layer_base + int64_t(sid) * small_bytes + (pos & ((1 << t_log2) - 1)) * row_bytes;
  const char* k_row = k_src + int64_t(tok) * n_kv_heads * row_bytes;
  const char* v_row = v_src + int64_t(tok) * n_kv_heads * row_bytes;
  for (int i = threadIdx.x; i < 2 * n_kv_heads * chunks; i += blockDim.x) {
    const int is_v = i >= n_kv_heads * chunks;
    const int j = is_v ? i - n_kv_heads * chunks : i;     // 16-byte piece inside the token's K (or V) rows
    const int h = j / chunks;
    const int c = j - h * chunks;
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>((is_v ? v_row : k_row) + j * 16));
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(page_base + int64_t(h) * head_stride +
                                                           (is_v ? v_offset : 0) + c * 16));
  }
}

__global__ __launch_bounds__(256) void stream_copy_kernel(u32x4* __restrict__ dst,
                                                          const u32x4* __restrict__ src, int64_t n) {
  const int64_t stride = int64_t(gridDim.x) * blockDim.x;
  for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride)
    __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, int64_t n,
                                                          unsigned* __restrict__ sink) {
  const int64_t stride = int64_t(gridDim.x) * blockDim.x;
  unsigned x = 0;
  for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride) {
    const u32x4 v = __builtin_nontemporal_load(src + i);
    x ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (x == 0x9e3779b9u) *sink = x;     // practically never taken; keeps the loads alive
}

// ---- host side: validation, partition geometry, launch --------------------------------

using DecodeFn = void (*)(DecodeParams);

bool attention_kind(const jenga::Kind& k) {
  return k.desc.type == JENGA_FULL || k.desc.type == JENGA_WINDOW || k.desc.type == JENGA_CROSS;
}

bool aligned16(const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }

// Only the combinations decode_geometry() can ask for are instantiated.
template <typename E, int D>
DecodeFn pick_g(bool mat, bool quad, int G) {
  constexpr int kRow = D * E::kBytes;
  if constexpr (E::kBytes == 2) {
    if (mat) {
      switch (G) {
        case 1: return decode_partial_kernel<MatEngine<D, 1>>;
        case 2: return decode_partial_kernel<MatEngine<D, 2>>;
        case 4: return decode_partial_kernel<MatEngine<D, 4>>;
        default: break;
      }
      if (G == 16) return decode_partial_kernel<MatEngine<D, 16>>;
      return decode_partial_kernel<MatEngine<D, 8>>;
    }
  }
  if constexpr (kRow <= 512 && (E::kBytes == 4 || kRow == 512)) {
    if (quad) {
      switch (G) {
        case 1: return decode_partial_kernel<QuadEngine<E, D, 1>>;
        case 2: return decode_partial_kernel<QuadEngine<E, D, 2>>;
        default: return decode_partial_kernel<QuadEngine<E, D, 4>>;
      }
    }
  }
  switch (G) {
    case 1: return decode_partial_kernel<RowEngine<E, D, 1>>;
    case 2: return decode_partial_kernel<RowEngine<E, D, 2>>;
    case 4: return decode_partial_kernel<RowEngine<E, D, 4>>;
    default: return decode_partial_kernel<RowEngine<E, D, 8>>;
  }
}

template <typename E>
DecodeFn pick_d(int D, bool mat, bool quad, int G) {
  switch (D) {
    case 64: return pick_g<E, 64>(mat, quad, G);
    case 128: return pick_g<E, 128>(mat, quad, G);
    default: return pick_g<E, 256>(mat, quad, G);
  }
}

// Partitions of the automatic mode: resident blocks of `fn`, at most one per SIMD, a multiple
// of 8 (one share per XCD), capped at kMaxPartitions.  Cached per kernel; 2048 when no device can be asked.
int resident_partitions(DecodeFn fn) {
  static std::mutex mu;
  static std::unordered_map<const void*, int> cache;
  std::lock_guard<std::mutex> lock(mu);
  auto it = cache.find(reinterpret_cast<const void*>(fn));
  if (it != cache.end()) return it->second;
  int n = 2048;
  int dev = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) == hipSuccess &&
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kWave, 0) == hipSuccess &&
      cus > 0 && per_cu > 0) {
    // one wavefront per SIMD (4 per compute unit): measured faster than filling every slot,
    // and it leaves each wavefront the registers for a deep load pipeline
    n = std::min(kMaxPartitions, cus * std::min(per_cu, 4)) / 8 * 8;
    n = std::max(n, 8);
    cache.emplace(reinterpret_cast<const void*>(fn), n);
  } else {
    (void)hipGetLastError();      // no device: do not leave a sticky error, do not cache
  }
  return n;
}

struct Geometry {
  const jenga::Kind* kind;
  int G;
  bool quad;             // 16-token pages, vector-ALU engine
  bool mat;              // bf16, pages of 16 tokens or more, matrix-core engine
  int tile_log2;
  int chunk_tiles;       // 0: automatic
  int min_chunk_tiles;
  int n_part_bound;      // partitions the workspace must have room for
  int64_t slots;
  DecodeFn fn;
};

// Everything the partial kernel and the reduction must agree on.
int decode_geometry(const jenga_pool* pool, int32_t kind, int32_t n_q_heads, int32_t batch,
                    int32_t max_seq_len, int32_t window, int32_t pages_per_split, Geometry* out) {
  if (!pool || kind < 0 || kind >= int32_t(pool->kinds.size())) return JENGA_ERR_INVALID;
  const jenga::Kind& k = pool->kinds[kind];
  if (!attention_kind(k)) return JENGA_ERR_INVALID;
  if (batch < 0 || max_seq_len < 0 || window < 0 || n_q_heads < 1 || pages_per_split < 0)
    return JENGA_ERR_INVALID;
  if (batch > kMaxBatch) return JENGA_ERR_UNSUPPORTED;
  if (n_q_heads % k.desc.n_kv_heads != 0) return JENGA_ERR_INVALID;
  const int G = n_q_heads / k.desc.n_kv_heads;
  if (G != 1 && G != 2 && G != 4 && G != 8 && G != 16) return JENGA_ERR_UNSUPPORTED;
  if (G == 16 && !(k.desc.dtype == JENGA_BF16 && k.t_log2 >= 4)) return JENGA_ERR_UNSUPPORTED;
  const int row = k.desc.head_dim * k.elem_bytes;
  const int T = k.desc.tokens_per_page;
  out->kind = &k;
  out->G = G;
  // bf16 K/V in pages of 16 tokens or more goes to the matrix-core engine, except 16-token pages of
  // 256-element rows with up to 4 query heads per KV head, where the quad engine measures 0.7 %
  // faster; fp32 K/V in 16-token pages goes to the quad engine up to 4 heads per KV head.
  // Everything else takes the general engine.
  out->quad = k.t_log2 == 4 && G <= 4 && row <= 512 &&
              (k.desc.dtype == JENGA_F32 || row == 512);
  out->mat = k.t_log2 >= 4 && k.desc.dtype == JENGA_BF16 && !out->quad;
  const bool paged16 = out->mat || out->quad;      // tiles of 8 KiB K + 8 KiB V in whole pages
  const int tile_tokens = paged16 ? (8 / (row / 64)) * 16 : 8 * (kWave / (row / 16));
  out->tile_log2 = 0;
  while ((1 << out->tile_log2) < tile_tokens) ++out->tile_log2;
  int64_t max_pages = (int64_t(max_seq_len) + T - 1) / T;
  if (window > 0) max_pages = std::min<int64_t>(max_pages, window / T + 2);
  const int64_t max_tiles = (max_pages * T + tile_tokens - 1) / tile_tokens;
  const int64_t w_max = (max_tiles + kSegStartUnits) * k.desc.n_kv_heads * std::max(batch, 1);
  if (w_max > 0x3fffffff) return JENGA_ERR_UNSUPPORTED;
  out->fn = k.desc.dtype == JENGA_F32 ? pick_d<F32>(k.desc.head_dim, out->mat, out->quad, G)
                                      : pick_d<BF16>(k.desc.head_dim, out->mat, out->quad, G);
  const int64_t tile_bytes = int64_t(tile_tokens) * row * 2;
  out->min_chunk_tiles = int(std::max<int64_t>(1, (64 * 1024) / tile_bytes));
  if (pages_per_split > 0) {
    out->chunk_tiles = int(std::max<int64_t>(1, int64_t(pages_per_split) * T / tile_tokens));
    const int64_t n = std::max<int64_t>(1, (w_max + out->chunk_tiles - 1) / out->chunk_tiles);
    if (n > (1 << 22)) return JENGA_ERR_UNSUPPORTED;
    out->n_part_bound = int(n);
  } else {
    out->chunk_tiles = 0;
    out->n_part_bound = kMaxPartitions;
  }
  out->slots = int64_t(out->n_part_bound) + int64_t(std::max(batch, 1)) * k.desc.n_kv_heads;
  return JENGA_OK;
}

int launch_partitions(const Geometry& g) {
  return g.chunk_tiles > 0 ? g.n_part_bound : resident_partitions(g.fn);
}

int64_t workspace_bytes_for(const Geometry& g) {
  return g.slots * g.G * (g.kind->desc.head_dim + 2) * 4;
}

int hip_status() { return hipGetLastError() == hipSuccess ? JENGA_OK : JENGA_ERR_HIP; }

int split_ws(const Geometry& g, void* workspace, int64_t workspace_bytes, float** acc, float** ml) {
  if (!workspace) return JENGA_ERR_INVALID;
  if (!aligned16(workspace)) return JENGA_ERR_ALIGN;
  if (workspace_bytes < workspace_bytes_for(g)) return JENGA_ERR_WORKSPACE;
  *acc = static_cast<float*>(workspace);
  *ml = *acc + g.slots * g.G * g.kind->desc.head_dim;
  return JENGA_OK;
}

}  // namespace

extern "C" {

int jenga_kv_append(const jenga_pool* pool, int32_t kind, int32_t layer, const void* k_new,
                    const void* v_new, const int32_t* block_table, int32_t bt_stride,
                    const int32_t* seq_lens, int32_t batch, jenga_stream stream) {
  if (!pool || kind < 0 || kind >= int32_t(pool->kinds.size())) return JENGA_ERR_INVALID;
  const jenga::Kind& k = pool->kinds[kind];
  if (k.desc.type != JENGA_FULL && k.desc.type != JENGA_WINDOW) return JENGA_ERR_INVALID;
  if (!pool->base || layer < 0 || layer >= k.desc.n_layers || !k_new || !v_new || !block_table ||
      !seq_lens || batch < 0 || bt_stride < 1)
    return JENGA_ERR_INVALID;
  if (!aligned16(k_new) || !aligned16(v_new)) return JENGA_ERR_ALIGN;
  if (batch == 0) return JENGA_OK;
  const int row_bytes = k.desc.head_dim * k.elem_bytes;
  const int64_t threads = int64_t(batch) * k.desc.n_kv_heads * 2 * (row_bytes / 16);
  const int64_t blocks = (threads + 255) / 256;
  if (blocks > 0x7fffffff) return JENGA_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(kv_append_kernel, dim3(unsigned(blocks)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), pool->base + int64_t(layer) * k.slice_bytes,
                     k.small_bytes, int32_t(2 * k.desc.tokens_per_page * row_bytes),
                     int32_t(k.desc.tokens_per_page * row_bytes), k.t_log2, k.desc.n_kv_heads,
                     row_bytes, static_cast<const char*>(k_new), static_cast<const char*>(v_new),
                     block_table, bt_stride, seq_lens, batch, int32_t(pool->n_large * k.per_large - 1));
  return hip_status();
}

int jenga_kv_write_range(const jenga_pool* pool, int32_t kind, int32_t layer, const void* k_src,
                         const void* v_src, const int32_t* cu_tokens, const int32_t* start_pos,
                         const int32_t* block_table, int32_t bt_stride, int32_t batch,
                         int32_t total_tokens, jenga_stream stream) {
  if (!pool || kind < 0 || kind >= int32_t(pool->kinds.size())) return JENGA_ERR_INVALID;
  const jenga::Kind& k = pool->kinds[kind];
  if (!attention_kind(k)) return JENGA_ERR_INVALID;
  if (!pool->base || layer < 0 || layer >= k.desc.n_layers || !k_src || !v_src || !cu_tokens ||
      !start_pos || !block_table || batch < 0 || total_tokens < 0 || bt_stride < 1)
    return JENGA_ERR_INVALID;
  if (!aligned16(k_src) || !aligned16(v_src)) return JENGA_ERR_ALIGN;
  if (batch == 0 || total_tokens == 0) return JENGA_OK;
  const int row_bytes = k.desc.head_dim * k.elem_bytes;
  const int per_token = k.desc.n_kv_heads * 2 * (row_bytes / 16);
  const int threads = per_token >= 256 ? 256 : per_token >= 128 ? 128 : 64;
  hipLaunchKernelGGL(kv_write_range_kernel, dim3(unsigned(total_tokens)), dim3(threads), 0,
                     static_cast<hipStream_t>(stream), pool->base + int64_t(layer) * k.slice_bytes,
                     k.small_bytes, int32_t(2 * k.desc.tokens_per_page * row_bytes),
                     int32_t(k.desc.tokens_per_page * row_bytes), k.t_log2, k.desc.n_kv_heads,
                     row_bytes, static_cast<const char*>(k_src), static_cast<const char*>(v_src),
                     cu_tokens, start_pos, block_table, bt_stride, batch,
                     int32_t(pool->n_large * k.per_large - 1));
  return hip_status();
}

int jenga_decode_num_partitions(const jenga_pool* pool, int32_t kind, int32_t n_q_heads, int32_t batch,
                                int32_t max_seq_len, int32_t window, int32_t pages_per_split) {
  Geometry g;
  const int rc = decode_geometry(pool, kind, n_q_heads, batch, max_seq_len, window, pages_per_split, &g);
  if (rc != JENGA_OK) return rc;
  return g.n_part_bound;
}

int64_t jenga_decode_workspace_bytes(const jenga_pool* pool, int32_t kind, int32_t n_q_heads,
                                     int32_t batch, int32_t max_seq_len, int32_t window,
                                     int32_t pages_per_split) {
  Geometry g;
  const int rc = decode_geometry(pool, kind, n_q_heads, batch, max_seq_len, window, pages_per_split, &g);
  if (rc != JENGA_OK) return rc;
  return workspace_bytes_for(g);
}

int jenga_paged_decode_partial(const jenga_pool* pool, int32_t kind, int32_t layer, const void* q,
                               int32_t n_q_heads, const void* k_new, const void* v_new,
                               const int32_t* block_table, int32_t bt_stride,
                               const int32_t* seq_lens, int32_t batch, int32_t max_seq_len,
                               int32_t window, float scale, int32_t pages_per_split, void* workspace,
                               int64_t workspace_bytes, jenga_stream stream) {
  Geometry g;
  int rc = decode_geometry(pool, kind, n_q_heads, batch, max_seq_len, window, pages_per_split, &g);
  if (rc != JENGA_OK) return rc;
  const jenga::Kind& k = *g.kind;
  if (!pool->base || layer < 0 || layer >= k.desc.n_layers || !q || !block_table || !seq_lens ||
      bt_stride < 1)
    return JENGA_ERR_INVALID;
  if (int64_t(bt_stride) * k.desc.tokens_per_page < max_seq_len) return JENGA_ERR_INVALID;
  if (!aligned16(q)) return JENGA_ERR_ALIGN;
  if ((k_new == nullptr) != (v_new == nullptr)) return JENGA_ERR_INVALID;
  if (k_new && k.desc.type != JENGA_FULL && k.desc.type != JENGA_WINDOW) return JENGA_ERR_INVALID;
  if (k_new && (!aligned16(k_new) || !aligned16(v_new))) return JENGA_ERR_ALIGN;
  float *acc = nullptr, *ml = nullptr;
  rc = split_ws(g, workspace, workspace_bytes, &acc, &ml);
  if (rc != JENGA_OK) return rc;
  if (batch == 0) return JENGA_OK;

  const int row_bytes = k.desc.head_dim * k.elem_bytes;
  DecodeParams p;
  p.layer_base = pool->base + int64_t(layer) * k.slice_bytes;
  p.small_bytes = k.small_bytes;
  p.head_stride = 2 * k.desc.tokens_per_page * row_bytes;
  p.v_offset = k.desc.tokens_per_page * row_bytes;
  p.t_log2 = k.t_log2;
  p.n_kv_heads = k.desc.n_kv_heads;
  p.n_q_heads = n_q_heads;
  p.max_page_id = int32_t(pool->n_large * k.per_large - 1);
  p.q = q;
  p.block_table = block_table;
  p.bt_stride = bt_stride;
  p.seq_lens = seq_lens;
  p.batch = batch;
  p.max_seq_len = max_seq_len;
  p.window = window;
  p.scale_log2 = scale * 1.4426950408889634f;
  p.chunk_tiles = g.chunk_tiles;
  p.min_chunk_tiles = g.min_chunk_tiles;
  p.k_new = k_new;
  p.v_new = v_new;
  p.ws_acc = acc;
  p.ws_ml = ml;
  const int n_part = launch_partitions(g);
  hipLaunchKernelGGL(g.fn, dim3(unsigned(n_part)), dim3(kWave), 0, static_cast<hipStream_t>(stream), p);
  return hip_status();
}

int jenga_splitk_reduce(const jenga_pool* pool, int32_t kind, int32_t n_q_heads,
                        const int32_t* seq_lens, int32_t batch, int32_t max_seq_len, int32_t window,
                        int32_t pages_per_split, const void* workspace, int64_t workspace_bytes,
                        float* out, jenga_stream stream) {
  Geometry g;
  int rc = decode_geometry(pool, kind, n_q_heads, batch, max_seq_len, window, pages_per_split, &g);
  if (rc != JENGA_OK) return rc;
  const jenga::Kind& k = *g.kind;
  if (!seq_lens || !out) return JENGA_ERR_INVALID;
  if (!aligned16(out)) return JENGA_ERR_ALIGN;
  float *acc = nullptr, *ml = nullptr;
  rc = split_ws(g, const_cast<void*>(workspace), workspace_bytes, &acc, &ml);
  if (rc != JENGA_OK) return rc;
  if (batch == 0) return JENGA_OK;
  const int n_part = launch_partitions(g);
  const dim3 grid(static_cast<unsigned>(n_q_heads), static_cast<unsigned>(batch));
  hipStream_t st = static_cast<hipStream_t>(stream);
#define JENGA_LAUNCH_REDUCE(DIM)                                                                   \
  hipLaunchKernelGGL((splitk_reduce_kernel<DIM>), grid, dim3(kWave), 0, st, acc, ml, seq_lens,    \
                     batch, max_seq_len, window, k.t_log2, g.tile_log2, g.chunk_tiles,             \
                     g.min_chunk_tiles, n_part, k.desc.n_kv_heads, n_q_heads, out)
  switch (k.desc.head_dim) {
    case 64: JENGA_LAUNCH_REDUCE(64); break;
    case 128: JENGA_LAUNCH_REDUCE(128); break;
    default: JENGA_LAUNCH_REDUCE(256); break;
  }
#undef JENGA_LAUNCH_REDUCE
  return hip_status();
}

int jenga_paged_decode(const jenga_pool* pool, int32_t kind, int32_t layer, const void* q,
                       int32_t n_q_heads, const void* k_new, const void* v_new,
                       const int32_t* block_table, int32_t bt_stride,
                       const int32_t* seq_lens, int32_t batch, int32_t max_seq_len, int32_t window,
                       float scale, int32_t pages_per_split, void* workspace, int64_t workspace_bytes,
                       float* out, jenga_stream stream) {
  if (!out) return JENGA_ERR_INVALID;
  if (!aligned16(out)) return JENGA_ERR_ALIGN;
  const int rc = jenga_paged_decode_partial(pool, kind, layer, q, n_q_heads, k_new, v_new, block_table, bt_stride,
                                            seq_lens, batch, max_seq_len, window, scale,
                                            pages_per_split, workspace, workspace_bytes, stream);
  if (rc != JENGA_OK) return rc;
  return jenga_splitk_reduce(pool, kind, n_q_heads, seq_lens, batch, max_seq_len, window,
                             pages_per_split, workspace, workspace_bytes, out, stream);
}

int jenga_stream_copy(void* dst, const void* src, int64_t bytes, jenga_stream stream) {
  if (!dst || !src || bytes < 0 || bytes % 16 != 0) return JENGA_ERR_INVALID;
  if (!aligned16(dst) || !aligned16(src)) return JENGA_ERR_ALIGN;
  if (bytes == 0) return JENGA_OK;
  const int64_t n = bytes / 16;
  const unsigned blocks = unsigned(std::min<int64_t>((n + 255) / 256, 256 * 32));
  hipLaunchKernelGGL(stream_copy_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<u32x4*>(dst), static_cast<const u32x4*>(src), n);
  return hip_status();
}

int jenga_stream_read(const void* src, int64_t bytes, void* sink, jenga_stream stream) {
  if (!src || !sink || bytes < 0 || bytes % 16 != 0) return JENGA_ERR_INVALID;
  if (!aligned16(src)) return JENGA_ERR_ALIGN;
  if (bytes == 0) return JENGA_OK;
  const int64_t n = bytes / 16;
  const unsigned blocks = unsigned(std::min<int64_t>((n + 255) / 256, 256 * 32));
  hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(src), n, static_cast<unsigned*>(sink));
  return hip_status();
}

}  // extern "C"
