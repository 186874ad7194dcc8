// Shared by the decode engines (device code, gfx950): launch parameters, the flat work
// partitioning, cross-lane helpers, element types, page-id registers and the partial record.
// Included by kernels.hip only; everything lives in that file's unnamed namespace.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

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

}  // namespace
