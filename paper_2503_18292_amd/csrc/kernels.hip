// Device half of the library, written for gfx950 (CDNA4, 64-wide wavefronts).
//
//   kv_append_kernel       stores the new token's K/V rows into their page
//   decode_partial_kernel  one wavefront per (request, KV head, split-K partition):
//                          streams K and V pages with 16-byte loads, fp32 online
//                          softmax, the G query heads of the group share every load
//   splitk_reduce_kernel   log-sum-exp merge of the partitions
//
// Decode attention is a bandwidth-bound matrix-vector product (G flop per byte of
// bf16 K/V), so no matrix-core instructions are used; the design goal is to keep
// many 1 KiB wave-wide loads in flight per wavefront and to spend few vector-ALU
// instructions per byte.
//
// The kernel view of the pool is the one of paper Sec. 4.2: a start pointer (pool
// base + layer offset), a page stride (the kind's small-page size) and page ids
// (the kind's block table).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "pool_internal.hpp"

namespace {

constexpr int kWave = 64;
constexpr int kLoadsPerTile = 8;     // 16-byte loads per lane per K (or V) tile: 8 KiB per wave
constexpr int kMaxPagesPerSplit = 256;
constexpr float kNegBig = -1.0e30f;  // finite stand-in for -inf: keeps exp2(m - m) well defined

struct DecodeParams {
  const char* layer_base;     // pool base + layer * slice_bytes
  int64_t small_bytes;        // page stride
  int32_t head_stride;        // bytes between KV heads inside a layer slice: 2 * T * D * e
  int32_t v_offset;           // bytes from a head's K rows to its V rows: T * D * e
  int32_t t_log2;
  int32_t n_kv_heads;
  int32_t n_q_heads;
  const void* q;
  const int32_t* block_table;
  int32_t bt_stride;
  const int32_t* seq_lens;
  int32_t batch;
  int32_t max_seq_len;
  int32_t window;
  float scale_log2;           // softmax scale * log2(e): scores live in the base-2 domain
  int32_t pages_per_split;
  int32_t n_split;
  float* ws_acc;              // [batch][n_q_heads][n_split][D]
  float* ws_ml;               // [batch][n_q_heads][n_split][2]  (running max, running sum)
};

// Visible pages [p_lo, p_hi) and first visible token of a request of length L.
__device__ __forceinline__ void visible_pages(int L, int window, int t_log2, int* lo_tok,
                                              int* p_lo, int* p_hi) {
  const int lo = window > 0 ? max(0, L - window) : 0;
  *lo_tok = lo;
  *p_lo = lo >> t_log2;
  *p_hi = (L + (1 << t_log2) - 1) >> t_log2;
}


// Number of live split-K partitions of a request of length L.
__device__ __forceinline__ int live_splits(int L, int window, int t_log2, int pages_per_split) {
  if (L <= 0) return 0;
  int lo_tok, p_lo, p_hi;
  visible_pages(L, window, t_log2, &lo_tok, &p_lo, &p_hi);
  return (p_hi - p_lo + pages_per_split - 1) / pages_per_split;
}

// Dense, XCD-aware task numbering.  The hardware deals consecutive blocks of the 1-D grid
// round-robin to the 8 XCDs (each with its own L2 and address-translation cache).  Live
// (request, partition) pairs are numbered densely as groups g = 0, 1, ...; group g runs on
// XCD g % 8 with all its KV heads, so
//   * the XCDs carry equal work whatever the mix of sequence lengths (a 3-D grid over
//     (partition, head, request) sends all blocks of one partition index to one XCD whenever
//     the partition count is a multiple of 8, and short requests leave the high partition
//     indices empty: the XCDs then finish up to 20 % apart);
//   * the KV heads of a page, which lie next to each other in the page's layer slice, are
//     read through one XCD, so every page translation is needed on one XCD only.
// Every block recomputes the prefix sum of live partitions from seq_lens, 64 requests per
// pass: one coalesced load, the same latency as reading its own length.
// Returns false for blocks past the last live group.
__device__ __forceinline__ bool locate_task(const DecodeParams& p, int lane, int* b_out, int* split_out,
                                            int* kvh_out, int* len_out) {
  // hardware block t -> (group g of one (request, partition), KV head): blocks t, t+8, t+16, ...
  // of a run of 8 * n_kv_heads blocks share g, so all KV heads of a page group run on one XCD
  const int run = 8 * p.n_kv_heads;
  const int r = blockIdx.x % run;
  const int g = (blockIdx.x / run) * 8 + (r & 7);
  *kvh_out = r >> 3;
  int base = 0;
  for (int c0 = 0; c0 < p.batch; c0 += kWave) {
    const int i = c0 + lane;
    const int Li = i < p.batch ? min(p.seq_lens[i], p.max_seq_len) : 0;
    const int n = live_splits(Li, p.window, p.t_log2, p.pages_per_split);
    int incl = n;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const int up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    const int total = __builtin_amdgcn_readlane(incl, kWave - 1);
    if (g < base + total) {
      const unsigned long long hit = __ballot(base + incl > g);
      const int who = __builtin_ctzll(hit);
      *b_out = c0 + who;
      *len_out = __builtin_amdgcn_readlane(Li, who);
      *split_out = g - (base + __builtin_amdgcn_readlane(incl, who) - __builtin_amdgcn_readlane(n, who));
      return true;
    }
    base += total;
  }
  return false;
}

// ---- cross-lane sums -------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true);
  return x + __int_as_float(y);
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
  using storage = float;
  static constexpr int kBytes = 4;
};
struct BF16 {
  using storage = uint16_t;
  static constexpr int kBytes = 2;
};

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));   // 16 bytes, a native vector so it can be loaded non-temporally

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

// ---- the decode kernel -------------------------------------------------------------
//
// Lane geometry.  A token's K (or V) row is D*e bytes = LPT lanes x 16 bytes, so one
// wave-wide 16-byte load covers TPL = 64 / LPT consecutive tokens (1 KiB, contiguous in
// the page).  Lane l holds elements [sub*EPL, sub*EPL + EPL) of token (l / LPT) of the
// load, sub = l % LPT.  A tile is kLoadsPerTile such loads of K and as many of V.
//
// Each group of LPT lanes runs its own online softmax over the tokens it sees (token
// index mod TPL == its group), so the only cross-lane traffic in the loop is the sum of
// the partial dot products inside a group; the TPL groups are merged once at the end.
template <typename E, int D, int G>
__global__ __launch_bounds__(kWave) void decode_partial_kernel(const DecodeParams p) {
  constexpr int EPL = 16 / E::kBytes;
  constexpr int LPT = D / EPL;
  constexpr int TPL = kWave / LPT;
  constexpr int NL = kLoadsPerTile;
  constexpr int TT = NL * TPL;             // tokens per tile
  constexpr int ROW = D * E::kBytes;       // bytes per token row

  const int lane = threadIdx.x;
  int b, split, kvh, L;
  if (!locate_task(p, lane, &b, &split, &kvh, &L)) return;
  int lo_tok, p_lo, p_hi;
  visible_pages(L, p.window, p.t_log2, &lo_tok, &p_lo, &p_hi);
  const int page0 = p_lo + split * p.pages_per_split;
  if (page0 >= p_hi) return;
  const int n_pages = min(p.pages_per_split, p_hi - page0);

  // block-table slice of this partition, staged once in LDS
  __shared__ int32_t s_pages[kMaxPagesPerSplit];
  for (int i = lane; i < n_pages; i += kWave)
    s_pages[i] = p.block_table[int64_t(b) * p.bt_stride + page0 + i];
  __syncthreads();

  const int sub = lane % LPT;
  const int grp = lane / LPT;
  const int t_mask = (1 << p.t_log2) - 1;
  const int tok0 = page0 << p.t_log2;                  // absolute index of the partition's first token
  const int n_tok = n_pages << p.t_log2;
  const int n_tiles = (n_tok + TT - 1) / TT;
  const char* head_base = p.layer_base + int64_t(kvh) * p.head_stride + lane * 16;

  // the G query rows of this KV head, 16 bytes per lane each
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

  // Issues the loads of one tile of K (v_off = 0) or V (v_off = p.v_offset).
  auto load_tile = [&](int tile, int v_off, u32x4* buf) {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int tok = tile * TT + i * TPL;               // first token of this load, wave-uniform
      const int page_rel = tok >> p.t_log2;
      if (page_rel < n_pages) {
        const int sid = __builtin_amdgcn_readfirstlane(s_pages[page_rel]);
        const char* src = head_base + int64_t(sid) * p.small_bytes + v_off + (tok & t_mask) * ROW;
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

    // scores of the tile's tokens against the G query heads (base-2 logits)
    float s[NL][G];
#pragma unroll
    for (int i = 0; i < NL; ++i)
#pragma unroll
      for (int g = 0; g < G; ++g)
        s[i][g] = group_sum<LPT>(dot16<E>(kbuf[i], qv[g])) * p.scale_log2;

    if (tile + 1 < n_tiles) load_tile(tile + 1, 0, kbuf);

    // tokens of this lane's group that are outside [lo_tok, L) or past the partition
    const int t_abs0 = tok0 + tile * TT + grp;
    const bool clean = (tok0 + tile * TT >= lo_tok) && (tok0 + (tile + 1) * TT <= L) &&
                       ((tile + 1) * TT <= n_tok);
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

  if (grp == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const int64_t slot = (int64_t(b) * p.n_q_heads + kvh * G + g) * p.n_split + split;
      float* dst = p.ws_acc + slot * D + sub * EPL;
#pragma unroll
      for (int j = 0; j < EPL; j += 4)
        *reinterpret_cast<float4*>(dst + j) =
            make_float4(acc[g][j], acc[g][j + 1], acc[g][j + 2], acc[g][j + 3]);
      if (lane == 0) *reinterpret_cast<float2*>(p.ws_ml + slot * 2) = make_float2(m[g], l[g]);
    }
  }
}

// ---- the decode kernel for 16-token pages ---------------------------------------------
//
// Same task decomposition and same results as the kernel above, with far fewer vector-ALU
// instructions per byte.  The two operands are read in two different lane geometries:
//
//   K  lane l reads token l/4 of the page, the (l%4)-th 16 bytes of every 64-byte piece of
//      that token's row (quads of lanes read 64 contiguous bytes).  A lane therefore sums
//      a quarter of ONE token's dot product in its own registers and the only cross-lane
//      work per score is a sum over 4 lanes.
//   V  lane l reads 16 contiguous bytes at l*16 of every KiB of the page (as above), i.e.
//      it owns EPL output elements and sees token (l / LPT) of each load.
//
// The softmax weights are produced in the K geometry (one token per quad of lanes) and
// consumed in the V geometry, so they cross lanes through a small LDS array (broadcast
// reads, no bank conflicts).  The running maximum is wave-uniform: it is reduced across the
// wave once per tile and page, which also makes the final merge of the V lane groups a
// plain sum.
template <typename E, int D, int G>
__global__ __launch_bounds__(kWave) void decode_partial_t16_kernel(const DecodeParams p) {
  constexpr int T = 16;
  constexpr int ROW = D * E::kBytes;            // bytes per token row
  constexpr int EPL = 16 / E::kBytes;           // elements per 16 bytes
  constexpr int KCH = ROW / 64;                 // 64-byte pieces per row == 1 KiB loads per page
  constexpr int PPT = KCH >= 8 ? 1 : 8 / KCH;   // pages per tile
  constexpr int NLD = PPT * KCH;                // loads per tile, K and V alike (8 or 16)
  constexpr int LPT = ROW / 16;                 // V geometry: lanes per token row
  constexpr int TPL = kWave / LPT;              // V geometry: tokens per load
  constexpr int V_OFF = T * ROW;                // K rows come first in a (page, head) block

  const int lane = threadIdx.x;
  int b, split, kvh, L;
  if (!locate_task(p, lane, &b, &split, &kvh, &L)) return;
  int lo_tok, p_lo, p_hi;
  visible_pages(L, p.window, 4, &lo_tok, &p_lo, &p_hi);
  const int page0 = p_lo + split * p.pages_per_split;
  if (page0 >= p_hi) return;
  const int n_pages = min(p.pages_per_split, p_hi - page0);

  __shared__ int32_t s_pages[kMaxPagesPerSplit];
  __shared__ float s_prob[2][PPT * T][G];       // softmax weights of a tile, double buffered
  for (int i = lane; i < n_pages; i += kWave)
    s_pages[i] = p.block_table[int64_t(b) * p.bt_stride + page0 + i];
  __syncthreads();

  const int tok0 = page0 * T;
  const int n_tiles = (n_pages + PPT - 1) / PPT;
  const char* kv_base = p.layer_base + int64_t(kvh) * p.head_stride;   // wave-uniform
  const unsigned k_voff = (lane >> 2) * ROW + (lane & 3) * 16;         // K geometry
  const unsigned v_voff = V_OFF + lane * 16;                           // V geometry
  const int k_tok = lane >> 2;                                         // token of the page this lane scores
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

  // Page ids of the partition live in one register per stream, lane j holding page
  // (chunk * 64 + j); v_readlane turns one into a scalar without an LDS round trip.
  int pid_k = 0, pid_v = 0;
  auto refill = [&](int page_rel, int& reg) {
    if ((page_rel & 63) == 0) reg = (page_rel + lane < n_pages) ? s_pages[page_rel + lane] : 0;
  };
  auto page_ptr = [&](int page_rel, int reg) -> const char* {
    const int sid = __builtin_amdgcn_readlane(reg, page_rel & 63);
    return kv_base + int64_t(sid) * p.small_bytes;
  };
  auto load_k = [&](int tile, u32x4* buf) {
    refill(tile * PPT, pid_k);
#pragma unroll
    for (int pp = 0; pp < PPT; ++pp) {
      const int page_rel = tile * PPT + pp;
      if (PPT == 1 || page_rel < n_pages) {
        const char* pb = page_ptr(page_rel, pid_k);
#pragma unroll
        for (int c = 0; c < KCH; ++c)
          buf[pp * KCH + c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pb + k_voff + c * 64));
      } else {
#pragma unroll
        for (int c = 0; c < KCH; ++c) buf[pp * KCH + c] = u32x4{0, 0, 0, 0};
      }
    }
  };
  auto load_v = [&](int tile, u32x4* buf) {
    refill(tile * PPT, pid_v);
#pragma unroll
    for (int pp = 0; pp < PPT; ++pp) {
      const int page_rel = tile * PPT + pp;
      if (PPT == 1 || page_rel < n_pages) {
        const char* pb = page_ptr(page_rel, pid_v);
#pragma unroll
        for (int j = 0; j < KCH; ++j)
          buf[pp * KCH + j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(pb + v_voff + j * 1024));
      } else {
#pragma unroll
        for (int j = 0; j < KCH; ++j) buf[pp * KCH + j] = u32x4{0, 0, 0, 0};
      }
    }
  };

  u32x4 kbuf[NLD], vbuf[NLD];
  load_k(0, kbuf);

  for (int tile = 0; tile < n_tiles; ++tile) {
    load_v(tile, vbuf);

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

    if (tile + 1 < n_tiles) load_k(tile + 1, kbuf);

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
      // wave maximum: rows of 16 lanes first, then row -> next row broadcasts, lane 63 has it
      mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(mx), __float_as_int(mx), 0x124, 0xf, 0xf, false)));  // row_ror:4
      mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(mx), __float_as_int(mx), 0x128, 0xf, 0xf, false)));  // row_ror:8
      mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(mx), __float_as_int(mx), 0x142, 0xa, 0xf, false)));  // row_bcast:15
      mx = fmaxf(mx, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(mx), __float_as_int(mx), 0x143, 0xc, 0xf, false)));  // row_bcast:31
      const float tile_max = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mx), 63));
      const float m_new = fmaxf(m[g], tile_max);
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

  if (v_grp == 0) {
    const int sub = lane % LPT;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const int64_t slot = (int64_t(b) * p.n_q_heads + kvh * G + g) * p.n_split + split;
      float* dst = p.ws_acc + slot * D + sub * EPL;
#pragma unroll
      for (int j = 0; j < EPL; j += 4)
        *reinterpret_cast<float4*>(dst + j) =
            make_float4(acc[g][j], acc[g][j + 1], acc[g][j + 2], acc[g][j + 3]);
      if (lane == 0) *reinterpret_cast<float2*>(p.ws_ml + slot * 2) = make_float2(m[g], l[g]);
    }
  }
}

// One block per (request, query head); thread i owns output elements [4i, 4i+4).
template <int D>
__global__ __launch_bounds__(D / 4) void splitk_reduce_kernel(
    const float* __restrict__ ws_acc, const float* __restrict__ ws_ml,
    const int32_t* __restrict__ seq_lens, int32_t max_seq_len, int32_t window, int32_t t_log2,
    int32_t pages_per_split, int32_t n_split, int32_t n_q_heads, float* __restrict__ out) {
  const int hq = blockIdx.x;
  const int b = blockIdx.y;
  const int tid = threadIdx.x;
  float4* dst = reinterpret_cast<float4*>(out + (int64_t(b) * n_q_heads + hq) * D) + tid;
  const int L = min(seq_lens[b], max_seq_len);
  if (L <= 0) {
    *dst = make_float4(0.f, 0.f, 0.f, 0.f);
    return;
  }
  const int n_live = live_splits(L, window, t_log2, pages_per_split);
  const int64_t slot0 = (int64_t(b) * n_q_heads + hq) * n_split;
  float m_star = kNegBig;
  for (int s = 0; s < n_live; ++s) m_star = fmaxf(m_star, ws_ml[(slot0 + s) * 2]);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  float l_star = 0.f;
  for (int s = 0; s < n_live; ++s) {
    const float2 ml = *reinterpret_cast<const float2*>(ws_ml + (slot0 + s) * 2);
    const float w = __builtin_amdgcn_exp2f(ml.x - m_star);
    const float4 a = *(reinterpret_cast<const float4*>(ws_acc + (slot0 + s) * D) + tid);
    acc.x = fmaf(a.x, w, acc.x); acc.y = fmaf(a.y, w, acc.y);
    acc.z = fmaf(a.z, w, acc.z); acc.w = fmaf(a.w, w, acc.w);
    l_star = fmaf(ml.y, w, l_star);
  }
  const float inv = l_star > 0.f ? 1.0f / l_star : 0.f;
  *dst = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
}

// One thread per 16 bytes of the new K and V rows.
__global__ __launch_bounds__(256) void kv_append_kernel(
    char* __restrict__ layer_base, int64_t small_bytes, int32_t head_stride, int32_t v_offset,
    int32_t t_log2, int32_t n_kv_heads, int32_t row_bytes, const char* __restrict__ k_new,
    const char* __restrict__ v_new, const int32_t* __restrict__ block_table, int32_t bt_stride,
    const int32_t* __restrict__ seq_lens, int32_t batch) {
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
  if (sid < 0) return;
  const char* src = (is_v ? v_new : k_new) + (int64_t(b) * n_kv_heads + h) * row_bytes + c * 16;
  char* dst = layer_base + int64_t(sid) * small_bytes + int64_t(h) * head_stride +
              (is_v ? v_offset : 0) + (pos & ((1 << t_log2) - 1)) * row_bytes + c * 16;
  *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
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

// ---- host side: validation, split geometry, launch ---------------------------------

bool attention_kind(const jenga::Kind& k) {
  return k.desc.type == JENGA_FULL || k.desc.type == JENGA_WINDOW || k.desc.type == JENGA_CROSS;
}

bool aligned16(const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }

// Tokens per tile of the decode kernel for this kind (see the lane geometry above).
int tile_tokens(const jenga::Kind& k) {
  const int lanes_per_token = k.desc.head_dim * k.elem_bytes / 16;
  return kLoadsPerTile * (kWave / lanes_per_token);
}

struct SplitGeom {
  int pages_per_split;
  int n_split;
};

// Split-K geometry.  A partition is a whole number of pages and of tiles.  Automatic
// choice: enough partitions to keep every SIMD of the 256 compute units busy with
// several wavefronts, without making partitions so small that the workspace traffic
// (one (D+2)-float record per partition and query head) shows up next to the K/V bytes.
int split_geometry(const jenga::Kind& k, int batch, int max_seq_len, int window, int pages_per_split,
                   SplitGeom* out) {
  const int T = k.desc.tokens_per_page;
  const int align = std::max(1, tile_tokens(k) / T);        // pages per tile
  int64_t max_pages = (int64_t(max_seq_len) + T - 1) / T;
  if (window > 0) max_pages = std::min<int64_t>(max_pages, window / T + 2);
  max_pages = std::max<int64_t>(max_pages, 1);
  int pps = pages_per_split;
  if (pps < 0) return JENGA_ERR_INVALID;
  if (pps == 0) {
    const int64_t units = int64_t(std::max(batch, 1)) * k.desc.n_kv_heads * max_pages;
    const int64_t target_partitions = 16384;
    const int64_t bytes_per_page_head = k.slice_bytes / k.desc.n_kv_heads;
    const int64_t min_pages = std::max<int64_t>(1, (128 * 1024) / bytes_per_page_head);  // >= 128 KiB each
    int64_t want = (units + target_partitions - 1) / target_partitions;
    want = std::max(want, min_pages);
    want = std::min<int64_t>(want, kMaxPagesPerSplit);
    pps = int(want);
  }
  pps = ((pps + align - 1) / align) * align;
  if (pps > kMaxPagesPerSplit) return JENGA_ERR_INVALID;
  // keep the partition count within the grid limit
  int64_t n_split = (max_pages + pps - 1) / pps;
  if (n_split > (1 << 20)) return JENGA_ERR_UNSUPPORTED;
  out->pages_per_split = pps;
  out->n_split = int(n_split);
  return JENGA_OK;
}

int64_t workspace_bytes_for(const jenga::Kind& k, int n_q_heads, int batch, int n_split) {
  const int64_t slots = int64_t(batch) * n_q_heads * n_split;
  return slots * k.desc.head_dim * 4 + slots * 2 * 4;
}

struct DecodeCheck {
  const jenga::Kind* kind;
  SplitGeom geom;
  int G;
};

int check_decode(const jenga_pool* pool, int32_t kind, int32_t n_q_heads, int32_t batch,
                 int32_t max_seq_len, int32_t window, int32_t pages_per_split, DecodeCheck* out) {
  if (!pool || kind < 0 || kind >= int32_t(pool->kinds.size())) return JENGA_ERR_INVALID;
  const jenga::Kind& k = pool->kinds[kind];
  if (!attention_kind(k)) return JENGA_ERR_INVALID;
  if (batch < 0 || batch > 65535 || max_seq_len < 0 || window < 0 || n_q_heads < 1)
    return JENGA_ERR_INVALID;
  if (n_q_heads % k.desc.n_kv_heads != 0) return JENGA_ERR_INVALID;
  const int G = n_q_heads / k.desc.n_kv_heads;
  if (G != 1 && G != 2 && G != 4 && G != 8) return JENGA_ERR_UNSUPPORTED;
  const int rc = split_geometry(k, batch, max_seq_len, window, pages_per_split, &out->geom);
  if (rc != JENGA_OK) return rc;
  out->kind = &k;
  out->G = G;
  return JENGA_OK;
}

template <typename E, int D>
void launch_partial_g(int G, dim3 grid, hipStream_t st, const DecodeParams& p) {
  if (p.t_log2 == 4 && G <= 4) {     // 16-token pages: the lane-per-token kernel
    switch (G) {
      case 1: hipLaunchKernelGGL((decode_partial_t16_kernel<E, D, 1>), grid, dim3(kWave), 0, st, p); break;
      case 2: hipLaunchKernelGGL((decode_partial_t16_kernel<E, D, 2>), grid, dim3(kWave), 0, st, p); break;
      default: hipLaunchKernelGGL((decode_partial_t16_kernel<E, D, 4>), grid, dim3(kWave), 0, st, p); break;
    }
    return;
  }
  switch (G) {
    case 1: hipLaunchKernelGGL((decode_partial_kernel<E, D, 1>), grid, dim3(kWave), 0, st, p); break;
    case 2: hipLaunchKernelGGL((decode_partial_kernel<E, D, 2>), grid, dim3(kWave), 0, st, p); break;
    case 4: hipLaunchKernelGGL((decode_partial_kernel<E, D, 4>), grid, dim3(kWave), 0, st, p); break;
    default: hipLaunchKernelGGL((decode_partial_kernel<E, D, 8>), grid, dim3(kWave), 0, st, p); break;
  }
}

template <typename E>
void launch_partial_d(int D, int G, dim3 grid, hipStream_t st, const DecodeParams& p) {
  switch (D) {
    case 64: launch_partial_g<E, 64>(G, grid, st, p); break;
    case 128: launch_partial_g<E, 128>(G, grid, st, p); break;
    default: launch_partial_g<E, 256>(G, grid, st, p); break;
  }
}

int hip_status() { return hipGetLastError() == hipSuccess ? JENGA_OK : JENGA_ERR_HIP; }

int split_ws(const jenga::Kind& k, int n_q_heads, int batch, int n_split, void* workspace,
             int64_t workspace_bytes, float** acc, float** ml) {
  if (!workspace) return JENGA_ERR_INVALID;
  if (!aligned16(workspace)) return JENGA_ERR_ALIGN;
  if (workspace_bytes < workspace_bytes_for(k, n_q_heads, batch, n_split)) return JENGA_ERR_WORKSPACE;
  const int64_t slots = int64_t(batch) * n_q_heads * n_split;
  *acc = static_cast<float*>(workspace);
  *ml = *acc + slots * k.desc.head_dim;
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
                     block_table, bt_stride, seq_lens, batch);
  return hip_status();
}

int jenga_decode_num_splits(const jenga_pool* pool, int32_t kind, int32_t batch, int32_t max_seq_len,
                            int32_t window, int32_t pages_per_split, int32_t* out_pages_per_split) {
  DecodeCheck c;
  if (!pool || kind < 0 || kind >= int32_t(pool->kinds.size())) return JENGA_ERR_INVALID;
  const int rc = check_decode(pool, kind, pool->kinds[kind].desc.n_kv_heads, batch, max_seq_len,
                              window, pages_per_split, &c);
  if (rc != JENGA_OK) return rc;
  if (out_pages_per_split) *out_pages_per_split = c.geom.pages_per_split;
  return c.geom.n_split;
}

int64_t jenga_decode_workspace_bytes(const jenga_pool* pool, int32_t kind, int32_t n_q_heads,
                                     int32_t batch, int32_t max_seq_len, int32_t window,
                                     int32_t pages_per_split) {
  DecodeCheck c;
  const int rc = check_decode(pool, kind, n_q_heads, batch, max_seq_len, window, pages_per_split, &c);
  if (rc != JENGA_OK) return rc;
  return std::max<int64_t>(16, workspace_bytes_for(*c.kind, n_q_heads, batch, c.geom.n_split));
}

int jenga_paged_decode_partial(const jenga_pool* pool, int32_t kind, int32_t layer, const void* q,
                               int32_t n_q_heads, const int32_t* block_table, int32_t bt_stride,
                               const int32_t* seq_lens, int32_t batch, int32_t max_seq_len,
                               int32_t window, float scale, int32_t pages_per_split, void* workspace,
                               int64_t workspace_bytes, jenga_stream stream) {
  DecodeCheck c;
  int rc = check_decode(pool, kind, n_q_heads, batch, max_seq_len, window, pages_per_split, &c);
  if (rc != JENGA_OK) return rc;
  const jenga::Kind& k = *c.kind;
  if (!pool->base || layer < 0 || layer >= k.desc.n_layers || !q || !block_table || !seq_lens ||
      bt_stride < 1)
    return JENGA_ERR_INVALID;
  if (int64_t(bt_stride) * k.desc.tokens_per_page < max_seq_len) return JENGA_ERR_INVALID;
  if (!aligned16(q)) return JENGA_ERR_ALIGN;
  float *acc = nullptr, *ml = nullptr;
  rc = split_ws(k, n_q_heads, batch, c.geom.n_split, workspace, workspace_bytes, &acc, &ml);
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
  p.q = q;
  p.block_table = block_table;
  p.bt_stride = bt_stride;
  p.seq_lens = seq_lens;
  p.batch = batch;
  p.max_seq_len = max_seq_len;
  p.window = window;
  p.scale_log2 = scale * 1.4426950408889634f;
  p.pages_per_split = c.geom.pages_per_split;
  p.n_split = c.geom.n_split;
  p.ws_acc = acc;
  p.ws_ml = ml;
  // 1-D grid with room for every request at max_seq_len; blocks past the live tasks exit
  const int64_t n_groups = (int64_t(c.geom.n_split) * batch + 7) / 8 * 8;    // whole runs of 8 groups
  const int64_t n_blocks = n_groups * k.desc.n_kv_heads;
  if (n_blocks > 0x7fffffff) return JENGA_ERR_UNSUPPORTED;
  const dim3 grid(static_cast<unsigned>(n_blocks));
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (k.desc.dtype == JENGA_F32)
    launch_partial_d<F32>(k.desc.head_dim, c.G, grid, st, p);
  else
    launch_partial_d<BF16>(k.desc.head_dim, c.G, grid, st, p);
  return hip_status();
}

int jenga_splitk_reduce(const jenga_pool* pool, int32_t kind, int32_t n_q_heads,
                        const int32_t* seq_lens, int32_t batch, int32_t max_seq_len, int32_t window,
                        int32_t pages_per_split, const void* workspace, int64_t workspace_bytes,
                        float* out, jenga_stream stream) {
  DecodeCheck c;
  int rc = check_decode(pool, kind, n_q_heads, batch, max_seq_len, window, pages_per_split, &c);
  if (rc != JENGA_OK) return rc;
  const jenga::Kind& k = *c.kind;
  if (!seq_lens || !out) return JENGA_ERR_INVALID;
  if (!aligned16(out)) return JENGA_ERR_ALIGN;
  float *acc = nullptr, *ml = nullptr;
  rc = split_ws(k, n_q_heads, batch, c.geom.n_split, const_cast<void*>(workspace), workspace_bytes,
                &acc, &ml);
  if (rc != JENGA_OK) return rc;
  if (batch == 0) return JENGA_OK;
  const dim3 grid(static_cast<unsigned>(n_q_heads), static_cast<unsigned>(batch));
  hipStream_t st = static_cast<hipStream_t>(stream);
  switch (k.desc.head_dim) {
    case 64:
      hipLaunchKernelGGL((splitk_reduce_kernel<64>), grid, dim3(16), 0, st, acc, ml, seq_lens,
                         max_seq_len, window, k.t_log2, c.geom.pages_per_split, c.geom.n_split,
                         n_q_heads, out);
      break;
    case 128:
      hipLaunchKernelGGL((splitk_reduce_kernel<128>), grid, dim3(32), 0, st, acc, ml, seq_lens,
                         max_seq_len, window, k.t_log2, c.geom.pages_per_split, c.geom.n_split,
                         n_q_heads, out);
      break;
    default:
      hipLaunchKernelGGL((splitk_reduce_kernel<256>), grid, dim3(64), 0, st, acc, ml, seq_lens,
                         max_seq_len, window, k.t_log2, c.geom.pages_per_split, c.geom.n_split,
                         n_q_heads, out);
      break;
  }
  return hip_status();
}

int jenga_paged_decode(const jenga_pool* pool, int32_t kind, int32_t layer, const void* q,
                       int32_t n_q_heads, const int32_t* block_table, int32_t bt_stride,
                       const int32_t* seq_lens, int32_t batch, int32_t max_seq_len, int32_t window,
                       float scale, int32_t pages_per_split, void* workspace, int64_t workspace_bytes,
                       float* out, jenga_stream stream) {
  if (!out) return JENGA_ERR_INVALID;
  if (!aligned16(out)) return JENGA_ERR_ALIGN;
  const int rc = jenga_paged_decode_partial(pool, kind, layer, q, n_q_heads, block_table, bt_stride,
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
