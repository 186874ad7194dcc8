// Decode engine on the matrix cores: bf16 and fp32 K/V, any page size (see kernels.hip for the front end).
#pragma once

#include "decode_common.hpp"

namespace {

// ---- both contractions of a 16-token block on the matrix cores ------------------------------
//
// The work per 16-token block is a small dense contraction, scores = K[16 x D] . Q^T[D x G] and
// out += P[G x 16] . V[16 x D], and the matrix cores take it off the vector ALUs altogether:
// with 8 heads on every K/V byte those can no longer keep up with HBM (an engine on the vector
// ALUs needed about 70 instructions per KiB), and with fewer heads the loads still issue
// earlier and more evenly when so little else competes for the issue slots.  The G heads are
// padded to the 16 rows / columns of the instructions, so any number from 1 to 16 can be served:
// G_ = 0 is a build that takes it at run time (3, 5, 6, 7 ... heads per KV head), the powers of
// two have builds of their own (1 % faster: the record stores and query loads are resolved at
// compile time).  Operand layouts (lane l, n = l % 16, j = l / 16), checked on the device: A
// holds row n and B holds column n, each with consecutive k (8j .. 8j+7 for 16x16x32, 4j .. 4j+3
// for 16x16x16); the result holds column n, rows 4j .. 4j+3.
//   scores  v_mfma_f32_16x16x32_bf16, A = K page (row = token, k = d): lane (n, j) reads the
//           16 bytes at d = 8j of each 64-byte piece of token n's row -- a plain 16-byte load,
//           64-byte runs per token.  B = Q (column = head, zero for the padding heads).
//           Result: lane (n, j) holds head n, tokens 4j .. 4j+3 of the page.
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
// MODE_ 0: pages of 16, 32, 64 or 128 tokens, i.e. 1, 2, 4 or 8 whole blocks.
// MODE_ 1: the pages hold 8 tokens, half a block (a build of its own, so that the usual case keeps
// a scalar page address plus a constant lane offset for every load).
// MODE_ 2: pages of any other size (1, 2, 4, 24 ... tokens): the rows of a block come from
// whatever pages its 16 tokens fall into, every lane looks up the page of the row it loads
// (a division and two cross-lane reads per load address).  The paper leaves the number of
// tokens per page open (Sec. 4.1 footnote); this build serves it, without the scalar addressing
// that makes the other two fast.
// fp32 K/V takes the same road with v_mfma_f32_16x16x4_f32 (A row n / B column n, k = j; result as
// above): lane (n, j) holds the four floats d = 16c + 4j + e of token n from each 16-byte load, and
// since the order inside the contraction is free, product (c, e) pairs them with the same four
// floats of the query rows.  For the values, product s of a block contracts over tokens 4j + s:
// the probability is register s of the lane's score result, and V[4j + s][16 blk + n] is one float
// per lane, read from the row-major LDS copy with an ordinary 4-byte read.
template <typename E_, int D_, int G_, int MODE_>
struct MatEngine {
  using E = E_;
  static constexpr bool F32K = E::kBytes == 4;
  static constexpr int D = D_;
  static_assert(G_ >= 0 && G_ <= 16, "heads are padded to 16");
  static constexpr int T = 16;                 // tokens per block; a page holds 1/2, 1, 2, 4 or 8 blocks
  static constexpr int ROW = D * E::kBytes;    // bytes per token row
  static constexpr int KCH = ROW / 64;         // k-steps of the score product == 1 KiB loads per page
  // A tile is one 16-token block for rows of 256 bytes and more (4 + 4 KiB of K and V, 8 + 8 for
  // 512-byte rows, 16 + 16 for the 1 KiB rows of 256-element fp32 heads) and four blocks for
  // 128-byte rows (8 + 8 KiB).  Measured: two blocks per tile are 1.2-3 % slower
  // over whole steps for 256-byte rows and 2.3 % for 512-byte rows -- the fewer bytes a wavefront
  // keeps in flight, the better -- while for 128-byte rows, where a block is only 2 + 2 KiB and the
  // per-tile softmax weighs more, one or two blocks per tile are 14 % and 3 % slower than four.
  static constexpr int PPT = KCH >= 4 ? 1 : 4;         // blocks per tile
  static constexpr int NLD = PPT * KCH;        // 16-byte loads per lane and tile, K and V alike
  static constexpr int LPT = ROW / 16;         // V loads: lanes per token row
  static constexpr int TPL = kWave / LPT;      // V loads: token rows per load
  static constexpr int NBLK = D / 16;          // 16-wide blocks of the output row
  // LDS row pitch: bf16, transposing 8-byte reads of 4 consecutive rows -> 8 banks further per
  // row; fp32, 4-byte reads of rows 4 apart -> 16 banks further per 4 rows
  static constexpr int LROW = ROW + (F32K ? 16 : 32);
  static constexpr int kTileLog2 = PPT == 1 ? 4 : PPT == 2 ? 5 : 6;
  static constexpr int kLdsFloats = PPT * T * LROW / 4;
  static constexpr int kG = G_;
  // LDS left for finished records when four blocks share a compute unit's 160 KiB: 38 KiB (two
  // are left to the allocation granularity) less the front end's two arrays of 4 KiB, this
  // engine's V tile and 256 bytes of bookkeeping
  static constexpr int kRecFloats = (38 * 1024 - 2 * 4 * kMaxBatch - 4 * kLdsFloats - 256) / 4;
  static_assert(kRecFloats > 0, "LDS budget");
  static_assert(KCH == 2 || KCH == 4 || KCH == 8 || KCH == 16, "row size");

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
                             int n_tiles, int append_tile, int64_t slot, float* rec, PageIds& ids, float* lds) {
    // A 16-token block is the unit of both products.  Pages of 16, 32, 64 or 128 tokens hold 1, 2,
    // 4 or 8 blocks: block q (counted from the first visible page) lies in page q >> sh at row
    // (q & sub_mask) * 16.  An 8-token page is half a block: a block takes its rows 0..7 from one
    // page and its rows 8..15 from the next.
    constexpr bool t8 = MODE_ == 1;
    constexpr bool gen = MODE_ == 2;
    const int G = G_ ? G_ : p.group;                           // query heads per KV head, at most 16
    const int sh = (t8 || gen) ? 0 : p.t_log2 - 4;
    const int sub_mask = (1 << sh) - 1;
    const int Tp = p.tokens_per_page;                          // (used by the any-size mode only)
    int lo_tok, p_lo, p_hi;
    visible_pages(L, p.window, p.t_log2, &lo_tok, &p_lo, &p_hi);
    const int blk0 = tile0 * PPT;                              // first block of the chunk
    const int tot_blk = gen ? ((p_hi - p_lo) * Tp + T - 1) / T : t8 ? (p_hi - p_lo + 1) >> 1 : (p_hi - p_lo) << sh;
    const int n_blk = min(n_tiles * PPT, tot_blk - blk0);
    const int page0 = p_lo + (gen ? blk0 * T / Tp : t8 ? 2 * blk0 : blk0 >> sh);
    const int off0 = (t8 || gen) ? 0 : blk0 & sub_mask;        // place of the first block inside page0
    const int off_tok = gen ? blk0 * T - (page0 - p_lo) * Tp : 0;   // any size: token of page0 the chunk starts at
    const int n_pages = gen ? min((off_tok + n_blk * T + Tp - 1) / Tp, p_hi - page0)
                        : t8 ? min(2 * n_blk, p_hi - page0) : (off0 + n_blk + sub_mask) >> sh;
    const int tok0 = first_token_of(p.t_log2, p_lo) + blk0 * T;
    char* v_lds = reinterpret_cast<char*>(lds);

    ids.init(p.block_table + int64_t(b) * p.bt_stride + page0, n_pages, lane, p.max_page_id);

    const int n = lane & 15, j = lane >> 4;
    const int v_row = lane / LPT;                                        // V loads: row v_row + TPL * c of the page
    const char* kv_base = p.layer_base + int64_t(kvh) * p.head_stride;   // wave-uniform
    const unsigned k_loff = (t8 ? n & 7 : n) * ROW + j * 16;             // A operand of the score product: row n of the block
    const unsigned v_loff = p.v_offset + (gen ? 0 : v_row * ROW) + (lane % LPT) * 16;
    const unsigned lds_wr = v_row * LROW + (lane % LPT) * 16;            // this lane's V bytes (+ row offset)
    const unsigned lds_rd = (4 * j + (n >> 2)) * LROW + (n & 3) * 8;     // transposed read (+ page, + block)

    // B operand of the score product: head n (zero rows for the padding heads)
    u32x4 qb[KCH];
#pragma unroll
    for (int c = 0; c < KCH; ++c) {
      qb[c] = u32x4{0, 0, 0, 0};
      if (n < G)
        qb[c] = *reinterpret_cast<const u32x4*>(static_cast<const char*>(p.q) +
                                               (int64_t(b) * p.n_q_heads + kvh * G + n) * ROW + j * 16 + c * 64);
    }

    float m = kNegBig, l = 0.f;        // of head n; l is this lane's share (its tokens only)
    f32x4 acc[NBLK];
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) acc[blk] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Address (wave-uniform) of row 8h of block r of the chunk in this KV head's K rows; the V
    // rows lie p.v_offset further.  With an odd number of 8-token pages the last block has no
    // second page: its rows 8..15 are read from the first one again and masked like any token >= L.
    auto half_base = [&](int r, int h) -> const char* {
      if (t8) return kv_base + int64_t(ids.get(min(2 * r + h, n_pages - 1))) * p.small_bytes;
      const int q = off0 + r;
      return kv_base + int64_t(ids.get(q >> sh)) * p.small_bytes + ((q & sub_mask) * T + 8 * h) * ROW;
    };
    // Pages of any size: address of the row of chunk-relative token t (a different one in every
    // lane) in this KV head's K rows.  Tokens past the last page (the tail of the last block, masked
    // like any token >= L) read the last page.
    auto row_of_token = [&](int t) -> const char* {
      const int tt = off_tok + t;
      const int pg = tt / Tp;
      return kv_base + int64_t(ids.get_lane(min(pg, n_pages - 1))) * p.small_bytes + (tt - pg * Tp) * ROW;
    };
    auto load_k = [&](int tile, u32x4* buf) {
#pragma unroll
      for (int pp = 0; pp < PPT; ++pp) {
        const int r = tile * PPT + pp;
        if (PPT == 1 || r < n_blk) {
          const char* src;
          if constexpr (gen) src = row_of_token(r * T + n) + j * 16;
          else src = half_base(r, 0) + k_loff;                           // wave-uniform base + lane offset
          if constexpr (t8) {
            const char* hi = half_base(r, 1);                            // taken by all lanes: it reads a lane
            if (n & 8) src = hi + k_loff;
          }
#pragma unroll
          for (int c = 0; c < KCH; ++c)
            buf[pp * KCH + c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + c * 64));
        } else {
#pragma unroll
          for (int c = 0; c < KCH; ++c) buf[pp * KCH + c] = u32x4{0, 0, 0, 0};
        }
      }
    };
    auto load_v = [&](int tile, u32x4* buf) {
#pragma unroll
      for (int pp = 0; pp < PPT; ++pp) {
        const int r = tile * PPT + pp;
        if (PPT == 1 || r < n_blk) {
          if constexpr (gen) {
#pragma unroll
            for (int c = 0; c < KCH; ++c)                    // load c covers rows TPL * c .. TPL * c + TPL - 1
              buf[pp * KCH + c] = __builtin_nontemporal_load(
                  reinterpret_cast<const u32x4*>(row_of_token(r * T + TPL * c + v_row) + v_loff));
          } else {
            const char* lo = half_base(r, 0);
            const char* hi = t8 ? half_base(r, 1) : lo + 8 * ROW;
#pragma unroll
            for (int c = 0; c < KCH; ++c) {                  // load c covers rows TPL * c .. TPL * c + TPL - 1
              const char* src = (((TPL * c) & 8) ? hi : lo) + ((TPL * c) & 7) * ROW;     // wave-uniform
              buf[pp * KCH + c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + v_loff));
            }
          }
        } else {
#pragma unroll
          for (int c = 0; c < KCH; ++c) buf[pp * KCH + c] = u32x4{0, 0, 0, 0};
        }
      }
    };
    // the K stream tells the page-id registers when it enters a new page
    auto k_entered = [&](int tile) {
      if (gen) {
        ids.k_stream_in((off_tok + tile * PPT * T) / Tp);
      } else if (t8) {
        ids.k_stream_at(2 * tile * PPT);
      } else {
        const int q = off0 + tile * PPT;
        if ((q & sub_mask) == 0) ids.k_stream_at(q >> sh);
      }
    };

    // One tile ahead, one register set each: a step first moves V(t) to LDS and issues the score
    // products of K(t), which frees both sets, then requests K(t+1) and V(t+1) -- adjacent in
    // memory -- back to back, with the rest of the step to arrive in.  Deeper pipelines measured
    // slower: K two tiles ahead in a second register set by 1.5 % over whole steps (3 % on
    // launches of 0.1-0.3 GB), a second V set by 0.3-0.5 %.  One wavefront per SIMD with 8-16 KiB in
    // flight already covers the memory latency; more outstanding requests only lengthen the queues.
    u32x4 kb[NLD], vb[NLD];
    load_k(0, kb);
    load_v(0, vb);

    // Fused append: the new token's rows and its page's table entry are requested now, so that the
    // tile that takes them in (often the last of the segment) does not wait for them.
    u32x4 k_app[KCH], v_app = u32x4{0, 0, 0, 0};
    int raw_new = -1;
    const int rel = (L - 1) - first_token_of(p.t_log2, p_lo);    // the new token, counted from the first visible page
    const int r_new = (rel >> 4) - blk0;                         // its block, relative to the chunk
    const int row_new = rel & 15;                                // its row in the block
    const int page_new = gen ? (off_tok + r_new * T + row_new) / Tp : t8 ? 2 * r_new + (row_new >> 3) : (off0 + r_new) >> sh;
#pragma unroll
    for (int c = 0; c < KCH; ++c) k_app[c] = u32x4{0, 0, 0, 0};
    if (append_tile >= 0) {
      const char* kn = static_cast<const char*>(p.k_new) + (int64_t(b) * p.n_kv_heads + kvh) * ROW;
      const char* vn = static_cast<const char*>(p.v_new) + (int64_t(b) * p.n_kv_heads + kvh) * ROW;
#pragma unroll
      for (int c = 0; c < KCH; ++c) k_app[c] = *reinterpret_cast<const u32x4*>(kn + j * 16 + c * 64);
      v_app = *reinterpret_cast<const u32x4*>(vn + (lane % LPT) * 16);
      raw_new = ids.row[page_new];
    }

    auto step = [&](int tile, u32x4* kbuf, u32x4* vbuf) {

      // fused append: the rows of the token at L - 1 come from k_new / v_new (they are stored into
      // the page after the loop)
      if (tile == append_tile) {
        const int pp_new = r_new - tile * PPT;
        if (n == row_new) {
#pragma unroll
          for (int c = 0; c < KCH; ++c)
#pragma unroll
            for (int pp = 0; pp < PPT; ++pp)
              if (pp == pp_new) kbuf[pp * KCH + c] = k_app[c];
        }
#pragma unroll
        for (int i = 0; i < NLD; ++i)
          if ((i / KCH) * T + (i % KCH) * TPL + v_row == pp_new * T + row_new) vbuf[i] = v_app;
      }

      const int tile_tok = tok0 + tile * PPT * T;
      const bool clean = tile_tok >= lo_tok && tile_tok + PPT * T <= L;
      if (!clean) {
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

      // scores: lane (n, j) gets head n, tokens 4j .. 4j+3 of each page
      f32x4 s[PPT];
#pragma unroll
      for (int pp = 0; pp < PPT; ++pp) {
        s[pp] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < KCH; ++c) {
          if constexpr (F32K) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              s[pp] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(kbuf[pp * KCH + c][e]),
                                                           __uint_as_float(qb[c][e]), s[pp], 0, 0, 0);
          } else {
            s[pp] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kbuf[pp * KCH + c]),
                                                            __builtin_bit_cast(bf16x8, qb[c]), s[pp], 0, 0, 0);
          }
        }
      }

      if (tile + 1 < n_tiles) {
        load_k(tile + 1, kbuf);
        load_v(tile + 1, vbuf);                            // the registers are free again
        k_entered(tile + 1);
      }

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
      }

      // online softmax of head n
      float mx = s[0][0];
#pragma unroll
      for (int pp = 0; pp < PPT; ++pp)
#pragma unroll
        for (int i = 0; i < 4; ++i) mx = fmaxf(mx, s[pp][i]);
      const float m_new = fmaxf(m, across_groups_max(mx));
      const float alpha = __builtin_amdgcn_exp2f(m - m_new);
      bf16x4 prob_hi[PPT], prob_lo[PPT];
      float prob[PPT][4];
      float sum = 0.f;
#pragma unroll
      for (int pp = 0; pp < PPT; ++pp)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float e = __builtin_amdgcn_exp2f(s[pp][i] - m_new);
          if (!clean) e = (s[pp][i] == kNegBig) ? 0.f : e;
          if constexpr (F32K) {
            prob[pp][i] = e;
          } else {
            const __bf16 hi = static_cast<__bf16>(e);
            prob_hi[pp][i] = hi;
            prob_lo[pp][i] = static_cast<__bf16>(e - static_cast<float>(hi));
          }
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
          if constexpr (F32K) {
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
              const float vt = *reinterpret_cast<const float*>(v_lds + (pp * T + 4 * j + s4) * LROW + (16 * blk + n) * 4);
              acc[blk] = __builtin_amdgcn_mfma_f32_16x16x4f32(prob[pp][s4], vt, acc[blk], 0, 0, 0);
            }
          } else {
            const s16x4 v4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (lds_s16x4_ptr)(v_lds + pp * T * LROW + lds_rd + blk * 32));
            const bf16x4 vt = __builtin_bit_cast(bf16x4, v4);
            acc[blk] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(prob_hi[pp], vt, acc[blk], 0, 0, 0);
            acc[blk] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(prob_lo[pp], vt, acc[blk], 0, 0, 0);
          }
        }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    };

    for (int tile = 0; tile < n_tiles; ++tile) step(tile, kb, vb);

    // The new token's rows go into their page only now.  Loads and stores share one in-order
    // counter and the waits are fixed at compile time for the path without stores, so a store
    // issued inside the step is waited for by the step's own loads: 1.7 us per segment, measured.
    // (The tile of the new token is the last of its segment, so the page-id registers still hold
    // its page.)
    if (append_tile >= 0 && raw_new >= 0 && raw_new <= p.max_page_id) {
      char* dst;
      if constexpr (gen)
        dst = const_cast<char*>(kv_base) + int64_t(ids.get(page_new)) * p.small_bytes +
              (off_tok + r_new * T + row_new - page_new * Tp) * ROW;
      else
        dst = const_cast<char*>(half_base(r_new, row_new >> 3)) + (row_new & 7) * ROW;
      if (n == row_new) {
#pragma unroll
        for (int c = 0; c < KCH; ++c) *reinterpret_cast<u32x4*>(dst + j * 16 + c * 64) = k_app[c];
      }
      if (v_row == (row_new & (TPL - 1))) *reinterpret_cast<u32x4*>(dst + p.v_offset + (lane % LPT) * 16) = v_app;
    }

    l = across_groups_sum(l);
    // one partial record: lane (n, j) holds element 16 * blk + n of heads 4j .. 4j+3.  It goes to
    // the LDS buffer `rec` ([G][D] accumulators, then G (max, sum) pairs; the front end stores the
    // buffered records when the wavefront is done), or straight to workspace slot `slot` when
    // the record is too large to be buffered.
    if (rec != nullptr) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int h = 4 * j + i;
        if (h < G) {
          float* dst = rec + h * D + n;
#pragma unroll
          for (int blk = 0; blk < NBLK; ++blk) dst[blk * 16] = acc[blk][i];
        }
      }
      if (j == 0 && n < G) *reinterpret_cast<float2*>(rec + G * D + 2 * n) = make_float2(m, l);
    } else {
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
  }
};

}  // namespace
