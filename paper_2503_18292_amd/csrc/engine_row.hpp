// General decode engine: any page size, rows spread over lanes (see kernels.hip for the front end).
#pragma once

#include "decode_common.hpp"

namespace {

// ---- engine for any page size: rows spread over lanes -----------------------------------
//
// K and V are read alike: a token's row is LPT lanes x 16 bytes, one wave-wide load covers
// TPL = 64 / LPT consecutive tokens (1 KiB, contiguous in the page).  Every partial dot
// product is summed over LPT lanes, so this engine spends several times more vector-ALU
// work per byte than the other two; it covers what they are not built for (fp32 K/V in pages
// other than 16 tokens, with 8 query heads per KV head, or with 1 KiB rows).  Each group of
// LPT lanes runs its own online softmax over the tokens it sees; the groups are merged once at
// the end.
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

}  // namespace
