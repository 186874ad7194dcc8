// Decode engine for 16-token pages on the vector ALUs (see kernels.hip for the front end).
#pragma once

#include "decode_common.hpp"

namespace {

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

    // Software pipeline, one tile deep: V(t+1) is requested when tile t starts (into the second V
    // set), K(t+1) as soon as the scores of tile t have freed the K registers; 8 to 16 KiB are in
    // flight per wavefront.  (K two tiles ahead in a second register set measured the same on
    // 512-byte rows with 2 query heads per KV head and needs 32 more registers.)
    u32x4 kb[NLD], vb[2][NLD];
    load_pages(0, k_voff, 64, kb);
    load_pages(0, v_voff, 1024, vb[0]);

    auto step = [&](int tile, u32x4* kbuf, u32x4* vbuf, u32x4* v_next) {
      if (tile + 1 < n_tiles) load_pages(tile + 1, v_voff, 1024, v_next);

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

      if (tile + 1 < n_tiles) {
        load_pages(tile + 1, k_voff, 64, kbuf);
        ids.k_stream_at((tile + 1) * PPT);
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

    for (int tile = 0; tile < n_tiles; tile += 2) {
      step(tile, kb, vb[0], vb[1]);
      if (tile + 1 < n_tiles) step(tile + 1, kb, vb[1], vb[0]);
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

}  // namespace
