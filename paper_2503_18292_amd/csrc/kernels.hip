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
// and (3) that the arithmetic stays out of the way of the loads: both products of a 16-token
// block are small dense contractions and go through MFMA (bf16 and fp32 K/V alike, any page
// size, 1 to 16 query heads per KV head), which leaves the vector ALUs almost idle and keeps
// even 16 heads per KV head at the HBM rate.
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

#include "pool_internal.hpp"
#include "decode_common.hpp"
#include "engine_mat.hpp"

namespace {

// Finished records wait in LDS and leave together when the wavefront is done (or the buffer is
// full): a store issued between two segments sits in the same in-order queue as the next
// segment's loads, whose first wait then also waits for the store's acknowledgement, and record
// traffic interleaved with the read stream costs HBM efficiency -- measured on batch 1024 with
// 100-600 tokens (nine records per wavefront): 15 % of the kernel's time.
constexpr int kMaxBufferedRecords = 16;

// Copies `count` buffered records (and the chunk spans of the segments that start in them) from
// LDS to the workspace.  Record r: G * D accumulator floats, then G (max, sum) pairs.
// A record that covers its whole segment (s_last < 0) is the segment's result but for the
// division: when the caller's output array is known it goes there directly, normalised exactly as
// the reduction would (a one-record merge multiplies by 1 and divides by the sum), and the
// segment's span is left empty, which tells the reduction to skip it.  With many short requests
// that is nearly every segment, and the reduction launch has next to nothing to do.
template <int D>
__device__ __forceinline__ void flush_records(const DecodeParams& p, const float* s_rec, const int* s_slot,
                                              const int* s_seg, const int* s_last, int count, int G,
                                              int rec_stride, int lane) {
  __syncthreads();                                  // the engine's LDS writes (one wavefront per block)
  for (int r = 0; r < count; ++r) {
    const float4* src = reinterpret_cast<const float4*>(s_rec + r * rec_stride);
    const float2* ml = reinterpret_cast<const float2*>(s_rec + r * rec_stride + G * D);
    if (s_last[r] < 0) {
      float4* dst = reinterpret_cast<float4*>(p.out + int64_t(s_seg[r]) * G * D);   // heads kvh*G .. of request b
      for (int i = lane; i < G * D / 4; i += kWave) {
        const float l = ml[i / (D / 4)].y;
        const float inv = l > 0.f ? 1.0f / l : 0.f;
        const float4 a = src[i];
        dst[i] = make_float4(a.x * inv, a.y * inv, a.z * inv, a.w * inv);
      }
      if (lane == 0) *reinterpret_cast<int2*>(p.ws_meta + int64_t(s_seg[r]) * 2) = make_int2(1, 0);
      continue;
    }
    const int64_t slot = s_slot[r];
    float4* dst = reinterpret_cast<float4*>(p.ws_acc + slot * G * D);
    for (int i = lane; i < G * D / 4; i += kWave) dst[i] = src[i];
    if (lane < G) reinterpret_cast<float2*>(p.ws_ml + slot * G * 2)[lane] = ml[lane];
    if (lane == 0 && s_seg[r] >= 0)
      *reinterpret_cast<int2*>(p.ws_meta + int64_t(s_seg[r]) * 2) = make_int2(int(blockIdx.x), s_last[r]);
  }
  __syncthreads();                                  // the buffer may be written again
}

// Batches above kMaxBatch: the prefix sums every decode block needs (see scan_requests) are made
// once, by one block, and read from the workspace.  Thread t takes the K consecutive requests
// t*K .. t*K + K - 1.
__global__ __launch_bounds__(1024) void scan_lengths_kernel(const int32_t* __restrict__ seq_lens, int batch,
                                                            int max_seq_len, int window, int t_log2,
                                                            int tile_log2, int n_kv_heads,
                                                            int32_t* __restrict__ incl, int32_t* __restrict__ lens) {
  __shared__ int s_wave[16];
  const int t = threadIdx.x;
  const int K = (batch + 1023) / 1024;
  const int first = t * K, last = min(first + K, batch);
  int total = 0;
  for (int i = first; i < last; ++i) {
    const int raw = seq_lens[i];
    const int Li = min(raw, max_seq_len);
    lens[i] = raw > max_seq_len ? -Li : Li;
    total += units_of(Li, window, t_log2, tile_log2) * n_kv_heads;
  }
  int scan = total;                                   // inclusive over the wavefront, then over the 16 wavefronts
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int up = __shfl_up(scan, off);
    if ((t & (kWave - 1)) >= off) scan += up;
  }
  if ((t & (kWave - 1)) == kWave - 1) s_wave[t / kWave] = scan;
  __syncthreads();
  int before = scan - total;
  for (int w = 0; w < t / kWave; ++w) before += s_wave[w];
  for (int i = first; i < last; ++i) {
    const int Li = abs(lens[i]);
    before += units_of(Li, window, t_log2, tile_log2) * n_kv_heads;
    incl[i] = before;
  }
}

// One wavefront per partition of the flat tile space (see the head of the file).
// BIG: the batch exceeds kMaxBatch and the prefix sums come from scan_lengths_kernel.
template <class Eng, bool BIG>
__global__ __launch_bounds__(kWave) void decode_partial_kernel(const DecodeParams p) {
  __shared__ int s_incl[BIG ? 1 : kMaxBatch];
  __shared__ int s_len[BIG ? 1 : kMaxBatch];
  __shared__ float s_eng[Eng::kLdsFloats > 0 ? Eng::kLdsFloats : 1];
  __shared__ __align__(16) float s_rec[Eng::kRecFloats];
  __shared__ int s_rslot[kMaxBufferedRecords], s_rseg[kMaxBufferedRecords], s_rlast[kMaxBufferedRecords];
  const int lane = threadIdx.x;
  const int* incl;
  const int* lens;
  int W;
  if constexpr (BIG) {
    incl = p.ws_incl;
    lens = p.ws_len;
    W = incl[p.batch - 1];
  } else {
    W = scan_requests(p.seq_lens, p.batch, p.max_seq_len, p.window, p.t_log2, Eng::kTileLog2,
                      p.n_kv_heads, lane, s_incl, s_len);
    incl = s_incl;
    lens = s_len;
  }
  const int C = chunk_of(p.chunk_tiles, p.min_chunk_tiles, W, gridDim.x);
  const int64_t x0 = int64_t(blockIdx.x) * C;
  if (x0 >= W) return;
  // records buffered in LDS: as many as fit (none for the largest records, which then go straight
  // to the workspace); a record is padded to a multiple of 16 bytes
  const int G = Eng::kG ? Eng::kG : p.group;
  const int rec_stride = G * Eng::D + ((2 * G + 3) & ~3);
  const int rec_cap = min(kMaxBufferedRecords, Eng::kRecFloats / rec_stride);
  int n_rec = 0;
  PageIds ids;
  ids.row = nullptr;
  ids.n_loaded = 0;
  int x = int(x0);
  const int x1 = int(min<int64_t>(W, x0 + C));
  int b = BIG ? find_request_global(incl, p.batch, x, lane) : find_request(incl, p.batch, x, lane);
  // The segments of a chunk follow one another: after the first one, (request, KV head) moves on
  // by one head, or to the next request that has tokens.  Only the first needs a division.
  int L_enc = lens[b];
  int units_b = units_of(abs(L_enc), p.window, p.t_log2, Eng::kTileLog2);   // start-up units + tiles, per head
  int kvh, seg0;                                                            // seg0: flat position of the segment
  {
    const int start_b = b > 0 ? incl[b - 1] : 0;
    kvh = (x - start_b) / units_b;
    seg0 = start_b + kvh * units_b;
  }
  while (x < x1) {
    const int xe = min(x1, seg0 + units_b);
    // tiles of the segment inside [x, xe): none if the chunk ends inside the start-up units
    const int tile0 = max(x - seg0 - kSegStartUnits, 0);
    const int n_tiles = xe - seg0 - kSegStartUnits - tile0;
    if (n_tiles > 0) {
      const int seg = b * p.n_kv_heads + kvh;
      const int slot = seg + int(blockIdx.x);
      // the wavefront that holds a segment's first tile tells the reduction where its records are
      // (a segment whose tiles all lie in this chunk ends in it: no division)
      const bool whole = tile0 == 0 && n_tiles == units_b - kSegStartUnits;
      const int last_chunk = whole ? int(blockIdx.x) : (seg0 + units_b - 1) / C;
      // (the last record of a wavefront has nothing behind it to delay: it goes straight out)
      float* rec = nullptr;
      if (rec_cap > 0 && xe < x1) {
        if (n_rec == rec_cap) {
          flush_records<Eng::D>(p, s_rec, s_rslot, s_rseg, s_rlast, n_rec, G, rec_stride, lane);
          n_rec = 0;
        }
        rec = s_rec + n_rec * rec_stride;
        if (lane == 0) {
          s_rslot[n_rec] = slot;
          s_rseg[n_rec] = tile0 == 0 ? seg : -1;
          s_rlast[n_rec] = whole && p.out != nullptr ? -1 : last_chunk;
        }
        ++n_rec;
      } else if (tile0 == 0 && lane == 0) {
        *reinterpret_cast<int2*>(p.ws_meta + int64_t(seg) * 2) = make_int2(int(blockIdx.x), last_chunk);
      }
      // fused append: the chunk that holds the tile of the newest token (position L - 1) writes it
      // (not for a request whose length was clamped to max_seq_len: see scan_requests)
      const int L = abs(L_enc);
      int append_tile = -1;
      if (p.k_new != nullptr && L_enc > 0) {
        int lo_tok, p_lo, p_hi;
        visible_pages(L, p.window, p.t_log2, &lo_tok, &p_lo, &p_hi);
        const int t_pos = ((L - 1) - first_token_of(p.t_log2, p_lo)) >> Eng::kTileLog2;
        if (t_pos >= tile0 && t_pos < tile0 + n_tiles) append_tile = t_pos - tile0;
      }
      Eng::run(p, lane, b, kvh, L, tile0, n_tiles, append_tile, slot, rec, ids, s_eng);
    }
    x = xe;
    if (x < x1) {                                   // the segment ended inside the chunk
      seg0 = x;
      if (++kvh == p.n_kv_heads) {
        kvh = 0;
        do ++b; while (b < p.batch - 1 && incl[b] <= x);          // requests without tokens take no units
        L_enc = lens[b];
        units_b = units_of(abs(L_enc), p.window, p.t_log2, Eng::kTileLog2);
      }
    }
  }
  if (n_rec > 0) flush_records<Eng::D>(p, s_rec, s_rslot, s_rseg, s_rlast, n_rec, G, rec_stride, lane);
}

// One block (one wavefront) per (request, query head): merges the records of its segment,
//   m* = max m_i,  out = sum_i acc_i 2^(m_i - m*) / sum_i l_i 2^(m_i - m*).
// D/4 lanes cover an output row (4 elements each), so the wavefront holds 256/D lane groups;
// group i takes every (256/D)-th record, eight records are in flight per step over all groups
// (all loads issued before any is used), and the groups are merged at the end.  Where the
// records are comes from the (first chunk, last chunk) pair the partial kernel left per segment.
// NW wavefronts per block share a segment's records the same way when a few long segments have
// many records each (a single request of 100 k tokens has 128 per KV head), and meet in LDS.
template <int D, int NW>
__global__ __launch_bounds__(kWave * NW) void splitk_reduce_kernel(
    const float* __restrict__ ws_acc, const float* __restrict__ ws_ml, const int32_t* __restrict__ ws_meta,
    const int32_t* __restrict__ seq_lens, int32_t max_seq_len, int32_t n_kv_heads, int32_t n_q_heads,
    float* __restrict__ out) {
  constexpr int LPR = D / 4;              // lanes per output row
  constexpr int NG = kWave / LPR;         // lane groups: 4, 2 or 1
  constexpr int R = 8 / NG;               // records per group and step
  const int hq = blockIdx.x;
  const int b = blockIdx.y;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int gi = lane / LPR, li = lane % LPR;
  const int G = n_q_heads / n_kv_heads;
  const int kvh = hq / G;
  const int g = hq - kvh * G;
  float4* dst = reinterpret_cast<float4*>(out + (int64_t(b) * n_q_heads + hq) * D) + li;
  if (min(seq_lens[b], max_seq_len) <= 0) {   // no visible token, no record (the whole block leaves)
    if (gi == 0 && wave == 0) *dst = make_float4(0.f, 0.f, 0.f, 0.f);
    return;
  }
  const int64_t seg = int64_t(b) * n_kv_heads + kvh;
  const int2 span = *reinterpret_cast<const int2*>(ws_meta + seg * 2);
  const int c_lo = span.x, c_hi = span.y;
  if (c_lo > c_hi) return;                // the partial kernel has written this segment's result itself
  float m_star = kNegBig, l_star = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int c0 = c_lo + wave * (R * NG); c0 <= c_hi; c0 += R * NG * NW) {
    float2 ml[R];
    float4 a[R];
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const int64_t rec = (seg + min(c0 + i * NG + gi, c_hi)) * G + g;
      ml[i] = *reinterpret_cast<const float2*>(ws_ml + rec * 2);
      a[i] = *(reinterpret_cast<const float4*>(ws_acc + rec * D) + li);
    }
    float m_new = m_star;
#pragma unroll
    for (int i = 0; i < R; ++i)
      if (c0 + i * NG + gi <= c_hi) m_new = fmaxf(m_new, ml[i].x);
    const float keep = __builtin_amdgcn_exp2f(m_star - m_new);
    l_star *= keep;
    acc.x *= keep; acc.y *= keep; acc.z *= keep; acc.w *= keep;
#pragma unroll
    for (int i = 0; i < R; ++i) {
      if (c0 + i * NG + gi > c_hi) continue;
      const float w = __builtin_amdgcn_exp2f(ml[i].x - m_new);
      l_star = fmaf(ml[i].y, w, l_star);
      acc.x = fmaf(a[i].x, w, acc.x); acc.y = fmaf(a[i].y, w, acc.y);
      acc.z = fmaf(a[i].z, w, acc.z); acc.w = fmaf(a[i].w, w, acc.w);
    }
    m_star = m_new;
  }
  // merge the lane groups (a group that saw no record still has m = -big, l = 0, acc = 0)
#pragma unroll
  for (int off = LPR; off < kWave; off <<= 1) {
    const float m_o = __shfl_xor(m_star, off);
    const float l_o = __shfl_xor(l_star, off);
    const float m_new = fmaxf(m_star, m_o);
    const float wa = __builtin_amdgcn_exp2f(m_star - m_new);
    const float wb = __builtin_amdgcn_exp2f(m_o - m_new);
    l_star = l_star * wa + l_o * wb;
    acc.x = acc.x * wa + __shfl_xor(acc.x, off) * wb;
    acc.y = acc.y * wa + __shfl_xor(acc.y, off) * wb;
    acc.z = acc.z * wa + __shfl_xor(acc.z, off) * wb;
    acc.w = acc.w * wa + __shfl_xor(acc.w, off) * wb;
    m_star = m_new;
  }
  if constexpr (NW > 1) {
    __shared__ float4 s_acc[NW][LPR];
    __shared__ float2 s_ml[NW];
    if (gi == 0) {
      s_acc[wave][li] = acc;
      if (li == 0) s_ml[wave] = make_float2(m_star, l_star);
    }
    __syncthreads();
    if (wave != 0) return;
    m_star = kNegBig;
#pragma unroll
    for (int w = 0; w < NW; ++w) m_star = fmaxf(m_star, s_ml[w].x);
    l_star = 0.f;
    acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float f = __builtin_amdgcn_exp2f(s_ml[w].x - m_star);
      const float4 a = s_acc[w][li];
      l_star = fmaf(s_ml[w].y, f, l_star);
      acc.x = fmaf(a.x, f, acc.x); acc.y = fmaf(a.y, f, acc.y);
      acc.z = fmaf(a.z, f, acc.z); acc.w = fmaf(a.w, f, acc.w);
    }
  }
  const float inv = l_star > 0.f ? 1.0f / l_star : 0.f;
  if (gi == 0) *dst = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
}

// One thread per 16 bytes of the new K and V rows.
__global__ __launch_bounds__(256) void kv_append_kernel(
    char* __restrict__ layer_base, int64_t small_bytes, int32_t head_stride, int32_t v_offset,
    int32_t t_log2, int32_t n_kv_heads, int32_t row_bytes, const char* __restrict__ k_new,
    const char* __restrict__ v_new, const int32_t* __restrict__ block_table, int32_t bt_stride,
    const int32_t* __restrict__ seq_lens, int32_t batch, int32_t max_len, int32_t max_page_id) {
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
  if (L <= 0 || L > max_len) return;
  const int pos = L - 1;
  const int page = page_of_token(t_log2, pos);
  if (page >= bt_stride) return;
  const int sid = block_table[int64_t(b) * bt_stride + page];
  if (sid < 0 || sid > max_page_id) return;
  const char* src = (is_v ? v_new : k_new) + (int64_t(b) * n_kv_heads + h) * row_bytes + c * 16;
  char* dst = layer_base + int64_t(sid) * small_bytes + int64_t(h) * head_stride +
              (is_v ? v_offset : 0) + (pos - first_token_of(t_log2, page)) * row_bytes + c * 16;
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
  if (pos < 0) return;
  const int page = page_of_token(t_log2, pos);
  if (page >= bt_stride) return;
  const int sid = block_table[int64_t(b) * bt_stride + page];
  if (sid < 0 || sid > max_page_id) return;       // page not resident (e.g. already slid out)
  const int chunks = row_bytes / 16;              // 16-byte pieces per (head, K or V) row
  char* page_base = layer_base + int64_t(sid) * small_bytes + (pos - first_token_of(t_log2, page)) * row_bytes;
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

// A read stream shaped like the decode kernel's: one wavefront per block, 16 KiB (16 loads of
// 16 bytes per lane) per step, the next step's loads issued before this step's are used.  Its
// rate is what the memory system gives a kernel that does nothing but read.
__global__ __launch_bounds__(kWave) void stream_read_kernel(const u32x4* __restrict__ src, int64_t n,
                                                            unsigned* __restrict__ sink) {
  constexpr int kLoads = 16;
  constexpr int64_t kChunk = int64_t(kLoads) * kWave;          // 16-byte units per step
  const int lane = threadIdx.x;
  const int64_t n_chunks = n / kChunk;
  unsigned x = 0;
  u32x4 v[2][kLoads];
  auto issue = [&](int64_t c, u32x4* buf) {
    const u32x4* p = src + c * kChunk + lane;
#pragma unroll
    for (int u = 0; u < kLoads; ++u) buf[u] = __builtin_nontemporal_load(p + u * kWave);
  };
  auto use = [&](const u32x4* buf) {
#pragma unroll
    for (int u = 0; u < kLoads; ++u) x ^= buf[u].x ^ buf[u].y ^ buf[u].z ^ buf[u].w;
  };
  int64_t c = blockIdx.x;
  if (c < n_chunks) issue(c, v[0]);
  while (c < n_chunks) {
    const int64_t c1 = c + gridDim.x;
    if (c1 < n_chunks) issue(c1, v[1]);
    use(v[0]);
    if (c1 >= n_chunks) break;
    const int64_t c2 = c1 + gridDim.x;
    if (c2 < n_chunks) issue(c2, v[0]);
    use(v[1]);
    c = c2;
  }
  if (blockIdx.x == 0)                                         // what does not fill a whole step
    for (int64_t i = n_chunks * kChunk + lane; i < n; i += kWave) {
      const u32x4 t = __builtin_nontemporal_load(src + i);
      x ^= t.x ^ t.y ^ t.z ^ t.w;
    }
  if (x == 0x9e3779b9u) *sink = x;     // practically never taken; keeps the loads alive
}

// The same merge for launches with many short segments (one to three records each): a wavefront
// serves 256 / D query heads, one per lane group, each group walking its own segment's records.
template <int D>
__global__ __launch_bounds__(kWave) void splitk_reduce_packed_kernel(
    const float* __restrict__ ws_acc, const float* __restrict__ ws_ml, const int32_t* __restrict__ ws_meta,
    const int32_t* __restrict__ seq_lens, int32_t max_seq_len, int32_t n_kv_heads, int32_t n_q_heads,
    float* __restrict__ out) {
  constexpr int LPR = D / 4;              // lanes per output row
  constexpr int NG = kWave / LPR;         // query heads per wavefront
  const int lane = threadIdx.x;
  const int gi = lane / LPR, li = lane % LPR;
  const int hq = blockIdx.x * NG + gi;
  const int b = blockIdx.y;
  if (hq >= n_q_heads) return;
  const int G = n_q_heads / n_kv_heads;
  const int kvh = hq / G;
  const int g = hq - kvh * G;
  float4* dst = reinterpret_cast<float4*>(out + (int64_t(b) * n_q_heads + hq) * D) + li;
  if (min(seq_lens[b], max_seq_len) <= 0) {
    *dst = make_float4(0.f, 0.f, 0.f, 0.f);
    return;
  }
  const int64_t seg = int64_t(b) * n_kv_heads + kvh;
  const int2 span = *reinterpret_cast<const int2*>(ws_meta + seg * 2);
  if (span.x > span.y) return;            // the partial kernel has written this segment's result itself
  float m_star = kNegBig, l_star = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int c0 = span.x; c0 <= span.y; c0 += 2) {
    float2 ml[2];
    float4 a[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int64_t rec = (seg + min(c0 + i, span.y)) * G + g;
      ml[i] = *reinterpret_cast<const float2*>(ws_ml + rec * 2);
      a[i] = *(reinterpret_cast<const float4*>(ws_acc + rec * D) + li);
    }
    float m_new = fmaxf(m_star, ml[0].x);
    if (c0 + 1 <= span.y) m_new = fmaxf(m_new, ml[1].x);
    const float keep = __builtin_amdgcn_exp2f(m_star - m_new);
    l_star *= keep;
    acc.x *= keep; acc.y *= keep; acc.z *= keep; acc.w *= keep;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      if (c0 + i > span.y) continue;
      const float w = __builtin_amdgcn_exp2f(ml[i].x - m_new);
      l_star = fmaf(ml[i].y, w, l_star);
      acc.x = fmaf(a[i].x, w, acc.x); acc.y = fmaf(a[i].y, w, acc.y);
      acc.z = fmaf(a[i].z, w, acc.z); acc.w = fmaf(a[i].w, w, acc.w);
    }
    m_star = m_new;
  }
  const float inv = l_star > 0.f ? 1.0f / l_star : 0.f;
  *dst = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
}

// ---- split-K scratch for callers that cannot allocate ------------------------------------
//
// jenga_paged_decode_static keeps the records between its two kernels here instead of in a
// caller-owned workspace.  Every device the library runs on holds its own copy of the array for
// the life of the process; host code never uses the array's name as an address (on the host it is
// only a stand-in for the symbol) but the device address hipGetSymbolAddress reports, looked up
// once per device with that device current.
constexpr int64_t kStaticScratchBytes = JENGA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, or nullptr (with *rc set) on failure.
void* static_scratch(int* rc) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    *rc = JENGA_ERR_HIP;
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
      (void)hipGetLastError();
      *rc = JENGA_ERR_HIP;
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  *rc = JENGA_OK;
  return g_scratch_ptr[dev];
}

// The address is looked up when a pool is created on the device, so that the first
// jenga_paged_decode_static call (which may run under stream capture) finds it there.
void setup_device() noexcept {
  int rc = JENGA_OK;
  (void)static_scratch(&rc);
}
const bool g_setup_hook_set = (jenga::device_setup_hook = &setup_device, true);

// ---- host side: validation, partition geometry, launch --------------------------------

using DecodeFn = void (*)(DecodeParams);

bool attention_kind(const jenga::Kind& k) {
  return k.desc.type == JENGA_FULL || k.desc.type == JENGA_WINDOW || k.desc.type == JENGA_CROSS;
}

bool aligned16(const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }

// Builds: element type x head size x page kind (8-token pages are half blocks) x head count
// (the powers of two at compile time, 0 = any other count up to 16 at run time).
// Builds: element type x head size x page mode (whole blocks, half blocks; any other page size
// in a build that takes the head count at run time) x head count (the powers of two at compile
// time, 0 = any other count up to 16 at run time) x batch range.
template <typename E, int D, int MODE>
DecodeFn pick_g(int G, bool big) {
#define JENGA_PICK(GG) (big ? decode_partial_kernel<MatEngine<E, D, GG, MODE>, true> \
                            : decode_partial_kernel<MatEngine<E, D, GG, MODE>, false>)
  if constexpr (MODE == 2) {
    return JENGA_PICK(0);
  } else {
    switch (G) {
      case 1: return JENGA_PICK(1);
      case 2: return JENGA_PICK(2);
      case 4: return JENGA_PICK(4);
      case 8: return JENGA_PICK(8);
      case 16: return JENGA_PICK(16);
      default: return JENGA_PICK(0);
    }
  }
#undef JENGA_PICK
}

template <typename E>
DecodeFn pick_d(int D, int mode, int G, bool big) {
#define JENGA_PICK_MODE(DD) (mode == 0 ? pick_g<E, DD, 0>(G, big) : mode == 1 ? pick_g<E, DD, 1>(G, big) : pick_g<E, DD, 2>(G, big))
  switch (D) {
    case 64: return JENGA_PICK_MODE(64);
    case 128: return JENGA_PICK_MODE(128);
    default: return JENGA_PICK_MODE(256);
  }
#undef JENGA_PICK_MODE
}

// Partitions of the automatic mode: resident blocks of `fn`, at most one per SIMD, a multiple
// of 8 (one share per XCD), capped at kMaxPartitions.  Remembered per kernel in a fixed table (no
// heap allocation on any call); 2048 when no device can be asked.
int resident_partitions(DecodeFn fn) noexcept {
  constexpr unsigned kSlots = 1024;                 // far more than there are decode kernels
  struct Entry { const void* fn; int n; };
  static std::mutex mu;
  static Entry table[kSlots] = {};
  const void* key = reinterpret_cast<const void*>(fn);
  std::lock_guard<std::mutex> lock(mu);
  unsigned i = unsigned((reinterpret_cast<uintptr_t>(key) >> 4) * 2654435761u) % kSlots;
  for (unsigned probes = 0; probes < kSlots && table[i].fn != nullptr; ++probes, i = (i + 1) % kSlots)
    if (table[i].fn == key) return table[i].n;
  int dev = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) == hipSuccess &&
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kWave, 0) == hipSuccess &&
      cus > 0 && per_cu > 0) {
    // one wavefront per SIMD (4 per compute unit): measured faster than filling every slot,
    // and it leaves each wavefront the registers for a deep load pipeline
    int n = std::min(kMaxPartitions, cus * std::min(per_cu, 4)) / 8 * 8;
    n = std::max(n, 8);
    if (table[i].fn == nullptr) table[i] = Entry{key, n};
    return n;
  }
  (void)hipGetLastError();      // no device: do not leave a sticky error, do not remember
  return 2048;
}

struct Geometry {
  const jenga::Kind* kind;
  int G;
  int chunk_tiles;       // 0: automatic
  int min_chunk_tiles;
  int n_part_bound;      // partitions the workspace must have room for
  int64_t slots;
  DecodeFn fn;
  int batch;
  int tile_log2;         // tokens per tile, as the engine's kTileLog2
  bool big;              // batch > kMaxBatch: prefix sums through the workspace
};

// Everything the partial kernel and the reduction must agree on.
int decode_geometry(const jenga_pool* pool, int32_t kind, int32_t n_q_heads, int32_t batch,
                    int32_t max_seq_len, int32_t window, int32_t pages_per_split, Geometry* out) {
  if (!pool || kind < 0 || kind >= int32_t(pool->kinds.size())) return JENGA_ERR_INVALID;
  const jenga::Kind& k = pool->kinds[kind];
  if (!attention_kind(k)) return JENGA_ERR_INVALID;
  if (batch < 0 || max_seq_len < 0 || window < 0 || n_q_heads < 1 || pages_per_split < 0)
    return JENGA_ERR_INVALID;
  // a sliding-window kind keeps only the pages of its window resident: a wider view would read
  // pages the allocator has already handed to someone else
  if (k.desc.type == JENGA_WINDOW && (window <= 0 || window > k.desc.window)) return JENGA_ERR_INVALID;
  // (the reduction's grid has one row of blocks per request)
  if (batch > kMaxGridBatch) return JENGA_ERR_UNSUPPORTED;
  if (n_q_heads % k.desc.n_kv_heads != 0) return JENGA_ERR_INVALID;
  const int G = n_q_heads / k.desc.n_kv_heads;
  // any number of query heads per KV head up to 16: the engine pads them to the 16 rows of the
  // matrix-core instructions anyway
  if (G > 16) return JENGA_ERR_UNSUPPORTED;
  const int row = k.desc.head_dim * k.elem_bytes;
  const int T = k.desc.tokens_per_page;
  out->kind = &k;
  out->G = G;
  // tokens per tile: one 16-token block, four of them for 128-byte rows
  const int tile_tokens = (row >= 256 ? 1 : 4) * 16;
  int64_t max_pages = (int64_t(max_seq_len) + T - 1) / T;
  if (window > 0) max_pages = std::min<int64_t>(max_pages, window / T + 2);
  const int64_t max_tiles = (max_pages * T + tile_tokens - 1) / tile_tokens;
  const int64_t w_max = (max_tiles + kSegStartUnits) * k.desc.n_kv_heads * std::max(batch, 1);
  if (w_max > 0x3fffffff) return JENGA_ERR_UNSUPPORTED;
  // whole 16-token blocks per page, half blocks, or any other page size
  const int mode = (T >= 16 && (T & (T - 1)) == 0) ? 0 : T == 8 ? 1 : 2;
  out->batch = batch;
  out->tile_log2 = tile_tokens == 16 ? 4 : 6;
  out->big = batch > kMaxBatch;
  out->fn = k.desc.dtype == JENGA_F32 ? pick_d<F32>(k.desc.head_dim, mode, G, out->big)
                                      : pick_d<BF16>(k.desc.head_dim, mode, G, out->big);
  if (out->fn == nullptr) return JENGA_ERR_UNSUPPORTED;
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

// Workspace layout: accumulators [slot][G][D], (max, sum) pairs [slot][G][2], then the
// (first chunk, last chunk) pair of every (request, KV head) segment, then, for batches above
// kMaxBatch, the requests' prefix sums and clamped lengths.
int64_t segments_of(const Geometry& g) { return g.slots - g.n_part_bound; }

int64_t workspace_bytes_for(const Geometry& g) {
  return g.slots * g.G * (g.kind->desc.head_dim + 2) * 4 + segments_of(g) * 8 + (g.big ? int64_t(g.batch) * 8 : 0);
}

int hip_status() { return hipGetLastError() == hipSuccess ? JENGA_OK : JENGA_ERR_HIP; }

struct Workspace {
  float* acc;
  float* ml;
  int32_t* meta;
  int32_t* incl;    // big batches only
  int32_t* len;
};

// Carves the three arrays out of `base` (the layout only depends on the geometry).
Workspace carve_ws(const Geometry& g, void* base) {
  Workspace ws;
  ws.acc = static_cast<float*>(base);
  ws.ml = ws.acc + g.slots * g.G * g.kind->desc.head_dim;
  ws.meta = reinterpret_cast<int32_t*>(ws.ml + g.slots * g.G * 2);
  ws.incl = ws.meta + segments_of(g) * 2;
  ws.len = ws.incl + g.batch;
  return ws;
}

int split_ws(const Geometry& g, void* workspace, int64_t workspace_bytes, Workspace* ws) {
  if (!workspace) return JENGA_ERR_INVALID;
  if (!aligned16(workspace)) return JENGA_ERR_ALIGN;
  if (workspace_bytes < workspace_bytes_for(g)) return JENGA_ERR_WORKSPACE;
  *ws = carve_ws(g, workspace);
  return JENGA_OK;
}

// Checks and launch of the append kernel; requests longer than max_len are left alone.
int launch_append(const jenga_pool* pool, int32_t kind, int32_t layer, const void* k_new,
                  const void* v_new, const int32_t* block_table, int32_t bt_stride,
                  const int32_t* seq_lens, int32_t batch, int32_t max_len, jenga_stream stream) {
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
                     block_table, bt_stride, seq_lens, batch, max_len,
                     int32_t(pool->n_large * k.per_large - 1));
  return hip_status();
}

// What the host can check of the partial kernel's arguments (the geometry is already valid).
int check_partial_args(const jenga_pool* pool, const Geometry& g, int32_t layer, const void* q,
                       const void* k_new, const void* v_new, const int32_t* block_table,
                       int32_t bt_stride, const int32_t* seq_lens, int32_t max_seq_len) {
  const jenga::Kind& k = *g.kind;
  if (!pool->base || layer < 0 || layer >= k.desc.n_layers || !q || !block_table || !seq_lens ||
      bt_stride < 1)
    return JENGA_ERR_INVALID;
  if (int64_t(bt_stride) * k.desc.tokens_per_page < max_seq_len) return JENGA_ERR_INVALID;
  if (!aligned16(q)) return JENGA_ERR_ALIGN;
  if ((k_new == nullptr) != (v_new == nullptr)) return JENGA_ERR_INVALID;
  if (k_new && k.desc.type != JENGA_FULL && k.desc.type != JENGA_WINDOW) return JENGA_ERR_INVALID;
  if (k_new && (!aligned16(k_new) || !aligned16(v_new))) return JENGA_ERR_ALIGN;
  return JENGA_OK;
}

// Launches the partial kernel (and, for large batches of short requests, the append in front of
// it) with checked arguments; the records go to `ws`.
int launch_partial(const jenga_pool* pool, int32_t kind, const Geometry& g, int32_t layer, const void* q,
                   int32_t n_q_heads, const void* k_new, const void* v_new, const int32_t* block_table,
                   int32_t bt_stride, const int32_t* seq_lens, int32_t batch, int32_t max_seq_len,
                   int32_t window, float scale, const Workspace& ws, float* out, jenga_stream stream) {
  if (batch == 0) return JENGA_OK;
  const jenga::Kind& k = *g.kind;
  const int row_bytes = k.desc.head_dim * k.elem_bytes;
  DecodeParams p;
  p.layer_base = pool->base + int64_t(layer) * k.slice_bytes;
  p.small_bytes = k.small_bytes;
  p.head_stride = 2 * k.desc.tokens_per_page * row_bytes;
  p.v_offset = k.desc.tokens_per_page * row_bytes;
  p.t_log2 = k.t_log2;
  p.tokens_per_page = k.desc.tokens_per_page;
  p.n_kv_heads = k.desc.n_kv_heads;
  p.n_q_heads = n_q_heads;
  p.group = g.G;
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
  p.ws_acc = ws.acc;
  p.ws_ml = ws.ml;
  p.ws_meta = ws.meta;
  p.out = out;
  p.ws_incl = ws.incl;
  p.ws_len = ws.len;
  const int n_part = launch_partitions(g);
  // Every appended row costs its wavefront the latency of a store (loads and stores share one
  // in-order counter): with many short requests -- six or more (request, KV head) segments per
  // wavefront -- the append is cheaper as a launch of its own in front (batch 1024 with 100-600
  // tokens: +2.3 % per step; equal at 4 segments per wavefront, 1.2 % slower at 1).
  if (k_new != nullptr && segments_of(g) >= 6 * int64_t(n_part)) {
    const int rc = launch_append(pool, kind, layer, k_new, v_new, block_table, bt_stride, seq_lens, batch,
                                 max_seq_len, stream);
    if (rc != JENGA_OK) return rc;
    p.k_new = nullptr;
    p.v_new = nullptr;
  }
  if (g.big)
    hipLaunchKernelGGL(scan_lengths_kernel, dim3(1), dim3(1024), 0, static_cast<hipStream_t>(stream), seq_lens,
                       batch, max_seq_len, window, k.t_log2, g.tile_log2, k.desc.n_kv_heads, ws.incl, ws.len);
  hipLaunchKernelGGL(g.fn, dim3(unsigned(n_part)), dim3(kWave), 0, static_cast<hipStream_t>(stream), p);
  return hip_status();
}

// Launches the reduction that merges the records in `ws` into `out`.
int launch_reduce(const Geometry& g, int32_t n_q_heads, const int32_t* seq_lens, int32_t batch,
                  int32_t max_seq_len, const Workspace& ws, float* out, jenga_stream stream) {
  if (batch == 0) return JENGA_OK;
  const jenga::Kind& k = *g.kind;
  float* acc = ws.acc;
  float* ml = ws.ml;
  int32_t* meta = ws.meta;
  const dim3 grid(static_cast<unsigned>(n_q_heads), static_cast<unsigned>(batch));
  hipStream_t st = static_cast<hipStream_t>(stream);
  // Four wavefronts per (request, query head) when the segments are few enough to have more than
  // about eight records each.
  const bool wide = launch_partitions(g) >= 8 * segments_of(g);
  // Many short segments (fewer than two records each on average): 256 / D query heads per
  // wavefront.  Batch 1024 with 100-600 tokens: +1.7 % per step with 128-element heads, +8 % with
  // 64-element heads; with two to three records per segment and some long ones (the Jamba-like
  // workload) the one-head kernel is 0.4 % faster, hence the bound.
  const int heads_per_wave = 256 / k.desc.head_dim;
  const bool packed = heads_per_wave > 1 && int64_t(launch_partitions(g)) < segments_of(g);
  const dim3 pgrid(static_cast<unsigned>((n_q_heads + heads_per_wave - 1) / heads_per_wave), static_cast<unsigned>(batch));
#define JENGA_LAUNCH_REDUCE(DIM)                                                                       \
  if (packed)                                                                                          \
    hipLaunchKernelGGL((splitk_reduce_packed_kernel<DIM>), pgrid, dim3(kWave), 0, st, acc, ml, meta,  \
                       seq_lens, max_seq_len, k.desc.n_kv_heads, n_q_heads, out);                      \
  else if (wide)                                                                                       \
    hipLaunchKernelGGL((splitk_reduce_kernel<DIM, 4>), grid, dim3(4 * kWave), 0, st, acc, ml, meta,   \
                       seq_lens, max_seq_len, k.desc.n_kv_heads, n_q_heads, out);                      \
  else                                                                                                 \
    hipLaunchKernelGGL((splitk_reduce_kernel<DIM, 1>), grid, dim3(kWave), 0, st, acc, ml, meta,       \
                       seq_lens, max_seq_len, k.desc.n_kv_heads, n_q_heads, out)
  switch (k.desc.head_dim) {
    case 64: JENGA_LAUNCH_REDUCE(64); break;
    case 128: JENGA_LAUNCH_REDUCE(128); break;
    default: JENGA_LAUNCH_REDUCE(256); break;
  }
#undef JENGA_LAUNCH_REDUCE
  return hip_status();
}

}  // namespace

extern "C" {

int jenga_kv_append(const jenga_pool* pool, int32_t kind, int32_t layer, const void* k_new,
                    const void* v_new, const int32_t* block_table, int32_t bt_stride,
                    const int32_t* seq_lens, int32_t batch, jenga_stream stream) {
  return launch_append(pool, kind, layer, k_new, v_new, block_table, bt_stride, seq_lens, batch,
                       0x7fffffff, stream);
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
  rc = check_partial_args(pool, g, layer, q, k_new, v_new, block_table, bt_stride, seq_lens, max_seq_len);
  if (rc != JENGA_OK) return rc;
  Workspace ws;
  rc = split_ws(g, workspace, workspace_bytes, &ws);
  if (rc != JENGA_OK) return rc;
  return launch_partial(pool, kind, g, layer, q, n_q_heads, k_new, v_new, block_table, bt_stride, seq_lens,
                        batch, max_seq_len, window, scale, ws, nullptr, stream);
}

int jenga_splitk_reduce(const jenga_pool* pool, int32_t kind, int32_t n_q_heads,
                        const int32_t* seq_lens, int32_t batch, int32_t max_seq_len, int32_t window,
                        int32_t pages_per_split, const void* workspace, int64_t workspace_bytes,
                        float* out, jenga_stream stream) {
  Geometry g;
  int rc = decode_geometry(pool, kind, n_q_heads, batch, max_seq_len, window, pages_per_split, &g);
  if (rc != JENGA_OK) return rc;
  if (!seq_lens || !out) return JENGA_ERR_INVALID;
  if (!aligned16(out)) return JENGA_ERR_ALIGN;
  Workspace ws;
  rc = split_ws(g, const_cast<void*>(workspace), workspace_bytes, &ws);
  if (rc != JENGA_OK) return rc;
  return launch_reduce(g, n_q_heads, seq_lens, batch, max_seq_len, ws, out, stream);
}

int jenga_paged_decode(const jenga_pool* pool, int32_t kind, int32_t layer, const void* q,
                       int32_t n_q_heads, const void* k_new, const void* v_new,
                       const int32_t* block_table, int32_t bt_stride,
                       const int32_t* seq_lens, int32_t batch, int32_t max_seq_len, int32_t window,
                       float scale, int32_t pages_per_split, void* workspace, int64_t workspace_bytes,
                       float* out, jenga_stream stream) {
  if (!out) return JENGA_ERR_INVALID;
  if (!aligned16(out)) return JENGA_ERR_ALIGN;
  Geometry g;
  int rc = decode_geometry(pool, kind, n_q_heads, batch, max_seq_len, window, pages_per_split, &g);
  if (rc != JENGA_OK) return rc;
  rc = check_partial_args(pool, g, layer, q, k_new, v_new, block_table, bt_stride, seq_lens, max_seq_len);
  if (rc != JENGA_OK) return rc;
  Workspace ws;
  rc = split_ws(g, workspace, workspace_bytes, &ws);
  if (rc != JENGA_OK) return rc;
  // (the partial kernel knows `out`: segments it covers in one piece are finished there)
  rc = launch_partial(pool, kind, g, layer, q, n_q_heads, k_new, v_new, block_table, bt_stride, seq_lens,
                      batch, max_seq_len, window, scale, ws, out, stream);
  if (rc != JENGA_OK) return rc;
  return launch_reduce(g, n_q_heads, seq_lens, batch, max_seq_len, ws, out, stream);
}

int jenga_paged_decode_static(const jenga_pool* pool, int32_t kind, int32_t layer, const void* q,
                              int32_t n_q_heads, const void* k_new, const void* v_new,
                              const int32_t* block_table, int32_t bt_stride,
                              const int32_t* seq_lens, int32_t batch, int32_t max_seq_len, int32_t window,
                              float scale, int32_t pages_per_split, float* out, jenga_stream stream) {
  if (!out) return JENGA_ERR_INVALID;
  if (!aligned16(out)) return JENGA_ERR_ALIGN;
  Geometry g;
  int rc = decode_geometry(pool, kind, n_q_heads, batch, max_seq_len, window, pages_per_split, &g);
  if (rc != JENGA_OK) return rc;
  rc = check_partial_args(pool, g, layer, q, k_new, v_new, block_table, bt_stride, seq_lens, max_seq_len);
  if (rc != JENGA_OK) return rc;
  // A caller-owned workspace is sized for the largest grid the automatic mode may ever use; here
  // the grid is known, so the records need room for exactly its partitions.
  if (g.chunk_tiles == 0) {
    const int64_t segs = segments_of(g);
    g.n_part_bound = launch_partitions(g);
    g.slots = int64_t(g.n_part_bound) + segs;
  }
  if (workspace_bytes_for(g) > kStaticScratchBytes) return JENGA_ERR_WORKSPACE;
  void* base = static_scratch(&rc);
  if (!base) return rc;
  const Workspace ws = carve_ws(g, base);
  rc = launch_partial(pool, kind, g, layer, q, n_q_heads, k_new, v_new, block_table, bt_stride, seq_lens,
                      batch, max_seq_len, window, scale, ws, out, stream);
  if (rc != JENGA_OK) return rc;
  return launch_reduce(g, n_q_heads, seq_lens, batch, max_seq_len, ws, out, stream);
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
  // one wavefront per SIMD of a 256-unit device, fewer for short streams
  const unsigned blocks = unsigned(std::max<int64_t>(1, std::min<int64_t>(n / (16 * kWave), 1024)));
  hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(kWave), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(src), n, static_cast<unsigned*>(sink));
  return hip_status();
}

}  // extern "C"
