// Decode attention over a paged KV cache (the attention part of forward_decode(B),
// Algorithm 2 of the paper; Section 2.1 describes decoding as one new token per
// request against all of its cached tokens).  HBM-bound: every cached K and V
// element of every running request is read exactly once per step.
//
// Decomposition.  Order all (sequence r, kv head h, KV block b) triples of the batch
// as r-major, then h, then b, and call that sequence of gtot blocks the *stream*.
// The stream is cut into W equal ranges, one per resident wavefront, regardless of
// where sequences begin and end, so every wave moves the same number of bytes:
//   plan    one workgroup: blocks per sequence -> exclusive prefix; then for each
//           wave the (r, h, b) at which its range starts and the range length.
//   attend  one 64-lane wave per range.  The wave walks its range block by block,
//           always one block of loads ahead of the arithmetic, across sequence and
//           head boundaries without draining.  Each maximal run of blocks of one
//           (r, h) inside the range is a *piece*; when a piece ends the wave writes
//           either the final output (the piece is the whole sequence) or an fp32
//           partial (m, l, acc[128] per q head).  A wave owns at most two partial
//           pieces: one cut at its range start and one cut at its range end.
//   merge   one wave per range boundary: if the boundary cuts a (r, h), combines the
//           partials of the waves that share it exactly (rescale by exp2(m_c - m))
//           and writes the output; also writes zeros for empty sequences.
//
// Lane mapping inside a wave: lane = 16 * row + sub.  A 16-byte load instruction
// covers 4 tokens x 128 dims: row picks the token (4 * i + row for load i of a
// block), sub picks dims 8*sub .. 8*sub+7.  A K.q dot product is 4 packed dot2
// operations per lane plus a 4-step DPP all-reduce inside the 16-lane row; the V
// update needs no cross-lane traffic.  The 4 rows keep separate softmax states
// that are merged once per piece.
#include "vtc_internal.h"

namespace vtc {

constexpr int kPlanThreads = 1024;

// Start of wave w's range in the stream, floor(gtot * w / waves), from quot = gtot / waves and
// rem = gtot % waves (rem * w < 2^26 because waves <= kMaxDecodeWaves): no 64-bit division.
struct RangeMap {
  long long quot;
  uint32_t rem;
  uint32_t waves;
  __device__ __forceinline__ long long start(int w) const {
    return quot * (long long)w + (long long)(rem * (uint32_t)w / waves);
  }
};

// ------------------------------------------------------------------ plan ----
constexpr int kPlanLdsSeqs = 8192;     // sequences whose block prefix is also kept in LDS for the range search

__global__ __launch_bounds__(kPlanThreads) void decode_plan_kernel(const int32_t* __restrict__ seq_lens,
                                                                   int32_t num_seqs, int32_t num_kv_heads,
                                                                   int32_t max_tokens, int32_t max_waves,
                                                                   DecodeHeader* __restrict__ header,
                                                                   int32_t* __restrict__ seg_prefix,
                                                                   int4* __restrict__ wave_desc) {
  __shared__ int32_t prefix_lds[kPlanLdsSeqs + 1];
  __shared__ int32_t wave_sums[kPlanThreads / kWave];
  __shared__ int32_t carry;
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wid = tid / kWave;
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int base = 0; base < num_seqs; base += kPlanThreads) {
    const int r = base + tid;
    int32_t n = 0;
    if (r < num_seqs) n = (min(max(seq_lens[r], 0), max_tokens) + kBlockSize - 1) / kBlockSize;
    // inclusive scan inside the wave, then across the 16 waves
    int32_t x = n;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const int32_t y = __shfl_up(x, off);
      if (lane >= off) x += y;
    }
    if (lane == kWave - 1) wave_sums[wid] = x;
    __syncthreads();
    int32_t before = carry;
    for (int j = 0; j < wid; ++j) before += wave_sums[j];
    if (r < num_seqs) {
      const int32_t excl = before + x - n;
      seg_prefix[r] = excl;
      if (r < kPlanLdsSeqs) prefix_lds[r] = excl;
    }
    __syncthreads();
    if (tid == kPlanThreads - 1) carry = before + x;
    __syncthreads();
  }
  const int32_t total_blocks = carry;
  if (tid == 0) {
    seg_prefix[num_seqs] = total_blocks;
    if (num_seqs <= kPlanLdsSeqs) prefix_lds[num_seqs] = total_blocks;
  }
  const long long gtot = (long long)total_blocks * num_kv_heads;
  // every active wave gets at least kMinBlocksPerWave blocks
  const long long want = (gtot + kMinBlocksPerWave - 1) / kMinBlocksPerWave;
  const int waves = (int)(want < (long long)max_waves ? want : (long long)max_waves);
  RangeMap map{0, 0u, 1u};
  if (waves > 0) map = RangeMap{gtot / waves, (uint32_t)(gtot % waves), (uint32_t)waves};
  if (tid == 0) {
    header->gtot = gtot;
    header->quot = map.quot;
    header->rem = (int)map.rem;
    header->waves = waves;
  }
  __syncthreads();                                           // the prefix is complete and visible to the workgroup
  const bool in_lds = num_seqs <= kPlanLdsSeqs;
  for (int w = tid; w < max_waves; w += kPlanThreads) {
    int4 d = make_int4(0, 0, 0, 0);
    if (w < waves) {
      const long long g = map.start(w);
      const long long n = map.start(w + 1) - g;
      // the sequence r with prefix[r] * Hkv <= g < prefix[r+1] * Hkv
      int lo = 0, hi = num_seqs - 1;
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        const int32_t pm = in_lds ? prefix_lds[mid + 1] : seg_prefix[mid + 1];
        if ((long long)pm * num_kv_heads > g) hi = mid; else lo = mid + 1;
      }
      const int32_t p0 = in_lds ? prefix_lds[lo] : seg_prefix[lo];
      const int32_t p1 = in_lds ? prefix_lds[lo + 1] : seg_prefix[lo + 1];
      const int nb = p1 - p0;
      const uint32_t off = (uint32_t)(g - (long long)p0 * num_kv_heads);   // < nb * Hkv < 2^31
      d = make_int4(lo, (int)(off / (uint32_t)nb), (int)(off % (uint32_t)nb), (int)n);
    }
    wave_desc[w] = d;
  }
}

// ---------------------------------------------------------------- attend ----
template <int G>
struct RowState {
  float m[G];        // running max of the scaled logits (log2 domain)
  float l[G];        // running sum of exp2(logit - m)
  float acc[G][8];   // running sum of exp2(logit - m) * v, dims 8*sub .. 8*sub+7
  __device__ __forceinline__ void reset() {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      m[g] = -INFINITY;
      l[g] = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
    }
  }
};

// Process one K/V block (16 tokens).  `nvalid` < 16 marks a ragged last block:
// tokens >= nvalid are excluded and their (possibly garbage) V rows zeroed.
template <typename T, int G, bool kTail>
__device__ __forceinline__ void block_update(RowState<G>& st, const u32x4 (&q)[G], const u32x4 (&k)[4],
                                             u32x4 (&v)[4], float scale2, int row, int nvalid) {
  float s[G][4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float d = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) d = dot2<T>(q[g][w], k[i][w], d);
      s[g][i] = row16_allreduce_sum(d) * scale2;
    }
  }
  if (kTail) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool ok = 4 * i + row < nvalid;
#pragma unroll
      for (int g = 0; g < G; ++g) s[g][i] = ok ? s[g][i] : -INFINITY;
      if (!ok) v[i] = u32x4{0u, 0u, 0u, 0u};
    }
  }
  float p[G][4];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const float mx = fmaxf(fmaxf(s[g][0], s[g][1]), fmaxf(s[g][2], s[g][3]));
    const float m_new = fmaxf(st.m[g], mx);
    // a row that has seen no valid token yet keeps m = -inf; subtract 0 instead so
    // that exp2 yields 0 rather than NaN
    const float m_sub = (kTail && m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = fast_exp2(st.m[g] - m_sub);
#pragma unroll
    for (int i = 0; i < 4; ++i) p[g][i] = fast_exp2(s[g][i] - m_sub);
    st.l[g] = st.l[g] * alpha + ((p[g][0] + p[g][1]) + (p[g][2] + p[g][3]));
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[g][e] *= alpha;
    st.m[g] = m_new;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float lo = lo_f32<T>(v[i][w]);
      const float hi = hi_f32<T>(v[i][w]);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        st.acc[g][2 * w] = fmaf(p[g][i], lo, st.acc[g][2 * w]);
        st.acc[g][2 * w + 1] = fmaf(p[g][i], hi, st.acc[g][2 * w + 1]);
      }
    }
  }
}

// Load one 4 KiB tile (4 x 1 KiB across the wave).  `stride16` is kWave for a real tile; 0 turns the
// four loads into re-reads of one 1 KiB line set (the throw-away prefetch at the end of a range).
__device__ __forceinline__ void load_tile(u32x4 (&dst)[4], const uint16_t* __restrict__ tile, int lane, int stride16) {
  const u32x4* src = reinterpret_cast<const u32x4*>(tile) + lane;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#if VTC_DECODE_NT_LOADS
    dst[i] = __builtin_nontemporal_load(src + i * stride16);  // streamed once: keep it out of the caches' way
#else
    dst[i] = src[i * stride16];
#endif
  }
}

// A position in the stream: which block, and where its K/V tile lives.
struct StreamPos {
  int r, h, b;       // sequence, kv head, block index inside the sequence
  int nb;            // blocks of sequence r
  int s_len;         // context length of sequence r (clamped)
  size_t off;        // element offset of the (block, head) tile in k_cache / v_cache
};

template <typename T, int G>
__global__ __launch_bounds__(kWave) void decode_attend_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_cache, const uint16_t* __restrict__ v_cache,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_lens, uint16_t* __restrict__ out,
    const int4* __restrict__ wave_desc, float2* __restrict__ part_ml, float* __restrict__ part_acc,
    int32_t num_kv_heads, int32_t max_blocks_per_seq, float scale2) {
  const int lane = threadIdx.x;
  const int row = lane >> 4;
  const int sub = lane & 15;
  const int num_q_heads = num_kv_heads * G;
  const int max_tokens = max_blocks_per_seq * kBlockSize;
  const int wave = blockIdx.x;
  const int4 desc_v = wave_desc[wave];
  // the descriptor is the same for all lanes: keep it (and everything derived from it) in scalar registers
  const int4 desc = make_int4(__builtin_amdgcn_readfirstlane(desc_v.x), __builtin_amdgcn_readfirstlane(desc_v.y),
                              __builtin_amdgcn_readfirstlane(desc_v.z), __builtin_amdgcn_readfirstlane(desc_v.w));
  const int n_blocks = desc.w;
  if (n_blocks <= 0) return;
  const size_t block_stride = (size_t)num_kv_heads * kTileElems;

  auto locate = [&](StreamPos& p) {        // fill in the tile offset of p
    p.off = (size_t)block_table[(size_t)p.r * max_blocks_per_seq + p.b] * block_stride + (size_t)p.h * kTileElems;
  };
  auto step = [&](StreamPos& p) {          // move p to the next block of the stream (there is one)
    if (++p.b == p.nb) {
      p.b = 0;
      if (++p.h == num_kv_heads) {
        p.h = 0;
        do {
          ++p.r;
          p.s_len = min(max(seq_lens[p.r], 0), max_tokens);
          p.nb = (p.s_len + kBlockSize - 1) / kBlockSize;
        } while (p.nb == 0);
      }
    }
    locate(p);
  };
  auto load_q = [&](u32x4 (&dst)[G], const StreamPos& p) {
#pragma unroll
    for (int g = 0; g < G; ++g)
      dst[g] = *reinterpret_cast<const u32x4*>(q + ((size_t)p.r * num_q_heads + p.h * G + g) * kHeadDim + sub * 8);
  };

  // cur: the block being consumed; nxt: the block whose loads are in flight; far: one further, so
  // that its (scalar) block-table lookup is never waited for between a tile's loads and their use.
  StreamPos cur;
  cur.r = desc.x;
  cur.h = desc.y;
  cur.b = desc.z;
  cur.s_len = min(max(seq_lens[cur.r], 0), max_tokens);
  cur.nb = (cur.s_len + kBlockSize - 1) / kBlockSize;
  locate(cur);
  StreamPos nxt = cur, far = cur;
  if (n_blocks > 1) {
    step(nxt);
    far = nxt;
  }
  if (n_blocks > 2) step(far);

  RowState<G> st;
  st.reset();
  int piece_lo = cur.b;                    // first block of the current piece

  // Two register sets (q, K tile, V tile), used alternately.  The q rows travel with the
  // tiles, so a set always holds the query of the block it holds.
  u32x4 qa[G], ka[4], va[4], qb[G], kb[4], vb[4];
  load_q(qa, cur);
  load_tile(ka, k_cache + cur.off, lane, kWave);
  load_tile(va, v_cache + cur.off, lane, kWave);
  // where the prefetch goes when there is no next block: 1 KiB of the (cache-resident) range table
  const uint16_t* const dummy = reinterpret_cast<const uint16_t*>(wave_desc);

  // Consume the block at `cur` from (qreg, kx, vx); close the piece if it ends here.
  auto consume = [&](const u32x4 (&qreg)[G], u32x4 (&kx)[4], u32x4 (&vx)[4], bool last_of_range) {
    const bool last_of_seq = cur.b + 1 == cur.nb;
    const int nvalid = last_of_seq ? cur.s_len - cur.b * kBlockSize : kBlockSize;
    if (nvalid < kBlockSize)
      block_update<T, G, true>(st, qreg, kx, vx, scale2, row, nvalid);
    else
      block_update<T, G, false>(st, qreg, kx, vx, scale2, row, kBlockSize);
    if (!(last_of_seq || last_of_range)) return;

    // merge the four 16-lane rows (lanes l, l^16, l^32, l^48 hold the same dims)
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float m_o = __shfl_xor(st.m[g], off);
        const float l_o = __shfl_xor(st.l[g], off);
        const float m_n = fmaxf(st.m[g], m_o);
        const float m_sub = m_n == -INFINITY ? 0.f : m_n;
        const float a = fast_exp2(st.m[g] - m_sub);
        const float b = fast_exp2(m_o - m_sub);
        st.l[g] = st.l[g] * a + l_o * b;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.acc[g][e] = st.acc[g][e] * a + __shfl_xor(st.acc[g][e], off) * b;
        st.m[g] = m_n;
      }
    }
    const bool whole = piece_lo == 0 && last_of_seq;     // the piece is the entire sequence
    if (row == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        if (whole) {
          const float inv = 1.f / st.l[g];
          u32x4 o;
#pragma unroll
          for (int w2 = 0; w2 < 4; ++w2) o[w2] = pack2<T>(st.acc[g][2 * w2] * inv, st.acc[g][2 * w2 + 1] * inv);
          *reinterpret_cast<u32x4*>(out + ((size_t)cur.r * num_q_heads + cur.h * G + g) * kHeadDim + sub * 8) = o;
        } else {
          // slot 0: the piece cut at the start of this wave's range; slot 1: the one cut at its end
          const size_t pi = ((size_t)wave * 2 + (piece_lo == 0 ? 1 : 0)) * G + g;
          float4* dst = reinterpret_cast<float4*>(part_acc + pi * kPartialFloats + sub * 8);
          dst[0] = make_float4(st.acc[g][0], st.acc[g][1], st.acc[g][2], st.acc[g][3]);
          dst[1] = make_float4(st.acc[g][4], st.acc[g][5], st.acc[g][6], st.acc[g][7]);
          if (sub == 0) part_ml[pi] = make_float2(st.m[g], st.l[g]);
        }
      }
    }
    st.reset();                             // a new (r, h) starts with the next block
    piece_lo = 0;
  };

  // The prefetch of the next block is unconditional (no branch around the loads, so the
  // hardware load counter stays exact and a tile's wait never covers the loads issued after
  // it).  On the last block of the range it is pointed at 1 KiB that is already in cache and
  // its result is dropped.  q is re-read with every block for the same reason (a 256-byte
  // row that stays in cache); it only changes when the next block starts a new (r, h).
  int i = 0;
  while (true) {
    // -- even step: consume set a, prefetch into set b
    {
      const bool more = i + 1 < n_blocks;
      load_q(qb, nxt);
      load_tile(kb, more ? k_cache + nxt.off : dummy, lane, more ? kWave : 0);
      load_tile(vb, more ? v_cache + nxt.off : dummy, lane, more ? kWave : 0);
    }
    consume(qa, ka, va, i + 1 == n_blocks);
    if (++i == n_blocks) break;
    cur = nxt;
    nxt = far;
    if (i + 2 < n_blocks) step(far);
    // -- odd step: consume set b, prefetch into set a
    {
      const bool more = i + 1 < n_blocks;
      load_q(qa, nxt);
      load_tile(ka, more ? k_cache + nxt.off : dummy, lane, more ? kWave : 0);
      load_tile(va, more ? v_cache + nxt.off : dummy, lane, more ? kWave : 0);
    }
    consume(qb, kb, vb, i + 1 == n_blocks);
    if (++i == n_blocks) break;
    cur = nxt;
    nxt = far;
    if (i + 2 < n_blocks) step(far);
  }
}

// ----------------------------------------------------------------- merge ----
// Only a sequence-head that a range boundary cuts needs merging, so the merge is driven by the
// boundaries: block w looks at the cut between waves w-1 and w.  If that cut falls inside a
// (r, kv head) and wave w-1 holds its beginning, the block combines the pieces of waves
// w-1, w, w+1, ... for one of the G query heads of that kv head (blockIdx.y).  Blocks past the
// waves zero the output rows of empty sequences.
template <typename T>
__global__ __launch_bounds__(kWave) void decode_merge_kernel(const DecodeHeader* __restrict__ header,
                                                             const int32_t* __restrict__ seg_prefix,
                                                             const int4* __restrict__ wave_desc,
                                                             const float2* __restrict__ part_ml,
                                                             const float* __restrict__ part_acc,
                                                             uint16_t* __restrict__ out, int32_t num_seqs,
                                                             int32_t num_q_heads, int32_t num_kv_heads,
                                                             int32_t max_waves) {
  const int lane = threadIdx.x;                          // dims 2*lane, 2*lane+1
  const int group = num_q_heads / num_kv_heads;
  const int g = blockIdx.y;                              // query head inside the group
  if ((int)blockIdx.x >= max_waves) {                    // empty sequences: all-zero rows
    const int r = blockIdx.x - max_waves;
    if (g != 0 || seg_prefix[r + 1] - seg_prefix[r] > 0) return;
    uint32_t* dst = reinterpret_cast<uint32_t*>(out + (size_t)r * num_q_heads * kHeadDim);
    for (int i = lane; i < num_q_heads * (kHeadDim / 2); i += kWave) dst[i] = 0u;
    return;
  }
  const int w = blockIdx.x;
  const int waves = header->waves;
  if (w == 0 || w >= waves) return;
  const int4 d = wave_desc[w];                           // (r, kv head, block) where wave w starts
  if (d.z == 0) return;                                  // the cut coincides with a sequence-head boundary
  if (d.z > wave_desc[w - 1].w) return;                  // the beginning lies before wave w-1: an earlier block merges it
  const int nb = seg_prefix[d.x + 1] - seg_prefix[d.x];
  const RangeMap map{header->quot, (uint32_t)header->rem, (uint32_t)waves};
  const long long g1 = map.start(w) + (nb - d.z);         // end of the sequence-head in the stream
  {
    // wave w-1 holds the beginning (its slot 1); waves w.. hold continuations (their slot 0)
    float m = part_ml[((size_t)(w - 1) * 2 + 1) * group + g].x;
    int w_end = w;
    while (w_end < waves && map.start(w_end) < g1) {
      m = fmaxf(m, part_ml[((size_t)w_end * 2) * group + g].x);
      ++w_end;
    }
    float l = 0.f, a0 = 0.f, a1 = 0.f;
    for (int j = w - 1; j < w_end; ++j) {
      const size_t pi = ((size_t)j * 2 + (j == w - 1 ? 1 : 0)) * group + g;
      const float2 ml = part_ml[pi];
      const float wgt = fast_exp2(ml.x - m);
      const float2 a = *reinterpret_cast<const float2*>(part_acc + pi * kPartialFloats + 2 * lane);
      l = fmaf(ml.y, wgt, l);
      a0 = fmaf(a.x, wgt, a0);
      a1 = fmaf(a.y, wgt, a1);
    }
    const float inv = 1.f / l;
    uint32_t* dst = reinterpret_cast<uint32_t*>(out + ((size_t)d.x * num_q_heads + d.y * group + g) * kHeadDim) + lane;
    *dst = pack2<T>(a0 * inv, a1 * inv);
  }
}

// -------------------------------------------------------------- launcher ----
template <typename T, int G>
static int launch_typed(const vtc_attn_params& p, int32_t num_seqs, const void* q, const void* k_cache,
                        const void* v_cache, const int32_t* block_table, const int32_t* seq_lens, void* out,
                        void* workspace, hipStream_t stream, hipEvent_t ev_begin, hipEvent_t ev_end) {
  const DecodeWorkspace ws = decode_workspace_layout(p, num_seqs, 0);
  char* base = static_cast<char*>(workspace);
  DecodeHeader* header = reinterpret_cast<DecodeHeader*>(base + ws.header_off);
  int32_t* seg_prefix = reinterpret_cast<int32_t*>(base + ws.seg_prefix_off);
  int4* wave_desc = reinterpret_cast<int4*>(base + ws.wave_desc_off);
  float2* part_ml = reinterpret_cast<float2*>(base + ws.ml_off);
  float* part_acc = reinterpret_cast<float*>(base + ws.acc_off);
  const int32_t max_tokens = p.max_blocks_per_seq * kBlockSize;

  // Grid = the waves the chip holds at once (never more, so no wave waits for a slot while
  // the others are already half way through their share).
  static int waves_per_cu = 0;
  if (waves_per_cu == 0) {
    int occ = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, decode_attend_kernel<T, G>, kWave, 0) != hipSuccess || occ <= 0)
      occ = 8;
    waves_per_cu = occ < VTC_DECODE_WAVES_PER_CU ? occ : VTC_DECODE_WAVES_PER_CU;
  }
  long long resident = (long long)device_cu_count() * waves_per_cu;
  const int grid = (int)(resident < kMaxDecodeWaves ? resident : kMaxDecodeWaves);

  hipLaunchKernelGGL(decode_plan_kernel, dim3(1), dim3(kPlanThreads), 0, stream, seq_lens, num_seqs, p.num_kv_heads,
                     max_tokens, grid, header, seg_prefix, wave_desc);
  if (ev_begin && hipEventRecord(ev_begin, stream) != hipSuccess) return VTC_ERR_HIP;
  hipLaunchKernelGGL((decode_attend_kernel<T, G>), dim3(grid), dim3(kWave), 0, stream,
                     static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k_cache),
                     static_cast<const uint16_t*>(v_cache), block_table, seq_lens, static_cast<uint16_t*>(out),
                     wave_desc, part_ml, part_acc, p.num_kv_heads, p.max_blocks_per_seq, p.scale * kLog2e);
  if (ev_end && hipEventRecord(ev_end, stream) != hipSuccess) return VTC_ERR_HIP;
  hipLaunchKernelGGL((decode_merge_kernel<T>), dim3(grid + num_seqs, G), dim3(kWave), 0, stream, header, seg_prefix,
                     wave_desc, part_ml, part_acc, static_cast<uint16_t*>(out), num_seqs, p.num_q_heads,
                     p.num_kv_heads, grid);
  return hipGetLastError() == hipSuccess ? VTC_OK : VTC_ERR_HIP;
}

template <typename T>
static int launch_group(const vtc_attn_params& p, int32_t num_seqs, const void* q, const void* k_cache,
                        const void* v_cache, const int32_t* block_table, const int32_t* seq_lens, void* out,
                        void* workspace, hipStream_t stream, hipEvent_t ev_begin, hipEvent_t ev_end) {
  switch (p.num_q_heads / p.num_kv_heads) {
    case 1: return launch_typed<T, 1>(p, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace, stream, ev_begin, ev_end);
    case 2: return launch_typed<T, 2>(p, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace, stream, ev_begin, ev_end);
    case 4: return launch_typed<T, 4>(p, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace, stream, ev_begin, ev_end);
    case 8: return launch_typed<T, 8>(p, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace, stream, ev_begin, ev_end);
    default: return VTC_ERR_UNSUPPORTED;
  }
}

int launch_decode(const vtc_attn_params& p, int32_t num_seqs, const void* q, const void* k_cache,
                  const void* v_cache, const int32_t* block_table, const int32_t* seq_lens, void* out,
                  void* workspace, hipStream_t stream, hipEvent_t ev_begin, hipEvent_t ev_end) {
  // the flattened block index must fit the 64-bit products used above and the grid limits of the merge launch
  if ((long long)num_seqs * p.max_blocks_per_seq >= (1ll << 31)) return VTC_ERR_UNSUPPORTED;
  if (p.dtype == VTC_F16)
    return launch_group<F16>(p, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace, stream, ev_begin, ev_end);
  return launch_group<BF16>(p, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace, stream, ev_begin, ev_end);
}

}  // namespace vtc
