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
//   merge   one wave per (r, q head): finds the waves whose ranges overlap the
//           sequence, combines their partials exactly (rescale by exp2(m_c - m))
//           and writes the output; writes zeros for empty sequences.
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

// 64-bit helpers shared by plan and merge: start of wave w's range, and the wave that owns block g.
__device__ __forceinline__ long long range_start(long long gtot, int waves, int w) {
  return gtot * (long long)w / (long long)waves;
}
__device__ __forceinline__ int wave_of(long long gtot, int waves, long long g) {
  int w = (int)(g * (long long)waves / gtot);
  if (w + 1 < waves && range_start(gtot, waves, w + 1) <= g) ++w;
  return w;
}

// ------------------------------------------------------------------ plan ----
__global__ __launch_bounds__(kPlanThreads) void decode_plan_kernel(const int32_t* __restrict__ seq_lens,
                                                                   int32_t num_seqs, int32_t num_kv_heads,
                                                                   int32_t max_tokens, int32_t max_waves,
                                                                   DecodeHeader* __restrict__ header,
                                                                   int32_t* __restrict__ seg_prefix,
                                                                   int4* __restrict__ wave_desc) {
  __shared__ int32_t scan[kPlanThreads];
  __shared__ int32_t carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (int base = 0; base < num_seqs; base += kPlanThreads) {
    const int r = base + (int)threadIdx.x;
    int32_t n = 0;
    if (r < num_seqs) n = (min(max(seq_lens[r], 0), max_tokens) + kBlockSize - 1) / kBlockSize;
    scan[threadIdx.x] = n;
    __syncthreads();
    for (int off = 1; off < kPlanThreads; off <<= 1) {     // inclusive Hillis-Steele scan
      int32_t v = (int)threadIdx.x >= off ? scan[threadIdx.x - off] : 0;
      __syncthreads();
      scan[threadIdx.x] += v;
      __syncthreads();
    }
    if (r < num_seqs) seg_prefix[r] = carry + scan[threadIdx.x] - n;
    __syncthreads();
    if (threadIdx.x == kPlanThreads - 1) carry += scan[threadIdx.x];
    __syncthreads();
  }
  const int32_t total_blocks = carry;
  if (threadIdx.x == 0) seg_prefix[num_seqs] = total_blocks;
  const long long gtot = (long long)total_blocks * num_kv_heads;
  // every active wave gets at least kMinBlocksPerWave blocks
  const long long want = (gtot + kMinBlocksPerWave - 1) / kMinBlocksPerWave;
  const int waves = (int)(want < (long long)max_waves ? want : (long long)max_waves);
  if (threadIdx.x == 0) {
    header->gtot = gtot;
    header->waves = waves;
  }
  __threadfence();
  __syncthreads();                                           // seg_prefix is complete and visible
  for (int w = threadIdx.x; w < max_waves; w += kPlanThreads) {
    int4 d = make_int4(0, 0, 0, 0);
    if (w < waves) {
      const long long g = range_start(gtot, waves, w);
      const long long n = range_start(gtot, waves, w + 1) - g;
      // the sequence r with seg_prefix[r] * Hkv <= g < seg_prefix[r+1] * Hkv
      int lo = 0, hi = num_seqs - 1;
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if ((long long)seg_prefix[mid + 1] * num_kv_heads > g) hi = mid; else lo = mid + 1;
      }
      const int nb = seg_prefix[lo + 1] - seg_prefix[lo];
      const long long off = g - (long long)seg_prefix[lo] * num_kv_heads;
      d = make_int4(lo, (int)(off / nb), (int)(off % nb), (int)n);
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

__device__ __forceinline__ void load_tile(u32x4 (&dst)[4], const uint16_t* __restrict__ tile, int lane) {
  const u32x4* src = reinterpret_cast<const u32x4*>(tile) + lane;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#if VTC_DECODE_NT_LOADS
    dst[i] = __builtin_nontemporal_load(src + i * kWave);     // streamed once: keep it out of the caches' way
#else
    dst[i] = src[i * kWave];
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
  const int4 desc = wave_desc[wave];
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

  u32x4 qreg[G], qnext[G];
  load_q(qreg, cur);
  RowState<G> st;
  st.reset();
  int piece_lo = cur.b;                    // first block of the current piece

  u32x4 ka[4], va[4], kb[4], vb[4];
  load_tile(ka, k_cache + cur.off, lane);
  load_tile(va, v_cache + cur.off, lane);

  // Consume the block at `cur` from (kx, vx); close the piece if it ends here.
  auto consume = [&](u32x4 (&kx)[4], u32x4 (&vx)[4], bool last_of_range) {
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
    if (!last_of_range) {                   // a new (r, h) starts with the next block
      st.reset();
      piece_lo = 0;
#pragma unroll
      for (int g = 0; g < G; ++g) qreg[g] = qnext[g];
    }
  };

  int i = 0;
  while (true) {
    // -- even step: consume from (ka, va), prefetch into (kb, vb)
    if (i + 1 < n_blocks) {
      if (nxt.b == 0) load_q(qnext, nxt);
      load_tile(kb, k_cache + nxt.off, lane);
      load_tile(vb, v_cache + nxt.off, lane);
    }
    consume(ka, va, i + 1 == n_blocks);
    if (++i == n_blocks) break;
    cur = nxt;
    nxt = far;
    if (i + 2 < n_blocks) step(far);
    // -- odd step: consume from (kb, vb), prefetch into (ka, va)
    if (i + 1 < n_blocks) {
      if (nxt.b == 0) load_q(qnext, nxt);
      load_tile(ka, k_cache + nxt.off, lane);
      load_tile(va, v_cache + nxt.off, lane);
    }
    consume(kb, vb, i + 1 == n_blocks);
    if (++i == n_blocks) break;
    cur = nxt;
    nxt = far;
    if (i + 2 < n_blocks) step(far);
  }
}

// ----------------------------------------------------------------- merge ----
template <typename T>
__global__ __launch_bounds__(kWave) void decode_merge_kernel(const DecodeHeader* __restrict__ header,
                                                             const int32_t* __restrict__ seg_prefix,
                                                             const float2* __restrict__ part_ml,
                                                             const float* __restrict__ part_acc,
                                                             uint16_t* __restrict__ out, int32_t num_q_heads,
                                                             int32_t num_kv_heads) {
  const int r = blockIdx.x;
  const int h = blockIdx.y;
  const int lane = threadIdx.x;                          // dims 2*lane, 2*lane+1
  const int group = num_q_heads / num_kv_heads;
  const int nb = seg_prefix[r + 1] - seg_prefix[r];
  uint32_t* dst = reinterpret_cast<uint32_t*>(out + ((size_t)r * num_q_heads + h) * kHeadDim) + lane;
  if (nb <= 0) {
    *dst = 0u;
    return;
  }
  const long long gtot = header->gtot;
  const int waves = header->waves;
  const long long g0 = (long long)seg_prefix[r] * num_kv_heads + (long long)(h / group) * nb;
  const int w_first = wave_of(gtot, waves, g0);
  const int w_last = wave_of(gtot, waves, g0 + nb - 1);
  if (w_first == w_last) return;                         // one wave saw the whole sequence and wrote the output
  float m = -INFINITY;
  for (int w = w_first; w <= w_last; ++w) {
    const size_t pi = ((size_t)w * 2 + (range_start(gtot, waves, w) > g0 ? 0 : 1)) * group + h % group;
    m = fmaxf(m, part_ml[pi].x);
  }
  float l = 0.f, a0 = 0.f, a1 = 0.f;
  for (int w = w_first; w <= w_last; ++w) {
    const size_t pi = ((size_t)w * 2 + (range_start(gtot, waves, w) > g0 ? 0 : 1)) * group + h % group;
    const float2 ml = part_ml[pi];
    const float wgt = fast_exp2(ml.x - m);
    const float2 a = *reinterpret_cast<const float2*>(part_acc + pi * kPartialFloats + 2 * lane);
    l = fmaf(ml.y, wgt, l);
    a0 = fmaf(a.x, wgt, a0);
    a1 = fmaf(a.y, wgt, a1);
  }
  const float inv = 1.f / l;
  *dst = pack2<T>(a0 * inv, a1 * inv);
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
  hipLaunchKernelGGL((decode_merge_kernel<T>), dim3(num_seqs, p.num_q_heads), dim3(kWave), 0, stream, header,
                     seg_prefix, part_ml, part_acc, static_cast<uint16_t*>(out), p.num_q_heads, p.num_kv_heads);
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
  if (p.num_q_heads > 65535) return VTC_ERR_UNSUPPORTED;
  if (p.dtype == VTC_F16)
    return launch_group<F16>(p, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace, stream, ev_begin, ev_end);
  return launch_group<BF16>(p, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace, stream, ev_begin, ev_end);
}

}  // namespace vtc
