// Decode attention over a paged KV cache (the attention part of forward_decode(B),
// Algorithm 2 of the paper; Section 2.1 describes decoding as one new token per
// request against all of its cached tokens).  HBM-bound: every cached K and V
// element of every running request is read exactly once per step.
//
// Decomposition
//   plan    one workgroup: chunks per sequence -> exclusive prefix -> a flat list
//           of work items (sequence, chunk).  A chunk is kChunkTokens tokens.
//   attend  one 64-lane wavefront per (work item, kv head), in a grid-stride loop.
//           The wave streams the chunk's K and V tiles (4 KiB each per block) with
//           16-byte loads that are contiguous across the wave, keeps an online
//           softmax per 16-lane row, and either writes the final output (sequence
//           has a single chunk) or an fp32 partial (m, l, acc[128]).
//   merge   one workgroup per (sequence, q head) with more than one chunk: combines
//           the partials exactly (rescale by exp2(m_c - m)) and writes the output;
//           writes zeros for empty sequences.
//
// Lane mapping inside a wave: lane = 16 * row + sub.  A 16-byte load instruction
// covers 4 tokens x 128 dims: row picks the token (4 * i + row for load i of a
// block), sub picks dims 8*sub .. 8*sub+7.  A K.q dot product is 4 packed dot2
// operations per lane plus a 4-step DPP all-reduce inside the 16-lane row; the V
// update needs no cross-lane traffic.  The 4 rows keep separate softmax states
// that are merged once per work item.
#include "vtc_internal.h"

namespace vtc {

constexpr int kPlanThreads = 1024;

// ------------------------------------------------------------------ plan ----
__global__ __launch_bounds__(kPlanThreads) void decode_plan_kernel(const int32_t* __restrict__ seq_lens,
                                                                   int32_t num_seqs, int32_t max_tokens,
                                                                   int32_t* __restrict__ chunk_start,
                                                                   int2* __restrict__ items) {
  __shared__ int32_t scan[kPlanThreads];
  __shared__ int32_t carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (int base = 0; base < num_seqs; base += kPlanThreads) {
    const int r = base + (int)threadIdx.x;
    int32_t n = 0;
    if (r < num_seqs) {
      const int32_t s = min(max(seq_lens[r], 0), max_tokens);
      n = (s + kChunkTokens - 1) / kChunkTokens;
    }
    scan[threadIdx.x] = n;
    __syncthreads();
    for (int off = 1; off < kPlanThreads; off <<= 1) {     // inclusive Hillis-Steele scan
      int32_t v = (int)threadIdx.x >= off ? scan[threadIdx.x - off] : 0;
      __syncthreads();
      scan[threadIdx.x] += v;
      __syncthreads();
    }
    const int32_t start = carry + scan[threadIdx.x] - n;
    if (r < num_seqs) {
      chunk_start[r] = start;
      for (int c = 0; c < n; ++c) items[start + c] = make_int2(r, c);
    }
    __syncthreads();
    if (threadIdx.x == kPlanThreads - 1) carry += scan[threadIdx.x];
    __syncthreads();
  }
  if (threadIdx.x == 0) chunk_start[num_seqs] = carry;
}

// ---------------------------------------------------------------- attend ----
template <typename T, int G>
struct RowState {
  float m[G];        // running max of the scaled logits (log2 domain)
  float l[G];        // running sum of exp2(logit - m)
  float acc[G][8];   // running sum of exp2(logit - m) * v, dims 8*sub .. 8*sub+7
};

// Process one K/V block (16 tokens).  `nvalid` < 16 marks a ragged last block:
// tokens >= nvalid are excluded and their (possibly garbage) V rows zeroed.
template <typename T, int G, bool kTail>
__device__ __forceinline__ void block_update(RowState<T, G>& st, const u32x4 (&q)[G], const u32x4 (&k)[4],
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
  for (int i = 0; i < 4; ++i) dst[i] = src[i * kWave];
}

template <typename T, int G>
__global__ __launch_bounds__(kWave) void decode_attend_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_cache, const uint16_t* __restrict__ v_cache,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_lens, uint16_t* __restrict__ out,
    const int32_t* __restrict__ chunk_start, const int2* __restrict__ items, float2* __restrict__ part_ml,
    float* __restrict__ part_acc, int32_t num_seqs, int32_t num_kv_heads, int32_t max_blocks_per_seq, float scale2) {
  const int lane = threadIdx.x;
  const int row = lane >> 4;
  const int sub = lane & 15;
  const int num_q_heads = num_kv_heads * G;
  const int max_tokens = max_blocks_per_seq * kBlockSize;
  const uint32_t total = (uint32_t)chunk_start[num_seqs] * (uint32_t)num_kv_heads;

  for (uint32_t w = blockIdx.x; w < total; w += gridDim.x) {
    const int slot = (int)(w / (uint32_t)num_kv_heads);  // index into items / partials
    const int kvh = (int)(w - (uint32_t)slot * (uint32_t)num_kv_heads);
    const int2 item = items[slot];
    const int r = item.x;
    const int c = item.y;
    const int s_len = min(seq_lens[r], max_tokens);
    const int n_chunks = (s_len + kChunkTokens - 1) / kChunkTokens;
    const int t0 = c * kChunkTokens;
    const int t1 = min(s_len, t0 + kChunkTokens);
    const int n_full = (t1 - t0) / kBlockSize;          // complete blocks in this chunk
    const int tail = (t1 - t0) % kBlockSize;            // valid tokens of the ragged last block
    const int32_t* __restrict__ table = block_table + (size_t)r * max_blocks_per_seq + t0 / kBlockSize;

    u32x4 qreg[G];
#pragma unroll
    for (int g = 0; g < G; ++g)
      qreg[g] = *reinterpret_cast<const u32x4*>(q + ((size_t)r * num_q_heads + kvh * G + g) * kHeadDim + sub * 8);

    RowState<T, G> st;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      st.m[g] = -INFINITY;
      st.l[g] = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) st.acc[g][e] = 0.f;
    }

    const int n_blocks = n_full + (tail ? 1 : 0);
    const int last = n_blocks - 1;
    const size_t head_off = (size_t)kvh * kTileElems;
    const size_t block_stride = (size_t)num_kv_heads * kTileElems;
    // Two register buffers, used alternately; block ids are fetched two blocks ahead so
    // that the (scalar) table lookup never sits between a tile's loads and their use.
    u32x4 ka[4], va[4], kb[4], vb[4];
    int32_t id_next = table[min(1, last)];
    int32_t id_after = table[min(2, last)];
    {
      const size_t off = (size_t)table[0] * block_stride + head_off;
      load_tile(ka, k_cache + off, lane);
      load_tile(va, v_cache + off, lane);
    }
    int b = 0;
    while (b < n_full) {
      if (b + 1 < n_blocks) {                            // fetch block b+1 while block b is consumed
        const size_t off = (size_t)id_next * block_stride + head_off;
        load_tile(kb, k_cache + off, lane);
        load_tile(vb, v_cache + off, lane);
      }
      id_next = id_after;
      id_after = table[min(b + 3, last)];
      block_update<T, G, false>(st, qreg, ka, va, scale2, row, kBlockSize);
      ++b;
      if (b >= n_full) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          ka[i] = kb[i];
          va[i] = vb[i];
        }
        break;
      }
      if (b + 1 < n_blocks) {
        const size_t off = (size_t)id_next * block_stride + head_off;
        load_tile(ka, k_cache + off, lane);
        load_tile(va, v_cache + off, lane);
      }
      id_next = id_after;
      id_after = table[min(b + 3, last)];
      block_update<T, G, false>(st, qreg, kb, vb, scale2, row, kBlockSize);
      ++b;
    }
    if (tail) block_update<T, G, true>(st, qreg, ka, va, scale2, row, tail);

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

    if (row == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const int h = kvh * G + g;
        if (n_chunks == 1) {
          const float inv = 1.f / st.l[g];
          u32x4 o;
#pragma unroll
          for (int w2 = 0; w2 < 4; ++w2) o[w2] = pack2<T>(st.acc[g][2 * w2] * inv, st.acc[g][2 * w2 + 1] * inv);
          *reinterpret_cast<u32x4*>(out + ((size_t)r * num_q_heads + h) * kHeadDim + sub * 8) = o;
        } else {
          const size_t pi = (size_t)slot * num_q_heads + h;
          float4* dst = reinterpret_cast<float4*>(part_acc + pi * kPartialFloats + sub * 8);
          dst[0] = make_float4(st.acc[g][0], st.acc[g][1], st.acc[g][2], st.acc[g][3]);
          dst[1] = make_float4(st.acc[g][4], st.acc[g][5], st.acc[g][6], st.acc[g][7]);
          if (sub == 0) part_ml[pi] = make_float2(st.m[g], st.l[g]);
        }
      }
    }
  }
}

// ----------------------------------------------------------------- merge ----
template <typename T>
__global__ __launch_bounds__(kWave) void decode_merge_kernel(const int32_t* __restrict__ seq_lens,
                                                             const int32_t* __restrict__ chunk_start,
                                                             const float2* __restrict__ part_ml,
                                                             const float* __restrict__ part_acc,
                                                             uint16_t* __restrict__ out, int32_t num_q_heads,
                                                             int32_t max_tokens) {
  const int r = blockIdx.x;
  const int h = blockIdx.y;
  const int lane = threadIdx.x;                          // dims 2*lane, 2*lane+1
  const int s_len = min(seq_lens[r], max_tokens);
  const int n_chunks = (s_len + kChunkTokens - 1) / kChunkTokens;
  if (n_chunks == 1) return;                             // written directly by the attend kernel
  uint32_t* dst = reinterpret_cast<uint32_t*>(out + ((size_t)r * num_q_heads + h) * kHeadDim) + lane;
  if (n_chunks <= 0) {
    *dst = 0u;
    return;
  }
  const size_t first = (size_t)chunk_start[r] * num_q_heads + h;
  float m = -INFINITY;
  for (int c = 0; c < n_chunks; ++c) m = fmaxf(m, part_ml[first + (size_t)c * num_q_heads].x);
  float l = 0.f, a0 = 0.f, a1 = 0.f;
  for (int c = 0; c < n_chunks; ++c) {
    const size_t pi = first + (size_t)c * num_q_heads;
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
  int32_t* chunk_start = reinterpret_cast<int32_t*>(base + ws.chunk_start_off);
  int2* items = reinterpret_cast<int2*>(base + ws.items_off);
  float2* part_ml = reinterpret_cast<float2*>(base + ws.ml_off);
  float* part_acc = reinterpret_cast<float*>(base + ws.acc_off);
  const int32_t max_tokens = p.max_blocks_per_seq * kBlockSize;

  hipLaunchKernelGGL(decode_plan_kernel, dim3(1), dim3(kPlanThreads), 0, stream, seq_lens, num_seqs, max_tokens,
                     chunk_start, items);

  const long long max_work = ws.max_items * p.num_kv_heads;
  if (max_work >= (1ll << 31)) return VTC_ERR_UNSUPPORTED;
  const long long resident = (long long)device_cu_count() * 16;      // waves the chip can hold at once
  const int grid = (int)(max_work < resident ? (max_work < 1 ? 1 : max_work) : resident);
  if (ev_begin && hipEventRecord(ev_begin, stream) != hipSuccess) return VTC_ERR_HIP;
  hipLaunchKernelGGL((decode_attend_kernel<T, G>), dim3(grid), dim3(kWave), 0, stream,
                     static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k_cache),
                     static_cast<const uint16_t*>(v_cache), block_table, seq_lens, static_cast<uint16_t*>(out),
                     chunk_start, items, part_ml, part_acc, num_seqs, p.num_kv_heads, p.max_blocks_per_seq,
                     p.scale * kLog2e);
  if (ev_end && hipEventRecord(ev_end, stream) != hipSuccess) return VTC_ERR_HIP;

  hipLaunchKernelGGL((decode_merge_kernel<T>), dim3(num_seqs, p.num_q_heads), dim3(kWave), 0, stream, seq_lens,
                     chunk_start, part_ml, part_acc, static_cast<uint16_t*>(out), p.num_q_heads, max_tokens);
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
  if (num_seqs > 65535 * 1024) return VTC_ERR_UNSUPPORTED;
  if (p.dtype == VTC_F16)
    return launch_group<F16>(p, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace, stream, ev_begin, ev_end);
  return launch_group<BF16>(p, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace, stream, ev_begin, ev_end);
}

}  // namespace vtc
