// Causal prefill-chunk attention over a paged KV cache on the CDNA4 matrix cores
// (the attention part of forward_prefill(B_new), Algorithm 2 of the paper;
// Section 2.1 describes prefilling as processing all prompt tokens at once).
//
// One workgroup (4 wavefronts) handles 64 consecutive chunk tokens of one
// (sequence, q head); each wave owns 16 query rows.  The workgroup walks the
// visible keys in tiles of 64, staging the K and V tiles of the head's KV group
// in LDS.  Per tile and wave:
//   S^T = K . Q^T      16 x v_mfma_f32_16x16x32  (A = K rows from LDS, B = Q^T in registers)
//   online softmax     per query row (= per lane column), fp32, exp2 domain
//   O^T += V^T . P^T   16 x v_mfma_f32_16x16x32  (A = V^T gathered from LDS, B = P^T)
// Working with the transposed products makes the accumulator layout of S^T
// (lane: query row l%16, keys 4*(l/16)+v) directly usable as the B operand of the
// second product: the 8 contraction slots of lane group l/16 are assigned to keys
// {4*(l/16)+v} of two neighbouring 16-key blocks, and V^T is gathered to match.
#include "vtc_internal.h"

namespace vtc {

using f32x4 = float __attribute__((ext_vector_type(4)));
using f16x8 = _Float16 __attribute__((ext_vector_type(8)));
using bf16x8 = __bf16 __attribute__((ext_vector_type(8)));

constexpr int kQTile = 64;          // query rows per workgroup
constexpr int kKTile = 64;          // keys per LDS tile
constexpr int kPitch = kHeadDim + 8;   // LDS row pitch in elements (272 B): conflict-free 16-byte row reads

template <typename T>
__device__ __forceinline__ f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c);
template <>
__device__ __forceinline__ f32x4 mfma16<F16>(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <>
__device__ __forceinline__ f32x4 mfma16<BF16>(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

template <typename T>
__global__ __launch_bounds__(256) void prefill_chunk_kernel(
    const uint16_t* __restrict__ q, const int32_t* __restrict__ cu_q_lens, const uint16_t* __restrict__ k_cache,
    const uint16_t* __restrict__ v_cache, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ seq_lens, uint16_t* __restrict__ out, int32_t num_q_heads, int32_t num_kv_heads,
    int32_t max_blocks_per_seq, float scale2) {
  __shared__ __attribute__((aligned(16))) uint16_t k_lds[kKTile * kPitch];
  __shared__ __attribute__((aligned(16))) uint16_t v_lds[kKTile * kPitch];

  const int qt = blockIdx.x;
  const int h = blockIdx.y;
  const int r = blockIdx.z;
  const int q_begin = cu_q_lens[r];
  const int lq = cu_q_lens[r + 1] - q_begin;
  if (qt * kQTile >= lq) return;                                   // uniform over the workgroup
  const int s_len = min(seq_lens[r], max_blocks_per_seq * kBlockSize);
  const int p0 = max(s_len - lq, 0);                               // absolute position of chunk token 0
  const int kvh = h / (num_q_heads / num_kv_heads);
  const int32_t* __restrict__ table = block_table + (size_t)r * max_blocks_per_seq;

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int col = lane & 15;       // query row within the wave's 16 (MFMA column index)
  const int kg = lane >> 4;        // lane group: contraction slots 8*kg .. 8*kg+7

  const int i_row = qt * kQTile + wave * 16 + col;                 // chunk token of this lane's column
  const int i_load = min(i_row, lq - 1);
  const int pq = p0 + i_row;                                       // its absolute position
  // keys the workgroup / the wave can see
  const int wg_kv_end = min(s_len, p0 + min(lq, qt * kQTile + kQTile));
  const int wave_kv_end = min(s_len, p0 + min(lq, qt * kQTile + wave * 16 + 16));

  u32x4 qf[4];
  {
    const uint16_t* src = q + ((size_t)(q_begin + i_load) * num_q_heads + h) * kHeadDim + kg * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) qf[ks] = *reinterpret_cast<const u32x4*>(src + ks * 32);
  }

  f32x4 oacc[8];
#pragma unroll
  for (int db = 0; db < 8; ++db) oacc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY;
  float l_run = 0.f;               // partial: this lane group's keys only

  const int n_tiles = (wg_kv_end + kKTile - 1) / kKTile;
  for (int kt = 0; kt < n_tiles; ++kt) {
    const int k0 = kt * kKTile;
    __syncthreads();                                               // previous tile fully consumed
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + 256 * i;                                // 16-byte piece of the 64 x 128 tile
      const int row = id >> 4;
      const int c16 = id & 15;
      const int key = k0 + row;
      u32x4 kv = u32x4{0u, 0u, 0u, 0u}, vv = u32x4{0u, 0u, 0u, 0u};
      if (key < s_len) {
        const size_t off = (((size_t)table[key / kBlockSize] * num_kv_heads + kvh) * kBlockSize + key % kBlockSize) * kHeadDim + c16 * 8;
        kv = *reinterpret_cast<const u32x4*>(k_cache + off);
        vv = *reinterpret_cast<const u32x4*>(v_cache + off);
      }
      *reinterpret_cast<u32x4*>(&k_lds[row * kPitch + c16 * 8]) = kv;
      *reinterpret_cast<u32x4*>(&v_lds[row * kPitch + c16 * 8]) = vv;
    }
    __syncthreads();
    if (k0 >= wave_kv_end) continue;                               // whole tile masked for this wave

    // S^T tile: 4 key blocks x (16 keys x 16 query rows)
    f32x4 sacc[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      sacc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const u32x4 kf = *reinterpret_cast<const u32x4*>(&k_lds[(nb * 16 + col) * kPitch + ks * 32 + kg * 8]);
        sacc[nb] = mfma16<T>(kf, qf[ks], sacc[nb]);
      }
    }
    // scale, causal mask, row maximum
    float mx = -INFINITY;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int key = k0 + nb * 16 + kg * 4 + v;
        const float s = key <= pq ? sacc[nb][v] * scale2 : -INFINITY;
        sacc[nb][v] = s;
        mx = fmaxf(mx, s);
      }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float m_sub = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = fast_exp2(m_run - m_sub);
    m_run = m_new;
    float psum = 0.f;
    u32x4 pb[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      float p[8];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        p[v] = fast_exp2(sacc[2 * t][v] - m_sub);
        p[4 + v] = fast_exp2(sacc[2 * t + 1][v] - m_sub);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) psum += p[e];
#pragma unroll
      for (int w = 0; w < 4; ++w) pb[t][w] = pack2<T>(p[2 * w], p[2 * w + 1]);
    }
    l_run = l_run * alpha + psum;
#pragma unroll
    for (int db = 0; db < 8; ++db) oacc[db] *= alpha;

    // O^T += V^T . P^T
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int db = 0; db < 8; ++db) {
        const uint16_t* vsrc = &v_lds[(t * 32 + kg * 4) * kPitch + db * 16 + col];
        uint32_t e[8];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          e[v] = vsrc[v * kPitch];
          e[4 + v] = vsrc[(16 + v) * kPitch];
        }
        u32x4 vf;
#pragma unroll
        for (int w = 0; w < 4; ++w) vf[w] = e[2 * w] | (e[2 * w + 1] << 16);
        oacc[db] = mfma16<T>(vf, pb[t], oacc[db]);
      }
    }
  }

  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  if (i_row < lq) {
    const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
    uint16_t* dst = out + ((size_t)(q_begin + i_row) * num_q_heads + h) * kHeadDim + kg * 4;
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      uint2 o;
      o.x = pack2<T>(oacc[db][0] * inv, oacc[db][1] * inv);
      o.y = pack2<T>(oacc[db][2] * inv, oacc[db][3] * inv);
      *reinterpret_cast<uint2*>(dst + db * 16) = o;
    }
  }
}

int launch_prefill(const vtc_attn_params& p, int32_t num_seqs, const void* q, const int32_t* cu_q_lens,
                   int32_t max_q_len, const void* k_cache, const void* v_cache, const int32_t* block_table,
                   const int32_t* seq_lens, void* out, hipStream_t stream) {
  if (num_seqs > 65535 || p.num_q_heads > 65535) return VTC_ERR_UNSUPPORTED;
  dim3 grid((max_q_len + kQTile - 1) / kQTile, p.num_q_heads, num_seqs);
  const float scale2 = p.scale * kLog2e;
  if (p.dtype == VTC_F16)
    hipLaunchKernelGGL(prefill_chunk_kernel<F16>, grid, dim3(256), 0, stream, static_cast<const uint16_t*>(q),
                       cu_q_lens, static_cast<const uint16_t*>(k_cache), static_cast<const uint16_t*>(v_cache),
                       block_table, seq_lens, static_cast<uint16_t*>(out), p.num_q_heads, p.num_kv_heads,
                       p.max_blocks_per_seq, scale2);
  else
    hipLaunchKernelGGL(prefill_chunk_kernel<BF16>, grid, dim3(256), 0, stream, static_cast<const uint16_t*>(q),
                       cu_q_lens, static_cast<const uint16_t*>(k_cache), static_cast<const uint16_t*>(v_cache),
                       block_table, seq_lens, static_cast<uint16_t*>(out), p.num_q_heads, p.num_kv_heads,
                       p.max_blocks_per_seq, scale2);
  return hipGetLastError() == hipSuccess ? VTC_OK : VTC_ERR_HIP;
}

}  // namespace vtc
