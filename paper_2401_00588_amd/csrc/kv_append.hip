// Append the K/V rows of newly processed tokens to the paged cache: the step between
// the projection of a token and the attention over its sequence (forward_prefill /
// forward_decode of Algorithm 2 both run on a cache that already holds the new tokens).
// Pure data movement: 16-byte pieces, a 256-byte (token, kv head) row per 16 lanes.
#include "vtc_internal.h"

namespace vtc {

constexpr int kAppendThreads = 256;
constexpr int kAppendTokens = 8;       // new tokens of one sequence per workgroup

__global__ __launch_bounds__(kAppendThreads) void kv_append_kernel(
    const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new, const int32_t* __restrict__ cu_new_lens,
    uint16_t* __restrict__ k_cache, uint16_t* __restrict__ v_cache, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ seq_lens, int32_t num_kv_heads, int32_t max_blocks_per_seq, int32_t block_size) {
  const int r = blockIdx.x;
  const int first = cu_new_lens[r];
  const int n_new = cu_new_lens[r + 1] - first;
  const int i0 = blockIdx.y * kAppendTokens;
  if (i0 >= n_new) return;
  const int s_len = min(max(seq_lens[r], 0), max_blocks_per_seq * block_size);
  const int pieces_per_token = num_kv_heads * (kHeadDim / 8);          // 16-byte pieces of one token's K (or V)
  const int n_tok = min(kAppendTokens, n_new - i0);
  for (int it = threadIdx.x; it < n_tok * pieces_per_token; it += kAppendThreads) {
    const int i = i0 + it / pieces_per_token;                          // new token index inside the sequence
    const int piece = it % pieces_per_token;
    const int head = piece / (kHeadDim / 8);
    const int c16 = piece % (kHeadDim / 8);
    const int p = s_len - n_new + i;                                   // absolute position
    if (p < 0) continue;                                               // seq_lens shorter than the append: nothing to place
    const size_t src = ((size_t)(first + i) * num_kv_heads + head) * kHeadDim + c16 * 8;
    const int32_t slot = slot_of(block_table + (size_t)r * max_blocks_per_seq, p, block_size);   // physical block * block_size + row
    const size_t dst = cache_row_offset(slot, head, num_kv_heads, block_size) + c16 * 8;
    *reinterpret_cast<u32x4*>(k_cache + dst) = *reinterpret_cast<const u32x4*>(k_new + src);
    *reinterpret_cast<u32x4*>(v_cache + dst) = *reinterpret_cast<const u32x4*>(v_new + src);
  }
}

int launch_kv_append(const vtc_attn_params& p, int32_t num_seqs, const void* k_new, const void* v_new,
                     const int32_t* cu_new_lens, int32_t max_new_len, void* k_cache, void* v_cache,
                     const int32_t* block_table, const int32_t* seq_lens, hipStream_t stream) {
  const int gy = (max_new_len + kAppendTokens - 1) / kAppendTokens;
  if (gy > 65535) return VTC_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(kv_append_kernel, dim3(num_seqs, gy), dim3(kAppendThreads), 0, stream,
                     static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new), cu_new_lens,
                     static_cast<uint16_t*>(k_cache), static_cast<uint16_t*>(v_cache), block_table, seq_lens,
                     p.num_kv_heads, p.max_blocks_per_seq, p.block_size);
  return hipGetLastError() == hipSuccess ? VTC_OK : VTC_ERR_HIP;
}

}  // namespace vtc
