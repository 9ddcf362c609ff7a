// Test hook: physical slot of every valid (sequence, position) of a paged cache.
#include "vtc_internal.h"

namespace vtc {

__global__ __launch_bounds__(256) void gather_slots_kernel(const int32_t* __restrict__ block_table,
                                                           int32_t max_blocks_per_seq, int32_t block_size,
                                                           const int32_t* __restrict__ seq_lens,
                                                           const int32_t* __restrict__ cu_out,
                                                           int32_t* __restrict__ slots_out) {
  const int r = blockIdx.x;
  const int p = blockIdx.y * 256 + threadIdx.x;
  const int s = min(seq_lens[r], max_blocks_per_seq * block_size);
  if (p >= s) return;
  slots_out[cu_out[r] + p] = slot_of(block_table + (size_t)r * max_blocks_per_seq, p, block_size);
}

int launch_gather_slots(const vtc_attn_params& p, int32_t num_seqs, const int32_t* block_table,
                        const int32_t* seq_lens, const int32_t* cu_out, int32_t max_seq_len, int32_t* slots_out,
                        hipStream_t stream) {
  if ((max_seq_len + 255) / 256 > 65535) return VTC_ERR_UNSUPPORTED;
  dim3 grid(num_seqs, (max_seq_len + 255) / 256);
  hipLaunchKernelGGL(gather_slots_kernel, grid, dim3(256), 0, stream, block_table, p.max_blocks_per_seq, p.block_size, seq_lens,
                     cu_out, slots_out);
  return hipGetLastError() == hipSuccess ? VTC_OK : VTC_ERR_HIP;
}

}  // namespace vtc
