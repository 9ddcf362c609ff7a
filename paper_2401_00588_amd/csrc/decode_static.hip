// vtc_attn_decode_static: decode attention for callers that cannot allocate or hand over a workspace
// (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  It is
// vtc_attn_decode with the workspace -- range table and fp32 partial results of the launch -- placed in a
// device array that is part of the library image, so the call takes inputs and outputs only.
#include "vtc_internal.h"

#include <mutex>

namespace vtc {

constexpr size_t kStaticScratchBytes = 10u << 20;      // 10 MiB on every device the library runs on
constexpr int32_t kStaticMaxSeqs = 65536;              // 256 KiB of it for the per-sequence prefix

// In host code this name is a stand-in for the symbol, not a device address: host code uses the pointer that
// hipGetSymbolAddress returns for the current device, never the name.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Address of `scratch` on the current device, looked up once per device (each device holds its own copy).
static int static_scratch(void** ptr_out) {
  static std::mutex mu;
  static void* ptrs[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return VTC_ERR_HIP;
  std::lock_guard<std::mutex> lock(mu);
  if (ptrs[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return VTC_ERR_HIP;
    ptrs[dev] = p;
  }
  *ptr_out = ptrs[dev];
  return VTC_OK;
}

}  // namespace vtc

extern "C" int vtc_attn_decode_static(const vtc_attn_params* params, int32_t num_seqs, const void* q,
                                      const void* k_cache, const void* v_cache, const int32_t* block_table,
                                      const int32_t* seq_lens, void* out, void* hip_stream) {
  int rc = vtc::check_params(params);
  if (rc != VTC_OK) return rc;
  if (num_seqs < 0) return VTC_ERR_INVALID_ARG;
  if (num_seqs == 0) return VTC_OK;
  if (num_seqs > vtc::kStaticMaxSeqs) return VTC_ERR_STATIC_LIMIT;
  if (!q || !k_cache || !v_cache || !block_table || !seq_lens || !out) return VTC_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(q) & 15u) || (reinterpret_cast<uintptr_t>(out) & 15u) ||
      (reinterpret_cast<uintptr_t>(k_cache) & 15u) || (reinterpret_cast<uintptr_t>(v_cache) & 15u))
    return VTC_ERR_INVALID_ARG;
  if (params->block_size != vtc::kBlockSize)              // small blocks: the general path uses no scratch at all
    return vtc::launch_attend_general(*params, num_seqs, q, nullptr, 1, k_cache, v_cache, block_table, seq_lens, out,
                                      static_cast<hipStream_t>(hip_stream));
  // as many waves as the array has room for (all the device holds, for every supported shape on 256 compute units)
  const int max_waves = vtc::decode_wave_capacity(*params, num_seqs, vtc::kStaticScratchBytes, vtc::decode_wave_bound(*params));
  if (max_waves < 1) return VTC_ERR_STATIC_LIMIT;
  void* workspace = nullptr;
  rc = vtc::static_scratch(&workspace);
  if (rc != VTC_OK) return rc;
  // nothing in the workspace has to start at zero: the launch writes the range table and every partial
  // result before the merge reads it
  return vtc::launch_decode(*params, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace, max_waves,
                            static_cast<hipStream_t>(hip_stream), nullptr, nullptr, vtc::CounterJob{});
}
