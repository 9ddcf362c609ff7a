// C ABI entry points: host-side validation, then the kernel launchers.
// Every check on host-visible arguments runs before the first HIP call.
#include "vtc_internal.h"

#include <mutex>

namespace vtc {

DeviceShape device_shape() {
  static std::mutex mu;
  static DeviceShape cached[64];
  const DeviceShape assumed{256, 8};                     // an MI355X in its default partition mode
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return assumed;
  std::lock_guard<std::mutex> lock(mu);
  if (cached[dev].cus == 0) {
    int cus = 0, xcds = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = assumed.cus;
    if (hipDeviceGetAttribute(&xcds, hipDeviceAttributeNumberOfXccs, dev) != hipSuccess || xcds <= 0 || cus % xcds != 0)
      xcds = 1;                                          // unknown: treat the device as one die (plain block order)
    cached[dev] = DeviceShape{cus, xcds};
  }
  return cached[dev];
}

int device_cu_count() { return device_shape().cus; }

}  // namespace vtc

extern "C" {

int vtc_version(void) { return 300; }   // 0.3.0

const char* vtc_strerror(int code) {
  switch (code) {
    case VTC_OK: return "success";
    case VTC_ERR_INVALID_ARG: return "invalid argument (null pointer, negative or inconsistent size)";
    case VTC_ERR_UNSUPPORTED:
      return "unsupported configuration (need head_dim 128, block_size 1, 2, 4, 8 or 16, fp16/bf16, "
             "num_q_heads/num_kv_heads in {1,2,4,8})";
    case VTC_ERR_WORKSPACE_TOO_SMALL: return "workspace smaller than vtc_attn_workspace_bytes()";
    case VTC_ERR_HIP: return "HIP runtime error (launch failed or no usable device)";
    case VTC_ERR_STATIC_LIMIT:
      return "more sequences than vtc_attn_decode_static's built-in scratch array is laid out for (65536)";
    default: return "unknown error code";
  }
}

size_t vtc_attn_workspace_bytes(const vtc_attn_params* params, int32_t max_num_seqs, int32_t max_seq_len) {
  if (vtc::check_params(params) != VTC_OK || max_num_seqs < 0) return 0;
  return vtc::decode_workspace_layout(*params, max_num_seqs, vtc::decode_waves_for(*params, max_num_seqs, max_seq_len))
      .total_bytes;
}

static int decode_common(const vtc_attn_params* params, int32_t num_seqs, const void* q, const void* k_cache,
                         const void* v_cache, const int32_t* block_table, const int32_t* seq_lens, void* out,
                         void* workspace, size_t workspace_bytes, void* hip_stream, void* ev_begin, void* ev_end,
                         const vtc::CounterJob& job) {
  int rc = vtc::check_params(params);
  if (rc != VTC_OK) return rc;
  if (num_seqs < 0) return VTC_ERR_INVALID_ARG;
  if (num_seqs == 0) return VTC_OK;
  if (!q || !k_cache || !v_cache || !block_table || !seq_lens || !out) return VTC_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(q) & 15u) || (reinterpret_cast<uintptr_t>(out) & 15u) ||
      (reinterpret_cast<uintptr_t>(k_cache) & 15u) || (reinterpret_cast<uintptr_t>(v_cache) & 15u))
    return VTC_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (params->block_size != vtc::kBlockSize) {            // small blocks: the general path, which needs no workspace
    if (ev_begin) (void)hipEventRecord(static_cast<hipEvent_t>(ev_begin), stream);
    rc = vtc::launch_attend_general(*params, num_seqs, q, nullptr, 1, k_cache, v_cache, block_table, seq_lens, out, stream);
    if (ev_end) (void)hipEventRecord(static_cast<hipEvent_t>(ev_end), stream);
    if (rc == VTC_OK && job.n > 0)
      rc = vtc::launch_counter_update(reinterpret_cast<int64_t*>(job.counters), job.num_clients, job.client_ids, job.n_in,
                                      job.n_out, job.n, (int64_t)job.w_p, (int64_t)job.w_q, stream);
    return rc;
  }
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return VTC_ERR_INVALID_ARG;
  // the launch uses as many waves as the workspace has room for (and the device can hold)
  const int max_waves = vtc::decode_wave_capacity(*params, num_seqs, workspace_bytes, vtc::decode_wave_bound(*params));
  if (max_waves < 1) return VTC_ERR_WORKSPACE_TOO_SMALL;
  return vtc::launch_decode(*params, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace, max_waves,
                            stream, static_cast<hipEvent_t>(ev_begin),
                            static_cast<hipEvent_t>(ev_end), job);
}

int vtc_attn_decode_profiled(const vtc_attn_params* params, int32_t num_seqs, const void* q, const void* k_cache,
                             const void* v_cache, const int32_t* block_table, const int32_t* seq_lens, void* out,
                             void* workspace, size_t workspace_bytes, void* hip_stream, void* ev_begin,
                             void* ev_end) {
  return decode_common(params, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace,
                       workspace_bytes, hip_stream, ev_begin, ev_end, vtc::CounterJob{});
}

int vtc_attn_decode(const vtc_attn_params* params, int32_t num_seqs, const void* q, const void* k_cache,
                    const void* v_cache, const int32_t* block_table, const int32_t* seq_lens, void* out,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  return decode_common(params, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace,
                       workspace_bytes, hip_stream, nullptr, nullptr, vtc::CounterJob{});
}

int vtc_step_decode_profiled(const vtc_attn_params* params, int32_t num_seqs, const void* q, const void* k_cache,
                             const void* v_cache, const int32_t* block_table, const int32_t* seq_lens, void* out,
                             int64_t* counters, int32_t num_clients, const int32_t* client_ids,
                             const int32_t* n_input_tokens, const int32_t* n_output_tokens, int32_t n,
                             int64_t w_p, int64_t w_q, void* workspace, size_t workspace_bytes, void* hip_stream,
                             void* ev_begin, void* ev_end) {
  // every host-visible argument of both halves is checked before anything is enqueued
  int rc = vtc::check_params(params);
  if (rc != VTC_OK) return rc;
  if (num_seqs < 0 || n < 0 || num_clients < 0) return VTC_ERR_INVALID_ARG;
  const bool charge = n > 0 && num_clients > 0;
  if (charge && (!counters || !client_ids)) return VTC_ERR_INVALID_ARG;
  if (num_seqs == 0)                           // nothing to attend to: the charge alone
    return charge ? vtc::launch_counter_update(counters, num_clients, client_ids, n_input_tokens, n_output_tokens, n,
                                               w_p, w_q, static_cast<hipStream_t>(hip_stream))
                  : VTC_OK;
  vtc::CounterJob job{};
  if (charge)
    job = vtc::CounterJob{reinterpret_cast<unsigned long long*>(counters), num_clients, client_ids, n_input_tokens,
                          n_output_tokens, n, (unsigned long long)w_p, (unsigned long long)w_q};
  return decode_common(params, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace,
                       workspace_bytes, hip_stream, ev_begin, ev_end, job);
}

int vtc_step_decode(const vtc_attn_params* params, int32_t num_seqs, const void* q, const void* k_cache,
                    const void* v_cache, const int32_t* block_table, const int32_t* seq_lens, void* out,
                    int64_t* counters, int32_t num_clients, const int32_t* client_ids,
                    const int32_t* n_input_tokens, const int32_t* n_output_tokens, int32_t n, int64_t w_p,
                    int64_t w_q, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return vtc_step_decode_profiled(params, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, counters,
                                  num_clients, client_ids, n_input_tokens, n_output_tokens, n, w_p, w_q, workspace,
                                  workspace_bytes, hip_stream, nullptr, nullptr);
}

int vtc_attn_prefill_chunk(const vtc_attn_params* params, int32_t num_seqs, const void* q,
                           const int32_t* cu_q_lens, int32_t max_q_len, const void* k_cache,
                           const void* v_cache, const int32_t* block_table, const int32_t* seq_lens,
                           void* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  (void)workspace;
  (void)workspace_bytes;
  int rc = vtc::check_params(params);
  if (rc != VTC_OK) return rc;
  if (num_seqs < 0 || max_q_len < 0) return VTC_ERR_INVALID_ARG;
  if (num_seqs == 0 || max_q_len == 0) return VTC_OK;
  if (!q || !cu_q_lens || !k_cache || !v_cache || !block_table || !seq_lens || !out) return VTC_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(q) & 15u) || (reinterpret_cast<uintptr_t>(out) & 15u) ||
      (reinterpret_cast<uintptr_t>(k_cache) & 15u) || (reinterpret_cast<uintptr_t>(v_cache) & 15u))
    return VTC_ERR_INVALID_ARG;
  if (params->block_size != vtc::kBlockSize)
    return vtc::launch_attend_general(*params, num_seqs, q, cu_q_lens, max_q_len, k_cache, v_cache, block_table, seq_lens,
                                      out, static_cast<hipStream_t>(hip_stream));
  return vtc::launch_prefill(*params, num_seqs, q, cu_q_lens, max_q_len, k_cache, v_cache, block_table,
                             seq_lens, out, static_cast<hipStream_t>(hip_stream));
}

int vtc_counter_update(int64_t* counters, int32_t num_clients, const int32_t* client_ids,
                       const int32_t* n_input_tokens, const int32_t* n_output_tokens, int32_t n, int64_t w_p,
                       int64_t w_q, void* hip_stream) {
  if (n < 0 || num_clients < 0) return VTC_ERR_INVALID_ARG;
  if (n == 0) return VTC_OK;
  if (num_clients == 0) return VTC_OK;   // every id is out of range: nothing to charge
  if (!counters || !client_ids) return VTC_ERR_INVALID_ARG;
  return vtc::launch_counter_update(counters, num_clients, client_ids, n_input_tokens, n_output_tokens, n, w_p,
                                    w_q, static_cast<hipStream_t>(hip_stream));
}

int vtc_counter_update_cost(int64_t* counters, int32_t num_clients, const int32_t* client_ids,
                            const int32_t* n_p_old, const int32_t* n_q_old, const int32_t* n_p_new,
                            const int32_t* n_q_new, int32_t n, const vtc_cost_poly* h,
                            const int64_t* client_multiplier, void* hip_stream) {
  if (n < 0 || num_clients < 0 || !h) return VTC_ERR_INVALID_ARG;
  if (n == 0 || num_clients == 0) return VTC_OK;
  if (!counters || !client_ids || !n_p_old || !n_q_old || !n_p_new || !n_q_new) return VTC_ERR_INVALID_ARG;
  return vtc::launch_counter_update_cost(counters, num_clients, client_ids, n_p_old, n_q_old, n_p_new, n_q_new, n, *h,
                                         client_multiplier, static_cast<hipStream_t>(hip_stream));
}

int vtc_counter_update_predicted(int64_t* counters, int32_t num_clients, const int32_t* client_ids,
                                 const int32_t* n_output, const int32_t* n_predicted, const int32_t* finished,
                                 int32_t n, int64_t w_q, void* hip_stream) {
  if (n < 0 || num_clients < 0) return VTC_ERR_INVALID_ARG;
  if (n == 0 || num_clients == 0) return VTC_OK;
  if (!counters || !client_ids || !n_output || !n_predicted || !finished) return VTC_ERR_INVALID_ARG;
  return vtc::launch_counter_update_predicted(counters, num_clients, client_ids, n_output, n_predicted, finished, n,
                                              w_q, static_cast<hipStream_t>(hip_stream));
}

int vtc_kv_append(const vtc_attn_params* params, int32_t num_seqs, const void* k_new, const void* v_new,
                  const int32_t* cu_new_lens, int32_t max_new_len, void* k_cache, void* v_cache,
                  const int32_t* block_table, const int32_t* seq_lens, void* hip_stream) {
  int rc = vtc::check_params(params);
  if (rc != VTC_OK) return rc;
  if (num_seqs < 0 || max_new_len < 0) return VTC_ERR_INVALID_ARG;
  if (num_seqs == 0 || max_new_len == 0) return VTC_OK;
  if (!k_new || !v_new || !cu_new_lens || !k_cache || !v_cache || !block_table || !seq_lens) return VTC_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(k_new) & 15u) || (reinterpret_cast<uintptr_t>(v_new) & 15u) ||
      (reinterpret_cast<uintptr_t>(k_cache) & 15u) || (reinterpret_cast<uintptr_t>(v_cache) & 15u))
    return VTC_ERR_INVALID_ARG;
  return vtc::launch_kv_append(*params, num_seqs, k_new, v_new, cu_new_lens, max_new_len, k_cache, v_cache,
                               block_table, seq_lens, static_cast<hipStream_t>(hip_stream));
}

int vtc_debug_gather_slots(const vtc_attn_params* params, int32_t num_seqs, const int32_t* block_table,
                           const int32_t* seq_lens, const int32_t* cu_out, int32_t max_seq_len,
                           int32_t* slots_out, void* hip_stream) {
  int rc = vtc::check_params(params);
  if (rc != VTC_OK) return rc;
  if (num_seqs < 0 || max_seq_len < 0) return VTC_ERR_INVALID_ARG;
  if (num_seqs == 0 || max_seq_len == 0) return VTC_OK;
  if (!block_table || !seq_lens || !cu_out || !slots_out) return VTC_ERR_INVALID_ARG;
  return vtc::launch_gather_slots(*params, num_seqs, block_table, seq_lens, cu_out, max_seq_len, slots_out,
                                  static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
