// Virtual-token-counter charge: a segmented int64 reduction keyed by client id.
//
// Algorithm 2 of the paper charges w_p * input_length(r) at admission and
// w_q per running request after each decode step; with the weighted-token cost
// of Section 3.1 both are  counters[client(r)] += w_p * n_p(r) + w_q * n_q(r).
//
// Each workgroup reduces its slice of the requests into an LDS table (one int64
// per client, LDS atomics), then adds the non-zero entries to the global
// counters with 64-bit integer atomics.  Integer addition is associative, so
// the result is the same for every execution order.  Client tables larger than
// the LDS table fall back to global atomics per request.
#include "vtc_internal.h"

namespace vtc {

constexpr int kCounterThreads = 256;
constexpr int kLdsClients = 4096;              // 32 KiB of int64
constexpr int kRequestsPerWorkgroup = 4096;

__global__ __launch_bounds__(kCounterThreads) void counter_update_kernel(
    unsigned long long* __restrict__ counters, int32_t num_clients, const int32_t* __restrict__ client_ids,
    const int32_t* __restrict__ n_in, const int32_t* __restrict__ n_out, int32_t n, long long w_p, long long w_q) {
  __shared__ unsigned long long table[kLdsClients];
  const bool use_lds = num_clients <= kLdsClients;
  if (use_lds) {
    for (int i = threadIdx.x; i < num_clients; i += kCounterThreads) table[i] = 0ull;
    __syncthreads();
  }
  const int begin = blockIdx.x * kRequestsPerWorkgroup;
  const int end = min(n, begin + kRequestsPerWorkgroup);
  for (int r = begin + (int)threadIdx.x; r < end; r += kCounterThreads) {
    const int32_t c = client_ids[r];
    if (c < 0 || c >= num_clients) continue;
    const long long np = n_in ? (long long)n_in[r] : 0ll;
    const long long nq = n_out ? (long long)n_out[r] : 0ll;
    // two's-complement wrap-around arithmetic, done unsigned to keep it defined
    const unsigned long long delta =
        (unsigned long long)w_p * (unsigned long long)np + (unsigned long long)w_q * (unsigned long long)nq;
    if (delta == 0ull) continue;
    if (use_lds)
      atomicAdd(&table[c], delta);
    else
      atomicAdd(&counters[c], delta);
  }
  if (use_lds) {
    __syncthreads();
    for (int i = threadIdx.x; i < num_clients; i += kCounterThreads) {
      const unsigned long long d = table[i];
      if (d != 0ull) atomicAdd(&counters[i], d);
    }
  }
}

int launch_counter_update(int64_t* counters, int32_t num_clients, const int32_t* client_ids, const int32_t* n_in,
                          const int32_t* n_out, int32_t n, int64_t w_p, int64_t w_q, hipStream_t stream) {
  const int grid = (n + kRequestsPerWorkgroup - 1) / kRequestsPerWorkgroup;
  hipLaunchKernelGGL(counter_update_kernel, dim3(grid), dim3(kCounterThreads), 0, stream,
                     reinterpret_cast<unsigned long long*>(counters), num_clients, client_ids, n_in, n_out, n,
                     (long long)w_p, (long long)w_q);
  return hipGetLastError() == hipSuccess ? VTC_OK : VTC_ERR_HIP;
}

}  // namespace vtc
