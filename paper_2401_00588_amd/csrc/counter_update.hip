// Virtual-token-counter charges: segmented int64 reductions keyed by client id.
//
// Algorithm 2 of the paper charges w_p * input_length(r) at admission and w_q per
// running request after each decode step; with the weighted-token cost of
// Section 3.1 both are  counters[client(r)] += w_p * n_p(r) + w_q * n_q(r).
// Algorithm 4 generalises the charge to the increase of a cost function h(n_p, n_q)
// (Section 4.2), weighted VTC scales a client's increment (Section 4.3), and
// Algorithm 3 replaces the per-step charge by a prediction-aware adjustment
// (Section 4.4).  All of them are the same reduction with a different per-request term.
//
// Each workgroup reduces its slice of the requests into an LDS table (one int64
// per client, LDS atomics), then adds the non-zero entries to the global
// counters with 64-bit integer atomics.  Integer addition is associative, so
// the result is the same for every execution order.  Client tables larger than
// the LDS table fall back to global atomics per request.  Arithmetic is done on
// unsigned 64-bit values, i.e. exact two's-complement wrap-around.
#include "counter_terms.h"

namespace vtc {

constexpr int kCounterThreads = 256;
constexpr int kLdsClients = 4096;              // 32 KiB of int64
constexpr int kRequestsPerWorkgroup = 4096;

template <typename Term>
__global__ __launch_bounds__(kCounterThreads) void counter_reduce_kernel(u64* __restrict__ counters,
                                                                         int32_t num_clients,
                                                                         const int32_t* __restrict__ client_ids,
                                                                         int32_t n, Term term) {
  __shared__ u64 table[kLdsClients];
  const int begin = blockIdx.x * kRequestsPerWorkgroup;
  counter_reduce_slice<kCounterThreads, kLdsClients>(table, counters, num_clients, client_ids, begin,
                                                     min(n, begin + kRequestsPerWorkgroup), term, threadIdx.x);
}

template <typename Term>
static int launch_reduce(int64_t* counters, int32_t num_clients, const int32_t* client_ids, int32_t n, Term term,
                         hipStream_t stream) {
  const int grid = (n + kRequestsPerWorkgroup - 1) / kRequestsPerWorkgroup;
  hipLaunchKernelGGL(counter_reduce_kernel<Term>, dim3(grid), dim3(kCounterThreads), 0, stream,
                     reinterpret_cast<u64*>(counters), num_clients, client_ids, n, term);
  return hipGetLastError() == hipSuccess ? VTC_OK : VTC_ERR_HIP;
}

int launch_counter_update(int64_t* counters, int32_t num_clients, const int32_t* client_ids, const int32_t* n_in,
                          const int32_t* n_out, int32_t n, int64_t w_p, int64_t w_q, hipStream_t stream) {
  return launch_reduce(counters, num_clients, client_ids, n, LinearTerm{n_in, n_out, (u64)w_p, (u64)w_q}, stream);
}

int launch_counter_update_cost(int64_t* counters, int32_t num_clients, const int32_t* client_ids,
                               const int32_t* p_old, const int32_t* q_old, const int32_t* p_new,
                               const int32_t* q_new, int32_t n, const vtc_cost_poly& h,
                               const int64_t* client_multiplier, hipStream_t stream) {
  return launch_reduce(counters, num_clients, client_ids, n,
                       CostTerm{p_old, q_old, p_new, q_new, client_multiplier, (u64)h.c0, (u64)h.cp, (u64)h.cq,
                                (u64)h.cpp, (u64)h.cpq, (u64)h.cqq},
                       stream);
}

int launch_counter_update_predicted(int64_t* counters, int32_t num_clients, const int32_t* client_ids,
                                    const int32_t* n_output, const int32_t* n_predicted, const int32_t* finished,
                                    int32_t n, int64_t w_q, hipStream_t stream) {
  return launch_reduce(counters, num_clients, client_ids, n, PredictedTerm{n_output, n_predicted, finished, (u64)w_q},
                       stream);
}

}  // namespace vtc
