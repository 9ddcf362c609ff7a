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
#include "vtc_internal.h"

namespace vtc {

constexpr int kCounterThreads = 256;
constexpr int kLdsClients = 4096;              // 32 KiB of int64
constexpr int kRequestsPerWorkgroup = 4096;

using u64 = unsigned long long;

// ---- per-request terms -------------------------------------------------------
struct LinearTerm {                            // w_p * n_p + w_q * n_q
  const int32_t* __restrict__ n_in;
  const int32_t* __restrict__ n_out;
  u64 w_p, w_q;
  __device__ __forceinline__ u64 operator()(int r, int) const {
    const long long np = n_in ? (long long)n_in[r] : 0ll;
    const long long nq = n_out ? (long long)n_out[r] : 0ll;
    return w_p * (u64)np + w_q * (u64)nq;
  }
};

struct CostTerm {                              // (h(new) - h(old)) * multiplier[client]
  const int32_t* __restrict__ p_old;
  const int32_t* __restrict__ q_old;
  const int32_t* __restrict__ p_new;
  const int32_t* __restrict__ q_new;
  const int64_t* __restrict__ multiplier;      // may be null
  u64 c0, cp, cq, cpp, cpq, cqq;
  __device__ __forceinline__ u64 h(long long np, long long nq) const {
    const u64 p = (u64)np, q = (u64)nq;
    return c0 + cp * p + cq * q + cpp * p * p + cpq * p * q + cqq * q * q;
  }
  __device__ __forceinline__ u64 operator()(int r, int client) const {
    const long long po = p_old[r], qo = q_old[r];
    // a request none of whose tokens has been processed has cost 0, not h(0, 0)
    const u64 old_cost = (po == 0 && qo == 0) ? 0ull : h(po, qo);
    u64 delta = h(p_new[r], q_new[r]) - old_cost;
    if (multiplier) delta *= (u64)multiplier[client];
    return delta;
  }
};

struct PredictedTerm {                         // Algorithm 3, "adjust the cost of output tokens"
  const int32_t* __restrict__ n_output;
  const int32_t* __restrict__ n_predicted;
  const int32_t* __restrict__ finished;
  u64 w_q;
  __device__ __forceinline__ u64 operator()(int r, int) const {
    const long long delta = (long long)n_output[r] - (long long)n_predicted[r];
    u64 add = 0ull;
    if (delta > 0) add += w_q;                                   // prediction used up: pay per token
    if (finished[r] != 0 && delta < 0) add += w_q * (u64)delta;  // refund the unused pre-payment
    return add;
  }
};

template <typename Term>
__global__ __launch_bounds__(kCounterThreads) void counter_reduce_kernel(u64* __restrict__ counters,
                                                                         int32_t num_clients,
                                                                         const int32_t* __restrict__ client_ids,
                                                                         int32_t n, Term term) {
  __shared__ u64 table[kLdsClients];
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
    const u64 delta = term(r, c);
    if (delta == 0ull) continue;
    if (use_lds)
      atomicAdd(&table[c], delta);
    else
      atomicAdd(&counters[c], delta);
  }
  if (use_lds) {
    __syncthreads();
    for (int i = threadIdx.x; i < num_clients; i += kCounterThreads) {
      const u64 d = table[i];
      if (d != 0ull) atomicAdd(&counters[i], d);
    }
  }
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
