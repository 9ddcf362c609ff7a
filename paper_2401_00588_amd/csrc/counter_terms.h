// Per-request terms of the virtual-token-counter charges and the workgroup-level reduction that
// applies them.  Shared by the stand-alone counter kernels and by the decode step that carries a
// counter update in its last launch.
//
// Algorithm 2 of the paper charges w_p * input_length(r) at admission and w_q per running request
// after each decode step (Section 3.1: cost w_p * n_p + w_q * n_q); Algorithm 4 charges the increase
// of a cost function h(n_p, n_q) (Section 4.2); weighted VTC scales a client's increment
// (Section 4.3); Algorithm 3 adjusts for a predicted output length (Section 4.4).
#pragma once

#include "vtc_internal.h"

namespace vtc {

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

struct PredictedTerm {                         // per-step adjustment under length prediction (Section 4.4)
  const int32_t* __restrict__ n_output;
  const int32_t* __restrict__ n_predicted;
  const int32_t* __restrict__ finished;
  u64 w_q;
  // The predicted tokens were paid for at admission.  A token beyond the prediction costs w_q when it is
  // generated; a request that ends short of its prediction gets the unused part back, w_q per token.
  __device__ __forceinline__ u64 operator()(int r, int) const {
    const long long beyond = (long long)n_output[r] - (long long)n_predicted[r];      // > 0: prediction used up
    const long long tokens = (beyond > 0 ? 1ll : 0ll) + ((finished[r] != 0 && beyond < 0) ? beyond : 0ll);
    return w_q * (u64)tokens;
  }
};

// One workgroup of kThreads threads charges requests [begin, end): per-client sums in an LDS table
// (LDS atomics), then one 64-bit global atomic per client that received something.  Client tables
// larger than kTable go to global atomics per request.  Unsigned 64-bit arithmetic, i.e. exact
// two's-complement wrap-around; integer addition is associative, so any order gives the same counters.
// `tid` is the thread's index among the kThreads of the workgroup (which need not be one-dimensional).
template <int kThreads, int kTable, typename Term>
__device__ __forceinline__ void counter_reduce_slice(u64* __restrict__ table, u64* __restrict__ counters,
                                                     int32_t num_clients, const int32_t* __restrict__ client_ids,
                                                     int begin, int end, const Term& term, int tid) {
  const bool use_lds = num_clients <= kTable;
  if (use_lds) {
    for (int i = tid; i < num_clients; i += kThreads) table[i] = 0ull;
    __syncthreads();
  }
  for (int r = begin + tid; r < end; r += kThreads) {
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
    for (int i = tid; i < num_clients; i += kThreads) {
      const u64 d = table[i];
      if (d != 0ull) atomicAdd(&counters[i], d);
    }
  }
}

}  // namespace vtc
