/*
 * vtc.h -- C ABI of the MI355X (gfx950) hot path of one Virtual Token Counter
 * serving step: paged-KV decode attention, causal prefill-chunk attention and
 * the per-client virtual-token-counter charge.
 *
 * Paper: "Fairness in Serving Large Language Models" (arXiv 2401.00588).
 * One iteration of the execution stream of Algorithm 2 calls
 *     (new tokens' K/V into the cache)  ->  vtc_kv_append
 *     forward_prefill(B_new)            ->  vtc_attn_prefill_chunk   (attention part)
 *     forward_decode(B)                 ->  vtc_attn_decode          (attention part)
 *     c_i += ...                        ->  vtc_counter_update
 *     the last two in one call          ->  vtc_step_decode
 * and the variants of the charge: vtc_counter_update_cost (Algorithm 4, general cost function;
 * weighted VTC), vtc_counter_update_predicted (Algorithm 3, length prediction).
 * The paper names a paged KV cache as its substrate (Section 5.1) and gives no
 * attention formula; the kernels compute standard scaled dot-product softmax
 * attention (see each entry point).
 *
 * Conventions
 *   - Every pointer marked [device] is a device pointer valid on the current
 *     HIP device; [host] pointers are ordinary host memory.
 *   - The caller owns every buffer (including workspace and counters).  The
 *     library allocates no device memory and never frees caller memory.
 *   - Calls enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL
 *     is the default stream) and return without synchronising; results are
 *     valid once the caller has synchronised that stream.
 *   - Return value: VTC_OK (0) or a negative VTC_ERR_* code.  Arguments that
 *     are visible on the host are validated before any HIP call is made, so
 *     every error path below can be exercised on a machine without a GPU.
 *     Device-resident contents (seq_lens, block_table, client_ids, ...) are
 *     trusted, except where a clamp is documented.
 *
 * Layouts (row-major, last index fastest; E = 2-byte element, fp16 or bf16;
 * O = the element type named by out_dtype: E, or 4-byte float)
 *   q             E [num_q_tokens, num_q_heads, head_dim]
 *   out           O [num_q_tokens, num_q_heads, head_dim]
 *   k_cache,
 *   v_cache       E [num_blocks, num_kv_heads, block_size, head_dim]
 *   block_table   int32 [num_seqs, max_blocks_per_seq]   physical block ids
 *   seq_lens      int32 [num_seqs]
 * Token p of sequence r lives in block block_table[r][p / block_size], row
 * p % block_size.  Query head h reads KV head h / (num_q_heads/num_kv_heads).
 *
 * Block sizes.  The kernels are built for blocks of 16 tokens: a (block, kv head)
 * tile is then 4 KiB of contiguous K and of V.  The paper's own system pages its
 * cache one token at a time (Section 5.1); block sizes 1, 2, 4 and 8 are served by
 * the same entry points through a general path (one wavefront per sequence and KV
 * head, 16 tokens gathered through the block table at a time) with the same
 * results and error behaviour.  That path runs at 60-80 % of the tuned one's
 * rate, takes no workspace (the workspace arguments are ignored) and makes
 * vtc_step_decode launch its charge separately.
 */
#ifndef VTC_H_
#define VTC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { VTC_F16 = 0, VTC_BF16 = 1, VTC_F32 = 2 /* output rows only */ } vtc_dtype;

enum {
  VTC_OK = 0,
  VTC_ERR_INVALID_ARG = -1,         /* null pointer, negative size, inconsistent sizes   */
  VTC_ERR_UNSUPPORTED = -2,         /* head_dim != 128, block_size not 1/2/4/8/16, unknown dtype,
                                       out_dtype neither dtype nor VTC_F32,
                                       num_q_heads/num_kv_heads not in {1,2,4,8}          */
  VTC_ERR_WORKSPACE_TOO_SMALL = -3, /* workspace_bytes < vtc_attn_workspace_bytes(...)   */
  VTC_ERR_HIP = -4,                 /* a HIP runtime call or kernel launch failed        */
  VTC_ERR_STATIC_LIMIT = -5         /* vtc_attn_decode_static: more sequences than its
                                       built-in scratch array is laid out for             */
};

/* Host struct, passed by const pointer; never retained by the library. */
typedef struct {
  int32_t num_q_heads;        /* Hq                                              */
  int32_t num_kv_heads;       /* Hkv, must divide Hq                             */
  int32_t head_dim;           /* 128                                             */
  int32_t block_size;         /* tokens per KV block: 16 (the tuned kernels), or 1,
                                 2, 4, 8 (a general path, see below)             */
  int32_t max_blocks_per_seq; /* row stride of block_table                       */
  int32_t dtype;              /* vtc_dtype of q, k_cache and v_cache: F16 or BF16 */
  float scale;                /* logit scale, normally 1/sqrt(head_dim)          */
  int32_t out_dtype;          /* vtc_dtype of out: equal to dtype (the fp32 result
                                 is rounded to nearest even), or VTC_F32 (the fp32
                                 result as it stands, no final rounding)          */
} vtc_attn_params;

/*
 * Bytes of device workspace with which vtc_attn_decode can put every wave to use
 * that the current device holds at once, for up to max_num_seqs sequences of up
 * to max_seq_len context tokens each (max_seq_len <= 0, or larger than the block
 * table can address, means max_blocks_per_seq * block_size).  The footprint is a
 * fixed part plus a share per wave (two fp32 partial results per query head of a
 * group), and short batches cannot use many waves, so it grows with
 * max_num_seqs * max_seq_len until the device's wave count caps it (2 to 9 MB
 * on 256 compute units, depending on num_q_heads / num_kv_heads).  Host arithmetic plus one query of the current device's
 * compute-unit count (256 is assumed when there is no usable device).  Returns 0
 * if params is NULL or unsupported.  vtc_attn_prefill_chunk needs no workspace.
 */
size_t vtc_attn_workspace_bytes(const vtc_attn_params* params /*[host]*/, int32_t max_num_seqs,
                                int32_t max_seq_len);

/*
 * Decode attention -- the attention part of forward_decode(B) in Algorithm 2
 * (one new token per running request, Section 2.1 "decoding").
 *
 * For each sequence r < num_seqs and query head h:
 *     out[r,h,:] = sum_j softmax_j(scale * <q[r,h,:], K_j>) * V_j,  j in [0, seq_lens[r])
 * over the cached tokens of KV head h / (Hq/Hkv).  The K/V of the current
 * token must already be in the cache (seq_lens includes it).  Accumulation is
 * fp32; out is rounded to out_dtype (nearest even; no rounding for VTC_F32).  seq_lens[r] == 0
 * gives an all-zero row.  seq_lens[r] is clamped to max_blocks_per_seq *
 * block_size.  Rows of the last block past seq_lens[r], and block_table
 * entries past the last block, are never used (they may hold anything).
 *
 *   q [device]          E [num_seqs, Hq, 128]
 *   k_cache, v_cache    [device] paged caches, read only
 *   block_table         [device] int32 [num_seqs, max_blocks_per_seq]
 *   seq_lens            [device] int32 [num_seqs]
 *   out [device]        O [num_seqs, Hq, 128], written
 *   workspace [device]  256-byte aligned, contents undefined before and after.
 *                       vtc_attn_workspace_bytes(params, num_seqs, L) bytes serve
 *                       contexts of up to L tokens at full speed; the call uses as
 *                       many waves as workspace_bytes has room for, so a smaller
 *                       workspace gives the same results more slowly, and
 *                       VTC_ERR_WORKSPACE_TOO_SMALL only if not even one wave fits
 *                       (vtc_attn_workspace_bytes(params, num_seqs, 1) always does).
 * num_seqs == 0 is a successful no-op.  The call enqueues the attention kernel
 * and a merge kernel on hip_stream (batches of more than 1024 sequences: a
 * planning kernel first); two calls that share one workspace must be ordered on
 * the same stream.  It allocates nothing, never synchronises and keeps no state
 * between calls, so it may be captured into a HIP graph.  On VTC_ERR_HIP the
 * contents of out are undefined.
 */
int vtc_attn_decode(const vtc_attn_params* params /*[host]*/, int32_t num_seqs, const void* q,
                    const void* k_cache, const void* v_cache, const int32_t* block_table,
                    const int32_t* seq_lens, void* out, void* workspace, size_t workspace_bytes,
                    void* hip_stream);

/*
 * vtc_attn_decode for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and error behaviour as
 * vtc_attn_decode, except that the workspace is a 10 MiB device array inside the
 * library image (every device the library runs on holds its own copy until the
 * process ends).  The call allocates and frees nothing.
 *   - num_seqs may be at most 65536; more returns VTC_ERR_STATIC_LIMIT.  10 MiB
 *     hold the full wave count of a 256-compute-unit device for every supported
 *     shape; on a larger device the launch uses the waves that fit.
 *   - Every call on a device shares that device's array: calls that overlap on
 *     one device (different streams, different threads) race.  Order them on one
 *     stream.  The array keeps the last call's contents; nothing in it has to be
 *     cleared between calls.
 *   - The first call on a device looks up the array's address (a HIP runtime
 *     query, no allocation); make it outside any stream capture.
 */
int vtc_attn_decode_static(const vtc_attn_params* params /*[host]*/, int32_t num_seqs, const void* q,
                           const void* k_cache, const void* v_cache, const int32_t* block_table,
                           const int32_t* seq_lens, void* out, void* hip_stream);

/*
 * Measurement hook: exactly vtc_attn_decode, and in addition records the HIP
 * events ev_begin / ev_end (hipEvent_t passed as void*, created by the caller
 * with timing enabled) on hip_stream immediately before and after the attention
 * kernel proper, i.e. excluding the planning and merge kernels.  Either event
 * may be NULL.  Used by the benchmark to time the HBM-bound kernel of the decode
 * step (Algorithm 2, forward_decode) by itself.
 */
int vtc_attn_decode_profiled(const vtc_attn_params* params /*[host]*/, int32_t num_seqs, const void* q,
                             const void* k_cache, const void* v_cache, const int32_t* block_table,
                             const int32_t* seq_lens, void* out, void* workspace,
                             size_t workspace_bytes, void* hip_stream, void* ev_begin, void* ev_end);

/*
 * One decode iteration of the execution stream of Algorithm 2 in a single call:
 * forward_decode(B) (its attention part, exactly vtc_attn_decode) followed by
 * the counter charge c_i += w_p * n_input_tokens + w_q * n_output_tokens summed
 * over the requests of client i (exactly vtc_counter_update, declared below;
 * for a pure decode step n_output_tokens is all ones and n_input_tokens NULL,
 * i.e. c_i += w_q * |{r in B : client(r) = i}|).  The charge travels in the
 * last launch of the attention, so the step costs no extra kernel launch.
 *
 * The two halves have separate request lists: attention runs over num_seqs
 * sequences, the charge over n requests (a mixed step also charges the requests
 * that were prefilled in the same iteration).  Arguments, layouts, clamping and
 * error behaviour of each half are those of vtc_attn_decode and
 * vtc_counter_update; all host-visible arguments of both halves are validated
 * before anything is enqueued.  num_seqs == 0 performs the charge alone; n == 0
 * or num_clients == 0 performs the attention alone.  The charge is not ordered
 * against the attention inside the call; both are complete when the work
 * enqueued by the call on hip_stream is.
 */
int vtc_step_decode(const vtc_attn_params* params /*[host]*/, int32_t num_seqs, const void* q,
                    const void* k_cache, const void* v_cache, const int32_t* block_table,
                    const int32_t* seq_lens, void* out, int64_t* counters, int32_t num_clients,
                    const int32_t* client_ids, const int32_t* n_input_tokens,
                    const int32_t* n_output_tokens, int32_t n, int64_t w_p, int64_t w_q, void* workspace,
                    size_t workspace_bytes, void* hip_stream);

/* Measurement hook: vtc_step_decode with the two events of vtc_attn_decode_profiled. */
int vtc_step_decode_profiled(const vtc_attn_params* params /*[host]*/, int32_t num_seqs, const void* q,
                             const void* k_cache, const void* v_cache, const int32_t* block_table,
                             const int32_t* seq_lens, void* out, int64_t* counters, int32_t num_clients,
                             const int32_t* client_ids, const int32_t* n_input_tokens,
                             const int32_t* n_output_tokens, int32_t n, int64_t w_p, int64_t w_q,
                             void* workspace, size_t workspace_bytes, void* hip_stream, void* ev_begin,
                             void* ev_end);

/*
 * Causal prefill-chunk attention -- the attention part of forward_prefill(B_new)
 * in Algorithm 2 (Section 2.1 "prefilling"), for one chunk of each newly
 * admitted prompt.  Chunking is this library's batching unit; the paper
 * prefills whole prompts, which is the single-chunk case.
 *
 * Sequence r contributes Lq_r = cu_q_lens[r+1] - cu_q_lens[r] query tokens,
 * stored at rows cu_q_lens[r] .. cu_q_lens[r+1]-1 of q and out.  seq_lens[r]
 * is its context length AFTER the chunk's K/V were appended to the cache, so
 * chunk token i sits at absolute position p = seq_lens[r] - Lq_r + i and
 * attends to cached tokens 0..p inclusive:
 *     out[row,h,:] = sum_{j<=p} softmax_j(scale * <q[row,h,:], K_j>) * V_j
 * fp32 accumulation, output rounded to out_dtype.  The softmax weights enter the
 * P*V product as matrix-core operands of the storage type: fp16 weights with
 * their 11 significant bits, bf16 weights as two operands (the rounded weight
 * and what the rounding dropped), i.e. with 16 significant bits.
 * A sequence whose seq_lens[r] (clamped to 0 .. max_blocks_per_seq * block_size)
 * is smaller than Lq_r has no positions for its chunk tokens: all its output
 * rows are zero and no cache block is read for it (its block_table row may hold
 * anything).
 *
 *   q [device]          E [total_q_tokens, Hq, 128], total_q_tokens = cu_q_lens[num_seqs]
 *   cu_q_lens [device]  int32 [num_seqs + 1], non-decreasing, cu_q_lens[0] == 0
 *   max_q_len           host-side upper bound on every Lq_r (sizes the launch)
 *   seq_lens [device]   int32 [num_seqs], seq_lens[r] >= Lq_r (see above for the other case)
 *   out [device]        O [total_q_tokens, Hq, 128], written
 *   workspace           unused, may be NULL
 * num_seqs == 0 or max_q_len == 0 is a successful no-op.
 */
int vtc_attn_prefill_chunk(const vtc_attn_params* params /*[host]*/, int32_t num_seqs,
                           const void* q, const int32_t* cu_q_lens, int32_t max_q_len,
                           const void* k_cache, const void* v_cache, const int32_t* block_table,
                           const int32_t* seq_lens, void* out, void* workspace,
                           size_t workspace_bytes, void* hip_stream);

/*
 * Virtual-token-counter charge (Algorithm 2: admission charge
 * c_k += w_p * input_length(r), and decode charge
 * c_i += w_q * |{r in B : client(r) = i}|; Algorithm 4 states both as "when new
 * tokens have been processed" with the weighted-token cost of Section 3.1):
 *     counters[client_ids[r]] += w_p * n_input_tokens[r] + w_q * n_output_tokens[r]
 * for every r < n, as exact two's-complement int64 arithmetic (the result does
 * not depend on the order of summation).  Either token array may be NULL,
 * meaning all zero.  Requests whose client id is outside [0, num_clients) are
 * ignored.  Token counts may be negative (a refund).
 *
 *   counters [device]         int64 [num_clients], updated in place
 *   client_ids [device]       int32 [n]
 *   n_input_tokens [device]   int32 [n] or NULL
 *   n_output_tokens [device]  int32 [n] or NULL
 * n == 0 is a successful no-op.
 */
int vtc_counter_update(int64_t* counters, int32_t num_clients, const int32_t* client_ids,
                       const int32_t* n_input_tokens, const int32_t* n_output_tokens, int32_t n,
                       int64_t w_p, int64_t w_q, void* hip_stream);

/*
 * Integer (fixed-point) cost polynomial
 *     h(n_p, n_q) = c0 + cp*n_p + cq*n_q + cpp*n_p^2 + cpq*n_p*n_q + cqq*n_q^2
 * for the general cost function of Section 4.2.  The weighted-token cost of Section 3.1 is
 * {0, w_p, w_q, 0, 0, 0}; the profiled cost printed in Appendix B.2,
 * 2.1 n_p + n_q + 0.04 n_p n_q + 0.032 n_q^2 + 11.46, is {11460, 2100, 1000, 0, 40, 32} in units of 1/1000.
 */
typedef struct {
  int64_t c0, cp, cq, cpp, cpq, cqq;
} vtc_cost_poly;

/*
 * General VTC counter update (Algorithm 4: "when new tokens have been processed",
 * c_i += sum over the client's requests of h(n_p, n_q) - h(n_p(old), n_q(old)); Section 4.2
 * gives the two instances used by Algorithm 2: h(n_p, 0) at admission and
 * h(n_p, n_q) - h(n_p, n_q - 1) per decode step):
 *     counters[client_ids[r]] += (h(n_p_new[r], n_q_new[r]) - old_r) * mult
 * with old_r = 0 if n_p_old[r] == n_q_old[r] == 0 (none of the request's tokens processed yet, so the
 * first update charges h(n_p, 0) in full, constant term included) and h(n_p_old[r], n_q_old[r])
 * otherwise; mult = client_multiplier[client_ids[r]], or 1 if client_multiplier is NULL.  The
 * multiplier expresses weighted VTC (Section 4.3) exactly: dividing client i's increment by its
 * weight w_i is multiplying it by W / w_i for a common multiple W of the weights.
 * Exact two's-complement int64 arithmetic, independent of summation order; client ids outside
 * [0, num_clients) are ignored.
 *
 *   counters [device]           int64 [num_clients], updated in place
 *   client_ids [device]         int32 [n]
 *   n_p_old, n_q_old,
 *   n_p_new, n_q_new [device]   int32 [n], processed input / output tokens before and after
 *   h [host]                    cost polynomial
 *   client_multiplier [device]  int64 [num_clients] or NULL
 * n == 0 is a successful no-op.
 */
int vtc_counter_update_cost(int64_t* counters, int32_t num_clients, const int32_t* client_ids,
                            const int32_t* n_p_old, const int32_t* n_q_old, const int32_t* n_p_new,
                            const int32_t* n_q_new, int32_t n, const vtc_cost_poly* h /*[host]*/,
                            const int64_t* client_multiplier, void* hip_stream);

/*
 * Per-step counter adjustment of VTC with length prediction (Algorithm 3, the loop after
 * forward_decode; Section 4.4).  At admission the caller has charged
 * w_p * input_len + w_q * predicted_output_len with vtc_counter_update.  After each decode step,
 * for every running request r, with delta = n_output[r] - n_predicted[r] (n_output counts the token
 * just generated):
 *     delta > 0                    : counters[client] += w_q          (prediction used up)
 *     finished[r] != 0 and delta<0 : counters[client] += w_q * delta  (refund of the unused part)
 * so that a finished request has paid w_p*n_p + w_q*n_q whatever was predicted.
 * Exact int64 arithmetic; client ids outside [0, num_clients) are ignored.
 *
 *   counters [device]     int64 [num_clients], updated in place
 *   client_ids, n_output, n_predicted, finished [device]   int32 [n]
 * n == 0 is a successful no-op.
 */
int vtc_counter_update_predicted(int64_t* counters, int32_t num_clients, const int32_t* client_ids,
                                 const int32_t* n_output, const int32_t* n_predicted,
                                 const int32_t* finished, int32_t n, int64_t w_q, void* hip_stream);

/*
 * Append newly processed tokens to the paged cache -- the step that precedes the attention
 * calls above, which expect the current token / chunk to be cached already (Algorithm 2 runs
 * forward_prefill and forward_decode on the running batch's KV memory pool).
 *
 * Sequence r contributes n_r = cu_new_lens[r+1] - cu_new_lens[r] tokens, stored at rows
 * cu_new_lens[r] .. of k_new / v_new.  seq_lens[r] is the context length AFTER the append
 * (the value the attention call will be given): new token i gets position
 * p = seq_lens[r] - n_r + i and is written to block block_table[r][p / block_size], row
 * p % block_size, of every KV head.  Bit-exact copy.  The blocks must be allocated by the caller.
 *
 *   k_new, v_new [device]   E [total_new_tokens, num_kv_heads, 128]
 *   cu_new_lens [device]    int32 [num_seqs + 1], cu_new_lens[0] == 0
 *   max_new_len             host-side upper bound on every n_r (sizes the launch)
 *   k_cache, v_cache        [device] paged caches, written
 *   block_table, seq_lens   [device] as for the attention calls
 * num_seqs == 0 or max_new_len == 0 is a successful no-op.
 */
int vtc_kv_append(const vtc_attn_params* params /*[host]*/, int32_t num_seqs, const void* k_new,
                  const void* v_new, const int32_t* cu_new_lens, int32_t max_new_len, void* k_cache,
                  void* v_cache, const int32_t* block_table, const int32_t* seq_lens,
                  void* hip_stream);

/*
 * Test hook for the paged-cache index arithmetic: writes, for every sequence r
 * and position p < seq_lens[r], the physical slot
 *     slot(r,p) = block_table[r][p / block_size] * block_size + p % block_size
 * to slots_out[cu_out[r] + p].  cu_out [device] int32 [num_seqs+1] are the
 * exclusive prefix sums of seq_lens; max_seq_len is a host-side upper bound on
 * seq_lens (sizes the launch).  The attention kernels address whole blocks
 * (block_table[r][b] times the block stride), which is this formula at
 * p = b * block_size; vtc_kv_append and the general path for small blocks address
 * single rows with it.
 */
int vtc_debug_gather_slots(const vtc_attn_params* params /*[host]*/, int32_t num_seqs,
                           const int32_t* block_table, const int32_t* seq_lens,
                           const int32_t* cu_out, int32_t max_seq_len, int32_t* slots_out,
                           void* hip_stream);

/* Static, NUL-terminated description of a return code.  Never NULL. */
const char* vtc_strerror(int code);

/* Library version as major*10000 + minor*100 + patch. */
int vtc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* VTC_H_ */
