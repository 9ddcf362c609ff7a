// Internal helpers shared by the gfx950 kernels of the VTC serving step.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "vtc.h"

namespace vtc {

constexpr int kHeadDim = 128;       // the only supported head_dim
constexpr int kBlockSize = 16;      // tokens per KV block of the tuned kernels (smaller powers of two: general path)
constexpr int kWave = 64;           // CDNA wavefront
constexpr int kTileElems = kBlockSize * kHeadDim;   // elements of one (block, kv head) K or V tile
constexpr float kLog2e = 1.4426950408889634f;

// Decode attention cuts the batch's stream of KV blocks into one range per resident wave.
// Waves launched per compute unit.  Four already saturate the memory system; with many more, the waves
// dispatched last progress so much more slowly than the first that the end of the launch drags (measured: one
// query head per KV head, 64 and 256 sequences: 8 per CU 1.5 % faster than 16; grouped queries, 256 and 512
// sequences: 4 per CU 1.5 % faster than 8).
constexpr int kDecodeWavesPerCuMha = 8;      // num_q_heads == num_kv_heads (vector-ALU engine)
constexpr int kDecodeWavesPerCuGqa = 4;      // grouped queries (matrix-core engine)
constexpr int kMaxDecodeWaves = 8192;        // upper bound on the launch on any device
constexpr int kPieceUnits = 1;               // cost of beginning a (sequence, kv head), in units of one KV block
constexpr int kMinUnitsPerWave = 1 + kPieceUnits;   // a range of that many units holds at least one block: small batches use fewer waves

// One fp32 partial result of a piece: running max m (log2 domain), sum l, acc[128].
constexpr int kPartialFloats = kHeadDim;

// Written by the planning kernel (or by wave 0 of a self-planning launch), read by the merge kernel.
struct DecodeHeader {
  long long gtot;   // cost units in the stream: (sum over non-empty sequences of blocks + kPieceUnits) * num_kv_heads
  long long quot;   // gtot / waves
  int rem;          // gtot % waves
  int waves;        // waves that received a non-empty range
};

using u32x4 = uint32_t __attribute__((ext_vector_type(4)));
using f16x2 = _Float16 __attribute__((ext_vector_type(2)));
using bf16x2 = __bf16 __attribute__((ext_vector_type(2)));

struct F16 {};
struct BF16 {};

// Physical slot of token p of a sequence whose block-table row is `row`, for blocks of `bs` tokens.
// Paged KV cache (Section 5.1 of the paper names it, with blocks of one token; this is the usual index).
__device__ __forceinline__ int32_t slot_of(const int32_t* __restrict__ row, int32_t p, int32_t bs) {
  return row[p / bs] * bs + p % bs;
}
// Element offset of the 128-wide row of (slot, kv head) in a cache laid out [block, kv head, row of the block, dim].
__device__ __forceinline__ size_t cache_row_offset(int32_t slot, int32_t head, int32_t num_kv_heads, int32_t bs) {
  return (((size_t)(slot / bs) * num_kv_heads + head) * bs + slot % bs) * kHeadDim;
}

// ---- 16-bit element helpers -------------------------------------------------
template <typename T>
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c);
template <>
__device__ __forceinline__ float dot2<F16>(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, a), __builtin_bit_cast(f16x2, b), c, false);
}
template <>
__device__ __forceinline__ float dot2<BF16>(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}

template <typename T>
__device__ __forceinline__ float lo_f32(uint32_t w);
template <typename T>
__device__ __forceinline__ float hi_f32(uint32_t w);
template <>
__device__ __forceinline__ float lo_f32<F16>(uint32_t w) {
  return (float)__builtin_bit_cast(f16x2, w)[0];
}
template <>
__device__ __forceinline__ float hi_f32<F16>(uint32_t w) {
  return (float)__builtin_bit_cast(f16x2, w)[1];
}
template <>
__device__ __forceinline__ float lo_f32<BF16>(uint32_t w) {
  return (float)__builtin_bit_cast(bf16x2, w)[0];     // lets the compiler fold the widening into v_fma_mix_f32_bf16
}
template <>
__device__ __forceinline__ float hi_f32<BF16>(uint32_t w) {
  return (float)__builtin_bit_cast(bf16x2, w)[1];
}

// Round two floats to the storage type (nearest even) and pack them.
template <typename T>
__device__ __forceinline__ uint32_t pack2(float a, float b);
template <>
__device__ __forceinline__ uint32_t pack2<F16>(float a, float b) {
  f16x2 v = {(_Float16)a, (_Float16)b};
  return __builtin_bit_cast(uint32_t, v);
}
template <>
__device__ __forceinline__ uint32_t pack2<BF16>(float a, float b) {
  using f32x2 = float __attribute__((ext_vector_type(2)));
  const f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));   // v_cvt_pk_bf16_f32, nearest even
}

// ---- cross-lane helpers -----------------------------------------------------
// Sum over the 16 lanes of a DPP row; every lane of the row gets the total.
__device__ __forceinline__ float row16_allreduce_sum(float x) {
  x += __builtin_amdgcn_update_dpp(0.f, x, 0xB1, 0xf, 0xf, false);    // quad_perm [1,0,3,2]
  x += __builtin_amdgcn_update_dpp(0.f, x, 0x4E, 0xf, 0xf, false);    // quad_perm [2,3,0,1]
  x += __builtin_amdgcn_update_dpp(0.f, x, 0x141, 0xf, 0xf, false);   // row_half_mirror
  x += __builtin_amdgcn_update_dpp(0.f, x, 0x140, 0xf, 0xf, false);   // row_mirror
  return x;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---- host side --------------------------------------------------------------
struct DecodeWorkspace {
  size_t header_off;        // DecodeHeader
  size_t seg_prefix_off;    // uint64[num_seqs + 1]      exclusive prefix per sequence: non-empty sequences << 32 | KV blocks
  size_t wave_desc_off;     // int4  [max(waves, 64)]    (r, h, b, n_blocks): start and length of a wave's range
  size_t ml_off;            // float2[2 * waves * G]     (m, l) of each partial piece
  size_t acc_off;           // float [2 * waves * G * 128]
  size_t total_bytes;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct DeviceShape {
  int cus;    // compute units
  int xcds;   // accelerator complex dies they are spread over (each with its own L2); 1 if unknown
};
DeviceShape device_shape();   // of the current device (cached per device; 256 / 8 when there is no device)
int device_cu_count();        // device_shape().cus

// The most waves a decode launch uses on the current device.
inline int decode_wave_bound(const vtc_attn_params& p) {
  const int per_cu = p.num_q_heads == p.num_kv_heads ? kDecodeWavesPerCuMha : kDecodeWavesPerCuGqa;
  const long long w = (long long)device_cu_count() * per_cu;
  return (int)(w < kMaxDecodeWaves ? w : kMaxDecodeWaves);
}

// Layout for a launch of `waves` waves over num_seqs sequences.  A wave owns at most two partial pieces
// however long the contexts are, so the footprint is linear in the number of waves.
inline DecodeWorkspace decode_workspace_layout(const vtc_attn_params& p, int32_t num_seqs, int32_t waves) {
  const size_t group = (size_t)(p.num_q_heads / p.num_kv_heads);
  const size_t w = (size_t)(waves > 0 ? waves : 0);
  DecodeWorkspace ws{};
  size_t at = 0;
  ws.header_off = at;
  at = 256;
  ws.seg_prefix_off = at;
  at = align_up(at + sizeof(uint64_t) * ((size_t)num_seqs + 1), 256);
  ws.wave_desc_off = at;
  at = align_up(at + sizeof(int32_t) * 4 * (w > 64 ? w : 64), 256);    // at least 1 KiB: also the target of dummy prefetches
  ws.ml_off = at;
  at = align_up(at + sizeof(float) * 2 * 2 * w * group, 256);
  ws.acc_off = at;
  at = align_up(at + sizeof(float) * kPartialFloats * 2 * w * group, 256);
  ws.total_bytes = at;
  return ws;
}

// Waves that a launch over sequences of at most max_seq_len tokens can put to use (0 or less: the block
// table's capacity): every wave gets at least kMinUnitsPerWave cost units of the batch, a unit being a KV block
// or the start of a (sequence, kv head).
inline int decode_waves_for(const vtc_attn_params& p, int32_t num_seqs, int32_t max_seq_len) {
  const long long cap = (long long)p.max_blocks_per_seq;
  long long nb = max_seq_len > 0 ? ((long long)max_seq_len + p.block_size - 1) / p.block_size : cap;
  if (nb > cap) nb = cap;
  const long long want = (nb + kPieceUnits) * num_seqs * p.num_kv_heads / kMinUnitsPerWave;
  const long long bound = decode_wave_bound(p);
  const long long w = want < bound ? want : bound;
  return (int)(w > 1 ? w : 1);
}

// The most waves (<= limit) whose layout fits into `bytes`; 0 if not even one does.
inline int decode_wave_capacity(const vtc_attn_params& p, int32_t num_seqs, size_t bytes, int limit) {
  int lo = 0, hi = limit;                      // the footprint is monotone in the number of waves
  while (lo < hi) {
    const int mid = lo + (hi - lo + 1) / 2;
    if (decode_workspace_layout(p, num_seqs, mid).total_bytes <= bytes) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// Host-side validation of the parameter struct; no HIP calls.
inline int check_params(const vtc_attn_params* p) {
  if (p == nullptr) return VTC_ERR_INVALID_ARG;
  if (p->num_q_heads <= 0 || p->num_kv_heads <= 0 || p->max_blocks_per_seq <= 0) return VTC_ERR_INVALID_ARG;
  if (!(p->scale == p->scale)) return VTC_ERR_INVALID_ARG;
  if (p->num_q_heads % p->num_kv_heads != 0) return VTC_ERR_UNSUPPORTED;
  const int g = p->num_q_heads / p->num_kv_heads;
  if (g != 1 && g != 2 && g != 4 && g != 8) return VTC_ERR_UNSUPPORTED;
  if (p->head_dim != kHeadDim) return VTC_ERR_UNSUPPORTED;
  if (p->block_size != 1 && p->block_size != 2 && p->block_size != 4 && p->block_size != 8 && p->block_size != kBlockSize)
    return VTC_ERR_UNSUPPORTED;
  if (p->dtype != VTC_F16 && p->dtype != VTC_BF16) return VTC_ERR_UNSUPPORTED;
  if (p->out_dtype != p->dtype && p->out_dtype != VTC_F32) return VTC_ERR_UNSUPPORTED;
  return VTC_OK;
}

// A counter update that rides in the last launch of a decode step (Algorithm 2 charges the
// counters right after forward_decode).  n == 0: none.
struct CounterJob {
  unsigned long long* counters;
  int32_t num_clients;
  const int32_t* client_ids;
  const int32_t* n_in;
  const int32_t* n_out;
  int32_t n;
  unsigned long long w_p, w_q;
};

// Kernel launchers (one translation unit each).
int launch_decode(const vtc_attn_params& p, int32_t num_seqs, const void* q, const void* k_cache,
                  const void* v_cache, const int32_t* block_table, const int32_t* seq_lens, void* out,
                  void* workspace, int32_t max_waves, hipStream_t stream, hipEvent_t ev_begin, hipEvent_t ev_end,
                  const CounterJob& counter_job);
// Attention for KV blocks of fewer than 16 tokens (one wave per query row, no workspace): decode when cu_q_lens
// is null (one query row per sequence), else the causal prefill chunk.
int launch_attend_general(const vtc_attn_params& p, int32_t num_seqs, const void* q, const int32_t* cu_q_lens,
                          int32_t max_q_len, const void* k_cache, const void* v_cache, const int32_t* block_table,
                          const int32_t* seq_lens, void* out, hipStream_t stream);
int launch_prefill(const vtc_attn_params& p, int32_t num_seqs, const void* q, const int32_t* cu_q_lens,
                   int32_t max_q_len, const void* k_cache, const void* v_cache, const int32_t* block_table,
                   const int32_t* seq_lens, void* out, hipStream_t stream);
int launch_counter_update(int64_t* counters, int32_t num_clients, const int32_t* client_ids,
                          const int32_t* n_in, const int32_t* n_out, int32_t n, int64_t w_p, int64_t w_q,
                          hipStream_t stream);
int launch_counter_update_cost(int64_t* counters, int32_t num_clients, const int32_t* client_ids,
                               const int32_t* p_old, const int32_t* q_old, const int32_t* p_new,
                               const int32_t* q_new, int32_t n, const vtc_cost_poly& h,
                               const int64_t* client_multiplier, hipStream_t stream);
int launch_counter_update_predicted(int64_t* counters, int32_t num_clients, const int32_t* client_ids,
                                    const int32_t* n_output, const int32_t* n_predicted, const int32_t* finished,
                                    int32_t n, int64_t w_q, hipStream_t stream);
int launch_kv_append(const vtc_attn_params& p, int32_t num_seqs, const void* k_new, const void* v_new,
                     const int32_t* cu_new_lens, int32_t max_new_len, void* k_cache, void* v_cache,
                     const int32_t* block_table, const int32_t* seq_lens, hipStream_t stream);
int launch_gather_slots(const vtc_attn_params& p, int32_t num_seqs, const int32_t* block_table,
                        const int32_t* seq_lens, const int32_t* cu_out, int32_t max_seq_len,
                        int32_t* slots_out, hipStream_t stream);

}  // namespace vtc
