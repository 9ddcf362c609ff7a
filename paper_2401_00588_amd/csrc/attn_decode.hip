// Decode attention over a paged KV cache (the attention part of forward_decode(B),
// Algorithm 2 of the paper; Section 2.1 describes decoding as one new token per
// request against all of its cached tokens).  HBM-bound: every cached K and V
// element of every running request is read exactly once per step.
//
// Decomposition.  Order all (sequence r, kv head h, KV block b) triples of the batch
// as r-major, then h, then b, and call that sequence of blocks the *stream*.
// The stream is cut into W ranges of equal *cost*, one per resident wavefront, regardless
// of where sequences begin and end.  A block costs one unit and so does every (r, h)
// that begins (closing it -- merging the softmax rows, normalising, writing -- takes a
// wave about as long as one block), so every wave needs about the same time:
//   plan    units per sequence -> exclusive prefix; then for each wave the (r, h, b)
//           at which its range starts and its number of blocks.  Batches of up to 1024
//           sequences need no launch for this: every attend wave derives its own
//           range from seq_lens in registers.  Larger batches run a one-workgroup
//           planning kernel first.
//   attend  one 64-lane wave per range.  The wave walks its range block by block,
//           always one block of loads ahead of the arithmetic, across sequence and
//           head boundaries without draining.  Each maximal run of blocks of one
//           (r, h) inside the range is a *piece*; a piece that ends becomes either the
//           final output (the piece is the whole sequence) or an fp32 partial
//           (m, l, acc[128] per q head).  A wave owns at most two partial pieces: one
//           cut at its range start and one cut at its range end.  Closed pieces wait
//           in an LDS patch and leave for global memory together, few instructions
//           for many rows, when the patch is full or the range ends.
//   merge   one wave per range boundary: if the boundary cuts a (r, h), combines the
//           partials of the waves that share it exactly (rescale by exp2(m_c - m))
//           and writes the output; also writes zeros for empty sequences.  When the
//           caller asked for the step's counter update as well (Algorithm 2 charges
//           the counters right after forward_decode), extra workgroups of this launch
//           do it.
//
// Lane mapping inside a wave: lane = 16 * row + sub.  A 16-byte load instruction
// covers 4 tokens x 128 dims: row picks the token (4 * i + row for load i of a
// block), sub picks dims 8*sub .. 8*sub+7.  A K.q dot product is 4 packed dot2
// operations per lane plus a 4-step DPP all-reduce inside the 16-lane row; the V
// update needs no cross-lane traffic.  The 4 rows keep separate softmax states
// that are merged once per piece.
#include "counter_terms.h"

namespace vtc {

constexpr int kPlanThreads = 1024;

// The stream in cost units: sequence r with nb_r > 0 blocks takes Hkv * (nb_r + kPieceUnits) units, head by head,
// each head's kPieceUnits of overhead first and its blocks after them.  A cut that falls into the overhead
// starts the range at block 0 of that head.
//
// Start of wave w's range, floor(total * w / waves), from quot = total / waves and rem = total % waves
// (rem * w < 2^26 because waves <= kMaxDecodeWaves): no 64-bit division per lookup.
struct RangeMap {
  long long quot;
  uint32_t rem;
  uint32_t waves;
  __device__ __forceinline__ long long start(int w) const {
    return quot * (long long)w + (long long)(rem * (uint32_t)w / waves);
  }
};
__device__ __forceinline__ RangeMap make_range_map(long long total, int waves) {
  if (waves <= 0) return RangeMap{0, 0u, 1u};
  if (total <= 0xffffffffll)                         // the usual case: 32-bit division
    return RangeMap{(long long)((uint32_t)total / (uint32_t)waves), (uint32_t)total % (uint32_t)waves, (uint32_t)waves};
  return RangeMap{total / waves, (uint32_t)(total % waves), (uint32_t)waves};
}

// Where a position v of the unit stream lies, given the sequence r that contains it: p_blocks / p_seqs = blocks /
// non-empty sequences before r, nb = blocks of r.  Returns (r, kv head, block, real blocks of the stream before v).
struct UnitPos {
  int r, h, b;
  long long blocks_before;
};
__device__ __forceinline__ UnitPos unit_pos(long long v, int r, long long p_blocks, long long p_seqs, uint32_t nb,
                                            int num_kv_heads) {
  const uint32_t per_head = nb + kPieceUnits;
  const uint32_t off = (uint32_t)(v - (p_blocks + p_seqs * kPieceUnits) * num_kv_heads);     // < per_head * Hkv < 2^31
  const uint32_t h = off / per_head, u = off - h * per_head;
  const uint32_t b = u > (uint32_t)kPieceUnits ? u - kPieceUnits : 0u;
  return UnitPos{r, (int)h, (int)b, p_blocks * num_kv_heads + (long long)h * nb + b};
}

// ------------------------------------------------------------------ plan ----
constexpr int kPlanLdsSeqs = 4096;     // sequences whose prefix is also kept in LDS for the range search

__global__ __launch_bounds__(kPlanThreads) void decode_plan_kernel(const int32_t* __restrict__ seq_lens,
                                                                   int32_t num_seqs, int32_t num_kv_heads,
                                                                   int32_t max_tokens, int32_t max_waves,
                                                                   DecodeHeader* __restrict__ header,
                                                                   unsigned long long* __restrict__ seg_prefix,
                                                                   int4* __restrict__ wave_desc) {
  // a prefix entry: non-empty sequences before r in the high half, their blocks in the low half
  __shared__ unsigned long long prefix_lds[kPlanLdsSeqs + 1];
  __shared__ unsigned long long wave_sums[kPlanThreads / kWave];
  __shared__ unsigned long long carry;
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wid = tid / kWave;
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int base = 0; base < num_seqs; base += kPlanThreads) {
    const int r = base + tid;
    unsigned long long n = 0;
    if (r < num_seqs) {
      const uint32_t nb = (uint32_t)(min(max(seq_lens[r], 0), max_tokens) + kBlockSize - 1) / kBlockSize;
      n = nb > 0 ? (1ull << 32) | nb : 0ull;
    }
    // inclusive scan inside the wave, then across the 16 waves
    unsigned long long x = n;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const unsigned long long y = __shfl_up(x, off);
      if (lane >= off) x += y;
    }
    if (lane == kWave - 1) wave_sums[wid] = x;
    __syncthreads();
    unsigned long long before = carry;
    for (int j = 0; j < wid; ++j) before += wave_sums[j];
    if (r < num_seqs) {
      const unsigned long long excl = before + x - n;
      seg_prefix[r] = excl;
      if (r < kPlanLdsSeqs) prefix_lds[r] = excl;
    }
    __syncthreads();
    if (tid == kPlanThreads - 1) carry = before + x;
    __syncthreads();
  }
  const unsigned long long total = carry;
  if (tid == 0) {
    seg_prefix[num_seqs] = total;
    if (num_seqs <= kPlanLdsSeqs) prefix_lds[num_seqs] = total;
  }
  const long long total_blocks = (long long)(total & 0xffffffffull), total_seqs = (long long)(total >> 32);
  const long long utot = (total_blocks + total_seqs * kPieceUnits) * num_kv_heads;
  // every active wave gets at least kMinUnitsPerWave units, i.e. at least one block
  const long long want = utot / kMinUnitsPerWave;
  const int waves = (int)(want < (long long)max_waves ? want : (long long)max_waves);
  const RangeMap map = make_range_map(utot, waves);
  if (tid == 0) {
    header->gtot = utot;
    header->quot = map.quot;
    header->rem = (int)map.rem;
    header->waves = waves;
  }
  __syncthreads();                                           // the prefix is complete and visible to the workgroup
  const bool in_lds = num_seqs <= kPlanLdsSeqs;
  auto units_before = [&](int r) {                           // units of the sequences before r, per kv head
    const unsigned long long e = in_lds ? prefix_lds[r] : seg_prefix[r];
    return (long long)(e & 0xffffffffull) + (long long)(e >> 32) * kPieceUnits;
  };
  auto locate = [&](long long v) {                           // v < utot
    // the sequence r with units_before(r) * Hkv <= v < units_before(r + 1) * Hkv
    int lo = 0, hi = num_seqs - 1;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (units_before(mid + 1) * num_kv_heads > v) hi = mid; else lo = mid + 1;
    }
    const unsigned long long e0 = in_lds ? prefix_lds[lo] : seg_prefix[lo];
    const unsigned long long e1 = in_lds ? prefix_lds[lo + 1] : seg_prefix[lo + 1];
    return unit_pos(v, lo, (long long)(e0 & 0xffffffffull), (long long)(e0 >> 32),
                    (uint32_t)((e1 & 0xffffffffull) - (e0 & 0xffffffffull)), num_kv_heads);
  };
  for (int w = tid; w < max_waves; w += kPlanThreads) {
    int4 d = make_int4(0, 0, 0, 0);
    if (w < waves) {
      const UnitPos p0 = locate(map.start(w));
      const long long end_blocks = w + 1 < waves ? locate(map.start(w + 1)).blocks_before : total_blocks * num_kv_heads;
      d = make_int4(p0.r, p0.h, p0.b, (int)(end_blocks - p0.blocks_before));
    }
    wave_desc[w] = d;
  }
}

// Inclusive prefix sum over the 64 lanes with data-parallel-primitive moves (vector instructions; a shuffle-based
// scan is six dependent LDS round trips, and every wave of a self-planning launch runs two of them before its first
// load): shifts by 1, 2, 4, 8 inside the 16-lane rows, then row 0's total into row 1 and row 2's into row 3, then
// the first half's total into the second.  Lanes without a source add 0.
__device__ __forceinline__ int wave_inclusive_sum(int x) {
  x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, false);      // row_shr:1
  x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, false);      // row_shr:2
  x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, false);      // row_shr:4
  x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, false);      // row_shr:8
  x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false);      // row_bcast:15 into rows 1 and 3
  x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false);      // row_bcast:31 into rows 2 and 3
  return x;
}

// ------------------------------------------------------------- self-plan ----
// The same plan without a launch, for batches of at most 64 x 16 sequences: every wave computes
// the prefix in registers (lane i holds sequences i*c .. i*c+c-1, c = ceil(N / 64)) and looks
// up only the two ends of its own range.  Returns (r, h, b, n_blocks); n_blocks = 0 for a wave without a range.
// Wave 0 also writes the header that the merge kernel reads.
constexpr int kSelfPlanPerLane = 16;
constexpr int kSelfPlanMaxSeqs = kWave * kSelfPlanPerLane;

__device__ __forceinline__ int4 self_plan(const int32_t* __restrict__ seq_lens, int num_seqs, int num_kv_heads,
                                          int max_tokens, int max_waves, int wave, int lane,
                                          DecodeHeader* __restrict__ header, int32_t* lens_lds) {
  // Every resident wave runs this before its first load, so it is kept short: sequences are handled four
  // at a time and groups past ceil(N / 64) are skipped by a uniform branch.
  const int per_lane = (num_seqs + kWave - 1) / kWave;
  const int first = lane * per_lane;
  // seq_lens is read with coalesced loads (thousands of waves read the same few lines at the same
  // moment) and redistributed through LDS so that each lane ends up with its own run of sequences
#pragma unroll
  for (int c = 0; c < kSelfPlanPerLane; c += 4) {
    if (c < per_lane) {
      int len[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) len[j] = seq_lens[min((c + j) * kWave + lane, num_seqs - 1)];   // clamped: always valid
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int r = (c + j) * kWave + lane;          // < 1024 = the size of lens_lds
        lens_lds[r] = r < num_seqs ? (min(max(len[j], 0), max_tokens) + kBlockSize - 1) / kBlockSize : 0;
      }
    }
  }
  __syncthreads();                         // one wave per workgroup: orders the LDS writes before the reads
  int nbv[kSelfPlanPerLane];
#pragma unroll
  for (int j = 0; j < kSelfPlanPerLane; ++j) nbv[j] = 0;
#pragma unroll
  for (int c = 0; c < kSelfPlanPerLane; c += 4) {
    if (c < per_lane) {
#pragma unroll
      for (int j = 0; j < 4; ++j) nbv[c + j] = c + j < per_lane ? lens_lds[first + c + j] : 0;
    }
  }
  int mine_b = 0, mine_s = 0;              // blocks and non-empty sequences of this lane's run
#pragma unroll
  for (int j = 0; j < kSelfPlanPerLane; ++j) {
    mine_b += nbv[j];
    mine_s += nbv[j] > 0 ? 1 : 0;
  }
  const int incl_b = wave_inclusive_sum(mine_b), incl_s = wave_inclusive_sum(mine_s);
  const int total_blocks = __builtin_amdgcn_readlane(incl_b, kWave - 1);
  const int total_seqs = __builtin_amdgcn_readlane(incl_s, kWave - 1);
  const int excl_b = incl_b - mine_b, excl_s = incl_s - mine_s;      // of all sequences before this lane's
  const int excl_u = excl_b + excl_s * kPieceUnits;                   // units before this lane's run, per kv head
  const long long utot = ((long long)total_blocks + (long long)total_seqs * kPieceUnits) * num_kv_heads;
  const bool narrow = utot <= 0xffffffffll;                           // the usual case: 32-bit divisions
  const long long want = utot / kMinUnitsPerWave;                     // every active wave gets at least one block
  const int waves = (int)(want < (long long)max_waves ? want : (long long)max_waves);
  const RangeMap map = make_range_map(utot, waves);
  if (wave == 0 && lane == 0) {
    header->gtot = utot;
    header->quot = map.quot;
    header->rem = (int)map.rem;
    header->waves = waves;
  }
  if (wave >= waves) return make_int4(0, 0, 0, 0);
  auto locate = [&](long long v) {                                    // v < utot
    // Sequence r owns the positions [Hkv * before_r, Hkv * (before_r + units_r)), so v lies in the
    // sequence whose unit range [before_r, before_r + units_r) contains floor(v / Hkv).
    const int vq = narrow ? (int)((uint32_t)v / (uint32_t)num_kv_heads) : (int)(v / num_kv_heads);
    // the prefix is non-decreasing over the lanes: the last lane that starts at or before vq owns it
    const unsigned long long below = __ballot(excl_u <= vq);
    const int owner = __builtin_amdgcn_readfirstlane(__popcll(below) - 1);
    int before_b = excl_b, before_s = excl_s, found_r = 0, found_b = 0, found_s = 0, found_nb = 1;
#pragma unroll
    for (int c = 0; c < kSelfPlanPerLane; c += 4) {
      if (c < per_lane) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int nb = nbv[c + j];
          const int before_u = before_b + before_s * kPieceUnits;
          if (nb > 0 && before_u <= vq && vq < before_u + nb + kPieceUnits) {
            found_r = first + c + j;
            found_b = before_b;
            found_s = before_s;
            found_nb = nb;
          }
          before_b += nb;
          before_s += nb > 0 ? 1 : 0;
        }
      }
    }
    return unit_pos(v, __builtin_amdgcn_readlane(found_r, owner), __builtin_amdgcn_readlane(found_b, owner),
                    __builtin_amdgcn_readlane(found_s, owner), (uint32_t)__builtin_amdgcn_readlane(found_nb, owner),
                    num_kv_heads);
  };
  const UnitPos p0 = locate(map.start(wave));
  const long long end_blocks =
      wave + 1 < waves ? locate(map.start(wave + 1)).blocks_before : (long long)total_blocks * num_kv_heads;
  return make_int4(p0.r, p0.h, p0.b, (int)(end_blocks - p0.blocks_before));
}

// ---------------------------------------------------------------- attend ----
// Load one 4 KiB tile (4 x 1 KiB across the wave).  `stride16` is kWave for a real tile; 0 turns the
// four loads into re-reads of one 1 KiB line set (the throw-away prefetch at the end of a range).
__device__ __forceinline__ void load_tile(u32x4 (&dst)[4], const uint16_t* __restrict__ tile, int lane, int stride16) {
  const u32x4* src = reinterpret_cast<const u32x4*>(tile) + lane;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    dst[i] = __builtin_nontemporal_load(src + i * stride16);  // streamed once: keep it out of the caches' way
  }
}

// Pieces a wave has closed are parked in LDS and written to global memory together, when the patch is full or the
// range ends, with as few store instructions as their bytes allow.  In this kernel a store instruction costs a wave
// 0.3-0.8 us whatever it carries (the memory pipeline is full of the other waves' loads; measured on batches of the
// same bytes in 4 x as many sequences with and without the stores), and stores issued between a tile's loads and
// their wait also make that wait cover their completion (the compiler cannot count stores that only some
// iterations issue).  A lane of a store can write anywhere, so one instruction carries the 16-bit output rows of
// four (sequence, query head) pairs, or two fp32 rows, or every parked partial's (m, l).
// A parked piece: for each of the group's G query heads 128 unnormalised fp32 sums, the running maximum m and the
// sum l (kParkFloats apart, 16-byte aligned), then the descriptor.
constexpr int kParkFloats = kHeadDim + 4;
struct ParkedPiece {
  uint32_t whole;        // 1: the piece is a whole (sequence, kv head): normalise and write the output rows
  uint32_t slot0;        // 0: write partial slots slot0 .. slot0 + G - 1
  uint32_t out_row_lo;   // element offset of the first of the G output rows
  uint32_t out_row_hi;
};
template <int G>
constexpr int park_stride() { return G * kParkFloats + 4; }     // in 4-byte words

// Write n parked pieces out.  Their n * G rows (at most 64) are taken four (16-bit output) or two (fp32 output,
// partial sums) at a time; a lane whose row is of the other kind stays idle.
template <typename T, int G>
__device__ __forceinline__ void flush_pieces(const float* __restrict__ parked, int n, int lane, void* __restrict__ out,
                                             int32_t out_f32, float2* __restrict__ part_ml,
                                             float* __restrict__ part_acc) {
  using f32x4 = float __attribute__((ext_vector_type(4)));
  const int rows = n * G;
  auto row_of = [&](int rho, const float*& row, u32x4& d) {      // rho < rows
    const int pi = rho / G, g = rho % G;
    const float* piece = parked + pi * park_stride<G>();
    row = piece + g * kParkFloats;
    d = *reinterpret_cast<const u32x4*>(piece + G * kParkFloats);
    return g;
  };
  if (!out_f32) {
    for (int base = 0; base < rows; base += 4) {                 // 16 lanes x 8 dims per row
      const int rho = base + (lane >> 4), chunk = lane & 15;
      if (rho < rows) {
        const float* row;
        u32x4 d;
        const int g = row_of(rho, row, d);
        if (d[0] != 0u) {
          const f32x4 a0 = *reinterpret_cast<const f32x4*>(row + chunk * 8);
          const f32x4 a1 = *reinterpret_cast<const f32x4*>(row + chunk * 8 + 4);
          const float inv = 1.f / row[kHeadDim + 1];
          const u32x4 o = u32x4{pack2<T>(a0[0] * inv, a0[1] * inv), pack2<T>(a0[2] * inv, a0[3] * inv),
                                pack2<T>(a1[0] * inv, a1[1] * inv), pack2<T>(a1[2] * inv, a1[3] * inv)};
          const size_t at = ((size_t)d[2] | ((size_t)d[3] << 32)) + (size_t)g * kHeadDim + chunk * 8;
          *reinterpret_cast<u32x4*>(static_cast<uint16_t*>(out) + at) = o;
        }
      }
    }
  }
  for (int base = 0; base < rows; base += 2) {                   // 32 lanes x 4 dims per row
    const int rho = base + (lane >> 5), chunk = lane & 31;
    if (rho < rows) {
      const float* row;
      u32x4 d;
      const int g = row_of(rho, row, d);
      const f32x4 a = *reinterpret_cast<const f32x4*>(row + chunk * 4);
      if (d[0] == 0u) {
        *reinterpret_cast<f32x4*>(part_acc + (size_t)(d[1] + g) * kPartialFloats + chunk * 4) = a;
      } else if (out_f32) {
        const float inv = 1.f / row[kHeadDim + 1];
        const size_t at = ((size_t)d[2] | ((size_t)d[3] << 32)) + (size_t)g * kHeadDim + chunk * 4;
        *reinterpret_cast<f32x4*>(static_cast<float*>(out) + at) = f32x4{a[0] * inv, a[1] * inv, a[2] * inv, a[3] * inv};
      }
    }
  }
  if (lane < rows) {                                              // the partials' (m, l): one instruction for all
    const float* row;
    u32x4 d;
    const int g = row_of(lane, row, d);
    if (d[0] == 0u) part_ml[d[1] + g] = *reinterpret_cast<const float2*>(row + kHeadDim);
  }
}

// Where a finished piece goes: the output row block of its (sequence, kv head) and its partial slot.
struct PieceSink {
  void* out_rows;       // G consecutive output rows of 128 (of the storage type, or fp32 when out_f32)
  bool out_f32;
  float* part_acc;      // part_acc + slot0 * 128, slot0 = (wave * 2 + end) * G: G consecutive partials
  float2* part_ml;      // part_ml + slot0
};

// ---- vector-ALU engine: lane = 16 * row + sub handles token 4i + row of load i, dims 8*sub..8*sub+7 ----
template <typename T, int G>
struct ValuEngine {
  static constexpr int kQRegs = G;       // one 16-byte q slice per query head
  static constexpr int kLdsElems = 0;
  static constexpr int kMinWavesPerSimd = G == 1 ? 4 : (G == 2 ? 3 : (G == 4 ? 2 : 1));   // register budget (used with G = 1)
  static constexpr int kWavesPerCu = kDecodeWavesPerCuMha;
  static constexpr int kParked = 16;                // pieces parked in LDS before they are written out (8.3 KiB)
  int row, sub;
  float m[G];        // running max of the scaled logits (log2 domain), per 16-lane row
  float l[G];        // running sum of exp2(logit - m)
  float acc[G][8];   // running sum of exp2(logit - m) * v, dims 8*sub .. 8*sub+7

  __device__ __forceinline__ void init(int lane, uint16_t*) {
    row = lane >> 4;
    sub = lane & 15;
    reset();
  }
  __device__ __forceinline__ void reset() {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      m[g] = -INFINITY;
      l[g] = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
    }
  }
  // q_rows = q + (r * Hq + h * G) * 128
  __device__ __forceinline__ void load_q(u32x4 (&dst)[kQRegs], const uint16_t* __restrict__ q_rows) const {
#pragma unroll
    for (int g = 0; g < G; ++g) dst[g] = *reinterpret_cast<const u32x4*>(q_rows + g * kHeadDim + sub * 8);
  }

  // One K/V block (16 tokens).  kTail: tokens >= nvalid are excluded and their (possibly garbage) V rows zeroed.
  template <bool kTail>
  __device__ __forceinline__ void block_t(const u32x4 (&q)[kQRegs], const u32x4 (&k)[4], u32x4 (&v)[4], float scale2,
                                          int nvalid) {
    float s[G][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) d = dot2<T>(q[g][w], k[i][w], d);
        s[g][i] = row16_allreduce_sum(d) * scale2;
      }
    }
    if (kTail) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool ok = 4 * i + row < nvalid;
#pragma unroll
        for (int g = 0; g < G; ++g) s[g][i] = ok ? s[g][i] : -INFINITY;
        if (!ok) v[i] = u32x4{0u, 0u, 0u, 0u};
      }
    }
    float p[G][4];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float mx = fmaxf(fmaxf(s[g][0], s[g][1]), fmaxf(s[g][2], s[g][3]));
      const float m_new = fmaxf(m[g], mx);
      // a row that has seen no valid token yet keeps m = -inf; subtract 0 instead so
      // that exp2 yields 0 rather than NaN
      const float m_sub = (kTail && m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = fast_exp2(m[g] - m_sub);
#pragma unroll
      for (int i = 0; i < 4; ++i) p[g][i] = fast_exp2(s[g][i] - m_sub);
      l[g] = l[g] * alpha + ((p[g][0] + p[g][1]) + (p[g][2] + p[g][3]));
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[g][e] *= alpha;
      m[g] = m_new;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float lo = lo_f32<T>(v[i][w]);
        const float hi = hi_f32<T>(v[i][w]);
#pragma unroll
        for (int g = 0; g < G; ++g) {
          acc[g][2 * w] = fmaf(p[g][i], lo, acc[g][2 * w]);
          acc[g][2 * w + 1] = fmaf(p[g][i], hi, acc[g][2 * w + 1]);
        }
      }
    }
  }
  __device__ __forceinline__ void block(const u32x4 (&q)[kQRegs], const u32x4 (&k)[4], u32x4 (&v)[4], float scale2,
                                        int nvalid) {
    if (nvalid < kBlockSize)
      block_t<true>(q, k, v, scale2, nvalid);
    else
      block_t<false>(q, k, v, scale2, kBlockSize);
  }

  // Merge the four 16-lane rows of the softmax state (the result is complete in the lanes of row 0).
  __device__ __forceinline__ void merge_rows() {
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float m_o = __shfl_xor(m[g], off);
        const float l_o = __shfl_xor(l[g], off);
        const float m_n = fmaxf(m[g], m_o);
        const float m_sub = m_n == -INFINITY ? 0.f : m_n;
        const float a = fast_exp2(m[g] - m_sub);
        const float b = fast_exp2(m_o - m_sub);
        l[g] = l[g] * a + l_o * b;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = acc[g][e] * a + __shfl_xor(acc[g][e], off) * b;
        m[g] = m_n;
      }
    }
  }
  // Close a piece into an LDS patch (see ParkedPiece) and reset.
  __device__ __forceinline__ void park(float* piece) {
    merge_rows();
    if (row == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float4* dst = reinterpret_cast<float4*>(piece + g * kParkFloats + sub * 8);
        dst[0] = make_float4(acc[g][0], acc[g][1], acc[g][2], acc[g][3]);
        dst[1] = make_float4(acc[g][4], acc[g][5], acc[g][6], acc[g][7]);
        if (sub == 0) *reinterpret_cast<float2*>(piece + g * kParkFloats + kHeadDim) = make_float2(m[g], l[g]);
      }
    }
    reset();
  }
  // Close a piece: merge the four 16-lane rows, write the output (whole sequence) or a partial, reset.
  __device__ __forceinline__ void finish(bool whole, const PieceSink& sink) {
    merge_rows();
    if (row == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        if (whole) {
          const float inv = 1.f / l[g];
          if (sink.out_f32) {
            float4* dst = reinterpret_cast<float4*>(static_cast<float*>(sink.out_rows) + g * kHeadDim + sub * 8);
            dst[0] = make_float4(acc[g][0] * inv, acc[g][1] * inv, acc[g][2] * inv, acc[g][3] * inv);
            dst[1] = make_float4(acc[g][4] * inv, acc[g][5] * inv, acc[g][6] * inv, acc[g][7] * inv);
          } else {
            u32x4 o;
#pragma unroll
            for (int w2 = 0; w2 < 4; ++w2) o[w2] = pack2<T>(acc[g][2 * w2] * inv, acc[g][2 * w2 + 1] * inv);
            *reinterpret_cast<u32x4*>(static_cast<uint16_t*>(sink.out_rows) + g * kHeadDim + sub * 8) = o;
          }
        } else {
          float4* dst = reinterpret_cast<float4*>(sink.part_acc + g * kPartialFloats + sub * 8);
          dst[0] = make_float4(acc[g][0], acc[g][1], acc[g][2], acc[g][3]);
          dst[1] = make_float4(acc[g][4], acc[g][5], acc[g][6], acc[g][7]);
          if (sub == 0) sink.part_ml[g] = make_float2(m[g], l[g]);
        }
      }
    }
    reset();
  }
};

// ---- matrix-core engine for grouped-query attention (2 <= G <= 16) --------------------------------------
// With G query heads per KV head the vector-ALU engine spends ~110 instructions per head and block and
// becomes ALU-bound (measured: 75 % VALU busy at G = 4).  Here a block is two small matrix products on the
// G x 16-token problem, padded to 16 x 16:
//   S^T[token][head] = K . Q^T     4 x v_mfma_f32_16x16x32   A = K rows (tile staged in LDS, 16-byte reads)
//                                                            B = Q^T in registers
//   O^T[dim][head]  += V^T . P^T   8 x v_mfma_f32_16x16x16   A = V^T via the transposing LDS read
//                                                            B = P^T = the accumulator layout of S^T
// lane = 16 * kg + j: j is the head (columns) or token/dim (rows), kg the contraction group.  Columns
// j >= G are padding (they repeat head G-1 and are never written).
template <typename T, int G>
struct MfmaEngine {
  static_assert(G >= 2 && G <= 16, "group size");
  static constexpr int kQRegs = (G + 3) / 4;      // the G q rows (256 B each) as 16 bytes per lane, 4 rows per register set
  static constexpr int kPitchK = kHeadDim + 8;    // 272 B rows: conflict-free 16-byte row reads
  static constexpr int kPitchV = kHeadDim + 16;   // 288 B rows: the 16-row x 32-byte transposing reads use every bank twice
  static constexpr int kPitchQ = kHeadDim + 8;
  static constexpr int kLdsElems = kBlockSize * (kPitchK + kPitchV) + 4 * kQRegs * kPitchQ;
  static constexpr int kMinWavesPerSimd = 2;      // register budget = 512 / this (three waves spill)
  static constexpr int kWavesPerCu = kDecodeWavesPerCuGqa;
  static constexpr int kParked = G <= 2 ? 8 : 24 / G;   // pieces parked in LDS before they are written out (12.5 KiB)
  using f32x4 = float __attribute__((ext_vector_type(4)));
  using f16x8 = _Float16 __attribute__((ext_vector_type(8)));
  using bf16x8 = __bf16 __attribute__((ext_vector_type(8)));
  using f16x4 = _Float16 __attribute__((ext_vector_type(4)));
  using s16x4 = short __attribute__((ext_vector_type(4)));
  using u32x2 = uint32_t __attribute__((ext_vector_type(2)));

  int row, sub;      // staging layout of a loaded tile: token 4i + row, dims 8*sub..
  int j, kg;         // matrix layout
  uint16_t* k_lds;
  uint16_t* v_lds;
  uint16_t* q_lds;
  float m, l;        // softmax state of head j (m identical in the 4 lane groups, l partial per group)
  f32x4 acc[8];      // O^T: dims 16*db + 4*kg + v of head j

  __device__ __forceinline__ void init(int lane, uint16_t* lds) {
    row = kg = lane >> 4;
    sub = j = lane & 15;
    k_lds = lds;
    v_lds = lds + kBlockSize * kPitchK;
    q_lds = v_lds + kBlockSize * kPitchV;
    reset();
  }
  __device__ __forceinline__ void reset() {
    m = -INFINITY;
    l = 0.f;
#pragma unroll
    for (int db = 0; db < 8; ++db) acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  // The q rows are fetched like a tile (lane = 16 * row + sub: head 4i + row, dims 8*sub..) and turned into the
  // Q^T operand through LDS when the block is consumed; heads >= G repeat head G-1.
  __device__ __forceinline__ void load_q(u32x4 (&dst)[kQRegs], const uint16_t* __restrict__ q_rows) const {
#pragma unroll
    for (int i = 0; i < kQRegs; ++i)
      dst[i] = *reinterpret_cast<const u32x4*>(q_rows + min(4 * i + row, G - 1) * kHeadDim + sub * 8);
  }

  static __device__ __forceinline__ f32x4 mfma_qk(u32x4 a, u32x4 b, f32x4 c) {
    if constexpr (__is_same(T, F16))
      return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
      return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ f32x4 mfma_pv(u32x2 a, u32x2 b, f32x4 c) {
    if constexpr (__is_same(T, F16))
      return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4, a), __builtin_bit_cast(f16x4, b), c, 0, 0, 0);
    else
      return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, a), __builtin_bit_cast(s16x4, b), c, 0, 0, 0);
  }

  __device__ __forceinline__ void block(const u32x4 (&q)[kQRegs], const u32x4 (&k)[4], u32x4 (&v)[4], float scale2,
                                        int nvalid) {
    const bool tail = nvalid < kBlockSize;
    // stage the tile row-major in this wave's LDS patch (the wave's LDS operations complete in order)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (tail && 4 * i + row >= nvalid) v[i] = u32x4{0u, 0u, 0u, 0u};   // garbage rows must not meet a zero weight as NaN
      *reinterpret_cast<u32x4*>(&k_lds[(4 * i + row) * kPitchK + sub * 8]) = k[i];
      *reinterpret_cast<u32x4*>(&v_lds[(4 * i + row) * kPitchV + sub * 8]) = v[i];
    }
#pragma unroll
    for (int i = 0; i < kQRegs; ++i) *reinterpret_cast<u32x4*>(&q_lds[(4 * i + row) * kPitchQ + sub * 8]) = q[i];
    // S^T[token 4*kg + v][head j]
    f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};
    const uint16_t* qrow = q_lds + min(j, 4 * kQRegs - 1) * kPitchQ + kg * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const u32x4 kf = *reinterpret_cast<const u32x4*>(&k_lds[j * kPitchK + ks * 32 + kg * 8]);
      const u32x4 qf = *reinterpret_cast<const u32x4*>(qrow + ks * 32);
      s = mfma_qk(kf, qf, s);
    }
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      s[e] *= scale2;
      if (tail && 4 * kg + e >= nvalid) s[e] = -INFINITY;
      mx = fmaxf(mx, s[e]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m, mx);
    const float m_sub = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = fast_exp2(m - m_sub);
    m = m_new;
    float p[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) p[e] = fast_exp2(s[e] - m_sub);
    l = l * alpha + ((p[0] + p[1]) + (p[2] + p[3]));
    if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0ull) {          // skip the rescale when no head's maximum moved
#pragma unroll
      for (int db = 0; db < 8; ++db) acc[db] *= alpha;
    }
    const u32x2 pb = u32x2{pack2<T>(p[0], p[1]), pack2<T>(p[2], p[3])};   // P^T: tokens 4*kg + 0..3 of head j
    // bf16 keeps 8 bits of a weight.  What the rounding dropped goes through the second product as an
    // operand of its own, so the weights act with 16 bits (fp16's 11 bits are left as they are).
    constexpr bool kSplitP = __is_same(T, BF16);
    u32x2 pr = u32x2{0u, 0u};
    if constexpr (kSplitP) {
      pr = u32x2{pack2<T>(p[0] - __builtin_bit_cast(float, pb[0] << 16),
                          p[1] - __builtin_bit_cast(float, pb[0] & 0xffff0000u)),
                 pack2<T>(p[2] - __builtin_bit_cast(float, pb[1] << 16),
                          p[3] - __builtin_bit_cast(float, pb[1] & 0xffff0000u))};
    }
    // O^T[dim][head] += V^T . P^T; lane j of group kg addresses token 4*kg + j/4, dims 4*(j%4).. of each 16-dim block
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const uint16_t* vrow = v_lds + (4 * kg + (j >> 2)) * kPitchV + 4 * (j & 3);
    u32x2 vt[8];
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      vt[db] = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vrow + db * 16)));
      acc[db] = mfma_pv(vt[db], pb, acc[db]);
    }
    if constexpr (kSplitP) {                 // second pass, so that no product waits for the one before it
#pragma unroll
      for (int db = 0; db < 8; ++db) acc[db] = mfma_pv(vt[db], pr, acc[db]);
    }
  }

  // Close a piece into an LDS patch (see ParkedPiece) and reset.
  __device__ __forceinline__ void park(float* piece) {
    float l_tot = l + __shfl_xor(l, 16);
    l_tot += __shfl_xor(l_tot, 32);
    if (j < G) {
      float* dst = piece + j * kParkFloats + 4 * kg;
#pragma unroll
      for (int db = 0; db < 8; ++db) *reinterpret_cast<f32x4*>(dst + db * 16) = acc[db];
      if (kg == 0) *reinterpret_cast<float2*>(piece + j * kParkFloats + kHeadDim) = make_float2(m, l_tot);
    }
    reset();
  }
  __device__ __forceinline__ void finish(bool whole, const PieceSink& sink) {
    float l_tot = l + __shfl_xor(l, 16);
    l_tot += __shfl_xor(l_tot, 32);
    if (j < G) {
      if (whole) {
        const float inv = 1.f / l_tot;
        if (sink.out_f32) {
          float* dst = static_cast<float*>(sink.out_rows) + j * kHeadDim + 4 * kg;
#pragma unroll
          for (int db = 0; db < 8; ++db)
            *reinterpret_cast<float4*>(dst + db * 16) =
                make_float4(acc[db][0] * inv, acc[db][1] * inv, acc[db][2] * inv, acc[db][3] * inv);
        } else {
          uint16_t* dst = static_cast<uint16_t*>(sink.out_rows) + j * kHeadDim + 4 * kg;
#pragma unroll
          for (int db = 0; db < 8; ++db) {
            const u32x2 o = u32x2{pack2<T>(acc[db][0] * inv, acc[db][1] * inv), pack2<T>(acc[db][2] * inv, acc[db][3] * inv)};
            *reinterpret_cast<u32x2*>(dst + db * 16) = o;
          }
        }
      } else {
        float* dst = sink.part_acc + j * kPartialFloats + 4 * kg;
#pragma unroll
        for (int db = 0; db < 8; ++db)
          *reinterpret_cast<float4*>(dst + db * 16) = make_float4(acc[db][0], acc[db][1], acc[db][2], acc[db][3]);
        if (kg == 0) sink.part_ml[j] = make_float2(m, l_tot);
      }
    }
    reset();
  }
};

// A position in the stream: which block, and where its K/V tile lives.
struct StreamPos {
  int r, h, b;       // sequence, kv head, block index inside the sequence
  int nb;            // blocks of sequence r
  int s_len;         // context length of sequence r (clamped)
  size_t off;        // element offset of the (block, head) tile in k_cache / v_cache
};

template <typename T, int G, typename Engine>
__global__ __launch_bounds__(kWave, Engine::kMinWavesPerSimd) void decode_attend_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_cache, const uint16_t* __restrict__ v_cache,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_lens, void* __restrict__ out,
    int32_t out_f32, int4* __restrict__ wave_desc, float2* __restrict__ part_ml, float* __restrict__ part_acc,
    int32_t num_kv_heads, int32_t max_blocks_per_seq, float scale2, int32_t self_plan_seqs,
    DecodeHeader* __restrict__ header) {
  constexpr int kQRegs = Engine::kQRegs;
  __shared__ __attribute__((aligned(16))) uint16_t lds[Engine::kLdsElems > 0 ? Engine::kLdsElems : 8];
  __shared__ __attribute__((aligned(16))) float parked[Engine::kParked * park_stride<G>()];
  const int lane = threadIdx.x;
  const int num_q_heads = num_kv_heads * G;
  const int max_tokens = max_blocks_per_seq * kBlockSize;
  const int wave = blockIdx.x;
  int4 desc_v;
  if (self_plan_seqs > 0) {                // no planning launch: derive the range here, leave it for the merge
    __shared__ int32_t lens_lds[kSelfPlanMaxSeqs];
    desc_v = self_plan(seq_lens, self_plan_seqs, num_kv_heads, max_tokens, gridDim.x, wave, lane, header, lens_lds);
    if (lane == 0) wave_desc[wave] = desc_v;
  } else {
    desc_v = wave_desc[wave];
  }
  // the descriptor is the same for all lanes: keep it (and everything derived from it) in scalar registers
  const int4 desc = make_int4(__builtin_amdgcn_readfirstlane(desc_v.x), __builtin_amdgcn_readfirstlane(desc_v.y),
                              __builtin_amdgcn_readfirstlane(desc_v.z), __builtin_amdgcn_readfirstlane(desc_v.w));
  const int n_blocks = desc.w;
  if (n_blocks <= 0) return;
  const size_t block_stride = (size_t)num_kv_heads * kTileElems;

  auto locate = [&](StreamPos& p) {        // fill in the tile offset of p
    p.off = (size_t)block_table[(size_t)p.r * max_blocks_per_seq + p.b] * block_stride + (size_t)p.h * kTileElems;
  };
  auto step = [&](StreamPos& p) {          // move p to the next block of the stream (there is one)
    if (++p.b == p.nb) {
      p.b = 0;
      if (++p.h == num_kv_heads) {
        p.h = 0;
        do {
          ++p.r;
          p.s_len = min(max(seq_lens[p.r], 0), max_tokens);
          p.nb = (p.s_len + kBlockSize - 1) / kBlockSize;
        } while (p.nb == 0);
      }
    }
    locate(p);
  };
  auto q_rows = [&](const StreamPos& p) { return q + ((size_t)p.r * num_q_heads + p.h * G) * kHeadDim; };

  // cur: the block being consumed; nxt: the block whose loads are in flight; far: one further, so
  // that its (scalar) block-table lookup is never waited for between a tile's loads and their use.
  StreamPos cur;
  cur.r = desc.x;
  cur.h = desc.y;
  cur.b = desc.z;
  cur.s_len = min(max(seq_lens[cur.r], 0), max_tokens);
  cur.nb = (cur.s_len + kBlockSize - 1) / kBlockSize;
  locate(cur);
  StreamPos nxt = cur, far = cur;
  if (n_blocks > 1) {
    step(nxt);
    far = nxt;
  }
  if (n_blocks > 2) step(far);

  Engine eng;
  eng.init(lane, lds);
  int piece_lo = cur.b;                    // first block of the current piece

  // Two register sets (q, K tile, V tile), used alternately.  The q rows travel with the
  // tiles, so a set always holds the query of the block it holds.
  u32x4 qa[kQRegs], ka[4], va[4], qb[kQRegs], kb[4], vb[4];
  eng.load_q(qa, q_rows(cur));
  load_tile(ka, k_cache + cur.off, lane, kWave);
  load_tile(va, v_cache + cur.off, lane, kWave);
  // where the prefetch goes when there is no next block: 1 KiB of the (cache-resident) range table
  const uint16_t* const dummy = reinterpret_cast<const uint16_t*>(wave_desc);

  int n_parked = 0;                        // pieces closed and not yet written out
  auto flush_parked = [&]() {
    flush_pieces<T, G>(parked, n_parked, lane, out, out_f32, part_ml, part_acc);
    n_parked = 0;
  };
  // Consume the block at `cur` from (qreg, kx, vx); close the piece if it ends here.
  auto consume = [&](const u32x4 (&qreg)[kQRegs], u32x4 (&kx)[4], u32x4 (&vx)[4], bool last_of_range) {
    const bool last_of_seq = cur.b + 1 == cur.nb;
    const int nvalid = last_of_seq ? cur.s_len - cur.b * kBlockSize : kBlockSize;
    eng.block(qreg, kx, vx, scale2, nvalid);
    if (!(last_of_seq || last_of_range)) return;
    const bool whole = piece_lo == 0 && last_of_seq;     // the piece is the entire sequence
    if (n_parked == Engine::kParked) flush_parked();
    float* piece = parked + n_parked * park_stride<G>();
    eng.park(piece);
    if (lane == 0) {
      // partial slot 0: the piece cut at the start of this wave's range; slot 1: the one cut at its end
      const size_t out_row = ((size_t)cur.r * num_q_heads + cur.h * G) * kHeadDim;      // in elements
      ParkedPiece d;
      d.whole = whole ? 1u : 0u;
      d.slot0 = (uint32_t)((wave * 2 + (piece_lo == 0 ? 1 : 0)) * G);
      d.out_row_lo = (uint32_t)out_row;
      d.out_row_hi = (uint32_t)(out_row >> 32);
      *reinterpret_cast<ParkedPiece*>(piece + G * kParkFloats) = d;
    }
    ++n_parked;
    piece_lo = 0;                           // a new (r, h) starts with the next block
  };

  // The prefetch of the next block is unconditional (no branch around the loads, so the
  // hardware load counter stays exact and a tile's wait never covers the loads issued after
  // it).  On the last block of the range it is pointed at 1 KiB that is already in cache and
  // its result is dropped.  q is re-read with every block for the same reason (256-byte
  // rows that stay in cache); it only changes when the next block starts a new (r, h).
  int i = 0;
  while (true) {
    // -- even step: consume set a, prefetch into set b
    {
      const bool more = i + 1 < n_blocks;
      eng.load_q(qb, q_rows(nxt));
      load_tile(kb, more ? k_cache + nxt.off : dummy, lane, more ? kWave : 0);
      load_tile(vb, more ? v_cache + nxt.off : dummy, lane, more ? kWave : 0);
    }
    consume(qa, ka, va, i + 1 == n_blocks);
    if (++i == n_blocks) break;
    cur = nxt;
    nxt = far;
    if (i + 2 < n_blocks) step(far);
    // -- odd step: consume set b, prefetch into set a
    {
      const bool more = i + 1 < n_blocks;
      eng.load_q(qa, q_rows(nxt));
      load_tile(ka, more ? k_cache + nxt.off : dummy, lane, more ? kWave : 0);
      load_tile(va, more ? v_cache + nxt.off : dummy, lane, more ? kWave : 0);
    }
    consume(qb, kb, vb, i + 1 == n_blocks);
    if (++i == n_blocks) break;
    cur = nxt;
    nxt = far;
    if (i + 2 < n_blocks) step(far);
  }
  flush_parked();                          // nothing waits for these stores any more
}

// ----------------------------------------------------------------- merge ----
// Only a sequence-head that a range boundary cuts needs merging, so the merge is driven by the
// boundaries: block w looks at the cut between waves w-1 and w.  If that cut falls inside a
// (r, kv head) and wave w-1 holds its beginning, the block combines the pieces of waves
// w-1, w, w+1, ... for the G query heads of that kv head, one wave of the workgroup per head
// (threadIdx.y).  Blocks past the waves zero the output rows of empty sequences.
constexpr int kFusedCounterTable = 512;          // clients whose sums a merge-launch workgroup keeps in LDS
constexpr int kFusedCounterRequests = 1024;      // requests per such workgroup

template <typename T, int G>
__global__ __launch_bounds__(kWave * G) void decode_merge_kernel(const DecodeHeader* __restrict__ header,
                                                             const int32_t* __restrict__ seq_lens,
                                                             const int4* __restrict__ wave_desc,
                                                             const float2* __restrict__ part_ml,
                                                             const float* __restrict__ part_acc,
                                                             void* __restrict__ out, int32_t out_f32,
                                                             int32_t num_seqs,
                                                             int32_t num_q_heads, int32_t num_kv_heads,
                                                             int32_t max_waves, int32_t max_tokens,
                                                             CounterJob job) {
  __shared__ u64 counter_table[kFusedCounterTable];
  const int lane = threadIdx.x;                          // dims 2*lane, 2*lane+1
  constexpr int group = G;
  const int g = threadIdx.y;                             // query head inside the group
  const int tid = g * kWave + lane;
  if ((int)blockIdx.x >= max_waves + num_seqs) {         // the step's counter update
    const int begin = ((int)blockIdx.x - max_waves - num_seqs) * kFusedCounterRequests;
    counter_reduce_slice<kWave * G, kFusedCounterTable>(counter_table, job.counters, job.num_clients, job.client_ids,
                                                        begin, min(job.n, begin + kFusedCounterRequests),
                                                        LinearTerm{job.n_in, job.n_out, job.w_p, job.w_q}, tid);
    return;
  }
  if ((int)blockIdx.x >= max_waves) {                    // empty sequences: all-zero rows
    const int r = blockIdx.x - max_waves;
    if (min(seq_lens[r], max_tokens) > 0) return;
    const int words = num_q_heads * (out_f32 ? kHeadDim : kHeadDim / 2);    // 4-byte words of one output row block
    uint32_t* dst = static_cast<uint32_t*>(out) + (size_t)r * words;
    for (int i = tid; i < words; i += kWave * G) dst[i] = 0u;
    return;
  }
  const int w = blockIdx.x;
  const int waves = header->waves;
  if (w == 0 || w >= waves) return;
  const int4 d = wave_desc[w];                           // (r, kv head, block) where wave w starts
  if (d.z == 0) return;                                  // the cut coincides with a sequence-head boundary
  if (d.z > wave_desc[w - 1].w) return;                  // the beginning lies before wave w-1: an earlier block merges it
  const int nb = (min(max(seq_lens[d.x], 0), max_tokens) + kBlockSize - 1) / kBlockSize;
  const RangeMap map{header->quot, (uint32_t)header->rem, (uint32_t)waves};
  const long long g1 = map.start(w) + (nb - d.z);         // end of the sequence-head in the unit stream (only blocks lie between)
  {
    // wave w-1 holds the beginning (its slot 1); waves w.. hold continuations (their slot 0)
    float m = part_ml[((size_t)(w - 1) * 2 + 1) * group + g].x;
    int w_end = w;
    while (w_end < waves && map.start(w_end) < g1) {
      m = fmaxf(m, part_ml[((size_t)w_end * 2) * group + g].x);
      ++w_end;
    }
    float l = 0.f, a0 = 0.f, a1 = 0.f;
    for (int j = w - 1; j < w_end; ++j) {
      const size_t pi = ((size_t)j * 2 + (j == w - 1 ? 1 : 0)) * group + g;
      const float2 ml = part_ml[pi];
      const float wgt = fast_exp2(ml.x - m);
      const float2 a = *reinterpret_cast<const float2*>(part_acc + pi * kPartialFloats + 2 * lane);
      l = fmaf(ml.y, wgt, l);
      a0 = fmaf(a.x, wgt, a0);
      a1 = fmaf(a.y, wgt, a1);
    }
    const float inv = 1.f / l;
    const size_t row = ((size_t)d.x * num_q_heads + d.y * group + g) * kHeadDim;       // in elements
    if (out_f32)
      reinterpret_cast<float2*>(static_cast<float*>(out) + row)[lane] = make_float2(a0 * inv, a1 * inv);
    else
      reinterpret_cast<uint32_t*>(static_cast<uint16_t*>(out) + row)[lane] = pack2<T>(a0 * inv, a1 * inv);
  }
}

// ---------------------------------------------------- general block size ----
// KV blocks of fewer than 16 tokens (the paper's own system pages its cache one token at a time, Section 5.1).
// One wave per (sequence, kv head) of a decode step, or per (chunk token, kv head) of a prefill chunk with its
// causal limit, gathers 16 tokens at a time through the block table, whatever the block size, and hands them to
// the vector-ALU engine of the tuned decode kernel for the G query heads of the group at once (so K and V are
// read once, not once per query head).  No workspace; not tuned beyond that (measured on 256 / 512-sequence
// batches like cfg3 / cfg4: 5.2-5.4 TB/s with one query head per KV head against 6.5 through 16-token blocks).
template <typename T, int G>
__global__ __launch_bounds__(kWave) void attend_general_kernel(
    const uint16_t* __restrict__ q, const int32_t* __restrict__ cu_q_lens, const uint16_t* __restrict__ k_cache,
    const uint16_t* __restrict__ v_cache, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ seq_lens, void* __restrict__ out, int32_t out_f32, int32_t num_kv_heads,
    int32_t max_blocks_per_seq, int32_t block_size, float scale2) {
  const int r = blockIdx.z, kv_head = blockIdx.y, lane = threadIdx.x;
  const int num_q_heads = num_kv_heads * G;
  const int s_len = min(max(seq_lens[r], 0), max_blocks_per_seq * block_size);
  int q_row = r, n_keys = s_len;                       // decode: every cached token is visible
  if (cu_q_lens != nullptr) {                          // prefill chunk: token i at position s_len - lq + i sees keys 0 .. position
    const int q_begin = cu_q_lens[r];
    const int lq = cu_q_lens[r + 1] - q_begin;
    if ((int)blockIdx.x >= lq) return;
    q_row = q_begin + blockIdx.x;
    n_keys = s_len < lq ? 0 : s_len - lq + (int)blockIdx.x + 1;     // a context shorter than its chunk: zero rows
  }
  const size_t row_elems = ((size_t)q_row * num_q_heads + kv_head * G) * kHeadDim;     // G consecutive rows
  void* const out_rows = static_cast<char*>(out) + row_elems * (out_f32 ? 4 : 2);
  if (n_keys == 0) {
    uint32_t* dst = static_cast<uint32_t*>(out_rows);
    for (int i = lane; i < G * (out_f32 ? kHeadDim : kHeadDim / 2); i += kWave) dst[i] = 0u;
    return;
  }
  ValuEngine<T, G> eng;
  eng.init(lane, nullptr);
  u32x4 qreg[G], k[4], v[4];
  eng.load_q(qreg, q + row_elems);
  const int32_t* __restrict__ table = block_table + (size_t)r * max_blocks_per_seq;
  for (int j0 = 0; j0 < n_keys; j0 += kBlockSize) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {                      // lane = 16 * row + sub: token j0 + 4i + row, dims 8 sub ..
      const int tok = min(j0 + 4 * i + eng.row, n_keys - 1);        // past the end: a real row, masked by the engine
      const size_t off = cache_row_offset(slot_of(table, tok, block_size), kv_head, num_kv_heads, block_size) + eng.sub * 8;
      k[i] = *reinterpret_cast<const u32x4*>(k_cache + off);
      v[i] = *reinterpret_cast<const u32x4*>(v_cache + off);
    }
    eng.block(qreg, k, v, scale2, min(kBlockSize, n_keys - j0));
  }
  eng.finish(true, PieceSink{out_rows, out_f32 != 0, nullptr, nullptr});
}

template <typename T>
static int launch_general_typed(const vtc_attn_params& p, int32_t num_seqs, const void* q, const int32_t* cu_q_lens,
                                int32_t max_q_len, const void* k_cache, const void* v_cache,
                                const int32_t* block_table, const int32_t* seq_lens, void* out, hipStream_t stream) {
  const dim3 grid(cu_q_lens ? max_q_len : 1, p.num_kv_heads, num_seqs);
  auto go = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, grid, dim3(kWave), 0, stream, static_cast<const uint16_t*>(q), cu_q_lens,
                       static_cast<const uint16_t*>(k_cache), static_cast<const uint16_t*>(v_cache), block_table,
                       seq_lens, out, p.out_dtype == VTC_F32 ? 1 : 0, p.num_kv_heads, p.max_blocks_per_seq,
                       p.block_size, p.scale * kLog2e);
  };
  switch (p.num_q_heads / p.num_kv_heads) {
    case 1: go(attend_general_kernel<T, 1>); break;
    case 2: go(attend_general_kernel<T, 2>); break;
    case 4: go(attend_general_kernel<T, 4>); break;
    case 8: go(attend_general_kernel<T, 8>); break;
    default: return VTC_ERR_UNSUPPORTED;
  }
  return hipGetLastError() == hipSuccess ? VTC_OK : VTC_ERR_HIP;
}

int launch_attend_general(const vtc_attn_params& p, int32_t num_seqs, const void* q, const int32_t* cu_q_lens,
                          int32_t max_q_len, const void* k_cache, const void* v_cache, const int32_t* block_table,
                          const int32_t* seq_lens, void* out, hipStream_t stream) {
  if (num_seqs > 65535 || p.num_kv_heads > 65535) return VTC_ERR_UNSUPPORTED;      // grid limits
  if (p.dtype == VTC_F16)
    return launch_general_typed<F16>(p, num_seqs, q, cu_q_lens, max_q_len, k_cache, v_cache, block_table, seq_lens, out,
                                     stream);
  return launch_general_typed<BF16>(p, num_seqs, q, cu_q_lens, max_q_len, k_cache, v_cache, block_table, seq_lens, out,
                                    stream);
}

// -------------------------------------------------------------- launcher ----
template <typename T, int G, typename Engine>
static int launch_typed(const vtc_attn_params& p, int32_t num_seqs, const void* q, const void* k_cache,
                        const void* v_cache, const int32_t* block_table, const int32_t* seq_lens, void* out,
                        void* workspace, int32_t max_waves, hipStream_t stream, hipEvent_t ev_begin,
                        hipEvent_t ev_end, const CounterJob& job) {
  // Grid: a fixed number of waves per compute unit, all resident at once (no wave waits for a slot while the
  // others are already half way through their share), or as many of them as the caller's workspace has room for.
  static_assert(Engine::kWavesPerCu <= 4 * Engine::kMinWavesPerSimd, "the launch must fit the kernel's guaranteed occupancy");
  const long long resident = (long long)device_cu_count() * Engine::kWavesPerCu;
  const int grid = (int)(resident < max_waves ? resident : max_waves);

  const DecodeWorkspace ws = decode_workspace_layout(p, num_seqs, grid);
  char* base = static_cast<char*>(workspace);
  DecodeHeader* header = reinterpret_cast<DecodeHeader*>(base + ws.header_off);
  unsigned long long* seg_prefix = reinterpret_cast<unsigned long long*>(base + ws.seg_prefix_off);
  int4* wave_desc = reinterpret_cast<int4*>(base + ws.wave_desc_off);
  float2* part_ml = reinterpret_cast<float2*>(base + ws.ml_off);
  float* part_acc = reinterpret_cast<float*>(base + ws.acc_off);
  const int32_t max_tokens = p.max_blocks_per_seq * kBlockSize;
  const int32_t out_f32 = p.out_dtype == VTC_F32 ? 1 : 0;

  const bool self_plan = num_seqs <= kSelfPlanMaxSeqs;
  if (!self_plan)
    hipLaunchKernelGGL(decode_plan_kernel, dim3(1), dim3(kPlanThreads), 0, stream, seq_lens, num_seqs,
                       p.num_kv_heads, max_tokens, grid, header, seg_prefix, wave_desc);
  if (ev_begin) (void)hipEventRecord(ev_begin, stream);      // a failure shows up in hipGetLastError() below
  hipLaunchKernelGGL((decode_attend_kernel<T, G, Engine>), dim3(grid), dim3(kWave), 0, stream,
                     static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k_cache),
                     static_cast<const uint16_t*>(v_cache), block_table, seq_lens, out, out_f32,
                     wave_desc, part_ml, part_acc, p.num_kv_heads, p.max_blocks_per_seq, p.scale * kLog2e,
                     self_plan ? num_seqs : 0, header);
  if (ev_end) (void)hipEventRecord(ev_end, stream);
  const int counter_blocks = (job.n + kFusedCounterRequests - 1) / kFusedCounterRequests;
  hipLaunchKernelGGL((decode_merge_kernel<T, G>), dim3(grid + num_seqs + counter_blocks), dim3(kWave, G), 0, stream,
                     header, seq_lens, wave_desc, part_ml, part_acc, out, out_f32, num_seqs,
                     p.num_q_heads, p.num_kv_heads, grid, max_tokens, job);
  return hipGetLastError() == hipSuccess ? VTC_OK : VTC_ERR_HIP;
}

template <typename T>
static int launch_group(const vtc_attn_params& p, int32_t num_seqs, const void* q, const void* k_cache,
                        const void* v_cache, const int32_t* block_table, const int32_t* seq_lens, void* out,
                        void* workspace, int32_t max_waves, hipStream_t stream, hipEvent_t ev_begin,
                        hipEvent_t ev_end, const CounterJob& job) {
#define VTC_DECODE_CASE(G, ENGINE)                                                                             \
  case G:                                                                                                      \
    return launch_typed<T, G, ENGINE<T, G>>(p, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out,      \
                                            workspace, max_waves, stream, ev_begin, ev_end, job)
  switch (p.num_q_heads / p.num_kv_heads) {
    VTC_DECODE_CASE(1, ValuEngine);      // one query head per KV head: 1 flop per byte, vector ALUs
    VTC_DECODE_CASE(2, MfmaEngine);      // grouped queries: the vector path becomes ALU-bound, matrix cores
    VTC_DECODE_CASE(4, MfmaEngine);
    VTC_DECODE_CASE(8, MfmaEngine);
    default: return VTC_ERR_UNSUPPORTED;
  }
#undef VTC_DECODE_CASE
}

int launch_decode(const vtc_attn_params& p, int32_t num_seqs, const void* q, const void* k_cache,
                  const void* v_cache, const int32_t* block_table, const int32_t* seq_lens, void* out,
                  void* workspace, int32_t max_waves, hipStream_t stream, hipEvent_t ev_begin, hipEvent_t ev_end,
                  const CounterJob& job) {
  // the batch's cost units per kv head, and one sequence's over all kv heads, must fit 31 bits (the plan's prefixes
  // and offsets are 32-bit)
  if ((long long)num_seqs * ((long long)p.max_blocks_per_seq + kPieceUnits) >= (1ll << 31) ||
      ((long long)p.max_blocks_per_seq + kPieceUnits) * p.num_kv_heads >= (1ll << 31))
    return VTC_ERR_UNSUPPORTED;
  if (p.dtype == VTC_F16)
    return launch_group<F16>(p, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace, max_waves, stream,
                             ev_begin, ev_end, job);
  return launch_group<BF16>(p, num_seqs, q, k_cache, v_cache, block_table, seq_lens, out, workspace, max_waves, stream,
                            ev_begin, ev_end, job);
}

}  // namespace vtc
