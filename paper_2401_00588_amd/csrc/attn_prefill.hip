// Causal prefill-chunk attention over a paged KV cache on the CDNA4 matrix cores
// (the attention part of forward_prefill(B_new), Algorithm 2 of the paper;
// Section 2.1 describes prefilling as processing all prompt tokens at once).
//
// Work split.  A workgroup is 4 wavefronts; each wave owns 32 query rows, where a
// row is a (chunk token, query head) pair.  All rows of a workgroup read the same
// KV head, so with grouped-query attention the 4 waves take up to 4 query heads of
// the group for the same 32 tokens (HW = heads per workgroup), and with HW < 4 the
// remaining waves take further 32-token tiles.  The workgroup walks the keys it can
// see in tiles of 64 keys.  A K and a V tile live in LDS once for all 4 waves, double-
// buffered, and get there without passing through registers: wave w copies KV block
// k0/16 + w of the tile with 16-byte global-to-LDS loads (a load instruction fills
// 1 KiB = 4 rows of LDS contiguously, lane l at byte 16 l), the loads of tile j+1 being
// in flight while tile j is used.  Rows are 256 bytes with no padding; instead the
// 16-byte chunks of a row are permuted on the way in (the lane picks which chunk of the
// global row it fetches): K chunk c of row r sits at position c ^ (r & 15), V chunk c at
// c ^ 4 (r & 3), which makes the 16-byte row reads of K and the 8-byte transposing reads
// of V hit every LDS bank equally.
//
// Per tile and wave, with v_mfma_f32_32x32x16 (A: 32 rows x 16, B: 16 x 32 columns):
//   S^T = K . Q^T      2 key blocks x 8 steps over head_dim; A = 32 keys of the K tile
//                      (16-byte LDS row reads), B = Q^T kept in registers
//   online softmax     per query row = per lane column; fp32; exp2 domain
//   O^T += V^T . P^T   A = V^T fragments: 4 consecutive keys at one dim per 8-byte
//                      transposing LDS read (ds_read_b64_tr_b16) from the row-major
//                      V tile; B = P^T, which is the accumulator layout of S^T as it
//                      stands (lane: query row l%32, keys 8*(v/4) + 4*(l/32) + v%4)
// The contraction slots of the second product are assigned to keys so that no data
// moves between the two products: slots 0..3 of lane half hg are keys 16t+4hg+0..3
// and slots 4..7 are keys 16t+8+4hg+0..3 of a 32-key block, for t = 0, 1.
#include "vtc_internal.h"

namespace vtc {

using f32x16 = float __attribute__((ext_vector_type(16)));
using f32x4 = float __attribute__((ext_vector_type(4)));
using f16x8 = _Float16 __attribute__((ext_vector_type(8)));
using bf16x8 = __bf16 __attribute__((ext_vector_type(8)));
using s16x4 = short __attribute__((ext_vector_type(4)));
using u32x2 = uint32_t __attribute__((ext_vector_type(2)));

constexpr int kQkAhead = 6;              // K fragments in flight ahead of the product that uses them
constexpr int kPvAhead = 4;              // V^T fragments in flight ahead of the product(s) that use them
constexpr int kPfThreads = 256;
constexpr int kPfRows = 32;              // query rows per wave
constexpr int kPfKTile = 64;             // keys per LDS tile
constexpr int kTileElems64 = kPfKTile * kHeadDim;    // one K or V tile in LDS, unpadded (16 KiB)
constexpr int kPitchO = kHeadDim + 8;                // output patch rows: 272 B
static_assert(4 * kPfRows * kPitchO <= 4 * kTileElems64, "the four output patches must fit the tile buffers");

template <typename T>
__device__ __forceinline__ f32x16 mfma32(u32x4 a, u32x4 b, f32x16 c);
template <>
__device__ __forceinline__ f32x16 mfma32<F16>(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <>
__device__ __forceinline__ f32x16 mfma32<BF16>(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// 8-byte transposing LDS read: inside each group of 16 lanes, lane j receives element j%4 of the
// 8-byte chunks addressed by lanes j/4, 4 + j/4, 8 + j/4 and 12 + j/4 (verified on gfx950).
__device__ __forceinline__ u32x2 lds_read_tr16(const uint16_t* p) {
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
  return __builtin_bit_cast(u32x2, v);
}

// 16 bytes per lane from global memory straight into LDS: lane l of the wave writes LDS bytes
// [dst + 16 l, dst + 16 l + 16); dst is wave-uniform (it travels in M0).  Issued as inline assembly so that
// the compiler does not order every later LDS read behind it: completion is waited for explicitly
// (s_waitcnt vmcnt(0) + barrier) before the buffer is read.  Loads the compiler does not know about can
// only make its own vmcnt waits longer, never shorter (the counter retires in issue order).
__device__ __forceinline__ void lds_dma16(const uint16_t* src, uint16_t* dst_uniform) {
  typedef __attribute__((address_space(3))) uint16_t lds_u16;
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_u16*)dst_uniform);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(src) : "memory", "m0");
}

// The same for data that is read once (the q rows): marked non-temporal so that it does not displace the K/V
// tiles, which several workgroups share, from the L2.
__device__ __forceinline__ void lds_dma16_once(const uint16_t* src, uint16_t* dst_uniform) {
  typedef __attribute__((address_space(3))) uint16_t lds_u16;
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_u16*)dst_uniform);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" ::"s"(lds_addr), "v"(src) : "memory", "m0");
}

// The same with a wave-uniform base address and 32-bit per-lane byte offsets, four loads at once: load i reads
// base + o_i + 1024 i and writes LDS bytes [dst + 1024 i + 16 l, + 16) (the instruction's immediate offset moves
// both addresses).  One KV block's K or V rows (4 KiB) are four such 1 KiB slices; the addresses cost no vector
// arithmetic per tile.
__device__ __forceinline__ void lds_dma16_x4(const uint16_t* base_uniform, uint32_t o0, uint32_t o1, uint32_t o2,
                                             uint32_t o3, uint16_t* dst_uniform) {
  typedef __attribute__((address_space(3))) uint16_t lds_u16;
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_u16*)dst_uniform);
  // Pin the base to scalar registers also where the compiler would rather form the address with vector arithmetic
  // (an "s" operand does not force that by itself).  The builtin returns int: widen through uint32_t.
  const uint64_t base_bits = (uint64_t)(uintptr_t)base_uniform;
  base_uniform = (const uint16_t*)(uintptr_t)(
      (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)base_bits) |
      ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(base_bits >> 32)) << 32));
  asm volatile(
      "s_mov_b32 m0, %0\n\ts_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %5\n\t"
      "global_load_lds_dwordx4 %2, %5 offset:1024\n\t"
      "global_load_lds_dwordx4 %3, %5 offset:2048\n\t"
      "global_load_lds_dwordx4 %4, %5 offset:3072" ::"s"(lds_addr),
      "v"(o0), "v"(o1), "v"(o2), "v"(o3), "s"(base_uniform)
      : "memory", "m0");
}

template <typename T, int HW, bool kPosScale>
__global__ __launch_bounds__(kPfThreads, 2) void prefill_chunk_kernel(
    const uint16_t* __restrict__ q, const int32_t* __restrict__ cu_q_lens, const uint16_t* __restrict__ k_cache,
    const uint16_t* __restrict__ v_cache, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ seq_lens, void* __restrict__ out, int32_t out_f32, int32_t num_q_heads,
    int32_t num_kv_heads, int32_t max_blocks_per_seq, float scale2, int32_t xcds, int32_t cus_per_xcd) {
  constexpr int TT = 4 / HW;                       // 32-token tiles per workgroup
  constexpr int kTokensPerWg = kPfRows * TT;
  __shared__ __attribute__((aligned(1024))) uint16_t lds[4 * kTileElems64];    // K buffers 0, 1, then V buffers 0, 1
  uint16_t* const k_lds = lds;
  uint16_t* const v_lds = lds + 2 * kTileElems64;

  // Workgroups are dispatched round-robin over the device's XCDs (each with its own L2) in linear
  // block order.  All query tiles that read the same K/V -- one (sequence, kv head) -- are
  // placed on one XCD, so that K/V comes out of that XCD's L2 after the first tile's read.
  const int n_qt = gridDim.x;                                      // query tiles per (sequence, head slot)
  const int n_units = gridDim.y * gridDim.z;                       // (head slot, sequence) pairs
  const int linear = blockIdx.x + n_qt * (blockIdx.y + gridDim.y * blockIdx.z);
  int qt, unit;
  if (xcds > 1 && n_units % xcds == 0) {
    const int per_xcd = n_units / xcds;
    const int j = linear / xcds;
    // Units go in groups whose query tiles come to about one workgroup per CU of the XCD, and inside a group the
    // order is query tile first, unit second: the XCD's 4 MB L2 then serves the K/V of a few units at a time, each
    // of them to all its query tiles at once, instead of a slice of every unit's K/V in every round of workgroups.
    // (Measured on 16 units x 8 query tiles per XCD: groups of 4 units -7 % on a 256-key chunk, -1.5 % on a
    // 512-key chunk against no grouping; groups of 1, 2, 3 or 8 units are slower than 4.)
    const int gsz = min(per_xcd, max(1, cus_per_xcd / n_qt));
    const int per_group = gsz * n_qt;
    const int grp = j / per_group, jj = j % per_group;
    const int in_grp = min(gsz, per_xcd - grp * gsz);             // the last group may be smaller
    unit = (grp * gsz + jj % in_grp) * xcds + linear % xcds;
    qt = jj / in_grp;
  } else {                                                         // odd shapes, or one die: plain order
    qt = blockIdx.x;
    unit = blockIdx.y + gridDim.y * blockIdx.z;
  }
  qt = n_qt - 1 - qt;                                              // later tiles see more keys: start them first
  const int slot = unit % gridDim.y;
  const int r = unit / gridDim.y;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // uniform: block ids and LDS bases stay scalar
  // Everything the first tile's addresses depend on is fetched in one round trip: the chunk bounds, the context
  // length and -- on the guess that the sequence has that many blocks -- the id of this wave's first KV block.
  const int32_t* __restrict__ table = block_table + (size_t)r * max_blocks_per_seq;
  const int q_begin = cu_q_lens[r];
  const int q_end = cu_q_lens[r + 1];
  const int s_raw = seq_lens[r];
  const int32_t guessed_id = table[min(wave, max_blocks_per_seq - 1)];
  // ... and the sequence's first 64 block ids, one per lane; later tiles read theirs out of this register, so the
  // key loop holds no scalar memory loads (their returns would share a counter with the LDS reads of the products)
  int32_t ids = table[min((int)(threadIdx.x & 63), max_blocks_per_seq - 1)];
  int ids_chunk = 0;                                               // ids holds blocks 64 ids_chunk .. + 63
  asm volatile("" ::: "memory");                                   // keep the four loads together, ahead of their first use
  const int lq = q_end - q_begin;
  if (qt * kTokensPerWg >= lq) return;                             // uniform over the workgroup
  if (min(max(s_raw, 0), max_blocks_per_seq * kBlockSize) < lq) {
    // The context is shorter than the chunk that is said to end it: there is no position to give the chunk's
    // tokens.  Their output rows are zeroed and no cache block is read for the sequence.
    const int words_per_row = out_f32 ? kHeadDim : kHeadDim / 2;   // 4-byte words of one (token, head) row
    const int tok_lo = qt * kTokensPerWg, tok_hi = min(lq, tok_lo + kTokensPerWg);
    const int group0 = num_q_heads / num_kv_heads;
    const int head_lo = (slot / (group0 / HW)) * group0 + (slot % (group0 / HW)) * HW;
    for (int i = tid; i < (tok_hi - tok_lo) * HW * words_per_row; i += kPfThreads) {
      const int w = i % words_per_row, hh = (i / words_per_row) % HW, t = i / (words_per_row * HW);
      static_cast<uint32_t*>(out)[((size_t)(q_begin + tok_lo + t) * num_q_heads + head_lo + hh) * words_per_row + w] = 0u;
    }
    return;
  }
  const int group = num_q_heads / num_kv_heads;
  const int subs = group / HW;                                     // workgroups per kv head
  const int kvh = slot / subs;
  const int sub = slot % subs;
  const int s_len = min(max(s_raw, 0), max_blocks_per_seq * kBlockSize);
  const int p0 = max(s_len - lq, 0);                               // absolute position of chunk token 0

  const int lane = tid & 63;
  const int col = lane & 31;       // query row within the wave (MFMA column index)
  const int hg = lane >> 5;        // lane half: contraction slots 8*hg .. 8*hg+7
  const int kswz = hg ^ (col & 15);   // K chunk 2 ks + hg of this lane's row sits at position kswz ^ 2 ks
  const int h = kvh * group + sub * HW + wave % HW;                // this wave's query head
  const int tok0 = qt * kTokensPerWg + (wave / HW) * kPfRows;      // its first chunk token
  const bool wave_has_rows = tok0 < lq;
  const int i_row = tok0 + col;
  const int pq = p0 + i_row;                                       // absolute position of this lane's query row
  // keys the workgroup / the wave can see
  const int wg_kv_end = min(s_len, p0 + min(lq, qt * kTokensPerWg + kTokensPerWg));
  const int wave_kv_end = wave_has_rows ? min(s_len, p0 + min(lq, tok0 + kPfRows)) : 0;

  // The wave's 32 q rows (8 KiB) go global -> LDS -> registers: fetched as whole 256-byte rows (4 rows per load
  // instruction, every cache line used in full), parked in the tile buffers that the second tile will overwrite
  // later, with the chunk permutation of the K tiles, then read in the B-operand layout of the first product.
  u32x4 qf[8];                                                      // Q^T operand, filled once the rows are in LDS
  uint16_t* const q_park = (wave < 2 ? k_lds : v_lds) + kTileElems64 + (wave & 1) * (kPfRows * kHeadDim);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int j = 4 * i + (lane >> 4);                                                   // row of the wave's 32
    const uint16_t* src = q + ((size_t)(q_begin + min(tok0 + j, lq - 1)) * num_q_heads + h) * kHeadDim;
    lds_dma16_once(src + (((lane & 15) ^ (j & 15)) * 8), q_park + i * 4 * kHeadDim);
  }

  f32x16 oacc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
  float m_run = -INFINITY;         // reference exponent of the weights: within 8 of the running maximum of the scaled logits (log2 domain)
  float l_run = 0.f;               // running sum; this lane half's keys only

  // Tile loads.  Wave w brings KV block (k0/16 + w) into rows 16w .. 16w+15 of the K and V buffers: load i
  // of a wave fills rows 16w + 4i .. +3, lane l row 4i + l/16 of the block, chunk position l%16.  The block id
  // is wave-uniform and is read out of the id register one tile ahead of the loads that need it.  A key the
  // workgroup cannot see is replaced by the last key it can see, whose rows are real, finite and already in
  // cache; its weight is zero through the causal mask.
  const int kv_last = max(wg_kv_end - 1, 0);
  const int last_block = kv_last / kBlockSize;
  auto lookup = [&](int k0) {
    const int b = min(k0 / kBlockSize + wave, last_block);
    if ((b >> 6) != ids_chunk) {                                   // uniform; once per 1024 keys
      ids_chunk = b >> 6;
      ids = table[min(ids_chunk * 64 + (int)(threadIdx.x & 63), last_block)];
    }
    return __builtin_amdgcn_readlane(ids, b & 63);
  };
  const int pos16 = lane & 15;                                     // chunk position inside the LDS row
  const int row4 = lane >> 4;
  // per-lane byte offsets inside a (block, head) tile for the four loads of a block (see lds_dma16_x4); they do not
  // change from tile to tile
  uint32_t koff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) koff[i] = row4 * 256 + ((pos16 ^ (4 * i + row4)) * 16);   // K: chunk c at c ^ (r & 15)
  const uint32_t voff = row4 * 256 + ((pos16 ^ (4 * row4)) * 16);                       // V: chunk c at c ^ 4 (r & 3)
  auto issue = [&](int k0, int buf, int32_t block_id) {
    const size_t block_base = ((size_t)block_id * num_kv_heads + kvh) * kBlockSize;
    uint16_t* const kdst = k_lds + buf * kTileElems64 + wave * (kBlockSize * kHeadDim);
    uint16_t* const vdst = v_lds + buf * kTileElems64 + wave * (kBlockSize * kHeadDim);
    if (k0 + wave * kBlockSize + kBlockSize - 1 <= kv_last) {       // the whole block is visible: uniform addresses
      lds_dma16_x4(k_cache + block_base * kHeadDim, koff[0], koff[1], koff[2], koff[3], kdst);
      lds_dma16_x4(v_cache + block_base * kHeadDim, voff, voff, voff, voff, vdst);
      return;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = 4 * i + row4;                                // row of the block = LDS row & 15
      const int key = min(k0 + wave * kBlockSize + row, kv_last);
      const size_t grow = (block_base + (key & 15)) * kHeadDim;
      const int ck = pos16 ^ row;
      const int cv = pos16 ^ (4 * row4);
      lds_dma16(k_cache + grow + ck * 8, kdst + i * 4 * kHeadDim);
      lds_dma16(v_cache + grow + cv * 8, vdst + i * 4 * kHeadDim);
    }
  };
  // This wave's tile loads have landed in LDS, then every wave's have, and every wave is done with the other buffer.
  auto tiles_ready = [&]() {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  };

  // ---- one tile of work for this wave, from LDS buffer `buf`
  auto compute = [&](int k0, int buf) {
    if (k0 < wave_kv_end) {
      const uint16_t* ks_tile = k_lds + buf * kTileElems64;
      const uint16_t* vs_tile = v_lds + buf * kTileElems64;
      // ---- S^T = K . Q^T
      f32x16 sacc[2];
#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[sb][v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const u32x4 kf = *reinterpret_cast<const u32x4*>(&ks_tile[(sb * 32 + col) * kHeadDim + ((kswz ^ (2 * ks)) * 8)]);
          sacc[sb] = mfma32<T>(kf, qf[ks], sacc[sb]);
        }
      }
      // order of the 16 fragment reads and 16 products above: reads run kQkAhead fragments ahead of their use
      __builtin_amdgcn_sched_group_barrier(0x100, kQkAhead, 0);
#pragma unroll
      for (int i = 0; i < 16 - kQkAhead; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, kQkAhead, 0);
      // ---- causal mask (only tiles that reach past the wave's first query position), row maximum
      const float masked = kPosScale ? -INFINITY : INFINITY;
      if (k0 + kPfKTile - 1 > p0 + tok0) {
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int key = k0 + sb * 32 + 8 * (v >> 2) + 4 * hg + (v & 3);
            if (key > pq) sacc[sb][v] = masked;
          }
      }
      float mx = -INFINITY;          // max over keys of sign(scale) * raw logit
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, kPosScale ? sacc[sb][v] : -sacc[sb][v]);
      {
        // The other half of the row's keys sits 32 lanes away.  v_permlane32_swap exchanges lanes 32..63 of its first
        // operand with lanes 0..31 of its second, so with the row maximum in both, every lane finds its own half in
        // one and the other half in the other: a vector instruction instead of an LDS round trip in the middle of the
        // tile's dependency chain.  (Inline assembly: through the builtin this compiler hands out the first result
        // register for both results.)
        uint32_t mx_a = __builtin_bit_cast(uint32_t, mx), mx_b = mx_a;
        asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(mx_a), "+v"(mx_b));
        mx = fmaxf(__builtin_bit_cast(float, mx_a), __builtin_bit_cast(float, mx_b));
      }
      const float m_tile = mx * (kPosScale ? scale2 : -scale2);     // = max of the scaled logits, or -inf
      // The reference exponent follows the maximum only when that has grown by more than 8 since it last moved,
      // so weights stay <= 2^8 (exact in either storage type's range) and the 64 accumulators are rescaled once or
      // twice per row instead of in almost every tile (-3 % kernel time).  The choice is per row and depends on
      // that row's keys alone, so a row's result does not depend on how the prompt was cut into chunks.
      const float m_new = m_tile > m_run + 8.f ? m_tile : m_run;
      const float m_sub = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = fast_exp2(m_run - m_sub);
      m_run = m_new;
      // ---- P^T = exp2(scaled logit - m), packed to the storage type as the B operands
      // bf16 keeps 8 bits of a weight.  What the rounding drops enters the second product as an operand of its
      // own (pr), so the weights act with 16 bits; fp16's 11 bits are left as they are.
      constexpr bool kSplitP = __is_same(T, BF16);
      // The row sum adds up the weights before rounding, with plain additions: the dot instruction that would add up
      // the rounded pair executes in the matrix pipeline and cannot overlap the products (measured: 64 of them under
      // 8 products take 636 cycles where 64 additions take 348).  The sum then differs from the sum of the operands
      // by their rounding, 2^-17 (bf16, two operands) or 2^-12 (fp16) of a weight, with either sign.
      float psum4[4] = {0.f, 0.f, 0.f, 0.f};
      u32x4 pb[2][2];
      u32x4 pr[kSplitP ? 2 : 1][2];
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const float pa = fast_exp2(fmaf(sacc[sb][8 * t + 2 * w], scale2, -m_sub));
            const float pc = fast_exp2(fmaf(sacc[sb][8 * t + 2 * w + 1], scale2, -m_sub));
            const uint32_t hi = pack2<T>(pa, pc);
            pb[sb][t][w] = hi;
            psum4[w] += pa + pc;
            if constexpr (kSplitP) {
              const uint32_t lo = pack2<T>(pa - __builtin_bit_cast(float, hi << 16),
                                           pc - __builtin_bit_cast(float, hi & 0xffff0000u));
              pr[sb][t][w] = lo;
            }
          }
      l_run = l_run * alpha + ((psum4[0] + psum4[1]) + (psum4[2] + psum4[3]));
      if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0ull) {      // skip the rescale when no row's maximum moved
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int v = 0; v < 16; ++v) oacc[db][v] *= alpha;
      }
      // ---- O^T += V^T . P^T
      // lane -> (key tr_row of 4, 4-dim group tr_col of 32 dims): chunk 4 db + tr_col / 8 of the row, moved by
      // the V permutation to 4 (db ^ tr_row) + tr_col / 8
      const int tr_row = (lane & 15) >> 2;
      const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const uint16_t* vrow = vs_tile + (sb * 32 + 16 * t + 4 * hg + tr_row) * kHeadDim + tr_col;
#pragma unroll
          for (int db = 0; db < 4; ++db) {
            const int dofs = 32 * (db ^ tr_row);
            const u32x2 lo = lds_read_tr16(vrow + dofs);                       // keys 16t+4hg+0..3
            const u32x2 hi = lds_read_tr16(vrow + 8 * kHeadDim + dofs);        // keys 16t+8+4hg+0..3
            const u32x4 vt = u32x4{lo[0], lo[1], hi[0], hi[1]};
            oacc[db] = mfma32<T>(vt, pb[sb][t], oacc[db]);
            if constexpr (kSplitP) oacc[db] = mfma32<T>(vt, pr[sb][t], oacc[db]);
          }
        }
      // order of the 32 transposing reads and the 16 (bf16: 32) products above: kPvAhead fragments (2 reads each)
      // ahead of use; the first reads may start while the weights are still being exponentiated
      constexpr int kPerFrag = kSplitP ? 2 : 1;                     // products that consume one V^T fragment
      __builtin_amdgcn_sched_group_barrier(0x100, 2 * kPvAhead, 0);
#pragma unroll
      for (int i = 0; i < 16 - kPvAhead; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, kPerFrag, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, kPerFrag * kPvAhead, 0);
    }

  };

  // Pipeline over key tiles: while tile kt is used from one LDS buffer, the loads of tile kt+1 fill the other.
  // One barrier per tile: behind it every wave's part of tile kt+1 is in LDS and nobody reads tile kt any more.
  const int n_tiles = (wg_kv_end + kPfKTile - 1) / kPfKTile;
  issue(0, 0, wave <= last_block ? guessed_id : table[last_block]);
  int32_t id1 = table[min(kPfKTile / kBlockSize + wave, last_block)];   // block id of the next tile (scalar load: the
                                                                        // id register is first needed in the loop)
  tiles_ready();
#pragma unroll
  for (int ks = 0; ks < 8; ++ks)
    qf[ks] = *reinterpret_cast<const u32x4*>(&q_park[col * kHeadDim + ((kswz ^ (2 * ks)) * 8)]);
  __syncthreads();                                                 // every wave holds its q before tile 1 lands there
  for (int kt = 0; kt < n_tiles; ++kt) {
    // (the lookup comes first: should it have to fetch the next 64 ids, no tile load is in flight behind which the
    // wait for them would queue up)
    const int32_t id2 = lookup((kt + 2) * kPfKTile);
    if (kt + 1 < n_tiles) issue((kt + 1) * kPfKTile, (kt + 1) & 1, id1);
    id1 = id2;
    compute(kt * kPfKTile, kt & 1);
    tiles_ready();
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                 // no load may still be writing LDS when the wave ends

  // ---- epilogue: normalise, round, and turn the wave's O^T (a query row per lane) into whole
  // 256-byte output rows through a private 32 x 128 LDS patch, so that the global stores are
  // 16 bytes per lane and contiguous per row.
  l_run += __shfl_xor(l_run, 32);
  // (the last tiles_ready() left every wave done with the tile buffers)
  if (wave_has_rows) {
    uint16_t* patch = lds + wave * (kPfRows * kPitchO);
    const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
    if (out_f32) {
      // fp32 rows, no rounding: the lane's 4 consecutive dims go out as one 16-byte store (the two lane halves
      // of a row fill 32 contiguous bytes per instruction)
      if (i_row < lq) {
        float* dst = static_cast<float*>(out) + ((size_t)(q_begin + i_row) * num_q_heads + h) * kHeadDim + 4 * hg;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            __builtin_nontemporal_store(
                f32x4{oacc[db][4 * j] * inv, oacc[db][4 * j + 1] * inv, oacc[db][4 * j + 2] * inv, oacc[db][4 * j + 3] * inv},
                reinterpret_cast<f32x4*>(dst + db * 32 + 8 * j));
      }
      return;
    }
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int j = 0; j < 4; ++j) {                                 // dims db*32 + 8j + 4hg + 0..3 of row `col`
        u32x2 o;
        o[0] = pack2<T>(oacc[db][4 * j] * inv, oacc[db][4 * j + 1] * inv);
        o[1] = pack2<T>(oacc[db][4 * j + 2] * inv, oacc[db][4 * j + 3] * inv);
        *reinterpret_cast<u32x2*>(&patch[col * kPitchO + db * 32 + 8 * j + 4 * hg]) = o;
      }
    // LDS operations of one wave complete in order: the reads below see the writes above
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = 4 * i + (lane >> 4);
      const u32x4 v = *reinterpret_cast<const u32x4*>(&patch[row * kPitchO + (lane & 15) * 8]);
      if (tok0 + row < lq)
        // (written once and not read again here: non-temporal, so that it does not displace K/V tiles from the L2)
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(static_cast<uint16_t*>(out) + ((size_t)(q_begin + tok0 + row) * num_q_heads + h) * kHeadDim + (lane & 15) * 8));
    }
  }
}

template <typename T, int HW>
static int launch_hw(const vtc_attn_params& p, int32_t num_seqs, const void* q, const int32_t* cu_q_lens,
                     int32_t max_q_len, const void* k_cache, const void* v_cache, const int32_t* block_table,
                     const int32_t* seq_lens, void* out, hipStream_t stream) {
  constexpr int kTokensPerWg = kPfRows * (4 / HW);
  const int group = p.num_q_heads / p.num_kv_heads;
  const long long gy = (long long)p.num_kv_heads * (group / HW);
  if (num_seqs > 65535 || gy > 65535) return VTC_ERR_UNSUPPORTED;
  dim3 grid((max_q_len + kTokensPerWg - 1) / kTokensPerWg, (unsigned)gy, num_seqs);
  float scale2 = p.scale * kLog2e;
  if (scale2 == 0.f) scale2 = 1e-30f;   // all logits equal either way; keeps (-inf) * scale of masked keys well defined
  const DeviceShape shape = device_shape();
  auto go = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, grid, dim3(kPfThreads), 0, stream, static_cast<const uint16_t*>(q), cu_q_lens,
                       static_cast<const uint16_t*>(k_cache), static_cast<const uint16_t*>(v_cache), block_table,
                       seq_lens, out, p.out_dtype == VTC_F32 ? 1 : 0, p.num_q_heads, p.num_kv_heads,
                       p.max_blocks_per_seq, scale2, shape.xcds, shape.cus / shape.xcds);
  };
  if (scale2 >= 0.f)
    go(prefill_chunk_kernel<T, HW, true>);
  else
    go(prefill_chunk_kernel<T, HW, false>);
  return hipGetLastError() == hipSuccess ? VTC_OK : VTC_ERR_HIP;
}

template <typename T>
static int launch_t(const vtc_attn_params& p, int32_t num_seqs, const void* q, const int32_t* cu_q_lens,
                    int32_t max_q_len, const void* k_cache, const void* v_cache, const int32_t* block_table,
                    const int32_t* seq_lens, void* out, hipStream_t stream) {
  switch (p.num_q_heads / p.num_kv_heads) {
    case 1: return launch_hw<T, 1>(p, num_seqs, q, cu_q_lens, max_q_len, k_cache, v_cache, block_table, seq_lens, out, stream);
    case 2: return launch_hw<T, 2>(p, num_seqs, q, cu_q_lens, max_q_len, k_cache, v_cache, block_table, seq_lens, out, stream);
    default: return launch_hw<T, 4>(p, num_seqs, q, cu_q_lens, max_q_len, k_cache, v_cache, block_table, seq_lens, out, stream);
  }
}

int launch_prefill(const vtc_attn_params& p, int32_t num_seqs, const void* q, const int32_t* cu_q_lens,
                   int32_t max_q_len, const void* k_cache, const void* v_cache, const int32_t* block_table,
                   const int32_t* seq_lens, void* out, hipStream_t stream) {
  if (p.dtype == VTC_F16)
    return launch_t<F16>(p, num_seqs, q, cu_q_lens, max_q_len, k_cache, v_cache, block_table, seq_lens, out, stream);
  return launch_t<BF16>(p, num_seqs, q, cu_q_lens, max_q_len, k_cache, v_cache, block_table, seq_lens, out, stream);
}

}  // namespace vtc
