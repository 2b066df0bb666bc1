// Attention over the paged KV pool, both phases, on MFMA with operands read straight from HBM/L2.
//
// Formulation.  Everything is computed transposed: S^T = K Q^T and O^T = V^T P^T.  With the pool
// layout K [block][head][d/32][16 positions][32] and V [block][head][d][16 slots], both left operands
// then have their contraction index contiguous in memory (d for K rows, slots for V^T rows), which is
// exactly what an MFMA lane holds (8 consecutive k of one row).  The right operand of the second product,
// P^T, is the accumulator of the first one: the row order of a key tile is a free choice (each lane
// loads its own K row), and choosing it so that a lane's accumulator registers are 8 consecutive slots
// of one block makes the registers of S^T the B operand of the PV product with no data movement
// between lanes and no LDS.  A query column is a lane, so softmax statistics are per-lane scalars.
//
// Masking is by select, never by multiplying with zero: slots past a sequence's end may hold NaN.
// V values of such slots are zeroed before the PV product for the same reason.
#include "attention.hpp"
#include "common.hpp"

#include <type_traits>

namespace molink {

namespace {

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ e16x8 zero_tail(e16x8 v, int nvalid) {
  // keep elements [0, nvalid), zero the rest (bitwise, so NaNs vanish)
  u32x4 w = __builtin_bit_cast(u32x4, v);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t lo = (2 * i < nvalid) ? 0x0000ffffu : 0u;
    const uint32_t hi = (2 * i + 1 < nvalid) ? 0xffff0000u : 0u;
    w[i] &= (lo | hi);
  }
  return __builtin_bit_cast(e16x8, w);
}

__device__ __forceinline__ e16x8 pack8(const float* p) {
  e16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = f32_to_e16(p[e]);
  return o;
}

// ------------------------------------------------------------------------------------------------
// Decode: one wave per (key range of a decode token, KV head); all query heads of the group ride in
// the 16 MFMA columns, so the cache is read once per KV head.  16x16x32 MFMA; a step is 32 keys
// (two blocks).  Row m of key tile A is (block m/8, slot 8*((m/4)%2) + m%4), tile B is 4 slots
// further, so lane group g = lane/16 ends up with keys 8g .. 8g+7 of the step in registers
// [A0..A3, B0..B3].  K of the next step is prefetched while the current step is processed.
// ------------------------------------------------------------------------------------------------
template <int D>
struct DecodeStepLoads {
  e16x8 ka[D / 32], kb[D / 32];   // key tiles A and B, D/32 MFMA k-steps each
  e16x8 v[D / 16];                // V^T tiles, one per 16 output dims
};

// ALIBI: attention with linear biases - the score of key j is lowered by slope[head] * (last_key - j), the distance
// of the key from the token's own logical index.
template <int D, bool QLO, bool ALIBI = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void attn_decode_kernel(AttnArgs a, const DecodeItem* __restrict__ items,
                                                          int num_items, float* __restrict__ part_o,
                                                          float2* __restrict__ part_ml) {
  constexpr int KS = D / 32;   // MFMA k-steps of the QK product
  constexpr int DT = D / 16;   // 16-row tiles of O^T
  const int lane = threadIdx.x & 63;
  // the four waves of a workgroup take four neighbouring KV heads of the same key range: their
  // blocks are adjacent in the pool, so the workgroup reads 16 KB runs
  // workgroup order: the head groups of one key range follow each other eight apart, i.e. on the same XCD (workgroups
  // go to the eight XCDs in turn) and close in time, so that they find each other's lines and translations
  const int hgroups = (a.nkv + 3) / 4;
  const int item_id = (int)(blockIdx.x / (8 * hgroups)) * 8 + (int)(blockIdx.x % 8);
  const int hg = (int)(blockIdx.x % (8 * hgroups)) / 8;
  if (item_id >= num_items) return;
  const int r = __builtin_amdgcn_readfirstlane(hg * 4 + (threadIdx.x >> 6));   // KV head
  if (r >= a.nkv) return;
  const int g = a.nq / a.nkv;
  const int row = __builtin_amdgcn_readfirstlane(items[item_id].row);
  const int bt_off = __builtin_amdgcn_readfirstlane(items[item_id].bt_off);
  const int key_begin = __builtin_amdgcn_readfirstlane(items[item_id].key_begin);
  const int key_end = __builtin_amdgcn_readfirstlane(items[item_id].key_end);
  const int part = __builtin_amdgcn_readfirstlane(items[item_id].part);
  // block ids are read through the constant address space (nothing writes the table during the kernel):
  // scalar loads, which do not queue behind the K/V loads in flight
  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  const const_i32_ptr bt = (const_i32_ptr)(a.bt_flat + bt_off);
  const int last_block = (key_end - 1) / kKvBlock;
  const int nsteps = (key_end - key_begin + 31) / 32;

  const int col = lane & 15, grp = lane >> 4;
  const int ldq = (a.nq + 2 * a.nkv) * D;
  // linear biases: this column's slope in the exponent's unit (log2), and the token's own index
  float slope_l2 = 0.f;
  int last_key = 0;
  if constexpr (ALIBI) {
    slope_l2 = a.alibi[r * g + (col < g ? col : 0)] * 1.4426950408889634f;
    last_key = __builtin_amdgcn_readfirstlane(items[item_id].last_key);
  }

  // Q^T operand: column = query head of the group, lane group holds d = 32*kk + 8*grp .. +7
  e16x8 qf[KS], qf_lo[QLO ? KS : 1];
  {
    const int head = r * g + (col < g ? col : 0);
    const e16* qp = a.qkv + (size_t)row * ldq + head * D + grp * 8;
    const e16* ql = QLO ? a.q_lo + ((size_t)row * a.nq + head) * D + grp * 8 : qp;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      e16x8 v = load8(qp + kk * 32);
      if (col >= g) v = e16x8{0, 0, 0, 0, 0, 0, 0, 0};
      qf[kk] = v;
      if constexpr (QLO) {
        e16x8 w = load8(ql + kk * 32);
        if (col >= g) w = e16x8{0, 0, 0, 0, 0, 0, 0, 0};
        qf_lo[kk] = w;
      }
    }
  }

  // per-lane constants of the K and V^T operand loads
  const int k_bsel = (lane & 15) >> 3;                                  // which block of the pair this lane's K row is in
  const int v_bsel = grp >> 1;
  // tile A takes positions 0..7 of the block this lane's key row is in (slots 0-3 and 8-11), tile B the
  // next eight: per instruction two runs of 512 bytes
  const size_t k_lane_off = (size_t)(lane & 7) * 32 + grp * 8;
  const size_t v_lane_off = (size_t)(lane & 15) * kKvBlock + 8 * (grp & 1);
  const size_t blk_stride = (size_t)a.nkv * kKvBlock * D;               // elements per block (all heads)
  const size_t head_off = (size_t)r * kKvBlock * D;

  auto block_id = [&](int step, int sel) -> int {
    int lb = key_begin / kKvBlock + 2 * step + sel;
    lb = lb < last_block ? lb : last_block;
    return bt[lb];
  };
  // all loads of one step: addresses are always in bounds (block indices are clamped), so a step can
  // be fetched without asking whether it exists and the loop body stays free of branches
  auto load_step = [&](DecodeStepLoads<D>& L, int b0, int b1) {
    const int pbk = k_bsel ? b1 : b0;
    const e16* kp = a.k_pool + (size_t)pbk * blk_stride + head_off + k_lane_off;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      L.ka[kk] = load8_stream(kp + kk * (kKvBlock * 32));
      L.kb[kk] = load8_stream(kp + 8 * 32 + kk * (kKvBlock * 32));
    }
    const int pbv = v_bsel ? b1 : b0;
    const e16* vp = a.v_pool + (size_t)pbv * blk_stride + head_off + v_lane_off;
#pragma unroll
    for (int t = 0; t < DT; ++t) L.v[t] = load8_stream(vp + (size_t)t * 16 * kKvBlock);
  };

  f32x4 acc[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;

  auto process = [&](const DecodeStepLoads<D>& L, int step) {
    f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      sa = mfma_16x16x32(L.ka[kk], qf[kk], sa);
      sb = mfma_16x16x32(L.kb[kk], qf[kk], sb);
      if constexpr (QLO) {   // second query plane into the same scores
        sa = mfma_16x16x32(L.ka[kk], qf_lo[kk], sa);
        sb = mfma_16x16x32(L.kb[kk], qf_lo[kk], sb);
      }
    }
    const int key0 = key_begin + 32 * step + 8 * grp;     // first of this lane's 8 keys
    const int nvalid = key_end - key0;                    // keys [0, nvalid) of the 8 are real
    float s[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float va = sa[e] * a.scale_log2e, vb = sb[e] * a.scale_log2e;
      if constexpr (ALIBI) {
        va -= slope_l2 * (float)(last_key - (key0 + e));
        vb -= slope_l2 * (float)(last_key - (key0 + 4 + e));
      }
      s[e] = (e < nvalid) ? va : -INFINITY;
      s[4 + e] = (4 + e < nvalid) ? vb : -INFINITY;
    }
    float m_tile = s[0];
#pragma unroll
    for (int e = 1; e < 8; ++e) m_tile = fmaxf(m_tile, s[e]);
    m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 16, 64));
    m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32, 64));
    const float m_new = fmaxf(m_run, m_tile);              // finite: every range has at least one real key
    const float alpha = fast_exp2(m_run - m_new);
    float p[8], psum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      p[e] = fast_exp2(s[e] - m_new);
      psum += p[e];
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    const e16x8 pf = pack8(p);
    const bool tail = key_begin + 32 * step + 32 > key_end;   // wave-uniform
#pragma unroll
    for (int t = 0; t < DT; ++t) {
      e16x8 v = L.v[t];
      if (tail) v = zero_tail(v, nvalid < 0 ? 0 : nvalid);
      acc[t] = acc[t] * alpha;
      acc[t] = mfma_16x16x32(v, pf, acc[t]);
    }
  };

  // Software pipeline: while step s is processed, all loads of step s+1 are in flight and the block
  // ids of step s+2 are being fetched.  The loop body has no branches, so the waits count exactly the
  // loads that must have landed.
  DecodeStepLoads<D> buf0, buf1;
  int c0 = block_id(1, 0), c1 = block_id(1, 1);          // ids of the step after the one in flight
  load_step(buf0, block_id(0, 0), block_id(0, 1));
  int step = 0;
  for (; step + 2 < nsteps; step += 2) {
    load_step(buf1, c0, c1);                              // step + 1
    c0 = block_id(step + 2, 0); c1 = block_id(step + 2, 1);
    process(buf0, step);
    load_step(buf0, c0, c1);                              // step + 2
    c0 = block_id(step + 3, 0); c1 = block_id(step + 3, 1);
    process(buf1, step + 1);
  }
  if (step + 1 < nsteps) {
    load_step(buf1, c0, c1);
    process(buf0, step);
    process(buf1, step + 1);
  } else {
    process(buf0, step);
  }

  // l_run holds this lane group's share of the row sum; combine the four groups
  float l_tot = l_run + __shfl_xor(l_run, 16, 64);
  l_tot += __shfl_xor(l_tot, 32, 64);
  if (col < g) {
    const size_t slot = ((size_t)part * a.nkv + r) * g + col;
    float* po = part_o + slot * D + 4 * grp;
#pragma unroll
    for (int t = 0; t < DT; ++t) *reinterpret_cast<f32x4*>(po + t * 16) = acc[t];
    if (grp == 0) part_ml[slot] = make_float2(m_run, l_tot);
  }
}

// Combine the key ranges of every decode token: out = sum_i 2^(m_i - M) O_i / sum_i 2^(m_i - M) l_i.
// One thread per (token, head, 4 consecutive dims).
template <int D>
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a, const DecodeToken* __restrict__ tokens,
                                                         int num_tokens, const float* __restrict__ part_o,
                                                         const float2* __restrict__ part_ml) {
  const int per_token = a.nq * (D / 4);
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= num_tokens * per_token) return;
  const int tok = idx / per_token, rem = idx % per_token;
  const int head = rem / (D / 4), d4 = rem % (D / 4);
  const int g = a.nq / a.nkv;
  const int r = head / g, col = head % g;
  const DecodeToken t = tokens[tok];
  // four ranges per trip in both passes: their loads are issued together, the sums stay in range order
  const size_t slot_step = (size_t)a.nkv * g;
  const size_t slot0 = ((size_t)t.first_item * a.nkv + r) * g + col;
  float m_max = -INFINITY;
  int i = 0;
  for (; i + 4 <= t.num_items; i += 4) {
    float mx[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) mx[u] = part_ml[slot0 + (size_t)(i + u) * slot_step].x;
    m_max = fmaxf(fmaxf(m_max, fmaxf(mx[0], mx[1])), fmaxf(mx[2], mx[3]));
  }
  for (; i < t.num_items; ++i) m_max = fmaxf(m_max, part_ml[slot0 + (size_t)i * slot_step].x);
  float l = 0.f;
  f32x4 o = {0.f, 0.f, 0.f, 0.f};
  i = 0;
  for (; i + 4 <= t.num_items; i += 4) {
    float2 ml[4];
    f32x4 po[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t slot = slot0 + (size_t)(i + u) * slot_step;
      ml[u] = part_ml[slot];
      po[u] = *reinterpret_cast<const f32x4*>(part_o + slot * D + d4 * 4);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float w = fast_exp2(ml[u].x - m_max);
      l += w * ml[u].y;
      o += po[u] * w;
    }
  }
  for (; i < t.num_items; ++i) {
    const size_t slot = slot0 + (size_t)i * slot_step;
    const float2 ml = part_ml[slot];
    const float w = fast_exp2(ml.x - m_max);
    l += w * ml.y;
    const f32x4 po = *reinterpret_cast<const f32x4*>(part_o + slot * D + d4 * 4);
    o += po * w;
  }
  const float inv = 1.0f / l;
  e16x4 ob, ol;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float val = o[e] * inv;
    ob[e] = f32_to_act(val, a.out_half);
    ol[e] = f32_to_e16(val - e16_to_f32(ob[e]));
  }
  const size_t at = (size_t)t.row * a.nq * D + head * D + d4 * 4;
  *reinterpret_cast<e16x4*>(a.out + at) = ob;
  if (a.out_lo) *reinterpret_cast<e16x4*>(a.out_lo + at) = ol;
}

// ------------------------------------------------------------------------------------------------
// Prefill: a workgroup of four waves takes 128 consecutive query columns of one (sequence, KV head);
// a column is a (token, head in group) pair, column = token * g + head_in_group, so grouped heads
// share every K/V read; wave w owns columns 32w .. 32w+31.  The four waves need the same keys, so a
// step's K and V tiles (32 keys = two blocks) are fetched once per workgroup, straight into LDS
// (global_load_lds), four stages deep.  32x32x16 MFMA.  Row m of the key tile is (block m/16, slot
// 8*((m/4)%2) + 4*((m/8)%2) + m%4): accumulator registers 0..7 of lane group G = lane/32 are then
// slots 8G..8G+7 of the first block, registers 8..15 the same slots of the second block, i.e. the
// S^T accumulators are the P^T operand of the PV product as they stand.
//
// Software pipeline inside a wave.  A step's work is a chain - scores (MFMA), their maximum, the
// exponentials and their rounding (vector unit), the PV product (MFMA) - and a wave that walks the chain
// in order leaves the matrix pipe idle during the vector work and the vector unit idle during the
// products.  Here the scores of step u+1 are multiplied while the exponentials of step u are taken
// (one basic block: the compiler interleaves the two), and the maximum of step u+1 is found while the PV
// product of step u runs (a second block).  What is rare - moving the reference of the exponentials -
// sits in a branch between iterations; what is occasional - the causal mask, slots past the sequence's
// end - in a second copy of the second block, chosen per step (wave-uniform).
//
// LDS stage: the K tile as it lies in the pool, [block][d/32][16 positions][64 bytes] (MFMA row m of the
// tile is position m % 16 of block m / 16; every load instruction copies one 1 KB run), with the four
// 16-byte chunks of a 64-byte piece exchanged by (position / 2) % 4 so that the 128-bit fragment reads
// of 8 consecutive rows hit 8 different bank groups; then the V^T tiles as [block][slot half][d][16
// bytes], so that the lanes of a fragment read (32 consecutive d, one half) are contiguous.  Both
// arrangements are made by choosing which 16 bytes each lane of a load instruction fetches.
// ------------------------------------------------------------------------------------------------

// the maximum of lane l and lane l ^ 32, on every lane, without a trip through LDS
__device__ __forceinline__ float max_across_halves(float v) {
  const uint32_t u = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

template <int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void attn_prefill_kernel(AttnArgs a, const PrefillTile* __restrict__ tiles,
                                                           int num_tiles) {
  constexpr int KS = D / 16;                 // MFMA k-steps of the QK product
  constexpr int DT = D / 32;                 // 32-row tiles of O^T
  constexpr int NST = 4;                     // LDS stages
  constexpr int K_BYTES = 32 * D * 2;        // K tile
  constexpr int STAGE_BYTES = 2 * K_BYTES;   // + V^T tiles of the same size
  constexpr int NI = STAGE_BYTES / 1024 / 4; // load instructions per wave per stage
  constexpr int NP = D / 32;                 // 32-element pieces per K row
  using Lds = LdsStages<STAGE_BYTES>;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // Work order.  The tile list is sorted by keys seen, longest first, and every tile exists once per KV head.  Two
  // workgroups fit on a CU; when the launch is between one and two workgroups per CU, all of them are resident at
  // once and a CU's time is the sum of its two.  The first 256 workgroups (one per CU) take the longest tiles in
  // order, the rest take the remaining ones shortest first, so that the longest tile shares its CU with the
  // shortest, the second longest with the second shortest, and so on.  Larger launches keep longest-first.
  const int total = num_tiles * a.nkv;
  constexpr int kFirstPass = 256;
  int pos = blockIdx.x;
  if (total > kFirstPass && total <= 2 * kFirstPass && pos >= kFirstPass) pos = total - 1 - (pos - kFirstPass);
  const int tile_id = pos / a.nkv;
  const int r = pos % a.nkv;
  const int g = a.nq / a.nkv;
  const int row0 = __builtin_amdgcn_readfirstlane(tiles[tile_id].row0);
  const int q_len = __builtin_amdgcn_readfirstlane(tiles[tile_id].q_len);
  const int ctx = __builtin_amdgcn_readfirstlane(tiles[tile_id].ctx);
  const int bt_off = __builtin_amdgcn_readfirstlane(tiles[tile_id].bt_off);
  const int tile_col0 = __builtin_amdgcn_readfirstlane(tiles[tile_id].col0);
  // The block table is read through the constant address space (nothing writes it during the kernel): the
  // reads become scalar loads, which do not queue behind the tile loads in flight.
  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  const const_i32_ptr bt = (const_i32_ptr)(a.bt_flat + bt_off);
  const int total_keys = ctx + q_len;
  const int last_block = (total_keys - 1) / kKvBlock;
  const int ncols = q_len * g;

  const int col = lane & 31, grp = lane >> 5;
  const int col0 = tile_col0 + 32 * wave;                      // this wave's first column
  const bool wave_active = col0 < ncols;
  const int my_col = min(col0 + col, ncols - 1);               // padding columns repeat the last real one
  const int tok = my_col / g, hg = my_col % g;
  const int limit = ctx + tok;                                  // last key this column may see
  // steps with a key visible to this wave (0 for a wave of padding columns only)
  const int wave_steps = wave_active ? (ctx + min(col0 + 31, ncols - 1) / g) / 32 + 1 : 0;
  const int wave_min_limit = ctx + min(col0, ncols - 1) / g;               // smallest limit among this wave's columns
  const int nsteps = (ctx + min(tile_col0 + 127, ncols - 1) / g) / 32 + 1; // ... to the workgroup
  const int ldq = (a.nq + 2 * a.nkv) * D;

  e16x8 qf[KS];
  {
    const e16* qp = a.qkv + (size_t)(row0 + tok) * ldq + (r * g + hg) * D + grp * 8;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qf[kk] = load8(qp + kk * 16);
  }

  // ---- what this lane fetches for load instruction i of its wave (instruction id j = 4 i + wave;
  // the first K_BYTES / 1024 instructions fill the K tile, the rest the V^T tiles)
  const size_t blk_stride = (size_t)a.nkv * kKvBlock * D;     // elements per block (all heads)
  const size_t head_off = (size_t)r * kKvBlock * D;
  // An instruction never straddles two blocks (4 or 8 K rows, 64 of the 2 D positions of a V block), so
  // the block is chosen per instruction (scalar) and only the offset inside the block is per lane.
  uint32_t ld_off[NI];     // byte offset of this lane's 16 bytes inside the (block, head) region
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int j = 4 * i + wave;
    if (j < K_BYTES / 1024) {
      // instruction j copies piece j % NP of block j / NP: 16 positions x 64 bytes, one run in the pool
      const int piece = j % NP, pos16 = lane >> 2, c = lane & 3;
      ld_off[i] = (uint32_t)((piece * kKvBlock + pos16) * 32 + ((c ^ ((pos16 >> 1) & 3)) * 8)) * 2u;
    } else {
      const int pos16 = (j - K_BYTES / 1024) * 64 + lane;   // 16-byte position in the V part: [block][half][d]
      const int d = pos16 % D, half = (pos16 / D) & 1;
      ld_off[i] = (uint32_t)(d * kKvBlock + half * 8) * 2u;
    }
  }
  // Every step issues the same loads (block indices past the sequence are clamped to its last block),
  // so the wait counts below hold without control flow around the loads.
  auto fetch = [&](auto stage_c, int step) {
    constexpr int S = decltype(stage_c)::value;
    int lb0 = 2 * step, lb1 = 2 * step + 1;
    lb0 = lb0 < last_block ? lb0 : last_block;
    lb1 = lb1 < last_block ? lb1 : last_block;
    const int b0 = bt[lb0], b1 = bt[lb1];
    char* stage = Lds::template get<S>();
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int j = 4 * i + wave;                                    // uniform
      const bool is_k = j < K_BYTES / 1024;
      const int second = is_k ? j / NP : ((j - K_BYTES / 1024) * 64) / (2 * D);
      const int pb = second ? b1 : b0;
      const char* base = reinterpret_cast<const char*>((is_k ? a.k_pool : a.v_pool) + (size_t)pb * blk_stride + head_off);
      __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(base + ld_off[i]),
                                       reinterpret_cast<uint32_t*>(stage + j * 1024), 16, 0, 0);
    }
  };

  f32x16 acc[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
  // m_run: reference of the exponentials (see maximum()); l_run: this lane's share of the row sum
  float m_run = -INFINITY, l_run = 0.f;

  // fragment addresses: K row m = lane % 32 is position m % 16 of block m / 16; MFMA step kk wants chunk
  // 2 (kk % 2) + grp of piece kk / 2;  V^T row d = 32 t + lane % 32 of half grp of block b
  const int k_pos = col & 15;
  const int k_row_off = ((col >> 4) * NP * kKvBlock + k_pos) * 64;
  const int k_swz = (k_pos >> 1) & 3;
  const int v_frag_off = K_BYTES + (grp * D + col) * 16;
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // scores of the step whose tiles are in stage S: register e of this lane is key 32*step + 16*(e/8) + 8*grp + e%8
  auto scores = [&](auto stage_c, f32x16& s) {
    constexpr int S = decltype(stage_c)::value;
    const char* stage = Lds::template get<S>();
    s = zero16;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      const e16x8 kf = *reinterpret_cast<const e16x8*>(stage + k_row_off + (kk >> 1) * (kKvBlock * 64) +
                                                         (((2 * (kk & 1) + grp) ^ k_swz) * 16));
      s = mfma_32x32x16(kf, qf[kk], s);
    }
  };
  // Hides the keys a column may not see (MASK) and finds the columns' new maxima; returns whether the reference of
  // the exponentials has to move.  The reference need not be the exact running maximum: softmax does not depend on
  // it, it only has to keep exp2(score - m_run) in range.  It is moved (and the accumulators rescaled, 16 DT
  // multiplications per lane) only when some column's maximum has grown by more than 2^8 since; until then
  // probabilities up to 256 are accumulated as they are.
  auto maximum = [&](auto mask_c, f32x16& s, int step, float& m_new) {
    constexpr bool MASK = decltype(mask_c)::value;
    float raw_max = -INFINITY;                               // maximum of the unscaled scores (the scale is positive)
    if constexpr (MASK) {
      const int key_base = 32 * step + 8 * grp;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int key = key_base + 16 * (e / 8) + (e % 8);
        s[e] = (key <= limit) ? s[e] : -INFINITY;
      }
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) raw_max = fmaxf(raw_max, s[e]);
    raw_max = max_across_halves(raw_max);
    m_new = fmaxf(m_run, raw_max * a.scale_log2e);           // finite from step 0 on: key 0 is visible to all
    return __builtin_amdgcn_ballot_w64(m_new > m_run + 8.0f) != 0;
  };
  auto move_reference = [&](float m_new) {
    const float alpha = fast_exp2(m_run - m_new);
    l_run *= alpha;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][e] *= alpha;
    m_run = m_new;
  };
  // probabilities of a step from its (masked) scores, rounded into the two P^T operands
  auto probabilities = [&](const f32x16& s, e16x8& p0, e16x8& p1) {
    float sv[16], psum = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      sv[e] = fast_exp2(__builtin_fmaf(s[e], a.scale_log2e, -m_run));    // (-inf) * scale - m = -inf -> 0
      psum += sv[e];
    }
    l_run += psum;
    p0 = pack8(sv);
    p1 = pack8(sv + 8);
  };
  auto pv = [&](auto stage_c, auto tail_c, const e16x8& p0, const e16x8& p1, int step) {
    constexpr int S = decltype(stage_c)::value;
    constexpr bool TAIL = decltype(tail_c)::value;
    const char* stage = Lds::template get<S>();
    const int nv0 = total_keys - (32 * step + 8 * grp), nv1 = nv0 - 16;    // slots past the sequence end hold anything
#pragma unroll
    for (int t = 0; t < DT; ++t) {
      e16x8 v0 = *reinterpret_cast<const e16x8*>(stage + v_frag_off + t * 512);
      e16x8 v1 = *reinterpret_cast<const e16x8*>(stage + v_frag_off + 2 * D * 16 + t * 512);
      if constexpr (TAIL) {
        v0 = zero_tail(v0, nv0 < 0 ? 0 : (nv0 > 8 ? 8 : nv0));
        v1 = zero_tail(v1, nv1 < 0 ? 0 : (nv1 > 8 ? 8 : nv1));
      }
      acc[t] = mfma_32x32x16(v0, p0, acc[t]);
      acc[t] = mfma_32x32x16(v1, p1, acc[t]);
    }
  };

  f32x16 sc[2];          // scores of the step being turned into probabilities and of the one after it
  float m_next = -INFINITY;
  bool move_next = false;
  // does step `step` need the causal mask or hold slots past the sequence's end (wave-uniform)?
  auto special = [&](int step) { return 32 * step + 31 > wave_min_limit; };

  // Iteration u: the tiles of steps u and u + 1 are in their stages, the masked scores of step u are in sc[u & 1]
  // and their maximum has been taken.  After the wait only the loads of step u + 2 can still be in flight, so this
  // wave's part of stage (u + 1) % 4 has landed; after the barrier everybody's has, and everybody is done with
  // stage (u - 1) % 4, which is refilled with step u + 3.
  auto iteration = [&](auto stage_c, auto par_c, int u) {
    constexpr int S = decltype(stage_c)::value;
    constexpr int P = decltype(par_c)::value;
    using Next = std::integral_constant<int, (S + 1) % NST>;
    wait_vmcnt<NI>();
    pipeline_barrier();
    fetch(std::integral_constant<int, (S + NST - 1) % NST>{}, u + NST - 1);
    if (u >= wave_steps) return;                              // nothing visible to this wave's columns any more
    if (move_next) move_reference(m_next);
    e16x8 p0, p1;
    // scores of step u + 1 under the exponentials of step u
    scores(Next{}, sc[P ^ 1]);
    probabilities(sc[P], p0, p1);
    __builtin_amdgcn_sched_barrier(0);
    // the PV product of step u over the maximum of step u + 1
    if (special(u + 1) || special(u)) {
      pv(stage_c, std::true_type{}, p0, p1, u);
      move_next = maximum(std::true_type{}, sc[P ^ 1], u + 1, m_next);
    } else {
      pv(stage_c, std::false_type{}, p0, p1, u);
      move_next = maximum(std::false_type{}, sc[P ^ 1], u + 1, m_next);
    }
  };

  fetch(std::integral_constant<int, 0>{}, 0);
  fetch(std::integral_constant<int, 1>{}, 1);
  fetch(std::integral_constant<int, 2>{}, 2);
  // step 0: its scores and their maximum before the pipeline starts
  wait_vmcnt<2 * NI>();
  pipeline_barrier();
  if (wave_steps > 0) {
    scores(std::integral_constant<int, 0>{}, sc[0]);
    move_next = maximum(std::true_type{}, sc[0], 0, m_next);
  }
  for (int u = 0; u < nsteps; u += NST) {
    iteration(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, u);
    iteration(std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{}, u + 1);
    iteration(std::integral_constant<int, 2>{}, std::integral_constant<int, 0>{}, u + 2);
    iteration(std::integral_constant<int, 3>{}, std::integral_constant<int, 1>{}, u + 3);
  }
  wait_vmcnt<0>();   // nothing may still be writing LDS when the workgroup ends

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (col0 + col < ncols) {
    const float inv = 1.0f / l_tot;
    const size_t at = (size_t)(row0 + tok) * a.nq * D + (r * g + hg) * D + 4 * grp;
#pragma unroll
    for (int t = 0; t < DT; ++t) {
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        e16x4 ob, ol;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float val = acc[t][q4 * 4 + e] * inv;
          ob[e] = f32_to_act(val, a.out_half);
          ol[e] = f32_to_e16(val - e16_to_f32(ob[e]));
        }
        *reinterpret_cast<e16x4*>(a.out + at + t * 32 + q4 * 8) = ob;
        if (a.out_lo) *reinterpret_cast<e16x4*>(a.out_lo + at + t * 32 + q4 * 8) = ol;
      }
    }
  }
}

// The same tiles for queries carried as two planes (q = hi + lo, every score takes both products): the steps of a
// tile are walked one after the other, each step's scores, softmax and PV product in order.  With twice the score
// MFMAs and the second plane's fragments in registers, the software-pipelined kernel above runs out of registers at
// two waves per SIMD and was measured slower on these launches (116 against 80 us on the 2048-token chunk of the
// Qwen2-shaped stage); overlap here comes from the second workgroup on the CU.
// QLO = false: one query plane; ALIBI: attention with linear biases (the score of key j for the query at logical
// index i is lowered by slope[head] * (i - j)) - every prefill launch with linear biases runs here.
template <int D, bool QLO = true, bool ALIBI = false>
__global__ __launch_bounds__(256) void attn_prefill_two_plane_kernel(AttnArgs a, const PrefillTile* __restrict__ tiles,
                                                           int num_tiles) {
  constexpr int KS = D / 16;                 // MFMA k-steps of the QK product
  constexpr int DT = D / 32;                 // 32-row tiles of O^T
  constexpr int NST = 4;                     // LDS stages
  constexpr int K_BYTES = 32 * D * 2;        // K tile
  constexpr int STAGE_BYTES = 2 * K_BYTES;   // + V^T tiles of the same size
  constexpr int NI = STAGE_BYTES / 1024 / 4; // load instructions per wave per stage
  constexpr int NP = D / 32;                 // 32-element pieces per K row
  using Lds = LdsStages<STAGE_BYTES>;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // Work order.  The tile list is sorted by keys seen, longest first, and every tile exists once per KV head.  Two
  // workgroups fit on a CU; when the launch is between one and two workgroups per CU, all of them are resident at
  // once and a CU's time is the sum of its two.  The first 256 workgroups (one per CU) take the longest tiles in
  // order, the rest take the remaining ones shortest first, so that the longest tile shares its CU with the
  // shortest, the second longest with the second shortest, and so on.  Larger launches keep longest-first.
  const int total = num_tiles * a.nkv;
  constexpr int kFirstPass = 256;
  int pos = blockIdx.x;
  if (total > kFirstPass && total <= 2 * kFirstPass && pos >= kFirstPass) pos = total - 1 - (pos - kFirstPass);
  const int tile_id = pos / a.nkv;
  const int r = pos % a.nkv;
  const int g = a.nq / a.nkv;
  const int row0 = __builtin_amdgcn_readfirstlane(tiles[tile_id].row0);
  const int q_len = __builtin_amdgcn_readfirstlane(tiles[tile_id].q_len);
  const int ctx = __builtin_amdgcn_readfirstlane(tiles[tile_id].ctx);
  const int bt_off = __builtin_amdgcn_readfirstlane(tiles[tile_id].bt_off);
  const int tile_col0 = __builtin_amdgcn_readfirstlane(tiles[tile_id].col0);
  // The block table is read through the constant address space (nothing writes it during the kernel): the
  // reads become scalar loads, which do not queue behind the tile loads in flight.
  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  const const_i32_ptr bt = (const_i32_ptr)(a.bt_flat + bt_off);
  const int total_keys = ctx + q_len;
  const int last_block = (total_keys - 1) / kKvBlock;
  const int ncols = q_len * g;

  const int col = lane & 31, grp = lane >> 5;
  const int col0 = tile_col0 + 32 * wave;                      // this wave's first column
  const bool wave_active = col0 < ncols;
  const int my_col = min(col0 + col, ncols - 1);               // padding columns repeat the last real one
  const int tok = my_col / g, hg = my_col % g;
  const int limit = ctx + tok;                                  // last key this column may see
  const int wave_steps = (ctx + min(col0 + 31, ncols - 1) / g) / 32 + 1;   // steps with a key visible to this wave
  const int wave_min_limit = ctx + min(col0, ncols - 1) / g;               // smallest limit among this wave's columns
  const int nsteps = (ctx + min(tile_col0 + 127, ncols - 1) / g) / 32 + 1; // ... to the workgroup
  const int ldq = (a.nq + 2 * a.nkv) * D;

  e16x8 qf[KS], qf_lo[QLO ? KS : 1];
  {
    const e16* qp = a.qkv + (size_t)(row0 + tok) * ldq + (r * g + hg) * D + grp * 8;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qf[kk] = load8(qp + kk * 16);
    if constexpr (QLO) {
      const e16* ql = a.q_lo + ((size_t)(row0 + tok) * a.nq + r * g + hg) * D + grp * 8;
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) qf_lo[kk] = load8(ql + kk * 16);
    }
  }
  // linear biases, in the unit of the unscaled scores: score * scale_log2e is the exponent, so a bias of
  // slope * log2(e) per key of distance there is slope * log2(e) / scale_log2e here
  float slope_raw = 0.f;
  if constexpr (ALIBI) slope_raw = a.alibi[r * g + hg] * 1.4426950408889634f / a.scale_log2e;

  // ---- what this lane fetches for load instruction i of its wave (instruction id j = 4 i + wave;
  // the first K_BYTES / 1024 instructions fill the K tile, the rest the V^T tiles)
  const size_t blk_stride = (size_t)a.nkv * kKvBlock * D;     // elements per block (all heads)
  const size_t head_off = (size_t)r * kKvBlock * D;
  // An instruction never straddles two blocks (4 or 8 K rows, 64 of the 2 D positions of a V block), so
  // the block is chosen per instruction (scalar) and only the offset inside the block is per lane.
  uint32_t ld_off[NI];     // byte offset of this lane's 16 bytes inside the (block, head) region
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int j = 4 * i + wave;
    if (j < K_BYTES / 1024) {
      // instruction j copies piece j % NP of block j / NP: 16 positions x 64 bytes, one run in the pool
      const int piece = j % NP, pos = lane >> 2, c = lane & 3;
      ld_off[i] = (uint32_t)((piece * kKvBlock + pos) * 32 + ((c ^ ((pos >> 1) & 3)) * 8)) * 2u;
    } else {
      const int pos = (j - K_BYTES / 1024) * 64 + lane;   // 16-byte position in the V part: [block][half][d]
      const int d = pos % D, half = (pos / D) & 1;
      ld_off[i] = (uint32_t)(d * kKvBlock + half * 8) * 2u;
    }
  }
  // Every step issues the same loads (block indices past the sequence are clamped to its last block),
  // so the wait counts below hold without control flow around the loads.
  auto fetch = [&](auto stage_c, int step) {
    constexpr int S = decltype(stage_c)::value;
    int lb0 = 2 * step, lb1 = 2 * step + 1;
    lb0 = lb0 < last_block ? lb0 : last_block;
    lb1 = lb1 < last_block ? lb1 : last_block;
    const int b0 = bt[lb0], b1 = bt[lb1];
    char* stage = Lds::template get<S>();
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int j = 4 * i + wave;                                    // uniform
      const bool is_k = j < K_BYTES / 1024;
      const int second = is_k ? j / NP : ((j - K_BYTES / 1024) * 64) / (2 * D);
      const int pb = second ? b1 : b0;
      const char* base = reinterpret_cast<const char*>((is_k ? a.k_pool : a.v_pool) + (size_t)pb * blk_stride + head_off);
      __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(base + ld_off[i]),
                                       reinterpret_cast<uint32_t*>(stage + j * 1024), 16, 0, 0);
    }
  };

  f32x16 acc[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // fragment addresses: K row m = lane % 32 is position m % 16 of block m / 16; MFMA step kk wants chunk
  // 2 (kk % 2) + grp of piece kk / 2;  V^T row d = 32 t + lane % 32 of half grp of block b
  const int k_pos = col & 15;
  const int k_row_off = ((col >> 4) * NP * kKvBlock + k_pos) * 64;
  const int k_swz = (k_pos >> 1) & 3;
  const int v_frag_off = K_BYTES + (grp * D + col) * 16;

  auto process = [&](auto stage_c, int step) {
    constexpr int S = decltype(stage_c)::value;
    if (!wave_active || step >= wave_steps) return;          // nothing visible to this wave's columns
    const char* stage = Lds::template get<S>();
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 s = zero16;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      const e16x8 kf = *reinterpret_cast<const e16x8*>(stage + k_row_off + (kk >> 1) * (kKvBlock * 64) +
                                                         (((2 * (kk & 1) + grp) ^ k_swz) * 16));
      s = mfma_32x32x16(kf, qf[kk], s);
      if constexpr (QLO) s = mfma_32x32x16(kf, qf_lo[kk], s);     // second query plane into the same scores
    }
    // register e of this lane is key 32*step + 16*(e/8) + 8*grp + e%8
    const int key_base = 32 * step + 8 * grp;
    if constexpr (ALIBI) {
#pragma unroll
      for (int e = 0; e < 16; ++e) s[e] -= slope_raw * (float)(limit - (key_base + 16 * (e / 8) + (e % 8)));
    }
    float sv[16];
    float raw_max = -INFINITY;                               // maximum of the unscaled scores (the scale is positive)
    if (32 * step + 31 <= wave_min_limit) {                  // wave-uniform: every key of the step is visible to every column
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        sv[e] = s[e];
        raw_max = fmaxf(raw_max, sv[e]);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int key = key_base + 16 * (e / 8) + (e % 8);
        sv[e] = (key <= limit) ? s[e] : -INFINITY;
        raw_max = fmaxf(raw_max, sv[e]);
      }
    }
    raw_max = max_across_halves(raw_max);
    const float m_new = fmaxf(m_run, raw_max * a.scale_log2e);   // finite from step 0 on: key 0 is visible to all
    // The reference m_run of the exponentials need not be the exact running maximum: softmax does not
    // depend on it, it only has to keep exp2(score - m_run) in range.  It is moved (and the accumulators
    // rescaled, 16 DT multiplications per lane) only when some column's maximum has grown by more than
    // 2^8 since; until then probabilities up to 256 are accumulated as they are.
    const bool rescale = __builtin_amdgcn_ballot_w64(m_new > m_run + 8.0f) != 0;
    if (rescale) {
      const float alpha = fast_exp2(m_run - m_new);
      l_run *= alpha;
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] *= alpha;
      m_run = m_new;
    }
    float psum = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      sv[e] = fast_exp2(__builtin_fmaf(sv[e], a.scale_log2e, -m_run));    // (-inf) * scale - m = -inf -> 0
      psum += sv[e];
    }
    l_run += psum;
    const e16x8 p0 = pack8(sv), p1 = pack8(sv + 8);
    const bool tail = 32 * step + 32 > total_keys;            // wave-uniform: slots past the sequence end
    const int nv0 = total_keys - key_base, nv1 = nv0 - 16;
#pragma unroll
    for (int t = 0; t < DT; ++t) {
      e16x8 v0 = *reinterpret_cast<const e16x8*>(stage + v_frag_off + t * 512);
      e16x8 v1 = *reinterpret_cast<const e16x8*>(stage + v_frag_off + 2 * D * 16 + t * 512);
      if (tail) {
        v0 = zero_tail(v0, nv0 < 0 ? 0 : nv0);
        v1 = zero_tail(v1, nv1 < 0 ? 0 : nv1);
      }
      acc[t] = mfma_32x32x16(v0, p0, acc[t]);
      acc[t] = mfma_32x32x16(v1, p1, acc[t]);
    }
  };

  // Step u: after the wait only the loads of the two younger stages can still be in flight, so this
  // wave's part of stage u % 4 has landed; after the barrier everybody's has, and everybody is done with
  // stage (u - 1) % 4, which is refilled with step u + 3.
  auto step_fn = [&](auto stage_c, int u) {
    constexpr int S = decltype(stage_c)::value;
    wait_vmcnt<2 * NI>();
    pipeline_barrier();
    fetch(std::integral_constant<int, (S + NST - 1) % NST>{}, u + NST - 1);
    process(stage_c, u);
  };
  fetch(std::integral_constant<int, 0>{}, 0);
  fetch(std::integral_constant<int, 1>{}, 1);
  fetch(std::integral_constant<int, 2>{}, 2);
  for (int u = 0; u < nsteps; u += NST) {
    step_fn(std::integral_constant<int, 0>{}, u);
    step_fn(std::integral_constant<int, 1>{}, u + 1);
    step_fn(std::integral_constant<int, 2>{}, u + 2);
    step_fn(std::integral_constant<int, 3>{}, u + 3);
  }
  wait_vmcnt<0>();   // nothing may still be writing LDS when the workgroup ends

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (col0 + col < ncols) {
    const float inv = 1.0f / l_tot;
    const size_t at = (size_t)(row0 + tok) * a.nq * D + (r * g + hg) * D + 4 * grp;
#pragma unroll
    for (int t = 0; t < DT; ++t) {
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        e16x4 ob, ol;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float val = acc[t][q4 * 4 + e] * inv;
          ob[e] = f32_to_act(val, a.out_half);
          ol[e] = f32_to_e16(val - e16_to_f32(ob[e]));
        }
        *reinterpret_cast<e16x4*>(a.out + at + t * 32 + q4 * 8) = ob;
        if (a.out_lo) *reinterpret_cast<e16x4*>(a.out_lo + at + t * 32 + q4 * 8) = ol;
      }
    }
  }
}

}  // namespace

hipError_t launch_attn_prefill(const AttnArgs& a, const PrefillTile* tiles, int num_tiles, hipStream_t stream) {
  dim3 grid(num_tiles * a.nkv), block(256);
#define MOLINK_PREFILL(KERNEL) hipLaunchKernelGGL((KERNEL), grid, block, 0, stream, a, tiles, num_tiles)
  if (a.alibi) {   // linear biases: the stepwise kernel, with one query plane or two
    if (a.head_dim == 128) {
      if (a.q_lo) MOLINK_PREFILL((attn_prefill_two_plane_kernel<128, true, true>));
      else MOLINK_PREFILL((attn_prefill_two_plane_kernel<128, false, true>));
    } else {
      if (a.q_lo) MOLINK_PREFILL((attn_prefill_two_plane_kernel<64, true, true>));
      else MOLINK_PREFILL((attn_prefill_two_plane_kernel<64, false, true>));
    }
  } else if (a.head_dim == 128) {
    if (a.q_lo) MOLINK_PREFILL((attn_prefill_two_plane_kernel<128>));
    else MOLINK_PREFILL((attn_prefill_kernel<128>));
  } else {
    if (a.q_lo) MOLINK_PREFILL((attn_prefill_two_plane_kernel<64>));
    else MOLINK_PREFILL((attn_prefill_kernel<64>));
  }
#undef MOLINK_PREFILL
  return hipGetLastError();
}

hipError_t launch_attn_decode(const AttnArgs& a, const DecodeItem* items, int num_items, float* part_o,
                              float2* part_ml, hipStream_t stream) {
  dim3 grid(((num_items + 7) / 8) * 8 * ((a.nkv + 3) / 4)), block(256);
#define MOLINK_DECODE(D, QLO, ALIBI) \
  hipLaunchKernelGGL((attn_decode_kernel<D, QLO, ALIBI>), grid, block, 0, stream, a, items, num_items, part_o, part_ml)
  if (a.head_dim == 128) {
    if (a.alibi) { if (a.q_lo) MOLINK_DECODE(128, true, true); else MOLINK_DECODE(128, false, true); }
    else { if (a.q_lo) MOLINK_DECODE(128, true, false); else MOLINK_DECODE(128, false, false); }
  } else {
    if (a.alibi) { if (a.q_lo) MOLINK_DECODE(64, true, true); else MOLINK_DECODE(64, false, true); }
    else { if (a.q_lo) MOLINK_DECODE(64, true, false); else MOLINK_DECODE(64, false, false); }
  }
#undef MOLINK_DECODE
  return hipGetLastError();
}

hipError_t launch_attn_merge(const AttnArgs& a, const DecodeToken* tokens, int num_tokens, const float* part_o,
                             const float2* part_ml, hipStream_t stream) {
  const int total = num_tokens * a.nq * (a.head_dim / 4);
  dim3 grid((total + 255) / 256), block(256);
  if (a.head_dim == 128)
    hipLaunchKernelGGL(attn_merge_kernel<128>, grid, block, 0, stream, a, tokens, num_tokens, part_o, part_ml);
  else
    hipLaunchKernelGGL(attn_merge_kernel<64>, grid, block, 0, stream, a, tokens, num_tokens, part_o, part_ml);
  return hipGetLastError();
}

}  // namespace molink
