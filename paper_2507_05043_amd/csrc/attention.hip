// Attention over the paged KV pool, both phases, on MFMA with operands read straight from HBM/L2.
//
// Formulation.  Everything is computed transposed: S^T = K Q^T and O^T = V^T P^T.  With the pool
// layout K [block][head][16 slots][d] and V [block][head][d][16 slots], both left operands then have
// their contraction index contiguous in memory (d for K rows, slots for V^T rows), which is exactly
// what an MFMA lane holds (8 consecutive k of one row).  The right operand of the second product,
// P^T, is the accumulator of the first one: the row order of a key tile is a free choice (each lane
// loads its own K row), and choosing it so that a lane's accumulator registers are 8 consecutive slots
// of one block makes the registers of S^T the B operand of the PV product with no data movement
// between lanes and no LDS.  A query column is a lane, so softmax statistics are per-lane scalars.
//
// Masking is by select, never by multiplying with zero: slots past a sequence's end may hold NaN.
// V values of such slots are zeroed before the PV product for the same reason.
#include "attention.hpp"
#include "common.hpp"

namespace molink {

namespace {

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ bf16x8 zero_tail(bf16x8 v, int nvalid) {
  // keep elements [0, nvalid), zero the rest (bitwise, so NaNs vanish)
  u32x4 w = __builtin_bit_cast(u32x4, v);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t lo = (2 * i < nvalid) ? 0x0000ffffu : 0u;
    const uint32_t hi = (2 * i + 1 < nvalid) ? 0xffff0000u : 0u;
    w[i] &= (lo | hi);
  }
  return __builtin_bit_cast(bf16x8, w);
}

__device__ __forceinline__ bf16x8 pack8(const float* p) {
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = f32_to_bf16(p[e]);
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
  bf16x8 ka[D / 32], kb[D / 32];   // key tiles A and B, D/32 MFMA k-steps each
  bf16x8 v[D / 16];                // V^T tiles, one per 16 output dims
};

template <int D, bool QLO>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void attn_decode_kernel(AttnArgs a, const DecodeItem* __restrict__ items,
                                                          int num_items, float* __restrict__ part_o,
                                                          float2* __restrict__ part_ml) {
  constexpr int KS = D / 32;   // MFMA k-steps of the QK product
  constexpr int DT = D / 16;   // 16-row tiles of O^T
  const int lane = threadIdx.x & 63;
  // the four waves of a workgroup take four neighbouring KV heads of the same key range: their
  // blocks are adjacent in the pool, so the workgroup reads 16 KB runs
  const int item_id = blockIdx.x;
  const int r = __builtin_amdgcn_readfirstlane(blockIdx.y * 4 + (threadIdx.x >> 6));   // KV head
  if (r >= a.nkv) return;
  const int g = a.nq / a.nkv;
  const int row = __builtin_amdgcn_readfirstlane(items[item_id].row);
  const int bt_off = __builtin_amdgcn_readfirstlane(items[item_id].bt_off);
  const int key_begin = __builtin_amdgcn_readfirstlane(items[item_id].key_begin);
  const int key_end = __builtin_amdgcn_readfirstlane(items[item_id].key_end);
  const int part = __builtin_amdgcn_readfirstlane(items[item_id].part);
  const int32_t* bt = a.bt_flat + bt_off;
  const int last_block = (key_end - 1) / kKvBlock;
  const int nsteps = (key_end - key_begin + 31) / 32;

  const int col = lane & 15, grp = lane >> 4;
  const int ldq = (a.nq + 2 * a.nkv) * D;

  // Q^T operand: column = query head of the group, lane group holds d = 32*kk + 8*grp .. +7
  bf16x8 qf[KS], qf_lo[QLO ? KS : 1];
  {
    const int head = r * g + (col < g ? col : 0);
    const __bf16* qp = a.qkv + (size_t)row * ldq + head * D + grp * 8;
    const __bf16* ql = QLO ? a.q_lo + ((size_t)row * a.nq + head) * D + grp * 8 : qp;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      bf16x8 v = load8(qp + kk * 32);
      if (col >= g) v = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
      qf[kk] = v;
      if constexpr (QLO) {
        bf16x8 w = load8(ql + kk * 32);
        if (col >= g) w = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        qf_lo[kk] = w;
      }
    }
  }

  // per-lane constants of the K and V^T operand loads
  const int k_bsel = (lane & 15) >> 3;                                  // which block of the pair this lane's K row is in
  const int k_slot = 8 * (((lane & 15) >> 2) & 1) + (lane & 3);         // tile A slot; tile B is +4
  const int v_bsel = grp >> 1;
  const size_t k_lane_off = (size_t)k_slot * D + grp * 8;
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
    const __bf16* kp = a.k_pool + (size_t)pbk * blk_stride + head_off + k_lane_off;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      L.ka[kk] = load8(kp + kk * 32);
      L.kb[kk] = load8(kp + 4 * D + kk * 32);
    }
    const int pbv = v_bsel ? b1 : b0;
    const __bf16* vp = a.v_pool + (size_t)pbv * blk_stride + head_off + v_lane_off;
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
      sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(L.ka[kk], qf[kk], sa, 0, 0, 0);
      sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(L.kb[kk], qf[kk], sb, 0, 0, 0);
      if constexpr (QLO) {   // second query plane into the same scores
        sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(L.ka[kk], qf_lo[kk], sa, 0, 0, 0);
        sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(L.kb[kk], qf_lo[kk], sb, 0, 0, 0);
      }
    }
    const int key0 = key_begin + 32 * step + 8 * grp;     // first of this lane's 8 keys
    const int nvalid = key_end - key0;                    // keys [0, nvalid) of the 8 are real
    float s[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      s[e] = (e < nvalid) ? sa[e] * a.scale_log2e : -INFINITY;
      s[4 + e] = (4 + e < nvalid) ? sb[e] * a.scale_log2e : -INFINITY;
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
    const bf16x8 pf = pack8(p);
    const bool tail = key_begin + 32 * step + 32 > key_end;   // wave-uniform
#pragma unroll
    for (int t = 0; t < DT; ++t) {
      bf16x8 v = L.v[t];
      if (tail) v = zero_tail(v, nvalid < 0 ? 0 : nvalid);
      acc[t] = acc[t] * alpha;
      acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v, pf, acc[t], 0, 0, 0);
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
  float m_max = -INFINITY;
  for (int i = 0; i < t.num_items; ++i) {
    const size_t slot = ((size_t)(t.first_item + i) * a.nkv + r) * g + col;
    m_max = fmaxf(m_max, part_ml[slot].x);
  }
  float l = 0.f;
  f32x4 o = {0.f, 0.f, 0.f, 0.f};
  for (int i = 0; i < t.num_items; ++i) {
    const size_t slot = ((size_t)(t.first_item + i) * a.nkv + r) * g + col;
    const float2 ml = part_ml[slot];
    const float w = fast_exp2(ml.x - m_max);
    l += w * ml.y;
    const f32x4 po = *reinterpret_cast<const f32x4*>(part_o + slot * D + d4 * 4);
    o += po * w;
  }
  const float inv = 1.0f / l;
  bf16x4 ob, ol;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float val = o[e] * inv;
    ob[e] = f32_to_bf16(val);
    ol[e] = f32_to_bf16(val - bf16_to_f32(ob[e]));
  }
  const size_t at = (size_t)t.row * a.nq * D + head * D + d4 * 4;
  *reinterpret_cast<bf16x4*>(a.out + at) = ob;
  if (a.out_lo) *reinterpret_cast<bf16x4*>(a.out_lo + at) = ol;
}

// ------------------------------------------------------------------------------------------------
// Prefill: one wave per 32 query columns of one (sequence, KV head); a column is a (token, head in
// group) pair, column = token * g + head_in_group, so grouped heads share every K/V read.  32x32x16
// MFMA; a step is 32 keys (two blocks).  Row m of the key tile is (block m/16, slot
// 8*((m/4)%2) + 4*((m/8)%2) + m%4): accumulator registers 0..7 of lane group G = lane/32 are then
// slots 8G..8G+7 of the first block, registers 8..15 the same slots of the second block.
// ------------------------------------------------------------------------------------------------
template <int D, bool QLO>
__global__ __launch_bounds__(256) void attn_prefill_kernel(AttnArgs a, const PrefillTile* __restrict__ tiles,
                                                           int num_tiles) {
  constexpr int KS = D / 16;   // MFMA k-steps of the QK product
  constexpr int DT = D / 32;   // 32-row tiles of O^T
  const int lane = threadIdx.x & 63;
  const int tile_id = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6));
  if (tile_id >= num_tiles) return;
  const int r = blockIdx.y;
  const int g = a.nq / a.nkv;
  const int row0 = __builtin_amdgcn_readfirstlane(tiles[tile_id].row0);
  const int q_len = __builtin_amdgcn_readfirstlane(tiles[tile_id].q_len);
  const int ctx = __builtin_amdgcn_readfirstlane(tiles[tile_id].ctx);
  const int bt_off = __builtin_amdgcn_readfirstlane(tiles[tile_id].bt_off);
  const int col0 = __builtin_amdgcn_readfirstlane(tiles[tile_id].col0);
  const int32_t* bt = a.bt_flat + bt_off;
  const int total_keys = ctx + q_len;
  const int last_block = (total_keys - 1) / kKvBlock;
  const int ncols = q_len * g;

  const int col = lane & 31, grp = lane >> 5;
  const int my_col = min(col0 + col, ncols - 1);           // padding columns repeat the last real one
  const int tok = my_col / g, hg = my_col % g;
  const int limit = ctx + tok;                              // last key this column may see
  const int last_col = min(col0 + 31, ncols - 1);
  const int max_limit = ctx + last_col / g;                 // wave-uniform loop bound
  const int nsteps = max_limit / 32 + 1;
  const int ldq = (a.nq + 2 * a.nkv) * D;

  bf16x8 qf[KS], qf_lo[QLO ? KS : 1];
  {
    const __bf16* qp = a.qkv + (size_t)(row0 + tok) * ldq + (r * g + hg) * D + grp * 8;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qf[kk] = load8(qp + kk * 16);
    if constexpr (QLO) {
      const __bf16* ql = a.q_lo + ((size_t)(row0 + tok) * a.nq + r * g + hg) * D + grp * 8;
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) qf_lo[kk] = load8(ql + kk * 16);
    }
  }

  const int k_bsel = col >> 4;
  const int k_slot = 8 * ((col >> 2) & 1) + 4 * ((col >> 3) & 1) + (col & 3);
  const size_t k_lane_off = (size_t)k_slot * D + grp * 8;
  const size_t v_lane_off = (size_t)col * kKvBlock + 8 * grp;
  const size_t blk_stride = (size_t)a.nkv * kKvBlock * D;
  const size_t head_off = (size_t)r * kKvBlock * D;

  auto block_id = [&](int step, int sel) -> int {
    int lb = 2 * step + sel;
    lb = lb < last_block ? lb : last_block;
    return bt[lb];
  };
  auto load_k = [&](bf16x8* kf, int b0, int b1) {
    const int pb = k_bsel ? b1 : b0;
    const __bf16* kp = a.k_pool + (size_t)pb * blk_stride + head_off + k_lane_off;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) kf[kk] = load8(kp + kk * 16);
  };

  f32x16 acc[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  auto process = [&](const bf16x8* kf, int step, int b0, int b1) {
    bf16x8 vf[DT][2];
    {
      const __bf16* vp0 = a.v_pool + (size_t)b0 * blk_stride + head_off + v_lane_off;
      const __bf16* vp1 = a.v_pool + (size_t)b1 * blk_stride + head_off + v_lane_off;
#pragma unroll
      for (int t = 0; t < DT; ++t) {
        vf[t][0] = load8(vp0 + (size_t)t * 32 * kKvBlock);
        vf[t][1] = load8(vp1 + (size_t)t * 32 * kKvBlock);
      }
    }
    f32x16 s;
#pragma unroll
    for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], s, 0, 0, 0);
      if constexpr (QLO) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf_lo[kk], s, 0, 0, 0);
    }
    // register e of this lane is key 32*step + 16*(e/8) + 8*grp + e%8
    const int key_base = 32 * step + 8 * grp;
    float sv[16];
    float m_tile = -INFINITY;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int key = key_base + 16 * (e / 8) + (e % 8);
      sv[e] = (key <= limit) ? s[e] * a.scale_log2e : -INFINITY;
      m_tile = fmaxf(m_tile, sv[e]);
    }
    m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32, 64));
    const float m_new = fmaxf(m_run, m_tile);               // finite from step 0 on: key 0 is visible to all
    const float alpha = fast_exp2(m_run - m_new);
    float psum = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      sv[e] = fast_exp2(sv[e] - m_new);
      psum += sv[e];
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    const bf16x8 p0 = pack8(sv), p1 = pack8(sv + 8);
    const bool tail = 32 * step + 32 > total_keys;            // wave-uniform: slots past the sequence end
    const int nv0 = total_keys - key_base, nv1 = nv0 - 16;
#pragma unroll
    for (int t = 0; t < DT; ++t) {
      bf16x8 v0 = vf[t][0], v1 = vf[t][1];
      if (tail) {
        v0 = zero_tail(v0, nv0 < 0 ? 0 : nv0);
        v1 = zero_tail(v1, nv1 < 0 ? 0 : nv1);
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][e] *= alpha;
      acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v0, p0, acc[t], 0, 0, 0);
      acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v1, p1, acc[t], 0, 0, 0);
    }
  };

  bf16x8 kbuf0[KS], kbuf1[KS];
  int b0 = block_id(0, 0), b1 = block_id(0, 1);
  int n0 = block_id(1, 0), n1 = block_id(1, 1);
  load_k(kbuf0, b0, b1);
  for (int step = 0; step < nsteps; step += 2) {
    const bool has1 = step + 1 < nsteps;
    if (has1) load_k(kbuf1, n0, n1);
    const int f0 = block_id(step + 2, 0), f1 = block_id(step + 2, 1);
    process(kbuf0, step, b0, b1);
    if (has1) {
      const bool has2 = step + 2 < nsteps;
      if (has2) load_k(kbuf0, f0, f1);
      const int h0 = block_id(step + 3, 0), h1 = block_id(step + 3, 1);
      process(kbuf1, step + 1, n0, n1);
      b0 = f0; b1 = f1;
      n0 = h0; n1 = h1;
    }
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (col0 + col < ncols) {
    const float inv = 1.0f / l_tot;
    const size_t at = (size_t)(row0 + tok) * a.nq * D + (r * g + hg) * D + 4 * grp;
#pragma unroll
    for (int t = 0; t < DT; ++t) {
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        bf16x4 ob, ol;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float val = acc[t][q4 * 4 + e] * inv;
          ob[e] = f32_to_bf16(val);
          ol[e] = f32_to_bf16(val - bf16_to_f32(ob[e]));
        }
        *reinterpret_cast<bf16x4*>(a.out + at + t * 32 + q4 * 8) = ob;
        if (a.out_lo) *reinterpret_cast<bf16x4*>(a.out_lo + at + t * 32 + q4 * 8) = ol;
      }
    }
  }
}

}  // namespace

hipError_t launch_attn_prefill(const AttnArgs& a, const PrefillTile* tiles, int num_tiles, hipStream_t stream) {
  dim3 grid((num_tiles + 3) / 4, a.nkv), block(256);
  if (a.head_dim == 128) {
    if (a.q_lo) hipLaunchKernelGGL((attn_prefill_kernel<128, true>), grid, block, 0, stream, a, tiles, num_tiles);
    else hipLaunchKernelGGL((attn_prefill_kernel<128, false>), grid, block, 0, stream, a, tiles, num_tiles);
  } else {
    if (a.q_lo) hipLaunchKernelGGL((attn_prefill_kernel<64, true>), grid, block, 0, stream, a, tiles, num_tiles);
    else hipLaunchKernelGGL((attn_prefill_kernel<64, false>), grid, block, 0, stream, a, tiles, num_tiles);
  }
  return hipGetLastError();
}

hipError_t launch_attn_decode(const AttnArgs& a, const DecodeItem* items, int num_items, float* part_o,
                              float2* part_ml, hipStream_t stream) {
  dim3 grid(num_items, (a.nkv + 3) / 4), block(256);
  if (a.head_dim == 128) {
    if (a.q_lo) hipLaunchKernelGGL((attn_decode_kernel<128, true>), grid, block, 0, stream, a, items, num_items, part_o, part_ml);
    else hipLaunchKernelGGL((attn_decode_kernel<128, false>), grid, block, 0, stream, a, items, num_items, part_o, part_ml);
  } else {
    if (a.q_lo) hipLaunchKernelGGL((attn_decode_kernel<64, true>), grid, block, 0, stream, a, items, num_items, part_o, part_ml);
    else hipLaunchKernelGGL((attn_decode_kernel<64, false>), grid, block, 0, stream, a, items, num_items, part_o, part_ml);
  }
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
