// Paged-KV attention kernels: MFMA causal prefill, split-KV decode and its merge (host-side declarations).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "elem.hpp"

namespace molink {

// One unit of decode work: a contiguous key range of one decode token's sequence.
struct DecodeItem {
  int32_t row;        // row of the token in the packed [T] tensors
  int32_t bt_off;     // offset of the sequence's first block in the flat block-table array
  int32_t key_begin;  // first key of the range (multiple of 32)
  int32_t key_end;    // one past the last key (<= ctx + 1)
  int32_t part;       // index of this range's partial result (ranges of a token are consecutive)
  int32_t last_key;   // the token's own logical index = its last key (linear biases count distances from it)
  int32_t pad[2];
};

// One decode token: where its partial results live.
struct DecodeToken {
  int32_t row;
  int32_t first_item;
  int32_t num_items;
  int32_t pad;
};

// One unit of prefill work (one workgroup): 128 query columns (token, head-in-group pairs) of one sequence.
struct PrefillTile {
  int32_t row0;       // row of the chunk's first token
  int32_t q_len;      // tokens in the chunk
  int32_t ctx;        // tokens cached before the chunk
  int32_t bt_off;     // offset of the sequence's first block in the flat block-table array
  int32_t col0;       // first query column of this tile; column = token * g + head_in_group
  int32_t pad[3];
};

struct AttnArgs {
  const e16* qkv;        // [T][(nq + 2 nkv) d], q already rotated
  const e16* q_lo;       // optional [T][nq d]: second plane of the rotated queries (q = hi + lo); nullptr = none
  const e16* k_pool;     // this layer's K region
  const e16* v_pool;     // this layer's V region
  const int32_t* bt_flat;   // flat block tables
  e16* out;              // [T][nq d]
  e16* out_lo;           // optional [T][nq d]: e16(result - e16(result)) for the two-plane output projection
  int nq, nkv, head_dim;
  float scale_log2e;        // log2(e) / sqrt(d)
  bool out_half;            // bfloat16 library only: `out` receives IEEE half bits (for a projection that takes half activations)
  const float* alibi;       // optional [nq] head slopes: scores are lowered by slope * (query index - key index)
};

hipError_t launch_attn_prefill(const AttnArgs& a, const PrefillTile* tiles, int num_tiles, hipStream_t stream);
hipError_t launch_attn_decode(const AttnArgs& a, const DecodeItem* items, int num_items, float* part_o,
                              float2* part_ml, hipStream_t stream);
hipError_t launch_attn_merge(const AttnArgs& a, const DecodeToken* tokens, int num_tokens, const float* part_o,
                             const float2* part_ml, hipStream_t stream);

}  // namespace molink
