// RMSNorm, RoPE angle table and RoPE + paged KV append (host-side declarations).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "elem.hpp"

namespace molink {

// a[t][:] = x[t][:] * gain / sqrt(mean(x[t][:]^2) + eps), rounded to e16; or, with norm.layer, the LayerNorm
// (x - mean) / sqrt(mean((x - mean)^2) + eps) * gain + bias.
// from_e16: the row source is in_e16 (the stage input) and the fp32 residual stream x is also
// initialised from it; otherwise the source is x.
// out_lo (optional): receives e16(value - e16(value)), the second activation plane of the two-plane GEMMs.
// out_half (bfloat16 library only): the output is written as IEEE half bits, for GEMMs that take half activations.
hipError_t launch_rmsnorm(const e16* in_e16, float* x, const NormSpec& norm, e16* out, e16* out_lo, int rows,
                          int hidden, bool from_e16, bool out_half, hipStream_t stream);

// x[t][:] += bias[:] on the fp32 residual stream x [rows][hidden]: the bias of a projection whose product is added to
// x, put there ahead of the product (the sum is the same up to fp32 rounding order).
hipError_t launch_add_row_bias(float* x, const e16* bias, int rows, int hidden, hipStream_t stream);

// The ungated MLP between its two matrix products: out[t][f] = gelu(sum over `planes` planes of src[t][f] + bias[f]),
// planes `plane_stride` floats apart (split-K partial sums, or one plane), gelu in its tanh form or (erf_form) as
// z Phi(z); rounded once to e16 (or IEEE half with out_half), with the optional second plane out_lo.
hipError_t launch_bias_gelu(const float* src, int planes, size_t plane_stride, const e16* bias, bool erf_form, e16* out,
                            e16* out_lo, int rows, int ffn, bool out_half, hipStream_t stream);

// cos_sin[t][i] = (cos, sin)(positions[t] * theta^(-2i/r)), i < r/2, evaluated in fp64; r = rotary_dim, the
// number of leading elements of a head that rotate (head_dim unless the rotary embedding is partial).
// scaling: the frequencies theta^(-2i/r) are replaced by their scaled values (stage_config.rope_scaling: 0 none,
// 1 every frequency / factor, 2 by wavelength against the trained length).
struct RopeScaling {
  int kind;
  float factor, low_freq_factor, high_freq_factor;
  int original_max_position;
};
hipError_t launch_rope_table(const int32_t* positions, float2* cos_sin, int rows, int rotary_dim, float theta,
                             const RopeScaling& scaling, hipStream_t stream);

struct RopeAppendArgs {
  const float* qkv_f32;    // [planes][T][(nq + 2 nkv) d] projection output, fp32 (rounded to e16 only after the
                           // rotation); with planes > 1 the split-K partial sums, added here in plane order
  int planes;
  size_t plane_stride;     // floats between planes
  const e16* bias;      // optional [(nq + 2 nkv) d] projection bias, added before the rotation
  const e16* q_gain;    // optional [d] (with k_gain): per-head RMSNorm of every query head / key head after the
  const e16* k_gain;    // bias and before the rotation, u * gain / sqrt(mean(u^2) + head_eps)
  float head_eps;
  e16* qkv;             // [T][(nq + 2 nkv) d] e16: rotated q heads, rotated k heads, v heads
  e16* q_lo;            // optional [T][nq d]: e16(q - e16(q)), second plane of the rotated queries
  const float2* cos_sin;   // [T][rotary_dim/2]
  const int64_t* slots;    // [T] pool slot of every row
  e16* k_pool;          // this layer's K region [blocks][nkv][16][d]
  e16* v_pool;          // this layer's V region [blocks][nkv][d][16]
  int rows, nq, nkv, head_dim;
  int rotary_dim;          // leading elements of every q and k head that rotate (a multiple of 16, <= head_dim)
  int interleaved;         // 0: element i rotates with element i + rotary_dim/2; 1: element 2i with element 2i + 1
};
hipError_t launch_rope_append(const RopeAppendArgs& args, hipStream_t stream);

// out[t][:] = table[ids[t]][:]  (e16 rows of `hidden` elements, hidden % 8 == 0)
hipError_t launch_embed_gather(const e16* table, const int32_t* ids, e16* out, int rows, int hidden,
                               hipStream_t stream);

// out[s][:] = e16(norm(in[rows[s]][:])), the norm (RMSNorm, or LayerNorm with optional bias) in fp32
hipError_t launch_gather_rmsnorm(const e16* in, const int32_t* rows, const NormSpec& norm, e16* out, int n_rows,
                                 int hidden, hipStream_t stream);

// Per row: logits = sum over `planes` of src[plane][row][:] (in plane order), optionally stored, and the
// index of their maximum (the smallest index among equals) written to tokens[row].
hipError_t launch_argmax_rows(const float* src, int planes, size_t plane_stride, int rows, int vocab, float* logits_out,
                              int32_t* tokens, hipStream_t stream);

}  // namespace molink
