// Bandwidth-bound row kernels of the decoder block: RMSNorm, the RoPE angle table, and the fused
// RoPE + KV-cache append.  All global accesses are 16-byte vectors along the contiguous dimension,
// except the transposed V writes of the append (2-byte elements, 32 bytes apart by construction of
// the V block layout [d][16 slots]).
#include "elementwise.hpp"
#include "common.hpp"

namespace molink {

namespace {

// One row per workgroup.  RMSNorm: one pass for the mean square, one to scale.  LayerNorm (ns.layer): a pass for the
// mean first, then the mean of the squared deviations, then (x - mean) * rs * gain + bias; the row stays in the
// caches between the passes.
template <bool FROM_BF16>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const e16* __restrict__ in_e16, float* __restrict__ x,
                                                      NormSpec ns, e16* __restrict__ out,
                                                      e16* __restrict__ out_lo, int hidden, bool out_half) {
  __shared__ float partial[4];
  __shared__ float partial_sum[4];
  const int row = blockIdx.x, tid = threadIdx.x;
  const int chunks = hidden / 8;
  const e16* src_b = in_e16 + (size_t)row * hidden;
  float* xr = x + (size_t)row * hidden;
  auto load_row8 = [&](int c, float* v) {
    if constexpr (FROM_BF16) {
      const e16x8 b = load8(src_b + c * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = e16_to_f32(b[e]);
    } else {
      const float4 p = *reinterpret_cast<const float4*>(xr + c * 8);
      const float4 q = *reinterpret_cast<const float4*>(xr + c * 8 + 4);
      v[0] = p.x; v[1] = p.y; v[2] = p.z; v[3] = p.w; v[4] = q.x; v[5] = q.y; v[6] = q.z; v[7] = q.w;
    }
  };
  float mean = 0.f;
  if (ns.layer) {
    float sum = 0.f;
    for (int c = tid; c < chunks; c += 256) {
      float v[8];
      load_row8(c, v);
#pragma unroll
      for (int e = 0; e < 8; ++e) sum += v[e];
    }
    sum = wave_sum(sum);
    if ((tid & 63) == 0) partial_sum[tid >> 6] = sum;
    __syncthreads();
    mean = (partial_sum[0] + partial_sum[1] + partial_sum[2] + partial_sum[3]) / (float)hidden;
  }
  float ss = 0.f;
  for (int c = tid; c < chunks; c += 256) {
    float v[8];
    load_row8(c, v);
    if constexpr (FROM_BF16) {
      *reinterpret_cast<float4*>(xr + c * 8) = make_float4(v[0], v[1], v[2], v[3]);
      *reinterpret_cast<float4*>(xr + c * 8 + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += (v[e] - mean) * (v[e] - mean);
  }
  ss = wave_sum(ss);
  if ((tid & 63) == 0) partial[tid >> 6] = ss;
  __syncthreads();
  const float total = partial[0] + partial[1] + partial[2] + partial[3];
  const float rs = 1.0f / sqrtf(total / (float)hidden + ns.eps);
  for (int c = tid; c < chunks; c += 256) {
    float v[8];
    load_row8(c, v);
    const e16x8 g = load8(ns.gain + c * 8);
    float add[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (ns.bias) {
      const e16x8 b = load8(ns.bias + c * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) add[e] = e16_to_f32(b[e]);
    }
    e16x8 o, lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float val = (v[e] - mean) * rs * e16_to_f32(g[e]);
      if (ns.bias) val += add[e];
      o[e] = f32_to_act(val, out_half);
      lo[e] = f32_to_act(val - act_to_f32(o[e], out_half), out_half);     // what the rounding dropped, for two-plane GEMMs
    }
    store8(out + (size_t)row * hidden + c * 8, o);
    if (out_lo) store8(out_lo + (size_t)row * hidden + c * 8, lo);
  }
}

__device__ __forceinline__ float gelu_tanh_f(float z) {
  // 0.5 z (1 + tanh(t)) = z / (1 + exp(-2 t)),  t = sqrt(2/pi) (z + 0.044715 z^3)
  const float t = 0.7978845608028654f * (z + 0.044715f * z * z * z);
  return z / (1.0f + __expf(-2.0f * t));
}
__device__ __forceinline__ float gelu_erf_f(float z) { return 0.5f * z * (1.0f + erff(z * 0.7071067811865476f)); }

// x[t][:] += bias, ahead of a projection whose product is added to x and carries a bias.
__global__ __launch_bounds__(256) void add_row_bias_kernel(float* __restrict__ x, const e16* __restrict__ bias, int hidden,
                                                           size_t count8) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= count8) return;
  const int col = (int)(idx % (size_t)(hidden / 8)) * 8;
  const e16x8 b = load8(bias + col);
  f32x4 p = *reinterpret_cast<const f32x4*>(x + idx * 8), q = *reinterpret_cast<const f32x4*>(x + idx * 8 + 4);
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    p[e] += e16_to_f32(b[e]);
    q[e] += e16_to_f32(b[e + 4]);
  }
  *reinterpret_cast<f32x4*>(x + idx * 8) = p;
  *reinterpret_cast<f32x4*>(x + idx * 8 + 4) = q;
}

// The ungated MLP's first half after its matrix product: out[t][f] = gelu(sum of the product's split-K planes + bias),
// rounded once.  One thread per 8 consecutive features.
__global__ __launch_bounds__(256) void bias_gelu_kernel(const float* __restrict__ src, int planes, size_t plane_stride,
                                                        const e16* __restrict__ bias, int erf_form,
                                                        e16* __restrict__ out, e16* __restrict__ out_lo, int ffn,
                                                        size_t count8, bool out_half) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= count8) return;
  const int col = (int)(idx % (size_t)(ffn / 8)) * 8;
  const float* q = src + idx * 8;
  f32x4 a = *reinterpret_cast<const f32x4*>(q), b = *reinterpret_cast<const f32x4*>(q + 4);
  for (int k = 1; k < planes; ++k) {
    a += *reinterpret_cast<const f32x4*>(q + k * plane_stride);
    b += *reinterpret_cast<const f32x4*>(q + k * plane_stride + 4);
  }
  float v[8] = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  if (bias) {
    const e16x8 bb = load8(bias + col);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] += e16_to_f32(bb[e]);
  }
  e16x8 o, lo;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float val = erf_form ? gelu_erf_f(v[e]) : gelu_tanh_f(v[e]);
    o[e] = f32_to_act(val, out_half);
    lo[e] = f32_to_act(val - act_to_f32(o[e], out_half), out_half);
  }
  store8(out + idx * 8, o);
  if (out_lo) store8(out_lo + idx * 8, lo);
}

__global__ __launch_bounds__(256) void rope_table_kernel(const int32_t* __restrict__ positions,
                                                         float2* __restrict__ cos_sin, int rows, int half,
                                                         double log2_theta, RopeScaling sc) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * half) return;
  const int t = idx / half, i = idx % half;
  double inv_freq = exp2(-(double)i / (double)half * log2_theta);   // theta^(-2i/d), d = 2*half
  if (sc.kind == 1) {
    inv_freq /= (double)sc.factor;
  } else if (sc.kind == 2) {
    // by wavelength against the trained length: fast pairs keep their frequency, slow ones are divided by the
    // factor, those in between get the mix that is continuous at both borders
    const double wavelength = 6.283185307179586 / inv_freq, length = (double)sc.original_max_position;
    if (wavelength > length / (double)sc.low_freq_factor) {
      inv_freq /= (double)sc.factor;
    } else if (!(wavelength < length / (double)sc.high_freq_factor)) {
      const double smooth = (length / wavelength - (double)sc.low_freq_factor) /
                            ((double)sc.high_freq_factor - (double)sc.low_freq_factor);
      inv_freq = (1.0 - smooth) * inv_freq / (double)sc.factor + smooth * inv_freq;
    }
  }
  const double ang = (double)positions[t] * inv_freq;
  double s, c;
  sincos(ang, &s, &c);
  cos_sin[idx] = make_float2((float)c, (float)s);
}

// One workgroup per token row.  Work units of 8 elements:
//   rotated heads (q then k): unit = (head, chunk of 8 pairs; a pair is (i, i + rotary_dim/2) or, with neighbour
//   pairing, (2i, 2i + 1)): reads the 16 fp32 values, rotates, rounds to
//   e16 once, writes the e16 row and, for k heads, also the K pool row of the token's slot;
//   with a partial rotary embedding, the elements of q and k heads past rotary_dim: unit = (head, chunk of 8),
//   rounded and written like the rotated ones, unrotated;
//   v heads: unit = (head, chunk of 8 dims): rounded once and scattered into the transposed V block.
__global__ __launch_bounds__(256) void rope_append_kernel(RopeAppendArgs p) {
  const int t = blockIdx.x;
  const int u = blockIdx.y * 256 + threadIdx.x;                  // one unit of 8 (rotated: 8 pairs) per thread
  const int d = p.head_dim, half = p.rotary_dim / 2, cpr = half / 8;       // chunks per rotated head
  const int ppr = (d - p.rotary_dim) / 8;                                    // unrotated chunks per q / k head
  const int rot_units = (p.nq + p.nkv) * cpr;
  const int pass_units = (p.nq + p.nkv) * ppr;
  const int v_units = p.nkv * (d / 8);
  if (u >= rot_units + pass_units + v_units) return;
  const int row_elems = (p.nq + 2 * p.nkv) * d;
  const float* src = p.qkv_f32 + (size_t)t * row_elems;
  e16* row = p.qkv + (size_t)t * row_elems;
  const int64_t slot = p.slots[t];
  const int64_t blk = slot / kKvBlock;
  const int s = (int)(slot % kKvBlock);
  // 8 consecutive fp32 values, summed over the split-K planes in plane order
  auto load8f = [&](const float* q, float* v) {
    f32x4 a = *reinterpret_cast<const f32x4*>(q), b = *reinterpret_cast<const f32x4*>(q + 4);
    for (int k = 1; k < p.planes; ++k) {
      a += *reinterpret_cast<const f32x4*>(q + k * p.plane_stride);
      b += *reinterpret_cast<const f32x4*>(q + k * p.plane_stride + 4);
    }
    v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3]; v[4] = b[0]; v[5] = b[1]; v[6] = b[2]; v[7] = b[3];
    if (p.bias) {
      const e16x8 bb = load8(p.bias + (q - src));
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += e16_to_f32(bb[e]);
    }
  };
  if (u < rot_units) {
    const int head = u / cpr, c = u % cpr;
    const float2* cs = p.cos_sin + (size_t)t * half + c * 8;
    // the unit's 8 pairs (first[e], second[e]), pair index 8 c + e: elements (8 c + e, half + 8 c + e), or with
    // neighbour pairing elements (16 c + 2 e, 16 c + 2 e + 1) - two consecutive chunks either way, at at0 and at1
    const int at0 = p.interleaved ? 16 * c : 8 * c, at1 = p.interleaved ? 16 * c + 8 : half + 8 * c;
    auto pairs_of = [&](const float* x0, const float* x1, float* first, float* second) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        first[e] = p.interleaved ? (e < 4 ? x0[2 * e] : x1[2 * e - 8]) : x0[e];
        second[e] = p.interleaved ? (e < 4 ? x0[2 * e + 1] : x1[2 * e - 7]) : x1[e];
      }
    };
    float lo[8], hi[8];
    {
      float x0[8], x1[8];
      load8f(src + head * d + at0, x0);
      load8f(src + head * d + at1, x1);
      pairs_of(x0, x1, lo, hi);
    }
    if (p.q_gain) {
      // per-head RMSNorm: the head's d values sit in cpr consecutive lanes (cpr = 4 or 8, heads start at
      // multiples of cpr), all of them in this branch
      float ss = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += lo[e] * lo[e] + hi[e] * hi[e];
      for (int off = 1; off < cpr; off <<= 1) ss += __shfl_xor(ss, off, 64);
      const float inv = 1.0f / sqrtf(ss / (float)d + p.head_eps);
      const e16* gain = head < p.nq ? p.q_gain : p.k_gain;
      const e16x8 g0 = load8(gain + at0), g1 = load8(gain + at1);
      float x0[8], x1[8], gl[8], gh[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) { x0[e] = e16_to_f32(g0[e]); x1[e] = e16_to_f32(g1[e]); }
      pairs_of(x0, x1, gl, gh);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        lo[e] = lo[e] * inv * gl[e];
        hi[e] = hi[e] * inv * gh[e];
      }
    }
    // rotate, round once, and put every value back where its input came from
    float y0[8], y1[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float2 f = cs[e];
      y0[e] = lo[e] * f.x - hi[e] * f.y;
      y1[e] = hi[e] * f.x + lo[e] * f.y;
    }
    e16x8 o0, o1, l0, l1;     // the chunks at at0 and at1: values, and what rounding dropped
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float v0 = p.interleaved ? ((e & 1) ? y1[e >> 1] : y0[e >> 1]) : y0[e];
      const float v1 = p.interleaved ? ((e & 1) ? y1[4 + (e >> 1)] : y0[4 + (e >> 1)]) : y1[e];
      o0[e] = f32_to_e16(v0);
      o1[e] = f32_to_e16(v1);
      l0[e] = f32_to_e16(v0 - e16_to_f32(o0[e]));
      l1[e] = f32_to_e16(v1 - e16_to_f32(o1[e]));
    }
    e16* base = row + head * d;
    store8(base + at0, o0);
    store8(base + at1, o1);
    if (head < p.nq) {
      if (p.q_lo) {
        e16* lb = p.q_lo + ((size_t)t * p.nq + head) * d;
        store8(lb + at0, l0);
        store8(lb + at1, l1);
      }
    } else {
      const int r = head - p.nq;
      e16* dst = p.k_pool + ((size_t)blk * p.nkv + r) * kKvBlock * d;
      store8(dst + k_offset_in_block(s, at0), o0);
      store8(dst + k_offset_in_block(s, at1), o1);
    }
  } else if (u < rot_units + pass_units) {
    const int w = u - rot_units;
    const int head = w / ppr, at = p.rotary_dim + (w % ppr) * 8;     // element of the head this unit starts at
    float v[8];
    load8f(src + head * d + at, v);
    e16x8 hi, lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      hi[e] = f32_to_e16(v[e]);
      lo[e] = f32_to_e16(v[e] - e16_to_f32(hi[e]));
    }
    store8(row + head * d + at, hi);
    if (head < p.nq) {
      if (p.q_lo) store8(p.q_lo + ((size_t)t * p.nq + head) * d + at, lo);
    } else {
      e16* dst = p.k_pool + ((size_t)blk * p.nkv + (head - p.nq)) * kKvBlock * d;
      store8(dst + k_offset_in_block(s, at), hi);
    }
  } else {
    const int w = u - rot_units - pass_units;
    const int r = w / (d / 8), c = w % (d / 8);
    float v[8];
    load8f(src + (p.nq + p.nkv + r) * d + c * 8, v);
    e16x8 vb;
#pragma unroll
    for (int e = 0; e < 8; ++e) vb[e] = f32_to_e16(v[e]);
    store8(row + (p.nq + p.nkv + r) * d + c * 8, vb);
    e16* dst = p.v_pool + (((size_t)blk * p.nkv + r) * d + c * 8) * kKvBlock + s;
#pragma unroll
    for (int e = 0; e < 8; ++e) dst[e * kKvBlock] = vb[e];
  }
}

__global__ __launch_bounds__(256) void embed_gather_kernel(const e16* __restrict__ table, const int32_t* __restrict__ ids,
                                                           e16* __restrict__ out, int hidden) {
  const int t = blockIdx.x;
  const e16* src = table + (size_t)ids[t] * hidden;
  e16* dst = out + (size_t)t * hidden;
  for (int c = threadIdx.x * 8; c < hidden; c += 256 * 8) store8(dst + c, load8(src + c));
}

__global__ __launch_bounds__(256) void gather_rmsnorm_kernel(const e16* __restrict__ in, const int32_t* __restrict__ rows,
                                                             NormSpec ns, e16* __restrict__ out, int hidden) {
  __shared__ float wsum[4];
  __shared__ float wmean[4];
  const int s = blockIdx.x, tid = threadIdx.x;
  const e16* src = in + (size_t)rows[s] * hidden;
  float mean = 0.f;
  if (ns.layer) {                       // LayerNorm: the mean first, then the squared deviations from it
    float sum = 0.f;
    for (int c = tid * 8; c < hidden; c += 256 * 8) {
      const e16x8 v = load8(src + c);
#pragma unroll
      for (int e = 0; e < 8; ++e) sum += e16_to_f32(v[e]);
    }
    sum = wave_sum(sum);
    if ((tid & 63) == 0) wmean[tid >> 6] = sum;
    __syncthreads();
    mean = ((wmean[0] + wmean[1]) + (wmean[2] + wmean[3])) / (float)hidden;
  }
  float ss = 0.f;
  for (int c = tid * 8; c < hidden; c += 256 * 8) {
    const e16x8 v = load8(src + c);
#pragma unroll
    for (int e = 0; e < 8; ++e) { const float f = e16_to_f32(v[e]) - mean; ss += f * f; }
  }
  ss = wave_sum(ss);
  if ((tid & 63) == 0) wsum[tid >> 6] = ss;
  __syncthreads();
  const float tot = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
  const float rs = 1.0f / sqrtf(tot / (float)hidden + ns.eps);
  for (int c = tid * 8; c < hidden; c += 256 * 8) {
    const e16x8 v = load8(src + c), g = load8(ns.gain + c);
    e16x8 o;
    if (ns.bias) {
      const e16x8 b = load8(ns.bias + c);
#pragma unroll
      for (int e = 0; e < 8; ++e)
        o[e] = f32_to_e16((e16_to_f32(v[e]) - mean) * rs * e16_to_f32(g[e]) + e16_to_f32(b[e]));
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = f32_to_e16((e16_to_f32(v[e]) - mean) * rs * e16_to_f32(g[e]));
    }
    store8(out + (size_t)s * hidden + c, o);
  }
}

// One workgroup per row.  Every thread keeps the best (value, index) of the columns it visits in
// increasing order (so `>` keeps the earliest), then the pairs are combined preferring the larger
// value and, among equal values, the smaller index.
__global__ __launch_bounds__(1024) void argmax_rows_kernel(const float* __restrict__ src, int planes, size_t plane_stride,
                                                           int vocab, float* __restrict__ logits_out,
                                                           int32_t* __restrict__ tokens) {
  __shared__ float bv[16];
  __shared__ int bi[16];
  const int row = blockIdx.x, tid = threadIdx.x;
  const float* base = src + (size_t)row * vocab;
  float best = -INFINITY;
  int best_i = 0x7fffffff;
  for (int c = tid * 4; c < vocab; c += 1024 * 4) {
    f32x4 v = *reinterpret_cast<const f32x4*>(base + c);
    for (int k = 1; k < planes; ++k) v += *reinterpret_cast<const f32x4*>(base + k * plane_stride + c);
    if (logits_out) *reinterpret_cast<f32x4*>(logits_out + (size_t)row * vocab + c) = v;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (v[e] > best || best_i == 0x7fffffff) { best = v[e]; best_i = c + e; }
  }
  auto better = [](float v, int i, float w, int j) { return v > w || (v == w && i < j); };
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float ov = __shfl_xor(best, off, 64);
    const int oi = __shfl_xor(best_i, off, 64);
    if (oi != 0x7fffffff && (best_i == 0x7fffffff || better(ov, oi, best, best_i))) { best = ov; best_i = oi; }
  }
  if ((tid & 63) == 0) { bv[tid >> 6] = best; bi[tid >> 6] = best_i; }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < 16; ++w)
      if (bi[w] != 0x7fffffff && (best_i == 0x7fffffff || better(bv[w], bi[w], best, best_i))) { best = bv[w]; best_i = bi[w]; }
    tokens[row] = best_i == 0x7fffffff ? 0 : best_i;
  }
}

}  // namespace

hipError_t launch_embed_gather(const e16* table, const int32_t* ids, e16* out, int rows, int hidden,
                               hipStream_t stream) {
  hipLaunchKernelGGL(embed_gather_kernel, dim3(rows), dim3(256), 0, stream, table, ids, out, hidden);
  return hipGetLastError();
}

hipError_t launch_gather_rmsnorm(const e16* in, const int32_t* rows, const NormSpec& norm, e16* out, int n_rows,
                                 int hidden, hipStream_t stream) {
  hipLaunchKernelGGL(gather_rmsnorm_kernel, dim3(n_rows), dim3(256), 0, stream, in, rows, norm, out, hidden);
  return hipGetLastError();
}

hipError_t launch_argmax_rows(const float* src, int planes, size_t plane_stride, int rows, int vocab, float* logits_out,
                              int32_t* tokens, hipStream_t stream) {
  hipLaunchKernelGGL(argmax_rows_kernel, dim3(rows), dim3(1024), 0, stream, src, planes, plane_stride, vocab, logits_out,
                     tokens);
  return hipGetLastError();
}

hipError_t launch_rmsnorm(const e16* in_e16, float* x, const NormSpec& norm, e16* out, e16* out_lo, int rows,
                          int hidden, bool from_e16, bool out_half, hipStream_t stream) {
  if (from_e16)
    hipLaunchKernelGGL(rmsnorm_kernel<true>, dim3(rows), dim3(256), 0, stream, in_e16, x, norm, out, out_lo, hidden,
                       out_half);
  else
    hipLaunchKernelGGL(rmsnorm_kernel<false>, dim3(rows), dim3(256), 0, stream, in_e16, x, norm, out, out_lo, hidden,
                       out_half);
  return hipGetLastError();
}

hipError_t launch_add_row_bias(float* x, const e16* bias, int rows, int hidden, hipStream_t stream) {
  const size_t count8 = (size_t)rows * (size_t)(hidden / 8);
  hipLaunchKernelGGL(add_row_bias_kernel, dim3((unsigned)((count8 + 255) / 256)), dim3(256), 0, stream, x, bias, hidden,
                     count8);
  return hipGetLastError();
}

hipError_t launch_bias_gelu(const float* src, int planes, size_t plane_stride, const e16* bias, bool erf_form, e16* out,
                            e16* out_lo, int rows, int ffn, bool out_half, hipStream_t stream) {
  const size_t count8 = (size_t)rows * (size_t)(ffn / 8);
  hipLaunchKernelGGL(bias_gelu_kernel, dim3((unsigned)((count8 + 255) / 256)), dim3(256), 0, stream, src, planes,
                     plane_stride, bias, erf_form ? 1 : 0, out, out_lo, ffn, count8, out_half);
  return hipGetLastError();
}

hipError_t launch_rope_table(const int32_t* positions, float2* cos_sin, int rows, int rotary_dim, float theta,
                             const RopeScaling& scaling, hipStream_t stream) {
  const int half = rotary_dim / 2;
  const int total = rows * half;
  hipLaunchKernelGGL(rope_table_kernel, dim3((total + 255) / 256), dim3(256), 0, stream, positions, cos_sin, rows, half,
                     log2((double)theta), scaling);
  return hipGetLastError();
}

hipError_t launch_rope_append(const RopeAppendArgs& args, hipStream_t stream) {
  const int units = (args.nq + args.nkv) * (args.rotary_dim / 16 + (args.head_dim - args.rotary_dim) / 8) +
                    args.nkv * (args.head_dim / 8);
  hipLaunchKernelGGL(rope_append_kernel, dim3(args.rows, (units + 255) / 256), dim3(256), 0, stream, args);
  return hipGetLastError();
}

}  // namespace molink
