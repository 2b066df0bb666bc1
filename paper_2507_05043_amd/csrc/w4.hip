// 4-bit group-quantised projection weights (the precision the paper runs its 70B model at, section 5
// "Models").  Format: codes uint32 [N][K/8], element k of a row in bits 4*(k%8)..4*(k%8)+3 of word k/8;
// scales and zero points bf16 [N][K/group];  W[n][k] = (code - zero) * scale.
#include "w4.hpp"
#include "common.hpp"

namespace molink {

namespace {

// One thread expands one word (8 consecutive k of one row) into 16 bytes of bf16.
__global__ __launch_bounds__(256) void dequant_w4_kernel(const uint32_t* __restrict__ codes, const __bf16* __restrict__ scales,
                                                        const __bf16* __restrict__ zeros, int words_per_row, int group,
                                                        size_t total_words, __bf16* __restrict__ out) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total_words) return;
  const size_t row = idx / words_per_row;
  const int word = (int)(idx % words_per_row);
  const int groups_per_row = words_per_row * 8 / group;
  const size_t g = row * groups_per_row + (size_t)(word * 8 / group);
  const float s = bf16_to_f32(scales[g]), z = bf16_to_f32(zeros[g]);
  const uint32_t x = codes[idx];
  bf16x8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = f32_to_bf16(((float)((x >> (4 * i)) & 15u) - z) * s);
  *reinterpret_cast<bf16x8*>(out + idx * 8) = o;
}

}  // namespace

hipError_t launch_dequant_w4(const W4Matrix& w, int n, int k, int group, __bf16* out, hipStream_t stream) {
  if (k % 8 || group % 8 || k % group) return hipErrorInvalidValue;
  const size_t total = (size_t)n * (k / 8);
  hipLaunchKernelGGL(dequant_w4_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, w.codes, w.scales,
                     w.zeros, k / 8, group, total, out);
  return hipGetLastError();
}

}  // namespace molink
