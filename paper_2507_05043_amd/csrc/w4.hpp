// 4-bit group-quantised weights: W[n][k] = (code[n][k] - zero[n][k/group]) * scale[n][k/group]
// (host-side declarations).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace molink {

// One quantised matrix [n][k]: codes uint32 [n][k/8] (element k in bits 4*(k%8).. of word k/8), scales and
// zero points bf16 [n][k/group].
struct W4Matrix {
  const uint32_t* codes;
  const __bf16* scales;
  const __bf16* zeros;
};

// Writes the matrix as bf16 [n][k] (the product formed in fp32, rounded once).  k % group == 0, group % 8 == 0.
hipError_t launch_dequant_w4(const W4Matrix& w, int n, int k, int group, __bf16* out, hipStream_t stream);

}  // namespace molink
