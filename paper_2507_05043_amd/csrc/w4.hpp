// 4-bit group-quantised weights: W[n][k] = (code[n][k] - zero[n][k/group]) * scale[n][k/group]
// (host-side declarations).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "elem.hpp"

#include "gemm.hpp"

namespace molink {

// Writes the matrix as e16 [n][k] (the product formed in fp32, rounded once).  k % group == 0, group % 8 == 0.
hipError_t launch_dequant_w4(const W4Matrix& w, int n, int k, int group, e16* out, hipStream_t stream);

// Whether the weight-streaming kernel below takes this shape as it is stored: at most 64 rows, one activation
// plane, groups of 128, an even number of groups per row.  (Above 64 rows see tile_w4_supports in gemm.hpp; what
// neither takes the caller expands with launch_dequant_w4 and hands to a e16 GEMM.)
bool skinny_w4_supports(int m, int k, int group, bool two_planes);

// Decode-sized GEMM on 4-bit weights, args.q0 (and args.q1 for the gate/up pair) in place of w0 / w1.
// Same decomposition and output as the e16 weight-streaming kernel: fp32 partial sums
// [splits][m][nv] in args.partial, to be added by the reduction kernels.
hipError_t launch_gemm_skinny_w4(const GemmArgs& args, int nv, int splits, int swiglu, hipStream_t stream);

}  // namespace molink
