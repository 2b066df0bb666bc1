// e16 MFMA GEMM  C[M][N] = A[M][K] * W[N][K]^T  with fused epilogues (host-side declarations).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "elem.hpp"

namespace molink {

enum GemmEpilogue : int {
  kEpiStoreF32 = 0,     // out_f32[m][n] = acc                   (q/k/v before RoPE: rounded only once, after it)
  kEpiResidualF32 = 1,  // resid[m][n] += acc                      (fp32 residual stream, in place)
  kEpiResidualOut = 2,  // out_e16[m][n] = resid[m][n] + acc      (last layer: packed payload)
  kEpiSwiGLU = 3,       // out_e16[m][f] = silu(acc_gate[f]) * acc_up[f]
};

// One 4-bit group-quantised matrix [n][k]: codes uint32 [n][k/8] (element k in bits 4*(k%8).. of word k/8),
// scales and zero points e16 [n][k/group];  W[n][k] = (code - zero) * scale.
struct W4Matrix {
  const uint32_t* codes;
  const e16* scales;
  const e16* zeros;
};

struct GemmArgs {
  const e16* a;      // [M][lda]
  const e16* a_lo;   // optional second plane [M][lda]: the activations are a + a_lo (the part of the fp32
                        // value that e16 rounding dropped); both planes are multiplied into the same
                        // accumulators.  nullptr = single plane.
  e16* out_lo;       // SwiGLU epilogue only, optional: receives e16(result - e16(result)) [M][ldo]
  const e16* w0;     // [N][K]; for SwiGLU the gate matrix [F][K]
  const e16* w1;     // SwiGLU only: the up matrix [F][K]
  const e16* wa0;    // optional: the same matrices once more in operand order (launch_arrange_weights), in the format
  const e16* wa1;    // of the MFMA operands (IEEE half when a_half); read by plans of the kTileArranged kind
  W4Matrix q0, q1;      // q0.codes != nullptr: the weights are 4-bit (groups of 128) and w0 / w1 are unused;
                        // only plans of the weight-streaming kind (at most 64 rows) and of the kTileW4 kind take them
  e16* out_e16;     // see GemmEpilogue
  float* out_f32;       // kEpiStoreF32 output [M][ldo]
  float* resid;         // fp32 residual stream [M][N]
  float* partial;       // split-K scratch [splits][M][Nv] fp32
  int m, n, k;          // n = output features (F for SwiGLU)
  int lda, ldo;         // leading dimensions (elements) of a and of out_e16 / out_f32
  bool a_half;          // bfloat16 library only: `a` holds IEEE half bits (one plane); the weight fragments are
                        // converted to half on their way into the matrix instruction
  bool out_half;        // bfloat16 library only: the SwiGLU epilogue writes IEEE half bits (no out_lo then)
};

// kTileSkinny: at most 64 rows; K cut into slices of 1024, weights streamed in groups of 16 rows, always
// through partial sums (the reduction applies the epilogue).
// kTileW4, kTileW4x128: 256 x 256 and 128 x 256 tiles on 4-bit weights in their stored form (more than 64 rows,
// half operands).  kTileArranged, kTileArranged128: 256 x 256 and 128 x 256 tiles that read the weights' copy in operand order (GemmArgs::wa0 / wa1)
// straight into registers.
enum GemmTile : int { kTile256x256 = 0, kTile256x128 = 1, kTile128x128 = 2, kTile64x128 = 3, kTileSkinny = 4, kTile128x256 = 5, kTileW4 = 6, kTileW4x128 = 7, kTileArranged = 8, kTileArranged128 = 9 };

struct GemmPlan {
  int tile;             // GemmTile: workgroup tile shape
  int splits;           // K splits across workgroups
  bool partials;        // the GEMM kernel writes partial sums [splits][M][nv]; a reduction applies the epilogue
  int k_tiles_per_split;
  int nv;               // width of the column space the kernel iterates (gate/up interleaved for SwiGLU, else N)
};

// How a product of at most 64 rows (one activation plane) is planned: on the weight-streaming kernel, on 64-row
// tiles, or by shape.  Wide projections (K of 8192 and more, 64 M weights and more) do better on the tiles: the
// streaming kernel cuts K into slices of 1024 and writes one plane of partial sums per slice, and with 8 to 28
// slices its reductions cost more than the tiles' few K splits (70B-shaped stage, 52 sequences: 8.5 ms of
// projections and reductions per micro-batch against 7.2); at 7B shapes the streaming kernel is ahead (2.86 ms per
// micro-batch against 3.00).  The stage plans by shape, or on the streaming kernel where 4-bit weights are read in
// their stored form; kFewRowsTiles exists for sizing the scratch of either choice.
enum GemmFewRows : int { kFewRowsByShape = 0, kFewRowsStreaming = 1, kFewRowsTiles = 2 };

// arranged: the weights exist in operand order too, so plans of the kTileArranged kind may be chosen.
GemmPlan plan_gemm(int m, int n, int k, GemmEpilogue epi, int num_cus, bool split_a = false,
                   GemmFewRows few_rows = kFewRowsByShape, bool arranged = false);
// Floats of split-K scratch that any GEMM with m <= max_m rows of this (n, k, epilogue) may need, however its
// products of at most 64 rows are planned.
size_t gemm_partial_floats(int max_m, int n, int k, GemmEpilogue epi, int num_cus, bool split_a = false, bool arranged = false);

// Weights in operand order (see gemm_tile_arranged_kernel): K must be a multiple of 256; the copy holds
// arranged_weights_elems(n, k) elements (rows padded to a multiple of 32 with zeros).  to_half (bfloat16 library only):
// the copy is IEEE half, converted as the GEMMs' registers would (exact within half's range).
bool arranged_weights_supported(int k);
size_t arranged_weights_elems(int n, int k);
hipError_t launch_arrange_weights(const e16* w, int n, int k, bool to_half, e16* out, hipStream_t stream);

// 4-bit weights, more than 64 rows: whether the tiled kernel reads this shape as it is stored (otherwise the
// caller expands the matrix and runs a e16 GEMM).  One activation plane held as IEEE half (`operands_half`: half
// activations in the bfloat16 library, or the half-precision library), groups of 128, K a multiple of 256.
bool tile_w4_supports(int m, int k, int group, bool two_planes, bool operands_half);
// The plan of such a product (tile kTileW4), and the split-K scratch any m <= max_m may need under these plans.
GemmPlan plan_gemm_w4_tile(int m, int n, int k, GemmEpilogue epi, int num_cus);
size_t gemm_partial_floats_w4_tile(int max_m, int n, int k, GemmEpilogue epi, int num_cus);

hipError_t launch_gemm_main(const GemmArgs& args, GemmEpilogue epi, const GemmPlan& plan, hipStream_t stream);
// Only when plan.partials: sums the partial results in split order and applies the epilogue.
hipError_t launch_gemm_reduce(const GemmArgs& args, GemmEpilogue epi, const GemmPlan& plan, hipStream_t stream);

// Only when plan.partials and the epilogue is a residual one: one kernel that sums the partial
// results in split order, adds them to the fp32 residual stream x[m][n] (in place), and then either
// writes the norm of x (RMSNorm or LayerNorm: NormSpec) as e16 to norm_out (norm.gain != nullptr) or rounds x to e16 into
// args.out_e16 (kEpiResidualOut).  Replaces launch_gemm_reduce plus the following RMSNorm.
hipError_t launch_gemm_reduce_residual_norm(const GemmArgs& args, GemmEpilogue epi, const GemmPlan& plan,
                                            const NormSpec& norm, e16* norm_out, e16* norm_out_lo,
                                            bool norm_out_half, hipStream_t stream);

}  // namespace molink
