// 4-bit group-quantised projection weights (the precision the paper runs its 70B model at, section 5
// "Models").  Format: codes uint32 [N][K/8], element k of a row in bits 4*(k%8)..4*(k%8)+3 of word k/8;
// scales and zero points bf16 [N][K/group];  W[n][k] = (code - zero) * scale.
#include "w4.hpp"
#include "common.hpp"

#include <type_traits>

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

// ------------------------------------------------------------------------------------------------
// Weight-streaming GEMM on the stored 4-bit form, for micro-batches of at most 64 rows (decode).
//
// Decomposition as in the bf16 weight-streaming kernel: K is cut into slices of 1024, a workgroup (one
// per CU, eight waves) keeps one slice and walks over units of 16 weight rows; the slices' partial
// sums are added by the reduction kernels.  A quarter of the bytes per weight changes what is scarce:
//  - Every weight is expanded exactly once.  Multiplying wave w owns the k range [256 w, 256 w + 256) of
//    the slice for ALL activation rows (four blocks of 16 rows, held in registers as MFMA operands), so
//    no two waves read the same code.  The four waves' sums over their k ranges meet in LDS: every wave
//    owns one block of activation rows, takes the four contributions to it one unit
//    later (double-buffered, so the unit's single barrier serves both the pipeline and the exchange)
//    and writes the block's partial sums.
//  - Expansion is folded into the contraction.  A code c becomes the bf16 number 128 + c by or-ing its
//    four bits into 0x4300 (two codes per 32-bit operation; the word's fields k and k+4 land in one
//    register, and the activation operands are permuted once to the same order).  Per group of 128
//    input features the MFMAs give T = sum (128 + c) a; the group's scale and zero point enter once per
//    accumulator register:  s * (T - (128 + z) * sum a), with sum a from one MFMA against ones per slice.
//    The weights are the MFMA's row operand, so a lane ends up with four consecutive weight rows of one
//    activation row: 16-byte stores, and one activation sum per lane.
//    Products and sums are fp32, so nothing but the activations is ever rounded to bf16.
// Waves 4-7 only load (global_load_lds): a stage is 64 weight rows x 512 bytes of codes, laid out so that
// the 4-byte fragment reads of 16 rows fall into 64 different banks, plus the rows' scales and zero
// points of the slice; three stages, two in flight.
// ------------------------------------------------------------------------------------------------
constexpr int kW4KS = 1024;            // K elements per slice (must equal the bf16 streaming kernel's)
constexpr int kW4Rows = 16;            // weight rows per unit
constexpr int kW4UnitsPerStage = 4;
constexpr int kW4Stages = 3;
constexpr int kW4StageBytes = 64 * 512 + 1024 + 1024;   // codes, scales [4][64] dwords, zero points [4][64] dwords
constexpr int kW4Group = 128;

// Two 4-bit codes (bits 0-3 and 16-19 of x) as two bf16 numbers 128 + code: (x & 0x000F000F) | 0x43004300 in one
// instruction (the mask in a scalar register, 0x43004300 in a vector register: one scalar operand per
// instruction; the compiler emits an AND and an OR otherwise).
__device__ __forceinline__ uint32_t expand_pair(uint32_t x) {
  uint32_t r;
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "s"(0x000F000Fu), "v"(0x43004300u));
  return r;
}

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// NBLK: blocks of 16 activation rows in use (1..4); waves NBLK..3 own no block and only contribute.
template <int NBLK>
__global__ __launch_bounds__(512) void gemm_skinny_w4_kernel(GemmArgs p, int nv, int splits, int groups, int swiglu) {
  constexpr int NI = 10;                   // load instructions per loading wave per stage (8 of codes, scales, zero points)
  using Lds = LdsStages<kW4StageBytes>;
  __shared__ __attribute__((aligned(16))) char red[2][4][4][1024];   // [unit parity][owner block][source wave][lane x 16 B]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nwg = gridDim.x;
  const int split = blockIdx.x % splits, slot = blockIdx.x / splits;
  const int peers = (nwg - split + splits - 1) / splits;          // workgroups that share this slice
  const int g_begin = (int)((long)groups * slot / peers);
  const int g_end = (int)((long)groups * (slot + 1) / peers);
  const int n_units = g_end - g_begin;
  if (n_units <= 0) return;
  const int n_stages = (n_units + kW4UnitsPerStage - 1) / kW4UnitsPerStage;
  const int kbase = split * kW4KS;
  const int row_words = p.k / 8, row_groups = p.k / kW4Group;

  // Virtual row v of the column space -> (matrix, row); SwiGLU: 32 gate rows, then the 32 up rows of the same
  // features.  The matrices' pointers are held as values and chosen by select: a choice between pointers to
  // the argument structs would turn every use into a memory load that waits on the loads in flight.
  const uint32_t* const codes0 = p.q0.codes;
  const uint32_t* const codes1 = swiglu ? p.q1.codes : p.q0.codes;
  const __bf16* const scales0 = p.q0.scales;
  const __bf16* const scales1 = swiglu ? p.q1.scales : p.q0.scales;
  const __bf16* const zeros0 = p.q0.zeros;
  const __bf16* const zeros1 = swiglu ? p.q1.zeros : p.q0.zeros;
  auto row_of = [&](int v) -> int {
    const int r = swiglu ? (v >> 6) * 32 + (v & 31) : v;
    return r < p.n ? r : p.n - 1;            // rows past the matrix repeat its last row (never stored)
  };
  auto is_up = [&](int v) -> bool { return swiglu && (v & 32); };

  if (wave >= 4) {
    // ---- loading waves: wave lw fills unit lw of every stage, and dword lw of the stage's scales and zero points ----
    const int lw = wave - 4;
    // codes: instruction i covers rows 2i, 2i+1 of the unit; position lane%32 of a row's 512 bytes receives chunk
    // (lane%32) ^ row (16 bytes each), which spreads the 16 rows of a fragment read over all banks
    uint32_t code_off[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = 2 * i + (lane >> 5);
      int byte = kbase / 2 + (((lane & 31) ^ row) * 16);
      byte = byte < p.k / 2 - 16 ? byte : p.k / 2 - 16;      // past the end of K: any codes, the activations there are zero
      code_off[i] = (uint32_t)byte;
    }
    int pair = kbase / kW4Group / 2 + lw;                     // the two groups of multiplying wave lw
    pair = pair < row_groups / 2 - 1 ? pair : row_groups / 2 - 1;
    auto fetch = [&](auto stage_c, int st) {
      constexpr int S = decltype(stage_c)::value;
      char* stage = Lds::template get<S>();
      int unit = st * kW4UnitsPerStage + lw;
      unit = unit < n_units ? unit : n_units - 1;              // past the last unit: the last one again
      const int v0 = (g_begin + unit) * kW4Rows;            // uniform; a unit never straddles gate and up rows
      const uint32_t* const codes = is_up(v0) ? codes1 : codes0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int r = row_of(v0 + 2 * i + (lane >> 5));
        const char* src = reinterpret_cast<const char*>(codes + (size_t)r * row_words) + code_off[i];
        __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(src),
                                         reinterpret_cast<uint32_t*>(stage + lw * 8192 + i * 1024), 16, 0, 2);
      }
      // scales and zero points: lane l serves row l of the stage's 64
      int urow = st * kW4UnitsPerStage + (lane >> 4);
      urow = urow < n_units ? urow : n_units - 1;
      const int vr = (g_begin + urow) * kW4Rows + (lane & 15);
      const size_t at = (size_t)row_of(vr) * row_groups + 2 * pair;
      const __bf16* const sc = is_up(vr) ? scales1 : scales0;
      const __bf16* const zp = is_up(vr) ? zeros1 : zeros0;
      __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(sc + at),
                                       reinterpret_cast<uint32_t*>(stage + 32768 + lw * 256), 4, 0, 0);
      __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(zp + at),
                                       reinterpret_cast<uint32_t*>(stage + 32768 + 1024 + lw * 256), 4, 0, 0);
    };
    // At the first barrier of stage st only the loads of stage st + 1 may still be in flight; after it the
    // multiplying waves are done with stage st - 1, whose memory takes stage st + 2.
    auto run_stage = [&](auto stage_c, int st) {
      constexpr int S = decltype(stage_c)::value;
      wait_vmcnt<NI>();
      pipeline_barrier();
      fetch(std::integral_constant<int, (S + 2) % kW4Stages>{}, st + 2);
      pipeline_barrier();
      pipeline_barrier();
      pipeline_barrier();
    };
    fetch(std::integral_constant<int, 0>{}, 0);
    fetch(std::integral_constant<int, 1>{}, 1);
    int st = 0;
    for (; st + 3 <= n_stages; st += 3) {
      run_stage(std::integral_constant<int, 0>{}, st);
      run_stage(std::integral_constant<int, 1>{}, st + 1);
      run_stage(std::integral_constant<int, 2>{}, st + 2);
    }
    if (st < n_stages) run_stage(std::integral_constant<int, 0>{}, st);
    if (st + 1 < n_stages) run_stage(std::integral_constant<int, 1>{}, st + 1);
    pipeline_barrier();   // the multiplying waves' last exchange
    wait_vmcnt<0>();      // nothing may still be writing LDS when the workgroup ends
    return;
  }

  // ---- multiplying waves ----
  const int col = lane & 15, quarter = lane >> 4;
  const int kw = kbase + 256 * wave;                // this wave's k range
  // activations as MFMA column operands: lane (row col of block j, quarter) holds k = kw + 32 t + 8 quarter .. +7 of
  // MFMA step t, in the order (k0 k4 k1 k5 k2 k6 k3 k7) the expanded weights come out in
  bf16x8 act[NBLK][8];
#pragma unroll
  for (int j = 0; j < NBLK; ++j) {
    int m = 16 * j + col;
    m = m < p.m ? m : p.m - 1;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int k = kw + 32 * t + 8 * quarter;
      u32x4 x = {0u, 0u, 0u, 0u};
      if (k < p.k) x = __builtin_bit_cast(u32x4, load8(p.a + (size_t)m * p.lda + k));
      const u32x4 y = {(x[0] & 0xFFFFu) | (x[2] << 16), (x[0] >> 16) | (x[2] & 0xFFFF0000u),
                       (x[1] & 0xFFFFu) | (x[3] << 16), (x[1] >> 16) | (x[3] & 0xFFFF0000u)};
      act[j][t] = __builtin_bit_cast(bf16x8, y);
    }
  }
  // sum of this lane's activation row (row col of block j) over each of the wave's two groups
  float asum[2][NBLK];
  {
    const u32x4 ones_bits = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
    const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_bits);
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
      for (int j = 0; j < NBLK; ++j) {
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 4; ++t) s = mfma16(ones, act[j][4 * g + t], s);   // every row of the result is the sum
        asum[g][j] = s[0];
      }
  }

  // fragment of MFMA step t: lane (weight row col, quarter) wants the word with k = 256 wave + 32 t + 8 quarter .. +7 of
  // its row: byte 128 wave + 16 t + 4 quarter, stored at chunk (8 wave + t) ^ col
  // (the low three bits of the chunk index are t ^ (col & 7); the rest does not depend on t)
  const int frag_base = col * 512 + (((8 * wave) ^ (col & 8)) * 16) + 4 * quarter;
  const int col7 = col & 7;

  auto flush = [&](int unit) {
    // partial sums of `unit` for this wave's own block of activation rows: the four waves' contributions in
    // wave order, then out
    if (wave >= NBLK) return;
    const char* slot_base = &red[unit & 1][wave][0][0] + lane * 16;
    const f32x4 p0 = *reinterpret_cast<const f32x4*>(slot_base);
    const f32x4 p1 = *reinterpret_cast<const f32x4*>(slot_base + 1024);
    const f32x4 p2 = *reinterpret_cast<const f32x4*>(slot_base + 2048);
    const f32x4 p3 = *reinterpret_cast<const f32x4*>(slot_base + 3072);
    const f32x4 sum = ((p0 + p1) + p2) + p3;
    // accumulator register r of lane l is C[weight row 4 (l/16) + r][activation row l%16]
    const int v = (g_begin + unit) * kW4Rows + 4 * quarter;
    const int m = 16 * wave + col;
    if (m < p.m && v < nv) *reinterpret_cast<f32x4*>(p.partial + ((size_t)split * p.m + m) * nv + v) = sum;
  };

  auto compute = [&](auto stage_c, int unit, int sub) {
    constexpr int S = decltype(stage_c)::value;
    const char* stage = Lds::template get<S>();
    const char* codes = stage + sub * 8192;
    // the LDS reads of a group go out together, so that their latency is paid once
    uint32_t xs[2][4];
#pragma unroll
    for (int t = 0; t < 4; ++t) xs[0][t] = *reinterpret_cast<const uint32_t*>(codes + frag_base + ((t ^ col7) << 4));
    // scales and zero points of this lane's four weight rows (each word: the wave's two groups)
    const u32x4 sc = *reinterpret_cast<const u32x4*>(stage + 32768 + wave * 256 + (sub * 16 + 4 * quarter) * 4);
    const u32x4 zp = *reinterpret_cast<const u32x4*>(stage + 32768 + 1024 + wave * 256 + (sub * 16 + 4 * quarter) * 4);
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
    f32x4 fin[NBLK];
#pragma unroll
    for (int j = 0; j < NBLK; ++j) fin[j] = zero4;
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      f32x4 tmp[NBLK];
#pragma unroll
      for (int j = 0; j < NBLK; ++j) tmp[j] = zero4;
      if (g == 0) {   // the second group's words are fetched under the first group's MFMAs
#pragma unroll
        for (int t = 0; t < 4; ++t)
          xs[1][t] = *reinterpret_cast<const uint32_t*>(codes + frag_base + (((4 + t) ^ col7) << 4));
      }
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        const int t = 4 * g + tt;
        const uint32_t x = xs[g][tt];
        const u32x4 wbits = {expand_pair(x), expand_pair(x >> 4), expand_pair(x >> 8), expand_pair(x >> 12)};
        const bf16x8 wf = __builtin_bit_cast(bf16x8, wbits);
#pragma unroll
        for (int j = 0; j < NBLK; ++j) tmp[j] = mfma16(wf, act[j][t], tmp[j]);
      }
      f32x4 s, zc;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        s[r] = __uint_as_float(g == 0 ? sc[r] << 16 : sc[r] & 0xFFFF0000u);
        zc[r] = 128.f + __uint_as_float(g == 0 ? zp[r] << 16 : zp[r] & 0xFFFF0000u);
      }
#pragma unroll
      for (int j = 0; j < NBLK; ++j) fin[j] += (tmp[j] - zc * asum[g][j]) * s;
    }
    // hand every block's contribution to its owner (this wave's own block included)
#pragma unroll
    for (int j = 0; j < NBLK; ++j) *reinterpret_cast<f32x4*>(&red[unit & 1][j][wave][lane * 16]) = fin[j];
  };

  int pending = -1;   // unit whose exchange is complete after the next barrier
  auto run_stage = [&](auto stage_c, int st) {
#pragma unroll 1
    for (int sub = 0; sub < kW4UnitsPerStage; ++sub) {
      const int unit = st * kW4UnitsPerStage + sub;
      pipeline_barrier();
      if (pending >= 0) flush(pending);
      if (unit < n_units) {
        compute(stage_c, unit, sub);
        pending = unit;
      } else {
        pending = -1;
      }
    }
  };
  int st = 0;
  for (; st + 3 <= n_stages; st += 3) {
    run_stage(std::integral_constant<int, 0>{}, st);
    run_stage(std::integral_constant<int, 1>{}, st + 1);
    run_stage(std::integral_constant<int, 2>{}, st + 2);
  }
  if (st < n_stages) run_stage(std::integral_constant<int, 0>{}, st);
  if (st + 1 < n_stages) run_stage(std::integral_constant<int, 1>{}, st + 1);
  pipeline_barrier();
  if (pending >= 0) flush(pending);
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

namespace molink {

bool skinny_w4_supports(int m, int k, int group, bool two_planes) {
  return m <= 64 && !two_planes && group == kW4Group && k % kW4Group == 0 && (k / kW4Group) % 2 == 0 && k >= 256;
}

hipError_t launch_gemm_skinny_w4(const GemmArgs& a, int nv, int splits, int swiglu, hipStream_t stream) {
  if (a.m > 64 || a.a_lo || !a.q0.codes || (swiglu && !a.q1.codes)) return hipErrorInvalidValue;
  if (splits != (a.k + kW4KS - 1) / kW4KS) return hipErrorInvalidValue;
  const int groups = (nv + kW4Rows - 1) / kW4Rows;
  const long units = (long)groups * splits;
  const int cus = 256;
  const int nwg = units < cus ? (int)units : (cus > splits ? cus : splits);
  switch ((a.m + 15) / 16) {
    case 1: hipLaunchKernelGGL(gemm_skinny_w4_kernel<1>, dim3(nwg), dim3(512), 0, stream, a, nv, splits, groups, swiglu); break;
    case 2: hipLaunchKernelGGL(gemm_skinny_w4_kernel<2>, dim3(nwg), dim3(512), 0, stream, a, nv, splits, groups, swiglu); break;
    case 3: hipLaunchKernelGGL(gemm_skinny_w4_kernel<3>, dim3(nwg), dim3(512), 0, stream, a, nv, splits, groups, swiglu); break;
    default: hipLaunchKernelGGL(gemm_skinny_w4_kernel<4>, dim3(nwg), dim3(512), 0, stream, a, nv, splits, groups, swiglu); break;
  }
  return hipGetLastError();
}

}  // namespace molink
