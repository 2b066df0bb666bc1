// 4-bit group-quantised projection weights (the precision the paper runs its 70B model at, section 5
// "Models").  Format: codes uint32 [N][K/8], element k of a row in bits 4*(k%8)..4*(k%8)+3 of word k/8;
// scales and zero points e16 [N][K/group];  W[n][k] = (code - zero) * scale.
#include "w4.hpp"
#include "common.hpp"

#include <type_traits>

namespace molink {

namespace {

// One thread expands one word (8 consecutive k of one row) into 16 bytes of e16.
__global__ __launch_bounds__(256) void dequant_w4_kernel(const uint32_t* __restrict__ codes, const e16* __restrict__ scales,
                                                        const e16* __restrict__ zeros, int words_per_row, int group,
                                                        size_t total_words, e16* __restrict__ out) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total_words) return;
  const size_t row = idx / words_per_row;
  const int word = (int)(idx % words_per_row);
  const int groups_per_row = words_per_row * 8 / group;
  const size_t g = row * groups_per_row + (size_t)(word * 8 / group);
  const float s = e16_to_f32(scales[g]), z = e16_to_f32(zeros[g]);
  const uint32_t x = codes[idx];
  e16x8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = f32_to_e16(((float)((x >> (4 * i)) & 15u) - z) * s);
  *reinterpret_cast<e16x8*>(out + idx * 8) = o;
}

// ------------------------------------------------------------------------------------------------
// Weight-streaming GEMM on the stored 4-bit form, for micro-batches of at most 64 rows (decode).
//
// Decomposition as in the e16 weight-streaming kernel: K is cut into slices of 1024, a workgroup (one
// per CU, eight waves) keeps one slice and walks over units of 16 weight rows; the slices' partial
// sums are added by the reduction kernels.  A quarter of the bytes per weight changes what is scarce:
//  - Every weight is expanded exactly once.  Wave w owns the k range [128 w, 128 w + 128) of the slice -
//    one quantisation group - for ALL activation rows (up to four blocks of 16 rows, held in registers
//    as MFMA operands), so no two waves read the same code.  The eight waves' sums over their k ranges
//    meet in LDS: waves 0-3 each own one block of activation rows, take the eight contributions to it
//    after a barrier, add them in wave order and write the block's partial sums.
//  - Expansion is folded into the contraction.  A code c becomes the e16 number 128 + c by or-ing its
//    four bits into 0x4300 (bfloat16; IEEE half: 1024 + c, into 0x6400; "128" below stands for either
//    offset; two codes per 32-bit operation; the word's fields k and k+4 land in one
//    register, and the activation operands are permuted once to the same order).  The MFMAs give
//    T = sum (128 + c) a over the wave's group; scale and zero point enter once per accumulator register:
//    s * (T - (128 + z) * sum a), with sum a from one MFMA against ones per slice.  The weights are the
//    MFMA's row operand, so a lane ends up with four consecutive weight rows of one activation row:
//    16-byte stores, and one activation sum per lane.  Products and sums are fp32, so nothing but the
//    activations is ever rounded to e16.
//  - Two waves per SIMD and two units between barriers: a unit is a chain of LDS reads, expansion, MFMAs,
//    scaling and exchange whose latencies a wave can only hide behind another such chain.
// Waves 4-7 also issue the loads (global_load_lds) and no stores, waves 0-3 the stores and no loads, so
// each wave's memory counter counts one kind of operation and the waits on it stay exact.  A stage is 32
// weight rows x 512 bytes of codes, laid out so that the 4-byte fragment reads of 16 rows fall into 64
// different banks, plus the rows' scales and zero points of the slice; four stages, up to four in flight.
// ------------------------------------------------------------------------------------------------
constexpr int kW4KS = 1024;            // K elements per slice (must equal the e16 streaming kernel's)
constexpr int kW4Rows = 16;            // weight rows per unit
constexpr int kW4UnitsPerStage = 2;
constexpr int kW4Stages = 4;
constexpr int kW4StageBytes = 32 * 512 + 512 + 512;   // codes, scales [4 pairs][32 rows] dwords, zero points likewise
constexpr int kW4Group = 128;

// The 16-bit format of the MFMA operands: e16, or IEEE half when a bfloat16 stage keeps its activations as half
// (HALF_ACT).  Per format: the offset whose pattern has its four lowest mantissa bits worth 1, 2, 4, 8 (as a
// pair), 1.0 as a pair, and the offset as a number.  Scales and zero points are e16 in either case.
template <bool HALF_ACT> struct OperandFormat {
  static constexpr bool kHalf = HALF_ACT || kElemIsF16 != 0;
  static constexpr uint32_t kCodeBasePair = kHalf ? 0x64006400u : 0x43004300u;
  static constexpr uint32_t kOnesPair = kHalf ? 0x3C003C00u : 0x3F803F80u;
  static constexpr float kCodeBase = kHalf ? 1024.f : 128.f;
};

// Two 4-bit codes (bits 0-3 and 16-19 of x) as two 16-bit numbers offset + code.  Plain C on purpose: written as an
// inline-assembly v_and_or_b32 the result fed the next MFMA without the wait states the compiler inserts
// between a vector write and a matrix read (it does not look inside assembly), and results were wrong.
template <bool HALF_ACT> __device__ __forceinline__ uint32_t expand_pair(uint32_t x) {
  return (x & 0x000F000Fu) | OperandFormat<HALF_ACT>::kCodeBasePair;
}

template <bool HALF_ACT> __device__ __forceinline__ f32x4 mfma16(e16x8 a, e16x8 b, f32x4 c) {
  if constexpr (OperandFormat<HALF_ACT>::kHalf)
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h16x8, a), __builtin_bit_cast(h16x8, b), c, 0, 0, 0);
  else
    return mfma_16x16x32(a, b, c);
}

// NBLK: blocks of 16 activation rows in use (1..4); wave j < NBLK owns block j.
template <int NBLK, bool HALF_ACT>
__global__ __launch_bounds__(512) void gemm_skinny_w4_kernel(GemmArgs p, int nv, int splits, int groups, int swiglu) {
  constexpr int NI = 5;                    // load instructions per loading wave per stage (4 of codes, 1 of scales or zero points)
  using Lds = LdsStages<kW4StageBytes>;
  __shared__ __attribute__((aligned(16))) char red[2][4][8][1024];   // [unit of the stage][owner block][source wave][lane x 16 B]

  // the arguments as plain values (the lambdas below capture these, not the struct)
  const e16* const arg_a = p.a;
  float* const arg_partial = p.partial;
  const int arg_m = p.m, arg_n = p.n, arg_k = p.k, arg_lda = p.lda;
  const uint32_t* const codes0 = p.q0.codes;
  const uint32_t* const codes1 = swiglu ? p.q1.codes : p.q0.codes;
  const e16* const scales0 = p.q0.scales;
  const e16* const scales1 = swiglu ? p.q1.scales : p.q0.scales;
  const e16* const zeros0 = p.q0.zeros;
  const e16* const zeros1 = swiglu ? p.q1.zeros : p.q0.zeros;

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
  const int row_words = arg_k / 8, row_groups = arg_k / kW4Group;
  const bool loader = wave >= 4;
  const int lw = wave - 4;

  // Virtual row v of the column space -> (matrix, row); SwiGLU: 32 gate rows, then the 32 up rows of the same
  // features.  (The lambdas of this kernel capture by value.)  The matrices' pointers are held as values and chosen by select: a choice between pointers to
  // the argument structs would turn every use into a memory load that waits on the loads in flight.
  auto row_of = [=](int v) __attribute__((always_inline)) -> int {
    const int r = swiglu ? (v >> 6) * 32 + (v & 31) : v;
    return r < arg_n ? r : arg_n - 1;            // rows past the matrix repeat its last row (never stored)
  };
  auto is_up = [=](int v) __attribute__((always_inline)) -> bool { return swiglu && (v & 32); };

  // ---- loading (waves 4-7): wave lw fills rows 8 lw .. 8 lw + 7 of every stage's 32, and a quarter of its scales / zero points ----
  // codes: instruction i covers two rows; position lane%32 of a row's 512 bytes receives chunk (lane%32) ^ (row in
  // unit) (16 bytes each), which spreads the 16 rows of a fragment read over all banks
  // Gate or up matrix: chosen by adding a byte distance, not by selecting between two captured pointers (the
  // compiler turns such a select into an indexed read of the closure, which then stays in private memory).
  const ptrdiff_t codes_up = reinterpret_cast<const char*>(codes1) - reinterpret_cast<const char*>(codes0);
  const char* const small0 = reinterpret_cast<const char*>(lw < 2 ? scales0 : zeros0);
  const ptrdiff_t small_up = reinterpret_cast<const char*>(lw < 2 ? scales1 : zeros1) - small0;
  // scales (waves 4, 5) and zero points (waves 6, 7): lane l serves row l%32 of the stage, group pair 2 (lw%2) + l/32
  int pair = kbase / kW4Group / 2 + 2 * (lw & 1) + (lane >> 5);
  pair = pair < row_groups / 2 - 1 ? pair : row_groups / 2 - 1;
  auto fetch = [=](auto stage_c, int st) __attribute__((always_inline)) {
    constexpr int S = decltype(stage_c)::value;
    char* stage = Lds::template get<S>();
    int unit = st * kW4UnitsPerStage + (lw >> 1);
    unit = unit < n_units ? unit : n_units - 1;              // past the last unit: the last one again
    const int v0 = (g_begin + unit) * kW4Rows;               // uniform; a unit never straddles gate and up rows
    const char* const codes = reinterpret_cast<const char*>(codes0) + (is_up(v0) ? codes_up : (ptrdiff_t)0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = ((8 * lw + 2 * i) & 15) + (lane >> 5);     // row inside its unit
      int byte = kbase / 2 + (((lane & 31) ^ row) * 16);
      byte = byte < arg_k / 2 - 16 ? byte : arg_k / 2 - 16;      // past the end of K: any codes, the activations there are zero
      const int r = row_of(v0 + row);
      const char* src = codes + (size_t)r * row_words * 4 + byte;
      __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(src),
                                       reinterpret_cast<uint32_t*>(stage + (4 * lw + i) * 1024), 16, 0, 2);
    }
    int urow = st * kW4UnitsPerStage + ((lane >> 4) & 1);
    urow = urow < n_units ? urow : n_units - 1;
    const int vr = (g_begin + urow) * kW4Rows + (lane & 15);
    const size_t at = (size_t)row_of(vr) * row_groups + 2 * pair;
    const char* const src = small0 + (is_up(vr) ? small_up : (ptrdiff_t)0);
    __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(src + at * 2),
                                     reinterpret_cast<uint32_t*>(stage + 16384 + (lw >> 1) * 512 + (lw & 1) * 256), 4, 0, 0);
  };

  if (loader) {   // the first four stages are requested before anything else
    fetch(std::integral_constant<int, 0>{}, 0);
    fetch(std::integral_constant<int, 1>{}, 1);
    fetch(std::integral_constant<int, 2>{}, 2);
    fetch(std::integral_constant<int, 3>{}, 3);
  }

  // ---- multiplying (all waves) ----
  const int col = lane & 15, quarter = lane >> 4;
  const int kw = kbase + 128 * wave;                // this wave's k range: one group
  // activations as MFMA column operands: lane (row col of block j, quarter) holds k = kw + 32 t + 8 quarter .. +7 of
  // MFMA step t, in the order (k0 k4 k1 k5 k2 k6 k3 k7) the expanded weights come out in
  e16x8 act[NBLK][4];
#pragma unroll
  for (int j = 0; j < NBLK; ++j) {
    int m = 16 * j + col;
    m = m < arg_m ? m : arg_m - 1;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int k = kw + 32 * t + 8 * quarter;
      u32x4 x = {0u, 0u, 0u, 0u};
      if (k < arg_k) x = __builtin_bit_cast(u32x4, load8(arg_a + (size_t)m * arg_lda + k));
      const u32x4 y = {(x[0] & 0xFFFFu) | (x[2] << 16), (x[0] >> 16) | (x[2] & 0xFFFF0000u),
                       (x[1] & 0xFFFFu) | (x[3] << 16), (x[1] >> 16) | (x[3] & 0xFFFF0000u)};
      act[j][t] = __builtin_bit_cast(e16x8, y);
    }
  }
  // sum of this lane's activation row (row col of block j) over the wave's group
  float asum[NBLK];
  {
    constexpr uint32_t kOnesPair = OperandFormat<HALF_ACT>::kOnesPair;
    const u32x4 ones_bits = {kOnesPair, kOnesPair, kOnesPair, kOnesPair};
    const e16x8 ones = __builtin_bit_cast(e16x8, ones_bits);
#pragma unroll
    for (int j = 0; j < NBLK; ++j) {
      f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int t = 0; t < 4; ++t) s = mfma16<HALF_ACT>(ones, act[j][t], s);   // every row of the result is the sum
      asum[j] = s[0];
    }
  }
  // (the activation loads were issued after the first stages' loads and have been waited for by now, so in the
  // loading waves the memory counter counts tile loads only from here on)

  // fragment of MFMA step t: lane (weight row col, quarter) wants the word with k = 128 wave + 32 t + 8 quarter .. +7 of
  // its row: byte 64 wave + 16 t + 4 quarter, stored at chunk (4 wave + t) ^ col
  // (the low two bits of the chunk index are t ^ (col & 3); the rest does not depend on t)
  const int frag_base = col * 512 + (((4 * wave) ^ (col & 12)) * 16) + 4 * quarter;
  const int col3 = col & 3;

  auto flush = [=](int unit, int sub) __attribute__((always_inline)) {
    // partial sums of `unit` for this wave's own block of activation rows: the eight waves' contributions in
    // wave order, then out
    if (wave >= NBLK) return;
    const char* slot_base = &red[sub][wave][0][0] + lane * 16;
    f32x4 sum = *reinterpret_cast<const f32x4*>(slot_base);
#pragma unroll
    for (int w = 1; w < 8; ++w) sum += *reinterpret_cast<const f32x4*>(slot_base + w * 1024);
    // accumulator register r of lane l is C[weight row 4 (l/16) + r][activation row l%16]
    const int v = (g_begin + unit) * kW4Rows + 4 * quarter;
    const int m = 16 * wave + col;
    if (m < arg_m && v < nv) *reinterpret_cast<f32x4*>(arg_partial + ((size_t)split * arg_m + m) * nv + v) = sum;
  };

  auto compute = [=](auto stage_c, int unit, int sub) __attribute__((always_inline)) {
    constexpr int S = decltype(stage_c)::value;
    const char* stage = Lds::template get<S>();
    const char* codes = stage + sub * 8192;
    uint32_t xs[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) xs[t] = *reinterpret_cast<const uint32_t*>(codes + frag_base + ((t ^ col3) << 4));
    // scales and zero points of this lane's four weight rows (each word: the groups of waves 2p and 2p + 1)
    const u32x4 sc = *reinterpret_cast<const u32x4*>(stage + 16384 + (wave >> 1) * 128 + (sub * 16 + 4 * quarter) * 4);
    const u32x4 zp = *reinterpret_cast<const u32x4*>(stage + 16384 + 512 + (wave >> 1) * 128 + (sub * 16 + 4 * quarter) * 4);
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
    f32x4 tmp[NBLK];
#pragma unroll
    for (int j = 0; j < NBLK; ++j) tmp[j] = zero4;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const uint32_t x = xs[t];
      const u32x4 wbits = {expand_pair<HALF_ACT>(x), expand_pair<HALF_ACT>(x >> 4), expand_pair<HALF_ACT>(x >> 8),
                           expand_pair<HALF_ACT>(x >> 12)};
      const e16x8 wf = __builtin_bit_cast(e16x8, wbits);
#pragma unroll
      for (int j = 0; j < NBLK; ++j) tmp[j] = mfma16<HALF_ACT>(wf, act[j][t], tmp[j]);
    }
    f32x4 s, zc;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      s[r] = (wave & 1) ? e16_hi(sc[r]) : e16_lo(sc[r]);
      zc[r] = OperandFormat<HALF_ACT>::kCodeBase + ((wave & 1) ? e16_hi(zp[r]) : e16_lo(zp[r]));
    }
    // hand every block's contribution to its owner
#pragma unroll
    for (int j = 0; j < NBLK; ++j)
      *reinterpret_cast<f32x4*>(&red[sub][j][wave][lane * 16]) = (tmp[j] - zc * asum[j]) * s;
  };

  // A stage: wait until its loads have landed (those of the next three stages may still be in flight) and meet;
  // every wave multiplies the stage's two units - two independent chains of LDS reads, expansion, MFMAs and
  // scaling that overlap each other - and leaves its contributions in LDS; meet again; then the loading
  // waves refill the stage just read with stage st + 4 while the owning waves add up and store both units.
  // The first barrier of the next stage keeps the contributions from being overwritten before they are read.
#define MOLINK_W4_STAGE(S, ST)                                                                        \
  {                                                                                                  \
    const int u0_ = (ST) * kW4UnitsPerStage;                                                          \
    if (loader) wait_vmcnt<3 * NI>();                                                                 \
    pipeline_barrier();                                                                              \
    if (u0_ < n_units) compute(std::integral_constant<int, (S)>{}, u0_, 0);                           \
    if (u0_ + 1 < n_units) compute(std::integral_constant<int, (S)>{}, u0_ + 1, 1);                   \
    pipeline_barrier();                                                                              \
    if (loader) fetch(std::integral_constant<int, (S)>{}, (ST) + kW4Stages);                          \
    if (u0_ < n_units) flush(u0_, 0);                                                                 \
    if (u0_ + 1 < n_units) flush(u0_ + 1, 1);                                                         \
  }
  static_assert(kW4UnitsPerStage == 2, "two units per stage are written out");
  int st = 0;
  for (; st + 4 <= n_stages; st += 4) {
    MOLINK_W4_STAGE(0, st)
    MOLINK_W4_STAGE(1, st + 1)
    MOLINK_W4_STAGE(2, st + 2)
    MOLINK_W4_STAGE(3, st + 3)
  }
  if (st < n_stages) MOLINK_W4_STAGE(0, st)
  if (st + 1 < n_stages) MOLINK_W4_STAGE(1, st + 1)
  if (st + 2 < n_stages) MOLINK_W4_STAGE(2, st + 2)
#undef MOLINK_W4_STAGE
  if (loader) wait_vmcnt<0>();   // nothing may still be writing LDS when the workgroup ends
}

}  // namespace

hipError_t launch_dequant_w4(const W4Matrix& w, int n, int k, int group, e16* out, hipStream_t stream) {
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
  const int blocks = (a.m + 15) / 16;
#define MOLINK_W4_LAUNCH(NB, HALF) \
  hipLaunchKernelGGL((gemm_skinny_w4_kernel<NB, HALF>), dim3(nwg), dim3(512), 0, stream, a, nv, splits, groups, swiglu)
  if (a.a_half) {
#ifdef MOLINK_F16
    return hipErrorInvalidValue;   // the element type is half already
#else
    switch (blocks) {
      case 1: MOLINK_W4_LAUNCH(1, true); break;
      case 2: MOLINK_W4_LAUNCH(2, true); break;
      case 3: MOLINK_W4_LAUNCH(3, true); break;
      default: MOLINK_W4_LAUNCH(4, true); break;
    }
#endif
  } else {
    switch (blocks) {
      case 1: MOLINK_W4_LAUNCH(1, false); break;
      case 2: MOLINK_W4_LAUNCH(2, false); break;
      case 3: MOLINK_W4_LAUNCH(3, false); break;
      default: MOLINK_W4_LAUNCH(4, false); break;
    }
  }
#undef MOLINK_W4_LAUNCH
  return hipGetLastError();
}

}  // namespace molink
