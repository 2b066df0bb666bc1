// e16 MFMA GEMM for the stage's projections: C[M][N] = A[M][K] * W[N][K]^T, fp32 accumulate.
//
// Both operands are K-contiguous, which is the layout the 32x32x16 e16 MFMA wants in its lanes
// (lane l holds 8 consecutive k of row l%32).  Tiles travel HBM/L2 -> LDS directly (16 bytes per lane,
// 8 rows x 128 bytes per wave instruction, XOR-swizzled so 128-bit LDS reads are conflict free) ->
// MFMA operands.  Two to three K tiles are kept in flight in separate LDS stages; one barrier per K
// tile, placed before the tile's last MFMA step so that the matrix pipe does not drain at it; LDS reads
// and tile loads are interleaved with the MFMAs by explicit scheduling hints.
//
// Workgroup ids are remapped so that consecutive logical tiles share an XCD, and tiles are walked in
// bands of eight tile rows: the workgroups that run together on one XCD form a compact block of the
// output, so each operand tile that enters the XCD's L2 is used by several of them.
//
// Shapes without enough output tiles to fill 256 CUs split the K dimension across workgroups; the
// partial sums go to fp32 scratch and a second kernel adds them in a fixed order (deterministic) and
// applies the epilogue.  Micro-batches of at most 64 rows (decode) have a kernel of their own,
// gemm_skinny_kernel below, built around streaming the weights; the widest projections (K of 8192 and more)
// run on 64-row tiles instead (see GemmFewRows).
//
// 4-bit group-quantised weights: micro-batches of more than 64 rows with half operands run on gemm_tile_w4_kernel,
// which carries the codes into LDS as they are stored and expands them in registers; decode-sized ones on the
// streaming kernel of w4.hip.
//
// Half activations (bfloat16 library, deep stages): with A_HALF the A operand holds IEEE half bits, every weight
// fragment read from LDS is converted from bfloat16 to half in registers (exact) and the f16 MFMA is used; the
// tiles, their pipeline and their epilogues are otherwise the same code.
#include "gemm.hpp"
#include "w4.hpp"
#include "common.hpp"

#include <type_traits>

namespace molink {

namespace {

constexpr int kBK = 64;               // K elements per tile
constexpr int kBandRows = 8;          // tile rows per band of the tile order

// Scheduling hint for one MFMA step of NMFMA MFMAs.  After each MFMA come the memory operations that
// run in its shadow: the NREAD LDS reads of the next step's fragments are placed behind the first
// MFMAs (so they have landed when the step ends), and the step's NLOAD tile loads are spread evenly
// over the whole step - a wave that issues its loads in one burst sits in the address unit's queue and
// issues no MFMA meanwhile.  Group sizes must be compile-time constants, hence the recursion.
template <int R, int NMFMA, int NREAD, int NLOAD>
__device__ __forceinline__ void sched_step() {
  if constexpr (R < NMFMA) {
    constexpr int RSLOTS = NMFMA < NREAD ? NMFMA : (NREAD > 0 ? NREAD : 1);
    constexpr int reads = R < RSLOTS ? (R + 1) * NREAD / RSLOTS - R * NREAD / RSLOTS : 0;
    constexpr int loads = (R + 1) * NLOAD / NMFMA - R * NLOAD / NMFMA;
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if constexpr (reads > 0) __builtin_amdgcn_sched_group_barrier(0x100, reads, 0);
    if constexpr (loads > 0) __builtin_amdgcn_sched_group_barrier(0x010, loads, 0);
    sched_step<R + 1, NMFMA, NREAD, NLOAD>();
  }
}

// z * sigmoid(z); the reciprocal is the hardware's (one ulp), not the IEEE division sequence: the result is rounded
// to 16 bits right after, and the division would be ten vector instructions per output in a tile's epilogue.
__device__ __forceinline__ float silu_f(float z) { return z * __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }

// Epilogue of a wave's MT x NT block of 32x32 accumulator tiles whose first row / column are m_base / n_base.
// Accumulator register r of lane l is C[row 8*(r/4) + 4*(l/32) + r%4][col l%32] of its tile.
// CHECKED = false: the whole block lies inside the output (no per-element bounds tests).
// OUT: how the SwiGLU epilogue stores - kOutByFlags: by p.out_half / p.out_lo, tested per element; kOutHalf: IEEE
// half bits, one plane; kOutOnePlane: the element type, one plane (the two cases that matter, decided once per block).
enum { kOutByFlags = 0, kOutHalf = 1, kOutOnePlane = 2 };
template <int EPI, bool SPLIT, int MT, int NT, bool CHECKED, int OUT = kOutByFlags>
__device__ __forceinline__ void tile_epilogue_body(const GemmArgs& p, f32x16 (&acc)[MT][NT], int m_base, int n_base,
                                                   int nv, int split, int lane) {
  const int col_in_tile = lane & 31;
  const int row_base = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < MT; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m_base + i * 32 + 8 * (r / 4) + row_base + (r % 4);
      if (CHECKED && m >= p.m) continue;
      if constexpr (SPLIT) {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          const int v = n_base + j * 32 + col_in_tile;
          if (!CHECKED || v < nv) p.partial[((size_t)split * p.m + m) * nv + v] = acc[i][j][r];
        }
      } else if constexpr (EPI == kEpiSwiGLU) {
#pragma unroll
        for (int j = 0; j < NT; j += 2) {
          const int v = n_base + j * 32 + col_in_tile;   // gate column; its up column is 32 further
          const int f = (v >> 6) * 32 + (v & 31);
          if (!CHECKED || f < p.n) {
            const float val = silu_f(acc[i][j][r]) * acc[i][j + 1][r];
            if constexpr (OUT == kOutByFlags) {
              const e16 hi = f32_to_act(val, p.out_half);
              p.out_e16[(size_t)m * p.ldo + f] = hi;
              if (p.out_lo) p.out_lo[(size_t)m * p.ldo + f] = f32_to_e16(val - e16_to_f32(hi));
            } else {
              p.out_e16[(size_t)m * p.ldo + f] = f32_to_act(val, OUT == kOutHalf);
            }
          }
        }
      } else {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          const int n = n_base + j * 32 + col_in_tile;
          if (CHECKED && n >= p.n) continue;
          const float c = acc[i][j][r];
          if constexpr (EPI == kEpiStoreF32) {
            p.out_f32[(size_t)m * p.ldo + n] = c;
          } else if constexpr (EPI == kEpiResidualF32) {
            p.resid[(size_t)m * p.n + n] += c;
          } else {
            p.out_e16[(size_t)m * p.ldo + n] = f32_to_e16(p.resid[(size_t)m * p.n + n] + c);
          }
        }
      }
    }
  }
}

template <int EPI, bool SPLIT, int MT, int NT>
__device__ __forceinline__ void tile_epilogue(const GemmArgs& p, f32x16 (&acc)[MT][NT], int m_base, int n_base, int nv,
                                              int split, int lane) {
  // a block is interior when its last row and its last column exist (wave-uniform): partial sums live in the nv
  // columns the kernel iterates, outputs in p.n columns (for SwiGLU: features, two 32-wide column tiles each 32)
  const bool rows_in = m_base + MT * 32 <= p.m;
  bool cols_in = n_base + NT * 32 <= nv;
  if constexpr (!SPLIT && EPI == kEpiSwiGLU) {
    const int v_last = n_base + NT * 32 - 1;             // an up column; its feature index is the block's largest
    cols_in = ((v_last >> 6) * 32 + (v_last & 31)) < p.n;
  } else if constexpr (!SPLIT) {
    cols_in = n_base + NT * 32 <= p.n;
  }
  if (rows_in && cols_in) {
    if constexpr (!SPLIT && EPI == kEpiSwiGLU) {
      if (p.out_lo) tile_epilogue_body<EPI, SPLIT, MT, NT, false>(p, acc, m_base, n_base, nv, split, lane);
      else if (p.out_half) tile_epilogue_body<EPI, SPLIT, MT, NT, false, kOutHalf>(p, acc, m_base, n_base, nv, split, lane);
      else tile_epilogue_body<EPI, SPLIT, MT, NT, false, kOutOnePlane>(p, acc, m_base, n_base, nv, split, lane);
    } else {
      tile_epilogue_body<EPI, SPLIT, MT, NT, false>(p, acc, m_base, n_base, nv, split, lane);
    }
  } else
    tile_epilogue_body<EPI, SPLIT, MT, NT, true>(p, acc, m_base, n_base, nv, split, lane);
}

// Workgroup of 4 waves (2 x 2); wave tile (BM/2) x (BN/2) made of 32x32 MFMA tiles; K tile of 64.
//
// Tiles go from global memory straight into LDS (global_load_lds_dwordx4: each lane's 16 bytes land at
// the wave's LDS base + 16*lane), so data in flight costs no registers and the pipeline depth is set
// by how many stages fit in the 160 KB of LDS (NSTAGE-1 tiles in flight).  One wave instruction
// fills 8 rows x 128 bytes.  Rows are unpadded; bank conflicts are avoided by an XOR swizzle applied
// to the *global* address each lane fetches: slot p of row r holds the row's 16-byte chunk p ^ (r & 7),
// so the 8 lanes of a 128-bit LDS read that hit rows r..r+7 at the same logical chunk touch 8
// different slots.  LDS reads of MFMA step kk+1 are issued under the MFMAs of step kk, across tile
// boundaries too.
template <int BM, int BN, int WAVES_M, int WAVES_N, int NSTAGE, int EPI, bool SPLIT, bool SPLIT_A, bool A_HALF>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gemm_tile_kernel(GemmArgs p, int nv, int tiles_m, int tiles_n, int splits,
                                                        int k_tiles_per_split) {
  constexpr int NWAVES = WAVES_M * WAVES_N;
  constexpr int TM = BM / WAVES_M, TN = BN / WAVES_N;
  constexpr int MT = TM / 32, NT = TN / 32;
  constexpr int AROWS = SPLIT_A ? 2 * BM : BM;  // activation rows per stage: the high plane, then the low plane
  constexpr int GROUPS = (AROWS + BN) / 8;     // 8-row groups per stage (A rows first, then B rows)
  constexpr int NI = GROUPS / NWAVES;          // load instructions per wave per tile
  static_assert(GROUPS % NWAVES == 0, "row groups must divide evenly among the waves");
  constexpr int STAGE_BYTES = (AROWS + BN) * 128;
  static_assert(EPI != kEpiSwiGLU || TN % 64 == 0, "SwiGLU pairs two 32-wide column tiles per wave");
  static_assert(NSTAGE >= 2 && NSTAGE <= 3 && NSTAGE * STAGE_BYTES <= 160 * 1024, "stages must fit in LDS");
  using Lds = LdsStages<STAGE_BYTES>;

  const int total = tiles_m * tiles_n * splits;
  const int lid = xcd_logical_id(blockIdx.x, total);
  if (lid < 0) return;
  int tile_m, tile_n, split;
  if (splits == 1 && tiles_m > kBandRows) {
    // bands of kBandRows tile rows, each walked column by column
    const int band_size = kBandRows * tiles_n;
    const int band = lid / band_size, rem = lid % band_size;
    const int rows_in_band = min(kBandRows, tiles_m - band * kBandRows);
    tile_m = band * kBandRows + rem % rows_in_band;
    tile_n = rem / rows_in_band;
    split = 0;
  } else {
    // split-major: the workgroups of one K range are neighbours, i.e. share an XCD, so the slice of the activation
    // matrix they all read enters that XCD's L2 once instead of every XCD streaming the whole matrix
    tile_m = lid % tiles_m;
    tile_n = (lid / tiles_m) % tiles_n;
    split = lid / (tiles_m * tiles_n);
  }
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  const int k_tiles = (p.k + kBK - 1) / kBK;
  const int kt_begin = split * k_tiles_per_split;
  const int kt_end = min(kt_begin + k_tiles_per_split, k_tiles);
  const int nkt = kt_end - kt_begin;

  // Load instruction j of this wave fills row group g = 4*j + wave.  This lane's slot in the group is
  // (row 8*g + lane/8, position lane%8) and receives the row's chunk (lane%8) ^ (lane/8).
  const int sw_chunk = (lane & 7) ^ (lane >> 3);
  // Byte offset of this lane's chunk from the first row of the workgroup's tile at k = 0.  Offsets are taken from
  // the tile's own first row (a 64-bit base per workgroup), so 32 bits hold them for any matrix size: a tile spans
  // at most 256 rows.
  uint32_t g_off[NI];
  const int b_row0 = EPI == kEpiSwiGLU ? (n0 >> 6) * 32 : n0;   // first weight row of the tile (gate/up: per matrix)
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    const int g = NWAVES * j + wave;
    const int r = 8 * g + (lane >> 3);            // row inside the stage (A rows, then B rows)
    if (r < AROWS) {
      int gm = m0 + (r < BM ? r : r - BM);         // the low plane has the same rows as the high plane
      gm = gm < p.m ? gm : p.m - 1;
      g_off[j] = ((uint32_t)(gm - m0) * (uint32_t)p.lda + sw_chunk * 8) * 2u;
    } else {
      int row;
      if constexpr (EPI == kEpiSwiGLU) {
        // 32 gate rows, then the 32 up rows of the same features (which matrix is decided per 8-row group)
        const int v = n0 + (r - AROWS);
        row = (v >> 6) * 32 + (v & 31);
      } else {
        row = n0 + (r - AROWS);
      }
      row = row < p.n ? row : p.n - 1;
      g_off[j] = ((uint32_t)(row - b_row0) * (uint32_t)p.k + sw_chunk * 8) * 2u;
    }
  }
  const size_t a_tile0 = (size_t)m0 * p.lda, b_tile0 = (size_t)b_row0 * p.k;   // elements

  int zero_below[NSTAGE];   // per stage: leading k columns that repeat the previous tile (shifted last tile)
  auto fetch = [&](auto stage_c, int idx) {
    constexpr int S = decltype(stage_c)::value;
    int kt = kt_begin + idx;
    kt = kt < kt_end - 1 ? kt : kt_end - 1;
    // The last tile of a K that is not a multiple of 64 is shifted back to end exactly at K (every load
    // stays inside its row); the columns it shares with the previous tile are zeroed in LDS afterwards.
    int k0 = kt * kBK;
    const int k_last = p.k - kBK;
    zero_below[S] = k0 > k_last ? k0 - k_last : 0;
    k0 = k0 > k_last ? k_last : k0;
    const char* abase = reinterpret_cast<const char*>(p.a + a_tile0 + k0);
    const char* alobase = SPLIT_A ? reinterpret_cast<const char*>(p.a_lo + a_tile0 + k0) : abase;
    const char* w0base = reinterpret_cast<const char*>(p.w0 + b_tile0 + k0);
    const char* w1base = EPI == kEpiSwiGLU ? reinterpret_cast<const char*>(p.w1 + b_tile0 + k0) : w0base;
    char* stage = Lds::template get<S>();
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int g = NWAVES * j + wave;                          // uniform
      const char* base = g < BM / 8 ? abase
                         : g < AROWS / 8 ? alobase
                                         : ((EPI == kEpiSwiGLU && ((g - AROWS / 8) & 4)) ? w1base : w0base);
      __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(base + g_off[j]),
                                       reinterpret_cast<uint32_t*>(stage + g * 1024), 16, 0, 0);
    }
  };
  // Zero the duplicated columns of a shifted last tile: each lane patches the slots it loaded itself.
  auto patch_tail = [&](auto stage_c) {
    constexpr int S = decltype(stage_c)::value;
    if (zero_below[S] > 0 && sw_chunk * 8 < zero_below[S]) {
      char* stage = Lds::template get<S>();
      const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int j = 0; j < NI; ++j) *reinterpret_cast<u32x4*>(stage + (NWAVES * j + wave) * 1024 + lane * 16) = zero;
    }
  };

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // fragment reads: lane (row l%32, k half l/32) of step kk wants chunk 2*kk + l/32 of its row, which
  // sits at slot (2*kk + l/32) ^ (l % 8) since every fragment's first row is a multiple of 32
  const int frag_row = lane & 31;
  int frag_off[kBK / 16];
#pragma unroll
  for (int kk = 0; kk < kBK / 16; ++kk) frag_off[kk] = frag_row * 128 + (((2 * kk + (lane >> 5)) ^ (lane & 7)) * 16);

  constexpr int NPLANE = SPLIT_A ? 2 : 1;
  constexpr int KSTEPS = kBK / 16, NMFMA = NPLANE * MT * NT, NREAD = NPLANE * MT + NT;
  static_assert(KSTEPS == 4, "four MFMA steps per K tile");
  e16x8 af[2][NPLANE][MT], bfr[2][NT];
  // fragments of MFMA step kk of the tile in stage S into register set s
  auto read_frags = [&](auto stage_c, int s, int kk) {
    constexpr int S = decltype(stage_c)::value;
    const char* la = Lds::template get<S>() + wm * TM * 128;
    const char* lb = Lds::template get<S>() + (AROWS + wn * TN) * 128;
    auto read_a = [&] {
#pragma unroll
      for (int pl = 0; pl < NPLANE; ++pl)
#pragma unroll
        for (int i = 0; i < MT; ++i)
          af[s][pl][i] = *reinterpret_cast<const e16x8*>(la + (pl * BM + i * 32) * 128 + frag_off[kk]);
    };
    // half activations: the weight fragments are read first, so that they land - and can be turned into half, once
    // per read - as early as possible (placing the conversions behind chosen MFMAs with scheduling hints was
    // measured slower: 765 against 712 us on the Qwen2-shaped gate/up product)
    if constexpr (!A_HALF) read_a();
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const e16x8 w = *reinterpret_cast<const e16x8*>(lb + j * 32 * 128 + frag_off[kk]);
      bfr[s][j] = A_HALF ? __builtin_bit_cast(e16x8, bf16x8_to_half(w)) : w;
    }
    if constexpr (A_HALF) read_a();
  };
  auto mfmas = [&](int s) {
#pragma unroll
    for (int pl = 0; pl < NPLANE; ++pl)
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[i][j] = A_HALF ? mfma_32x32x16_half(__builtin_bit_cast(h16x8, af[s][pl][i]), __builtin_bit_cast(h16x8, bfr[s][j]), acc[i][j])
                             : mfma_32x32x16(af[s][pl][i], bfr[s][j], acc[i][j]);
  };

  // One pipeline step: tile idx is in stage S and the fragments of its first MFMA step are already in
  // registers (two register sets alternate).  The wait for tile idx + 1 and the barrier come BEFORE the
  // last MFMA step: by then every fragment of tile idx has been read, so the barrier also frees stage S,
  // and the fragment reads of tile idx + 1 run under the MFMAs of the last step - the matrix pipe does
  // not drain at the barrier.  Where the next tile's loads go depends on the depth:
  //  - three stages: the stage read in the previous step takes tile idx + 2, its loads spread evenly over
  //    the first three MFMA steps (a wave that issues loads faster than the address unit takes them sits
  //    in its queue and issues no MFMA meanwhile; at this tile size the even spread is just that rate);
  //  - two stages: stage S takes tile idx + 2 right after the barrier, under the last MFMA step, which
  //    gives the loads the longest lead a double buffer allows.
  constexpr bool kRefillAfterBarrier = NSTAGE == 2;
  constexpr int L0 = kRefillAfterBarrier ? 0 : NI / 3, L1 = kRefillAfterBarrier ? 0 : (2 * NI) / 3 - NI / 3,
                L2 = kRefillAfterBarrier ? 0 : NI - (2 * NI) / 3, L3 = kRefillAfterBarrier ? NI : 0;
  constexpr int kInFlight = kRefillAfterBarrier ? NSTAGE : NSTAGE - 1;   // tiles requested ahead of the one multiplied
  auto step = [&](auto stage_c, int idx) {
    constexpr int S = decltype(stage_c)::value;
    using Next = std::integral_constant<int, (S + 1) % NSTAGE>;
    if constexpr (!kRefillAfterBarrier) fetch(std::integral_constant<int, (S + NSTAGE - 1) % NSTAGE>{}, idx + NSTAGE - 1);
    read_frags(stage_c, 1, 1);
    mfmas(0);
    sched_step<0, NMFMA, NREAD, L0>();
    read_frags(stage_c, 0, 2);
    mfmas(1);
    sched_step<0, NMFMA, NREAD, L1>();
    read_frags(stage_c, 1, 3);
    mfmas(0);
    sched_step<0, NMFMA, NREAD, L2>();
    __builtin_amdgcn_sched_barrier(0);
    wait_vmcnt<(NSTAGE - 2) * NI>();
    patch_tail(Next{});
    pipeline_barrier();
    if constexpr (kRefillAfterBarrier) fetch(stage_c, idx + NSTAGE);
    read_frags(Next{}, 0, 0);
    mfmas(1);
    sched_step<0, NMFMA, NREAD, L3>();
    __builtin_amdgcn_sched_barrier(0);
  };

  if (nkt > 0) {
    // prologue: the first tiles in flight, tile 0 landed, its first fragments read
    fetch(std::integral_constant<int, 0>{}, 0);
    if constexpr (kInFlight > 1) fetch(std::integral_constant<int, 1>{}, 1);
    if constexpr (kInFlight > 2) fetch(std::integral_constant<int, 2>{}, 2);
    wait_vmcnt<(kInFlight - 1) * NI>();
    patch_tail(std::integral_constant<int, 0>{});
    pipeline_barrier();
    read_frags(std::integral_constant<int, 0>{}, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    int i = 0;
    for (; i + NSTAGE <= nkt; i += NSTAGE) {
      step(std::integral_constant<int, 0>{}, i);
      step(std::integral_constant<int, 1>{}, i + 1);
      if constexpr (NSTAGE > 2) step(std::integral_constant<int, 2>{}, i + 2);
    }
    if (i < nkt) step(std::integral_constant<int, 0>{}, i);
    if constexpr (NSTAGE > 2) {
      if (i + 1 < nkt) step(std::integral_constant<int, 1>{}, i + 1);
    }
    wait_vmcnt<0>();   // nothing may still be writing LDS when the workgroup ends
  }

  tile_epilogue<EPI, SPLIT, MT, NT>(p, acc, m0 + wm * TM, n0 + wn * TN, nv, split, lane);
}

// The 256 x 256 tile on K tiles of 32.
//
// What holds the matrix pipe of the tiles above back is LDS traffic: a ds_read_b128 occupies LDS for 12 clocks
// instead of 8 while tile fills arrive (counters), about 85 bytes per clock, and at full MFMA rate a 128 x 256 tile
// asks for 96 bytes per clock of fragment reads plus 48 of fills.  A 2 x 2 arrangement of 128 x 128 wave tiles
// reads 64 + 32.  Its stages are too large for three of them at a K tile of 64 (the two-stage pipeline of
// gemm_tile_kernel<256, 256> must refill a stage in one burst), so this kernel halves the K tile instead: rows of
// 64 bytes, stages of 32 KB, four of them, three tiles in flight, the next tile's loads spread over the first
// MFMA step.  One load instruction fills 16 rows; chunk c (16 bytes) of row r sits at position c ^ ((r >> 1) & 3),
// which makes the 128-bit fragment reads of eight consecutive rows conflict free.
constexpr int kBK32 = 32;

template <int EPI, bool SPLIT, bool A_HALF>
__global__ __launch_bounds__(256) void gemm_tile32_kernel(GemmArgs p, int nv, int tiles_m, int tiles_n, int splits,
                                                          int k_tiles_per_split) {
  constexpr int BM = 256, BN = 256, NWAVES = 4, TM = 128, TN = 128, MT = 4, NT = 4, NSTAGE = 4;
  constexpr int GROUPS = (BM + BN) / 16;       // 16-row groups per stage (A rows first, then B rows)
  constexpr int NI = GROUPS / NWAVES;          // load instructions per wave per tile
  constexpr int STAGE_BYTES = (BM + BN) * 64;
  constexpr int KSTEPS = kBK32 / 16;
  static_assert(NSTAGE * STAGE_BYTES <= 160 * 1024 && KSTEPS == 2, "stages must fit in LDS");
  using Lds = LdsStages<STAGE_BYTES>;

  const int total = tiles_m * tiles_n * splits;
  const int lid = xcd_logical_id(blockIdx.x, total);
  if (lid < 0) return;
  int tile_m, tile_n, split;
  if (splits == 1 && tiles_m > kBandRows) {
    const int band_size = kBandRows * tiles_n;
    const int band = lid / band_size, rem = lid % band_size;
    const int rows_in_band = min(kBandRows, tiles_m - band * kBandRows);
    tile_m = band * kBandRows + rem % rows_in_band;
    tile_n = rem / rows_in_band;
    split = 0;
  } else {
    // split-major: the workgroups of one K range are neighbours, i.e. share an XCD, so the slice of the activation
    // matrix they all read enters that XCD's L2 once instead of every XCD streaming the whole matrix
    tile_m = lid % tiles_m;
    tile_n = (lid / tiles_m) % tiles_n;
    split = lid / (tiles_m * tiles_n);
  }
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  const int k_tiles = (p.k + kBK32 - 1) / kBK32;
  const int kt_begin = split * k_tiles_per_split;
  const int kt_end = min(kt_begin + k_tiles_per_split, k_tiles);
  const int nkt = kt_end - kt_begin;

  // Load instruction j of this wave fills row group g = 4 j + wave: rows 16 g .. 16 g + 15 of the stage.  This
  // lane's slot is (row 16 g + lane / 4, position lane % 4) and receives the row's chunk (lane % 4) ^ ((row >> 1) & 3).
  const int sw_chunk = (lane & 3) ^ ((lane >> 3) & 3);
  const int b_row0 = EPI == kEpiSwiGLU ? (n0 >> 6) * 32 : n0;
  uint32_t g_off[NI];
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    const int r = 16 * (NWAVES * j + wave) + (lane >> 2);
    if (r < BM) {
      int gm = m0 + r;
      gm = gm < p.m ? gm : p.m - 1;
      g_off[j] = ((uint32_t)(gm - m0) * (uint32_t)p.lda + sw_chunk * 8) * 2u;
    } else {
      int row;
      if constexpr (EPI == kEpiSwiGLU) {
        const int v = n0 + (r - BM);
        row = (v >> 6) * 32 + (v & 31);
      } else {
        row = n0 + (r - BM);
      }
      row = row < p.n ? row : p.n - 1;
      g_off[j] = ((uint32_t)(row - b_row0) * (uint32_t)p.k + sw_chunk * 8) * 2u;
    }
  }
  const size_t a_tile0 = (size_t)m0 * p.lda, b_tile0 = (size_t)b_row0 * p.k;

  int zero_below[NSTAGE];
  auto fetch = [&](auto stage_c, int idx) {
    constexpr int S = decltype(stage_c)::value;
    int kt = kt_begin + idx;
    kt = kt < kt_end - 1 ? kt : kt_end - 1;
    int k0 = kt * kBK32;
    const int k_last = p.k - kBK32;
    zero_below[S] = k0 > k_last ? k0 - k_last : 0;
    k0 = k0 > k_last ? k_last : k0;
    const char* abase = reinterpret_cast<const char*>(p.a + a_tile0 + k0);
    const char* w0base = reinterpret_cast<const char*>(p.w0 + b_tile0 + k0);
    const char* w1base = EPI == kEpiSwiGLU ? reinterpret_cast<const char*>(p.w1 + b_tile0 + k0) : w0base;
    char* stage = Lds::template get<S>();
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int g = NWAVES * j + wave;                          // uniform
      // gate/up: rows 32..63 of every 64 virtual columns are up rows, i.e. groups 2 and 3 of every four
      const char* base = g < BM / 16 ? abase : ((EPI == kEpiSwiGLU && ((g - BM / 16) & 2)) ? w1base : w0base);
      __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(base + g_off[j]),
                                       reinterpret_cast<uint32_t*>(stage + g * 1024), 16, 0, 0);
    }
  };
  auto patch_tail = [&](auto stage_c) {
    constexpr int S = decltype(stage_c)::value;
    if (zero_below[S] > 0 && sw_chunk * 8 < zero_below[S]) {
      char* stage = Lds::template get<S>();
      const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int j = 0; j < NI; ++j) *reinterpret_cast<u32x4*>(stage + (NWAVES * j + wave) * 1024 + lane * 16) = zero;
    }
  };

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // fragment reads: lane (row l % 32, k half l / 32) of step kk wants chunk 2 kk + l / 32 of its row
  const int frag_row = lane & 31;
  int frag_off[KSTEPS];
#pragma unroll
  for (int kk = 0; kk < KSTEPS; ++kk) frag_off[kk] = frag_row * 64 + (((2 * kk + (lane >> 5)) ^ ((frag_row >> 1) & 3)) * 16);

  e16x8 af[2][MT], bfr[2][NT];
  auto read_frags = [&](auto stage_c, int s, int kk) {
    constexpr int S = decltype(stage_c)::value;
    const char* la = Lds::template get<S>() + wm * TM * 64;
    const char* lb = Lds::template get<S>() + (BM + wn * TN) * 64;
    auto read_a = [&] {
#pragma unroll
      for (int i = 0; i < MT; ++i) af[s][i] = *reinterpret_cast<const e16x8*>(la + i * 32 * 64 + frag_off[kk]);
    };
    if constexpr (!A_HALF) read_a();
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const e16x8 w = *reinterpret_cast<const e16x8*>(lb + j * 32 * 64 + frag_off[kk]);
      bfr[s][j] = A_HALF ? __builtin_bit_cast(e16x8, bf16x8_to_half(w)) : w;
    }
    if constexpr (A_HALF) read_a();
  };
  auto mfmas = [&](int s) {
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j)
        acc[i][j] = A_HALF ? mfma_32x32x16_half(__builtin_bit_cast(h16x8, af[s][i]), __builtin_bit_cast(h16x8, bfr[s][j]), acc[i][j])
                           : mfma_32x32x16(af[s][i], bfr[s][j], acc[i][j]);
  };

  constexpr int NMFMA = MT * NT, NREAD = MT + NT;
  // Tile idx is in stage S and the fragments of its first MFMA step are in register set 0.  The stage read in the
  // previous step takes tile idx + 3, its loads spread over the first MFMA step; before the second (last) step all
  // loads but those of tiles idx + 2 and idx + 3 must have landed, and the barrier that publishes tile idx + 1 also
  // frees stage S.
  auto step = [&](auto stage_c, int idx) {
    constexpr int S = decltype(stage_c)::value;
    using Next = std::integral_constant<int, (S + 1) % NSTAGE>;
    fetch(std::integral_constant<int, (S + NSTAGE - 1) % NSTAGE>{}, idx + NSTAGE - 1);
    read_frags(stage_c, 1, 1);
    mfmas(0);
    sched_step<0, NMFMA, NREAD, NI>();
    __builtin_amdgcn_sched_barrier(0);
    wait_vmcnt<2 * NI>();
    patch_tail(Next{});
    pipeline_barrier();
    read_frags(Next{}, 0, 0);
    mfmas(1);
    sched_step<0, NMFMA, NREAD, 0>();
    __builtin_amdgcn_sched_barrier(0);
  };

  if (nkt > 0) {
    fetch(std::integral_constant<int, 0>{}, 0);
    fetch(std::integral_constant<int, 1>{}, 1);
    fetch(std::integral_constant<int, 2>{}, 2);
    wait_vmcnt<2 * NI>();
    patch_tail(std::integral_constant<int, 0>{});
    pipeline_barrier();
    read_frags(std::integral_constant<int, 0>{}, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    int i = 0;
    for (; i + NSTAGE <= nkt; i += NSTAGE) {
      step(std::integral_constant<int, 0>{}, i);
      step(std::integral_constant<int, 1>{}, i + 1);
      step(std::integral_constant<int, 2>{}, i + 2);
      step(std::integral_constant<int, 3>{}, i + 3);
    }
    if (i < nkt) step(std::integral_constant<int, 0>{}, i);
    if (i + 1 < nkt) step(std::integral_constant<int, 1>{}, i + 1);
    if (i + 2 < nkt) step(std::integral_constant<int, 2>{}, i + 2);
    wait_vmcnt<0>();   // nothing may still be writing LDS when the workgroup ends
  }
  tile_epilogue<EPI, SPLIT, MT, NT>(p, acc, m0 + wm * TM, n0 + wn * TN, nv, split, lane);
}

// 4-bit group-quantised weights (groups of 128) on 256 x 256 tiles, for more than 64 rows.
//
// The weights stay in their stored form all the way into LDS and are expanded in registers, per MFMA operand:
// a quarter of the bytes from memory and in LDS, no expanded copy.  The matrix instruction is the f16 one, so the
// activations must be IEEE half (a bfloat16 stage that keeps its projection inputs as half, or the
// half-precision library); a weight enters it as half((code - zero) * scale), formed as one fused multiply-add
// code * scale + (-zero * scale) on exact operands - the same eleven significant bits a bfloat16 weight converted
// to half would carry, three more than the expanded bfloat16 copy.  Scales are assumed to lie in half's normal
// range (2^-14 .. 65504), which per-group scales of weights of ordinary magnitude do.
//
// A K tile is 64 wide: 128 bytes per activation row (swizzled as in gemm_tile_kernel), 32 bytes of codes per
// weight row, and per weight row the two words that hold the scale and the zero point of the tile's group (a word
// holds two consecutive groups, i.e. serves four tiles; it travels with every tile so that each stage is
// self-contained and every pipeline step issues the same number of loads).  43 KB per stage, three stages.
// Within a tile, MFMA step s takes k = 32 h + 8 s .. + 7 from lane half h (not 16 s + 8 h): the four words a lane
// needs for the four steps of a tile are then one 16-byte LDS read of its row's codes.
//
// Expansion of one word (eight codes, k ascending from bit 0), per pair (k, k + 1): a byte permute puts the
// byte that holds both codes into either half, and-or isolates one code per half as the half number
// 1024 + code (bits or-ed into 0x6400), a packed subtraction removes the 1024 (exact), the packed fused
// multiply-add applies scale and zero point: 17 vector operations per 8 weights.  Mask and offset are held in
// registers: as literals they would split the and-or into two instructions.

__device__ __forceinline__ h16x8 expand_w4_word(uint32_t x, h16x2 scale2, h16x2 bias2, uint32_t mask, uint32_t base) {
  const uint32_t u = x >> 4;
  const h16x2 offset = {(h16)1024.f, (h16)1024.f};
  u32x4 o;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    // bytes (x.byte i, 0, u.byte i, 0): the low nibbles are codes 2 i and 2 i + 1
    const uint32_t t = __builtin_amdgcn_perm(u, x, 0x0c000c00u | (uint32_t)i | ((uint32_t)(4 + i) << 16));
    const h16x2 code = __builtin_bit_cast(h16x2, (t & mask) | base) - offset;
    o[i] = __builtin_bit_cast(uint32_t, __builtin_elementwise_fma(code, scale2, bias2));
  }
  return __builtin_bit_cast(h16x8, o);
}

template <int BM, int EPI, bool SPLIT>
__global__ __launch_bounds__(256, BM == 128 ? 2 : 1) void gemm_tile_w4_kernel(GemmArgs p, int nv, int tiles_m, int tiles_n,
                                                                             int splits, int k_tiles_per_split) {
  static_assert(BM == 128 || BM == 256, "tile rows");
  constexpr int BN = 256, NWAVES = 4, TM = BM / 2, TN = 128, MT = TM / 32, NT = 4, NSTAGE = 3;
  constexpr int A_BYTES = BM * 128, CODE_BYTES = BN * 32, QP_BYTES = BN * 4;
  constexpr int STAGE_BYTES = A_BYTES + CODE_BYTES + 2 * QP_BYTES;
  constexpr int NA = BM / 8 / NWAVES;          // activation loads per wave per tile (8 rows x 128 bytes each)
  constexpr int NB = BN / 32 / NWAVES;         // code loads per wave per tile (32 rows x 32 bytes each)
  constexpr int NI = NA + NB + 2;              // + this wave's 64 rows of scale words and of zero-point words
  static_assert(NSTAGE * STAGE_BYTES * (BM == 128 ? 2 : 1) <= 160 * 1024, "stages must fit in LDS");
  using Lds = LdsStages<STAGE_BYTES>;

  const int total = tiles_m * tiles_n * splits;
  const int lid = xcd_logical_id(blockIdx.x, total);
  if (lid < 0) return;
  int tile_m, tile_n, split;
  if (splits == 1 && tiles_m > kBandRows) {
    const int band_size = kBandRows * tiles_n;
    const int band = lid / band_size, rem = lid % band_size;
    const int rows_in_band = min(kBandRows, tiles_m - band * kBandRows);
    tile_m = band * kBandRows + rem % rows_in_band;
    tile_n = rem / rows_in_band;
    split = 0;
  } else {
    // split-major: the workgroups of one K range are neighbours, i.e. share an XCD, so the slice of the activation
    // matrix they all read enters that XCD's L2 once instead of every XCD streaming the whole matrix
    tile_m = lid % tiles_m;
    tile_n = (lid / tiles_m) % tiles_n;
    split = lid / (tiles_m * tiles_n);
  }
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  const int k_tiles = p.k / kBK;               // K is a multiple of 256 (launcher)
  const int kt_begin = split * k_tiles_per_split;
  const int kt_end = min(kt_begin + k_tiles_per_split, k_tiles);
  const int nkt = kt_end - kt_begin;

  // virtual column v of the tile's column space -> weight row (gate/up: 32 gate rows, then the 32 up rows of the
  // same features); rows past the matrix repeat its last row (never stored)
  auto row_of = [&](int v) {
    const int r = EPI == kEpiSwiGLU ? (v >> 6) * 32 + (v & 31) : v;
    return r < p.n ? r : p.n - 1;
  };
  const int b_row0 = EPI == kEpiSwiGLU ? (n0 >> 6) * 32 : n0;

  // activations: as in gemm_tile_kernel - load j of this wave fills rows 8 g .. 8 g + 7, g = 4 j + wave; slot
  // lane % 8 of row lane / 8 receives the row's chunk (lane % 8) ^ (lane / 8)
  uint32_t a_off[NA];
#pragma unroll
  for (int j = 0; j < NA; ++j) {
    int gm = m0 + 8 * (NWAVES * j + wave) + (lane >> 3);
    gm = gm < p.m ? gm : p.m - 1;
    a_off[j] = ((uint32_t)(gm - m0) * (uint32_t)p.lda + (uint32_t)(((lane & 7) ^ (lane >> 3)) * 8)) * 2u;
  }
  // codes: load j fills rows 32 g .. 32 g + 31, g = 4 j + wave; lane l carries bytes 16 (l % 2) .. + 15 of row l / 2.
  // g and wave have the same parity, so with gate/up a wave reads one of the two matrices only.
  const int row_bytes = p.k / 2;
  uint32_t c_off[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const int v = n0 + 32 * (NWAVES * j + wave) + (lane >> 1);
    c_off[j] = (uint32_t)(row_of(v) - b_row0) * (uint32_t)row_bytes + (uint32_t)((lane & 1) * 16);
  }
  const bool up_wave = EPI == kEpiSwiGLU && (wave & 1);
  const char* const codes_tile = reinterpret_cast<const char*>(up_wave ? p.q1.codes : p.q0.codes) + (size_t)b_row0 * row_bytes;
  // scale and zero-point words: lane l serves row 64 wave + l of the tile (gate/up: lanes 32-63 are up rows)
  const char* scale_lane;
  const char* zero_lane;
  {
    const int v = n0 + 64 * wave + lane;
    const bool up = EPI == kEpiSwiGLU && (v & 32);
    const size_t at = (size_t)row_of(v) * (p.k / 128) * 2;
    scale_lane = reinterpret_cast<const char*>(up ? p.q1.scales : p.q0.scales) + at;
    zero_lane = reinterpret_cast<const char*>(up ? p.q1.zeros : p.q0.zeros) + at;
  }
  const size_t a_tile0 = (size_t)m0 * p.lda;

  auto fetch = [&](auto stage_c, int idx) {
    constexpr int S = decltype(stage_c)::value;
    int kt = kt_begin + idx;
    kt = kt < kt_end - 1 ? kt : kt_end - 1;
    const char* abase = reinterpret_cast<const char*>(p.a + a_tile0 + kt * kBK);
    const char* cbase = codes_tile + kt * 32;
    char* stage = Lds::template get<S>();
#pragma unroll
    for (int j = 0; j < NA; ++j)
      __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(abase + a_off[j]),
                                       reinterpret_cast<uint32_t*>(stage + (NWAVES * j + wave) * 1024), 16, 0, 0);
#pragma unroll
    for (int j = 0; j < NB; ++j)
      __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(cbase + c_off[j]),
                                       reinterpret_cast<uint32_t*>(stage + A_BYTES + (NWAVES * j + wave) * 1024), 16, 0, 0);
    const int word = (kt >> 2) * 4;            // the word of groups 2 (kt / 4) and 2 (kt / 4) + 1
    __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(scale_lane + word),
                                     reinterpret_cast<uint32_t*>(stage + A_BYTES + CODE_BYTES + wave * 256), 4, 0, 0);
    __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(zero_lane + word),
                                     reinterpret_cast<uint32_t*>(stage + A_BYTES + CODE_BYTES + QP_BYTES + wave * 256), 4, 0, 0);
  };

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // fragment reads: lane (row l % 32, half h = l / 32) of step s wants chunk 4 h + s of its activation row, stored
  // at slot (4 h + s) ^ (l % 8), and word s of the 16 bytes of codes at 16 h of its weight row
  const int frag_row = lane & 31, half = lane >> 5;
  int frag_off[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) frag_off[s] = frag_row * 128 + (((4 * half + s) ^ (lane & 7)) * 16);
  const int code_off = A_BYTES + (wn * TN + frag_row) * 32 + half * 16;
  const int qp_off = A_BYTES + CODE_BYTES + (wn * TN + frag_row) * 4;

  uint32_t mask, base;
  asm("s_mov_b32 %0, 0x000F000F" : "=s"(mask));
  asm("v_mov_b32 %0, 0x64006400" : "=v"(base));

  e16x8 af[2][MT];
  h16x8 bfr[2][NT];
  u32x4 codes[NT];           // the current tile's codes of this lane's NT weight rows: word s feeds MFMA step s
  h16x2 scale2[NT], bias2[NT];
  auto read_a = [&](auto stage_c, int set, int s) {
    constexpr int S = decltype(stage_c)::value;
    const char* la = Lds::template get<S>() + wm * TM * 128;
#pragma unroll
    for (int i = 0; i < MT; ++i) af[set][i] = *reinterpret_cast<const e16x8*>(la + i * 32 * 128 + frag_off[s]);
  };
  // the codes, scales and zero points of the tile in stage S, whose K tile index is kt
  auto read_b = [&](auto stage_c, int kt) {
    constexpr int S = decltype(stage_c)::value;
    const char* st = Lds::template get<S>();
    const bool odd_group = (kt >> 1) & 1;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      codes[j] = *reinterpret_cast<const u32x4*>(st + code_off + j * 32 * 32);
      const uint32_t sw = *reinterpret_cast<const uint32_t*>(st + qp_off + j * 32 * 4);
      const uint32_t zw = *reinterpret_cast<const uint32_t*>(st + qp_off + QP_BYTES + j * 32 * 4);
      const float sc = odd_group ? e16_hi(sw) : e16_lo(sw);
      const float zp = odd_group ? e16_hi(zw) : e16_lo(zw);
      const h16 sh = (h16)sc, bh = (h16)(-zp * sc);
      scale2[j] = h16x2{sh, sh};
      bias2[j] = h16x2{bh, bh};
    }
  };
  auto expand = [&](int set, int s) {
#pragma unroll
    for (int j = 0; j < NT; ++j) bfr[set][j] = expand_w4_word(codes[j][s], scale2[j], bias2[j], mask, base);
  };
  auto mfmas = [&](int set) {
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j)
        acc[i][j] = mfma_32x32x16_half(__builtin_bit_cast(h16x8, af[set][i]), bfr[set][j], acc[i][j]);
  };

  // The pipeline of gemm_tile_kernel at three stages: tile idx is in stage S with the operands of its first MFMA
  // step in register set 0; tile idx + 2 is requested into the stage read in the previous step, its loads spread
  // over the first three MFMA steps; wait and barrier come before the last step, whose MFMAs cover the first reads
  // and the first expansion of tile idx + 1.
  constexpr int NMFMA = MT * NT;
  constexpr int L0 = NI / 3, L1 = (2 * NI) / 3 - NI / 3, L2 = NI - (2 * NI) / 3;
  auto step = [&](auto stage_c, int idx) {
    constexpr int S = decltype(stage_c)::value;
    using Next = std::integral_constant<int, (S + 1) % NSTAGE>;
    fetch(std::integral_constant<int, (S + NSTAGE - 1) % NSTAGE>{}, idx + NSTAGE - 1);
    read_a(stage_c, 1, 1);
    expand(1, 1);
    mfmas(0);
    sched_step<0, NMFMA, MT, L0>();
    read_a(stage_c, 0, 2);
    expand(0, 2);
    mfmas(1);
    sched_step<0, NMFMA, MT, L1>();
    read_a(stage_c, 1, 3);
    expand(1, 3);
    mfmas(0);
    sched_step<0, NMFMA, MT, L2>();
    __builtin_amdgcn_sched_barrier(0);
    wait_vmcnt<(NSTAGE - 2) * NI>();
    pipeline_barrier();
    read_a(Next{}, 0, 0);
    int kt_next = kt_begin + idx + 1;
    kt_next = kt_next < kt_end - 1 ? kt_next : kt_end - 1;
    read_b(Next{}, kt_next);
    expand(0, 0);
    mfmas(1);
    sched_step<0, NMFMA, MT + 3 * NT, 0>();
    __builtin_amdgcn_sched_barrier(0);
  };

  if (nkt > 0) {
    fetch(std::integral_constant<int, 0>{}, 0);
    fetch(std::integral_constant<int, 1>{}, 1);
    wait_vmcnt<NI>();
    pipeline_barrier();
    read_a(std::integral_constant<int, 0>{}, 0, 0);
    read_b(std::integral_constant<int, 0>{}, kt_begin);
    expand(0, 0);
    __builtin_amdgcn_sched_barrier(0);
    int i = 0;
    for (; i + NSTAGE <= nkt; i += NSTAGE) {
      step(std::integral_constant<int, 0>{}, i);
      step(std::integral_constant<int, 1>{}, i + 1);
      step(std::integral_constant<int, 2>{}, i + 2);
    }
    if (i < nkt) step(std::integral_constant<int, 0>{}, i);
    if (i + 1 < nkt) step(std::integral_constant<int, 1>{}, i + 1);
    wait_vmcnt<0>();   // nothing may still be writing LDS when the workgroup ends
  }

  tile_epilogue<EPI, SPLIT, MT, NT>(p, acc, m0 + wm * TM, n0 + wn * TN, nv, split, lane);
}

// ---- weights in operand order, read straight into registers ----
//
// A stage may keep a second copy of its projection weights (made once, at set-up, in the operand format of its
// matrix instructions), arranged so that a wave instruction of 64 x 16 bytes, fully coalesced, IS one MFMA column
// operand.  The tiled kernel below then takes its weights from memory straight into registers: no LDS fill and no
// LDS fragment reads for them - half of the LDS traffic of gemm_tile_kernel, whose matrix pipe waits on LDS - and,
// in a stage with half activations, no conversion either.
//
// Block (nb, ks) = rows 32 nb .. + 31, k 16 ks .. + 15 of a weight matrix is 1 KB in the order the 32x32x16 MFMA
// takes its column operand: lane l (16 bytes) holds row 32 nb + l % 32, k = 16 ks + 8 (l / 32) .. + 7.  Blocks are
// stored [nb][ks], so the operands a wave needs for consecutive MFMA steps of one 32-row strip are consecutive KBs.
__global__ __launch_bounds__(256) void arrange_weights_kernel(const e16* __restrict__ w, int n, int k, int to_half,
                                                             e16* __restrict__ out, size_t chunks) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= chunks) return;
  const int lane = (int)(idx & 63);
  const size_t blk = idx >> 6;
  const int ksteps = k / 16;
  const int nb = (int)(blk / ksteps), ks = (int)(blk % ksteps);
  const int row = nb * 32 + (lane & 31), k0 = ks * 16 + 8 * (lane >> 5);
  e16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
  if (row < n) v = load8(w + (size_t)row * k + k0);
  if (to_half) v = __builtin_bit_cast(e16x8, bf16x8_to_half(v));
  store8(out + idx * 8, v);
}

// s_waitcnt vmcnt(N) lgkmcnt(0)
template <int N> __device__ __forceinline__ void wait_vm_lgkm0() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0070);
}

// 256 x 256 output tile, 2 x 2 waves, K tiles of 64 (K a multiple of 256, a split a multiple of four K tiles).
// Activations go through LDS as in gemm_tile_kernel (four stages of 32 KB, direct loads, XOR swizzle); the weight
// operands of MFMA step s are requested eight steps (two K tiles) ahead, into a ring of eight register sets, each
// set refilled right behind the last MFMA that reads it.  Every wave loads the operands of its own 128 columns, so
// a block is read by the two waves that share those columns (the second read hits the CU's cache).
// Loads into registers, loads into LDS and fragment reads all run on explicit counts: the first and the last are
// written as assembly because the compiler counts a mixture of register loads and LDS-directed loads as unordered
// and answers it with full waits, and scheduling barriers keep every wait between the instructions it separates.
// HALF_OPS: the operands are IEEE half (f16 MFMA), else e16.
// BM: 256, or 128 for products of at most 128 rows (half the MFMA work per weight operand: bound by the weight stream).
// The tile of workgroup `block_id` of a launch of xcd_grid(tiles_m * tiles_n * splits) workgroups; STAGE_BYTES: size of
// an LDS stage (at least BM * 128; a kernel that runs tiles of both heights gives both the larger).
template <int BM, int STAGE_BYTES, int EPI, bool SPLIT, bool HALF_OPS>
__device__ __forceinline__ void arranged_tile(const GemmArgs& p, int nv, int tiles_m, int tiles_n, int splits, int k_tiles_per_split,
                                              int block_id) {
  static_assert(BM == 128 || BM == 256, "tile rows");
  static_assert(STAGE_BYTES >= BM * 128, "a stage holds the tile's activation rows");
  constexpr int BN = 256, NWAVES = 4, TM = BM / 2, TN = 128, MT = TM / 32, NT = 4, NSTAGE = 4, RING = 8;
  constexpr int NA = BM / 8 / NWAVES;            // activation loads per wave per tile, issued in three parts
  using Lds = LdsStages<STAGE_BYTES>;

  const int total = tiles_m * tiles_n * splits;
  const int lid = xcd_logical_id(block_id, total);
  if (lid < 0) return;
  int tile_m, tile_n, split;
  if (splits == 1 && tiles_m > kBandRows) {
    const int band_size = kBandRows * tiles_n;
    const int band = lid / band_size, rem = lid % band_size;
    const int rows_in_band = min(kBandRows, tiles_m - band * kBandRows);
    tile_m = band * kBandRows + rem % rows_in_band;
    tile_n = rem / rows_in_band;
    split = 0;
  } else {
    tile_m = lid % tiles_m;
    tile_n = (lid / tiles_m) % tiles_n;
    split = lid / (tiles_m * tiles_n);
  }
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  const int k_tiles = p.k / kBK;               // K is a multiple of 256, a split a multiple of four K tiles (launcher)
  const int kt_begin = split * k_tiles_per_split;
  const int kt_end = min(kt_begin + k_tiles_per_split, k_tiles);
  const int nkt = kt_end - kt_begin;
  const int ksteps = p.k / 16;

  uint32_t a_off[NA];
#pragma unroll
  for (int j = 0; j < NA; ++j) {
    int gm = m0 + 8 * (NWAVES * j + wave) + (lane >> 3);
    gm = gm < p.m ? gm : p.m - 1;
    a_off[j] = ((uint32_t)(gm - m0) * (uint32_t)p.lda + (uint32_t)(((lane & 7) ^ (lane >> 3)) * 8)) * 2u;
  }
  const size_t a_tile0 = (size_t)m0 * p.lda;

  // first block of this split of each of the wave's NT strips of 32 weight rows (wave-uniform addresses)
  uint64_t bbase[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int v0 = n0 + wn * TN + j * 32;                       // first virtual column of the strip
    const bool up = EPI == kEpiSwiGLU && (v0 & 32);
    int nb = EPI == kEpiSwiGLU ? (v0 >> 6) : (v0 >> 5);
    const int nb_last = (p.n + 31) / 32 - 1;
    nb = nb < nb_last ? nb : nb_last;                           // strips past the matrix repeat the last one (never stored)
    bbase[j] = reinterpret_cast<uint64_t>(up ? p.wa1 : p.wa0) + ((uint64_t)nb * ksteps + (uint64_t)kt_begin * 4) * 1024;
  }
  const uint32_t lane_off = lane * 16;

  // part `part` (0..2) of the loads of activation tile idx into stage S: load j belongs to part 3 j / NA
  // (3 + 3 + 2 instructions at 256 rows, 2 + 1 + 1 at 128)
  auto fetch_a = [&](auto stage_c, int idx, int part) {
    constexpr int S = decltype(stage_c)::value;
    int kt = kt_begin + idx;
    kt = kt < kt_end - 1 ? kt : kt_end - 1;
    const char* abase = reinterpret_cast<const char*>(p.a + a_tile0 + kt * kBK);
    char* stage = Lds::template get<S>();
#pragma unroll
    for (int j = 0; j < NA; ++j)
      if (3 * j / NA == part)
        __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(abase + a_off[j]),
                                         reinterpret_cast<uint32_t*>(stage + (NWAVES * j + wave) * 1024), 16, 0, 0);
  };

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int frag_row = lane & 31;
  int frag_off[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) frag_off[kk] = frag_row * 128 + (((2 * kk + (lane >> 5)) ^ (lane & 7)) * 16);

  u32x4 af[2][MT];
  u32x4 bq[RING][NT];      // weight operands of eight consecutive MFMA steps, a ring
  // Fragment reads and weight loads are written as assembly and waited for explicitly (see below).
  typedef __attribute__((address_space(3))) char* lds_ptr;
  const uint32_t lds_a[NSTAGE] = {(uint32_t)(uintptr_t)(lds_ptr)(Lds::template get<0>()), (uint32_t)(uintptr_t)(lds_ptr)(Lds::template get<1>()),
                                  (uint32_t)(uintptr_t)(lds_ptr)(Lds::template get<2>()), (uint32_t)(uintptr_t)(lds_ptr)(Lds::template get<3>())};
  auto read_a = [&](int stage, int set, int kk) {
    const uint32_t at = lds_a[stage] + wm * TM * 128 + frag_off[kk];
    static_assert(MT == 2 || MT == 4, "the fragment reads are written out");
    asm volatile("ds_read_b128 %0, %1" : "=v"(af[set][0]) : "v"(at));
    asm volatile("ds_read_b128 %0, %1 offset:4096" : "=v"(af[set][1]) : "v"(at));
    if constexpr (MT == 4) {
      asm volatile("ds_read_b128 %0, %1 offset:8192" : "=v"(af[set][2]) : "v"(at));
      asm volatile("ds_read_b128 %0, %1 offset:12288" : "=v"(af[set][3]) : "v"(at));
    }
  };
  // The operands of local MFMA step `step` (counted from the split's first) into ring slot `slot`; steps past the
  // split's last repeat it (loaded, never multiplied).  Written as assembly so that the wait for them is the
  // explicit one below: the compiler does not count loads into registers and loads into LDS on one counter and
  // answers their mixture with full waits.
  const int last_step = nkt * 4 - 1;
  auto load_b = [&](int slot, int j, int step) {
    step = step < last_step ? step : last_step;
    const uint64_t addr = bbase[j] + (uint64_t)step * 1024;
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(bq[slot][j]) : "v"(lane_off), "s"(addr));
  };
  // The MFMAs of one step, strip by strip; each strip's operand register is refilled, for the step eight steps
  // ahead, right behind the last MFMA that reads it.
  auto multiply = [&](int set, int slot, int refill_step) {
#pragma unroll
    for (int j = 0; j < NT; ++j) {
#pragma unroll
      for (int i = 0; i < MT; ++i)
        acc[i][j] = HALF_OPS ? mfma_32x32x16_half(__builtin_bit_cast(h16x8, af[set][i]), __builtin_bit_cast(h16x8, bq[slot][j]), acc[i][j])
                             : mfma_32x32x16(__builtin_bit_cast(e16x8, af[set][i]), __builtin_bit_cast(e16x8, bq[slot][j]), acc[i][j]);
      __builtin_amdgcn_sched_barrier(0);
      load_b(slot, j, refill_step);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Loads issued per MFMA step: a part of the next activation tile (3, 3, 2, 0 instructions at 256 rows) and the
  // step's NT weight operands, i.e. 7, 7, 6, 4; 24 per tile.  The weight operands of a step were requested eight steps
  // earlier, at the end of that step: when the step begins, everything but the loads of the seven steps in between
  // has to have landed (loads complete in order) - 48 minus the issuing step's own count.  That wait also covers the
  // activation tile, whose last part was requested earlier still.
  constexpr int kPart0 = (NA + 2) / 3, kPart1 = (2 * NA + 2) / 3 - kPart0, kPart2 = NA - kPart0 - kPart1;
  static_assert(kPart0 == (NA == 8 ? 3 : 2) && kPart1 == (NA == 8 ? 3 : 1) && kPart2 == (NA == 8 ? 2 : 1), "parts as fetch_a cuts them");
  constexpr int kTwoTiles = 2 * (NA + 4 * NT);
  constexpr int kWait0 = kTwoTiles - (kPart0 + NT), kWait1 = kTwoTiles - (kPart1 + NT), kWait2 = kTwoTiles - (kPart2 + NT),
                kWait3 = kTwoTiles - NT;
  // Tile idx (activations in stage S, weight operands in ring slots 4 P .. 4 P + 3); the activation tile idx + 3 goes
  // into the stage read in the previous tile; a step's weight operands are requested eight steps ahead, into the
  // slot the step's MFMAs have just read.
  auto tile_step = [&](auto stage_c, auto parity_c, int idx) {
    constexpr int S = decltype(stage_c)::value;
    constexpr int P = decltype(parity_c)::value;
    using Next = std::integral_constant<int, (S + 1) % NSTAGE>;
    using Fill = std::integral_constant<int, (S + NSTAGE - 1) % NSTAGE>;
    wait_vm_lgkm0<kWait0>();
    __builtin_amdgcn_sched_barrier(0);
    read_a(S, 1, 1);
    fetch_a(Fill{}, idx + NSTAGE - 1, 0);
    __builtin_amdgcn_sched_barrier(0);
    multiply(0, 4 * P + 0, 4 * (idx + 2) + 0);
    wait_vm_lgkm0<kWait1>();
    __builtin_amdgcn_sched_barrier(0);
    read_a(S, 0, 2);
    fetch_a(Fill{}, idx + NSTAGE - 1, 1);
    __builtin_amdgcn_sched_barrier(0);
    multiply(1, 4 * P + 1, 4 * (idx + 2) + 1);
    wait_vm_lgkm0<kWait2>();
    __builtin_amdgcn_sched_barrier(0);
    read_a(S, 1, 3);
    fetch_a(Fill{}, idx + NSTAGE - 1, 2);
    __builtin_amdgcn_sched_barrier(0);
    multiply(0, 4 * P + 2, 4 * (idx + 2) + 2);
    wait_vm_lgkm0<kWait3>();
    pipeline_barrier();
    __builtin_amdgcn_sched_barrier(0);
    read_a(Next::value, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    multiply(1, 4 * P + 3, 4 * (idx + 2) + 3);
  };

  if (nkt > 0) {
    // the order of requests the loop would have made in the two tiles before the first
    fetch_a(std::integral_constant<int, 0>{}, 0, 0);
    fetch_a(std::integral_constant<int, 0>{}, 0, 1);
    fetch_a(std::integral_constant<int, 0>{}, 0, 2);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        if (kk < 3) {
          if (t == 0) fetch_a(std::integral_constant<int, 1>{}, 1, kk);
          else fetch_a(std::integral_constant<int, 2>{}, 2, kk);
        }
#pragma unroll
        for (int j = 0; j < NT; ++j) load_b(4 * t + kk, j, 4 * t + kk);
      }
    }
    wait_vmcnt<kWait3>();
    pipeline_barrier();
    __builtin_amdgcn_sched_barrier(0);
    read_a(0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    // (a split holds a multiple of four K tiles - the launcher sees to it -, so the loop has no remainder: no branch
    // joins while assembly-issued loads are in flight, where the compiler might copy a register that has not landed)
    for (int i = 0; i + NSTAGE <= nkt; i += NSTAGE) {
      tile_step(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, i);
      tile_step(std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{}, i + 1);
      tile_step(std::integral_constant<int, 2>{}, std::integral_constant<int, 0>{}, i + 2);
      tile_step(std::integral_constant<int, 3>{}, std::integral_constant<int, 1>{}, i + 3);
    }
    wait_vmcnt<0>();   // nothing may still be writing LDS or registers when the workgroup ends
  }

  tile_epilogue<EPI, SPLIT, MT, NT>(p, acc, m0 + wm * TM, n0 + wn * TN, nv, split, lane);
}

template <int BM, int EPI, bool SPLIT, bool HALF_OPS>
__global__ __launch_bounds__(256) void gemm_tile_arranged_kernel(GemmArgs p, int nv, int tiles_m, int tiles_n, int splits,
                                                                 int k_tiles_per_split) {
  arranged_tile<BM, BM * 128, EPI, SPLIT, HALF_OPS>(p, nv, tiles_m, tiles_n, splits, k_tiles_per_split, blockIdx.x);
}

// A product whose last tile row holds at most 128 rows, without K splits, where that row would cost a whole round of
// workgroups of its own: the first head_blocks workgroups take the 256-row tiles of `head` (all full tile rows), the
// rest take `tail` (the remaining rows, with every pointer moved to its first row) on 128-row tiles, which run
// beside the last, partly filled round of the big tiles instead of after it.
template <int EPI, bool HALF_OPS>
__global__ __launch_bounds__(256) void gemm_tile_arranged_ragged_kernel(GemmArgs head, GemmArgs tail, int nv, int tiles_m_head,
                                                                        int tiles_n, int k_tiles, int head_blocks) {
  if ((int)blockIdx.x < head_blocks)
    arranged_tile<256, 256 * 128, EPI, false, HALF_OPS>(head, nv, tiles_m_head, tiles_n, 1, k_tiles, blockIdx.x);
  else
    arranged_tile<128, 256 * 128, EPI, false, HALF_OPS>(tail, nv, 1, tiles_n, 1, k_tiles, blockIdx.x - head_blocks);
}

// Adds the split-K partial sums (split 0 first) and applies the epilogue.  Four consecutive outputs per
// thread (n is a multiple of 8, so a group of four never straddles a row or a gate/up block of 32).
template <int EPI>
__global__ __launch_bounds__(256) void gemm_splitk_reduce_kernel(GemmArgs p, int nv, int splits) {
  const size_t idx = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  const size_t count = (size_t)p.m * p.n;
  if (idx >= count) return;
  const int m = (int)(idx / p.n), n = (int)(idx % p.n);
  const size_t plane = (size_t)p.m * nv;
  if constexpr (EPI == kEpiSwiGLU) {
    const int vg = (n >> 5) * 64 + (n & 31);
    const float* src = p.partial + (size_t)m * nv + vg;
    f32x4 g = {0.f, 0.f, 0.f, 0.f}, u = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < splits; ++s) {
      g += *reinterpret_cast<const f32x4*>(src + s * plane);
      u += *reinterpret_cast<const f32x4*>(src + s * plane + 32);
    }
    e16x4 hi, lo;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float val = silu_f(g[e]) * u[e];
      hi[e] = f32_to_act(val, p.out_half);
      lo[e] = f32_to_e16(val - e16_to_f32(hi[e]));     // only stored with a second plane, never with half
    }
    *reinterpret_cast<e16x4*>(p.out_e16 + (size_t)m * p.ldo + n) = hi;
    if (p.out_lo) *reinterpret_cast<e16x4*>(p.out_lo + (size_t)m * p.ldo + n) = lo;
  } else {
    const float* src = p.partial + (size_t)m * nv + n;
    f32x4 c = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < splits; ++s) c += *reinterpret_cast<const f32x4*>(src + s * plane);
    if constexpr (EPI == kEpiStoreF32) {
      *reinterpret_cast<f32x4*>(p.out_f32 + (size_t)m * p.ldo + n) = c;
    } else if constexpr (EPI == kEpiResidualF32) {
      *reinterpret_cast<f32x4*>(p.resid + idx) += c;
    } else {
      const f32x4 r = *reinterpret_cast<const f32x4*>(p.resid + idx) + c;
      e16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = f32_to_e16(r[e]);
      *reinterpret_cast<e16x4*>(p.out_e16 + (size_t)m * p.ldo + n) = o;
    }
  }
}

// Sum of the split-K partial results + residual add + (norm | e16 rounding), one workgroup
// per row.  The norm is an RMSNorm, or (ns.layer) a LayerNorm, which takes one more pass over the row for its mean.
template <bool NORM>
__global__ __launch_bounds__(1024) void reduce_residual_norm_kernel(const float* __restrict__ partial, int splits,
                                                                   int m_rows, int n, float* __restrict__ x,
                                                                   NormSpec ns,
                                                                   e16* __restrict__ out, e16* __restrict__ out_lo,
                                                                   int ldo, bool out_half) {
  __shared__ float wsum[16];
  __shared__ float wmean[16];
  const int row = blockIdx.x, tid = threadIdx.x;
  const int stride = blockDim.x * 4, nwaves = blockDim.x >> 6;
  const size_t plane = (size_t)m_rows * n;
  float* xr = x + (size_t)row * n;
  const float* pr = partial + (size_t)row * n;
  float ss = 0.f, sum = 0.f;
  for (int c = tid * 4; c < n; c += stride) {
    f32x4 v = *reinterpret_cast<const f32x4*>(xr + c);
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    for (int k = 0; k < splits; ++k) s += *reinterpret_cast<const f32x4*>(pr + k * plane + c);
    v += s;
    if constexpr (NORM) {
      *reinterpret_cast<f32x4*>(xr + c) = v;
      ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
      sum += v[0] + v[1] + v[2] + v[3];
    } else {
      e16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = f32_to_e16(v[e]);
      *reinterpret_cast<e16x4*>(out + (size_t)row * ldo + c) = o;
    }
  }
  if constexpr (NORM) {
    float mean = 0.f;
    if (ns.layer) {
      sum = wave_sum(sum);
      if ((tid & 63) == 0) wmean[tid >> 6] = sum;
      __syncthreads();
      float tot = 0.f;
      for (int w = 0; w < nwaves; ++w) tot += wmean[w];
      mean = tot / (float)n;
      ss = 0.f;
      for (int c = tid * 4; c < n; c += stride) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(xr + c);     // written by this same thread above
#pragma unroll
        for (int e = 0; e < 4; ++e) ss += (v[e] - mean) * (v[e] - mean);
      }
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) wsum[tid >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
    for (int w = 0; w < nwaves; ++w) tot += wsum[w];
    const float rs = 1.0f / sqrtf(tot / (float)n + ns.eps);
    for (int c = tid * 4; c < n; c += stride) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(xr + c);     // written by this same thread above
      const e16x4 g = *reinterpret_cast<const e16x4*>(ns.gain + c);
      f32x4 add = {0.f, 0.f, 0.f, 0.f};
      if (ns.bias) {
        const e16x4 b = *reinterpret_cast<const e16x4*>(ns.bias + c);
#pragma unroll
        for (int e = 0; e < 4; ++e) add[e] = e16_to_f32(b[e]);
      }
      e16x4 o, lo;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float val = (v[e] - mean) * rs * e16_to_f32(g[e]);
        if (ns.bias) val += add[e];
        o[e] = f32_to_act(val, out_half);
        lo[e] = f32_to_act(val - act_to_f32(o[e], out_half), out_half);
      }
      *reinterpret_cast<e16x4*>(out + (size_t)row * ldo + c) = o;
      if (out_lo) *reinterpret_cast<e16x4*>(out_lo + (size_t)row * ldo + c) = lo;
    }
  }
}

// Weight-streaming GEMM for micro-batches of at most 64 rows (decode): the projection is bound by
// reading W once from HBM, so the kernel is built around that stream.
//
// K is cut into slices of 1024; a workgroup keeps one slice for its whole life and walks over groups
// of 16 weight rows.  A stage is 16 weight rows x 2 KB, filled by global_load_lds instructions that
// each fetch 1 KB of ONE row (the longest run a wave instruction can ask for, and what the memory
// system streams fastest); four stages, three in flight (96 KB per CU).  Chunk c (16 bytes) of row r is
// stored at position c ^ (r & 7) of its 1 KB piece - done by choosing which chunk each lane fetches -
// so that the 128-bit fragment reads of 16 rows at one k are conflict free.
//
// Eight waves with two roles.  Waves 4-7 only issue the loads: a wave that has filled the address
// unit's queue stalls at its next load until older ones have drained, and a wave that also had to
// multiply would do so only after that stall - load time and multiply time would add up.  Waves 0-3
// multiply: wave w holds the activations of rows 16w..16w+15 for the whole slice in registers as MFMA
// operands (loaded once), multiplies every stage with them (16x16x32 MFMA, weights as the row operand)
// and writes its 16 x 16 block of the slice's partial sums; the split-K reduction kernels add the
// slices in order and apply the epilogue.  One barrier per stage joins the two roles.
constexpr int kSkinnyKS = 1024;     // K elements per slice
constexpr int kSkinnyRows = 16;     // weight rows per stage
constexpr int kSkinnyStages = 4;

//
// A_HALF (bfloat16 library, half activations): the activations are IEEE half bits; every weight fragment is turned
// into half in registers after its LDS read (exact) and the f16 instruction multiplies.  The conversion is vector
// work of the multiplying waves only and stays far below the time the stage's bytes take to arrive.
template <bool A_HALF>
__global__ __launch_bounds__(512) void gemm_skinny_kernel(GemmArgs p, int nv, int splits, int groups, int swiglu) {
  constexpr int KS = kSkinnyKS, ROWS = kSkinnyRows, NST = kSkinnyStages;
  constexpr int STAGE_BYTES = ROWS * KS * 2;
  constexpr int NI = ROWS * 2 / 4;             // load instructions per loading wave per stage (two 1 KB pieces per row)
  constexpr int STEPS = KS / 32;               // MFMA steps per stage
  using Lds = LdsStages<STAGE_BYTES>;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nwg = gridDim.x;
  const int split = blockIdx.x % splits, slot = blockIdx.x / splits;
  const int peers = (nwg - split + splits - 1) / splits;         // workgroups that share this slice
  const int g_begin = (int)((long)groups * slot / peers);
  const int g_end = (int)((long)groups * (slot + 1) / peers);
  const int n_units = g_end - g_begin;
  const int n_steps = (n_units + NST - 1) / NST * NST;           // both roles run the same number of barriers
  const int kbase = split * KS;
  if (n_units <= 0) return;

  if (wave >= 4) {
    // ---- loading waves ----
    const int lw = wave - 4;
    // byte offset inside a row of the chunk this lane fetches: position `lane` of a 1 KB piece receives
    // chunk lane ^ (row & 7)
    uint32_t koff[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int idx = NI * lw + i, row = idx >> 1, half = idx & 1;
      int k = kbase + 8 * (64 * half + (lane ^ (row & 7)));
      k = k < p.k - 8 ? k : p.k - 8;           // past the end of K: any finite value, the activations there are zero
      koff[i] = (uint32_t)k * 2u;
    }
    // Every pipeline step issues the same number of loads, so that the wait count below holds without
    // control flow around the loads (which the compiler would answer with full waits).  A fetch past the
    // workgroup's last unit degenerates to one cache line: every lane reads the start of a row.
    auto fetch = [&](auto stage_c, int unit) {
      constexpr int S = decltype(stage_c)::value;
      const bool real = unit < n_units;
      unit = real ? unit : n_units - 1;
      const int v0 = (g_begin + unit) * ROWS;    // first (virtual) row of the group
      // SwiGLU: 32 gate rows, then the 32 up rows of the same features
      const e16* w = (swiglu && (v0 & 32)) ? p.w1 : p.w0;
      const int r0 = swiglu ? (v0 >> 6) * 32 + (v0 & 31) : v0;
      const int last = p.n - 1 - r0;              // rows past the matrix repeat its last row (never stored)
      char* stage = Lds::template get<S>();
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int idx = NI * lw + i;
        int row = idx >> 1;
        row = row < last ? row : last;
        const char* base = reinterpret_cast<const char*>(w + (size_t)(r0 + row) * p.k);
        __builtin_amdgcn_global_load_lds(reinterpret_cast<const uint32_t*>(base + (real ? koff[i] : 0u)),
                                         reinterpret_cast<uint32_t*>(stage + idx * 1024), 16, 0, 2);   // aux 2 = nontemporal
      }
    };
    // Step u: after the wait only the 2 * NI loads of the two younger stages can still be in flight, so
    // this wave's part of stage u % 4 has landed; after the barrier everybody's has, and the multiplying
    // waves are done with stage (u - 1) % 4, which is refilled next.
    auto step = [&](auto stage_c, int u) {
      constexpr int S = decltype(stage_c)::value;
      wait_vmcnt<2 * NI>();
      pipeline_barrier();
      fetch(std::integral_constant<int, (S + NST - 1) % NST>{}, u + NST - 1);
    };
    fetch(std::integral_constant<int, 0>{}, 0);
    fetch(std::integral_constant<int, 1>{}, 1);
    fetch(std::integral_constant<int, 2>{}, 2);
    for (int u = 0; u < n_steps; u += NST) {
      step(std::integral_constant<int, 0>{}, u);
      step(std::integral_constant<int, 1>{}, u + 1);
      step(std::integral_constant<int, 2>{}, u + 2);
      step(std::integral_constant<int, 3>{}, u + 3);
    }
    wait_vmcnt<0>();   // nothing may still be writing LDS when the workgroup ends
    return;
  }

  // ---- multiplying waves ----
  // activations: lane (row l%16, quarter l/16) holds k = 32 s + 8 (l/16) .. +7 of step s
  const int a_row = 16 * wave + (lane & 15), quarter = lane >> 4;
  const bool wave_active = 16 * wave < p.m;
  e16x8 act[STEPS];
  {
    const int m = a_row < p.m ? a_row : p.m - 1;
    const e16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      const int k = kbase + 32 * s + 8 * quarter;
      act[s] = wave_active && k < p.k ? load8(p.a + (size_t)m * p.lda + k) : zero;
    }
  }

  // fragment of step s: lane (row n = l%16, quarter q) wants chunk 4s + q of row n, stored at position
  // (4s + q) ^ (n & 7) = 4 (s ^ ((n >> 2) & 1)) + (q ^ (n & 3)) of the piece s / 16 of the row
  const int n_in = lane & 15;
  const int frag_base = n_in * 2048 + ((quarter ^ (n_in & 3)) * 16);
  const int flip = (n_in >> 2) & 1;
  const int frag_even = frag_base + flip * 64, frag_odd = frag_base - flip * 64;

  auto compute = [&](auto stage_c, int unit) {
    constexpr int S = decltype(stage_c)::value;
    pipeline_barrier();
    if (!wave_active || unit >= n_units) return;
    const char* stage = Lds::template get<S>();
    f32x4 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      const int off = (s >> 4) * 1024 + (s & 15) * 64 + ((s & 1) ? frag_odd : frag_even);
      const e16x8 wf = *reinterpret_cast<const e16x8*>(stage + off);
      if constexpr (A_HALF)
        acc[s & 3] = mfma_16x16x32_half(bf16x8_to_half(wf), __builtin_bit_cast(h16x8, act[s]), acc[s & 3]);
      else
        acc[s & 3] = mfma_16x16x32(wf, act[s], acc[s & 3]);
    }
    // eight fragment reads run ahead of the MFMA that consumes the oldest of them
    __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
    for (int s = 0; s < STEPS - 8; ++s) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
    const f32x4 sum = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    // accumulator register r of lane l is C[weight row 4 (l/16) + r][activation row l%16]
    const int v = (g_begin + unit) * ROWS + 4 * quarter;
    if (a_row < p.m && v < nv) *reinterpret_cast<f32x4*>(p.partial + ((size_t)split * p.m + a_row) * nv + v) = sum;
  };
  for (int u = 0; u < n_steps; u += NST) {
    compute(std::integral_constant<int, 0>{}, u);
    compute(std::integral_constant<int, 1>{}, u + 1);
    compute(std::integral_constant<int, 2>{}, u + 2);
    compute(std::integral_constant<int, 3>{}, u + 3);
  }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int NSTAGE, int EPI, bool SPLIT_A, bool A_HALF = false>
hipError_t launch_tile(const GemmArgs& a, const GemmPlan& plan, hipStream_t stream) {
  const int tiles_m = (a.m + BM - 1) / BM;
  const int tiles_n = (plan.nv + BN - 1) / BN;
  const int total = tiles_m * tiles_n * plan.splits;
  dim3 grid(xcd_grid(total)), block(WAVES_M * WAVES_N * 64);
  if (plan.splits > 1) {
    hipLaunchKernelGGL((gemm_tile_kernel<BM, BN, WAVES_M, WAVES_N, NSTAGE, EPI, true, SPLIT_A, A_HALF>), grid, block, 0, stream, a,
                       plan.nv, tiles_m, tiles_n, plan.splits, plan.k_tiles_per_split);
  } else {
    hipLaunchKernelGGL((gemm_tile_kernel<BM, BN, WAVES_M, WAVES_N, NSTAGE, EPI, false, SPLIT_A, A_HALF>), grid, block, 0, stream,
                       a, plan.nv, tiles_m, tiles_n, 1, plan.k_tiles_per_split);
  }
  return hipGetLastError();
}

template <int EPI, bool A_HALF>
hipError_t launch_tile32(const GemmArgs& a, const GemmPlan& plan, hipStream_t stream) {
  const int tiles_m = (a.m + 255) / 256;
  const int tiles_n = (plan.nv + 255) / 256;
  const int total = tiles_m * tiles_n * plan.splits;
  dim3 grid(xcd_grid(total)), block(256);
  // K tiles of 32: a split takes twice the plan's count of 64-wide K tiles
  if (plan.splits > 1)
    hipLaunchKernelGGL((gemm_tile32_kernel<EPI, true, A_HALF>), grid, block, 0, stream, a, plan.nv, tiles_m, tiles_n, plan.splits,
                       2 * plan.k_tiles_per_split);
  else
    hipLaunchKernelGGL((gemm_tile32_kernel<EPI, false, A_HALF>), grid, block, 0, stream, a, plan.nv, tiles_m, tiles_n, 1,
                       2 * plan.k_tiles_per_split);
  return hipGetLastError();
}

template <int BM, int EPI>
hipError_t launch_tile_w4(const GemmArgs& a, const GemmPlan& plan, hipStream_t stream) {
  const int tiles_m = (a.m + BM - 1) / BM;
  const int tiles_n = (plan.nv + 255) / 256;
  const int total = tiles_m * tiles_n * plan.splits;
  dim3 grid(xcd_grid(total)), block(256);
  if (plan.splits > 1)
    hipLaunchKernelGGL((gemm_tile_w4_kernel<BM, EPI, true>), grid, block, 0, stream, a, plan.nv, tiles_m, tiles_n, plan.splits,
                       plan.k_tiles_per_split);
  else
    hipLaunchKernelGGL((gemm_tile_w4_kernel<BM, EPI, false>), grid, block, 0, stream, a, plan.nv, tiles_m, tiles_n, 1,
                       plan.k_tiles_per_split);
  return hipGetLastError();
}
template <int EPI>
hipError_t launch_tile_w4(const GemmArgs& a, const GemmPlan& plan, hipStream_t stream) {
  return plan.tile == kTileW4x128 ? launch_tile_w4<128, EPI>(a, plan, stream) : launch_tile_w4<256, EPI>(a, plan, stream);
}

template <int BM, int EPI>
hipError_t launch_tile_arranged(const GemmArgs& a, const GemmPlan& plan, hipStream_t stream) {
  const int tiles_m = (a.m + BM - 1) / BM;
  const int tiles_n = (plan.nv + 255) / 256;
  const int total = tiles_m * tiles_n * plan.splits;
  dim3 grid(xcd_grid(total)), block(256);
  if (a.a_half) {
#ifdef MOLINK_F16
    return hipErrorInvalidValue;   // the element type is half already
#else
    if (plan.splits > 1)
      hipLaunchKernelGGL((gemm_tile_arranged_kernel<BM, EPI, true, true>), grid, block, 0, stream, a, plan.nv, tiles_m, tiles_n,
                         plan.splits, plan.k_tiles_per_split);
    else
      hipLaunchKernelGGL((gemm_tile_arranged_kernel<BM, EPI, false, true>), grid, block, 0, stream, a, plan.nv, tiles_m, tiles_n, 1,
                         plan.k_tiles_per_split);
    return hipGetLastError();
#endif
  }
  if (plan.splits > 1)
    hipLaunchKernelGGL((gemm_tile_arranged_kernel<BM, EPI, true, false>), grid, block, 0, stream, a, plan.nv, tiles_m, tiles_n, plan.splits,
                       plan.k_tiles_per_split);
  else
    hipLaunchKernelGGL((gemm_tile_arranged_kernel<BM, EPI, false, false>), grid, block, 0, stream, a, plan.nv, tiles_m, tiles_n, 1,
                       plan.k_tiles_per_split);
  return hipGetLastError();
}
template <int EPI>
hipError_t launch_tile_arranged(const GemmArgs& a, const GemmPlan& plan, hipStream_t stream) {
  return plan.tile == kTileArranged128 ? launch_tile_arranged<128, EPI>(a, plan, stream) : launch_tile_arranged<256, EPI>(a, plan, stream);
}

template <int EPI>
hipError_t launch_epi(const GemmArgs& a, const GemmPlan& plan, hipStream_t stream) {
  if (a.a_lo) {
    // two activation planes: only the tiles whose stages still fit in LDS
    if (a.a_half) {
#ifdef MOLINK_F16
      return hipErrorInvalidValue;
#else
      if (plan.tile == kTile128x128) return launch_tile<128, 128, 2, 2, 3, EPI, true, true>(a, plan, stream);
      if (plan.tile == kTile64x128) return launch_tile<64, 128, 2, 2, 2, EPI, true, true>(a, plan, stream);
      return hipErrorInvalidValue;
#endif
    }
    if (plan.tile == kTile128x128) return launch_tile<128, 128, 2, 2, 3, EPI, true>(a, plan, stream);
    if (plan.tile == kTile64x128) return launch_tile<64, 128, 2, 2, 2, EPI, true>(a, plan, stream);
    return hipErrorInvalidValue;
  }
  if (a.a_half) {
#ifdef MOLINK_F16
    return hipErrorInvalidValue;   // the element type is half already
#else
    if (plan.tile == kTile64x128) return launch_tile<64, 128, 2, 2, 2, EPI, false, true>(a, plan, stream);
    switch (plan.tile) {
      // (the 256x256 tile has no registers left for the converted fragments: its plans run on 128x256 tiles,
      // twice as many workgroups over the same splits)
      // The 128x256 tile is cut 1 x 4 among the waves here (each wave all 128 rows of a 64-column strip): every
      // weight fragment is then converted by one wave instead of two, half the conversion work per MFMA.
      case kTile256x256: return launch_tile32<EPI, true>(a, plan, stream);
      case kTile256x128: return launch_tile<256, 128, 2, 2, 3, EPI, false, true>(a, plan, stream);
      case kTile128x128: return launch_tile<128, 128, 2, 2, 2, EPI, false, true>(a, plan, stream);
      case kTile128x256: return launch_tile<128, 256, 1, 4, 3, EPI, false, true>(a, plan, stream);
      default: return hipErrorInvalidValue;
    }
#endif
  }
  switch (plan.tile) {
    case kTile64x128: return launch_tile<64, 128, 2, 2, 2, EPI, false>(a, plan, stream);
    case kTile256x256: return launch_tile32<EPI, false>(a, plan, stream);
    case kTile256x128: return launch_tile<256, 128, 2, 2, 3, EPI, false>(a, plan, stream);
    case kTile128x128: return launch_tile<128, 128, 2, 2, 2, EPI, false>(a, plan, stream);
    case kTile128x256: return launch_tile<128, 256, 2, 2, 3, EPI, false>(a, plan, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

GemmPlan plan_gemm(int m, int n, int k, GemmEpilogue epi, int num_cus, bool split_a, GemmFewRows few_rows, bool arranged) {
  GemmPlan plan;
  plan.nv = epi == kEpiSwiGLU ? ((n + 31) / 32) * 64 : n;
  if (arranged && arranged_weights_supported(k) && !split_a && m > 64) {
    // The kernel that reads the weights in operand order: 256-row tiles (128-row ones up to 128 rows), 256 columns,
    // one workgroup per CU, a split a multiple of four K tiles.  Measured against the tiles below on the shapes of
    // the 7B, 70B and Qwen2 stages at 128 to 2176 rows it is 4 to 32 % ahead everywhere except where few tiles meet
    // many short splits (256 rows, 32 - 40 tiles, 6 - 8 splits of 16 - 24 K tiles: 7 - 17 % behind; 192 rows, 8
    // splits of 56: 7 % behind; 128 rows, 6 - 8 splits: level), hence the rule.
    // (Two rows of 128-row tiles where the 256-row tile is turned down at 256 rows - half the splits - measured
    // level or ahead alone, 53 -> 48 us on 8192 x 8192, but level or behind inside the 70B-shaped stage, 58 -> 65 us
    // on its q/k/v projection: not taken.)
    const int k_tiles = k / kBK;
    {
      const int bm = m <= 128 ? 128 : 256;
      const int tiles = ((m + bm - 1) / bm) * ((plan.nv + 255) / 256);
      int splits = 1;
      if (tiles * 2 <= num_cus) {
        splits = num_cus / tiles;
        const int max_by_k = k_tiles / 4 > 0 ? k_tiles / 4 : 1;
        if (splits > max_by_k) splits = max_by_k;
        if (splits > 16) splits = 16;
      }
      const int per = ((k_tiles + splits - 1) / splits + 3) / 4 * 4;
      splits = (k_tiles + per - 1) / per;
      if (splits <= 4 || (bm == 256 && per >= 48 && m > 192)) {
        plan.tile = bm == 128 ? kTileArranged128 : kTileArranged;
        plan.k_tiles_per_split = per;
        plan.splits = splits;
        plan.partials = splits > 1;
        return plan;
      }
    }
  }
  const bool wide = k >= 8192 && (long)plan.nv * k >= (64L << 20);
  const bool streaming = few_rows == kFewRowsStreaming || (few_rows == kFewRowsByShape && !wide);
  const int k_tiles = (k + kBK - 1) / kBK;
  struct Cand { int tile, bm, bn, wg_per_cu; float eff; };
  // measured relative efficiency of the tile shapes and how many workgroups of each fit on a CU (LDS)
  static const Cand cands[] = {{kTile128x256, 128, 256, 1, 1.0f}, {kTile256x128, 256, 128, 1, 0.99f},
                               {kTile256x256, 256, 256, 1, 1.08f}, {kTile128x128, 128, 128, 2, 0.86f}};
  if (m <= 64 && !split_a && streaming) {
    plan.tile = kTileSkinny;
    plan.splits = (k + kSkinnyKS - 1) / kSkinnyKS;
    plan.k_tiles_per_split = kSkinnyKS / kBK;
    plan.partials = true;
    return plan;
  }
  float best = 0.f;
  int bm = m <= 64 ? 64 : 128, bn = 128, wg_per_cu = m <= 64 ? 2 : (split_a ? 1 : 2);
  plan.tile = m <= 64 ? kTile64x128 : kTile128x128;
  for (const Cand& c : cands) {
    if (m <= 64) break;
    if (split_a && c.tile != kTile128x128) continue;   // with two activation planes only this tile's stages fit
    const int per_cu = split_a ? 1 : c.wg_per_cu;
    const long tiles = (long)((m + c.bm - 1) / c.bm) * ((plan.nv + c.bn - 1) / c.bn);
    const long slots = (long)num_cus * per_cu;
    const long rounds = (tiles + slots - 1) / slots;
    const float cost = (float)rounds * c.bm * c.bn * per_cu / c.eff;
    if (best == 0.f || cost < best) {
      best = cost;
      plan.tile = c.tile;
      bm = c.bm; bn = c.bn; wg_per_cu = per_cu;
    }
  }
  // One round of one workgroup per CU leaves a tile's prologue and epilogue exposed: nothing else runs on the CU
  // meanwhile.  If the 128x128 tiles (two per CU) also fit in one round they overlap each other's ends
  // (measured on 2176 x 3584 x 3584: 75 us against 87).  Only for short K: with 296 K tiles instead of 56 the ends
  // no longer count and the larger tile's lower traffic per flop wins again (277 us against 295).
  if (!split_a && m > 64 && wg_per_cu == 1 && best > 0.f && k_tiles <= 96) {
    const long t_big = (long)((m + bm - 1) / bm) * ((plan.nv + bn - 1) / bn);
    const long t_small = (long)((m + 127) / 128) * ((plan.nv + 127) / 128);
    if (t_big <= num_cus && t_big * 2 > num_cus && t_small <= 2L * num_cus) {
      plan.tile = kTile128x128;
      bm = 128; bn = 128; wg_per_cu = 2;
    }
  }
  const int tiles = ((m + bm - 1) / bm) * ((plan.nv + bn - 1) / bn);
  int splits = 1;
  if (tiles * 2 <= num_cus * wg_per_cu) {
    // as many splits as still fit one round of workgroups: one more would start a second, nearly empty round
    // that takes as long as the first
    splits = (num_cus * wg_per_cu) / tiles;
    const int max_by_k = k_tiles / 4 > 0 ? k_tiles / 4 : 1;   // at least 4 K tiles per split
    if (splits > max_by_k) splits = max_by_k;
    if (splits > 16) splits = 16;
  }
  plan.k_tiles_per_split = (k_tiles + splits - 1) / splits;
  plan.splits = (k_tiles + plan.k_tiles_per_split - 1) / plan.k_tiles_per_split;
  plan.partials = plan.splits > 1;
  return plan;
}

// Which of the two 4-bit tile heights a product of m rows runs on.  Up to 128 rows the 128-row tiles (two workgroups
// per CU) are ahead - 70B-shaped stage, 128 tokens: 16.6 against 17.8 ms per micro-batch; at 256 and 512 rows the
// 256-row tiles are (26.9 against 28.6 and 45.7 against 49.2 ms): every workgroup expands the codes of its own
// columns, so two tile rows expand everything twice.
static bool w4_tile_rows_128(int m) { return m <= 128; }

bool tile_w4_supports(int m, int k, int group, bool two_planes, bool operands_half) {
  return m > 64 && operands_half && !two_planes && group == 128 && k >= 256 && k % 256 == 0;
}

GemmPlan plan_gemm_w4_tile(int m, int n, int k, GemmEpilogue epi, int num_cus) {
  GemmPlan plan;
  plan.nv = epi == kEpiSwiGLU ? ((n + 31) / 32) * 64 : n;
  const int k_tiles = k / kBK;
  const int tiles_n = (plan.nv + 255) / 256;
  // 128-row tiles run two workgroups per CU, 256-row tiles one
  const bool rows128 = w4_tile_rows_128(m);
  plan.tile = rows128 ? kTileW4x128 : kTileW4;
  const int tiles = (rows128 ? (m + 127) / 128 : (m + 255) / 256) * tiles_n;
  const int slots = rows128 ? 2 * num_cus : num_cus;
  int splits = 1;
  if (tiles * 2 <= slots) {
    // as in plan_gemm: as many splits as fit one round of workgroups, at least 4 K tiles each, at most 16
    splits = slots / tiles;
    const int max_by_k = k_tiles / 4 > 0 ? k_tiles / 4 : 1;
    if (splits > max_by_k) splits = max_by_k;
    if (splits > 16) splits = 16;
  }
  plan.k_tiles_per_split = (k_tiles + splits - 1) / splits;
  plan.splits = (k_tiles + plan.k_tiles_per_split - 1) / plan.k_tiles_per_split;
  plan.partials = plan.splits > 1;
  return plan;
}

size_t gemm_partial_floats_w4_tile(int max_m, int n, int k, GemmEpilogue epi, int num_cus) {
  // The split count depends on the number of tile rows only, so the largest m of every such count is the worst:
  // the multiples of 128 below max_m, and max_m itself.
  size_t worst = 0;
  for (int top = 128;; top += 128) {
    const int m = top < max_m ? top : max_m;
    if (m <= 64) break;
    const GemmPlan p = plan_gemm_w4_tile(m, n, k, epi, num_cus);
    if (p.partials) {
      const size_t need = (size_t)p.splits * m * p.nv;
      if (need > worst) worst = need;
    }
    if (top >= max_m) break;
  }
  return worst;
}

bool arranged_weights_supported(int k) { return k >= 256 && k % 256 == 0; }

size_t arranged_weights_elems(int n, int k) { return (size_t)((n + 31) / 32) * 32 * (size_t)k; }

hipError_t launch_arrange_weights(const e16* w, int n, int k, bool to_half, e16* out, hipStream_t stream) {
  if (!arranged_weights_supported(k)) return hipErrorInvalidValue;
#ifdef MOLINK_F16
  if (to_half) return hipErrorInvalidValue;      // the element type is half already
#endif
  const size_t chunks = arranged_weights_elems(n, k) / 8;
  hipLaunchKernelGGL(arrange_weights_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, stream, w, n, k, to_half ? 1 : 0, out,
                     chunks);
  return hipGetLastError();
}

size_t gemm_partial_floats(int max_m, int n, int k, GemmEpilogue epi, int num_cus, bool split_a, bool arranged) {
  // The scratch of a shape is splits * m * nv; the split count falls as m grows, so every m at which the
  // plan can change (multiples of 64) is tried.
  size_t worst = 0;
  for (int m = 1; m <= max_m; m = (m < 64 ? 64 : m + 64)) {
    for (GemmFewRows few : {kFewRowsStreaming, kFewRowsTiles}) {
      if (m > 64 && few == kFewRowsTiles) continue;            // above 64 rows there is one plan
      const GemmPlan p = plan_gemm(m, n, k, epi, num_cus, split_a, few, arranged);
      if (p.partials) {
        const int mm = m < 64 ? (max_m < 64 ? max_m : 64) : m;   // the plan of m = 1 holds up to 64 rows
        const size_t need = (size_t)p.splits * mm * p.nv;
        if (need > worst) worst = need;
      }
    }
  }
  const GemmPlan p = plan_gemm(max_m, n, k, epi, num_cus, split_a, kFewRowsByShape, arranged);
  if (p.partials) {
    const size_t need = (size_t)p.splits * max_m * p.nv;
    if (need > worst) worst = need;
  }
  return worst;
}

hipError_t launch_gemm_main(const GemmArgs& a, GemmEpilogue epi, const GemmPlan& plan, hipStream_t stream) {
  if (plan.tile == kTileSkinny) {
    if (a.m > 64 || a.a_lo) return hipErrorInvalidValue;
    if (a.q0.codes) return launch_gemm_skinny_w4(a, plan.nv, plan.splits, epi == kEpiSwiGLU ? 1 : 0, stream);
    const int groups = (plan.nv + kSkinnyRows - 1) / kSkinnyRows;
    const long units = (long)groups * plan.splits;
    const int cus = 256;
    const int nwg = units < cus ? (int)units : (cus > plan.splits ? cus : plan.splits);
    dim3 grid(nwg);
    if (a.a_half) {
#ifdef MOLINK_F16
      return hipErrorInvalidValue;                 // the element type is half already
#else
      hipLaunchKernelGGL(gemm_skinny_kernel<true>, grid, dim3(512), 0, stream, a, plan.nv, plan.splits, groups,
                         epi == kEpiSwiGLU ? 1 : 0);
      return hipGetLastError();
#endif
    }
    hipLaunchKernelGGL(gemm_skinny_kernel<false>, grid, dim3(512), 0, stream, a, plan.nv, plan.splits, groups,
                       epi == kEpiSwiGLU ? 1 : 0);
    return hipGetLastError();
  }
  if (plan.tile == kTileArranged || plan.tile == kTileArranged128) {
    if (!a.wa0 || (epi == kEpiSwiGLU && !a.wa1) || a.a_lo || a.m <= 64 || a.k % 256 || plan.k_tiles_per_split % 4)
      return hipErrorInvalidValue;
    auto launch = [&](const GemmArgs& g, const GemmPlan& pl) {
      switch (epi) {
        case kEpiStoreF32: return launch_tile_arranged<kEpiStoreF32>(g, pl, stream);
        case kEpiResidualF32: return launch_tile_arranged<kEpiResidualF32>(g, pl, stream);
        case kEpiResidualOut: return launch_tile_arranged<kEpiResidualOut>(g, pl, stream);
        case kEpiSwiGLU: return launch_tile_arranged<kEpiSwiGLU>(g, pl, stream);
      }
      return hipErrorInvalidValue;
    };
    // A last tile row of at most 128 rows, where it costs a whole round of workgroups of its own (2176 rows x 148
    // tile columns: 1332 tiles are six rounds on 256 CUs, 1184 are five), runs on 128-row tiles - about 0.55 of a
    // 256-row tile's time - in the same launch, behind the big tiles.  Without K splits only.
    const int rest = a.m % 256;
    if (plan.tile == kTileArranged && plan.splits == 1 && a.m > 256 && rest > 0 && rest <= 128) {
      const long tiles_n = (plan.nv + 255) / 256, cus = 256;
      const long full_rows = a.m / 256;
      const float one = (float)(((full_rows + 1) * tiles_n + cus - 1) / cus);
      const float mixed = ceilf(((float)(full_rows * tiles_n) + 0.55f * (float)tiles_n) / (float)cus);   // rounds of 256-row tiles
      if (mixed < one - 0.1f) {
        GemmArgs head = a;
        head.m = a.m - rest;
        GemmArgs tail = a;
        const size_t at = (size_t)head.m;
        tail.m = rest;
        tail.a = a.a + at * a.lda;
        if (a.out_e16) tail.out_e16 = a.out_e16 + at * a.ldo;
        if (a.out_lo) tail.out_lo = a.out_lo + at * a.ldo;
        if (a.out_f32) tail.out_f32 = a.out_f32 + at * a.ldo;
        if (a.resid) tail.resid = a.resid + at * a.n;
        const int head_blocks = xcd_grid((int)(full_rows * tiles_n)), tail_blocks = xcd_grid((int)tiles_n);
        dim3 grid(head_blocks + tail_blocks), block(256);
        const int k_tiles = plan.k_tiles_per_split;
#define MOLINK_RAGGED(EPI, HALF)                                                                                          \
  hipLaunchKernelGGL((gemm_tile_arranged_ragged_kernel<EPI, HALF>), grid, block, 0, stream, head, tail, plan.nv, (int)full_rows, \
                     (int)tiles_n, k_tiles, head_blocks)
        if (a.a_half) {
#ifdef MOLINK_F16
          return hipErrorInvalidValue;   // the element type is half already
#else
          switch (epi) {
            case kEpiStoreF32: MOLINK_RAGGED(kEpiStoreF32, true); break;
            case kEpiResidualF32: MOLINK_RAGGED(kEpiResidualF32, true); break;
            case kEpiResidualOut: MOLINK_RAGGED(kEpiResidualOut, true); break;
            case kEpiSwiGLU: MOLINK_RAGGED(kEpiSwiGLU, true); break;
          }
#endif
        } else {
          switch (epi) {
            case kEpiStoreF32: MOLINK_RAGGED(kEpiStoreF32, false); break;
            case kEpiResidualF32: MOLINK_RAGGED(kEpiResidualF32, false); break;
            case kEpiResidualOut: MOLINK_RAGGED(kEpiResidualOut, false); break;
            case kEpiSwiGLU: MOLINK_RAGGED(kEpiSwiGLU, false); break;
          }
        }
#undef MOLINK_RAGGED
        return hipGetLastError();
      }
    }
    return launch(a, plan);
  }
  if (plan.tile == kTileW4 || plan.tile == kTileW4x128) {
    if (!a.q0.codes || (epi == kEpiSwiGLU && !a.q1.codes) || a.a_lo || !(a.a_half || kElemIsF16) || a.k % 256)
      return hipErrorInvalidValue;
    switch (epi) {
      case kEpiStoreF32: return launch_tile_w4<kEpiStoreF32>(a, plan, stream);
      case kEpiResidualF32: return launch_tile_w4<kEpiResidualF32>(a, plan, stream);
      case kEpiResidualOut: return launch_tile_w4<kEpiResidualOut>(a, plan, stream);
      case kEpiSwiGLU: return launch_tile_w4<kEpiSwiGLU>(a, plan, stream);
    }
    return hipErrorInvalidValue;
  }
  if (a.q0.codes) return hipErrorInvalidValue;   // the other tiled kernels take e16 weights only
  switch (epi) {
    case kEpiStoreF32: return launch_epi<kEpiStoreF32>(a, plan, stream);
    case kEpiResidualF32: return launch_epi<kEpiResidualF32>(a, plan, stream);
    case kEpiResidualOut: return launch_epi<kEpiResidualOut>(a, plan, stream);
    case kEpiSwiGLU: return launch_epi<kEpiSwiGLU>(a, plan, stream);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_gemm_reduce(const GemmArgs& a, GemmEpilogue epi, const GemmPlan& plan, hipStream_t stream) {
  const size_t count = (size_t)a.m * a.n / 4;
  dim3 grid((unsigned)((count + 255) / 256)), block(256);
  switch (epi) {
    case kEpiStoreF32:
      hipLaunchKernelGGL((gemm_splitk_reduce_kernel<kEpiStoreF32>), grid, block, 0, stream, a, plan.nv, plan.splits);
      break;
    case kEpiResidualF32:
      hipLaunchKernelGGL((gemm_splitk_reduce_kernel<kEpiResidualF32>), grid, block, 0, stream, a, plan.nv, plan.splits);
      break;
    case kEpiResidualOut:
      hipLaunchKernelGGL((gemm_splitk_reduce_kernel<kEpiResidualOut>), grid, block, 0, stream, a, plan.nv, plan.splits);
      break;
    case kEpiSwiGLU:
      hipLaunchKernelGGL((gemm_splitk_reduce_kernel<kEpiSwiGLU>), grid, block, 0, stream, a, plan.nv, plan.splits);
      break;
  }
  return hipGetLastError();
}

hipError_t launch_gemm_reduce_residual_norm(const GemmArgs& a, GemmEpilogue epi, const GemmPlan& plan,
                                            const NormSpec& norm, e16* norm_out, e16* norm_out_lo,
                                            bool norm_out_half, hipStream_t stream) {
  const int threads = a.n >= 4096 ? 1024 : (a.n >= 2048 ? 512 : 256);
  if (epi == kEpiResidualOut) {
    hipLaunchKernelGGL(reduce_residual_norm_kernel<false>, dim3(a.m), dim3(threads), 0, stream, a.partial, plan.splits, a.m,
                       a.n, a.resid, NormSpec{nullptr, nullptr, norm.eps, 0}, a.out_e16, (e16*)nullptr, a.ldo, false);
  } else {
    hipLaunchKernelGGL(reduce_residual_norm_kernel<true>, dim3(a.m), dim3(threads), 0, stream, a.partial, plan.splits, a.m,
                       a.n, a.resid, norm, norm_out, norm_out_lo, a.n, norm_out_half);
  }
  return hipGetLastError();
}

}  // namespace molink
