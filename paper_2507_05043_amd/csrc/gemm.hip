// bf16 MFMA GEMM for the stage's projections: C[M][N] = A[M][K] * W[N][K]^T, fp32 accumulate.
//
// Both operands are K-contiguous, which is the layout the 32x32x16 bf16 MFMA wants in its lanes
// (lane l holds 8 consecutive k of row l%32).  Tiles travel HBM -> registers (16-byte coalesced
// loads) -> LDS (row stride padded by 16 bytes, so 128-bit LDS reads of 8 consecutive rows cover all
// banks) -> MFMA operands.  The next K tile is prefetched into registers while the current one is
// multiplied; LDS is double buffered so one barrier per K tile suffices.
//
// Workgroup ids are remapped so that consecutive logical tiles share an XCD: the M tiles that reuse
// one weight tile run next to each other on one L2.
//
// Small-M shapes (decode micro-batches) do not have enough output tiles to fill 256 CUs, so the K
// dimension is split across workgroups; the partial sums go to fp32 scratch and a second kernel adds
// them in a fixed order (deterministic) and applies the epilogue.
#include "gemm.hpp"
#include "common.hpp"

namespace molink {

namespace {

constexpr int kBK = 64;               // K elements per tile
constexpr int kLdsStride = kBK + 8;   // padded row stride in bf16 elements (144 bytes)

// Scheduling hint: NOPS memory operations of class OPMASK (0x100 LDS read, 0x200 LDS write) spread evenly
// between NMFMA MFMAs.  The group sizes must be compile-time constants, hence the recursion.
template <int R, int NOPS, int NMFMA, int OPMASK, bool OP_FIRST>
__device__ __forceinline__ void sched_interleave() {
  if constexpr (R < NOPS) {
    constexpr int n = (R + 1) * NMFMA / NOPS - R * NMFMA / NOPS;
    if constexpr (OP_FIRST) __builtin_amdgcn_sched_group_barrier(OPMASK, 1, 0);
    if constexpr (n > 0) __builtin_amdgcn_sched_group_barrier(0x008, n, 0);
    if constexpr (!OP_FIRST) __builtin_amdgcn_sched_group_barrier(OPMASK, 1, 0);
    sched_interleave<R + 1, NOPS, NMFMA, OPMASK, OP_FIRST>();
  }
}

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

// Workgroup of 4 waves (2 x 2); wave tile (BM/2) x (BN/2) made of 32x32 MFMA tiles.
// PF = number of K tiles kept in flight in registers ahead of the one being multiplied.  Small tiles
// finish a K tile faster than a load returns, so they look two tiles ahead; 256x256 needs only one.
// Fetches are unconditional (the tile index is clamped at the end of the range, which re-reads the
// last tile once or twice) so that the loop body has no branches and the waits on outstanding loads
// count exactly the loads that must have landed.
template <int BM, int BN, int PF, int EPI, bool SPLIT>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs p, int nv, int tiles_m, int tiles_n, int splits,
                                                        int k_tiles_per_split) {
  constexpr int NTHREADS = 256;
  constexpr int TM = BM / 2, TN = BN / 2;
  constexpr int MT = TM / 32, NT = TN / 32;
  constexpr int A_CHUNKS = BM * (kBK / 8) / NTHREADS;   // 16-byte chunks per thread per tile
  constexpr int B_CHUNKS = BN * (kBK / 8) / NTHREADS;
  static_assert(A_CHUNKS >= 1 && B_CHUNKS >= 1, "tile too small for the workgroup");
  static_assert(EPI != kEpiSwiGLU || TN % 64 == 0, "SwiGLU pairs two 32-wide column tiles per wave");
  static_assert(PF == 1 || PF == 2, "one or two K tiles in flight");

  __shared__ __attribute__((aligned(16))) __bf16 lds_a[2][BM * kLdsStride];
  __shared__ __attribute__((aligned(16))) __bf16 lds_b[2][BN * kLdsStride];

  const int total = tiles_m * tiles_n * splits;
  const int lid = xcd_logical_id(blockIdx.x, total);
  if (lid < 0) return;
  const int tile_m = lid % tiles_m;
  const int split = (lid / tiles_m) % splits;
  const int tile_n = lid / (tiles_m * splits);
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  const int k_tiles = (p.k + kBK - 1) / kBK;
  const int kt_begin = split * k_tiles_per_split;
  const int kt_end = min(kt_begin + k_tiles_per_split, k_tiles);
  const int nkt = kt_end - kt_begin;

  // Global->LDS copy.  Chunk i of a thread is 16 bytes of row 32*i + tid/8 at k offset 8*(tid%8); the
  // byte offsets from the (uniform) matrix bases are fixed across K tiles, so a load is one
  // instruction with a scalar base that advances along K and a 32-bit per-thread offset.
  const int kc = (tid & 7) * 8;
  const int row_in_pass = tid >> 3;
  uint32_t a_off[A_CHUNKS], b_off[B_CHUNKS];
#pragma unroll
  for (int i = 0; i < A_CHUNKS; ++i) {
    int gm = m0 + i * 32 + row_in_pass;
    gm = gm < p.m ? gm : p.m - 1;
    a_off[i] = ((uint32_t)gm * (uint32_t)p.lda + kc) * 2u;
  }
#pragma unroll
  for (int i = 0; i < B_CHUNKS; ++i) {
    int row;
    if constexpr (EPI == kEpiSwiGLU) {
      // 32 gate rows, then the 32 up rows of the same features: chunk i is gate for even i, up for odd i
      row = ((n0 >> 6) + (i >> 1)) * 32 + row_in_pass;
    } else {
      row = n0 + i * 32 + row_in_pass;
    }
    row = row < p.n ? row : p.n - 1;
    b_off[i] = ((uint32_t)row * (uint32_t)p.k + kc) * 2u;
  }
  const int lds_dst = row_in_pass * kLdsStride + kc;

  bf16x8 a_reg[PF][A_CHUNKS], b_reg[PF][B_CHUNKS];
  int zero_below[PF];   // leading k columns of the tile in a register set that repeat the previous tile
  auto fetch = [&](int set, int idx) {
    int kt = kt_begin + idx;
    kt = kt < kt_end - 1 ? kt : kt_end - 1;
    // The last tile of a K that is not a multiple of 64 is shifted back to end exactly at K (so every
    // load stays inside its row); the columns it then shares with the previous tile are zeroed on
    // their way into LDS.  All of this is uniform: nothing below depends on loaded data.
    int k0 = kt * kBK;
    const int k_last = p.k - kBK;
    zero_below[set] = k0 > k_last ? k0 - k_last : 0;
    k0 = k0 > k_last ? k_last : k0;
    const char* abase = reinterpret_cast<const char*>(p.a + k0);
    const char* w0base = reinterpret_cast<const char*>(p.w0 + k0);
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) a_reg[set][i] = *reinterpret_cast<const bf16x8*>(abase + a_off[i]);
    if constexpr (EPI == kEpiSwiGLU) {
      const char* w1base = reinterpret_cast<const char*>(p.w1 + k0);
#pragma unroll
      for (int i = 0; i < B_CHUNKS; ++i)
        b_reg[set][i] = *reinterpret_cast<const bf16x8*>(((i & 1) ? w1base : w0base) + b_off[i]);
    } else {
#pragma unroll
      for (int i = 0; i < B_CHUNKS; ++i) b_reg[set][i] = *reinterpret_cast<const bf16x8*>(w0base + b_off[i]);
    }
    __builtin_amdgcn_sched_barrier(0);   // keep the loads here, ahead of the MFMAs they overlap with
  };
  // LDS writes of one register set: plain copies, nothing is computed on the loaded data (any
  // arithmetic on it would be scheduled early and stall on the loads that were just issued).
  auto stash = [&](int set, int buf) {
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i)
      *reinterpret_cast<bf16x8*>(&lds_a[buf][lds_dst + i * 32 * kLdsStride]) = a_reg[set][i];
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i)
      *reinterpret_cast<bf16x8*>(&lds_b[buf][lds_dst + i * 32 * kLdsStride]) = b_reg[set][i];
  };
  // The shifted last tile of a K that is not a multiple of 64: overwrite the columns it shares with
  // the previous tile with zeros (after this thread's own copies; LDS operations of a wave are ordered).
  auto patch_tail = [&](int set, int buf) {
    if (zero_below[set] > 0 && kc < zero_below[set]) {
      const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int i = 0; i < A_CHUNKS; ++i) *reinterpret_cast<bf16x8*>(&lds_a[buf][lds_dst + i * 32 * kLdsStride]) = zero;
#pragma unroll
      for (int i = 0; i < B_CHUNKS; ++i) *reinterpret_cast<bf16x8*>(&lds_b[buf][lds_dst + i * 32 * kLdsStride]) = zero;
    }
  };

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
  // One K tile: 4 steps of 16 k.  The LDS reads of step kk+1 are issued under the MFMAs of step kk
  // (fragments are double buffered in registers), and the LDS writes of the next tile (register set
  // `st_set` into buffer `st_buf`, if st_set >= 0) are spread under the MFMAs of the last step.
  auto multiply = [&](int buf, int st_set, int st_buf) {
    const __bf16* la = &lds_a[buf][(wm * TM + frag_row) * kLdsStride + frag_k];
    const __bf16* lb = &lds_b[buf][(wn * TN + frag_row) * kLdsStride + frag_k];
    bf16x8 af[2][MT], bfr[2][NT];
    auto read_frags = [&](int s, int kk) {
#pragma unroll
      for (int i = 0; i < MT; ++i) af[s][i] = *reinterpret_cast<const bf16x8*>(la + i * 32 * kLdsStride + kk * 16);
#pragma unroll
      for (int j = 0; j < NT; ++j) bfr[s][j] = *reinterpret_cast<const bf16x8*>(lb + j * 32 * kLdsStride + kk * 16);
    };
    constexpr int KSTEPS = kBK / 16, NMFMA = MT * NT, NREAD = MT + NT, NWRITE = A_CHUNKS + B_CHUNKS;
    read_frags(0, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, NREAD, 0);   // the first step's fragments cannot overlap anything
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
      if (kk + 1 < KSTEPS) read_frags((kk + 1) & 1, kk + 1);
      if (kk + 1 == KSTEPS && st_set >= 0) stash(st_set, st_buf);
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j], acc[i][j], 0, 0, 0);
      // scheduling pattern for this step: memory operations spread evenly between the MFMAs
      if (kk + 1 < KSTEPS) {
        sched_interleave<0, NREAD, NMFMA, 0x100, true>();
      } else if (st_set >= 0) {
        sched_interleave<0, NWRITE, NMFMA, 0x200, false>();
      }
    }
  };

  if (nkt > 0) {
    if constexpr (PF == 1) {
      fetch(0, 0);
      stash(0, 0);
      patch_tail(0, 0);
      __syncthreads();
      for (int i = 0; i < nkt; ++i) {
        fetch(0, i + 1);
        multiply(i & 1, 0, (i & 1) ^ 1);
        patch_tail(0, (i & 1) ^ 1);
        __syncthreads();
      }
    } else {
      // tile i is in LDS buffer i&1; register set (i+1)&1 holds tile i+1; set i&1 is free for tile i+2
      fetch(0, 0);
      fetch(1, 1);
      stash(0, 0);
      patch_tail(0, 0);
      __syncthreads();
      int i = 0;
      for (; i + 2 <= nkt; i += 2) {
        fetch(0, i + 2);
        multiply(0, 1, 1);
        patch_tail(1, 1);
        __syncthreads();
        fetch(1, i + 3);
        multiply(1, 0, 0);
        patch_tail(0, 0);
        __syncthreads();
      }
      if (i < nkt) multiply(0, -1, 0);
    }
  }

  // Epilogue.  Accumulator register r of lane l is C[row 8*(r/4) + 4*(l/32) + r%4][col l%32] of its tile.
  const int col_in_tile = lane & 31;
  const int row_base = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < MT; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + wm * TM + i * 32 + 8 * (r / 4) + row_base + (r % 4);
      if (m >= p.m) continue;
      if constexpr (SPLIT) {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          const int v = n0 + wn * TN + j * 32 + col_in_tile;
          if (v < nv) p.partial[((size_t)split * p.m + m) * nv + v] = acc[i][j][r];
        }
      } else if constexpr (EPI == kEpiSwiGLU) {
#pragma unroll
        for (int j = 0; j < NT; j += 2) {
          const int v = n0 + wn * TN + j * 32 + col_in_tile;   // gate column; its up column is 32 further
          const int f = (v >> 6) * 32 + (v & 31);
          if (f < p.n) p.out_bf16[(size_t)m * p.ldo + f] = f32_to_bf16(silu_f(acc[i][j][r]) * acc[i][j + 1][r]);
        }
      } else {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          const int n = n0 + wn * TN + j * 32 + col_in_tile;
          if (n >= p.n) continue;
          const float c = acc[i][j][r];
          if constexpr (EPI == kEpiStoreBf16) {
            p.out_bf16[(size_t)m * p.ldo + n] = f32_to_bf16(c);
          } else if constexpr (EPI == kEpiResidualF32) {
            p.resid[(size_t)m * p.n + n] += c;
          } else {
            p.out_bf16[(size_t)m * p.ldo + n] = f32_to_bf16(p.resid[(size_t)m * p.n + n] + c);
          }
        }
      }
    }
  }
}

// Adds the split-K partial sums (split 0 first) and applies the epilogue.  One thread per output.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_splitk_reduce_kernel(GemmArgs p, int nv, int splits) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t count = (size_t)p.m * p.n;
  if (idx >= count) return;
  const int m = (int)(idx / p.n), n = (int)(idx % p.n);
  const size_t plane = (size_t)p.m * nv;
  if constexpr (EPI == kEpiSwiGLU) {
    const int vg = (n >> 5) * 64 + (n & 31);
    const float* src = p.partial + (size_t)m * nv + vg;
    float g = 0.f, u = 0.f;
    for (int s = 0; s < splits; ++s) {
      g += src[s * plane];
      u += src[s * plane + 32];
    }
    p.out_bf16[(size_t)m * p.ldo + n] = f32_to_bf16(silu_f(g) * u);
  } else {
    const float* src = p.partial + (size_t)m * nv + n;
    float c = 0.f;
    for (int s = 0; s < splits; ++s) c += src[s * plane];
    if constexpr (EPI == kEpiStoreBf16) {
      p.out_bf16[(size_t)m * p.ldo + n] = f32_to_bf16(c);
    } else if constexpr (EPI == kEpiResidualF32) {
      p.resid[idx] += c;
    } else {
      p.out_bf16[(size_t)m * p.ldo + n] = f32_to_bf16(p.resid[idx] + c);
    }
  }
}

// Sum of the split-K partial results + residual add + (RMSNorm | bf16 rounding), one workgroup per row.
template <bool NORM>
__global__ __launch_bounds__(1024) void reduce_residual_norm_kernel(const float* __restrict__ partial, int splits,
                                                                   int m_rows, int n, float* __restrict__ x,
                                                                   const __bf16* __restrict__ gain, float eps,
                                                                   __bf16* __restrict__ out, int ldo) {
  __shared__ float wsum[16];
  const int row = blockIdx.x, tid = threadIdx.x;
  const int stride = blockDim.x * 4, nwaves = blockDim.x >> 6;
  const size_t plane = (size_t)m_rows * n;
  float* xr = x + (size_t)row * n;
  const float* pr = partial + (size_t)row * n;
  float ss = 0.f;
  for (int c = tid * 4; c < n; c += stride) {
    f32x4 v = *reinterpret_cast<const f32x4*>(xr + c);
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    for (int k = 0; k < splits; ++k) s += *reinterpret_cast<const f32x4*>(pr + k * plane + c);
    v += s;
    if constexpr (NORM) {
      *reinterpret_cast<f32x4*>(xr + c) = v;
      ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
    } else {
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = f32_to_bf16(v[e]);
      *reinterpret_cast<bf16x4*>(out + (size_t)row * ldo + c) = o;
    }
  }
  if constexpr (NORM) {
    ss = wave_sum(ss);
    if ((tid & 63) == 0) wsum[tid >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
    for (int w = 0; w < nwaves; ++w) tot += wsum[w];
    const float rs = 1.0f / sqrtf(tot / (float)n + eps);
    for (int c = tid * 4; c < n; c += stride) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(xr + c);     // written by this same thread above
      const bf16x4 g = *reinterpret_cast<const bf16x4*>(gain + c);
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = f32_to_bf16(v[e] * rs * bf16_to_f32(g[e]));
      *reinterpret_cast<bf16x4*>(out + (size_t)row * ldo + c) = o;
    }
  }
}

template <int BM, int BN, int PF, int EPI>
hipError_t launch_tile(const GemmArgs& a, const GemmPlan& plan, hipStream_t stream) {
  const int tiles_m = (a.m + BM - 1) / BM;
  const int tiles_n = (plan.nv + BN - 1) / BN;
  const int total = tiles_m * tiles_n * plan.splits;
  dim3 grid(xcd_grid(total)), block(256);
  if (plan.splits > 1) {
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, PF, EPI, true>), grid, block, 0, stream, a, plan.nv, tiles_m, tiles_n,
                       plan.splits, plan.k_tiles_per_split);
  } else {
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, PF, EPI, false>), grid, block, 0, stream, a, plan.nv, tiles_m, tiles_n,
                       1, plan.k_tiles_per_split);
  }
  return hipGetLastError();
}

template <int EPI>
hipError_t launch_epi(const GemmArgs& a, const GemmPlan& plan, hipStream_t stream) {
  switch (plan.tile) {
    case kTile256x256: return launch_tile<256, 256, 1, EPI>(a, plan, stream);
    case kTile256x128: return launch_tile<256, 128, 2, EPI>(a, plan, stream);
    case kTile128x128: return launch_tile<128, 128, 2, EPI>(a, plan, stream);
    default: return launch_tile<64, 128, 2, EPI>(a, plan, stream);
  }
}

}  // namespace

GemmPlan plan_gemm(int m, int n, int k, GemmEpilogue epi, int num_cus) {
  GemmPlan plan;
  plan.nv = epi == kEpiSwiGLU ? ((n + 31) / 32) * 64 : n;
  const int k_tiles = (k + kBK - 1) / kBK;
  struct Cand { int tile, bm, bn, wg_per_cu; float eff; };
  // relative MFMA efficiency of a tile shape (LDS traffic per MFMA) and how many fit on a CU (LDS)
  static const Cand cands[] = {{kTile256x256, 256, 256, 1, 1.0f}, {kTile256x128, 256, 128, 1, 0.85f},
                               {kTile128x128, 128, 128, 2, 0.7f}};
  if (m <= 64) {
    plan.tile = kTile64x128;
  } else {
    float best = 0.f;
    plan.tile = kTile128x128;
    for (const Cand& c : cands) {
      const long tiles = (long)((m + c.bm - 1) / c.bm) * ((plan.nv + c.bn - 1) / c.bn);
      const long slots = (long)num_cus * c.wg_per_cu;
      const long rounds = (tiles + slots - 1) / slots;
      const float cost = (float)rounds * c.bm * c.bn * c.wg_per_cu / c.eff;
      if (best == 0.f || cost < best) { best = cost; plan.tile = c.tile; }
    }
  }
  const int bm = plan.tile == kTile64x128 ? 64 : (plan.tile == kTile128x128 ? 128 : 256);
  const int bn = plan.tile == kTile256x256 ? 256 : 128;
  const int wg_per_cu = (plan.tile == kTile128x128 || plan.tile == kTile64x128) ? 2 : 1;
  const int tiles = ((m + bm - 1) / bm) * ((plan.nv + bn - 1) / bn);
  int splits = 1;
  if (tiles * 2 <= num_cus * wg_per_cu) {
    splits = (num_cus * wg_per_cu + tiles - 1) / tiles;
    const int max_by_k = k_tiles / 4 > 0 ? k_tiles / 4 : 1;   // at least 4 K tiles per split
    if (splits > max_by_k) splits = max_by_k;
    if (splits > 16) splits = 16;
  }
  plan.k_tiles_per_split = (k_tiles + splits - 1) / splits;
  plan.splits = (k_tiles + plan.k_tiles_per_split - 1) / plan.k_tiles_per_split;
  return plan;
}

size_t gemm_partial_floats(int max_m, int n, int k, GemmEpilogue epi, int num_cus) {
  // Splitting only happens when there are fewer tiles than CUs; the scratch of any such shape is
  // bounded by 16 splits of the largest m that still splits.
  size_t worst = 0;
  for (int m = 1; m <= max_m; m = (m < 64 ? 64 : m + 64)) {
    const int mm = m > max_m ? max_m : m;
    GemmPlan p = plan_gemm(mm, n, k, epi, num_cus);
    if (p.splits > 1) {
      const size_t need = (size_t)p.splits * mm * p.nv;
      if (need > worst) worst = need;
    }
  }
  GemmPlan p = plan_gemm(max_m, n, k, epi, num_cus);
  if (p.splits > 1) {
    const size_t need = (size_t)p.splits * max_m * p.nv;
    if (need > worst) worst = need;
  }
  return worst;
}

hipError_t launch_gemm_main(const GemmArgs& a, GemmEpilogue epi, const GemmPlan& plan, hipStream_t stream) {
  switch (epi) {
    case kEpiStoreBf16: return launch_epi<kEpiStoreBf16>(a, plan, stream);
    case kEpiResidualF32: return launch_epi<kEpiResidualF32>(a, plan, stream);
    case kEpiResidualOut: return launch_epi<kEpiResidualOut>(a, plan, stream);
    case kEpiSwiGLU: return launch_epi<kEpiSwiGLU>(a, plan, stream);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_gemm_reduce(const GemmArgs& a, GemmEpilogue epi, const GemmPlan& plan, hipStream_t stream) {
  const size_t count = (size_t)a.m * a.n;
  dim3 grid((unsigned)((count + 255) / 256)), block(256);
  switch (epi) {
    case kEpiStoreBf16:
      hipLaunchKernelGGL((gemm_splitk_reduce_kernel<kEpiStoreBf16>), grid, block, 0, stream, a, plan.nv, plan.splits);
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
                                            const __bf16* gain, float eps, __bf16* norm_out, hipStream_t stream) {
  const int threads = a.n >= 4096 ? 1024 : (a.n >= 2048 ? 512 : 256);
  if (epi == kEpiResidualOut) {
    hipLaunchKernelGGL(reduce_residual_norm_kernel<false>, dim3(a.m), dim3(threads), 0, stream, a.partial, plan.splits, a.m,
                       a.n, a.resid, (const __bf16*)nullptr, eps, a.out_bf16, a.ldo);
  } else {
    hipLaunchKernelGGL(reduce_residual_norm_kernel<true>, dim3(a.m), dim3(threads), 0, stream, a.partial, plan.splits, a.m,
                       a.n, a.resid, gain, eps, norm_out, a.n);
  }
  return hipGetLastError();
}

}  // namespace molink
