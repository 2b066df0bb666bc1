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

template <int EPI>
struct ColumnMap {
  // Maps a column v of the iterated column space to (matrix, row).  For SwiGLU, columns come in
  // groups of 64: 32 gate rows f..f+31 followed by the 32 up rows with the same f, so that one
  // wave's two 32-wide MFMA column tiles hold gate and up of the same features.
  __device__ static __forceinline__ const __bf16* row_ptr(const GemmArgs& p, int v) {
    if constexpr (EPI == kEpiSwiGLU) {
      int f = (v >> 6) * 32 + (v & 31);
      f = f < p.n ? f : p.n - 1;
      const __bf16* w = (v & 32) ? p.w1 : p.w0;
      return w + (size_t)f * p.k;
    } else {
      const int n = v < p.n ? v : p.n - 1;
      return p.w0 + (size_t)n * p.k;
    }
  }
};

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, bool SPLIT>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gemm_bf16_kernel(GemmArgs p, int nv, int tiles_m, int tiles_n,
                                                                          int splits, int k_tiles_per_split) {
  constexpr int NTHREADS = WAVES_M * WAVES_N * 64;
  constexpr int TM = BM / WAVES_M, TN = BN / WAVES_N;
  constexpr int MT = TM / 32, NT = TN / 32;
  constexpr int A_CHUNKS = BM * (kBK / 8) / NTHREADS;   // 16-byte chunks per thread per tile
  constexpr int B_CHUNKS = BN * (kBK / 8) / NTHREADS;
  static_assert(A_CHUNKS >= 1 && B_CHUNKS >= 1, "tile too small for the workgroup");
  static_assert(EPI != kEpiSwiGLU || TN == 64, "SwiGLU pairs two 32-wide column tiles per wave");

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
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  const int k_tiles = (p.k + kBK - 1) / kBK;
  const int kt_begin = split * k_tiles_per_split;
  const int kt_end = min(kt_begin + k_tiles_per_split, k_tiles);

  // per-thread source rows of the global->LDS copy (fixed across K tiles)
  const __bf16* a_src[A_CHUNKS];
  const __bf16* b_src[B_CHUNKS];
  int a_dst[A_CHUNKS], b_dst[B_CHUNKS];
  const int kc = (tid & 7) * 8;  // this thread's k offset inside a tile
#pragma unroll
  for (int i = 0; i < A_CHUNKS; ++i) {
    const int row = (i * NTHREADS + tid) >> 3;
    int gm = m0 + row;
    gm = gm < p.m ? gm : p.m - 1;
    a_src[i] = p.a + (size_t)gm * p.lda + kc;
    a_dst[i] = row * kLdsStride + kc;
  }
#pragma unroll
  for (int i = 0; i < B_CHUNKS; ++i) {
    const int row = (i * NTHREADS + tid) >> 3;
    b_src[i] = ColumnMap<EPI>::row_ptr(p, n0 + row) + kc;
    b_dst[i] = row * kLdsStride + kc;
  }

  bf16x8 a_reg[A_CHUNKS], b_reg[B_CHUNKS];
  auto fetch = [&](int kt) {
    const int k0 = kt * kBK;
    const bool in_k = (k0 + kc) < p.k;            // K is a multiple of 8: a chunk is all in or all out
    const int koff = in_k ? k0 : 0;               // keep the address in bounds, zero the data below
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
      bf16x8 v = load8(a_src[i] + koff - (in_k ? 0 : kc));
      if (!in_k) v = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
      a_reg[i] = v;
    }
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i) {
      bf16x8 v = load8(b_src[i] + koff - (in_k ? 0 : kc));
      if (!in_k) v = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
      b_reg[i] = v;
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) *reinterpret_cast<bf16x8*>(&lds_a[buf][a_dst[i]]) = a_reg[i];
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i) *reinterpret_cast<bf16x8*>(&lds_b[buf][b_dst[i]]) = b_reg[i];
  };

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  if (kt_begin < kt_end) {
    fetch(kt_begin);
    stash(0);
  }
  __syncthreads();

  const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
  for (int kt = kt_begin; kt < kt_end; ++kt) {
    const int buf = (kt - kt_begin) & 1;
    const bool more = kt + 1 < kt_end;
    if (more) fetch(kt + 1);
    const __bf16* la = &lds_a[buf][(wm * TM + frag_row) * kLdsStride + frag_k];
    const __bf16* lb = &lds_b[buf][(wn * TN + frag_row) * kLdsStride + frag_k];
#pragma unroll
    for (int kk = 0; kk < kBK / 16; ++kk) {
      bf16x8 af[MT], bfr[NT];
#pragma unroll
      for (int i = 0; i < MT; ++i) af[i] = *reinterpret_cast<const bf16x8*>(la + i * 32 * kLdsStride + kk * 16);
#pragma unroll
      for (int j = 0; j < NT; ++j) bfr[j] = *reinterpret_cast<const bf16x8*>(lb + j * 32 * kLdsStride + kk * 16);
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (more) stash(buf ^ 1);
    __syncthreads();
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
        const int v = n0 + wn * TN + col_in_tile;          // gate column; up is 32 further
        const int f = (v >> 6) * 32 + (v & 31);
        if (f < p.n) p.out_bf16[(size_t)m * p.ldo + f] = f32_to_bf16(silu_f(acc[i][0][r]) * acc[i][1][r]);
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

template <int BM, int BN, int EPI>
hipError_t launch_tile(const GemmArgs& a, const GemmPlan& plan, hipStream_t stream) {
  const int tiles_m = (a.m + BM - 1) / BM;
  const int tiles_n = (plan.nv + BN - 1) / BN;
  const int total = tiles_m * tiles_n * plan.splits;
  dim3 grid(xcd_grid(total)), block(256);
  if (plan.splits > 1) {
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, 2, 2, EPI, true>), grid, block, 0, stream, a, plan.nv, tiles_m, tiles_n,
                       plan.splits, plan.k_tiles_per_split);
  } else {
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, 2, 2, EPI, false>), grid, block, 0, stream, a, plan.nv, tiles_m,
                       tiles_n, 1, plan.k_tiles_per_split);
  }
  return hipGetLastError();
}

template <int EPI>
hipError_t launch_epi(const GemmArgs& a, const GemmPlan& plan, hipStream_t stream) {
  return plan.tile == 0 ? launch_tile<128, 128, EPI>(a, plan, stream) : launch_tile<64, 128, EPI>(a, plan, stream);
}

}  // namespace

GemmPlan plan_gemm(int m, int n, int k, GemmEpilogue epi, int num_cus) {
  GemmPlan plan;
  plan.tile = m <= 64 ? 1 : 0;
  const int bm = plan.tile == 0 ? 128 : 64, bn = 128;
  plan.nv = epi == kEpiSwiGLU ? ((n + 31) / 32) * 64 : n;
  const int tiles = ((m + bm - 1) / bm) * ((plan.nv + bn - 1) / bn);
  const int k_tiles = (k + kBK - 1) / kBK;
  int splits = 1;
  if (tiles < num_cus) {
    splits = (2 * num_cus + tiles - 1) / tiles;
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
