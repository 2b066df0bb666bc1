// Shared device-side types and small helpers for the gfx950 stage kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "elem.hpp"

namespace molink {

typedef __attribute__((ext_vector_type(8))) e16 e16x8;
typedef __attribute__((ext_vector_type(4))) e16 e16x4;
typedef __attribute__((ext_vector_type(2))) e16 e16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kWave = 64;        // lanes per wavefront
constexpr int kKvBlock = 16;     // tokens per KV block (fixed by the ABI)

// K layout inside one (block, KV head): [d / 32][16 positions][32 elements]; the key of slot s sits at
// position s with bits 2 and 3 exchanged (slots 0-3, 8-11, 4-7, 12-15).  In that order the key rows an
// MFMA key tile takes (whose accumulator registers must come out as 8 consecutive slots per lane group)
// are consecutive, so that one load instruction reads a 512-byte or 1 KB run instead of 64-byte pieces.
__host__ __device__ __forceinline__ int k_position_of_slot(int slot) {
  return (slot & 3) | ((slot & 8) >> 1) | ((slot & 4) << 1);
}
// element offset of (slot, dim) inside a (block, KV head) region of K
__host__ __device__ __forceinline__ int k_offset_in_block(int slot, int dim) {
  return ((dim >> 5) * kKvBlock + k_position_of_slot(slot)) * 32 + (dim & 31);
}

__device__ __forceinline__ float e16_to_f32(e16 v) { return static_cast<float>(v); }
__device__ __forceinline__ e16 f32_to_e16(float v) { return static_cast<e16>(v); }

// widen the low / high e16 of a packed 32-bit word
#ifdef MOLINK_F16
__device__ __forceinline__ float e16_lo(uint32_t w) { return static_cast<float>(__builtin_bit_cast(e16x2, w)[0]); }
__device__ __forceinline__ float e16_hi(uint32_t w) { return static_cast<float>(__builtin_bit_cast(e16x2, w)[1]); }
#else
__device__ __forceinline__ float e16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float e16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
#endif

// matrix instructions on e16 operands, fp32 accumulators
__device__ __forceinline__ f32x4 mfma_16x16x32(e16x8 a, e16x8 b, f32x4 c) {
#ifdef MOLINK_F16
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
#else
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
#endif
}
__device__ __forceinline__ f32x16 mfma_32x32x16(e16x8 a, e16x8 b, f32x16 c) {
#ifdef MOLINK_F16
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
#else
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
#endif
}

__device__ __forceinline__ uint32_t pack_e16(float lo, float hi) {
  e16x2 p;
  p[0] = static_cast<e16>(lo);
  p[1] = static_cast<e16>(hi);
  return __builtin_bit_cast(uint32_t, p);
}

// ---- half-precision activations inside the bfloat16 library ----
// Deep stages keep the inputs of their projections (norm outputs, attention output, silu(gate)*up) as IEEE
// half - eleven significant bits instead of eight - in the same 16-bit buffers, and the GEMMs convert the
// bfloat16 weight fragments to half on their way into the matrix instruction (exact: a bfloat16 number has
// eight significant bits; only magnitudes below 2^-17 lose bits, toward zero, by less than 2^-24).  In the
// half-precision library the element type is half already and none of this is used.
typedef _Float16 h16;
typedef __attribute__((ext_vector_type(8))) h16 h16x8;
typedef __attribute__((ext_vector_type(4))) h16 h16x4;
typedef __attribute__((ext_vector_type(2))) h16 h16x2;

// a value as the 16 bits of an activation: half (clamped to its finite range) when as_half, else e16
__device__ __forceinline__ e16 f32_to_act(float v, bool as_half) {
#ifdef MOLINK_F16
  (void)as_half;
  return static_cast<e16>(v);
#else
  if (as_half) return __builtin_bit_cast(e16, static_cast<h16>(fminf(fmaxf(v, -65504.f), 65504.f)));
  return static_cast<e16>(v);
#endif
}

// the value of an activation stored by f32_to_act
__device__ __forceinline__ float act_to_f32(e16 v, bool as_half) {
#ifdef MOLINK_F16
  (void)as_half;
  return static_cast<float>(v);
#else
  return as_half ? static_cast<float>(__builtin_bit_cast(h16, v)) : static_cast<float>(v);
#endif
}

// eight bfloat16 numbers as eight halves (round toward zero: exact wherever half has the range)
__device__ __forceinline__ h16x8 bf16x8_to_half(e16x8 v) {
#ifdef MOLINK_F16
  return v;
#else
  const u32x4 w = __builtin_bit_cast(u32x4, v);
  u32x4 o;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    o[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(__uint_as_float(w[i] << 16), __uint_as_float(w[i] & 0xffff0000u)));
  return __builtin_bit_cast(h16x8, o);
#endif
}
__device__ __forceinline__ f32x16 mfma_32x32x16_half(h16x8 a, h16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma_16x16x32_half(h16x8 a, h16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// 16-byte global load / store of 8 e16
__device__ __forceinline__ e16x8 load8(const e16* p) { return *reinterpret_cast<const e16x8*>(p); }
// The same load for data that is read exactly once (cached KV, streamed weights): marked nontemporal,
// so it does not displace what the caches hold; measured about 15 % more read bandwidth on long streams.
__device__ __forceinline__ e16x8 load8_stream(const e16* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const e16x8*>(p));
}
__device__ __forceinline__ void store8(e16* p, e16x8 v) { *reinterpret_cast<e16x8*>(p) = v; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// The 8 XCDs take workgroups round-robin.  Remap the hardware workgroup id so that ids that are
// consecutive in the logical order run on the same XCD (and share its L2).
// Returns the logical id, or -1 for a padding workgroup.  Launch with xcd_grid(total) workgroups.
__host__ __device__ __forceinline__ int xcd_grid(int total) { return ((total + 7) / 8) * 8; }
__device__ __forceinline__ int xcd_logical_id(int pid, int total) {
  const int per = (total + 7) / 8;
  const int lid = (pid % 8) * per + pid / 8;
  return lid < total ? lid : -1;
}

// ---- software-pipelined tiles in LDS (used by the GEMM and the prefill attention kernels) ----

// LDS stages live in separate arrays so that the compiler can tell a stage being filled from the
// stage being read (a single array indexed by the stage would force every LDS read to wait for all
// loads in flight).
template <int BYTES> struct LdsStages {
  template <int S> static __device__ __forceinline__ char* get() {
    __shared__ __attribute__((aligned(1024))) char stage[BYTES];
    return stage;
  }
};

// s_waitcnt on the vector-memory counter only (gfx9 encoding: vmcnt in bits 3:0 and 15:14).
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0070 | 0x0F00);
}

// Workgroup barrier without the memory fence of __syncthreads(): that fence would wait for every load
// in flight, including the tiles being prefetched into other LDS stages.  The caller has already
// waited for exactly the loads the other waves are about to read; this only drains the wave's own LDS
// operations and keeps the compiler from moving memory accesses across the barrier.
__device__ __forceinline__ void pipeline_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0), vmcnt and expcnt untouched
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

}  // namespace molink
