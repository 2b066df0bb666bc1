// The library's 16-bit element type.
#pragma once

namespace molink {

// e16 is the 16-bit element type of everything the library stores (weights, activations, KV cache, payload):
// bfloat16 by default, IEEE half when the sources are compiled with -DMOLINK_F16 (a second library with the
// same C ABI).  Arithmetic is fp32 in both; only the storage format and the MFMA operand type differ.
#ifdef MOLINK_F16
typedef _Float16 e16;
constexpr int kElemIsF16 = 1;
#else
typedef __bf16 e16;
constexpr int kElemIsF16 = 0;
#endif

// The norm in front of a branch of the block: RMSNorm (layer = 0; gain only) or LayerNorm (layer = 1; bias optional).
struct NormSpec {
  const e16* gain;   // nullptr: no norm asked for
  const e16* bias;   // LayerNorm only, may be nullptr
  float eps;
  int layer;
};

}  // namespace molink
