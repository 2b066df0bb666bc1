// C ABI of the stage library: configuration checks, workspace carving, per-call metadata (slot
// mapping, work lists) and the launch sequence of one micro-batch.  See include/molink_stage.h.
#include "../../include/molink_stage.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "attention.hpp"
#include "elementwise.hpp"
#include "common.hpp"
#include "gemm.hpp"
#include "w4.hpp"

using namespace molink;

// Scratch of stage_forward_static: the workspace of callers that cannot bring one.  One copy per GPU the library
// runs on, held until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress;
// the device address of each GPU's copy is looked up once per device (static_scratch_of) and kernels only ever
// see that pointer.
static constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local char g_error[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                          \
  do {                                                                                         \
    hipError_t e_ = (expr);                                                                    \
    if (e_ != hipSuccess) return fail(STAGE_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

constexpr size_t kAlign = 256;
size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
char* g_scratch_ptr[kMaxDevices] = {};

// Device address of this device's copy of `scratch`; `device` must be the current device.
int static_scratch_of(int device, char** out) {
  if (device < 0 || device >= kMaxDevices) return fail(STAGE_ERR_CONFIG, "device %d: at most %d devices are supported", device, kMaxDevices);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr || (uintptr_t)ptr % kAlign) return fail(STAGE_ERR_HIP, "the static scratch array has no usable device address");
    g_scratch_ptr[device] = (char*)ptr;
  }
  *out = g_scratch_ptr[device];
  return STAGE_OK;
}

constexpr int kStagingSlots = 4;
constexpr int kMaxTimed = 8192;
// Decode work items: at most this many per CU (sets the key-range length of large launches), and no key range shorter
// than kMinDecodeRange unless the sequence is.  Measured on 70B-shaped decode launches of 0.84 / 4.9 GB and a
// 7B-shaped one of 1.3 GB: 16 / 24 / 32 / 48 / 64 items per CU give 146 / 153 / 158 / 161 / 163 us, 766 / 761 / 768 /
// 779 / 792 us and 217 / 214 / 216 / 217 / 218 us - about 400 keys per wave and more is what all three want.
constexpr int kDecodeWavesPerCu = 24;
constexpr int kMinDecodeRange = 384;

struct Dims {
  int L, H, nq, nkv, d, F, qkv_out, g;
  int rd;   // leading elements of a head that rotate
};

struct WorkspaceLayout {
  size_t x, a, a_lo, qkv_f32, qkv, q_lo, attn, attn_lo, mlp, mlp_lo, cos_sin, splitk, part_o, part_ml, meta, total;
  size_t b2, b2_lo;                        // parallel block: the second norm of the block's input (and its second plane)
  size_t up_f32;                           // ungated MLP: the first product before bias and gelu, fp32
  size_t splitk_floats;                    // capacity of the split-K scratch
  size_t head_a, head_logits, ends_meta;   // output head: normalised last rows, fp32 logits, token ids / row indices
  size_t wexp;                             // 4-bit weights: one projection's matrices expanded to e16
  size_t meta_bytes;
  int max_items, max_tiles;
};

int check_config(const stage_config* c) {
  if (!c) return fail(STAGE_ERR_NULL, "stage_config is NULL");
  if (c->struct_size != sizeof(stage_config))
    return fail(STAGE_ERR_CONFIG, "stage_config.struct_size %u != %zu", c->struct_size, sizeof(stage_config));
  if (c->num_layers < 1 || c->num_q_heads < 1 || c->num_kv_heads < 1)
    return fail(STAGE_ERR_CONFIG, "non-positive dimension in stage_config");
  if (c->hidden < 64 || c->ffn < 64) return fail(STAGE_ERR_CONFIG, "hidden and ffn must be at least 64");
  if (c->kv_block_size != 16) return fail(STAGE_ERR_CONFIG, "kv_block_size must be 16, got %d", c->kv_block_size);
  if (c->head_dim != 64 && c->head_dim != 128)
    return fail(STAGE_ERR_CONFIG, "head_dim must be 64 or 128, got %d", c->head_dim);
  if (c->hidden % 8 || c->ffn % 8) return fail(STAGE_ERR_CONFIG, "hidden and ffn must be multiples of 8");
  if (c->num_q_heads % c->num_kv_heads) return fail(STAGE_ERR_CONFIG, "num_q_heads must be a multiple of num_kv_heads");
  if (c->num_q_heads / c->num_kv_heads > 16)
    return fail(STAGE_ERR_CONFIG, "at most 16 query heads per KV head are supported");
  if (!(c->rms_eps > 0.f) || !(c->rope_theta > 1.f)) return fail(STAGE_ERR_CONFIG, "rms_eps must be > 0 and rope_theta > 1");
  if (c->activation_planes < 0 || c->activation_planes > 4)
    return fail(STAGE_ERR_CONFIG, "activation_planes must be 0 (automatic), 1, 2, 3 or 4 (half activations)");
  if (c->activation_planes >= 3 && kElemIsF16)
    return fail(STAGE_ERR_CONFIG, "activation_planes 3 and 4 (half activations) are modes of the bfloat16 library; this one stores half already");
  if (c->vocab_size != 0 && (c->vocab_size < 64 || c->vocab_size % 8))
    return fail(STAGE_ERR_CONFIG, "vocab_size must be 0 or a multiple of 8 that is at least 64");
  if (c->rope_interleaved != 0 && c->rope_interleaved != 1)
    return fail(STAGE_ERR_CONFIG, "rope_interleaved must be 0 or 1, got %d", c->rope_interleaved);
  if (c->weight_copies != 0 && c->weight_copies != 1)
    return fail(STAGE_ERR_CONFIG, "weight_copies must be 0 (keep copies in operand order) or 1 (none), got %d", c->weight_copies);
  if (c->norm_kind != 0 && c->norm_kind != 1)
    return fail(STAGE_ERR_CONFIG, "norm_kind must be 0 (RMSNorm) or 1 (LayerNorm), got %d", c->norm_kind);
  if (c->mlp_kind < 0 || c->mlp_kind > 2)
    return fail(STAGE_ERR_CONFIG, "mlp_kind must be 0 (gated, SiLU), 1 (ungated, tanh GELU) or 2 (ungated, erf GELU), got %d", c->mlp_kind);
  if (c->parallel_block != 0 && c->parallel_block != 1)
    return fail(STAGE_ERR_CONFIG, "parallel_block must be 0 or 1, got %d", c->parallel_block);
  if (c->rope_scaling < 0 || c->rope_scaling > 2)
    return fail(STAGE_ERR_CONFIG, "rope_scaling must be 0 (none), 1 (linear) or 2 (by wavelength), got %d", c->rope_scaling);
  if (c->rope_scaling == 0 && (c->rope_scaling_factor != 0.f || c->rope_low_freq_factor != 0.f ||
                               c->rope_high_freq_factor != 0.f || c->rope_original_max_position != 0))
    return fail(STAGE_ERR_CONFIG, "the rope scaling parameters must be 0 unless rope_scaling is set");
  if (c->rope_scaling != 0 && !(c->rope_scaling_factor >= 1.f))
    return fail(STAGE_ERR_CONFIG, "rope_scaling_factor must be at least 1");
  if (c->rope_scaling == 1 && (c->rope_low_freq_factor != 0.f || c->rope_high_freq_factor != 0.f || c->rope_original_max_position != 0))
    return fail(STAGE_ERR_CONFIG, "linear rope scaling takes rope_scaling_factor only");
  if (c->rope_scaling == 2 && (!(c->rope_low_freq_factor > 0.f) || !(c->rope_high_freq_factor > c->rope_low_freq_factor) ||
                               c->rope_original_max_position < 1))
    return fail(STAGE_ERR_CONFIG, "rope scaling by wavelength needs 0 < rope_low_freq_factor < rope_high_freq_factor and a positive rope_original_max_position");
  if (c->weight_bits == 4 && (c->mlp_kind != 0 || c->parallel_block != 0))
    return fail(STAGE_ERR_CONFIG, "4-bit weights are supported for the gated, sequential block only (mlp_kind 0, parallel_block 0)");
  if (c->weight_bits != 0 && c->weight_bits != 16 && c->weight_bits != 4)
    return fail(STAGE_ERR_CONFIG, "weight_bits must be 0, 16 or 4, got %d", c->weight_bits);
  if (c->weight_bits == 4) {
    const int g = c->weight_group_size;
    if (g != 32 && g != 64 && g != 128) return fail(STAGE_ERR_CONFIG, "weight_group_size must be 32, 64 or 128, got %d", g);
    if (c->hidden % g || c->ffn % g || (c->num_q_heads * c->head_dim) % g)
      return fail(STAGE_ERR_CONFIG, "hidden, num_q_heads*head_dim and ffn must be multiples of weight_group_size %d", g);
  } else if (c->weight_group_size != 0) {
    return fail(STAGE_ERR_CONFIG, "weight_group_size must be 0 unless weight_bits is 4");
  }
  if (c->rotary_dim != 0 && (c->rotary_dim < 16 || c->rotary_dim > c->head_dim || c->rotary_dim % 16))
    return fail(STAGE_ERR_CONFIG, "rotary_dim must be 0 or a multiple of 16 in [16, head_dim], got %d", c->rotary_dim);
  if (c->num_kv_blocks < 1 || c->max_tokens < 1 || c->max_seqs < 1 || c->max_blocks_per_seq < 1)
    return fail(STAGE_ERR_CONFIG, "capacities must be positive");
  const size_t layer_bytes = (size_t)c->num_kv_blocks * c->num_kv_heads * 16 * c->head_dim * 2 * 2;
  if (c->kv_layer_stride_bytes != 0 &&
      (c->kv_layer_stride_bytes < (int64_t)layer_bytes || c->kv_layer_stride_bytes % 256))
    return fail(STAGE_ERR_CONFIG, "kv_layer_stride_bytes must be 0 or a multiple of 256 >= %zu", layer_bytes);
  return STAGE_OK;
}

Dims dims_of(const stage_config& c) {
  Dims d;
  d.L = c.num_layers; d.H = c.hidden; d.nq = c.num_q_heads; d.nkv = c.num_kv_heads; d.d = c.head_dim; d.F = c.ffn;
  d.qkv_out = (c.num_q_heads + 2 * c.num_kv_heads) * c.head_dim;
  d.g = c.num_q_heads / c.num_kv_heads;
  d.rd = c.rotary_dim == 0 ? c.head_dim : c.rotary_dim;
  return d;
}

// Number of compute units the work decomposition is sized for.  The library targets MI355X only.
constexpr int kNumCus = 256;

// One bfloat16 rounding per GEMM input costs about 2.8e-3 relative error per layer on the residual
// stream; the errors of the layers add in quadrature (8.0e-3 measured at eight layers, 9.5e-3 on the rows of
// a long prefill chunk at seven), which leaves no margin to the 1e-2 relative-L2 budget on the stage output
// from about five layers on.  Two ways to carry more bits (stage_config.activation_planes):
//  - two planes (2): every GEMM input - both norm outputs, the attention output, silu(gate)*up - and the
//    rotated queries as two e16 planes, value = hi + lo, both multiplied into the same accumulators:
//    sixteen bits at twice the matrix work of the projections.
//  - half activations (3, bfloat16 library): every GEMM input is kept as IEEE half (eleven significant
//    bits) in the same buffers and the GEMMs convert the bfloat16 weight fragments to half in registers,
//    which is exact; the matrix work stays what it is.  The rotated queries keep a second bfloat16 plane
//    for the attention kernels, whose cache operands are bfloat16.
// Mode 4 is mode 3 that, for micro-batches with prefill chunks, also gives the q/k/v projection's input - the
// first norm's output - a second half plane: the rows of a chunk that attend to few keys amplify input rounding about ninefold,
// mostly through keys and values that land on the other side of a rounding boundary of the bfloat16 cache
// (measured on 20 layers, a chunk with a short cached prefix: relative error of its rows 1.2e-2 with one
// half plane everywhere, its largest error above the max-abs bar; decode rows 3.0e-3).  Left to the library (0),
// a bfloat16 stage takes one bfloat16 plane up to four layers, half activations (3) from five, and mode 4 from
// nine.  The half-precision library keeps three more mantissa bits in e16 itself and chooses none of this.
constexpr int kHalfFromLayers = 5;       // automatic mode: half activations from this depth on
constexpr int kQkvPlaneFromLayers = 9;   // automatic mode: also the second half plane of the q/k/v input
// the mode a configuration runs in: its own, or by depth when left to the library
int mode_of(const stage_config& c) {
  if (c.activation_planes != 0) return c.activation_planes;
  if (kElemIsF16) return 1;
  return c.num_layers >= kQkvPlaneFromLayers ? 4 : (c.num_layers >= kHalfFromLayers ? 3 : 1);
}
// workspace: are the second planes of the GEMM inputs / of the rotated queries laid out?
bool lo_planes_of(const stage_config& c) { return mode_of(c) == 2; }
bool norm1_lo_plane_of(const stage_config& c) { return mode_of(c) == 2 || mode_of(c) == 4; }
bool q_lo_plane_of(const stage_config& c) { return mode_of(c) >= 2; }
// per micro-batch
bool half_act_of(const stage_config& c) { return !kElemIsF16 && mode_of(c) >= 3; }
bool two_plane_of(const stage_config& c) { return mode_of(c) == 2; }
// half activations: does the q/k/v projection's input get a second (half) plane?
bool qkv_lo_of(const stage_config& c, bool has_prefill) { return mode_of(c) == 4 && has_prefill; }

int decode_target_items(const Dims& d) { return (kNumCus * kDecodeWavesPerCu + d.nkv - 1) / d.nkv; }

// Second copies of the projection weights in operand order (gemm_tile_arranged_kernel), behind the workspace proper.
// Possible whenever the weights are 16-bit and the stage runs one activation plane; made when the stage can see a
// micro-batch of more than 64 rows (smaller ones never use them).  A matrix whose K is not a multiple of 256 has none.
constexpr size_t kNoCopy = ~(size_t)0;
struct CopyLayout {
  size_t qkv, o, gate, up, down;   // byte offsets inside one layer's copies, or kNoCopy
  size_t per_layer;                // bytes per layer (0: nothing is copied)
};
bool copies_possible(const stage_config& c) { return c.weight_copies == 0 && c.weight_bits != 4 && !two_plane_of(c); }

CopyLayout copy_layout_of(const stage_config& c) {
  const Dims d = dims_of(c);
  CopyLayout cl{kNoCopy, kNoCopy, kNoCopy, kNoCopy, kNoCopy, 0};
  if (!copies_possible(c) || c.max_tokens <= 64) return cl;
  size_t off = 0;
  auto take = [&](int n, int k) {
    if (!arranged_weights_supported(k)) return kNoCopy;
    const size_t o = off;
    off += align_up(arranged_weights_elems(n, k) * 2);
    return o;
  };
  cl.qkv = take(d.qkv_out, d.H);
  cl.o = take(d.H, d.nq * d.d);
  cl.gate = c.mlp_kind == 0 ? take(d.F, d.H) : kNoCopy;
  cl.up = take(d.F, d.H);
  cl.down = take(d.H, d.F);
  cl.per_layer = off;
  return cl;
}

WorkspaceLayout layout_of(const stage_config& c) {
  const Dims d = dims_of(c);
  WorkspaceLayout w;
  const size_t T = (size_t)c.max_tokens;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  w.x = take(T * d.H * 4);
  w.a = take(T * d.H * 2);
  w.a_lo = take(norm1_lo_plane_of(c) ? T * d.H * 2 : 0);
  w.qkv_f32 = take(T * d.qkv_out * 4);
  w.qkv = take(T * d.qkv_out * 2);
  w.q_lo = take(q_lo_plane_of(c) ? T * d.nq * d.d * 2 : 0);
  w.attn = take(T * d.nq * d.d * 2);
  w.attn_lo = take(lo_planes_of(c) ? T * d.nq * d.d * 2 : 0);
  w.mlp = take(T * d.F * 2);
  w.mlp_lo = take(lo_planes_of(c) ? T * d.F * 2 : 0);
  w.cos_sin = take(T * (d.d / 2) * 8);
  w.b2 = take(c.parallel_block ? T * d.H * 2 : 0);
  w.b2_lo = take(c.parallel_block && lo_planes_of(c) ? T * d.H * 2 : 0);
  w.up_f32 = take(c.mlp_kind != 0 ? T * d.F * 4 : 0);
  // split-K scratch for every way the projections may be planned: as for one activation plane, and - with two
  // planes, or with half activations, whose decode-sized projections take the two-plane plans' 64-row tiles -
  // as for two
  size_t pf = 0, v;
  for (int sp = 0; sp < 2; ++sp) {
    if (sp == 1 && !(lo_planes_of(c) || half_act_of(c))) continue;
    if (sp == 0 && lo_planes_of(c)) continue;
    for (int arr = 0; arr < 2; ++arr) {      // with and without the copies in operand order (whether a call has them
      if (arr && (sp || !copies_possible(c))) continue;   // depends on the handle, not on the capacity this is sized for)
      if ((v = gemm_partial_floats(c.max_tokens, d.qkv_out, d.H, kEpiStoreF32, kNumCus, sp, arr)) > pf) pf = v;
      if ((v = gemm_partial_floats(c.max_tokens, d.H, d.nq * d.d, kEpiResidualF32, kNumCus, sp, arr)) > pf) pf = v;
      if ((v = gemm_partial_floats(c.max_tokens, d.F, d.H, c.mlp_kind == 0 ? kEpiSwiGLU : kEpiStoreF32, kNumCus, sp, arr)) > pf) pf = v;
      if ((v = gemm_partial_floats(c.max_tokens, d.H, d.F, kEpiResidualF32, kNumCus, sp, arr)) > pf) pf = v;
    }
  }
  if (c.vocab_size > 0 && (v = gemm_partial_floats(c.max_seqs, c.vocab_size, d.H, kEpiStoreF32, kNumCus, false)) > pf) pf = v;
  if (c.weight_bits == 4) {   // the tiles that read 4-bit weights as stored plan on their own
    if ((v = gemm_partial_floats_w4_tile(c.max_tokens, d.qkv_out, d.H, kEpiStoreF32, kNumCus)) > pf) pf = v;
    if ((v = gemm_partial_floats_w4_tile(c.max_tokens, d.H, d.nq * d.d, kEpiResidualF32, kNumCus)) > pf) pf = v;
    if ((v = gemm_partial_floats_w4_tile(c.max_tokens, d.F, d.H, kEpiSwiGLU, kNumCus)) > pf) pf = v;
    if ((v = gemm_partial_floats_w4_tile(c.max_tokens, d.H, d.F, kEpiResidualF32, kNumCus)) > pf) pf = v;
  }
  w.splitk = take(pf * 4 + 16);
  w.splitk_floats = pf;
  // 4-bit weights: room for the largest projection (gate and up together) expanded to e16
  {
    size_t elems = (size_t)d.qkv_out * d.H;
    if ((size_t)2 * d.F * d.H > elems) elems = (size_t)2 * d.F * d.H;
    w.wexp = take(c.weight_bits == 4 ? elems * 2 : 0);
  }
  w.head_a = take(c.vocab_size > 0 ? (size_t)c.max_seqs * d.H * 2 : 0);
  w.head_logits = take(c.vocab_size > 0 ? (size_t)c.max_seqs * c.vocab_size * 4 : 0);
  w.ends_meta = take((T > (size_t)c.max_seqs ? T : (size_t)c.max_seqs) * 4 + 256);
  w.max_items = decode_target_items(d) + c.max_seqs;
  w.part_o = take((size_t)w.max_items * d.nq * d.d * 4);
  w.part_ml = take((size_t)w.max_items * d.nq * 8);
  w.max_tiles = (int)((T * d.g + 31) / 32) + c.max_seqs;
  size_t mb = 0;
  mb += align_up(T * 4);                                                    // positions
  mb += align_up(T * 8);                                                    // slots
  mb += align_up((size_t)c.max_seqs * c.max_blocks_per_seq * 4);            // flat block tables
  mb += align_up((size_t)w.max_items * sizeof(DecodeItem));
  mb += align_up((size_t)c.max_seqs * sizeof(DecodeToken));
  mb += align_up((size_t)w.max_tiles * sizeof(PrefillTile));
  w.meta_bytes = mb;
  w.meta = take(mb);
  w.total = off;
  return w;
}

struct BatchCounts {
  int64_t total_blocks, decode_keys;
  int n_decode, n_tiles;
};

// Host-only checks of a micro-batch against the stage's capacities; also counts the work.
int validate_batch(const stage_config& c, int32_t T, const int32_t* positions, int32_t S, const int32_t* q_lens,
                   const int32_t* ctx_lens, const int32_t* block_tables, BatchCounts* out) {
  if (!positions || !q_lens || !ctx_lens || !block_tables) return fail(STAGE_ERR_NULL, "a metadata array is NULL");
  if (T < 1 || T > c.max_tokens) return fail(STAGE_ERR_BATCH, "num_tokens %d outside [1, max_tokens=%d]", T, c.max_tokens);
  if (S < 1 || S > c.max_seqs) return fail(STAGE_ERR_BATCH, "num_seqs %d outside [1, max_seqs=%d]", S, c.max_seqs);
  const int g = c.num_q_heads / c.num_kv_heads;
  BatchCounts bc{0, 0, 0, 0};
  int64_t sum_q = 0;
  for (int s = 0; s < S; ++s) {
    const int q = q_lens[s], cx = ctx_lens[s];
    if (q < 1) return fail(STAGE_ERR_BATCH, "q_lens[%d] = %d must be >= 1", s, q);
    if (cx < 0) return fail(STAGE_ERR_BATCH, "ctx_lens[%d] = %d must be >= 0", s, cx);
    const int64_t tot = (int64_t)q + cx;
    const int64_t nb = (tot + 15) / 16;
    if (nb > c.max_blocks_per_seq)
      return fail(STAGE_ERR_BLOCK_TABLE, "sequence %d needs %lld blocks, block table rows hold %d", s, (long long)nb,
                  c.max_blocks_per_seq);
    const int32_t* row = block_tables + (size_t)s * c.max_blocks_per_seq;
    for (int b = 0; b < nb; ++b)
      if (row[b] < 0 || row[b] >= c.num_kv_blocks)
        return fail(STAGE_ERR_BLOCK_TABLE, "block_tables[%d][%d] = %d outside [0, %d)", s, b, row[b], c.num_kv_blocks);
    sum_q += q;
    bc.total_blocks += nb;
    if (q == 1) { ++bc.n_decode; bc.decode_keys += tot; }
    else bc.n_tiles += (int)(((int64_t)q * g + 127) / 128);
  }
  if (sum_q != T) return fail(STAGE_ERR_BATCH, "sum(q_lens) = %lld != num_tokens = %d", (long long)sum_q, T);
  for (int t = 0; t < T; ++t)
    if (positions[t] < 0) return fail(STAGE_ERR_BATCH, "positions[%d] = %d must be >= 0", t, positions[t]);
  *out = bc;
  return STAGE_OK;
}

void fill_slot_mapping(const stage_config& c, int32_t S, const int32_t* q_lens, const int32_t* ctx_lens,
                       const int32_t* block_tables, int64_t* slots) {
  int row = 0;
  for (int s = 0; s < S; ++s) {
    const int32_t* tab = block_tables + (size_t)s * c.max_blocks_per_seq;
    for (int i = 0; i < q_lens[s]; ++i) {
      const int j = ctx_lens[s] + i;
      slots[row++] = (int64_t)tab[j / 16] * 16 + j % 16;
    }
  }
}

struct TimedLaunch {
  hipEvent_t begin, end;
  int kernel;
};

}  // namespace

struct stage_handle {
  stage_config cfg;
  Dims dim;
  WorkspaceLayout ws;
  std::vector<stage_layer_weights> layers;
  char* kv_pool;
  char* workspace;
  char* static_scratch;                 // this device's copy of the library's static scratch array
  // workspace and layout of the call being enqueued (the handle's own, or the static scratch carved for the call)
  char* call_ws;
  const WorkspaceLayout* call_layout;
  // the weights' copies in operand order: layer l's start at wcopy + l * copies.per_layer (wcopy NULL: none were made)
  char* wcopy;
  CopyLayout copies;
  int device;
  // pinned staging ring for the per-call metadata
  char* staging[kStagingSlots];
  hipEvent_t staging_done[kStagingSlots];
  bool staging_used[kStagingSlots];
  int next_slot;
  // timing
  uint32_t profile_mask;
  std::vector<TimedLaunch> timed;       // recorded, not yet read
  std::vector<TimedLaunch> free_events; // recycled event pairs
};

namespace {

struct Timer {
  stage_handle* st;
  hipStream_t stream;
  bool on;
  TimedLaunch cur;
  Timer(stage_handle* s, hipStream_t str, int kernel) : st(s), stream(str), on(false) {
    if (!((s->profile_mask >> kernel) & 1u) || (int)s->timed.size() >= kMaxTimed) return;
    if (!s->free_events.empty()) {
      cur = s->free_events.back();
      s->free_events.pop_back();
    } else {
      if (hipEventCreate(&cur.begin) != hipSuccess) return;
      if (hipEventCreate(&cur.end) != hipSuccess) { (void)hipEventDestroy(cur.begin); return; }
    }
    cur.kernel = kernel;
    on = hipEventRecord(cur.begin, stream) == hipSuccess;
    if (!on) st->free_events.push_back(cur);
  }
  ~Timer() {
    if (!on) return;
    (void)hipEventRecord(cur.end, stream);
    st->timed.push_back(cur);
  }
};

__global__ __launch_bounds__(256) void f32_to_e16_kernel(const float* __restrict__ src, e16* __restrict__ dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = static_cast<e16>(src[i]);
}

// IEEE half bits -> e16, for the taps of a stage that keeps its GEMM inputs as half
__global__ __launch_bounds__(256) void half_bits_to_e16_kernel(const e16* __restrict__ src, e16* __restrict__ dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = f32_to_e16(static_cast<float>(__builtin_bit_cast(h16, src[i])));
}

// A tap of a GEMM input: a plain copy, or a conversion when the stage holds it as half.
hipError_t copy_activation_tap(void* dst, const e16* src, size_t n, bool src_half, hipStream_t stream) {
  if (!src_half) return hipMemcpyAsync(dst, src, n * 2, hipMemcpyDeviceToDevice, stream);
  hipLaunchKernelGGL(half_bits_to_e16_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, src, (e16*)dst, n);
  return hipGetLastError();
}

// Whether the operands of a stage's matrix instructions are IEEE half: the half-precision library, or half
// activations in the bfloat16 one.
bool operands_half_of(const stage_config& c) { return kElemIsF16 != 0 || half_act_of(c); }

// Points a projection's GEMM at its weights.  e16 weights are used where they lie (and, where the stage keeps a copy
// in operand order, there too).  4-bit weights are read as
// they are stored by the weight-streaming kernel (decode-sized micro-batches) and by the 4-bit tiles (more rows,
// half operands); otherwise they are expanded to e16 in the workspace first (one projection at a time; `w1` is
// the second matrix of the gate/up pair or NULL) and the GEMM reads the expanded copy.
int bind_weights(stage_handle* st, hipStream_t stream, GemmArgs& g, const void* w0, const void* s0, const void* z0,
                 const void* w1, const void* s1, const void* z1, int layer, size_t copy0, size_t copy1) {
  if (st->cfg.weight_bits != 4) {
    g.w0 = (const e16*)w0;
    g.w1 = (const e16*)w1;
    // the copies in operand order, where the stage keeps them (plans of the kind that reads them exist only then)
    if (st->wcopy && copy0 != kNoCopy) {
      const char* base = st->wcopy + (size_t)layer * st->copies.per_layer;
      g.wa0 = (const e16*)(base + copy0);
      if (w1) g.wa1 = (const e16*)(base + copy1);
    }
    return STAGE_OK;
  }
  const W4Matrix m0{(const uint32_t*)w0, (const e16*)s0, (const e16*)z0};
  if (skinny_w4_supports(g.m, g.k, st->cfg.weight_group_size, g.a_lo != nullptr) ||
      tile_w4_supports(g.m, g.k, st->cfg.weight_group_size, g.a_lo != nullptr, g.a_half || kElemIsF16 != 0)) {
    // the kernel the projection was planned on reads the stored form itself
    g.q0 = m0;
    if (w1) g.q1 = W4Matrix{(const uint32_t*)w1, (const e16*)s1, (const e16*)z1};
    return STAGE_OK;
  }
  e16* exp0 = (e16*)(st->call_ws + st->call_layout->wexp);
  Timer t(st, stream, STAGE_K_DEQUANT);
  HIP_TRY(launch_dequant_w4(m0, g.n, g.k, st->cfg.weight_group_size, exp0, stream));
  g.w0 = exp0;
  if (w1) {
    e16* exp1 = exp0 + (size_t)g.n * g.k;
    const W4Matrix m1{(const uint32_t*)w1, (const e16*)s1, (const e16*)z1};
    HIP_TRY(launch_dequant_w4(m1, g.n, g.k, st->cfg.weight_group_size, exp1, stream));
    g.w1 = exp1;
  }
  return STAGE_OK;
}

// The plan of a projection.  4-bit weights with more than 64 rows and half operands: the tiles that read the stored
// form.  At most 64 rows: 4-bit weights in their stored form need the streaming kernel; otherwise the shape decides
// between it and the 64-row tiles.
GemmPlan plan_projection(const stage_config& c, int m, int n, int k, GemmEpilogue epi, bool two_planes, bool arranged) {
  if (c.weight_bits == 4 && tile_w4_supports(m, k, c.weight_group_size, two_planes, operands_half_of(c)))
    return plan_gemm_w4_tile(m, n, k, epi, kNumCus);
  const bool stored_w4 = c.weight_bits == 4 && skinny_w4_supports(m, k, c.weight_group_size, two_planes);
  return plan_gemm(m, n, k, epi, kNumCus, two_planes, stored_w4 ? kFewRowsStreaming : kFewRowsByShape, arranged);
}

// The plans of a layer's four projections for one micro-batch; they depend on the shapes only, so they are made -
// and checked against the workspace - once per call, before anything is enqueued.
struct LayerPlans {
  GemmPlan qkv, o, gateup, down, down_out;   // down_out: the last layer's down projection writing the payload
};

// The partial sums a plan writes must fit the scratch the workspace was laid out with.
int check_plan(const stage_handle* st, int m, const GemmPlan& plan) {
  if (!plan.partials) return STAGE_OK;
  const size_t need = (size_t)plan.splits * m * plan.nv;
  if (need > st->call_layout->splitk_floats)
    return fail(STAGE_ERR_SIZE, "internal: a projection's plan needs %zu floats of split-K scratch, the workspace holds %zu",
                need, st->call_layout->splitk_floats);
  return STAGE_OK;
}

int plan_layer(const stage_handle* st, int T, bool qkv_two_planes, bool two_planes, LayerPlans* out) {
  const stage_config& c = st->cfg;
  const Dims& d = st->dim;
  const CopyLayout& cl = st->copies;
  const bool have = st->wcopy != nullptr;     // copies in operand order: a projection may be planned on the kernel that reads them
  out->qkv = plan_projection(c, T, d.qkv_out, d.H, kEpiStoreF32, qkv_two_planes, have && cl.qkv != kNoCopy);
  out->o = plan_projection(c, T, d.H, d.nq * d.d, kEpiResidualF32, two_planes, have && cl.o != kNoCopy);
  out->gateup = c.mlp_kind == 0 ? plan_projection(c, T, d.F, d.H, kEpiSwiGLU, two_planes, have && cl.gate != kNoCopy)
                                : plan_projection(c, T, d.F, d.H, kEpiStoreF32, two_planes, have && cl.up != kNoCopy);
  out->down = plan_projection(c, T, d.H, d.F, kEpiResidualF32, two_planes, have && cl.down != kNoCopy);
  out->down_out = plan_projection(c, T, d.H, d.F, kEpiResidualOut, two_planes, have && cl.down != kNoCopy);
  for (const GemmPlan* p : {&out->qkv, &out->o, &out->gateup, &out->down, &out->down_out})
    if (int rc = check_plan(st, T, *p)) return rc;
  return STAGE_OK;
}

int run_gemm(stage_handle* st, hipStream_t stream, int kernel_class, const GemmArgs& args, GemmEpilogue epi,
             const GemmPlan& plan) {
  {
    Timer t(st, stream, kernel_class);
    HIP_TRY(launch_gemm_main(args, epi, plan, stream));
  }
  if (plan.partials) {
    Timer t(st, stream, STAGE_K_SPLITK_REDUCE);
    HIP_TRY(launch_gemm_reduce(args, epi, plan, stream));
  }
  return STAGE_OK;
}

// A projection whose result is added to the fp32 residual stream x, followed by what consumes x next:
// a norm into `norm_out` (norm.gain != nullptr), or nothing.  When the GEMM splits K across workgroups
// the sum of the partial results, the residual add and the norm run as one kernel.
int run_residual_gemm(stage_handle* st, hipStream_t stream, int kernel_class, const GemmArgs& args, GemmEpilogue epi,
                      const GemmPlan& plan, const NormSpec& norm, e16* norm_out, e16* norm_out_lo, bool norm_out_half) {
  const e16* gain = norm.gain;
  {
    Timer t(st, stream, kernel_class);
    HIP_TRY(launch_gemm_main(args, epi, plan, stream));
  }
  const bool fused = plan.partials && (gain != nullptr || epi == kEpiResidualOut);
  if (fused) {
    Timer t(st, stream, STAGE_K_SPLITK_REDUCE);
    HIP_TRY(launch_gemm_reduce_residual_norm(args, epi, plan, norm, norm_out, norm_out_lo, norm_out_half, stream));
    return STAGE_OK;
  }
  if (plan.partials) {
    Timer t(st, stream, STAGE_K_SPLITK_REDUCE);
    HIP_TRY(launch_gemm_reduce(args, epi, plan, stream));
  }
  if (gain) {
    Timer t(st, stream, STAGE_K_RMSNORM);
    HIP_TRY(launch_rmsnorm(nullptr, args.resid, norm, norm_out, norm_out_lo, args.m, args.n, false, norm_out_half, stream));
  }
  return STAGE_OK;
}

int forward_impl(stage_handle* st, void* hip_stream, int32_t T, const void* hidden_in, const int32_t* positions,
                 int32_t S, const int32_t* q_lens, const int32_t* ctx_lens, const int32_t* block_tables,
                 void* hidden_out, int64_t* slot_mapping_out, const stage_taps* taps, bool use_static_scratch = false) {
  if (!st) return fail(STAGE_ERR_NULL, "stage handle is NULL");
  if (!hidden_in || !positions || !q_lens || !ctx_lens || !block_tables || !hidden_out)
    return fail(STAGE_ERR_NULL, "a required argument of stage_forward is NULL");
  // whatever workspace this call uses, the handle points at its own again when the call returns
  struct CallWorkspaceReset {
    stage_handle* st;
    ~CallWorkspaceReset() { st->call_ws = st->workspace; st->call_layout = &st->ws; }
  } reset_call_workspace{st};
  const stage_config& c = st->cfg;
  const Dims& d = st->dim;
  if (taps && (taps->tap_layer < 0 || taps->tap_layer >= d.L))
    return fail(STAGE_ERR_BATCH, "tap_layer %d outside [0, %d)", taps->tap_layer, d.L);
  if (T >= 1) {
    const char* in0 = (const char*)hidden_in;
    const char* out0 = (const char*)hidden_out;
    const size_t bytes = (size_t)T * d.H * 2;
    if (in0 < out0 + bytes && out0 < in0 + bytes) return fail(STAGE_ERR_ALIAS, "hidden_out overlaps hidden_in");
  }

  // ---- validate the micro-batch and size the metadata (host only, nothing enqueued yet)
  BatchCounts bc;
  {
    int rc = validate_batch(c, T, positions, S, q_lens, ctx_lens, block_tables, &bc);
    if (rc) return rc;
  }
  const int64_t total_blocks = bc.total_blocks, decode_keys = bc.decode_keys;
  const int n_decode = bc.n_decode, n_tiles = bc.n_tiles;

  // ---- the workspace of this call: the handle's, or the static scratch carved for exactly this micro-batch
  WorkspaceLayout carved;
  st->call_ws = st->workspace;
  st->call_layout = &st->ws;
  if (use_static_scratch) {
    stage_config rc = c;
    rc.max_tokens = T;
    rc.max_seqs = S;
    rc.vocab_size = 0;
    carved = layout_of(rc);
    if (carved.total > kStaticScratchBytes)
      return fail(STAGE_ERR_SIZE, "this micro-batch needs %zu bytes of scratch; the static scratch holds %zu", carved.total,
                  kStaticScratchBytes);
    if (carved.meta_bytes > st->ws.meta_bytes) return fail(STAGE_ERR_SIZE, "internal: metadata staging too small");
    st->call_ws = st->static_scratch;
    st->call_layout = &carved;
  }
  const WorkspaceLayout& wl = *st->call_layout;

  // key-range length of the decode work items: aim at a fixed number of items, never below the minimum
  int range = kMinDecodeRange;
  if (n_decode) {
    const int64_t target = decode_target_items(d);
    int64_t r = (decode_keys + target - 1) / target;
    r = (r + 31) / 32 * 32;
    if (r > range) range = (int)r;
  }
  int n_items = 0;
  for (int s = 0; s < S; ++s)
    if (q_lens[s] == 1) n_items += (ctx_lens[s] + 1 + range - 1) / range;
  if (n_items > wl.max_items || n_tiles > wl.max_tiles)
    return fail(STAGE_ERR_BATCH, "internal: work list larger than planned (%d items, %d tiles)", n_items, n_tiles);

  // the projections' plans (they depend on the shapes only) and their fit into the workspace
  const bool two_plane = two_plane_of(c);
  const bool half_act = half_act_of(c);                // GEMM inputs as IEEE half bits (bfloat16 library)
  const bool qkv_lo = half_act && qkv_lo_of(c, n_tiles > 0);
  LayerPlans plans;
  if (int rc = plan_layer(st, T, two_plane || qkv_lo, two_plane, &plans)) return rc;
  // The q/k/v input's second plane is there for the rows of prefill chunks.  When chunk rows and decode rows lie in a
  // few contiguous runs (a scheduler that puts its chunks first or last gives two), every run gets its own product:
  // chunk rows with both planes, decode rows with one - on the kernel that reads the weights' copy in operand order
  // where the stage keeps one.  Otherwise one product with both planes covers all rows.
  struct QkvRun { int row0, rows; bool two_planes; GemmPlan plan; };
  std::vector<QkvRun> qkv_runs;
  if (qkv_lo && !two_plane) {
    int row = 0, decode_rows = 0;
    for (int s = 0; s < S; ++s) {
      const bool chunk = q_lens[s] > 1;
      if (!qkv_runs.empty() && qkv_runs.back().two_planes == chunk) qkv_runs.back().rows += q_lens[s];
      else qkv_runs.push_back(QkvRun{row, q_lens[s], chunk, GemmPlan{}});
      row += q_lens[s];
      if (!chunk) ++decode_rows;
    }
    // below about 128 decode rows the products are bound by the weight stream, and two products read it twice
    constexpr int kMaxQkvRuns = 4, kMinDecodeRows = 128;
    if (qkv_runs.size() < 2 || qkv_runs.size() > kMaxQkvRuns || decode_rows < kMinDecodeRows) qkv_runs.clear();
    const bool copy = st->wcopy != nullptr && st->copies.qkv != kNoCopy;
    for (QkvRun& r : qkv_runs) {
      r.plan = plan_projection(c, r.rows, d.qkv_out, d.H, kEpiStoreF32, r.two_planes, copy && !r.two_planes);
      if (int rc = check_plan(st, r.rows, r.plan)) return rc;
    }
  }

  HIP_TRY(hipSetDevice(st->device));
  hipStream_t stream = (hipStream_t)hip_stream;

  // ---- build the metadata blob in a pinned staging slot
  const int slot_id = st->next_slot;
  st->next_slot = (st->next_slot + 1) % kStagingSlots;
  if (st->staging_used[slot_id]) HIP_TRY(hipEventSynchronize(st->staging_done[slot_id]));
  char* blob = st->staging[slot_id];
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  const size_t o_pos = take((size_t)T * 4), o_slots = take((size_t)T * 8), o_bt = take((size_t)total_blocks * 4);
  const size_t o_items = take((size_t)n_items * sizeof(DecodeItem));
  const size_t o_dtok = take((size_t)n_decode * sizeof(DecodeToken));
  const size_t o_tiles = take((size_t)n_tiles * sizeof(PrefillTile));
  if (off > wl.meta_bytes) return fail(STAGE_ERR_BATCH, "internal: metadata larger than planned");
  int32_t* h_pos = (int32_t*)(blob + o_pos);
  int64_t* h_slots = (int64_t*)(blob + o_slots);
  int32_t* h_bt = (int32_t*)(blob + o_bt);
  DecodeItem* h_items = (DecodeItem*)(blob + o_items);
  DecodeToken* h_dtok = (DecodeToken*)(blob + o_dtok);
  PrefillTile* h_tiles = (PrefillTile*)(blob + o_tiles);
  memcpy(h_pos, positions, (size_t)T * 4);
  {
    int row = 0, bt_off = 0, it = 0, dt = 0, tl = 0;
    for (int s = 0; s < S; ++s) {
      const int q = q_lens[s], cx = ctx_lens[s];
      const int nb = (q + cx + 15) / 16;
      const int32_t* tab = block_tables + (size_t)s * c.max_blocks_per_seq;
      memcpy(h_bt + bt_off, tab, (size_t)nb * 4);
      for (int i = 0; i < q; ++i) {
        const int j = cx + i;
        h_slots[row + i] = (int64_t)tab[j / 16] * 16 + j % 16;
      }
      if (q == 1) {
        const int keys = cx + 1;
        const int n = (keys + range - 1) / range;
        h_dtok[dt++] = DecodeToken{row, it, n, 0};
        // the sequence's ranges get equal lengths (a multiple of 32 keys) instead of n - 1 full ones and a
        // short remainder: less spread between the work items
        const int len = ((keys + n - 1) / n + 31) / 32 * 32;
        for (int k = 0; k < n; ++k) {
          const int kb = k * len;
          const int ke = kb + len < keys ? kb + len : keys;
          h_items[it] = DecodeItem{row, bt_off, kb, ke, it, keys - 1, {0, 0}};
          ++it;
        }
      } else {
        const int ncols = q * d.g;
        for (int c0 = 0; c0 < ncols; c0 += 128) h_tiles[tl++] = PrefillTile{row, q, cx, bt_off, c0, {0, 0, 0}};
      }
      row += q;
      bt_off += nb;
    }
  }
  // longest key ranges first, so the short ones fill the tail of the launch
  if (n_items > 1)
    std::stable_sort(h_items, h_items + n_items, [](const DecodeItem& x, const DecodeItem& y) {
      return (x.key_end - x.key_begin) > (y.key_end - y.key_begin);
    });
  // prefill tiles that see the most keys first (a late tile of a long chunk runs twice as long as an early one)
  if (n_tiles > 1) {
    const int gq = d.g;
    std::stable_sort(h_tiles, h_tiles + n_tiles, [gq](const PrefillTile& x, const PrefillTile& y) {
      return x.ctx + (x.col0 + 127) / gq > y.ctx + (y.col0 + 127) / gq;
    });
  }
  if (slot_mapping_out) memcpy(slot_mapping_out, h_slots, (size_t)T * 8);

  // ---- enqueue
  char* ws = st->call_ws;
  char* meta = ws + wl.meta;
  HIP_TRY(hipMemcpyAsync(meta, blob, off, hipMemcpyHostToDevice, stream));
  HIP_TRY(hipEventRecord(st->staging_done[slot_id], stream));
  st->staging_used[slot_id] = true;

  float* x = (float*)(ws + wl.x);
  e16* a = (e16*)(ws + wl.a);
  e16* a_lo = two_plane ? (e16*)(ws + wl.a_lo) : nullptr;
  e16* norm1_lo = (two_plane || qkv_lo) ? (e16*)(ws + wl.a_lo) : nullptr;   // second plane of the first norm's output
  e16* mlp_lo = two_plane ? (e16*)(ws + wl.mlp_lo) : nullptr;
  e16* q_lo = (two_plane || half_act) ? (e16*)(ws + wl.q_lo) : nullptr;
  e16* attn_lo = two_plane ? (e16*)(ws + wl.attn_lo) : nullptr;
  float* qkv_f32 = (float*)(ws + wl.qkv_f32);
  e16* qkv = (e16*)(ws + wl.qkv);
  e16* attn = (e16*)(ws + wl.attn);
  e16* mlp = (e16*)(ws + wl.mlp);
  float2* cos_sin = (float2*)(ws + wl.cos_sin);
  float* splitk = (float*)(ws + wl.splitk);
  float* part_o = (float*)(ws + wl.part_o);
  float2* part_ml = (float2*)(ws + wl.part_ml);
  const int32_t* d_pos = (const int32_t*)(meta + o_pos);
  const int64_t* d_slots = (const int64_t*)(meta + o_slots);
  const int32_t* d_bt = (const int32_t*)(meta + o_bt);
  const DecodeItem* d_items = (const DecodeItem*)(meta + o_items);
  const DecodeToken* d_dtok = (const DecodeToken*)(meta + o_dtok);
  const PrefillTile* d_tiles = (const PrefillTile*)(meta + o_tiles);

  // the norm in front of layer l's attention branch (second = false) or MLP branch
  auto norm_of = [&](int l, bool second) {
    const stage_layer_weights& lw = st->layers[l];
    return NormSpec{(const e16*)(second ? lw.norm2 : lw.norm1), (const e16*)(second ? lw.norm2_bias : lw.norm1_bias),
                    c.rms_eps, c.norm_kind};
  };
  const NormSpec no_norm{nullptr, nullptr, c.rms_eps, 0};
  const bool parallel = c.parallel_block != 0;
  e16* b2 = parallel ? (e16*)(ws + wl.b2) : nullptr;
  e16* b2_lo = parallel && two_plane ? (e16*)(ws + wl.b2_lo) : nullptr;
  float* up_f32 = (float*)(ws + wl.up_f32);
  const bool alibi = st->layers[0].alibi != nullptr;   // linear biases in the attention scores: nothing rotates
  const int rotating = alibi ? 0 : d.rd;
  if (rotating) {
    Timer t(st, stream, STAGE_K_ROPE_TABLE);
    HIP_TRY(launch_rope_table(d_pos, cos_sin, T, d.rd, c.rope_theta,
                              RopeScaling{c.rope_scaling, c.rope_scaling_factor, c.rope_low_freq_factor,
                                          c.rope_high_freq_factor, c.rope_original_max_position}, stream));
  }
  const size_t kv_region = (size_t)c.num_kv_blocks * d.nkv * 16 * d.d;   // elements of one K (or V) region
  {
    // the first layer's input norm also initialises the fp32 residual stream from the e16 input
    Timer t(st, stream, STAGE_K_RMSNORM);
    HIP_TRY(launch_rmsnorm((const e16*)hidden_in, x, norm_of(0, false), a, norm1_lo, T, d.H, true, half_act, stream));
  }
  for (int l = 0; l < d.L; ++l) {
    const stage_layer_weights& w = st->layers[l];
    const bool last = l == d.L - 1;
    const bool tap = taps && taps->tap_layer == l;
    e16* k_pool = (e16*)(st->kv_pool + (size_t)l * (size_t)c.kv_layer_stride_bytes);
    e16* v_pool = k_pool + kv_region;
    // `a` holds RMSNorm(x; norm1 of this layer) here
    if (tap && taps->tap_norm1) HIP_TRY(copy_activation_tap(taps->tap_norm1, a, (size_t)T * d.H, half_act, stream));
    // parallel block: the MLP branch starts from the block's input too - its norm is taken now, before the
    // attention branch is added to x (a block with one norm reads `a` in both branches)
    const bool own_norm2 = parallel && w.norm2 != nullptr;
    if (own_norm2) {
      Timer t(st, stream, STAGE_K_RMSNORM);
      HIP_TRY(launch_rmsnorm(nullptr, x, norm_of(l, true), b2, b2_lo, T, d.H, false, half_act, stream));
    }
    const e16* mlp_in = parallel ? (own_norm2 ? b2 : a) : a;
    const e16* mlp_in_lo = own_norm2 ? b2_lo : a_lo;
    // q/k/v projection, rotation and cache append of rows row0 .. row0 + rows - 1
    auto qkv_rows = [&](int row0, int rows, bool second_plane, const GemmPlan& plan) -> int {
      GemmArgs g{};
      g.a = a + (size_t)row0 * d.H; g.a_lo = second_plane ? norm1_lo + (size_t)row0 * d.H : nullptr; g.a_half = half_act;
      g.out_f32 = qkv_f32 + (size_t)row0 * d.qkv_out; g.partial = splitk;
      g.m = rows; g.n = d.qkv_out; g.k = d.H; g.lda = d.H; g.ldo = d.qkv_out;
      if (int rc = bind_weights(st, stream, g, w.wqkv, w.sqkv, w.zqkv, nullptr, nullptr, nullptr, l, st->copies.qkv, kNoCopy)) return rc;
      // the rotation kernel adds the split-K partial sums itself: no separate reduction pass
      {
        Timer t(st, stream, STAGE_K_GEMM_QKV);
        HIP_TRY(launch_gemm_main(g, kEpiStoreF32, plan, stream));
      }
      Timer t(st, stream, STAGE_K_ROPE_APPEND);
      RopeAppendArgs r{plan.partials ? splitk : g.out_f32, plan.partials ? plan.splits : 1, (size_t)rows * d.qkv_out,
                       (const e16*)w.bqkv, (const e16*)w.qnorm, (const e16*)w.knorm, c.rms_eps,
                       qkv + (size_t)row0 * d.qkv_out, q_lo ? q_lo + (size_t)row0 * d.nq * d.d : nullptr,
                       cos_sin + (size_t)row0 * (rotating / 2), d_slots + row0, k_pool, v_pool, rows, d.nq, d.nkv, d.d,
                       rotating, c.rope_interleaved};
      HIP_TRY(launch_rope_append(r, stream));
      return STAGE_OK;
    };
    if (qkv_runs.empty()) {
      if (int rc = qkv_rows(0, T, norm1_lo != nullptr, plans.qkv)) return rc;
    } else {
      for (const QkvRun& r : qkv_runs)
        if (int rc = qkv_rows(r.row0, r.rows, r.two_planes, r.plan)) return rc;
    }
    if (tap && taps->tap_qkv)
      HIP_TRY(hipMemcpyAsync(taps->tap_qkv, qkv, (size_t)T * d.qkv_out * 2, hipMemcpyDeviceToDevice, stream));
    AttnArgs aa{qkv, q_lo, k_pool, v_pool, d_bt, attn, attn_lo, d.nq, d.nkv, d.d, 1.4426950408889634f / sqrtf((float)d.d),
                half_act, (const float*)w.alibi};
    if (n_tiles) {
      Timer t(st, stream, STAGE_K_ATTN_PREFILL);
      // half activations without the q/k/v input's second plane (mode 3, stages of five to eight layers): the chunk
      // rows take the queries' first plane alone - the pipelined kernel, a quarter faster than the two-plane one, for a
      // tenth more error on those rows (2.8e-3 against 2.5e-3 relative at seven layers); decode rows and deeper stages
      // keep both planes
      AttnArgs ap = aa;
      if (mode_of(c) == 3) ap.q_lo = nullptr;
      HIP_TRY(launch_attn_prefill(ap, d_tiles, n_tiles, stream));
    }
    if (n_items) {
      {
        Timer t(st, stream, STAGE_K_ATTN_DECODE);
        HIP_TRY(launch_attn_decode(aa, d_items, n_items, part_o, part_ml, stream));
      }
      Timer t(st, stream, STAGE_K_ATTN_MERGE);
      HIP_TRY(launch_attn_merge(aa, d_dtok, n_decode, part_o, part_ml, stream));
    }
    if (tap && taps->tap_attn) HIP_TRY(copy_activation_tap(taps->tap_attn, attn, (size_t)T * d.nq * d.d, half_act, stream));
    {
      GemmArgs g{};
      g.a = attn; g.a_lo = attn_lo; g.a_half = half_act; g.resid = x; g.partial = splitk;
      g.m = T; g.n = d.H; g.k = d.nq * d.d; g.lda = d.nq * d.d; g.ldo = d.H;
      if (int rc = bind_weights(st, stream, g, w.wo, w.so, w.zo, nullptr, nullptr, nullptr, l, st->copies.o, kNoCopy)) return rc;
      if (w.bo) {        // the projection's bias joins the residual stream ahead of its product
        Timer t(st, stream, STAGE_K_SPLITK_REDUCE);
        HIP_TRY(launch_add_row_bias(x, (const e16*)w.bo, T, d.H, stream));
      }
      int rc = run_residual_gemm(st, stream, STAGE_K_GEMM_O, g, kEpiResidualF32, plans.o,
                                 parallel ? no_norm : norm_of(l, true), a, a_lo, half_act);
      if (rc) return rc;
    }
    if (tap && taps->tap_h)
      HIP_TRY(hipMemcpyAsync(taps->tap_h, x, (size_t)T * d.H * 4, hipMemcpyDeviceToDevice, stream));
    {
      GemmArgs g{};
      g.a = mlp_in; g.a_lo = mlp_in_lo; g.a_half = half_act; g.out_e16 = mlp; g.out_lo = mlp_lo; g.out_half = half_act;
      g.partial = splitk;
      g.m = T; g.n = d.F; g.k = d.H; g.lda = d.H; g.ldo = d.F;
      if (c.mlp_kind == 0) {
        if (int rc = bind_weights(st, stream, g, w.wgate, w.sgate, w.zgate, w.wup, w.sup, w.zup, l, st->copies.gate, st->copies.up)) return rc;
        int rc = run_gemm(st, stream, STAGE_K_GEMM_GATEUP, g, kEpiSwiGLU, plans.gateup);
        if (rc) return rc;
      } else {
        // ungated: the product in fp32 (one plane, or the split-K partial sums), then bias + gelu + rounding in one pass
        g.out_f32 = up_f32;
        if (int rc = bind_weights(st, stream, g, w.wup, w.sup, w.zup, nullptr, nullptr, nullptr, l, st->copies.up, kNoCopy)) return rc;
        const GemmPlan& plan = plans.gateup;
        {
          Timer t(st, stream, STAGE_K_GEMM_GATEUP);
          HIP_TRY(launch_gemm_main(g, kEpiStoreF32, plan, stream));
        }
        Timer t(st, stream, STAGE_K_SPLITK_REDUCE);
        HIP_TRY(launch_bias_gelu(plan.partials ? splitk : up_f32, plan.partials ? plan.splits : 1, (size_t)T * d.F,
                                 (const e16*)w.bup, c.mlp_kind == 2, mlp, mlp_lo, T, d.F, half_act, stream));
      }
    }
    if (tap && taps->tap_mlp) HIP_TRY(copy_activation_tap(taps->tap_mlp, mlp, (size_t)T * d.F, half_act, stream));
    {
      // With a tap on the last layer the fp32 stream is completed first and rounded by a separate
      // kernel, so the tap sees it; the sum and its rounding are the same as in the fused epilogue.
      const bool fused_out = last && !(tap && taps->tap_x);
      GemmArgs g{};
      g.a = mlp; g.a_lo = mlp_lo; g.a_half = half_act; g.resid = x; g.out_e16 = (e16*)hidden_out;
      g.partial = splitk;
      g.m = T; g.n = d.H; g.k = d.F; g.lda = d.F; g.ldo = d.H;
      if (int rc = bind_weights(st, stream, g, w.wdown, w.sdown, w.zdown, nullptr, nullptr, nullptr, l, st->copies.down, kNoCopy)) return rc;
      if (w.bdown) {
        Timer t(st, stream, STAGE_K_SPLITK_REDUCE);
        HIP_TRY(launch_add_row_bias(x, (const e16*)w.bdown, T, d.H, stream));
      }
      int rc = run_residual_gemm(st, stream, STAGE_K_GEMM_DOWN, g, fused_out ? kEpiResidualOut : kEpiResidualF32,
                                 fused_out ? plans.down_out : plans.down, last ? no_norm : norm_of(l + 1, false), a,
                                 norm1_lo, half_act);
      if (rc) return rc;
      if (tap && taps->tap_x)
        HIP_TRY(hipMemcpyAsync(taps->tap_x, x, (size_t)T * d.H * 4, hipMemcpyDeviceToDevice, stream));
      if (last && !fused_out) {
        const size_t n = (size_t)T * d.H;
        hipLaunchKernelGGL(f32_to_e16_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, x,
                           (e16*)hidden_out, n);
        HIP_TRY(hipGetLastError());
      }
    }
  }
  return STAGE_OK;
}

}  // namespace

extern "C" {

int stage_kv_layer_bytes(const stage_config* cfg, size_t* out_bytes) {
  if (!out_bytes) return fail(STAGE_ERR_NULL, "out_bytes is NULL");
  int rc = check_config(cfg);
  if (rc) return rc;
  *out_bytes = (size_t)cfg->num_kv_blocks * cfg->num_kv_heads * 16 * cfg->head_dim * 2 * 2;
  return STAGE_OK;
}

int stage_kv_element_offset(const stage_config* cfg, int32_t kv, int32_t block, int32_t kv_head, int32_t slot,
                            int32_t dim, int64_t* out_offset) {
  if (!out_offset) return fail(STAGE_ERR_NULL, "out_offset is NULL");
  int rc = check_config(cfg);
  if (rc) return rc;
  if (kv < 0 || kv > 1 || block < 0 || block >= cfg->num_kv_blocks || kv_head < 0 || kv_head >= cfg->num_kv_heads ||
      slot < 0 || slot >= 16 || dim < 0 || dim >= cfg->head_dim)
    return fail(STAGE_ERR_CONFIG, "KV coordinate out of range");
  const int64_t d = cfg->head_dim, nkv = cfg->num_kv_heads;
  const int64_t region = (int64_t)cfg->num_kv_blocks * nkv * 16 * d;
  const int64_t base = ((int64_t)block * nkv + kv_head) * 16 * d;
  *out_offset = kv == 0 ? base + k_offset_in_block(slot, dim) : region + base + (int64_t)dim * 16 + slot;
  return STAGE_OK;
}

int stage_workspace_bytes(const stage_config* cfg, size_t* out_bytes) {
  if (!out_bytes) return fail(STAGE_ERR_NULL, "out_bytes is NULL");
  int rc = check_config(cfg);
  if (rc) return rc;
  *out_bytes = layout_of(*cfg).total + (size_t)cfg->num_layers * copy_layout_of(*cfg).per_layer;
  return STAGE_OK;
}

int stage_check_batch(const stage_config* cfg, int32_t num_tokens, const int32_t* positions, int32_t num_seqs,
                      const int32_t* q_lens, const int32_t* ctx_lens, const int32_t* block_tables,
                      int64_t* slot_mapping_out) {
  int rc = check_config(cfg);
  if (rc) return rc;
  BatchCounts bc;
  rc = validate_batch(*cfg, num_tokens, positions, num_seqs, q_lens, ctx_lens, block_tables, &bc);
  if (rc) return rc;
  if (slot_mapping_out) fill_slot_mapping(*cfg, num_seqs, q_lens, ctx_lens, block_tables, slot_mapping_out);
  return STAGE_OK;
}

int stage_init(const stage_config* cfg, const stage_layer_weights* layers, void* kv_pool, size_t kv_pool_bytes,
               void* workspace, size_t workspace_bytes, int32_t device, stage_handle** out) {
  if (!out) return fail(STAGE_ERR_NULL, "out handle pointer is NULL");
  *out = nullptr;
  int rc = check_config(cfg);
  if (rc) return rc;
  if (!layers || !kv_pool || !workspace) return fail(STAGE_ERR_NULL, "layers, kv_pool or workspace is NULL");
  for (int l = 0; l < cfg->num_layers; ++l) {
    const stage_layer_weights& w = layers[l];
    if (!w.norm1 || !w.wqkv || !w.wo || !w.wup || !w.wdown)
      return fail(STAGE_ERR_NULL, "layer %d has a NULL weight pointer", l);
    if ((w.wgate == nullptr) != (cfg->mlp_kind != 0))
      return fail(cfg->mlp_kind ? STAGE_ERR_CONFIG : STAGE_ERR_NULL,
                  "layer %d: wgate must be set for the gated MLP (mlp_kind 0) and NULL for the ungated one", l);
    if (!w.norm2 && !cfg->parallel_block) return fail(STAGE_ERR_NULL, "layer %d: norm2 is NULL (allowed with parallel_block only)", l);
    if ((w.norm2 == nullptr) != (layers[0].norm2 == nullptr))
      return fail(STAGE_ERR_NULL, "layer %d: norm2 must be set in every layer or in none", l);
    if ((w.norm1_bias || w.norm2_bias) && cfg->norm_kind != 1)
      return fail(STAGE_ERR_CONFIG, "layer %d: norm1_bias / norm2_bias belong to LayerNorms (norm_kind 1)", l);
    if (w.norm2_bias && !w.norm2) return fail(STAGE_ERR_CONFIG, "layer %d: norm2_bias without norm2", l);
    if (w.bup && cfg->mlp_kind == 0) return fail(STAGE_ERR_CONFIG, "layer %d: bup belongs to the ungated MLP (mlp_kind 1 or 2)", l);
    const void* ptrs[12] = {w.norm1, w.wqkv, w.wo, w.norm2, w.wgate, w.wup, w.wdown, w.norm1_bias, w.norm2_bias, w.bo, w.bup, w.bdown};
    for (const void* p : ptrs)
      if ((uintptr_t)p % 16) return fail(STAGE_ERR_CONFIG, "layer %d has a weight or bias pointer that is not 16-byte aligned", l);
    if ((uintptr_t)w.bqkv % 16) return fail(STAGE_ERR_CONFIG, "layer %d: bqkv is not 16-byte aligned", l);
    if ((w.alibi == nullptr) != (layers[0].alibi == nullptr))
      return fail(STAGE_ERR_NULL, "layer %d: alibi slopes must be set in every layer or in none", l);
    if (w.alibi && (w.qnorm || cfg->rotary_dim != 0 || cfg->rope_interleaved != 0 || cfg->rope_scaling != 0))
      return fail(STAGE_ERR_CONFIG, "layer %d: linear biases replace the rotation: rotary_dim and rope_interleaved must be 0, "
                  "qnorm / knorm NULL", l);
    if ((uintptr_t)w.alibi % 4) return fail(STAGE_ERR_CONFIG, "layer %d: alibi is not 4-byte aligned", l);
    if ((w.qnorm == nullptr) != (w.knorm == nullptr))
      return fail(STAGE_ERR_NULL, "layer %d: qnorm and knorm must both be set or both be NULL", l);
    if (w.qnorm && cfg->rotary_dim != 0 && cfg->rotary_dim != cfg->head_dim)
      return fail(STAGE_ERR_CONFIG, "layer %d: qnorm / knorm are not supported together with a partial rotary embedding", l);
    if ((uintptr_t)w.qnorm % 16 || (uintptr_t)w.knorm % 16)
      return fail(STAGE_ERR_CONFIG, "layer %d: qnorm or knorm is not 16-byte aligned", l);
    if (cfg->weight_bits == 4) {
      const void* q[10] = {w.sqkv, w.so, w.sgate, w.sup, w.sdown, w.zqkv, w.zo, w.zgate, w.zup, w.zdown};
      for (const void* p : q) {
        if (!p) return fail(STAGE_ERR_NULL, "layer %d has a NULL scale or zero-point pointer", l);
        if ((uintptr_t)p % 16) return fail(STAGE_ERR_CONFIG, "layer %d has a scale or zero-point pointer that is not 16-byte aligned", l);
      }
    }
  }
  if ((uintptr_t)kv_pool % 256 || (uintptr_t)workspace % 256)
    return fail(STAGE_ERR_CONFIG, "kv_pool and workspace must be 256-byte aligned");
  const size_t layer_bytes = (size_t)cfg->num_kv_blocks * cfg->num_kv_heads * 16 * cfg->head_dim * 2 * 2;
  const size_t need_pool = (size_t)(cfg->num_layers - 1) * (size_t)cfg->kv_layer_stride_bytes + layer_bytes;
  if (kv_pool_bytes < need_pool) return fail(STAGE_ERR_SIZE, "kv_pool_bytes %zu < %zu", kv_pool_bytes, need_pool);
  const WorkspaceLayout ws = layout_of(*cfg);
  const CopyLayout copies = copy_layout_of(*cfg);
  const size_t need_ws = ws.total + (size_t)cfg->num_layers * copies.per_layer;
  if (workspace_bytes < need_ws) return fail(STAGE_ERR_SIZE, "workspace_bytes %zu < %zu", workspace_bytes, need_ws);
  int ndev = 0;
  HIP_TRY(hipGetDeviceCount(&ndev));
  if (device < 0 || device >= ndev) return fail(STAGE_ERR_CONFIG, "device %d outside [0, %d)", device, ndev);
  HIP_TRY(hipSetDevice(device));

  stage_handle* st = new (std::nothrow) stage_handle();
  if (!st) return fail(STAGE_ERR_SIZE, "out of host memory");
  st->cfg = *cfg;
  st->dim = dims_of(*cfg);
  st->ws = ws;
  st->layers.assign(layers, layers + cfg->num_layers);
  st->kv_pool = (char*)kv_pool;
  st->workspace = (char*)workspace;
  st->static_scratch = nullptr;
  st->call_ws = (char*)workspace;
  st->call_layout = &st->ws;
  st->copies = copies;
  st->wcopy = copies.per_layer ? (char*)workspace + ws.total : nullptr;
  st->device = device;
  st->next_slot = 0;
  st->profile_mask = 0;
  for (int i = 0; i < kStagingSlots; ++i) { st->staging[i] = nullptr; st->staging_done[i] = nullptr; st->staging_used[i] = false; }
  for (int i = 0; i < kStagingSlots; ++i) {
    hipError_t e = hipHostMalloc((void**)&st->staging[i], ws.meta_bytes, hipHostMallocDefault);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&st->staging_done[i], hipEventDisableTiming);
    if (e != hipSuccess) {
      stage_destroy(st);
      return fail(STAGE_ERR_HIP, "allocating pinned staging: %s", hipGetErrorString(e));
    }
  }
  if (int rc2 = static_scratch_of(device, &st->static_scratch)) {
    stage_destroy(st);
    return rc2;
  }
  if (st->wcopy) {
    // the weights once more, in operand order and in the operand format of this stage's matrix instructions
    const Dims& d = st->dim;
    const bool to_half = half_act_of(*cfg);
    hipError_t e = hipSuccess;
    for (int l = 0; l < d.L && e == hipSuccess; ++l) {
      const stage_layer_weights& w = st->layers[l];
      char* base = st->wcopy + (size_t)l * copies.per_layer;
      struct { const void* src; size_t at; int n, k; } jobs[5] = {{w.wqkv, copies.qkv, d.qkv_out, d.H}, {w.wo, copies.o, d.H, d.nq * d.d},
                                                                 {w.wgate, copies.gate, d.F, d.H}, {w.wup, copies.up, d.F, d.H},
                                                                 {w.wdown, copies.down, d.H, d.F}};
      for (const auto& j : jobs)
        if (j.at != kNoCopy && j.src && e == hipSuccess)
          e = launch_arrange_weights((const e16*)j.src, j.n, j.k, to_half, (e16*)(base + j.at), nullptr);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
    if (e != hipSuccess) {
      stage_destroy(st);
      return fail(STAGE_ERR_HIP, "copying the weights into operand order: %s", hipGetErrorString(e));
    }
  }
  *out = st;
  return STAGE_OK;
}

int stage_forward_static(stage_handle* st, void* hip_stream, int32_t num_tokens, const void* hidden_in,
                         const int32_t* positions, int32_t num_seqs, const int32_t* q_lens, const int32_t* ctx_lens,
                         const int32_t* block_tables, void* hidden_out, int64_t* slot_mapping_out) {
  if (!st) return fail(STAGE_ERR_NULL, "stage handle is NULL");
  // per-kernel timing creates events on demand; this entry point creates nothing
  const uint32_t mask = st->profile_mask;
  st->profile_mask = 0;
  const int rc = forward_impl(st, hip_stream, num_tokens, hidden_in, positions, num_seqs, q_lens, ctx_lens, block_tables,
                              hidden_out, slot_mapping_out, nullptr, true);
  st->profile_mask = mask;
  return rc;
}

int stage_forward(stage_handle* st, void* hip_stream, int32_t num_tokens, const void* hidden_in,
                  const int32_t* positions, int32_t num_seqs, const int32_t* q_lens, const int32_t* ctx_lens,
                  const int32_t* block_tables, void* hidden_out, int64_t* slot_mapping_out) {
  return forward_impl(st, hip_stream, num_tokens, hidden_in, positions, num_seqs, q_lens, ctx_lens, block_tables,
                      hidden_out, slot_mapping_out, nullptr);
}

int stage_forward_taps(stage_handle* st, void* hip_stream, int32_t num_tokens, const void* hidden_in,
                       const int32_t* positions, int32_t num_seqs, const int32_t* q_lens, const int32_t* ctx_lens,
                       const int32_t* block_tables, void* hidden_out, int64_t* slot_mapping_out,
                       const stage_taps* taps) {
  if (!taps) return fail(STAGE_ERR_NULL, "taps is NULL");
  return forward_impl(st, hip_stream, num_tokens, hidden_in, positions, num_seqs, q_lens, ctx_lens, block_tables,
                      hidden_out, slot_mapping_out, taps);
}

// Start-up profiling: one point of the latency table (see the header).  Identity paging: sequence s owns the
// blocks s * B .. s * B + B - 1, B = blocks of ctx_len + q_len tokens.
int stage_profile(stage_handle* st, void* hip_stream, int32_t num_seqs, int32_t q_len, int32_t ctx_len, int32_t warmup,
                  int32_t iters, const void* hidden_in, void* hidden_out, double* out_ms) {
  if (!st || !out_ms) return fail(STAGE_ERR_NULL, "stage handle or out_ms is NULL");
  const stage_config& c = st->cfg;
  if (num_seqs < 1 || q_len < 1 || ctx_len < 0 || warmup < 0 || iters < 1)
    return fail(STAGE_ERR_BATCH, "stage_profile: need num_seqs, q_len, iters >= 1 and ctx_len, warmup >= 0");
  const int64_t T = (int64_t)num_seqs * q_len;
  const int64_t blocks = ((int64_t)ctx_len + q_len + 15) / 16;
  if (num_seqs > c.max_seqs || T > c.max_tokens)
    return fail(STAGE_ERR_BATCH, "stage_profile: %d sequences of %d new tokens exceed max_seqs %d / max_tokens %d", num_seqs,
                q_len, c.max_seqs, c.max_tokens);
  if (blocks > c.max_blocks_per_seq || blocks * num_seqs > c.num_kv_blocks)
    return fail(STAGE_ERR_BLOCK_TABLE, "stage_profile: %d sequences of %lld blocks exceed the block tables or the pool",
                num_seqs, (long long)blocks);
  std::vector<int32_t> positions((size_t)T), q_lens((size_t)num_seqs, q_len), ctx_lens((size_t)num_seqs, ctx_len);
  std::vector<int32_t> tables((size_t)num_seqs * c.max_blocks_per_seq, -1);
  for (int s = 0; s < num_seqs; ++s) {
    for (int i = 0; i < q_len; ++i) positions[(size_t)s * q_len + i] = ctx_len + i;
    for (int b = 0; b < blocks; ++b) tables[(size_t)s * c.max_blocks_per_seq + b] = (int32_t)(s * blocks + b);
  }
  hipStream_t stream = (hipStream_t)hip_stream;
  HIP_TRY(hipSetDevice(st->device));
  hipEvent_t begin, end;
  HIP_TRY(hipEventCreate(&begin));
  if (hipEventCreate(&end) != hipSuccess) {
    (void)hipEventDestroy(begin);
    return fail(STAGE_ERR_HIP, "hipEventCreate failed");
  }
  int rc = STAGE_OK;
  for (int i = 0; i < warmup + iters && rc == STAGE_OK; ++i) {
    if (i == warmup && hipEventRecord(begin, stream) != hipSuccess) rc = fail(STAGE_ERR_HIP, "hipEventRecord failed");
    if (rc == STAGE_OK)
      rc = forward_impl(st, hip_stream, (int32_t)T, hidden_in, positions.data(), num_seqs, q_lens.data(), ctx_lens.data(),
                        tables.data(), hidden_out, nullptr, nullptr);
  }
  if (rc == STAGE_OK) {
    float ms = 0.f;
    if (hipEventRecord(end, stream) != hipSuccess || hipEventSynchronize(end) != hipSuccess ||
        hipEventElapsedTime(&ms, begin, end) != hipSuccess)
      rc = fail(STAGE_ERR_HIP, "timing the profiled runs failed: %s", hipGetErrorString(hipGetLastError()));
    else
      *out_ms = (double)ms / iters;
  }
  (void)hipEventDestroy(begin);
  (void)hipEventDestroy(end);
  return rc;
}

// Copies a small host array to the device through a pinned staging slot (the caller may reuse the host
// array as soon as the call returns).
static int stage_small_h2d(stage_handle* st, hipStream_t stream, const void* host, size_t bytes, void* dev) {
  const int slot_id = st->next_slot;
  st->next_slot = (st->next_slot + 1) % kStagingSlots;
  if (st->staging_used[slot_id]) HIP_TRY(hipEventSynchronize(st->staging_done[slot_id]));
  memcpy(st->staging[slot_id], host, bytes);
  HIP_TRY(hipMemcpyAsync(dev, st->staging[slot_id], bytes, hipMemcpyHostToDevice, stream));
  HIP_TRY(hipEventRecord(st->staging_done[slot_id], stream));
  st->staging_used[slot_id] = true;
  return STAGE_OK;
}

int stage_embed(stage_handle* st, void* hip_stream, const void* table, int32_t vocab, int32_t num_tokens,
                const int32_t* token_ids, void* hidden_out) {
  if (!st) return fail(STAGE_ERR_NULL, "stage handle is NULL");
  if (!table || !token_ids || !hidden_out) return fail(STAGE_ERR_NULL, "a required argument of stage_embed is NULL");
  if (vocab < 1) return fail(STAGE_ERR_BATCH, "vocab %d must be positive", vocab);
  if (num_tokens < 1 || num_tokens > st->cfg.max_tokens)
    return fail(STAGE_ERR_BATCH, "num_tokens %d outside [1, max_tokens=%d]", num_tokens, st->cfg.max_tokens);
  for (int t = 0; t < num_tokens; ++t)
    if (token_ids[t] < 0 || token_ids[t] >= vocab)
      return fail(STAGE_ERR_BATCH, "token_ids[%d] = %d outside [0, %d)", t, token_ids[t], vocab);
  HIP_TRY(hipSetDevice(st->device));
  hipStream_t stream = (hipStream_t)hip_stream;
  int32_t* d_ids = (int32_t*)(st->workspace + st->ws.ends_meta);
  int rc = stage_small_h2d(st, stream, token_ids, (size_t)num_tokens * 4, d_ids);
  if (rc) return rc;
  Timer t(st, stream, STAGE_K_EMBED);
  HIP_TRY(launch_embed_gather((const e16*)table, d_ids, (e16*)hidden_out, num_tokens, st->dim.H, stream));
  return STAGE_OK;
}

static int head_impl(stage_handle* st, void* hip_stream, int32_t num_tokens, const void* hidden, int32_t num_seqs,
              const int32_t* q_lens, const void* final_norm, const void* final_norm_bias, const void* lm_head,
              int32_t vocab, void* logits_out, int32_t* next_tokens) {
  if (!hidden || !q_lens || !final_norm || !lm_head || !next_tokens)
    return fail(STAGE_ERR_NULL, "a required argument of the output head is NULL");
  const stage_config& c = st->cfg;
  const Dims& d = st->dim;
  if (c.vocab_size == 0 || vocab != c.vocab_size)
    return fail(STAGE_ERR_CONFIG, "vocab %d does not match the stage's vocab_size %d", vocab, c.vocab_size);
  if (num_tokens < 1 || num_tokens > c.max_tokens)
    return fail(STAGE_ERR_BATCH, "num_tokens %d outside [1, max_tokens=%d]", num_tokens, c.max_tokens);
  if (num_seqs < 1 || num_seqs > c.max_seqs)
    return fail(STAGE_ERR_BATCH, "num_seqs %d outside [1, max_seqs=%d]", num_seqs, c.max_seqs);
  std::vector<int32_t> rows((size_t)num_seqs);
  int64_t sum_q = 0;
  for (int s = 0; s < num_seqs; ++s) {
    if (q_lens[s] < 1) return fail(STAGE_ERR_BATCH, "q_lens[%d] = %d must be >= 1", s, q_lens[s]);
    sum_q += q_lens[s];
    rows[(size_t)s] = (int32_t)(sum_q - 1);
  }
  if (sum_q != num_tokens)
    return fail(STAGE_ERR_BATCH, "sum(q_lens) = %lld != num_tokens = %d", (long long)sum_q, num_tokens);
  const GemmPlan plan = plan_gemm(num_seqs, vocab, d.H, kEpiStoreF32, kNumCus, false);
  if (int rc2 = check_plan(st, num_seqs, plan)) return rc2;
  HIP_TRY(hipSetDevice(st->device));
  hipStream_t stream = (hipStream_t)hip_stream;
  char* ws = st->workspace;
  int32_t* d_rows = (int32_t*)(ws + st->ws.ends_meta);
  int rc = stage_small_h2d(st, stream, rows.data(), (size_t)num_seqs * 4, d_rows);
  if (rc) return rc;
  e16* head_a = (e16*)(ws + st->ws.head_a);
  {
    Timer t(st, stream, STAGE_K_HEAD_NORM);
    HIP_TRY(launch_gather_rmsnorm((const e16*)hidden, d_rows,
                                  NormSpec{(const e16*)final_norm, (const e16*)final_norm_bias, c.rms_eps, c.norm_kind},
                                  head_a, num_seqs, d.H, stream));
  }
  GemmArgs g{};
  g.a = head_a; g.w0 = (const e16*)lm_head; g.partial = (float*)(ws + st->ws.splitk);
  g.m = num_seqs; g.n = vocab; g.k = d.H; g.lda = d.H; g.ldo = vocab;
  // without partial sums the GEMM writes the logits itself (to the caller's buffer if there is one)
  float* direct = logits_out ? (float*)logits_out : (float*)(ws + st->ws.head_logits);
  g.out_f32 = direct;
  {
    Timer t(st, stream, STAGE_K_GEMM_HEAD);
    HIP_TRY(launch_gemm_main(g, kEpiStoreF32, plan, stream));
  }
  Timer t(st, stream, STAGE_K_HEAD_ARGMAX);
  if (plan.partials)
    HIP_TRY(launch_argmax_rows(g.partial, plan.splits, (size_t)num_seqs * vocab, num_seqs, vocab, (float*)logits_out,
                               next_tokens, stream));
  else
    HIP_TRY(launch_argmax_rows(direct, 1, 0, num_seqs, vocab, nullptr, next_tokens, stream));
  return STAGE_OK;
}

int stage_head(stage_handle* st, void* hip_stream, int32_t num_tokens, const void* hidden, int32_t num_seqs,
               const int32_t* q_lens, const void* final_norm, const void* lm_head, int32_t vocab, void* logits_out,
               int32_t* next_tokens) {
  if (!st) return fail(STAGE_ERR_NULL, "stage handle is NULL");
  if (st->cfg.norm_kind != 0)
    return fail(STAGE_ERR_CONFIG, "stage_head normalises with an RMSNorm; this stage's blocks use LayerNorms (norm_kind 1): "
                                  "call stage_head_layernorm");
  return head_impl(st, hip_stream, num_tokens, hidden, num_seqs, q_lens, final_norm, nullptr, lm_head, vocab, logits_out,
                   next_tokens);
}

int stage_head_layernorm(stage_handle* st, void* hip_stream, int32_t num_tokens, const void* hidden, int32_t num_seqs,
                         const int32_t* q_lens, const void* final_norm, const void* final_norm_bias, const void* lm_head,
                         int32_t vocab, void* logits_out, int32_t* next_tokens) {
  if (!st) return fail(STAGE_ERR_NULL, "stage handle is NULL");
  if (st->cfg.norm_kind != 1)
    return fail(STAGE_ERR_CONFIG, "stage_head_layernorm belongs to stages whose blocks use LayerNorms (norm_kind 1): "
                                  "call stage_head");
  if ((uintptr_t)final_norm_bias % 16) return fail(STAGE_ERR_CONFIG, "final_norm_bias is not 16-byte aligned");
  return head_impl(st, hip_stream, num_tokens, hidden, num_seqs, q_lens, final_norm, final_norm_bias, lm_head, vocab,
                   logits_out, next_tokens);
}


int stage_profile_enable(stage_handle* st, uint32_t kernel_mask) {
  if (!st) return fail(STAGE_ERR_NULL, "stage handle is NULL");
  st->profile_mask = kernel_mask;
  return STAGE_OK;
}

int stage_profile_read(stage_handle* st, int32_t kernel, double* out_total_ms, int64_t* out_launches) {
  if (!st || !out_total_ms || !out_launches) return fail(STAGE_ERR_NULL, "NULL argument");
  if (kernel < 0 || kernel >= STAGE_K_COUNT) return fail(STAGE_ERR_CONFIG, "unknown kernel class %d", kernel);
  double total = 0.0;
  int64_t n = 0;
  std::vector<TimedLaunch> keep;
  for (const TimedLaunch& t : st->timed) {
    if (t.kernel != kernel) { keep.push_back(t); continue; }
    HIP_TRY(hipEventSynchronize(t.end));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, t.begin, t.end));
    total += ms;
    ++n;
    st->free_events.push_back(t);
  }
  st->timed.swap(keep);
  *out_total_ms = total;
  *out_launches = n;
  return STAGE_OK;
}

const char* stage_kernel_name(int32_t kernel) {
  switch (kernel) {
    case STAGE_K_RMSNORM: return "rmsnorm_kernel";
    case STAGE_K_GEMM_QKV:
    case STAGE_K_GEMM_O:
    case STAGE_K_GEMM_GATEUP:
    case STAGE_K_GEMM_DOWN: return "gemm_tile_kernel";
    case STAGE_K_ROPE_APPEND: return "rope_append_kernel";
    case STAGE_K_ATTN_PREFILL: return "attn_prefill_kernel";
    case STAGE_K_ATTN_DECODE: return "attn_decode_kernel";
    case STAGE_K_ATTN_MERGE: return "attn_merge_kernel";
    case STAGE_K_SPLITK_REDUCE: return "gemm_splitk_reduce_kernel";
    case STAGE_K_ROPE_TABLE: return "rope_table_kernel";
    case STAGE_K_EMBED: return "embed_gather_kernel";
    case STAGE_K_HEAD_NORM: return "gather_rmsnorm_kernel";
    case STAGE_K_GEMM_HEAD: return "gemm_tile_kernel";
    case STAGE_K_HEAD_ARGMAX: return "argmax_rows_kernel";
    case STAGE_K_DEQUANT: return "dequant_w4_kernel";
    default: return nullptr;
  }
}

void stage_destroy(stage_handle* st) {
  if (!st) return;
  (void)hipSetDevice(st->device);
  (void)hipDeviceSynchronize();
  for (int i = 0; i < kStagingSlots; ++i) {
    if (st->staging[i]) (void)hipHostFree(st->staging[i]);
    if (st->staging_done[i]) (void)hipEventDestroy(st->staging_done[i]);
  }
  for (auto* list : {&st->timed, &st->free_events})
    for (const TimedLaunch& t : *list) {
      (void)hipEventDestroy(t.begin);
      (void)hipEventDestroy(t.end);
    }
  delete st;
}

const char* stage_last_error(void) { return g_error; }

int32_t stage_elem_type(void) { return kElemIsF16 ? STAGE_ELEM_F16 : STAGE_ELEM_BF16; }

}  // extern "C"
