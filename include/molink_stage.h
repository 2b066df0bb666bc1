/*
 * molink_stage.h -- C ABI of one pipeline stage's decoder-layer forward pass on one MI355X.
 *
 * The serving system launches every inference engine with the run of consecutive decoder
 * layers assigned to it (paper section 3.2.1) and feeds it micro-batches that mix prefill
 * chunks and decode tokens; the engine's runtime holds the weights, runs the micro-batch through
 * them and hands the resulting intermediate activations to the next stage (paper section
 * 3.2.2, "Distributed Inference Engine").  That output is one hidden vector per processed
 * token (section 4.2).  This library is that computation:
 *   stage_init     -- bind the stage's layer weights, a paged KV pool and a workspace;
 *   stage_forward  -- run all layers on one micro-batch and write the packed activations.
 *
 * Per layer (Llama-style pre-norm block, bf16 storage, fp32 accumulation):
 *   a = RMSNorm(x; norm1)            q,k,v = a Wqkv^T        q,k <- RoPE(q,k; positions)
 *   append k,v to the paged pool     o = causal GQA attention of q over the sequence's cache
 *   h = x + o Wo^T                   b = RMSNorm(h; norm2)
 *   x' = h + (silu(b Wgate^T) * (b Wup^T)) Wdown^T
 * Switches of stage_config and optional tensors of stage_layer_weights turn this block into the other dense
 * blocks of the paper's model table (section 3.1.3): a bias on q/k/v, per-head norms of q and k, a partial or
 * neighbour-pairing rotation, linear score biases instead of a rotation, LayerNorms, an ungated GELU MLP with
 * biases, and branches that both start from x (norm_kind, mlp_kind, parallel_block).
 *
 * All device buffers (weights, KV pool, workspace, input, output) are allocated and owned by
 * the caller and must stay valid until stage_destroy; the library allocates no device memory.
 * Every entry point returns 0 on success or a negative STAGE_ERR_* code and never throws;
 * stage_last_error() gives a message for the calling thread's last failure.
 *
 * Element type.  The same sources build two libraries with this one ABI: libmolink_stage.so stores
 * every 16-bit tensor (weights, activations, KV cache, payload, 4-bit scales and zero points) as
 * bfloat16, libmolink_stage_f16.so as IEEE half, the precision the paper serves its 7B model in
 * (section 5, "Models").  Wherever this header says bf16 it means the loaded library's element type;
 * stage_elem_type() tells which one that is.  Accumulation, softmax, norms and the residual stream are
 * fp32 in both.
 *
 * The library targets gfx950 only and requires kv_block_size == 16, head_dim in {64, 128},
 * hidden and ffn multiples of 8 and at least 64, num_q_heads a multiple of num_kv_heads
 * with at most 16 query heads per KV head.
 */
#ifndef MOLINK_STAGE_H
#define MOLINK_STAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  STAGE_OK = 0,
  STAGE_ERR_NULL = -1,        /* a required pointer is NULL */
  STAGE_ERR_CONFIG = -2,      /* unsupported or inconsistent stage_config */
  STAGE_ERR_SIZE = -3,        /* a caller buffer is too small */
  STAGE_ERR_BATCH = -4,       /* micro-batch metadata invalid (lengths, counts, capacity) */
  STAGE_ERR_BLOCK_TABLE = -5, /* block table too short, or a used block id out of range */
  STAGE_ERR_HIP = -6,         /* a HIP runtime call failed (message has the HIP error string) */
  STAGE_ERR_ALIAS = -7        /* hidden_out overlaps hidden_in */
};

/* Plain data, versioned by struct_size (= sizeof(stage_config) of the caller's header). */
typedef struct {
  uint32_t struct_size;
  int32_t num_layers;          /* L: decoder layers hosted by this stage */
  int32_t hidden;              /* H */
  int32_t num_q_heads;         /* nq */
  int32_t num_kv_heads;        /* nkv; query head h reads KV head h / (nq / nkv) */
  int32_t head_dim;            /* d: 64 or 128 */
  int32_t ffn;                 /* F: SwiGLU inner width */
  float rms_eps;               /* added to the mean square inside the square root */
  float rope_theta;            /* RoPE base; pair (i, i + d/2) turns by position * theta^(-2i/d) */
  int32_t kv_block_size;       /* tokens per KV block; must be 16 */
  int32_t num_kv_blocks;       /* blocks in each layer's pool */
  int64_t kv_layer_stride_bytes; /* distance between consecutive layers' pools; >= stage_kv_layer_bytes,
                                    or 0 to alias every layer onto one pool (timing experiments only:
                                    values are then meaningless) */
  int32_t max_tokens;          /* capacity: new tokens per micro-batch (T) */
  int32_t max_seqs;            /* capacity: sequences per micro-batch (S) */
  int32_t max_blocks_per_seq;  /* row length of block_tables */
  int32_t activation_planes;   /* How the inputs of the projections are carried between kernels:
                                  1  one plane of the element type;
                                  2  two planes (also of the rotated queries), value = hi + lo, both multiplied
                                     into the same fp32 accumulators: activations that are effectively 16-bit, at
                                     twice the MFMA work of the projections;
                                  3  (bfloat16 library only) one plane of IEEE half - eleven significant bits
                                     instead of eight - with the bfloat16 weights converted to half, exactly, on
                                     their way into the matrix instruction; the rotated queries keep a second
                                     bfloat16 plane for the attention kernels (the decode kernel multiplies both; the
                                     prefill kernel both in mode 4, the first alone in mode 3).  Values beyond the half range
                                     saturate: a projection input larger than 65504 in magnitude is carried as
                                     +-65504 (finite, no longer the unclamped result; activations of that size
                                     do not occur behind an RMSNorm with gains of order one);
                                  4  (bfloat16 library only) as 3, and for micro-batches with prefill chunks the
                                     input of the q/k/v projection gets a second half plane (rows that attend to
                                     few keys amplify the rounding of that input);
                                  0  automatic: 1 for the half-precision library; for the bfloat16 library by
                                     depth, because the rounding errors of the layers add up on the residual
                                     stream: 1 up to 4 layers, 3 from 5 layers, 4 from 9 layers (one bfloat16
                                     plane comes to 8e-3 of the 1e-2 relative-L2 budget at 8 layers). */
  int32_t vocab_size;          /* 0, or the vocabulary size (multiple of 8, >= 64) of the output head this
                                  stage may run with stage_head (sizes the workspace for it) */
  int32_t weight_bits;         /* 0 or 16: the five projection matrices of a layer are bf16.  4: they are
                                  group-quantised to 4 bits (see stage_layer_weights); the paper runs its 70B
                                  model that way (section 5 "Models") */
  int32_t weight_group_size;   /* weight_bits == 4 only: 32, 64 or 128 consecutive input features share one
                                  scale and one zero point; hidden, num_q_heads*head_dim and ffn must be
                                  multiples of it.  Otherwise 0. */
  int32_t rotary_dim;          /* 0 (or head_dim): whole heads rotate.  Otherwise a multiple of 16 below head_dim: only
                                  the first rotary_dim elements of every query and key head rotate, as a head of that
                                  size would (pairs (i, i + rotary_dim/2), angle position * theta^(-2i/rotary_dim)); the
                                  rest pass through unrotated.  The GLM / ChatGLM families of the paper's model table
                                  (section 3.1.3) rotate half of each head (see also rope_interleaved).  Not together
                                  with qnorm / knorm. */
  int32_t rope_interleaved;    /* 0: the rotation pairs element i with element i + d/2 (d: head_dim, or rotary_dim).
                                  1: it pairs neighbours, element 2i with element 2i + 1, at the same angle
                                  position * theta^(-2i/d).  The GLM / ChatGLM families pair neighbours (and rotate
                                  half of each head: rotary_dim). */
  int32_t weight_copies;       /* 0: the stage keeps a second copy of its 16-bit projection weights, made by stage_init
                                  in the order and format its matrix instructions take them (IEEE half in a stage
                                  with half activations), which the tiled GEMMs of micro-batches of more than 64
                                  rows read straight into registers: about a quarter faster than reading the
                                  caller's row-major matrices through LDS, for one more copy of the weights in the
                                  workspace (stage_workspace_bytes counts it).  Made only when max_tokens > 64, the
                                  weights are 16-bit and activation_planes is not 2; a matrix whose input width is
                                  not a multiple of 256 has none.  1: no copies.  Results agree to the rounding of
                                  the fp32 summation order. */
  int32_t norm_kind;           /* 0: both norms of the block are RMSNorms (gain only).  1: LayerNorms,
                                    (x - mean(x)) / sqrt(mean((x - mean(x))^2) + rms_eps) * gain + bias,
                                  bias optional (stage_layer_weights.norm1_bias / norm2_bias).  The Falcon, GPT-2 and
                                  Cohere families of the paper's model table (section 3.1.3). */
  int32_t mlp_kind;            /* 0: the gated MLP down(silu(gate(b)) * up(b)).  1, 2: the ungated MLP
                                  down(gelu(up(b) + bup)) + bdown, with gelu in its tanh form
                                  0.5 z (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3))) (1: GPT-2) or as z Phi(z) (2: Falcon);
                                  wgate is then unused and must be NULL.  16-bit weights only. */
  int32_t parallel_block;      /* 0: y = h + mlp(norm2(h)) with h = x + attention(norm1(x)).  1: both branches start
                                  from the block's input, y = x + attention(norm1(x)) + mlp(norm2(x)) (Falcon, Cohere);
                                  norm2 may then be NULL in every layer: the MLP reads norm1(x) too (one norm per block).
                                  16-bit weights only. */
  int32_t rope_scaling;        /* Frequency scaling of the rotary embedding for contexts beyond the trained length (the
                                  Llama family publishes its long-context models this way).  0: none.  1: linear - every
                                  frequency theta^(-2i/d) is divided by rope_scaling_factor.  2: by wavelength
                                  w = 2 pi / frequency against rope_original_max_position L: w < L / rope_high_freq_factor
                                  keeps its frequency, w > L / rope_low_freq_factor gets frequency / rope_scaling_factor,
                                  in between the mix (1 - s) frequency / factor + s frequency with
                                  s = (L / w - low) / (high - low).  The four fields below are 0 unless this is set. */
  float rope_scaling_factor;       /* >= 1 */
  float rope_low_freq_factor;      /* kind 2: > 0 and below rope_high_freq_factor */
  float rope_high_freq_factor;     /* kind 2 */
  int32_t rope_original_max_position;  /* kind 2: the trained context length L, > 0 */
} stage_config;

/* Device pointers to one layer's weights, row-major [out_features][in_features], bf16 unless
 * stage_config.weight_bits says otherwise. Borrowed, read-only. */
typedef struct {
  const void *norm1;  /* [H]  gain of the input RMSNorm */
  const void *wqkv;   /* [(nq + 2 nkv) d][H]: q head rows, then k head rows, then v head rows */
  const void *wo;     /* [H][nq d] */
  const void *norm2;  /* [H]  gain of the norm in front of the MLP (NULL: see stage_config.parallel_block) */
  const void *wgate;  /* [F][H]  (NULL with an ungated MLP: stage_config.mlp_kind) */
  const void *wup;    /* [F][H] */
  const void *wdown;  /* [H][F] */
  const void *bqkv;   /* [(nq + 2 nkv) d] bias of the q/k/v projection, added before the rotation
                         (the Qwen2 family has one), or NULL */
  /*
   * weight_bits == 4 only (ignored otherwise).  Each projection matrix W [N][K] (wqkv, wo, wgate, wup,
   * wdown above) is then given as
   *   codes        uint32 [N][K/8], in the w* pointer: element k of row n is the 4-bit field at bits
   *                4*(k%8) .. 4*(k%8)+3 of word [n][k/8]
   *   scales       bf16 [N][K/group]   (s* below)
   *   zero points  bf16 [N][K/group]   (z* below; in code units, usually an integer in 0..15)
   * and stands for   W[n][k] = (code[n][k] - zero[n][k/group]) * scale[n][k/group].
   * Norm gains, the bias and the output head stay bf16.  How a projection reads its weights depends on the
   * micro-batch (the result is the same product, to the stated tolerance, either way):
   *   - at most 64 rows, one activation plane, groups of 128, K a multiple of 256: the stored form is streamed,
   *     scale and zero point applied to fp32 sums - W itself is never rounded;
   *   - more rows, the matrix instructions' operands IEEE half (half activations in the bfloat16 library -
   *     activation_planes 3, 4 or the automatic choice of a deep stage - or the half-precision library), one
   *     plane, groups of 128, K a multiple of 256: the stored form is read by the tiled kernel, each weight formed
   *     as half(code * scale - zero * scale) on its way into the matrix instruction (scales below 2^-14 lose
   *     precision there, products beyond 65504 overflow: per-group scales of weights of ordinary magnitude are
   *     far from either);
   *   - otherwise the matrix is expanded in the workspace first, the fp32 product (exact for integer zero points)
   *     rounded to bf16 once, and the ordinary kernels read the copy: complete, but it costs a write and a read
   *     of 2 bytes per weight per call.
   */
  const void *sqkv, *so, *sgate, *sup, *sdown;
  const void *zqkv, *zo, *zgate, *zup, *zdown;
  /*
   * Both NULL, or both set: gains [d] of a per-head RMSNorm (same rms_eps) applied to every query head
   * (qnorm) and every key head (knorm) of the projection output, after the bias and before the rotation:
   *   u <- u * gain / sqrt(mean(u^2) + rms_eps)   over the d elements of one head.
   * The Qwen3 family of the paper's model table (section 3.1.3) normalises its queries and keys this way;
   * values are not normalised.
   */
  const void *qnorm, *knorm;
  /*
   * NULL in every layer, or set in every layer: fp32 [num_q_heads] head slopes of attention with linear biases.
   * The stage then rotates nothing (positions are ignored; rotary_dim, rope_interleaved and rope_scaling must be 0,
   * qnorm / knorm NULL), and the score of the query at logical index i of its sequence for the key at logical index j <= i is
   * lowered by slope[head] * (i - j) before the softmax.  The larger Baichuan model of the paper's model table
   * (section 3.1.3) is the Llama-style block with these biases in place of the rotary embedding.
   */
  const void *alibi;
  /*
   * Optional biases, each NULL or set independently per layer, element type of the library:
   *   norm1_bias, norm2_bias [H]  of the LayerNorms (norm_kind 1 only; must be NULL otherwise)
   *   bo    [H]  added to the attention's output projection
   *   bup   [F]  added to up(b) before the gelu (mlp_kind 1 or 2 only; must be NULL otherwise)
   *   bdown [H]  added to the MLP's down projection
   * A block with neither a rotation nor score biases (GPT-2: its positions enter with the embedding, outside the
   * layers) is the linear-bias block with all slopes zero.
   */
  const void *norm1_bias, *norm2_bias, *bo, *bup, *bdown;
} stage_layer_weights;

typedef struct stage_handle stage_handle;

/*
 * KV pool layout (part of the ABI: the caller pre-fills the cached context).
 * Layer l starts at kv_pool + l * kv_layer_stride_bytes and holds two bf16 regions:
 *   K: [num_kv_blocks][nkv][d/32][16 positions][32]   a key vector is cut into pieces of 32 elements; the
 *                                                      key of slot s sits at position s with bits 2 and 3
 *                                                      exchanged (slots 0-3, 8-11, 4-7, 12-15)
 *   V: [num_kv_blocks][nkv][d][16 slots]               values are stored transposed inside a block
 * (the orders in which the attention kernels' matrix-core tiles take their rows, so that every load
 * instruction reads runs of 512 bytes or more; stage_kv_element_offset is the map)
 * The V region starts stage_kv_layer_bytes/2 bytes after the K region.  Token j of a sequence
 * lives in block block_table[j / 16] at slot j % 16.
 * stage_kv_layer_bytes: bytes of one layer's pool (both regions).
 */
int stage_kv_layer_bytes(const stage_config *cfg, size_t *out_bytes);

/*
 * Element offset (in bf16 elements from the start of a layer's pool) of cached element
 * (kv = 0 key / 1 value, block, kv_head, slot, dim).  Host-only helper for callers and tests.
 */
int stage_kv_element_offset(const stage_config *cfg, int32_t kv, int32_t block, int32_t kv_head,
                            int32_t slot, int32_t dim, int64_t *out_offset);

/*
 * Host-only check of a micro-batch against a configuration: exactly the validation stage_forward
 * performs before it enqueues anything (same arguments, same error codes), usable without a GPU.
 * On success, and if slot_mapping_out is not NULL, writes the pool slot of every row as
 * stage_forward would report it.
 */
int stage_check_batch(const stage_config *cfg, int32_t num_tokens, const int32_t *positions,
                      int32_t num_seqs, const int32_t *q_lens, const int32_t *ctx_lens,
                      const int32_t *block_tables, int64_t *slot_mapping_out);

/* Bytes of device workspace stage_init needs for this config (activations, split-K and
 * split-KV partial results, per-call metadata, and - see stage_config.weight_copies - the second copy of
 * the projection weights). */
int stage_workspace_bytes(const stage_config *cfg, size_t *out_bytes);

/*
 * Create a stage.  layers: host array [num_layers] of device-pointer structs (copied).
 * kv_pool / workspace: device memory, 256-byte aligned, of at least kv_pool_bytes >=
 * (L-1)*stride + stage_kv_layer_bytes and stage_workspace_bytes.  device: HIP device ordinal
 * that owns all buffers.  Unless the stage keeps copies of its weights (stage_config.weight_copies) no kernel
 * is launched and no device memory is touched; with copies, the weights must be complete on the device when
 * stage_init is called (it reads them on the default stream and returns when the copies are written) and must
 * not change afterwards.
 * Errors: STAGE_ERR_NULL, STAGE_ERR_CONFIG, STAGE_ERR_SIZE, STAGE_ERR_HIP.
 */
int stage_init(const stage_config *cfg, const stage_layer_weights *layers, void *kv_pool,
               size_t kv_pool_bytes, void *workspace, size_t workspace_bytes, int32_t device,
               stage_handle **out);

/*
 * Run the stage's layers on one micro-batch, asynchronously on hip_stream (a hipStream_t;
 * NULL = the default stream).
 *   num_tokens T      rows of hidden_in / hidden_out; T == sum(q_lens), 0 < T <= max_tokens
 *   hidden_in         device bf16 [T][H]; sequences packed one after another
 *   positions         host int32 [T]; RoPE position of every row (>= 0)
 *   num_seqs S        0 < S <= max_seqs
 *   q_lens            host int32 [S]; new tokens of each sequence (1 = decode token, >1 = prefill chunk)
 *   ctx_lens          host int32 [S]; tokens of the sequence already cached (>= 0)
 *   block_tables      host int32 [S][max_blocks_per_seq]; entries beyond ceil((ctx+q)/16) are ignored
 *   hidden_out        device bf16 [T][H]; row t is the output for input row t (the activation
 *                     payload for the next stage).  Must not overlap hidden_in.
 *   slot_mapping_out  host int64 [T] or NULL; receives, for every row, the pool slot
 *                     block_table[j/16]*16 + j%16 (j = ctx + offset in the chunk) its K/V is written to
 * Row i of a sequence attends to cached tokens 0..ctx-1 and to rows 0..i of its own chunk.
 * All metadata, and the fit of every kernel's scratch into the workspace, is checked on the host before
 * anything is enqueued: on STAGE_ERR_NULL / BATCH / BLOCK_TABLE / ALIAS / SIZE nothing was launched and the
 * KV pool is unchanged.  STAGE_ERR_HIP reports a failing HIP runtime call (a copy or a launch itself), which
 * can come after earlier kernels of the call were enqueued.  The host arrays may be reused as soon as the call
 * returns.  The call does not synchronise; asynchronous HIP failures surface at the caller's
 * next synchronisation.  One handle must not be used from two threads at once, and calls on
 * one handle must be issued to streams that execute them in order (the workspace is shared).
 * Errors: STAGE_ERR_NULL, STAGE_ERR_BATCH, STAGE_ERR_BLOCK_TABLE, STAGE_ERR_ALIAS, STAGE_ERR_HIP.
 */
int stage_forward(stage_handle *st, void *hip_stream, int32_t num_tokens, const void *hidden_in,
                  const int32_t *positions, int32_t num_seqs, const int32_t *q_lens,
                  const int32_t *ctx_lens, const int32_t *block_tables, void *hidden_out,
                  int64_t *slot_mapping_out);

/*
 * stage_forward for callers that cannot allocate device memory and so cannot bring a workspace sized for
 * the stage's capacities: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same result (bit for bit) and same errors as stage_forward, but every
 * intermediate of the call - activations between kernels, split-K and split-KV partial results, the per-call
 * metadata - lives in a scratch array of STAGE_STATIC_SCRATCH_BYTES that is part of the library's device
 * image (each GPU the library runs on holds one copy until the process ends); of the workspace given to
 * stage_init nothing is written, and nothing is read but the weights' second copies that stage_init may
 * have put there (stage_config.weight_copies).  The array is carved for exactly this micro-batch (num_tokens rows, num_seqs
 * sequences); a micro-batch that needs more is rejected with STAGE_ERR_SIZE before anything is enqueued.
 * The call allocates nothing, on the device or through the HIP runtime (no hipMalloc, hipFree, event or
 * stream creation; per-kernel timing is off for the call), and nothing in the array has to start at zero:
 * every buffer carved from it is written by the call before it is read.  All calls on one GPU, from any
 * handle, share that GPU's array: calls that overlap on one GPU race; issue them to streams that run them
 * in order.  Additional error: STAGE_ERR_SIZE.
 */
#define STAGE_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int stage_forward_static(stage_handle *st, void *hip_stream, int32_t num_tokens, const void *hidden_in,
                         const int32_t *positions, int32_t num_seqs, const int32_t *q_lens,
                         const int32_t *ctx_lens, const int32_t *block_tables, void *hidden_out,
                         int64_t *slot_mapping_out);

/*
 * Debug taps (for parity tests).  Same as stage_forward, and additionally copies, for layer
 * tap_layer, intermediate tensors into caller device buffers (any may be NULL to skip):
 *   tap_norm1 bf16 [T][H]            RMSNorm output a
 *   tap_qkv   bf16 [T][(nq+2nkv)d]   projection output with q and k already rotated
 *   tap_attn  bf16 [T][nq d]         attention output
 *   tap_h     f32  [T][H]            residual stream after the attention branch
 *   tap_mlp   bf16 [T][F]            silu(gate) * up
 *   tap_x     f32  [T][H]            residual stream after the layer
 */
typedef struct {
  int32_t tap_layer;
  void *tap_norm1, *tap_qkv, *tap_attn, *tap_h, *tap_mlp, *tap_x;
} stage_taps;

int stage_forward_taps(stage_handle *st, void *hip_stream, int32_t num_tokens, const void *hidden_in,
                       const int32_t *positions, int32_t num_seqs, const int32_t *q_lens,
                       const int32_t *ctx_lens, const int32_t *block_tables, void *hidden_out,
                       int64_t *slot_mapping_out, const stage_taps *taps);

/*
 * The two ends of the pipeline.  The head engine turns requests into the first stage's input and
 * the system's output is generated tokens (paper section 3.2.2 "Distributed Inference Engine";
 * section 5 "Metrics"); the definitions are the Llama family's (section 5 "Models").
 *
 * stage_embed: hidden_out[t] = table[token_ids[t]], the input of the first stage.
 *   table       device bf16 [vocab][H] (H = the handle's hidden size), borrowed for the call
 *   token_ids   host int32 [T], each in [0, vocab); validated before anything is enqueued
 *   hidden_out  device bf16 [T][H]
 * Needs no vocab_size in the config.  Errors: STAGE_ERR_NULL, STAGE_ERR_BATCH, STAGE_ERR_HIP.
 *
 * stage_head: for every sequence s of a micro-batch, on its LAST row r(s) = q_lens[0] + .. + q_lens[s] - 1:
 *   logits[s] = RMSNorm(hidden[r(s)]; final_norm, rms_eps) * lm_head^T,  next_tokens[s] = argmax_v logits[s][v]
 * (the smallest index among equal maxima).  The norm is computed in fp32 and rounded to bf16 once, the
 * projection accumulates in fp32, logits stay fp32.
 *   hidden       device bf16 [T][H]: the last stage's hidden_out
 *   q_lens       host int32 [S], sum == T
 *   final_norm   device bf16 [H];  lm_head  device bf16 [vocab][H]; both borrowed for the call
 *   vocab        must equal the config's vocab_size
 *   logits_out   device f32 [S][vocab], or NULL when only the tokens are wanted
 *   next_tokens  device int32 [S]
 * Asynchronous on hip_stream like stage_forward, shares the handle's workspace with it (same ordering
 * rule).  Errors: STAGE_ERR_NULL, STAGE_ERR_CONFIG (vocab mismatch; the wrong head for the stage's norm_kind),
 * STAGE_ERR_BATCH, STAGE_ERR_HIP.
 *
 * stage_head_layernorm: the same for a stage whose blocks use LayerNorms (norm_kind 1; the GPT-2, Falcon and Cohere
 * families end with a LayerNorm too):
 *   logits[s] = LayerNorm(hidden[r(s)]; final_norm, final_norm_bias, rms_eps) * lm_head^T
 *   final_norm_bias  device bf16 [H], or NULL for a LayerNorm without bias
 * stage_head serves stages with norm_kind 0 only, stage_head_layernorm stages with norm_kind 1 only.
 */
int stage_embed(stage_handle *st, void *hip_stream, const void *table, int32_t vocab, int32_t num_tokens,
                const int32_t *token_ids, void *hidden_out);
int stage_head(stage_handle *st, void *hip_stream, int32_t num_tokens, const void *hidden, int32_t num_seqs,
               const int32_t *q_lens, const void *final_norm, const void *lm_head, int32_t vocab,
               void *logits_out, int32_t *next_tokens);
int stage_head_layernorm(stage_handle *st, void *hip_stream, int32_t num_tokens, const void *hidden,
                         int32_t num_seqs, const int32_t *q_lens, const void *final_norm,
                         const void *final_norm_bias, const void *lm_head, int32_t vocab, void *logits_out,
                         int32_t *next_tokens);

/*
 * Start-up profiling (paper section 4.1: every engine times its own stage over a grid of batch sizes and
 * sequence lengths when it starts, and the scheduler sizes its micro-batches from that table).  One point of
 * the table: the stage's latency for a micro-batch of num_seqs sequences, each with q_len new tokens
 * (1 = decode, > 1 = a prefill chunk) after ctx_len cached ones.  Runs stage_forward on such a micro-batch
 * `warmup` times untimed and `iters` times timed (HIP events on hip_stream), synchronises, and writes
 * milliseconds per micro-batch to out_ms.  Sequence s is paged onto blocks s*B .. s*B+B-1 (B = blocks of
 * ctx_len + q_len tokens): the runs append to those blocks and read whatever the pool holds there, so
 * this belongs before the pool holds live sequences.  The values in hidden_in do not matter for the time.
 *   hidden_in / hidden_out   device bf16 [num_seqs * q_len][H], not overlapping
 * Errors: STAGE_ERR_NULL, STAGE_ERR_BATCH (counts outside the stage's capacities), STAGE_ERR_BLOCK_TABLE
 * (the sequences do not fit the block tables or the pool), STAGE_ERR_ALIAS, STAGE_ERR_HIP.
 */
int stage_profile(stage_handle *st, void *hip_stream, int32_t num_seqs, int32_t q_len, int32_t ctx_len,
                  int32_t warmup, int32_t iters, const void *hidden_in, void *hidden_out, double *out_ms);

/*
 * Per-kernel timing with HIP events recorded on the stream the kernels are launched on.
 * stage_profile_enable(st, mask): bit k of mask turns timing of kernel class k on (0 = off).
 * stage_profile_read: synchronises the events recorded so far, adds up the elapsed time of
 * class `kernel` and returns it with the number of timed launches, then forgets them.
 * At most 8192 launches are kept between two reads; later ones are not timed.
 */
enum {
  STAGE_K_RMSNORM = 0,
  STAGE_K_GEMM_QKV = 1,
  STAGE_K_ROPE_APPEND = 2,
  STAGE_K_ATTN_PREFILL = 3,
  STAGE_K_ATTN_DECODE = 4,
  STAGE_K_ATTN_MERGE = 5,
  STAGE_K_GEMM_O = 6,
  STAGE_K_GEMM_GATEUP = 7,
  STAGE_K_GEMM_DOWN = 8,
  STAGE_K_SPLITK_REDUCE = 9,
  STAGE_K_ROPE_TABLE = 10,
  STAGE_K_EMBED = 11,
  STAGE_K_HEAD_NORM = 12,
  STAGE_K_GEMM_HEAD = 13,
  STAGE_K_HEAD_ARGMAX = 14,
  STAGE_K_DEQUANT = 15,      /* 4-bit weights expanded to bf16 ahead of a GEMM */
  STAGE_K_COUNT = 16
};
int stage_profile_enable(stage_handle *st, uint32_t kernel_mask);
int stage_profile_read(stage_handle *st, int32_t kernel, double *out_total_ms, int64_t *out_launches);

/* Name of the device kernel family (as a profiler lists it, without template arguments) that implements a kernel
 * class, for matching profiler output; the projections name their tiled kernel (gemm_tile_kernel) although a
 * launch may run on gemm_tile_arranged_kernel (the weights' copies in operand order), gemm_tile32_kernel (256 x
 * 256 tiles), gemm_tile_w4_kernel (4-bit weights) or gemm_skinny_kernel (at most 64 rows), and prefill
 * attention with two query planes runs on attn_prefill_two_plane_kernel.  Returns NULL for an unknown class. */
const char *stage_kernel_name(int32_t kernel);

/* Release the handle (host memory, events, pinned staging).  Synchronises the device first. */
void stage_destroy(stage_handle *st);

/* Message describing the calling thread's most recent error ("" if none). */
const char *stage_last_error(void);

/* The 16-bit element type this library was built for (see "Element type" at the top): which of the two
 * builds of the half-precision serving configuration of paper section 5 the caller has loaded. */
enum { STAGE_ELEM_BF16 = 0, STAGE_ELEM_F16 = 1 };
int32_t stage_elem_type(void);

#ifdef __cplusplus
}
#endif
#endif /* MOLINK_STAGE_H */
