"""ctypes binding of libmolink_stage.so (bfloat16 elements) and libmolink_stage_f16.so (IEEE half
elements, the same sources and ABI): argument marshalling only.

Every step of the forward pass runs in the library's HIP kernels; torch is used for device
memory, the current stream handle and nothing else.  The library is loaded from the package
directory and there is no fallback: without it every call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmolink_stage.so")
LIB_PATHS = {torch.bfloat16: LIB_PATH, torch.float16: os.path.join(_HERE, "libmolink_stage_f16.so")}
ELEM_TYPES = {torch.bfloat16: 0, torch.float16: 1}      # what stage_elem_type() of each library returns

KERNEL_CLASSES = {
    "rmsnorm": 0, "gemm_qkv": 1, "rope_append": 2, "attn_prefill": 3, "attn_decode": 4, "attn_merge": 5,
    "gemm_o": 6, "gemm_gateup": 7, "gemm_down": 8, "splitk_reduce": 9, "rope_table": 10,
    "embed": 11, "head_norm": 12, "gemm_head": 13, "head_argmax": 14, "dequant": 15,
}


class StageError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"stage error {code}: {message}")
        self.code = code


class StageConfig(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("num_layers", ctypes.c_int32), ("hidden", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("ffn", ctypes.c_int32),
        ("rms_eps", ctypes.c_float), ("rope_theta", ctypes.c_float),
        ("kv_block_size", ctypes.c_int32), ("num_kv_blocks", ctypes.c_int32),
        ("kv_layer_stride_bytes", ctypes.c_int64),
        ("max_tokens", ctypes.c_int32), ("max_seqs", ctypes.c_int32), ("max_blocks_per_seq", ctypes.c_int32),
        ("activation_planes", ctypes.c_int32), ("vocab_size", ctypes.c_int32),
        ("weight_bits", ctypes.c_int32), ("weight_group_size", ctypes.c_int32), ("rotary_dim", ctypes.c_int32),
        ("rope_interleaved", ctypes.c_int32), ("weight_copies", ctypes.c_int32),
        ("norm_kind", ctypes.c_int32), ("mlp_kind", ctypes.c_int32), ("parallel_block", ctypes.c_int32),
        ("rope_scaling", ctypes.c_int32), ("rope_scaling_factor", ctypes.c_float),
        ("rope_low_freq_factor", ctypes.c_float), ("rope_high_freq_factor", ctypes.c_float),
        ("rope_original_max_position", ctypes.c_int32),
    ]


W4_MATRICES = ("wqkv", "wo", "wgate", "wup", "wdown")
W4_SCALES = ("sqkv", "so", "sgate", "sup", "sdown")
W4_ZEROS = ("zqkv", "zo", "zgate", "zup", "zdown")


BLOCK_BIASES = ("norm1_bias", "norm2_bias", "bo", "bup", "bdown")
# tensors a layer may leave out (wgate: the ungated MLP; norm2: a parallel block with one norm)
OPTIONAL_TENSORS = ("bqkv", "qnorm", "knorm", "alibi", "wgate", "norm2") + BLOCK_BIASES
NORM_KINDS = {"rms": 0, "layer": 1}
MLP_KINDS = {"swiglu": 0, "gelu_tanh": 1, "gelu_erf": 2}


class StageLayerWeights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("norm1", "wqkv", "wo", "norm2", "wgate", "wup", "wdown", "bqkv")
                + W4_SCALES + W4_ZEROS + ("qnorm", "knorm", "alibi") + BLOCK_BIASES]


class StageTaps(ctypes.Structure):
    _fields_ = [("tap_layer", ctypes.c_int32)] + [
        (n, ctypes.c_void_p) for n in ("tap_norm1", "tap_qkv", "tap_attn", "tap_h", "tap_mlp", "tap_x")]


_libs: Dict[torch.dtype, ctypes.CDLL] = {}


def load_library(dtype: torch.dtype = torch.bfloat16) -> ctypes.CDLL:
    """Load the built shared library for a 16-bit element type (raises if it has not been built)."""
    if dtype in _libs:
        return _libs[dtype]
    if dtype not in LIB_PATHS:
        raise ValueError(f"no library for element type {dtype}: bfloat16 and float16 are built")
    path = LIB_PATHS[dtype]
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} is missing: build it with `python -m paper_2507_05043_amd.build`")
    lib = ctypes.CDLL(path)
    i32p, i64p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
    cfgp = ctypes.POINTER(StageConfig)
    lib.stage_kv_layer_bytes.argtypes = [cfgp, ctypes.POINTER(ctypes.c_size_t)]
    lib.stage_kv_element_offset.argtypes = [cfgp] + [ctypes.c_int32] * 5 + [i64p]
    lib.stage_check_batch.argtypes = [cfgp, ctypes.c_int32, i32p, ctypes.c_int32, i32p, i32p, i32p, i64p]
    lib.stage_workspace_bytes.argtypes = [cfgp, ctypes.POINTER(ctypes.c_size_t)]
    lib.stage_init.argtypes = [cfgp, ctypes.POINTER(StageLayerWeights), ctypes.c_void_p, ctypes.c_size_t,
                               ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.POINTER(ctypes.c_void_p)]
    fwd = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, i32p, ctypes.c_int32, i32p, i32p,
           i32p, ctypes.c_void_p, i64p]
    lib.stage_forward.argtypes = fwd
    lib.stage_forward_static.argtypes = fwd
    lib.stage_forward_taps.argtypes = fwd + [ctypes.POINTER(StageTaps)]
    lib.stage_embed.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, i32p,
                                ctypes.c_void_p]
    lib.stage_head.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, i32p,
                               ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
    lib.stage_head_layernorm.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32,
                                         i32p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                         ctypes.c_void_p, ctypes.c_void_p]
    lib.stage_profile.argtypes = [ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int32] * 5 + [
        ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(ctypes.c_double)]
    lib.stage_profile_enable.argtypes = [ctypes.c_void_p, ctypes.c_uint32]
    lib.stage_profile_read.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_double), i64p]
    lib.stage_kernel_name.argtypes = [ctypes.c_int32]
    lib.stage_kernel_name.restype = ctypes.c_char_p
    lib.stage_destroy.argtypes = [ctypes.c_void_p]
    lib.stage_destroy.restype = None
    lib.stage_last_error.restype = ctypes.c_char_p
    for name in ("stage_kv_layer_bytes", "stage_kv_element_offset", "stage_check_batch", "stage_workspace_bytes",
                 "stage_init", "stage_forward", "stage_forward_static", "stage_forward_taps", "stage_profile", "stage_profile_enable",
                 "stage_profile_read", "stage_embed", "stage_head", "stage_head_layernorm"):
        getattr(lib, name).restype = ctypes.c_int
    lib.stage_elem_type.restype = ctypes.c_int32
    if lib.stage_elem_type() != ELEM_TYPES[dtype]:
        raise RuntimeError(f"{path} was not built for {dtype}")
    _libs[dtype] = lib
    return lib


def _check(rc: int, lib: Optional[ctypes.CDLL] = None) -> None:
    if rc != 0:
        raise StageError(rc, (lib or load_library()).stage_last_error().decode())


def make_config(*, num_layers, hidden, num_q_heads, num_kv_heads, head_dim, ffn, rms_eps, rope_theta,
                num_kv_blocks, max_tokens, max_seqs, max_blocks_per_seq, kv_block_size=16,
                kv_layer_stride_bytes=None, activation_planes=0, vocab_size=0, weight_bits=0,
                weight_group_size=0, rotary_dim=0, weight_copies=0, rope_interleaved=0, norm_kind=0, mlp_kind=0,
                parallel_block=0, rope_scaling=None) -> StageConfig:
    """rope_scaling: None, ("linear", factor) or ("llama3", factor, low_freq_factor, high_freq_factor,
    original_max_position)."""
    if rope_scaling is None:
        scaling = (0, 0.0, 0.0, 0.0, 0)
    elif rope_scaling[0] == "linear":
        scaling = (1, float(rope_scaling[1]), 0.0, 0.0, 0)
    elif rope_scaling[0] == "llama3":
        scaling = (2, float(rope_scaling[1]), float(rope_scaling[2]), float(rope_scaling[3]), int(rope_scaling[4]))
    else:
        scaling = tuple(rope_scaling)          # raw field values (tests of the validation)
    cfg = StageConfig(ctypes.sizeof(StageConfig), num_layers, hidden, num_q_heads, num_kv_heads, head_dim, ffn,
                      rms_eps, rope_theta, kv_block_size, num_kv_blocks, 0, max_tokens, max_seqs, max_blocks_per_seq,
                      activation_planes, vocab_size, weight_bits, weight_group_size, rotary_dim, int(rope_interleaved),
                      weight_copies, NORM_KINDS.get(norm_kind, norm_kind), MLP_KINDS.get(mlp_kind, mlp_kind),
                      int(parallel_block), *scaling)
    if kv_layer_stride_bytes is None:
        kv_layer_stride_bytes = stage_kv_layer_bytes(cfg)
    cfg.kv_layer_stride_bytes = kv_layer_stride_bytes
    return cfg


def stage_kv_layer_bytes(cfg: StageConfig) -> int:
    out = ctypes.c_size_t()
    _check(load_library().stage_kv_layer_bytes(ctypes.byref(cfg), ctypes.byref(out)))
    return out.value


def stage_workspace_bytes(cfg: StageConfig, dtype: torch.dtype = torch.bfloat16) -> int:
    """Workspace the library for `dtype` needs (the half-precision one never adds a second activation
    plane by itself, so deep stages need less there)."""
    out = ctypes.c_size_t()
    lib = load_library(dtype)
    _check(lib.stage_workspace_bytes(ctypes.byref(cfg), ctypes.byref(out)), lib)
    return out.value


def stage_kv_element_offset(cfg: StageConfig, kv: int, block: int, kv_head: int, slot: int, dim: int) -> int:
    out = ctypes.c_int64()
    _check(load_library().stage_kv_element_offset(ctypes.byref(cfg), kv, block, kv_head, slot, dim, ctypes.byref(out)))
    return out.value


def stage_kernel_name(kernel: int) -> Optional[str]:
    r = load_library().stage_kernel_name(kernel)
    return r.decode() if r else None


def _i32_array(values, count: Optional[int] = None):
    t = torch.as_tensor(values, dtype=torch.int32).contiguous().cpu()
    if count is not None and t.numel() != count:
        raise ValueError(f"expected {count} int32 values, got {t.numel()}")
    return t, ctypes.cast(t.data_ptr(), ctypes.POINTER(ctypes.c_int32))


def stage_check_batch(cfg: StageConfig, positions, q_lens, ctx_lens, block_tables, num_tokens=None) -> List[int]:
    """Host-only validation; returns the slot mapping."""
    pos_t, pos_p = _i32_array(positions)
    q_t, q_p = _i32_array(q_lens)
    c_t, c_p = _i32_array(ctx_lens)
    b_t, b_p = _i32_array(block_tables)
    n = pos_t.numel() if num_tokens is None else num_tokens
    slots = torch.empty(max(n, 1), dtype=torch.int64)
    _check(load_library().stage_check_batch(ctypes.byref(cfg), n, pos_p, q_t.numel(), q_p, c_p, b_p,
                                            ctypes.cast(slots.data_ptr(), ctypes.POINTER(ctypes.c_int64))))
    return slots[:n].tolist()


class Stage:
    """One pipeline stage bound to its weights, KV pool and workspace (all torch CUDA tensors)."""

    def __init__(self, cfg: StageConfig, layers: Sequence[Dict[str, torch.Tensor]], *, device="cuda:0",
                 kv_pool: Optional[torch.Tensor] = None, dtype: torch.dtype = torch.bfloat16):
        lib = load_library(dtype)
        self._lib = lib
        self.dtype = dtype            # the 16-bit element type of weights, activations and the KV pool
        self.cfg = cfg
        self.device = torch.device(device)
        self.layers = [dict(l) for l in layers]          # keep the tensors alive
        arr = (StageLayerWeights * cfg.num_layers)()
        for l, w in enumerate(self.layers):
            four_bit = cfg.weight_bits == 4
            for name, _ in StageLayerWeights._fields_:
                if name in OPTIONAL_TENSORS and w.get(name) is None:
                    continue
                if not four_bit and (name in W4_SCALES or name in W4_ZEROS):
                    continue
                t = w[name]
                want = torch.int32 if four_bit and name in W4_MATRICES else dtype   # code words / elements
                if name == "alibi":
                    want = torch.float32                                             # head slopes
                if t.dtype != want or not t.is_contiguous() or t.device != self.device:
                    raise ValueError(f"layer {l} {name}: need a contiguous {want} tensor on {self.device}")
                setattr(arr[l], name, t.data_ptr())
        layer_bytes = stage_kv_layer_bytes(cfg)
        pool_bytes = (cfg.num_layers - 1) * cfg.kv_layer_stride_bytes + layer_bytes
        if kv_pool is None:
            kv_pool = torch.empty(pool_bytes, dtype=torch.uint8, device=self.device)
        self.kv_pool = kv_pool
        self.workspace = torch.empty(stage_workspace_bytes(cfg, dtype), dtype=torch.uint8, device=self.device)
        handle = ctypes.c_void_p()
        self._check(lib.stage_init(ctypes.byref(cfg), arr, kv_pool.data_ptr(), kv_pool.numel() * kv_pool.element_size(),
                              self.workspace.data_ptr(), self.workspace.numel(), self.device.index or 0,
                              ctypes.byref(handle)))
        self._handle = handle

    def _check(self, rc: int) -> None:
        _check(rc, self._lib)

    # ---- KV pool views (layout of the ABI: K [blocks][nkv][d/32][16 positions][32], V [blocks][nkv][d][16])
    # position of slot s = s with bits 2 and 3 exchanged; the exchange is its own inverse
    _K_SLOT_OF_POSITION = [0, 1, 2, 3, 8, 9, 10, 11, 4, 5, 6, 7, 12, 13, 14, 15]

    def _region(self, layer: int, kv: int) -> torch.Tensor:
        c = self.cfg
        region_bytes = stage_kv_layer_bytes(c) // 2
        start = layer * c.kv_layer_stride_bytes + kv * region_bytes
        return self.kv_pool.view(torch.uint8)[start:start + region_bytes].view(self.dtype)

    def k_view(self, layer: int) -> torch.Tensor:
        c = self.cfg
        return self._region(layer, 0).view(c.num_kv_blocks, c.num_kv_heads, c.head_dim // 32, 16, 32)

    def v_view(self, layer: int) -> torch.Tensor:
        c = self.cfg
        return self._region(layer, 1).view(c.num_kv_blocks, c.num_kv_heads, c.head_dim, 16)

    def write_kv_blocks(self, layer: int, kv: int, blocks: torch.Tensor, values: torch.Tensor) -> None:
        """Store values [n, 16 slots, nkv, d] (bf16, on the device) into the given physical blocks."""
        if kv == 0:
            n, _, nkv, d = values.shape
            order = torch.tensor(self._K_SLOT_OF_POSITION, device=values.device)
            v = values[:, order].reshape(n, 16, nkv, d // 32, 32)          # [n, position, nkv, piece, 32]
            self.k_view(layer)[blocks] = v.permute(0, 2, 3, 1, 4)
        else:
            self.v_view(layer)[blocks] = values.permute(0, 2, 3, 1)

    def read_kv_blocks(self, layer: int, kv: int, blocks: torch.Tensor) -> torch.Tensor:
        """Inverse of write_kv_blocks: [n, 16 slots, nkv, d]."""
        if kv == 0:
            v = self.k_view(layer)[blocks].permute(0, 3, 1, 2, 4)             # [n, position, nkv, piece, 32]
            n, _, nkv, pieces, _ = v.shape
            order = torch.tensor(self._K_SLOT_OF_POSITION, device=v.device)  # slot of position == position of slot
            return v.reshape(n, 16, nkv, pieces * 32)[:, order]
        return self.v_view(layer)[blocks].permute(0, 3, 1, 2)

    # ---- start-up profiling: one point of the latency table, timed by the library
    def profile(self, num_seqs: int, q_len: int, ctx_len: int, *, warmup: int = 2, iters: int = 5) -> float:
        """Milliseconds per micro-batch of `num_seqs` sequences with `q_len` new tokens after `ctx_len` cached ones."""
        t = num_seqs * q_len
        hidden = torch.zeros(max(t, 1), self.cfg.hidden, dtype=self.dtype, device=self.device)
        out = torch.empty_like(hidden)
        ms = ctypes.c_double()
        stream = torch.cuda.current_stream(self.device).cuda_stream
        self._check(self._lib.stage_profile(self._handle, ctypes.c_void_p(stream), num_seqs, q_len, ctx_len, warmup, iters,
                                            ctypes.c_void_p(hidden.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                                            ctypes.byref(ms)))
        return ms.value

    # ---- the forward pass
    def forward(self, hidden: torch.Tensor, positions, q_lens, ctx_lens, block_tables, *,
                out: Optional[torch.Tensor] = None, want_slots: bool = False, taps_layer: Optional[int] = None,
                static_scratch: bool = False):
        """static_scratch: call stage_forward_static (the library's own scratch array instead of the workspace)."""
        lib = self._lib
        c = self.cfg
        t = hidden.shape[0]
        if hidden.dtype != self.dtype or not hidden.is_contiguous() or hidden.shape[1] != c.hidden:
            raise ValueError("hidden must be a contiguous 16-bit [T, hidden] tensor")
        pos_t, pos_p = _i32_array(positions, t)
        q_t, q_p = _i32_array(q_lens)
        c_t, c_p = _i32_array(ctx_lens, q_t.numel())
        b_t, b_p = _i32_array(block_tables, q_t.numel() * c.max_blocks_per_seq)
        if out is None:
            out = torch.empty_like(hidden)
        slots = torch.empty(t, dtype=torch.int64) if want_slots else None
        slots_p = ctypes.cast(slots.data_ptr(), ctypes.POINTER(ctypes.c_int64)) if want_slots else None
        stream = torch.cuda.current_stream(self.device).cuda_stream
        args = [self._handle, ctypes.c_void_p(stream), t, hidden.data_ptr(), pos_p, q_t.numel(), q_p, c_p, b_p,
                out.data_ptr(), slots_p]
        taps = None
        if static_scratch:
            if taps_layer is not None:
                raise ValueError("the static-scratch entry point has no taps")
            self._check(lib.stage_forward_static(*args))
        elif taps_layer is None:
            self._check(lib.stage_forward(*args))
        else:
            qkv_out = (c.num_q_heads + 2 * c.num_kv_heads) * c.head_dim
            dev = self.device
            taps = {
                "a": torch.empty(t, c.hidden, dtype=self.dtype, device=dev),
                "qkv": torch.empty(t, qkv_out, dtype=self.dtype, device=dev),
                "attn": torch.empty(t, c.num_q_heads * c.head_dim, dtype=self.dtype, device=dev),
                "h": torch.empty(t, c.hidden, dtype=torch.float32, device=dev),
                "m": torch.empty(t, c.ffn, dtype=self.dtype, device=dev),
                "x": torch.empty(t, c.hidden, dtype=torch.float32, device=dev),
            }
            st = StageTaps(taps_layer, taps["a"].data_ptr(), taps["qkv"].data_ptr(), taps["attn"].data_ptr(),
                           taps["h"].data_ptr(), taps["m"].data_ptr(), taps["x"].data_ptr())
            self._check(lib.stage_forward_taps(*args, ctypes.byref(st)))
        result = [out]
        if want_slots:
            result.append(slots.tolist())
        if taps is not None:
            result.append(taps)
        return result[0] if len(result) == 1 else tuple(result)

    # ---- the two ends of the pipeline
    def embed(self, table: torch.Tensor, token_ids, *, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        c = self.cfg
        if table.dtype != self.dtype or not table.is_contiguous() or table.shape[1] != c.hidden:
            raise ValueError("table must be a contiguous 16-bit [vocab, hidden] tensor")
        ids_t, ids_p = _i32_array(token_ids)
        t = ids_t.numel()
        if out is None:
            out = torch.empty(t, c.hidden, dtype=self.dtype, device=self.device)
        stream = torch.cuda.current_stream(self.device).cuda_stream
        self._check(self._lib.stage_embed(self._handle, ctypes.c_void_p(stream), table.data_ptr(), table.shape[0], t,
                                          ids_p, out.data_ptr()))
        return out

    def head(self, hidden: torch.Tensor, q_lens, final_norm: torch.Tensor, lm_head: torch.Tensor, *,
             want_logits: bool = True, final_norm_bias: Optional[torch.Tensor] = None):
        """(next_tokens int32 [S], logits f32 [S, vocab] or None) for the last row of every sequence.
        A stage whose blocks use LayerNorms ends with one (stage_head_layernorm; final_norm_bias optional)."""
        c = self.cfg
        if hidden.dtype != self.dtype or not hidden.is_contiguous() or hidden.shape[1] != c.hidden:
            raise ValueError("hidden must be a contiguous 16-bit [T, hidden] tensor")
        for w in (final_norm, lm_head):
            if w.dtype != self.dtype or not w.is_contiguous():
                raise ValueError("final_norm and lm_head must be contiguous 16-bit tensors")
        if lm_head.shape[1] != c.hidden or final_norm.numel() != c.hidden:
            raise ValueError("final_norm must be [hidden] and lm_head [vocab, hidden]")
        q_t, q_p = _i32_array(q_lens)
        s = q_t.numel()
        vocab = lm_head.shape[0]
        logits = torch.empty(s, vocab, dtype=torch.float32, device=self.device) if want_logits else None
        tokens = torch.empty(s, dtype=torch.int32, device=self.device)
        stream = torch.cuda.current_stream(self.device).cuda_stream
        if c.norm_kind == 0 and final_norm_bias is None:
            self._check(self._lib.stage_head(self._handle, ctypes.c_void_p(stream), hidden.shape[0], hidden.data_ptr(), s,
                                             q_p, final_norm.data_ptr(), lm_head.data_ptr(), vocab,
                                             logits.data_ptr() if want_logits else None, tokens.data_ptr()))
        else:
            if final_norm_bias is not None and (final_norm_bias.dtype != self.dtype or not final_norm_bias.is_contiguous()
                                                or final_norm_bias.numel() != c.hidden):
                raise ValueError("final_norm_bias must be a contiguous 16-bit [hidden] tensor")
            self._check(self._lib.stage_head_layernorm(
                self._handle, ctypes.c_void_p(stream), hidden.shape[0], hidden.data_ptr(), s, q_p, final_norm.data_ptr(),
                final_norm_bias.data_ptr() if final_norm_bias is not None else None, lm_head.data_ptr(), vocab,
                logits.data_ptr() if want_logits else None, tokens.data_ptr()))
        return tokens, logits

    # ---- per-kernel timing
    def profile_enable(self, kernels: Sequence[str]) -> None:
        mask = 0
        for k in kernels:
            mask |= 1 << KERNEL_CLASSES[k]
        self._check(self._lib.stage_profile_enable(self._handle, mask))

    def profile_read(self, kernel: str):
        ms, n = ctypes.c_double(), ctypes.c_int64()
        self._check(self._lib.stage_profile_read(self._handle, KERNEL_CLASSES[kernel], ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, n.value

    def close(self) -> None:
        if getattr(self, "_handle", None):
            self._lib.stage_destroy(self._handle)
            self._handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
