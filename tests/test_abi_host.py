"""Host-side checks that need no GPU: the library loads, exports what the header declares,
validates micro-batches, and maps slots and KV coordinates exactly."""
import ctypes
import os
import random
import re

import pytest
import torch

import oracle
from paper_2507_05043_amd import StageError, stage as S, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not all(os.path.exists(p) for p in S.LIB_PATHS.values()):
        from paper_2507_05043_amd import build
        build.build()
    return S.load_library()


@pytest.fixture(scope="module", params=[torch.bfloat16, torch.float16], ids=["bf16", "f16"])
def each_lib(request, lib):
    return S.load_library(request.param)


def tiny_cfg(**kw):
    args = dict(num_layers=2, hidden=256, num_q_heads=4, num_kv_heads=2, head_dim=64, ffn=688, rms_eps=1e-5,
                rope_theta=1e4, num_kv_blocks=40, max_tokens=128, max_seqs=8, max_blocks_per_seq=12)
    args.update(kw)
    return S.make_config(**args)


def test_library_exports_every_declared_symbol(each_lib):
    lib = each_lib
    header = open(os.path.join(ROOT, "include", "molink_stage.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(stage_[a-z_]+)\s*\(", header))
    assert {"stage_init", "stage_forward", "stage_forward_taps", "stage_check_batch", "stage_destroy"} <= names
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} is declared in the header but not exported"


def test_library_exports_every_handoff_symbol(each_lib):
    lib = each_lib
    header = open(os.path.join(ROOT, "include", "molink_handoff.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(handoff_[a-z_]+)\s*\(", header))
    assert {"handoff_plan", "handoff_sender_create", "handoff_sender_submit", "handoff_sender_destroy"} <= names
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} is declared in the header but not exported"


def test_handoff_plan_equals_the_model_on_random_layouts(lib):
    from oracle import handoff_oracle as M
    from paper_2507_05043_amd import handoff
    rng = random.Random(0)
    for _ in range(200):
        q = [rng.choice([1, 1, 1, rng.randint(2, 50)]) for _ in range(rng.randint(1, 20))]
        row, chunk = rng.choice([2, 512, 7168]), rng.choice([3, 100, 4096, 1 << 20])
        d, p = M.split_payload(q, row, chunk)
        assert handoff.plan(q, row, chunk) == d + p
    with pytest.raises(handoff.HandoffError):
        handoff.plan([3, 0], 8, 8)
    with pytest.raises(handoff.HandoffError):
        handoff.plan([3], 8, 0)


def test_each_library_reports_its_element_type_and_the_same_host_answers(lib):
    f16 = S.load_library(torch.float16)
    assert lib.stage_elem_type() == 0 and f16.stage_elem_type() == 1
    cfg = tiny_cfg(vocab_size=1000)
    for fn in ("stage_kv_layer_bytes", "stage_workspace_bytes"):       # a shallow stage has the same sizes in both (deep ones differ by the second activation plane)
        a, b = ctypes.c_size_t(), ctypes.c_size_t()
        assert getattr(lib, fn)(ctypes.byref(cfg), ctypes.byref(a)) == 0
        assert getattr(f16, fn)(ctypes.byref(cfg), ctypes.byref(b)) == 0
        assert a.value == b.value > 0
    with pytest.raises(ValueError):
        S.load_library(torch.float32)


def test_half_activations_are_a_mode_of_the_bfloat16_library_only(lib):
    cfg = tiny_cfg(activation_planes=3)
    out = ctypes.c_size_t()
    assert lib.stage_workspace_bytes(ctypes.byref(cfg), ctypes.byref(out)) == 0
    one = ctypes.c_size_t()
    cfg1 = tiny_cfg(activation_planes=1)
    assert lib.stage_workspace_bytes(ctypes.byref(cfg1), ctypes.byref(one)) == 0
    assert out.value > one.value                       # the second plane of the rotated queries
    assert S.load_library(torch.float16).stage_workspace_bytes(ctypes.byref(cfg), ctypes.byref(out)) == -2


def test_automatic_activation_mode_goes_by_depth(lib):
    """Left to the library, the bfloat16 stage carries one bfloat16 plane up to four layers, half activations from
    five and the extra half plane of the q/k/v input from nine; seen from the host as the workspace each mode needs."""
    def ws(layers, planes, dtype=torch.bfloat16):
        return S.stage_workspace_bytes(tiny_cfg(num_layers=layers, activation_planes=planes, weight_copies=1), dtype)
    for layers, mode in ((1, 1), (4, 1), (5, 3), (8, 3), (9, 4), (20, 4)):
        assert ws(layers, 0) == ws(layers, mode), (layers, mode)
    assert ws(8, 1) < ws(8, 3) < ws(8, 4) <= ws(8, 2)
    # the half-precision library never takes a mode of its own accord
    assert ws(20, 0, torch.float16) == ws(20, 1, torch.float16)


def test_matrices_of_four_gib_and_more_are_accepted(lib):
    """Tile addressing takes a 64-bit base per workgroup, so an output head of 262144 x 8192 (4 GiB) and
    projections of that size are within the configuration limits."""
    cfg = tiny_cfg(hidden=8192, num_q_heads=64, num_kv_heads=8, head_dim=128, ffn=8192 * 36, vocab_size=262144,
                   max_tokens=64, max_seqs=64)
    assert S.stage_workspace_bytes(cfg) > 64 * 262144 * 4


def test_config_struct_matches_header_size(lib):
    # uint32 + 6 int32 + 2 float + 2 int32 (+ 4 pad) + int64 + 14 int32 + 3 float + int32
    assert ctypes.sizeof(S.StageConfig) == 128
    assert ctypes.sizeof(S.StageLayerWeights) == 26 * ctypes.sizeof(ctypes.c_void_p)
    assert S.stage_workspace_bytes(tiny_cfg()) > 0


@pytest.mark.parametrize("bad", [dict(kv_block_size=32), dict(head_dim=96), dict(hidden=252), dict(num_q_heads=5),
                                 dict(num_q_heads=34, num_kv_heads=2), dict(rms_eps=0.0), dict(num_layers=0),
                                 dict(activation_planes=5), dict(vocab_size=1001), dict(vocab_size=32),
                                 dict(rotary_dim=8), dict(rotary_dim=40), dict(rotary_dim=80),
                                 dict(weight_bits=3), dict(weight_group_size=128), dict(weight_bits=4, weight_group_size=48),
                                 dict(weight_bits=4, weight_group_size=128, ffn=768 + 64),
                                 dict(weight_bits=4, weight_group_size=128),    # ffn 688 is no multiple of 128
                                 dict(rope_scaling=(3, 2.0, 0.0, 0.0, 0)), dict(rope_scaling=(0, 2.0, 0.0, 0.0, 0)),
                                 dict(rope_scaling=("linear", 0.5)), dict(rope_scaling=(1, 2.0, 1.0, 4.0, 8192)),
                                 dict(rope_scaling=("llama3", 8.0, 4.0, 1.0, 8192)), dict(rope_scaling=("llama3", 8.0, 1.0, 4.0, 0)),
                                 dict(norm_kind=2), dict(mlp_kind=3), dict(mlp_kind=-1), dict(parallel_block=2),
                                 dict(weight_bits=4, weight_group_size=128, ffn=768, mlp_kind=1),
                                 dict(weight_bits=4, weight_group_size=128, ffn=768, parallel_block=1)])
def test_unsupported_configs_are_rejected(lib, bad):
    with pytest.raises(StageError) as ei:
        cfg = tiny_cfg(**bad)
        S.stage_workspace_bytes(cfg)
    assert ei.value.code == -2


def test_struct_size_is_checked(lib):
    cfg = tiny_cfg()
    cfg.struct_size = 64
    with pytest.raises(StageError) as ei:
        S.stage_workspace_bytes(cfg)
    assert ei.value.code == -2


def test_slot_mapping_is_bit_exact_against_the_oracle(lib):
    rng = random.Random(5)
    for trial in range(20):
        n_seq = rng.randint(1, 8)
        q_lens = [rng.choice([1, 1, 1, 2, 7, 16, 17, 33]) for _ in range(n_seq)]
        ctx_lens = [rng.choice([0, 1, 15, 16, 17, 31, 64, 100]) for _ in range(n_seq)]
        mb = synth.make_microbatch(q_lens, ctx_lens, seed=trial, max_blocks_per_seq=12)
        cfg = tiny_cfg(num_kv_blocks=mb.num_kv_blocks, max_tokens=max(128, mb.num_tokens))
        got = S.stage_check_batch(cfg, mb.positions, mb.q_lens, mb.ctx_lens, mb.block_tables)
        assert got == oracle.slot_mapping(q_lens, ctx_lens, mb.block_tables, 16)


def test_batch_validation_errors(lib):
    mb = synth.make_microbatch([5, 1, 1], [0, 20, 3], seed=1, max_blocks_per_seq=12)
    cfg = tiny_cfg(num_kv_blocks=mb.num_kv_blocks)
    ok = dict(positions=mb.positions, q_lens=mb.q_lens, ctx_lens=mb.ctx_lens, block_tables=mb.block_tables)
    S.stage_check_batch(cfg, **ok)

    def expect(code, **change):
        args = dict(ok)
        args.update(change)
        with pytest.raises(StageError) as ei:
            S.stage_check_batch(cfg, **args)
        assert ei.value.code == code, ei.value

    expect(-4, q_lens=[5, 0, 1])
    expect(-4, q_lens=[4, 1, 1])                              # sum(q_lens) != T
    expect(-4, ctx_lens=[0, -1, 3])
    expect(-4, positions=torch.tensor([0, 1, 2, 3, -4, 20, 3], dtype=torch.int32))
    bad = mb.block_tables.clone()
    bad[1, 1] = mb.num_kv_blocks
    expect(-5, block_tables=bad)
    bad = mb.block_tables.clone()
    bad[0, 0] = -1
    expect(-5, block_tables=bad)
    expect(-5, ctx_lens=[0, 16 * 12, 3])                      # needs 13 blocks, rows hold 12
    small = tiny_cfg(num_kv_blocks=mb.num_kv_blocks, max_tokens=6)
    with pytest.raises(StageError) as ei:
        S.stage_check_batch(small, **ok)
    assert ei.value.code == -4
    few = tiny_cfg(num_kv_blocks=mb.num_kv_blocks, max_seqs=2)
    with pytest.raises(StageError) as ei:
        S.stage_check_batch(few, **ok)
    assert ei.value.code == -4
    # entries past a sequence's need are ignored, whatever they hold
    junk = mb.block_tables.clone()
    junk[2, 1:] = 10 ** 6
    S.stage_check_batch(cfg, **dict(ok, block_tables=junk))


def test_kv_element_offset_is_a_bijection_with_the_documented_layout(lib):
    cfg = tiny_cfg(num_kv_blocks=3)
    nb, nkv, d = 3, cfg.num_kv_heads, cfg.head_dim
    layer_elems = S.stage_kv_layer_bytes(cfg) // 2
    assert layer_elems == 2 * nb * nkv * 16 * d
    seen = set()
    for kv in (0, 1):
        for b in range(nb):
            for h in range(nkv):
                for s in (0, 1, 15):
                    for e in (0, 1, d - 1):
                        off = S.stage_kv_element_offset(cfg, kv, b, h, s, e)
                        assert 0 <= off < layer_elems and off not in seen
                        seen.add(off)
                        region = kv * (layer_elems // 2)
                        base = (b * nkv + h) * 16 * d
                        pos = (s & 3) | ((s & 8) >> 1) | ((s & 4) << 1)     # bits 2 and 3 of the slot exchanged
                        want = region + base + (((e // 32) * 16 + pos) * 32 + e % 32 if kv == 0 else e * 16 + s)
                        assert off == want
    with pytest.raises(StageError):
        S.stage_kv_element_offset(cfg, 0, 3, 0, 0, 0)


def test_output_head_adds_its_scratch_to_the_workspace(lib):
    base = S.stage_workspace_bytes(tiny_cfg())
    with_head = S.stage_workspace_bytes(tiny_cfg(vocab_size=1000))
    # at least the normalised rows [S, H] bf16 and the fp32 logits [S, vocab]
    assert with_head - base >= 8 * 256 * 2 + 8 * 1000 * 4


def test_four_bit_weights_add_room_for_one_expanded_projection(lib):
    base = S.stage_workspace_bytes(tiny_cfg(ffn=768, weight_copies=1))
    w4 = S.stage_workspace_bytes(tiny_cfg(ffn=768, weight_bits=4, weight_group_size=128))
    assert w4 - base >= 2 * 768 * 256 * 2          # gate and up [F][H] as bf16


def test_kernel_names(lib):
    assert S.stage_kernel_name(S.KERNEL_CLASSES["gemm_head"]) == "gemm_tile_kernel"
    assert S.stage_kernel_name(S.KERNEL_CLASSES["head_argmax"]) == "argmax_rows_kernel"
    assert S.stage_kernel_name(S.KERNEL_CLASSES["attn_decode"]) == "attn_decode_kernel"
    assert S.stage_kernel_name(S.KERNEL_CLASSES["dequant"]) == "dequant_w4_kernel"
    assert S.stage_kernel_name(99) is None


def test_weight_copies_are_counted_in_the_workspace(lib):
    """The second copy of the weights (operand order) sits behind the workspace proper: one more copy of every
    projection matrix whose input width is a multiple of 256, rows padded to 32, when the stage can see more than 64
    rows, the weights are 16-bit and the stage runs one activation plane."""
    def ws(**kw):
        return S.stage_workspace_bytes(tiny_cfg(**kw))
    big = dict(hidden=512, num_q_heads=4, num_kv_heads=2, head_dim=128, ffn=1000, max_tokens=300, max_seqs=8)
    # q/k/v [1024][512], o [512][512], gate and up [1000 -> 1024][512]; down has K = 1000: no copy
    per_layer = (1024 * 512 + 512 * 512 + 2 * 1024 * 512) * 2
    assert ws(**big) - ws(weight_copies=1, **big) == 2 * per_layer
    assert ws(**dict(big, max_tokens=64)) == ws(weight_copies=1, **dict(big, max_tokens=64))
    assert ws(activation_planes=2, **big) == ws(activation_planes=2, weight_copies=1, **big)
    w4 = dict(big, ffn=1024, weight_bits=4, weight_group_size=128)
    assert ws(**w4) == ws(weight_copies=1, **w4)
    with pytest.raises(S.StageError):
        ws(weight_copies=2, **big)


def test_rope_pairing_flag_is_validated(lib):
    assert S.stage_workspace_bytes(tiny_cfg(rope_interleaved=1)) == S.stage_workspace_bytes(tiny_cfg())
    with pytest.raises(S.StageError):
        S.stage_workspace_bytes(tiny_cfg(rope_interleaved=2))


def test_block_kinds_size_the_workspace(lib):
    """A parallel block keeps the second norm of the block's input (one more [T][H] plane), an ungated MLP its first
    product in fp32 before bias and gelu ([T][F] floats) - and has one matrix less to copy into operand order."""
    base = S.stage_workspace_bytes(tiny_cfg(weight_copies=1))
    assert S.stage_workspace_bytes(tiny_cfg(weight_copies=1, norm_kind="layer")) == base
    par = S.stage_workspace_bytes(tiny_cfg(weight_copies=1, parallel_block=1))
    assert 128 * 256 * 2 <= par - base < 128 * 256 * 2 + 512
    ung = S.stage_workspace_bytes(tiny_cfg(weight_copies=1, mlp_kind="gelu_tanh"))
    assert ung - base >= 128 * 688 * 4 - 2 * 1024 * 1024        # the split-K scratch may shrink: no gate/up pair
    wide = dict(ffn=768, max_tokens=128)
    with_gate = S.stage_workspace_bytes(tiny_cfg(**wide)) - S.stage_workspace_bytes(tiny_cfg(weight_copies=1, **wide))
    without = (S.stage_workspace_bytes(tiny_cfg(mlp_kind="gelu_erf", **wide))
               - S.stage_workspace_bytes(tiny_cfg(mlp_kind="gelu_erf", weight_copies=1, **wide)))
    assert 0 < without < with_gate


def test_rope_scaling_settings_are_accepted(lib):
    base = S.stage_workspace_bytes(tiny_cfg())
    assert S.stage_workspace_bytes(tiny_cfg(rope_scaling=("linear", 4.0))) == base
    assert S.stage_workspace_bytes(tiny_cfg(rope_scaling=("llama3", 8.0, 1.0, 4.0, 8192))) == base
