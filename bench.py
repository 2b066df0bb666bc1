#!/usr/bin/env python3
"""Benchmark of one pipeline stage's forward pass on one MI355X.

A step is one stage_forward (all layers, every kernel of the path) over one seeded synthetic
micro-batch whose inputs are already resident in HBM.  Headline workload: the largest single-GPU
configuration, the Llama-3-70B-shaped stage (20 of 80 layers) on a pure-decode micro-batch of 256
sequences with contexts in [1024, 8192].  Prints one JSON line: stage tokens/s, latency per micro-batch,
the roofline of the dominant kernel measured with HIP events on the launch stream, the CPU oracle
timed on a bounded sample, and - unless a single workload was asked for - one entry per other
configuration (Llama-2-7B-shaped decode, Qwen2-7B-shaped mixed, token-budget sweep) with its own
latency and roofline line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# HBM bytes per launch (reads + writes) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled by what the
# same counter reads for a plain 1 GiB copy (profiles/hbm_traffic_*.md).  A figure is only reported while the
# kernel source it was taken on is unchanged.
MEASURED_TRAFFIC = {
    ("attn_decode", "llama3-70b", 0): {"bytes": 4.92216e9 + 2.95565e7, "source": "csrc/attention.hip",
                                       "sha256_16": "7730ca679be14cef"},
    ("attn_decode", "llama2-7b", 0): {"bytes": 1.29793e9 + 3.71088e6, "source": "csrc/attention.hip",
                                      "sha256_16": "7730ca679be14cef"},
}

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0
HEADLINE = "llama3-70b"
# (workload, sweep budget) of the per-configuration entries; the headline's own entry is the headline run itself
# the stage's other builds: the half-precision library and 4-bit weights on the small decode workload, 4-bit weights
# on the headline workload (the paper serves its 70B model with 4-bit weights, section 5 "Models")
VARIANTS = [("llama2-7b", {"dtype": "f16"}), ("llama2-7b", {"weights": "w4"}), ("llama3-70b", {"weights": "w4"})]
PER_CONFIG = [("llama2-7b", None), ("qwen2-7b", None), ("llama3-70b", None), ("sweep", 64), ("sweep", 128), ("sweep", 256),
              ("sweep", 512), ("sweep", 1024), ("sweep", 2048)]


def algorithmic_work(shape, mb, weight_bytes_per_param=2.0):
    """Bytes and flops the method must move / compute per call (weights once, KV once per KV head)."""
    kv_tok = 4 * shape.num_kv_heads * shape.head_dim                       # K+V bytes per token per layer
    dec_keys = sum(c + 1 for q, c in zip(mb.q_lens, mb.ctx_lens) if q == 1)
    pre_keys = sum(c + q for q, c in zip(mb.q_lens, mb.ctx_lens) if q > 1)
    t = mb.num_tokens
    attn_flops = 0
    for q, c in zip(mb.q_lens, mb.ctx_lens):
        attn_flops += 4 * shape.num_q_heads * shape.head_dim * sum(c + i + 1 for i in range(q))
    weight_bytes = int(weight_bytes_per_param * shape.params_per_layer)
    per_layer_bytes = weight_bytes + (dec_keys + pre_keys) * kv_tok + t * kv_tok
    return {
        "decode_attn_bytes_per_layer": dec_keys * kv_tok,
        "weight_bytes_per_layer": weight_bytes,
        "bytes_per_call": shape.num_layers * per_layer_bytes + 2 * t * shape.hidden * 2,
        "gemm_flops_per_layer": 2 * shape.params_per_layer * t,
        "attn_flops_per_layer": attn_flops,
        "flops_per_call": shape.num_layers * (2 * shape.params_per_layer * t + attn_flops),
    }


def measured_traffic(kernel, workload, seed):
    import hashlib
    rec = MEASURED_TRAFFIC.get((kernel, workload, seed))
    if rec is None:
        return None
    path = os.path.join(ROOT, "paper_2507_05043_amd", rec["source"])
    with open(path, "rb") as f:
        if hashlib.sha256(f.read()).hexdigest()[:16] != rec["sha256_16"]:
            return None
    return rec["bytes"]


def cpu_baseline(shape, mb, seed, sample_seqs):
    """The oracle, as it stands, on a sample of whole sequences at full depth (rows of different
    sequences are independent).  Returns tokens/s of the host cores."""
    import torch
    import oracle
    from paper_2507_05043_amd import synth
    from tests.gpu_harness import sub_problem
    from tests.helpers import oracle_shape
    seqs = list(range(0, mb.num_seqs, max(1, mb.num_seqs // sample_seqs)))[:sample_seqs]
    sub, rows, pool = sub_problem(shape, mb, seqs, seed, dtype=torch.float32, draw_device="cuda:0")
    layers = [{k: v.cpu() for k, v in synth.draw_layer_weights(shape, l, seed=seed, device="cuda:0").items()}
              for l in range(shape.num_layers)]
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=seed)[rows]
    t0 = time.perf_counter()
    oracle.stage_forward(oracle_shape(shape), layers, hidden, sub.positions, sub.q_lens, sub.ctx_lens,
                         sub.block_tables, pool, dtype=torch.float32)
    dt = time.perf_counter() - t0
    return {"value": sub.num_tokens / dt, "unit": "tokens/s", "cores": torch.get_num_threads(), "kind": "oracle",
            "sample": f"{len(seqs)} of {mb.num_seqs} sequences ({sub.num_tokens} tokens) of the {shape.name} workload at "
                      f"full depth, fp32, {dt:.1f} s"}


def run_workload(args, workload, budget, steps, warmup, extras):
    """Time `steps` forward passes of one workload; returns the result fields of that workload."""
    import torch
    from paper_2507_05043_amd import KERNEL_CLASSES, synth
    from paper_2507_05043_amd import stage as _stage
    from paper_2507_05043_amd.harness import make_stage

    # progress goes to stderr (stdout carries the one JSON line): a run of several minutes must not look hung
    t_begin = time.time()
    print(f"[bench] {workload}{'' if budget is None else ' budget ' + str(budget)} weights={args.weights} "
          f"dtype={args.dtype}: setting up", file=sys.stderr, flush=True)
    shape, mb = synth.workload(workload, seed=args.seed, budget=budget or 256)
    w4 = args.weights == "w4"
    elem = torch.float16 if args.dtype == "f16" else torch.bfloat16
    # 4 bits per weight plus a bf16 scale and a bf16 zero point per 128 weights
    work = algorithmic_work(shape, mb, 0.5 + 4.0 / 128 if w4 else 2.0)
    kv_bytes = shape.num_layers * mb.num_kv_blocks * 16 * 4 * shape.num_kv_heads * shape.head_dim
    alias = kv_bytes + work["weight_bytes_per_layer"] * shape.num_layers > 250e9     # timing only: layers share one pool
    want_ends = extras and args.ends
    st = make_stage(shape, mb, args.seed, alias_layers=alias, vocab_size=shape.vocab if want_ends else 0,
                    qkv_bias=workload == "qwen2-7b",     # the Qwen2 family has a q/k/v bias
                    weight_group_size=128 if w4 else 0, dtype=elem, pool_first=not args.weights_first)
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=args.seed, device="cuda:0", dtype=elem)
    out = torch.empty_like(hidden)
    n_dec = sum(1 for q in mb.q_lens if q == 1)
    decode_bound = work["decode_attn_bytes_per_layer"] / (HBM_PEAK_GBS * 1e9) >= \
        (work["gemm_flops_per_layer"] + work["attn_flops_per_layer"]) / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    dominant = "attn_decode" if (n_dec and decode_bound) else "gemm_gateup"

    def step():
        st.forward(hidden, mb.positions, mb.q_lens, mb.ctx_lens, mb.block_tables, out=out)

    print(f"[bench]   stage ready after {time.time() - t_begin:.0f} s, timing {steps} steps", file=sys.stderr, flush=True)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    st.profile_enable([dominant])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    dom_ms, dom_n = st.profile_read(dominant)
    st.profile_enable([])
    ms_per_step = elapsed / steps * 1e3
    tokens_per_s = mb.num_tokens * steps / elapsed

    avg_ms = dom_ms / max(dom_n, 1)
    if dominant == "attn_decode":
        achieved = work["decode_attn_bytes_per_layer"] / (avg_ms * 1e-3) / 1e9
        roofline = {"kernel": _stage.stage_kernel_name(KERNEL_CLASSES[dominant]), "bound": "hbm",
                    "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": measured_traffic(dominant, workload, args.seed) if args.dtype == "bf16" and not w4 else None,
                    "avg_launch_ms": round(avg_ms, 5), "launches": dom_n,
                    "algorithmic_bytes_per_launch": work["decode_attn_bytes_per_layer"]}
    else:
        flops = 2 * (2 * shape.hidden * shape.ffn) * mb.num_tokens
        achieved = flops / (avg_ms * 1e-3) / 1e12
        roofline = {"kernel": _stage.stage_kernel_name(KERNEL_CLASSES[dominant]), "bound": "mfma",
                    "achieved": round(achieved, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                    "avg_launch_ms": round(avg_ms, 5), "launches": dom_n, "flops_per_launch": flops}

    # what the library does by itself by depth (see stage_config.activation_planes)
    if args.dtype != "bf16" or shape.num_layers < 5:
        inputs = args.dtype
    else:
        inputs = "IEEE half (bf16 weights converted in the GEMMs, or once into the stage's copies)"
    without = type(st.cfg).from_buffer_copy(st.cfg)
    without.weight_copies = 1
    copy_bytes = _stage.stage_workspace_bytes(st.cfg, st.dtype) - _stage.stage_workspace_bytes(without, st.dtype)
    copies = (f"second copy of the projection weights in MFMA operand order, written by stage_init "
              f"({copy_bytes / 1e9:.2f} GB incl. its split-K scratch)" if copy_bytes > 0 else "none")
    if roofline["bound"] == "mfma" and copy_bytes > 0 and mb.num_tokens > 128:
        # the projection kernel of a stage that keeps the copies; a last tile row of at most 128 rows runs on 128-row
        # tiles in the same launch (the kernel trace lists that launch under the second name)
        ragged = mb.num_tokens > 256 and 0 < mb.num_tokens % 256 <= 128
        roofline["kernel"] = "gemm_tile_arranged_ragged_kernel" if ragged else "gemm_tile_arranged_kernel"
    tag = f"sweep budget {budget}: " if workload == "sweep" else ""
    result = {
        "value": round(tokens_per_s, 1), "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 4),
        "config": {"workload": f"{tag}{shape.name}: L={shape.num_layers} H={shape.hidden} nq={shape.num_q_heads} "
                               f"nkv={shape.num_kv_heads} d={shape.head_dim} F={shape.ffn}; micro-batch T={mb.num_tokens} "
                               f"S={mb.num_seqs} ({mb.num_seqs - n_dec} prefill chunks, {n_dec} decode tokens), KV block 16",
                   "seed": args.seed, "kv_layers_aliased": bool(alias), "projection_inputs": inputs,
                   "weights": f"4-bit codes, {args.dtype} scale and zero point per 128 input features" if w4 else args.dtype,
                   "weight_copies": copies,
                   "allocation_order": "weights, then KV pool" if args.weights_first else "KV pool, then weights"},
        "stage_latency_ms": round(ms_per_step, 4),
        "ideal_ms": {"hbm": round(work["bytes_per_call"] / (HBM_PEAK_GBS * 1e9) * 1e3, 4),
                     "mfma": round(work["flops_per_call"] / (MFMA_BF16_PEAK_TFLOPS * 1e12) * 1e3, 4)},
        "roofline": roofline,
    }

    if extras and args.breakdown:
        names = list(KERNEL_CLASSES)
        st.profile_enable(names)
        reps = max(3, min(steps, 10))
        for _ in range(reps):
            step()
        torch.cuda.synchronize()
        result["breakdown_ms_per_step"] = {n: round(st.profile_read(n)[0] / reps, 5) for n in names}
        st.profile_enable([])
        proj_ms = sum(result["breakdown_ms_per_step"][n] for n in ("gemm_qkv", "gemm_o", "gemm_gateup", "gemm_down", "dequant"))
        result["projections"] = {"ms_per_step": round(proj_ms, 5),
                                 "weight_bytes_per_step": work["weight_bytes_per_layer"] * shape.num_layers,
                                 "weight_stream_GBps": round(work["weight_bytes_per_layer"] * shape.num_layers / (proj_ms * 1e-3) / 1e9, 1)}

    if want_ends:
        # The pipeline's two ends, timed on their own after the stage (not part of `value`): token
        # embedding of the micro-batch and final norm + vocabulary projection + greedy choice.
        ends = synth.draw_ends_weights(shape, seed=args.seed, device="cuda:0", dtype=elem)
        ids = synth.draw_token_ids(shape, mb.num_tokens, seed=args.seed)
        names = ["embed", "head_norm", "gemm_head", "head_argmax"]
        reps = max(3, min(steps, 20))
        for timed in (False, True):
            if timed:
                st.profile_enable(names)
            for _ in range(reps):
                st.embed(ends["embed"], ids, out=hidden)
                st.head(out, mb.q_lens, ends["final_norm"], ends["lm_head"], want_logits=False)
            torch.cuda.synchronize()
        ms = {n: st.profile_read(n)[0] / reps for n in names}
        st.profile_enable([])
        head_bytes = 2 * shape.vocab * shape.hidden
        result["ends"] = {"vocab": shape.vocab, "ms": {n: round(v, 5) for n, v in ms.items()},
                          "head_gemm_GBps": round(head_bytes / (ms["gemm_head"] * 1e-3) / 1e9, 1),
                          "head_gemm_algorithmic_bytes": head_bytes}

    # the oracle baseline is timed on the benchmark configuration
    if extras and not args.no_cpu_baseline and not w4 and args.dtype == "bf16":
        sample = {"tiny": mb.num_seqs, "llama2-7b": 64, "qwen2-7b": 8, "llama3-70b": 16, "sweep": 8}[workload]
        result["cpu_baseline"] = cpu_baseline(shape, mb, args.seed, sample)
    st.close()
    del st, hidden, out
    torch.cuda.empty_cache()
    print(f"[bench]   {ms_per_step:.3f} ms per micro-batch ({time.time() - t_begin:.0f} s in all)", file=sys.stderr, flush=True)
    return result


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None, choices=["tiny", "llama2-7b", "qwen2-7b", "llama3-70b", "sweep"],
                    help="time this workload alone (default: the headline workload plus one entry per configuration)")
    ap.add_argument("--budget", type=int, default=256, help="token budget of the sweep workload")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--weights", default="bf16", choices=["bf16", "w4"],
                    help="w4: 4-bit projection weights in groups of 128 (a variant, not the benchmark configuration)")
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f16"],
                    help="f16: the IEEE-half library (a variant, not the benchmark configuration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--weights-first", action="store_true",
                    help="allocate the weights before the KV pool (default: the pool first, as an engine that reserves "
                         "its cache when it starts; the decode kernel's stream is 2-5 %% faster over a pool mapped first)")
    ap.add_argument("--no-per-config", action="store_true", help="headline workload only")
    ap.add_argument("--ends", action="store_true",
                    help="also time the pipeline's two ends (embedding; final norm + output head + greedy choice)")
    ap.add_argument("--breakdown", action="store_true", help="also time every kernel class (extra untimed steps)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain 1 GiB device copy ten times and exit (reference for hardware counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: one pipeline stage is one GPU's share and this benchmark measures exactly that; use --gpus 1")

    import torch
    if args.copy_calibration:
        src = torch.full((1 << 28,), 1.0, dtype=torch.float32, device="cuda:0")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4, "launches": 10}))
        return
    from paper_2507_05043_amd import stage as _stage
    if not all(os.path.exists(p) for p in _stage.LIB_PATHS.values()):
        import __graft_entry__
        __graft_entry__.build()

    headline = args.workload or HEADLINE
    head = run_workload(args, headline, args.budget if headline == "sweep" else None, args.steps, args.warmup, extras=True)
    result = {"metric": "stage_tokens_per_sec", "value": head.pop("value"), "unit": "tokens/s", "n_gpus": 1,
              "steps": head.pop("steps"), "warmup": head.pop("warmup"), "ms_per_step": head.pop("ms_per_step"),
              "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic"}
    result.update(head)

    if args.workload is None and not args.no_per_config:
        # One entry per configuration, each timed like the headline (same seed, same measurement) with fewer steps
        # for the long ones so that the whole run stays within a few minutes.
        entries = []
        for workload, budget in PER_CONFIG:
            if workload == headline:
                r = {k: result[k] for k in ("value", "steps", "warmup", "ms_per_step", "config", "ideal_ms", "roofline")}
            else:
                steps = max(3, min(args.steps, 10)) if (workload == "sweep" and budget >= 1024) else args.steps
                r = run_workload(args, workload, budget, steps, args.warmup, extras=False)
                r.pop("stage_latency_ms")
            r["unit"] = "tokens/s"
            entries.append(r)
        result["per_config"] = entries
        if args.weights == "bf16" and args.dtype == "bf16":
            import copy
            variants = []
            for workload, override in VARIANTS:
                a2 = copy.copy(args)
                for k, v in override.items():
                    setattr(a2, k, v)
                r = run_workload(a2, workload, None, args.steps, args.warmup, extras=False)
                r.pop("stage_latency_ms")
                r["unit"] = "tokens/s"
                r["variant"] = override
                variants.append(r)
            result["variants"] = variants
    print(json.dumps(result))


if __name__ == "__main__":
    main()
