#!/usr/bin/env python3
"""Decode-step benchmark: shared-prefix attention (all layers) + token sampling.

One "step" is one pass of the whole hot path over one batch of synthetic input:
`shared_prefix_decode_attn` once per layer, then `sample_tokens` once.  Inputs
are resident in HBM before the timed region.  To keep the caches from serving
repeated reads, the step rotates over several copies of the inputs placed at
distinct addresses (working set between reuses > 512 MB).

Prints ONE JSON line (see the keys below).  `roofline` describes the kernel that
takes the most time in a step; `kernels` lists every stage.  `cpu_baseline` is
the fp64 checker timed on the host cores on the same workload (a reported
baseline, not a target).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16

# HBM-side traffic per launch (bytes) from hardware counters: rocprofv3 --pmc FETCH_SIZE and
# --pmc WRITE_SIZE (KiB per dispatch), each scaled by what the same counter reads for an
# elementwise kernel of known size in the same run (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0 on this
# machine).  Keyed by (kernel, workload); anything not listed is reported as null.  The entry
# must be dropped when the kernel changes.  Source: profiles/hbm_traffic_cfg3_pmc.txt
TRAFFIC_BYTES = {
    ("attn_fused", "cfg3-bf16-p8192-n64"): int((95249.2 * 2.0 + 11341.9) * 1024),
    ("prefix", "cfg3-bf16-p8192-n64"): int((18536.9 * 2.0 + 9216.0) * 1024),
    ("suffix", "cfg3-bf16-p8192-n64"): int((77085.8 * 2.0 + 2064.5) * 1024),
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--copies", type=int, default=0, help="input copies to rotate over (0 = auto)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-iters", type=int, default=50)
    ap.add_argument("--loop-steps", type=int, default=48,
                    help="decode steps of the append + attention + sampler loop timed eagerly and as a "
                         "replayed graph (0 = skip; single-layer workloads only)")
    ap.add_argument("--no-also", action="store_true",
                    help="skip the small configuration measured beside the main one (profiling runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy three times (reference for HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only; --gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2502_02534_amd import binding as B
    from paper_2502_02534_amd import device, workloads

    B.load()  # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    sp = workloads.SPECS[args.config]
    elt = 2 if sp.dtype == "bf16" else 4

    # ---- inputs ---------------------------------------------------------------------------
    layers_host = [workloads.make_attn_inputs(args.config, layer=l) for l in range(sp.layers)]
    sin = workloads.make_sampler_inputs(args.config)
    first = layers_host[0]
    kvB = 2 * sp.num_kv_heads * sp.head_dim * elt                     # bytes per token, K and V, all heads
    prefix_bytes = int(first.prefix_lens.astype(np.int64).sum()) * kvB
    suffix_bytes = int(first.suffix_lens.astype(np.int64).sum()) * kvB
    q_bytes = sp.num_samples * sp.num_q_heads * sp.head_dim * elt
    sampler_bytes = sin.logits.shape[0] * sin.logits.shape[1] * 4 + 16 * sin.logits.shape[0]
    step_bytes = sp.layers * (prefix_bytes + suffix_bytes + 2 * q_bytes) + sampler_bytes
    prefix_flops = 4.0 * sp.group * sp.head_dim * sp.num_kv_heads * float(
        sum(int(first.prefix_lens[b]) * int(first.sample_indptr[b + 1] - first.sample_indptr[b])
            for b in range(sp.num_prompts)))
    copies = args.copies or max(1, min(8, int(np.ceil(600e6 / max(step_bytes, 1)))))

    sets = []
    for c in range(copies):
        lay = [device.upload_attn(h) for h in layers_host]
        sets.append((lay, device.upload_sampler(sin)))
    torch.cuda.synchronize()

    def step(i: int) -> None:
        lay, smp = sets[i % copies]
        for d in lay:
            d.run()
        smp.run()

    # ---- whole-step timing ----------------------------------------------------------------
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3

    # ---- per-stage timing with events on the launching stream -------------------------------
    def time_stage(fn, iters: int) -> float:
        """Mean duration of one call: `iters` calls back to back between one pair of events on the
        launching stream (a pair of events around every single call would add its own few
        microseconds to each)."""
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(iters):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / iters * 1e3  # microseconds per call

    def attn_stage(mask):
        def fn(i):
            lay, _ = sets[i % copies]
            lay[i % len(lay)].run(mask)
        return fn

    # merge: every valid partial state is read once (fp32 accumulator + (m, l)), the output written
    plan = B.spd_attn_plan(sets[0][0][0].desc, first.max_prefix_len, first.max_suffix_len)
    split_tok, _, chunk_tok, _ = plan
    rows_q = sp.num_q_heads
    n_partials = 0
    for b in range(sp.num_prompts):
        nsamp = int(first.sample_indptr[b + 1] - first.sample_indptr[b])
        n_partials += nsamp * rows_q * -(-int(first.prefix_lens[b]) // split_tok)
    n_partials += rows_q * int(sum(-(-int(l) // chunk_tok) for l in first.suffix_lens))
    part_elt = 2 if sp.dtype == "bf16" else 4  # stored partial outputs: fp16 on the bf16 path
    merge_bytes = n_partials * (sp.head_dim * part_elt + 8) + q_bytes

    it = args.kernel_iters
    # A step runs the prefix and the suffix pass in one launch when the library's fused kernel takes
    # the shape (bf16, head_dim 128, group size <= 16); the
    # two passes are also timed as launches of their own for their separate rooflines.
    fused = sp.dtype == "bf16" and sp.head_dim == 128 and sp.group <= 16 and suffix_bytes > 0
    us = {
        "attn_fused": time_stage(attn_stage(B.STAGE_PREFIX | B.STAGE_SUFFIX), it),
        "prefix": time_stage(attn_stage(B.STAGE_PREFIX), it),
        "suffix": time_stage(attn_stage(B.STAGE_SUFFIX), it),
        "merge": time_stage(attn_stage(B.STAGE_MERGE), it),
        "sampler": time_stage(lambda i: sets[i % copies][1].run(), it),
    }
    attn_bytes = prefix_bytes + suffix_bytes + 2 * q_bytes
    kernels = {
        "attn_fused": {"us": us["attn_fused"], "bytes": attn_bytes, "flops": prefix_flops,
                       "GBps": attn_bytes / us["attn_fused"] / 1e3,
                       "TFLOPs": prefix_flops / us["attn_fused"] / 1e6,
                       "calls_per_step": sp.layers if fused else 0,
                       "note": "prefix + suffix pass" + (" in one launch (what a step runs)" if fused
                                                         else " as two launches back to back (what a step runs)")},
        "prefix": {"us": us["prefix"], "bytes": prefix_bytes + q_bytes, "flops": prefix_flops,
                   "GBps": (prefix_bytes + q_bytes) / us["prefix"] / 1e3,
                   "TFLOPs": prefix_flops / us["prefix"] / 1e6, "calls_per_step": 0 if fused else sp.layers},
        "suffix": {"us": us["suffix"], "bytes": suffix_bytes + q_bytes,
                   "GBps": (suffix_bytes + q_bytes) / us["suffix"] / 1e3,
                   "calls_per_step": 0 if fused else sp.layers},
        "merge": {"us": us["merge"], "bytes": merge_bytes, "GBps": merge_bytes / us["merge"] / 1e3,
                  "calls_per_step": sp.layers},
        "sampler": {"us": us["sampler"], "bytes": sampler_bytes,
                    "GBps": sampler_bytes / us["sampler"] / 1e3, "calls_per_step": 1},
    }
    for k in kernels.values():
        k["frac_hbm_peak"] = k.get("GBps", 0.0) / HBM_PEAK_GBS
    kernels["prefix"]["frac_mfma_peak"] = kernels["prefix"]["TFLOPs"] / MFMA_BF16_PEAK_TFLOPS
    # the dominant kernel is looked for among the stages that are one kernel each; the sampler
    # stage is two to four kernels (its event time is their sum) and is listed under "kernels"
    per_step = {k: v["us"] * v["calls_per_step"] for k, v in kernels.items()
                if k in ("attn_fused", "prefix", "suffix")}
    dom = max(per_step, key=per_step.get)
    if dom == "attn_fused" and prefix_flops / MFMA_BF16_PEAK_TFLOPS / 1e12 > attn_bytes / HBM_PEAK_GBS / 1e9:
        roofline = {"kernel": "attn_fused", "bound": "mfma", "achieved": kernels["attn_fused"]["TFLOPs"],
                    "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": kernels["attn_fused"]["TFLOPs"] / MFMA_BF16_PEAK_TFLOPS,
                    "traffic": TRAFFIC_BYTES.get(("attn_fused", sp.name))}
    elif dom == "prefix" and prefix_flops / MFMA_BF16_PEAK_TFLOPS / 1e12 > (prefix_bytes + q_bytes) / HBM_PEAK_GBS / 1e9:
        roofline = {"kernel": "prefix", "bound": "mfma", "achieved": kernels["prefix"]["TFLOPs"],
                    "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": kernels["prefix"]["frac_mfma_peak"],
                    "traffic": TRAFFIC_BYTES.get(("prefix", sp.name))}
    else:
        roofline = {"kernel": dom, "bound": "hbm", "achieved": kernels[dom]["GBps"], "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": kernels[dom]["frac_hbm_peak"],
                    "traffic": TRAFFIC_BYTES.get((dom, sp.name))}

    # ---- loop of decode steps with KV append (device-side lengths), eager and as a replayed graph ----
    loop_info = None
    if args.loop_steps > 0 and sp.layers == 1:
        L = args.loop_steps
        host = layers_host[0]
        import copy as _copy
        hl = _copy.copy(host)
        hl.suffix_lens = np.maximum(host.suffix_lens - L - 1, 0).astype(np.int32)  # room for the steps
        rng = np.random.default_rng(12345)
        n = sp.num_samples

        def draw(shape):
            x = rng.standard_normal(shape).astype(np.float32)
            t = torch.from_numpy(workloads.f32_to_bf16_bits(x) if sp.dtype == "bf16" else x).cuda()
            return t.view(torch.int16).view(torch.bfloat16) if sp.dtype == "bf16" else t

        q_s = draw((L, n, sp.num_q_heads, sp.head_dim))
        k_s = draw((L, n, sp.num_kv_heads, sp.head_dim))
        v_s = draw((L, n, sp.num_kv_heads, sp.head_dim))
        u_s = torch.from_numpy(rng.random((L, sin.logits.shape[0]), dtype=np.float32)).cuda()

        def make_loop():
            return device.DecodeLoop(device.upload_attn(hl), device.upload_sampler(sin), q_s, k_s, v_s, u_s, -1)

        lp = make_loop()
        lp.one_step()
        lp.step.zero_()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(L - 1):
            lp.one_step()
        torch.cuda.synchronize()
        eager_us = (time.perf_counter() - t0) / (L - 1) * 1e6
        gl = make_loop()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            gl.one_step()
        torch.cuda.current_stream().wait_stream(side)
        gl.step.zero_()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            gl.one_step()
        graph.replay()
        gl.step.zero_()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(L - 2):
            graph.replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - t0) / (L - 2) * 1e6
        loop_info = {"steps": L, "us_per_step_eager": eager_us, "us_per_step_graph": graph_us,
                     "tokens_per_sec_graph": sp.num_samples * 1e6 / graph_us,
                     "note": "append_suffix_kv + attention + sample_tokens per step, per-step inputs gathered "
                             "on the device, lengths on the device; graph = one captured step replayed"}
        del lp, gl, graph, q_s, k_s, v_s, u_s

    # ---- the small configuration next to the main one: whole-step rate only -------------------------
    also = {}
    if args.config == 3 and not args.no_also:
        sp2 = workloads.SPECS[2]
        lay2 = [device.upload_attn(workloads.make_attn_inputs(2)) for _ in range(4)]
        smp2 = [device.upload_sampler(workloads.make_sampler_inputs(2)) for _ in range(4)]

        def step2(i):
            lay2[i % 4].run()
            smp2[i % 4].run()

        for i in range(20):
            step2(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(400):
            step2(i)
        torch.cuda.synchronize()
        ms2 = (time.perf_counter() - t0) / 400 * 1e3
        also[sp2.name] = {"value": 1e3 / ms2, "unit": "steps/s", "ms_per_step": ms2,
                          "tokens_per_sec": sp2.num_samples * 1e3 / ms2,
                          "note": "16 samples, 2048-token prompt: launch-latency bound (about 10 MB per step)"}
        del lay2, smp2

    if args.calibrate_copy:
        # a plain elementwise kernel of known size in the same process: 256 MiB read and 256 MiB
        # written per call (torch's out-of-place multiply; a tensor copy would go to the runtime's
        # blit path instead of a kernel of known shape)
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 2.0, out=dst)
        torch.cuda.synchronize()

    # ---- CPU baseline: the fp64 checker on the same workload ---------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        ncores = os.cpu_count() or 1
        env_threads = int(os.environ.get("OMP_NUM_THREADS", ncores))
        total_rows = sp.num_samples * sp.num_q_heads
        # bounded sample: at most 4096 attention rows of one layer and 128 sampler rows, scaled up
        # (configuration 3 fits whole: about ten core-seconds)
        rows = np.arange(total_rows, dtype=np.int64)
        if total_rows > 4096:
            rows = np.linspace(0, total_rows - 1, 4096).astype(np.int64)
        t0 = time.perf_counter()
        oracle.attention_inputs(first, rows=rows)
        t_attn = (time.perf_counter() - t0) * (total_rows / len(rows)) * sp.layers
        srows = min(128, sin.logits.shape[0])
        t0 = time.perf_counter()
        oracle.sample_tokens(sin.logits[:srows], sin.temperature[:srows], sin.top_p[:srows], sin.uniforms[:srows])
        t_samp = (time.perf_counter() - t0) * (sin.logits.shape[0] / srows)
        cpu = {"value": 1.0 / (t_attn + t_samp), "unit": "steps/s", "cores": min(env_threads, ncores),
               "kind": "oracle",
               "sample": f"{len(rows)} of {total_rows} attention rows of one layer (x{sp.layers} layers) "
                         f"and {srows} of {sin.logits.shape[0]} sampler rows, scaled linearly to one step"}

    line = {
        "metric": "decode_steps_per_sec", "value": 1e3 / ms_per_step, "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": sp.dtype, "data": "synthetic",
        "config": {"workload": sp.name, "config_id": args.config, "num_samples": sp.num_samples,
                   "q_heads": sp.num_q_heads, "kv_heads": sp.num_kv_heads, "head_dim": sp.head_dim,
                   "prefix_tokens": int(first.prefix_lens.sum()), "suffix_tokens": int(first.suffix_lens.sum()),
                   "vocab": sp.vocab, "layers": sp.layers, "page_size": sp.page_size,
                   "input_copies_rotated": copies},
        "tokens_per_sec": sp.num_samples * 1e3 / ms_per_step,
        "step_algorithmic_bytes": step_bytes,
        "step_GBps": step_bytes / ms_per_step / 1e6,
        "roofline": roofline, "kernels": kernels, "decode_loop": loop_info, "also": also, "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
