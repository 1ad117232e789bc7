#!/usr/bin/env python3
"""Decode-step benchmark: shared-prefix attention (all layers) + token sampling.

One "step" is one pass of the whole hot path over one batch of synthetic input:
`shared_prefix_decode_attn` once per layer, then `sample_tokens` once.  Inputs
are resident in HBM before the timed region.  To keep the caches from serving
repeated reads, the step rotates over several copies of the inputs placed at
distinct addresses whenever one copy is smaller than 600 MB.

The default workload is the largest single-GPU configuration (configuration 5:
8 prompts x 128 samples, paged KV, 4.3 GB of KV and 525 MB of logits per step);
the whole-step rates of configurations 3 and 4 are reported beside it under `also`.

Prints ONE JSON line.  `roofline` describes the kernel that takes the most time
in a step; `kernels` lists every stage with its fraction of the roofline that
bounds it.  `cpu_baseline` is the fp64 checker timed on the host cores on a
bounded sample of the same workload (a reported baseline, not a target).
"""
import argparse
import dataclasses
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16

CSRC = os.path.join(ROOT, "paper_2502_02534_amd", "csrc")
# Source files that define each timed kernel: a measured traffic figure is only reported while
# these files are the ones it was measured on.
KERNEL_SOURCES = {
    "attn_fused": ["attn_fused.hip", "attn_prefix_body.h", "attn_suffix_body.h", "spd_internal.h", "plan.h"],
    "prefix": ["attn_prefix_mfma.hip", "attn_prefix_body.h", "spd_internal.h", "plan.h"],
    "suffix": ["attn_suffix_mfma.hip", "attn_suffix_body.h", "spd_internal.h", "plan.h"],
    "merge": ["attn_merge.hip", "spd_internal.h", "plan.h"],
    "sampler": ["sampler.hip", "spd_internal.h"],
}
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_table.txt")


def source_hash(kernel: str) -> str:
    h = hashlib.sha256()
    for name in KERNEL_SOURCES[kernel]:
        with open(os.path.join(CSRC, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(kernel: str, workload: str):
    """HBM-side bytes per launch from hardware counters (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE,
    KiB per dispatch, each scaled by what the same counter reads for an elementwise kernel of known
    size), as recorded in profiles/hbm_traffic_table.txt; None when no line matches this kernel,
    this workload and the present source files."""
    if kernel not in KERNEL_SOURCES or not os.path.exists(TRAFFIC_TABLE):
        return None
    want = source_hash(kernel)
    with open(TRAFFIC_TABLE) as f:
        for line in f:
            parts = line.split()
            if len(parts) == 7 and parts[0] == kernel and parts[1] == workload and parts[2] == want:
                fetch_kib, write_kib, f_fetch, f_write = (float(v) for v in parts[3:])
                return int((fetch_kib * f_fetch + write_kib * f_write) * 1024)
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=5, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--copies", type=int, default=0, help="input copies to rotate over (0 = auto)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-iters", type=int, default=20)
    ap.add_argument("--loop-steps", type=int, default=24,
                    help="decode steps of the append + attention + sampler loop timed eagerly and as a "
                         "replayed graph (0 = skip; single-layer workloads only)")
    ap.add_argument("--completion-steps", type=int, default=1024,
                    help="tokens per sample of the end-to-end sampling job (64 samples, 8192-token prompt); 0 = skip")
    ap.add_argument("--no-also", action="store_true",
                    help="skip the other configurations and the end-to-end job measured beside the main one (profiling runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run an elementwise kernel over 256 MiB three times (reference for HBM traffic counters)")
    ap.add_argument("--page-order", choices=["shuffled", "sequential"], default="shuffled",
                    help="paged workloads: page table dealt out at random (the default recipe) or in order of use")
    ap.add_argument("--print-source-hashes", action="store_true",
                    help="print the source hash of every timed kernel (for profiles/hbm_traffic_table.txt) and exit")
    args = ap.parse_args()
    if args.print_source_hashes:
        for k in KERNEL_SOURCES:
            print(k, source_hash(k))
        return 0
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

    def events_us(fn, iters: int) -> float:
        """Mean duration of one call: `iters` calls back to back between one pair of events on the
        launching stream."""
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(iters):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / iters * 1e3

    def whole_step(cfg: int, steps: int, warmup: int):
        """Uploads configuration `cfg` and times `steps` whole steps; returns (ms per step, context)."""
        sp = workloads.SPECS[cfg]
        if sp.page_size and args.page_order != sp.page_order:
            sp = dataclasses.replace(sp, page_order=args.page_order)
        layers_host = [workloads.make_attn_inputs(cfg, layer=l, spec=sp) for l in range(sp.layers)]
        sin = workloads.make_sampler_inputs(cfg)
        elt = 2 if sp.dtype == "bf16" else 4
        first = layers_host[0]
        kvB = 2 * sp.num_kv_heads * sp.head_dim * elt
        prefix_bytes = int(first.prefix_lens.astype(np.int64).sum()) * kvB
        suffix_bytes = int(first.suffix_lens.astype(np.int64).sum()) * kvB
        q_bytes = sp.num_samples * sp.num_q_heads * sp.head_dim * elt
        sampler_bytes = sin.logits.shape[0] * sin.logits.shape[1] * 4 + 16 * sin.logits.shape[0]
        step_bytes = sp.layers * (prefix_bytes + suffix_bytes + 2 * q_bytes) + sampler_bytes
        copies = args.copies or max(1, min(8, int(np.ceil(600e6 / max(step_bytes, 1)))))
        sets = []
        for _ in range(copies):
            sets.append(([device.upload_attn(h) for h in layers_host], device.upload_sampler(sin)))
        torch.cuda.synchronize()

        def step(i: int) -> None:
            lay, smp = sets[i % copies]
            for d in lay:
                d.run()
            smp.run()

        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(warmup + i)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        ctx = dict(sp=sp, layers_host=layers_host, sin=sin, sets=sets, copies=copies, first=first,
                   prefix_bytes=prefix_bytes, suffix_bytes=suffix_bytes, q_bytes=q_bytes,
                   sampler_bytes=sampler_bytes, step_bytes=step_bytes)
        return ms, ctx

    ms_per_step, cx = whole_step(args.config, args.steps, args.warmup)
    sp, sets, copies, first, sin = cx["sp"], cx["sets"], cx["copies"], cx["first"], cx["sin"]
    prefix_bytes, suffix_bytes, q_bytes = cx["prefix_bytes"], cx["suffix_bytes"], cx["q_bytes"]
    sampler_bytes, step_bytes = cx["sampler_bytes"], cx["step_bytes"]
    prefix_flops = 4.0 * sp.group * sp.head_dim * sp.num_kv_heads * float(
        sum(int(first.prefix_lens[b]) * int(first.sample_indptr[b + 1] - first.sample_indptr[b])
            for b in range(sp.num_prompts)))

    # ---- per-stage timing with events on the launching stream -------------------------------------
    def attn_stage(mask):
        def fn(i):
            lay, _ = sets[i % copies]
            lay[i % len(lay)].run(mask)
        return fn

    # merge: every valid partial state is read once (accumulator + (m, l)), the output written
    split_tok, _, chunk_tok, _ = B.spd_attn_plan(sets[0][0][0].desc, first.max_prefix_len, first.max_suffix_len)
    n_partials = 0
    for b in range(sp.num_prompts):
        nsamp = int(first.sample_indptr[b + 1] - first.sample_indptr[b])
        n_partials += nsamp * sp.num_q_heads * -(-int(first.prefix_lens[b]) // split_tok)
    n_partials += sp.num_q_heads * int(sum(-(-int(l) // chunk_tok) for l in first.suffix_lens))
    part_elt = 2 if sp.dtype == "bf16" else 4  # stored partial outputs: fp16 on the bf16 path
    merge_bytes = n_partials * (sp.head_dim * part_elt + 8) + q_bytes

    it = args.kernel_iters
    # A step runs the prefix and the suffix pass in one launch when the library's fused kernel takes
    # the shape (bf16, head_dim 128, group size <= 16); the two passes are also timed as launches of
    # their own for their separate rooflines.
    fused = sp.dtype == "bf16" and sp.head_dim == 128 and sp.group <= 16 and suffix_bytes > 0
    us = {
        "attn_fused": events_us(attn_stage(B.STAGE_PREFIX | B.STAGE_SUFFIX), it),
        "prefix": events_us(attn_stage(B.STAGE_PREFIX), it),
        "suffix": events_us(attn_stage(B.STAGE_SUFFIX), it),
        "merge": events_us(attn_stage(B.STAGE_MERGE), it),
        "sampler": events_us(lambda i: sets[i % copies][1].run(), it),
    }
    attn_bytes = prefix_bytes + suffix_bytes + 2 * q_bytes
    prefix_floor_us = max((prefix_bytes + q_bytes) / HBM_PEAK_GBS / 1e3, prefix_flops / MFMA_BF16_PEAK_TFLOPS / 1e6)
    kernels = {
        "attn_fused": {"us": us["attn_fused"], "bytes": attn_bytes, "flops": prefix_flops,
                       "GBps": attn_bytes / us["attn_fused"] / 1e3,
                       "TFLOPs": prefix_flops / us["attn_fused"] / 1e6,
                       "calls_per_step": sp.layers if fused else 0,
                       "note": "prefix + suffix pass" + (" in one launch (what a step runs)" if fused
                                                         else " as two launches back to back (what a step runs)")},
        "prefix": {"us": us["prefix"], "bytes": prefix_bytes + q_bytes, "flops": prefix_flops,
                   "GBps": (prefix_bytes + q_bytes) / us["prefix"] / 1e3,
                   "TFLOPs": prefix_flops / us["prefix"] / 1e6, "calls_per_step": 0 if fused else sp.layers,
                   "frac_binding_roofline": prefix_floor_us / us["prefix"],
                   "binding_roofline": "mfma" if prefix_flops / MFMA_BF16_PEAK_TFLOPS / 1e6 >=
                   (prefix_bytes + q_bytes) / HBM_PEAK_GBS / 1e3 else "hbm"},
        "suffix": {"us": us["suffix"], "bytes": suffix_bytes + q_bytes,
                   "GBps": (suffix_bytes + q_bytes) / us["suffix"] / 1e3,
                   "calls_per_step": 0 if fused else sp.layers},
        "merge": {"us": us["merge"], "bytes": merge_bytes, "GBps": merge_bytes / us["merge"] / 1e3,
                  "calls_per_step": sp.layers},
        "sampler": {"us": us["sampler"], "bytes": sampler_bytes,
                    "GBps": sampler_bytes / us["sampler"] / 1e3, "calls_per_step": 1,
                    "note": "all kernels of one sample_tokens call"},
    }
    for name, k in kernels.items():
        k["frac_hbm_peak"] = k.get("GBps", 0.0) / HBM_PEAK_GBS
        # the counters were taken on the recipe's own page table
        k["traffic"] = measured_traffic(name, sp.name) if sp.page_order == workloads.SPECS[args.config].page_order else None
    kernels["prefix"]["frac_mfma_peak"] = kernels["prefix"]["TFLOPs"] / MFMA_BF16_PEAK_TFLOPS
    # the dominant kernel is looked for among the stages that are one kernel each
    per_step = {k: v["us"] * v["calls_per_step"] for k, v in kernels.items()
                if k in ("attn_fused", "prefix", "suffix")}
    dom = max(per_step, key=per_step.get)
    dom_flops_us = prefix_flops / MFMA_BF16_PEAK_TFLOPS / 1e6 if dom in ("attn_fused", "prefix") else 0.0
    dom_bytes_us = kernels[dom]["bytes"] / HBM_PEAK_GBS / 1e3
    if dom_flops_us > dom_bytes_us:
        roofline = {"kernel": dom, "bound": "mfma", "achieved": kernels[dom]["TFLOPs"],
                    "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": kernels[dom]["TFLOPs"] / MFMA_BF16_PEAK_TFLOPS, "traffic": kernels[dom]["traffic"]}
    else:
        roofline = {"kernel": dom, "bound": "hbm", "achieved": kernels[dom]["GBps"], "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": kernels[dom]["frac_hbm_peak"], "traffic": kernels[dom]["traffic"]}

    # ---- loop of decode steps with KV append (device-side lengths), eager and as a replayed graph ----
    loop_info = None
    if args.loop_steps > 2 and sp.layers == 1:
        L = args.loop_steps
        host = cx["layers_host"][0]
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
                     "note": "decode_step_advance (record, select and KV append in one launch) + attention + "
                             "sample_tokens per step: library launches only, step counter and lengths on the "
                             "device; graph = one captured step replayed"}
        del lp, gl, graph, q_s, k_s, v_s, u_s

    if args.calibrate_copy:
        # an elementwise kernel of known size in the same process: 256 MiB read and 256 MiB written
        # per call (torch's out-of-place multiply; a tensor copy would go to the runtime's blit path
        # instead of a kernel of known shape)
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 2.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    # ---- CPU baseline: the fp64 checker on a bounded sample of the same workload ----------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        ncores = os.cpu_count() or 1
        env_threads = int(os.environ.get("OMP_NUM_THREADS", ncores))
        total_rows = sp.num_samples * sp.num_q_heads
        # at most 2048 attention rows of one layer and 64 sampler rows, spread evenly, scaled linearly
        rows = np.arange(total_rows, dtype=np.int64)
        if total_rows > 2048:
            rows = np.linspace(0, total_rows - 1, 2048).astype(np.int64)
        t0 = time.perf_counter()
        oracle.attention_inputs(first, rows=rows)
        t_attn = (time.perf_counter() - t0) * (total_rows / len(rows)) * sp.layers
        nrows = sin.logits.shape[0]
        pick = np.arange(nrows) if nrows <= 64 else np.linspace(0, nrows - 1, 64).astype(np.int64)
        t0 = time.perf_counter()
        oracle.sample_tokens(sin.logits[pick], sin.temperature[pick], sin.top_p[pick], sin.uniforms[pick])
        t_samp = (time.perf_counter() - t0) * (nrows / len(pick))
        cpu = {"value": 1.0 / (t_attn + t_samp), "unit": "steps/s", "cores": min(env_threads, ncores),
               "kind": "oracle",
               "sample": f"{len(rows)} of {total_rows} attention rows of one layer (x{sp.layers} layers) "
                         f"and {len(pick)} of {nrows} sampler rows, scaled linearly to one step"}

    config = {"workload": sp.name, "config_id": args.config, "num_samples": sp.num_samples,
              "q_heads": sp.num_q_heads, "kv_heads": sp.num_kv_heads, "head_dim": sp.head_dim,
              "prefix_tokens": int(first.prefix_lens.sum()), "suffix_tokens": int(first.suffix_lens.sum()),
              "vocab": sp.vocab, "layers": sp.layers, "page_size": sp.page_size, "input_copies_rotated": copies}
    if sp.page_size:
        config["page_order"] = sp.page_order

    # ---- the other configurations: whole-step rate only ------------------------------------------------
    also = {}
    if not args.no_also:
        del sets, cx
        torch.cuda.empty_cache()
        notes = {2: "16 samples, 2048-token prompt: launch-latency bound (about 10 MB per step)",
                 3: "64 samples of one 8192-token prompt (the paper's sampling shape), suffixes U[128,1024]",
                 4: "32 layers, 32 samples of one 16384-token prompt, 512-token suffixes; sampler once per step",
                 5: "8 prompts x 128 samples, paged KV"}
        for cfg in (3, 4, 5):
            if cfg == args.config:
                continue
            ms, c2 = whole_step(cfg, 100 if cfg != 4 else 30, 10 if cfg != 4 else 3)
            sp2 = c2["sp"]
            also[sp2.name] = {"value": 1e3 / ms, "unit": "steps/s", "ms_per_step": ms,
                              "tokens_per_sec": sp2.num_samples * 1e3 / ms,
                              "step_algorithmic_bytes": c2["step_bytes"],
                              "step_GBps": c2["step_bytes"] / ms / 1e6,
                              "input_copies_rotated": c2["copies"], "note": notes[cfg]}
            del c2
            torch.cuda.empty_cache()

    # ---- the paper's sampling job end to end: 64 samples of one 8192-token prompt, every sample from
    # an empty suffix to `completion_steps` generated tokens, one captured decode step replayed ----------
    completions = None
    if args.completion_steps > 0 and not args.no_also:
        torch.cuda.empty_cache()
        sp3 = dataclasses.replace(workloads.SPECS[3], suffix_len=(0, args.completion_steps))
        h3 = workloads.make_attn_inputs(3, spec=sp3)
        h3.suffix_lens[:] = 0
        sin3 = workloads.make_sampler_inputs(3)
        rng = np.random.default_rng(4321)
        rows = 16   # distinct per-step inputs; later steps reuse the last row (the timing does not depend on the values)

        def draw3(shape):
            t = torch.from_numpy(workloads.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))).cuda()
            return t.view(torch.int16).view(torch.bfloat16)

        n3 = sp3.num_samples
        lp3 = device.DecodeLoop(device.upload_attn(h3), device.upload_sampler(sin3),
                                draw3((rows, n3, sp3.num_q_heads, sp3.head_dim)),
                                draw3((rows, n3, sp3.num_kv_heads, sp3.head_dim)),
                                draw3((rows, n3, sp3.num_kv_heads, sp3.head_dim)),
                                torch.from_numpy(rng.random((rows, n3), dtype=np.float32)).cuda(), -1)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            lp3.one_step()                      # warm-up outside the capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph3 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph3):
            lp3.one_step()
        graph3.replay()
        torch.cuda.synchronize()
        lp3.step.zero_()
        lp3.attn.suffix_lens.zero_()
        lp3.finished.zero_()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.completion_steps):
            graph3.replay()
        torch.cuda.synchronize()
        total = time.perf_counter() - t0
        final_lens = lp3.attn.suffix_lens.cpu().numpy()
        assert int(final_lens.min()) == args.completion_steps == int(final_lens.max()), "the loop did not append every step"
        completions = {"workload": "64 samples of one 8192-token prompt, suffixes grown from 0 to "
                                   f"{args.completion_steps} tokens", "steps": args.completion_steps,
                       "samples": n3, "total_ms": total * 1e3, "us_per_step_mean": total / args.completion_steps * 1e6,
                       "tokens_per_sec": n3 * args.completion_steps / total,
                       "note": "per step: decode_step_advance (record, select and KV append in one launch) + "
                               "attention + sample_tokens, replayed from one captured graph; no host "
                               "synchronisation between steps"}
        del lp3, graph3
        torch.cuda.empty_cache()

    line = {
        "metric": "decode_steps_per_sec", "value": 1e3 / ms_per_step, "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": sp.dtype, "data": "synthetic", "config": config,
        "tokens_per_sec": sp.num_samples * 1e3 / ms_per_step,
        "step_algorithmic_bytes": step_bytes,
        "step_GBps": step_bytes / ms_per_step / 1e6,
        "roofline": roofline, "kernels": kernels, "decode_loop": loop_info, "completions": completions, "also": also,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
