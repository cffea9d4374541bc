#!/usr/bin/env python3
"""Benchmark of the absorbed-MLA decode hot path on one MI355X.

A step is one pass of the whole path (paged KV gather, QK^T, online softmax, rescale, PV,
epilogue, and the split-KV combine when the shape needs it) over one synthetic batch that
is already resident in HBM.  The default workload is the 128-head, s_q = 2 decode batch the
headline metric is quoted on.  One JSON line is printed:

  value      whole-job TFLOP/s, FLOPs = 2 * H * s_q * sum(kv_len) * (576 + 512)  (Section 2.4)
  roofline   the decode kernel against the bf16 dense MFMA peak (2516.6 TFLOP/s)
  cpu_baseline  the fp64 CPU oracle timed on the host cores on a bounded sample
  rescale    ADD (exponent add) and MUL (FP32 multiply) variants timed side by side
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "MLA decode TFLOPS + % of MI355X bf16 MFMA peak (H=128, s_q=2)"
MFMA_BF16_PEAK_TFLOPS = 2516.6          # 256 CU x 4096 FLOP/clk x 2.4 GHz
HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="index into the measured configurations (0-4)")
    ap.add_argument("--balanced", action="store_true",
                    help="balanced decomposition for ragged batches (needs AMLA_ENABLE_BALANCED=1; --splits then "
                         "means workers)")
    _names = ["add", "mul", "add_lazy", "mul_lazy", "add_ldexp", "add_ldexp_lazy"]
    ap.add_argument("--variant", choices=["auto", "add_comp"] + _names + [n + "_pf" for n in _names] + [n + "_w8" for n in _names + ["add_comp"]],
                    default="auto",
                    help="auto = the fastest exponent-add variant whose output agrees with the strict add variant on this "
                         "input; _pf = the loop that issues its LDS operand reads ahead of their MFMA; _w8 = the eight-wave kernel")
    ap.add_argument("--table5", default=None, metavar="SQ,SK",
                    help="use a shape of the paper's performance table instead of --config: batch 96, 128 heads, "
                         "s_q SQ, every sequence SK keys, contiguous cache")
    ap.add_argument("--impl", choices=["compiler", "asm"], default="compiler",
                    help="compiler = the HIP C++ kernel (default); asm = the hand-scheduled kernels, which the "
                         "library only runs when AMLA_ENABLE_ASM_KERNELS=1")
    ap.add_argument("--splits", type=int, default=0, help="split-KV factor, 0 = library default")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-mfma-probe", action="store_true", help="skip the measured-MFMA-peak probe")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="instead of the benchmark: copy a buffer of this many MiB `steps` times with a plain "
                         "copy kernel (torch copy_), for scaling the FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--no-ab", action="store_true", help="skip the ADD-vs-MUL side-by-side timing")
    return ap.parse_args()


def time_steps(torch, fn, steps, warmup):
    """Returns (total_ms over exactly `steps` calls, per-step ms list) using events on the
    stream the kernels are launched on (torch's current stream)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    marks[0].record()
    for i in range(steps):
        fn()
        marks[i + 1].record()
    torch.cuda.synchronize()
    total = marks[0].elapsed_time(marks[steps])
    per = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
    return total, per


def cpu_baseline(case, flops_per_seq, budget_s=12.0):
    """The oracle as it stands, one sequence at a time, until ~budget_s of CPU work."""
    from oracle import amla_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    done, flops = 0, 0
    t0 = time.perf_counter()
    for b in range(case.batch):
        orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale, seq_ids=[b])
        done += 1
        flops += flops_per_seq[b]
        if time.perf_counter() - t0 >= budget_s:
            break
    dt = time.perf_counter() - t0
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {done} of {case.batch} sequences of the same workload, fp64 numpy, {dt:.1f} s"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); the path would shard by batch "
              "with no exchange between GPUs", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2509_25224_amd import accounting as acc, amla, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.copy_probe_mib:
        n = args.copy_probe_mib << 20
        src = torch.full((n,), 3, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe": True, "bytes_read_per_launch": n, "bytes_written_per_launch": n,
                          "launches": args.steps}))
        return
    if args.table5:
        sq, sk = (int(x) for x in args.table5.split(","))
        case = wl.make_table5_case(sq, sk)
        workload_tag = f"paper Table 5 shape {case.name}"
    else:
        case = wl.make_config(args.config)
        workload_tag = f"configs[{args.config}] {case.name}"
    dev = torch.device("cuda:0")
    q = torch.from_numpy(case.q_bits.view(np.int16)).to(dev).view(torch.bfloat16)
    kv = torch.from_numpy(case.kv_bits.view(np.int16)).to(dev).view(torch.bfloat16)
    tab = torch.from_numpy(case.block_table).to(dev)
    lens = torch.from_numpy(case.seqlens).to(dev)
    out = torch.empty((case.batch, case.s_q, case.heads, 512), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((case.batch, case.s_q, case.heads), dtype=torch.float32, device=dev)

    impl_flag = amla.AMLA_FLAG_ASM_KERNEL if args.impl == "asm" else 0
    if args.balanced:
        impl_flag |= amla.AMLA_FLAG_BALANCED
    desc = amla.make_desc(case.batch, case.s_q, case.heads, case.num_blocks, case.max_blocks_per_seq,
                          num_splits=args.splits, flags=impl_flag)
    splits = amla.amla_effective_splits(desc)
    ws_bytes = amla.amla_workspace_bytes(desc)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

    VARIANTS = {"mul": (amla.AMLA_RESCALE_MUL, 0), "add": (amla.AMLA_RESCALE_ADD, 0),
                "mul_lazy": (amla.AMLA_RESCALE_MUL, amla.AMLA_FLAG_LAZY_RESCALE),
                "add_lazy": (amla.AMLA_RESCALE_ADD, amla.AMLA_FLAG_LAZY_RESCALE),
                "add_comp": (amla.AMLA_RESCALE_ADD_COMP, 0),
                "add_ldexp": (amla.AMLA_RESCALE_ADD_LDEXP, 0),
                "add_ldexp_lazy": (amla.AMLA_RESCALE_ADD_LDEXP, amla.AMLA_FLAG_LAZY_RESCALE)}
    # "_pf": the build of the compiler kernels' loop that issues its LDS operand reads one MFMA ahead
    # (same arithmetic in the same order); equal-share compiler-built kernels only
    PREFETCHABLE = ("mul", "add", "mul_lazy", "add_lazy", "add_ldexp", "add_ldexp_lazy")
    have_pf = args.impl == "compiler" and not args.balanced
    if have_pf:
        for name in PREFETCHABLE:
            v, f = VARIANTS[name]
            VARIANTS[name + "_pf"] = (v, f | amla.AMLA_FLAG_PREFETCH)
    # "_w8": the eight-wave kernels (16 rows per wave, two waves per SIMD, 16 x 16 x 32 MFMA), equal-share
    # or balanced
    have_w8 = args.impl == "compiler"
    if have_w8:
        for name in PREFETCHABLE + ("add_comp",):
            v, f = VARIANTS[name]
            VARIANTS[name + "_w8"] = (v, f | amla.AMLA_FLAG_EIGHT_WAVES)
    if args.variant not in VARIANTS and args.variant != "auto":
        print(f"bench.py: variant {args.variant} does not exist for this --impl / --balanced", file=sys.stderr)
        sys.exit(2)

    def step(name, o=out, l=lse):
        v, f = VARIANTS[name]
        f |= impl_flag
        amla.amla_decode(q, kv, tab, lens, case.softmax_scale, o, l, variant=v, flags=f,
                         num_splits=args.splits, workspace=ws)

    # The strict add variant is the one checked against the oracle on every row of this workload
    # by the GPU tests.  Another exponent-add variant (lazy reference, or the paper's compensated
    # form) becomes the headline only if, on this very input, its output stays within one bf16 step
    # of the strict one and its lse within 1e-4, and a short timing shows it to be faster.
    chosen, self_check = args.variant, None
    if args.variant == "auto":
        chosen = "add"
        self_check = {}
        try:
            o2 = torch.empty_like(out)
            l2 = torch.empty_like(lse)
            step("add")
            torch.cuda.synchronize()
            passed = ["add"]
            # what each build of the kernels offers: the compensated form only compiler-built, the ldexp
            # form compiler-built without the balanced decomposition and hand-scheduled with or without it
            others = ["add_lazy"]
            if args.impl == "compiler":
                others.append("add_comp")
            if args.impl == "asm" or not args.balanced:
                others += ["add_ldexp", "add_ldexp_lazy"]
            if have_pf:
                others += ["add_pf", "add_lazy_pf", "add_ldexp_pf", "add_ldexp_lazy_pf"]
            if have_w8:
                others += ["add_w8", "add_lazy_w8", "add_ldexp_w8", "add_ldexp_lazy_w8", "add_comp_w8"]
            for name in others:
                try:
                    step(name, o2, l2)
                    torch.cuda.synchronize()
                    a, b = out.float(), o2.float()
                    d_out = float(((a - b).abs() / a.abs().clamp(min=1.0)).max())
                    d_lse = float((lse - l2).abs().max())
                    ok = d_out <= 2.0 ** -7 and d_lse <= 1e-4
                    self_check[name] = {"max_rel_out_diff_vs_strict": d_out, "max_lse_diff_vs_strict": d_lse,
                                        "passed": ok}
                    if ok:
                        passed.append(name)
                except Exception as e:  # noqa: BLE001
                    self_check[name] = {"passed": False, "error": repr(e)}
            del o2, l2
            quick = {}
            for name in passed * 2:
                t, _ = time_steps(torch, lambda: step(name), 20, 3)
                quick[name] = min(quick.get(name, float("inf")), t / 20)
            chosen = min(quick, key=quick.get)
            self_check["quick_ms"] = quick
        except Exception as e:  # noqa: BLE001  (fall back to the variant every GPU test covers)
            chosen = "add"
            self_check["error"] = repr(e)
    torch.cuda.synchronize()
    total_ms, per = time_steps(torch, lambda: step(chosen), args.steps, args.warmup)
    torch.cuda.synchronize()

    flops = acc.decode_flops(case.heads, case.s_q, case.total_kv)
    abytes = acc.algorithmic_bytes(case.heads, case.s_q, case.batch, case.total_kv)
    ms_per_step = total_ms / args.steps
    tflops = flops / (ms_per_step * 1e-3) / 1e12
    kern_ms = sum(per) / len(per)          # one decode launch per step (+ combine when split)
    achieved = flops / (kern_ms * 1e-3) / 1e12

    result = {
        "metric": METRIC, "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{workload_tag}: batch {case.batch}, s_q {case.s_q}, "
                               f"{case.heads} heads, sum kv_len {case.total_kv}, paged bf16 latent cache "
                               f"(block 64), d_qk 576 / d_v 512",
                   "variant": chosen, "kernel_build": args.impl, "kv_splits": splits, "balanced": bool(args.balanced),
                   "seed": case.seed},
        "pct_of_mfma_peak": 100.0 * tflops / MFMA_BF16_PEAK_TFLOPS,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                     "kernel": ("amla_decode_asm_" + chosen) if args.impl == "asm" else
                               ("amla_decode_prefetch_kernel" if chosen.endswith("_pf") else
                                "amla_decode_w8_kernel" if chosen.endswith("_w8") else "amla_decode_kernel"),
                     "kernel_ms": kern_ms,
                     "algorithmic_flops_per_launch": flops, "algorithmic_bytes_per_launch": abytes,
                     "algorithmic_GBps": abytes / (kern_ms * 1e-3) / 1e9, "hbm_peak_GBps": HBM_PEAK_GBS},
    }

    if self_check is not None:
        result["config"]["auto_self_check"] = self_check
    notes = []
    try:
        # what ran it: the datasheet peak above assumes 256 compute units at 2.4 GHz
        prop = torch.cuda.get_device_properties(0)
        result["config"]["device"] = {"name": prop.name, "compute_units": int(prop.multi_processor_count),
                                      "clock_mhz": float(getattr(prop, "clock_rate", 0)) / 1e3}
    except Exception as e:  # noqa: BLE001
        notes.append(f"device properties unavailable: {e!r}")
    if not args.no_ab:
        try:
            ab = {}
            names = ("mul", "add", "mul_lazy", "add_lazy") + (("add_comp",) if args.impl == "compiler" else ()) + \
                (("add_ldexp", "add_ldexp_lazy") if args.impl == "asm" or not args.balanced else ()) + \
                (tuple(n + "_pf" for n in PREFETCHABLE) if have_pf else ()) + \
                (tuple(n + "_w8" for n in PREFETCHABLE + ("add_comp",)) if have_w8 else ())
            for name in names * 2:
                t, _ = time_steps(torch, lambda: step(name), args.steps, 2)
                ab.setdefault(name, []).append(t / args.steps)
            best = {k: min(v) for k, v in ab.items()}
            result["rescale"] = {"add_ms": best["add"], "mul_ms": best["mul"], "add_lazy_ms": best["add_lazy"],
                                 "mul_lazy_ms": best["mul_lazy"],
                                 "add_over_mul_speedup": best["mul"] / best["add"],
                                 "add_lazy_over_mul_lazy_speedup": best["mul_lazy"] / best["add_lazy"],
                                 "tflops": {k: flops / (v * 1e-3) / 1e12 for k, v in best.items()},
                                 "note": "interleaved runs, best of 2 per variant, same binary; strict = "
                                         "reference moves with every new row max, lazy = only past 2^8, "
                                         "add_comp = Algorithm 2 with its BF16 scale compensation, add_ldexp = the exponent add "
                                         "done by v_ldexp_f32, _pf = LDS operand reads issued ahead of their MFMA, _w8 = eight waves of "
                                         "16 rows with the 16 x 16 x 32 MFMA"}
        except Exception as e:  # noqa: BLE001  (an optional leg must not cost the headline line)
            notes.append(f"rescale side-by-side failed: {e!r}")

    if not args.no_mfma_probe:
        try:
            # sustained rate of a register-resident MFMA loop on this device, same process: what the
            # chip delivers under its power limit
            probe_flops = [0.0]

            def probe():
                probe_flops[0] = amla.amla_mfma_probe(20000, 256)
            t, _ = time_steps(torch, probe, 5, 2)
            measured = probe_flops[0] / (t / 5 * 1e-3) / 1e12
            result["roofline"]["measured_mfma_peak"] = measured
            result["roofline"]["frac_of_measured_peak"] = achieved / measured
        except Exception as e:  # noqa: BLE001
            notes.append(f"mfma probe failed: {e!r}")
    if not args.no_cpu_baseline:
        try:
            per_seq = [acc.decode_flops(case.heads, case.s_q, int(L)) for L in case.seqlens]
            result["cpu_baseline"] = cpu_baseline(case, per_seq)
        except Exception as e:  # noqa: BLE001
            notes.append(f"cpu baseline failed: {e!r}")
    if notes:
        result["notes"] = notes

    print(json.dumps(result))


if __name__ == "__main__":
    main()
