#!/usr/bin/env python3
"""Benchmark of the absorbed-MLA decode hot path on one MI355X.

A step is one pass of the whole path (paged KV gather, QK^T, online softmax, rescale, PV, epilogue, and the
split-KV combine when the shape needs it) over one synthetic batch that is already resident in HBM.  The
default workload is the 128-head, s_q = 2 decode batch the headline metric is quoted on, and the timed kernel
is the paper's method as the library runs it by default: the strict INT32 exponent add of Lemma 3.1 /
Algorithm 2 (AMLA_RESCALE_ADD) on the row-rescale kernels.  One JSON line is printed:

  value         whole-job TFLOP/s, FLOPs = 2 * H * s_q * sum(kv_len) * (576 + 512)  (Section 2.4)
  roofline      the decode kernel against the bf16 dense MFMA peak (2516.6 TFLOP/s)
  parity        the timed kernel's output against the fp64 CPU oracle on the same input
  cpu_baseline  the oracle timed on the host cores on a bounded sample
  rescale       every rescale variant of both kernel families timed side by side, and the ADD / MUL
                ratio as interleaved medians
  per_config    the other measured configurations (HBM-bound s_q = 1, ragged, long context) and a
                low-head-count batch (16 heads: achieved HBM GB/s)
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
# HBM traffic of one launch of the headline kernel on the headline workload, from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs scaled by a copy kernel of known size (profiles/amla_decode_rg_kernel_mtp_b128.md); null for
# any other kernel or workload
MEASURED_TRAFFIC = {
    # FETCH_SIZE 313918 KiB x 2.000 + WRITE_SIZE 33408 KiB x 1.000 (factors: profiles/copy_probe_512mib.md)
    ("amla_decode_rg_kernel", "add", "mtp_b128", 1): {"read": 643.7e6, "written": 35.0e6},
    ("amla_decode_rg_kernel", "mul", "mtp_b128", 1): {"read": 643.6e6, "written": 35.0e6},
    ("amla_decode_rg_kernel", "add_512", "mtp_b128", 1): {"read": 643.9e6, "written": 35.0e6},
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="index into the measured configurations (0-4)")
    ap.add_argument("--variant", default="add",
                    help="the kernel that is timed: mul, add, add_comp (row-rescale kernels, the default family), "
                         "mul_512, add_512 (the same with one iteration of the recurrence per 512 keys), "
                         "mul_t, add_t, add_comp_t, mul_lazy, add_lazy, add_ldexp, add_ldexp_lazy "
                         "(transposed-accumulator kernels)")
    ap.add_argument("--balanced", action="store_true",
                    help="balanced decomposition for ragged batches (--splits then means workers)")
    ap.add_argument("--table5", default=None, metavar="SQ,SK",
                    help="use a shape of the paper's performance table instead of --config: batch 96, 128 heads, "
                         "s_q SQ, every sequence SK keys, contiguous cache; 'all' times the table's 12 shapes")
    ap.add_argument("--low-heads", type=int, default=0, metavar="H",
                    help="use the low-head-count batch instead of --config: 256 sequences, s_q 1, H heads (16 = one GPU "
                         "of an eight-way tensor-parallel group), 4096 keys each")
    ap.add_argument("--splits", type=int, default=0, help="split-KV factor, 0 = library default")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle leg (and with it the parity block)")
    ap.add_argument("--no-mfma-probe", action="store_true", help="skip the measured-MFMA-peak probe")
    ap.add_argument("--no-ab", action="store_true", help="skip the side-by-side timing of the rescale variants")
    ap.add_argument("--no-per-config", action="store_true", help="skip the other measured configurations")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="instead of the benchmark: copy a buffer of this many MiB `steps` times with a plain "
                         "copy kernel (torch copy_), for scaling the FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


def variants(amla):
    T, L, I = amla.AMLA_FLAG_TRANSPOSED_ACC, amla.AMLA_FLAG_LAZY_RESCALE, amla.AMLA_FLAG_ITERATION_512
    return {"mul": (amla.AMLA_RESCALE_MUL, 0), "add": (amla.AMLA_RESCALE_ADD, 0), "add_comp": (amla.AMLA_RESCALE_ADD_COMP, 0),
            "mul_512": (amla.AMLA_RESCALE_MUL, I), "add_512": (amla.AMLA_RESCALE_ADD, I),
            "mul_t": (amla.AMLA_RESCALE_MUL, T), "add_t": (amla.AMLA_RESCALE_ADD, T),
            "add_comp_t": (amla.AMLA_RESCALE_ADD_COMP, T),
            "mul_lazy": (amla.AMLA_RESCALE_MUL, L), "add_lazy": (amla.AMLA_RESCALE_ADD, L),
            "add_ldexp": (amla.AMLA_RESCALE_ADD_LDEXP, 0), "add_ldexp_lazy": (amla.AMLA_RESCALE_ADD_LDEXP, L)}


def kernel_name(name, balanced):
    row = name in ("mul", "add", "add_comp", "mul_512", "add_512")
    return ("amla_decode_rg" if row else "amla_decode") + ("_balanced_kernel" if balanced else "_kernel")


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


def median(xs):
    s = sorted(xs)
    return s[len(s) // 2]


class Problem:
    """One workload resident in HBM, with output buffers and a workspace large enough for any decomposition."""

    def __init__(self, torch, amla, case):
        import numpy as np
        self.torch, self.amla, self.case = torch, amla, case
        dev = torch.device("cuda:0")
        self.q = torch.from_numpy(case.q_bits.view(np.int16)).to(dev).view(torch.bfloat16)
        self.kv = torch.from_numpy(case.kv_bits.view(np.int16)).to(dev).view(torch.bfloat16)
        self.tab = torch.from_numpy(case.block_table).to(dev)
        self.lens = torch.from_numpy(case.seqlens).to(dev)
        self.out = torch.empty((case.batch, case.s_q, case.heads, 512), dtype=torch.bfloat16, device=dev)
        self.lse = torch.empty((case.batch, case.s_q, case.heads), dtype=torch.float32, device=dev)
        self.ws = {}

    def desc(self, name, balanced=False, splits=0):
        v, f = variants(self.amla)[name]
        if balanced:
            f |= self.amla.AMLA_FLAG_BALANCED
        c = self.case
        return self.amla.make_desc(c.batch, c.s_q, c.heads, c.num_blocks, c.max_blocks_per_seq, v, splits, f)

    def second_pool(self):
        """A second copy of the cache pool; step() then alternates between the two, so that a pool of about the
        size of the 256 MB memory-side cache is read from HBM every time."""
        self.kv_other = self.kv.clone()

    def step(self, name, balanced=False, splits=0):
        if getattr(self, "kv_other", None) is not None:
            self.kv, self.kv_other = self.kv_other, self.kv
        key = (name, balanced, splits)
        if key not in self.ws:
            d = self.desc(name, balanced, splits)
            need = max(self.amla.amla_workspace_bytes(d), 16)
            self.ws[key] = (d.variant, d.flags, self.torch.empty(need, dtype=self.torch.uint8, device=self.q.device))
        v, f, ws = self.ws[key]
        self.amla.amla_decode(self.q, self.kv, self.tab, self.lens, self.case.softmax_scale, self.out, self.lse,
                              variant=v, flags=f, num_splits=splits, workspace=ws)

    def time(self, name, steps, warmup, balanced=False, splits=0):
        self.step(name, balanced, splits)            # allocates the workspace outside the timed region
        return time_steps(self.torch, lambda: self.step(name, balanced, splits), steps, warmup)


def oracle_leg(case, flops_per_seq, out, lse, budget_s=14.0):
    """The oracle as it stands, one sequence at a time, until ~budget_s of CPU work: its speed (the CPU
    baseline) and, for the sequences it got through, the timed kernel's worst deviation from it (the parity
    block)."""
    import numpy as np
    from oracle import amla_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    done, flops, worst_out, worst_lse, big = 0, 0, 0.0, 0.0, 0
    spent = 0.0
    for b in range(case.batch):
        t0 = time.perf_counter()
        want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale, seq_ids=[b])
        spent += time.perf_counter() - t0
        done += 1
        flops += flops_per_seq[b]
        fin = np.isfinite(want_lse[b])
        small = np.abs(want[b]) < 4.0           # where |exact| >= 4 the bf16 output format's half step alone is 1.56e-2
        big += int((~small).sum())
        if small.any():
            worst_out = max(worst_out, float(np.abs(out[b] - want[b])[small].max()))
        if fin.any():
            worst_lse = max(worst_lse, float(np.abs(lse[b] - want_lse[b])[fin].max()))
        if spent >= budget_s:
            break
    cpu = {"value": flops / spent / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
           "sample": f"first {done} of {case.batch} sequences of the same workload, fp64 numpy, {spent:.1f} s"}
    parity = {"max_out_err": worst_out, "max_lse_err": worst_lse, "rows_checked": done * case.s_q * case.heads,
              "rows_total": case.batch * case.s_q * case.heads, "out_bound": 1e-2, "lse_bound": 1e-3,
              "elements_with_exact_ge_4_left_to_the_bf16_half_step": big,
              "passed": bool(worst_out <= 1e-2 and worst_lse <= 1e-3)}
    return cpu, parity


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
    names = variants(amla)
    if args.variant not in names:
        print(f"bench.py: no variant {args.variant}; one of {', '.join(names)}", file=sys.stderr)
        sys.exit(2)
    if args.table5 == "all":
        rows = []
        for sq in (1, 2):
            for sk in (1024, 2048, 3072, 4096, 6144, 16384):
                case = wl.make_table5_case(sq, sk)
                prob = Problem(torch, amla, case)
                total, _ = prob.time(args.variant, 50, 5)
                fl = acc.decode_flops(case.heads, case.s_q, case.total_kv)
                rows.append({"s_q": sq, "s_k": sk, "duration_us": total / 50 * 1e3, "tflops": fl / (total / 50 * 1e-3) / 1e12,
                             "frac_of_mfma_peak": fl / (total / 50 * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS})
                del prob
        print(json.dumps({"table5": rows, "variant": args.variant, "batch": 96, "heads": 128,
                          "note": "the shapes of the paper's Table 5 (Section 5.2); its own rows were measured on other hardware"}))
        return
    if args.table5:
        sq, sk = (int(x) for x in args.table5.split(","))
        case = wl.make_table5_case(sq, sk)
        workload_tag = f"paper Table 5 shape {case.name}"
    elif args.low_heads:
        case = wl.make_low_head_case(heads=args.low_heads)
        workload_tag = f"low-head-count batch {case.name}"
    else:
        case = wl.make_config(args.config)
        workload_tag = f"configs[{args.config}] {case.name}"
    prob = Problem(torch, amla, case)
    chosen = args.variant
    splits = amla.amla_effective_splits(prob.desc(chosen, args.balanced, args.splits))

    torch.cuda.synchronize()
    total_ms, per = prob.time(chosen, args.steps, args.warmup, args.balanced, args.splits)
    torch.cuda.synchronize()
    out_host = prob.out.float().cpu().numpy().astype(np.float64)
    lse_host = prob.lse.cpu().numpy().astype(np.float64)

    flops = acc.decode_flops(case.heads, case.s_q, case.total_kv)
    abytes = acc.algorithmic_bytes(case.heads, case.s_q, case.batch, case.total_kv)
    ms_per_step = total_ms / args.steps
    tflops = flops / (ms_per_step * 1e-3) / 1e12
    kern_ms = sum(per) / len(per)          # one decode launch per step (+ the combine kernel when split)
    achieved = flops / (kern_ms * 1e-3) / 1e12
    kname = kernel_name(chosen, args.balanced)
    measured = MEASURED_TRAFFIC.get((kname, chosen, case.name, splits))
    traffic = measured["read"] + measured["written"] if measured else None

    result = {
        "metric": METRIC, "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{workload_tag}: batch {case.batch}, s_q {case.s_q}, "
                               f"{case.heads} heads, sum kv_len {case.total_kv}, paged bf16 latent cache "
                               f"(block 64), d_qk 576 / d_v 512",
                   "variant": chosen, "rescale": {"mul": "FP32 multiply (Algorithm 1)", "add": "INT32 exponent add (Lemma 3.1)",
                                                  "add_comp": "INT32 add with Algorithm 2's BF16 scale compensation"}.get(
                                                      chosen.replace("_t", ""), chosen),
                   "kv_splits": splits, "decomposition": "balanced" if args.balanced else "equal_share", "seed": case.seed},
        "pct_of_mfma_peak": 100.0 * tflops / MFMA_BF16_PEAK_TFLOPS,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic, "traffic_unit": "B per launch",
                     "traffic_read_written": measured, "traffic_over_algorithmic": traffic / abytes if traffic else None,
                     "kernel": kname, "kernel_ms": kern_ms, "kernel_ms_median": median(per), "kernel_ms_min": min(per),
                     "algorithmic_flops_per_launch": flops, "algorithmic_bytes_per_launch": abytes,
                     "algorithmic_GBps": abytes / (kern_ms * 1e-3) / 1e9, "hbm_peak_GBps": HBM_PEAK_GBS},
    }
    notes = []
    try:
        cus, khz = amla.amla_device_info()
        prop = torch.cuda.get_device_properties(0)
        result["config"]["device"] = {"name": prop.name, "compute_units": cus, "max_engine_clock_mhz": khz / 1e3,
                                      "datasheet_peak_from_these_tflops": cus * 4096 * khz * 1e3 / 1e12}
    except Exception as e:  # noqa: BLE001
        notes.append(f"device properties unavailable: {e!r}")

    if not args.no_mfma_probe:
        try:
            # sustained rate of a register-resident MFMA loop on this device, same process: what the
            # chip delivers under its power limit with nothing else running
            probe_flops = [0.0]

            def probe():
                probe_flops[0] = amla.amla_mfma_probe(20000, 256)
            t, _ = time_steps(torch, probe, 5, 2)
            measured = probe_flops[0] / (t / 5 * 1e-3) / 1e12
            result["roofline"]["measured_mfma_peak"] = measured
            result["roofline"]["frac_of_measured_peak"] = achieved / measured
        except Exception as e:  # noqa: BLE001
            notes.append(f"mfma probe failed: {e!r}")

    if not args.no_ab:
        try:
            # every variant of both families, interleaved, median of the per-launch times
            ab = {}
            reps = 2
            n = max(10, min(40, args.steps))
            for _ in range(reps):
                for name in names:
                    try:
                        _, p = prob.time(name, n, 2, args.balanced, args.splits)
                        ab.setdefault(name, []).extend(p)
                    except Exception as e:  # noqa: BLE001  (a variant that does not exist for this decomposition)
                        ab.setdefault(name, None)
            med = {k: median(v) for k, v in ab.items() if v}
            # the paper's comparison, strict ADD against strict MUL on the same kernel: alternate launches
            pairs = {}
            for a, b in (("add", "mul"), ("add_512", "mul_512"), ("add_t", "mul_t")):
                ta, tb = [], []
                for _ in range(4):
                    ta.extend(prob.time(a, 10, 2, args.balanced, args.splits)[1])
                    tb.extend(prob.time(b, 10, 2, args.balanced, args.splits)[1])
                pairs[f"{a}_over_{b}_speedup"] = median(tb) / median(ta)
                pairs[f"{a}_ms_median_of_{len(ta)}"] = median(ta)
                pairs[f"{b}_ms_median_of_{len(tb)}"] = median(tb)
            result["rescale"] = {"ms_median": med, "tflops": {k: flops / (v * 1e-3) / 1e12 for k, v in med.items()}, **pairs,
                                 "note": "same binary; mul / add / add_comp = row-rescale kernels (rescale per moved row, reference moves "
                                         "once per 64-key cache block); _512 = the same with the reference moving once per 512 keys, "
                                         "the KV block of Section 4.2; _t = "
                                         "transposed-accumulator kernels (rescale of all 256 registers whenever a row of the "
                                         "wave moved); lazy = reference moves only past 2^8; add_ldexp = the exponent add done "
                                         "by v_ldexp_f32; strict = reference moves with every new row max"}
        except Exception as e:  # noqa: BLE001  (an optional leg must not cost the headline line)
            notes.append(f"rescale side-by-side failed: {e!r}")

    if not args.no_cpu_baseline:
        try:
            per_seq = [acc.decode_flops(case.heads, case.s_q, int(L)) for L in case.seqlens]
            result["cpu_baseline"], result["parity"] = oracle_leg(case, per_seq, out_host, lse_host)
            result["parity"]["kernel"] = kname
            result["parity"]["variant"] = chosen
        except Exception as e:  # noqa: BLE001
            notes.append(f"oracle leg failed: {e!r}")

    if not args.no_per_config and not args.table5 and not args.low_heads and args.config == 2:
        per_config = {}
        del prob
        torch.cuda.empty_cache()
        for idx in (1, 3, 4, "low_heads"):
            try:
                c = wl.make_low_head_case() if idx == "low_heads" else wl.make_config(idx)
                pr = Problem(torch, amla, c)
                if idx == 1:
                    pr.second_pool()      # 302 MB pool: alternate two copies so that it comes from HBM each launch
                fl = acc.decode_flops(c.heads, c.s_q, c.total_kv)
                ab_ = acc.algorithmic_bytes(c.heads, c.s_q, c.batch, c.total_kv)
                entry = {"workload": f"batch {c.batch}, s_q {c.s_q}, {c.heads} heads, sum kv_len {c.total_kv}"
                                     + (", two pool copies read alternately" if idx == 1 else "")}
                legs = [("add", False), ("mul", False), ("add_512", False)] + ([("add", True), ("mul", True), ("add_512", True)] if idx == 3 else [])
                times = {}
                # the first launches on a fresh problem run slow whatever the variant (clocks and address
                # translation settle): one untimed pass over every leg, then interleaved passes in alternating order
                for name, bal in legs:
                    pr.time(name, 10, 10, bal)
                for order in (legs, legs[::-1]):
                    for name, bal in order:
                        _, p = pr.time(name, 20, 3, bal)
                        times.setdefault((name, bal), []).extend(p)
                for (name, bal), p in times.items():
                    ms = median(p)
                    tf = fl / (ms * 1e-3) / 1e12
                    gbs = ab_ / (ms * 1e-3) / 1e9
                    mfma_t, hbm_t = fl / (MFMA_BF16_PEAK_TFLOPS * 1e12), ab_ / (HBM_PEAK_GBS * 1e9)
                    entry[name + ("_balanced" if bal else "")] = {
                        "ms_median_of_40": ms, "tflops": tf, "algorithmic_GBps": gbs,
                        "kv_splits": amla.amla_effective_splits(pr.desc(name, bal)),
                        "binding_roof": "hbm" if hbm_t > mfma_t else "mfma",
                        "frac_of_binding_roof": max(mfma_t, hbm_t) / (ms * 1e-3),
                        "frac_of_mfma_peak": tf / MFMA_BF16_PEAK_TFLOPS, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}
                entry["add_over_mul_speedup"] = median(times[("mul", False)]) / median(times[("add", False)])
                per_config[f"configs[{idx}] {c.name}" if idx != "low_heads" else
                           f"{c.name} (one GPU's 16 heads of an eight-way tensor-parallel group)"] = entry
                del pr
                torch.cuda.empty_cache()
            except Exception as e:  # noqa: BLE001
                notes.append(f"per_config {idx} failed: {e!r}")
        result["per_config"] = per_config
    if notes:
        result["notes"] = notes

    print(json.dumps(result))


if __name__ == "__main__":
    main()
