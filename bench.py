"""Benchmark of the quantized GEMV hot path on one MI355X.

A step is one pass of the whole path over the LLaMA-7B-shaped decoder layer set at batch 1,
4-bit codes, group 128 (seven matrices: four 4096x4096, two 11008x4096, one 4096x11008, each
with its own fp32 x): ONE grouped kernel launch reading the packed weights from HBM.
Weights are quantized and packed by the library before the timed region (by default into the
narrow device layout, qg_pack + qg_to_narrow, read by qg_gemv_grouped_narrow; --layout wide
times qg_gemv_grouped on the wide layout, and the default run reports it beside) and stay resident
in HBM; to keep the 256 MB last-level cache from serving them, the timed loop rotates over
enough distinct packed copies of the set that consecutive uses of a copy are more than 1.2 GB
of traffic apart.

Prints one JSON line.  `value` is microseconds per layer set; `roofline` prices the GEMV
kernel against the 8 TB/s HBM peak with the algorithmic bytes of the set (codes + fp32 scale
+ b-bit zero per group + x + y); `cpu_baseline` is the CPU oracle on the same packed data, and
its result doubles as the check of what was timed: `parity_max_scaled_err` compares the y of
the last timed launch with it and the run fails above 1e-4.  `other_workloads` carries the
13B- and 65B-shaped layer sets (3-bit g64, 2-bit g32; timing only, weights drawn on the GPU)
and the nine small-M GEMM problems, timed the same way.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np
import torch

HBM_PEAK_GBS = 8000.0          # MI355X public peak
# HBM bytes of one grouped launch as rocprofv3 counted them (FETCH_SIZE + WRITE_SIZE, scaled by the
# same counters of a 256 MiB device copy): kept in a tracked file with the kernel they were
# measured on, and reported only while that kernel is still the one that runs
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
ROTATE_BYTES = 1.3e9           # distinct packed bytes touched between two uses of one copy
TOL_FP32 = 1e-4                # bound on max |y - y*| / (|What[n,:]| |x|) of the GEMV


def measured_traffic(name, kernel):
    """(bytes, source) of the profiled HBM traffic of workload `name`, or (None, reason)."""
    try:
        with open(TRAFFIC_FILE) as fh:
            rec = json.load(fh).get(name)
    except (OSError, ValueError):
        return None, "no profiles/hbm_traffic.json"
    if not rec:
        return None, f"no counter run recorded for {name}"
    recs = rec if isinstance(rec, list) else [rec]
    match = [r for r in recs if r["kernel"] == kernel]
    if not match:
        return None, f"counters were taken on {', '.join(r['kernel'] for r in recs)}, this run used {kernel}"
    rec = match[0]
    return rec["bytes"], f"{rec['source']} ({rec['date']}; rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, carried over)"


def algorithmic_bytes(cfg) -> int:
    """Bytes the method itself has to move for one layer set: b bits per weight, one fp32
    scale and one b-bit zero per group (the paper's memory formula, Section 3, with K/G
    groups per output), x read once and y written once per matrix."""
    total = 0
    for n, k in cfg.shapes:
        bits = cfg.bits * n * k + (32 + cfg.bits) * n * (k // cfg.group)
        total += bits // 8 + 4 * k + 4 * n
    return total


def prepare_set(cfg, qg):
    """Quantize and pack every matrix of the set on the GPU; returns problem dicts."""
    from paper_2307_03738_amd import synth
    problems = []
    for i, (n, k) in enumerate(cfg.shapes):
        W, (x,) = synth.matrix(cfg, i)
        Wd = torch.from_numpy(W).cuda()
        q, s, z = qg.qg_quantize(Wd, cfg.bits, cfg.group)
        blob = qg.qg_pack(q, s, z, cfg.bits, cfg.group)
        problems.append(dict(packed=blob, N=n, K=k, bits=cfg.bits, group=cfg.group,
                             x=torch.from_numpy(x).cuda(),
                             y=torch.empty(n, dtype=torch.float32, device="cuda"),
                             host=(q.cpu().numpy(), s.cpu().numpy(), z.cpu().numpy(), x)))
        del Wd, q, s, z
    torch.cuda.synchronize()
    return problems


def cpu_baseline(cfg, problems, timed_y, passes=5):
    """The oracle's packed-format matvec over the whole layer set on the host cores, timed; its
    result also checks the y of the last timed GPU launch (`timed_y`, host arrays).  Returns
    (cpu_baseline record, max scaled error)."""
    from oracle import oracle
    packed = []
    for p in problems:
        q, s, z, x = p["host"]
        packed.append((oracle.pack_codes(q, cfg.bits), oracle.transpose_scales(s),
                       oracle.pack_zeros(z, cfg.bits), p["K"], x))
    results = []
    def one_pass():
        t0 = time.perf_counter()
        results[:] = [oracle.matvec_packed(P, St, Zp, K, cfg.bits, cfg.group, x) for P, St, Zp, K, x in packed]
        return time.perf_counter() - t0
    cores = len(os.sched_getaffinity(0))       # the host cores this process may use
    oracle.set_threads(cores)
    times = [one_pass() for _ in range(passes)]
    oracle.set_threads(1)
    single = [one_pass() for _ in range(2)]
    oracle.set_threads(cores)
    worst = 0.0
    for p, y_ref, y in zip(problems, results, timed_y):
        q, s, z, x = p["host"]
        den = oracle.row_norms(q, s, z, cfg.group) * np.linalg.norm(x.astype(np.float64))
        worst = max(worst, float(np.max(np.abs(y.astype(np.float64) - y_ref) / np.where(den == 0, 1.0, den))))
    return {"value": round(float(np.median(times)) * 1e6, 1), "unit": "us per layer set",
            "cores": cores, "kind": "oracle",
            "sample": f"full {cfg.name} layer set from the canonical packed format, median of {passes} passes",
            "single_thread_us": round(float(min(single)) * 1e6, 1)}, worst


MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X public dense bf16 peak


def bench_gemm(cfg, qg, args):
    """Prompt-phase form (configuration 5): every (shape, M) problem timed on its own, packed
    copies rotated like the GEMV's.  A step is one pass over the nine problems."""
    from paper_2307_03738_amd import synth
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    stream_steps, warm = max(20, args.steps // 10), max(5, args.warmup // 10)
    rows, total_us = [], 0.0
    for idx, (N, K) in enumerate(cfg.shapes):
        W, acts = synth.matrix(cfg, idx)
        q, s, z = qg.qg_quantize(torch.from_numpy(W).cuda(), cfg.bits, cfg.group)
        blob = qg.qg_pack(q, s, z, cfg.bits, cfg.group)
        del q, s, z
        copies = max(2, int(np.ceil(ROTATE_BYTES / blob.numel())))
        blobs = [blob] + [blob.clone() for _ in range(copies - 1)]
        for M, X in zip(cfg.batch, acts):
            Xd = torch.from_numpy(X).cuda()
            Y = torch.empty((M, N), dtype=torch.float32, device="cuda")
            ws = qg.new_workspace(qg.qg_workspace_bytes(N, K, cfg.bits, cfg.group, M))
            searched = None
            if args.autotune:        # the launch-shape search, recorded for this problem; untimed
                sp, sh, _ = qg.qg_gemm_autotune(blobs, N, K, cfg.bits, cfg.group, Xd, Y, ws, repeats=2 * copies)
                _, n_timed, n_dropped = qg.qg_gemm_autotune_report()
                searched = {"K_ranges": sp, "shape": sh, "candidates_timed": n_timed,
                            "candidates_dropped_by_the_price": n_dropped}
            for i in range(warm):
                qg.qg_gemm_small(blobs[i % copies], N, K, cfg.bits, cfg.group, Xd, Y, ws)
            torch.cuda.synchronize()
            start.record()
            for i in range(stream_steps):
                qg.qg_gemm_small(blobs[i % copies], N, K, cfg.bits, cfg.group, Xd, Y, ws)
            stop.record()
            torch.cuda.synchronize()
            us = start.elapsed_time(stop) / stream_steps * 1e3
            flops = 2.0 * M * N * K
            byts = (cfg.bits * N * K + (32 + cfg.bits) * N * (K // cfg.group)) // 8 + 4 * M * K + 4 * M * N
            rows.append({"N": N, "K": K, "M": M, "us": round(us, 2),
                         "TFLOPs": round(flops / us / 1e6, 1),
                         "frac_of_bf16_mfma_peak": round(flops / us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4),
                         "GBps": round(byts / us / 1e3, 1),
                         "frac_of_hbm_peak": round(byts / us / 1e3 / HBM_PEAK_GBS, 4)})
            if searched:
                rows[-1]["autotuned"] = searched
            total_us += us
        del blobs, blob
    top = max(rows, key=lambda r: r["TFLOPs"])
    return {
        "metric": "us per pass over the small-M GEMM problems (3 LLaMA-7B shapes x M = 16, 64, 128), 4-bit g128",
        "value": round(total_us, 2), "unit": "us", "n_gpus": 1, "steps": stream_steps, "warmup": warm,
        "ms_per_step": round(total_us / 1e3, 6), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: Y = X What^T, shapes {list(cfg.shapes)}, M in {list(cfg.batch)}, "
                               f"{cfg.bits}-bit, group {cfg.group}, bf16 MFMA with fp32 accumulation"},
        "problems": rows,
        "roofline": {"bound": "mfma", "achieved": top["TFLOPs"], "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": top["frac_of_bf16_mfma_peak"], "traffic": None,
                     "problem": {k: top[k] for k in ("N", "K", "M")}},
    }


def bench_sweep(qg, args):
    """Group size x bit width on the three LLaMA-shaped layer sets (timing only; weights are
    seeded Gaussian noise drawn on the GPU, since the kernels have no data-dependent control
    flow).  Group 0 stands for one group per output (G = K, the full-column form of eq. (1))."""
    from paper_2307_03738_amd import synth
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    stream = torch.cuda.current_stream().cuda_stream
    steps, warm = max(1, args.steps // 10), max(1, args.warmup // 10)
    rows = []
    for name in ("C2", "C3", "C4"):
        shapes = synth.CONFIGS[name].shapes
        gen = torch.Generator(device="cuda").manual_seed(100 + synth.CONFIGS[name].seed)
        Ws = {}
        for n, k in set(shapes):
            Ws[(n, k)] = torch.randn((n, k), device="cuda", generator=gen) * 0.02
        xs = {k: torch.randn((k,), device="cuda", generator=gen) for k in {k for _, k in shapes}}
        for bits in (4, 3, 2):
            for group in args.sweep_groups:
                if group and group % qg.qg_cell(bits):
                    continue
                packed = {}
                for (n, k), W in Ws.items():
                    g = group or k
                    q, s, z = qg.qg_quantize(W, bits, g)
                    packed[(n, k)] = qg.qg_pack(q, s, z, bits, g)
                    del q, s, z
                set_bytes = sum(packed[s_].numel() for s_ in shapes)
                copies = max(2, int(np.ceil(ROTATE_BYTES / set_bytes)))
                launches = []
                for c in range(copies):
                    probs = [dict(packed=(packed[(n, k)] if c == 0 else packed[(n, k)].clone()), N=n, K=k,
                                  bits=bits, group=group or k, x=xs[k],
                                  y=torch.empty(n, dtype=torch.float32, device="cuda")) for n, k in shapes]
                    launches.append(qg.GroupedGemv(probs))
                for i in range(warm):
                    launches[i % copies].launch(stream)
                torch.cuda.synchronize()
                start.record()
                for i in range(steps):
                    launches[i % copies].launch(stream)
                stop.record()
                torch.cuda.synchronize()
                us = start.elapsed_time(stop) / steps * 1e3
                alg = sum((bits * n * k + (32 + bits) * n * (k // (group or k))) // 8 + 4 * k + 4 * n for n, k in shapes)
                rows.append({"shapes": name, "bits": bits, "group": group or "K", "us": round(us, 2),
                             "GBps": round(alg / us / 1e3, 1), "frac_of_hbm_peak": round(alg / us / 1e3 / HBM_PEAK_GBS, 4)})
                print(json.dumps(rows[-1]), file=sys.stderr, flush=True)
                del launches, packed
        del Ws
    return {"metric": "us per GEMV layer set over group size x bit width", "unit": "us", "n_gpus": 1,
            "steps": steps, "warmup": warm, "dtype": "f32", "data": "synthetic (timing only)",
            "config": {"workload": "layer sets with the shapes of C2, C3, C4; bits in {4,3,2}; group in {16,32,64,128,K}"},
            "rows": rows}


def bench_offline(qg, args):
    """The off-line steps (quantize, pack, unpack) on the largest matrix of each layer set.
    Each is a streaming pass; its bytes are what the step has to read and write once."""
    L = qg.lib()
    stream = torch.cuda.current_stream().cuda_stream
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(3, args.steps // 100)

    def timed(fn):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        start.record()
        for _ in range(reps):
            fn()
        stop.record()
        torch.cuda.synchronize()
        return start.elapsed_time(stop) / reps * 1e3

    rows = []
    for bits, group, N, K in ((4, 128, 11008, 4096), (3, 64, 13824, 5120), (2, 32, 22016, 8192)):
        gen = torch.Generator(device="cuda").manual_seed(bits)
        W = torch.randn((N, K), generator=gen, device="cuda", dtype=torch.float32) * 0.02
        q, s, z = qg.qg_quantize(W, bits, group)
        G = K // group
        row = {"N": N, "K": K, "bits": bits, "group": group}

        def check(rc):
            if rc != 0:
                raise RuntimeError(f"library call failed with status {rc}")
        us = timed(lambda: check(L.qg_quantize(W.data_ptr(), N, K, bits, group, q.data_ptr(), s.data_ptr(),
                                               z.data_ptr(), stream)))
        nbytes = 4 * N * K + N * K + 5 * N * G
        row["quantize_us"], row["quantize_GBps"] = round(us, 1), round(nbytes / us / 1e3, 1)
        for name, layout in (("device", qg.QG_LAYOUT_DEVICE), ("canonical", qg.QG_LAYOUT_CANONICAL)):
            pb = qg.qg_packed_bytes(N, K, bits, group, layout)
            blob = torch.empty(pb, dtype=torch.uint8, device="cuda")
            us = timed(lambda: check(L.qg_pack(q.data_ptr(), s.data_ptr(), z.data_ptr(), N, K, bits, group,
                                               layout, blob.data_ptr(), stream)))
            nbytes = N * K + 5 * N * G + pb
            row[f"pack_{name}_us"], row[f"pack_{name}_GBps"] = round(us, 1), round(nbytes / us / 1e3, 1)
            q2, s2, z2 = torch.empty_like(q), torch.empty_like(s), torch.empty_like(z)
            us = timed(lambda: check(L.qg_unpack(blob.data_ptr(), N, K, bits, group, layout, q2.data_ptr(),
                                                 s2.data_ptr(), z2.data_ptr(), stream)))
            row[f"unpack_{name}_us"], row[f"unpack_{name}_GBps"] = round(us, 1), round(nbytes / us / 1e3, 1)
            if not (torch.equal(q, q2) and torch.equal(s, s2) and torch.equal(z, z2)):
                raise RuntimeError("pack / unpack round trip changed the data")
            del blob, q2, s2, z2
        rows.append(row)
        del W, q, s, z
    return {"metric": "us per off-line step (quantize, pack, unpack) on the largest matrix of each layer set",
            "unit": "us", "n_gpus": 1, "data": "synthetic", "repeats": reps, "hbm_peak_GBps": HBM_PEAK_GBS,
            "rows": rows}


def narrow_launch(qg, problems):
    """The same grouped launch on the narrow layout (same x and y tensors, repacked weights)."""
    return qg.GroupedGemvNarrow([dict(p, packed=qg.qg_to_narrow(p["packed"], p["N"], p["K"], p["bits"], p["group"]))
                                 for p in problems])


def gpu_drawn_launches(qg, name, layout="wide"):
    """Rotated grouped launches of configuration `name` with Gaussian weights drawn on the GPU
    (timing only: the kernels have no data-dependent control flow)."""
    from paper_2307_03738_amd import synth
    cfg = synth.CONFIGS[name]
    gen = torch.Generator(device="cuda").manual_seed(100 + cfg.seed)
    packed = {}
    for n, k in set(cfg.shapes):
        W = torch.randn((n, k), device="cuda", generator=gen) * cfg.std
        q, s, z = qg.qg_quantize(W, cfg.bits, cfg.group)
        packed[(n, k)] = qg.qg_pack(q, s, z, cfg.bits, cfg.group)
        del W, q, s, z
    xs = {k: torch.randn((k,), device="cuda", generator=gen) for k in {k for _, k in cfg.shapes}}
    set_bytes = sum(packed[s_].numel() for s_ in cfg.shapes)
    copies = max(2, int(np.ceil(ROTATE_BYTES / set_bytes)))
    launches = []
    for c in range(copies):
        probs = [dict(packed=(packed[(n, k)] if c == 0 else packed[(n, k)].clone()), N=n, K=k, bits=cfg.bits,
                      group=cfg.group, x=xs[k], y=torch.empty(n, dtype=torch.float32, device="cuda"))
                 for n, k in cfg.shapes]
        launches.append(narrow_launch(qg, probs) if layout == "narrow" else qg.GroupedGemv(probs))
    torch.cuda.synchronize()
    return cfg, launches


def time_launches(launches, steps, warmup):
    """Microseconds per launch over `steps` launches that rotate over the prepared copies."""
    stream = torch.cuda.current_stream().cuda_stream
    copies = len(launches)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(warmup):
        launches[i % copies].launch(stream)
    torch.cuda.synchronize()
    start.record()
    for i in range(steps):
        launches[i % copies].launch(stream)
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / steps * 1e3


def other_workloads(qg, args):
    """The other layer sets and the small-M GEMM problems, each timed like the headline one."""
    from paper_2307_03738_amd import synth
    out = {}
    for name in ("C3", "C4"):
        row = {}
        for layout in ("narrow", "wide"):
            cfg, launches = gpu_drawn_launches(qg, name, layout)
            us = time_launches(launches, max(20, args.steps // 4), max(5, args.warmup // 4))
            alg = algorithmic_bytes(cfg)
            row[layout] = {"kernel": qg.qg_last_narrow_kernel() if layout == "narrow" else qg.qg_last_gemv_kernel(),
                           "us": round(us, 3), "GBps": round(alg / us / 1e3, 1),
                           "frac_of_hbm_peak": round(alg / us / 1e3 / HBM_PEAK_GBS, 4),
                           "packed_copies_rotated": len(launches)}
            del launches
        best = min(row, key=lambda k: row[k]["us"])
        out[name] = {"workload": f"{name}: decoder layer set {list(cfg.shapes)}, {cfg.bits}-bit, group {cfg.group}, "
                                 "batch 1, one grouped launch per set (timing only, weights drawn on the GPU)",
                     "algorithmic_bytes_per_set": alg, "layout": best, **row[best],
                     "other_layout": {"layout": [k for k in row if k != best][0], **row[[k for k in row if k != best][0]]}}
    gemm = bench_gemm(synth.CONFIGS["C5"], qg, args)
    out["C5"] = {"workload": gemm["config"]["workload"], "us_all_problems": gemm["value"],
                 "problems": gemm["problems"]}
    out["gemm_other_widths_M16"] = bench_gemm_other_widths(qg, args)
    out["stacked_qkv"] = bench_stacked_qkv(qg, args)
    return out


def bench_gemm_other_widths(qg, args, Ms=(16,)):
    """The small-M product at 3 and 2 bits: M = 16 (or `Ms`) on the three shapes of the 13B- and
    65B-shaped layer sets (timing only, weights drawn on the GPU), packed copies rotated."""
    from paper_2307_03738_amd import synth
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    steps, warm = max(20, args.steps // 10), max(5, args.warmup // 10)
    rows = []
    for name in ("C3", "C4"):
        cfg = synth.CONFIGS[name]
        gen = torch.Generator(device="cuda").manual_seed(200 + cfg.seed)
        for N, K in sorted(set(cfg.shapes)):
            W = torch.randn((N, K), device="cuda", generator=gen) * cfg.std
            q, s, z = qg.qg_quantize(W, cfg.bits, cfg.group)
            blob = qg.qg_pack(q, s, z, cfg.bits, cfg.group)
            del W, q, s, z
            copies = max(2, int(np.ceil(ROTATE_BYTES / blob.numel())))
            blobs = [blob] + [blob.clone() for _ in range(copies - 1)]
            for M in Ms:
                X = torch.randn((M, K), device="cuda", generator=gen)
                Y = torch.empty((M, N), dtype=torch.float32, device="cuda")
                ws = qg.new_workspace(qg.qg_workspace_bytes(N, K, cfg.bits, cfg.group, M))
                for i in range(warm):
                    qg.qg_gemm_small(blobs[i % copies], N, K, cfg.bits, cfg.group, X, Y, ws)
                torch.cuda.synchronize()
                start.record()
                for i in range(steps):
                    qg.qg_gemm_small(blobs[i % copies], N, K, cfg.bits, cfg.group, X, Y, ws)
                stop.record()
                torch.cuda.synchronize()
                us = start.elapsed_time(stop) / steps * 1e3
                byts = (cfg.bits * N * K + (32 + cfg.bits) * N * (K // cfg.group)) // 8 + 4 * M * K + 4 * M * N
                rows.append({"N": N, "K": K, "bits": cfg.bits, "group": cfg.group, "M": M, "us": round(us, 2),
                             "GBps": round(byts / us / 1e3, 1), "frac_of_hbm_peak": round(byts / us / 1e3 / HBM_PEAK_GBS, 4),
                             "TFLOPs": round(2.0 * M * N * K / us / 1e6, 1),
                             "frac_of_bf16_mfma_peak": round(2.0 * M * N * K / us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4)})
            del blobs, blob
    return rows


def bench_stacked_qkv(qg, args):
    """q, k and v of a 7B-shaped block (4-bit, group 128) as ONE 3H x H product against the same
    three products as problems of one grouped launch (timing only), packed copies rotated."""
    H, bits, group = 4096, 4, 128
    gen = torch.Generator(device="cuda").manual_seed(300)
    W3 = torch.randn((3 * H, H), device="cuda", generator=gen) * 0.02
    x = torch.randn((H,), device="cuda", generator=gen)
    q, s, z = qg.qg_quantize(W3, bits, group)
    stacked = qg.qg_pack(q, s, z, bits, group)
    parts = [qg.qg_pack(q[i * H:(i + 1) * H].contiguous(), s[i * H:(i + 1) * H].contiguous(),
                        z[i * H:(i + 1) * H].contiguous(), bits, group) for i in range(3)]
    del W3, q, s, z
    copies = max(2, int(np.ceil(ROTATE_BYTES / stacked.numel())))
    one, three = [], []
    for c in range(copies):
        one.append(qg.GroupedGemv([dict(packed=stacked.clone(), N=3 * H, K=H, bits=bits, group=group, x=x,
                                        y=torch.empty(3 * H, dtype=torch.float32, device="cuda"))]))
        three.append(qg.GroupedGemv([dict(packed=p.clone(), N=H, K=H, bits=bits, group=group, x=x,
                                          y=torch.empty(H, dtype=torch.float32, device="cuda")) for p in parts]))
    steps, warm = max(20, args.steps // 4), max(5, args.warmup // 4)
    return {"workload": "q/k/v of a 7B-shaped block, 4-bit group 128: one 12288 x 4096 product / three 4096 x 4096 problems in one launch",
            "one_stacked_product_us": round(time_launches(one, steps, warm), 3),
            "three_grouped_problems_us": round(time_launches(three, steps, warm), 3)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=1000)
    ap.add_argument("--config", default="C2", choices=["C2", "C3", "C4", "C5"])
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the oracle leg (and with it the check of the timed result)")
    ap.add_argument("--gemm-widths", action="store_true",
                    help="the small-M product at 3 and 2 bits on the 13B- and 65B-shaped matrices, M = 16, 64, 128")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="time the headline workload only")
    ap.add_argument("--autotune", action="store_true",
                    help="let qg_gemv_autotune (C5: qg_gemm_autotune per problem) pick the launch shape, timed over the "
                         "rotated copies, before the run")
    ap.add_argument("--sweep-groups", type=lambda s: [int(v) for v in s.split(",")], default=[16, 32, 64, 128, 0],
                    help="group sizes of --sweep; 0 = one group per output")
    ap.add_argument("--sweep", action="store_true",
                    help="time every group size x bit width on the three layer-set shapes instead")
    ap.add_argument("--offline", action="store_true",
                    help="time the off-line steps (quantize, pack, unpack) instead")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain device copy of 256 MiB (reference for HBM byte counters)")
    ap.add_argument("--gemm-shape", type=int, default=0,
                    help="--config C5: workgroup shape / kernel of qg_gemm_small (qg_set_gemm_tuning); 13 = raw-code kernel")
    ap.add_argument("--gemm-splits", type=int, default=0, help="--config C5: K ranges over workgroups (0 = built-in choice)")
    ap.add_argument("--layout", default="narrow", choices=["narrow", "wide"],
                    help="device layout of the packed weights for the GEMV: narrow (rows of 16 outputs x 4 steps of K, "
                         "qg_to_narrow + qg_gemv_grouped_narrow) or wide (rows of 64 outputs, qg_gemv_grouped)")
    ap.add_argument("--narrow-tiles-per-wave", type=int, default=0, help="qg_set_narrow_tuning (0 = built-in choice)")
    ap.add_argument("--wpb", type=int, default=0)
    ap.add_argument("--bytes-per-wave", type=int, default=0)
    ap.add_argument("--kernel", type=int, default=0, help="0 built-in choice, 1 vector-ALU GEMV, 2 matrix-core GEMV (32x32x16), 3 matrix-core GEMV (4x4x4, bf16), 4 matrix-core GEMV (4x4x4, int8)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: the path has no multi-GPU part (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    from paper_2307_03738_amd import binding as qg, synth
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.config]
    if args.gemm_widths:
        rows = bench_gemm_other_widths(qg, args, (16, 64, 128))
        print(json.dumps({"metric": "us per small-M product, 3-bit g64 and 2-bit g32", "unit": "us", "n_gpus": 1,
                          "data": "synthetic", "dtype": "bf16", "problems": rows}))
        return
    if args.sweep:
        qg.qg_set_gemv_tuning(args.wpb, args.bytes_per_wave, args.kernel)
        print(json.dumps(bench_sweep(qg, args)))
        return
    if args.offline:
        print(json.dumps(bench_offline(qg, args)))
        return
    if args.config == "C5":
        qg.qg_set_gemm_tuning(args.gemm_splits, args.gemm_shape)
        print(json.dumps(bench_gemm(cfg, qg, args)))
        return
    qg.qg_set_gemv_tuning(args.wpb, args.bytes_per_wave, args.kernel)

    base = prepare_set(cfg, qg)
    set_bytes = sum(p["packed"].numel() for p in base)
    copies = max(2, int(np.ceil(ROTATE_BYTES / set_bytes)))
    narrow = args.layout == "narrow"
    if narrow and (args.autotune or args.wpb or args.bytes_per_wave or args.kernel):
        print("--autotune, --wpb, --bytes-per-wave and --kernel belong to the wide layout (--layout wide)", file=sys.stderr)
        sys.exit(2)
    qg.qg_set_narrow_tuning(args.narrow_tiles_per_wave)
    launches, wide_launches = [], []
    for c in range(copies):
        probs = [dict(p, packed=(p["packed"] if c == 0 else p["packed"].clone())) for p in base]
        wide_launches.append(qg.GroupedGemv(probs))
        launches.append(narrow_launch(qg, probs) if narrow else wide_launches[-1])
    torch.cuda.synchronize()

    if args.copy_calibration:
        # a copy of known size: 256 MiB read + 256 MiB written; profilers' byte counters for this
        # kernel give the factor between counter units and bytes
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    tuned = None
    if args.autotune:
        tuned = qg.qg_gemv_autotune(launches, repeats=2 * copies)
    stream = torch.cuda.current_stream().cuda_stream
    for i in range(args.warmup):
        launches[i % copies].launch(stream)
    torch.cuda.synchronize()
    kernel_name = qg.qg_last_narrow_kernel() if narrow else qg.qg_last_gemv_kernel()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for i in range(args.steps):
        launches[i % copies].launch(stream)
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = start.elapsed_time(stop) / args.steps
    # what the last timed launch left in y (all copies share the y vectors of `base`)
    timed_y = [p["y"].cpu().numpy() for p in base]
    # the same timed loop four more times: spread of the measurement (the first one is `value`)
    repeats = [ms_per_step * 1e3]
    for _ in range(4):
        repeats.append(time_launches(launches, args.steps, 0))

    # the same launches on a single copy: weights served largely by the last-level cache
    warm_ms = time_launches(launches[:1], args.steps, 20) / 1e3
    # the other layout, for comparison
    wide_us = time_launches(wide_launches, max(args.steps, 400), max(50, args.warmup // 10)) if narrow else None
    wide_kernel = qg.qg_last_gemv_kernel() if narrow else None

    alg = algorithmic_bytes(cfg)
    achieved = alg / (ms_per_step * 1e-3) / 1e9
    traffic, traffic_source = measured_traffic(cfg.name, kernel_name)
    out = {
        "metric": "us per LLaMA-7B-shaped 4-bit g128 GEMV layer set (batch 1); % of HBM peak"
                  if args.config == "C2" else f"us per {cfg.name} GEMV layer set (batch 1); % of HBM peak",
        "value": round(ms_per_step * 1e3, 3), "unit": "us",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None,
        # what the multiply-adds run in: 4-bit codes as int8 against the int8 digits of x in 32-bit
        # fixed point (per step) on the 4x4x4 matrix instruction, int32 sums, fp32 per group and beyond
        "dtype": "i8 mfma (x as 32-bit fixed point), f32 accumulate"
                 if ("mma4i" in kernel_name or "narrow" in kernel_name) else "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: decoder layer set {list(cfg.shapes)}, {cfg.bits}-bit, "
                               f"group {cfg.group}, batch 1, one grouped launch per set",
                   "kernel": kernel_name,
                   "layout": "narrow: rows of 16 outputs x 4 steps of K (qg_pack, qg_to_narrow, qg_gemv_grouped_narrow)"
                             if narrow else "wide: rows of 64 outputs (qg_pack, qg_gemv_grouped)",
                   "packed_copies_rotated": copies, "packed_bytes_per_set": set_bytes,
                   "algorithmic_bytes_per_set": alg},
        "effective_weight_GBps": round(achieved, 1),
        "pct_of_hbm_peak": round(100 * achieved / HBM_PEAK_GBS, 2),
        "repeats_us": [round(r, 3) for r in repeats],
        "repeats_median_us": round(float(np.median(repeats)), 3), "repeats_min_us": round(min(repeats), 3),
        "cache_warm_single_copy_us": round(warm_ms * 1e3, 3),
        "host_wall_ms_per_step": round(wall_ms / args.steps, 6),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "traffic_source": traffic_source},
    }
    if narrow:
        out["wide_layout"] = {"kernel": wide_kernel, "us": round(wide_us, 3),
                              "frac_of_hbm_peak": round(alg / wide_us / 1e3 / HBM_PEAK_GBS, 4)}
    if tuned is not None:
        _, timed, dropped = qg.qg_gemv_autotune_report()
        out["autotuned"] = {"waves_per_block": tuned[0], "bytes_per_wave": tuned[1], "kernel": tuned[2],
                            "us_while_tuning": round(tuned[3], 3), "candidates_timed": timed,
                            "candidates_dropped_by_the_resource_budget": dropped}
    failed = False
    if not args.no_cpu_baseline:
        out["cpu_baseline"], err = cpu_baseline(cfg, base, timed_y)
        out["parity_max_scaled_err"] = float(f"{err:.3e}")
        out["parity_bound"] = TOL_FP32
        failed = not (err <= TOL_FP32)
    del launches, wide_launches, base
    if not args.no_other_workloads:
        qg.qg_set_gemv_tuning(0, 0, 0)
        out["other_workloads"] = other_workloads(qg, args)
    print(json.dumps(out))
    if failed:
        print(f"the timed launch's y is off by {err:.3e} of |What[n,:]| |x| (bound {TOL_FP32})", file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
