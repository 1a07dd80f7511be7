#!/usr/bin/env python3
"""Benchmark of the QSDP fused quantized SGD step on one MI355X.

Workload (the configuration the headline metric is quoted on): a GPT-1.3B-shaped flat fp32
parameter vector (1,315,723,264 elements: 24 layers, d = 2048, vocabulary 50257), weights
~ 0.02*N(0,1), gradients ~ 1e-3*Student-t(3); 8-bit weights, 4-bit gradients, bucket 1024,
lr 1e-3; step k uses seed k and updates x in place, g stays fixed.

A step is one call of qsdp_fused_step over the whole vector: x <- Q^w(x - lr*Q^g(g)), i.e.
bucket statistics, stochastic gradient rounding, decode, axpy, random-shift weight rounding
and decode, in one pass over HBM. Algorithmic traffic: 12 bytes per parameter (read x, read
g, write x). Inputs are resident in HBM before the timed region.

Prints ONE JSON line. `--gpus` above 1 is refused: this build is single-GPU.
"""
import argparse
import hashlib
import json
import os
import sys
import time

HBM_PEAK_GBS = 8000.0
BYTES_PER_PARAM = 12.0
ROOT = os.path.dirname(os.path.abspath(__file__))


def kernel_sources_digest():
    """SHA-256 over the codec's kernel sources and build flags: names the kernels a profile was taken on."""
    from paper_2302_02390_amd import build
    h = hashlib.sha256()
    for name in sorted(os.listdir(build.CSRC)):
        if name.endswith((".hip", ".hpp")) and name != "qsdp_bench_stream.hip":
            h.update(name.encode())
            with open(os.path.join(build.CSRC, name), "rb") as f:
                h.update(f.read())
    h.update(" ".join(build.FLAGS).encode())
    return h.hexdigest()


def profiled_traffic():
    """HBM bytes per fused-step launch on the headline workload, from the rocprofv3 --pmc summary committed as
    profiles/fused_step_gpt1p3b.json (FETCH_SIZE and WRITE_SIZE runs, each scaled by what the same counter reads
    for a plain copy of known size). The figure is offline evidence, not a measurement of this run: it is
    reported only while the kernel sources are byte for byte those the profile was taken on, else null."""
    try:
        with open(os.path.join(ROOT, "profiles", "fused_step_gpt1p3b.json")) as f:
            prof = json.load(f)
        if prof.get("kernel_sources_sha256") == kernel_sources_digest():
            return int(prof["traffic_bytes_per_launch"]), prof.get("commit")
    except (OSError, ValueError, KeyError):
        pass
    return None, None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="gpt-1.3b", choices=["gpt-1.3b", "gpt-350m", "gpt-125m", "1m"])
    ap.add_argument("--wbits", type=int, default=8)
    ap.add_argument("--gbits", type=int, default=None)
    ap.add_argument("--bucket", type=int, default=1024)
    ap.add_argument("--delta", type=float, default=0.0)
    ap.add_argument("--emit-codes", action="store_true", help="also write packed Q^w codes + meta")
    ap.add_argument("--per-layer", action="store_true",
                    help="run the step tensor by tensor (bucketing restarts per tensor, one call each)")
    ap.add_argument("--segmented", action="store_true",
                    help="bucketing restarts per tensor, all tensors in ONE segmented launch")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip timing the other entry points")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the headline run: the bits / bucket / delta sweep and the layer-by-layer "
                         "decode to bf16 on the chosen workload; still one JSON line (key 'sweep')")
    ap.add_argument("--levels-report", action="store_true",
                    help="instead of the headline run: relative L2 compression error of uniform and fitted "
                         "(learned) levels at 2..6 bits on the chosen workload, with the fit and codec timings; "
                         "one JSON line (key 'levels')")
    ap.add_argument("--cpu-sample", type=int, default=0,
                    help="elements of the workload the bucket-parallel CPU oracle is timed on (0: one whole step)")
    ap.add_argument("--cpu-single-sample", type=int, default=0,
                    help="elements the single-threaded CPU oracle is timed on (0: one whole step, about half a "
                         "minute on the 1.3B vector)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain device copy of the weight vector a few times (a kernel of "
                         "known traffic, to scale rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


def time_call(fn, iters, torch):
    """Average duration in ms of fn() over iters calls, from events on the current stream."""
    start = [torch.cuda.Event(enable_timing=True) for _ in range(iters)]
    stop = [torch.cuda.Event(enable_timing=True) for _ in range(iters)]
    for i in range(iters):
        start[i].record()
        fn(i)
        stop[i].record()
    torch.cuda.synchronize()
    ts = [a.elapsed_time(b) for a, b in zip(start, stop)]
    return sum(ts) / len(ts), sorted(ts)[len(ts) // 2]


def main():
    a = parse()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the codec has no collectives); "
              "run with --gpus 1", file=sys.stderr)
        return 2
    import torch
    from paper_2302_02390_amd import binding as qb
    from paper_2302_02390_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    qb.lib()  # fail loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if a.workload == "1m":
        n, cfg_id, heavy = 1 << 20, 0, False
    else:
        shape = {"gpt-1.3b": wl.GPT_1P3B, "gpt-350m": wl.GPT_350M, "gpt-125m": wl.GPT_125M}[a.workload]
        n, cfg_id, heavy = wl.model_numel(shape), {"gpt-125m": 1, "gpt-350m": 2, "gpt-1.3b": 3}[a.workload], True
    gbits = a.gbits if a.gbits is not None else (4 if a.workload in ("gpt-1.3b", "gpt-350m") else 8)
    wbits, bucket, delta, lr = a.wbits, a.bucket, a.delta, 1e-3

    x = wl.weights(n, 1234 + 2 * cfg_id, dev)
    g = wl.grads_student_t3(n, 1235 + 2 * cfg_id, dev) if heavy else wl.grads_normal(n, 1235 + 2 * cfg_id, dev)
    x0 = x.clone()
    wcodes = wmeta = None
    if a.emit_codes:
        wcodes, wmeta = qb.alloc_packed(n, wbits, bucket, dev)
        wmeta = wmeta.reshape(-1)
    torch.cuda.synchronize()

    def step(k):
        qb.qsdp_fused_step(x, g, lr, wbits, gbits, bucket, delta, k, 0, wcodes, wmeta, None)

    if a.sweep:
        print(json.dumps(sweep(torch, qb, wl, x, g, n, a.workload, dev)))
        return 0

    if a.levels_report:
        rep = levels_report(torch, qb, x, g, n, a.workload, bucket, dev)
        if a.workload != "1m":
            rep["per_layer_W5G4"] = levels_per_layer(torch, qb, wl, x, g, shape, bucket, dev)
        print(json.dumps(rep))
        return 0

    if a.segmented:
        if a.workload == "1m":
            print("bench.py: --segmented needs a GPT workload", file=sys.stderr)
            return 2
        segs = qb.Segments([size for _, size in wl.model_tensors(shape)], bucket, dev)
        if a.emit_codes:
            wcodes, wmeta = segs.alloc_packed(wbits)
            wmeta = wmeta.reshape(-1)

        def step(k):  # noqa: F811
            qb.qsdp_fused_step_segmented(x, g, segs, lr, wbits, gbits, delta, k, 0, wcodes, wmeta, None)

    if a.per_layer:
        if a.workload == "1m" or a.emit_codes or a.segmented:
            print("bench.py: --per-layer needs a GPT workload and no --emit-codes/--segmented", file=sys.stderr)
            return 2
        views, off = [], 0
        for _, size in wl.model_tensors(shape):
            views.append((x[off:off + size], g[off:off + size], off))
            off += size

        def step(k):  # noqa: F811
            for xs, gs, o in views:
                qb.qsdp_fused_step(xs, gs, lr, wbits, gbits, bucket, delta, k, o, None, None, None)

    for k in range(a.warmup):
        step(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(a.steps):
        step(a.warmup + k)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / max(a.steps, 1)

    # per-launch kernel duration from events on the launch stream (for the roofline entry)
    ev_iters = max(5, min(a.steps, 50))
    ev_mean, ev_median = time_call(lambda i: step(1000 + i), ev_iters, torch)

    # The measurement protocol of the 10-step configuration: the sequence of 10 steps (seeds 0..9, x carried) is
    # the unit, timed five times, each time from the restored x0.
    seq_ms = []
    for _ in range(5):
        x.copy_(x0)
        torch.cuda.synchronize()
        ms, _ = time_call(lambda i: [step(k) for k in range(10)], 1, torch)
        seq_ms.append(ms)

    bytes_per_param = BYTES_PER_PARAM + ((wbits / 8.0 + 8.0 / bucket) if a.emit_codes else 0.0)
    alg_bytes = bytes_per_param * n
    value_gbs = alg_bytes / (wall_ms * 1e-3) / 1e9
    achieved = alg_bytes / (ev_mean * 1e-3) / 1e9

    out = {
        "metric": "fused quantize+step GB/s (fraction of HBM peak) and params/s, 1.3B fp32 shard",
        "value": round(value_gbs, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": round(wall_ms, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "params_per_s": round(n / (wall_ms * 1e-3), 1),
        "hbm_peak_frac": round(value_gbs / HBM_PEAK_GBS, 4),
        "config": {
            "workload": f"{a.workload}-shaped flat fp32 vector, n={n}, W{wbits} G{gbits}, bucket {bucket}, "
                        f"delta {delta}, lr {lr}, seed = step index, in-place fused step"
                        + (", packed codes emitted" if a.emit_codes else "")
                        + (", one call per layer tensor" if a.per_layer else "")
                        + (", per-layer tensors in one segmented launch" if a.segmented else ""),
            "n": n, "wbits": wbits, "gbits": gbits, "bucket": bucket, "delta": delta,
            "spec_version": qb.spec_version(),
        },
        "roofline": {
            "bound": "hbm",
            "achieved": round(achieved, 2),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": None,
            "kernel": "qsdp::wave_kernel<MODE_FUSED, G=64, R=4, BITS=0, W=1> (qsdp_fused_step, bucket 1024, no code output)"
                      if (bucket == 1024 and not a.emit_codes) else "qsdp::wave_kernel<MODE_FUSED, ...> (qsdp_fused_step)",
            "algorithmic_bytes_per_launch": alg_bytes,
            "kernel_ms_mean": round(ev_mean, 4),
            "kernel_ms_median": round(ev_median, 4),
        },
    }

    headline = (a.workload == "gpt-1.3b" and not (a.emit_codes or a.per_layer or a.segmented)
                and (wbits, gbits, bucket, delta) == (8, 4, 1024, 0.0))
    if headline:
        traffic, commit = profiled_traffic()
        out["roofline"]["traffic"] = traffic
        out["roofline"]["traffic_source"] = (
            f"profiles/fused_step_gpt1p3b.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, taken at commit {commit} on "
            "these kernel sources)" if traffic is not None else
            "null: the committed counter profile was taken on other kernel sources than the ones in this tree")
    seq_sorted = sorted(seq_ms)
    out["ten_step_sequence"] = {
        "protocol": "10 fused steps (seeds 0..9, x carried) from the restored x0, timed 5 times",
        "ms_per_sequence": [round(v, 4) for v in seq_ms],
        "ms_per_step_median": round(seq_sorted[2] / 10.0, 4),
        "GB/s_median": round(alg_bytes * 10 / (seq_sorted[2] * 1e-3) / 1e9, 2)}

    if a.calibration_copy:
        y = torch.empty_like(x)
        for _ in range(3):
            y.copy_(x)
        torch.cuda.synchronize()
        out["calibration_copy_bytes"] = {"read": 4 * n, "write": 4 * n}
        del y

    if not a.no_extras:
        out["attainable"] = attainable(torch, x, g, n, achieved, lr)
        out["other_entry_points"] = extras(torch, qb, x, g, n, wbits, gbits, bucket, dev)
        att, oth = out["attainable"], out["other_entry_points"]
        att["adamw_mix_best_GB/s"] = max(att["adamw_mix_GB/s"], att["adamw_mix_2_workgroups_per_cu_GB/s"])
        att["fused_adamw_step_vs_adamw_mix"] = round(oth[f"fused_adamw_step_W{wbits}G{gbits}"]["GB/s"] /
                                                     att["adamw_mix_best_GB/s"], 3)
        att[f"quantize_grad_b{gbits}_vs_encode_mix"] = round(
            oth[f"quantize_grad_b{gbits}"]["GB/s"] / att[f"encode_{gbits}bit_mix_GB/s"], 3) \
            if f"encode_{gbits}bit_mix_GB/s" in att else None
        if a.segmented:
            out["segmented_entry_points"] = segmented_extras(torch, qb, x, n, segs, wbits, bucket, dev)

    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(x0, g, a.cpu_sample, a.cpu_single_sample, lr, wbits, gbits, bucket, delta,
                                           bytes_per_param)
    print(json.dumps(out))
    return 0


def attainable(torch, x, g, n, fused_achieved, lr):
    """What this memory system sustains for plain streaming kernels with the fused step's access pattern (hand-written
    gfx950 kernels of libqsdp_bench.so: 16-byte non-temporal accesses, a contiguous 4 KiB tile per wave and operand),
    next to the runtime's own device-to-device copy: the ceilings the fused step's HBM fraction is to be read against.
    The read-read-write kernel x <- x - lr*g moves the fused step's 12 bytes per element with one fma per element."""
    from paper_2302_02390_amd import bench_support as bs
    m = n // bs.TILE * bs.TILE
    xa, ga = x[:m].clone(), g[:m]
    y = torch.empty_like(xa)
    sink = torch.zeros(4, dtype=torch.float32, device=x.device)
    codes = torch.empty(m // 4, dtype=torch.int32, device=x.device)
    mo, vo = torch.zeros_like(xa), torch.zeros_like(xa)
    kernels = (("read_only", lambda i: bs.read(xa, sink), 4.0), ("write_only", lambda i: bs.fill(y, 0.5), 4.0),
               ("copy", lambda i: bs.copy(xa, y), 8.0), ("rrw", lambda i: bs.axpy(xa, ga, lr), 12.0),
               ("rrw_5_workgroups_per_cu", lambda i: bs.axpy(xa, ga, lr, 27000), 12.0),
               ("rrw_3_workgroups_per_cu", lambda i: bs.axpy(xa, ga, lr, 50000), 12.0),
               ("encode_4bit_mix", lambda i: bs.encode(xa, 4, codes), 4.5),
               ("encode_8bit_mix", lambda i: bs.encode(xa, 8, codes), 5.0),
               ("adamw_mix", lambda i: bs.moments(xa, ga, mo, vo, lr, 0.5), 28.0),
               ("adamw_mix_2_workgroups_per_cu", lambda i: bs.moments(xa, ga, mo, vo, lr, 0.5, 60000), 28.0),
               ("runtime_device_copy", lambda i: y.copy_(xa), 8.0))
    res = {"kernels": "float4 non-temporal streaming kernels, 4 KiB per wave and operand; rrw = x <- x - lr*g "
                      "(2 reads : 1 write, the fused step's mix; also launched with the workgroups per compute unit "
                      "capped the way the fused step is, the best of the three is the ceiling); encode_Nbit_mix = read 4 B, write N/8 B per "
                      "element (the encoders' mix); adamw_mix = 4 operands read, 3 written (the AdamW step's 28 B per element, also "
                      "with that step's residency cap)", "elements": m}
    for name, fn, bpe in kernels:
        for i in range(3):
            fn(i)
        mean, _ = time_call(fn, 10, torch)
        res[f"{name}_GB/s"] = round(bpe * m / (mean * 1e-3) / 1e9, 1)
        res[f"{name}_ms"] = round(mean, 4)
    res["rrw_best_GB/s"] = max(res["rrw_GB/s"], res["rrw_5_workgroups_per_cu_GB/s"], res["rrw_3_workgroups_per_cu_GB/s"])
    res["fused_step_vs_rrw"] = round(fused_achieved / res["rrw_best_GB/s"], 3)
    res["fused_step_vs_read_only"] = round(fused_achieved / res["read_only_GB/s"], 3)
    res["fused_step_vs_runtime_device_copy"] = round(fused_achieved / res["runtime_device_copy_GB/s"], 3)
    return res


def levels_report(torch, qb, x, g, n, workload, bucket, dev):
    """Learned (non-uniform) levels against the uniform table: relative L2 error |decode(encode(v)) - v| / |v| of
    the deterministic nearest-level codec on the weights and on the gradients, levels fitted on the first 4096
    buckets (rate 0.01, one pass), codec applied to the whole vector. The norms are torch reductions (measurement
    only)."""
    rows = []
    fit_buckets = 4096
    out = torch.empty(n, dtype=torch.float32, device=dev)
    for name, v in (("weights", x), ("gradients", g)):
        vnorm = float(torch.linalg.vector_norm(v.double()))
        for bits in (2, 3, 4, 5, 6):
            codes, meta = qb.alloc_packed(n, bits, bucket, dev)
            meta = meta.reshape(-1)
            uniform = qb.levels_uniform(bits, dev)
            fitted = uniform.clone()
            fit_ms, _ = time_call(lambda i: qb.qsdp_fit_levels(v, bits, bucket, 0.01, fitted, fit_buckets), 1, torch)
            row = {"tensor": name, "bits": bits, "fit_ms": round(fit_ms, 3), "fit_batches": fit_buckets}
            for label, table in (("uniform", uniform), ("fitted", fitted)):
                # untimed first calls: enough of them for the clocks to recover from the fit (one workgroup
                # running alone for 10 ms leaves the chip nearly idle, and the next kernels run slow for a while)
                for _ in range(8):
                    qb.qsdp_quantize_levels(v, bits, bucket, table, codes, meta)
                qb.qsdp_dequantize_levels(codes, meta, n, bits, bucket, table, out)
                _, enc_ms = time_call(lambda i: qb.qsdp_quantize_levels(v, bits, bucket, table, codes, meta), 9, torch)
                _, dec_ms = time_call(lambda i: qb.qsdp_dequantize_levels(codes, meta, n, bits, bucket, table, out), 9,
                                      torch)  # medians
                err = float(torch.linalg.vector_norm((out - v).double())) / vnorm
                # the quantity the fit minimises: rms error in bucket-normalised coordinates (full buckets only)
                nbf = n // bucket
                rng = meta.view(-1, 2)[:nbf, 1].double().clamp_min(1e-30)
                zerr = ((out[:nbf * bucket] - v[:nbf * bucket]).view(nbf, bucket).double() / rng[:, None])
                row[label] = {"rel_l2_error": round(err, 6), "normalised_rms_error": round(float(zerr.pow(2).mean().sqrt()), 6),
                              "encode_ms": round(enc_ms, 4), "decode_ms": round(dec_ms, 4)}
                del zerr
            row["error_ratio_fitted_over_uniform"] = round(row["fitted"]["rel_l2_error"] / row["uniform"]["rel_l2_error"], 4)
            rows.append(row)
            del codes, meta
    return {"metric": "relative L2 compression error, uniform vs fitted levels", "workload": workload, "n": n,
            "bucket": bucket, "data": "synthetic", "levels": rows}


def levels_per_layer(torch, qb, wl, x, g, shape, bucket, dev):
    """The learned-level pipeline the way Section 5.2 / Appendix C run it: every layer tensor of the model has a
    table of its own, fitted on that tensor (tensors of at most 1e5 elements keep the uniform table); W5 for the
    weights, G4 with the unbiased coin flip for the gradients; fit, encode and decode are one launch each over
    all tensors."""
    sizes = [size for _, size in wl.model_tensors(shape)]
    n = sum(sizes)
    segs = qb.Segments(sizes, bucket, dev)
    small = torch.tensor([s <= 100000 for s in sizes], device=dev)
    out = torch.empty(n, dtype=torch.bfloat16, device=dev)
    res = {"tensors": len(sizes), "tensors_with_fitted_table": int((~small).sum()), "fit_batches_per_tensor": 1024}
    for name, v, bits, coin in (("weights_W5", x, 5, False), ("gradients_G4", g, 4, True)):
        uniform = qb.levels_uniform(bits, dev)
        tables = uniform.repeat(len(sizes), 1).contiguous()
        fit_ms, _ = time_call(lambda i: qb.qsdp_fit_levels_segmented(v, segs, bits, 0.01, tables, 1024), 1, torch)
        tables[small] = uniform
        codes, meta = segs.alloc_packed(bits)
        meta = meta.reshape(-1)
        for _ in range(8):                                                                      # untimed first calls
            qb.qsdp_quantize_levels_segmented(v, segs, bits, tables, codes, meta, coin, 0, 0)
        qb.qsdp_dequantize_levels_segmented(codes, meta, segs, bits, tables, out)
        _, enc_ms = time_call(lambda i: qb.qsdp_quantize_levels_segmented(v, segs, bits, tables, codes, meta, coin, i, 0),
                              9, torch)
        _, dec_ms = time_call(lambda i: qb.qsdp_dequantize_levels_segmented(codes, meta, segs, bits, tables, out), 9,
                              torch)  # medians
        res[name] = {"fit_ms": round(fit_ms, 3), "encode_ms": round(enc_ms, 4), "decode_bf16_ms": round(dec_ms, 4),
                     "encode_GB/s": round((4 + bits / 8 + 8 / bucket) * n / enc_ms / 1e6, 1),
                     "decode_GB/s": round((2 + bits / 8 + 8 / bucket) * n / dec_ms / 1e6, 1),
                     "rounding": "coin flip between the enclosing levels" if coin else "nearest level"}
        del codes, meta
    return res


def sweep(torch, qb, wl, x, g, n, workload, dev):
    """Fused step over gradient bits x weight bits x bucket, the explicit-delta pairings, the
    quantizers, and the decode of the transformer blocks to bf16 one by one (median of 10 calls)."""
    def med(fn, iters=10):
        for i in range(2):
            fn(i)
        return time_call(fn, iters, torch)[1]

    rows = []
    for B in (128, 512, 1024, 4096):
        for gb in (2, 3, 4, 6, 8):
            for wb in (4, 6, 8):
                t = med(lambda i: qb.qsdp_fused_step(x, g, 1e-3, wb, gb, B, 0.0, i))
                rows.append({"call": "fused_step", "bucket": B, "gbits": gb, "wbits": wb, "ms": round(t, 4),
                             "GB/s": round(12.0 * n / t / 1e6, 1)})
    for d, wb in ((2.0 ** -6, 4), (2.0 ** -8, 6), (2.0 ** -10, 8)):
        sat = torch.zeros(1, dtype=torch.int64, device=dev)
        t = med(lambda i: qb.qsdp_fused_step(x, g, 1e-3, wb, 4, 1024, d, i, 0, None, None, sat))
        rows.append({"call": "fused_step", "bucket": 1024, "gbits": 4, "wbits": wb, "delta": d, "ms": round(t, 4),
                     "GB/s": round(12.0 * n / t / 1e6, 1), "saturated_per_call": int(sat) // 12})
    for B in (128, 1024, 4096):
        for b in (2, 3, 4, 6, 8):
            c, m = qb.alloc_packed(n, b, B, dev)
            bp = 4 + b / 8.0 + 8.0 / B
            t = med(lambda i: qb.qsdp_quantize_grad(g, b, B, i, 0, c, m.reshape(-1)))
            rows.append({"call": "quantize_grad", "bucket": B, "bits": b, "ms": round(t, 4),
                         "GB/s": round(bp * n / t / 1e6, 1)})
            t = med(lambda i: qb.qsdp_quantize_weight(x, b, B, 0.0, i, c, m.reshape(-1)))
            rows.append({"call": "quantize_weight", "bucket": B, "bits": b, "ms": round(t, 4),
                         "GB/s": round(bp * n / t / 1e6, 1)})
            del c, m
    layer = None
    if workload != "1m":
        shape = {"gpt-1.3b": wl.GPT_1P3B, "gpt-350m": wl.GPT_350M, "gpt-125m": wl.GPT_125M}[workload]
        blk = wl.block_numel(shape.d)
        start = (wl.VOCAB + wl.N_CTX) * shape.d
        out = torch.empty(blk, dtype=torch.bfloat16, device=dev)
        packed = []
        for layer_id in range(shape.layers):
            c, m = qb.alloc_packed(blk, 8, 1024, dev)
            qb.qsdp_quantize_weight(x[start + layer_id * blk: start + (layer_id + 1) * blk], 8, 1024, 0.0, layer_id, c,
                                    m.reshape(-1))
            packed.append((c, m.reshape(-1)))

        def all_layers(i):
            for c, m in packed:
                qb.qsdp_dequantize(c, m, blk, 8, 1024, out)

        t_all = med(all_layers, 5)
        t_one = med(lambda i: qb.qsdp_dequantize(packed[0][0], packed[0][1], blk, 8, 1024, out))
        bp = 2 + 1 + 8.0 / 1024
        layer = {"block_elements": blk, "layers": shape.layers, "ms_one_block": round(t_one, 4),
                 "GB/s_one_block": round(bp * blk / t_one / 1e6, 1), "ms_all_blocks": round(t_all, 4),
                 "GB/s_all_blocks": round(bp * blk * shape.layers / t_all / 1e6, 1)}
    return {"metric": "sweep of the codec entry points (algorithmic GB/s)", "workload": workload, "n": n,
            "data": "synthetic", "sweep": rows, "layerwise_dequantize_to_bf16": layer}


def segmented_extras(torch, qb, x, n, segs, wbits, bucket, dev):
    """Encode and decode of all layer tensors in one segmented launch each (algorithmic GB/s over
    the n real elements; the padding slots of short tensors are not counted)."""
    res = {}
    meta_b = 8.0 / bucket
    wc, wm = segs.alloc_packed(wbits)
    wm = wm.reshape(-1)
    out16 = torch.empty(n, dtype=torch.bfloat16, device=dev)
    out32 = torch.empty(n, dtype=torch.float32, device=dev)
    for name, fn, bpp in (
            (f"quantize_weight_segmented_b{wbits}",
             lambda i: qb.qsdp_quantize_weight_segmented(x, segs, wbits, 0.0, i, wc, wm), 4 + wbits / 8.0 + meta_b),
            (f"dequantize_segmented_b{wbits}_bf16",
             lambda i: qb.qsdp_dequantize_segmented(wc, wm, segs, wbits, out16), 2 + wbits / 8.0 + meta_b),
            (f"dequantize_segmented_b{wbits}_f32",
             lambda i: qb.qsdp_dequantize_segmented(wc, wm, segs, wbits, out32), 4 + wbits / 8.0 + meta_b)):
        for i in range(3):
            fn(i)
        mean, _ = time_call(fn, 10, torch)
        res[name] = {"ms": round(mean, 4), "GB/s": round(bpp * n / (mean * 1e-3) / 1e9, 1),
                     "bytes_per_param": round(bpp, 4), "tensors": segs.nseg}
    return res


def extras(torch, qb, x, g, n, wbits, gbits, bucket, dev):
    """Algorithmic GB/s of the other entry points on the same tensors (not part of `value`)."""
    res = {}
    meta_b = 8.0 / bucket
    gc, gm = qb.alloc_packed(n, gbits, bucket, dev)
    wc, wm = qb.alloc_packed(n, wbits, bucket, dev)
    gm, wm = gm.reshape(-1), wm.reshape(-1)

    def run(name, fn, bytes_per_param):
        for i in range(3):
            fn(i)
        mean, median = time_call(fn, 10, torch)
        res[name] = {"ms": round(mean, 4), "GB/s": round(bytes_per_param * n / (mean * 1e-3) / 1e9, 1),
                     "bytes_per_param": round(bytes_per_param, 4)}

    run(f"quantize_grad_b{gbits}", lambda i: qb.qsdp_quantize_grad(g, gbits, bucket, i, 0, gc, gm),
        4 + gbits / 8.0 + meta_b)
    run(f"quantize_weight_b{wbits}", lambda i: qb.qsdp_quantize_weight(x, wbits, bucket, 0.0, i, wc, wm),
        4 + wbits / 8.0 + meta_b)
    out32 = torch.empty(n, dtype=torch.float32, device=dev)
    run(f"dequantize_b{wbits}_f32", lambda i: qb.qsdp_dequantize(wc, wm, n, wbits, bucket, out32),
        4 + wbits / 8.0 + meta_b)
    del out32
    out16 = torch.empty(n, dtype=torch.bfloat16, device=dev)
    run(f"dequantize_b{wbits}_bf16", lambda i: qb.qsdp_dequantize(wc, wm, n, wbits, bucket, out16),
        2 + wbits / 8.0 + meta_b)
    run(f"dequantize_b{gbits}_bf16", lambda i: qb.qsdp_dequantize(gc, gm, n, gbits, bucket, out16),
        2 + gbits / 8.0 + meta_b)
    del out16
    outh = torch.empty(n, dtype=torch.float16, device=dev)
    run(f"dequantize_b{wbits}_f16", lambda i: qb.qsdp_dequantize(wc, wm, n, wbits, bucket, outh),
        2 + wbits / 8.0 + meta_b)
    del outh
    # learned levels at 4 bits (table fitted on the first 2048 buckets): nearest-level and coin-flip encoders
    lv = qb.levels_uniform(4, dev)
    qb.qsdp_fit_levels(x, 4, bucket, 0.01, lv, 2048)
    lc, lm = qb.alloc_packed(n, 4, bucket, dev)
    lm = lm.reshape(-1)
    for _ in range(8):  # untimed: the fit (one workgroup for some ms) left the chip nearly idle, let the clocks recover
        qb.qsdp_quantize_levels(x, 4, bucket, lv, lc, lm)
    run("quantize_levels_b4_fitted_table", lambda i: qb.qsdp_quantize_levels(x, 4, bucket, lv, lc, lm), 4.5 + meta_b)
    run("quantize_levels_stochastic_b4_fitted_table",
        lambda i: qb.qsdp_quantize_levels_stochastic(g, 4, bucket, lv, i, 0, lc, lm), 4.5 + meta_b)
    del lc, lm
    # the fused step with x resident as codes (wc, wm hold Q^w(x) from the call above)
    run(f"fused_step_codes_W{wbits}G{gbits}",
        lambda i: qb.qsdp_fused_step_codes(wc, wm, g, 1e-3, wbits, gbits, bucket, 0.0, i),
        4 + 2 * (wbits / 8.0 + meta_b))
    run(f"fused_step_codes_W{wbits}G{gbits}_shared_shift_gradients",
        lambda i: qb.qsdp_fused_step_codes(wc, wm, g, 1e-3, wbits, gbits, bucket, 0.0, i, 0, None,
                                           qb.QSDP_FLAG_GRAD_SHIFT), 4 + 2 * (wbits / 8.0 + meta_b))
    # gradients handed over in 16 bits (widened exactly on load): 2 bytes of gradient traffic per parameter
    for name, dt in (("f16", torch.float16), ("bf16", torch.bfloat16)):
        g16 = g.to(dt)
        run(f"quantize_grad_b{gbits}_{name}_gradient",
            lambda i: qb.qsdp_quantize_grad_g16(g16, gbits, bucket, i, 0, gc, gm), 2 + gbits / 8.0 + meta_b)
        xh = x.clone()
        run(f"fused_step_W{wbits}G{gbits}_{name}_gradient",
            lambda i: qb.qsdp_fused_step_g16(xh, g16, 1e-3, wbits, gbits, bucket, 0.0, i), 10.0)
        if name == "bf16":
            # ... and the new weights written once more as bf16 for the next forward pass
            x16 = torch.empty(n, dtype=dt, device=dev)
            run(f"fused_step_mp_W{wbits}G{gbits}_bf16_gradient_bf16_weights_out",
                lambda i: qb.qsdp_fused_step_mp(xh, g16, 1e-3, wbits, gbits, bucket, 0.0, i, x16=x16), 12.0)
            del x16
        del g16, xh
    # AdamW between the quantizers (moments in fp32): read x, g, m, v; write x, m, v
    mom = torch.zeros(n, dtype=torch.float32, device=dev)
    var = torch.zeros(n, dtype=torch.float32, device=dev)
    xa = x.clone()
    run(f"fused_adamw_step_W{wbits}G{gbits}",
        lambda i: qb.qsdp_fused_adamw_step(xa, g, mom, var, 2e-4, 0.9, 0.95, 1e-8, 0.0, 1 - 0.9 ** (i + 1),
                                           1 - 0.95 ** (i + 1), wbits, gbits, bucket, 0.0, i), 28.0)
    # ... as a mixed-precision training step: bf16 gradient in (2 B), bf16 copy of the new weights out (2 B)
    g16 = g.to(torch.bfloat16)
    x16 = torch.empty(n, dtype=torch.bfloat16, device=dev)
    run(f"fused_adamw_step_mp_W{wbits}G{gbits}_bf16_gradient_bf16_weights_out",
        lambda i: qb.qsdp_fused_adamw_step_mp(xa, g16, mom, var, 2e-4, 0.9, 0.95, 1e-8, 0.0, 1 - 0.9 ** (i + 1),
                                              1 - 0.95 ** (i + 1), wbits, gbits, bucket, 0.0, i, x16=x16), 28.0)
    del g16, x16
    # the same with the weights resident as codes: read codes, g, m, v; write codes, m, v
    qb.qsdp_quantize_weight(x, wbits, bucket, 0.0, 5, wc, wm)
    run(f"fused_adamw_step_codes_W{wbits}G{gbits}",
        lambda i: qb.qsdp_fused_adamw_step_codes(wc, wm, g, mom, var, 2e-4, 0.9, 0.95, 1e-8, 0.0, 1 - 0.9 ** (i + 1),
                                                 1 - 0.95 ** (i + 1), wbits, gbits, bucket, 0.0, i),
        20 + 2 * (wbits / 8.0 + meta_b))
    del mom, var, xa
    # decode-and-sum of 8 peers' gradient slices on one GPU's 1/8 shard (the receive side of the
    # quantized gradient exchange): the 8 slices are 8 quantizations of the shard with different seeds
    peers = 8
    m = (n // peers) // bucket * bucket
    nbm = m // bucket
    pc = torch.empty((peers, nbm * bucket * gbits // 32), dtype=torch.int32, device=dev)
    pm = torch.empty((peers, (nbm * 2 + 3) // 4 * 4), dtype=torch.float32, device=dev)  # rows stay 16-byte aligned
    for p in range(peers):
        qb.qsdp_quantize_grad(g[:m], gbits, bucket, 100 + p, 0, pc[p], pm[p])
    acc = torch.empty(m, dtype=torch.float32, device=dev)
    n_saved, n = n, m

    def run_small(name, fn, bytes_per_param):
        for i in range(3):
            fn(i)
        mean, _ = time_call(fn, 10, torch)
        res[name] = {"ms": round(mean, 4), "GB/s": round(bytes_per_param * m / (mean * 1e-3) / 1e9, 1),
                     "bytes_per_param": round(bytes_per_param, 4), "n": m}

    run_small(f"dequantize_add_{peers}peers_b{gbits}",
              lambda i: qb.qsdp_dequantize_add(pc, pm, peers, m, gbits, bucket, 1.0 / peers, acc),
              peers * (gbits / 8.0 + meta_b) + 4)
    # the same receive side fused with the update and Q^w (codes of the new weights emitted)
    xs = x[:m].clone()
    sc, sm = qb.alloc_packed(m, wbits, bucket, dev)
    run_small(f"recv_step_{peers}peers_W{wbits}G{gbits}",
              lambda i: qb.qsdp_recv_step(xs, pc, pm, peers, 1.0 / peers, 1e-3, wbits, gbits, bucket, 0.0, i, 0,
                                          sc, sm.reshape(-1)),
              8 + peers * (gbits / 8.0 + meta_b) + wbits / 8.0 + meta_b)
    # ... and with AdamW on the full-precision partition (Algorithm 2's weight update as the experiments run it)
    mom = torch.zeros(m, dtype=torch.float32, device=dev)
    var = torch.zeros(m, dtype=torch.float32, device=dev)
    run_small(f"recv_adamw_step_{peers}peers_W{wbits}G{gbits}_keep_master",
              lambda i: qb.qsdp_recv_adamw_step(xs, mom, var, pc, pm, peers, 1.0 / peers, 2e-4, 0.9, 0.95, 1e-8, 0.0,
                                                1 - 0.9 ** (i + 1), 1 - 0.95 ** (i + 1), wbits, gbits, bucket, 0.0, i,
                                                qb.QSDP_FLAG_KEEP_MASTER, sc, sm.reshape(-1)),
              24 + peers * (gbits / 8.0 + meta_b) + wbits / 8.0 + meta_b)
    del xs, sc, sm, mom, var
    n = n_saved
    del pc, pm, acc
    # decode of a gathered layer: the vector as 8 peers' weight shards, each quantized on its own, one
    # slot [codes | meta] per peer in a single receive buffer, decoded to bf16 in one launch
    shard = -(-(n // peers) // bucket) * bucket
    npeers = -(-n // shard)
    cw = shard * wbits // 32
    mw = (2 * (shard // bucket) + 3) // 4 * 4
    recv = torch.empty((npeers, cw + mw), dtype=torch.int32, device=dev)
    slot_codes, slot_meta = recv[:, :cw], recv.view(torch.float32)[:, cw:]
    for p in range(npeers):
        xs = x[p * shard:min((p + 1) * shard, n)]
        mlen = 2 * (-(-xs.numel() // bucket))
        qb.qsdp_quantize_weight(xs, wbits, bucket, 0.0, 7, slot_codes[p], slot_meta[p, :mlen])
    out16 = torch.empty(n, dtype=torch.bfloat16, device=dev)
    run(f"dequantize_gathered_{npeers}slots_b{wbits}_bf16",
        lambda i: qb.qsdp_dequantize_gathered(slot_codes, slot_meta, npeers, n, shard, wbits, bucket, out16),
        2 + wbits / 8.0 + meta_b)
    return res


def cpu_baseline(x0, g, sample, single_sample, lr, wbits, gbits, bucket, delta, bytes_per_param):
    """The CPU oracle, as it stands, on the same tensors: one fused step (seed 0) from x0, by default over the whole
    vector, once with the bucket-parallel loop on the host's cores and once on a single thread."""
    from oracle import ref
    threads = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16")), 16)
    n = x0.numel()
    m = n if sample <= 0 else max(bucket, min(n, sample) // bucket * bucket)
    m1 = n if single_sample <= 0 else max(bucket, min(n, single_sample) // bucket * bucket)
    big = max(m, m1)
    xs = x0[:big].cpu().numpy()
    gs = g[:big].cpu().numpy()
    work = xs[:m].copy()
    ref.set_threads(threads)
    t0 = time.perf_counter()
    ref.fused_step_inplace(work, gs[:m], lr, wbits, gbits, bucket, delta, 0)
    dt = time.perf_counter() - t0
    ref.set_threads(1)
    work = xs[:m1].copy()
    t0 = time.perf_counter()
    ref.fused_step_inplace(work, gs[:m1], lr, wbits, gbits, bucket, delta, 0)
    dt1 = time.perf_counter() - t0

    def what(k):
        return "one whole fused step (seed 0) of the same workload" if k == n else \
            f"one fused step (seed 0) on the first {k} elements of the same x and g"

    return {"value": round(bytes_per_param * m / dt / 1e9, 3), "unit": "GB/s", "cores": threads,
            "kind": "oracle", "params_per_s": round(m / dt, 1), "seconds": round(dt, 3),
            "sample": f"{what(m)}, bucket-parallel oracle on {threads} threads",
            "single_thread": {"value": round(bytes_per_param * m1 / dt1 / 1e9, 3), "unit": "GB/s", "cores": 1,
                              "params_per_s": round(m1 / dt1, 1), "seconds": round(dt1, 3),
                              "sample": f"{what(m1)}, the same oracle on one thread"}}


if __name__ == "__main__":
    sys.exit(main())
