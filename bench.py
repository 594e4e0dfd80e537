#!/usr/bin/env python3
"""Benchmark of the attention-carving hot path on one MI355X.

One "step" is one pass of the whole path over one synthetic layer input:
    3 x jenga_curve_permute (Q, K, V)  ->  jenga_select_blocks  ->  jenga_block_sparse_attn
    ->  jenga_unpermute
with Q/K/V already resident in HBM.  The headline value is the time of what recurs per layer
(select + attention); the permutes, which the paper pays once per DiT forward, are reported beside
it.  Prints ONE JSON line.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0


def cpu_baseline(w, q, k, v, seconds_budget=20.0):
    """The CPU oracle as it stands, timed on a bounded sample of the same workload."""
    import numpy as np
    import jenga_inputs as ji
    from oracle import jenga_oracle as jo
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    t_all = time.time()
    lay = jo.Layout(w["T"], w["H"], w["W"], w["n_text"], w["block"], w["topk"])
    t_plan = time.time() - t_all
    heads = w["heads"]
    h = 0
    qs, ks, vs = [jo.permute(jo.bf16_bits_to_f64(ji.bits(x[:, :, h:h + 1, :])), lay) for x in (q, k, v)]
    t0 = time.time()
    mask = jo.build_mask(qs, ks, lay, w["p"])
    t_select_head = time.time() - t0
    rng = np.random.default_rng(0)
    order = rng.permutation(lay.M_v)
    n_blocks, t0 = 0, time.time()
    for i in order:
        jo.attention_block(qs[0, 0], ks[0, 0], vs[0, 0], mask[0, 0, i], lay, int(i))
        n_blocks += 1
        if time.time() - t0 > seconds_budget:
            break
    t_attn = time.time() - t0
    mean_sel = float(mask[0, 0, : lay.M_v].sum(-1).mean())
    # extrapolate to the full layer: every head, every vision block at the sampled cost per block,
    # text blocks at the dense cost (M / mean_sel times a sampled block)
    per_block = t_attn / n_blocks
    layer_s = heads * w["batch"] * (t_select_head + per_block * (lay.M_v + lay.M_c * lay.M / mean_sel))
    return {"value": layer_s * 1e3, "unit": "ms per layer (extrapolated)", "cores": cores, "kind": "oracle",
            "sample": "head 0: masks of all %d query blocks (%.2f s) + attention of %d random vision query blocks "
                      "(%.2f s); scaled to %d heads x %d blocks; plan %.2f s not included"
                      % (lay.M_v, t_select_head, n_blocks, t_attn, heads, lay.M, t_plan),
            "measured_s": t_select_head + t_attn}


class Telemetry:
    """Samples the package power and the shader clocks with `amd-smi metric -p -c` (read-only) in a thread while
    a block of work runs; reports what the part held under that load.  Absent tool or parse failure: None."""

    def __init__(self, period=0.25):
        import threading
        self.period, self.samples, self._stop = period, [], False
        self._thread = threading.Thread(target=self._run, daemon=True)

    def _run(self):
        import subprocess
        while not self._stop:
            try:
                r = subprocess.run(["amd-smi", "metric", "-p", "-c"], capture_output=True, text=True, timeout=10)
                power, clocks, in_gfx = None, [], False
                for line in r.stdout.splitlines():
                    t = line.strip()
                    if t.startswith("SOCKET_POWER"):
                        power = float(t.split(":")[1].split()[0])
                    elif t.startswith("GFX_"):
                        in_gfx = True
                    elif in_gfx and t.startswith("CLK:"):
                        clocks.append(float(t.split(":")[1].split()[0]))
                        in_gfx = False
                if power is not None and clocks:
                    self.samples.append((time.time(), power, sum(clocks) / len(clocks)))
            except Exception:
                return
            time.sleep(self.period)

    def __enter__(self):
        self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop = True
        self._thread.join(timeout=15)

    def summary(self, t_from, t_to):
        inside = [(p, c) for (t, p, c) in self.samples if t_from <= t <= t_to]
        if not inside:
            return None
        return {"samples": len(inside), "socket_power_w": sum(p for p, _ in inside) / len(inside),
                "gfx_clock_mhz": sum(c for _, c in inside) / len(inside)}


def attention_under_load(layer, seconds=4.0):
    """Runs the attention kernel back to back for about `seconds` and samples power and clock meanwhile: the
    clock the part holds under this kernel (it runs at the package power limit) is what the percentage of the
    nominal peak has to be read against."""
    import torch
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    layer.attend_packed()
    b.record()
    torch.cuda.synchronize()
    reps = max(4, int(seconds * 1e3 / max(a.elapsed_time(b), 1e-3)))
    with Telemetry() as tel:
        time.sleep(0.3)
        t0 = time.time()
        a.record()
        for _ in range(reps):
            layer.attend_packed()
        b.record()
        torch.cuda.synchronize()
        t1 = time.time()
    out = tel.summary(t0 + 1.0, t1)      # skip the ramp at the start
    if out is not None:
        out["attn_ms_back_to_back"] = a.elapsed_time(b) / reps
    return out


def stage_switch_bench(dev, reps=20):
    """The resolution switch between stages (Eq. 4) at the 540p -> 720p latent shape: HBM-bound, beside the layer."""
    import torch
    import jenga_inputs as ji
    from paper_2505_16864_amd import binding as jb
    w = ji.STAGE_SWITCHES["hy540to720"]
    x, e, n = ji.make_latents(w, 7030, device=dev)
    out = torch.empty_like(n)
    stream = torch.cuda.current_stream().cuda_stream
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for it in range(2):
        a.record()
        for _ in range(reps):
            jb.jenga_stage_switch(x, e, n, out, w["channels"], w["in"], w["out"], w["sigma"], stream)
        b.record()
        torch.cuda.synchronize()
    ms = a.elapsed_time(b) / reps
    nbytes = 4.0 * (2 * x.numel() + 2 * n.numel())
    return {"workload": "hy540to720", "ms": ms, "algorithmic_bytes": nbytes, "gbs": nbytes / (ms * 1e-3) / 1e9,
            "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS}


def sustained_mfma_tflops(dev, seconds=0.15):
    """What the matrix cores sustain on random bf16 operands under the power limit (MFMA-only loop)."""
    import ctypes
    import torch
    lib_path = os.path.join(ROOT, "bench_mfma_probe.so")
    if not os.path.exists(lib_path):
        return None
    probe = ctypes.CDLL(lib_path).bench_mfma_probe
    probe.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32,
                      ctypes.c_int32, ctypes.c_void_p]
    probe.restype = ctypes.c_int
    g = torch.Generator().manual_seed(99)
    ops = torch.randn(65536, generator=g, dtype=torch.float32).to(torch.bfloat16).to(dev)
    n_wg = 2 * torch.cuda.get_device_properties(0).multi_processor_count     # two waves per SIMD
    sink = torch.empty(n_wg * 256, device=dev, dtype=torch.float32)
    stream = torch.cuda.current_stream().cuda_stream
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    iters, rate = 20000, 0.0
    for _ in range(3):            # calibrate the length, then measure a run of about `seconds`
        a.record()
        if probe(ops.data_ptr(), ops.numel() * 2, sink.data_ptr(), sink.numel(), iters, n_wg, stream) != 0:
            return None
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b)
        rate = n_wg * 4 * iters * 4 * 32768.0 / (ms * 1e-3) / 1e12
        iters = max(2, int(iters * seconds * 1e3 / ms) // 2 * 2)
    return rate


def valu_under_mfma(dev):
    """ns per MFMA and SIMD of a loop of MFMAs with a fixed group of vector ALU instructions after each of them,
    at one to four wavefronts per SIMD (bench_mfma_probe.so: bench_valu_under_mfma)."""
    import ctypes
    import torch
    lib_path = os.path.join(ROOT, "bench_mfma_probe.so")
    if not os.path.exists(lib_path):
        sys.exit("bench.py: bench_mfma_probe.so is not built")
    probe = ctypes.CDLL(lib_path).bench_valu_under_mfma
    probe.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
    probe.restype = ctypes.c_int
    kinds = ["mfma only", "attention step per mfma: exp, fma, add, half a bf16 pack", "the same plus half a v_max3",
             "4 v_add_f32 per mfma", "5 v_add_f32 per mfma", "6 v_add_f32 per mfma"]
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    stream = torch.cuda.current_stream().cuda_stream
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    iters = 40000
    table = {}
    for kind, name in enumerate(kinds):
        row = {}
        for waves in (1, 2, 4):                 # one workgroup of four wavefronts per CU and per wave of a SIMD
            n_wg = n_cu * waves
            sink = torch.empty(n_wg * 256, device=dev, dtype=torch.float32)
            for timed in (False, True):
                a.record()
                if probe(kind, sink.data_ptr(), sink.numel(), iters if timed else 2000, n_wg, stream) != 0:
                    sys.exit("bench.py: bench_valu_under_mfma failed")
                b.record()
                torch.cuda.synchronize()
            row["%d_waves_per_simd" % waves] = round(a.elapsed_time(b) * 1e6 / (iters * 4 * waves), 2)
        table[name] = row
    return {"unit": "ns per MFMA and SIMD", "mfma": "v_mfma_f32_32x32x16_bf16", "iters": iters, "table": table}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="hy720p")
    ap.add_argument("--seed", type=int, default=5000)
    ap.add_argument("--walk", choices=["paced", "ordered"], default="paced",
                    help="order in which the attention kernel visits the selected blocks: paced by a chip-wide clock "
                         "(library flag JENGA_FLAG_PACED_WALK, the faster one) or in list order (bit-reproducible)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-telemetry", action="store_true", help="skip the power/clock sampling run")
    ap.add_argument("--zero-operands", action="store_true",
                    help="attribution run: the lists are selected on the real inputs, then Q, K, V are zeroed before "
                         "the attention is timed (same work, no data-dependent switching power)")
    ap.add_argument("--valu-under-mfma", action="store_true",
                    help="microbenchmark only: how many vector ALU instructions fit beside an MFMA on this part "
                         "(prints its own JSON line and exits)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build targets one GPU; run with --gpus 1 (no multi-GPU path exists)")

    import torch
    if args.valu_under_mfma:
        if not torch.cuda.is_available():
            sys.exit("bench.py: needs a GPU")
        print(json.dumps({"microbenchmark": "valu_under_mfma", **valu_under_mfma("cuda:0")}))
        return
    import jenga_inputs as ji
    from paper_2505_16864_amd import binding as B
    from paper_2505_16864_amd.layer import CarveLayer

    if not torch.cuda.is_available():
        sys.exit("bench.py: needs a GPU")
    w = ji.WORKLOADS[args.workload]
    dev = "cuda:0"
    q, k, v = ji.make_qkv(w, args.seed, device=dev)
    flags = (w.get("flags", 7) & 7) | (8 if args.walk == "paced" else 0)
    layer = CarveLayer(w, dev, flags=flags)
    info = layer.info

    def ev():
        return torch.cuda.Event(enable_timing=True)

    names = ["permute_in", "select", "pack", "attn", "permute_out"]
    acc = {n: 0.0 for n in names}
    samples = {n: [] for n in names}
    total_ms = 0.0
    for it in range(args.warmup + args.steps):
        marks = [ev() for _ in range(6)]
        torch.cuda.synchronize()
        marks[0].record()
        layer.permute_in(q, k, v)
        marks[1].record()
        layer.select()
        marks[2].record()
        if args.zero_operands:
            layer.q_c.zero_()
            layer.k_c.zero_()
            layer.v_c.zero_()
            torch.cuda.synchronize()
            marks[2].record()
        layer.pack()
        marks[3].record()
        layer.attend_packed()
        marks[4].record()
        layer.permute_out()
        marks[5].record()
        torch.cuda.synchronize()
        if it >= args.warmup:
            for n, a, b in zip(names, marks[:-1], marks[1:]):
                t = a.elapsed_time(b)
                acc[n] += t
                samples[n].append(t)
            total_ms += marks[0].elapsed_time(marks[5])
    ms = {n: acc[n] / args.steps for n in names}
    ms_step = total_ms / args.steps
    layer_ms = ms["select"] + ms["pack"] + ms["attn"]

    m, d, heads, batch = w["block"], w["head_dim"], w["heads"], w["batch"]
    sel_total = int(layer.sel_count.sum().item())
    executed_flop = 4.0 * m * m * d * sel_total              # QK^T and PV of every visited m x m tile
    dense_flop = 4.0 * float(info.N_pad) ** 2 * d * heads * batch
    density = sel_total / float(batch * heads * info.M * info.M)
    attn_tflops = executed_flop / (ms["attn"] * 1e-3) / 1e12
    tensor_bytes = 2.0 * (info.N_v + w["n_text"]) * heads * d * batch
    permute_gbs = 2 * tensor_bytes * 4 / ((ms["permute_in"] + ms["permute_out"]) * 1e-3) / 1e9

    # algorithmic bytes of the HBM-bound stages: pooling reads Q and K once, the index lists are written once;
    # packing reads K and V and writes both re-tiled
    n_pad_bytes = 2.0 * info.N_pad * heads * d * batch
    select_gbs = (2 * n_pad_bytes + 4.0 * sel_total) / (ms["select"] * 1e-3) / 1e9
    pack_gbs = 4 * n_pad_bytes / (ms["pack"] * 1e-3) / 1e9

    # HBM-side traffic of the attention kernel comes from rocprofv3 counters, which cannot be read from inside this
    # process: the figure of the committed profile of this workload is quoted, with its source
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "attn_kernel_%s_traffic.json" % args.workload)
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(args.walk, {}).get("hbm_bytes_per_launch")
        traffic_source = "profiles/" + os.path.basename(tpath) + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, not measured in this run)"

    out = {
        "metric": "ms per block-sparse attention layer (select + pack + attention)",
        "value": layer_ms, "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "grid": [w["T"], w["H"], w["W"]], "n_text": w["n_text"],
                   "heads": heads, "head_dim": d, "block": m, "topk": w["topk"], "p": w["p"],
                   "tokens_padded": info.N_pad, "blocks": info.M, "seed": args.seed, "walk": args.walk},
        "ms": ms,
        "ms_median": {n: sorted(samples[n])[len(samples[n]) // 2] for n in names},
        "ms_min": {n: min(samples[n]) for n in names},
        "executed_tflop": executed_flop / 1e12, "dense_equiv_tflop": dense_flop / 1e12,
        "executed_tflops": attn_tflops, "dense_equiv_tflops": dense_flop / (ms["attn"] * 1e-3) / 1e12,
        "layer_executed_tflops": executed_flop / (layer_ms * 1e-3) / 1e12,
        "density": density, "mean_selected_blocks": sel_total / float(batch * heads * info.M),
        "permute_gbs": permute_gbs, "select_gbs": select_gbs, "pack_gbs": pack_gbs,
        "roofline": {"kernel": "attn_h_kernel<128>" if m == 128 else "attn_kernel", "bound": "mfma", "achieved": attn_tflops, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": attn_tflops / PEAK_BF16_TFLOPS, "traffic": traffic,
                     "traffic_source": traffic_source},
    }
    sustained = sustained_mfma_tflops(dev)
    if sustained:
        out["roofline"]["mfma_only_random_operands_tflops"] = sustained
        out["roofline"]["frac_of_mfma_only"] = attn_tflops / sustained
    # the other walk of the same kernel on the same lists and tiles, for comparison (a few launches)
    other = CarveLayer(w, dev, flags=flags ^ 8)
    a, b = ev(), ev()
    times = []
    for _ in range(4):
        a.record()
        B.jenga_block_sparse_attn_packed(other.plan, layer.q_c, layer.ws_attn, layer.ws_attn.numel(), layer.sel_count,
                                         layer.sel_index, layer.o_c, None, torch.cuda.current_stream().cuda_stream)
        b.record()
        torch.cuda.synchronize()
        times.append(a.elapsed_time(b))
    out["attn_ms_other_walk"] = {"walk": "ordered" if args.walk == "paced" else "paced", "ms": sum(times[1:]) / 3}
    del other
    if args.zero_operands:
        out["data"] = "synthetic; lists from the real inputs, attention timed on all-zero Q, K, V (attribution run)"
    if not args.no_telemetry:
        out["under_load"] = attention_under_load(layer)
    out["stage_switch"] = stage_switch_bench(dev)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, q, k, v)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
