#!/usr/bin/env python3
"""Benchmark of the BNS-GCN partition step on one MI355X.

One "step" is one pass of the whole hot path (sample -> sampled CSR + transpose -> L layers
forward -> loss -> backward) over one synthetic workload, with every input already resident in
HBM.  The headline workload is the largest partition share (config 5, "very-large-one-share"),
run the plain way: every layer aggregates all of its entries in every step (no cached input
aggregate).  `value` = entries aggregated in the timed steps / their time.

Prints ONE JSON line: the headline (median step time of K timed steps, each step bracketed by HIP
events on the stream it runs on), the roofline figure of its dominant kernel class (per-phase HIP
events in a second pass of K steps), the same steps as graph replays and with the input-aggregate
cache, the CPU oracle timed on the host cores on the same work, and a `workloads` array with the
other synthetic workloads (1-4; workload 2 at its three sampling rates).
"""
import argparse
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
FP32_MFMA_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix, published

# (config, p) of the other workloads reported in `workloads`
SWEEP = [(1, 0.1), (2, 1.0), (2, 0.1), (2, 0.01), (3, 0.1), (4, 0.1)]


def kernel_source_hash():
    """Hash of the kernel sources: a committed PMC summary only feeds `roofline.traffic` if it was
    taken from the same sources."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2203_10983_amd", "csrc")
    for name in sorted(os.listdir(d)):
        with open(os.path.join(d, name), "rb") as fh:
            h.update(name.encode())
            h.update(fh.read())
    return h.hexdigest()[:16]


def mfma_regimes():
    """Issue rate of v_mfma_f32_32x32x2_f32 with nothing else in the loop, over wavefronts resident per SIMD
    and independent accumulators per wavefront (one workgroup of 4 w wavefronts per compute unit gives w per
    SIMD; two or three workgroups per compute unit reach 6 and 8)."""
    import torch
    import paper_2203_10983_amd as pkg
    dev = torch.device("cuda:0")
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    stream = torch.cuda.current_stream()
    out = torch.zeros(8 * cus, dtype=torch.float32, device=dev)
    # (wavefronts per workgroup, workgroups per compute unit, accumulators)
    cases = [(4, 1, 1), (4, 1, 2), (4, 1, 4), (8, 1, 1), (8, 1, 2), (8, 1, 4), (8, 1, 6), (4, 3, 4), (4, 4, 4), (16, 1, 4),
             (4, 4, 1), (4, 4, 2), (16, 1, 1), (16, 1, 2), (8, 3, 2), (8, 4, 2), (16, 2, 1), (16, 2, 2), (4, 8, 2)]
    rows = []
    for wpb, bpc, n_acc in cases:
        per_simd = wpb * bpc // 4
        iters = max(200, 16000 // (per_simd * n_acc))
        blocks = cus * bpc
        for _ in range(2):
            pkg.probe_mfma(n_acc, wpb, blocks, iters, out)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        torch.cuda.synchronize()
        ev[0].record(stream)
        for i in range(3):
            pkg.probe_mfma(n_acc, wpb, blocks, iters, out)
            ev[i + 1].record(stream)
        torch.cuda.synchronize()
        ms = statistics.median(ev[i].elapsed_time(ev[i + 1]) for i in range(3))
        flops = 4096.0 * 8 * n_acc * iters * wpb * blocks
        rows.append({"wavefronts_per_simd": per_simd, "accumulators": n_acc, "wavefronts_per_workgroup": wpb,
                     "workgroups_per_cu": bpc, "ms": round(ms, 3), "TFLOPs": round(flops / ms / 1e9, 1)})
    return {"metric": "issue rate of v_mfma_f32_32x32x2_f32, nothing else in the loop", "unit": "TFLOP/s",
            "peak": FP32_MFMA_PEAK_TFLOPS, "compute_units": cus, "regimes": rows}


def run_workload(cfg, p, kind, steps, warmup, dropout=0.0, extras=False, cpu_baseline=True, calibrate=False,
                 local_order="native"):
    """Times one workload; -> dict.  extras: also the graph-replay and the cached-input variants,
    the whole-step roofline and the memory figures (the headline workload)."""
    import torch
    import paper_2203_10983_amd as pkg
    from bns_inputs import SAMPLING_SEED, make_workload
    from bns_inputs.workloads import sage_weights

    t0 = time.time()
    w = make_workload(cfg, local_order=local_order)
    if kind == 1:
        w.W = sage_weights(220310983 + w.cfg + 300, w.dims)
    P, L = w.part, w.n_layers
    dev = torch.device("cuda:0")
    ctx = pkg.Context(P, w.dims, w.loss_kind, device=dev, layer_kind=kind)
    ctx.set_dropout(dropout)
    X = torch.from_numpy(w.X).to(dev)
    halo_h = [torch.from_numpy(h).to(dev) for h in w.halo_h]
    labels = torch.from_numpy(w.labels).to(dev)
    W = [torch.from_numpy(x).to(dev) for x in w.W]
    dW = [torch.empty_like(x) for x in W]
    dhalo = [None] + [torch.empty(P.n_halo + 1, w.dims[l], dtype=torch.float32, device=dev) for l in range(1, L)]
    loss = torch.zeros(1, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    t_setup = time.time() - t0
    stream = torch.cuda.current_stream()

    def step(epoch):
        ctx.train_step(SAMPLING_SEED, epoch, p, X, halo_h, labels, W, dW, dhalo, loss, 0.0)

    if calibrate:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)        # one elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    def timed(first_epoch):
        """K steps, one event between consecutive steps on the steps' stream -> (wall ms, per-step ms)."""
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ev[0].record(stream)
        for e in range(steps):
            step(first_epoch + e)
            ev[e + 1].record(stream)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        return (t2 - t1) * 1e3, [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]

    for e in range(warmup):
        step(e)
    torch.cuda.synchronize()
    # pass 1, the headline: nothing but the steps and one event per step
    wall_ms, per_step = timed(warmup)
    ms_median = statistics.median(per_step)
    n_kept = int(ctx.ws_tensor(pkg.VIEW_N_KEPT)[0])
    nnz = int(ctx.ws_tensor(pkg.VIEW_NNZ)[0])          # of the last epoch (varies by < 1% over epochs)
    # pass 2: the same K steps with HIP-event brackets around every kernel class
    ctx.profile_enable(0xFFFFFFFF, steps * (12 * L + 8))
    for e in range(steps):
        step(warmup + e)
    torch.cuda.synchronize()
    phases = ctx.profile_read()
    ctx.profile_enable(0, 0)

    n_in, dims = P.n_in, w.dims
    e_u = nnz - P.e_in                                   # kept boundary entries
    edges_per_step = nnz * (2 * L - 1)                   # L forward + (L - 1) transposed aggregates, each over nnz entries
    fused = [l for l in range(1, L + 1) if ctx.layer_plan(l) == pkg.LAYER_ONE_KERNEL]
    first = [l for l in range(1, L + 1) if ctx.layer_plan(l) == pkg.LAYER_UPDATE_FIRST]

    # ---- algorithmic bytes / flops per kernel class ---------------------------------------------
    # how train_step runs each layer: one kernel for aggregate + update (its update is timed and counted
    # with the aggregate: it also writes H_out and reads W there, and A is not read back), or update
    # first (the aggregate then runs at the output width)
    fw = {l: dims[l] if l in first else dims[l - 1] for l in range(1, L + 1)}        # forward aggregate width
    bw = {l: dims[l] if (kind == 0 and dims[l] < dims[l - 1]) else dims[l - 1] for l in range(2, L + 1)}

    def fwd_alg(l, cached=False):
        if cached:      # the cached inner sum and the kept boundary rows instead of all neighbours
            return 4 * e_u + 4 * (n_in + 1) + 4 * fw[l] * (n_in + n_kept) + 4 * fw[l] * n_in
        return 4 * nnz + 4 * (n_in + 1) + 4 * fw[l] * (n_in + n_kept) + 4 * fw[l] * n_in

    fwd_bytes = sum(fwd_alg(l) for l in range(1, L + 1))
    fwd_bytes += sum(4 * n_in * dims[l] + 4 * dims[l - 1] * dims[l] for l in fused)
    bwd_bytes = sum(4 * nnz + 4 * (n_in + n_kept + 1) + 4 * bw[l] * n_in + 4 * bw[l] * (n_in + n_kept)
                    for l in range(2, L + 1))
    # bytes the aggregates ask for when no neighbour row is found in a cache (index + one row per entry + output)
    fwd_req = sum(4 * nnz + 4 * fw[l] * nnz + 4 * fw[l] * n_in for l in range(1, L + 1))
    bwd_req = sum(4 * nnz + 4 * bw[l] * nnz + 4 * bw[l] * (n_in + n_kept) for l in range(2, L + 1))
    kw = 2 if kind == 1 else 1      # the concat update doubles the depth of every product
    gemm_flops = {"gemm_fwd": sum(2 * kw * n_in * dims[l - 1] * dims[l] for l in range(1, L + 1) if l not in fused),
                  "gemm_dw": sum(2 * kw * n_in * dims[l - 1] * dims[l] for l in range(1, L + 1)),
                  "gemm_da": sum(2 * kw * n_in * dims[l - 1] * dims[l] for l in range(2, L + 1))}
    per_step_ms = {k: v[0] / steps for k, v in phases.items()}
    launches = {k: v[1] // steps for k, v in phases.items()}
    # the forward aggregate class = the one-kernel / plain aggregate launches plus, before one-kernel layers,
    # the pass over the rows longer than one segment (timed apart so that launch times match a kernel trace)
    long_ms = per_step_ms.pop("spmm_long")
    fwd_kernel_ms = per_step_ms["spmm_fwd"]
    per_step_ms["spmm_fwd"] += long_ms
    cand = {k: per_step_ms[k] for k in ("spmm_fwd", "spmm_bwd", "gemm_fwd", "gemm_dw", "gemm_da")}
    dom = max(cand, key=cand.get)
    if dom.startswith("spmm"):
        alg = fwd_bytes if dom == "spmm_fwd" else bwd_bytes
        achieved = alg / (per_step_ms[dom] * 1e-3) / 1e9
        roof = {"kernel": dom, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                "launches_per_step": launches[dom], "avg_launch_ms": per_step_ms[dom] / max(launches[dom], 1),
                "algorithmic_bytes_per_step": alg}
        # another reading of the same time: what the kernel asks for without any cache re-use
        roof["requested_GBps"] = (fwd_req if dom == "spmm_fwd" else bwd_req) / (per_step_ms[dom] * 1e-3) / 1e9
        if dom == "spmm_fwd" and fused:
            # per launch: the dominant kernel itself, and the long-row pass that precedes it
            roof["avg_launch_ms"] = fwd_kernel_ms / max(launches[dom], 1)
            roof["kernel_name"] = "spmm_gemm_kernel (aggregate + update)"
            roof["long_row_pass_ms_per_launch"] = long_ms / max(launches[dom], 1)
            roof["note"] = ("achieved = algorithmic bytes of the layer (aggregate + H_out + W) / (long-row pass + "
                            "one-kernel launch); avg_launch_ms is the one-kernel launch alone, as a kernel trace shows it")
    else:
        fl = gemm_flops[dom]
        achieved = fl / (per_step_ms[dom] * 1e-3) / 1e12
        roof = {"kernel": dom, "bound": "mfma", "achieved": achieved, "peak": FP32_MFMA_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / FP32_MFMA_PEAK_TFLOPS, "traffic": None,
                "launches_per_step": launches[dom], "avg_launch_ms": per_step_ms[dom] / max(launches[dom], 1),
                "algorithmic_flops_per_step": fl}
    # HBM-side bytes per launch from the committed rocprofv3 PMC summary of this workload, if there is one
    # taken from these kernel sources (its "bench-traffic:" line)
    src = os.path.join("profiles", f"train_step_config{w.cfg}_hbm_traffic.md")
    try:
        with open(os.path.join(ROOT, src)) as fh:
            line = [ln for ln in fh if ln.strip().startswith("bench-traffic:")][-1]
        tr = json.loads(line.split("bench-traffic:", 1)[1])
        if tr["workload"] == f"config {w.cfg}: {w.name}" and abs(tr["p"] - p) < 1e-12 and kind == 0 \
                and not tr.get("input_aggregate_cached", True):
            if tr.get("csrc_sha") == kernel_source_hash():
                roof["traffic"] = tr["bytes_per_launch"].get(dom)
                roof["traffic_source"] = src
                # what crossed the L2 <-> fabric interface (above the Infinity Cache) per launch of the kernel
                if roof["traffic"] and roof.get("avg_launch_ms"):
                    roof["traffic_GBps"] = roof["traffic"] / (roof["avg_launch_ms"] * 1e-3) / 1e9
            else:
                roof["traffic_stale"] = f"{src} was taken from other kernel sources ({tr.get('csrc_sha')})"
    except (OSError, KeyError, ValueError, IndexError):
        pass
    classes = {
        "spmm_fwd_GBps": fwd_bytes / (per_step_ms["spmm_fwd"] * 1e-3) / 1e9 if per_step_ms["spmm_fwd"] else None,
        "spmm_bwd_GBps": bwd_bytes / (per_step_ms["spmm_bwd"] * 1e-3) / 1e9 if per_step_ms["spmm_bwd"] else None,
        "spmm_fwd_frac": fwd_bytes / (per_step_ms["spmm_fwd"] * 1e-3) / 1e9 / HBM_PEAK_GBS if per_step_ms["spmm_fwd"] else None,
        "spmm_bwd_frac": bwd_bytes / (per_step_ms["spmm_bwd"] * 1e-3) / 1e9 / HBM_PEAK_GBS if per_step_ms["spmm_bwd"] else None,
    }
    classes["spmm_fwd_requested_GBps"] = fwd_req / (per_step_ms["spmm_fwd"] * 1e-3) / 1e9 if per_step_ms["spmm_fwd"] else None
    classes["spmm_bwd_requested_GBps"] = bwd_req / (per_step_ms["spmm_bwd"] * 1e-3) / 1e9 if per_step_ms["spmm_bwd"] else None
    classes["spmm_fwd_long_row_pass_ms"] = long_ms      # part of spmm_fwd above
    for k, fl in gemm_flops.items():
        classes[k + "_TFLOPs"] = fl / (per_step_ms[k] * 1e-3) / 1e12 if per_step_ms[k] else None
    # the integer stage (sample + sampled CSR + transposed rows) against HBM: bytes it has to move / its time
    int_bytes = 12 * P.n_halo + 4 * n_kept + 8 * P.e_bd + 12 * P.e_in + 8 * e_u + 8 * (n_in + 1) + 4 * n_kept
    int_ms = per_step_ms["sample"] + per_step_ms["build"]
    classes["sample_build_GBps"] = int_bytes / (int_ms * 1e-3) / 1e9 if int_ms else None

    out = {
        "workload": f"config {w.cfg}: {w.name}", "p": p, "layer": "gcn" if kind == 0 else "graphsage-mean",
        "n_in": n_in, "n_halo": P.n_halo, "n_kept": n_kept, "nnz": nnz, "dims": dims,
        "ms_per_step": ms_median, "ms_per_step_mean": wall_ms / steps, "ms_per_step_min": min(per_step),
        "edges_per_step": edges_per_step, "edges_per_s": edges_per_step / (ms_median * 1e-3),
        "one_kernel_layers": fused, "update_first_layers": first,
        "roofline": roof, "phases_ms_per_step": {k: round(v, 4) for k, v in per_step_ms.items()},
        "kernel_classes": classes, "sampling_overhead": int_ms / ms_median, "setup_s": round(t_setup, 1),
    }

    if extras:
        # the same K epochs as replays of one captured step (no launch gaps)
        side = torch.cuda.Stream(device=dev)
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            ctx.graph_capture(SAMPLING_SEED, warmup, p, X, halo_h, labels, W, dW, dhalo, loss, 0.0)
            ctx.graph_replay(2)
            side.synchronize()
            t3 = time.perf_counter()
            ctx.graph_replay(steps)
            side.synchronize()
            t4 = time.perf_counter()
        out["ms_per_step_graph_replay"] = (t4 - t3) * 1e3 / steps
        # static-inner caching of layer 1: its inner entries are aggregated once, outside the timed steps,
        # so a step aggregates e_in fewer entries; own edge count and bytes
        ctx.cache_input_aggregate(X)
        for e in range(2):
            step(e)
        _, per_c = timed(warmup)
        ctx.profile_enable(0xFFFFFFFF, steps * (12 * L + 8))
        for e in range(steps):
            step(warmup + e)
        torch.cuda.synchronize()
        ph_c = {k: v[0] / steps for k, v in ctx.profile_read().items()}
        ctx.profile_enable(0, 0)
        plan1_cached = ctx.layer_plan(1)
        ctx.cache_input_aggregate(None)
        ms_c = statistics.median(per_c)
        edges_c = edges_per_step - P.e_in
        fwd_c = fwd_bytes - fwd_alg(1) + (4 * e_u + 4 * (n_in + 1) + 4 * dims[0] * (n_in + n_kept) + 4 * dims[0] * n_in) \
            if 1 not in first else None
        out["cached_input_aggregate"] = {
            "ms_per_step": ms_c, "edges_per_step": edges_c, "edges_per_s": edges_c / (ms_c * 1e-3),
            "layer_1_plan": plan1_cached,
            "spmm_fwd_ms_per_step": ph_c["spmm_fwd"] + ph_c["spmm_long"],
            "spmm_fwd_algorithmic_bytes_per_step": fwd_c,
            "note": "layer 1 adds only the kept boundary entries of each row to the inner sum aggregated once at set-up",
        }
        # ---- the ceiling of the aggregate's access pattern on this machine, measured beside it: a bare gather
        # (bns_probe_gather) of as many uniformly random rows as a layer has entries, of the width the forward
        # aggregates run at, from a table as large as the stacked features, as many rows per wavefront as the
        # average row has entries.  The generator's graphs have no locality beyond their degree distribution,
        # so no order of the same reads does better than this rate times the share of reads that hit in L2.
        widths = [fw[l] for l in range(1, L + 1)]
        d_probe = max(set(widths), key=widths.count)
        if d_probe in (16, 32, 64, 128, 256):
            n_rows = n_in + n_kept
            gen = torch.Generator(device=dev)
            gen.manual_seed(220310983)
            table = torch.randn(n_rows, d_probe, dtype=torch.float32, device=dev, generator=gen)
            idx = torch.randint(0, n_rows, (nnz,), dtype=torch.int32, device=dev, generator=gen)
            per_wave = max(1, round(nnz / n_in))
            waves = (nnz + per_wave - 1) // per_wave
            outp = torch.empty(waves, d_probe, dtype=torch.float32, device=dev)
            for _ in range(3):
                pkg.probe_gather(table, idx, per_wave, outp)
            evp = [torch.cuda.Event(enable_timing=True) for _ in range(11)]
            torch.cuda.synchronize()
            evp[0].record(stream)
            for i in range(10):
                pkg.probe_gather(table, idx, per_wave, outp)
                evp[i + 1].record(stream)
            torch.cuda.synchronize()
            ms_g = statistics.median(evp[i].elapsed_time(evp[i + 1]) for i in range(10))
            req = 4 * nnz + 4 * d_probe * nnz + 4 * d_probe * waves
            ceiling = req / (ms_g * 1e-3) / 1e9
            out["gather_ceiling"] = {
                "requested_GBps": ceiling, "ms": ms_g, "rows_gathered": nnz, "row_floats": d_probe,
                "table_MB": n_rows * d_probe * 4 / 1e6, "rows_per_wavefront": per_wave,
                "note": "bare gather of uniformly random rows (index + row per entry + one row stored per wavefront), "
                        "same loads in flight as the aggregate kernels; the aggregates' requested_GBps is to be read "
                        "against this, their algorithmic GB/s against it times algorithmic / requested bytes"}
            del table, idx, outp
        # ---- whole-step roofline: sum over kernel classes of max(compulsory bytes / HBM peak, flops / MFMA peak)
        gemm_bytes = {"gemm_fwd": sum(4 * n_in * (kw * dims[l - 1] + dims[l]) for l in range(1, L + 1) if l not in fused),
                      "gemm_dw": sum(4 * n_in * (kw * dims[l - 1] + dims[l]) for l in range(1, L + 1)),
                      "gemm_da": sum(4 * n_in * (kw * dims[l - 1] + dims[l]) for l in range(2, L + 1))}
        t_roof = (fwd_bytes + bwd_bytes) / (HBM_PEAK_GBS * 1e9)
        t_roof += sum(max(gemm_flops[k] / (FP32_MFMA_PEAK_TFLOPS * 1e12), gemm_bytes[k] / (HBM_PEAK_GBS * 1e9))
                      for k in gemm_flops)
        t_roof += sum(2 * n_in * dims[l - 1] * dims[l] for l in fused) / (FP32_MFMA_PEAK_TFLOPS * 1e12)  # fused updates
        t_roof += 8 * n_in * dims[L] / (HBM_PEAK_GBS * 1e9)                                          # loss
        t_roof += int_bytes / (HBM_PEAK_GBS * 1e9)                                                   # sample + CSRs
        out["step_roofline"] = {"t_roof_ms": t_roof * 1e3, "frac": t_roof * 1e3 / ms_median,
                                "note": "sum over kernel classes of max(compulsory bytes / 8 TB/s, flops / 157.3 TFLOP/s) / ms_per_step"}
        # activations held for the backward pass per layer (floats), beside the memory model of Eq. 4
        held = [n_in * dims[l - 1] + n_in * dims[l] + n_kept * dims[l - 1] for l in range(1, L + 1)]
        eq4 = [(3 * n_in + n_kept) * dims[l] for l in range(1, L + 1)]
        out["memory"] = {"held_floats_per_layer": held, "eq4_floats_per_layer": eq4, "workspace_bytes": ctx.ws_bytes}

    # ---- CPU baseline: the oracle as it stands, one full step of the same workload (same work: every
    # layer aggregates every entry) on the host cores
    if cpu_baseline:
        from oracle import bns_oracle as orc
        tc = time.perf_counter()
        ref = orc.step(P, w.loss_kind, w.X, w.halo_h, w.labels, w.W, SAMPLING_SEED, 0, p, layer_kind=kind,
                       dropout=dropout)
        dt = time.perf_counter() - tc
        nnz0 = int(ref["sub"]["col_idx"].size)
        out["cpu_baseline"] = {"value": nnz0 * (2 * L - 1) / dt, "unit": "edges/s", "cores": orc.num_threads(),
                               "kind": "oracle", "sample": f"1 full step (epoch 0) of the same workload, {dt:.1f} s",
                               "ms_per_step": dt * 1e3}
        del ref
    ctx.close()
    del ctx, X, halo_h, labels, W, dW, dhalo
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", type=int, default=5, help="headline workload, 1..5")
    ap.add_argument("--p", type=float, default=0.1, help="sampling rate of the headline workload")
    ap.add_argument("--model", choices=["gcn", "sage"], default="gcn",
                    help="gcn: the GCN layer of the five configs; sage: GraphSAGE-mean, the paper's own model")
    ap.add_argument("--dropout", type=float, default=0.0,
                    help="dropout rate on the hidden activations (the five workloads name none: default 0)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mfma-regimes", action="store_true",
                    help="instead of a workload: time the bare fp32 matrix instruction (bns_probe_mfma) over wavefronts "
                         "per SIMD x independent accumulators per wavefront and print the rates as one JSON line")
    ap.add_argument("--local-order", choices=["native", "degree"], default="native",
                    help="numbering of the partition's inner nodes: the generator's (default, what every reported figure "
                         "uses) or descending degree (the measurement of what node order does to the aggregates)")
    ap.add_argument("--only", action="store_true", help="the headline workload only (no `workloads` sweep, no "
                    "graph-replay / cached variants): what the rocprofv3 summaries under profiles/ run")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 1 GiB device-to-device copies (a kernel of known traffic, "
                         "to scale rocprofv3's FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs one partition on ONE GPU; --gpus must be 1 "
                 "(no collectives or sharding are part of it)")

    if args.mfma_regimes:
        print(json.dumps(mfma_regimes()))
        return
    kind = 1 if args.model == "sage" else 0
    head = run_workload(args.workload, args.p, kind, args.steps, args.warmup, dropout=args.dropout,
                        extras=not args.only, cpu_baseline=not args.no_cpu_baseline, calibrate=args.calibrate_copy,
                        local_order=args.local_order)
    others = []
    if not args.only:
        for cfg, p in SWEEP:
            if cfg == args.workload and abs(p - args.p) < 1e-12:
                continue
            r = run_workload(cfg, p, kind, min(args.steps, 20), min(args.warmup, 3),
                             cpu_baseline=not args.no_cpu_baseline)
            keep = ("workload", "p", "n_in", "n_kept", "nnz", "dims", "ms_per_step", "ms_per_step_mean",
                    "edges_per_step", "edges_per_s", "one_kernel_layers", "update_first_layers", "sampling_overhead")
            o = {k: r[k] for k in keep}
            o["dominant"] = {k: r["roofline"][k] for k in ("kernel", "bound", "achieved", "peak", "unit", "frac")}
            o["kernel_classes"] = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in r["kernel_classes"].items()}
            if "cpu_baseline" in r:
                o["oracle_ms_per_step"] = r["cpu_baseline"]["ms_per_step"]
                o["oracle_cores"] = r["cpu_baseline"]["cores"]
            others.append(o)

    out = {
        "metric": "aggregated edges/s of one partition's BNS-GCN epoch (fwd+bwd); ms per epoch in ms_per_step",
        "value": head["edges_per_s"], "unit": "edges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "ms_per_step_mean": head["ms_per_step_mean"],
        "ms_per_step_min": head["ms_per_step_min"],
        "timing": "median over the timed steps, each bracketed by HIP events on its stream; no other events in that pass",
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": head["workload"], "p": head["p"], "n_in": head["n_in"], "n_halo": head["n_halo"],
                   "n_kept": head["n_kept"], "nnz": head["nnz"], "dims": head["dims"], "layers": len(head["dims"]) - 1,
                   "edges_per_step": head["edges_per_step"], "setup_s": head["setup_s"],
                   "input_aggregate_cached": False, "layer": head["layer"], "dropout": args.dropout,
                   "one_kernel_layers": head["one_kernel_layers"], "update_first_layers": head["update_first_layers"],
                   "kernel_source_hash": kernel_source_hash()},
        "roofline": head["roofline"],
        "phases_ms_per_step": head["phases_ms_per_step"],
        "kernel_classes": head["kernel_classes"],
        "sampling_overhead": head["sampling_overhead"],
    }
    for k in ("ms_per_step_graph_replay", "cached_input_aggregate", "gather_ceiling", "step_roofline", "memory"):
        if k in head:
            out[k] = head[k]
    out["cpu_baseline"] = head.get("cpu_baseline")
    if others:
        out["workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
