#!/usr/bin/env python3
"""Benchmark of the S-STE 2:4 sparse linear-layer hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input, for EVERY linear layer of the
workload, back to back on one stream:
  project + scale + pack of W  ->  forward sparse GEMM  ->  MVUE weight-gradient sparse GEMM.
The default (headline) workload is the largest one: the four linears of a GPT-2-774M block in the 8-bit
format (e4m3 weights, activations and gradients, 32768 tokens).  The same measurement on the bf16 block
(16384 tokens), the GPT-2-350M FFN pair and the GPT-2-124M fc1 layer rides along in `secondary`.
Prints ONE JSON line.  `value` = dense-equivalent TFLOP/s of forward + weight gradient of all layers
(sum of 2 * 2*T*I*O flops) over the whole step time, pruning included.
"""
import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# published MI355X peaks
PEAK_HBM_GBS = 8000.0
PEAK_DENSE_TFLOPS = {"bf16": 2500.0, "e4m3": 5000.0}
FMT_MAX = {"e4m3": 448.0, "e5m2": 57344.0}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=5, help="workload number (1-5); 5 is the headline one")
    ap.add_argument("--layer", type=int, default=-1, help="layer index inside the workload; -1 = every layer (the block)")
    ap.add_argument("--sets", type=int, default=0,
                    help="activation buffer sets rotated over steps; 0 = as many as it takes to exceed the 256 MB cache twice over")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true", help="skip the bf16 block and the 124M layer")
    ap.add_argument("--grad-e5m2", action="store_true",
                    help="8-bit workloads: output gradients in e5m2 (the paper's backward format) instead of e4m3")
    ap.add_argument("--dense-context", action="store_true",
                    help="also time the vendor dense bf16 GEMM (torch.matmul) on the same shapes: context, not the product")
    ap.add_argument("--no-prune-model", action="store_true",
                    help="skip the whole-model re-projection measurement (144 weight tensors of GPT-2-774M, 2.2 GB)")
    ap.add_argument("--no-kernel-timing", action="store_true", help="do not bracket kernels with events (for counter runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 256 MiB device copies before the warm-up (reference for HBM byte counters)")
    return ap.parse_args()


def hbm_traffic_table():
    """(workload, kernel kind) -> HBM bytes per launch, read from the committed rocprofv3 counter summary
    profiles/hbm_traffic.md (FETCH_SIZE and WRITE_SIZE runs of this file, scaled as that summary states).
    Rows look like `| 5 | wgrad | 123456 | 65432 |` (KiB fetched, KiB written, averages per launch)."""
    table = {}
    path = os.path.join(ROOT, "profiles", "hbm_traffic.md")
    if not os.path.exists(path):
        return table
    for line in open(path):
        m = re.match(r"^\|\s*(\d+)\s*\|\s*([a-z_]+)\s*\|\s*([0-9.]+)\s*\|\s*([0-9.]+)\s*\|", line)
        if m:
            table[(int(m.group(1)), m.group(2))] = (float(m.group(3)) + float(m.group(4))) * 1024.0
    return table


class LayerState:
    """Device-resident operands and outputs of one linear layer (several rotating sets of the big ones)."""
    pass


def make_layer(sste, torch, np, WL, wl, li, nsets, grad_e5m2):
    L = wl.layers[li]
    T, O, I = wl.T, L.O, L.I
    fp8 = wl.dtype == "e4m3"
    st = LayerState()
    st.name, st.T, st.O, st.I, st.fp8 = L.name, T, O, I, fp8
    st.dt = sste.F8E4M3 if fp8 else sste.BF16
    st.gdt = sste.F8E5M2 if (fp8 and grad_e5m2) else st.dt
    st.esize = 1 if fp8 else 2

    def up(bits):
        return torch.from_numpy(np.ascontiguousarray(bits.view(np.int16))).cuda().view(torch.bfloat16)

    st.wb = WL.weight_bits(wl, li)
    st.W = up(st.wb)
    xb = WL.activations(wl, li)[0]
    dyb = WL.output_gradient(wl, li)[0]
    Xb, dYb = up(xb), up(dyb)
    del xb, dyb
    if fp8:
        # operand preparation of Sec. 5.2 on the GPU, before the timed region: per-tensor largest magnitude,
        # then rescale + cast
        def quantise(t, fmt_code, fmt_max):
            _, amax = sste.cast_fp8(t, 1.0, fmt_code, store=False)
            scale = float(np.float32(float(amax.cpu()[0]) / fmt_max))
            q, _ = sste.cast_fp8(t, scale, fmt_code)
            return q, scale
        X0, st.xs = quantise(Xb, sste.F8E4M3, FMT_MAX["e4m3"])
        dY0, st.dys = quantise(dYb, st.gdt, FMT_MAX["e5m2" if st.gdt == sste.F8E5M2 else "e4m3"])
        del Xb, dYb
    else:
        X0, dY0, st.xs, st.dys = Xb, dYb, 1.0, 1.0
    st.Xs = [X0] + [X0.clone() for _ in range(nsets - 1)]
    st.dYs = [dY0] + [dY0.clone() for _ in range(nsets - 1)]
    st.Zs = [torch.empty((T, O), dtype=torch.bfloat16, device="cuda") for _ in range(nsets)]
    st.dWs = [torch.empty((O, I), dtype=torch.float32, device="cuda") for _ in range(nsets)]
    st.vals, st.meta = sste.packed_buffers(O, I, st.dt, "cuda")
    st.ws_bytes = sste.wgrad_workspace_bytes(T, O, I, st.gdt)
    st.wss = [torch.empty(max(st.ws_bytes, 16), dtype=torch.uint8, device="cuda") for _ in range(nsets)]
    # beta: computed once from the initial weights, then frozen (Sec. 4.2)
    st.beta = float(sste.compute_beta(st.W).cpu()[0])
    if fp8:
        amax = torch.zeros(1, dtype=torch.float32, device="cuda")
        sste.project_pack(st.W, st.beta, sste.BF16, 1.0, amax_out=amax)
        st.w_scale = float(np.float32(float(amax.cpu()[0]) / 448.0))
    else:
        st.w_scale = 1.0
    st.flops = 2.0 * T * I * O                        # dense-equivalent flops of one GEMM
    st.nsets = nsets
    return st


def layer_step(sste, st, seed, i, project=True):
    s = i % st.nsets
    if project:
        sste.project_pack(st.W, st.beta, st.dt, st.w_scale, vals=st.vals, meta=st.meta)
    sste.linear_fwd(st.Xs[s], st.vals, st.meta, st.O, st.dt, st.xs, st.w_scale, Z=st.Zs[s])
    sste.linear_wgrad(st.dYs[s], st.Xs[s], seed=seed, offset=i, dtype=st.gdt, dy_scale=st.dys, x_scale=st.xs,
                      dW=st.dWs[s], workspace=st.wss[s])


def kernel_table(sste, layers, kt, dtype):
    """Per-kind averages over all launches of the events pass, with the algorithmic work the launches did."""
    def avg_ms(name):
        ms, n = kt[name]
        return ms / n if n else float("nan")

    n_layers = len(layers)
    flops = sum(st.flops for st in layers) / n_layers                     # mean dense-equivalent flops per GEMM launch
    # project + pack: one launch per layer, or one multi-tensor launch per step for a block of layers
    pp_per_step = sum(st.O * st.I * (2 + st.esize / 2 + 0.125) for st in layers)
    pp_bytes = pp_per_step * (kt["fwd"][1] / n_layers) / max(1, kt["project_pack"][1])
    mv_bytes = sum(st.T * st.O * st.esize * (1 + 0.5 + 0.0625) for st in layers if st.ws_bytes) / max(1, sum(1 for st in layers if st.ws_bytes))
    kernels = {}
    ms = avg_ms("project_pack")
    kernels["project_pack"] = {"ms": ms, "launches": kt["project_pack"][1], "GB_per_s": pp_bytes / (ms * 1e-3) * 1e-9,
                               "frac_hbm_peak": pp_bytes / (ms * 1e-3) * 1e-9 / PEAK_HBM_GBS}
    for k in ("fwd", "wgrad"):
        ms = avg_ms(k)
        kernels[k] = {"ms": ms, "launches": kt[k][1], "dense_equiv_TFLOP_per_s": flops / (ms * 1e-3) * 1e-12}
        kernels[k]["frac_sparse_mfma_peak"] = kernels[k]["dense_equiv_TFLOP_per_s"] / (2 * PEAK_DENSE_TFLOPS[dtype])
    if kt["wgrad_reduce"][1]:
        kernels["wgrad_reduce"] = {"ms": avg_ms("wgrad_reduce"), "launches": kt["wgrad_reduce"][1]}
    if kt["mvue_pack"][1]:
        ms = avg_ms("mvue_pack")
        kernels["mvue_pack"] = {"ms": ms, "launches": kt["mvue_pack"][1], "GB_per_s": mv_bytes / (ms * 1e-3) * 1e-9,
                                "frac_hbm_peak": mv_bytes / (ms * 1e-3) * 1e-9 / PEAK_HBM_GBS}
    # the weight-gradient row as a whole: estimator pre-pass + GEMM + reduction, per layer
    row_ms = sum(kt[k][0] for k in ("wgrad", "wgrad_reduce", "mvue_pack")) / max(1, kt["wgrad"][1])
    kernels["wgrad_row"] = {"ms": row_ms, "dense_equiv_TFLOP_per_s": flops / (row_ms * 1e-3) * 1e-12,
                            "frac_sparse_mfma_peak": flops / (row_ms * 1e-3) * 1e-12 / (2 * PEAK_DENSE_TFLOPS[dtype])}
    return kernels, flops


def roofline_of(kernels, flops, dtype, cfg, traffic):
    """The `roofline` object for the kernel kind with the longest average launch, and `roofline_row` for the
    weight-gradient row (pre-pass + GEMM + reduction together).  The sparse MFMA executes half of the
    dense-equivalent multiply-adds: algorithmic flops per launch = T*I*O (I/2 or T/2 MACs per output element),
    held against the published dense MFMA peak of the operand type."""
    dom = max([k for k in ("project_pack", "fwd", "wgrad", "mvue_pack") if k in kernels], key=lambda k: kernels[k]["ms"])
    if dom in ("project_pack", "mvue_pack"):
        achieved = kernels[dom]["GB_per_s"]
        roof = {"kernel": dom, "bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS}
    else:
        peak = PEAK_DENSE_TFLOPS[dtype]
        achieved = 0.5 * flops / (kernels[dom]["ms"] * 1e-3) * 1e-12
        roof = {"kernel": dom, "bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak}
    roof["avg_launch_ms"] = kernels[dom]["ms"]
    roof["traffic"] = traffic.get((cfg, dom))
    peak = PEAK_DENSE_TFLOPS[dtype]
    row = {"kernel": "mvue_pack + wgrad + wgrad_reduce", "bound": "mfma",
           "achieved": 0.5 * flops / (kernels["wgrad_row"]["ms"] * 1e-3) * 1e-12, "peak": peak, "unit": "TFLOP/s",
           "avg_row_ms": kernels["wgrad_row"]["ms"]}
    row["frac"] = row["achieved"] / peak
    parts = [traffic.get((cfg, k)) for k in ("mvue_pack", "wgrad", "wgrad_reduce") if k in kernels]
    row["traffic"] = sum(parts) if parts and all(p is not None for p in parts) else None
    return roof, row


def measure(sste, torch, np, WL, cfg, layer_sel, steps, warmup, sets, grad_e5m2, with_events, traffic, chunks=10):
    """Builds the workload's layers in HBM, runs `warmup` untimed and exactly `steps` timed steps between two
    synchronisations, then (optionally) the same steps again with an event pair around every hot kernel."""
    wl = WL.WORKLOADS[cfg]
    sel = list(range(len(wl.layers))) if layer_sel < 0 else [layer_sel]
    # bytes one set of a step's big operands and outputs occupies; rotate enough sets to exceed the cache twice
    esize = 1 if wl.dtype == "e4m3" else 2
    set_bytes = sum(wl.T * (wl.layers[i].I * esize + wl.layers[i].O * (esize + 2)) for i in sel)
    nsets = sets if sets > 0 else max(1, min(8, -(-(512 << 20) // set_bytes)))
    layers = [make_layer(sste, torch, np, WL, wl, i, nsets, grad_e5m2) for i in sel]

    # The re-projection of every layer's weight is one multi-tensor launch at the head of the step (what the
    # batch entry point is for: single layers are launch-bound); forward and weight gradient follow per layer.
    batch = sste.PackBatch([st.W for st in layers], [st.beta for st in layers], layers[0].dt, [st.w_scale for st in layers],
                           vals=[st.vals for st in layers], metas=[st.meta for st in layers]) if len(layers) > 1 else None

    def step(i):
        if batch is not None:
            batch.launch()
        for st in layers:
            layer_step(sste, st, cfg, i, project=batch is None)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps between two synchronisations -> `value`
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i)
    t_enq = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps

    # ---- spread: the same steps in `chunks` separately synchronised pieces (median / min per step)
    per = max(1, steps // chunks)
    chunk_ms = []
    for c in range(chunks):
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for i in range(per):
            step(warmup + steps + c * per + i)
        torch.cuda.synchronize()
        chunk_ms.append((time.perf_counter() - c0) * 1e3 / per)

    # ---- cache-warm regime: one buffer set reused (what fits stays in the 256 MB Infinity Cache)
    for st in layers:
        st.nsets_saved, st.nsets = st.nsets, 1
    for i in range(3):
        step(i)
    torch.cuda.synchronize()
    w0 = time.perf_counter()
    for i in range(per * 2):
        step(i)
    torch.cuda.synchronize()
    warm_ms = (time.perf_counter() - w0) * 1e3 / (per * 2)
    for st in layers:
        st.nsets = st.nsets_saved

    flops_step = sum(2 * st.flops for st in layers)
    out = {
        "workload": "cfg%d %s: %s" % (wl.cfg, wl.name, ", ".join("%s %dx%d" % (st.name, st.O, st.I) for st in layers)),
        "value": flops_step / (ms_per_step * 1e-3) * 1e-12,
        "ms_per_step": ms_per_step,
        "ms_per_step_median_of_chunks": statistics.median(chunk_ms),
        "ms_per_step_min_of_chunks": min(chunk_ms),
        "ms_per_step_cache_warm": warm_ms,
        "host_enqueue_ms_per_step": (t_enq - t0) * 1e3 / steps,
        "buffer_sets": nsets,
        "dtype": wl.dtype,
        "frac_sparse_mfma_peak_whole_step": flops_step / (ms_per_step * 1e-3) * 1e-12 / (2 * PEAK_DENSE_TFLOPS[wl.dtype]),
    }
    if with_events:
        # the same steps again, every hot kernel bracketed by its own HIP event pair -> per-kernel durations.
        # The event pairs serialise the queue (about 8 us per launch), so this pass is slower per step than the
        # one above and is not what `value` is quoted on.
        sste.timing_begin(8 * len(layers) * steps + 16)
        torch.cuda.synchronize()
        e0 = time.perf_counter()
        for i in range(steps):
            step(warmup + 2 * steps + i)
        torch.cuda.synchronize()
        out["ms_per_step_with_kernel_events"] = (time.perf_counter() - e0) * 1e3 / steps
        kt = sste.timing_end()
        kernels, flops = kernel_table(sste, layers, kt, wl.dtype)
        out["kernels"] = kernels
        out["roofline"], out["roofline_row"] = roofline_of(kernels, flops, wl.dtype, wl.cfg, traffic)
        # per layer: one short events pass each, so that every GEMM shape has its own figures
        per_layer = {}
        for st in layers:
            sste.timing_begin(8 * 20 + 16)
            for i in range(20):
                layer_step(sste, st, cfg, i)
            torch.cuda.synchronize()
            lk = sste.timing_end()
            row = {k: (lk[k][0] / lk[k][1] if lk[k][1] else 0.0) for k in ("project_pack", "fwd", "mvue_pack", "wgrad", "wgrad_reduce")}
            wrow = row["mvue_pack"] + row["wgrad"] + row["wgrad_reduce"]
            peak2 = 2 * PEAK_DENSE_TFLOPS[wl.dtype]
            per_layer[st.name] = {"us": {k: v * 1e3 for k, v in row.items()},
                                  "fwd_frac_sparse_peak": st.flops / (row["fwd"] * 1e-3) * 1e-12 / peak2,
                                  "wgrad_gemm_frac_sparse_peak": st.flops / (row["wgrad"] * 1e-3) * 1e-12 / peak2,
                                  "wgrad_row_frac_sparse_peak": st.flops / (wrow * 1e-3) * 1e-12 / peak2}
        out["layers"] = per_layer
    return out, layers


def cpu_baseline(np, WL, cfg):
    """Times the oracle, as it stands (its numpy forms), on a bounded sample of the headline workload: one
    step (8-bit casts of X and dY, project + pack, forward, estimator + weight gradient) of the block's
    attention-projection layer (the smallest of the four; the whole block would take minutes).  Median of three runs."""
    from oracle import formats as OF
    from oracle import linear as OL
    from oracle import projection as OP
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    wl = WL.WORKLOADS[cfg]
    li = 1 if len(wl.layers) > 1 else 0
    L = wl.layers[li]
    T = wl.T
    wb = WL.weight_bits(wl, li)
    xb = WL.activations(wl, li, T=T)[0]
    dyb = WL.output_gradient(wl, li, T=T)[0]
    beta32 = np.float32(OP.beta_mse(OF.bf16_to_f32(wb).astype(np.float64)))
    times = []
    for _ in range(3):
        t0 = time.perf_counter()
        if wl.dtype == "e4m3":
            def q(bits):
                amax = np.float32(np.max(np.abs(OF.bf16_to_f32(bits))))
                scale = np.float32(float(amax) / 448.0)
                return OF.cast_fp8(bits, scale, "e4m3")[0], scale
            xc, xs = q(xb)
            dyc, dys = q(dyb)
            _, _, amax = OP.project_pack(wb, beta32)
            ws = np.float32(float(amax) / 448.0)
            rv, rm, _ = OP.project_pack(wb, beta32, "e4m3", ws)
        else:
            xc, xs, dyc, dys, ws = xb, np.float32(1.0), dyb, np.float32(1.0), np.float32(1.0)
            rv, rm, _ = OP.project_pack(wb, beta32)
        OL.linear_fwd(xc, rv, rm, wl.dtype, xs, ws)
        OL.linear_wgrad(dyc, xc, 0, 0, wl.dtype, dys, xs)
        times.append(time.perf_counter() - t0)
    flops = 2 * 2.0 * T * L.I * L.O
    t = statistics.median(times)
    return {
        "value": flops / t * 1e-12,
        "unit": "TFLOP/s",
        "cores": int(cores),
        "kind": "oracle",
        "sample": "one step of cfg%d layer %s (W %dx%d, all %d tokens; the smallest of the block's four layers): casts, project+pack, "
                  "forward, estimator + weight gradient; median of 3 runs (%.2f s each)" % (wl.cfg, L.name, L.O, L.I, T, t),
    }


def prune_model(sste, torch, iters=20):
    """Re-projection + packing of every sparse linear layer of GPT-2-774M (36 blocks x QKV, attention
    projection, fc1, fc2 = 144 distinct bf16 tensors, 1.4 GB read: larger than the Infinity Cache), the
    per-iteration work workload 4 models, as ONE multi-tensor launch and as 144 single launches."""
    shapes = [(3840, 1280), (1280, 1280), (5120, 1280), (1280, 5120)] * 36
    g = torch.Generator(device="cuda")
    g.manual_seed(4000)
    Ws = [(torch.randn(s, generator=g, device="cuda", dtype=torch.float32) * 0.02).to(torch.bfloat16) for s in shapes]
    weights = sum(o * i for o, i in shapes)
    algo_bytes = weights * 3.125                           # 2 B read + 1 B values + 0.125 B positions per weight
    batch = sste.PackBatch(Ws, [1.48] * len(Ws), sste.BF16)

    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / iters

    def singles():
        for W, v, m in zip(Ws, batch.vals, batch.metas):
            sste.project_pack(W, 1.48, sste.BF16, 1.0, vals=v, meta=m)

    ms_batch = timed(batch.launch)
    ms_single = timed(singles)
    out = {
        "tensors": len(shapes), "weights": weights, "algorithmic_bytes": algo_bytes,
        "one_launch": {"ms": ms_batch, "GB_per_s": algo_bytes / ms_batch * 1e-6, "frac_hbm_peak": algo_bytes / ms_batch * 1e-6 / PEAK_HBM_GBS},
        "launch_per_tensor": {"ms": ms_single, "GB_per_s": algo_bytes / ms_single * 1e-6,
                              "frac_hbm_peak": algo_bytes / ms_single * 1e-6 / PEAK_HBM_GBS},
    }
    # The dense-weight step fused with the re-projection, one launch for all 144 tensors: W and the
    # float32 gradient are read, W is written back, the packed form is written.  alpha = 0 keeps the
    # weights where they are over the repetitions.
    Gs = [torch.randn(s, generator=g, device="cuda", dtype=torch.float32) * 1e-4 for s in shapes]
    for master, wbytes in (("bf16", 2), ("f32", 4)):
        Wm = Ws if master == "bf16" else [W.float() for W in Ws]
        upd_bytes = weights * (2 * wbytes + 4 + 1.125)
        ub = sste.UpdateBatch(Wm, Gs, [1.48] * len(Wm), sste.BF16, vals=batch.vals, metas=batch.metas)
        ms = timed(lambda: ub.launch(0.0))
        out["update_fused_" + master] = {"ms": ms, "algorithmic_bytes": upd_bytes, "GB_per_s": upd_bytes / ms * 1e-6,
                                         "frac_hbm_peak": upd_bytes / ms * 1e-6 / PEAK_HBM_GBS}
        del Wm, ub
    return out


def extras(sste, torch, np, WL, cfg, layers, steps, grad_e5m2, dense_context, output_variants=True):
    """Figures that are not part of `value`: the layer's third GEMM (input gradient, dense by the paper's
    choice), the 8-bit operand casts, the flip rate of workload 4, the vendor's dense GEMM as context."""
    out = {}
    wl = WL.WORKLOADS[cfg]
    dgrad = {}
    for st in layers:
        dX = torch.empty((st.T, st.I), dtype=torch.bfloat16, device="cuda")
        for i in range(3):
            sste.linear_dgrad(st.dYs[i % st.nsets], st.vals, st.meta, st.I, st.gdt, st.dys, st.w_scale, dX=dX)
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        n = max(10, steps // 4)
        for i in range(n):
            sste.linear_dgrad(st.dYs[i % st.nsets], st.vals, st.meta, st.I, st.gdt, st.dys, st.w_scale, dX=dX)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - g0) * 1e3 / n
        dgrad[st.name] = {"ms": ms, "TFLOP_per_s": st.flops / (ms * 1e-3) * 1e-12,
                          "frac_dense_mfma_peak": st.flops / (ms * 1e-3) * 1e-12 / PEAK_DENSE_TFLOPS[wl.dtype]}
        del dX
    out["dgrad_dense"] = dgrad
    if wl.dtype == "e4m3":
        casts = {}
        T = wl.T
        for name, cols, fmt in (("X 32768x1280", 1280, sste.F8E4M3), ("dY 32768x5120", 5120, sste.F8E5M2 if grad_e5m2 else sste.F8E4M3)):
            src = torch.randn((T, cols), device="cuda", dtype=torch.float32).to(torch.bfloat16)
            q = torch.empty((T, cols), dtype=torch.uint8, device="cuda")
            amax = torch.empty(1, dtype=torch.float32, device="cuda")
            for _ in range(3):
                sste.cast_fp8(src, 0.01, fmt, Q=q, amax_out=amax)
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            for _ in range(20):
                sste.cast_fp8(src, 0.01, fmt, Q=q, amax_out=amax)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - c0) * 1e3 / 20
            casts[name] = {"ms": ms, "GB_per_s": T * cols * 3 / ms * 1e-6, "frac_hbm_peak": T * cols * 3 / ms * 1e-6 / PEAK_HBM_GBS}
            del src, q
        out["cast_fp8"] = casts
    if wl.dtype == "e4m3" and output_variants:
        # the forward product written as e4m3 where it is produced (Sec. 5.2: the next layer's operand), with its
        # largest magnitude, beside the bf16 output the step uses: half the output bytes
        outs = {}
        for st in layers:
            Z8 = torch.empty((st.T, st.O), dtype=torch.uint8, device="cuda")
            amax = torch.empty(1, dtype=torch.float32, device="cuda")

            def run8(i, st=st, Z8=Z8, amax=amax):
                sste.linear_fwd_ex(st.Xs[i % st.nsets], st.vals, st.meta, st.O, st.dt, st.xs, st.w_scale, sste.F8E4M3, 1.0,
                                   Z=Z8, amax_out=amax)

            def run16(i, st=st):
                sste.linear_fwd(st.Xs[i % st.nsets], st.vals, st.meta, st.O, st.dt, st.xs, st.w_scale, Z=st.Zs[i % st.nsets])
            row = {}
            for key, fn in (("bf16_out_ms", run16), ("e4m3_out_with_amax_ms", run8)):
                for i in range(3):
                    fn(i)
                torch.cuda.synchronize()
                f0 = time.perf_counter()
                for i in range(20):
                    fn(i)
                torch.cuda.synchronize()
                row[key] = (time.perf_counter() - f0) * 1e3 / 20
            row["e4m3_out_frac_sparse_mfma_peak"] = st.flops / (row["e4m3_out_with_amax_ms"] * 1e-3) * 1e-12 / (2 * PEAK_DENSE_TFLOPS[wl.dtype])
            outs[st.name] = row
            del Z8
        out["fwd_e4m3_output"] = outs
    if wl.cfg == 4:
        # workload 4: the dense weight moves a little every step and is re-projected with the frozen beta; the
        # fraction of positions whose kept / pruned state changes (flip rate, Sec. 3.3) is a sanity number
        st = layers[min(2, len(layers) - 1)]
        li = [l.name for l in wl.layers].index(st.name)

        def up(bits):
            return torch.from_numpy(np.ascontiguousarray(bits.view(np.int16))).cuda().view(torch.bfloat16)
        flips, w_bits = [], st.wb
        _, m_prev = sste.project_pack(up(w_bits), st.beta, st.dt, st.w_scale)
        for k in range(10):
            w_bits = WL.weight_update_bits(w_bits, wl, li, k)
            _, m_new = sste.project_pack(up(w_bits), st.beta, st.dt, st.w_scale)
            flips.append(int(sste.flip_count(m_prev, m_new, st.O).cpu()[0]) / float(st.O * st.I))
            m_prev = m_new
        out["flip_rate_per_step"] = {"layer": st.name, "rates": flips}
    if dense_context and wl.dtype == "bf16":
        ctx = {}
        for st in layers:
            def dense_us(fn, iters=30):
                for i in range(3):
                    fn(i)
                torch.cuda.synchronize()
                d0 = time.perf_counter()
                for i in range(iters):
                    fn(i)
                torch.cuda.synchronize()
                return (time.perf_counter() - d0) / iters * 1e6
            f_us = dense_us(lambda i: torch.matmul(st.Xs[i % st.nsets], st.W.t(), out=st.Zs[i % st.nsets]))
            w_us = dense_us(lambda i: torch.matmul(st.dYs[i % st.nsets].t(), st.Xs[i % st.nsets]))
            d_us = dense_us(lambda i: torch.matmul(st.dYs[i % st.nsets], st.W))
            ctx[st.name] = {"fwd_us": f_us, "wgrad_us": w_us, "dgrad_us": d_us}
        out["dense_context"] = {"library": "torch.matmul (bf16 in, bf16 out)", "layers": ctx}
    return out


def ffn_block(sste, torch, np, WL, cfg=4, iters=30):
    """One training step of a feed-forward block (fc1 -> GELU -> fc2; the block the paper's appendix times) through
    the library, bf16: re-projection of both weights, fc1 forward with the activation in its epilogue, fc2 forward,
    fc2 input gradient with the activation's derivative in its epilogue, both weight gradients, fc1 input gradient.
    Beside it, as context, the same block as dense torch.matmul + autograd on the same box."""
    wl = WL.WORKLOADS[cfg]
    names = [l.name for l in wl.layers]
    l1, l2 = wl.layers[names.index("fc1")], wl.layers[names.index("fc2")]
    T, d, h = wl.T, l1.I, l1.O

    def up(bits):
        return torch.from_numpy(np.ascontiguousarray(bits.view(np.int16))).cuda().view(torch.bfloat16)
    W1, W2 = up(WL.weight_bits(wl, names.index("fc1"))), up(WL.weight_bits(wl, names.index("fc2")))
    X = up(WL.activations(wl, names.index("fc1"))[0])
    dY = up(WL.output_gradient(wl, names.index("fc2"))[0])
    v1, m1 = sste.packed_buffers(h, d, sste.BF16, "cuda")
    v2, m2 = sste.packed_buffers(d, h, sste.BF16, "cuda")
    H = torch.empty((T, h), dtype=torch.bfloat16, device="cuda")
    A = torch.empty_like(H)
    Y = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
    dH = torch.empty_like(H)
    dX = torch.empty_like(X)
    dW1 = torch.empty((h, d), dtype=torch.float32, device="cuda")
    dW2 = torch.empty((d, h), dtype=torch.float32, device="cuda")
    ws1 = torch.empty(max(16, sste.wgrad_workspace_bytes(T, h, d, sste.BF16)), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty(max(16, sste.wgrad_workspace_bytes(T, d, h, sste.BF16)), dtype=torch.uint8, device="cuda")
    beta = 1.4830322

    def step(i):
        sste.project_pack(W1, beta, vals=v1, meta=m1)
        sste.project_pack(W2, beta, vals=v2, meta=m2)
        sste.linear_fwd_act(X, v1, m1, h, H=H, A=A)
        sste.linear_fwd(A, v2, m2, d, Z=Y)
        sste.linear_dgrad_act(dY, v2, m2, h, H, dX=dH)
        sste.linear_wgrad(dY, A, seed=cfg, offset=2 * i, dW=dW2, workspace=ws2)
        sste.linear_wgrad(dH, X, seed=cfg, offset=2 * i + 1, dW=dW1, workspace=ws1)
        sste.linear_dgrad(dH, v1, m1, d, dX=dX)

    def timed(fn, n):
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    ms = timed(step, iters)
    # the same products with the activation as separate passes (plain calls + torch elementwise ops): what the fusion saves
    def unfused(i):
        sste.project_pack(W1, beta, vals=v1, meta=m1)
        sste.project_pack(W2, beta, vals=v2, meta=m2)
        sste.linear_fwd(X, v1, m1, h, Z=H)
        torch.nn.functional.gelu(H, approximate="tanh")
        sste.linear_fwd(A, v2, m2, d, Z=Y)
        sste.linear_dgrad(dY, v2, m2, h, dX=dH)
        torch.ops.aten.gelu_backward(dH, H, approximate="tanh")
        sste.linear_wgrad(dY, A, seed=cfg, offset=2 * i, dW=dW2, workspace=ws2)
        sste.linear_wgrad(dH, X, seed=cfg, offset=2 * i + 1, dW=dW1, workspace=ws1)
        sste.linear_dgrad(dH, v1, m1, d, dX=dX)
    ms_unfused = timed(unfused, iters)

    Xr = X.clone().requires_grad_(True)
    W1r, W2r = W1.clone().requires_grad_(True), W2.clone().requires_grad_(True)

    def dense(i):
        Xr.grad = W1r.grad = W2r.grad = None
        out = torch.nn.functional.gelu(Xr @ W1r.t(), approximate="tanh") @ W2r.t()
        out.backward(dY)
    ms_dense = timed(dense, iters)
    flops = 6 * 2.0 * T * d * h                                  # six GEMMs of 2 T d h dense-equivalent flops
    return {"workload": "cfg%d FFN block: fc1 %dx%d, GELU, fc2 %dx%d, %d tokens, bf16" % (cfg, h, d, d, h, T),
            "ms_per_step": ms, "dense_equiv_TFLOP_per_s": flops / (ms * 1e-3) * 1e-12,
            "ms_per_step_activation_as_separate_passes": ms_unfused,
            "dense_context": {"library": "torch.matmul + torch gelu(tanh) + autograd, bf16", "ms_per_step": ms_dense,
                              "speedup_over_dense": ms_dense / ms}}


def ffn_block_fp8(sste, torch, np, WL, cfg=5, iters=20, grad_e5m2=True):
    """The same feed-forward step in the 8-bit recipe of Sec. 5.2 at workload 5's shapes: e4m3 weights and
    activations, e5m2 (or e4m3) gradients, per-tensor scales taken from a calibration pass and then held (delayed
    scaling: no value is read back inside the step).  X arrives as e4m3 (what the preceding layer's output stage
    writes), dY as bf16 and is cast inside the step; fc1's epilogue writes the pre-activation (bf16, for the
    backward pass) and the e4m3 activation; fc2's input-gradient epilogue applies the activation's derivative, and
    its bf16 result is cast once for the two products that consume it.  Context: the dense bf16 block in torch at
    the same shapes."""
    wl = WL.WORKLOADS[cfg]
    names = [l.name for l in wl.layers]
    l1 = wl.layers[names.index("fc1")]
    T, d, h = wl.T, l1.I, l1.O
    gfmt, gmax = (sste.F8E5M2, FMT_MAX["e5m2"]) if grad_e5m2 else (sste.F8E4M3, FMT_MAX["e4m3"])

    def up(bits):
        return torch.from_numpy(np.ascontiguousarray(bits.view(np.int16))).cuda().view(torch.bfloat16)

    def amax_of(t):
        return float(sste.cast_fp8(t, 1.0, sste.F8E4M3, store=False)[1].cpu()[0])
    W1, W2 = up(WL.weight_bits(wl, names.index("fc1"))), up(WL.weight_bits(wl, names.index("fc2")))
    Xb = up(WL.activations(wl, names.index("fc1"))[0])
    dYb = up(WL.output_gradient(wl, names.index("fc2"))[0])
    beta = 1.4830322
    f32 = lambda v: float(np.float32(v))
    # calibration pass (untimed): the scales a window of earlier iterations would have left behind
    xs = f32(amax_of(Xb) / 448.0)
    X8, _ = sste.cast_fp8(Xb, xs, sste.F8E4M3)
    del Xb
    am = torch.zeros(1, dtype=torch.float32, device="cuda")
    sste.project_pack(W1, beta, sste.BF16, 1.0, amax_out=am)
    ws1 = f32(float(am.cpu()[0]) / 448.0)
    sste.project_pack(W2, beta, sste.BF16, 1.0, amax_out=am)
    ws2 = f32(float(am.cpu()[0]) / 448.0)
    v1, m1 = sste.packed_buffers(h, d, sste.F8E4M3, "cuda")
    v2, m2 = sste.packed_buffers(d, h, sste.F8E4M3, "cuda")
    sste.project_pack(W1, beta, sste.F8E4M3, ws1, vals=v1, meta=m1)
    sste.project_pack(W2, beta, sste.F8E4M3, ws2, vals=v2, meta=m2)
    H = torch.empty((T, h), dtype=torch.bfloat16, device="cuda")
    A16 = torch.empty_like(H)
    sste.linear_fwd_act(X8, v1, m1, h, sste.F8E4M3, xs, ws1, H=H, A=A16)
    a_scale = f32(1.25 * amax_of(A16) / 448.0)
    del A16
    A8 = torch.empty((T, h), dtype=torch.uint8, device="cuda")
    dys = f32(1.25 * amax_of(dYb) / gmax)
    dY8 = torch.empty((T, d), dtype=torch.uint8, device="cuda")
    sste.cast_fp8(dYb, dys, gfmt, Q=dY8, amax_out=am)
    dH = torch.empty((T, h), dtype=torch.bfloat16, device="cuda")
    sste.linear_dgrad_act(dY8, v2, m2, h, H, gfmt, dys, ws2, dX=dH)
    dhs = f32(1.25 * amax_of(dH) / gmax)
    dH8 = torch.empty((T, h), dtype=torch.uint8, device="cuda")
    Y = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
    dW1 = torch.empty((h, d), dtype=torch.float32, device="cuda")
    dW2 = torch.empty((d, h), dtype=torch.float32, device="cuda")
    wsb1 = torch.empty(max(16, sste.wgrad_workspace_bytes(T, h, d, gfmt)), dtype=torch.uint8, device="cuda")
    wsb2 = torch.empty(max(16, sste.wgrad_workspace_bytes(T, d, h, gfmt)), dtype=torch.uint8, device="cuda")
    amaxes = [torch.zeros(1, dtype=torch.float32, device="cuda") for _ in range(3)]

    def step(i):
        sste.project_pack(W1, beta, sste.F8E4M3, ws1, vals=v1, meta=m1)
        sste.project_pack(W2, beta, sste.F8E4M3, ws2, vals=v2, meta=m2)
        sste.linear_fwd_act(X8, v1, m1, h, sste.F8E4M3, xs, ws1, a_dtype=sste.F8E4M3, a_scale=a_scale, H=H, A=A8, amax_out=amaxes[0])
        sste.linear_fwd(A8, v2, m2, d, sste.F8E4M3, a_scale, ws2, Z=Y)
        sste.cast_fp8(dYb, dys, gfmt, Q=dY8, amax_out=amaxes[1])
        sste.linear_dgrad_act(dY8, v2, m2, h, H, gfmt, dys, ws2, dX=dH)
        sste.cast_fp8(dH, dhs, gfmt, Q=dH8, amax_out=amaxes[2])
        sste.linear_wgrad(dY8, A8, seed=cfg, offset=2 * i, dtype=gfmt, dy_scale=dys, x_scale=a_scale, dW=dW2, workspace=wsb2)
        sste.linear_wgrad(dH8, X8, seed=cfg, offset=2 * i + 1, dtype=gfmt, dy_scale=dhs, x_scale=xs, dW=dW1, workspace=wsb1)
        sste.linear_dgrad(dH8, v1, m1, d, gfmt, dhs, ws1, dX=dX)

    def timed(fn, n):
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n
    ms = timed(step, iters)
    del H, A8, dH, dH8, dY8, Y, dX
    Xr = (X8.float() * xs).to(torch.bfloat16).requires_grad_(True)     # any bf16 data of the shape: the context is a timing
    W1r, W2r = W1.clone().requires_grad_(True), W2.clone().requires_grad_(True)

    def dense(i):
        Xr.grad = W1r.grad = W2r.grad = None
        out = torch.nn.functional.gelu(Xr @ W1r.t(), approximate="tanh") @ W2r.t()
        out.backward(dYb)
    ms_dense = timed(dense, max(5, iters // 2))
    flops = 6 * 2.0 * T * d * h
    return {"workload": "cfg%d FFN block: fc1 %dx%d, GELU, fc2 %dx%d, %d tokens, e4m3 weights and activations, %s gradients, held scales"
                        % (cfg, h, d, d, h, T, "e5m2" if grad_e5m2 else "e4m3"),
            "ms_per_step": ms, "dense_equiv_TFLOP_per_s": flops / (ms * 1e-3) * 1e-12,
            "dense_context": {"library": "torch.matmul + torch gelu(tanh) + autograd, bf16", "ms_per_step": ms_dense,
                              "speedup_over_dense_bf16": ms_dense / ms}}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2409_09099_amd as sste
    from paper_2409_09099_amd import workloads as WL

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    sste.library()
    traffic = hbm_traffic_table()
    events = not args.no_kernel_timing

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    head, layers = measure(sste, torch, np, WL, args.config, args.layer, args.steps, args.warmup, args.sets,
                           args.grad_e5m2, events, traffic)
    wl = WL.WORKLOADS[args.config]
    out = {
        "metric": "S-STE 2:4 linear fwd+wgrad TFLOP/s (dense-equivalent, project+pack inside the step)",
        "value": head["value"],
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": head["workload"], "tokens": wl.T, "buffer_sets": head["buffer_sets"],
                   "grad_format": "e5m2" if (args.grad_e5m2 and wl.dtype == "e4m3") else wl.dtype},
    }
    for k in ("ms_per_step_median_of_chunks", "ms_per_step_min_of_chunks", "ms_per_step_cache_warm", "host_enqueue_ms_per_step",
              "ms_per_step_with_kernel_events", "frac_sparse_mfma_peak_whole_step", "kernels", "layers", "roofline", "roofline_row"):
        if k in head:
            out[k] = head[k]
    out.update(extras(sste, torch, np, WL, args.config, layers, args.steps, args.grad_e5m2, args.dense_context,
                      output_variants=not args.no_secondary))
    del layers
    torch.cuda.empty_cache()

    if not args.no_secondary and args.layer < 0 and args.config == 5:
        secondary = {}
        for cfg in (4, 3, 2):
            sec, sl = measure(sste, torch, np, WL, cfg, -1, max(20, args.steps // 2), args.warmup, 0, False, events, traffic)
            del sl
            torch.cuda.empty_cache()
            secondary["cfg%d" % cfg] = sec
        out["secondary"] = secondary
    if not args.no_secondary:
        out["ffn_block"] = ffn_block(sste, torch, np, WL)
        torch.cuda.empty_cache()
        out["ffn_block_fp8"] = ffn_block_fp8(sste, torch, np, WL)
        torch.cuda.empty_cache()
    if not args.no_prune_model:
        out["prune_pack_model"] = prune_model(sste, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(np, WL, args.config)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
