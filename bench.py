#!/usr/bin/env python3
"""Benchmark of the S-STE 2:4 sparse linear-layer hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
  project + scale + pack of W  ->  forward sparse GEMM  ->  MVUE weight-gradient sparse GEMM.
The default workload is the GPT-2-124M FFN fc1 layer (W 3072 x 768, 8192 tokens, bf16).
Prints ONE JSON line.  `value` = dense-equivalent TFLOP/s of forward + weight gradient
(2 * 2*T*I*O flops per step) over the whole step time, pruning included.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# published MI355X peaks
PEAK_HBM_GBS = 8000.0
PEAK_DENSE_TFLOPS = {"bf16": 2500.0, "e4m3": 5000.0}

# HBM bytes per launch on the headline workload, from two rocprofv3 --pmc runs of this file (FETCH_SIZE
# scaled by 2.000, WRITE_SIZE by 1.000: what a plain 256 MiB copy reads on the same counters); the
# summary with the commands is committed under profiles/.  KiB read + KiB written.
HBM_TRAFFIC_KIB = {
    (2, "project_pack"): 4658 + 2592,
    (2, "fwd"): 42304 + 49211,
    (2, "mvue_pack"): 49246 + 27648,
    (2, "wgrad"): 67784 + 36887,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="workload number (1-5); 2 is the headline one")
    ap.add_argument("--layer", type=int, default=0, help="layer index inside the workload")
    ap.add_argument("--sets", type=int, default=4, help="activation buffer sets rotated over steps (1 = cache-warm)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--grad-e5m2", action="store_true",
                    help="8-bit workloads: output gradients in e5m2 (the paper's backward format) instead of e4m3")
    ap.add_argument("--dense-context", action="store_true",
                    help="also time the vendor dense bf16 GEMM (torch.matmul) on the same shapes: context, not the product")
    ap.add_argument("--no-prune-model", action="store_true",
                    help="skip the whole-model re-projection measurement (144 weight tensors of GPT-2-774M, 2.2 GB)")
    ap.add_argument("--no-kernel-timing", action="store_true", help="do not bracket kernels with events (debug)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 256 MiB device copies before the warm-up (reference for HBM byte counters)")
    return ap.parse_args()


def cpu_baseline(wl, layer, wb, xc, xs, dyc, dys, beta32, grad_e5m2=False):
    """Times the oracle, as it stands, on one full step of the same workload (host cores)."""
    import numpy as np
    from oracle import linear as OL
    from oracle import projection as OP
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    L = wl.layers[layer]
    t0 = time.perf_counter()
    if wl.dtype == "bf16":
        rv, rm, _ = OP.project_pack(wb, beta32)
        ws = np.float32(1.0)
    else:
        _, _, amax = OP.project_pack(wb, beta32)
        ws = np.float32(float(amax) / 448.0)
        rv, rm, _ = OP.project_pack(wb, beta32, "e4m3", ws)
    t1 = time.perf_counter()
    OL.linear_fwd(xc, rv, rm, wl.dtype, xs, ws)
    t2 = time.perf_counter()
    OL.linear_wgrad(dyc, xc, 0, 0, "e5m2" if grad_e5m2 else wl.dtype, dys, xs, x_dtype=wl.dtype)
    t3 = time.perf_counter()
    flops = 2 * 2.0 * wl.T * L.I * L.O
    return {
        "value": flops / (t3 - t0) * 1e-12,
        "unit": "TFLOP/s",
        "cores": int(cores),
        "kind": "oracle",
        "sample": "one full step of the same workload (project+pack %.2fs, fwd %.2fs, MVUE+wgrad %.2fs)" % (t1 - t0, t2 - t1, t3 - t2),
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

    wl = WL.WORKLOADS[args.config]
    L = wl.layers[args.layer]
    T, O, I = wl.T, L.O, L.I
    fp8 = wl.dtype == "e4m3"
    dt = sste.F8E4M3 if fp8 else sste.BF16
    esize = 1 if fp8 else 2

    # ---- seeded synthetic inputs, generated on the host and made resident in HBM before timing
    wb = WL.weight_bits(wl, args.layer)
    xc, xs = WL.activations(wl, args.layer)
    grad_e5m2 = bool(args.grad_e5m2 and fp8)
    dyc, dys = WL.output_gradient(wl, args.layer, e5m2=grad_e5m2)
    gdt = sste.F8E5M2 if grad_e5m2 else dt           # format of dY in the backward calls

    def up(a):
        t = torch.from_numpy(np.ascontiguousarray(a.view(np.int16) if a.dtype == np.uint16 else a)).cuda()
        return t.view(torch.bfloat16) if a.dtype == np.uint16 else t

    W = up(wb)
    nsets = max(1, args.sets)
    Xs = [up(xc)] + [up(xc).clone() for _ in range(nsets - 1)]
    dYs = [up(dyc)] + [up(dyc).clone() for _ in range(nsets - 1)]
    Zs = [torch.empty((T, O), dtype=torch.bfloat16, device="cuda") for _ in range(nsets)]
    dWs = [torch.empty((O, I), dtype=torch.float32, device="cuda") for _ in range(nsets)]
    vals, meta = sste.packed_buffers(O, I, dt, "cuda")
    ws_bytes = sste.wgrad_workspace_bytes(T, O, I, dt)
    wss = [torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda") for _ in range(nsets)]

    # beta: computed once from the initial weights, then frozen (paper Sec. 4.2)
    beta = float(sste.compute_beta(W).cpu()[0])
    if fp8:
        amax = torch.zeros(1, dtype=torch.float32, device="cuda")
        sste.project_pack(W, beta, sste.BF16, 1.0, amax_out=amax)
        w_scale = float(amax.cpu()[0]) / 448.0
    else:
        w_scale = 1.0

    def step(i):
        s = i % nsets
        sste.project_pack(W, beta, dt, w_scale, vals=vals, meta=meta)
        sste.linear_fwd(Xs[s], vals, meta, O, dt, float(xs), w_scale, Z=Zs[s])
        sste.linear_wgrad(dYs[s], Xs[s], seed=args.config, offset=i, dtype=gdt, dy_scale=float(dys), x_scale=float(xs),
                          dW=dWs[s], workspace=wss[s])

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps between two synchronisations -> `value`
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    t_enq = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    # ---- the same K steps again, every hot kernel bracketed by its own HIP event pair -> per-kernel
    # durations and the roofline.  The event pairs serialise the queue (about 8 us per launch on this
    # box), so this pass is slower per step than the one above and is not what `value` is quoted on.
    ms_per_step_events = float("nan")
    if not args.no_kernel_timing:
        sste.timing_begin(8 * args.steps + 16)
        torch.cuda.synchronize()
        e0 = time.perf_counter()
        for i in range(args.steps):
            step(args.warmup + args.steps + i)
        torch.cuda.synchronize()
        ms_per_step_events = (time.perf_counter() - e0) * 1e3 / args.steps
        kt = sste.timing_end()
    else:
        kt = {k: (float("nan"), 1) for k in sste.binding.KERNEL_NAMES}

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    gemm_flops = 2.0 * T * I * O                 # dense-equivalent flops of one GEMM
    value = 2 * gemm_flops / (ms_per_step * 1e-3) * 1e-12

    def avg_ms(name):
        ms, n = kt[name]
        return ms / n if n else float("nan")

    pp_bytes = O * I * (2 + esize / 2 + 0.125)   # algorithmic bytes: read W, write values + metadata
    kernels = {
        "project_pack": {"ms": avg_ms("project_pack"), "GB_per_s": pp_bytes / (avg_ms("project_pack") * 1e-3) * 1e-9,
                         "frac_hbm_peak": pp_bytes / (avg_ms("project_pack") * 1e-3) * 1e-9 / PEAK_HBM_GBS},
        "fwd": {"ms": avg_ms("fwd"), "dense_equiv_TFLOP_per_s": gemm_flops / (avg_ms("fwd") * 1e-3) * 1e-12},
        "wgrad": {"ms": avg_ms("wgrad"), "dense_equiv_TFLOP_per_s": gemm_flops / (avg_ms("wgrad") * 1e-3) * 1e-12},
        "wgrad_reduce": {"ms": avg_ms("wgrad_reduce")},
    }
    if kt["mvue_pack"][1]:
        mv_bytes = T * O * esize * (1 + 0.5 + 0.0625)          # read dY, write packed values + position bits
        kernels["mvue_pack"] = {"ms": avg_ms("mvue_pack"), "GB_per_s": mv_bytes / (avg_ms("mvue_pack") * 1e-3) * 1e-9,
                                "frac_hbm_peak": mv_bytes / (avg_ms("mvue_pack") * 1e-3) * 1e-9 / PEAK_HBM_GBS}
    wgrad_total_ms = sum(kernels[k]["ms"] for k in ("wgrad", "wgrad_reduce", "mvue_pack") if k in kernels and kernels[k]["ms"] == kernels[k]["ms"])
    kernels["wgrad_all"] = {"ms": wgrad_total_ms, "dense_equiv_TFLOP_per_s": gemm_flops / (max(wgrad_total_ms, 1e-9) * 1e-3) * 1e-12}
    for k in ("fwd", "wgrad"):
        kernels[k]["frac_sparse_mfma_peak"] = kernels[k]["dense_equiv_TFLOP_per_s"] / (2 * PEAK_DENSE_TFLOPS[wl.dtype])

    # roofline of the dominant kernel.  The sparse MFMA executes half of the dense-equivalent
    # multiply-adds: algorithmic flops per launch = T*I*O (I/2 MACs per output element), held against
    # the published dense MFMA peak of the operand type.
    dom = max([k for k in ("project_pack", "fwd", "wgrad", "mvue_pack") if k in kernels], key=lambda k: kernels[k]["ms"])
    if dom in ("project_pack", "mvue_pack"):
        achieved = kernels[dom]["GB_per_s"]
        roofline = {"kernel": dom, "bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": achieved / PEAK_HBM_GBS, "traffic": None}
    else:
        achieved = 0.5 * gemm_flops / (kernels[dom]["ms"] * 1e-3) * 1e-12
        peak = PEAK_DENSE_TFLOPS[wl.dtype]
        roofline = {"kernel": dom, "bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                    "frac": achieved / peak, "traffic": None}
    roofline["avg_launch_ms"] = kernels[dom]["ms"]
    kib = HBM_TRAFFIC_KIB.get((wl.cfg, dom)) if args.layer == 0 else None
    roofline["traffic"] = kib * 1024 if kib is not None else None

    out = {
        "metric": "S-STE 2:4 linear fwd+wgrad TFLOP/s (dense-equivalent, project+pack inside the step)",
        "value": value,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "host_enqueue_ms_per_step": (t_enq - t0) * 1e3 / args.steps,
        "ms_per_step_with_kernel_events": ms_per_step_events,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": wl.dtype if fp8 else "bf16",
        "data": "synthetic",
        "config": {"workload": "cfg%d %s layer %s (W %dx%d, %d tokens)" % (wl.cfg, wl.name, L.name, O, I, T),
                   "buffer_sets": nsets, "wgrad_workspace_bytes": int(ws_bytes),
                   "grad_format": "e5m2" if grad_e5m2 else wl.dtype},
        "frac_sparse_mfma_peak_whole_step": value / (2 * PEAK_DENSE_TFLOPS[wl.dtype]),
        "kernels": kernels,
        "roofline": roofline,
    }
    if True:
        # the layer's third GEMM, grad_X = grad_Z S(W): dense by the paper's choice, not part of `value`
        dXs = [torch.empty((T, I), dtype=torch.bfloat16, device="cuda") for _ in range(nsets)]
        for i in range(5):
            sste.linear_dgrad(dYs[i % nsets], vals, meta, I, gdt, float(dys), w_scale, dX=dXs[i % nsets])
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for i in range(args.steps):
            sste.linear_dgrad(dYs[i % nsets], vals, meta, I, gdt, float(dys), w_scale, dX=dXs[i % nsets])
        torch.cuda.synchronize()
        dg_ms = (time.perf_counter() - g0) * 1e3 / args.steps
        out_dgrad = {"ms": dg_ms, "TFLOP_per_s": gemm_flops / (dg_ms * 1e-3) * 1e-12, "frac_dense_mfma_peak": gemm_flops / (dg_ms * 1e-3) * 1e-12 / PEAK_DENSE_TFLOPS[wl.dtype]}
        del dXs
    if fp8:
        # operand preparation of the 8-bit path: per-tensor rescale + cast of bf16 X and dY (3 B per element)
        casts = {}
        for name, rows, cols, fmt in (("X", T, I, sste.F8E4M3), ("dY", T, O, gdt if grad_e5m2 else sste.F8E4M3)):
            src = torch.randn((rows, cols), device="cuda", dtype=torch.float32).to(torch.bfloat16)
            q = torch.empty((rows, cols), dtype=torch.uint8, device="cuda")
            amax = torch.empty(1, dtype=torch.float32, device="cuda")
            for _ in range(3):
                sste.cast_fp8(src, 0.01, fmt, Q=q, amax_out=amax)
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            for _ in range(20):
                sste.cast_fp8(src, 0.01, fmt, Q=q, amax_out=amax)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - c0) * 1e3 / 20
            casts[name] = {"ms": ms, "GB_per_s": rows * cols * 3 / ms * 1e-6, "frac_hbm_peak": rows * cols * 3 / ms * 1e-6 / PEAK_HBM_GBS}
            del src, q
        out["cast_fp8"] = casts
    if args.dense_context and not fp8:
        # what the vendor's dense GEMM reaches on the same layer (forward Z = X W^T; weight gradient dY^T X)
        def dense_us(fn, iters=50):
            for i in range(5):
                fn(i)
            torch.cuda.synchronize()
            d0 = time.perf_counter()
            for i in range(iters):
                fn(i)
            torch.cuda.synchronize()
            return (time.perf_counter() - d0) / iters * 1e6
        f_us = dense_us(lambda i: torch.matmul(Xs[i % nsets], W.t(), out=Zs[i % nsets]))
        w_us = dense_us(lambda i: torch.matmul(dYs[i % nsets].t(), Xs[i % nsets]))
        d_us = dense_us(lambda i: torch.matmul(dYs[i % nsets], W))
        out["dense_context"] = {"library": "torch.matmul (bf16 in, bf16 out)", "fwd_us": f_us, "fwd_TFLOP_per_s": gemm_flops / f_us * 1e-6,
                                "wgrad_us": w_us, "wgrad_TFLOP_per_s": gemm_flops / w_us * 1e-6,
                                "dgrad_us": d_us, "dgrad_TFLOP_per_s": gemm_flops / d_us * 1e-6}
    if out_dgrad is not None:
        out["dgrad_dense"] = out_dgrad
    if wl.cfg == 4:
        # workload 4: the dense weight moves a little every step and is re-projected with the frozen beta;
        # the fraction of positions whose kept / pruned state changes (flip rate, paper Sec. 3.3) is a sanity number
        flips, w_bits = [], wb
        v_prev, m_prev = sste.project_pack(up(w_bits), beta, dt, w_scale)
        for k in range(10):
            w_bits = WL.weight_update_bits(w_bits, wl, args.layer, k)
            v_new, m_new = sste.project_pack(up(w_bits), beta, dt, w_scale)
            flips.append(int(sste.flip_count(m_prev, m_new, O).cpu()[0]) / float(O * I))
            m_prev = m_new
        out["flip_rate_per_step"] = flips
    if not args.no_prune_model:
        out["prune_pack_model"] = prune_model(sste, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, args.layer, wb, xc, xs, dyc, dys, np.float32(beta), grad_e5m2)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
