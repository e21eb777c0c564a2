#!/usr/bin/env python3
"""Benchmark of the TWN hot path on one MI355X.

A step is one pass of the whole hot path over one batch of the VGG-7 / CIFAR
workload (batch 128, bf16 activations): ternarize all 8 weight tensors
(Delta, alpha, 2-bit codes and the transposed copy), forward every conv / FC
layer with the fused scale-shift-ReLU tail, then the straight-through backward
of every layer (dX and dW on two streams, they are independent of each other).  Inputs are seeded synthetic tensors already
resident in HBM.  Prints ONE JSON line on stdout; per-layer detail goes to stderr.
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # dense bf16 MFMA, MI355X
PEAK_HBM_GBPS = 8000.0
# HBM-side bytes per launch of the roofline sample (L2 fills + write-backs, rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE scaled by a 1 GiB copy), taken from profiles/vgg7_b128_step_kernels.txt; it is a property of
# the committed kernels and tile choices at this workload, re-measured whenever those change.
ROOFLINE_SAMPLE_TRAFFIC_BYTES = 33194744
F = 0.7


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-extras", action="store_true", help="skip the GEMM / ternarize-2^28 / ResNet-18 side measurements")
    ap.add_argument("--cpu-batch", type=int, default=128)
    ap.add_argument("--only", choices=["gemm", "ternarize", "resnet18"], default=None,
                    help="run one side measurement alone (used for the rocprofv3 summaries in profiles/)")
    ap.add_argument("--variants", action="store_true", help="with --only gemm: also time the comparison weight formats")
    ap.add_argument("--graph", action="store_true", help="also capture the step into a HIP graph and time its replay")
    ap.add_argument("--eager-backward", action="store_true", help="launch the backward eagerly instead of replaying its HIP graph")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1")

    import numpy as np
    import torch

    from paper_1605_04711_amd import api
    from paper_1605_04711_amd import workloads as wl

    if not os.path.exists(api.library_path()):
        from paper_1605_04711_amd import build as b
        b.build()
    api.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    def dev_bf16(a):
        return torch.from_numpy(wl.f32_to_bf16_bits(a).view(np.int16)).to(dev).view(torch.bfloat16).reshape(a.shape)

    def time_call(fn, reps=10, warm=2):
        for _ in range(warm):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps


    def side_gemm():
        # stand-alone GEMM: X [8192 x 4096] bf16, W [4096 x 4096] N(0, 0.02^2)
        g = wl.gemm_config()
        gx = dev_bf16(wl.normal(3, wl.IDX_INPUT, (g.N, g.C)))
        gw = torch.from_numpy(wl.normal(3, 1, (g.O, g.C), std=0.02)).to(dev)
        gtw = api.twn_ternarize(gw, F)
        gy = torch.empty((g.N, g.O), dtype=torch.bfloat16, device=dev)
        t = time_call(lambda: api.twn_gemm_fwd(gx, gtw, out=gy), reps=300, warm=100)
        log("gemm 8192x4096x4096: %.1f us, %.1f TFLOP/s-eq" % (t * 1e3, g.flops / t / 1e9))
        res = {"us": round(t * 1e3, 1), "tflops": round(g.flops / t / 1e9, 1),
               "frac_mfma_peak": round(g.flops / t / 1e9 / PEAK_BF16_TFLOPS, 4)}
        if args.only == "gemm" and not args.variants:
            return res
        # The two comparison variants live in the register-staged 128x128 kernel only; the product format is
        # timed in that same kernel (TWN_TILE=4 selects it) so that only the weight format differs.
        os.environ["TWN_TILE"] = "4"
        same = {"postscale_2bit": time_call(lambda: api.twn_gemm_fwd(gx, gtw, out=gy), reps=60, warm=20)}
        del os.environ["TWN_TILE"]
        for name, var in (("alpha_at_expansion_2bit", api.TWN_VAR_BF16_ALPHA_LDS),
                          ("int8_stored", api.TWN_VAR_I8_STORED_POSTSCALE)):
            same[name] = time_call(lambda: api.twn_gemm_fwd(gx, gtw, out=gy, variant=var), reps=60, warm=20)
        for k, v in same.items():
            log("gemm weight format %-24s %.1f us, %.1f TFLOP/s-eq (register-staged 128x128 kernel)" % (k, v * 1e3, g.flops / v / 1e9))
        res["weight_formats_same_kernel_us"] = {k: round(v * 1e3, 1) for k, v in same.items()}
        return res

    def side_ternarize(calibrate=False):
        # ternarize-only: 2^28 float32 N(0,1) shaped [16384][16384]
        rows = 1 << 14
        big = torch.from_numpy(wl.normal(3, 0, (rows, rows))).to(dev)
        ws = torch.empty(1 << 17, dtype=torch.uint8, device=dev)
        if calibrate:
            # plain copy of known size (1 GiB read + 1 GiB written): calibrates the HBM byte counters
            dst = torch.empty_like(big)
            for _ in range(3):
                dst.copy_(big)
            torch.cuda.synchronize()
            del dst
        btw = api.twn_ternarize(big, F)
        t = time_call(lambda: api.twn_ternarize(big, F, out=btw, workspace=ws), reps=100, warm=20)
        nbytes = (1 << 28) * 8.25
        log("ternarize 2^28: %.1f us, %.1f GB/s algorithmic (8.25 B/weight)" % (t * 1e3, nbytes / t / 1e6))
        return {"us": round(t * 1e3, 1), "GBps": round(nbytes / t / 1e6, 1),
                "frac_hbm_peak": round(nbytes / t / 1e6 / PEAK_HBM_GBPS, 4)}

    def side_resnet18():
        # ResNet-18, batch 64: forward (per-layer synthetic inputs, fused scale/shift/ReLU tail) and STE backward
        rl = wl.resnet18(64)
        tot = 0.0
        tot_b = 0.0
        for li, L in enumerate(rl):
            x = dev_bf16(wl.normal(2, wl.IDX_INPUT + li, L.x_shape))
            tw = api.twn_ternarize(torch.from_numpy(wl.kaiming_weights(2, li, L)).to(dev), F)
            y = torch.empty(L.y_shape, dtype=torch.bfloat16, device=dev)
            sc = torch.ones(L.O, dtype=torch.float32, device=dev)
            sf = torch.zeros(L.O, dtype=torch.float32, device=dev)
            st, pd, dl = (L.stride,) * 2, (L.pad,) * 2, (L.dil,) * 2
            ws = torch.empty(max(16, api.twn_conv2d_fwd_workspace_bytes(L.x_shape, tw, st, pd, dl)), dtype=torch.uint8,
                             device=dev)
            t = time_call(lambda: api.twn_conv2d_fwd(x, tw, st, pd, dl, scale=sc, shift=sf, relu=True, out=y,
                                                     workspace=ws), reps=100, warm=20)
            tot += t
            # straight-through backward of the same layer (serial: data gradient, then weight gradient)
            twt = api.twn_ternarize(torch.from_numpy(wl.kaiming_weights(2, li, L)).to(dev), F, transposed=True)
            dy = dev_bf16(wl.normal(2, wl.IDX_DY + 10 * li, L.y_shape))
            wsb_ = torch.empty(max(16, api.twn_conv2d_bwd_ste_workspace_bytes(L.x_shape, twt, st, pd, dl)),
                               dtype=torch.uint8, device=dev)
            dxo = torch.empty(L.x_shape, dtype=torch.bfloat16, device=dev)
            dwo = torch.empty(L.w_shape, dtype=torch.float32, device=dev)
            tb = time_call(lambda: api.twn_conv2d_bwd_ste(x, dy, twt, st, pd, dl, need_dx=(li > 0), need_dw=True, dX=dxo,
                                                          dW=dwo, workspace=wsb_), reps=50, warm=10)
            tot_b += tb
            log("resnet18 %-12s %24s %9.1f us %8.1f TFLOP/s-eq | bwd %8.1f us" % (L.name, str(L.gemm_mnk), t * 1e3,
                                                                                L.flops / t / 1e9, tb * 1e3))
            del x, y, dy, dxo, dwo, wsb_
        rflops = sum(L.flops for L in rl)
        log("resnet18 b64 conv/fc layers: fwd %.3f ms, %.0f img/s; STE backward (dX + dW, serial) %.3f ms" %
            (tot, 64 / (tot * 1e-3), tot_b))
        return {"ms": round(tot, 4), "img_per_s": round(64 / (tot * 1e-3), 1), "tflops": round(rflops / tot / 1e9, 1),
                "frac_mfma_peak": round(rflops / tot / 1e9 / PEAK_BF16_TFLOPS, 4), "bwd_serial_ms": round(tot_b, 4)}

    if args.only:
        res = {"gemm": side_gemm, "ternarize": lambda: side_ternarize(calibrate=True), "resnet18": side_resnet18}[args.only]()
        print(json.dumps({"only": args.only, **res}), flush=True)
        return

    # ---------------- workload: VGG-7, batch 128 ----------------
    CFG = 1
    layers = wl.vgg7(128)
    W, X, dY, Y, dX, dW, tws, wsb, wsw, scale, shift = [], [], [], [], [], [], [], [], [], [], []
    tern_ws = None
    for li, L in enumerate(layers):
        w = wl.kaiming_weights(CFG, li, L)
        W.append(torch.from_numpy(w).to(dev))
        X.append(dev_bf16(wl.normal(CFG, wl.IDX_INPUT + li, L.x_shape)))
        dY.append(dev_bf16(wl.normal(CFG, wl.IDX_DY + 10 * li, L.y_shape)))
        Y.append(torch.empty(L.y_shape, dtype=torch.bfloat16, device=dev))
        dX.append(torch.empty(L.x_shape, dtype=torch.bfloat16, device=dev) if li > 0 else None)
        dW.append(torch.empty(L.w_shape, dtype=torch.float32, device=dev))
        scale.append(torch.ones(L.O, dtype=torch.float32, device=dev))
        shift.append(torch.zeros(L.O, dtype=torch.float32, device=dev))
        tws.append(api.twn_ternarize(W[li], F, transposed=True))
        nws = max(16, api.twn_conv2d_bwd_ste_workspace_bytes(L.x_shape, tws[li], (L.stride,) * 2, (L.pad,) * 2,
                                                             (L.dil,) * 2))
        wsb.append(torch.empty(nws, dtype=torch.uint8, device=dev))      # backward-data (split-K partials)
        wsw.append(torch.empty(nws, dtype=torch.uint8, device=dev))      # backward-weight (split partials)
    tern_ws = torch.empty(api.lib().twn_ternarize_batch_workspace_bytes(len(layers)), dtype=torch.uint8, device=dev)
    geo = [((L.stride,) * 2, (L.pad,) * 2, (L.dil,) * 2) for L in layers]
    wsf = [torch.empty(max(16, api.twn_conv2d_fwd_workspace_bytes(L.x_shape, tws[li], *geo[li])), dtype=torch.uint8,
                       device=dev) for li, L in enumerate(layers)]

    flops_fwd = sum(L.flops for L in layers)
    flops_dx = sum(L.flops for L in layers[1:])
    flops_dw = flops_fwd
    flops_step = flops_fwd + flops_dx + flops_dw
    tern_bytes = sum(L.n_weights for L in layers) * 8.5      # two reads + two 2-bit copies

    # One step.  Main stream: ONE multi-tensor ternarize call (three launches for the eight tensors), then the
    # forward of every layer.  Backward: the data gradients and the weight gradients of a layer do not depend
    # on each other (nor do the weight gradients of different layers), so they run on side streams forked from
    # the main stream after the forward and joined at
    # the end (the tail of one kernel is filled by the other stream's work).  `calls` lists every library
    # call as (phase, layer index, callable(stream)); the one-tensor ternarize entry point is timed per
    # layer in the detail pass below.
    calls = [("ternarize", 0, lambda st_=None: api.twn_ternarize_batch(W, F, transposed=True, out=tws, workspace=tern_ws))]
    tern_single = [lambda li=li: api.twn_ternarize(W[li], F, transposed=True, out=tws[li], workspace=tern_ws)
                   for li in range(len(layers))]
    for li in range(len(layers)):
        st, pd, dl = geo[li]
        calls.append(("fwd", li, lambda st_=None, li=li, st=st, pd=pd, dl=dl: api.twn_conv2d_fwd(
            X[li], tws[li], st, pd, dl, scale=scale[li], shift=shift[li], relu=True, out=Y[li], workspace=wsf[li])))
    n_main = len(calls)
    for li in range(len(layers) - 1, 0, -1):
        st, pd, dl = geo[li]
        calls.append(("bwd_data", li, lambda st_=None, li=li, st=st, pd=pd, dl=dl: api.twn_conv2d_bwd_ste(
            None, dY[li], tws[li], st, pd, dl, need_dx=True, need_dw=False, dX=dX[li], x_shape=layers[li].x_shape,
            workspace=wsb[li], stream=st_)))
    for li in range(len(layers) - 1, -1, -1):
        st, pd, dl = geo[li]
        calls.append(("bwd_weight", li, lambda st_=None, li=li, st=st, pd=pd, dl=dl: api.twn_conv2d_bwd_ste(
            X[li], dY[li], tws[li], st, pd, dl, need_dx=False, need_dw=True, dW=dW[li], workspace=wsw[li], stream=st_)))
    dx_calls = [c for c in calls if c[0] == "bwd_data"]
    dw_calls = [c for c in calls if c[0] == "bwd_weight"]
    # default priority; the weight gradients of different layers are independent too, so they alternate between
    # two streams: the reduction pass of one layer overlaps the main pass of the next
    side_a, side_b, side_c = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    n_dw_streams = int(os.environ.get("TWN_BENCH_DW_STREAMS", "2"))

    def backward():
        cur = torch.cuda.current_stream()
        fork = torch.cuda.Event()
        fork.record(cur)
        sides = [side_a, side_b] + ([side_c] if n_dw_streams > 1 else [])
        for st_ in sides:
            st_.wait_event(fork)
        # interleave the launches layer by layer so no stream runs ahead of the host
        for i in range(len(dw_calls)):
            if i < len(dx_calls):
                dx_calls[i][2](side_a)
            dw_calls[i][2](side_c if (n_dw_streams > 1 and i % 2) else side_b)
        for st_ in sides:
            j = torch.cuda.Event()
            j.record(st_)
            cur.wait_event(j)

    bwd_graph = None

    def one_step(marks=None):
        for ci in range(n_main):
            if marks is not None and ci in marks:
                marks[ci].record()
            calls[ci][2]()
        if marks is not None and n_main in marks:
            marks[n_main].record()
        if bwd_graph is not None:
            bwd_graph.replay()
        else:
            backward()

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()

    # The backward (27 launches on three streams) is captured once into a HIP graph and replayed in every step:
    # the library only launches kernels and takes its workspaces from the caller, so it captures as is.  The
    # forward stays eager because the roofline events sit between its launches.  Replays are checked against
    # the eager results (bit for bit) before they are used.
    def capture_backward():
        outs_b = [t for t in dX[1:]] + list(dW)
        ref_b = [t.clone() for t in outs_b]
        cap = torch.cuda.Stream()
        cap.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(cap):
            backward()
        torch.cuda.synchronize()
        g_ = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_, stream=cap):
            backward()
        torch.cuda.synchronize()
        for _ in range(2):
            for t in outs_b:
                t.zero_()
            calls[1][2]()                  # eager work between two replays
            torch.cuda.synchronize()
            g_.replay()
            torch.cuda.synchronize()
            if not all(torch.equal(a, b) for a, b in zip(ref_b, outs_b)):
                return None
        return g_

    if not args.eager_backward:
        try:
            bwd_graph = capture_backward()
        except RuntimeError as e:          # capture not available: the step runs eagerly
            log("backward graph capture failed (%s): eager backward" % str(e).splitlines()[0])
            bwd_graph = None
            torch.cuda.synchronize()
        if bwd_graph is None:
            log("backward runs eagerly (no graph)")
        for _ in range(args.warmup):
            one_step()
        torch.cuda.synchronize()

    # Timed region.  HIP events on the launch stream (torch's current stream) bracket each forward call that is
    # exactly one launch of the contraction kernel (the roofline sample: forward c2-c6, which run alone on
    # the GPU); phases and the per-layer table are taken in separate passes afterwards.
    name_of = [L.name for L in layers]
    single = {("fwd", n) for n in ("c2", "c3", "c4", "c5", "c6")}
    is_single = [(c[0], name_of[c[1]]) in single for c in calls]

    def new_ev():
        return torch.cuda.Event(enable_timing=True)

    # An event between two launches costs several microseconds of idle GPU, so the timed region records only
    # two per step: before the first and after the last call of the run of consecutive single-launch calls.
    first_single = min(ci for ci in range(n_main) if is_single[ci])
    last_single = max(ci for ci in range(n_main) if is_single[ci])
    assert all(is_single[ci] for ci in range(first_single, last_single + 1))
    marks = [first_single, last_single + 1]
    mev = [{ci: new_ev() for ci in marks} for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        one_step(mev[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    span_ms = sum(mev[s][first_single].elapsed_time(mev[s][last_single + 1]) for s in range(args.steps)) / args.steps
    single_calls = list(range(first_single, last_single + 1))

    # phase times: a second pass with one event pair per phase (the two backward streams form one phase)
    phase_names = ["ternarize", "fwd", "bwd_two_streams"]
    NPH = max(5, min(50, args.steps))
    pev = [[new_ev() for _ in range(4)] for _ in range(NPH)]
    for s in range(NPH):
        pev[s][0].record()
        calls[0][2]()
        pev[s][1].record()
        for ci in range(1, n_main):
            calls[ci][2]()
        pev[s][2].record()
        if bwd_graph is not None:
            bwd_graph.replay()
        else:
            backward()
        pev[s][3].record()
    torch.cuda.synchronize()
    phase_ms = [sum(pev[s][i].elapsed_time(pev[s][i + 1]) for s in range(NPH)) / NPH for i in range(3)]
    value = flops_step / (ms_per_step * 1e-3) / 1e12
    log("step %.3f ms | " % ms_per_step + " | ".join("%s %.3f ms" % (phase_names[i], phase_ms[i]) for i in range(3)))

    # per-layer detail: a second, untimed pass with events around every call
    NP = 20
    ev = [[(new_ev(), new_ev()) for _ in calls] for _ in range(NP)]
    for s in range(NP):
        for ci, (_, _, fn) in enumerate(calls):
            ev[s][ci][0].record()
            fn()
            ev[s][ci][1].record()
    torch.cuda.synchronize()
    call_ms = [sum(ev[s][ci][0].elapsed_time(ev[s][ci][1]) for s in range(NP)) / NP for ci in range(len(calls))]
    per = {(c[0], c[1]): call_ms[ci] for ci, c in enumerate(calls)}
    for li, fn in enumerate(tern_single):
        per[("ternarize", li)] = time_call(fn, reps=NP, warm=2)
    log("%-6s %22s %9s %9s %9s %9s %9s %9s" % ("layer", "(M,N,K)", "tern us", "fwd us", "fwd TF/s", "dX TF/s", "dW us", "dW TF/s"))
    for li, L in enumerate(layers):
        tf, tdx, tdw = per[("fwd", li)], per.get(("bwd_data", li), float("nan")), per[("bwd_weight", li)]
        log("%-6s %22s %9.1f %9.1f %9.1f %9.1f %9.1f %9.1f" % (L.name, str(L.gemm_mnk), per[("ternarize", li)] * 1e3,
                                                             tf * 1e3, L.flops / tf / 1e9, L.flops / tdx / 1e9,
                                                             tdw * 1e3, L.flops / tdw / 1e9))

    # Roofline of the contraction kernel named by the task (gather_gemm_dma_kernel): the forward calls that
    # consist of exactly ONE launch of it (no split-K finish, no first-layer copy, no odd-channel fallback)
    # and run alone on the GPU: forward c2-c6.
    def call_bytes(ph, L):
        # algorithmic bytes of one call: bf16 activations in and out plus the 2-bit codes
        x_b = 2 * L.N * L.H * L.W * L.C
        y_b = 2 * L.N * L.P * L.Q * L.O
        return x_b + y_b + L.n_weights // 4     # the same three tensors forward (X -> Y) and backward (dY -> dX)
    sample_bytes = {ci: call_bytes(calls[ci][0], layers[calls[ci][1]]) for ci in single_calls}
    r_flops = sum(layers[calls[ci][1]].flops for ci in single_calls)
    r_ms = span_ms
    gg_tflops = r_flops / (r_ms * 1e-3) / 1e12
    roof = {"kernel": "gather_gemm_dma_kernel", "bound": "mfma", "achieved": round(gg_tflops, 2),
            "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(gg_tflops / PEAK_BF16_TFLOPS, 4),
            "traffic": ROOFLINE_SAMPLE_TRAFFIC_BYTES,
            "algorithmic_bytes_per_launch": round(sum(sample_bytes.values()) / len(sample_bytes)),
            "launches_per_step": len(single_calls), "avg_launch_us": round(r_ms * 1e3 / len(single_calls), 2),
            "flops_per_launch_avg": round(r_flops / len(single_calls) / 1e9, 2),
            "calls": "fwd c2-c6 (one launch each)"}
    # serial per-layer times of the detail pass give the per-phase rates of the two backward parts
    dx_ms = sum(per[("bwd_data", li)] for li in range(1, len(layers)))
    dw_ms = sum(per[("bwd_weight", li)] for li in range(len(layers)))
    extras = {"phase_ms": {phase_names[i]: round(phase_ms[i], 4) for i in range(3)},
              "fwd_tflops": round(flops_fwd / (phase_ms[1] * 1e-3) / 1e12, 2),
              "bwd_tflops": round((flops_dx + flops_dw) / (phase_ms[2] * 1e-3) / 1e12, 2),
              "bwd_data_serial_ms": round(dx_ms, 4), "bwd_weight_serial_ms": round(dw_ms, 4),
              "ternarize_layers_GBps": round(tern_bytes / (phase_ms[0] * 1e-3) / 1e9, 1),
              "backward_launch": "hip_graph_replay" if bwd_graph is not None else "eager"}

    if args.graph:
        # the same step captured once into a HIP graph and replayed (the library only launches kernels and takes
        # its workspaces from the caller, so a step captures as is); outputs are compared with the eager step's
        outs = (Y[1], Y[7], dX[1], dW[1], dW[5], dW[7])

        def full_step():
            for ci in range(n_main):
                calls[ci][2]()
            backward()

        full_step()
        torch.cuda.synchronize()
        ref = [t.clone() for t in outs]
        cap = torch.cuda.Stream()
        cap.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(cap):
            full_step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=cap):
            full_step()
        torch.cuda.synchronize()
        same = True
        for _ in range(3):
            for t in outs:
                t.fill_(0.0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            same = same and all(torch.equal(a, b) for a, b in zip(ref, outs))
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - g0) * 1e3 / args.steps
        log("graph replay: %.3f ms per step (eager %.3f), outputs identical to eager: %s" % (g_ms, ms_per_step, same))
        extras["graph_replay"] = {"ms_per_step": round(g_ms, 4), "outputs_identical_to_eager": bool(same)}

    if not args.no_extras:
        del X, dY, Y, dX, dW
        torch.cuda.empty_cache()
        extras["gemm_8192x4096x4096"] = side_gemm()
        extras["ternarize_2p28"] = side_ternarize()
        extras["resnet18_b64_fwd"] = side_resnet18()

    cpu = None
    if not args.no_cpu:
        from oracle import conv as oc
        from oracle import ternarize as ot
        oc.build()
        cores = oc.max_threads()
        nb = args.cpu_batch
        t_tern = 0.0
        t_conv = 0.0
        for li, L in enumerate(layers):
            w = wl.kaiming_weights(CFG, li, L)
            a = time.perf_counter()
            codes, delta, alpha, nnz = ot.ternarize(w, F)
            t_tern += time.perf_counter() - a
            Ls = L.with_batch(nb)
            x = wl.bf16_round(wl.normal(CFG, wl.IDX_INPUT + li, Ls.x_shape))
            dy = wl.bf16_round(wl.normal(CFG, wl.IDX_DY + 10 * li, Ls.y_shape))
            st, pd, dl = geo[li]
            a = time.perf_counter()
            oc.conv2d_fwd(x, codes, alpha, st, pd, dl)
            if li:
                oc.conv2d_bwd_data(dy, codes, alpha, Ls.x_shape, st, pd, dl)
            oc.conv2d_bwd_weight(x, dy, Ls.w_shape, st, pd, dl)
            t_conv += time.perf_counter() - a
        t_full = t_tern + t_conv * (128.0 / nb)
        cpu = {"value": round(flops_step / t_full / 1e12, 6), "unit": "TFLOP/s-eq", "cores": cores, "kind": "oracle",
               "sample": "ternarize of all 8 VGG-7 tensors in full (%.2f s, numpy sort, 1 thread) + fwd/dX/dW of every layer "
                         "at batch %d of 128 (%.2f s, C direct loops, %d OpenMP threads)%s"
                         % (t_tern, nb, t_conv, cores, "" if nb == 128 else ", conv time scaled linearly to batch 128")}
        log("cpu oracle: ternarize %.2f s, conv(b%d) %.2f s -> %.5f TFLOP/s-eq" % (t_tern, nb, t_conv, cpu["value"]))

    out = {
        "metric": "ternary conv/GEMM throughput, dense-equivalent (2MNK per contraction; ternarize + fwd + STE bwd per step)",
        "value": round(value, 3), "unit": "TFLOP/s-eq", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "vgg7_cifar_b128_twn_step", "layers": len(layers), "batch": 128, "delta_factor": F,
                   "gflop_per_step": round(flops_step / 1e9, 1), "img_per_s": round(128 / (ms_per_step * 1e-3), 1)},
        "roofline": roof,
        "cpu_baseline": cpu,
        "extras": extras,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
