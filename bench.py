#!/usr/bin/env python3
"""Benchmark of the TWN hot path on one MI355X.

Headline workload: ResNet-18, batch 64, bf16 (the configuration both the metric and the target are stated on).
A step is one pass of the forward hot path over one batch: ONE multi-tensor ternarize call for all 21 weight
tensors (Delta, alpha, 2-bit codes), then the forward of every conv / FC layer with its fused block tail
(scale, shift, residual on the second conv of a block, ReLU).  Inside a basic block the tensors flow as in the
network (conv2 reads conv1's output and adds the block input or its down-sampled copy, the next block reads
conv2's output); the stem, the first block and the classifier start from seeded synthetic tensors because the
pooling between them is glue outside the hot path.  All inputs are resident in HBM and the layers run one after
the other on one stream, as the data dependences of the network demand.  `value` is the dense-equivalent throughput of the step (2MNK per
contraction / step time); images per second are in `config`.

Side measurements (structured, each with its own roofline object): the 8192x4096x4096 GEMM, the 2^28-element
ternarize, and timings of the other configurations (LeNet b64 fp32, VGG-7 b128 forward + straight-through
backward, the VGG-16-style backbone b32, ResNet-18 backward, ResNet-18 with one alpha per filter).

Prints ONE JSON line on stdout; per-layer detail goes to stderr.
"""

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # dense bf16 MFMA, MI355X
PEAK_HBM_GBPS = 8000.0
PEAK_ADDS_T = 256 * 64 * 2.4e9 / 1e12   # float32 additions per second (non-packed), in units of 1e12
F = 0.7
PROFILES = os.path.join(ROOT, "profiles")
# consecutive forward calls of the headline step that are ONE launch each of the same kernel on the same shape:
# the sample the `roofline` object is measured on (two events per step bracket the run)
ROOFLINE_LAYERS = ("l1.0.conv1", "l1.0.conv2", "l1.1.conv1", "l1.1.conv2")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def profile_value(fname, key):
    """`key=<number>` from a committed rocprofv3 summary under profiles/ (None if the file or the key is absent)."""
    path = os.path.join(PROFILES, fname)
    if not os.path.exists(path):
        return None
    m = re.search(r"^%s\s*=\s*([0-9.eE+-]+)" % re.escape(key), open(path).read(), re.M)
    return float(m.group(1)) if m else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-extras", action="store_true", help="skip the side measurements")
    ap.add_argument("--cpu-batch", type=int, default=64,
                    help="batch the CPU oracle runs every layer at (64 = the whole workload, no extrapolation)")
    ap.add_argument("--only", choices=["gemm", "ternarize", "resnet18", "resnet18_bwd", "lenet", "vgg7", "vgg16_ssd", "sgd",
                                       "per_filter", "addsub", "resnet18b"], default=None,
                    help="run one measurement alone (used for the rocprofv3 summaries in profiles/)")
    ap.add_argument("--variants", action="store_true", help="with --only gemm: also time the comparison weight formats")
    ap.add_argument("--calibrate", action="store_true",
                    help="first run three plain 1 GiB device copies: a kernel of known traffic for the HBM byte counters "
                         "of a rocprofv3 --pmc run")
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

    def new_ev():
        return torch.cuda.Event(enable_timing=True)

    def time_call(fn, reps=10, warm=2):
        for _ in range(warm):
            fn()
        a, b = new_ev(), new_ev()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    def geo(L):
        return (L.stride,) * 2, (L.pad,) * 2, (L.dil,) * 2

    def layer_bytes(L):
        # algorithmic bytes of one forward call: bf16 activations in and out plus the 2-bit codes
        return 2 * L.N * L.H * L.W * L.C + 2 * L.N * L.P * L.Q * L.O + L.n_weights // 4

    def roof_obj(kernel, bound, achieved, peak, unit, alg_bytes, traffic_file, launch_us, **more):
        traffic = profile_value(traffic_file, "traffic_bytes_per_launch") if traffic_file else None
        o = {"kernel": kernel, "bound": bound, "achieved": round(achieved, 2), "peak": peak, "unit": unit,
             "frac": round(achieved / peak, 4), "traffic": None if traffic is None else int(traffic),
             "traffic_source": ("profiles/" + traffic_file) if traffic is not None else None,
             "algorithmic_bytes_per_launch": int(alg_bytes), "avg_launch_us": round(launch_us, 2)}
        o.update(more)
        return o

    # ------------------------------------------------------------------ network forward builders
    def build_forward(layers, cfg, fp32=False, residual_on=("conv2",), groups_per_filter=False, transposed=False,
                      chain_blocks=False, variant=None):
        """Device tensors and prepared calls for the forward of a list of layers.  Every layer reads its own
        synthetic input, except with chain_blocks (residual networks): inside a basic block the data flows as in
        the network (conv1 and the down-sample read the block input, conv2 reads conv1's output and adds the
        block input or the down-sampled one, the next block reads conv2's output); only where the network has
        glue that is outside the hot path (pooling before the first block and before the classifier) does a
        layer start from a synthetic tensor."""
        W, X, Y, tws, calls = [], [], [], [], []
        for li, L in enumerate(layers):
            w = wl.kaiming_weights(cfg, li, L)
            W.append(torch.from_numpy(w).to(dev))
            Y.append(torch.empty(L.y_shape, dtype=torch.float32 if fp32 else torch.bfloat16, device=dev))
            groups = L.O if groups_per_filter else 1
            tws.append(api.twn_ternarize(W[li], F, groups=groups, transposed=transposed))

        def synthetic(li, L):
            if fp32:
                return torch.from_numpy(wl.uniform01(cfg, wl.IDX_INPUT + li, L.x_shape)).to(dev)
            return dev_bf16(wl.normal(cfg, wl.IDX_INPUT + li, L.x_shape))

        RES = [None] * len(layers)
        block_in = conv1_out = down_out = None
        for li, L in enumerate(layers):
            x = None
            part = L.name.rsplit(".", 1)[-1]
            if chain_blocks and part in ("conv1", "down", "conv2"):
                if part == "conv1":
                    if block_in is None or tuple(block_in.shape) != tuple(L.x_shape):
                        block_in = synthetic(li, L)
                    x, conv1_out, down_out = block_in, Y[li], None
                elif part == "down":
                    x, down_out = block_in, Y[li]
                else:
                    x = conv1_out
                    RES[li] = down_out if down_out is not None else block_in
                    block_in = Y[li]
                assert tuple(x.shape) == tuple(L.x_shape)
            else:
                x = synthetic(li, L)
                if not fp32 and any(L.name.endswith(s) for s in residual_on):
                    RES[li] = dev_bf16(wl.normal(cfg, 700 + li, L.y_shape))
            X.append(x)
        for li, L in enumerate(layers):
            st, pd, dl = geo(L)
            is_fc = (L.R == 1 and L.S == 1 and L.H == 1 and L.W == 1)
            last = (li == len(layers) - 1)
            sc = torch.ones(L.O, dtype=torch.float32, device=dev)
            sf = torch.zeros(L.O, dtype=torch.float32, device=dev)
            if is_fc:
                calls.append(api.prepare_gemm_fwd(X[li].reshape(L.N, L.C), tws[li], out=Y[li].reshape(L.N, L.O),
                                                  scale=None if last else sc, shift=sf, relu=not last, variant=variant))
            else:
                calls.append(api.prepare_conv2d_fwd(X[li], tws[li], st, pd, dl, out=Y[li], scale=sc, shift=sf,
                                                    residual=RES[li], relu=True, variant=variant))
        return W, X, Y, tws, calls

    def per_layer_table(tag, layers, calls, reps=100, warm=20):
        tot = 0.0
        rows = []
        for L, c in zip(layers, calls):
            t = time_call(c, reps=reps, warm=warm)
            tot += t
            rows.append((L.name, t))
            log("%s %-12s %26s %9.1f us %8.1f TFLOP/s-eq" % (tag, L.name, str(L.gemm_mnk), t * 1e3, L.flops / t / 1e9))
        return tot, rows

    def graph_of(fn):
        """Capture fn (library calls only launch kernels and take their workspaces from the caller) and return the
        replayable graph, or None when capture is not available."""
        try:
            cap = torch.cuda.Stream()
            cap.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(cap):
                fn()
            torch.cuda.synchronize()
            g_ = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_, stream=cap):
                fn()
            torch.cuda.synchronize()
            return g_
        except RuntimeError as e:
            log("graph capture failed (%s)" % str(e).splitlines()[0])
            torch.cuda.synchronize()
            return None

    # ------------------------------------------------------------------ side measurements
    def side_gemm():
        g = wl.gemm_config()
        gx = dev_bf16(wl.normal(3, wl.IDX_INPUT, (g.N, g.C)))
        gw = torch.from_numpy(wl.normal(3, 1, (g.O, g.C), std=0.02)).to(dev)
        gtw = api.twn_ternarize(gw, F)
        gy = torch.empty((g.N, g.O), dtype=torch.bfloat16, device=dev)
        call = api.prepare_gemm_fwd(gx, gtw, out=gy)
        t = time_call(call, reps=300, warm=100)
        tf = g.flops / t / 1e9
        log("gemm 8192x4096x4096: %.1f us, %.1f TFLOP/s-eq (%.3f of 2.5 PFLOP/s)" % (t * 1e3, tf, tf / PEAK_BF16_TFLOPS))
        res = roof_obj("contraction kernel, 128x256 tile", "mfma", tf, PEAK_BF16_TFLOPS, "TFLOP/s", layer_bytes(g),
                       "gemm_8192x4096x4096_kernels.txt", t * 1e3, workload="gemm_8192x4096x4096_bf16", us=round(t * 1e3, 1),
                       flops_per_launch=g.flops,
                       # the same launch with everything but the MFMAs removed ran 128.9 us on this chip (ablation build,
                       # clock 2.49 GHz): the rate the matrix pipes sustain when nothing else draws power
                       mfma_only_rate_tflops=round(g.flops / 128.9e-6 / 1e12, 1),
                       frac_of_mfma_only_rate=round(tf / (g.flops / 128.9e-6 / 1e12), 4))
        if args.variants:
            os.environ["TWN_TILE"] = "4"
            api.reload_env()
            same = {"postscale_2bit": time_call(lambda: api.twn_gemm_fwd(gx, gtw, out=gy), reps=60, warm=20)}
            del os.environ["TWN_TILE"]
            api.reload_env()
            for name, var in (("alpha_at_expansion_2bit", api.TWN_VAR_BF16_ALPHA_LDS),
                              ("int8_stored", api.TWN_VAR_I8_STORED_POSTSCALE)):
                same[name] = time_call(lambda: api.twn_gemm_fwd(gx, gtw, out=gy, variant=var), reps=60, warm=20)
            # the binary-weight comparison of Sec. 3: sign codes, one bit per weight, alpha = mean|W|
            gbw = api.twn_binarize(gw)
            same["sign_1bit (binary-weight comparison)"] = time_call(
                lambda: api.twn_gemm_fwd(gx, gbw, out=gy, variant=api.TWN_VAR_BF16_SIGN1_POSTSCALE), reps=60, warm=20)
            t_b = time_call(lambda: api.twn_binarize(gw), reps=30, warm=5)
            log("twn_binarize of the 4096x4096 weights: %.1f us" % (t_b * 1e3))
            res["binarize_4096x4096_us"] = round(t_b * 1e3, 1)
            for k, v in same.items():
                log("gemm weight format %-24s %.1f us (register-staged 128x128 kernel)" % (k, v * 1e3))
            res["weight_formats_same_kernel_us"] = {k: round(v * 1e3, 1) for k, v in same.items()}
        return res

    def side_ternarize(calibrate=False):
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
        gbps = nbytes / t / 1e6
        res = roof_obj("abs_sum_kernel + mask_pack_flat_kernel", "hbm", gbps, PEAK_HBM_GBPS, "GB/s", nbytes,
                       "ternarize_2p28_hbm.txt", t * 1e3, workload="ternarize_2p28_f32", us=round(t * 1e3, 1))
        # bytes requested from beyond the L2s (the counters of the committed profile; Infinity Cache hits are among
        # them: pass 2 walks W backwards, so the end of pass 1 can be served from that cache) over this run's time
        if res["traffic"] is not None:
            res["beyond_l2_GBps"] = round(res["traffic"] / t / 1e6, 1)
        # the same call with pass 2 walking forwards (nothing of pass 1 left in the cache): all 8.25 B/weight from HBM,
        # the figure to hold against the HBM peak
        os.environ["TWN_TERN_REVERSE"] = "0"
        api.reload_env()
        t_fwd = time_call(lambda: api.twn_ternarize(big, F, out=btw, workspace=ws), reps=50, warm=10)
        del os.environ["TWN_TERN_REVERSE"]
        api.reload_env()
        res["forward_walk_us"] = round(t_fwd * 1e3, 1)
        res["forward_walk_GBps"] = round(nbytes / t_fwd / 1e6, 1)
        res["forward_walk_frac"] = round(nbytes / t_fwd / 1e6 / PEAK_HBM_GBPS, 4)
        log("ternarize 2^28: %.1f us, %.1f GB/s algorithmic (8.25 B/weight); forward-walking pass 2: %.1f us, %.1f GB/s"
            % (t * 1e3, gbps, t_fwd * 1e3, nbytes / t_fwd / 1e6))
        return res

    def side_sgd():
        """Parameter update of 2^28 float32 weights (Alg. 1 step 10) fused with pass 1 of the next ternarization, and
        the ternarization that follows with and without the sums it leaves behind."""
        n = 1 << 28
        Wt = torch.from_numpy(wl.normal(3, 0, (1 << 14, 1 << 14), std=0.05)).to(dev)
        Vt = torch.zeros_like(Wt)
        dWt = torch.from_numpy(wl.normal(3, 1, (1 << 14, 1 << 14), std=0.02)).to(dev)
        ws = torch.empty(1 << 17, dtype=torch.uint8, device=dev)
        tw = api.twn_ternarize(Wt, F)
        t_u = time_call(lambda: api.twn_sgd_update(Wt, Vt, dWt, 1e-3, 0.9, 1e-4, tern_workspace=ws), reps=50, warm=10)
        t_p = time_call(lambda: api.twn_ternarize_presummed(Wt, tw, ws, F), reps=50, warm=10)
        t_t = time_call(lambda: api.twn_ternarize(Wt, F, out=tw, workspace=ws), reps=50, warm=10)
        nbytes = n * 20.0
        gbps = nbytes / t_u / 1e6
        res = roof_obj("sgd_update_kernel", "hbm", gbps, PEAK_HBM_GBPS, "GB/s", nbytes, None, t_u * 1e3,
                       workload="sgd_momentum_wd_2p28_f32 (+ |W| sums of the next ternarization)", us=round(t_u * 1e3, 1),
                       ternarize_after_update_us={"reusing_the_sums": round(t_p * 1e3, 1), "from_scratch": round(t_t * 1e3, 1)})
        log("sgd update 2^28: %.1f us, %.1f GB/s (20 B/weight); ternarize after it: %.1f us reusing the sums, %.1f us from "
            "scratch" % (t_u * 1e3, gbps, t_p * 1e3, t_t * 1e3))
        return res

    def side_lenet():
        layers = wl.lenet5(64)
        W, X, Y, tws, calls = build_forward(layers, 0, fp32=True)
        tot, rows = per_layer_table("lenet", layers, calls)

        def fwd():
            for c in calls:
                c()
        g_ = graph_of(fwd)
        t_graph = time_call(g_.replay, reps=200, warm=20) if g_ is not None else None
        flops = sum(L.flops for L in layers)
        best = t_graph if t_graph is not None else tot
        log("lenet b64 fp32 forward: serial %.1f us, graph replay %s us, %.0f img/s" %
            (tot * 1e3, "%.1f" % (t_graph * 1e3) if t_graph else "n/a", 64 / (best * 1e-3)))
        return {"workload": "lenet5_b64_fp32_forward", "serial_us": round(tot * 1e3, 1),
                "graph_replay_us": None if t_graph is None else round(t_graph * 1e3, 1),
                "img_per_s": round(64 / (best * 1e-3), 1), "gflops": round(flops / best / 1e6, 1),
                "per_layer_us": {n: round(t * 1e3, 1) for n, t in rows},
                "bound": "latency: 0.55 GFLOP in four dependent launches of 2 to 576 workgroups"}

    def side_vgg16():
        layers = wl.vgg16_ssd(32)
        tot = 0.0
        rows = {}
        for li, L in enumerate(layers):
            # one layer resident at a time (the first layers' activations are 0.7 GB each)
            W, X, Y, tws, calls = build_forward([L], 4, residual_on=())
            t = time_call(calls[0], reps=30, warm=5)
            tot += t
            rows[L.name] = round(t * 1e3, 1)
            log("vgg16_ssd %-8s %28s %9.1f us %8.1f TFLOP/s-eq" % (L.name, str(L.gemm_mnk), t * 1e3, L.flops / t / 1e9))
            del W, X, Y, tws, calls
            torch.cuda.empty_cache()
        flops = sum(L.flops for L in layers)
        log("vgg16-style backbone b32 forward: %.3f ms, %.0f img/s, %.1f TFLOP/s-eq" % (tot, 32 / (tot * 1e-3), flops / tot / 1e9))
        return {"workload": "vgg16_ssd_b32_bf16_forward", "ms": round(tot, 4), "img_per_s": round(32 / (tot * 1e-3), 1),
                "tflops": round(flops / tot / 1e9, 1), "frac_mfma_peak": round(flops / tot / 1e9 / PEAK_BF16_TFLOPS, 4),
                "per_layer_us": rows}

    def backward_table(tag, layers, cfg):
        tot_dx = tot_dw = 0.0
        for li, L in enumerate(layers):
            st, pd, dl = geo(L)
            x = dev_bf16(wl.normal(cfg, wl.IDX_INPUT + li, L.x_shape))
            dy = dev_bf16(wl.normal(cfg, wl.IDX_DY + 10 * li, L.y_shape))
            twt = api.twn_ternarize(torch.from_numpy(wl.kaiming_weights(cfg, li, L)).to(dev), F, transposed=True)
            ws = torch.empty(max(16, api.twn_conv2d_bwd_ste_workspace_bytes(L.x_shape, twt, st, pd, dl)), dtype=torch.uint8,
                             device=dev)
            dxo = torch.empty(L.x_shape, dtype=torch.bfloat16, device=dev)
            dwo = torch.empty(L.w_shape, dtype=torch.float32, device=dev)
            tdx = 0.0
            if li > 0:
                c = api.prepare_conv2d_bwd_ste(None, dy, twt, st, pd, dl, dX=dxo, workspace=ws, x_shape=L.x_shape)
                tdx = time_call(c, reps=50, warm=10)
            c = api.prepare_conv2d_bwd_ste(x, dy, twt, st, pd, dl, dW=dwo, workspace=ws)
            tdw = time_call(c, reps=50, warm=10)
            tot_dx += tdx
            tot_dw += tdw
            log("%s %-12s %26s  dX %8.1f us  dW %8.1f us" % (tag, L.name, str(L.gemm_mnk), tdx * 1e3, tdw * 1e3))
            del x, dy, dxo, dwo, ws
        return tot_dx, tot_dw

    def side_resnet18_bwd():
        layers = wl.resnet18(64)
        tdx, tdw = backward_table("resnet18-bwd", layers, 2)
        flops = sum(L.flops for L in layers) + sum(L.flops for L in layers[1:])
        log("resnet18 b64 straight-through backward, serial: dX %.3f ms + dW %.3f ms" % (tdx, tdw))
        return {"workload": "resnet18_b64_bf16_ste_backward", "dx_ms": round(tdx, 4), "dw_ms": round(tdw, 4),
                "tflops": round(flops / (tdx + tdw) / 1e9, 1),
                "frac_mfma_peak": round(flops / (tdx + tdw) / 1e9 / PEAK_BF16_TFLOPS, 4)}

    def side_vgg7():
        layers = wl.vgg7(128)
        W, X, Y, tws, calls = build_forward(layers, 1, residual_on=(), transposed=True)
        tern = api.prepare_ternarize_batch(W, tws, F)
        t_tern = time_call(tern, reps=50, warm=10)
        t_fwd, _ = per_layer_table("vgg7", layers, calls, reps=50, warm=10)
        del X, Y, calls
        torch.cuda.empty_cache()
        tdx, tdw = backward_table("vgg7-bwd", layers, 1)
        f_fwd = sum(L.flops for L in layers)
        f_all = 2 * f_fwd + sum(L.flops for L in layers[1:])
        t_all = t_tern + t_fwd + tdx + tdw
        log("vgg7 b128 step, serial: ternarize %.3f + fwd %.3f + dX %.3f + dW %.3f = %.3f ms, %.1f TFLOP/s-eq" %
            (t_tern, t_fwd, tdx, tdw, t_all, f_all / t_all / 1e9))
        return {"workload": "vgg7_cifar_b128_bf16_step_serial", "ternarize_ms": round(t_tern, 4), "fwd_ms": round(t_fwd, 4),
                "dx_ms": round(tdx, 4), "dw_ms": round(tdw, 4), "ms": round(t_all, 4),
                "tflops": round(f_all / t_all / 1e9, 1), "frac_mfma_peak": round(f_all / t_all / 1e9 / PEAK_BF16_TFLOPS, 4),
                "img_per_s": round(128 / (t_all * 1e-3), 1)}

    def side_per_filter():
        # Alg. 1 as printed: one (Delta, alpha) per filter; ResNet-18 has 4800 filters in 21 tensors
        layers = wl.resnet18(64)
        t_fwd = 0.0
        t_dx = 0.0
        Wall = [torch.from_numpy(wl.kaiming_weights(2, li, L)).to(dev) for li, L in enumerate(layers)]
        tws_all = api.twn_ternarize_batch(Wall, F, transposed=True, per_filter=True)
        t_tern = time_call(api.prepare_ternarize_batch(Wall, tws_all, F), reps=50, warm=10)
        for li, L in enumerate(layers):
            st, pd, dl = geo(L)
            w = Wall[li]
            tw = tws_all[li]
            W, X, Y, tws, calls = build_forward([L], 2, residual_on=(), groups_per_filter=True)
            t_fwd += time_call(calls[0], reps=50, warm=10)
            del W, X, Y, tws, calls
            if li > 0:
                # backward-data with one alpha per filter: alpha*dY carried as two bf16 terms, two contraction passes
                dy = dev_bf16(wl.normal(2, wl.IDX_DY + 10 * li, L.y_shape))
                wsb = torch.empty(max(16, api.twn_conv2d_bwd_ste_workspace_bytes(L.x_shape, tw, st, pd, dl)),
                                  dtype=torch.uint8, device=dev)
                dxo = torch.empty(L.x_shape, dtype=torch.bfloat16, device=dev)
                c = api.prepare_conv2d_bwd_ste(None, dy, tw, st, pd, dl, dX=dxo, workspace=wsb, x_shape=L.x_shape)
                t_dx += time_call(c, reps=30, warm=5)
                del dy, wsb, dxo
        log("resnet18 per-filter (Alg. 1): ternarize of 21 tensors with both packed copies, one multi-tensor call %.3f ms; forward %.3f ms; backward-data "
            "%.3f ms" % (t_tern, t_fwd, t_dx))
        return {"workload": "resnet18_b64_per_filter_alpha", "ternarize_ms": round(t_tern, 4), "fwd_ms": round(t_fwd, 4),
                "dx_ms": round(t_dx, 4)}

    def side_addsub():
        """Eq. 2's multiplication-free form on the vector ALUs (zero codes skipped) against the matrix-core kernels, on
        every ResNet-18 b64 layer whose channel count it accepts (all but the three-channel stem)."""
        layers = wl.resnet18(64)[1:]
        rows = {}
        t_as = t_mfma = 0.0
        adds = 0
        for li, L in enumerate(layers, start=1):
            W, X, Y, tws, calls = build_forward([L], 2, variant=api.TWN_VAR_ADDSUB_SPARSE)
            ta = time_call(calls[0], reps=10, warm=2)
            nnz = int(tws[0].nnz.sum().item())
            del W, X, Y, tws, calls
            W, X, Y, tws, calls = build_forward([L], 2)
            tm = time_call(calls[0], reps=50, warm=10)
            del W, X, Y, tws, calls
            m = L.gemm_mnk[0]
            adds += m * nnz
            t_as += ta
            t_mfma += tm
            rows[L.name] = {"addsub_us": round(ta * 1e3, 1), "mfma_us": round(tm * 1e3, 1),
                            "nonzero_fraction": round(nnz / L.n_weights, 4)}
            log("addsub %-12s %26s  add/sub %9.1f us (%6.1f TFLOP/s-eq, %5.2f Tadd/s)   matrix cores %8.1f us" %
                (L.name, str(L.gemm_mnk), ta * 1e3, L.flops / ta / 1e9, m * nnz / ta / 1e9, tm * 1e3))
        flops = sum(L.flops for L in layers)
        tadds = adds / t_as / 1e9
        log("addsub resnet18 b64 (20 layers): %.3f ms = %.1f TFLOP/s-eq, %.2f T additions/s; matrix-core path %.3f ms (%.1fx)"
            % (t_as, flops / t_as / 1e9, tadds, t_mfma, t_as / t_mfma))
        # peak: one float32 addition per lane and clock, 64 lanes per CU and clock (4 SIMDs x 16 lanes), 256 CUs, 2.4 GHz;
        # the library is built without packed-float32 instructions
        return roof_obj("conv_addsub_kernel", "alu", tadds, PEAK_ADDS_T, "Tadd/s", sum(layer_bytes(L) for L in layers),
                        None, t_as * 1e3 / len(layers), workload="resnet18_b64_bf16_forward_without_stem, TWN_VAR_ADDSUB_SPARSE",
                        ms=round(t_as, 4), tflops_eq=round(flops / t_as / 1e9, 1), additions=adds,
                        matrix_core_path_ms=round(t_mfma, 4), slowdown_vs_matrix_cores=round(t_as / t_mfma, 2),
                        per_layer=rows)

    def side_resnet18b():
        # ResNet-18B of Sec. 3.1: the same blocks with 1.5x the filters (96 / 192 / 384 / 768)
        layers = wl.resnet18(64, width_mult=1.5)
        W, X, Y, tws, calls = build_forward(layers, 5, chain_blocks=True)
        tot, rows = per_layer_table("resnet18b", layers, calls, reps=50, warm=10)
        flops = sum(L.flops for L in layers)
        log("resnet18b b64 forward, sum of per-layer times: %.3f ms, %.0f img/s, %.1f TFLOP/s-eq" %
            (tot, 64 / (tot * 1e-3), flops / tot / 1e9))
        return {"workload": "resnet18b_b64_bf16_forward (1.5x filters)", "ms": round(tot, 4),
                "img_per_s": round(64 / (tot * 1e-3), 1), "gflop": round(flops / 1e9, 1),
                "tflops": round(flops / tot / 1e9, 1), "frac_mfma_peak": round(flops / tot / 1e9 / PEAK_BF16_TFLOPS, 4),
                "per_layer_us": {n: round(t * 1e3, 1) for n, t in rows}}

    # ------------------------------------------------------------------ headline: ResNet-18 b64 forward
    def headline(with_cpu):
        CFG = 2
        layers = wl.resnet18(64)
        W, X, Y, tws, calls = build_forward(layers, CFG, chain_blocks=True)
        tern = api.prepare_ternarize_batch(W, tws, F)
        names = [L.name for L in layers]
        i0, i1 = names.index(ROOFLINE_LAYERS[0]), names.index(ROOFLINE_LAYERS[-1])
        assert tuple(names[i0:i1 + 1]) == ROOFLINE_LAYERS
        flops_fwd = sum(L.flops for L in layers)
        n_w = sum(L.n_weights for L in layers)

        # block heads with a projection shortcut: the first convolution and the 1x1 down-sample read the same
        # input and go through ONE twn_conv2d_fwd_pair call (the library runs them in one launch where that pays)
        step_calls = list(calls)
        n_pairs = 0
        for li, L in enumerate(layers):
            if L.name.endswith(".down"):
                assert layers[li - 1].name == L.name[:-5] + ".conv1" and X[li] is X[li - 1]
                ones = [torch.ones(l_.O, dtype=torch.float32, device=dev) for l_ in (layers[li - 1], L)]
                zeros = [torch.zeros(l_.O, dtype=torch.float32, device=dev) for l_ in (layers[li - 1], L)]
                step_calls[li - 1] = api.prepare_conv2d_fwd_pair(
                    X[li], (tws[li - 1], tws[li]), (geo(layers[li - 1]), geo(L)), (Y[li - 1], Y[li]),
                    scales=ones, shifts=zeros, relus=(True, True))
                step_calls[li] = None
                n_pairs += 1

        def one_step(marks=None):
            tern()
            for li, c in enumerate(step_calls):
                if marks is not None and li == i0:
                    marks[0].record()
                if c is not None:
                    c()
                if marks is not None and li == i1:
                    marks[1].record()

        def forward_only():
            for c in step_calls:
                if c is not None:
                    c()

        for _ in range(args.warmup):
            one_step()
        torch.cuda.synchronize()
        mev = [(new_ev(), new_ev()) for _ in range(args.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(args.steps):
            one_step(mev[s])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / args.steps
        span_ms = sum(a.elapsed_time(b) for a, b in mev) / args.steps
        value = flops_fwd / (ms_per_step * 1e-3) / 1e12

        # phases (separate pass): the ternarize call, then the forward
        NPH = max(5, min(50, args.steps))
        pev = [[new_ev() for _ in range(3)] for _ in range(NPH)]
        for s in range(NPH):
            pev[s][0].record()
            tern()
            pev[s][1].record()
            forward_only()
            pev[s][2].record()
        torch.cuda.synchronize()
        t_tern = sum(pev[s][0].elapsed_time(pev[s][1]) for s in range(NPH)) / NPH
        t_fwd = sum(pev[s][1].elapsed_time(pev[s][2]) for s in range(NPH)) / NPH
        log("resnet18 b64 step %.3f ms (ternarize %.3f + forward %.3f), %.0f img/s, %.1f TFLOP/s-eq" %
            (ms_per_step, t_tern, t_fwd, 64 / (ms_per_step * 1e-3), value))

        # the same step replayed from a HIP graph (no host launch cost); outputs compared with the eager step's
        graph_info = None
        outs = [Y[0], Y[i0], Y[-1], tws[0].packed, tws[5].alpha]
        one_step()
        torch.cuda.synchronize()
        ref = [t.clone() for t in outs]
        g_ = graph_of(one_step)
        if g_ is not None:
            same = True
            for rep in range(3):
                for t in outs:
                    t.zero_()
                if rep == 1:
                    calls[1]()                 # eager work between two replays
                torch.cuda.synchronize()
                g_.replay()
                torch.cuda.synchronize()
                same = same and all(torch.equal(a, b) for a, b in zip(ref, outs))
            t_g = time_call(g_.replay, reps=args.steps, warm=args.warmup)
            log("graph replay: %.3f ms per step (eager %.3f), outputs identical to eager: %s" % (t_g, ms_per_step, same))
            graph_info = {"ms_per_step": round(t_g, 4), "outputs_identical_to_eager": bool(same),
                          "img_per_s": round(64 / (t_g * 1e-3), 1)}

        tot, rows = per_layer_table("resnet18", layers, calls)
        log("resnet18 b64 forward, sum of per-layer times: %.3f ms" % tot)

        Ls = layers[i0]
        n_launch = i1 - i0 + 1
        # the second convolution of a block also reads the residual tensor (as large as its output): averaged over the launches
        res_bytes = sum(2 * layers[i].N * layers[i].P * layers[i].Q * layers[i].O
                        for i in range(i0, i1 + 1) if layers[i].name.endswith("conv2")) // n_launch
        r_tf = sum(layers[i].flops for i in range(i0, i1 + 1)) / (span_ms * 1e-3) / 1e12
        roof = roof_obj("conv_c64_kernel (layer1 3x3 convolutions, 64 -> 64 channels, 56x56)", "mfma", r_tf,
                        PEAK_BF16_TFLOPS, "TFLOP/s", layer_bytes(Ls) + res_bytes, "resnet18_b64_forward_kernels.txt",
                        span_ms * 1e3 / n_launch, launches_per_step=n_launch, flops_per_launch=Ls.flops,
                        calls="fwd " + " ".join(ROOFLINE_LAYERS) + " (one launch each)",
                        hbm_bound_us=round((layer_bytes(Ls) + res_bytes) / PEAK_HBM_GBPS / 1e3, 2))
        # the other kernel templates of the forward, from the per-layer pass (each layer looped alone, 100 launches)
        tmap = dict(rows)
        layer_roofs = []
        for kern, bound, names_ in (
                ("conv_first_kernel (stem, 7x7 / 2, 3 -> 64 channels)", "hbm", ["stem"]),
                ("conv_stream_pc_kernel 128x128 (layer2 3x3 convolutions, 128 channels, 28x28)", "mfma",
                 ["l2.0.conv2", "l2.1.conv1", "l2.1.conv2"]),
                ("conv_stream_pc_kernel 64x128 (layer3 3x3 convolutions, 256 channels, 14x14)", "mfma",
                 ["l3.0.conv2", "l3.1.conv1", "l3.1.conv2"]),
                ("conv_stream_pc_kernel 64x128 (layer4 3x3 convolutions, 512 channels, 7x7)", "mfma",
                 ["l4.0.conv2", "l4.1.conv1", "l4.1.conv2"])):
            Lg = [layers[names.index(n)] for n in names_]
            t_ms = sum(tmap[n] for n in names_)
            if bound == "mfma":
                ach, peak, unit = sum(L.flops for L in Lg) / t_ms / 1e9, PEAK_BF16_TFLOPS, "TFLOP/s"
            else:
                ach, peak, unit = sum(layer_bytes(L) for L in Lg) / t_ms / 1e6, PEAK_HBM_GBPS, "GB/s"
            layer_roofs.append(roof_obj(kern, bound, ach, peak, unit, layer_bytes(Lg[0]), None, t_ms * 1e3 / len(Lg),
                                        launches_per_step=len(Lg), flops_per_launch=Lg[0].flops,
                                        calls="fwd " + " ".join(names_) + " (each looped alone)",
                                        workload="resnet18_b64_bf16_twn_forward"))
        cpu = None
        if with_cpu:
            from oracle import conv as oc
            from oracle import ternarize as ot
            oc.build()
            cores = oc.max_threads()
            nb = args.cpu_batch
            t_t = t_c = 0.0
            for li, L in enumerate(layers):
                w = wl.kaiming_weights(CFG, li, L)
                a = time.perf_counter()
                codes, delta, alpha, nnz = ot.ternarize(w, F)
                t_t += time.perf_counter() - a
                Lb = L.with_batch(nb)
                x = wl.bf16_round(wl.normal(CFG, wl.IDX_INPUT + li, Lb.x_shape))
                a = time.perf_counter()
                oc.conv2d_fwd(x, codes, alpha, *geo(L))
                t_c += time.perf_counter() - a
            t_full = t_t + t_c * (64.0 / nb)
            cpu = {"value": round(flops_fwd / t_full / 1e12, 6), "unit": "TFLOP/s-eq", "cores": cores, "kind": "oracle",
                   "img_per_s": round(64 / t_full, 3),
                   "sample": "ternarize of all 21 ResNet-18 tensors in full (%.2f s, numpy sort, 1 thread) + forward of every "
                             "layer at batch %d of 64 (%.2f s, C direct loops, %d OpenMP threads)%s"
                             % (t_t, nb, t_c, cores, "" if nb == 64 else ", conv time scaled linearly to batch 64")}
            log("cpu oracle: ternarize %.2f s, conv(b%d) %.2f s -> %.5f TFLOP/s-eq" % (t_t, nb, t_c, cpu["value"]))
        info = {"ms_per_step": ms_per_step, "value": value, "roof": roof, "layer_roofs": layer_roofs, "cpu": cpu, "graph": graph_info,
                "phase_ms": {"ternarize": round(t_tern, 4), "forward": round(t_fwd, 4)},
                "forward_only": {"ms": round(t_fwd, 4), "tflops": round(flops_fwd / t_fwd / 1e9, 1),
                                 "frac_mfma_peak": round(flops_fwd / t_fwd / 1e9 / PEAK_BF16_TFLOPS, 4),
                                 "img_per_s": round(64 / (t_fwd * 1e-3), 1)},
                "per_layer_us": {n: round(t * 1e3, 1) for n, t in rows}, "per_layer_sum_ms": round(tot, 4),
                "ternarize_layers_GBps": round(n_w * 8.25 / (t_tern * 1e-3) / 1e9, 1),
                "gflop": flops_fwd / 1e9, "layers": len(layers), "block_heads_in_pair_calls": n_pairs}
        return info

    if args.calibrate:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    sides = {"gemm": side_gemm, "ternarize": lambda: side_ternarize(calibrate=True), "lenet": side_lenet,
             "vgg7": side_vgg7, "vgg16_ssd": side_vgg16, "resnet18_bwd": side_resnet18_bwd, "per_filter": side_per_filter,
             "sgd": side_sgd, "addsub": side_addsub, "resnet18b": side_resnet18b}
    if args.only and args.only != "resnet18":
        print(json.dumps({"only": args.only, **sides[args.only]()}), flush=True)
        return

    h = headline(with_cpu=not args.no_cpu and not args.only)
    extras = {"phase_ms": h["phase_ms"], "forward_only": h["forward_only"], "per_layer_us": h["per_layer_us"],
              "per_layer_sum_ms": h["per_layer_sum_ms"], "graph_replay": h["graph"],
              "ternarize_21_tensors_GBps": h["ternarize_layers_GBps"]}
    rooflines = [h["roof"]] + h["layer_roofs"]
    if not args.no_extras and not args.only:
        torch.cuda.empty_cache()
        args.variants = True
        rooflines.append(side_gemm())
        rooflines.append(side_ternarize())
        torch.cuda.empty_cache()
        rooflines.append(side_sgd())
        torch.cuda.empty_cache()
        rooflines.append(side_addsub())
        for name in ("lenet", "vgg7", "vgg16_ssd", "resnet18_bwd", "per_filter", "resnet18b"):
            torch.cuda.empty_cache()
            extras[name] = sides[name]()

    out = {
        "metric": "ternary conv/GEMM throughput, dense-equivalent TFLOP/s (2MNK per contraction) and fraction of bf16 MFMA "
                  "peak; ternarize GB/s; ResNet-18 img/s",
        "value": round(h["value"], 1), "unit": "TFLOP/s-eq", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(h["ms_per_step"], 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "resnet18_b64_bf16_twn_forward", "layers": h["layers"], "batch": 64, "delta_factor": F,
                   "step": "twn_ternarize_batch of all 21 weight tensors + forward of all 21 conv/FC layers (the three block "
                           "heads with a projection shortcut as one twn_conv2d_fwd_pair call each)",
                   "gflop_per_step": round(h["gflop"], 1), "img_per_s": round(64 / (h["ms_per_step"] * 1e-3), 1),
                   "frac_mfma_peak": round(h["value"] / PEAK_BF16_TFLOPS, 4)},
        "roofline": h["roof"],
        "rooflines": rooflines,
        "cpu_baseline": h["cpu"],
        "extras": extras,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
