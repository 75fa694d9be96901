#!/usr/bin/env python3
"""Benchmark of the fused-operator hot path on one MI355X.

A step is one pass of the whole hot path: one launch of each of the five fused
chains (GEMM+bias+ReLU+softmax, affine+ReLU+residual+avg-pool, layernorm+GELU,
conv3x3+bias+ReLU, GEMM-softmax-GEMM) at full size on seeded synthetic inputs
already resident in HBM.  The memory-bound chains rotate over buffer sets whose
total exceeds the 256 MB last-level cache, so their reads come from HBM.

Prints ONE JSON line.  `value` is the mean over the five operators of the
achieved fraction of the MI355X peak that bounds each (HBM 8 TB/s for the
memory-bound chains, 157.3 TFLOP/s fp32 MFMA for the contraction-anchored
ones), in percent; `per_op` carries every operator's absolute GB/s or TFLOP/s.
Per-kernel durations are measured inside the timed region with HIP events
recorded on the launch stream around each chain's group of launches.  `roofline` describes the
kernel that takes the largest share of a step.  `cpu_baseline` is the CPU
checker timed on this host (a reported baseline, not a target).
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

HBM_PEAK_GBS = 8000.0
MFMA_F32_PEAK_TFLOPS = 157.3
LLC_BYTES = 256 << 20

# algorithmic work per launch: inputs once, outputs once, fused intermediates never
OPS = {
    1: dict(name="gemm_bias_relu_softmax", bound="mfma", flop=2 * 64 * 256 * 256, bytes=(64 * 256 + 256 * 256 + 256 + 64 * 256) * 4),
    2: dict(name="scale_shift_relu_add_avgpool", bound="hbm", flop=0, bytes=(2 * 32 * 64 * 56 * 56 + 2 * 64 + 32 * 64) * 4),
    3: dict(name="layernorm_gelu", bound="hbm", flop=0, bytes=(2 * 8192 * 4096 + 2 * 4096) * 4),
    4: dict(name="conv3x3_bias_relu", bound="mfma", flop=2 * 32 * 128 * 56 * 56 * 64 * 9,
            bytes=(32 * 64 * 56 * 56 + 128 * 64 * 9 + 128 + 32 * 128 * 56 * 56) * 4),
    5: dict(name="attention_qk_softmax_v", bound="mfma", flop=4 * 16 * 2048 * 2048 * 64, bytes=4 * 16 * 2048 * 64 * 4),
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU checker")
    ap.add_argument("--only", type=int, default=0, help="run a single chain (1..5) instead of all five")
    ap.add_argument("--skip-extra", action="store_true",
                    help="leave out the side measurements of the later operators (GEMM + GELU, batched GEMM, first-layer conv, "
                         "pooling, group norm), whose kernels share symbols with the chains' and would mix into per-kernel counters")
    ap.add_argument("--with-copy", action="store_true",
                    help="after the timed region also launch the library's plain copy kernel on a 25 690 112-byte "
                         "tensor (reference dispatches for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this operator library is a one-GPU hot path with no collectives; run it with --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2506_10401_amd import datagen, hpct

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback", file=sys.stderr)
        return 2
    hpct.load()
    torch.cuda.set_device(0)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()  # noqa: E731
    which = [args.only] if args.only else [1, 2, 3, 4, 5]

    # ---- inputs (seeded, host-generated, uploaded once) -----------------------
    host = {i: datagen.make(i) for i in which}

    def rotated(t, k):
        # further buffer sets for cache-cold timing: same values, rolled, in distinct memory
        return t if k == 0 else torch.roll(t.flatten(), 1001 * k).reshape(t.shape).contiguous()

    sets = {}
    if 1 in which:
        h = host[1]
        sets[1] = [dict(ins=[dev(h["X"]), dev(h["W"]), dev(h["bias"])], out=torch.empty(64, 256, device="cuda"))]
    if 2 in which:
        h = host[2]
        X, R, sc, sh = dev(h["X"]), dev(h["R"]), dev(h["scale"]), dev(h["shift"])
        n = LLC_BYTES * 2 // (2 * X.numel() * 4) + 1
        sets[2] = [dict(ins=[rotated(X, k), sc, sh, rotated(R, k)], out=torch.empty(32, 64, device="cuda")) for k in range(n)]
    if 3 in which:
        h = host[3]
        X, g, b = dev(h["X"]), dev(h["gamma"]), dev(h["beta"])
        sets[3] = [dict(ins=[rotated(X, k), g, b], out=torch.empty(8192, 4096, device="cuda")) for k in range(3)]
    if 4 in which:
        h = host[4]
        sets[4] = [dict(ins=[dev(h["in"]), dev(h["wt"]), dev(h["bias"])], out=torch.empty(32, 128, 56, 56, device="cuda"))]
    if 5 in which:
        h = host[5]
        sets[5] = [dict(ins=[dev(h["Q"]), dev(h["K"]), dev(h["V"])], out=torch.empty(16, 2048, 64, device="cuda"))]

    def bound(i, s):
        a, o = s["ins"], s["out"]
        if i == 1:
            plan, ins = hpct.gemm_bias_relu_softmax_plan(a[0], a[1], a[2], o)
        elif i == 2:
            plan, ins = hpct.scale_shift_relu_add_pool_plan(a[0], a[1], a[2], a[3], o)
        elif i == 3:
            plan, ins = hpct.layernorm_gelu_plan(a[0], a[1], a[2], o, eps=1e-5)
        elif i == 4:
            plan, ins = hpct.conv2d_bias_relu_plan(a[0], a[1], a[2], o, stride=1, pad=1)
        else:
            plan, ins = hpct.attention_plan(a[0], a[1], a[2], o, scale=0.125)
        kernels[i] = plan.kernel_name
        return plan.bind(ins, [o])

    kernels = {}
    calls = {i: [bound(i, s) for s in sets[i]] for i in which}

    # A step is one launch of every chain.  The timed region runs K steps'
    # worth of launches grouped by chain (K launches of chain 1, then K of
    # chain 2, ...), each group bracketed by one HIP event pair on the launch
    # stream, so a chain's average launch duration is (its bracket) / K and
    # carries no event overhead per launch.
    def run(K, ev=None):
        for i in which:
            c = calls[i]
            n = len(c)
            if ev is not None:
                ev[i][0].record()
            for k in range(K):
                c[k % n]()
            if ev is not None:
                ev[i][1].record()

    run(args.warmup)
    torch.cuda.synchronize()
    ev = {i: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for i in which}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps, ev)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # ---- the same step as one captured HIP graph (the five launches in order, first buffer set of each chain),
    # replayed K times: what a serving loop that cannot afford five launch calls per step would run
    graph_step = None
    if not args.only:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            rebound = [bound(i, sets[i][0]) for i in which]   # bound to the stream the capture runs on
            for c in rebound:
                c()
            side.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for c in rebound:
                    c()
            for _ in range(min(args.warmup, 10)):
                graph.replay()
            side.synchronize()
            g0 = time.perf_counter()
            for _ in range(args.steps):
                graph.replay()
            side.synchronize()
            g1 = time.perf_counter()
        torch.cuda.current_stream().wait_stream(side)
        graph_step = dict(ms_per_step=round((g1 - g0) * 1e3 / args.steps, 4), launches_per_step=len(which),
                          note="one hipGraph replay per step (chains 2 and 3 on one buffer set, so warm in the last-level cache)")

    if args.with_copy:
        # no epilogue, no reduction: the affine chain degenerates to out = X, a copy of known size
        src = torch.empty(32, 64, 56, 56, device="cuda").normal_()
        dst = torch.empty_like(src)
        plan, ins = hpct.scale_shift_relu_add_pool_plan(src, None, None, None, dst, relu=False, pool=False)
        go = plan.bind(ins, [dst])
        for _ in range(args.steps):
            go()
        torch.cuda.synchronize()

    # ---- layout transforms (Table 1 LayoutTransform class; outside the step and the headline value)
    layout_ops = []
    if not args.only:
        def time_layout(name, views, outs, nbytes):
            calls_l = []
            for v, o in zip(views, outs):
                plan, ins = hpct.layout_transform_plan(v, o)
                calls_l.append(plan.bind(ins, [o]))
            for k in range(min(args.warmup, 10)):
                calls_l[k % len(calls_l)]()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for k in range(args.steps):
                calls_l[k % len(calls_l)]()
            e1.record()
            torch.cuda.synchronize()
            us = 1e3 * e0.elapsed_time(e1) / args.steps
            layout_ops.append(dict(op=name, kernel=plan.kernel_name, avg_us=round(us, 3), achieved=round(nbytes / us / 1e3, 1),
                                   unit="GB/s", peak=HBM_PEAK_GBS, frac=round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4),
                                   buffer_sets=len(calls_l)))
        xs = [s["ins"][0] for s in sets[2]]                    # 11 NCHW tensors [32,64,56,56]
        outs = [torch.empty(32, 56, 56, 64, device="cuda") for _ in xs]
        time_layout("nchw_to_nhwc_32x64x56x56", [x.permute(0, 2, 3, 1) for x in xs], outs, 2 * xs[0].numel() * 4)
        del outs
        ms = [s["ins"][0] for s in sets[3]]                    # 3 matrices [8192,4096]
        outs = [s["out"].view(4096, 8192) for s in sets[3]]    # reuse the layernorm outputs as destinations
        time_layout("transpose_8192x4096", [m.t() for m in ms], outs, 2 * ms[0].numel() * 4)

    # ---- reductions over one axis (Table 1 Reduction class; outside the step and the headline value)
    reduce_ops = []
    if not args.only:
        def time_reduce(name, views, axis, op, out_shape, nbytes):
            calls_r = []
            for v in views:
                o = torch.empty(out_shape, device="cuda", dtype=torch.int32 if op.startswith("arg") else torch.float32)
                plan, ins = hpct.reduce_axis_plan(v, o, axis, op)
                ws = torch.empty(plan.workspace_bytes // 4, device="cuda") if plan.workspace_bytes else None
                calls_r.append(plan.bind(ins, [o], workspace=ws))
            for k in range(min(args.warmup, 10)):
                calls_r[k % len(calls_r)]()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for k in range(args.steps):
                calls_r[k % len(calls_r)]()
            e1.record()
            torch.cuda.synchronize()
            us = 1e3 * e0.elapsed_time(e1) / args.steps
            reduce_ops.append(dict(op=name, kernel=plan.kernel_name, avg_us=round(us, 3), achieved=round(nbytes / us / 1e3, 1),
                                   unit="GB/s", peak=HBM_PEAK_GBS, frac=round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4),
                                   buffer_sets=len(calls_r)))
        ms = [s_["ins"][0] for s_ in sets[3]]                  # 3 matrices [8192,4096]
        time_reduce("sum_axis1_8192x4096", ms, 1, "sum", (8192,), ms[0].numel() * 4 + 8192 * 4)
        time_reduce("sum_axis0_8192x4096", ms, 0, "sum", (4096,), ms[0].numel() * 4 + 4096 * 4)
        time_reduce("argmax_axis1_8192x4096", ms, 1, "argmax", (8192,), ms[0].numel() * 4 + 8192 * 4)
        # row softmax (Table 1 Reduction "softmax") on the same matrices, into the layernorm outputs
        calls_s = []
        for s_ in sets[3]:
            plan_s, ins_s = hpct.softmax_rows_plan(s_["ins"][0], s_["out"])
            calls_s.append(plan_s.bind(ins_s, [s_["out"]]))
        for k in range(min(args.warmup, 10)):
            calls_s[k % len(calls_s)]()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for k in range(args.steps):
            calls_s[k % len(calls_s)]()
        e1.record()
        torch.cuda.synchronize()
        us = 1e3 * e0.elapsed_time(e1) / args.steps
        nb = 2 * ms[0].numel() * 4
        reduce_ops.append(dict(op="softmax_rows_8192x4096", kernel=plan_s.kernel_name, avg_us=round(us, 3),
                               achieved=round(nb / us / 1e3, 1), unit="GB/s", peak=HBM_PEAK_GBS,
                               frac=round(nb / us / 1e3 / HBM_PEAK_GBS, 4), buffer_sets=len(calls_s)))
        # elementwise chain on views (Table 1 Elementwise "add, relu"): matrix + bias row, ReLU
        calls_e = []
        for s_ in sets[3]:
            plan_e, ins_e = hpct.eltwise_plan(s_["ins"][0], s_["ins"][1].expand(8192, 4096), s_["out"], "add", True)
            calls_e.append(plan_e.bind(ins_e, [s_["out"]]))
        for k in range(min(args.warmup, 10)):
            calls_e[k % len(calls_e)]()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for k in range(args.steps):
            calls_e[k % len(calls_e)]()
        e1.record()
        torch.cuda.synchronize()
        us = 1e3 * e0.elapsed_time(e1) / args.steps
        nb = 2 * ms[0].numel() * 4 + 4096 * 4
        reduce_ops.append(dict(op="add_bias_row_relu_8192x4096", kernel=plan_e.kernel_name, avg_us=round(us, 3),
                               achieved=round(nb / us / 1e3, 1), unit="GB/s", peak=HBM_PEAK_GBS,
                               frac=round(nb / us / 1e3 / HBM_PEAK_GBS, 4), buffer_sets=len(calls_e)))
        # one-operand chain (Table 1 Elementwise "sin"): out = sin(X)
        calls_u = []
        for s_ in sets[3]:
            plan_u, ins_u = hpct.eltwise_map_plan(s_["ins"][0], s_["out"], ("sin",))
            calls_u.append(plan_u.bind(ins_u, [s_["out"]]))
        for k in range(min(args.warmup, 10)):
            calls_u[k % len(calls_u)]()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for k in range(args.steps):
            calls_u[k % len(calls_u)]()
        e1.record()
        torch.cuda.synchronize()
        us = 1e3 * e0.elapsed_time(e1) / args.steps
        nb = 2 * ms[0].numel() * 4
        reduce_ops.append(dict(op="sin_8192x4096", kernel=plan_u.kernel_name, avg_us=round(us, 3),
                               achieved=round(nb / us / 1e3, 1), unit="GB/s", peak=HBM_PEAK_GBS,
                               frac=round(nb / us / 1e3 / HBM_PEAK_GBS, 4), buffer_sets=len(calls_u)))
        xs = [s_["ins"][0] for s_ in sets[2]]                  # 11 NCHW tensors [32,64,56,56]
        calls_p = []
        for x in xs:
            o = torch.empty(32, 64, 28, 28, device="cuda")
            plan_p, ins_p = hpct.maxpool2x2_plan(x, o)
            calls_p.append(plan_p.bind(ins_p, [o]))
        for k in range(min(args.warmup, 10)):
            calls_p[k % len(calls_p)]()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for k in range(args.steps):
            calls_p[k % len(calls_p)]()
        e1.record()
        torch.cuda.synchronize()
        us = 1e3 * e0.elapsed_time(e1) / args.steps
        nb = xs[0].numel() * 4 * 5 // 4
        reduce_ops.append(dict(op="maxpool2x2_32x64x56x56", kernel=plan_p.kernel_name, avg_us=round(us, 3),
                               achieved=round(nb / us / 1e3, 1), unit="GB/s", peak=HBM_PEAK_GBS,
                               frac=round(nb / us / 1e3 / HBM_PEAK_GBS, 4), buffer_sets=len(calls_p)))
        time_reduce("argmax_channels_32x64x56x56", xs, 1, "argmax", (32, 56, 56), xs[0].numel() * 4 + 32 * 3136 * 4)
        time_reduce("mean_channels_32x64x56x56", xs, 1, "mean", (32, 56, 56), xs[0].numel() * 4 + 32 * 3136 * 4)

    # ---- [Matmul, Dropout, Mean, Softmax] (Section 5.3 case study; outside the step and the headline value)
    next_ops = []

    def timed(call, launches):
        """avg us per launch over `launches` launches after the same warm-up the five chains get"""
        for _ in range(args.warmup):
            call()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(launches):
            call()
        b.record()
        torch.cuda.synchronize()
        return 1e3 * a.elapsed_time(b) / launches

    if not args.only:
        t6 = {k: dev(v) for k, v in datagen.make(6).items()}
        M6, K6 = t6["X"].shape
        N6 = t6["W"].shape[1]
        out6 = torch.empty(M6, device="cuda")
        plan6, ins6 = hpct.matmul_dropout_mean_softmax_plan(t6["X"], t6["W"], t6["bias"], out6, datagen.CHAIN6_P,
                                                            datagen.CHAIN6_SEED)
        ws6 = torch.empty(max(1, plan6.workspace_bytes // 4), device="cuda")
        call6 = plan6.bind(ins6, [out6], workspace=ws6)
        n6 = max(1, args.steps // 2)
        us = timed(call6, n6)
        flop6 = 2.0 * M6 * K6 * N6
        next_ops.append(dict(op="matmul_dropout_mean_softmax_%dx%dx%d" % (M6, K6, N6), kernel=plan6.kernel_name,
                             launches=n6, avg_us=round(us, 3), achieved=round(flop6 / us / 1e6, 2), unit="TFLOP/s",
                             peak=MFMA_F32_PEAK_TFLOPS, frac=round(flop6 / us / 1e6 / MFMA_F32_PEAK_TFLOPS, 4),
                             note="all three kernels of the chain (GEMM with fused dropout and row sums, row means, softmax over rows)"))
        del t6, out6, ws6

        # VGG-style block: conv3x3 + bias + scale/shift + relu + 2x2 max pool at the shape of chain 4
        t7 = {k: dev(v) for k, v in datagen.make(7).items()}
        Nb7, C7, H7, W7 = t7["in"].shape
        K7 = t7["wt"].shape[0]
        out7 = torch.empty(Nb7, K7, H7 // 2, W7 // 2, device="cuda")
        plan7, ins7 = hpct.conv_block_plan(t7["in"], t7["wt"], t7["bias"], t7["scale"], t7["shift"], out7)
        call7 = plan7.bind(ins7, [out7])
        us = timed(call7, args.steps)
        flop7 = 2.0 * Nb7 * K7 * H7 * W7 * C7 * 9
        next_ops.append(dict(op="conv3x3_bias_scale_shift_relu_maxpool2_%dx%dx%dx%d_to_%d" % (Nb7, C7, H7, W7, K7),
                             kernel=plan7.kernel_name, launches=args.steps, avg_us=round(us, 3),
                             achieved=round(flop7 / us / 1e6, 2), unit="TFLOP/s", peak=MFMA_F32_PEAK_TFLOPS,
                             frac=round(flop7 / us / 1e6 / MFMA_F32_PEAK_TFLOPS, 4),
                             note="flop = the convolution's 2*N*K*Ho*Wo*C*R*S; the pooled output is a quarter of the conv output"))
        del t7, out7

        # causal attention at the shape of chain 5 (flop = only the visible (query, key) pairs)
        if 5 in sets:
            q5, k5, v5 = sets[5][0]["ins"]
            o5 = torch.empty_like(q5)
            plan5, ins5 = hpct.attention_plan(q5, k5, v5, o5, 0.125, causal=True)
            call5 = plan5.bind(ins5, [o5])
            us = timed(call5, args.steps)
            B5, L5, D5 = q5.shape
            flop5 = 4.0 * D5 * B5 * L5 * (L5 + 1) / 2
            next_ops.append(dict(op="causal_attention_%dx%dx%d" % (B5, L5, D5), kernel=plan5.kernel_name, launches=args.steps,
                                 avg_us=round(us, 3), achieved=round(flop5 / us / 1e6, 2), unit="TFLOP/s",
                                 peak=MFMA_F32_PEAK_TFLOPS, frac=round(flop5 / us / 1e6 / MFMA_F32_PEAK_TFLOPS, 4),
                                 note="flop = 4*D per visible (query, key) pair; masked pairs inside diagonal blocks are computed but not counted"))

        # depthwise 3x3 conv + bias + relu6 at a MobileNetV2 shape (memory-bound: bytes = input + output)
        dsets = []
        for v in range(3):
            xd = torch.randn(32, 144, 56, 56, device="cuda")
            od = torch.empty(32, 144, 56, 56, device="cuda")
            pland, insd = hpct.depthwise_conv_plan(xd, torch.randn(144, 1, 3, 3, device="cuda"), torch.randn(144, device="cuda"),
                                                   None, None, od, 1, 1, "relu6")
            dsets.append(pland.bind(insd, [od]))
        kd = [0]

        def calld():
            dsets[kd[0] % 3]()
            kd[0] += 1
        us = timed(calld, args.steps)
        nbd = 2 * 32 * 144 * 56 * 56 * 4
        next_ops.append(dict(op="depthwise_conv3x3_bias_relu6_32x144x56x56", kernel=pland.kernel_name, launches=args.steps,
                             avg_us=round(us, 3), achieved=round(nbd / us / 1e3, 1), unit="GB/s", peak=HBM_PEAK_GBS,
                             frac=round(nbd / us / 1e3 / HBM_PEAK_GBS, 4), buffer_sets=3))
        del dsets

        # operators built after those: one line each (rotated buffer sets for the memory-bound ones)
        def side_op(op, make, nsets, work, bound, note=None):
            if args.skip_extra:
                return
            calls, name = [], None
            for _ in range(nsets):
                plan_, ins_, out_, ws_ = make()
                name = plan_.kernel_name
                calls.append(plan_.bind(ins_, [out_], workspace=ws_))
            k = [0]

            def call():
                calls[k[0] % nsets]()
                k[0] += 1
            us_ = timed(call, args.steps)
            if bound == "hbm":
                ach, peak, unit = work / us_ / 1e3, HBM_PEAK_GBS, "GB/s"
            else:
                ach, peak, unit = work / us_ / 1e6, MFMA_F32_PEAK_TFLOPS, "TFLOP/s"
            e = dict(op=op, kernel=name, launches=args.steps, avg_us=round(us_, 3), achieved=round(ach, 1 if bound == "hbm" else 2),
                     unit=unit, peak=peak, frac=round(ach / peak, 4), buffer_sets=nsets)
            if note:
                e["note"] = note
            next_ops.append(e)

        def mk_mlp():
            X = torch.randn(4096, 1024, device="cuda"); W = torch.randn(1024, 4096, device="cuda") * 0.03
            b = torch.randn(4096, device="cuda"); o = torch.empty(4096, 4096, device="cuda")
            pl, ins_ = hpct.gemm_bias_relu_softmax_plan(X, W, b, o, relu="gelu", softmax=False)
            return pl, ins_, o, None
        side_op("gemm_bias_gelu_4096x1024x4096", mk_mlp, 1, 2.0 * 4096 * 1024 * 4096, "mfma")

        def mk_bmm():
            X = torch.randn(16, 1024, 1024, device="cuda"); W = torch.randn(16, 1024, 1024, device="cuda") * 0.03
            o = torch.empty(16, 1024, 1024, device="cuda")
            pl, ins_ = hpct.gemm_bias_relu_softmax_plan(X, W, None, o, relu=False, softmax=False)
            return pl, ins_, o, None
        side_op("batched_gemm_16x1024x1024x1024", mk_bmm, 1, 2.0 * 16 * 1024 ** 3, "mfma")

        def mk_qk():
            X = torch.randn(64, 512, 64, device="cuda"); W = torch.randn(64, 64, 512, device="cuda")
            o = torch.empty(64, 512, 512, device="cuda")
            pl, ins_ = hpct.gemm_bias_relu_softmax_plan(X, W, None, o, relu=False, softmax=False)
            return pl, ins_, o, None
        side_op("batched_gemm_short_k_64x512x64x512", mk_qk, 1, 2.0 * 64 * 512 * 64 * 512, "mfma",
             note="2K flop per 4 bytes written: at K = 64 the store and MFMA bounds are of the same size")

        def mk_first():
            x = torch.randn(32, 3, 224, 224, device="cuda"); w = torch.randn(64, 3, 3, 3, device="cuda") * 0.2
            b = torch.randn(64, device="cuda"); o = torch.empty(32, 64, 224, 224, device="cuda")
            pl, ins_ = hpct.conv_block_plan(x, w, b, None, None, o, 1, 1, True, False)
            return pl, ins_, o, None
        side_op("conv3x3_first_layer_32x3x224x224_to_64", mk_first, 1, (32 * 3 + 32 * 64) * 224 * 224 * 4.0, "hbm",
             note="store-bound: bytes = input + output (411 MB of output)")

        def mk_pool():
            x = torch.randn(32, 64, 112, 112, device="cuda"); o = torch.empty(32, 64, 56, 56, device="cuda")
            pl, ins_ = hpct.maxpool_plan(x, o, 3, 2, 1)
            return pl, ins_, o, None
        side_op("maxpool3x3_stride2_32x64x112x112", mk_pool, 4, 32 * 64 * (112 * 112 + 56 * 56) * 4.0, "hbm")

        def mk_gn():
            x = torch.randn(32, 64, 56, 56, device="cuda"); o = torch.empty_like(x)
            pl, ins_ = hpct.groupnorm_plan(x, torch.randn(64, device="cuda"), torch.randn(64, device="cuda"), o, 8, 1e-5, True)
            return pl, ins_, o, None
        side_op("groupnorm8_relu_32x64x56x56", mk_gn, 11, 2.0 * 32 * 64 * 56 * 56 * 4, "hbm")

    per_op, fracs = [], []
    for i in which:
        avg_us = 1e3 * ev[i][0].elapsed_time(ev[i][1]) / args.steps
        op = OPS[i]
        if op["bound"] == "hbm":
            ach, peak, unit = op["bytes"] / (avg_us * 1e-6) / 1e9, HBM_PEAK_GBS, "GB/s"
        else:
            ach, peak, unit = op["flop"] / (avg_us * 1e-6) / 1e12, MFMA_F32_PEAK_TFLOPS, "TFLOP/s"
        fracs.append(ach / peak)
        per_op.append(dict(config=i, op=op["name"], kernel=kernels[i], bound=op["bound"], avg_us=round(avg_us, 3),
                           achieved=round(ach, 3), unit=unit, peak=peak, frac=round(ach / peak, 4),
                           buffer_sets=len(sets[i])))
    for rec in per_op:
        rec["hbm_traffic_bytes"] = recorded_traffic(rec["kernel"])
    dom = max(per_op, key=lambda r: r["avg_us"])
    dop = OPS[dom["config"]]
    roofline = dict(kernel=dom["kernel"], bound=dom["bound"], achieved=dom["achieved"], peak=dom["peak"], unit=dom["unit"],
                    frac=dom["frac"], traffic=dom["hbm_traffic_bytes"], avg_us=dom["avg_us"],
                    algorithmic=dop["flop"] if dom["bound"] == "mfma" else dop["bytes"])

    out = dict(metric="per-op GB/s (memory-bound) or fp32 TFLOP/s (contraction) and % of MI355X peak",
               value=round(100.0 * sum(fracs) / len(fracs), 3), unit="% of MI355X peak, mean over the ops of a step",
               n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=round(ms_per_step, 4),
               higher_is_better=True, scaling="weak", vs_baseline=None, dtype="f32", data="synthetic",
               config=dict(workload="five fused chains at full size: gemm64x256x256+softmax, affine+pool 32x64x56x56, "
                                    "layernorm+gelu 8192x4096, conv3x3 32x64x56x56->128, attention 16x2048x64"
                           if not args.only else "chain %d only" % args.only,
                           ops=len(which), hbm_cold_sets={str(i): len(sets[i]) for i in which}),
               per_op=per_op, roofline=roofline, layout_ops=layout_ops, reduce_ops=reduce_ops, next_ops=next_ops,
               graph_step=graph_step)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(host, which)
    print(json.dumps(out))
    return 0


def recorded_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed FETCH_SIZE / WRITE_SIZE summary, or None if there is no
    record or the kernel's source file has changed since the counters were taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "hbm_traffic_five_chains.md")
    try:
        for line in open(path):
            if not line.startswith("TRAFFIC "):
                continue
            kv = dict(f.split("=", 1) for f in line.split()[1:])
            if kv.get("kernel") != kernel:
                continue
            src = os.path.join(ROOT, "paper_2506_10401_amd", "csrc", kv["source"])
            if hashlib.sha256(open(src, "rb").read()).hexdigest()[:16] != kv["sha256_16"]:
                return None
            return int(float(kv["bytes"]))
    except OSError:
        pass
    return None


def cpu_baseline(host, which):
    """The CPU checker as it stands, timed on this machine's host cores on the
    same five workloads at full size (one run each after loading the library)."""
    from oracle import ref
    ref.lib()
    threads = ref.max_threads()
    secs, fracs, per, total = {}, [], [], 0.0
    for i in which:
        h = host[i]
        def once():
            if i == 1:
                ref.chain1(h["X"], h["W"], h["bias"])
            elif i == 2:
                ref.chain2(h["X"], h["scale"], h["shift"], h["R"])
            elif i == 3:
                ref.chain3(h["X"], h["gamma"], h["beta"], 1e-5)
            elif i == 4:
                ref.relu(ref.conv2d_nchw_bias(h["in"], h["wt"], h["bias"], 1, 1))
            else:
                ref.attention(h["Q"], h["K"], h["V"], 0.125)
        once()  # first touch
        best, spent, reps = float("inf"), 0.0, 0
        while reps < 3 or (spent < 2.0 and reps < 50):
            t0 = time.perf_counter()
            once()
            dt = time.perf_counter() - t0
            best, spent, reps = min(best, dt), spent + dt, reps + 1
        secs[i] = best
        total += spent
        op = OPS[i]
        if op["bound"] == "hbm":
            ach, peak, unit = op["bytes"] / secs[i] / 1e9, HBM_PEAK_GBS, "GB/s"
        else:
            ach, peak, unit = op["flop"] / secs[i] / 1e12, MFMA_F32_PEAK_TFLOPS, "TFLOP/s"
        fracs.append(ach / peak)
        per.append(dict(config=i, seconds=round(secs[i], 4), achieved=round(ach, 5), unit=unit))
    return dict(value=round(100.0 * sum(fracs) / len(fracs), 5), unit="% of MI355X peak, mean over the ops of a step",
                cores=threads, kind="oracle",
                sample="all five workloads at full size; best of >= 3 passes each (about 2 s of passes per chain), "
                       "%.1f s of CPU time in total" % total,
                per_op=per)


if __name__ == "__main__":
    sys.exit(main())
