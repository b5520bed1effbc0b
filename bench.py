#!/usr/bin/env python3
"""Benchmark of the W2A4 GEMV path on one MI355X.

Workload ("llama2_7b_decode_bs1"): one decode token through the linear layers of a
LLaMA-2-7B-shaped model, 32 distinct decoder layers, batch 1.  Per layer the step runs

    quantise(x_attn)            -> GEMV q|k|v  (12288 x 4096: three 4096 x 4096 stacked)
    quantise(x_o)               -> GEMV o      ( 4096 x 4096)
    quantise(x_mlp)             -> GEMV gate|up (22016 x 4096: two 11008 x 4096 stacked)
    rotate H_64 (x) Q_172 + quantise(x_down) -> GEMV down (4096 x 11008)

i.e. the seven linears of the layer in four GEMV launches (projections that read the same
input share one launch; with one LUT per output channel stacking rows changes nothing).
The 32 layers hold different weights (1.6 GB packed), so every weight byte comes from HBM:
the working set is far larger than the 256 MB memory-side cache.  Weight packing is the
offline export step and is done once, outside the timed region.

One JSON line is printed: value = algorithmic bytes of the step / step time (GB/s).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
HIDDEN, INTER = 4096, 11008
KRON = (64, 172)


def gemv_bytes(N, K, M=1):
    """Algorithmic bytes of one GEMV: packed indices + LUT + x_q + S + fp16 output."""
    return N * K // 4 + 8 * N + M * K // 2 + 2 * M + 2 * M * N


def layer_launches():
    """(name, N, K, rotated) of the four GEMV launches of one decoder layer."""
    return [("qkv", 3 * HIDDEN, HIDDEN, False), ("o", HIDDEN, HIDDEN, False),
            ("gate_up", 2 * INTER, HIDDEN, False), ("down", HIDDEN, INTER, True)]


def make_layer(torch, rcp, dev, seed, layer):
    """Synthetic weights of one layer (same recipe as rcp_synth, drawn on the GPU), packed.
    The packed indices and LUTs of the layer's four launches sit in one contiguous buffer."""
    shapes = layer_launches()
    total = sum(N * K // 4 + 8 * N for (_, N, K, _) in shapes)
    blob = torch.empty(total, dtype=torch.uint8, device=dev)
    out, off = [], 0
    for i, (name, N, K, _) in enumerate(shapes):
        g = torch.Generator(device=dev)
        g.manual_seed(seed * 100003 + layer * 16 + i)
        W = (torch.randn((N, K), generator=g, device=dev, dtype=torch.float32) * 0.02).to(torch.float16)
        Wf = W.float()
        k_lo = max(1, int(round(0.01 * K)))
        lo = torch.kthvalue(Wf, k_lo, dim=1).values.contiguous()
        hi = torch.kthvalue(Wf, K - k_lo + 1, dim=1).values.contiguous()
        part = torch.softmax(torch.randn((N, 3), generator=g, device=dev, dtype=torch.float32), dim=1).contiguous()
        packed = blob[off:off + N * K // 4]
        cb = blob[off + N * K // 4:off + N * K // 4 + 8 * N].view(torch.float16).view(N, 4)
        off += N * K // 4 + 8 * N
        rcp.pack_weights(W, lo, hi, part, packed_out=packed, codebook_out=cb)
        out.append((packed, cb))
        del W, Wf
    return out, blob


def make_activation(torch, dev, seed, K):
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    x = torch.randn((1, K), generator=g, device=dev, dtype=torch.float32)
    outlier = torch.rand((1, K), generator=g, device=dev) < 0.01
    return torch.where(outlier, x * 20.0, x).to(torch.float16).contiguous()


def timed(torch, fn, reps):
    """Seconds per call of fn(), events on the current stream, synchronised on both sides."""
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / reps


def cpu_baseline():
    """The oracle as it stands, on the host cores: GEMVs of each LLaMA-2-7B shape plus the activation preparation,
    scaled to one decoder layer (4 x qkvo + 2 x gate/up + 1 x down); with all OpenMP threads (`value`, best of
    five per shape; the median beside it) and once more on a single thread."""
    import numpy as np

    import oracle
    import rcp_synth
    cores = oracle.max_threads()
    cases = []
    for (name, N, K, rot), count in zip(rcp_synth.CONFIGS["llama2_7b"], (4, 2, 1)):
        W, lo, hi, part = rcp_synth.linear_layer(0, "bench/" + name, N, K)
        packed, cb = oracle.pack_weights(W.astype(np.float32), lo, hi, part)
        x = rcp_synth.activation(0, "bench/" + name, 1, K)
        cases.append((N, K, rot, count, packed, cb, x))
    b_layer = sum(count * gemv_bytes(N, K) for (N, K, _, count, _, _, _) in cases)

    def layer_time(reps, pick):
        t_layer = 0.0
        for (N, K, rot, count, packed, cb, x) in cases:
            t0 = time.perf_counter()
            if rot is None:
                y = x.astype(np.float64)
            else:
                Q = rcp_synth.orthogonal(0, rot[2]).astype(np.float64)
                y = oracle.rotate(x.astype(np.float64), oracle.ROT_KRON, n_wht=rot[1], m=rot[2], Q=Q)
            xq, sc, _ = oracle.quantize_act(y.astype(np.float32), 1.0)
            t_act = time.perf_counter() - t0
            ts = []
            for _ in range(reps):
                t0 = time.perf_counter()
                oracle.w2a4_gemv(packed, cb, N, K, xq, sc, 1)
                ts.append(time.perf_counter() - t0)
            t_layer += count * pick(sorted(ts)) + t_act
        return t_layer
    t_min = layer_time(5, lambda ts: ts[0])
    t_med = layer_time(5, lambda ts: ts[len(ts) // 2])
    oracle.set_threads(1)
    t_one = layer_time(2, lambda ts: ts[0])
    oracle.set_threads(cores)
    return {"value": round(b_layer / t_min / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": "one GEMV of each llama2_7b shape (4096x4096, 11008x4096, 4096x11008; best of 5 runs each) + "
                      "activation preparation, scaled to one decoder layer (4+2+1 linears); oracle C code, fp64, OpenMP",
            "ms_per_layer": round(t_min * 1e3, 2), "ms_per_layer_median": round(t_med * 1e3, 2),
            "single_thread_ms_per_layer": round(t_one * 1e3, 2),
            "single_thread_GBps": round(b_layer / t_one / 1e9, 4)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly from python instead of replaying a HIP graph")
    ap.add_argument("--split", action="store_true",
                    help="separate rcp_rotate_quant_act + rcp_w2a4_gemv launches instead of the fused quantise+GEMV call")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sequence-only", action="store_true",
                    help="run only the chained layer as one rcp_quant_w2a4_gemv_sequence launch per layer (used for profiles)")
    ap.add_argument("--step-only", action="store_true",
                    help="skip the per-shape, plain-read and small-batch side measurements (used for profiles)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2502_15779_amd as rcp
    import rcp_synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    rcp.lib()  # raises if librcp.so is missing: there is no fallback
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    L = args.layers

    t_setup = time.perf_counter()
    made = [make_layer(torch, rcp, dev, args.seed, l) for l in range(L)]
    layers = [m[0] for m in made]
    blobs = [m[1] for m in made]
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup

    launches = layer_launches()
    Q = torch.from_numpy(rcp_synth.orthogonal(args.seed, KRON[1])).to(dev)
    rot_down = rcp.Rotation.kron(KRON[0], Q)
    xs = [make_activation(torch, dev, args.seed * 7 + i, K) for i, (_, _, K, _) in enumerate(launches)]
    xqs = [torch.empty((1, K // 2), dtype=torch.uint8, device=dev) for (_, _, K, _) in launches]
    scs = [torch.empty((1,), dtype=torch.float16, device=dev) for _ in launches]
    outs = [torch.empty((1, N), dtype=torch.float16, device=dev) for (_, N, _, _) in launches]
    ws = torch.empty(rcp.act_workspace_bytes(1, INTER, rot_down), dtype=torch.uint8, device=dev)

    ybuf = torch.empty((1, INTER), dtype=torch.float32, device=dev)
    fused = not args.split

    def act(i):
        """Activation preparation of linear i as its own launch(es)."""
        if fused:
            if launches[i][3]:
                rcp.rotate_act(xs[i], rot_down, y_out=ybuf)  # rotation only; quantised inside the GEMV
            return
        rot = rot_down if launches[i][3] else None
        rcp.rotate_quant_act(xs[i], rot, 1.0, xq_out=xqs[i], scale_out=scs[i], workspace=ws if rot else None)

    def gemv(l, i):
        _, N, K, rotated = launches[i]
        packed, cb = layers[l][i]
        if fused:
            rcp.quant_w2a4_gemv(packed, cb, N, K, ybuf if rotated else xs[i], 1.0, out=outs[i])
        else:
            rcp.w2a4_gemv(packed, cb, N, K, xqs[i], scs[i], 1, out=outs[i])

    def step_eager():
        for l in range(L):
            for i in range(4):
                act(i)
                gemv(l, i)

    def gemv_only_eager():
        for l in range(L):
            for i in range(4):
                gemv(l, i)

    def act_only_eager():
        for l in range(L):
            for i in range(4):
                act(i)

    def capture(fn):
        if args.no_graph:
            return fn
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g.replay

    if not fused:
        for i in range(4):  # the GEMV-only sweeps of the split path read these
            rot = rot_down if launches[i][3] else None
            rcp.rotate_quant_act(xs[i], rot, 1.0, xq_out=xqs[i], scale_out=scs[i], workspace=ws if rot else None)
    if args.sequence_only:
        co = [torch.zeros((1, N), dtype=torch.float16, device=dev) for (_, N, _, _) in launches]
        seqs = []
        for l in range(L):
            w = layers[l]
            seqs.append([rcp.GemvStep(w[0][0], w[0][1], 3 * HIDDEN, HIDDEN, xs[0], co[0]),
                         rcp.GemvStep(w[1][0], w[1][1], HIDDEN, HIDDEN, co[0][0, :HIDDEN], co[1]),
                         rcp.GemvStep(w[2][0], w[2][1], 2 * INTER, HIDDEN, co[1], co[2]),
                         rcp.GemvStep(w[3][0], w[3][1], HIDDEN, INTER, co[2][0, :INTER], co[3], rot=rot_down)])
        wsq = rcp.gemv_sequence_workspace(seqs[0])

        def seq_step():
            for st in seqs:
                rcp.quant_w2a4_gemv_sequence(st, wsq)
        seq_step()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            seq_step()
        for _ in range(args.warmup):
            g.replay()
        sec = timed(torch, g.replay, args.steps)
        lb = sum(gemv_bytes(N, K) for (_, N, K, _) in launches)
        print(json.dumps({"sequence_us_per_layer": round(sec / L * 1e6, 2), "GBps": round(L * lb / sec / 1e9, 1),
                          "layers": L, "steps": args.steps, "error_word": int(wsq[0].item())}))
        return

    step_eager()  # warm every code path before capture
    torch.cuda.synchronize()
    step = capture(step_eager)
    gemv_only = capture(gemv_only_eager)
    act_only = capture(act_only_eager)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # ---- the timed region: exactly args.steps steps ------------------------------------------
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    sec_per_step = e0.elapsed_time(e1) * 1e-3 / args.steps
    # ------------------------------------------------------------------------------------------

    step_bytes = L * sum(gemv_bytes(N, K) for (_, N, K, _) in launches)
    value = step_bytes / sec_per_step / 1e9

    # dominant kernel: the GEMV.  Average launch duration over the same 32-layer sweep,
    # GEMV launches only, events on the launch stream.
    reps = max(3, args.steps // 5)
    sec_gemv_sweep = timed(torch, gemv_only, reps)
    sec_act_sweep = timed(torch, act_only, reps)
    n_gemv = 4 * L
    gemv_avg_s = sec_gemv_sweep / n_gemv
    achieved = (step_bytes / n_gemv) / gemv_avg_s / 1e9

    # per-shape GEMV latency on the paper's own layer sizes, cold (32 different weight buffers):
    # the stacked buffers start with the q (resp. gate) rows, so a prefix is the single matrix
    per_shape = {}
    side_shapes = () if args.step_only else (("4096x4096", 1, HIDDEN), ("11008x4096", 2, INTER), ("4096x11008", 3, HIDDEN),
                                             ("12288x4096_qkv", 0, 3 * HIDDEN), ("22016x4096_gate_up", 2, 2 * INTER))
    for label, i, N in side_shapes:
        K = launches[i][2]

        def sweep(i=i, N=N, K=K):
            for l in range(L):
                packed, cb = layers[l][i]
                if fused:
                    rcp.quant_w2a4_gemv(packed, cb, N, K, ybuf if launches[i][3] else xs[i], 1.0, out=outs[i])
                else:
                    rcp.w2a4_gemv(packed, cb, N, K, xqs[i], scs[i], 1, out=outs[i])
        fn = capture(sweep)
        fn()
        s = timed(torch, fn, reps) / L
        b = gemv_bytes(N, K)
        per_shape[label] = {"us": round(s * 1e6, 3), "GBps": round(b / s / 1e9, 1),
                            "pct_hbm_peak": round(100.0 * b / s / 1e9 / HBM_PEAK_GBPS, 2)}

    # the same GEMV on activations quantised beforehand (rcp_w2a4_gemv): what the quantiser in the prologue costs
    if fused:
        for label, i, N in side_shapes:
            K = launches[i][2]
            rot = rot_down if launches[i][3] else None
            rcp.rotate_quant_act(xs[i], rot, 1.0, xq_out=xqs[i], scale_out=scs[i], workspace=ws if rot else None)

            def psweep(i=i, N=N, K=K):
                for l in range(L):
                    packed, cb = layers[l][i]
                    rcp.w2a4_gemv(packed, cb, N, K, xqs[i], scs[i], 1, out=outs[i])
            fn = capture(psweep)
            fn()
            per_shape[label]["prequantised_us"] = round(timed(torch, fn, reps) / L * 1e6, 3)

    # warm: the same launch on ONE layer's buffer over and over (weights resident in the 256 MB
    # memory-side cache after the first pass) -- reported apart from the cold numbers above
    for label, i, N in side_shapes:
        K = launches[i][2]

        def wsweep_warm(i=i, N=N, K=K):
            packed, cb = layers[0][i]
            for l in range(L):
                if fused:
                    rcp.quant_w2a4_gemv(packed, cb, N, K, ybuf if launches[i][3] else xs[i], 1.0, out=outs[i])
                else:
                    rcp.w2a4_gemv(packed, cb, N, K, xqs[i], scs[i], 1, out=outs[i])
        fn = capture(wsweep_warm)
        fn()
        s = timed(torch, fn, reps) / L
        per_shape[label]["warm_us"] = round(s * 1e6, 3)

    # the machine's streaming-read ceiling for buffers of these sizes: a plain 128-bit-load
    # kernel over the same packed weights (same cold 32-layer sweep), beside each shape
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    for label, i, N in side_shapes:
        K = launches[i][2]

        def rsweep(i=i, N=N, K=K):
            for l in range(L):
                rcp.stream_read(layers[l][i][0], N * K // 4, sink)
        fn = capture(rsweep)
        fn()
        s = timed(torch, fn, reps) / L
        per_shape[label]["plain_read_us"] = round(s * 1e6, 3)
        per_shape[label]["plain_read_GBps"] = round(N * K // 4 / s / 1e9, 1)

    # small-batch decode (M = 4, 8, 16 tokens): the same four launches per layer with M tokens,
    # activations prepared by rcp_rotate_quant_act; with three or more tokens the GEMMs run on the matrix cores
    small_batch = {}
    for M in (() if args.step_only else (4, 8, 16)):
        xm = [make_activation(torch, dev, 1000 + M * 7 + i, K).repeat(M, 1).contiguous() for i, (_, _, K, _) in enumerate(launches)]
        for i in range(4):
            xm[i] += torch.randn(xm[i].shape, device=dev, dtype=torch.float16) * 0.1
        xqm = [torch.empty((M, K // 2), dtype=torch.uint8, device=dev) for (_, _, K, _) in launches]
        scm = [torch.empty((M,), dtype=torch.float16, device=dev) for _ in launches]
        outm = [torch.empty((M, N), dtype=torch.float16, device=dev) for (_, N, _, _) in launches]
        wsm = torch.empty(rcp.act_workspace_bytes(M, INTER, rot_down), dtype=torch.uint8, device=dev)

        def mstep(M=M, xm=xm, xqm=xqm, scm=scm, outm=outm, wsm=wsm):
            for l in range(L):
                for i in range(4):
                    _, N, K, rotated = launches[i]
                    rot = rot_down if rotated else None
                    rcp.rotate_quant_act(xm[i], rot, 1.0, xq_out=xqm[i], scale_out=scm[i], workspace=wsm if rot else None)
                    packed, cb = layers[l][i]
                    rcp.w2a4_gemv(packed, cb, N, K, xqm[i], scm[i], M, out=outm[i])
        def mgemm(M=M, xqm=xqm, scm=scm, outm=outm):
            for l in range(L):
                for i in range(4):
                    _, N, K, _ = launches[i]
                    packed, cb = layers[l][i]
                    rcp.w2a4_gemv(packed, cb, N, K, xqm[i], scm[i], M, out=outm[i])
        mstep()
        fn = capture(mstep)
        fn()
        s = timed(torch, fn, max(2, reps // 2))
        fng = capture(mgemm)
        fng()
        sg = timed(torch, fng, max(2, reps // 2))
        macs = M * L * sum(N * K for (_, N, K, _) in launches)
        small_batch[f"M{M}"] = {"ms_per_step": round(s * 1e3, 4), "us_per_layer": round(s / L * 1e6, 2),
                                "gemm_only_us_per_layer": round(sg / L * 1e6, 2),
                                "gemm_only_GBps": round(L * sum(gemv_bytes(N, K, M) for (_, N, K, _) in launches) / sg / 1e9, 1),
                                "int4_TMAC_per_s": round(macs / s / 1e12, 2),
                                "tokens_per_s": round(M / s, 1)}
        del xm, xqm, scm, outm, wsm

    # group-wise LUTs (128 input channels per LUT, the paper's deployed setting): the grouped GEMV
    # on the same shapes, cold over L different buffers; indices and levels are random (the
    # kernel's time does not depend on their values), activations quantised by a separate launch
    grouped = {}
    for label, i, N in side_shapes:
        K = launches[i][2]
        NG = K // rcp.GROUP
        rot = rot_down if launches[i][3] else None
        rcp.rotate_quant_act(xs[i], rot, 1.0, xq_out=xqs[i], scale_out=scs[i], workspace=ws if rot else None)
        bufs = []
        for l in range(L):
            pk = torch.randint(0, 256, (N * K // 4,), dtype=torch.uint8, device=dev)
            lv = (torch.randn((N // 4, NG, 4, 4), device=dev) * 0.03).sort(dim=3).values.to(torch.float16).contiguous()
            bufs.append((pk, lv))
        og = torch.empty((1, N), dtype=torch.float16, device=dev)

        def gsweep(i=i, N=N, K=K, bufs=bufs, og=og):
            for pk, lv in bufs:
                rcp.w2a4_gemv_grouped(pk, lv, N, K, xqs[i], scs[i], out=og)
        gsweep()
        fn = capture(gsweep)
        fn()
        s = timed(torch, fn, reps) / L
        b = N * K // 4 + 8 * N * NG + K // 2 + 2 + 2 * N
        grouped[label] = {"us": round(s * 1e6, 3), "GBps": round(b / s / 1e9, 1), "bytes": b}
        del bufs, og

    # the whole one-token step with group-wise LUTs (the paper's deployed setting): same launch
    # structure as the headline step (rotation kernel + four fused quantise+GEMV launches per
    # layer), 32 different layers of random indices and levels
    grouped_step = None
    if not args.step_only:
        gl = []
        for l in range(L):
            per = []
            for (_, N, K, _) in launches:
                NG = K // rcp.GROUP
                pk = torch.randint(0, 256, (N * K // 4,), dtype=torch.uint8, device=dev)
                lv = (torch.randn((N // 4, NG, 4, 4), device=dev) * 0.03).sort(dim=3).values.to(torch.float16).contiguous()
                per.append((pk, lv))
            gl.append(per)

        def gstep():
            for l in range(L):
                for i, (_, N, K, rotated) in enumerate(launches):
                    if rotated:
                        rcp.rotate_act(xs[i], rot_down, y_out=ybuf)
                    pk, lv = gl[l][i]
                    rcp.quant_w2a4_gemv_grouped(pk, lv, N, K, ybuf if rotated else xs[i], 1.0, out=outs[i])
        gstep()
        fn = capture(gstep)
        fn()
        s = timed(torch, fn, max(3, args.steps // 2))
        gbytes = L * sum(N * K // 4 + 8 * N * (K // rcp.GROUP) + K // 2 + 2 + 2 * N for (_, N, K, _) in launches)
        grouped_step = {"ms_per_step": round(s * 1e3, 4), "GBps": round(gbytes / s / 1e9, 1),
                        "pct_of_hbm_peak": round(100.0 * gbytes / s / 1e9 / HBM_PEAK_GBPS, 2), "bytes_per_step": gbytes}
        # several tokens with group-wise LUTs: the four GEMMs of a layer, activations already quantised
        grouped_step["small_batch_gemm_only_us_per_layer"] = {}
        for M in (4, 8, 16):
            xqm = [torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device=dev) for (_, _, K, _) in launches]
            scm = [(torch.rand(M, device=dev) * 0.1 + 0.05).to(torch.float16) for _ in launches]
            outm = [torch.empty((M, N), dtype=torch.float16, device=dev) for (_, N, _, _) in launches]

            def ggemm(M=M, xqm=xqm, scm=scm, outm=outm):
                for l in range(L):
                    for i, (_, N, K, _) in enumerate(launches):
                        pk, lv = gl[l][i]
                        rcp.w2a4_gemm_grouped(pk, lv, N, K, xqm[i], scm[i], M, out=outm[i])
            ggemm()
            fn = capture(ggemm)
            fn()
            sg = timed(torch, fn, max(2, reps // 2))
            grouped_step["small_batch_gemm_only_us_per_layer"][f"M{M}"] = round(sg / L * 1e6, 2)
        del gl

    # activation preparation alone (latency-bound: microseconds only): rotation + int4 quantiser
    # as one call, one token, at the rotation sizes of the benchmark configurations
    act_us = {}
    if not args.step_only:
        cases = [("quant_only_4096", 4096, None), ("wht_512", 512, ("wht", 512, 1)), ("wht_2048", 2048, ("wht", 2048, 1)),
                 ("wht_4096", 4096, ("wht", 4096, 1)), ("wht_8192", 8192, ("wht", 8192, 1)),
                 ("kron_64x172", 11008, ("kron", 64, 172)), ("kron_512x28", 14336, ("kron", 512, 28)),
                 ("heads_32x128", 4096, ("heads", 32, 128))]
        for label, K, r in cases:
            xa = make_activation(torch, dev, 4242 + K, K)
            if r is None:
                rot = None
            elif r[0] == "wht":
                rot = rcp.Rotation.wht(K)
            elif r[0] == "heads":
                rot = rcp.Rotation.heads(r[1], r[2])
            else:
                rot = rcp.Rotation.kron(r[1], torch.from_numpy(rcp_synth.orthogonal(args.seed, r[2])).to(dev))
            wsa = torch.empty(max(rcp.act_workspace_bytes(1, K, rot), 16), dtype=torch.uint8, device=dev)
            xqa = torch.empty((1, K // 2), dtype=torch.uint8, device=dev)
            sca = torch.empty((1,), dtype=torch.float16, device=dev)

            def asweep(xa=xa, rot=rot, wsa=wsa, xqa=xqa, sca=sca):
                for _ in range(L):
                    rcp.rotate_quant_act(xa, rot, 1.0, xq_out=xqa, scale_out=sca, workspace=wsa)
            asweep()
            fn = capture(asweep)
            fn()
            act_us[label] = round(timed(torch, fn, reps) / L * 1e6, 3)

    # weight-only variant (fp16 activations, no quantiser): same packed weights, same cold sweep
    weight_only = {}
    for label, i, N in side_shapes:
        K = launches[i][2]
        xw = xs[i] if xs[i].dtype == torch.float16 else xs[i].to(torch.float16)

        def wsweep(i=i, N=N, K=K, xw=xw):
            for l in range(L):
                packed, cb = layers[l][i]
                rcp.w2a16_gemv(packed, cb, N, K, xw, out=outs[i])
        wsweep()
        fn = capture(wsweep)
        fn()
        s = timed(torch, fn, reps) / L
        b = N * K // 4 + 8 * N + 2 * K + 2 * N
        weight_only[label] = {"us": round(s * 1e6, 3), "GBps": round(b / s / 1e9, 1)}

    # the whole one-token step with 16-bit activations (the paper's W2-only decode setting): rotation kernel + four
    # rcp_w2a16_gemv launches per layer on the headline step's weights, the down input as the rotated binary32 vector
    weight_only_step = None
    if not args.step_only:
        def wostep():
            for l in range(L):
                for i, (_, N, K, rotated) in enumerate(launches):
                    if rotated:
                        rcp.rotate_act(xs[i], rot_down, y_out=ybuf)
                    packed, cb = layers[l][i]
                    rcp.w2a16_gemv(packed, cb, N, K, ybuf if rotated else xs[i], out=outs[i])
        wostep()
        fn = capture(wostep)
        fn()
        s = timed(torch, fn, max(3, args.steps // 2))
        wobytes = L * sum(N * K // 4 + 8 * N + (4 if rotated else 2) * K + 2 * N for (_, N, K, rotated) in launches)
        weight_only_step = {"ms_per_step": round(s * 1e3, 4), "GBps": round(wobytes / s / 1e9, 1),
                            "pct_of_hbm_peak": round(100.0 * wobytes / s / 1e9 / HBM_PEAK_GBPS, 2), "bytes_per_step": wobytes}

    # 3-bit variant (eight levels per output channel): pre-quantised activations, cold over L weight sets
    w3 = {}
    for label, i, N in side_shapes:
        K = launches[i][2]
        w3sets = [(torch.randint(0, 256, (3 * N * K // 8,), dtype=torch.uint8, device=dev),
                   (torch.randn((N, 8), device=dev) * 0.03).sort(dim=1).values.to(torch.float16).contiguous())
                  for _ in range(L)]
        xq3 = torch.randint(0, 256, (K // 2,), dtype=torch.uint8, device=dev)
        sc3 = torch.full((1,), 0.07, dtype=torch.float16, device=dev)

        def w3sweep(i=i, N=N, K=K, w3sets=w3sets, xq3=xq3, sc3=sc3):
            for pk, cb in w3sets:
                rcp.w3a4_gemv(pk, cb, N, K, xq3, sc3, out=outs[i])
        w3sweep()
        fn = capture(w3sweep)
        fn()
        s = timed(torch, fn, reps) / L
        b = 3 * N * K // 8 + 16 * N + K // 2 + 2 + 2 * N
        w3[label] = {"us": round(s * 1e6, 3), "GBps": round(b / s / 1e9, 1)}

        def w3fused(i=i, N=N, K=K, w3sets=w3sets):   # quantiser fused into the prologue, raw fp16 activations
            for pk, cb in w3sets:
                rcp.quant_w3a4_gemv(pk, cb, N, K, xs[i] if not launches[i][3] else ybuf, 1.0, out=outs[i])
        w3fused()
        fn = capture(w3fused)
        fn()
        s = timed(torch, fn, reps) / L
        w3[label]["fused_us"] = round(s * 1e6, 3)
        del w3sets

    # the whole one-token step with 3-bit weights: the launch structure of the headline step (rotation kernel +
    # four fused quantise+GEMV launches per layer), 32 different layers of random indices and levels
    w3_step = None
    if not args.step_only:
        wl = [[(torch.randint(0, 256, (3 * N * K // 8,), dtype=torch.uint8, device=dev),
                (torch.randn((N, 8), device=dev) * 0.03).sort(dim=1).values.to(torch.float16).contiguous())
               for (_, N, K, _) in launches] for _ in range(L)]

        def w3step():
            for l in range(L):
                for i, (_, N, K, rotated) in enumerate(launches):
                    if rotated:
                        rcp.rotate_act(xs[i], rot_down, y_out=ybuf)
                    pk, cb = wl[l][i]
                    rcp.quant_w3a4_gemv(pk, cb, N, K, ybuf if rotated else xs[i], 1.0, out=outs[i])
        w3step()
        fn = capture(w3step)
        fn()
        s = timed(torch, fn, max(3, args.steps // 2))
        wbytes = L * sum(3 * N * K // 8 + 16 * N + K // 2 + 2 + 2 * N for (_, N, K, _) in launches)
        w3_step = {"ms_per_step": round(s * 1e3, 4), "GBps": round(wbytes / s / 1e9, 1),
                   "pct_of_hbm_peak": round(100.0 * wbytes / s / 1e9 / HBM_PEAK_GBPS, 2), "bytes_per_step": wbytes}

    # 4-bit KV cache, one query token (LLaMA-2-7B: 32 heads of 128), cold over L layers' caches.  One layer's
    # keys and values are drawn and quantised by the library, then copied into L separate caches.
    kv4 = {}
    Hh = 32
    for S in (() if args.step_only else (1024, 4096)):
        kx = torch.from_numpy(rcp_synth.kv_vectors(args.seed, f"bench_k{S}", S, Hh)).to(dev)
        vx = torch.from_numpy(rcp_synth.kv_vectors(args.seed, f"bench_v{S}", S, Hh)).to(dev)
        kc0, kp0 = rcp.kv4_new_cache(Hh, S, dev)
        vc0, vp0 = rcp.kv4_new_cache(Hh, S, dev)
        rcp.kv4_append(kx, 0, kc0, kp0, rotate=True)
        rcp.kv4_append(vx, 0, vc0, vp0)
        kcaches = [(kc0.clone(), kp0.clone(), vc0.clone(), vp0.clone()) for _ in range(L)]
        qv = torch.from_numpy(rcp_synth.query_vectors(args.seed, "bench_q", Hh)).to(dev)
        ov = torch.empty((Hh, 128), dtype=torch.float32, device=dev)
        wsk = torch.empty(rcp.kv4_workspace_bytes(Hh, S), dtype=torch.uint8, device=dev)

        def ksweep(S=S, kcaches=kcaches, qv=qv, ov=ov, wsk=wsk):
            for c in kcaches:
                rcp.kv4_attn_decode(qv, S, *c, 0.08838834764831845, out=ov, workspace=wsk)
        ksweep()
        fn = capture(ksweep)
        fn()
        s = timed(torch, fn, reps) / L
        b = 2 * S * Hh * 68 + Hh * 128 * (2 + 4)

        def asweep_kv(kx=kx, kcaches=kcaches, S=S):
            for c in kcaches:
                rcp.kv4_append(kx[:1], S - 1, c[0], c[1], rotate=True)   # a new key: R3, then the quantiser
        asweep_kv()
        fn = capture(asweep_kv)
        fn()
        sa = timed(torch, fn, reps) / L
        qraw = qv.to(torch.float16)

        def ksweep_rot(S=S, kcaches=kcaches, qraw=qraw, ov=ov, wsk=wsk):   # R3 on the query inside the attention launch
            for c in kcaches:
                rcp.kv4_rotate_attn_decode(qraw, S, *c, 0.08838834764831845, out=ov, workspace=wsk)
        ksweep_rot()
        fn = capture(ksweep_rot)
        fn()
        sf = timed(torch, fn, reps) / L

        def asweep_kv2(kx=kx, vx=vx, kcaches=kcaches, S=S):   # new key and new value in one launch
            for c in kcaches:
                rcp.kv4_append_kv(kx[:1], vx[:1], S - 1, c[0], c[1], c[2], c[3], rotate_k=True)
        asweep_kv2()
        fn = capture(asweep_kv2)
        fn()
        sa2 = timed(torch, fn, reps) / L
        kv4[f"S{S}"] = {"attn_us": round(s * 1e6, 3), "attn_GBps": round(b / s / 1e9, 1),
                        "rotate_attn_us": round(sf * 1e6, 3),
                        "append_one_token_us": round(sa * 1e6, 3), "append_key_and_value_one_launch_us": round(sa2 * 1e6, 3)}
        del kcaches

    # several sequences in one call (pooled caches): enough distinct pools to exceed the 256 MB memory-side cache
    # several times (at least 1.2 GB in total), and at least 32 launches per graph replay
    kv4_batched = {}
    for B, S in (() if args.step_only else ((8, 1024), (16, 1024), (8, 4096), (16, 4096))):
        nl = min(32, max(4, int(1.2e9 // (2 * B * Hh * S * 68))))
        nrep = (32 + nl - 1) // nl
        pools = []
        for _ in range(nl):
            kc = torch.randint(0, 256, (B * Hh, S, 64), dtype=torch.uint8, device=dev)
            vc = torch.randint(0, 256, (B * Hh, S, 64), dtype=torch.uint8, device=dev)
            par = torch.empty((B * Hh, S, 2), dtype=torch.int16, device=dev)
            par[..., 0] = 0x2C00   # step 1/16
            par[..., 1] = 8
            kp = par.view(torch.uint8).reshape(B * Hh, S, 4).contiguous()
            pools.append((kc, kp, vc, kp.clone()))
        qb = torch.randn((B, Hh, 128), device=dev).to(torch.float16)
        ob = torch.empty((B, Hh, 128), dtype=torch.float32, device=dev)
        wsb = torch.empty(B * rcp.kv4_workspace_bytes(Hh, S), dtype=torch.uint8, device=dev)
        newtok = torch.randn((B, Hh, 128), device=dev).to(torch.float16)

        def bsweep(pools=pools, qb=qb, ob=ob, wsb=wsb, B=B, S=S, nrep=nrep):
            for _ in range(nrep):
                for c in pools:
                    rcp.kv4_attn_decode_batched(qb, [S] * B, *c, 0.08838834764831845, out=ob, workspace=wsb)
        bsweep()
        fn = capture(bsweep)
        fn()
        s = timed(torch, fn, reps) / (nl * nrep)

        def basweep(pools=pools, newtok=newtok, B=B, S=S, nrep=nrep):
            for _ in range(nrep):
                for c in pools:
                    rcp.kv4_append_batched(newtok, [S - 1] * B, c[0], c[1], rotate=True)
        basweep()
        fn = capture(basweep)
        fn()
        sa = timed(torch, fn, reps) / (nl * nrep)
        bb = 2 * B * S * Hh * 68
        kv4_batched[f"B{B}_S{S}"] = {"attn_us": round(s * 1e6, 3), "attn_GBps": round(bb / s / 1e9, 1),
                                    "append_us": round(sa * 1e6, 3), "pools": nl}
        del pools

    # The linear layers and the KV-cache launches of a W2A4KV4 decode step chained as in a decoder layer, 4096
    # cached tokens: q|k|v GEMV -> R3 on the query heads -> append k (rotated) and v -> attention over the 4-bit
    # cache -> o GEMV on its output -> gate|up GEMV -> Kronecker rotation -> down GEMV: 11 launches per layer.
    # (RoPE, norms, the gated activation and the residual adds are not part of this library: the o input is the
    # attention output itself, the other GEMVs read the synthetic activations of the headline step.)
    kv_layer = None
    if not args.step_only:
        S_ctx = 4096
        kx = torch.from_numpy(rcp_synth.kv_vectors(args.seed, "layer_k", S_ctx, Hh)).to(dev)
        vx = torch.from_numpy(rcp_synth.kv_vectors(args.seed, "layer_v", S_ctx, Hh)).to(dev)
        kc0, kp0 = rcp.kv4_new_cache(Hh, S_ctx, dev)
        vc0, vp0 = rcp.kv4_new_cache(Hh, S_ctx, dev)
        rcp.kv4_append(kx, 0, kc0, kp0, rotate=True)
        rcp.kv4_append(vx, 0, vc0, vp0)
        lcaches = [(kc0.clone(), kp0.clone(), vc0.clone(), vp0.clone()) for _ in range(L)]
        rot_head = rcp.Rotation.wht(128)
        q_rot = torch.empty((Hh, 128), dtype=torch.float32, device=dev)
        attn_out = torch.empty((Hh, 128), dtype=torch.float32, device=dev)
        wsl = torch.empty(rcp.kv4_workspace_bytes(Hh, S_ctx), dtype=torch.uint8, device=dev)
        i_qkv, i_o, i_gu, i_down = 0, 1, 2, 3
        assert launches[i_qkv][1] == 3 * HIDDEN and launches[i_o][1:3] == (HIDDEN, HIDDEN) and launches[i_down][3]
        qkv = outs[i_qkv]

        def w2(l, i, x, N, K, out):
            pk, cb = layers[l][i]
            rcp.quant_w2a4_gemv(pk, cb, N, K, x, 1.0, out=out)

        def w3g(l, i, x, N, K, out):
            pk, cb = wl[l][i]
            rcp.quant_w3a4_gemv(pk, cb, N, K, x, 1.0, out=out)

        def kvstep(gemv_call):
            for l in range(L):
                gemv_call(l, i_qkv, xs[i_qkv], 3 * HIDDEN, HIDDEN, qkv)
                rcp.rotate_act(qkv[0, :HIDDEN].view(Hh, 128), rot_head, y_out=q_rot)
                kc, kp, vc, vp = lcaches[l]
                rcp.kv4_append(qkv[0, HIDDEN:2 * HIDDEN].view(1, Hh, 128), S_ctx - 1, kc, kp, rotate=True)
                rcp.kv4_append(qkv[0, 2 * HIDDEN:].view(1, Hh, 128), S_ctx - 1, vc, vp)
                rcp.kv4_attn_decode(q_rot, S_ctx, kc, kp, vc, vp, 0.08838834764831845, out=attn_out, workspace=wsl)
                gemv_call(l, i_o, attn_out.view(1, HIDDEN), HIDDEN, HIDDEN, outs[i_o])
                gemv_call(l, i_gu, xs[i_gu], launches[i_gu][1], HIDDEN, outs[i_gu])
                rcp.rotate_act(xs[i_down], rot_down, y_out=ybuf)
                gemv_call(l, i_down, ybuf, HIDDEN, INTER, outs[i_down])

        def kvstep_fused(gemv_call):
            # the same chain in 8 launches: keys and values appended together, R3 on the query inside the attention
            # launch
            for l in range(L):
                gemv_call(l, i_qkv, xs[i_qkv], 3 * HIDDEN, HIDDEN, qkv)
                kc, kp, vc, vp = lcaches[l]
                rcp.kv4_append_kv(qkv[0, HIDDEN:2 * HIDDEN].view(1, Hh, 128), qkv[0, 2 * HIDDEN:].view(1, Hh, 128), S_ctx - 1,
                                  kc, kp, vc, vp, rotate_k=True)
                rcp.kv4_rotate_attn_decode(qkv[0, :HIDDEN].view(Hh, 128), S_ctx, kc, kp, vc, vp, 0.08838834764831845,
                                           out=attn_out, workspace=wsl)
                gemv_call(l, i_o, attn_out.view(1, HIDDEN), HIDDEN, HIDDEN, outs[i_o])
                gemv_call(l, i_gu, xs[i_gu], launches[i_gu][1], HIDDEN, outs[i_gu])
                rcp.rotate_act(xs[i_down], rot_down, y_out=ybuf)
                gemv_call(l, i_down, ybuf, HIDDEN, INTER, outs[i_down])
        kv_layer = {"launches_per_layer": 11, "launches_per_layer_fused": 8, "cached_tokens": S_ctx, "heads": Hh}
        for label, call in (("w2a4kv4", w2), ("w3a4kv4", w3g)):
            kvstep(call)
            fn = capture(lambda call=call: kvstep(call))
            fn()
            s = timed(torch, fn, max(3, args.steps // 2))
            ref_attn = attn_out.clone()
            kvstep_fused(call)
            fn = capture(lambda call=call: kvstep_fused(call))
            fn()
            sfu = timed(torch, fn, max(3, args.steps // 2))
            kv_layer[label] = {"ms_per_step": round(s * 1e3, 4), "us_per_layer": round(s / L * 1e6, 2),
                               "fused_ms_per_step": round(sfu * 1e3, 4), "fused_us_per_layer": round(sfu / L * 1e6, 2),
                               "fused_same_bits": bool(torch.equal(ref_attn, attn_out))}
        del lcaches, wl

    # The other layer sizes of the paper's GEMV-latency tables (LLaMA-3.2-1B and LLaMA-3-8B configurations, and the
    # tiny configuration), each with the rotation its input needs, cold over L different weight buffers (random
    # indices and levels: the kernel's time does not depend on their values), a plain read of the same bytes beside it.
    other = {}
    if not args.step_only:
        ocases = [("256x512_wht512", 256, 512, ("wht", 512)), ("2048x2048", 2048, 2048, None),
                  ("2048x2048_wht2048", 2048, 2048, ("wht", 2048)), ("8192x2048", 8192, 2048, None),
                  ("2048x8192_wht8192", 2048, 8192, ("wht", 8192)), ("1024x4096", 1024, 4096, None),
                  ("14336x4096", 14336, 4096, None), ("4096x14336_kron512x28", 4096, 14336, ("kron", 512, 28))]
        for label, N, K, r in ocases:
            nbuf = max(L, min(256, int(3.0e8 // (N * K // 4)) + 1))      # more than the 256 MB memory-side cache in total
            bufs = [(torch.randint(0, 256, (N * K // 4,), dtype=torch.uint8, device=dev),
                     (torch.randn((N, 4), device=dev) * 0.03).sort(dim=1).values.to(torch.float16).contiguous()) for _ in range(nbuf)]
            xa = make_activation(torch, dev, 777 + K, K)
            oo = torch.empty((1, N), dtype=torch.float16, device=dev)
            xqo = torch.empty((1, K // 2), dtype=torch.uint8, device=dev)
            sco = torch.empty((1,), dtype=torch.float16, device=dev)
            yo = torch.empty((1, K), dtype=torch.float32, device=dev)
            if r is None:
                rot = None
            elif r[0] == "wht":
                rot = rcp.Rotation.wht(K)
            else:
                rot = rcp.Rotation.kron(r[1], torch.from_numpy(rcp_synth.orthogonal(args.seed, r[2])).to(dev))

            def osweep(bufs=bufs, N=N, K=K, rot=rot, r=r, xa=xa, oo=oo, xqo=xqo, sco=sco, yo=yo, gemv_only=False, two=False):
                for pk, lv in bufs:
                    if r is None:
                        rcp.quant_w2a4_gemv(pk, lv, N, K, xa, 1.0, out=oo)
                    elif r[0] == "wht" and K <= 2048 and not two and not gemv_only:   # short rotation: inside the GEMV launch
                        rcp.rotate_quant_w2a4_gemv(pk, lv, N, K, xa, rot, 1.0, out=oo)
                    elif r[0] == "wht":        # rotate + quantise in one kernel, then the GEMV
                        if not gemv_only:
                            rcp.rotate_quant_act(xa, rot, 1.0, xq_out=xqo, scale_out=sco)
                        rcp.w2a4_gemv(pk, lv, N, K, xqo, sco, 1, out=oo)
                    else:                      # rotation kernel, then the fused quantise + GEMV
                        if not gemv_only:
                            rcp.rotate_act(xa, rot, y_out=yo)
                        rcp.quant_w2a4_gemv(pk, lv, N, K, yo, 1.0, out=oo)
            osweep()
            fn = capture(osweep)
            fn()
            sec = timed(torch, fn, reps) / nbuf
            b = gemv_bytes(N, K)
            other[label] = {"us": round(sec * 1e6, 3), "GBps": round(b / sec / 1e9, 1), "buffers": nbuf}
            if r is not None:
                fn = capture(lambda: osweep(gemv_only=True))
                fn()
                other[label]["gemv_launch_only_us"] = round(timed(torch, fn, reps) / nbuf * 1e6, 3)
                if r[0] == "wht" and K <= 2048:
                    fn = capture(lambda: osweep(two=True))
                    fn()
                    other[label]["rotation_as_its_own_launch_us"] = round(timed(torch, fn, reps) / nbuf * 1e6, 3)

            def orsweep(bufs=bufs, N=N, K=K):
                for pk, _ in bufs:
                    rcp.stream_read(pk, N * K // 4, sink)
            fn = capture(orsweep)
            fn()
            other[label]["plain_read_us"] = round(timed(torch, fn, reps) / nbuf * 1e6, 3)
            del bufs

    # The same kernel where the launch is a small part of the time: a matrix of 131072 x 4096 (134 MB of packed weights, the
    # size of a LLaMA-3 vocabulary projection), cold over 8 buffers, against a plain read of the same bytes -- what the
    # kernel sustains once a launch is long enough to stream.
    large = {}
    if not args.step_only:
        N, K, nbuf = 131072, HIDDEN, 8
        bufs = [(torch.randint(0, 256, (N * K // 4,), dtype=torch.uint8, device=dev),
                 (torch.randn((N, 4), device=dev) * 0.03).sort(dim=1).values.to(torch.float16).contiguous()) for _ in range(nbuf)]
        xl = torch.randn((1, K), device=dev).to(torch.float16)
        xql, scl = rcp.rotate_quant_act(xl)
        ol = torch.empty((1, N), dtype=torch.float16, device=dev)
        b = gemv_bytes(N, K)

        def lsweep_q():
            for pk, cb in bufs:
                rcp.w2a4_gemv(pk, cb, N, K, xql, scl, 1, out=ol)

        def lsweep_f():
            for pk, cb in bufs:
                rcp.quant_w2a4_gemv(pk, cb, N, K, xl, 1.0, out=ol)

        def lsweep_r():
            for pk, _ in bufs:
                rcp.stream_read(pk, N * K // 4, sink)
        for key, sweep in (("prequantised", lsweep_q), ("fused_quantise", lsweep_f), ("plain_read", lsweep_r)):
            sweep()
            fn = capture(sweep)
            fn()
            sec = min(timed(torch, fn, 3), timed(torch, fn, 3)) / nbuf
            bb = b if key != "plain_read" else N * K // 4
            large[key + "_us"] = round(sec * 1e6, 2)
            large[key + "_GBps"] = round(bb / sec / 1e9, 1)
        large.update({"shape": f"{N}x{K}", "bytes": b, "buffers": nbuf,
                      "pct_of_hbm_peak": round(large["prequantised_GBps"] / HBM_PEAK_GBPS * 100, 1)})
        # the widened kernels on the same shape (activations quantised beforehand where they are quantised at all)
        NG = K // rcp.GROUP
        lvs = [(torch.randn((N // 4, NG, 4, 4), device=dev) * 0.03).sort(dim=3).values.to(torch.float16).contiguous()
               for _ in range(nbuf)]

        def lsweep_g():
            for (pk, _), lv in zip(bufs, lvs):
                rcp.w2a4_gemv_grouped(pk, lv, N, K, xql, scl, out=ol)

        def lsweep_wo():
            for pk, cb in bufs:
                rcp.w2a16_gemv(pk, cb, N, K, xl, out=ol)
        others = {}
        for key, sweep, bb in (("grouped_128", lsweep_g, N * K // 4 + 8 * N * NG + K // 2 + 2 + 2 * N),
                               ("weight_only_fp16", lsweep_wo, N * K // 4 + 8 * N + 2 * K + 2 * N)):
            sweep()
            fn = capture(sweep)
            fn()
            sec = min(timed(torch, fn, 3), timed(torch, fn, 3)) / nbuf
            others[key] = {"us": round(sec * 1e6, 2), "GBps": round(bb / sec / 1e9, 1), "bytes": bb}
        del bufs, lvs
        bufs3 = [(torch.randint(0, 256, (3 * N * K // 8,), dtype=torch.uint8, device=dev),
                  (torch.randn((N, 8), device=dev) * 0.03).sort(dim=1).values.to(torch.float16).contiguous()) for _ in range(nbuf)]

        def lsweep_3():
            for pk, cb in bufs3:
                rcp.w3a4_gemv(pk, cb, N, K, xql, scl, out=ol)
        lsweep_3()
        fn = capture(lsweep_3)
        fn()
        sec = min(timed(torch, fn, 3), timed(torch, fn, 3)) / nbuf
        bb = 3 * N * K // 8 + 16 * N + K // 2 + 2 + 2 * N
        others["w3a4"] = {"us": round(sec * 1e6, 2), "GBps": round(bb / sec / 1e9, 1), "bytes": bb}
        large["other_kernels"] = others
        del bufs3

    # What a dependent launch costs on this machine, and what the same dependency costs inside one launch:
    # (a) a chain of launches that read 16 bytes each; (b) a chain of the smallest fused GEMV (64 x 128) as launches;
    # (c) the same 16 GEMVs as one rcp_quant_w2a4_gemv_sequence call -- per entry that is one meeting of all
    # workgroups plus the quantiser on 128 values.
    floor = {}
    if not args.step_only:
        tiny = torch.zeros(64, dtype=torch.uint8, device=dev)

        def fsweep():
            for _ in range(64):
                rcp.stream_read(tiny, 16, sink)
        fn = capture(fsweep)
        fn()
        floor["dependent_16_byte_read_launch_us"] = round(timed(torch, fn, reps * 4) / 64 * 1e6, 3)
        tw = torch.randint(0, 256, (64 * 128 // 4,), dtype=torch.uint8, device=dev)
        tl = (torch.randn((64, 4), device=dev) * 0.03).sort(dim=1).values.to(torch.float16).contiguous()
        ta = [torch.randn((1, 128), device=dev).to(torch.float16)] + [torch.zeros((1, 128), dtype=torch.float16, device=dev) for _ in range(16)]

        def tsweep():
            for _ in range(4):
                for i in range(16):
                    rcp.quant_w2a4_gemv(tw, tl, 64, 128, ta[i], 1.0, out=ta[i + 1][:, :64])
        tsweep()
        fn = capture(tsweep)
        fn()
        floor["dependent_smallest_gemv_launch_us"] = round(timed(torch, fn, reps * 4) / 64 * 1e6, 3)
        tsteps = [rcp.GemvStep(tw, tl, 64, 128, ta[i], ta[i + 1][0, :64]) for i in range(16)]
        tws = rcp.gemv_sequence_workspace(tsteps)

        def ssweep():
            for _ in range(4):
                rcp.quant_w2a4_gemv_sequence(tsteps, tws)
        ssweep()
        fn = capture(ssweep)
        fn()
        t_seq = timed(torch, fn, reps * 4) / 4
        floor["sequence_of_16_smallest_gemvs_us_per_entry"] = round(t_seq / 16 * 1e6, 3)
        floor["sequence_error_word"] = int(tws[0].item())

    # The four GEMVs of a layer as a real chain (o reads q, gate|up reads o's output, down reads the rotated gate half
    # of gate|up's output; every layer starts from the same synthetic input): launched one by one (5 launches per
    # layer) and as one rcp_quant_w2a4_gemv_sequence launch per layer (and per 4 layers).  Same bits either way.
    persistent = None
    if not args.step_only:
        co = [torch.zeros((1, N), dtype=torch.float16, device=dev) for (_, N, _, _) in launches]

        def chain_launches():
            for l in range(L):
                w = layers[l]
                rcp.quant_w2a4_gemv(w[0][0], w[0][1], 3 * HIDDEN, HIDDEN, xs[0], 1.0, out=co[0])
                rcp.quant_w2a4_gemv(w[1][0], w[1][1], HIDDEN, HIDDEN, co[0][0, :HIDDEN], 1.0, out=co[1])
                rcp.quant_w2a4_gemv(w[2][0], w[2][1], 2 * INTER, HIDDEN, co[1], 1.0, out=co[2])
                rcp.rotate_act(co[2][:, :INTER], rot_down, y_out=ybuf)
                rcp.quant_w2a4_gemv(w[3][0], w[3][1], HIDDEN, INTER, ybuf, 1.0, out=co[3])

        def chain_steps(l):
            w = layers[l]
            return [rcp.GemvStep(w[0][0], w[0][1], 3 * HIDDEN, HIDDEN, xs[0], co[0]),
                    rcp.GemvStep(w[1][0], w[1][1], HIDDEN, HIDDEN, co[0][0, :HIDDEN], co[1]),
                    rcp.GemvStep(w[2][0], w[2][1], 2 * INTER, HIDDEN, co[1], co[2]),
                    rcp.GemvStep(w[3][0], w[3][1], HIDDEN, INTER, co[2][0, :INTER], co[3], rot=rot_down)]
        per_layer = [chain_steps(l) for l in range(L)]
        per_four = [sum(per_layer[l:l + 4], []) for l in range(0, L - L % 4, 4)]
        wsq = rcp.gemv_sequence_workspace(per_four[0] if per_four else per_layer[0])

        def chain_sequence():
            for st in per_layer:
                rcp.quant_w2a4_gemv_sequence(st, wsq)

        def chain_sequence4():
            for st in per_four:
                rcp.quant_w2a4_gemv_sequence(st, wsq)
        chain_launches()
        fn = capture(chain_launches)
        fn()
        t_l = timed(torch, fn, max(3, args.steps // 2)) / L
        ref_out = co[3].clone()
        chain_sequence()
        fn = capture(chain_sequence)
        fn()
        t_s = timed(torch, fn, max(3, args.steps // 2)) / L
        same = bool(torch.equal(ref_out, co[3]))
        layer_bytes = sum(gemv_bytes(N, K) for (_, N, K, _) in launches)
        persistent = {"chained_launches_us_per_layer": round(t_l * 1e6, 2), "chained_launches_GBps": round(layer_bytes / t_l / 1e9, 1),
                      "sequence_us_per_layer": round(t_s * 1e6, 2), "sequence_GBps": round(layer_bytes / t_s / 1e9, 1),
                      "sequence_pct_of_hbm_peak": round(100.0 * layer_bytes / t_s / 1e9 / HBM_PEAK_GBPS, 2),
                      "same_bits_as_launches": same}
        if per_four:
            fn = capture(chain_sequence4)
            fn()
            t4 = timed(torch, fn, max(3, args.steps // 2)) / (4 * len(per_four))
            persistent["sequence_4_layers_per_launch_us_per_layer"] = round(t4 * 1e6, 2)
        persistent["error_word"] = int(wsq[0].item())

    # The down projection's prologue: the fused call quantises the 11008 rotated binary32 values in every workgroup;
    # the same GEMV on activations quantised beforehand shows what that costs (cold, same 32 weight buffers).
    down_split = None
    if not args.step_only:
        rcp.rotate_quant_act(xs[3], rot_down, 1.0, xq_out=xqs[3], scale_out=scs[3], workspace=ws)

        def dsweep():
            for l in range(L):
                packed, cb = layers[l][3]
                rcp.w2a4_gemv(packed, cb, HIDDEN, INTER, xqs[3], scs[3], 1, out=outs[3])
        fn = capture(dsweep)
        fn()
        down_split = {"prequantised_gemv_us": round(timed(torch, fn, reps) / L * 1e6, 3)}
        if "4096x11008" in per_shape:
            down_split["fused_quantise_gemv_us"] = per_shape["4096x11008"]["us"]

    # Stored profiler figures (profiles/gemv_traffic.json, written from rocprofv3 runs of this file; its "commit" field
    # names the build they were taken on): HBM bytes per GEMV launch from the FETCH_SIZE / WRITE_SIZE counters, and the
    # kernel-trace durations, whose clock differs from the events used here (see "clocks").
    traffic = None
    stored = {}
    tpath = os.path.join(ROOT, "profiles", "gemv_traffic.json")
    if os.path.exists(tpath):
        try:
            stored = json.load(open(tpath))
            traffic = stored.get("hbm_bytes_per_launch")
        except Exception:
            stored, traffic = {}, None
    roofline = {"bound": "hbm", "kernel": "gemv_kernel / gemv_oneshot_kernel (the four GEMV launches of a layer)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "frac_events": round(achieved / HBM_PEAK_GBPS, 4),
                "clocks": "achieved / frac / frac_events: algorithmic bytes per GEMV launch over the mean launch-to-launch time of "
                          "a GEMV-only graph replay, HIP events on the launch stream (dispatch gaps included); frac_rocprof: the "
                          "same bytes over the stored rocprofv3 kernel-trace mean duration",
                "traffic_source": "stored: profiles/gemv_traffic.json" + (" @ " + str(stored.get("commit")) if stored.get("commit") else "")}
    kt = stored.get("gemv_kernel_trace") or {}
    if kt.get("call_weighted_mean_ns"):
        roofline["frac_rocprof"] = round((step_bytes / n_gemv) / (kt["call_weighted_mean_ns"] * 1e-9) / 1e9 / HBM_PEAK_GBPS, 4)
        per_kernel = {}
        byname = {"qkv 12288x4096": (3 * HIDDEN, HIDDEN), "o 4096x4096": (HIDDEN, HIDDEN),
                  "gate_up 22016x4096": (2 * INTER, HIDDEN), "down 4096x11008": (HIDDEN, INTER)}
        for name, ns in (kt.get("avg_ns") or {}).items():
            if name in byname:
                b = gemv_bytes(*byname[name])
                per_kernel[name] = {"rocprof_avg_us": round(ns * 1e-3, 3), "frac_rocprof": round(b / (ns * 1e-9) / 1e9 / HBM_PEAK_GBPS, 4)}
        for name, label in (("qkv 12288x4096", "12288x4096_qkv"), ("o 4096x4096", "4096x4096"),
                            ("gate_up 22016x4096", "22016x4096_gate_up"), ("down 4096x11008", "4096x11008")):
            if name in per_kernel and label in per_shape:
                per_kernel[name]["events_us"] = per_shape[label]["us"]
                per_kernel[name]["frac_events"] = round(per_shape[label]["pct_hbm_peak"] / 100.0, 4)
        roofline["per_kernel"] = per_kernel

    line = {
        "metric": "w2a4_gemv_effective_hbm_bandwidth_llama2_7b_bs1",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int4 x 2-bit LUT index, int32 accumulate, fp32 epilogue",
        "data": "synthetic",
        "config": {"workload": "llama2_7b_decode_bs1", "layers": L, "linears_per_layer": 7,
                   "gemv_launches_per_layer": 4, "batch": 1, "graph": not args.no_graph,
                   "activation_quantiser": "fused into the GEMV prologue" if fused else "separate launch",
                   "down_rotation": "H_64 (x) Q_172"},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "us_per_gemv_launch": round(gemv_avg_s * 1e6, 3),
        "us_per_linear": round(sec_gemv_sweep / (7 * L) * 1e6, 3),
        "us_act_prep_per_layer": round(sec_act_sweep / L * 1e6, 3),
        "gemv_only_GBps": round(step_bytes / sec_gemv_sweep / 1e9, 1),
        "per_shape": per_shape,
        "small_batch": small_batch,
        "act_prep_us": act_us,
        "grouped_128": grouped,
        "grouped_128_step": grouped_step,
        "weight_only_fp16": weight_only,
        "weight_only_step": weight_only_step,
        "w3a4": w3,
        "w3a4_step": w3_step,
        "kv4_attention_32_heads": kv4,
        "kv4_attention_batched": kv4_batched,
        "kv4_layer_launches": kv_layer,
        "per_shape_other": other,
        "large_matrix": large,
        "launch_floor": floor,
        "persistent_layer": persistent,
        "down_projection_prologue": down_split,
        "roofline": roofline,
        "setup_s": round(t_setup, 1),
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
