#!/usr/bin/env python3
"""Benchmark of the hybrid dense / 2:4 tile linear layer on one MI355X.

Headline workload (the line's `value`): the LLaMA-2-7B MLP prefill set -- gate and up projections
11008 x 4096 and the down projection 4096 x 11008, bf16, 128 x 128 tiles, 60 % of the tiles 2:4, M = 4096
rows of X.  One step = one pass of patch_gemm over the three projections (inputs resident in HBM).
`value` = dense-equivalent TFLOP/s = 3 * 2 M N K / step time.

Also reported on the same JSON line:
  roofline      dominant (prefill) kernel: issued matrix-instruction flops M N K (2 - f) per launch over
                its average launch duration, against the published dense bf16 MFMA peak (2.5 PFLOP/s)
  decode        7B attention projection 4096 x 4096, M in {1, 4, 16}, five 2:4 fractions: GB/s on the
                compressed weight bytes against the HBM peak, rotating over enough distinct packed copies
                to defeat the 256 MB last-level cache
  speedup_vs_all_dense   same shapes with an all-dense tile map through the same library
  pack          compression throughput (one-off conversion; not part of a step)
  cpu_baseline  the CPU oracle timed on a bounded sample of the headline workload
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

import numpy as np

PEAK_HBM_GBS = 8000.0       # MI355X published HBM3E bandwidth
PEAK_MFMA_BF16_TF = 2500.0  # MI355X published dense bf16 matrix peak
PAPER_CONTEXT = "paper: 1.18x-1.38x end-to-end LLaMA-2 7B speedup on an A6000 at 25-45% sparsity (context, not a target)"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--m", type=int, default=4096, help="rows of X for the headline prefill workload")
    ap.add_argument("--f", type=float, default=0.6, help="fraction of 2:4 tiles of the headline workload")
    ap.add_argument("--skip", default="", help="comma list of sections to skip: decode,dense,cpu,pack,mid,sweep,layer")
    ap.add_argument("--variant", type=int, default=0)
    ap.add_argument("--decode-launches", type=int, default=200)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (known traffic, for scaling profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU by design (one MI355X); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    skip = set(s for s in args.skip.split(",") if s)

    import torch
    from paper_2509_23410_amd import binding as B, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.lib()  # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream

    def dev_bf16(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)

    def masked_packed(c, tile_map=None):
        tm = c.tile_map if tile_map is None else tile_map
        W = dev_bf16(c.W)
        m24 = torch.from_numpy(c.mask24).to(dev)
        W_hat = torch.empty_like(W)
        B.patch_apply_mask(W, m24, tm, c.N, c.K, c.tile, W_hat, stream)
        return W_hat, B.patch_pack(W_hat, c.N, c.K, tm, c.tile, stream)

    def timed(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(n):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3  # seconds

    out = {}
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    # ------------------------------------------------------------------ headline: 7B MLP prefill
    M, f, t = args.m, args.f, 128
    shapes = [("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
    t0 = time.time()
    layers = []
    for name, N, K in shapes:
        c = synth.make_case("llama7b_mlp_" + name, N, K, M, t, f, seed=0)
        W_hat, P = masked_packed(c)
        X = dev_bf16(c.X)
        Y = torch.empty((M, N), device=dev, dtype=torch.float32)
        layers.append(dict(name=name, c=c, P=P, X=X, Y=Y, W_hat=W_hat))
    prep_s = time.time() - t0
    opts = dict(variant=args.variant)

    def step(_i):
        for L in layers:
            B.patch_gemm(L["X"], M, L["P"], L["Y"], stream, **opts)

    timed(step, args.warmup)
    secs = timed(step, args.steps)
    Y_sample = {L["name"]: L["Y"].cpu().numpy() for L in layers[:1]} if "cpu" not in skip else {}
    ms_per_step = secs / args.steps * 1e3
    dense_flop = sum(2.0 * M * L["c"].N * L["c"].K for L in layers)
    issued_flop = 0.0
    for L in layers:
        N_, K_, _t, ns = L["P"].dims()
        fa = ns / (N_ // t * (K_ // t))
        issued_flop += M * N_ * K_ * (2.0 - fa)
    value = dense_flop / (ms_per_step * 1e-3) / 1e12
    n_launch = len(layers)
    avg_launch_s = ms_per_step * 1e-3 / n_launch
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "prefill_traffic.json")
    if os.path.exists(tpath) and M == 4096 and f == 0.6:
        with open(tpath) as fh:
            traffic = json.load(fh).get("hbm_bytes_per_launch")   # from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
    roof = dict(bound="mfma", achieved=issued_flop / n_launch / avg_launch_s / 1e12, peak=PEAK_MFMA_BF16_TF, unit="TFLOP/s",
                traffic=traffic, kernel="prefill_kernel_wreg" if args.variant in (0, 3) else "variant %d" % args.variant, avg_launch_us=avg_launch_s * 1e6,
                algorithmic_flop_per_launch=issued_flop / n_launch,
                note="achieved = issued matrix flops M N K (2 - f) per launch / average launch duration (HIP events); "
                     "traffic = measured HBM bytes per launch (profiles/)")
    roof["frac"] = roof["achieved"] / roof["peak"]

    # ------------------------------------------------------------------ same shapes, all-dense tile map
    speedup = None
    if "dense" not in skip:
        dl = []
        for L in layers:
            c = L["c"]
            P0 = B.patch_pack(L["W_hat"], c.N, c.K, np.ones_like(c.tile_map), t, stream)
            dl.append((L["X"], P0, L["Y"]))

        def dstep(_i):
            for X, P0, Y in dl:
                B.patch_gemm(X, M, P0, Y, stream, **opts)

        timed(dstep, args.warmup)
        dsecs = timed(dstep, args.steps)
        speedup = dsecs / secs
        out["all_dense_ms_per_step"] = dsecs / args.steps * 1e3
        for _, P0, _ in dl:
            P0.close()

    # ------------------------------------------------------------------ pack throughput (one-off conversion)
    if "pack" not in skip:
        L = layers[0]
        c = L["c"]
        tp = time.time()
        for _ in range(3):
            B.patch_pack(L["W_hat"], c.N, c.K, c.tile_map, t, stream).close()
        torch.cuda.synchronize()
        out["pack"] = dict(shape=[c.N, c.K], ms=(time.time() - tp) / 3 * 1e3,
                           note="patch_pack wall time incl. allocation and the status read-back")

    # ------------------------------------------------------------------ prefill time against the 2:4 tile fraction (gate projection)
    if "sweep" not in skip:
        c0 = layers[0]["c"]
        fr = (0.0, 0.25, 0.5, 0.75, 1.0)
        Pf = []
        for ff in fr:
            cf = synth.make_case("llama7b_mlp_gate", c0.N, c0.K, M, t, ff, seed=0)
            W_hat_f, P_f = masked_packed(cf)
            Pf.append(P_f)
            del W_hat_f
        Xf, Yf = layers[0]["X"], layers[0]["Y"]
        us = [[] for _ in fr]
        for _r in range(3):   # the fractions in turn, three rounds: the clock drifts by a few per cent over a run
            for i, P_f in enumerate(Pf):
                fn = lambda _i, P_f=P_f: B.patch_gemm(Xf, M, P_f, Yf, stream, **opts)
                timed(fn, 3)
                us[i].append(timed(fn, 10) / 10 * 1e6)
        med = [sorted(u)[1] for u in us]
        out["prefill_f_sweep"] = dict(shape=[c0.N, c0.K], M=M, f=list(fr), us=[round(u, 1) for u in med],
                                      speedup_over_all_dense=[round(med[0] / u, 3) for u in med],
                                      note="median of three interleaved rounds of 10 launches each")
        for P_f in Pf:
            P_f.close()

    # ------------------------------------------------------------------ mid M: 13B layer shapes at M = 512, 7B MLP at M = 2048
    if "mid" not in skip:
        rows = []
        for name, N_, K_, Mm in (("13b_attn", 5120, 5120, 512), ("13b_gate", 13824, 5120, 512), ("13b_down", 5120, 13824, 512),
                                 ("7b_gate", 11008, 4096, 2048), ("7b_attn", 4096, 4096, 32), ("7b_attn", 4096, 4096, 64), ("7b_attn", 4096, 4096, 256),
                                 ("13b_gate", 13824, 5120, 32), ("13b_gate", 13824, 5120, 64), ("13b_down", 5120, 13824, 64)):
            cm = synth.make_case("mid_" + name, N_, K_, Mm, t, 0.5, seed=0)
            W_hat, Pm = masked_packed(cm)
            Xm = dev_bf16(cm.X)
            Ym = torch.empty((Mm, N_), device=dev, dtype=torch.float32)
            need = B.patch_gemm_workspace_bytes(Mm, Pm)
            ws = torch.empty(max(need, 16) // 4, device=dev, dtype=torch.float32)
            res = {}
            for label, kw in (("unsplit", dict()), ("with_workspace", dict(workspace=ws))):
                fn = lambda i, kw=kw: B.patch_gemm(Xm, Mm, Pm, Ym, stream, **kw)
                timed(fn, 10)
                res[label] = sorted(timed(fn, 50) / 50 for _ in range(3))[1] * 1e6
            rows.append(dict(shape=[N_, K_], M=Mm, f=0.5, us_without_workspace=round(res["unsplit"], 2),
                             us=round(res["with_workspace"], 2), workspace_MB=round(need / 1e6, 1),
                             dense_equiv_TFLOPs=round(2.0 * Mm * N_ * K_ / res["with_workspace"] / 1e6, 1)))
            Pm.close()
            del W_hat, Xm, Ym, ws
        out["mid_m"] = dict(rows=rows, note="patch_gemm, automatic path; with a workspace the launch splits K over otherwise idle "
                                            "compute units (partials summed in slice order): M <= 64 one decode-path pass with 64 "
                                            "features per wavefront, beyond that the prefill kernel")

    # ------------------------------------------------------------------ decode: 7B attention projection
    if "decode" not in skip:
        dec = []
        N = K = 4096
        cd = synth.make_case("llama7b_attn", N, K, 16, t, 0.0, seed=0)
        Xd = dev_bf16(cd.X)
        Yd = torch.empty((16, N), device=dev, dtype=torch.float32)
        base_us = {}
        fused = []
        for fd in (0.0, 0.25, 0.5, 0.75, 1.0):
            tm = synth.tile_map(0, N // t, K // t, fd, "llama7b_attn", N, K, t, fd)
            W_hat, P0 = masked_packed(cd, tm)
            R = max(2, int(np.ceil(1.1e9 / P0.nbytes)))
            Ps = [P0] + [B.patch_pack(W_hat, N, K, tm, t, stream) for _ in range(R - 1)]
            for Md in (1, 4, 16):
                def launch(i, Md=Md):
                    B.patch_gemm(Xd, Md, Ps[i % R], Yd, stream)
                timed(launch, 20)
                reps = sorted(timed(launch, args.decode_launches) / args.decode_launches for _ in range(5))
                us = reps[2] * 1e6
                timed(lambda i: B.patch_gemm(Xd, Md, Ps[0], Yd, stream), 20)
                us_res = sorted(timed(lambda i: B.patch_gemm(Xd, Md, Ps[0], Yd, stream), args.decode_launches)
                                / args.decode_launches for _ in range(3))[1] * 1e6
                if fd == 0.0:
                    base_us[Md] = us
                gbs = P0.nbytes / (us * 1e-6) / 1e9
                dec.append(dict(f=fd, M=Md, us=round(us, 3), GBps=round(gbs, 1), frac_hbm=round(gbs / PEAK_HBM_GBS, 4),
                                speedup_vs_all_dense=round(base_us[Md] / us, 4), us_cache_resident=round(us_res, 3),
                                packed_MB=round(P0.nbytes / 1e6, 3), copies=R,
                                dense_equiv_TFLOPs=round(2.0 * Md * N * K / (us * 1e-6) / 1e12, 3)))
            if fd in (0.0, 0.5):
                # q / k / v: three projections sharing X in one launch (patch_gemm_many)
                nq = 3
                Rq = max(2, R // nq)
                sets = [Ps[i * nq:(i + 1) * nq] for i in range(Rq)]
                Yq = [torch.empty((16, N), device=dev, dtype=torch.float32) for _ in range(nq)]
                def launch_q(i):
                    B.patch_gemm_many(Xd, 1, sets[i % Rq], Yq, stream)
                timed(launch_q, 20)
                nl = max(1, args.decode_launches // nq)
                us = sorted(timed(launch_q, nl) / nl for _ in range(5))[2] * 1e6
                gbs = nq * P0.nbytes / (us * 1e-6) / 1e9
                fused.append(dict(f=fd, M=1, weights=nq, us=round(us, 3), GBps=round(gbs, 1), frac_hbm=round(gbs / PEAK_HBM_GBS, 4),
                                  speedup_vs_single_launches=round(nq * [r_ for r_ in dec if r_["M"] == 1 and r_["f"] == fd][0]["us"] / us, 4)))
            for P_ in Ps:
                P_.close()
            del W_hat
        # the MLP projections of the same model at M = 1 (two thirds of a decoder layer's weight bytes)
        mlp = []
        for name, N_, K_ in (("gate", 11008, 4096), ("down", 4096, 11008)):
            for fd in (0.0, 0.5):
                cm = synth.make_case("llama7b_mlp_dec_" + name, N_, K_, 1, t, fd, seed=0)
                W_hat, P0 = masked_packed(cm)
                Rm = max(2, int(np.ceil(1.1e9 / P0.nbytes)))
                Pm = [P0] + [B.patch_pack(W_hat, N_, K_, cm.tile_map, t, stream) for _ in range(Rm - 1)]
                Xm = dev_bf16(cm.X)
                Ym = torch.empty((1, N_), device=dev, dtype=torch.float32)
                fn = lambda i: B.patch_gemm(Xm, 1, Pm[i % Rm], Ym, stream)
                timed(fn, 20)
                nl = max(1, args.decode_launches // 2)
                us = sorted(timed(fn, nl) / nl for _ in range(5))[2] * 1e6
                gbs = P0.nbytes / (us * 1e-6) / 1e9
                mlp.append(dict(shape=[N_, K_], f=fd, M=1, us=round(us, 3), GBps=round(gbs, 1), frac_hbm=round(gbs / PEAK_HBM_GBS, 4),
                                packed_MB=round(P0.nbytes / 1e6, 3), copies=Rm))
                for P_ in Pm:
                    P_.close()
                del W_hat
        out["decode_mlp"] = dict(rows=mlp, note="7B MLP projections, M = 1, rotating packed copies")
        # one 7B decoder layer's seven projections at M = 1 (q/k/v in one launch, o, gate/up in one launch, down),
        # eager and as a captured HIP graph, rotating over copies of the layer so that no cache holds the weights
        if "layer" not in skip:
            lrows = []
            for fd in (0.0, 0.5):
                shapes7 = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
                           ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
                copies, nbytes = 3, 0
                layer = [dict() for _ in range(copies)]
                for name, N_, K_ in shapes7:
                    cl = synth.make_case("llama7b_layer_" + name, N_, K_, 1, t, fd, seed=0)
                    W_hat, P0 = masked_packed(cl)
                    nbytes += P0.nbytes
                    for ci in range(copies):
                        layer[ci][name] = P0 if ci == 0 else B.patch_pack(W_hat, N_, K_, cl.tile_map, t, stream)
                    del W_hat
                x4, x11 = dev_bf16(synth.make_case("llama7b_layer_x", 128, 4096, 1, t, 0.0, seed=1).X), None
                x11 = dev_bf16(synth.make_case("llama7b_layer_x2", 128, 11008, 1, t, 0.0, seed=2).X)
                y = {n: torch.empty((1, N_), device=dev, dtype=torch.float32) for n, N_, _ in shapes7}

                def layer_pass(L, st):
                    B.patch_gemm_many(x4, 1, [L["q"], L["k"], L["v"]], [y["q"], y["k"], y["v"]], st)
                    B.patch_gemm(x4, 1, L["o"], y["o"], st)
                    B.patch_gemm_many(x4, 1, [L["gate"], L["up"]], [y["gate"], y["up"]], st)
                    B.patch_gemm(x11, 1, L["down"], y["down"], st)

                fn = lambda i: layer_pass(layer[i % copies], stream)
                timed(fn, 12)
                eager_us = sorted(timed(fn, 60) / 60 for _ in range(3))[1] * 1e6
                side = torch.cuda.Stream()
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.stream(side):
                    with torch.cuda.graph(graph, stream=side):
                        for ci in range(copies):
                            layer_pass(layer[ci], side.cuda_stream)
                timed(lambda i: graph.replay(), 4)
                graph_us = sorted(timed(lambda i: graph.replay(), 20) / (20 * copies) for _ in range(3))[1] * 1e6
                lrows.append(dict(f=fd, M=1, packed_MB=round(nbytes / 1e6, 1), launches=4, us_eager=round(eager_us, 2),
                                  us_graph=round(graph_us, 2), GBps_graph=round(nbytes / (graph_us * 1e-6) / 1e9, 1),
                                  frac_hbm_graph=round(nbytes / (graph_us * 1e-6) / 1e9 / PEAK_HBM_GBS, 4)))
                del graph
                for L in layer:
                    for P_ in L.values():
                        P_.close()
            out["decode_layer_7b"] = dict(rows=lrows, note="the seven projections of one 7B decoder layer at M = 1 in four launches "
                                          "(q/k/v fused, o, gate/up fused, down), per layer; graph = one captured HIP graph of three "
                                          "layer copies replayed")
        m1 = [r_ for r_ in dec if r_["M"] == 1 and r_["f"] == 0.0][0]
        dtraffic = None
        dpath = os.path.join(ROOT, "profiles", "decode_traffic.json")
        if os.path.exists(dpath):
            with open(dpath) as fh:
                dtraffic = json.load(fh).get("hbm_bytes_per_launch")   # from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
        out["decode_roofline"] = dict(bound="hbm", achieved=m1["GBps"], peak=PEAK_HBM_GBS, unit="GB/s", frac=m1["frac_hbm"],
                                      traffic=dtraffic, kernel="decode_kernel", workload="4096x4096 f=0 M=1",
                                      algorithmic_bytes_per_launch=m1["packed_MB"] * 1e6,
                                      note="achieved = compressed weight bytes per launch / average launch duration; "
                                           "traffic = measured HBM bytes per launch (profiles/)")
        out["decode_fused_qkv"] = dict(rows=fused, note="three 4096x4096 projections sharing X in one patch_gemm_many launch, rotating packed copies")
        out["decode"] = dict(workload="llama7b_attn_decode 4096x4096 tile128", peak_GBps=PEAK_HBM_GBS, rows=dec,
                             note="us = median of 5 batches of back-to-back launches over rotating packed copies (HBM-resident)")

    # ------------------------------------------------------------------ CPU oracle on a bounded sample
    cpu = None
    if "cpu" not in skip:
        from oracle import oracle
        L = layers[0]
        c = L["c"]
        Ms = M
        W_hat_o = oracle.apply_mask(c.W, c.tile_map, c.mask24, t)
        vals, meta = oracle.pack(W_hat_o, c.tile_map, t)
        tc = time.time()
        Yo = oracle.gemm(c.X[:Ms], vals, meta, c.N, c.K, c.tile_map, t)
        cs = time.time() - tc
        cpu = dict(value=2.0 * Ms * c.N * c.K / cs / 1e12, unit="TFLOP/s (dense-equivalent)", cores=oracle.num_threads(),
                   kind="oracle", seconds=round(cs, 2),
                   sample=f"gate projection 11008x4096, first {Ms} of {M} rows of X, fp64, decompress + one dot product per output")
        Yg = Y_sample[L["name"]][:Ms].astype(np.float64)
        out["relF_vs_oracle_on_sample"] = float(np.linalg.norm(Yg - Yo) / np.linalg.norm(Yo))

    line = {
        "metric": "hybrid GEMM dense-equiv TFLOP/s + GB/s vs roofline; speedup over all-dense",
        "value": value, "unit": "TFLOP/s (dense-equivalent)", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "llama7b_mlp_prefill", "shapes": [[n, k] for _, n, k in shapes], "M": M, "tile": t,
                   "f_2to4_tiles": f, "launches_per_step": n_launch, "variant": args.variant},
        "roofline": roof, "cpu_baseline": cpu, "speedup_vs_all_dense": speedup, "context": PAPER_CONTEXT,
        "input_prep_s": round(prep_s, 1),
    }
    line.update(out)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
