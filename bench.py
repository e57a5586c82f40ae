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
  prefill_m2048 the headline step on 2048 rows (the configuration's other row count), with its all-dense counterpart
  prefill_bf16_out  the headline step with bf16 output (half the bytes stored; beside the headline, not instead of it)
  pack          compression throughput (one-off conversion; not part of a step)
  ceilings      measured ceilings from kernels of this library (register-resident loops of the two matrix
                instructions, streaming reads) and the vendor dense GEMM on the same shapes (context)
  stack_13b     the 13B decoder stack: 40 layers x 7 matrices, one 2:4 fraction per layer drawn U[0,1),
                M in {1, 512, 4096}, time = sum over the layers; stack_13b_per_matrix: the same with a fraction
                per (layer, matrix) that follows the allocation the paper reports (key / value dense, MLP heavy)
  decode_q4     decode from the 4-bit weight-only storage (7B shapes, M = 1 and 16) beside the bf16 storage;
                decode_q4_layer_7b: one 7B decoder layer from it in four launches
  prefill_tile64  the two MLP projections with mask tile 64 (the paper's other tile size)
  qwen_0p5b     the 0.5B-scale layer set (launch-latency-bound)
  cpu_baseline  the CPU oracle timed on a bounded sample of the headline workload

Before every timed region the workload runs until two consecutive batches agree within 1 % (the clock of
the part needs some tens of launches after idle to settle); `settle_steps` says how many steps that took.
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


def _keep_top2(torch, W):
    """(N K / 4, 4) uint8 keep-mask of the two largest |w| of every four consecutive elements (lower index on ties), on
    the device: an element is kept when fewer than two others beat it."""
    mag = W.abs().float().view(-1, 4)
    keep = torch.empty_like(mag, dtype=torch.uint8)
    for p_ in range(4):
        beaten = torch.zeros(mag.shape[0], device=W.device, dtype=torch.int32)
        for o in range(4):
            if o != p_:
                beaten += (mag[:, o] >= mag[:, p_]) if o < p_ else (mag[:, o] > mag[:, p_])
        keep[:, p_] = beaten < 2
    return keep


def stack_13b(torch, B, synth, dev, stream, timed, t, per_matrix=False, Ms=(1, 512, 4096), q4=False):
    """The 13B decoder stack: 40 layers x {q, k, v, o 5120 x 5120; gate, up 13824 x 5120; down 5120 x 13824}, one 2:4
    tile fraction per layer drawn U[0, 1) - or, with per_matrix, the fractions of synth.matrix_fractions (key / value
    dense, MLP heavy, middle blocks heavy; global target 0.5) - every GEMM with its own X; time = sum over the layers.
    A layer runs as four launches (q / k / v share X, gate / up share X).  Weights are packed layer by layer and freed;
    they are drawn on the device (N(0, 0.02^2), magnitude 2:4 mask) - the parity tests cover these shapes with the
    host-drawn inputs.  Every layer is also run with an all-dense map of the same weights.  With q4 the same pruned
    weights are also stored in 4 bits (patch_pack4) and run at M = 1 (four launches: patch_gemm4_many / patch_gemm4) and
    M = 512 (seven patch_gemm4_ex launches); a layer's 4-bit weights (about 150 MB) would stay in the last-level cache
    between repetitions, so two consecutive layers are timed alternately (300 MB) and half of the pair's time counts."""
    H, F = 5120, 13824
    shapes = [("q", H, H), ("k", H, H), ("v", H, H), ("o", H, H), ("gate", F, H), ("up", F, H), ("down", H, F)]
    if per_matrix:
        fr = synth.matrix_fractions(40, [N_ * K_ for _, N_, K_ in shapes], 0.5)
    else:
        fr = np.repeat(synth.layer_fractions(0, 40)[:, None], len(shapes), axis=1)
    gen = torch.Generator(device=dev)
    gen.manual_seed(13)
    xH = torch.randn(4096, H, device=dev, generator=gen).to(torch.bfloat16)
    xF = torch.randn(4096, F, device=dev, generator=gen).to(torch.bfloat16)
    y = {n: torch.empty((4096, N_), device=dev, dtype=torch.float32) for n, N_, _ in shapes}
    ws = torch.empty(96 << 20, device=dev, dtype=torch.float32)     # 384 MB: room for every split the launcher picks
    tot = {M_: dict(mix=0.0, dense=0.0) for M_ in Ms}
    tot4, bytes4, prev4 = {1: 0.0, 512: 0.0}, 0, None
    packed_bytes, dense_bytes, flop_w, ideal_s = 0, 0, 0.0, {M_: 0.0 for M_ in Ms}
    per_layer = []

    def layer_pass(L, M_):
        B.patch_gemm_many(xH, M_, [L["q"], L["k"], L["v"]], [y["q"], y["k"], y["v"]], stream, workspace=ws)
        B.patch_gemm(xH, M_, L["o"], y["o"], stream, workspace=ws)
        B.patch_gemm_many(xH, M_, [L["gate"], L["up"]], [y["gate"], y["up"]], stream, workspace=ws)
        B.patch_gemm(xF, M_, L["down"], y["down"], stream, workspace=ws)

    def layer_pass4(L4, M_):
        if M_ == 1:
            B.patch_gemm4_many(xH, 1, [L4["q"], L4["k"], L4["v"]], [y["q"], y["k"], y["v"]], stream)
            B.patch_gemm4(xH, 1, L4["o"], y["o"], stream)
            B.patch_gemm4_many(xH, 1, [L4["gate"], L4["up"]], [y["gate"], y["up"]], stream)
            B.patch_gemm4(xF, 1, L4["down"], y["down"], stream)
        else:
            for name, _, K_ in shapes:
                B.patch_gemm4(xH if K_ == H else xF, M_, L4[name], y[name], stream, workspace=ws)

    for li in range(40):
        layer, dense, layer4 = {}, {}, {}
        for mi, (name, N_, K_) in enumerate(shapes):
            f = float(fr[li, mi])
            W = (torch.randn(N_, K_, device=dev, generator=gen) * 0.02).to(torch.bfloat16)
            keep = _keep_top2(torch, W)
            tm = synth.tile_map(li, N_ // t, K_ // t, f, "stack13b", name)
            W_hat = torch.empty_like(W)
            B.patch_apply_mask(W, keep.view(N_, K_), tm, N_, K_, t, W_hat, stream)
            layer[name] = B.patch_pack(W_hat, N_, K_, tm, t, stream)
            dense[name] = B.patch_pack(W_hat, N_, K_, np.ones_like(tm), t, stream)
            if q4:
                layer4[name] = B.patch_pack4(W_hat, N_, K_, tm, t, stream)
                bytes4 += layer4[name].nbytes
            packed_bytes += layer[name].nbytes
            dense_bytes += dense[name].nbytes
            del W, keep, W_hat
        row = dict(layer=li, f=[round(float(v), 3) for v in fr[li]] if per_matrix else round(float(fr[li, 0]), 3))
        for M_ in Ms:
            reps = 10 if M_ == 1 else 4 if M_ == 512 else 2
            for key, L in (("mix", layer), ("dense", dense)):
                timed(lambda _i: layer_pass(L, M_), 2)
                s_ = min(timed(lambda _i: layer_pass(L, M_), reps) / reps for _ in range(2))
                tot[M_][key] += s_
                row[f"us_M{M_}" + ("" if key == "mix" else "_all_dense")] = round(s_ * 1e6, 1)
        if q4 and prev4 is not None:
            for M_ in (1, 512):
                reps = 10 if M_ == 1 else 4
                pair = lambda _i: (layer_pass4(prev4, M_), layer_pass4(layer4, M_))
                timed(pair, 2)
                s_ = min(timed(pair, reps) / reps for _ in range(2)) / 2.0
                tot4[M_] += s_ * 40.0 / 39.0          # 39 pairs stand for 40 layers
                row[f"us_M{M_}_q4_mean_with_previous_layer"] = round(s_ * 1e6, 1)
        per_layer.append(row)
        for L in (layer, dense) + ((prev4,) if prev4 is not None else ()):
            for P_ in L.values():
                P_.close()
        prev4 = layer4 if q4 else None
    layer_flop = sum(2.0 * N_ * K_ for _, N_, K_ in shapes)            # per row of X
    mat_flop = np.array([2.0 * N_ * K_ for _, N_, K_ in shapes])
    f_mean = float((fr * mat_flop[None, :]).sum() / (mat_flop.sum() * 40))   # parameter-weighted
    rows = []
    for M_ in Ms:
        secs = tot[M_]["mix"]
        issued = float((mat_flop[None, :] * M_ * (2.0 - fr) / 2.0).sum())
        r_ = dict(M=M_, ms_total=round(secs * 1e3, 3), ms_total_all_dense=round(tot[M_]["dense"] * 1e3, 3),
                  speedup_vs_all_dense=round(tot[M_]["dense"] / secs, 4),
                  dense_equiv_TFLOPs=round(40 * layer_flop * M_ / secs / 1e12, 1),
                  issued_TFLOPs=round(issued / secs / 1e12, 1), frac_mfma_peak=round(issued / secs / 1e12 / PEAK_MFMA_BF16_TF, 4),
                  GBps_compressed=round(packed_bytes / secs / 1e9, 1), frac_hbm_peak=round(packed_bytes / secs / 1e9 / PEAK_HBM_GBS, 4))
        rows.append(r_)
    extra = {}
    if prev4 is not None:
        for P_ in prev4.values():
            P_.close()
    if q4:
        extra["q4"] = dict(packed_GB=round(bytes4 / 1e9, 3), bytes_vs_bf16_storage=round(bytes4 / packed_bytes, 4),
                           ms_total_M1=round(tot4[1] * 1e3, 3), GBps_M1=round(bytes4 / tot4[1] / 1e9, 1),
                           frac_hbm_peak_M1=round(bytes4 / tot4[1] / 1e9 / PEAK_HBM_GBS, 4),
                           ms_total_M512=round(tot4[512] * 1e3, 3),
                           dense_equiv_TFLOPs_M512=round(40 * layer_flop * 512 / tot4[512] / 1e12, 1),
                           note="the same 40 layers from the 4-bit storage: M = 1 four launches per layer, M = 512 seven "
                                "patch_gemm4_ex launches with the workspace; consecutive layers are timed in alternation (a "
                                "layer's 4-bit weights alone would stay in the last-level cache) and half of the pair counts")
    return dict(layers=40, launches_per_layer=4, packed_GB=round(packed_bytes / 1e9, 3), dense_GB=round(dense_bytes / 1e9, 3), **extra,
                f_mean=round(f_mean, 4), fractions="per (layer, matrix): synth.matrix_fractions" if per_matrix else "one per layer, U[0, 1)",
                rows=rows, per_layer=per_layer,
                note="time = sum over the 40 layers of the layer's four launches (q/k/v fused, o, gate/up fused, down), each layer "
                     "timed on its own after two warm-up passes with a caller workspace; frac_mfma_peak = issued matrix flops "
                     "(flop-weighted over the layers' fractions) / time / 2.5 PFLOP/s, the bound at M = 4096; frac_hbm_peak = "
                     "compressed weight bytes / time / 8 TB/s, the bound at M = 1; M = 512 sits near the ridge: both are given")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--m", type=int, default=4096, help="rows of X for the headline prefill workload")
    ap.add_argument("--f", type=float, default=0.6, help="fraction of 2:4 tiles of the headline workload")
    ap.add_argument("--skip", default="", help="comma list of sections to skip: decode,dense,half,bf16out,cpu,pack,mid,sweep,layer,ceilings,stack,alloc,qwen,q4,tile64")
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

    def settle(fn, batch=10, max_batches=12, tol=0.01):
        """Run fn in batches until two consecutive batch means agree within tol; -> steps run."""
        prev, n = None, 0
        for _ in range(max_batches):
            t = timed(fn, batch)
            n += batch
            if prev is not None and abs(t - prev) <= tol * prev:
                break
            prev = t
        return n

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

    settle_steps = settle(step)
    timed(step, args.warmup)
    secs = timed(step, args.steps)
    Y_sample = {L["name"]: L["Y"].cpu().numpy() for L in (layers[0], layers[2])} if "cpu" not in skip else {}
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

    # ------------------------------------------------------------------ the configuration's other row count (2048 rows)
    M2 = 2048
    half = None
    if "half" not in skip and M > M2:
        def step2(_i):
            for L in layers:
                B.patch_gemm(L["X"], M2, L["P"], L["Y"], stream, **opts)

        settle(step2)
        timed(step2, args.warmup)
        secs2 = timed(step2, args.steps)
        def step2f(_i):      # gate and up share X: one launch over both weights, then down
            B.patch_gemm_many(layers[0]["X"], M2, [layers[0]["P"], layers[1]["P"]], [layers[0]["Y"], layers[1]["Y"]], stream, **opts)
            B.patch_gemm(layers[2]["X"], M2, layers[2]["P"], layers[2]["Y"], stream, **opts)

        settle(step2f)
        timed(step2f, args.warmup)
        secs2f = timed(step2f, args.steps)
        need2 = max(B.patch_gemm_workspace_bytes(M2, layers[2]["P"]), 16)
        ws2 = torch.empty(need2 // 4, device=dev, dtype=torch.float32)

        def step2w(_i):      # and the down projection (128 tiles) with a workspace: K split over the idle half of the chip
            B.patch_gemm_many(layers[0]["X"], M2, [layers[0]["P"], layers[1]["P"]], [layers[0]["Y"], layers[1]["Y"]], stream, **opts)
            B.patch_gemm(layers[2]["X"], M2, layers[2]["P"], layers[2]["Y"], stream, workspace=ws2, **opts)

        settle(step2w)
        timed(step2w, args.warmup)
        secs2w = timed(step2w, args.steps)
        del ws2
        half = dict(M=M2, ms_per_step=secs2 / args.steps * 1e3, ms_per_step_gate_up_in_one_launch=secs2f / args.steps * 1e3,
                    ms_per_step_one_launch_and_workspace=secs2w / args.steps * 1e3, workspace_MB=round(need2 / 1e6, 1), dense_equiv_TFLOPs=dense_flop * M2 / M / (secs2 / args.steps) / 1e12,
                    frac_mfma_peak=issued_flop * M2 / M / (secs2 / args.steps) / 1e12 / PEAK_MFMA_BF16_TF,
                    note="the same three launches on the first 2048 rows of X (the 7B MLP prefill configuration names both row "
                         "counts): 344 + 344 + 128 output tiles on 256 compute units, i.e. part-filled rounds; gate and up in one "
                         "launch (patch_gemm_many) are 688 tiles, three rounds instead of four; with a caller workspace the down "
                         "projection splits K over the idle half of the chip")

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

        settle(dstep)
        timed(dstep, args.warmup)
        dsecs = timed(dstep, args.steps)
        speedup = dsecs / secs
        out["all_dense_ms_per_step"] = dsecs / args.steps * 1e3
        if half is not None:
            def dstep2(_i):
                for X, P0, Y in dl:
                    B.patch_gemm(X, M2, P0, Y, stream, **opts)

            settle(dstep2)
            timed(dstep2, args.warmup)
            d2 = timed(dstep2, args.steps)
            half["all_dense_ms_per_step"] = d2 / args.steps * 1e3
            half["speedup_vs_all_dense"] = d2 / (half["ms_per_step"] * 1e-3 * args.steps)
        for _, P0, _ in dl:
            P0.close()

    if half is not None:
        out["prefill_m2048"] = half

    # ------------------------------------------------------------------ the headline step with bf16 output (half the stores)
    if "bf16out" not in skip:
        Yb = [torch.empty((M, L["c"].N), device=dev, dtype=torch.bfloat16) for L in layers]

        def bstep(_i):
            for L, Y16 in zip(layers, Yb):
                B.patch_gemm(L["X"], M, L["P"], Y16, stream, y_bf16=True, **opts)

        settle(bstep)
        timed(bstep, args.warmup)
        bsecs = timed(bstep, args.steps)
        out["prefill_bf16_out"] = dict(M=M, ms_per_step=bsecs / args.steps * 1e3, dense_equiv_TFLOPs=dense_flop / (bsecs / args.steps) / 1e12,
                                       frac_mfma_peak=issued_flop / (bsecs / args.steps) / 1e12 / PEAK_MFMA_BF16_TF,
                                       speedup_vs_fp32_output=secs / bsecs,
                                       note="the headline step with the accumulator rounded to bf16 in the output stage (patch_gemm_opts.y_bf16): "
                                            "half the bytes stored, a few per cent at most since the output stage stores whole rows (ceilings."
                                            "store_tiles has the stores on their own); not the headline, whose Y is fp32 (a bf16 Y alone is "
                                            "outside the 1e-3 bar against the fp64 oracle)")
        del Yb

    # ------------------------------------------------------------------ pack throughput (one-off conversion)
    if "pack" not in skip:
        L = layers[0]
        c = L["c"]
        tp = time.time()
        for _ in range(3):
            B.patch_pack(L["W_hat"], c.N, c.K, c.tile_map, t, stream).close()
        torch.cuda.synchronize()
        pack_ms = (time.time() - tp) / 3 * 1e3
        ts = time.time()
        saved = L["P"].serialize(stream)
        save_ms = (time.time() - ts) * 1e3
        ts = time.time()
        B.patch_deserialize(saved, stream).close()
        load_ms = (time.time() - ts) * 1e3
        out["pack"] = dict(shape=[c.N, c.K], ms=pack_ms, saved_MB=round(saved.size / 1e6, 2), serialize_ms=round(save_ms, 1),
                           deserialize_ms=round(load_ms, 1),
                           note="patch_pack wall time incl. allocation and the status read-back; patch_serialize / patch_deserialize "
                                "to and from pageable host memory, incl. the checksum over every byte")
        del saved

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
        settle(lambda _i: B.patch_gemm(Xf, M, Pf[2], Yf, stream, **opts), batch=30)
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

    # ------------------------------------------------------------------ mask tile 64 (the paper's other tile size) on the same projections
    if "tile64" not in skip:
        rows64 = []
        for name, N_, K_ in (("gate", 11008, 4096), ("down", 4096, 11008)):
            us_f = {}
            for ff in (0.0, 0.6, 1.0):
                c64 = synth.make_case("llama7b_mlp_t64_" + name, N_, K_, M, 64, ff, seed=0)
                W_hat64, P64 = masked_packed(c64)
                X64 = layers[0]["X"] if K_ == 4096 else layers[2]["X"]
                Y64 = layers[0]["Y"] if N_ == 11008 else layers[2]["Y"]
                fn = lambda _i: B.patch_gemm(X64, M, P64, Y64, stream)
                settle(fn, batch=10, max_batches=8)
                us_f[ff] = sorted(timed(fn, 10) / 10 for _ in range(3))[1] * 1e6
                P64.close()
                del W_hat64
            rows64.append(dict(shape=[N_, K_], M=M, tile=64, us_f0=round(us_f[0.0], 1), us_f06=round(us_f[0.6], 1), us_f1=round(us_f[1.0], 1),
                               dense_equiv_TFLOPs_f06=round(2.0 * M * N_ * K_ / us_f[0.6] / 1e6, 1),
                               speedup_f06_over_all_dense=round(us_f[0.0] / us_f[0.6], 3), speedup_f1_over_all_dense=round(us_f[0.0] / us_f[1.0], 3)))
        out["prefill_tile64"] = dict(rows=rows64, note="mask tile 64 x 64 on prefill_kernel_areg<64, 256> (256 x 256 workgroup tiles, weights straight into registers); "
                                     "the headline uses mask tile 128 on prefill_kernel_wreg")

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
                                            "features per wavefront (from 33 rows on weights of at least 10240 features the prefill "
                                            "kernel with 128-row blocks), beyond that the prefill kernels")

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

    # ------------------------------------------------------------------ decode from the 4-bit weight-only storage (Section 5.2)
    if "q4" not in skip:
        qrows = []
        for name, N_, K_ in (("attn", 4096, 4096), ("gate", 11008, 4096), ("down", 4096, 11008)):
            for fd in (0.0, 0.5):
                cq = synth.make_case("llama7b_q4_" + name, N_, K_, 16, t, fd, seed=0)
                W_hat, Pb = masked_packed(cq)
                P4 = B.patch_pack4(W_hat, N_, K_, cq.tile_map, t, stream)
                R4 = max(2, int(np.ceil(1.1e9 / P4.nbytes)))
                Rb = max(2, int(np.ceil(1.1e9 / Pb.nbytes)))
                P4s = [P4] + [B.patch_pack4(W_hat, N_, K_, cq.tile_map, t, stream) for _ in range(R4 - 1)]
                Pbs = [Pb] + [B.patch_pack(W_hat, N_, K_, cq.tile_map, t, stream) for _ in range(Rb - 1)]
                Xq = dev_bf16(cq.X)
                Yq4 = torch.empty((16, N_), device=dev, dtype=torch.float32)
                for Mq in (1, 16):
                    f4 = lambda i, Mq=Mq: B.patch_gemm4(Xq, Mq, P4s[i % R4], Yq4, stream)
                    fb = lambda i, Mq=Mq: B.patch_gemm(Xq, Mq, Pbs[i % Rb], Yq4, stream)
                    nl = max(1, args.decode_launches // 2)
                    timed(f4, 20)
                    us4 = sorted(timed(f4, nl) / nl for _ in range(5))[2] * 1e6
                    timed(fb, 20)
                    usb = sorted(timed(fb, nl) / nl for _ in range(5))[2] * 1e6
                    gbs = P4.nbytes / (us4 * 1e-6) / 1e9
                    qrows.append(dict(shape=[N_, K_], f=fd, M=Mq, us=round(us4, 3), GBps=round(gbs, 1), frac_hbm=round(gbs / PEAK_HBM_GBS, 4),
                                      packed_MB=round(P4.nbytes / 1e6, 3), copies=R4, us_bf16_storage=round(usb, 3),
                                      speedup_vs_bf16_storage=round(usb / us4, 3),
                                      bytes_vs_dense_bf16=round(P4.nbytes / (2.0 * N_ * K_), 4)))
                for P_ in P4s + Pbs:
                    P_.close()
                del W_hat
        # one 7B decoder layer from the 4-bit storage at M = 1: q/k/v fused, o, gate/up fused, down (4 launches), rotating
        # over copies of the layer; beside it the single launches of the same seven weights
        q4layer = []
        for fd in (0.0, 0.5):
            shapes7 = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
                       ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
            copies, nbytes = 12, 0
            layer = [dict() for _ in range(copies)]
            for name, N_, K_ in shapes7:
                cl = synth.make_case("llama7b_layer_" + name, N_, K_, 1, t, fd, seed=0)
                W_hat, P0 = masked_packed(cl)
                P0.close()
                for ci in range(copies):
                    layer[ci][name] = B.patch_pack4(W_hat, N_, K_, cl.tile_map, t, stream)
                nbytes += layer[0][name].nbytes
                del W_hat
            x4 = dev_bf16(synth.make_case("llama7b_layer_x", 128, 4096, 1, t, 0.0, seed=1).X)
            x11 = dev_bf16(synth.make_case("llama7b_layer_x2", 128, 11008, 1, t, 0.0, seed=2).X)
            y = {n: torch.empty((1, N_), device=dev, dtype=torch.float32) for n, N_, _ in shapes7}

            def layer4(L):
                B.patch_gemm4_many(x4, 1, [L["q"], L["k"], L["v"]], [y["q"], y["k"], y["v"]], stream)
                B.patch_gemm4(x4, 1, L["o"], y["o"], stream)
                B.patch_gemm4_many(x4, 1, [L["gate"], L["up"]], [y["gate"], y["up"]], stream)
                B.patch_gemm4(x11, 1, L["down"], y["down"], stream)

            def layer4_single(L):
                for n in ("q", "k", "v", "o", "gate", "up"):
                    B.patch_gemm4(x4, 1, L[n], y[n], stream)
                B.patch_gemm4(x11, 1, L["down"], y["down"], stream)

            res = {}
            for label, fn in (("fused", layer4), ("single", layer4_single)):
                run = lambda i, fn=fn: fn(layer[i % copies])
                timed(run, 24)
                res[label] = sorted(timed(run, 120) / 120 for _ in range(3))[1] * 1e6
            q4layer.append(dict(f=fd, M=1, packed_MB=round(nbytes / 1e6, 1), copies=copies, us_4_launches=round(res["fused"], 2),
                                us_7_launches=round(res["single"], 2), GBps=round(nbytes / (res["fused"] * 1e-6) / 1e9, 1),
                                frac_hbm=round(nbytes / (res["fused"] * 1e-6) / 1e9 / PEAK_HBM_GBS, 4)))
            for L in layer:
                for P_ in L.values():
                    P_.close()
        out["decode_q4_layer_7b"] = dict(rows=q4layer, note="the seven projections of one 7B decoder layer from the 4-bit storage at "
                                         "M = 1, per layer: q/k/v and gate/up in one launch each (patch_gemm4_many) against seven "
                                         "single launches; rotating over copies of the layer (> 1 GB)")
        out["decode_q4"] = dict(rows=qrows, note="patch_gemm4: 4-bit codes + bf16 scale per row of a tile (+ 2:4 positions), dequantized in "
                                "registers; rotating packed copies (HBM-resident); us_bf16_storage = patch_gemm on the same pruned weight")
        # the prefill-shaped product from the same 4-bit storage (patch_gemm4_ex), beside 64-row passes and the bf16 storage
        prow = []
        for name, N_, K_ in (("attn", 4096, 4096), ("gate", 11008, 4096)):
            cq = synth.make_case("llama7b_q4p_" + name, N_, K_, 2048, t, 0.5, seed=0)
            W_hat, Pb = masked_packed(cq)
            P4 = B.patch_pack4(W_hat, N_, K_, cq.tile_map, t, stream)
            Xq = dev_bf16(cq.X)
            Yq = torch.empty((2048, N_), device=dev, dtype=torch.float32)
            wsq = torch.empty(8 * 512 * N_, device=dev, dtype=torch.float32)
            for Mq in (128, 512, 2048):
                fns = (("us_passes_of_64_rows", lambda i: B.patch_gemm4_many(Xq, Mq, [P4], [Yq], stream)),
                       ("us", lambda i: B.patch_gemm4(Xq, Mq, P4, Yq, stream)),
                       ("us_with_workspace", lambda i: B.patch_gemm4(Xq, Mq, P4, Yq, stream, workspace=wsq)),
                       ("us_bf16_storage_with_workspace", lambda i: B.patch_gemm(Xq, Mq, Pb, Yq, stream, workspace=wsq)))
                row = dict(shape=[N_, K_], M=Mq, f=0.5, packed_MB=round(P4.nbytes / 1e6, 2), bf16_packed_MB=round(Pb.nbytes / 1e6, 2))
                for key, fn in fns:
                    n_ = 20 if Mq <= 512 else 5
                    timed(fn, n_)
                    row[key] = round(min(timed(fn, n_) / n_ for _ in range(3)) * 1e6, 1)
                row["dense_equiv_TFLOPs_with_workspace"] = round(2.0 * Mq * N_ * K_ / (row["us_with_workspace"] * 1e-6) / 1e12, 1)
                prow.append(row)
            P4.close(); Pb.close()
            del W_hat, Xq, Yq, wsq
        out["prefill_q4"] = dict(rows=prow, note="patch_gemm4_ex on mask tile 128: the weight stays in 4 bits (read once per 128 rows of X, "
                                 "dequantized in registers); passes = the decode-shaped kernel repeated per 64 rows; bf16 storage = "
                                 "patch_gemm on the bf16 packing of the same pruned weight (4 x the bytes)")

    # ------------------------------------------------------------------ measured ceilings (kernels of this library)
    if "ceilings" not in skip:
        n_cus = torch.cuda.get_device_properties(dev).multi_processor_count
        ceil = dict(compute_units=n_cus)
        res = torch.empty(2 * n_cus * 256, device=dev, dtype=torch.float32)
        iters = 12000
        best_rate = {}
        for label, ops in (("random_operands", torch.randn(B.PROBE_OPERAND_BYTES // 2, device=dev).to(torch.bfloat16)),
                           ("zero_operands", torch.zeros(B.PROBE_OPERAND_BYTES // 2, device=dev, dtype=torch.bfloat16))):
            for kind, name, flop in ((0, "dense_mfma_16x16x32_bf16", 16384.0), (1, "sparse_smfmac_16x16x64_bf16", 32768.0),
                                     (2, "dense_mfma_32x32x16_bf16_unused_shape", 16384.0), (3, "sparse_smfmac_32x32x32_bf16_unused_shape", 32768.0)):
                if kind >= 2 and label != "random_operands":
                    continue
                for wps in (1, 2):      # wavefronts per SIMD
                    fn = lambda _i, kind=kind, ops=ops, wps=wps: B.patch_probe_matrix_rate(kind, ops, wps * n_cus, iters, res, stream)
                    timed(fn, 2)
                    t_best = min(timed(fn, 3) / 3 for _ in range(3))
                    rate = round(wps * n_cus * 4 * iters * 16 * flop / t_best / 1e12, 1)   # a round is 16 x flop for every kind
                    ceil[f"{name}_{label}_{wps}_per_simd_TFLOPs"] = rate
                    best_rate[(kind, label)] = max(best_rate.get((kind, label), 0.0), rate)
        P_d, P_s = best_rate[(0, "random_operands")], best_rate[(1, "random_operands")]
        fa = 1.0 - issued_flop / dense_flop * 2.0 + 1.0     # f of the headline set: issued = dense (2 - f) / 2
        p_mix = 1.0 / ((1.0 - fa) / P_d + fa / P_s)
        ceil["headline_mix_weighted_measured_peak_TFLOPs"] = round(p_mix, 1)
        ceil["headline_frac_of_measured_mix_peak"] = round(value / p_mix, 4)
        # beside the fraction of the published peak: the same launch against the mix-weighted rate the two matrix
        # instructions reach on this part with random operands and no memory traffic (dense-equivalent flops on both sides)
        roof["frac_of_measured_mix_peak"] = round(value / p_mix, 4)
        roof["measured_mix_peak_TFLOPs_dense_equivalent"] = round(p_mix, 1)
        ceil["matrix_note"] = ("register-resident loops, one or two wavefronts per SIMD on every compute unit, no memory traffic; 2:4 in "
                               "dense-equivalent flops; the clock under matrix load depends on the operand data, hence both figures; the "
                               "mix-weighted peak uses the better random-operand figure of each instruction")
        big = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
        big.random_(0, 255)
        sink = torch.empty(4096 * 1024, dtype=torch.int32, device=dev)
        best = None
        for wg, th in ((n_cus * 8, 256), (n_cus * 4, 512), (n_cus * 2, 1024), (n_cus * 16, 256)):
            fn = lambda _i, wg=wg, th=th: B.patch_probe_stream_read(big, big.numel(), wg, th, sink, stream)
            timed(fn, 2)
            t_ = min(timed(fn, 5) / 5 for _ in range(3))
            if best is None or t_ < best[0]:
                best = (t_, wg, th)
        ceil["stream_read_2GiB_GBps"] = round(big.numel() / best[0] / 1e9, 1)
        ceil["stream_read_2GiB_launch"] = [best[1], best[2]]
        # the decode launch shape of the 4096 x 4096 projection (256 workgroups of 16 wavefronts) over 33.5 MB pieces,
        # rotating through the 2 GiB buffer so that no cache holds a piece when its turn comes again
        piece, n_piece = 4096 * 4096 * 2, (2 << 30) // (4096 * 4096 * 2)
        fn = lambda i: B.patch_probe_stream_read(big.data_ptr() + (i % n_piece) * piece, piece, 256, 1024, sink, stream)
        timed(fn, 20)
        t_ = sorted(timed(fn, 200) / 200 for _ in range(5))[2]
        ceil["stream_read_33MB_decode_launch_shape_us"] = round(t_ * 1e6, 2)
        ceil["stream_read_33MB_decode_launch_shape_GBps"] = round(piece / t_ / 1e9, 1)
        fn = lambda i: B.patch_probe_stream_read(big.data_ptr(), 16, 1, 64, sink, stream)
        timed(fn, 20)
        ceil["empty_launch_us"] = round(sorted(timed(fn, 200) / 200 for _ in range(5))[2] * 1e6, 2)
        # what one compute unit fetches per K-step of the LDS-staged prefill kernels, on its own: 48 KB rounds (or 24 KB
        # rounds, one or two in flight) by 8 wavefronts; every workgroup on its own cache-resident chunk, or walking 48 MB
        fill = dict()
        rounds = 256
        empty_us = ceil["empty_launch_us"]
        for label, wg, chunks in (("cache_resident_all_cus", n_cus, n_cus), ("streaming_16_workgroups", 16, 1024), ("streaming_all_cus", n_cus, 1024)):
            for kind, name, kb in ((0, "global_to_lds_48KB", 48), (2, "global_to_registers_48KB", 48), (4, "global_to_lds_24KB", 24),
                                   (3, "global_to_lds_24KB_two_in_flight", 24)):
                fn = lambda _i, kind=kind, wg=wg, chunks=chunks: B.patch_probe_lds_fill(kind, big, chunks * 48 * 1024, wg, rounds, sink, stream)
                timed(fn, 2)
                per_round = (min(timed(fn, 5) / 5 for _ in range(3)) * 1e6 - empty_us) / rounds
                fill[f"{name}_{label}"] = dict(us_per_round=round(per_round, 3), GBps_per_cu=round(kb * 1024 / per_round / 1e3, 1))
        ceil["cu_fetch"] = fill
        ceil["cu_fetch_note"] = ("a round = every wavefront of a workgroup of 8 issues its 1 KB pieces, waits for them and meets the others at a "
                                 "barrier; the per-compute-unit rate is the same with one or two rounds in flight, so it is a throughput, not "
                                 "a latency: it bounds a K-step of the kernels that stage both operands (48 KB with blocks of 128 rows)")
        del big, sink
        # the output stage of the prefill kernel on its own: one workgroup per 256 x 256 tile of a 4096 x 11008 output
        # (688 tiles, the gate projection's grid) and of a 1536 x 11008 one (258 tiles: one round and two stragglers, whose
        # time is what a compute unit needs when nothing else is storing), two Y buffers in alternation
        st = dict()
        for bf in (False, True):
            Ys = [torch.empty((4096, 11008), device=dev, dtype=torch.bfloat16 if bf else torch.float32) for _ in range(2)]
            for rows_ in (4096, 1536):
                for pat, pname in ((0, "16_rows_x_%d_bytes" % (32 if bf else 64)), (1, "4_rows_x_%d_bytes" % (128 if bf else 256))):
                    fn = lambda i, pat=pat, bf=bf, rows_=rows_: B.patch_probe_store_tiles(pat, bf, Ys[i & 1], rows_, 11008, stream)
                    timed(fn, 6)
                    t_ = sorted(timed(fn, 40) / 40 for _ in range(3))[1]
                    st[f"{'bf16' if bf else 'fp32'}_{rows_ // 256 * 43}_tiles_{pname}_us"] = round(t_ * 1e6, 1)
            del Ys
        ceil["store_tiles"] = st
        # LDS read rate of a compute unit with four wavefronts (the prefill kernel's X fragments): 128 KB per 64-column step
        lout = torch.empty(n_cus * 256, device=dev, dtype=torch.float32)
        l_iters = 20000
        fn = lambda _i: B.patch_probe_lds_read(n_cus, l_iters, lout, stream)
        timed(fn, 2)
        t_ = min(timed(fn, 3) / 3 for _ in range(3))
        ceil["lds_read_GBps_per_cu_4_wavefronts"] = round(l_iters * 32768 / t_ / 1e9, 1)
        ceil["lds_read_note"] = ("conflict-free ds_read_b128, 8 in flight per wavefront, one workgroup of 4 wavefronts per compute unit, no "
                                 "other work (the clock is not held down by matrix instructions as it is in the product kernels)")
        del lout
        ceil["store_tiles_note"] = ("stores only, 4 wavefronts x 64 store instructions per tile: 16 rows x 64 bytes per instruction is the "
                                    "accumulator layout stored as it lies, 4 rows x 256 bytes the same data after a turn through LDS (what the "
                                    "prefill kernels do); 688 tiles = 2.7 rounds of the chip, bound by the HBM write rate in either pattern "
                                    "for fp32; 258 tiles = one round and two stragglers, and bf16: the row pattern is the faster one")
        # vendor dense GEMM (bf16 output) on the headline shapes, for context: same macro tile class, same part
        vend = []
        for name, N_, K_ in (("gate", 11008, 4096), ("down", 4096, 11008)):
            Xv = torch.randn(M, K_, device=dev, dtype=torch.float32).to(torch.bfloat16)
            Wv = (torch.randn(N_, K_, device=dev, dtype=torch.float32) * 0.02).to(torch.bfloat16)
            Yv = torch.empty(M, N_, device=dev, dtype=torch.bfloat16)
            fn = lambda _i: torch.matmul(Xv, Wv.t(), out=Yv)
            settle(fn, batch=20)
            t_ = min(timed(fn, 20) / 20 for _ in range(3))
            P0 = B.patch_pack(Wv, N_, K_, np.ones((N_ // t, K_ // t), np.uint8), t, stream)
            Yo_ = torch.empty(M, N_, device=dev, dtype=torch.float32)
            fo = lambda _i: B.patch_gemm(Xv, M, P0, Yo_, stream)
            settle(fo, batch=20)
            t_o = min(timed(fo, 20) / 20 for _ in range(3))
            vend.append(dict(shape=[N_, K_], M=M, vendor_us=round(t_ * 1e6, 1), vendor_TFLOPs=round(2.0 * M * N_ * K_ / t_ / 1e12, 1),
                             this_library_all_dense_us=round(t_o * 1e6, 1), this_library_all_dense_TFLOPs=round(2.0 * M * N_ * K_ / t_o / 1e12, 1)))
            P0.close()
            del Xv, Wv, Yv, Yo_
        ceil["vendor_dense_gemm"] = dict(rows=vend, note="torch.matmul (the vendor library), bf16 in / bf16 out, random data; this library: "
                                         "all-dense tile map, fp32 out.  Context only.")
        out["ceilings"] = ceil

    # ------------------------------------------------------------------ 0.5B-scale layer set (launch-latency-bound)
    if "qwen" not in skip:
        rows = []
        for N_, K_ in ((896, 896), (4864, 896), (896, 4864)):
            for fd in (0.0, 0.5, 1.0):
                cq = synth.make_case("qwen0p5b", N_, K_, 64, t, fd, seed=0)
                W_hat, Pq = masked_packed(cq)
                Xq = dev_bf16(cq.X)
                Yq = torch.empty((64, N_), device=dev, dtype=torch.float32)
                r_ = dict(shape=[N_, K_], f=fd, packed_MB=round(Pq.nbytes / 1e6, 2))
                wsq = torch.empty(8 * 64 * N_, device=dev, dtype=torch.float32)
                for Mq in (1, 64):
                    fn = lambda _i, Mq=Mq: B.patch_gemm(Xq, Mq, Pq, Yq, stream)
                    timed(fn, 20)
                    r_[f"us_M{Mq}"] = round(sorted(timed(fn, 200) / 200 for _ in range(3))[1] * 1e6, 2)
                fn = lambda _i: B.patch_gemm(Xq, 64, Pq, Yq, stream, workspace=wsq)
                timed(fn, 20)
                r_["us_M64_with_workspace"] = round(sorted(timed(fn, 200) / 200 for _ in range(3))[1] * 1e6, 2)
                rows.append(r_)
                Pq.close()
                del W_hat, Xq, Yq
        out["qwen_0p5b"] = dict(rows=rows, note="0.5B-scale set, tile 128, cache-resident (1.6 - 8.7 MB): bounded by launch latency "
                                "(an empty launch is in ceilings.empty_launch_us), not by a roofline; with a caller workspace the "
                                "64-row pass over a weight of few features splits K over otherwise idle compute units")

    # ------------------------------------------------------------------ 13B decoder stack
    if "stack" not in skip:
        out["stack_13b"] = stack_13b(torch, B, synth, dev, stream, timed, t, q4="q4" not in skip)
        if "alloc" not in skip:
            out["stack_13b_per_matrix"] = stack_13b(torch, B, synth, dev, stream, timed, t, per_matrix=True)

    # ------------------------------------------------------------------ CPU oracle on a bounded sample
    cpu = None
    if "cpu" not in skip:
        from oracle import oracle
        Ms = M
        cs, flop, num, den = 0.0, 0.0, 0.0, 0.0
        for L in (layers[0], layers[2]):       # gate and down: two of the step's three launches (up has gate's shape)
            c = L["c"]
            W_hat_o = oracle.apply_mask(c.W, c.tile_map, c.mask24, t)
            vals, meta = oracle.pack(W_hat_o, c.tile_map, t)
            tc = time.time()
            Yo = oracle.gemm(c.X[:Ms], vals, meta, c.N, c.K, c.tile_map, t)
            cs += time.time() - tc
            flop += 2.0 * Ms * c.N * c.K
            Yg = Y_sample[L["name"]][:Ms].astype(np.float64)
            num += float(np.sum((Yg - Yo) ** 2))
            den += float(np.sum(Yo ** 2))
            del Yo, Yg
        cpu = dict(value=flop / cs / 1e12, unit="TFLOP/s (dense-equivalent)", cores=oracle.num_threads(),
                   kind="oracle", seconds=round(cs, 2),
                   sample=f"gate (11008x4096) and down (4096x11008) projections of the step, first {Ms} of {M} rows of X, fp64, "
                          "decompress + one dot product per output")
        out["relF_vs_oracle_on_sample"] = float(np.sqrt(num / den))

    line = {
        "metric": "hybrid GEMM dense-equiv TFLOP/s + GB/s vs roofline; speedup over all-dense",
        "value": value, "unit": "TFLOP/s (dense-equivalent)", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "settle_steps": settle_steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
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
