#!/usr/bin/env python3
"""Benchmark of the GAD per-processor hot path on one MI355X.

One "step" = one pass of the per-iteration hot path over one augmented subgraph resident in HBM:
gcn_forward + gcn_backward (full batch: one pass = one epoch of that subgraph), subgraph_variance on the
per-node gradients, and the K-way weighted_consensus of parameter copies.  The CSR build (a load-time
step) is timed separately and reported as `build_ms`.

Prints ONE JSON line (the README lists the fields).  `value` = layer-edges per second:
n_layers * nnz(A+I) / (forward + backward time), i.e. the per-layer edge rate of a full fwd+bwd.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E bandwidth


class HipEvents:
    """HIP events made through the runtime itself (hipEventCreate): their handles can be handed to the library,
    which records them on the stream it launches on."""

    def __init__(self, count):
        import ctypes as C
        self.C, self.hip = C, C.CDLL("libamdhip64.so")
        self.ev = []
        for _ in range(count):
            e = C.c_void_p()
            assert self.hip.hipEventCreate(C.byref(e)) == 0
            self.ev.append(e)

    def handles(self):
        return [e.value for e in self.ev]

    def ms(self, i, j):
        t = self.C.c_float()
        assert self.hip.hipEventElapsedTime(self.C.byref(t), self.ev[i], self.ev[j]) == 0
        return float(t.value)


def gather_sweep(args) -> int:
    """Uniform random graphs: no hub rows, so nearly every gathered row is a miss of whatever cache is smaller than
    the source matrix.  The rate over the gather-model bytes is then the ceiling of that level for 1 KB gathers."""
    import dataclasses
    import numpy as np
    import torch
    from paper_2110_02987_amd import gad, workloads as wl
    torch.cuda.set_device(0)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    w, out = 256, []
    for n in (2048, 16384, 65536, 131072, 262144, 690000, 2000000):
        cfg = dataclasses.replace(wl.CONFIGS["tiny"], name=f"er{n}", n_local=n, avg_degree=50.0)
        gr = wl.make_graph(cfg)
        g = gad.build_subgraph(dev(gr["src"]), dev(gr["dst"]), gr["n_global"], dev(gr["local_ids"]), dev(gr["halo_ids"]))
        T = torch.randn((n, w), device="cuda")
        O = torch.empty_like(T)
        sws = gad.spmm_workspace(g, w)
        for _ in range(3):
            gad.spmm(g, T, O, w, gad.F32, sws)
        ts = []
        for _ in range(args.kernel_reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            gad.spmm(g, T, O, w, gad.F32, sws)
            b.record()
            ts.append((a, b))
        torch.cuda.synchronize()
        ms = float(np.median([a.elapsed_time(b) for a, b in ts]))
        gather = g.nnz * (4 + 4 * w) + n * (12 + 4 * w)
        out.append(dict(n=n, nnz=g.nnz, source_MB=n * w * 4 / 1e6, ms=ms, gather_model_GBps=gather / ms * 1e-6))
        print(f"uniform random graph n={n:8d} nnz={g.nnz:10d} source matrix {n * w * 4 / 1e6:7.1f} MB: "
              f"{ms:8.4f} ms  {gather / ms * 1e-6:7.0f} GB/s of gather-model bytes", flush=True)
        del g, T, O, sws
    print(json.dumps(dict(gather_sweep=out, width=w)))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="products_part")
    ap.add_argument("--storage", choices=["f32", "bf16"], default=None,
                    help="storage type of features / activations (default: the workload's own)")
    ap.add_argument("--generator-row-order", action="store_true",
                    help="variant: rows in the generator's node order (Chung-Lu: sorted by expected degree) instead of "
                         "the seeded shuffle")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-reps", type=int, default=20, help="standalone launches of the dominant kernel")
    ap.add_argument("--gather-sweep", action="store_true",
                    help="measurement aid: the width-256 SpMM on uniform random graphs (average degree 50) whose source "
                         "matrix grows from 2 MB (fits one L2) over 268 MB (about the Infinity Cache) to 2 GB (HBM): "
                         "what random 1 KB row gathers reach at each level of the memory system; prints one line per size")
    ap.add_argument("--kernels-only", action="store_true",
                    help="profiling aid: run only a 1 GiB device copy (counter calibration) and the standalone SpMM "
                         "launches, no training steps, no CPU baseline")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs one augmented subgraph on ONE GPU; the only cross-GPU step of the method "
              "(the weighted all-reduce of Eq. 15) is not part of it. Run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2110_02987_amd import gad, workloads as wl

    if args.gather_sweep:
        return gather_sweep(args)
    cfg = wl.CONFIGS[args.workload]
    variant = ""
    if args.storage and args.storage != cfg.dtype:          # a variant of the named workload, reported as such
        import dataclasses
        cfg = dataclasses.replace(cfg, dtype=args.storage)
        variant = f" [{args.storage} storage variant]"
    if args.generator_row_order:
        import dataclasses
        cfg = dataclasses.replace(cfg, shuffle_rows=False)
        variant += " [rows in generator order]"
    dims, L = list(cfg.dims), cfg.n_layers
    torch.cuda.set_device(0)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    # ---- inputs (synthetic, seeded), resident in HBM before anything is timed
    gr = wl.make_graph(cfg)
    X = wl.make_features(cfg.n, dims[0])
    Ws = wl.make_weights(dims)
    y = wl.make_labels(cfg.n, dims[-1])
    mask = wl.make_mask(cfg)
    c = 1.0 / float(mask.sum())
    src, dst = dev(gr["src"]), dev(gr["dst"])
    loc, halo = dev(gr["local_ids"]), dev(gr["halo_ids"])
    bf16 = cfg.dtype == "bf16"
    dt = gad.BF16 if bf16 else gad.F32
    esz = 2 if bf16 else 4                                  # bytes per stored node-matrix element
    if bf16:                                                # features rounded to bfloat16 once (nearest even)
        bits = wl.to_bf16_rne(X)
        Xd = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
        X = wl.bf16_to_f32(bits)                            # what the oracle starts from
    else:
        Xd = dev(X)
    Wd, yd, md = [dev(w) for w in Ws], dev(y), dev(mask)
    K = max(cfg.consensus_k, 1)
    copies = [dev(p) for p in wl.make_param_copies(dims, K)]
    torch.cuda.synchronize()

    t0 = time.perf_counter()
    g = gad.build_subgraph(src, dst, gr["n_global"], loc, halo)
    torch.cuda.synchronize()
    build_ms = (time.perf_counter() - t0) * 1e3
    del src, dst

    ws = gad.alloc_workspace(g, dims, dt)
    loss = torch.zeros(1, dtype=torch.float64, device="cuda")
    dW = [torch.empty_like(w) for w in Wd]
    G_last = torch.empty((g.n, dims[-1]), device="cuda")
    G_out = [None] * (L - 1) + [G_last]
    out3 = torch.zeros(3, dtype=torch.float64, device="cuda")
    consensus = torch.empty(cfg.n_params, device="cuda")
    zetas = [1.0 + 0.1 * k for k in range(K)]

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(record=None, x_unchanged=False):
        e = [ev() for _ in range(4)] if record is not None else None
        if e: e[0].record()
        gad.gcn_forward(g, Xd, dims, Wd, yd, md, c, ws, None, loss, dt, x_unchanged=x_unchanged)
        if e: e[1].record()
        gad.gcn_backward(g, Xd, dims, Wd, ws, dW, G_out, dt)
        if e: e[2].record()
        gad.subgraph_variance(g, G_last, 1.0, out3)
        gad.weighted_consensus(copies, zetas, consensus)
        if e:
            e[3].record()
            record.append(e)

    if args.kernels_only:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)                       # plain copy: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b
        args.warmup, args.steps, args.no_cpu_baseline = 0, 1, True
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    rec = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(rec)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    med = lambda xs: float(np.median(xs))
    fwd_ms = med([e[0].elapsed_time(e[1]) for e in rec])
    bwd_ms = med([e[1].elapsed_time(e[2]) for e in rec])
    tail_ms = med([e[2].elapsed_time(e[3]) for e in rec])
    epoch_ms = med([e[0].elapsed_time(e[2]) for e in rec])
    value = L * g.nnz / (epoch_ms * 1e-3)
    # The same step when the caller vouches that X has not changed (static features): the first layer's aggregate
    # A~ X is then reused.  Reported beside the figures above, never in `value`.
    cached_epoch_ms = None
    if not args.kernels_only:
        rec_c = []
        for _ in range(args.steps):
            step(rec_c, x_unchanged=True)
        torch.cuda.synchronize()
        cached_epoch_ms = med([e[0].elapsed_time(e[2]) for e in rec_c])

    # ---- per layer: the library records events at the layer boundaries of both passes (its own stream).  The
    # instrumented backward waits for each layer's weight gradient before the next layer starts, so the layers add
    # up to a little more than the plain backward above.  edges/s of a layer = nnz / (its forward + its backward).
    per_layer = None
    if not args.kernels_only:
        hev = HipEvents(2 * L + 3)
        gad.gcn_layer_events(hev.handles())
        f_l, b_l, loss_l = [[] for _ in range(L)], [[] for _ in range(L)], []
        for _ in range(args.steps):
            step()
            torch.cuda.synchronize()
            for l in range(L):
                f_l[l].append(hev.ms(l, l + 1))
                b_l[l].append(hev.ms(L + 2 + (L - 1 - l), L + 3 + (L - 1 - l)))
            loss_l.append(hev.ms(L, L + 1))
        gad.gcn_layer_events([])
        per_layer = []
        for l in range(L):
            fm, bm = med(f_l[l]), med(b_l[l])
            per_layer.append(dict(layer=l + 1, dims=f"{dims[l]}x{dims[l + 1]}",
                                  order="aggregate-first" if dims[l] <= dims[l + 1] else "transform-first",
                                  spmm_width=min(dims[l], dims[l + 1]), forward_ms=fm, backward_ms=bm,
                                  edges_per_s=g.nnz / ((fm + bm) * 1e-3)))
        per_layer.append(dict(layer="loss", forward_ms=med(loss_l)))

    # ---- dominant kernel: the SpMM at each width the step uses, timed alone with events on the launch stream
    widths = []
    for l in range(L):
        w = dims[l] if dims[l] <= dims[l + 1] else dims[l + 1]
        widths.append(w)                                   # forward
        if not (l == 0 and dims[l] <= dims[l + 1]):
            widths.append(w)                               # backward (layer 1 needs none when it aggregates first)
    # the attainable ceiling of a plain device copy on this machine, in the same run: 1 GiB read + 1 GiB written
    a_ = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    b_ = torch.empty_like(a_)
    for _ in range(3):
        b_.copy_(a_)
    cp = []
    for _ in range(10):
        e0, e1 = ev(), ev()
        e0.record()
        b_.copy_(a_)
        e1.record()
        torch.cuda.synchronize()
        cp.append(e0.elapsed_time(e1))
    copy_ceiling = 2.0 * a_.numel() * 4 / med(cp) * 1e-6          # GB/s
    del a_, b_

    spmm = {}
    for w in sorted(set(widths)):
        ld = (w + 15) // 16 * 16
        T = torch.randn((g.n, ld), device="cuda").to(torch.bfloat16 if bf16 else torch.float32)
        O = torch.empty_like(T)
        sws = gad.spmm_workspace(g, w)
        for _ in range(3):
            gad.spmm(g, T, O, w, dt, sws)
        times = []
        for _ in range(args.kernel_reps):
            a, b = ev(), ev()
            a.record()
            gad.spmm(g, T, O, w, dt, sws)
            b.record()
            times.append((a, b))
        torch.cuda.synchronize()
        ms = med([a.elapsed_time(b) for a, b in times])
        compulsory = 4 * g.nnz + 12 * g.n + 2 * g.n * w * esz
        gather = g.nnz * (4 + w * esz) + g.n * (12 + w * esz)
        spmm[w] = dict(ms=ms, launches_per_step=widths.count(w), edges_per_s=g.nnz / (ms * 1e-3),
                       compulsory_GBps=compulsory / ms * 1e-6, gather_model_GBps=gather / ms * 1e-6,
                       compulsory_bytes=compulsory, gather_model_bytes=gather)
        del T, O, sws
    dom = max(spmm, key=lambda w: spmm[w]["ms"] * spmm[w]["launches_per_step"])
    d = spmm[dom]
    # Roofline of the dominant kernel against the 8 TB/s HBM peak.  `achieved` = bytes that cross from L2 to the
    # memory side per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter reads for a plain
    # 1 GiB copy) / the launch time measured here.  The counters cannot be read from inside this process: they come
    # from the committed summary under profiles/, which names the commit and the command it was taken with.  The
    # counter sits in front of the Infinity Cache, so this is an upper bound of the DRAM rate.  Beside it, the two
    # byte models of the method: gather (4 B index + one w-wide row per edge; rowptr + dinv + one written row per
    # node: what moves if no gathered row is reused from a cache; it can exceed the peak because L2 serves part of
    # it) and compulsory (every array once: the least HBM could move).
    roofline = dict(bound="hbm", kernel=f"spmm_kernel (A~ T at width {dom}, {cfg.dtype} storage)",
                    achieved=None, peak=HBM_PEAK_GBPS, unit="GB/s", frac=None, traffic=None, traffic_source=None,
                    avg_launch_ms=d["ms"],
                    gather_model=dict(bytes=d["gather_model_bytes"], GBps=d["gather_model_GBps"],
                                      formula=f"nnz*(4 + {esz}w) + n*(12 + {esz}w)"),
                    compulsory_model=dict(bytes=d["compulsory_bytes"], GBps=d["compulsory_GBps"],
                                          frac_of_peak=d["compulsory_GBps"] / HBM_PEAK_GBPS,
                                          formula=f"4 nnz + 12 n + 2 n w {esz}"),
                    time_over_compulsory=d["ms"] / (d["compulsory_bytes"] / HBM_PEAK_GBPS * 1e-6),
                    copy_ceiling_GBps=copy_ceiling)
    tr = os.path.join(ROOT, "profiles", f"spmm_{cfg.name}_hbm_traffic.txt")
    if os.path.exists(tr) and not variant:                  # the committed counters are those of the workload as named
        stamp = ""
        for line in open(tr):
            if line.startswith("# taken at commit"):
                stamp = line[1:].strip()
            if line.startswith("traffic "):
                kv = dict(t.split("=") for t in line.split()[1:])
                if int(kv["width"]) == dom:
                    nbytes = 1024.0 * (float(kv["fetch_kib"]) * float(kv["fetch_scale"]) +
                                       float(kv["write_kib"]) * float(kv["write_scale"]))
                    roofline["traffic"] = nbytes
                    roofline["traffic_source"] = f"profiles/{os.path.basename(tr)} ({stamp})"
                    roofline["traffic_launch_ms_in_profile"] = float(kv.get("avg_dur_us", "nan")) * 1e-3
                    roofline["achieved"] = nbytes / d["ms"] * 1e-6
                    roofline["traffic_over_gather_model"] = nbytes / d["gather_model_bytes"]
                    roofline["traffic_over_compulsory"] = nbytes / d["compulsory_bytes"]
    if roofline["achieved"] is None:                         # no counter summary for this workload / variant:
        roofline["achieved"] = d["compulsory_GBps"]          # the strict lower bound of the HBM rate stands in
        roofline["achieved_is"] = "compulsory-model bytes / time (lower bound; no counter summary for this workload)"
    roofline["frac"] = roofline["achieved"] / HBM_PEAK_GBPS
    roofline["frac_of_copy_ceiling"] = roofline["achieved"] / copy_ceiling

    # ---- the dense contractions of each layer, timed alone (MFMA kernels): H W forward and the weight gradient
    mfma_peak = 2500.0 if bf16 else 157.3                  # published dense TFLOP/s of the instruction's type
    gemm = {}
    tdt = torch.bfloat16 if bf16 else torch.float32
    for l in range(L):
        K_, N_ = dims[l], dims[l + 1]
        if f"{K_}x{N_}" in gemm:
            continue
        A_ = torch.randn((g.n, K_), device="cuda").to(tdt)
        G_ = torch.randn((g.n, N_), device="cuda").to(tdt)
        C_ = torch.empty((g.n, N_), device="cuda", dtype=tdt)
        dW_ = torch.empty((K_, N_), device="cuda")
        gws = gad.gemm_workspace(g.n, K_, N_)
        res = {}
        for tag, fn in (("forward", lambda: gad.gemm_w(A_, Wd[l], C_, False, gws)),
                        ("weight_grad", lambda: gad.gemm_tn(A_, G_, dW_, K_, N_, gws))):
            for _ in range(2):
                fn()
            a, b = ev(), ev()
            a.record()
            for _ in range(args.kernel_reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b) / args.kernel_reps
            tf = 2.0 * g.n * K_ * N_ / ms * 1e-9
            res[tag] = dict(ms=ms, TFLOPs=tf, frac_of_mfma_peak=tf / mfma_peak)
        gemm[f"{K_}x{N_}"] = res
        del A_, G_, C_, dW_, gws

    # ---- the rows built beyond the per-iteration step, each timed once on this workload's graph (not part of `value`)
    extras = {}
    if not args.kernels_only:
        def timed(fn):
            fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            r = fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3, r
        # Algorithm 1 with this graph in the role of the original graph: partition = the first half of its rows
        part = torch.arange(g.n // 2, dtype=torch.int64, device="cuda")
        ms, (halo, n_walks) = timed(lambda: gad.augment_subgraph(g, part, L, g.n // 20, 1))
        extras["augment_subgraph"] = dict(ms=ms, n_part=int(part.numel()), walk_len=L, budget=g.n // 20,
                                          n_walks=int(n_walks), n_halo=int(halo.numel()))
        # Eq. 14 with the distance inside the pair sum, all pairs, on the last layer's per-node gradients
        pairs = g.n * (g.n - 1) / 2
        if pairs <= 5e11:                                  # about 1.5 s per call; the larger graphs would take minutes
            out2 = torch.zeros(2, dtype=torch.float64, device="cuda")
            ms, _ = timed(lambda: gad.pair_importance(g, G_last, 1.0, out2))
            extras["pair_importance"] = dict(ms=ms, pairs=pairs, F=int(G_last.shape[1]),
                                             pairs_per_s=pairs / (ms * 1e-3), zeta_pair=float(out2[0].item()))
        else:
            extras["pair_importance"] = dict(skipped=f"{pairs:.3g} pairs")
        del part, halo

    out = dict(metric="GCN fwd+bwd edges/s per layer and epoch ms per subgraph; SpMM % of HBM peak",
               value=value, unit="edges/s", n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=ms_per_step,
               higher_is_better=True, scaling="weak", vs_baseline=None, dtype=cfg.dtype, data="synthetic",
               config=dict(workload=f"{cfg.name}{variant}: n={g.n} ({cfg.n_local} local + {cfg.n_halo} halo), nnz={g.nnz}, "
                                    f"GCN {'-'.join(map(str, dims))}, consensus K={K}",
                           n=g.n, nnz=g.nnz, dims=dims),
               epoch_ms=epoch_ms, forward_ms=fwd_ms, backward_ms=bwd_ms, variance_consensus_ms=tail_ms,
               epoch_ms_first_aggregate_reused=cached_epoch_ms,
               per_layer=per_layer, build_ms=build_ms, spmm={str(k): v for k, v in spmm.items()}, gemm=gemm, extras=extras,
               mfma_peak_TFLOPs=mfma_peak, roofline=roofline)

    # ---- the oracle, as it stands, on the host cores (reported baseline, not a target)
    if not args.no_cpu_baseline:
        from oracle import gad_csr as T1
        t0 = time.perf_counter()
        ref = T1.build(**gr)
        cpu_build = time.perf_counter() - t0
        t0 = time.perf_counter()
        f = T1.forward(ref, X, Ws, y, mask, c)
        T1.backward(ref, Ws, f, y, mask, c)
        cpu_s = time.perf_counter() - t0
        out["cpu_baseline"] = dict(value=L * ref.nnz / cpu_s, unit="edges/s", cores=int(T1.lib().t1_num_threads()),
                                   kind="oracle", sample=f"one full forward+backward of the same workload "
                                   f"({cpu_s:.1f} s; CSR build {cpu_build:.1f} s not included), float64",
                                   epoch_ms=cpu_s * 1e3)
        out["loss_gpu"], out["loss_oracle"] = float(loss.item()), f["loss"]
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
