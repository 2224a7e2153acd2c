#!/usr/bin/env python3
"""Benchmark of the decimation hot path on one MI355X.

One "step" = one whole picasso_decimate call (vertex quadrics, then every
round: edges, costs, selection, contraction, facet clean-up) on the
115k-vertex synthetic room mesh, decimated to 41,500 vertices (about 36 %),
inputs resident in HBM.  For the hierarchy workload (batch16x60k) a step is
the whole ladder: four batched decimations in a row, each to 40 % per mesh.
Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload room115k]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def source_hash():
    """sha256 over the HIP sources: what the stored HBM-traffic figures are stamped with."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2103_15076_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".h", ".hip")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()


def measured_traffic(workload):
    """HBM-side bytes per launch of the bracketed kernels from the rocprofv3 --pmc runs summarised in
    profiles/hbm_traffic.txt ({kernel key: bytes}), or {} when that file was taken with other kernel
    sources than the ones that are running now (the figures would be stale)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return {}
    out, ok = {}, False
    for line in open(path):
        w = line.split()
        if not w or w[0].startswith("#"):
            continue
        if w[0] == "source_sha256":
            ok = w[1] == source_hash()
        elif w[0] == workload and len(w) >= 3:
            out[w[1]] = float(w[2])
    return out if ok else {}


KERNEL_KEYS = ("sort", "unique_cost", "subround0", "facet_insert", "quadric_rows", "sort_incidence")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="room115k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="leave out the per-launch hipEvents of the roofline measurement")
    ap.add_argument("--kernel-events-every", type=int, default=10, metavar="N",
                    help="bracket the roofline kernels' launches with hipEvents in every N-th timed step (default 10)")
    ap.add_argument("--copy-calib", action="store_true",
                    help="only run the plain copy kernel on 1 GiB (HBM yardstick / counter calibration)")
    ap.add_argument("--pool", type=int, default=0, metavar="C",
                    help="also time pooling/unpooling of C-channel features over the recorded clusters")
    ap.add_argument("--conv", type=int, default=0, metavar="C",
                    help="also time the depth-wise vertex2facet / facet2vertex convolutions on the input mesh, "
                         "C channels, 6 Gaussian components")
    ap.add_argument("--stages", action="store_true", help="also print per-stage times to stderr")
    ap.add_argument("--placement", choices=["mean", "inverse"], default="mean",
                    help="contraction target: the pair's mean (default, the headline path) or the point of "
                         "least quadric error with fallback to the mean")
    ap.add_argument("--rcond-min", type=float, default=1e-3, help="rank threshold of --placement inverse")
    ap.add_argument("--shuffle-seed", type=int, default=0,
                    help="seeded order among pairs of equal cost (the paper's augmentation shuffle); 0 = index order")
    ap.add_argument("--absorb", action="store_true",
                    help="apply Alg. 2 line 11 (un-paired vertices join a neighbouring pair's cluster, under the "
                         "budget); the headline path contracts pairs only")
    ap.add_argument("--stream-sync", action="store_true",
                    help="the host waits by synchronising the stream (PICASSO_OPT_HOST_POLL = 0) instead of "
                         "watching the word its last kernel writes to pinned memory")
    ap.add_argument("--single-stream", action="store_true",
                    help="keep the first round's edge sort on the caller's stream (PICASSO_OPT_OVERLAP = 0)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU only (the path shards by mesh: with more GPUs every rank "
              "would decimate its own meshes, with no exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2103_15076_amd as pk
    from paper_2103_15076_amd import meshgen

    pk.load_library()  # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.copy_calib:
        # plain copy of a known size: achievable HBM rate, and the reference for profiler byte counters
        nbytes = 1 << 30
        src = torch.empty(nbytes // 4, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        s = torch.cuda.current_stream()
        for _ in range(3):
            pk.picasso_device_copy(dst, src, s)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 10
        e0.record(s)
        for _ in range(reps):
            pk.picasso_device_copy(dst, src, s)
        e1.record(s)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        print(json.dumps({"copy_kernel": "copy_kernel", "bytes_read": nbytes, "bytes_written": nbytes,
                          "ms": round(ms, 4), "GBps_read_plus_write": round(2 * nbytes / ms / 1e6, 1),
                          "frac_of_8TBps": round(2 * nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)}))
        return

    cfg = meshgen.config(args.workload)
    V, F = cfg["verts"], cfg["facets"]
    nv_in, nf_in, target = cfg["nv"], cfg["nf"], cfg["target"]
    N, NF, B = int(V.shape[0]), int(F.shape[0]), int(nv_in.shape[0])
    dV, dF = torch.from_numpy(V).to(dev), torch.from_numpy(F).to(dev)
    vo = torch.empty((N, 3), dtype=torch.float32, device=dev)
    fo = torch.empty((NF, 3), dtype=torch.int32, device=dev)
    cid = torch.empty((N,), dtype=torch.int32, device=dev)
    ctx = pk.Context(N, NF, B, device=0)
    stream = torch.cuda.current_stream()
    inverse = args.placement == "inverse"
    if (inverse or args.absorb or args.shuffle_seed) and B > 1 and not args.no_cpu_baseline:
        sys.exit("bench.py: --placement inverse / --absorb / --shuffle-seed on a batch need --no-cpu-baseline (the "
                 "oracle's batch entry point runs the default path)")
    if inverse:
        ctx.set_placement(pk.PICASSO_PLACE_INVERSE, args.rcond_min)
    if args.absorb:
        ctx.set_option(pk.PICASSO_OPT_ABSORB, 1)
    if args.shuffle_seed:
        ctx.set_option(pk.PICASSO_OPT_SHUFFLE_SEED, args.shuffle_seed)
    if args.stream_sync:
        ctx.set_option(pk.PICASSO_OPT_HOST_POLL, 0)

    levels = int(cfg.get("levels", 1))
    targets = [np.asarray(target, np.int32)]
    for _ in range(1, levels):   # every further level keeps 40 % of each mesh's vertices
        targets.append((targets[-1].astype(np.int64) * 4 // 10).astype(np.int32))
    lev_out = [(torch.empty((N, 3), dtype=torch.float32, device=dev), torch.empty((NF, 3), dtype=torch.int32, device=dev),
                torch.empty((N,), dtype=torch.int32, device=dev)) for _ in range(levels - 1)]
    lev_ev = [torch.cuda.Event(enable_timing=True) for _ in range(levels + 1)]

    def step(stats=None, record=False):
        """One pass of the whole path: one decimation, or for the hierarchy workload its levels in a row,
        each level's output mesh being the next level's input.  Returns the last level's result and, per
        level, (status, verts, facets, cluster ids, nv[B], nf[B])."""
        if levels == 1:
            if B == 1:
                return ctx.picasso_decimate(dV, dF, int(target[0]), vo, fo, cid, stats=stats, stream=stream), None
            return ctx.picasso_decimate_batch(dV, dF, nv_in, nf_in, target, vo, fo, cid, stats=stats, stream=stream), None
        per_level = []
        v_in, f_in, nvs, nfs = dV, dF, nv_in, nf_in
        if record:
            lev_ev[0].record(stream)
        for lv in range(levels):
            bufs = (vo, fo, cid) if lv == 0 else lev_out[lv - 1]
            r = ctx.picasso_decimate_batch(v_in, f_in, nvs, nfs, targets[lv], bufs[0], bufs[1],
                                           bufs[2][: int(v_in.shape[0])], stats=stats if lv == 0 else None, stream=stream)
            if record:
                lev_ev[lv + 1].record(stream)
            per_level.append(r)
            v_in, f_in, nvs, nfs = r[1], r[2], r[4], r[5]
        return per_level[-1], per_level

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # The collector is held off while timing (as timeit does): a full collection of this process
    # (torch, numpy and the mesh arrays alive) takes ~40 ms, two orders above one step.
    import gc
    gc.collect()
    gc.disable()

    # ---- timed region: exactly K steps, hipEvents on the launch stream + wall clock
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    every = max(1, args.kernel_events_every)   # kernel events in every `every`-th step: all calls of such a step
    if args.single_stream:
        ctx.set_option(pk.PICASSO_OPT_OVERLAP, 0)
    for k in range(pk.PICASSO_KERNEL_COUNT):
        ctx.picasso_kernel_timing(k, reset=True)
    torch.cuda.synchronize()
    level_ms = [0.0] * levels
    t0 = time.perf_counter()
    ev0.record(stream)
    for k_step in range(args.steps):
        if not args.no_kernel_events:
            ctx.set_option(pk.PICASSO_OPT_KERNEL_TIMING, 1 if k_step % every == 0 else 0)
        res, res_levels = step(record=levels > 1)
        if levels > 1:   # (the host has waited for every level's work; the last event follows it at once)
            lev_ev[levels].synchronize()
            for lv in range(levels):
                level_ms[lv] += lev_ev[lv].elapsed_time(lev_ev[lv + 1])
    ev1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ev_ms = ev0.elapsed_time(ev1)
    ms_per_step = max(wall_ms, ev_ms) / args.steps
    nv_out, nf_out = int(res[1].shape[0]), int(res[2].shape[0])
    gc.enable()
    # hipEvents around the largest kernels' launches in every N-th step of the timed region
    kts = [ctx.picasso_kernel_timing(k, reset=True) for k in range(pk.PICASSO_KERNEL_COUNT)]

    # ---- one extra call for the per-round shape and stage times
    st = pk.picasso_stats()
    ctx.set_option(pk.PICASSO_OPT_KERNEL_TIMING, 0)
    ctx.set_option(pk.PICASSO_OPT_STAGE_TIMING, 1)
    step(st)
    ctx.set_option(pk.PICASSO_OPT_STAGE_TIMING, 0)
    sd = st.as_dict()
    if args.stages:
        print(json.dumps(sd), file=sys.stderr)

    # Roofline: every bracketed kernel against the HBM peak (algorithmic bytes per launch / average
    # launch time); the headline entry is the kernel with the largest share of the step.
    traffic = measured_traffic(args.workload)
    timed_steps = (args.steps + every - 1) // every
    by_kernel = []
    for key, kt in zip(KERNEL_KEYS, kts):
        if kt["launches"] == 0:
            continue
        avg_ms = kt["ms_total"] / kt["launches"]
        bytes_per_launch = kt["bytes_total"] / kt["launches"]
        achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9
        by_kernel.append({"bound": "hbm", "kernel": kt["kernel"], "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                          "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5), "traffic": traffic.get(key),
                          "launches_timed": kt["launches"], "events_every_n_steps": every,
                          "avg_launch_us": round(avg_ms * 1e3, 3), "algorithmic_bytes_per_launch": int(bytes_per_launch),
                          "event_ms_per_timed_step": round(kt["ms_total"] / timed_steps, 4)})
    by_kernel.sort(key=lambda r: -r["event_ms_per_timed_step"])
    roofline = by_kernel[0] if by_kernel else None

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        times = []
        reps = 5 if N < 500000 else 2

        def oracle_pass():
            """The same work on one host core: one decimation, or the hierarchy's levels in a row."""
            if B == 1:
                return [oracle.decimate(V, F, int(target[0]), placement=1 if inverse else 0,
                                        rcond_min=args.rcond_min if inverse else 0.0, absorb=args.absorb,
                                        shuffle_seed=args.shuffle_seed)]
            outs, v_in, f_in, nvs, nfs = [], V, F, nv_in, nf_in
            for lv in range(levels):
                r = oracle.decimate_batch(v_in, f_in, nvs, nfs, targets[lv])
                outs.append(r)
                v_in, f_in, nvs, nfs = r["verts"], r["facets"], r["nv"], r["nf"]
            return outs

        for _ in range(reps):
            c0 = time.perf_counter()
            refs = oracle_pass()
            times.append(time.perf_counter() - c0)
        med = float(np.median(times))
        got = res_levels if res_levels is not None else [res]
        same = all(np.array_equal(g[3].cpu().numpy(), r["cluster_id"]) and np.array_equal(g[2].cpu().numpy(), r["facets"])
                   and np.array_equal(g[1].cpu().numpy().view(np.uint32), r["verts"].view(np.uint32))
                   for g, r in zip(got, refs))
        what = "decimation" if levels == 1 else f"pass over the {levels} levels"
        cpu_baseline = {"value": round(NF / med, 1), "unit": "facets/s", "cores": 1, "kind": "oracle",
                        "sample": f"the full workload, median of {reps} runs ({med * 1e3:.1f} ms per {what})",
                        "ms_per_decimation": round(med * 1e3, 2), "gpu_matches_oracle_bit_exact": bool(same)}

    pooling = None
    if args.pool:
        # pooling / unpooling of C-channel features over the clusters just recorded (network-style use)
        C = args.pool
        n_out = nv_out
        x = torch.randn((N, C), device=dev, dtype=torch.float32)
        g = torch.randn((n_out, C), device=dev, dtype=torch.float32)
        cid_c = res[3].contiguous()

        def timed(fn, reps=20):
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps

        t_csr = timed(lambda: ctx.picasso_cluster_csr(cid_c, n_out))
        off, mem = ctx.picasso_cluster_csr(cid_c, n_out)
        _, arg = ctx.picasso_pool_forward(pk.PICASSO_POOL_MAX, x, off, mem)
        rows = {
            "max_forward": (lambda: ctx.picasso_pool_forward(pk.PICASSO_POOL_MAX, x, off, mem), 4 * C * (N + 2 * n_out) + 8 * N),
            "avg_forward": (lambda: ctx.picasso_pool_forward(pk.PICASSO_POOL_AVG, x, off, mem), 4 * C * (N + n_out) + 8 * N),
            "max_backward": (lambda: ctx.picasso_pool_backward(pk.PICASSO_POOL_MAX, g, cid_c, off, mem, argmax=arg), 4 * C * (N + 2 * n_out) + 4 * N),
            "unpool_forward": (lambda: ctx.picasso_unpool_forward(g, cid_c), 4 * C * (N + n_out) + 4 * N),
            "unpool_backward": (lambda: ctx.picasso_unpool_backward(x, off, mem), 4 * C * (N + n_out) + 8 * N),
        }
        pooling = {"channels": C, "n_in": N, "n_out": n_out, "cluster_csr_ms": round(t_csr, 4)}
        for name, (fn, nbytes) in rows.items():
            ms = timed(fn)
            pooling[name] = {"ms": round(ms, 4), "algorithmic_MB": round(nbytes / 1e6, 2),
                             "GBps": round(nbytes / ms / 1e6, 1), "frac_of_8TBps": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)}

    convs = None
    if args.conv:
        # one vertex2vertex convolution's depth-wise kernels on the input mesh (forward and backward)
        C, T = args.conv, 6

        def timed_c(fn, reps=20):
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps

        xin = torch.randn((N, C), device=dev, dtype=torch.float32)
        w3 = torch.randn((3, C), device=dev, dtype=torch.float32)
        wt = torch.randn((T, C), device=dev, dtype=torch.float32)
        mu = torch.tensor([[1, 0, 0], [-1, 0, 0], [0, 1, 0], [0, -1, 0], [0, 0, 1], [0, 0, -1]], device=dev,
                          dtype=torch.float32)
        iv = torch.full((T,), 2.0, device=dev, dtype=torch.float32)
        nf_list = [int(v) for v in nf_in] if B > 1 else None
        t_csr = timed_c(lambda: ctx.picasso_vertex_corner_csr(dF, N), reps=5)
        off_c, cor_c = ctx.picasso_vertex_corner_csr(dF, N)
        t_geo = timed_c(lambda: ctx.picasso_facet_geometry(dV, dF, nf=nf_list), reps=5)
        nrm, _, lev = ctx.picasso_facet_geometry(dV, dF, nf=nf_list)
        t_fz = timed_c(lambda: ctx.picasso_fuzzy_coefficients(nrm, mu, iv))
        pi_c = ctx.picasso_fuzzy_coefficients(nrm, mu, iv)
        yb = torch.empty((NF, C), device=dev, dtype=torch.float32)
        xb = torch.empty((N, C), device=dev, dtype=torch.float32)
        ctx.picasso_v2f_forward(xin, dF, lev, w3, out=yb)
        idx_f, idx_v = 4 * (3 * NF + NF), 4 * (3 * NF + N)
        rows_c = {
            "v2f_forward": (lambda: ctx.picasso_v2f_forward(xin, dF, lev, w3, out=yb), 4 * C * (N + NF) + idx_f),
            "f2v_forward": (lambda: ctx.picasso_f2v_forward(yb, pi_c, wt, off_c, cor_c, N, out=xb),
                            4 * C * (N + NF) + idx_v + 4 * T * NF),
            "v2f_backward": (lambda: ctx.picasso_v2f_backward(yb, xin, dF, lev, w3, off_c, cor_c),
                             4 * C * (2 * N + 2 * NF) + idx_f + idx_v),
            "f2v_backward": (lambda: ctx.picasso_f2v_backward(xin, yb, pi_c, wt, dF, off_c, want_gpi=False),
                             4 * C * (2 * N + 3 * NF) + idx_f + 2 * 4 * T * NF),
        }
        convs = {"channels": C, "components": T, "verts": N, "facets": NF, "corner_csr_ms": round(t_csr, 4),
                 "facet_geometry_ms": round(t_geo, 4), "fuzzy_ms": round(t_fz, 4)}
        for name, (fn, nbytes) in rows_c.items():
            ms = timed_c(fn)
            convs[name] = {"ms": round(ms, 4), "algorithmic_MB": round(nbytes / 1e6, 2),
                           "GBps": round(nbytes / ms / 1e6, 1), "frac_of_8TBps": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)}

    out = {
        "metric": "input facets/s per decimation (ms per decimation in ms_per_step)",
        "value": round(NF / (ms_per_step * 1e-3), 1),
        "unit": "facets/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "n_meshes": B, "verts_in": N, "facets_in": NF,
                   "target_nv": int(np.sum(target)), "verts_out": nv_out, "facets_out": nf_out,
                   "rounds": sd["rounds"], "subrounds": sd["subrounds"], "edges": sd["ne"],
                   "placement": args.placement + (f" (rcond_min {args.rcond_min:g})" if inverse else ""),
                   "line_11": bool(args.absorb), "shuffle_seed": args.shuffle_seed,
                   "host_wait": "stream synchronisation" if args.stream_sync else "pinned-memory sequence number"},
        "paper_context": {"ms": 65.0, "gpu": "RTX 2080 Ti (paper's machine, its own 115,114-vertex mesh)"},
        "event_ms_per_step": round(ev_ms / args.steps, 4),
        "stage_ms": {k: round(sum(r[k] for r in sd["ms_stage"]), 4) for k in pk.binding.STAGE_NAMES},
        "roofline": roofline,
        "roofline_by_kernel": by_kernel,
        "cpu_baseline": cpu_baseline,
    }
    if levels > 1:
        # the hierarchy: per-level time (hipEvents between the levels of every timed step) and sizes
        out["levels"] = [{"level": lv + 1, "ms": round(level_ms[lv] / args.steps, 4),
                          "verts_in": int(np.sum(nv_in)) if lv == 0 else int(res_levels[lv - 1][1].shape[0]),
                          "facets_in": NF if lv == 0 else int(res_levels[lv - 1][2].shape[0]),
                          "verts_out": int(res_levels[lv][1].shape[0]), "facets_out": int(res_levels[lv][2].shape[0])}
                         for lv in range(levels)]
        out["config"]["levels"] = levels
        out["config"]["stage_ms_and_rounds_are_of"] = "level 1" 
    if pooling is not None:
        out["pooling"] = pooling
    if convs is not None:
        out["convolutions"] = convs
    print(json.dumps(out))
    ctx.close()


if __name__ == "__main__":
    main()
