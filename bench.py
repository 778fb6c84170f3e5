#!/usr/bin/env python3
"""Benchmark of the K-FAC hot path on one MI355X.

One "step" = kfac_update_factors + kfac_invert_batch + kfac_precondition over the whole
ResNet-50-shaped layer set (54 layers, 108 factor matrices, batch 32, 224x224), all inputs
resident in HBM.  Prints ONE JSON line with the step time, the algorithmic TFLOP/s, the
roofline position of the dominant kernel (measured with HIP events inside the library on the
stream the kernels run on) and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3   # 256 CUs x 256 flop/clk x 2.4 GHz
WORKLOAD_NAMES = {
    "fc": "fc: single fully-connected layer 64->32, 32 rows",
    "cnn": "cnn: 4 conv3x3 + FC, batch 32, 32x32 input",
    "r50": "r50: ResNet-50-shaped layer set, batch 32, 224x224 input (54 layers, 108 factor matrices)",
    "r152": "r152: ResNet-152-shaped layer set, batch 32, 224x224 input (156 layers, 312 factor matrices)",
    "bertl": "bertl: BERT-large linear layers, 24 blocks, 4096 tokens (144 layers, 288 factor matrices)",
    "d201": "d201: DenseNet-201-shaped layer set, batch 16, 224x224 input (201 layers, 402 factor matrices)",
    "iv4": "iv4: Inception-v4-shaped layer set, batch 16, 224x224 input (150 layers, 300 factor matrices)",
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="r50", choices=list(WORKLOAD_NAMES))
    ap.add_argument("--cpu-budget", type=float, default=20.0, help="seconds of oracle time for cpu_baseline (0 = skip)")
    ap.add_argument("--no-breakdown", action="store_true", help="skip the extra per-kernel timing pass")
    ap.add_argument("--stale-inverses", action="store_true",
                    help="also time the variant that preconditions with the previous step's inverses on a second "
                         "stream while the new ones are computed (reported as an extra field, never as `value`)")
    ap.add_argument("--fit-inverse-model", action="store_true",
                    help="instead of the step benchmark: time kfac_invert_batch on single matrices d = 64 .. 8192 "
                         "(10 warm-up + 100 runs each) and fit t = alpha_inv * exp(beta_inv * d)")
    ap.add_argument("--opt", action="append", default=[], metavar="NAME=VALUE",
                    help="set a tuning option of the context (kfac_set_option; names in paper_2107_06533_amd.OPTIONS), for A/B runs")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a 1 GiB device-to-device copy (reference dispatch for scaling rocprofv3 byte counters)")
    return ap.parse_args()


def make_inputs(layers, hp):
    from synth import inputs
    with ThreadPoolExecutor(max_workers=8) as ex:
        return list(ex.map(lambda il: inputs.layer_inputs(il[1], hp["cid"], 0, il[0], hp["relu"]), enumerate(layers)))


def cpu_baseline(layers, hp, budget_s, flops_total):
    """Time the fp64 oracle on whole layers (largest shape classes first) until the budget is
    spent; scale to a full step by algorithmic flops."""
    import numpy as np
    import oracle
    from synth import inputs, shapes
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    classes = {}
    for i, l in enumerate(layers):
        key = (l.kind, l.dA, l.dG, l.R, l.kh, l.stride)
        classes.setdefault(key, []).append(i)
    order = sorted(classes.values(), key=lambda idx: -shapes.flops([layers[idx[0]]])["total"])
    spent, done_flops, used = 0.0, 0, []
    for idx in order:
        i = idx[0]
        l = layers[i]
        a, g, v = inputs.layer_inputs(l, hp["cid"], 0, i, hp["relu"])
        t0 = time.perf_counter()
        oracle.kfac_step([l], [a], [g], [v], [np.eye(l.dA)], [np.eye(l.dG)], hp["xi"], hp["gamma"])
        spent += time.perf_counter() - t0
        done_flops += shapes.flops([l])["total"]
        used.append(l.name or str(i))
        if spent >= budget_s:
            break
    est_ms = spent * 1e3 * flops_total / done_flops
    return {
        "value": round(est_ms, 1), "unit": "ms", "cores": int(cores), "kind": "oracle",
        "sample": (f"fp64 NumPy oracle, whole step on {len(used)} of {len(layers)} layers (largest shape classes first: "
                   f"{', '.join(used)}), {spent:.1f} s measured, {100.0 * done_flops / flops_total:.1f}% of the step's "
                   f"algorithmic flops, scaled to the full step by flops"),
        "measured_s": round(spent, 2),
    }


def cpu_baseline_small(names=("fc", "cnn")):
    """The oracle on the two small workloads, whole and unsampled (fc: its 3 steps), with all host
    threads and with one: 1 warm-up + 3 runs each, median."""
    import numpy as np
    import oracle
    from synth import inputs, shapes
    from threadpoolctl import threadpool_limits
    out = {}
    for name in names:
        hp = shapes.config_hparams(name)
        layers = shapes.config_layers(name)
        steps = 3 if name == "fc" else 1
        ins = [[inputs.layer_inputs(l, hp["cid"], st, i, hp["relu"]) for i, l in enumerate(layers)] for st in range(steps)]

        def run():
            A = [np.eye(l.dA) for l in layers]
            G = [np.eye(l.dG) for l in layers]
            for st in range(steps):
                a, g, v = zip(*ins[st])
                A, G, _, _, _ = oracle.kfac_step(layers, a, g, v, A, G, hp["xi"], hp["gamma"])

        res = {}
        for label, limit in (("all_threads_ms", None), ("one_thread_ms", 1)):
            ts = []
            with threadpool_limits(limits=limit):
                for rep in range(4):
                    t0 = time.perf_counter()
                    run()
                    ts.append((time.perf_counter() - t0) * 1e3)
            res[label] = round(float(np.median(ts[1:])), 2)
        res["steps"] = steps
        out[name] = res
    return out


def fit_inverse_model(pk, torch, np):
    """The paper's computation model of the inverse (Eq. inverting-model) fitted to this GPU with the
    paper's protocol: matrices of dimension 64 .. 8192, 10 warm-up and 100 timed runs each."""
    ctx = pk.Context(0)
    pts = []
    for d in (64, 128, 256, 512, 1024, 2048, 4096, 8192):
        B = torch.randn((d, 64), device="cuda")
        F = 0.05 * (B @ B.T) / 64.0
        F.diagonal().add_(0.95)
        X = torch.empty_like(F)
        for _ in range(10):
            ctx.kfac_invert_batch([d], [F], [X], 0.03)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(100):
            ctx.kfac_invert_batch([d], [F], [X], 0.03)
        e1.record()
        torch.cuda.synchronize()
        pts.append((d, e0.elapsed_time(e1) / 100.0 * 1e-3))
    ds = np.array([p[0] for p in pts], dtype=np.float64)
    ts = np.array([p[1] for p in pts], dtype=np.float64)
    beta, lna = np.polyfit(ds, np.log(ts), 1)
    ctx.close()
    print(json.dumps({"fit": "t_comp(d) = alpha_inv * exp(beta_inv * d), seconds", "alpha_inv": float(np.exp(lna)),
                      "beta_inv": float(beta), "points_d_seconds": [[int(d), round(t, 7)] for d, t in pts],
                      "max_rel_misfit": float(np.max(np.abs(np.exp(lna + beta * ds) / ts - 1.0)))}))


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the hot path is one worker's share); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2107_06533_amd as pk
    from synth import shapes

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    pk.load()                                      # fails loudly when the HIP library is missing
    torch.cuda.set_device(0)
    if args.fit_inverse_model:
        fit_inverse_model(pk, torch, np)
        return
    hp = shapes.config_hparams(args.config)
    layers = shapes.config_layers(args.config)
    n = len(layers)
    fl = shapes.flops(layers)

    t0 = time.perf_counter()
    ins = make_inputs(layers, hp)
    up = lambda x: torch.from_numpy(x).cuda()
    a_d = [up(x[0]) for x in ins]
    g_d = [up(x[1]) for x in ins]
    v_d = [up(x[2]) for x in ins]
    del ins
    A_d = [torch.eye(l.dA, device="cuda") for l in layers]
    G_d = [torch.eye(l.dG, device="cuda") for l in layers]
    XA_d = [torch.empty_like(t) for t in A_d]
    XG_d = [torch.empty_like(t) for t in G_d]
    P_d = [torch.empty_like(v) for v in v_d]
    info = torch.zeros(2 * n, dtype=torch.int32, device="cuda")
    dims = [l.dA for l in layers] + [l.dG for l in layers]
    dG, dA = [l.dG for l in layers], [l.dA for l in layers]
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t0

    ctx = pk.Context(0)
    for kv in args.opt:
        name, _, val = kv.partition("=")
        ctx.set_option(name, int(val))
    stream = torch.cuda.current_stream()

    def step():
        ctx.kfac_update_factors(layers, a_d, g_d, A_d, G_d, hp["xi"], stream=stream)
        ctx.kfac_invert_batch(dims, A_d + G_d, XA_d + XG_d, hp["gamma"], info, stream=stream)
        ctx.kfac_precondition(dG, dA, XG_d, XA_d, v_d, P_d, stream=stream)

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: K steps; the dominant kernel (grouped factor build) is bracketed by HIP events
    ctx.timing_enable(["factor_tiles"])
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    call_ms = [0.0, 0.0, 0.0]
    evs = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        e[0].record(stream)
        ctx.kfac_update_factors(layers, a_d, g_d, A_d, G_d, hp["xi"], stream=stream)
        e[1].record(stream)
        ctx.kfac_invert_batch(dims, A_d + G_d, XA_d + XG_d, hp["gamma"], info, stream=stream)
        e[2].record(stream)
        ctx.kfac_precondition(dG, dA, XG_d, XA_d, v_d, P_d, stream=stream)
        e[3].record(stream)
        evs.append(e)
    torch.cuda.synchronize()
    wall_s = time.perf_counter() - t0
    ms_per_step = wall_s * 1e3 / args.steps
    per_call = [[], [], []]
    step_ev_ms = []
    for e in evs:
        for k in range(3):
            t = e[k].elapsed_time(e[k + 1])
            call_ms[k] += t / args.steps
            per_call[k].append(t)
        step_ev_ms.append(e[0].elapsed_time(e[3]))
    call_median = [float(np.median(x)) for x in per_call]
    dom_ms, dom_n = ctx.timing_read("factor_tiles")
    ctx.timing_enable([])
    assert int(info.abs().sum()) == 0, "a factor was reported not positive definite"
    assert dom_n == args.steps

    # ---- per-kernel breakdown (extra, untimed pass with every kernel class bracketed)
    breakdown = None
    if not args.no_breakdown:
        ctx.timing_enable(pk.KERNEL_CLASSES)
        reps = 3
        for _ in range(reps):
            step()
        torch.cuda.synchronize()
        breakdown = {}
        for k in pk.KERNEL_CLASSES:
            ms, cnt = ctx.timing_read(k)
            breakdown[k] = {"ms_per_step": round(ms / reps, 4), "launches_per_step": cnt // reps}
        ctx.timing_enable([])

    # ---- packed upper triangles of all factors (what a multi-GPU job would put on the wire): an
    # HBM-bound move, reported next to the step, not part of it
    packed_io = None
    if not args.no_breakdown:
        tot, _ = ctx.packed_elems(dims)
        pbuf = torch.empty((tot,), device="cuda")
        reps = 20
        ev_p = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        for _ in range(3):
            ctx.kfac_pack_triangles(dims, A_d + G_d, pbuf, stream=stream)
            ctx.kfac_unpack_triangles(dims, pbuf, XA_d + XG_d, stream=stream)
        ev_p[0].record(stream)
        for _ in range(reps):
            ctx.kfac_pack_triangles(dims, A_d + G_d, pbuf, stream=stream)
        ev_p[1].record(stream)
        for _ in range(reps):
            ctx.kfac_unpack_triangles(dims, pbuf, XA_d + XG_d, stream=stream)
        ev_p[2].record(stream)
        torch.cuda.synchronize()
        pack_ms, unpack_ms = ev_p[0].elapsed_time(ev_p[1]) / reps, ev_p[1].elapsed_time(ev_p[2]) / reps
        full_bytes = 4 * sum(d * d for d in dims)
        pack_bytes, unpack_bytes = 2 * 4 * tot, 4 * tot + full_bytes      # read + write, algorithmic
        packed_io = {"packed_elems": tot, "pack_ms": round(pack_ms, 4), "unpack_ms": round(unpack_ms, 4),
                     "pack_gbps": round(pack_bytes / pack_ms / 1e6, 1), "unpack_gbps": round(unpack_bytes / unpack_ms / 1e6, 1),
                     "bound": "hbm", "peak_gbps": 8000.0,
                     "pack_frac": round(pack_bytes / pack_ms / 1e6 / 8000.0, 4),
                     "unpack_frac": round(unpack_bytes / unpack_ms / 1e6 / 8000.0, 4)}
        # inverse with the packed triangles written by the same kernels, against inverse + pack
        ev_q = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        for _ in range(2):
            ctx.kfac_invert_batch_packed(dims, A_d + G_d, XA_d + XG_d, pbuf, hp["gamma"], info, stream=stream)
        ev_q[0].record(stream)
        for _ in range(reps):
            ctx.kfac_invert_batch_packed(dims, A_d + G_d, XA_d + XG_d, pbuf, hp["gamma"], info, stream=stream)
        ev_q[1].record(stream)
        for _ in range(reps):
            ctx.kfac_invert_batch(dims, A_d + G_d, XA_d + XG_d, hp["gamma"], info, stream=stream)
            ctx.kfac_pack_triangles(dims, XA_d + XG_d, pbuf, stream=stream)
        ev_q[2].record(stream)
        torch.cuda.synchronize()
        packed_io["invert_packed_ms"] = round(ev_q[0].elapsed_time(ev_q[1]) / reps, 4)
        packed_io["invert_then_pack_ms"] = round(ev_q[1].elapsed_time(ev_q[2]) / reps, 4)
        # factor build with the packed triangles written by the same kernels, against factor build + pack
        ev_f = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        for _ in range(2):
            ctx.kfac_update_factors_packed(layers, a_d, g_d, A_d, G_d, hp["xi"], pbuf, stream=stream)
        ev_f[0].record(stream)
        for _ in range(reps):
            ctx.kfac_update_factors_packed(layers, a_d, g_d, A_d, G_d, hp["xi"], pbuf, stream=stream)
        ev_f[1].record(stream)
        for _ in range(reps):
            ctx.kfac_update_factors(layers, a_d, g_d, A_d, G_d, hp["xi"], stream=stream)
            ctx.kfac_pack_triangles(dims, A_d + G_d, pbuf, stream=stream)
        ev_f[2].record(stream)
        torch.cuda.synchronize()
        packed_io["update_packed_ms"] = round(ev_f[0].elapsed_time(ev_f[1]) / reps, 4)
        packed_io["update_then_pack_ms"] = round(ev_f[1].elapsed_time(ev_f[2]) / reps, 4)
        del pbuf
        step()          # the unpack above overwrote the inverses: restore a consistent state
        torch.cuda.synchronize()

    # ---- stale-inverse variant: precondition with the last inverses while the new ones are computed
    stale = None
    if args.stale_inverses:
        XA2 = [torch.empty_like(t) for t in XA_d]
        XG2 = [torch.empty_like(t) for t in XG_d]
        s_inv, s_pre = torch.cuda.Stream(), torch.cuda.Stream()
        cur, nxt = (XA_d, XG_d), (XA2, XG2)
        def stale_step():
            nonlocal cur, nxt
            ctx.kfac_update_factors(layers, a_d, g_d, A_d, G_d, hp["xi"], stream=stream)
            s_inv.wait_stream(stream); s_pre.wait_stream(stream)
            ctx.kfac_invert_batch(dims, A_d + G_d, nxt[0] + nxt[1], hp["gamma"], info, stream=s_inv)
            ctx.kfac_precondition(dG, dA, cur[1], cur[0], v_d, P_d, stream=s_pre)
            stream.wait_stream(s_inv); stream.wait_stream(s_pre)
            cur, nxt = nxt, cur
        for _ in range(3):
            stale_step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            stale_step()
        torch.cuda.synchronize()
        stale = {"ms_per_step": round((time.perf_counter() - t1) * 1e3 / args.steps, 4),
                 "note": "update_factors, then invert_batch (new inverses) and precondition (previous inverses) on two streams"}

    factor_flops = fl["factor_a"] + fl["factor_g"]
    dom_avg_ms = dom_ms / dom_n
    achieved = factor_flops / (dom_avg_ms * 1e-3) / 1e12
    # flops the tile jobs really execute (tile granularity): fewer than the algorithmic count where
    # 3x3 activation factors are assembled from lag products, more where tiles are ragged
    executed = {name: ctx.plan_stats(i)["mfma_flops"] for i, name in enumerate(("update_factors", "invert_batch", "precondition"))}
    # HBM bytes per launch of the dominant kernel: rocprofv3 counters cannot be read from inside this
    # process, so the figure comes from the committed counter summary of the same command line
    # (profiles/traffic.json, written by `python -m paper_2107_06533_amd.profile_summary`)
    traffic, traffic_src = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            rec = json.load(open(tpath)).get(args.config, {})
            traffic = rec.get("factor_tiles_bytes_per_launch")
            traffic_src = f"{rec.get('source')} (rocprofv3 FETCH_SIZE + WRITE_SIZE runs of this command, not this run)" if traffic else None
        except Exception:
            traffic = None
    inv_stats, pre_stats = ctx.plan_stats(1), ctx.plan_stats(2)
    nblk_max = max((d + 127) // 128 for d in dims)
    right = (breakdown or {}).get("precond_right", {}).get("ms_per_step")
    pre_right_flops = sum(2 * l.dG * l.dA * l.dA for l in layers)
    out = {
        "metric": "kfac_step_ms (factors + inverses + precondition)",
        "value": round(ms_per_step, 4),
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": WORKLOAD_NAMES[args.config], "layers": n, "matrices": 2 * n,
                   "xi": hp["xi"], "gamma": hp["gamma"], "setup_s": round(setup_s, 1)},
        "tflops": round(fl["total"] / (ms_per_step * 1e-3) / 1e12, 2),
        "frac_of_fp32_mfma_peak": round(fl["total"] / (ms_per_step * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS, 4),
        "ms_per_step_median": round(float(np.median(step_ev_ms)), 4),
        # per call: mean and median of the K timed steps (HIP events on the caller's stream); tflops and
        # frac_peak by the ALGORITHMIC flop count, frac_peak_executed by the flops the tile jobs execute
        # (what the matrix cores sustain: lower where lag products skip work, higher where tiles are ragged)
        "calls": {
            name: {"ms": round(call_ms[k], 4), "ms_median": round(call_median[k], 4),
                   "tflops": round(alg / call_ms[k] / 1e9, 2),
                   "frac_peak": round(alg / call_ms[k] / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
                   "frac_peak_executed": round(executed[name] / call_ms[k] / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4)}
            for k, (name, alg) in enumerate((("update_factors", factor_flops), ("invert_batch", fl["inverse"]),
                                             ("precondition", fl["precondition"])))
        },
        "algorithmic_flops": fl,
        "roofline": {
            "kernel": "tile_any_kernel (grouped factor build, one launch per step)",
            "bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
            "frac": round(achieved / PEAK_FP32_MFMA_TFLOPS, 4), "traffic": traffic, "traffic_source": traffic_src,
            "basis": "achieved and frac credit the ALGORITHMIC flops R*d*(d+1) per factor; lag products execute fewer, so the "
                     "utilisation of the matrix cores is executed_frac (algorithmic frac may exceed it, and 1, on lag-heavy sets)",
            "avg_launch_ms": round(dom_avg_ms, 4), "flops_per_launch": factor_flops,
            "executed_flops_per_launch": executed["update_factors"],
            "executed_tflops": round(executed["update_factors"] / (dom_avg_ms * 1e-3) / 1e12, 2),
            "executed_frac": round(executed["update_factors"] / (dom_avg_ms * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS, 4),
        },
        "executed_flops": executed,
        # the other two calls against the same roofline (whole call, mean of the timed steps)
        "roofline_calls": {
            "invert_batch": {
                "bound": "mfma", "achieved": round(fl["inverse"] / call_ms[1] / 1e9, 2), "peak": PEAK_FP32_MFMA_TFLOPS,
                "unit": "TFLOP/s", "frac": round(fl["inverse"] / call_ms[1] / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
                "executed_frac": round(executed["invert_batch"] / call_ms[1] / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
                "launches_per_call": inv_stats["n_launches"],
                # the sweep is a chain of dependent pivot blocks: that of the largest matrix bounds the call from below
                "critical_path": {"pivot_blocks": nblk_max, "ms_per_pivot_block": round(call_ms[1] / nblk_max, 4),
                                  "note": "call time / pivot blocks of the largest matrix; in-kernel times of one chain step "
                                          "(pivot block sweep + panel) are in the design notes"}},
            "precondition": {
                "bound": "mfma", "achieved": round(fl["precondition"] / call_ms[2] / 1e9, 2), "peak": PEAK_FP32_MFMA_TFLOPS,
                "unit": "TFLOP/s", "frac": round(fl["precondition"] / call_ms[2] / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
                "executed_frac": round(executed["precondition"] / call_ms[2] / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
                "launches_per_call": pre_stats["n_launches"],
                "right_product": None if not right else {
                    "kernel": "tile_gemm_dl_kernel (out = T . Ainv, direct-to-LDS loop)", "ms": right,
                    "tflops": round(pre_right_flops / right / 1e9, 2),
                    "frac": round(pre_right_flops / right / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4)}},
        },
    }
    if breakdown is not None:
        out["kernel_breakdown"] = breakdown
    if packed_io is not None:
        out["packed_io"] = packed_io
    if stale is not None:
        out["stale_inverses"] = stale
    if args.cpu_budget > 0:
        out["cpu_baseline"] = cpu_baseline(layers, hp, args.cpu_budget, fl["total"])
        out["cpu_baseline_small"] = cpu_baseline_small()
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
