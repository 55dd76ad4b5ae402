#!/usr/bin/env python3
"""Benchmark of the merged global-attention layer stack on one MI355X.

A *step* is one pass of the whole hot path over one synthetic sequence: the cached-index
layer driver (`litevggt_layers_run`) running all global layers of the workload, including
the merge-index refreshes.  `value` = tokens of the sequence / seconds per step, with all
inputs resident in HBM before the timed region.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload f1000]

Prints one JSON line.  `roofline` describes the dominant kernel (the attention kernel):
its duration is measured with HIP events that the driver records on the launch stream
inside the timed steps.  `cpu_baseline` is the CPU oracle timed on a bounded sub-sequence
of the same workload and scaled by each step's operation count; `parity` compares the HIP
path with that oracle run on the same sub-sequence (outside the timed region).
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

PEAK_BF16_MFMA_TFLOPS = 2500.0     # MI355X dense bf16
PEAK_FP8_MFMA_TFLOPS = 5000.0      # MI355X dense fp8
PEAK_HBM_GBS = 8000.0              # MI355X HBM3E


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="f1000", help="f32 | f100 | f500 | f1000 | tiny2 | paper1000")
    ap.add_argument("--merge-ratio", type=float, default=None)
    ap.add_argument("--refresh-interval", type=int, default=None,
                    help="layers between index refreshes (default: the workload's, 6)")
    ap.add_argument("--attn-dtype", default="bf16", choices=["bf16", "fp8"])
    ap.add_argument("--anchor-policy", default="ga", choices=["ga", "fixed", "random"],
                    help="what ranks the tokens: the GA map, or a geometry-blind partition")
    ap.add_argument("--block", action="store_true",
                    help="global layer = LayerNorm, q|k|v projection, attention, output projection, "
                         "MLP with seeded synthetic weights instead of the projection-free attention")
    ap.add_argument("--linear-dtype", default="bf16", choices=["bf16", "fp8", "fp8-delayed"],
                    help="with --block: operand type of its four linear layers (fp8: E4M3 per tensor, "
                         "scales from the tensors; fp8-delayed: input scales from an 80-step amax history)")
    ap.add_argument("--frame-attn", action="store_true",
                    help="run a frame attention after every global layer (not part of the metric's default)")
    ap.add_argument("--graph", action="store_true",
                    help="also capture one step into a HIP graph and time its replays "
                         "(reported as config.graph_replay_ms_per_step; `value` stays the eager run)")
    ap.add_argument("--no-unmerged", action="store_true",
                    help="skip the one-launch unmerged attention baseline")
    ap.add_argument("--qk-norm", type=int, default=1, choices=[0, 1],
                    help="1 (default): q and k RMS-normalised per head as in the model; 0: as given "
                         "(per-wave score bound, running-maximum second pass where it is loose)")
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the oracle leg (cpu_baseline and the parity check that rides on it)")
    ap.add_argument("--no-variants", action="store_true",
                    help="skip the single-launch timings of the attention entry point's other kernels")
    ap.add_argument("--no-peaks", action="store_true",
                    help="skip the probes of what this box sustains (pure MFMA loops, plain copy)")
    ap.add_argument("--cpu-frames", type=int, default=96,
                    help="frames of the sub-sequence the CPU oracle is timed on")
    return ap.parse_args()


class HipEvents:
    """hipEvent_t handles created through the HIP runtime the library itself is linked to."""

    def __init__(self, lib, n):
        self.lib = lib
        lib.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        lib.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        lib.hipEventDestroy.argtypes = [C.c_void_p]
        self.arr = (C.c_void_p * n)()
        for i in range(n):
            ev = C.c_void_p()
            assert lib.hipEventCreate(C.byref(ev)) == 0
            self.arr[i] = ev

    def ms(self, a, b):
        out = C.c_float()
        rc = self.lib.hipEventElapsedTime(C.byref(out), self.arr[a], self.arr[b])
        assert rc == 0, f"hipEventElapsedTime rc={rc}"
        return out.value

    def close(self):
        for ev in self.arr:
            self.lib.hipEventDestroy(ev)


CALIBRATION_COPY_BYTES = 256 << 20     # read once and written once by one elementwise kernel


def measured_traffic(workload, dtype, kernel):
    """HBM bytes per launch of `kernel` from the committed counter summary of this workload
    (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by the calibration copy).  The counters
    cannot be read inside an unprofiled run, so the line names the file and its hash; a summary
    made for another kernel gives (None, source)."""
    import hashlib
    rel = os.path.join("profiles", f"attn_{dtype}_{workload}_hbm_traffic.txt")
    try:
        text = open(os.path.join(ROOT, rel)).read()
    except OSError:
        return None, None
    src = {"file": rel, "sha256_16": hashlib.sha256(text.encode()).hexdigest()[:16],
           "how": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this program, not measured in this run"}
    value = None
    for line in text.splitlines():
        if line.startswith("traffic_bytes_per_launch"):
            value = float(line.split("=")[1].split()[0])
    if f"traffic_kernel = {kernel}" not in text:
        return None, dict(src, note=f"the summary was not made for {kernel}")
    return value, src


def cpu_baseline(wl, pl_full, n_frames, qk_norm, attn_dtype, B, torch):
    """Time the oracle on the first n_frames of the workload, one layer with a refresh, and
    scale each step to the full sequence by its operation count.  The same sub-sequence then
    goes through the HIP path (one driver layer, outside any timed region) and the two results
    are compared: `parity`."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from helpers import oracle_params
    from oracle import litevggt_oracle as O
    from paper_2512_04939_amd import synth

    sub = synth.Workload(**{**wl.__dict__, "frames": n_frames})
    gen = synth.Generator(wl)                     # same canvases/offsets as the full workload
    bits = gen.tokens(range(n_frames))
    if bits.dtype != np.uint16:
        bits = synth.f32_to_bf16_bits(bits)
    x = synth.bf16_bits_to_f32(bits)
    im = gen.images(range(n_frames))
    po = oracle_params(sub, qk_norm=bool(qk_norm))
    pls = O.plan(po)
    t = {}
    t0 = time.perf_counter()
    score, psi_g = O.importance(im, x, po)
    t["importance"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    sel = O.select_anchors(score.astype(np.float32), po)
    t["select"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    mt = O.match(x, sel["dst_idx"], sel["src_idx"])
    idx = O.build_index(sel["role"], sel["src_idx"], mt["anchor"])
    t["match"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    z = O.merge(x, idx["group_off"], idx["group_mem"])
    t["merge"] = time.perf_counter() - t0
    zz = z.reshape(z.shape[0], po.heads, po.head_dim)
    t0 = time.perf_counter()
    qk = O.qk_normalize(zz) if qk_norm else zz
    y = O.attention(qk, qk, zz).reshape(z.shape)
    t["attn"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    ref_out = O.unmerge(y, idx["slot_of"], residual=x)
    t["unmerge"] = time.perf_counter() - t0
    fr = wl.frames / n_frames
    scale = dict(importance=fr, select=fr,
                 match=(pl_full.n_src * pl_full.n_dst) / max(pls["n_src"] * pls["n_dst"], 1),
                 merge=pl_full.N / pls["N"], unmerge=pl_full.N / pls["N"],
                 attn=(pl_full.M / pls["M"]) ** 2)
    refreshes = sum(O.refresh_schedule(wl.layers, wl.refresh_interval))
    full = (refreshes * sum(t[k] * scale[k] for k in ("importance", "select", "match"))
            + wl.layers * sum(t[k] * scale[k] for k in ("merge", "attn", "unmerge")))
    threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])

    # the HIP path on the same sub-sequence, against what the oracle just computed
    ph = B.make_params(sub.frames, sub.grid_h, sub.grid_w, sub.dim, sub.heads, n_special=sub.n_special,
                       patch=sub.patch, merge_ratio=sub.merge_ratio, refresh_interval=sub.refresh_interval,
                       qk_norm=int(bool(qk_norm)), attn_dtype=attn_dtype)
    pl = B.litevggt_plan(ph)
    x_dev = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    ib = B.alloc_index(pl)
    g_dev = torch.zeros(sub.frames, sub.patches, device="cuda")
    s_dev = torch.zeros(sub.frames, sub.patches, device="cuda")
    B.litevggt_layers_run(ph, 1, torch.from_numpy(im).cuda(), x_dev, ib, g_dev, s_dev, B.alloc_ws(pl.ws_bytes))
    torch.cuda.synchronize()
    got = x_dev.float().cpu().numpy().astype(np.float64)
    roles_differ = int((ib.role.cpu().numpy() != sel["role"]).sum())
    src = sel["src_idx"].astype(np.int64)
    a_hip = ib.anchor_of.cpu().numpy().astype(np.int64)[src]
    differ = a_hip != idx["anchor_of"][src]
    gap = mt["best"] - mt["second"]
    same_rows = np.ones(pls["N"], dtype=bool)      # rows whose merge group has the same members
    if differ.any() or roles_differ:
        a_all, r_all = ib.anchor_of.cpu().numpy().astype(np.int64), idx["anchor_of"].astype(np.int64)
        touched = np.union1d(a_all[a_all != r_all], r_all[a_all != r_all])
        same_rows = (a_all == r_all) & ~np.isin(r_all, touched)
    err = float(np.abs(got - ref_out)[same_rows].max() / np.abs(ref_out).max())
    parity = dict(sample=f"first {n_frames} frames: one refresh + one layer of the driver against the oracle "
                         f"(float64, unrounded), N={pls['N']}, M={pls['M']}",
                  score_max_abs_err=float(np.abs(s_dev.cpu().numpy().astype(np.float64) - score).max()),
                  roles_differ=roles_differ,
                  src_tokens=int(len(src)), anchors_differ=int(differ.sum()),
                  anchors_differ_documented_near_ties=int((differ & (gap < 1e-6)).sum()),
                  oracle_near_ties=int((gap < 1e-6).sum()),
                  layer_max_rel_err=err, rows_compared=int(same_rows.sum()),
                  tolerance=2e-2 if attn_dtype == B.ATTN_BF16 else 6e-2)
    parity["ok"] = bool(parity["anchors_differ"] == parity["anchors_differ_documented_near_ties"]
                        and err <= parity["tolerance"] and parity["score_max_abs_err"] <= 2e-5)
    return dict(value=pl_full.N / full, unit="tokens/s", cores=int(threads), os_cpu_count=os.cpu_count(),
                kind="oracle",
                sample=(f"oracle timed on the first {n_frames} of {wl.frames} frames "
                        f"(N={pls['N']}, M={pls['M']}), one refresh + one layer"
                        f"{' with q, k normalised' if qk_norm else ''}, "
                        f"{sum(t.values()):.1f} s measured; each step scaled to the full "
                        f"sequence by its operation count (extrapolated step: {full:.0f} s)"),
                measured_s={k: round(v, 3) for k, v in t.items()}), parity


def sustained_peaks(B, torch):
    """What this machine gives the simplest possible kernels (the library's probes): loops of
    independent MFMAs on data loaded once, a plain 16-byte-per-lane copy and read of 2 GiB.
    Run after the timed steps; context for the fractions of the published peaks."""
    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / reps
    out = torch.empty(2048 * 512, dtype=torch.float32, device="cuda")
    g = torch.Generator(device="cuda").manual_seed(1)
    vals = torch.randn(65536, device="cuda", generator=g)
    res = {}
    for name, dt, ops, iters in (("mfma_bf16_tflops", B.ATTN_BF16, vals.to(torch.bfloat16), 40000),
                                 ("mfma_fp8_tflops", B.ATTN_FP8_E4M3,
                                  torch.cat([vals, vals.flip(0)]).to(torch.float8_e4m3fn), 20000)):
        assert ops.numel() * ops.element_size() == 128 * 1024
        t = timed(lambda: B.litevggt_probe_mfma(dt, ops, iters, out), 2)
        res[name] = B.litevggt_probe_mfma_flop(dt, iters) / t / 1e12
    nbytes = 2 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").random_(0, 256, generator=g)
    dst = torch.empty_like(src)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    res["copy_gbs"] = 2 * nbytes / timed(lambda: B.litevggt_probe_stream(src, dst, nbytes, sink), 10) / 1e9
    res["read_gbs"] = nbytes / timed(lambda: B.litevggt_probe_stream(src, None, nbytes, sink), 10) / 1e9
    # 2 KB rows (one token at dim 1024) read in a random order: the merge step's access pattern
    n_rows = nbytes // 2048
    order = torch.randperm(n_rows, device="cuda", generator=g).to(torch.int32)
    res["gather_2kb_rows_gbs"] = nbytes / timed(lambda: B.litevggt_probe_gather(src, 2048, order, n_rows, sink), 10) / 1e9
    res["note"] = ("litevggt_probe_mfma / litevggt_probe_stream: 2048 x 8 waves of independent 32x32 MFMAs on "
                   "operands loaded once; copy = bytes read + written of a 2 GiB buffer")
    return res


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only; --gpus N with N > 1 is not "
              "supported (no collectives are part of it).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2512_04939_amd import binding as B
    from paper_2512_04939_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    lib = B.lib()

    over = {} if args.merge_ratio is None else dict(merge_ratio=args.merge_ratio)
    if args.refresh_interval is not None:
        over["refresh_interval"] = args.refresh_interval
    wl = synth.workload(args.workload, **over)
    attn_dtype = B.ATTN_BF16 if args.attn_dtype == "bf16" else B.ATTN_FP8_E4M3
    bw = None
    if args.block:
        w_host = synth.block_weights(wl.dim, seed=wl.seed)
        w_dev = {k: (torch.from_numpy(synth.f32_to_bf16_bits(v).view(np.int16)).cuda().view(torch.bfloat16)
                     if v.ndim == 2 else torch.from_numpy(v).cuda()) for k, v in w_host.items()}
        fp8_state = torch.zeros(B.FP8_STATE_BYTES, dtype=torch.uint8, device="cuda")
        bw = B.block_weights(w_dev, linear_dtype=B.LINEAR_BF16 if args.linear_dtype == "bf16" else B.LINEAR_FP8_E4M3,
                             fp8_recipe=B.FP8_DELAYED if args.linear_dtype == "fp8-delayed" else B.FP8_CURRENT,
                             fp8_state=fp8_state)
    ph = B.make_params(wl.frames, wl.grid_h, wl.grid_w, wl.dim, wl.heads, n_special=wl.n_special,
                       patch=wl.patch, merge_ratio=wl.merge_ratio,
                       refresh_interval=wl.refresh_interval, qk_norm=args.qk_norm, attn_dtype=attn_dtype,
                       anchor_policy=dict(ga=B.POLICY_GA, fixed=B.POLICY_FIXED,
                                          random=B.POLICY_RANDOM)[args.anchor_policy],
                       frame_attn=1 if args.frame_attn else 0, block=bw)
    wl_qk_norm = bool(ph.qk_norm)
    pl = B.litevggt_plan(ph)
    L, C_ = wl.layers, wl.dim

    t0 = time.perf_counter()
    gen = synth.Generator(wl)
    bits = gen.tokens(threads=min(16, os.cpu_count() or 1))
    if bits.dtype != np.uint16:
        bits = synth.f32_to_bf16_bits(bits)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    x0 = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    torch.cuda.synchronize()
    h2d_s = time.perf_counter() - t1       # pageable host memory -> HBM, not part of `value`
    h2d_bytes = bits.nbytes
    del bits
    im = torch.empty(wl.frames, 3, wl.img_h, wl.img_w, dtype=torch.float32, device="cuda")
    for f0 in range(0, wl.frames, 50):
        fr = range(f0, min(wl.frames, f0 + 50))
        host = torch.from_numpy(gen.images(fr))
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        im[f0:f0 + len(fr)].copy_(host)
        torch.cuda.synchronize()
        h2d_s += time.perf_counter() - t1
        h2d_bytes += host.numel() * 4
    gen_s = time.perf_counter() - t0

    # a plain copy of known size: the kernel the HBM counters of a profiler run are scaled by
    cal = torch.ones(CALIBRATION_COPY_BYTES // 4, dtype=torch.float32, device="cuda")
    cal_out = torch.mul(cal, 1.0)
    torch.cuda.synchronize()
    del cal, cal_out

    x = torch.empty_like(x0)
    ib = B.alloc_index(pl)
    grad = torch.zeros(wl.frames, wl.patches, device="cuda")
    score = torch.zeros(wl.frames, wl.patches, device="cuda")
    ws = B.alloc_ws(pl.ws_bytes)
    n_ev = B.EVENTS_PER_LAYER * L
    evs = [HipEvents(lib, n_ev) for _ in range(args.steps)]

    for _ in range(args.warmup):
        x.copy_(x0)
        B.litevggt_layers_run(ph, L, im, x, ib, grad, score, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        x.copy_(x0)                      # restore the input (0.03 % of a step at 1000 frames)
        log = B.litevggt_layers_run(ph, L, im, x, ib, grad, score, ws, events=evs[k].arr)
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t0
    ms_step = 1e3 * total_s / args.steps
    finite = bool(torch.isfinite(x.float()).all().item())

    graph_ms = None
    if args.graph:      # the driver only enqueues kernels, so a step can be captured and replayed
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                x.copy_(x0)
                B.litevggt_layers_run(ph, L, im, x, ib, grad, score, ws)
        torch.cuda.current_stream().wait_stream(side)
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = 1e3 * (time.perf_counter() - t0) / args.steps

    # per-step durations from the driver's events
    E = B.EVENTS_PER_LAYER
    names = {"importance": (B.EV_LAYER_BEGIN, B.EV_IMPORTANCE_END),
             "select": (B.EV_IMPORTANCE_END, B.EV_SELECT_END),
             "match": (B.EV_SELECT_END, B.EV_MATCH_END),
             "merge": (B.EV_MATCH_END, B.EV_MERGE_END),
             "attn_pack": (B.EV_MERGE_END, B.EV_ATTN_PACK_END),
             "attn": (B.EV_ATTN_PACK_END, B.EV_ATTN_END),
             "block_rest": (B.EV_ATTN_END, B.EV_BLOCK_END),
             "unmerge": (B.EV_BLOCK_END, B.EV_UNMERGE_END),
             "frame_attn": (B.EV_UNMERGE_END, B.EV_FRAME_ATTN_END)}
    dur = {k: [] for k in names}
    imp_by_layer = []
    for ev in evs:
        for l in range(L):
            for k, (a, b) in names.items():
                if k in ("importance", "select", "match") and not log[l]:
                    continue
                dur[k].append(ev.ms(l * E + a, l * E + b))
                if k == "importance":
                    imp_by_layer.append((dur[k][-1], l))
    avg = {k: (sum(v) / len(v) if v else 0.0) for k, v in dur.items()}
    # each step on the device's clock: first to last event of its driver call
    last_ev = (L - 1) * E + B.EV_FRAME_ATTN_END
    step_ms = sorted(ev.ms(B.EV_LAYER_BEGIN, last_ev) for ev in evs)
    step_median = step_ms[len(step_ms) // 2] if len(step_ms) % 2 else 0.5 * (step_ms[len(step_ms) // 2 - 1] + step_ms[len(step_ms) // 2])
    for ev in evs:
        ev.close()

    N, M = pl.N, pl.M
    peak_tf = PEAK_BF16_MFMA_TFLOPS if args.attn_dtype == "bf16" else PEAK_FP8_MFMA_TFLOPS
    attn_flop = 4.0 * M * M * C_
    attn_tf = attn_flop / (avg["attn"] * 1e-3) / 1e12
    match_flop = 2.0 * pl.n_src * pl.n_dst * C_
    merge_bytes = (N + M) * C_ * 2 + 4 * (N + M)
    unmerge_bytes = (M + 2 * N) * C_ * 2 + 4 * N
    ops = {
        "attn": dict(ms=avg["attn"], tflops=attn_tf, frac_mfma=attn_tf / peak_tf),
        "attn_pack": dict(ms=avg["attn_pack"]),
        "match": dict(ms=avg["match"],
                      tflops=(match_flop / (avg["match"] * 1e-3) / 1e12) if avg["match"] else 0.0),
        "merge": dict(ms=avg["merge"], gbs=merge_bytes / (avg["merge"] * 1e-3) / 1e9),
        "unmerge": dict(ms=avg["unmerge"], gbs=unmerge_bytes / (avg["unmerge"] * 1e-3) / 1e9),
        "importance": dict(ms=avg["importance"]),
        "select": dict(ms=avg["select"], note="per refresh: per-frame cell arg-mins and rank counting, latency-bound (5.5 MB in)"),
    }
    if args.anchor_policy == "ga":
        # refreshes after the first read the cached gradient map: x patch rows once + three maps
        imp_first = [ev_ms for ev_ms, l in imp_by_layer if l == 0]
        imp_cached = [ev_ms for ev_ms, l in imp_by_layer if l != 0]
        imp_bytes = wl.frames * wl.patches * (C_ * 2 + 3 * 4)
        if imp_first:
            ops["importance"]["ms_first_refresh_with_grad_map"] = sum(imp_first) / len(imp_first)
        if imp_cached:
            ms_c = sum(imp_cached) / len(imp_cached)
            ops["importance"].update(ms_cached_grad=ms_c, gbs=imp_bytes / (ms_c * 1e-3) / 1e9,
                                     frac_hbm=imp_bytes / (ms_c * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                     note="gbs / frac_hbm: variance map + fusion of the refreshes that reuse the "
                                          "cached gradient map, bytes = patch rows of x once + the three maps")
    if args.block:
        blk_flop = 2.0 * M * C_ * (3 * C_ + C_ + 4 * C_ + 4 * C_)
        ops["block_linear"] = dict(ms=avg["attn_pack"] + avg["block_rest"],
                                   tflops=blk_flop / ((avg["attn_pack"] + avg["block_rest"]) * 1e-3) / 1e12,
                                   frac_mfma=blk_flop / ((avg["attn_pack"] + avg["block_rest"]) * 1e-3) / 1e12
                                   / (PEAK_FP8_MFMA_TFLOPS if args.linear_dtype.startswith("fp8") else PEAK_BF16_MFMA_TFLOPS),
                                   note="everything of the block except the attention kernel: 2 LayerNorms, "
                                        "4 linear layers (24 M C^2 flop), operand re-layouts (FP8: amax and "
                                        "quantisation passes), K/V re-layout")
    if args.frame_attn:
        fa_flop = 4.0 * wl.frames * wl.tokens_per_frame ** 2 * C_
        ops["frame_attn"] = dict(ms=avg["frame_attn"], tflops=fa_flop / (avg["frame_attn"] * 1e-3) / 1e12,
                                 frac_mfma=fa_flop / (avg["frame_attn"] * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS,
                                 note="pack + kernel, F independent sequences of P + 5 tokens")
    ops["match"]["frac_mfma"] = ops["match"]["tflops"] / PEAK_BF16_MFMA_TFLOPS
    ops["merge"]["frac_hbm"] = ops["merge"]["gbs"] / PEAK_HBM_GBS
    ops["unmerge"]["frac_hbm"] = ops["unmerge"]["gbs"] / PEAK_HBM_GBS

    unmerged = None
    if not args.no_unmerged:
        need = B.litevggt_attn_ws_bytes(ph, N)
        ws_u = B.alloc_ws(need)
        o = torch.empty_like(x0)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        B.litevggt_global_attn(ph, N, x0, x0, x0, o, ws_u)
        b.record()
        torch.cuda.synchronize()
        u_ms = a.elapsed_time(b)
        unmerged = dict(ms_per_layer=u_ms, tflops=4.0 * N * N * C_ / (u_ms * 1e-3) / 1e12,
                        ms_stack_extrapolated=u_ms * L,
                        note="one launch of the same attention entry point on the unmerged "
                             "sequence (n_tokens = N, q = k = v = x), times the layer count")
        del ws_u, o

    # single launches of the attention entry point's other kernels at the merged length, on the
    # first layer's merged tokens (index of the input features), timed around the call
    variants = None
    if not args.no_variants and not args.block:
        B.litevggt_importance(ph, im, x0, grad, True, score, ws)
        B.litevggt_select_anchors(ph, score, ib)
        B.litevggt_match(ph, x0, ib, None, ws)
        zv = torch.empty(M, C_, dtype=torch.bfloat16, device="cuda")
        yv = torch.empty_like(zv)
        B.litevggt_merge(ph, x0, ib, zv)

        def launch_ms(p, reps=3, q=None):
            q = zv if q is None else q
            wsv = B.alloc_ws(B.litevggt_attn_ws_bytes(p, M))
            B.litevggt_global_attn(p, M, q, zv, zv, yv, wsv)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                B.litevggt_global_attn(p, M, q, zv, zv, yv, wsv)
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps

        def mk(**kw):
            base = dict(n_special=wl.n_special, patch=wl.patch, merge_ratio=wl.merge_ratio,
                        refresh_interval=wl.refresh_interval, qk_norm=1, attn_dtype=B.ATTN_BF16)
            base.update(kw)
            return B.make_params(wl.frames, wl.grid_h, wl.grid_w, wl.dim, wl.heads, **base)

        variants = {"note": "one litevggt_global_attn call (K/V re-layout + kernels) at M merged tokens of the first "
                            "layer, averaged over 3 calls; frac = 4 M^2 C flop / call time / peak, so the re-layout "
                            "(ops.attn_pack) is inside"}
        for key, p_v, peak_v, what in (
                ("bf16_qk_norm", mk(), PEAK_BF16_MFMA_TFLOPS, "k_attn_bf16_main<false, false>: fixed reference (unit-RMS q, k)"),
                ("bf16_as_given", mk(qk_norm=0), PEAK_BF16_MFMA_TFLOPS,
                 "k_attn_bf16_main<true, false> (online softmax, per-wave running reference raised lazily), then the gated per-row kernel"),
                ("bf16_online_softmax", mk(softmax_scale=0.7), PEAK_BF16_MFMA_TFLOPS,
                 "k_attn_bf16_main<true, false> on normalised q, k with a softmax scale of 0.7 (beyond the fixed "
                 "reference's exponent range), then the gated per-row kernel"),
                ("fp8_qk_norm", mk(attn_dtype=B.ATTN_FP8_E4M3), PEAK_FP8_MFMA_TFLOPS, "k_attn_fp8_bounded"),
                ("fp8_as_given", mk(attn_dtype=B.ATTN_FP8_E4M3, qk_norm=0), PEAK_FP8_MFMA_TFLOPS,
                 "k_attn_fp8: running maximum")):
            ms_v = launch_ms(p_v)
            variants[key] = dict(kernel=what, ms_call=ms_v, tflops=attn_flop / (ms_v * 1e-3) / 1e12,
                                 frac_mfma=attn_flop / (ms_v * 1e-3) / 1e12 / peak_v)
        # the same kernel and launch as bf16_qk_norm with an all-zero q: an identical instruction
        # stream whose score MFMAs and exponentials toggle no operand bits.  Whatever it gains is
        # clock (power), not work
        zq = torch.zeros_like(zv)
        ms_v = launch_ms(mk(), q=zq)
        variants["bf16_qk_norm_zero_q"] = dict(
            kernel="k_attn_bf16_main<false, false> with q = 0 (same instructions, operands that toggle no bits): "
                   "how much of the kernel's time is the clock the chip holds under this kernel's power draw",
            ms_call=ms_v, tflops=attn_flop / (ms_v * 1e-3) / 1e12,
            frac_mfma=attn_flop / (ms_v * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS)
        del zv, yv, zq
        # the whole stack with the other setting of qk_norm (one step, not part of `value`): with
        # q = k = v = the merged tokens as given, the residual stream doubles per layer and from
        # the third layer on every score lies beyond the range the folded softmax scale resolves,
        # so those layers run the online pass (which flags its blocks after the first key tile)
        # and then the per-row kernel
        p_other = mk(qk_norm=0 if wl_qk_norm else 1, attn_dtype=attn_dtype)
        x.copy_(x0)
        B.litevggt_layers_run(p_other, L, im, x, ib, grad, score, ws)
        torch.cuda.synchronize()
        ev_o = HipEvents(lib, n_ev)
        x.copy_(x0)
        t0 = time.perf_counter()
        B.litevggt_layers_run(p_other, L, im, x, ib, grad, score, ws, events=ev_o.arr)
        torch.cuda.synchronize()
        other_ms = 1e3 * (time.perf_counter() - t0)
        per_layer = [ev_o.ms(l * E + B.EV_ATTN_PACK_END, l * E + B.EV_ATTN_END) for l in range(L)]
        ev_o.close()
        variants["stack_with_qk_norm_%d" % (0 if wl_qk_norm else 1)] = dict(
            ms_per_step=other_ms, tokens_per_s=N / (other_ms * 1e-3),
            attn_ms_first_layers=[round(v, 2) for v in per_layer[:4]], attn_ms_last_layer=round(per_layer[-1], 2),
            output_finite=bool(torch.isfinite(x.float()).all().item()))

    roof_kernel = ("k_attn_fp8_bounded" if args.attn_dtype == "fp8" and wl_qk_norm else "k_attn_fp8" if args.attn_dtype == "fp8"
                   else "k_attn_bf16_main<false, false>" if wl_qk_norm else "k_attn_bf16_main<true, false>")
    traffic, traffic_src = measured_traffic(wl.name, args.attn_dtype, roof_kernel)
    out = {
        "metric": "merged global-attn tokens/s @%d frames" % wl.frames,
        "value": N / (ms_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.attn_dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.frames} frames x {wl.tokens_per_frame} tokens "
                               f"(N={N}), dim {C_}, {wl.heads} heads x 64, merge ratio "
                               f"{wl.merge_ratio} (M={M}), {L} global layers, index refreshed "
                               f"every {wl.refresh_interval}",
                   "token_layers_per_s": L * N / (ms_step * 1e-3),
                   "qk_norm": bool(args.qk_norm), "anchor_policy": args.anchor_policy, "frame_attn": bool(args.frame_attn), "block": bool(args.block),
                   "linear_dtype": args.linear_dtype if args.block else None,
                   "refresh_log": log, "output_finite": finite,
                   "graph_replay_ms_per_step": graph_ms,
                   "peak_hbm_alloc_gib": torch.cuda.max_memory_allocated() / 2 ** 30,
                   "input_generation_s": gen_s,
                   "h2d_upload_s": h2d_s, "h2d_upload_gbs": h2d_bytes / h2d_s / 1e9,
                   "tokens_per_s_with_upload": N / (ms_step * 1e-3 + h2d_s),
                   "calibration_copy_bytes": CALIBRATION_COPY_BYTES,
                   "device_ms_per_step_median": step_median, "device_ms_per_step_min": step_ms[0],
                   "device_ms_per_step_max": step_ms[-1]},
        "roofline": {"kernel": roof_kernel, "bound": "mfma", "achieved": attn_tf, "peak": peak_tf,
                     "unit": "TFLOP/s", "frac": attn_tf / peak_tf,
                     "traffic": traffic, "traffic_source": traffic_src,
                     "flop_per_launch": attn_flop, "avg_launch_ms": avg["attn"],
                     "launches_timed": len(dur["attn"])},
        "ops": ops,
        "attn_variants": variants,
        "unmerged_attention": unmerged,
    }
    if unmerged:
        out["speedup_vs_unmerged_stack"] = unmerged["ms_stack_extrapolated"] / ms_step
    if not args.no_peaks:
        out["sustained_peaks"] = sustained_peaks(B, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"], out["parity"] = cpu_baseline(wl, pl, min(args.cpu_frames, wl.frames), args.qk_norm,
                                                          attn_dtype, B, torch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
