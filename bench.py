"""Benchmark of the FNO block on one MI355X.

A step is one pass of the whole hot path (fno_block_fwd through the C ABI: forward pruned
transforms, mode mix, inverse transforms, fused W x + b + GELU epilogue) over one batch of
synthetic input resident in HBM.  Prints ONE JSON line with the throughput in
Gpoint-channels/s, the roofline of the dominant kernel (timed live with HIP events on the
launch stream) and the float64 CPU oracle timed on a bounded sample as a baseline.
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


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg4", help="workload name from synth.CONFIGS (block forward; cfg5: forward + backward), or time_lift, time_lift_bwd")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--forward-only", action="store_true",
                    help="with --network: the forward pass alone (lift, blocks, projection), nothing saved")
    ap.add_argument("--network", action="store_true",
                    help="time one training step of the whole network of the workload (cfg3: lift, blocks, "
                         "projection, relative L2 loss, backward, Adam) instead of one block")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run plain device copies of 4 GiB (reference reading for rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE), then exit")
    ap.add_argument("--traffic-file", default=os.path.join(ROOT, "profiles", "hbm_traffic.json.txt"),
                    help="measured HBM bytes per launch of the dominant kernel (from rocprofv3 --pmc)")
    return ap.parse_args()


def cpu_baseline(cfg):
    """The oracle as it stands on a bounded sample: a width-1 block on one channel slab of the grid."""
    import numpy as np
    from oracle import fno_oracle as O
    from paper_2204_01205_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    grid = tuple(cfg["grid"])
    spec = O.LayerSpec(grid, tuple(cfg["modes"]), 0)
    counts = tuple(len(k) for k in O.mode_lists(spec))
    x = synth.normal_field(0, synth.T_X, 1, 1, grid)
    R = synth.spectral_weights(0, 1, 1, counts)
    W = synth.linear_weights(0, 1, 1)
    b = synth.bias(0, 1)
    t0 = time.perf_counter()
    O.block_fwd(x, R, W, b, spec)
    dt = time.perf_counter() - t0
    pc = float(np.prod(grid))
    return {"value": pc / dt / 1e9, "unit": "Gpoint-channels/s", "cores": int(threads), "kind": "oracle",
            "sample": f"float64 oracle block_fwd, width 1 (one of the workload's channel slabs), grid "
                      f"{grid[0]}x{grid[1]}x{grid[2]}x{grid[3]}, modes as the workload; {dt:.1f} s",
            "host_cores_visible": len(os.sched_getaffinity(0))}


def time_lift_bench(args, torch, B, adjoint=False):
    """The fused input lifts (fno_time_lift), or their adjoint with respect to the parameters
    (fno_time_lift_bwd), at the largest grid: 2 -> 20 channels, 1 -> 32 time steps."""
    grid, nt, c_in, c_out = (256, 256, 128), 32, 2, 20
    ns = grid[0] * grid[1] * grid[2]
    torch.cuda.set_device(0)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0)
    a = torch.randn((1, c_in, ns), device="cuda", generator=gen)
    wt = torch.randn(nt, device="cuda", generator=gen)
    bt = torch.randn(nt, device="cuda", generator=gen)
    wc = torch.randn((c_out, c_in), device="cuda", generator=gen)
    bc = torch.randn(c_out, device="cuda", generator=gen)
    out = torch.empty((1, c_out, ns, nt), device="cuda")

    if adjoint:
        out.normal_(generator=gen)               # plays the cotangent of the lifted tensor
        ws = torch.empty(B.fno_time_lift_bwd_workspace_bytes(c_in, c_out, nt) // 4 + 2, dtype=torch.float32,
                         device="cuda")
        gwt, gbt = torch.empty_like(wt), torch.empty_like(bt)
        gwc, gbc = torch.empty_like(wc), torch.empty_like(bc)

    def step():
        if adjoint:
            B.fno_time_lift_bwd(1, c_in, c_out, ns, nt, a, wt, bt, wc, out, gwt, gbt, gwc, gbc, ws)
        else:
            B.fno_time_lift(1, c_in, c_out, ns, nt, a, wt, bt, wc, bc, out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()                      # the launches go to torch's current stream, which these events see
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = 1e3 * dt / args.steps
    launch_ms = e0.elapsed_time(e1) / args.steps
    pc = float(c_out) * ns * nt
    nbytes = 4.0 * pc + 4.0 * c_in * ns          # lifted tensor written (adjoint: its cotangent read) once, input read once
    name = "time_lift_bwd" if adjoint else "time_lift"
    print(json.dumps({
        "metric": "FNO spectral layer Gpoint-channels/s + achieved HBM GB/s on 1 MI355X",
        "value": pc / (ms * 1e-3) / 1e9, "unit": "Gpoint-channels/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{name}: fno_{name}, batch 1, {c_in} -> {c_out} channels, grid "
                               f"{grid[0]}x{grid[1]}x{grid[2]}, 1 -> {nt} time steps",
                   "global_batch": 1, "parallelism": "single GPU"},
        "roofline": {"kernel": name, "bound": "hbm", "achieved": nbytes / (launch_ms * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": nbytes / (launch_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "traffic": None, "avg_launch_ms": launch_ms, "algorithmic_bytes_per_launch": nbytes},
    }))


def network_step_bench(args, torch, B, synth):
    """One training step of a whole network: every stage through the C ABI, all tensors resident."""
    cfg = synth.CONFIGS[args.config]
    batch, width, grid, modes = cfg["batch"], cfg["width"], tuple(cfg["grid"]), tuple(cfg["modes"])
    c_in, hidden, nblocks = cfg.get("in_channels", 5), cfg.get("hidden", 128), cfg.get("blocks", 4)
    counts = B.kept_counts(B.make_desc(batch, width, width, grid, modes))
    npts = 1
    for n in grid:
        npts *= n
    torch.cuda.set_device(0)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0)
    rn = lambda *shape: torch.randn(shape, device="cuda", generator=gen)
    a, y = rn(batch, c_in, *grid), rn(batch, 1, *grid)
    lw, lb = rn(width, c_in) / c_in ** 0.5, 0.1 * rn(width)
    blocks = [(torch.view_as_complex(rn(width, width, *counts, 2) / width), rn(width, width) / width ** 0.5,
               0.1 * rn(width)) for _ in range(nblocks)]
    w1, b1, w2, b2 = rn(hidden, width) / width ** 0.5, 0.1 * rn(hidden), rn(1, hidden) / hidden ** 0.5, 0.1 * rn(1)
    desc = B.make_desc(batch, width, width, grid, modes, 0, B.FNO_ACT_GELU)
    ws = B.alloc_workspace(desc, B.FNO_OP_BLOCK_BWD)
    act = lambda: torch.empty((batch, width) + grid, device="cuda")
    vs = [act() for _ in range(nblocks + 1)]
    zs = [act() for _ in range(nblocks)]
    xhs = [torch.empty((batch, width) + counts, dtype=torch.complex64, device="cuda") for _ in range(nblocks)]
    u, gu = torch.empty_like(y), torch.empty_like(y)
    gva, gvb = act(), act()
    lws = torch.empty(B.fno_rel_l2_workspace_bytes() // 4, dtype=torch.float32, device="cuda")
    pws = torch.empty(max(B.fno_pointwise_bwd_workspace_bytes(width, hidden, 1),
                          B.fno_pointwise_bwd_workspace_bytes(c_in, 0, width)) // 4 + 2,
                      dtype=torch.float32, device="cuda")
    loss = torch.empty(1, device="cuda")
    params = [lw, lb, w1, b1, w2, b2] + [t for blk in blocks for t in blk]
    flat = [torch.view_as_real(p).reshape(-1) if p.is_complex() else p.reshape(-1) for p in params]
    grads = [torch.empty_like(p) for p in params]
    gflat = [torch.view_as_real(t).reshape(-1) if t.is_complex() else t.reshape(-1) for t in grads]
    moms = [(torch.zeros_like(f), torch.zeros_like(f)) for f in flat]
    glw, glb, gw1, gb1, gw2, gb2 = grads[:6]
    gblk = [tuple(grads[6 + 3 * k: 9 + 3 * k]) for k in range(nblocks)]
    state = {"step": 0}

    def forward():
        B.fno_pointwise_linear(batch, c_in, width, npts, a, lw, lb, vs[0])
        for k, (R, W, b) in enumerate(blocks):
            B.fno_block_fwd(desc, vs[k & 1], R, W, b, vs[(k + 1) & 1], None, None, ws)
        B.fno_pointwise_mlp2(batch, width, hidden, 1, npts, vs[nblocks & 1], w1, b1, w2, b2, u)

    def step():
        if args.forward_only:
            return forward()
        state["step"] += 1
        B.fno_pointwise_linear(batch, c_in, width, npts, a, lw, lb, vs[0])
        for k, (R, W, b) in enumerate(blocks):
            B.fno_block_fwd(desc, vs[k], R, W, b, vs[k + 1], zs[k], xhs[k], ws)
        B.fno_pointwise_mlp2(batch, width, hidden, 1, npts, vs[-1], w1, b1, w2, b2, u)
        B.fno_rel_l2_loss(u.numel(), u, y, loss, gu, lws)
        B.fno_pointwise_mlp2_bwd(batch, width, hidden, 1, npts, vs[-1], w1, b1, w2, gu, gva, gw1, gb1, gw2, gb2, pws)
        gin, gout = gva, gvb
        for k in reversed(range(nblocks)):
            R, W, b = blocks[k]
            B.fno_block_bwd(desc, vs[k], R, W, zs[k], xhs[k], gin, gout, gblk[k][0], gblk[k][1], gblk[k][2], ws)
            gin, gout = gout, gin
        B.fno_pointwise_linear_bwd(batch, c_in, width, npts, a, lw, gin, None, glw, glb, pws)
        for f, gf, (m, v) in zip(flat, gflat, moms):
            B.fno_adam_step(f.numel(), f, gf, m, v, 1e-3, 0.9, 0.999, 1e-8, state["step"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t0) / args.steps
    pc = float(batch) * width * npts
    print(json.dumps({
        "metric": "FNO spectral layer Gpoint-channels/s + achieved HBM GB/s on 1 MI355X",
        "value": nblocks * pc / (ms * 1e-3) / 1e9, "unit": "Gpoint-channels/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.config} network {'forward' if args.forward_only else 'training step'}: lift "
                               f"{c_in}->{width}, {nblocks} blocks, projection {width}->{hidden}->1"
                               f"{'' if args.forward_only else ', relative L2 loss, backward, Adam'}; batch {batch}, grid "
                               f"{grid[0]}x{grid[1]}x{grid[2]}x{grid[3]}; value counts the point-channels of the "
                               f"{nblocks} blocks once per step",
                   "global_batch": batch, "parallelism": "single GPU"},
        "loss": None if args.forward_only else float(loss.cpu()),
    }))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build covers one GPU's share of the work only; run with --gpus 1 "
              "(no collectives or sharding are built)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2204_01205_amd import binding as B
    from paper_2204_01205_amd import synth

    if args.calibrate_copy:
        torch.cuda.set_device(0)
        src = torch.ones(1 << 30, dtype=torch.float32, device="cuda")      # 4 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_each_way": 4 * (1 << 30), "copies": 3}))
        return
    if args.config in ("time_lift", "time_lift_bwd"):
        time_lift_bench(args, torch, B, adjoint=args.config == "time_lift_bwd")
        return
    if args.network:
        network_step_bench(args, torch, B, synth)
        return
    cfg = synth.CONFIGS[args.config]
    batch, width, grid, modes = cfg["batch"], cfg["width"], tuple(cfg["grid"]), tuple(cfg["modes"])
    counts = B.kept_counts(B.make_desc(batch, width, width, grid, modes))
    npts = 1
    for n in grid:
        npts *= n
    pc = batch * width * npts
    nmodes = counts[0] * counts[1] * counts[2] * counts[3]

    torch.cuda.set_device(0)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0)
    x = torch.randn((batch, width) + grid, device="cuda", generator=gen)
    R = torch.view_as_complex(torch.randn((width, width) + counts + (2,), device="cuda", generator=gen)
                              / float(width))
    W = torch.randn((width, width), device="cuda", generator=gen) / float(width) ** 0.5
    b = 0.1 * torch.randn((width,), device="cuda", generator=gen)
    out = torch.empty_like(x)
    train = cfg["op"] == "block_fwd_bwd"
    if train:
        # one training step of a block: forward keeping z and the spectrum, backward with the
        # MSE gradient against a seeded target fused into its first sweep
        desc = B.make_desc(batch, width, width, grid, modes, 0, B.FNO_ACT_GELU, B.FNO_FLAG_MSE_TARGET)
        ws = B.alloc_workspace(desc, B.FNO_OP_BLOCK_BWD)
        target = torch.randn(x.shape, device="cuda", generator=gen)
        z = torch.empty_like(x)
        xh = torch.empty((batch, width) + counts, dtype=torch.complex64, device="cuda")
        gx = torch.empty_like(x)
        gR = torch.empty_like(R)
        gW = torch.empty_like(W)
        gb = torch.empty_like(b)

        def step():
            B.fno_block_fwd(desc, x, R, W, b, out, z, xh, ws)
            B.fno_block_bwd(desc, x, R, W, z, xh, target, gx, gR, gW, gb, ws)
    else:
        desc = B.make_desc(batch, width, width, grid, modes, 0, B.FNO_ACT_GELU)
        ws = B.alloc_workspace(desc, B.FNO_OP_BLOCK_FWD)

        def step():
            B.fno_block_fwd(desc, x, R, W, b, out, None, None, ws)

    # Warm-up: untimed, with an event pair around every stage; it gives the per-stage breakdown and
    # names the dominant stage.  (An event pair costs a few microseconds of idle time between two
    # kernels, 0.09 ms per step over all stages at cfg4, which is why the timed region below keeps
    # only the pair around the dominant stage.)
    B.fno_timing_enable(True)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    warm = B.fno_timing_read()
    B.fno_timing_enable(False)
    if args.warmup >= 2:                       # the first step carries first-call effects
        warm = warm[len(warm) // args.warmup:]
    nwarm = max(args.warmup - 1, 1) if args.warmup >= 2 else max(args.warmup, 1)
    stage_ms = {}
    for name, ms in warm:
        stage_ms.setdefault(name, []).append(ms)
    # per step: a stage that runs several times in a step (forward chain of x and of gz) is summed
    stage_avg = {k: sum(v) / nwarm for k, v in stage_ms.items()}
    dominant = max(stage_avg, key=stage_avg.get) if stage_avg else "zt_inv"

    # Timed region: exactly K steps; HIP events only around the dominant stage's launches, on the
    # stream they are launched on
    B.fno_timing_enable([dominant])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    records = B.fno_timing_read()
    B.fno_timing_enable(False)

    ms_per_step = 1e3 * dt / args.steps
    dom_ms = [ms for name, ms in records if name == dominant]
    stage_avg[dominant] = sum(dom_ms) / args.steps
    stage_launches = {dominant: len(dom_ms) / args.steps}
    # algorithmic bytes per launch of each full-grid sweep: 4 B per point-channel per tensor touched
    # zt_inv reads the tensor W acts on and writes the result (pruned spectrum not counted); in a
    # training step the forward launch also writes z, and the figure is the mean of its two launches
    alg_bytes = {"zt_inv": 10.0 * pc if train else 8.0 * pc,
                 "tz_fwd": 4.0 * pc,      # reads x
                 "bwd_pointwise": 16.0 * pc}   # reads z, target, x; writes gz
    dom_bytes = alg_bytes.get(dominant, 0.0)
    dom_launch_ms = stage_avg[dominant] / stage_launches[dominant]
    achieved = dom_bytes / (dom_launch_ms * 1e-3) / 1e9
    traffic = None
    if os.path.exists(args.traffic_file):
        try:
            tf = json.load(open(args.traffic_file))
            ent = tf.get(args.config, {}).get(dominant)
            if ent is not None:
                traffic = ent
        except Exception:
            traffic = None
    whole_bytes = (40.0 * pc + 24.0 * width * width * nmodes) if train else (12.0 * pc + 8.0 * width * width * nmodes)
    line = {
        "metric": "FNO spectral layer Gpoint-channels/s + achieved HBM GB/s on 1 MI355X",
        "value": pc / (ms_per_step * 1e-3) / 1e9,
        "unit": "Gpoint-channels/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.config}: {'fno_block_fwd + fno_block_bwd (MSE)' if train else 'fno_block_fwd'}, batch {batch}, width {width}, grid "
                               f"{grid[0]}x{grid[1]}x{grid[2]}x{grid[3]}, kept modes {counts[0]}x{counts[1]}x{counts[2]}x{counts[3]}",
                   "global_batch": batch, "parallelism": "single GPU"},
        "whole_path": {"algorithmic_GB": whole_bytes / 1e9,
                       "achieved_GBps": whole_bytes / (ms_per_step * 1e-3) / 1e9,
                       "frac_of_hbm_peak": whole_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "roofline": {"kernel": dominant, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "avg_launch_ms": dom_launch_ms, "algorithmic_bytes_per_launch": dom_bytes},
        "stage_ms": stage_avg,
        "stage_ms_note": "dominant stage: HIP events in the timed region; the others: from the warm-up steps",
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
