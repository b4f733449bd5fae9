#!/usr/bin/env python3
"""Benchmark of the CDQuant hot path on one MI355X.

One "step" = one pass of the whole path over one synthetic layer already resident in HBM:
    H = X^T X  ->  MinMax/RTN grid  ->  greedy coordinate descent (gradient init + T iterations)
    ->  layer loss.
Prints ONE JSON line.  `value` = committed coordinate updates per second of whole-step time.
Extra objects: `roofline` for the kernel that dominates the step, `cpu_baseline` for the CPU
oracle timed on a bounded sample of the same workload, `stages` with per-stage times.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config attn_proj] [--mode rtn|stress] [--init config|rtn|owc|owc_cd]
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


class HipEvents:
    """Raw HIP events on a given stream (timing of kernels launched by the library on it)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed: {rc}")
        return ev

    def record(self, ev, stream):
        rc = self.hip.hipEventRecord(ev, ctypes.c_void_p(stream))
        if rc != 0:
            raise RuntimeError(f"hipEventRecord failed: {rc}")

    def elapsed_ms(self, a, b):
        self.hip.hipEventSynchronize(b)
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(ms.value)


def load_traffic(kernel, workload):
    """HBM bytes per launch measured offline with rocprofv3 --pmc (see profiles/); None if absent."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(f"{kernel}:{workload}")
    except (OSError, ValueError):
        return None


def cpu_baseline(cfg, mode, init, budget_s=20.0):
    """The oracle, as it stands, on the host cores: Hessian on a token sample, RTN + CD + loss on a
    column sample, each extrapolated linearly to the full layer; updates/s of the whole step."""
    import numpy as np

    from oracle import cdq_oracle as oracle
    from paper_2406_17542_amd import inputs

    # all tokens when the fp64 product stays near 2e11 flop (the 2048-wide layers), else a prefix
    n_tok = int(min(cfg.n, max(512, 2e11 / (2.0 * cfg.d_in * cfg.d_in))))
    X = inputs.make_x(cfg.x_kind, n_tok, cfg.d_in, cfg.seed, cfg.x_dtype)
    t0 = time.perf_counter()
    H64 = oracle.hessian(X)
    t_h = (time.perf_counter() - t0) * (cfg.n / n_tok)
    H32 = H64.astype(np.float32)

    def run(cols):
        Wt = inputs.make_wt(cols, cfg.d_in, cfg.seed)
        t = time.perf_counter()
        if init == "owc" and mode != "stress":
            a, b, q, _, _ = oracle.init_owc(H32, Wt, cfg.bits, cfg.group, 50)
        elif init == "owc_cd" and mode != "stress":
            o = oracle.owc_cd(H32, Wt, cfg.bits, cfg.group, 50)
            a, b, q = o["scale"], o["zero"], o["Q"]
        else:
            a, b, q = oracle.init_grid(Wt, cfg.bits, cfg.group)
        if mode == "stress":
            q = inputs.make_random_codes(cols, cfg.d_in, cfg.bits, cfg.seed)
        r = oracle.greedy_cd(H32, Wt, a, b, q, cfg.bits, cfg.group, cfg.T)
        oracle.loss(H32, Wt, r["Q"], a, b, cfg.group)
        return time.perf_counter() - t, int(r["moves"].sum())

    probe_cols = min(cfg.d_out, 2 * oracle.n_threads())
    t_probe, _ = run(probe_cols)
    cols = int(min(cfg.d_out, max(probe_cols, probe_cols * budget_s / max(t_probe, 1e-3))))
    t_cols, moves = run(cols)
    scale = cfg.d_out / cols
    total_s = t_h + t_cols * scale
    return {
        "value": moves * scale / total_s, "unit": "updates/s", "cores": oracle.n_threads(), "kind": "oracle",
        "sample": f"Hessian on {n_tok} of {cfg.n} tokens (fp64 numpy), {init} init+CD+loss on the first {cols} of "
                  f"{cfg.d_out} columns for the full T={cfg.T}; times scaled linearly to the full layer "
                  f"(est. {total_s:.1f} s)",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="attn_proj")
    ap.add_argument("--mode", default="rtn", choices=["rtn", "stress"],
                    help="rtn: initial codes as the configuration says; stress: uniform random initial codes")
    ap.add_argument("--init", default="config", choices=["config", "rtn", "owc", "owc_cd"],
                    help="initial grid: the configuration's own, MinMax/RTN, OWC (Eq. 2 grid search) or OWC-CD (Algorithm 3)")
    ap.add_argument("--waves", type=int, default=0)
    ap.add_argument("--elems", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probes", action="store_true", help="skip the achievable-bandwidth probes")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the output columns are independent problems and would shard "
              "over GPUs with a replica of H and no communication during the loop) -- rerun with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2406_17542_amd import cdq, inputs

    cfg = inputs.CONFIGS[args.config]
    init = cfg.init if args.init == "config" else args.init
    if args.mode == "stress":
        init = "rtn"
    torch.cuda.set_device(0)
    ev = HipEvents()
    stream = torch.cuda.current_stream().cuda_stream

    X, Wt = inputs.make_layer(cfg)
    if cfg.x_dtype == "bf16":
        Xd = torch.from_numpy(inputs.bf16_bits(X).view(np.int16)).cuda().view(torch.bfloat16)
    else:
        Xd = torch.from_numpy(X).cuda()
    del X
    Wd = torch.from_numpy(Wt).cuda()
    q_stress = None
    if args.mode == "stress":
        q_stress = torch.from_numpy(inputs.make_random_codes(cfg.d_out, cfg.d_in, cfg.bits, cfg.seed)).cuda()

    H = torch.empty((cfg.d_in, cfg.d_in), dtype=torch.float32, device="cuda")
    ws_h = torch.empty(max(cdq.workspace_bytes(cdq.OP_HESSIAN, cfg.n, 0, cfg.d_in), 256), dtype=torch.uint8, device="cuda")
    ws_cd = torch.empty(max(cdq.workspace_bytes(cdq.OP_GREEDY_CD, 0, cfg.d_out, cfg.d_in), 256), dtype=torch.uint8, device="cuda")
    ws_l = torch.empty(max(cdq.workspace_bytes(cdq.OP_LOSS, 0, cfg.d_out, cfg.d_in), 256), dtype=torch.uint8, device="cuda")
    ws_owc = None
    if init == "owc":
        ws_owc = torch.empty(max(cdq.workspace_bytes(cdq.OP_INIT_OWC, 0, cfg.d_out, cfg.d_in), 256), dtype=torch.uint8, device="cuda")
    elif init == "owc_cd":
        ws_owc = torch.empty(max(cdq.workspace_bytes(cdq.OP_INIT_OWC_CD, 0, cfg.d_out, cfg.d_in), 256), dtype=torch.uint8, device="cuda")

    stage_names = ["hessian", "init_grid", "cd_gradient_init", "cd_loop", "loss"]
    n_ev = 7
    events = [[ev.create() for _ in range(n_ev)] for _ in range(args.steps)]
    state = {}

    def step(evs=None):
        rec = (lambda k: ev.record(evs[k], stream)) if evs is not None else (lambda k: None)
        rec(0)
        cdq.hessian(Xd, H=H, workspace=ws_h)
        rec(1)
        if init == "owc":
            scale, zero, Q, _, _ = cdq.init_owc(H, Wd, cfg.bits, cfg.group, 50, workspace=ws_owc, want_loss=False)
        elif init == "owc_cd":
            o = cdq.init_owc_cd(H, Wd, cfg.bits, cfg.group, 50, workspace=ws_owc)
            scale, zero, Q = o["scale"], o["zero"], o["Q"]
            state["owc_cd_moves"] = o["moves"]
        else:
            scale, zero, Q = cdq.init_rtn(Wd, cfg.bits, cfg.group)
        if q_stress is not None:
            Q.copy_(q_stress)
        rec(2)
        out = cdq.greedy_cd(H, Wd, scale, zero, Q, cfg.bits, cfg.group, cfg.T, workspace=ws_cd,
                            waves_per_column=args.waves, elems_per_lane=args.elems,
                            loop_events=(evs[3], evs[4]) if evs is not None else None)
        rec(5)
        per, tot = cdq.loss(H, Wd, scale, zero, Q, cfg.group, workspace=ws_l)
        rec(6)
        state.update(stats=out["stats"], loss=tot, Q=Q, scale=scale, zero=zero)

    # a copy of known size (256 MiB read + 256 MiB written): reference dispatch for scaling the
    # FETCH_SIZE / WRITE_SIZE counters when this command runs under rocprofv3 --pmc
    cal_src = torch.zeros(64 << 20, dtype=torch.float32, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    cdq.probe_copy(cal_src, cal_dst)
    torch.cuda.synchronize()
    del cal_dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    moves = int(state["stats"][:, 0].sum().item())
    converged = int(state["stats"][:, 2].sum().item())
    loss_final = float(state["loss"].item())

    # per-stage device time from the events: [0,1] hessian, [1,2] rtn, [2,3] gradient init (+diag),
    # [3,4] the iteration-loop kernel, [5,6] loss
    spans = {"hessian": (0, 1), "init_grid": (1, 2), "cd_gradient_init": (2, 3), "cd_loop": (3, 4), "loss": (5, 6)}
    stages = {}
    for name in stage_names:
        a, b = spans[name]
        stages[name] = sum(ev.elapsed_ms(events[k][a], events[k][b]) for k in range(args.steps)) / args.steps

    # roofline of each candidate for "dominant kernel"
    cd_bytes = moves * 4.0 * cfg.d_in                         # one H row (4*d_in bytes) per committed update
    cd_gbs = cd_bytes / (stages["cd_loop"] * 1e-3) * 1e-9
    flop_eff = 2.0 * cfg.n * cfg.d_in * cfg.d_in
    tile = 256 if cfg.x_dtype == "bf16" else 128                  # tile edge of the Hessian kernels
    n_t = (cfg.d_in + tile - 1) // tile
    flop_exec = 2.0 * cfg.n * (n_t * (n_t + 1) // 2) * tile * tile   # upper-triangular tiles only
    h_tflops_exec = flop_exec / (stages["hessian"] * 1e-3) * 1e-12
    h_tflops_eff = flop_eff / (stages["hessian"] * 1e-3) * 1e-12
    mfma_peak = MFMA_PEAK_TFLOPS[cfg.x_dtype]

    # achievable bandwidth on this machine, same process: streaming read from HBM, and the loop's
    # access pattern (independent random rows of H, same row length and team width) without its
    # arithmetic
    achievable = {}
    if not args.no_probes:
        sink = torch.zeros(4, dtype=torch.float32, device="cuda")
        big = torch.empty(1 << 30, dtype=torch.float32, device="cuda")       # 4 GiB
        big.zero_()
        e0, e1 = ev.create(), ev.create()
        cdq.probe_read(big, big.numel() * 4, sink)
        torch.cuda.synchronize()
        ev.record(e0, stream)
        for _ in range(5):
            cdq.probe_read(big, big.numel() * 4, sink)
        ev.record(e1, stream)
        achievable["hbm_stream_read_GBps"] = 5 * big.numel() * 4 / (ev.elapsed_ms(e0, e1) * 1e-3) * 1e-9
        del big
        # the same streaming read over a buffer that stays in the last-level cache (32 MiB, repeated)
        small = torch.zeros(8 << 20, dtype=torch.float32, device="cuda")
        cdq.probe_read(small, small.numel() * 4, sink)
        torch.cuda.synchronize()
        ev.record(e0, stream)
        for _ in range(200):
            cdq.probe_read(small, small.numel() * 4, sink)
        ev.record(e1, stream)
        achievable["cache_stream_read_GBps_32MiB"] = 200 * small.numel() * 4 / (ev.elapsed_ms(e0, e1) * 1e-3) * 1e-9
        del small
        # matrix cores alone (no memory traffic): what the GEMM kernels could reach at most on this machine, clock included
        for kind, key in ((0, "mfma_bf16_only_TFLOPs"), (1, "mfma_f64_only_TFLOPs")):
            cdq.probe_mfma(kind, 256 * 2, 200, sink)
            torch.cuda.synchronize()
            ev.record(e0, stream)
            flop = cdq.probe_mfma(kind, 256 * 2, 20000 if kind == 0 else 5000, sink)
            ev.record(e1, stream)
            achievable[key] = flop / (ev.elapsed_ms(e0, e1) * 1e-3) * 1e-12
        waves_used = args.waves
        if waves_used == 0:                     # mirrors the library's default: 16 coordinates per lane
            waves_used = 1
            while 64 * waves_used * 16 < cfg.d_in and waves_used < 16:
                waves_used *= 2
        teams = 256 * max(1, 16 // waves_used)
        row_bytes = 4 * cfg.d_in
        iters = max(50, int(2e11 / (teams * row_bytes)))
        cdq.probe_gather(H, cfg.d_in, row_bytes, teams, waves_used, iters, sink)
        torch.cuda.synchronize()
        ev.record(e0, stream)
        cdq.probe_gather(H, cfg.d_in, row_bytes, teams, waves_used, iters, sink)
        ev.record(e1, stream)
        achievable["h_row_gather_GBps"] = teams * iters * row_bytes / (ev.elapsed_ms(e0, e1) * 1e-3) * 1e-9
        achievable["h_row_gather_shape"] = f"H {cfg.d_in}x{cfg.d_in} fp32, rows of {row_bytes} B, {teams} teams x {waves_used} wavefronts"

    workload = (f"{cfg.name}: d_in={cfg.d_in} d_out={cfg.d_out} n={cfg.n} X={cfg.x_dtype}/{cfg.x_kind} bits={cfg.bits} "
                f"group={'per-channel' if cfg.group == cfg.d_in else cfg.group} T={cfg.T} init={'random codes' if args.mode == 'stress' else init}")
    owc_cd_info = None
    if init == "owc_cd":
        # fp64 operations of Algorithm 3 as the tiled kernel organises it: the table of self terms
        # e_k^T H_ii e_k, one F pass per iteration, one rank-`group` update of z per move, plus He of the start
        n_grp, n_gamma = cfg.d_in // cfg.group, 50
        g_moves = int(state["owc_cd_moves"].sum().item())
        iters = g_moves + cfg.d_out                      # every column runs one F pass more than it moves, up to T
        flop = (2.0 * cfg.d_out * n_grp * n_gamma * cfg.group * cfg.group + 2.0 * cfg.d_out * cfg.d_in * cfg.d_in
                + 2.0 * min(iters, cfg.d_out * n_grp) * n_grp * n_gamma * cfg.group + 2.0 * g_moves * cfg.group * (cfg.d_in - cfg.group))
        owc_cd_info = {"strength_moves": g_moves, "fp64_flop": flop, "tflops": flop / (stages["init_grid"] * 1e-3) * 1e-12,
                       "fp64_vector_peak_tflops": 78.6}
    if owc_cd_info is not None and stages["init_grid"] >= max(stages["cd_loop"], stages["hessian"]):
        roofline = {"kernel": "owc_cd_tiled_kernel (+ RTN and fp64 GEMM of the start)", "bound": "alu", "achieved": owc_cd_info["tflops"],
                    "peak": 78.6, "unit": "TFLOP/s", "frac": owc_cd_info["tflops"] / 78.6, "traffic": None,
                    "algorithmic_flop_per_launch": owc_cd_info["fp64_flop"], "avg_launch_ms": stages["init_grid"]}
    elif stages["cd_loop"] >= stages["hessian"]:
        roofline = {"kernel": "cd_fused_kernel", "bound": "hbm", "achieved": cd_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": cd_gbs / HBM_PEAK_GBS, "traffic": load_traffic("cd_fused_kernel", f"{cfg.name}:{args.mode}"),
                    "algorithmic_bytes_per_launch": cd_bytes, "avg_launch_ms": stages["cd_loop"]}
        if "h_row_gather_GBps" in achievable:
            roofline["frac_of_achievable_gather"] = cd_gbs / achievable["h_row_gather_GBps"]
        if 4 * cfg.d_in * cfg.d_in <= 256 * 2 ** 20:
            # the rows of an H that fits the 256 MiB Infinity Cache are not served by HBM: achieved may exceed the HBM peak
            roofline["note"] = "H is cache-resident: rows come from L2 / Infinity Cache, see frac_of_achievable_gather"
    else:
        roofline = {"kernel": "hessian_kernel", "bound": "mfma", "achieved": h_tflops_exec, "peak": mfma_peak, "unit": "TFLOP/s",
                    "frac": h_tflops_exec / mfma_peak, "traffic": load_traffic("hessian_kernel", f"{cfg.name}:{args.mode}"),
                    "algorithmic_flop_per_launch": flop_exec, "avg_launch_ms": stages["hessian"]}

    result = {
        "metric": "greedy_cd_coordinate_updates_per_s", "value": moves / (ms_per_step * 1e-3), "unit": "updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload, "mode": args.mode},
        "roofline": roofline,
        "stages_ms": stages,
        "cd_loop": {"committed_updates": moves, "columns_converged": converged, "updates_per_s": moves / (stages["cd_loop"] * 1e-3),
                    "nominal_T_x_d_out_per_s": cfg.T * cfg.d_out / (stages["cd_loop"] * 1e-3), "H_row_GBps": cd_gbs,
                    "frac_of_hbm_peak": cd_gbs / HBM_PEAK_GBS},
        "hessian": {"tflops_executed": h_tflops_exec, "tflops_effective": h_tflops_eff, "mfma_peak_tflops": mfma_peak,
                    "frac_of_mfma_peak": h_tflops_exec / mfma_peak,
                    "frac_of_measured_mfma_only": (h_tflops_exec / achievable["mfma_bf16_only_TFLOPs"])
                    if cfg.x_dtype == "bf16" and "mfma_bf16_only_TFLOPs" in achievable else None},
        "fp64_gemm": {"gradient_init_tflops": 2.0 * cfg.d_out * cfg.d_in * cfg.d_in / (stages["cd_gradient_init"] * 1e-3) * 1e-12,
                      # the loss multiplies only the 128-wide blocks of H on and above the diagonal (H is symmetric)
                      "loss_tflops_executed": 2.0 * cfg.d_out * 128.0 * 128.0 * sum(range(1, (cfg.d_in + 127) // 128 + 1))
                      / (stages["loss"] * 1e-3) * 1e-12,
                      "loss_tflops_effective": 2.0 * cfg.d_out * cfg.d_in * cfg.d_in / (stages["loss"] * 1e-3) * 1e-12,
                      "mfma_f64_peak_tflops": 78.6},
        "loss_final": loss_final,
        "achievable": achievable,
    }
    if owc_cd_info is not None:
        result["owc_cd"] = owc_cd_info
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, args.mode, init)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
