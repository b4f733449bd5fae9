#!/usr/bin/env python3
"""Benchmark of the CDQuant hot path on one MI355X.

One "step" = one pass of the whole path over one synthetic layer already resident in HBM:
    H = X^T X  ->  start grid (MinMax/RTN, or OWC's grid search)  ->  greedy coordinate descent
    (gradient init + T iterations)  ->  layer loss.
The workload is the largest of the five configurations (`large`: d_in = 8192, d_out = 32768, 32768 tokens, 3 bit,
OWC start, T = 8192) unless --config says otherwise.  Prints ONE JSON line.  `value` = committed coordinate updates
per second of whole-step time.  Extra objects:
    roofline      the kernel that dominates the step, against the ceiling that binds it (see loop_roofline)
    cpu_baseline  the CPU oracle timed on a bounded sample of the same workload, all host threads and one
    parity        sampled columns of the run just timed, re-run by the oracle for the full T (outside the timed region)
    configs       the other four configurations, a few steps each: loop GB/s and Hessian TFLOP/s
    stages_ms, cd_loop, hessian, fp64_gemm, achievable: per-stage detail of the main workload

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config large] [--mode rtn|stress] [--init config|rtn|owc|owc_cd]
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
INFINITY_CACHE_BYTES = 256 * 2 ** 20
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
# wavefront instructions the chip can issue to its vector ALUs per second: 256 CUs x 4 SIMDs, one fp32 instruction
# of a 64-wide wavefront every 4 cycles, 2.4 GHz
VALU_ISSUE_PEAK = 256 * 4 * 2.4e9 / 4
# vector-ALU issue slots of the loop kernels per wavefront and iteration at 16 coordinates per lane, from SQ_INSTS_VALU
# (profiles/cd_loop_sq_counters.txt): 319 instructions in the register kernels (13 per coordinate for the score and the
# running arg-min, 1 per coordinate for the update, the rest reduction and bookkeeping); 405 in the kernel for two columns
# per compute unit, 16 of them v_rcp_f32, which takes four slots; 304 with one or two wavefronts per column (attn_proj).
# Scaled by coordinates per lane for other shapes: a model (the 2-bit grouped layer needs fewer, so its figure reads high).
VALU_PER_WAVE_ITER_AT_16 = 320.0
VALU_PER_WAVE_ITER_NARROW = 304.0
VALU_PER_WAVE_ITER_PAIR = 405.0 + 3.0 * 16.0


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

    def destroy(self, ev):
        self.hip.hipEventDestroy(ev)

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
    """HBM-side bytes per launch measured offline with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by the same
    counters on a copy of known size); (bytes, source) or (None, None) when profiles/traffic.json has no entry."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            table = json.load(f)
    except (OSError, ValueError):
        return None, None
    entry = table.get(f"{kernel}:{workload}")
    if entry is None:
        return None, None
    if isinstance(entry, dict):
        return entry.get("bytes"), "offline: " + entry.get("source", "profiles/traffic.json")
    return entry, "offline: " + table.get("_source", "profiles/traffic.json")


def set_omp_threads(n):
    """Number of threads the oracle's OpenMP loops use from now on (its code is left as it is)."""
    try:
        ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))
        return True
    except OSError:
        return False


def cpu_baseline(cfg, mode, init, budget_s=14.0):
    """The oracle, as it stands, on the host cores: Hessian on a token sample, start grid + CD + loss on a column
    sample, each scaled linearly to the full layer; updates/s of the whole step.  Timed with all threads and, on a
    smaller sample, with one."""
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
    del X, H64

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

    threads = oracle.n_threads()

    def sample(n_thr, budget):
        probe_cols = min(cfg.d_out, 2 * n_thr)
        t_probe, _ = run(probe_cols)
        cols = int(min(cfg.d_out, max(probe_cols, probe_cols * budget / max(t_probe, 1e-3))))
        t_cols, moves = run(cols)
        scale = cfg.d_out / cols
        total_s = t_h + t_cols * scale
        return moves * scale / total_s, cols, total_s

    v_all, cols_all, total_all = sample(threads, budget_s)
    out = {
        "value": v_all, "unit": "updates/s", "cores": threads, "kind": "oracle",
        "sample": f"Hessian on {n_tok} of {cfg.n} tokens (fp64 numpy), {init} init+CD+loss on the first {cols_all} of "
                  f"{cfg.d_out} columns for the full T={cfg.T}; times scaled linearly to the full layer "
                  f"(est. {total_all:.1f} s)",
    }
    if threads > 1 and set_omp_threads(1):
        v_one, cols_one, total_one = sample(1, budget_s / 3.0)
        set_omp_threads(threads)
        out["one_thread"] = {"value": v_one, "unit": "updates/s", "cores": 1,
                             "sample": f"same, the column part on one thread: first {cols_one} columns (est. {total_one:.1f} s; "
                                       f"the numpy Hessian keeps its own threads)"}
    return out


def workload_name(cfg, mode, init):
    return (f"{cfg.name}: d_in={cfg.d_in} d_out={cfg.d_out} n={cfg.n} X={cfg.x_dtype}/{cfg.x_kind} bits={cfg.bits} "
            f"group={'per-channel' if cfg.group == cfg.d_in else cfg.group} T={cfg.T} "
            f"init={'random codes' if mode == 'stress' else init}")


class Layer:
    """One configuration resident on the GPU, with everything a step needs allocated up front."""

    def __init__(self, cfg, mode, init, args):
        import numpy as np
        import torch

        from paper_2406_17542_amd import cdq, inputs
        self.cfg, self.mode, self.init, self.args = cfg, mode, init, args
        self.cdq = cdq
        X, Wt = inputs.make_layer(cfg)
        if cfg.x_dtype == "bf16":
            self.Xd = torch.from_numpy(inputs.bf16_bits(X).view(np.int16)).cuda().view(torch.bfloat16)
        else:
            self.Xd = torch.from_numpy(X).cuda()
        del X
        self.Wd = torch.from_numpy(Wt).cuda()
        del Wt
        self.q_stress = None
        if mode == "stress":
            self.q_stress = torch.from_numpy(inputs.make_random_codes(cfg.d_out, cfg.d_in, cfg.bits, cfg.seed)).cuda()

        def ws(op, n=0, d_out=cfg.d_out):
            return torch.empty(max(cdq.workspace_bytes(op, n, d_out, cfg.d_in), 256), dtype=torch.uint8, device="cuda")
        self.H = torch.empty((cfg.d_in, cfg.d_in), dtype=torch.float32, device="cuda")
        self.ws_h = ws(cdq.OP_HESSIAN, cfg.n, 0)
        # with the OWC start the grid search hands the start gradient over (it is a by-product of its fp64 pass), so
        # Algorithm 1's own gradient initialisation, and the room for it, fall away
        self.fused_g0 = init == "owc" and mode != "stress"
        if self.fused_g0:
            self.G0 = torch.empty((cfg.d_out, cfg.d_in), dtype=torch.float32, device="cuda")
            self.ws_cd = torch.empty((4 * cfg.d_in + 255) // 256 * 256, dtype=torch.uint8, device="cuda")
        else:
            self.G0 = None
            self.ws_cd = ws(cdq.OP_GREEDY_CD)
        self.ws_l = ws(cdq.OP_LOSS)
        self.ws_owc = ws(cdq.OP_INIT_OWC) if init == "owc" else ws(cdq.OP_INIT_OWC_CD) if init == "owc_cd" else None
        self.state = {}

    def step(self, ev=None, evs=None, stream=None):
        cfg, cdq, init = self.cfg, self.cdq, self.init
        rec = (lambda k: ev.record(evs[k], stream)) if evs is not None else (lambda k: None)
        rec(0)
        cdq.hessian(self.Xd, H=self.H, workspace=self.ws_h)
        rec(1)
        if init == "owc":
            scale, zero, Q, gamma, _, cnt = cdq.init_owc(self.H, self.Wd, cfg.bits, cfg.group, 50, workspace=self.ws_owc, want_loss=False,
                                                         want_researched=True, G_out=self.G0)
            self.state["gamma"] = gamma
            self.state["owc_researched"] = cnt
        elif init == "owc_cd":
            o = cdq.init_owc_cd(self.H, self.Wd, cfg.bits, cfg.group, 50, workspace=self.ws_owc)
            scale, zero, Q = o["scale"], o["zero"], o["Q"]
            self.state["owc_cd_moves"] = o["moves"]
        else:
            scale, zero, Q = cdq.init_rtn(self.Wd, cfg.bits, cfg.group)
        if self.q_stress is not None:
            Q.copy_(self.q_stress)
        if self.state.get("keep_q0"):
            self.state["Q0"] = Q.clone()
        rec(2)
        out = cdq.greedy_cd(self.H, self.Wd, scale, zero, Q, cfg.bits, cfg.group, cfg.T, workspace=self.ws_cd,
                            waves_per_column=self.args.waves, elems_per_lane=self.args.elems,
                            loop_events=(evs[3], evs[4]) if evs is not None else None, G0=self.G0, teams_per_cu=self.args.teams)
        rec(5)
        per, tot = cdq.loss(self.H, self.Wd, scale, zero, Q, cfg.group, workspace=self.ws_l)
        rec(6)
        self.state.update(stats=out["stats"], loss=tot, loss_per_col=per, Q=Q, scale=scale, zero=zero)

    def timed(self, ev, stream, steps, warmup):
        """W untimed steps, then exactly K timed ones between device synchronisations; per-stage times from events."""
        import torch
        events = [[ev.create() for _ in range(7)] for _ in range(steps)]
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            self.step(ev, events[k], stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        # [0,1] hessian, [1,2] start grid, [2,3] gradient init (+diag), [3,4] the iteration-loop kernel, [5,6] loss
        spans = {"hessian": (0, 1), "init_grid": (1, 2), "cd_gradient_init": (2, 3), "cd_loop": (3, 4), "loss": (5, 6)}
        stages = {name: sum(ev.elapsed_ms(events[k][a], events[k][b]) for k in range(steps)) / steps
                  for name, (a, b) in spans.items()}
        for evs in events:
            for e in evs:
                ev.destroy(e)
        return (t1 - t0) * 1e3 / steps, stages

    def hessian_rates(self, stages):
        cfg = self.cfg
        flop_eff = 2.0 * cfg.n * cfg.d_in * cfg.d_in
        tile = 256 if cfg.x_dtype == "bf16" else 128                  # tile edge of the Hessian kernels
        n_t = (cfg.d_in + tile - 1) // tile
        flop_exec = 2.0 * cfg.n * (n_t * (n_t + 1) // 2) * tile * tile   # tiles on and above the diagonal only
        t = stages["hessian"] * 1e-3
        return flop_exec, flop_exec / t * 1e-12, flop_eff / t * 1e-12


def loop_roofline(cfg, mode, moves, loop_ms, shape, gather_gbs):
    """Roofline of the loop kernel.  Algorithmic bytes = one row of H (4 d_in bytes) per committed update; g, q and
    diag(H) stay in registers.  What serves those rows decides the ceiling: HBM when H (4 d_in^2 bytes) exceeds the
    256 MiB Infinity Cache; L2 / Infinity Cache otherwise, where no published peak exists -- `frac` stays the
    recomputable fraction of the HBM peak (and may exceed 1), the ceiling that binds is the gather rate measured in
    the same run (independent random rows of the same H, same row length and team width, no arithmetic) and, on the
    narrow layers, the vector-ALU issue rate of the scoring."""
    h_bytes = 4.0 * cfg.d_in * cfg.d_in
    cd_bytes = moves * 4.0 * cfg.d_in
    gbs = cd_bytes / (loop_ms * 1e-3) * 1e-9
    waves, elems, teams_per_cu = shape
    kernel = "cd_fused_pair_kernel" if teams_per_cu == 2 else "cd_fused_kernel"
    per_wave = VALU_PER_WAVE_ITER_PAIR if teams_per_cu == 2 else VALU_PER_WAVE_ITER_NARROW if waves <= 2 else VALU_PER_WAVE_ITER_AT_16
    valu_per_update = waves * per_wave * elems / 16.0
    valu_rate = moves * valu_per_update / (loop_ms * 1e-3)
    traffic, source = load_traffic("cd_fused_kernel", f"{cfg.name}:{mode}")
    r = {"kernel": kernel, "bound": "hbm" if h_bytes > INFINITY_CACHE_BYTES else "cache",
         "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
         "traffic": traffic, "algorithmic_bytes_per_launch": cd_bytes, "avg_launch_ms": loop_ms,
         "launch_shape": {"wavefronts_per_column": waves, "coordinates_per_lane": elems,
                          "columns_resident_per_cu": teams_per_cu * max(1, 16 // waves)},
         "valu_issue": {"issue_slots_per_update_model": valu_per_update, "achieved_slots_per_s": valu_rate,
                        "chip_issue_rate_slots_per_s": VALU_ISSUE_PEAK, "frac": valu_rate / VALU_ISSUE_PEAK}}
    if traffic is not None:
        r["traffic_source"] = source
        r["traffic_over_algorithmic"] = traffic / cd_bytes if cd_bytes else None
    if gather_gbs:
        r["ceiling_measured_gather_GBps"] = gather_gbs
        r["frac_of_measured_gather"] = gbs / gather_gbs
    if r["bound"] == "cache":
        r["note"] = ("H fits the Infinity Cache: the rows come from L2 / Infinity Cache, not HBM; peak is the published HBM figure "
                     "kept for comparison, the binding ceilings are ceiling_measured_gather_GBps and valu_issue")
    return r


def probes(cfg, H, shape, ev, stream, cdq, want_stream=True):
    """Achievable figures on this machine, same process: streaming reads, the matrix cores alone, and the loop's access
    pattern (independent random rows of H) without its arithmetic."""
    import torch
    achievable = {}
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    e0, e1 = ev.create(), ev.create()
    if want_stream:
        big = torch.empty(1 << 30, dtype=torch.float32, device="cuda")       # 4 GiB
        big.zero_()
        cdq.probe_read(big, big.numel() * 4, sink)
        torch.cuda.synchronize()
        ev.record(e0, stream)
        for _ in range(5):
            cdq.probe_read(big, big.numel() * 4, sink)
        ev.record(e1, stream)
        achievable["hbm_stream_read_GBps"] = 5 * big.numel() * 4 / (ev.elapsed_ms(e0, e1) * 1e-3) * 1e-9
        del big
        small = torch.zeros(8 << 20, dtype=torch.float32, device="cuda")     # 32 MiB, stays in the last-level cache
        cdq.probe_read(small, small.numel() * 4, sink)
        torch.cuda.synchronize()
        ev.record(e0, stream)
        for _ in range(200):
            cdq.probe_read(small, small.numel() * 4, sink)
        ev.record(e1, stream)
        achievable["cache_stream_read_GBps_32MiB"] = 200 * small.numel() * 4 / (ev.elapsed_ms(e0, e1) * 1e-3) * 1e-9
        del small
        # the matrix cores alone, no memory traffic: on constant operands (the instruction rate at the clock an idle data
        # path allows) and on pseudo-random ones (what the chip sustains when the operand bits toggle as real data does)
        for kind, key, blocks, iters in ((0, "mfma_bf16_only_TFLOPs", 512, 20000), (2, "mfma_bf16_only_random_operands_TFLOPs", 1024, 4000),
                                         (1, "mfma_f64_only_TFLOPs", 512, 5000)):
            cdq.probe_mfma(kind, blocks, 200, sink)
            torch.cuda.synchronize()
            ev.record(e0, stream)
            flop = cdq.probe_mfma(kind, blocks, iters, sink)
            ev.record(e1, stream)
            achievable[key] = flop / (ev.elapsed_ms(e0, e1) * 1e-3) * 1e-12
    waves = shape[0]
    teams = 256 * max(1, 16 // waves) * shape[2]          # as many teams as the loop kernel keeps resident per CU
    row_bytes = 4 * cfg.d_in
    iters = max(50, int(2e11 / (teams * row_bytes)))
    cdq.probe_gather(H, cfg.d_in, row_bytes, teams, waves, iters, sink)
    torch.cuda.synchronize()
    ev.record(e0, stream)
    cdq.probe_gather(H, cfg.d_in, row_bytes, teams, waves, iters, sink)
    ev.record(e1, stream)
    achievable["h_row_gather_GBps"] = teams * iters * row_bytes / (ev.elapsed_ms(e0, e1) * 1e-3) * 1e-9
    achievable["h_row_gather_shape"] = f"H {cfg.d_in}x{cfg.d_in} fp32, rows of {row_bytes} B, {teams} teams x {waves} wavefronts"
    ev.destroy(e0)
    ev.destroy(e1)
    return achievable


def parity_check(layer, n_cols=8):
    """Sampled columns of the run just timed, re-run by the oracle from the same fp32 H for the full T: start grid,
    codes, move counts, per-column loss.  The columns with the most moves are part of the sample."""
    import numpy as np

    from oracle import cdq_oracle as oracle
    cfg, st = layer.cfg, layer.state
    stats = st["stats"].cpu().numpy()
    rng = np.random.default_rng(17)
    busiest = np.argsort(-stats[:, 0], kind="stable")[:max(1, n_cols // 4)]
    cols = np.unique(np.concatenate([busiest, rng.choice(cfg.d_out, size=n_cols, replace=False)]))[:n_cols + len(busiest)]
    H32 = layer.H.cpu().numpy()
    Wt = layer.Wd[torch_index(cols)].cpu().numpy()
    a = st["scale"][torch_index(cols)].cpu().numpy()
    b = st["zero"][torch_index(cols)].cpu().numpy()
    q0 = st["Q0"][torch_index(cols)].cpu().numpy()
    out = {"cols": int(len(cols)), "T": cfg.T, "max_moves_in_sample": int(stats[cols, 0].max())}
    if layer.init == "owc" and layer.mode != "stress":
        ra, rb, rq, rgam, rloss_all = oracle.init_owc(H32, Wt, cfg.bits, cfg.group, 50)
        rloss = rloss_all.min(axis=0)           # [n_gamma][columns] -> each column's best
        g_gpu = st["gamma"][torch_index(cols)].cpu().numpy()
        same = g_gpu == rgam
        out["start_grid_equal_cols"] = int(same.sum())
        # a column whose clipping strength differs must be a tie of the two grid points' losses
        ok = True
        for c in np.where(~same)[0]:
            l_gpu = oracle.loss(H32, Wt[c:c + 1], q0[c:c + 1], a[c:c + 1], b[c:c + 1], cfg.group)[0]
            ok &= abs(l_gpu - rloss[c]) <= 1e-6 * rloss[c]
        out["start_grid_differences_are_ties"] = bool(ok)
    ref = oracle.greedy_cd(H32, Wt, a, b, q0, cfg.bits, cfg.group, cfg.T)
    Qn = st["Q"][torch_index(cols)].cpu().numpy()
    out["codes_equal"] = float((Qn == ref["Q"]).mean())
    out["moves_equal_cols"] = int((stats[cols, 0] == ref["moves"]).sum())
    l_ref = oracle.loss(H32, Wt, ref["Q"], a, b, cfg.group)
    l_gpu = st["loss_per_col"][torch_index(cols)].cpu().numpy()
    out["loss_rel"] = float(np.max(np.abs(l_gpu - l_ref) / l_ref))
    out["ok"] = bool(out["codes_equal"] >= 0.999 and out["loss_rel"] <= 1e-4)
    return out


def torch_index(cols):
    import torch
    return torch.from_numpy(cols).cuda()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="large")
    ap.add_argument("--mode", default="rtn", choices=["rtn", "stress"],
                    help="rtn: initial codes as the configuration says; stress: uniform random initial codes")
    ap.add_argument("--init", default="config", choices=["config", "rtn", "owc", "owc_cd"],
                    help="initial grid: the configuration's own, MinMax/RTN, OWC (Eq. 2 grid search) or OWC-CD (Algorithm 3)")
    ap.add_argument("--waves", type=int, default=0)
    ap.add_argument("--elems", type=int, default=0)
    ap.add_argument("--teams", type=int, default=0, help="columns resident per compute unit for the 16 x 16 launch shape: 0 = library default, 1 or 2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probes", action="store_true", help="skip the achievable-bandwidth probes")
    ap.add_argument("--no-parity", action="store_true", help="skip the oracle check of sampled columns")
    ap.add_argument("--no-others", action="store_true", help="skip the short runs of the other configurations")
    ap.add_argument("--others-steps", type=int, default=3)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the output columns are independent problems and would shard "
              "over GPUs with a replica of H and no communication during the loop) -- rerun with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2406_17542_amd import cdq, inputs

    cfg = inputs.CONFIGS[args.config]
    init = cfg.init if args.init == "config" else args.init
    if args.mode == "stress":
        init = "rtn"
    torch.cuda.set_device(0)
    ev = HipEvents()
    stream = torch.cuda.current_stream().cuda_stream

    layer = Layer(cfg, args.mode, init, args)

    # a copy of known size (256 MiB read + 256 MiB written): reference dispatch for scaling the
    # FETCH_SIZE / WRITE_SIZE counters when this command runs under rocprofv3 --pmc
    cal_src = torch.zeros(64 << 20, dtype=torch.float32, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    cdq.probe_copy(cal_src, cal_dst)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    ms_per_step, stages = layer.timed(ev, stream, args.steps, args.warmup)
    state = layer.state
    moves = int(state["stats"][:, 0].sum().item())
    converged = int(state["stats"][:, 2].sum().item())
    loss_final = float(state["loss"].item())
    shape = (args.waves, args.elems, 1) if args.waves and args.elems else cdq.greedy_cd_launch(cfg.d_out, cfg.d_in, cfg.group)
    if args.teams:
        shape = (shape[0], shape[1], args.teams)

    achievable = {} if args.no_probes else probes(cfg, layer.H, shape, ev, stream, cdq)
    flop_exec, h_tflops_exec, h_tflops_eff = layer.hessian_rates(stages)
    mfma_peak = MFMA_PEAK_TFLOPS[cfg.x_dtype]

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
        roofline = loop_roofline(cfg, args.mode, moves, stages["cd_loop"], shape, achievable.get("h_row_gather_GBps"))
    else:
        traffic, source = load_traffic("hessian_kernel", f"{cfg.name}:{args.mode}")
        roofline = {"kernel": "hessian_kernel", "bound": "mfma", "achieved": h_tflops_exec, "peak": mfma_peak, "unit": "TFLOP/s",
                    "frac": h_tflops_exec / mfma_peak, "traffic": traffic, "algorithmic_flop_per_launch": flop_exec,
                    "avg_launch_ms": stages["hessian"]}
        if traffic is not None:
            roofline["traffic_source"] = source

    cd_gbs = moves * 4.0 * cfg.d_in / (stages["cd_loop"] * 1e-3) * 1e-9
    result = {
        "metric": "greedy_cd_coordinate_updates_per_s", "value": moves / (ms_per_step * 1e-3), "unit": "updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload_name(cfg, args.mode, init), "mode": args.mode},
        "roofline": roofline,
        "stages_ms": stages,
        "cd_loop": {"committed_updates": moves, "columns_converged": converged, "updates_per_s": moves / (stages["cd_loop"] * 1e-3),
                    "nominal_T_x_d_out_per_s": cfg.T * cfg.d_out / (stages["cd_loop"] * 1e-3), "H_row_GBps": cd_gbs,
                    "frac_of_hbm_peak": cd_gbs / HBM_PEAK_GBS},
        "hessian": {"tflops_executed": h_tflops_exec, "tflops_effective": h_tflops_eff, "mfma_peak_tflops": mfma_peak,
                    "frac_of_mfma_peak": h_tflops_exec / mfma_peak,
                    "frac_of_measured_mfma_only": (h_tflops_exec / achievable["mfma_bf16_only_TFLOPs"])
                    if cfg.x_dtype == "bf16" and "mfma_bf16_only_TFLOPs" in achievable else None,
                    # the ceiling that binds on data: the matrix cores alone on pseudo-random operands (clock under that load included)
                    "frac_of_measured_mfma_only_random_operands": (h_tflops_exec / achievable["mfma_bf16_only_random_operands_TFLOPs"])
                    if cfg.x_dtype == "bf16" and "mfma_bf16_only_random_operands_TFLOPs" in achievable else None},
        "fp64_gemm": {"gradient_init_tflops": None if layer.fused_g0 else
                      2.0 * cfg.d_out * cfg.d_in * cfg.d_in / (stages["cd_gradient_init"] * 1e-3) * 1e-12,
                      "gradient_init": "inside init_grid: the grid search's fp64 pass leaves the start gradient" if layer.fused_g0
                      else "cdq_greedy_cd's own",
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
    if "owc_researched" in state:
        # columns whose fp16 estimate of the grid search failed its check against the fp64 loss and were searched exhaustively
        result["owc"] = {"grid": 50, "columns_searched_exhaustively": int(state["owc_researched"].item()), "ms": stages["init_grid"]}

    if not args.no_parity:
        # one more, untimed, step that keeps the start codes, then the oracle on sampled columns of exactly that run
        state["keep_q0"] = True
        layer.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        result["parity"] = parity_check(layer)
        result["parity"]["oracle_s"] = time.perf_counter() - t0

    del layer, state
    torch.cuda.empty_cache()

    if not args.no_others:
        others = []
        for name in inputs.CONFIG_ORDER:
            if name == cfg.name:
                continue
            c = inputs.CONFIGS[name]
            lay = Layer(c, "rtn", c.init, args)
            ms, stg = lay.timed(ev, stream, args.others_steps, 1)
            mv = int(lay.state["stats"][:, 0].sum().item())
            shp = cdq.greedy_cd_launch(c.d_out, c.d_in, c.group)
            gath = None if args.no_probes else probes(c, lay.H, shp, ev, stream, cdq, want_stream=False).get("h_row_gather_GBps")
            roof = loop_roofline(c, "rtn", mv, stg["cd_loop"], shp, gath)
            _, h_exec, h_eff = lay.hessian_rates(stg)
            others.append({"workload": workload_name(c, "rtn", c.init), "steps": args.others_steps, "ms_per_step": ms,
                           "updates_per_s": mv / (ms * 1e-3), "committed_updates": mv, "stages_ms": stg,
                           "loop": {k: roof[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic", "launch_shape")
                                    } | {k: roof[k] for k in ("ceiling_measured_gather_GBps", "frac_of_measured_gather", "traffic_over_algorithmic") if k in roof}
                                    | {"valu_issue_frac": roof["valu_issue"]["frac"]},
                           "hessian": {"tflops_executed": h_exec, "tflops_effective": h_eff,
                                       "frac_of_mfma_peak": h_exec / MFMA_PEAK_TFLOPS[c.x_dtype]},
                           "loss_final": float(lay.state["loss"].item())})
            del lay
            torch.cuda.empty_cache()
        result["configs"] = others

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, args.mode, init)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
