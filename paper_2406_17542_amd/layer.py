"""Layer driver: the paper's unit of work (quantize one linear layer from streamed calibration
activations), assembled from the library's entry points only.

    H   <- sum over token chunks of X_c^T X_c  (+ lambda I)        cdq_hessian(accumulate)
    a, b, Q0 <- MinMax / OWC / OWC-CD                                 cdq_init_rtn / _owc / _owc_cd
    Q   <- greedy coordinate descent, T iterations                    cdq_greedy_cd      (Algorithm 1/4)
    Q   <- optionally block coordinate descent from that             cdq_bcd            (Algorithm 2/5)
    loss = tr(E^T H E)                                                cdq_loss           (Eq. 1)

Section 4 of the paper calibrates on 1280 sequences of 2048 tokens, runs CD and BCD for d_in
iterations, OWC-CD for d_in/g, initialises BCD with CD, and reports per-layer seconds for the
FFN1 / FFN1-gate / FFN2 matrices of the Gemma models (appendix "Runtime Analysis").  `main`
prints the same rows for synthetic layers of those shapes (activations and weights are seeded
random numbers; the trained models and their calibration data are not available here).

No arithmetic of the method happens in this file: it moves tensors and calls the library.
"""
from __future__ import annotations

import argparse
import json
import time
from typing import Iterable

import numpy as np
import torch

from . import cdq, inputs

# (d_model, d_ff) of the FFN blocks whose runtimes the paper tabulates
MODEL_SHAPES = {
    "gemma1_7b": (3072, 24576),
    "gemma2_9b": (3584, 14336),
    "gemma2_27b": (4608, 36864),
}


class HessianAccumulator:
    """H = sum_c X_c^T X_c over chunks of tokens, then optional damping lambda_rel * mean(diag H) * I
    on the last chunk (Section 4: the Hessian is regularised as in GPTQ)."""

    def __init__(self, d_in: int, device="cuda"):
        self.d_in = d_in
        self.H = torch.empty((d_in, d_in), dtype=torch.float32, device=device)
        self.n_tokens = 0
        self._ws = None

    def add(self, X: torch.Tensor, last: bool = False, lambda_rel: float = 0.0) -> None:
        if X.shape[1] != self.d_in:
            raise ValueError("chunk width differs from d_in")
        need = cdq.workspace_bytes(cdq.OP_HESSIAN, X.shape[0], 0, self.d_in)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device=X.device)
        cdq.hessian(X, H=self.H, accumulate=self.n_tokens > 0, lambda_rel=lambda_rel if last else 0.0, workspace=self._ws)
        self.n_tokens += X.shape[0]


def quantize_layer(chunks: Iterable[torch.Tensor], Wt: torch.Tensor, bits: int, group: int, T: int | None = None,
                   init: str = "rtn", lambda_rel: float = 0.0, bcd_parts: torch.Tensor | None = None, n_gamma: int = 50):
    """Quantize one layer.  chunks: iterable of [n_c][d_in] bf16/fp32 GPU tensors (the calibration
    activations, streamed); Wt [d_out][d_in] fp32 GPU.  Returns a dict with H, scale, zero, Q, loss
    per column, total loss, stats and wall-clock seconds per stage (each stage synchronised)."""
    d_out, d_in = Wt.shape
    T = d_in if T is None else T
    sec = {}

    def timed(name, fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        r = fn()
        torch.cuda.synchronize()
        sec[name] = sec.get(name, 0.0) + time.perf_counter() - t0
        return r

    acc = HessianAccumulator(d_in, Wt.device)
    it = iter(chunks)
    cur = next(it)
    while cur is not None:
        nxt = next(it, None)
        timed("hessian", lambda: acc.add(cur, last=nxt is None, lambda_rel=lambda_rel))
        cur = nxt
    H = acc.H

    G0 = None
    if init == "rtn":
        scale, zero, Q = timed("init", lambda: cdq.init_rtn(Wt, bits, group))
    elif init == "owc":
        # the grid search's fp64 pass leaves the start gradient of Algorithm 1 behind: CD below starts from it
        G0 = torch.empty(Wt.shape, dtype=torch.float32, device=Wt.device)
        scale, zero, Q, _, _ = timed("init", lambda: cdq.init_owc(H, Wt, bits, group, n_gamma, want_loss=False, G_out=G0))
    elif init == "owc_cd":
        o = timed("init", lambda: cdq.init_owc_cd(H, Wt, bits, group, n_gamma))
        scale, zero, Q = o["scale"], o["zero"], o["Q"]
    else:
        raise ValueError(f"unknown init {init!r}")
    loss_init = timed("loss", lambda: cdq.loss(H, Wt, scale, zero, Q, group))[1]

    out = timed("cd", lambda: cdq.greedy_cd(H, Wt, scale, zero, Q, bits, group, T, G0=G0))
    del G0
    res = {"H": H, "scale": scale, "zero": zero, "Q": Q, "stats": out["stats"], "n_tokens": acc.n_tokens,
           "loss_init": float(loss_init.item())}
    per, tot = timed("loss", lambda: cdq.loss(H, Wt, scale, zero, Q, group))
    res["loss_cd"] = float(tot.item())
    if bcd_parts is not None:
        b = timed("bcd", lambda: cdq.bcd(H, Wt, scale, zero, Q, bits, group, bcd_parts))
        res["bcd_moves"] = b["moves"]
        per, tot = timed("loss", lambda: cdq.loss(H, Wt, scale, zero, Q, group))
        res["loss_bcd"] = float(tot.item())
    res["loss_per_column"] = per
    res["seconds"] = sec
    return res


def synthetic_chunks(n_tokens: int, d_in: int, chunk: int, seed: int, dtype=torch.bfloat16, device="cuda"):
    """Seeded Gaussian activations with a heavy-tailed per-channel scale, generated on the GPU chunk by
    chunk (the full calibration set of Section 4, 1280 x 2048 tokens, would not fit at once for the
    wide layers).  Stand-in for real activations; not part of the method."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    ch = torch.exp(0.5 * torch.randn(d_in, generator=g, device=device))
    done = 0
    while done < n_tokens:
        n = min(chunk, n_tokens - done)
        x = torch.randn((n, d_in), generator=g, device=device) * ch
        yield x.to(dtype).contiguous()
        done += n


def main():
    ap = argparse.ArgumentParser(description="Per-layer quantization seconds for synthetic FFN layers of the Gemma shapes")
    ap.add_argument("--model", default="gemma2_9b", choices=sorted(MODEL_SHAPES))
    ap.add_argument("--bits", type=int, default=3)
    ap.add_argument("--tokens", type=int, default=1280 * 2048, help="calibration tokens (Section 4: 1280 sequences of 2048)")
    ap.add_argument("--chunk", type=int, default=131072, help="tokens per cdq_hessian call (each call ends with a pass over H: larger chunks, fewer passes)")
    ap.add_argument("--lambda-rel", type=float, default=0.01)
    ap.add_argument("--t-div", type=int, default=1, help="run CD for d_in / t_div iterations (appendix: d_in/8 suffices)")
    ap.add_argument("--bcd", action="store_true", help="also run BCD (k=2, d_in iterations) from CD's result where it is supported")
    ap.add_argument("--init", default="owc", choices=["rtn", "owc"], help="Section 4: per-channel CD starts from OWC")
    ap.add_argument("--layers", default="ffn1,ffn2", help="comma-separated: ffn1, ffn1_gate (same shape as ffn1, other weights), ffn2")
    args = ap.parse_args()
    d_model, d_ff = MODEL_SHAPES[args.model]
    rows = []
    for name in args.layers.split(","):
        if name not in ("ffn1", "ffn1_gate", "ffn2"):
            raise SystemExit(f"unknown layer {name!r}: ffn1, ffn1_gate or ffn2")
        d_in, d_out = (d_model, d_ff) if name in ("ffn1", "ffn1_gate") else (d_ff, d_model)
        if d_in > cdq.MAX_D_IN:
            rows.append({"layer": name, "d_in": d_in, "d_out": d_out, "skipped": f"d_in above the fused loop's limit of {cdq.MAX_D_IN}"})
            print(json.dumps(rows[-1]), flush=True)
            continue
        Wt = torch.from_numpy(inputs.make_wt(d_out, d_in, seed=7 if name == "ffn1_gate" else 1)).cuda()
        parts = None
        if args.bcd and d_in <= 65534:
            parts = torch.from_numpy(inputs.make_partitions(d_in, d_in, seed=2)).cuda()
        r = quantize_layer(synthetic_chunks(args.tokens, d_in, args.chunk, seed=3), Wt, args.bits, d_in, T=d_in // args.t_div,
                           init=args.init, lambda_rel=args.lambda_rel, bcd_parts=parts)
        st = r["stats"]
        row = {"layer": name, "d_in": d_in, "d_out": d_out, "bits": args.bits, "init": args.init, "tokens": r["n_tokens"], "T": d_in // args.t_div,
               "seconds": {k: round(v, 4) for k, v in r["seconds"].items()},
               "cd_moves": int(st[:, 0].sum().item()), "cd_converged_columns": int(st[:, 2].sum().item()),
               "loss_init": r["loss_init"], "loss_cd": r["loss_cd"]}
        if "loss_bcd" in r:
            row["loss_bcd"] = r["loss_bcd"]
            row["bcd_moves"] = int(r["bcd_moves"].sum().item())
        rows.append(row)
        print(json.dumps(row), flush=True)
        del r, Wt
        torch.cuda.empty_cache()
    return rows


if __name__ == "__main__":
    main()
