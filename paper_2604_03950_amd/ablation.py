#!/usr/bin/env python3
"""Synthetic analogues of the paper's ablation tables, on one MI355X.

    python -m paper_2604_03950_amd.ablation [--workload prefill_8k] [--steps 50]

Three tables on the seeded synthetic inputs of a workload (no dataset, no model weights):
  formats      the fixed-format baselines against the mixed kernel (Sec. 5.2, latency breakdown by format),
  windows      diagonal window and sink window sizes (Sec. 5.3, table of diagonal and sink sizes),
  granularity  the Step-2 scale: none, per token, per block, per tensor (Sec. 5.3, table of granularities).
Each row gives the latency of the forward (HIP events, sustained clocks; TFLOP/s in the causal convention 2 B Hq S^2 D) and how close its output is to the library's
own unquantized bf16 forward on the same inputs: cosine similarity, relative L1 error, RMSE and PSNR over all output
elements.  These are reports, not pass/fail checks; the metric formulas are the usual ones (the paper does not print
them).  Everything runs in the HIP library; nothing here touches the CPU oracle.
"""
from __future__ import annotations

import argparse
import json

import torch

from . import binding, workloads as wl


def similarity(x: torch.Tensor, ref: torch.Tensor) -> dict:
    """Cosine similarity, relative L1, RMSE and PSNR (peak = largest reference magnitude) of x against ref, in float64."""
    x = x.double().flatten()
    r = ref.double().flatten()
    d = x - r
    mse = float((d * d).mean())
    peak = float(r.abs().max())
    return {
        "cos": float(torch.dot(x, r) / (x.norm() * r.norm())),
        "rel_l1": float(d.abs().sum() / r.abs().sum()),
        "rmse": mse ** 0.5,
        "psnr_db": float("inf") if mse == 0 else 10.0 * float(torch.log10(torch.tensor(peak * peak / mse))),
    }


def timed(fn, steps: int) -> float:
    """Microseconds per call after at least 60 ms of untimed calls (the clocks need that long to settle)."""
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    fn()
    e1.record()
    torch.cuda.synchronize()
    one = max(e0.elapsed_time(e1), 1e-3)
    for _ in range(int(60.0 / one) + 1):
        fn()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps * 1e3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="prefill_8k")
    ap.add_argument("--steps", type=int, default=50)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("ablation: no GPU visible")
    binding.load()
    w = wl.CONFIGS[args.workload]
    q, k, v = (binding.bits_to_bf16_tensor(a) for a in wl.generate(w))
    out = torch.empty((w.B, w.Hq, w.S, w.D), dtype=torch.float32, device="cuda")
    tile = None if w.tile == 128 else w.tile
    F = binding

    def forward(**kw):
        kw.setdefault("diag_band_tiles", w.band)
        return binding.dma_attn_fwd(q, k, v, tile=tile, out=out, **kw)

    ref = forward(hi_fmt=F.FMT_BF16, lo_fmt=F.FMT_BF16).clone()
    n_tiles = -(-w.S // w.tile)

    causal_flops = 2.0 * w.B * w.Hq * w.S * w.S * w.D      # causal flash-attention convention: 4 S^2 D per head, halved

    def row(table, name, **kw):
        us = timed(lambda: forward(**kw), args.steps)
        rec = {"table": table, "case": name, "us": round(us, 1), "tflops": round(causal_flops / us * 1e-6, 1)}
        rec.update({m: (round(x, 6) if m != "psnr_db" else round(x, 2)) for m, x in similarity(forward(**kw), ref).items()})
        print(json.dumps(rec), flush=True)

    print(json.dumps({"workload": f"{w.name}: B={w.B} Hq={w.Hq} Hkv={w.Hkv} S={w.S} D={w.D} tile={w.tile}, synthetic, seed {w.seed}",
                      "reference": "the library's unquantized bf16 forward on the same inputs"}), flush=True)
    row("formats", "bf16 (unquantized)", hi_fmt=F.FMT_BF16, lo_fmt=F.FMT_BF16)
    row("formats", "all MXFP4", hi_fmt=F.FMT_MXFP4_E2M1, lo_fmt=F.FMT_MXFP4_E2M1)
    row("formats", "all MXFP8 (E4M3)", hi_fmt=F.FMT_MXFP8_E4M3, lo_fmt=F.FMT_MXFP8_E4M3)
    row("formats", "all MXFP8 (E5M2)", hi_fmt=F.FMT_MXFP8_E5M2, lo_fmt=F.FMT_MXFP8_E5M2)
    row("formats", f"DMA: MXFP4 + MXFP8 window of {w.band} tiles")
    row("formats", f"DMA with the MX-format P V (beyond the paper)", pv_mx=True)
    for band in (0, 1, 2, 4, 8, 16):
        if band <= n_tiles:
            row("windows", f"diagonal {band * w.tile} tokens, no sink", diag_band_tiles=band)
    for band, sink in ((1, 1), (2, 1), (4, 1), (2, 2)):
        row("windows", f"diagonal {band * w.tile} tokens, sink {sink * w.tile} tokens", diag_band_tiles=band, sink_tiles=sink)
    row("granularity", "no Step-2 scale (E8M0 block scales only)")
    row("granularity", "per token", per_token_scale=True)
    for name, gran in (("per block (one tile of one head)", F.GRAN_BLOCK), ("per tensor", F.GRAN_TENSOR)):
        def fn(gran=gran):
            ga = (binding.dma_mx_group_amax(q, True, gran, w.tile), binding.dma_mx_group_amax(k, False, gran, w.tile))
            return forward(per_token_scale=True, group_amax=ga)
        us = timed(fn, args.steps)
        rec = {"table": "granularity", "case": name + " (group maxima included in the time)", "us": round(us, 1),
               "tflops": round(causal_flops / us * 1e-6, 1)}
        rec.update({m: (round(x, 6) if m != "psnr_db" else round(x, 2)) for m, x in similarity(fn(), ref).items()})
        print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
