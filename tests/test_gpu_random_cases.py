"""Seeded random sweep over shapes and options of the fused forward (GPU vs the CPU oracle).

Every case draws head dimension, batch, head counts (with GQA ratios), a sequence length that may or may not be a whole
number of tiles, a format pair, window and sink sizes, the mask, the Step-2 scale with its granularity and the MX-format
P V, and checks up to 1500 rows against the oracle at the bar of the fixed cases."""
import random

import numpy as np
import pytest
import torch

import parity
from paper_2604_03950_amd import workloads as wl

MAX_ABS, REL_L2 = 2e-3, 1e-3
PAIRS = [("e2m1", "e4m3"), ("e2m1", "e2m1"), ("e4m3", "e4m3"), ("e2m1", "e5m2"), ("e5m2", "e5m2"), ("bf16", "bf16")]


@pytest.fixture(scope="module")
def dma():
    from paper_2604_03950_amd import binding
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    binding.load()
    return binding


@pytest.mark.gpu
@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_cases(dma, oracle, seed):
    fm = {"bf16": (dma.FMT_BF16, oracle.FMT_BF16), "e4m3": (dma.FMT_MXFP8_E4M3, oracle.FMT_E4M3),
          "e2m1": (dma.FMT_MXFP4_E2M1, oracle.FMT_E2M1), "e5m2": (dma.FMT_MXFP8_E5M2, oracle.FMT_E5M2)}
    rnd = random.Random(seed)
    for it in range(12):
        d128 = rnd.random() < 0.5
        base = wl.CONFIGS["prefill_8k"] if d128 else wl.CONFIGS["tiny"]
        tile = 128 if d128 else 64
        hkv = rnd.choice([1, 2, 3, 8])
        group = rnd.choice([1, 1, 2, 4])
        batch = rnd.choice([1, 1, 2, 3])
        S = rnd.choice([tile, 2 * tile, 3 * tile, 4 * tile, 6 * tile, rnd.randint(1, 5 * tile)])
        w = wl.small_variant(base, S=S, Hq=hkv * group, Hkv=hkv, B=batch, seed=100 * seed + it)
        q, k, v = wl.generate(w)
        lo, hi = rnd.choice(PAIRS)
        band = rnd.choice([0, 1, 2, 3, 100])
        sink = rnd.choice([0, 0, 1, 2])
        causal = rnd.random() < 0.6
        per_token = rnd.random() < 0.3 and lo != "bf16"
        gran = rnd.choice(["token", "block", "tensor"]) if per_token else None
        pv_mx = (lo, hi) == ("e2m1", "e4m3") and not per_token and rnd.random() < 0.3
        what = (f"seed {seed} case {it}: D={w.D} B={batch} Hq={w.Hq} Hkv={hkv} S={S} {lo}/{hi} band={band} sink={sink} "
                f"causal={causal} scale={gran} pv_mx={pv_mx}")
        print(what, flush=True)
        qd, kd, vd = (dma.bits_to_bf16_tensor(a) for a in (q, k, v))
        group_amax = None
        if per_token and gran != "token":
            gid = dma.GRAN_BLOCK if gran == "block" else dma.GRAN_TENSOR
            group_amax = (dma.dma_mx_group_amax(qd, True, gid, tile), dma.dma_mx_group_amax(kd, False, gid, tile))
        out = torch.full((w.B, w.Hq, w.S, w.D), float("nan"), dtype=torch.float32, device="cuda")    # unwritten rows stay NaN
        dma.dma_attn_fwd(qd, kd, vd, diag_band_tiles=band, hi_fmt=fm[hi][0], lo_fmt=fm[lo][0], causal=causal,
                         sink_tiles=sink, per_token_scale=per_token, pv_mx=pv_mx, group_amax=group_amax, tile=tile, out=out)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out).all()), what
        rows = oracle.all_rows(w.B, w.Hq, w.S)
        if len(rows) > 1500:
            pick = np.random.Generator(np.random.Philox(100 * seed + it)).choice(len(rows), 1500, replace=False)
            rows = oracle.sort_rows(rows[np.sort(pick)])
        kw = dict(tile=tile, band=band, hi_fmt=fm[hi][1], lo_fmt=fm[lo][1], sink=sink, causal=causal,
                  per_token=(gran if per_token else False), pv_mx=pv_mx)
        want = oracle.dma_attn_rows(q, k, v, rows, **kw)
        got = out.cpu().numpy()[rows[:, 0], rows[:, 1], rows[:, 2]].astype(np.float64)
        parity.compare(got, want, rows, "    result", oracle, (q, k, v), kw, max_abs=MAX_ABS, rel_l2=REL_L2)


@pytest.mark.gpu
@pytest.mark.parametrize("seed", [21, 22])
def test_random_midsize_cases(dma, oracle, seed):
    """Mid-size shapes with odd head counts and batches: more work items than workgroups (several rounds of the static
    schedule, with and without the per-XCD split), lengths that are not whole tiles.  Every row must be written; 600
    uniformly drawn rows go to the oracle."""
    rnd = random.Random(seed)
    tile = 128
    for it in range(4):
        hkv = rnd.choice([3, 5, 7, 8, 12, 16])
        group = rnd.choice([1, 2, 3, 4])
        batch = rnd.choice([1, 2, 3, 5])
        S = rnd.choice([1024, 1152, 1536, 2048, 2432, 3072, rnd.randint(900, 3000)])    # even and odd tile counts
        w = wl.small_variant(wl.CONFIGS["prefill_8k"], S=S, Hq=hkv * group, Hkv=hkv, B=batch, seed=1000 * seed + it)
        q, k, v = wl.generate(w)
        band = rnd.choice([0, 1, 2, 3])
        sink = rnd.choice([0, 0, 1])
        causal = rnd.random() < 0.7
        per_token = rnd.random() < 0.25
        pv_mx = (not per_token) and rnd.random() < 0.25
        what = (f"seed {seed} case {it}: B={batch} Hq={w.Hq} Hkv={hkv} S={S} band={band} sink={sink} causal={causal} "
                f"per_token={per_token} pv_mx={pv_mx}")
        print(what, flush=True)
        qd, kd, vd = (dma.bits_to_bf16_tensor(a) for a in (q, k, v))
        out = torch.full((w.B, w.Hq, w.S, w.D), float("nan"), dtype=torch.float32, device="cuda")
        dma.dma_attn_fwd(qd, kd, vd, diag_band_tiles=band, causal=causal, sink_tiles=sink, per_token_scale=per_token,
                         pv_mx=pv_mx, out=out)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out).all()), what
        rows = oracle.all_rows(w.B, w.Hq, w.S)
        pick = np.random.Generator(np.random.Philox(1000 * seed + it)).choice(len(rows), 600, replace=False)
        rows = oracle.sort_rows(rows[np.sort(pick)])
        kw = dict(tile=tile, band=band, sink=sink, causal=causal, per_token=per_token, pv_mx=pv_mx)
        want = oracle.dma_attn_rows(q, k, v, rows, **kw)
        got = out.cpu().numpy()[rows[:, 0], rows[:, 1], rows[:, 2]].astype(np.float64)
        parity.compare(got, want, rows, "    result", oracle, (q, k, v), kw, max_abs=MAX_ABS, rel_l2=REL_L2)
