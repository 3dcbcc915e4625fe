"""Is the parity bar tight enough to mean something?  The HIP forward is compared with private copies of the CPU oracle
in which ONE arithmetic choice of the method was changed (on the CPU, in the copy's C source): the unmodified copy must
agree with the GPU within the bar, every changed copy must not.  The choices are the fine ones -- where P is rounded,
what the row sum adds up, the order of the key tiles -- each of which moves the output by only a few 1e-3."""
import numpy as np
import pytest
import torch

import parity
import test_oracle_mutations as tm
from paper_2604_03950_amd import workloads as wl

MAX_ABS, REL_L2 = 2e-3, 1e-3
FINE_CHOICES = ["P never rounded to 16 bit", "bf16 rounding keeps 7 bits", "row sum from the rounded P",
                "key tiles visited in descending order"]
COARSE_CHOICES = ["causal mask also hides the diagonal", "window one tile too wide", "sink window one tile too wide",
                  "e_max of E2M1 off by one", "E2M1 ties round half up", "query formats swapped between the phases"]


@pytest.fixture(scope="module")
def gpu_outputs():
    from paper_2604_03950_amd import binding as dma
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    dma.load()
    cases = []
    for w in (wl.CONFIGS["tiny"], wl.small_variant(wl.CONFIGS["prefill_8k"], S=640, Hq=2, Hkv=2)):
        q, k, v = wl.generate(w)
        qd, kd, vd = (dma.bits_to_bf16_tensor(a) for a in (q, k, v))
        out = dma.dma_attn_fwd(qd, kd, vd, diag_band_tiles=1, sink_tiles=1, tile=w.tile)
        torch.cuda.synchronize()
        cases.append((w, q, k, v, out.cpu().numpy().astype(np.float64)))
    return cases


def within_bar(oracle, cases):
    """The bar of tests/parity.py, with `oracle` (a private copy) as the reference."""
    ok = True
    for w, q, k, v, out in cases:
        rows = oracle.all_rows(w.B, w.Hq, w.S)
        kw = dict(tile=w.tile, band=1, sink=1)
        want = oracle.dma_attn_rows(q, k, v, rows, **kw)
        got = out[rows[:, 0], rows[:, 1], rows[:, 2]]
        try:
            parity.compare(got, want, rows, f"    {w.name}", oracle, (q, k, v), kw, max_abs=MAX_ABS, rel_l2=REL_L2)
        except AssertionError as e:            # a NaN on either side fails the comparison too
            print(f"    {w.name}: outside the bar: {str(e)[:200]}", flush=True)
            ok = False
    return ok


@pytest.mark.gpu
def test_unmodified_copy_is_within_the_bar(tmp_path, gpu_outputs):
    assert within_bar(tm.private_oracle(tmp_path, "oracle_ref_copy"), gpu_outputs)


@pytest.mark.gpu
@pytest.mark.parametrize("what", FINE_CHOICES + COARSE_CHOICES)
def test_changed_copy_is_outside_the_bar(tmp_path, gpu_outputs, what):
    case = [i for i, m in enumerate(tm.MUTATIONS) if m[0] == what][0]
    _, pattern, replacement, _ = tm.MUTATIONS[case]
    oracle = tm.private_oracle(tmp_path, f"oracle_changed_{case}", pattern, replacement)
    assert not within_bar(oracle, gpu_outputs), what
