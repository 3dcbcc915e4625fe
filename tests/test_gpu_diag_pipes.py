"""dma_diag_pipes: instruction streams side by side on one SIMD (the measurement `bench.py --pipes` prints).

Only what holds on any box at any clock is asserted: every stream makes progress, a slot that is idle counts nothing,
the matrix pipe serves one wave at a time (two matrix waves together issue no more than one alone), and a vector wave
next to a matrix wave is not faster than alone.  The figures themselves are in profiles/.
"""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dma():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2604_03950_amd import binding
    binding.load()
    return binding


def test_streams_run_and_stop_by_the_clock(dma):
    us = 200
    for _ in range(100):                                   # clocks up
        dma.dma_diag_pipes((dma.PIPE_FMA, dma.PIPE_FMA), us)
    torch.cuda.synchronize()
    for kind in (dma.PIPE_MFMA_BF16, dma.PIPE_MFMA_FP4, dma.PIPE_MFMA_FP8, dma.PIPE_FMA, dma.PIPE_EXP, dma.PIPE_CVT_PK_BF16):
        counts, wgs = dma.dma_diag_pipes((kind,), us)
        assert wgs > 0 and counts[0] > 0, kind
        per_wave = counts[0] / (4 * wgs)
        print(f"stream {kind}: {per_wave:.0f} instructions per wave in {us} us", flush=True)
        assert 100 < per_wave < 1e6, (kind, per_wave)     # between 0.5 and 5000 clocks per instruction at any sane clock
    counts, _ = dma.dma_diag_pipes((dma.PIPE_FMA, dma.PIPE_IDLE, dma.PIPE_FMA), us)
    assert counts[0] > 0 and counts[1] == 0 and counts[2] > 0


def test_matrix_pipe_serves_one_wave_and_slows_vector_waves(dma):
    us = 300
    M, F = dma.PIPE_MFMA_BF16, dma.PIPE_FMA
    for _ in range(100):
        dma.dma_diag_pipes((F, F), us)
    torch.cuda.synchronize()
    (m1,), _ = dma.dma_diag_pipes((M,), us)
    (ma, mb), _ = dma.dma_diag_pipes((M, M), us)
    (f1,), _ = dma.dma_diag_pipes((F,), us)
    (m2, f2), _ = dma.dma_diag_pipes((M, F), us)
    print(f"matrix alone {m1}, two matrix waves {ma} + {mb}; vector alone {f1}, next to a matrix wave {f2} (matrix {m2})", flush=True)
    assert ma + mb <= 1.25 * m1                            # one pipe: two waves share what one wave gets (measured 1.04)
    assert f2 <= 1.1 * f1                                  # not faster next to a matrix wave (measured 0.83; clocks may drift a little)
    assert m2 >= 0.5 * m1                                  # and the matrix wave keeps most of its rate
