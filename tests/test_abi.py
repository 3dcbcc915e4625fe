"""The C-ABI library loads and exports every symbol include/dma.h declares; argument checks that
return before any GPU work behave as documented.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

from paper_2604_03950_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dma.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dma_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.lib_path()):
        from paper_2604_03950_amd import build
        build.build()
    return binding.load()


def test_header_and_library_agree(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_version_and_error_strings(lib):
    assert binding.version() >= 100
    assert binding.error_string(0) == "ok"
    for code in (-1, -2, -3, -99):
        assert isinstance(binding.error_string(code), str) and binding.error_string(code)


def test_argument_checks_return_before_any_launch(lib):
    fake = ctypes.c_void_p(0x1000)       # never dereferenced: every call below fails validation first
    assert lib.dma_mx_quantize(None, 4, 128, 2, 0, fake, fake, None) == -1
    assert lib.dma_mx_quantize(fake, 4, 100, 2, 0, fake, fake, None) == -1          # D not a multiple of 32
    assert lib.dma_mx_quantize(fake, -1, 128, 2, 0, fake, fake, None) == -1
    assert lib.dma_mx_quantize(fake, 4, 128, 0, 0, fake, fake, None) == -1          # bf16 is not a quantized format
    assert lib.dma_mx_quantize(ctypes.c_void_p(0x1004), 4, 128, 2, 0, fake, fake, None) == -1   # misaligned
    assert lib.dma_mx_quantize_dual(fake, 4, 128, 0, fake, None, fake, fake, None) == -1
    assert lib.dma_mx_group_amax(fake, 2, 256, 128, 0, 0, 0, fake, None) == -1       # no such granularity
    assert lib.dma_mx_group_amax(fake, 2, 256, 128, 0, 2, 0, fake, None) == -1       # per-block needs block_rows > 0
    assert lib.dma_mx_group_amax(fake, 2, 256, 96, 0, 1, 0, fake, None) == -2        # head dimension 64 or 128 only
    assert lib.dma_mx_group_amax(None, 2, 256, 128, 0, 1, 0, fake, None) == -1
    assert lib.dma_mx_group_amax(fake, 0, 256, 128, 0, 1, 0, fake, None) == 0        # nothing to do
    args = dict(B=1, Hq=4, Hkv=2, S=256, D=128, causal=1, band=1, hi=1, lo=2)

    def attn(**kw):
        a = dict(args, **kw)
        return lib.dma_attn_fwd(fake, fake, fake, fake, a["B"], a["Hq"], a["Hkv"], a["S"], a["D"], a["causal"],
                                a["band"], a["hi"], a["lo"], None)
    assert attn(Hq=3) == -1                   # Hq % Hkv != 0
    assert attn(band=-1) == -1
    assert attn(hi=7) == -1
    assert attn(B=0) == -1
    assert attn(S=1 << 23) == -2              # one head of the output would not fit a 4 GiB buffer resource
    assert attn(S=(1 << 23) - 200) == -2      # ... nor may the rows of a filled-up last tile pair wrap around its offsets
    assert attn(D=96) == -2                   # no kernel for this head dimension
    assert attn(hi=2, lo=1) == -2             # unsupported format pair
    assert lib.dma_attn_fwd(None, fake, fake, fake, 1, 4, 2, 256, 128, 1, 1, 1, 2, None) == -1
    assert attn(hi=3, lo=1) == -2             # unsupported format pair (E5M2 over E4M3)
    def attn_ex(hi=1, **kw):
        opts = binding.AttnOpts(**{**dict(tile=128, sink_tiles=0, pv_fmt=0, per_token_scale=0, fp8_mfma=0), **kw})
        return lib.dma_attn_fwd_ex(fake, fake, fake, fake, 1, 4, 2, 256, 128, 1, 1, hi, 2, ctypes.byref(opts), None)
    assert attn_ex(sink_tiles=-1) == -1
    assert attn_ex(per_token_scale=2) == -1
    assert attn_ex(per_token_scale=1, fp8_mfma=1) == -2   # per-token scale only on the exact product paths
    assert attn_ex(pv_fmt=2) == -2            # P V formats: bf16 or MXFP8-E4M3 only
    assert attn_ex(per_token_scale=1, q_group_amax=0x1000) == -1     # group maxima: both or neither ...
    assert attn_ex(q_group_amax=0x1000, k_group_amax=0x1000) == -1     # ... and only with the Step-2 scale
    assert attn_ex(pv_fmt=1, per_token_scale=1) == -2   # MX-format P V: not with the per-token scale ...
    assert attn_ex(pv_fmt=1, hi=2) == -2      # ... and only for the default format pair
    assert attn_ex(hi=3, fp8_mfma=1) == -2    # E5M2 only has the decoded-to-bf16 path
    assert attn_ex(fp8_mfma=2) == -1
    assert lib.dma_attn_fwd_workspace_bytes(1, 32, 8, 32768, 128) == 0
    # the diagnostics
    assert lib.dma_diag_mfma(fake, fake, fake, fake, 3, fake, None) == -1            # E5M2 has no instruction path of its own
    assert lib.dma_diag_mfma(fake, fake, None, fake, 1, fake, None) == -1            # MX formats need both scale arrays
    assert lib.dma_diag_mfma(None, fake, None, None, 0, fake, None) == -1
    assert lib.dma_diag_mfma(fake, ctypes.c_void_p(0x1008), None, None, 0, fake, None) == -1   # misaligned
    assert lib.dma_diag_copy(fake, fake, 24, None) == -1                             # not a multiple of 16 bytes
    assert lib.dma_diag_copy(fake, fake, 0, None) == 0
    kinds = (ctypes.c_int * 3)(1, 4, 4)
    assert lib.dma_diag_pipes(kinds, 0, 100, fake, None, None) == -1                 # one to three slots
    assert lib.dma_diag_pipes(kinds, 4, 100, fake, None, None) == -1
    assert lib.dma_diag_pipes(kinds, 3, 0, fake, None, None) == -1                   # 1 .. 100 000 microseconds
    assert lib.dma_diag_pipes(kinds, 3, 100001, fake, None, None) == -1
    assert lib.dma_diag_pipes(kinds, 3, 100, None, None, None) == -1
    assert lib.dma_diag_pipes(kinds, 3, 100, ctypes.c_void_p(0x1004), None, None) == -1     # misaligned counters
    assert lib.dma_diag_pipes((ctypes.c_int * 3)(1, 7, 4), 3, 100, fake, None, None) == -1   # no such stream
    assert lib.dma_diag_pipes(None, 3, 100, fake, None, None) == -1
