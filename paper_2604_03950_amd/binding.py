"""Thin Python binding of the C-ABI library (``include/dma.h``): argument marshalling only.

Every function takes PyTorch tensors that live on the GPU, passes their device pointers and the
current HIP stream to the entry point of the same name, and raises ``DmaError`` on a non-zero
return code.  There is no CPU fallback: if ``libdma_mi355x.so`` has not been built
(``python -m paper_2604_03950_amd.build``) loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os

import torch

FMT_BF16 = 0
FMT_MXFP8_E4M3 = 1
FMT_MXFP4_E2M1 = 2
FMT_MXFP8_E5M2 = 3

EXPORTS = ("dma_mx_quantize", "dma_mx_quantize_token", "dma_mx_quantize_dual", "dma_mx_group_amax", "dma_attn_fwd", "dma_attn_fwd_ex",
           "dma_attn_fwd_workspace_bytes", "dma_diag_copy", "dma_diag_mfma", "dma_diag_pipes", "dma_error_string", "dma_version")

PIPE_IDLE, PIPE_MFMA_BF16, PIPE_MFMA_FP4, PIPE_MFMA_FP8, PIPE_FMA, PIPE_EXP, PIPE_CVT_PK_BF16 = range(7)

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdma_mi355x.so")
_lib = None


class DmaError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {error_string(code)} (code {code})")


class AttnOpts(ctypes.Structure):
    _fields_ = [("tile", ctypes.c_int), ("sink_tiles", ctypes.c_int), ("pv_fmt", ctypes.c_int),
                ("per_token_scale", ctypes.c_int), ("q_group_amax", ctypes.c_void_p), ("k_group_amax", ctypes.c_void_p),
                ("fp8_mfma", ctypes.c_int)]


def lib_path() -> str:
    return _LIB_PATH


def load() -> ctypes.CDLL:
    """Load the shared library (once).  Raises if it is missing: there is no other code path."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(f"{_LIB_PATH} not found: build it with `python -m paper_2604_03950_amd.build`")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.dma_mx_quantize.restype = ci
        L.dma_mx_quantize.argtypes = [vp, i64, ci, ci, ci, vp, vp, vp]
        L.dma_mx_quantize_token.restype = ci
        L.dma_mx_quantize_token.argtypes = [vp, i64, ci, ci, ci, vp, vp, vp, vp]
        L.dma_mx_group_amax.restype = ci
        L.dma_mx_group_amax.argtypes = [vp, i64, i64, ci, ci, ci, i64, vp, vp]
        L.dma_mx_quantize_dual.restype = ci
        L.dma_mx_quantize_dual.argtypes = [vp, i64, ci, ci, vp, vp, vp, vp, vp]
        L.dma_attn_fwd.restype = ci
        L.dma_attn_fwd.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, ci, vp]
        L.dma_attn_fwd_ex.restype = ci
        L.dma_attn_fwd_ex.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, ci, ctypes.POINTER(AttnOpts), vp]
        L.dma_attn_fwd_workspace_bytes.restype = ctypes.c_size_t
        L.dma_attn_fwd_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
        L.dma_diag_copy.restype = ci
        L.dma_diag_copy.argtypes = [vp, vp, i64, vp]
        L.dma_diag_mfma.restype = ci
        L.dma_diag_mfma.argtypes = [vp, vp, vp, vp, ci, vp, vp]
        L.dma_diag_pipes.restype = ci
        L.dma_diag_pipes.argtypes = [ctypes.POINTER(ci), ci, ci, vp, ctypes.POINTER(ci), vp]
        L.dma_error_string.restype = ctypes.c_char_p
        L.dma_error_string.argtypes = [ci]
        L.dma_version.restype = ci
        L.dma_version.argtypes = []
        _lib = L
    return _lib


def error_string(code: int) -> str:
    return load().dma_error_string(int(code)).decode()


def version() -> int:
    return int(load().dma_version())


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, dtype, what: str, shape=None) -> int:
    """Device pointer of a contiguous GPU tensor of the given dtype (and, for buffers the kernels write, shape: an
    undersized caller buffer would otherwise be written past its end)."""
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{what}: need a contiguous {dtype} tensor on the GPU")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{what}: shape {tuple(t.shape)}, expected {tuple(shape)}")
    return t.data_ptr()


def dma_mx_quantize(x: torch.Tensor, fmt: int, is_query: bool, codes: torch.Tensor | None = None,
                    scales: torch.Tensor | None = None):
    """x: [..., D] bf16 -> (codes uint8 [..., D] or [..., D/2], scales uint8 [..., D/32])."""
    D = x.shape[-1]
    rows = x.numel() // D
    cb = D // 2 if fmt == FMT_MXFP4_E2M1 else D
    if codes is None:
        codes = torch.empty(x.shape[:-1] + (cb,), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty(x.shape[:-1] + (D // 32,), dtype=torch.uint8, device=x.device)
    rc = load().dma_mx_quantize(_dev(x, torch.bfloat16, "x"), rows, D, fmt, int(bool(is_query)),
                                _dev(codes, torch.uint8, "codes", x.shape[:-1] + (cb,)),
                                _dev(scales, torch.uint8, "scales", x.shape[:-1] + (D // 32,)), _stream())
    if rc:
        raise DmaError(rc, "dma_mx_quantize")
    return codes, scales


def dma_mx_quantize_token(x: torch.Tensor, fmt: int, is_query: bool):
    """dma_mx_quantize with the per-token scale of Alg. 2 Step 2: returns (codes, scales, token_scales float32 [...])."""
    D = x.shape[-1]
    rows = x.numel() // D
    cb = D // 2 if fmt == FMT_MXFP4_E2M1 else D
    codes = torch.empty(x.shape[:-1] + (cb,), dtype=torch.uint8, device=x.device)
    scales = torch.empty(x.shape[:-1] + (D // 32,), dtype=torch.uint8, device=x.device)
    ts = torch.empty(x.shape[:-1], dtype=torch.float32, device=x.device)
    rc = load().dma_mx_quantize_token(_dev(x, torch.bfloat16, "x"), rows, D, fmt, int(bool(is_query)),
                                      _dev(codes, torch.uint8, "codes"), _dev(scales, torch.uint8, "scales"),
                                      _dev(ts, torch.float32, "token_scales"), _stream())
    if rc:
        raise DmaError(rc, "dma_mx_quantize_token")
    return codes, scales, ts


GRAN_TOKEN, GRAN_BLOCK, GRAN_TENSOR = 1, 2, 3


def dma_mx_group_amax(x: torch.Tensor, is_query: bool, granularity: int, block_rows: int = 0,
                      out: torch.Tensor | None = None) -> torch.Tensor:
    """x [..., S, D] bf16 -> float32 [..., S]: for every row the largest magnitude (queries: after the Step-1 pre-scale) of
    the group that shares its Step-2 scale: the row, block_rows rows of its [S, D] matrix, or all of x."""
    S, D = x.shape[-2], x.shape[-1]
    n_mat = x.numel() // (S * D)
    if out is None:
        out = torch.empty(x.shape[:-1], dtype=torch.float32, device=x.device)
    rc = load().dma_mx_group_amax(_dev(x, torch.bfloat16, "x"), n_mat, S, D, int(bool(is_query)), int(granularity),
                                  int(block_rows), _dev(out, torch.float32, "amax", x.shape[:-1]), _stream())
    if rc:
        raise DmaError(rc, "dma_mx_group_amax")
    return out


def dma_mx_quantize_dual(x: torch.Tensor, is_query: bool, out=None):
    """One read of x -> (codes_lo, scales_lo, codes_hi, scales_hi): MXFP4 E2M1 and MXFP8 E4M3 copies."""
    D = x.shape[-1]
    rows = x.numel() // D
    if out is None:
        mk = lambda n: torch.empty(x.shape[:-1] + (n,), dtype=torch.uint8, device=x.device)
        out = (mk(D // 2), mk(D // 32), mk(D), mk(D // 32))
    c4, s4, c8, s8 = out
    rc = load().dma_mx_quantize_dual(_dev(x, torch.bfloat16, "x"), rows, D, int(bool(is_query)),
                                     _dev(c4, torch.uint8, "codes_lo", x.shape[:-1] + (D // 2,)),
                                     _dev(s4, torch.uint8, "scales_lo", x.shape[:-1] + (D // 32,)),
                                     _dev(c8, torch.uint8, "codes_hi", x.shape[:-1] + (D,)),
                                     _dev(s8, torch.uint8, "scales_hi", x.shape[:-1] + (D // 32,)), _stream())
    if rc:
        raise DmaError(rc, "dma_mx_quantize_dual")
    return out


def dma_attn_fwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, *, diag_band_tiles: int,
                 hi_fmt: int = FMT_MXFP8_E4M3, lo_fmt: int = FMT_MXFP4_E2M1, causal: bool = True,
                 tile: int | None = None, fp8_mfma: bool = False, sink_tiles: int = 0, per_token_scale: bool = False,
                 pv_mx: bool = False, group_amax=None, out: torch.Tensor | None = None) -> torch.Tensor:
    """q [B,Hq,S,D], k/v [B,Hkv,S,D] bf16 -> out [B,Hq,S,D] float32.  With tile=None, fp8_mfma=False and
    sink_tiles=0 this is dma_attn_fwd (logical tile 128); otherwise dma_attn_fwd_ex with those options.
    pv_mx: the P V product in MXFP8-E4M3 with blocks of 32 keys (opts.pv_fmt) instead of 16-bit.
    group_amax: (q_amax [B,Hq,S], k_amax [B,Hkv,S]) float32 from dma_mx_group_amax: with per_token_scale, the Step-2 scale
    of a row comes from its group's maximum instead of its own."""
    B, Hq, S, D = q.shape
    Hkv = k.shape[1]
    if k.shape != (B, Hkv, S, D) or v.shape != k.shape:
        raise ValueError("k and v must be [B, Hkv, S, D] matching q")
    if out is None:
        out = torch.empty((B, Hq, S, D), dtype=torch.float32, device=q.device)
    args = [_dev(q, torch.bfloat16, "q"), _dev(k, torch.bfloat16, "k"), _dev(v, torch.bfloat16, "v"),
            _dev(out, torch.float32, "out", (B, Hq, S, D)), B, Hq, Hkv, S, D, int(bool(causal)), int(diag_band_tiles),
            int(hi_fmt), int(lo_fmt)]
    if tile is None and not fp8_mfma and not sink_tiles and not per_token_scale and not pv_mx and group_amax is None:
        rc = load().dma_attn_fwd(*args, _stream())
    else:
        qam = kam = None
        if group_amax is not None:
            qam = _dev(group_amax[0], torch.float32, "q_group_amax")
            kam = _dev(group_amax[1], torch.float32, "k_group_amax")
            if group_amax[0].shape != (B, Hq, S) or group_amax[1].shape != (B, Hkv, S):
                raise ValueError("group_amax must be ([B, Hq, S], [B, Hkv, S])")
        opts = AttnOpts(tile=int(tile or 0), sink_tiles=int(sink_tiles), pv_fmt=FMT_MXFP8_E4M3 if pv_mx else FMT_BF16, per_token_scale=int(bool(per_token_scale)),
                        q_group_amax=qam, k_group_amax=kam,
                        fp8_mfma=int(bool(fp8_mfma)))
        rc = load().dma_attn_fwd_ex(*args, ctypes.byref(opts), _stream())
    if rc:
        raise DmaError(rc, "dma_attn_fwd")
    return out


def dma_diag_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    """Plain copy kernel over the bytes of two equally sized contiguous GPU tensors (counter calibration)."""
    n = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != n or not (src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()):
        raise ValueError("dma_diag_copy: need two contiguous GPU tensors of equal byte size")
    rc = load().dma_diag_copy(src.data_ptr(), dst.data_ptr(), n, _stream())
    if rc:
        raise DmaError(rc, "dma_diag_copy")


def dma_diag_mfma(a: torch.Tensor, b: torch.Tensor, a_scales: torch.Tensor | None, b_scales: torch.Tensor | None, fmt: int) -> torch.Tensor:
    """One 32 x 32 x 64 product on the matrix instruction of format fmt (diagnostic): a, b uint8 [32, 64] (E4M3 codes) or
    [32, 32] (packed E2M1 codes) with scales uint8 [32, 2], or bf16 [32, 64] without scales -> float32 [32, 32]."""
    if fmt == FMT_BF16:
        pa, pb, psa, psb = _dev(a, torch.bfloat16, "a", (32, 64)), _dev(b, torch.bfloat16, "b", (32, 64)), None, None
    else:
        cols = 32 if fmt == FMT_MXFP4_E2M1 else 64
        pa, pb = _dev(a, torch.uint8, "a", (32, cols)), _dev(b, torch.uint8, "b", (32, cols))
        psa, psb = _dev(a_scales, torch.uint8, "a_scales", (32, 2)), _dev(b_scales, torch.uint8, "b_scales", (32, 2))
    out = torch.empty((32, 32), dtype=torch.float32, device=a.device)
    rc = load().dma_diag_mfma(pa, pb, psa, psb, int(fmt), out.data_ptr(), _stream())
    if rc:
        raise DmaError(rc, "dma_diag_mfma")
    return out


def dma_diag_pipes(kinds, microseconds: int = 300) -> tuple[list[int], int]:
    """Instruction streams kinds[s] (PIPE_* ids, one to three) side by side on every SIMD for `microseconds` (diagnostic).
    Returns (instructions issued per slot, summed over all waves; workgroups launched): a slot has 4 waves per workgroup."""
    kinds = [int(k) for k in kinds]
    counts = torch.zeros(3, dtype=torch.int64, device="cuda")
    arr = (ctypes.c_int * len(kinds))(*kinds)
    wgs = ctypes.c_int(0)
    rc = load().dma_diag_pipes(arr, len(kinds), int(microseconds), counts.data_ptr(), ctypes.byref(wgs), _stream())
    if rc:
        raise DmaError(rc, "dma_diag_pipes")
    return [int(c) for c in counts.cpu().tolist()[:len(kinds)]], int(wgs.value)


def bits_to_bf16_tensor(bits, device="cuda") -> torch.Tensor:
    """uint16 numpy bit patterns -> bf16 tensor on the GPU (no value conversion)."""
    import numpy as np
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.view(torch.bfloat16).to(device)
