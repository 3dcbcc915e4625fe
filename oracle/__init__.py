"""CPU oracle for Diagonal-Tiled Mixed-Precision Attention -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``dma_oracle.c`` (plain C, double arithmetic).  Only the tests, the smoke
check and the benchmark's CPU-baseline leg may import this package; the GPU library and its
Python binding never do, and nothing here imports them.

bf16 tensors are passed as ``numpy.uint16`` arrays holding the raw bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

FMT_BF16 = 0
FMT_E4M3 = 1
FMT_E2M1 = 2
FMT_E5M2 = 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dma_oracle.c")
_LIB = os.path.join(_HERE, "libdma_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile dma_oracle.c with gcc (-O2, no fast-math, OpenMP) into libdma_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared",
               "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        u16p, u8p, i64p = (ctypes.POINTER(ctypes.c_uint16), ctypes.POINTER(ctypes.c_uint8),
                           ctypes.POINTER(ctypes.c_int64))
        f32p, f64p = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)
        L.oracle_bf16_to_f32.restype = ctypes.c_float
        L.oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.oracle_round_to_bf16.restype = ctypes.c_double
        L.oracle_round_to_bf16.argtypes = [ctypes.c_double]
        L.oracle_e2m1_decode.restype = ctypes.c_double
        L.oracle_e2m1_decode.argtypes = [ctypes.c_uint8]
        L.oracle_e2m1_encode.restype = ctypes.c_uint8
        L.oracle_e2m1_encode.argtypes = [ctypes.c_double, ctypes.c_int]
        L.oracle_e4m3_decode.restype = ctypes.c_double
        L.oracle_e4m3_decode.argtypes = [ctypes.c_uint8]
        L.oracle_e4m3_encode.restype = ctypes.c_uint8
        L.oracle_e4m3_encode.argtypes = [ctypes.c_double, ctypes.c_int]
        L.oracle_e5m2_decode.restype = ctypes.c_double
        L.oracle_e5m2_decode.argtypes = [ctypes.c_uint8]
        L.oracle_e5m2_encode.restype = ctypes.c_uint8
        L.oracle_e5m2_encode.argtypes = [ctypes.c_double, ctypes.c_int]
        L.oracle_e8m0_from_amax.restype = ctypes.c_uint8
        L.oracle_e8m0_from_amax.argtypes = [ctypes.c_float, ctypes.c_int]
        L.oracle_query_prescale.restype = ctypes.c_float
        L.oracle_query_prescale.argtypes = [ctypes.c_int]
        L.oracle_mx_quantize.restype = ctypes.c_int
        L.oracle_mx_quantize.argtypes = [u16p, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, u8p, u8p]
        L.oracle_mx_quantize_ex.restype = ctypes.c_int
        L.oracle_mx_quantize_ex.argtypes = [u16p, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, u8p, u8p, f32p]
        L.oracle_mx_dequantize.restype = ctypes.c_int
        L.oracle_mx_dequantize.argtypes = [u8p, u8p, ctypes.c_int64, ctypes.c_int, ctypes.c_int, f64p]
        L.oracle_dma_attn_rows.restype = ctypes.c_int
        L.oracle_dma_attn_rows.argtypes = [u16p, u16p, u16p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_int, ctypes.c_int, ctypes.c_int, i64p, ctypes.c_int64, f32p]
        L.oracle_dma_attn_rows_ex.restype = ctypes.c_int
        L.oracle_dma_attn_rows_ex.argtypes = [u16p, u16p, u16p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_int, i64p, ctypes.c_int64, f32p]
        i32p = ctypes.POINTER(ctypes.c_int32)
        L.oracle_dma_attn_row_alt.restype = ctypes.c_int
        L.oracle_dma_attn_row_alt.argtypes = [u16p, u16p, u16p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                              i64p, i32p, ctypes.c_int64, f32p, ctypes.c_double, ctypes.c_int64,
                                              i64p, i32p, f64p, f64p, i64p]
        L.oracle_ref_attn_rows.restype = ctypes.c_int
        L.oracle_ref_attn_rows.argtypes = [u16p, u16p, u16p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_int64, ctypes.c_int, i64p, ctypes.c_int64, f64p]
        L.oracle_ref_attn_rows_ex.restype = ctypes.c_int
        L.oracle_ref_attn_rows_ex.argtypes = [u16p, u16p, u16p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_int64, ctypes.c_int, ctypes.c_int, i64p, ctypes.c_int64, f64p]
        L.oracle_group_amax.restype = ctypes.c_int
        L.oracle_group_amax.argtypes = [u16p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                        ctypes.c_int64, f32p]
        L.oracle_mx_quantize_grouped.restype = ctypes.c_int
        L.oracle_mx_quantize_grouped.argtypes = [u16p, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, f32p, u8p, u8p, f32p]
        L.oracle_values_as_seen_mxfp8.restype = ctypes.c_int
        L.oracle_values_as_seen_mxfp8.argtypes = [u16p, ctypes.c_int64, ctypes.c_int, ctypes.c_int64, f64p, u8p]
        L.oracle_num_threads.restype = ctypes.c_int
        L.oracle_num_threads.argtypes = []
        _lib = L
    return _lib


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _as_bits(x) -> np.ndarray:
    a = np.ascontiguousarray(x)
    if a.dtype != np.uint16:
        raise TypeError("bf16 data must be passed as uint16 bit patterns")
    return a


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"{what} failed with code {rc}")


# ---- scalar helpers (used by the pins) ---------------------------------------------------------

def bf16_to_f32(bits: int) -> float:
    return float(lib().oracle_bf16_to_f32(int(bits)))


def round_to_bf16(p: float) -> float:
    return float(lib().oracle_round_to_bf16(float(p)))


def e2m1_encode(y: float) -> int:
    neg = 1 if np.signbit(y) else 0
    return int(lib().oracle_e2m1_encode(float(y), neg))


def e2m1_decode(code: int) -> float:
    return float(lib().oracle_e2m1_decode(int(code)))


def e4m3_encode(y: float) -> int:
    neg = 1 if np.signbit(y) else 0
    return int(lib().oracle_e4m3_encode(float(y), neg))


def e4m3_decode(code: int) -> float:
    return float(lib().oracle_e4m3_decode(int(code)))


def e5m2_encode(y: float) -> int:
    neg = 1 if np.signbit(y) else 0
    return int(lib().oracle_e5m2_encode(float(y), neg))


def e5m2_decode(code: int) -> float:
    return float(lib().oracle_e5m2_decode(int(code)))


def e8m0_from_amax(amax: float, fmt: int) -> int:
    return int(lib().oracle_e8m0_from_amax(float(np.float32(amax)), int(fmt)))


def query_prescale(D: int) -> float:
    return float(lib().oracle_query_prescale(int(D)))


def num_threads() -> int:
    return int(lib().oracle_num_threads())


# ---- tensor functions --------------------------------------------------------------------------

def mx_quantize(x_bits, fmt: int, is_query: bool, per_token: bool = False):
    """x_bits: [..., D] uint16 (bf16 bits).  Returns (codes uint8 [..., D or D/2], scales uint8 [..., D/32]) and,
    with per_token (Alg. 2 Step 2), also the per-row scale S_q as float32 [...]."""
    x = _as_bits(x_bits)
    D = x.shape[-1]
    rows = x.size // D
    cb = D // 2 if fmt == FMT_E2M1 else D
    codes = np.zeros(x.shape[:-1] + (cb,), dtype=np.uint8)
    scales = np.zeros(x.shape[:-1] + (D // 32,), dtype=np.uint8)
    if per_token:
        ts = np.zeros(x.shape[:-1], dtype=np.float32)
        _check(lib().oracle_mx_quantize_ex(_p(x, ctypes.c_uint16), rows, D, fmt, int(bool(is_query)),
                                           _p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint8), _p(ts, ctypes.c_float)),
               "oracle_mx_quantize_ex")
        return codes, scales, ts
    _check(lib().oracle_mx_quantize(_p(x, ctypes.c_uint16), rows, D, fmt, int(bool(is_query)),
                                    _p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint8)), "oracle_mx_quantize")
    return codes, scales


def mx_dequantize(codes, scales, fmt: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    D = scales.shape[-1] * 32
    rows = scales.size // scales.shape[-1]
    out = np.empty(scales.shape[:-1] + (D,), dtype=np.float64)
    _check(lib().oracle_mx_dequantize(_p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint8), rows, D, fmt,
                                      _p(out, ctypes.c_double)), "oracle_mx_dequantize")
    return out


def sort_rows(rows) -> np.ndarray:
    """Order (b, hq, i) triples so that rows of one (b, hq) are adjacent (the C loops then reuse the
    decoded keys of a kv head when consecutive q heads share it)."""
    r = np.asarray(rows, dtype=np.int64).reshape(-1, 3)
    order = np.lexsort((r[:, 2], r[:, 1], r[:, 0]))
    return np.ascontiguousarray(r[order])


def dma_attn_rows(q_bits, k_bits, v_bits, rows, *, tile: int, band: int, hi_fmt: int = FMT_E4M3,
                  lo_fmt: int = FMT_E2M1, p_round: bool = True, sink: int = 0, causal: bool = True,
                  per_token: bool = False, pv_mx: bool = False):
    """Diagonal-tiled attention output for the given (b, hq, i) rows -> float32 [n_rows, D].
    sink: number of leading key tiles kept in the high format; causal=False: every key tile is visited and the
    high-precision window is |jt - it| < band.  per_token: Alg. 2 Step 2 on queries and keys (True / "token": from the
    row's own maximum; "block": from the maximum of the row's tile of its head; "tensor": from the maximum of Q resp. K).
    pv_mx: the MX-format P V product (P and V in MXFP8-E4M3 with blocks of 32 keys) instead of the 16-bit one."""
    q, k, v = _as_bits(q_bits), _as_bits(k_bits), _as_bits(v_bits)
    B, Hq, S, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (B, Hkv, S, D) and v.shape == k.shape
    r = np.ascontiguousarray(np.asarray(rows, dtype=np.int64).reshape(-1, 3))
    out = np.empty((r.shape[0], D), dtype=np.float32)
    _check(lib().oracle_dma_attn_rows_ex(_p(q, ctypes.c_uint16), _p(k, ctypes.c_uint16), _p(v, ctypes.c_uint16),
                                         B, Hq, Hkv, S, D, tile, band, int(sink), int(bool(causal)), granularity_id(per_token),
                                         hi_fmt, lo_fmt,
                                         2 if pv_mx else int(bool(p_round)), _p(r, ctypes.c_int64), r.shape[0],
                                         _p(out, ctypes.c_float)),
           "oracle_dma_attn_rows_ex")
    return out


# Rounding decisions a parity test may ask to see taken the other way (dma_attn_row_alt)
ALT_NEIGHBOUR, ALT_SCALE_UP, ALT_SCALE_DOWN = 1, 2, 3


def _row_alt(q_bits, k_bits, v_bits, row, alts, cand, *, tile, band, hi_fmt=FMT_E4M3, lo_fmt=FMT_E2M1, sink=0, causal=True,
             per_token=False, pv_mx=False):
    q, k, v = _as_bits(q_bits), _as_bits(k_bits), _as_bits(v_bits)
    B, Hq, S, D = q.shape
    Hkv = k.shape[1]
    b, hq, i = (int(x) for x in row)
    keys = np.ascontiguousarray([a[0] for a in alts], dtype=np.int64)
    kinds = np.ascontiguousarray([a[1] for a in alts], dtype=np.int32)
    out = np.empty(D, dtype=np.float32)
    if cand is None:
        min_move, max_cand, ck, cn, cm, cr, nc = 0.0, 0, None, None, None, None, None
    else:
        min_move, max_cand = cand
        ck = np.zeros(max_cand, dtype=np.int64)
        cn = np.zeros(max_cand, dtype=np.int32)
        cm = np.zeros((max_cand, D), dtype=np.float64)
        cr = np.zeros(max_cand, dtype=np.float64)
        nc = np.zeros(1, dtype=np.int64)
    _check(lib().oracle_dma_attn_row_alt(_p(q, ctypes.c_uint16), _p(k, ctypes.c_uint16), _p(v, ctypes.c_uint16),
                                         B, Hq, Hkv, S, D, tile, band, int(sink), int(bool(causal)), granularity_id(per_token),
                                         hi_fmt, lo_fmt, 2 if pv_mx else 1, b, hq, i,
                                         _p(keys, ctypes.c_int64) if len(alts) else None,
                                         _p(kinds, ctypes.c_int32) if len(alts) else None, len(alts), _p(out, ctypes.c_float),
                                         float(min_move), int(max_cand),
                                         None if ck is None else _p(ck, ctypes.c_int64),
                                         None if cn is None else _p(cn, ctypes.c_int32),
                                         None if cm is None else _p(cm, ctypes.c_double),
                                         None if cr is None else _p(cr, ctypes.c_double),
                                         None if nc is None else _p(nc, ctypes.c_int64)),
           "oracle_dma_attn_row_alt")
    if cand is None:
        return out
    n = int(min(nc[0], max_cand))
    return out, [(int(ck[t]), int(cn[t])) for t in range(n)], cm[:n], int(nc[0]), cr[:n]


def dma_attn_row_alt(q_bits, k_bits, v_bits, row, alts, **kw) -> np.ndarray:
    """The row (b, hq, i) with the rounding decisions `alts` = [(key, ALT_*), ...] taken the other way -> float32 [D].
    Keywords as dma_attn_rows (the probabilities are always rounded: p_round is not one of them)."""
    return _row_alt(q_bits, k_bits, v_bits, row, list(alts), None, **kw)


def dma_attn_row_candidates(q_bits, k_bits, v_bits, row, *, min_move: float = 0.0, max_cand: int = 16, **kw):
    """The rounding decisions of the row (b, hq, i) that an implementation with binary32 scores may take the other way
    (see oracle_dma_attn_row_alt in dma_oracle.c): (row output float32 [D], [(key, ALT_*), ...] with the largest effect first
    (at most max_cand), their first-order effect on the output float64 [n, D], the number of all such decisions whose
    effect reaches min_move, and per listed decision the share of the noise allowance it uses, 0 .. 1)."""
    return _row_alt(q_bits, k_bits, v_bits, row, [], (min_move, max_cand), **kw)


GRANULARITY = {False: 0, None: 0, True: 1, "token": 1, "block": 2, "tensor": 3}


def granularity_id(per_token) -> int:
    """per_token argument -> 0 (no Step 2), 1 (per-token), 2 (per-block: the rows of one tile of one head), 3 (per-tensor)."""
    return GRANULARITY[per_token]


def group_amax(x_bits, is_query: bool, granularity, block_rows: int = 0) -> np.ndarray:
    """x_bits: [..., S, D] bf16 bits.  Maximum magnitude (after the query pre-scale) of the group every row belongs to:
    the row ("token"), block_rows consecutive rows of one [S, D] matrix ("block"), everything ("tensor"); float32 [..., S]."""
    x = _as_bits(x_bits)
    S, D = x.shape[-2], x.shape[-1]
    n_mat = x.size // (S * D)
    out = np.empty(x.shape[:-1], dtype=np.float32)
    _check(lib().oracle_group_amax(_p(x, ctypes.c_uint16), n_mat, S, D, int(bool(is_query)), granularity_id(granularity),
                                   int(block_rows), _p(out, ctypes.c_float)), "oracle_group_amax")
    return out


def mx_quantize_grouped(x_bits, fmt: int, is_query: bool, amax):
    """Alg. 2 with Step 2 driven by the given group maxima (float32 [...], one per row): (codes, scales, S_q)."""
    x = _as_bits(x_bits)
    D = x.shape[-1]
    rows = x.size // D
    am = np.ascontiguousarray(amax, dtype=np.float32).reshape(-1)
    assert am.size == rows
    cb = D // 2 if fmt == FMT_E2M1 else D
    codes = np.zeros(x.shape[:-1] + (cb,), dtype=np.uint8)
    scales = np.zeros(x.shape[:-1] + (D // 32,), dtype=np.uint8)
    ts = np.zeros(x.shape[:-1], dtype=np.float32)
    _check(lib().oracle_mx_quantize_grouped(_p(x, ctypes.c_uint16), rows, D, fmt, int(bool(is_query)), _p(am, ctypes.c_float),
                                            _p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint8), _p(ts, ctypes.c_float)),
           "oracle_mx_quantize_grouped")
    return codes, scales, ts


def values_as_seen_mxfp8(v_bits):
    """V of one kv head, [S, D] bf16 bits, as the MX-format P V product sees it: (decoded values float64 [S, D],
    scale bytes uint8 [ceil(S/32), D]); blocks of 32 consecutive keys per column, zero-padded past S."""
    v = _as_bits(v_bits)
    S, D = v.shape
    seen = np.empty((S, D), dtype=np.float64)
    scales = np.empty(((S + 31) // 32, D), dtype=np.uint8)
    _check(lib().oracle_values_as_seen_mxfp8(_p(v, ctypes.c_uint16), S, D, S, _p(seen, ctypes.c_double),
                                             _p(scales, ctypes.c_uint8)), "oracle_values_as_seen_mxfp8")
    return seen, scales


def all_rows(B: int, Hq: int, S: int) -> np.ndarray:
    b, h, i = np.meshgrid(np.arange(B), np.arange(Hq), np.arange(S), indexing="ij")
    return np.stack([b.ravel(), h.ravel(), i.ravel()], axis=1).astype(np.int64)


def dma_attn(q_bits, k_bits, v_bits, **kw) -> np.ndarray:
    """Full output [B, Hq, S, D] float32 (small problems only)."""
    B, Hq, S, D = q_bits.shape
    return dma_attn_rows(q_bits, k_bits, v_bits, all_rows(B, Hq, S), **kw).reshape(B, Hq, S, D)


def ref_attn_rows(q_bits, k_bits, v_bits, rows, causal: bool = True) -> np.ndarray:
    """Exact softmax attention of the unquantized inputs (causal or full), float64 [n_rows, D]."""
    q, k, v = _as_bits(q_bits), _as_bits(k_bits), _as_bits(v_bits)
    B, Hq, S, D = q.shape
    Hkv = k.shape[1]
    r = np.ascontiguousarray(np.asarray(rows, dtype=np.int64).reshape(-1, 3))
    out = np.empty((r.shape[0], D), dtype=np.float64)
    _check(lib().oracle_ref_attn_rows_ex(_p(q, ctypes.c_uint16), _p(k, ctypes.c_uint16), _p(v, ctypes.c_uint16),
                                         B, Hq, Hkv, S, D, int(bool(causal)), _p(r, ctypes.c_int64), r.shape[0],
                                         _p(out, ctypes.c_double)), "oracle_ref_attn_rows_ex")
    return out
