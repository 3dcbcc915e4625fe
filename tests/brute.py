"""Brute-force, per-element definitions used to pin the CPU oracle (tiny inputs only).

Written from the definitions (nearest grid value, largest power of two not above a number, plain
row softmax), not from the oracle's formulas, and sharing no code with it.
"""
from __future__ import annotations

import numpy as np

# Representable magnitudes by code.  E2M1: Alg. 3 (bias 1, codes (E<<1)|M).  E4M3: OCP layout,
# bias 7, exponent field 15 is an ordinary binade (Sec. 4.2), 0x7F is not a number.
E2M1_GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
E4M3_GRID = np.array([(m * 2.0 ** -9) if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7)
                      for e in range(16) for m in range(8)][:0x7F])
# E5M2: bias 15, exponent field 31 reserved (infinities / NaN), so 0x7B = 57344 is the largest value.
E5M2_GRID = np.array([(m * 2.0 ** -16) if e == 0 else (1 + m / 4.0) * 2.0 ** (e - 15)
                      for e in range(31) for m in range(4)])
FORMATS = {"e2m1": (E2M1_GRID, 2, 8), "e4m3": (E4M3_GRID, 8, 0x80), "e5m2": (E5M2_GRID, 15, 0x80)}


def nearest_code(grid: np.ndarray, a: float) -> int:
    """Index of the grid value nearest to a >= 0; exact ties go to the even index; values beyond
    the largest grid value saturate."""
    a = float(a)
    if a >= grid[-1]:
        return len(grid) - 1
    d = np.abs(grid - a)               # exact: grid values and a are doubles with few bits
    best = np.flatnonzero(d == d.min())
    if len(best) == 1:
        return int(best[0])
    even = [int(b) for b in best if b % 2 == 0]
    return even[0]


def floor_log2(a: float) -> int:
    """Largest integer e with 2**e <= a, by search (a > 0)."""
    e = 0
    while 2.0 ** (e + 1) <= a:
        e += 1
    while 2.0 ** e > a:
        e -= 1
    return e


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def quantize_block(x32: np.ndarray, fmt: str):
    """One MX block (32 float32 values, already pre-scaled if a query).
    Returns (scale_byte, codes[32] with sign bit, decoded float64[32])."""
    grid, emax, signbit = FORMATS[fmt]
    amax = float(np.max(np.abs(x32)))
    if amax == 0.0:
        sb = 0
    else:
        sb = min(max(floor_log2(amax) - emax + 127, 0), 254)
    codes = np.zeros(32, dtype=np.uint8)
    dec = np.zeros(32)
    for t in range(32):
        y = float(x32[t]) * 2.0 ** (127 - sb)     # exact in double
        c = nearest_code(grid, abs(y))
        neg = bool(np.signbit(x32[t]))
        codes[t] = c | (signbit if neg else 0)
        dec[t] = (-grid[c] if neg else grid[c]) * 2.0 ** (sb - 127)
    return sb, codes, dec


def group_maxima(bits: np.ndarray, is_query: bool, granularity: str, block_rows: int = 0) -> np.ndarray:
    """bits [n_mat, S, D] -> float32 [n_mat, S]: the largest magnitude (queries: after the float32 pre-scale) in the
    group of each row: the row, the block of block_rows rows of its matrix, or everything."""
    n_mat, S, D = bits.shape
    x = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    if is_query:
        x = (x * np.float32(np.log2(np.e) / np.sqrt(np.float64(D)))).astype(np.float32)
    a = np.abs(x)
    out = np.zeros((n_mat, S), dtype=np.float32)
    for m_ in range(n_mat):
        for r in range(S):
            if granularity == "token":
                grp = a[m_, r]
            elif granularity == "block":
                r0 = (r // block_rows) * block_rows
                grp = a[m_, r0:r0 + block_rows]
            else:
                grp = a
            out[m_, r] = grp.max()
    return out


def quantize_rows(bits: np.ndarray, fmt: str, is_query: bool, per_token: bool = False, return_token_scale=False, amax=None):
    """bits: [rows, D] uint16.  Returns (scales[rows, D/32], codes[rows, D] unpacked, decoded[rows, D]).
    per_token: Alg. 2 Step 2: every row is first multiplied by 2688 / rowmax (float32), and the decoded row by
    rowmax / 2688 (float32); rows whose maximum is below 2^-100 are left alone."""
    rows, D = bits.shape
    x = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    if is_query:
        c = np.float32(np.log2(np.e) / np.sqrt(np.float64(D)))
        x = (x * c).astype(np.float32)            # one float32 multiply per element
    s_q = np.ones(rows, dtype=np.float32)
    if per_token:
        rmax = np.max(np.abs(x), axis=1).astype(np.float32) if amax is None else np.asarray(amax, dtype=np.float32)
        ok = rmax >= np.float32(2.0 ** -100)
        inv = np.ones(rows, dtype=np.float32)
        inv[ok] = np.float32(2688.0) / rmax[ok]
        s_q[ok] = rmax[ok] / np.float32(2688.0)
        x = (x * inv[:, None]).astype(np.float32)
    scales = np.zeros((rows, D // 32), dtype=np.uint8)
    codes = np.zeros((rows, D), dtype=np.uint8)
    dec = np.zeros((rows, D))
    for r in range(rows):
        for b in range(D // 32):
            sb, cd, de = quantize_block(x[r, 32 * b:32 * b + 32], fmt)
            scales[r, b] = sb
            codes[r, 32 * b:32 * b + 32] = cd
            dec[r, 32 * b:32 * b + 32] = de
    dec = dec * s_q.astype(np.float64)[:, None]
    if return_token_scale:
        return scales, codes, dec, s_q
    return scales, codes, dec


def pack_fp4(codes: np.ndarray) -> np.ndarray:
    """Two 4-bit codes per byte, the higher index in the high nibble (Alg. 2 Step 5)."""
    return (codes[..., 1::2].astype(np.uint8) << 4) | codes[..., 0::2].astype(np.uint8)


def round_bf16_nearest_of_two(p: np.ndarray) -> np.ndarray:
    """Round positive doubles to bf16 by comparing the two neighbouring bf16 numbers."""
    p = np.asarray(p, dtype=np.float64)
    out = np.zeros_like(p)
    nz = p > 0
    _, ex = np.frexp(p[nz])
    q = np.exp2((ex - 1 - 7).astype(np.float64))          # spacing of bf16 numbers around p
    q = np.maximum(q, 2.0 ** -133)
    lo_n = np.floor(p[nz] / q)
    lo, hi = lo_n * q, (lo_n + 1) * q
    dl, dh = p[nz] - lo, hi - p[nz]
    pick_hi = (dh < dl) | ((dh == dl) & (lo_n % 2 == 1))
    out[nz] = np.where(pick_hi, hi, lo)
    return out


def other_bf16_neighbour(p: np.ndarray, rounded: np.ndarray) -> np.ndarray:
    """For positive doubles p and their bf16 roundings: the bf16 number on the other side of p (p itself if exact)."""
    p = np.asarray(p, dtype=np.float64)
    _, ex = np.frexp(p)
    q = np.maximum(np.exp2((ex - 1 - 7).astype(np.float64)), 2.0 ** -133)
    lo = np.floor(p / q) * q
    return np.where(lo == p, rounded, np.where(rounded == lo, lo + q, lo))


def dma_attention(q_bits, k_bits, v_bits, *, tile, band, hi="e4m3", lo="e2m1", p_round=True, sink=0, causal=True,
                  score_dtype=np.float64, per_token=False, pv_mx=False, binary32_exponent=False, other_way=None, probe=None):
    """Per-element rewrite of the diagonal-tiled attention for q[Hq,S,D], k,v[Hkv,S,D] (one batch).

    For every visible pair (i, j) the score comes from the format of the tile pair (i // tile, j // tile):
    high when the tiles are closer than `band` or the key tile is one of the first `sink`; with
    p_round the probabilities are formed against the running maximum over key-tile prefixes and
    rounded to bf16, otherwise it is a plain base-2 row softmax.  causal=False: every key is visible.
    score_dtype=np.float32 rounds every score to binary32 first (what an implementation with binary32 scores sees).
    pv_mx: instead of the bf16 rounding, every block of 32 consecutive keys (aligned to multiples of 32, masked keys
    and keys past the end counting as zeros) of a row's probabilities, and of every column of V, is an MXFP8-E4M3 block.
    binary32_exponent: the probability that gets rounded is formed the way a binary32 implementation forms it (the row
    sum still adds the double-precision p, so only rounding decisions change).  True: the running maximum and the
    difference s - m' rounded to binary32, then 2^x rounded to binary32.  "chain": a running binary32 accumulator per
    key that starts at minus the binary32 running maximum and adds the exact partial product of one MX block after
    the other, rounding after each; the running maximum itself is a binary32 number that moves by binary32 additions;
    the accumulator is shifted by a binary32 subtraction when the maximum moves; then 2^x rounded to binary32.
    other_way: {(h, i): [keys]}: those probabilities of row i of head h take the OTHER of their two bf16 neighbours.
    probe: a dict that receives, per (h, i), the rounded probabilities of the row as they enter the second product."""
    Hq, S, D = q_bits.shape
    Hkv = k_bits.shape[0]
    g = Hq // Hkv
    out = np.zeros((Hq, S, D))
    v = bf16_bits_to_f64(v_bits)
    if pv_mx:
        v = np.stack([values_in_key_blocks(v[hk]) for hk in range(Hkv)])
    qam = kam = None
    if per_token in ("block", "tensor"):             # coarser granularities of the Step-2 scale: group maxima first
        qam = group_maxima(q_bits, True, per_token, tile)
        kam = group_maxima(k_bits, False, per_token, tile)
    pt = bool(per_token)
    for h in range(Hq):
        _, _, q_hi = quantize_rows(q_bits[h], hi, True, pt, amax=None if qam is None else qam[h])
        _, _, q_lo = quantize_rows(q_bits[h], lo, True, pt, amax=None if qam is None else qam[h])
        _, _, k_hi = quantize_rows(k_bits[h // g], hi, False, pt, amax=None if kam is None else kam[h // g])
        _, _, k_lo = quantize_rows(k_bits[h // g], lo, False, pt, amax=None if kam is None else kam[h // g])
        s_hi = q_hi @ k_hi.T
        s_lo = q_lo @ k_lo.T
        ti = np.arange(S)[:, None] // tile
        tj = np.arange(S)[None, :] // tile
        use_hi = (np.abs(ti - tj) < band) | (tj < sink)
        s = np.where(use_hi, s_hi, s_lo).astype(score_dtype).astype(np.float64)
        if binary32_exponent == "chain":
            nb = D // 32
            parts = np.where(use_hi[:, :, None],
                             np.einsum("ibd,jbd->ijb", q_hi.reshape(S, nb, 32), k_hi.reshape(S, nb, 32)),
                             np.einsum("ibd,jbd->ijb", q_lo.reshape(S, nb, 32), k_lo.reshape(S, nb, 32)))
        for i in range(S):
            nk = i + 1 if causal else S                  # keys this row sees
            si = s[i, :nk]
            if not p_round:
                p = np.exp2(si - si.max())
                out[h, i] = (p @ v[h // g, :nk]) / p.sum()
                continue
            nt = (nk + tile - 1) // tile
            # running maximum after each key tile
            run = np.array([si[:min((t + 1) * tile, nk)].max() for t in range(nt)])
            mj = run[np.arange(nk) // tile]              # maximum in force when key j was processed
            mfin = run[-1]
            p_at = np.exp2(si - mj)
            p_seen = p_at                                # the value the rounding decision is taken on
            if binary32_exponent == "chain":
                x32 = np.zeros(nk, dtype=np.float32)
                m_run, first = np.float32(0.0), True
                for t in range(nt):
                    j0, j1 = t * tile, min((t + 1) * tile, nk)
                    acc = np.full(j1 - j0, -m_run, dtype=np.float32)
                    for b in range(nb):
                        acc = (acc.astype(np.float64) + parts[i, j0:j1, b]).astype(np.float32)
                    delta = acc.max() if first else max(acc.max(), np.float32(0.0))
                    if delta != 0:
                        acc = (acc - np.float32(delta)).astype(np.float32)
                        m_run = np.float32(m_run + np.float32(delta))
                    x32[j0:j1] = acc
                    first = False
                p_seen = np.exp2(x32.astype(np.float64)).astype(np.float32).astype(np.float64)
            elif binary32_exponent:
                x32 = (si.astype(np.float32) - mj.astype(np.float32)).astype(np.float32)
                p_seen = np.exp2(x32.astype(np.float64)).astype(np.float32).astype(np.float64)
            if pv_mx:
                p_hat = np.zeros(nk)
                for b0 in range(0, nk, 32):
                    blk = np.zeros(32)
                    n = min(32, nk - b0)
                    blk[:n] = p_seen[b0:b0 + n]
                    p_hat[b0:b0 + n] = quantize_block(blk, "e4m3")[2][:n]
            else:
                p_hat = round_bf16_nearest_of_two(p_seen)
                if other_way and (h, i) in other_way:
                    jj = np.asarray(other_way[(h, i)], dtype=np.int64)
                    p_hat[jj] = other_bf16_neighbour(p_at[jj], p_hat[jj])
            if probe is not None:
                probe[(h, i)] = p_hat.copy()
            w_num = p_hat * np.exp2(mj - mfin)
            w_den = (p_at * np.exp2(mj - mfin)).sum()
            out[h, i] = (w_num @ v[h // g, :nk]) / w_den
    return out


def values_in_key_blocks(v: np.ndarray) -> np.ndarray:
    """v [S, D] real values -> every column cut into blocks of 32 consecutive keys (zero-padded at the end), each an
    MXFP8-E4M3 block; the decoded values, [S, D]."""
    S, D = v.shape
    out = np.zeros((S, D))
    for b0 in range(0, S, 32):
        n = min(32, S - b0)
        for d in range(D):
            blk = np.zeros(32)
            blk[:n] = v[b0:b0 + n, d]
            out[b0:b0 + n, d] = quantize_block(blk, "e4m3")[2][:n]
    return out


def softmax_attention_fp64(q, k, v, causal=True):
    """Plain softmax attention (causal or full) of real-valued q[Hq,S,D], k,v[Hkv,S,D] (doubles)."""
    Hq, S, D = q.shape
    g = Hq // k.shape[0]
    out = np.zeros((Hq, S, D))
    for h in range(Hq):
        s = (q[h] @ k[h // g].T) / np.sqrt(D)
        if causal:
            s = np.where(np.arange(S)[None, :] > np.arange(S)[:, None], -np.inf, s)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        out[h] = (p / p.sum(axis=1, keepdims=True)) @ v[h // g]
    return out
