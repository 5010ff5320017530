"""TEST INFRASTRUCTURE: Python face of the fp64 CPU oracle.

* ``attention`` / ``attention_rows`` marshal numpy arrays into the C routine of
  ``ifx_oracle.c`` (plain three-pass softmax attention over cache + block, the
  operation of the paper's Introduction, framework paragraph).
* ``BlockCacheOracle`` is the generate-and-cache loop's cache (same paragraph:
  after a block is generated its K/V update the cache) with the sliding-window,
  whole-block eviction the paper's KV Management section asks for.  It is a
  ``collections.deque`` of byte copies: append at the back, drop the front when
  full.  No modular slot arithmetic appears here on purpose; the HIP library
  uses slot arithmetic and the two are compared bit for bit.

Nothing here is imported by the product path.
"""
from __future__ import annotations

import collections
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ifx_oracle.c")
_LIB = os.path.join(_HERE, "libifx_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ifx_oracle.c with gcc (OpenMP) next to its source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", _SRC, "-o", _LIB, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        lib.ifx_oracle_attention.restype = ctypes.c_int
        lib.ifx_oracle_attention.argtypes = [
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
            dp, dp, dp, dp, dp, ctypes.c_double,
            ctypes.c_int64, ip, ip, dp, dp,
        ]
        lib.ifx_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    """OpenMP threads the attention routine uses."""
    return int(_load().ifx_oracle_threads())


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Widen raw bfloat16 bit patterns (uint16) exactly to float64."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    with np.errstate(invalid="ignore"):  # signalling-NaN patterns are quieted by the cast
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ---- fp8 cache variant (KV Management section: a compressed KV store; Challenges section: KV-cache
# quantisation and compression) -----------------------------------------------------------------
# The paper names no format.  The reading taken: OCP FP8 E4M3 ("e4m3fn": 1 sign, 4 exponent bits with
# bias 7, 3 mantissa bits; exponent 0 holds subnormals m/8 * 2^-6; exponent 15 with mantissa 7 is
# NaN, there are no infinities; largest magnitude 448), no scale factors, one code per element.
# A block is rounded to that format when it is committed: to the nearest code, ties to the even
# code, magnitudes beyond 448 (infinities included) to +-448, NaN to NaN.  Attention then reads the
# rounded values exactly (every E4M3 value is a bfloat16 value).

def e4m3_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """The value of every FP8 E4M3 code (uint8), from the format's definition, as float64."""
    bits = np.ascontiguousarray(bits, dtype=np.uint8).astype(np.int64)
    sign = np.where(bits & 0x80, -1.0, 1.0)
    e = (bits >> 3) & 0xF
    m = bits & 0x7
    normal = np.ldexp(1.0 + m / 8.0, e - 7)
    subnormal = np.ldexp(m / 8.0, -6)
    val = sign * np.where(e == 0, subnormal, normal)
    return np.where((e == 15) & (m == 7), np.nan, val)


def quantize_e4m3(x: np.ndarray) -> np.ndarray:
    """float64 values -> FP8 E4M3 codes (uint8) by the commit's rounding rule, written out as a
    search: among the 127 finite non-negative values of the format (code c has the c-th smallest
    value) take the one nearest to min(|x|, 448); of two equally near ones the one with the even
    code; then put the sign back."""
    x = np.asarray(x, dtype=np.float64)
    table = e4m3_bits_to_f64(np.arange(127, dtype=np.uint8))  # ascending: 0, 2^-9, ..., 448
    mag = np.minimum(np.abs(x), 448.0)
    mag = np.where(np.isnan(x), 0.0, mag)
    hi = np.clip(np.searchsorted(table, mag, side="left"), 0, 126)  # first code whose value is >= mag
    lo = np.maximum(hi - 1, 0)
    d_lo, d_hi = mag - table[lo], table[hi] - mag
    code = np.where(d_lo < d_hi, lo, np.where(d_hi < d_lo, hi, np.where(lo % 2 == 0, lo, hi)))
    code = np.where(np.isnan(x), 0x7F, code).astype(np.uint8)
    return (code | np.where(np.signbit(x), 0x80, 0).astype(np.uint8)).astype(np.uint8)


def bf16_bits_through_e4m3(bits: np.ndarray) -> np.ndarray:
    """What an fp8 cache holds for a block given as bfloat16 bit patterns (uint16), again as
    bfloat16 bit patterns: each element rounded to E4M3 and widened back (exactly)."""
    q = e4m3_bits_to_f64(quantize_e4m3(bf16_bits_to_f64(bits)))
    with np.errstate(invalid="ignore"):
        return (q.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)


def _f64(a, shape):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if a.shape != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def attention_rows(q, kc, vc, kb, vb, rows, heads, scale=None):
    """Oracle attention for selected (row, head) pairs.

    q, kb, vb: [n, H, D]; kc, vc: [C, H, D] (C may be 0, or None).  kb = vb = None: the key set
    is the C cached tokens alone.
    rows, heads: equal-length integer sequences.  Returns (out [S, D], lse [S]).
    """
    q = np.ascontiguousarray(q, dtype=np.float64)
    n, H, D = q.shape
    if (kb is None) != (vb is None):
        raise ValueError("kb and vb must both be given or both be None")
    if kb is not None:
        kb = _f64(kb, (n, H, D))
        vb = _f64(vb, (n, H, D))
    if kc is None or len(kc) == 0:
        C = 0
        kc = vc = None
    else:
        C = int(np.shape(kc)[0])
        kc = _f64(kc, (C, H, D))
        vc = _f64(vc, (C, H, D))
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    heads = np.ascontiguousarray(heads, dtype=np.int64)
    if rows.shape != heads.shape or rows.ndim != 1:
        raise ValueError("rows and heads must be 1-D and of equal length")
    S = rows.shape[0]
    out = np.empty((S, D), dtype=np.float64)
    lse = np.empty((S,), dtype=np.float64)
    dp = ctypes.POINTER(ctypes.c_double)
    ip = ctypes.POINTER(ctypes.c_int64)

    def p(a):
        return a.ctypes.data_as(dp) if a is not None else ctypes.cast(None, dp)

    rc = _load().ifx_oracle_attention(
        n, C, H, D, p(q), p(kc), p(vc), p(kb), p(vb), float(scale),
        S, rows.ctypes.data_as(ip), heads.ctypes.data_as(ip), p(out), p(lse),
    )
    if rc != 0:
        raise RuntimeError("ifx_oracle_attention rejected its arguments")
    return out, lse


def attention(q, kc, vc, kb, vb, scale=None):
    """Oracle attention for every row and head.  Returns (out [n,H,D], lse [n,H])."""
    n, H, D = np.shape(q)
    rows = np.repeat(np.arange(n, dtype=np.int64), H)
    heads = np.tile(np.arange(H, dtype=np.int64), n)
    out, lse = attention_rows(q, kc, vc, kb, vb, rows, heads, scale)
    return out.reshape(n, H, D), lse.reshape(n, H)


def merge(out_a, lse_a, out_b, lse_b):
    """Combine attention results over two disjoint key sets (paper, Parallelism section: ring
    attention computes attention per chunk of keys and combines the partial results).

    With L_x = ln sum_j exp(s_ij) over key set x, the softmax weight of set a inside the union is
    e^{L_a} / (e^{L_a} + e^{L_b}).  Returns (out [.., D], lse [..]) in fp64.
    """
    out_a, out_b = np.asarray(out_a, np.float64), np.asarray(out_b, np.float64)
    lse_a, lse_b = np.asarray(lse_a, np.float64), np.asarray(lse_b, np.float64)
    top = np.maximum(lse_a, lse_b)
    ea, eb = np.exp(lse_a - top), np.exp(lse_b - top)
    tot = ea + eb
    out = (ea / tot)[..., None] * out_a + (eb / tot)[..., None] * out_b
    return out, top + np.log(tot)


class BlockCacheOracle:
    """Per-layer cache of whole blocks with first-in-first-out eviction.

    Holds at most ``capacity_blocks`` blocks.  ``commit`` appends a byte-exact
    copy of the block's K and V; when the cache is already full the oldest block
    is dropped first.  ``ordinals`` lists the resident blocks oldest first
    (ordinal = how many blocks had been committed before it).
    """

    def __init__(self, capacity_blocks: int):
        if capacity_blocks <= 0:
            raise ValueError("capacity_blocks must be positive")
        self.capacity_blocks = int(capacity_blocks)
        self._blocks = collections.deque()
        self._committed = 0

    def commit(self, k_blk: np.ndarray, v_blk: np.ndarray) -> None:
        if len(self._blocks) == self.capacity_blocks:
            self._blocks.popleft()
        self._blocks.append((self._committed, np.array(k_blk, copy=True), np.array(v_blk, copy=True)))
        self._committed += 1

    def reset(self) -> None:
        self._blocks.clear()
        self._committed = 0

    def grow(self, capacity_blocks: int) -> None:
        """More room (paper, abstract: variable-length generation): nothing is lost, the window
        only starts to evict again once the larger capacity is full."""
        if capacity_blocks <= self.capacity_blocks:
            raise ValueError("the new capacity must be larger")
        self.capacity_blocks = int(capacity_blocks)

    @property
    def committed(self) -> int:
        return self._committed

    @property
    def ordinals(self):
        return [o for (o, _, _) in self._blocks]

    def tokens(self) -> int:
        return sum(k.shape[0] for (_, k, _) in self._blocks)

    def logical(self, ranges=None, blocks=None):
        """(K, V) of resident blocks, oldest first, concatenated along tokens.

        ranges: None for all of them, else (first_block, block_count) pairs counted from the
        oldest resident block (paper, KV Management section: range-based chunked access).
        blocks: instead of ranges, a list of block numbers counted the same way, taken in the
        list's order (same section: index-based selective fetch).
        """
        resident = list(self._blocks)
        if ranges is not None and blocks is not None:
            raise ValueError("ranges or blocks, not both")
        if blocks is not None:
            if len(set(blocks)) != len(blocks) or any(b < 0 or b >= len(resident) for b in blocks):
                raise IndexError("block list names a block twice or one that is not resident")
            resident = [resident[b] for b in blocks]
        if ranges is not None:
            picked = []
            for first, count in ranges:
                if first < 0 or count < 0 or first + count > len(resident):
                    raise IndexError("block range is not resident")
                picked.extend(resident[first:first + count])
            resident = picked
        blocks = resident
        if not blocks:
            return None, None
        ks = np.concatenate([k for (_, k, _) in blocks], axis=0)
        vs = np.concatenate([v for (_, _, v) in blocks], axis=0)
        return ks, vs
