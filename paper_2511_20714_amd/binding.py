"""ctypes binding of libifx.so: the same names and arguments as include/ifx.h.

Only argument marshalling happens here (tensor -> device pointer, stream ->
hipStream_t).  Every step of the path runs in the library's kernels.  If the
library has not been built, importing this module's functions raises: there is
no fallback.
"""
from __future__ import annotations

import ctypes
import os

IFX_F32 = 0
IFX_BF16 = 1
IFX_FP8_E4M3 = 2
IFX_OK = 0
IFX_ERR_INVALID_ARG = -1
IFX_ERR_NOT_CONFIGURED = -2
IFX_ERR_OOM = -3
IFX_ERR_HIP = -4
IFX_ERR_UNSUPPORTED = -5
IFX_MAX_LISTED_BLOCKS = 63
IFX_NOALLOC_MAX_LISTED_BLOCKS = 4096

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libifx.so")
_lib = None

_vp = ctypes.c_void_p
_i64 = ctypes.c_int64
_int = ctypes.c_int
class ifx_block_range(ctypes.Structure):
    _fields_ = [("first_block", ctypes.c_int64), ("block_count", ctypes.c_int64)]


_SIGS = {
    "ifx_kv_cache_create": (_vp, [_int, _int, _int, _i64]),
    "ifx_block_attention": (_int, [_vp, _int, _vp, _vp, _vp, _vp, _vp]),
    "ifx_kv_cache_commit": (_int, [_vp, _int, _vp, _vp, _vp]),
    "ifx_kv_cache_commit_layers": (_int, [_vp, _int, _int, ctypes.POINTER(_vp), ctypes.POINTER(_vp), _vp]),
    "ifx_block_attention_ranges": (_int, [_vp, _int, _vp, _vp, _vp, ctypes.POINTER(ifx_block_range), _int, _vp, _vp, _vp]),
    "ifx_block_attention_blocks": (_int, [_vp, _int, _vp, _vp, _vp, ctypes.POINTER(ctypes.c_int64), _int, _vp, _vp, _vp]),
    "ifx_block_attention_blocks_noalloc": (_int, [_vp, _int, _vp, _vp, _vp, ctypes.POINTER(ctypes.c_int64), _int, _vp, _vp, _vp]),
    "ifx_attention_merge": (_int, [_vp, _vp, _vp, _vp, _vp, _vp, _i64, _int, _int, _vp]),
    "ifx_kv_cache_reserve": (_int, [_vp, _i64]),
    "ifx_kv_cache_configure": (_int, [_vp, _i64, _int, ctypes.c_float]),
    "ifx_kv_cache_destroy": (None, [_vp]),
    "ifx_kv_cache_reset": (_int, [_vp, _int]),
    "ifx_kv_cache_grow": (_int, [_vp, _i64]),
    "ifx_kv_cache_len": (_i64, [_vp, _int]),
    "ifx_kv_cache_committed": (_i64, [_vp, _int]),
    "ifx_kv_cache_block_ids": (_int, [_vp, _int, ctypes.POINTER(_i64), _int]),
    "ifx_kv_cache_read": (_int, [_vp, _int, _vp, _vp, _int, _vp]),
    "ifx_kv_cache_profile": (_int, [_vp, _int]),
    "ifx_kv_cache_profile_read": (_int, [_vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(_i64),
                                         ctypes.POINTER(ctypes.c_double), ctypes.POINTER(_i64)]),
    "ifx_last_error": (ctypes.c_char_p, []),
    "ifx_ring_create": (_vp, [_i64]),
    "ifx_ring_destroy": (None, [_vp]),
    "ifx_ring_commit": (_i64, [_vp]),
    "ifx_ring_next_slot": (_i64, [_vp]),
    "ifx_ring_resident": (_i64, [_vp]),
    "ifx_ring_committed": (_i64, [_vp]),
    "ifx_ring_slot_of_logical": (_i64, [_vp, _i64]),
    "ifx_ring_block_ids": (_int, [_vp, ctypes.POINTER(_i64), _int]),
    "ifx_ring_reset": (None, [_vp]),
    "ifx_ring_grow": (_int, [_vp, _i64, _int]),
    "ifx_attention_launch_grid": (_int, [_int, _int]),
    "ifx_attention_launch_item": (_int, [_int, _int, _int, ctypes.POINTER(_int)]),
}


class IfxError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"ifx error {code}: {message}")
        self.code = code


def lib() -> ctypes.CDLL:
    """The loaded library.  Builds it first if there is none, or if the one that is there was built
    from other sources or flags than the tree holds now (a digest is kept next to it)."""
    global _lib
    if _lib is None:
        from .build import build_library, is_current

        if not is_current():
            build_library()
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def ifx_last_error() -> str:
    return lib().ifx_last_error().decode()


def _check(rc: int) -> int:
    if rc < 0:
        raise IfxError(int(rc), ifx_last_error())
    return int(rc)


def _ptr(t) -> int:
    """Device (or host) address of a tensor / raw integer address / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        import torch

        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


# ---- one function per C entry point ------------------------------------------

def ifx_kv_cache_create(layers: int, heads: int, head_dim: int, capacity_tokens: int):
    h = lib().ifx_kv_cache_create(layers, heads, head_dim, capacity_tokens)
    if not h:
        raise IfxError(IFX_ERR_INVALID_ARG, ifx_last_error())
    return h


def ifx_kv_cache_configure(cache, block_tokens: int, dtype: int, softmax_scale: float = 0.0) -> None:
    _check(lib().ifx_kv_cache_configure(cache, block_tokens, dtype, softmax_scale))


def ifx_kv_cache_reserve(cache, max_capacity_tokens: int) -> None:
    _check(lib().ifx_kv_cache_reserve(cache, max_capacity_tokens))


def ifx_kv_cache_destroy(cache) -> None:
    lib().ifx_kv_cache_destroy(cache)


def ifx_block_attention(cache, layer: int, q, k_blk, v_blk, out, stream=None) -> None:
    _check(lib().ifx_block_attention(cache, layer, _ptr(q), _ptr(k_blk), _ptr(v_blk), _ptr(out), _stream(stream)))


def ifx_kv_cache_commit(cache, layer: int, k_blk, v_blk, stream=None) -> None:
    _check(lib().ifx_kv_cache_commit(cache, layer, _ptr(k_blk), _ptr(v_blk), _stream(stream)))


def ifx_kv_cache_commit_layers(cache, first_layer: int, k_blks, v_blks, stream=None) -> None:
    """k_blks, v_blks: one tensor (or address) per layer, for layers first_layer, first_layer + 1, ..."""
    k_blks, v_blks = list(k_blks), list(v_blks)
    if len(k_blks) != len(v_blks):
        raise ValueError("k_blks and v_blks must have one entry per layer each")
    ka = (_vp * max(len(k_blks), 1))(*[_ptr(t) for t in k_blks])
    va = (_vp * max(len(v_blks), 1))(*[_ptr(t) for t in v_blks])
    _check(lib().ifx_kv_cache_commit_layers(cache, first_layer, len(k_blks), ka, va, _stream(stream)))


def ifx_block_attention_ranges(cache, layer: int, q, k_blk, v_blk, ranges, out, lse=None, stream=None) -> None:
    """ranges: sequence of (first_block, block_count) pairs, logical blocks, 0 = oldest resident."""
    ranges = list(ranges)
    arr = (ifx_block_range * max(len(ranges), 1))()
    for i, (first, count) in enumerate(ranges):
        arr[i].first_block, arr[i].block_count = first, count
    _check(lib().ifx_block_attention_ranges(cache, layer, _ptr(q), _ptr(k_blk), _ptr(v_blk), arr, len(ranges), _ptr(out),
                                            _ptr(lse), _stream(stream)))


def ifx_block_attention_blocks(cache, layer: int, q, k_blk, v_blk, blocks, out, lse=None, stream=None) -> None:
    """blocks: sequence of logical block numbers (0 = oldest resident), any order, each at most once;
    None: every resident block (the key set of ifx_block_attention, with lse)."""
    count = -1 if blocks is None else len(list(blocks))
    blocks = [] if blocks is None else list(blocks)
    arr = (ctypes.c_int64 * max(len(blocks), 1))(*blocks)
    _check(lib().ifx_block_attention_blocks(cache, layer, _ptr(q), _ptr(k_blk), _ptr(v_blk), arr, count, _ptr(out),
                                            _ptr(lse), _stream(stream)))


def ifx_block_attention_blocks_noalloc(cache, layer: int, q, k_blk, v_blk, blocks, out, lse=None, stream=None) -> None:
    """ifx_block_attention_blocks with the block list kept in the library's static device memory."""
    count = -1 if blocks is None else len(list(blocks))
    blocks = [] if blocks is None else list(blocks)
    arr = (ctypes.c_int64 * max(len(blocks), 1))(*blocks)
    _check(lib().ifx_block_attention_blocks_noalloc(cache, layer, _ptr(q), _ptr(k_blk), _ptr(v_blk), arr, count, _ptr(out),
                                                    _ptr(lse), _stream(stream)))


def ifx_attention_merge(out_a, lse_a, out_b, lse_b, out, lse, rows: int, head_dim: int, dtype: int, stream=None) -> None:
    _check(lib().ifx_attention_merge(_ptr(out_a), _ptr(lse_a), _ptr(out_b), _ptr(lse_b), _ptr(out), _ptr(lse), rows,
                                     head_dim, dtype, _stream(stream)))


def ifx_kv_cache_reset(cache, layer: int = -1) -> None:
    _check(lib().ifx_kv_cache_reset(cache, layer))


def ifx_kv_cache_grow(cache, new_capacity_tokens: int) -> None:
    _check(lib().ifx_kv_cache_grow(cache, new_capacity_tokens))


def ifx_kv_cache_len(cache, layer: int) -> int:
    return _check(lib().ifx_kv_cache_len(cache, layer))


def ifx_kv_cache_committed(cache, layer: int) -> int:
    return _check(lib().ifx_kv_cache_committed(cache, layer))


def ifx_kv_cache_block_ids(cache, layer: int, max_slots: int = 1 << 16):
    buf = (ctypes.c_int64 * max_slots)()
    k = _check(lib().ifx_kv_cache_block_ids(cache, layer, buf, max_slots))
    return list(buf[:k])


def ifx_kv_cache_read(cache, layer: int, k_out, v_out, logical_order: bool = True, stream=None) -> None:
    _check(lib().ifx_kv_cache_read(cache, layer, _ptr(k_out), _ptr(v_out), int(bool(logical_order)), _stream(stream)))


def ifx_kv_cache_profile(cache, enable: bool) -> None:
    _check(lib().ifx_kv_cache_profile(cache, int(bool(enable))))


def ifx_kv_cache_profile_read(cache):
    """(attention_ms, attention_launches, commit_ms, commit_launches) since the last read."""
    a, c = ctypes.c_double(), ctypes.c_double()
    na, nc = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().ifx_kv_cache_profile_read(cache, ctypes.byref(a), ctypes.byref(na), ctypes.byref(c), ctypes.byref(nc)))
    return a.value, na.value, c.value, nc.value


def ifx_ring_create(capacity_blocks: int):
    h = lib().ifx_ring_create(capacity_blocks)
    if not h:
        raise IfxError(IFX_ERR_INVALID_ARG, ifx_last_error())
    return h


def ifx_ring_destroy(ring) -> None:
    lib().ifx_ring_destroy(ring)


def ifx_ring_commit(ring) -> int:
    return _check(lib().ifx_ring_commit(ring))


def ifx_ring_next_slot(ring) -> int:
    return _check(lib().ifx_ring_next_slot(ring))


def ifx_ring_resident(ring) -> int:
    return _check(lib().ifx_ring_resident(ring))


def ifx_ring_committed(ring) -> int:
    return _check(lib().ifx_ring_committed(ring))


def ifx_ring_slot_of_logical(ring, logical: int) -> int:
    return int(lib().ifx_ring_slot_of_logical(ring, logical))


def ifx_ring_block_ids(ring, max_slots: int = 1 << 16):
    buf = (ctypes.c_int64 * max_slots)()
    k = _check(lib().ifx_ring_block_ids(ring, buf, max_slots))
    return list(buf[:k])


def ifx_ring_reset(ring) -> None:
    lib().ifx_ring_reset(ring)


def ifx_ring_grow(ring, new_capacity_blocks: int, in_place: bool = False) -> None:
    _check(lib().ifx_ring_grow(ring, new_capacity_blocks, int(bool(in_place))))


def ifx_attention_launch_grid(block_tokens: int, heads: int) -> int:
    g = lib().ifx_attention_launch_grid(block_tokens, heads)
    if g < 0:
        _check(g)
    return g


def ifx_attention_launch_item(block_tokens: int, heads: int, workgroup: int):
    """(head, q_tile, first row, wavefronts with rows, xcd) of one workgroup of the bf16 attention launch."""
    item = (_int * 5)()
    _check(lib().ifx_attention_launch_item(block_tokens, heads, workgroup, item))
    return tuple(item)


# ---- a small owner object so handles are not leaked ---------------------------

class KVCache:
    """Owns one ifx_kv_cache handle; every method is one C call."""

    def __init__(self, layers, heads, head_dim, capacity_tokens, block_tokens, dtype, softmax_scale=0.0, reserve_tokens=None):
        self.layers, self.heads, self.head_dim = layers, heads, head_dim
        self.capacity_tokens, self.block_tokens, self.dtype = capacity_tokens, block_tokens, dtype
        self.handle = ifx_kv_cache_create(layers, heads, head_dim, capacity_tokens)
        try:
            if reserve_tokens is not None:
                ifx_kv_cache_reserve(self.handle, reserve_tokens)
            ifx_kv_cache_configure(self.handle, block_tokens, dtype, softmax_scale)
        except Exception:
            ifx_kv_cache_destroy(self.handle)
            self.handle = None
            raise

    def attention(self, layer, q, k_blk, v_blk, out, stream=None):
        ifx_block_attention(self.handle, layer, q, k_blk, v_blk, out, stream)

    def commit(self, layer, k_blk, v_blk, stream=None):
        ifx_kv_cache_commit(self.handle, layer, k_blk, v_blk, stream)

    def commit_layers(self, first_layer, k_blks, v_blks, stream=None):
        ifx_kv_cache_commit_layers(self.handle, first_layer, k_blks, v_blks, stream)

    def attention_ranges(self, layer, q, k_blk, v_blk, ranges, out, lse=None, stream=None):
        ifx_block_attention_ranges(self.handle, layer, q, k_blk, v_blk, ranges, out, lse, stream)

    def attention_blocks(self, layer, q, k_blk, v_blk, blocks, out, lse=None, stream=None):
        ifx_block_attention_blocks(self.handle, layer, q, k_blk, v_blk, blocks, out, lse, stream)

    def attention_blocks_noalloc(self, layer, q, k_blk, v_blk, blocks, out, lse=None, stream=None):
        ifx_block_attention_blocks_noalloc(self.handle, layer, q, k_blk, v_blk, blocks, out, lse, stream)

    def reset(self, layer=-1):
        ifx_kv_cache_reset(self.handle, layer)

    def grow(self, new_capacity_tokens):
        ifx_kv_cache_grow(self.handle, new_capacity_tokens)

    def len(self, layer):
        return ifx_kv_cache_len(self.handle, layer)

    def committed(self, layer):
        return ifx_kv_cache_committed(self.handle, layer)

    def block_ids(self, layer):
        return ifx_kv_cache_block_ids(self.handle, layer)

    def read(self, layer, k_out, v_out, logical_order=True, stream=None):
        ifx_kv_cache_read(self.handle, layer, k_out, v_out, logical_order, stream)

    def profile(self, enable):
        ifx_kv_cache_profile(self.handle, enable)

    def profile_read(self):
        return ifx_kv_cache_profile_read(self.handle)

    def close(self):
        if self.handle:
            ifx_kv_cache_destroy(self.handle)
            self.handle = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
