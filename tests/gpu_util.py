"""Helpers shared by the GPU parity tests: run the HIP library through its C
ABI and compare with the fp64 oracle on the very same input bits."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2511_20714_amd import binding as ifx
from paper_2511_20714_amd import synth

TORCH_DTYPE = {ifx.IFX_F32: torch.float32, ifx.IFX_BF16: torch.bfloat16}


def f64(t):
    return synth.to_f64_numpy(t)


def oracle_rows(q, k, v, ocache, rows, heads):
    """Oracle output for selected (row, head) pairs; ocache holds device-tensor copies (torch, CPU)."""
    kc, vc = ocache.logical()
    kc64 = None if kc is None else kc.astype(np.float64)
    vc64 = None if vc is None else vc.astype(np.float64)
    out, _ = oracle.attention_rows(f64(q), kc64, vc64, f64(k), f64(v), rows, heads)
    return out


def to_np_exact(t):
    """Device tensor -> numpy float32 array holding exactly the same values (bf16 widened)."""
    return t.detach().to("cpu").to(torch.float32).numpy()


def sample_rows(n, H, q_tile=128, per_head=64, full_heads=(0, -1), seed=0):
    """(rows, heads): every row of the heads in full_heads; elsewhere first/last row, both
    sides of every q-tile boundary, the tail tile, plus random rows."""
    rng = np.random.default_rng(seed)
    rows, heads = [], []
    full = {h % H for h in full_heads}
    for h in range(H):
        if h in full:
            r = np.arange(n)
        else:
            edge = {0, n - 1}
            for b in range(q_tile, n, q_tile):
                edge.update((b - 1, b))
            edge.update(range(max(0, n - 8), n))
            edge = sorted(edge)
            if len(edge) > per_head:
                keep = {0, n - 1}
                keep.update(rng.choice(edge, size=per_head - 2, replace=False).tolist())
                edge = sorted(keep)
            extra = rng.choice(n, size=max(0, per_head - len(edge)), replace=False)
            r = np.unique(np.concatenate([np.array(edge, dtype=np.int64), extra]))
        rows.append(r)
        heads.append(np.full(r.shape, h, dtype=np.int64))
    return np.concatenate(rows).astype(np.int64), np.concatenate(heads)


def error_stats(got_rows, want_rows):
    err = np.abs(got_rows - want_rows)
    rms = float(np.sqrt(np.mean(want_rows ** 2)))
    return float(err.max()), float(err.mean()), rms


def assert_attention_close(got_rows, want_rows, dtype, label="", input_scale=1.0):
    """Spec tolerances, plus the same numbers relative to the RMS of the
    oracle's output (outputs shrink like 1/sqrt(keys), so the absolute gate alone
    would accept an all-zero result at long key lengths).  The fp32 bound is for
    unit-scale inputs: logit rounding error grows with the logits' magnitude, so a
    test that multiplies q by ``input_scale`` widens the fp32 bound by that factor."""
    mx, mean, rms = error_stats(got_rows, want_rows)
    msg = f"{label}: max|err|={mx:.3e} mean|err|={mean:.3e} rms(out)={rms:.3e}"
    assert np.isfinite(got_rows).all(), msg
    if dtype == ifx.IFX_F32:
        assert mx <= 1e-5 * input_scale, msg
    else:
        assert mx <= 2e-2 and mean <= 2e-3, msg
        assert mx <= 5e-2 * max(rms, 1e-30) and mean <= 2e-3 * max(rms, 1e-30), msg
    return mx, mean, rms


# ---- the cache on both sides --------------------------------------------------

def read_cache(cache, layer, H, D, tdtype, dev, logical=True):
    C = cache.len(layer)
    k = torch.empty((max(C, 1), H, D), dtype=tdtype, device=dev)
    v = torch.empty_like(k)
    cache.read(layer, k, v, logical)
    torch.cuda.synchronize()
    return k[:C], v[:C]


def assert_cache_bits(cache, layer, ocache, H, D, tdtype, dev):
    k, v = read_cache(cache, layer, H, D, tdtype, dev)
    ok, ov = ocache.logical()
    if ok is None:
        assert k.shape[0] == 0
        return
    assert synth.raw_bytes(k) == ok.tobytes()
    assert synth.raw_bytes(v) == ov.tobytes()


def as_oracle_block(t):
    """Device tensor -> numpy array with the same bits (bf16 as uint16)."""
    t = t.detach().to("cpu").contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()


class OracleCacheF:
    """The deque oracle holding raw bits, plus float views for the attention oracle."""

    def __init__(self, cap_blocks, tdtype):
        self.raw = oracle.BlockCacheOracle(cap_blocks)
        self.tdtype = tdtype

    def commit(self, k, v):
        self.raw.commit(as_oracle_block(k), as_oracle_block(v))

    def logical(self):
        k, v = self.raw.logical()
        if k is None:
            return None, None
        if self.tdtype == torch.bfloat16:
            return oracle.bf16_bits_to_f64(k), oracle.bf16_bits_to_f64(v)
        return k.astype(np.float64), v.astype(np.float64)


def expected_ids(raw, cap_blocks):
    """slot -> ordinal from the deque model: ordinal t sits in slot t mod cap."""
    ids = [-1] * cap_blocks
    for o in raw.ordinals:
        ids[o % cap_blocks] = o
    return ids


class OracleCacheFP8(OracleCacheF):
    """The deque oracle of an fp8 (E4M3) cache: a committed block is rounded to E4M3 by the oracle's
    own rule and kept as the bfloat16 bit patterns of the rounded values, which is what
    ifx_kv_cache_read returns for such a cache."""

    def __init__(self, cap_blocks):
        super().__init__(cap_blocks, torch.bfloat16)

    def commit(self, k, v):
        self.raw.commit(oracle.bf16_bits_through_e4m3(as_oracle_block(k)), oracle.bf16_bits_through_e4m3(as_oracle_block(v)))
