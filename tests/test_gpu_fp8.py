"""The fp8 (OCP E4M3) cache variant: commit rounds a block to E4M3 exactly as the oracle's rule
says (every bfloat16 value checked), attention over the rounded cache matches the fp64 oracle over
the same rounded values within the bf16 tolerance, on every kind of key set."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_20714_amd import binding as ifx
from paper_2511_20714_amd import synth

from gpu_util import (OracleCacheFP8, as_oracle_block, assert_attention_close, assert_cache_bits, expected_ids, read_cache,
                      sample_rows, to_np_exact)

pytestmark = pytest.mark.gpu
FP8 = ifx.IFX_FP8_E4M3
BF = torch.bfloat16


def all_pairs(n, H):
    return np.repeat(np.arange(n), H), np.tile(np.arange(H), n)


def test_fp8_commit_rounds_every_bf16_value_like_the_oracle(gpu_device):
    """One block of 512 tokens x 1 head x 128 holds each of the 65536 bfloat16 bit patterns once, as
    K (row layout) and, in another order, as V (granule layout).  What the cache then holds, read
    back widened to bf16, must be the oracle's rounding of every element: the same bits wherever
    the result is a number, a NaN wherever it is a NaN (which NaN is not defined)."""
    dev = gpu_device
    n, H, D = 512, 1, 128
    bits_k = np.arange(65536, dtype=np.uint16).reshape(n, H, D)
    bits_v = np.random.default_rng(5).permutation(65536).astype(np.uint16).reshape(n, H, D)
    with ifx.KVCache(1, H, D, 2 * n, n, FP8) as cache:
        k = torch.from_numpy(bits_k.view(np.int16).copy()).view(BF).to(dev)
        v = torch.from_numpy(bits_v.view(np.int16).copy()).view(BF).to(dev)
        cache.commit(0, k, v)
        kk, vv = read_cache(cache, 0, H, D, BF, dev)
        for got_t, src in ((kk, bits_k), (vv, bits_v)):
            got = as_oracle_block(got_t)
            want = oracle.bf16_bits_through_e4m3(src)
            want_nan = np.isnan(oracle.bf16_bits_to_f64(want))
            got_nan = np.isnan(oracle.bf16_bits_to_f64(got))
            assert np.array_equal(got_nan, want_nan)
            assert np.array_equal(got[~want_nan], want[~want_nan])
            assert want_nan.sum() == np.isnan(oracle.bf16_bits_to_f64(src)).sum()  # only NaN becomes NaN: everything else saturates


def test_fp8_generate_and_cache_loop(gpu_device):
    """Ragged block (n = 200), ring of 3 over 6 commits, 2 layers: attention of every row against
    the oracle over the rounded cache, contents and slot ids after every commit."""
    dev = gpu_device
    L, H, D, n, cap = 2, 3, 128, 200, 3
    rows, heads = all_pairs(n, H)
    with ifx.KVCache(L, H, D, cap * n, n, FP8) as cache:
        ocs = [OracleCacheFP8(cap) for _ in range(L)]
        for b in range(6):
            for l in range(L):
                q, k, v = synth.draw_qkv(131, b, 0, l, n, H, D, BF, dev, True)
                out = torch.full((n, H, D), float("nan"), dtype=BF, device=dev)
                cache.attention(l, q, k, v, out)
                torch.cuda.synchronize()
                kc, vc = ocs[l].logical()
                want, _ = oracle.attention_rows(synth.to_f64_numpy(q), kc, vc, synth.to_f64_numpy(k), synth.to_f64_numpy(v), rows, heads)
                assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, ifx.IFX_BF16, f"fp8 loop block {b} layer {l}")
                cache.commit(l, k, v)
                ocs[l].commit(k, v)
                assert cache.block_ids(l) == expected_ids(ocs[l].raw, cap)
                assert_cache_bits(cache, l, ocs[l].raw, H, D, BF, dev)


@pytest.mark.parametrize("gain", [1.0, 8.0])
def test_fp8_key_sets_and_softmax_variants(gpu_device, gain):
    """Listed blocks in any order, ranges on a wrapped ring, cache only, a list longer than one pass
    of the block table, with unit-scale queries (fixed maximum from the norms of the rounded keys)
    and 8 x longer ones (running maximum); log-sum-exp too."""
    dev = gpu_device
    H, D, n, cap = 2, 128, 72, 70
    rows, heads = all_pairs(n, H)
    with ifx.KVCache(1, H, D, cap * n, n, FP8) as cache:
        oc = OracleCacheFP8(cap)
        for b in range(cap + 5):
            _, k, v = synth.draw_qkv(137, b, 0, 0, n, H, D, BF, dev, True)
            cache.commit(0, k, v)
            oc.commit(k, v)
        q, k, v = synth.draw_qkv(137, 999, 0, 0, n, H, D, BF, dev, True, gain)
        rng = np.random.default_rng(9)
        selections = [[3, 0, 69, 41], list(range(cap)), rng.permutation(cap)[:66].tolist(), [7], list(range(10, 30))]
        for picks in selections:
            for kk, vv in ((k, v), (None, None)):
                out = torch.full((n, H, D), float("nan"), dtype=BF, device=dev)
                lse = torch.full((n, H), float("nan"), dtype=torch.float32, device=dev)
                cache.attention_blocks(0, q, kk, vv, picks, out, lse)
                torch.cuda.synchronize()
                kc, vc = oc.raw.logical(blocks=picks)
                kc, vc = oracle.bf16_bits_to_f64(kc), oracle.bf16_bits_to_f64(vc)
                kb = None if kk is None else synth.to_f64_numpy(kk)
                vb = None if vv is None else synth.to_f64_numpy(vv)
                want, want_lse = oracle.attention_rows(synth.to_f64_numpy(q), kc, vc, kb, vb, rows, heads)
                label = f"fp8 gain {gain} picks {len(picks)} block {kk is not None}"
                assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, ifx.IFX_BF16, label, input_scale=gain)
                assert np.abs(lse.cpu().numpy().astype(np.float64)[rows, heads] - want_lse).max() <= 2e-3 * gain, label
        out = torch.full((n, H, D), float("nan"), dtype=BF, device=dev)
        cache.attention_ranges(0, q, k, v, [(0, 1), (cap - 3, 3)], out)
        torch.cuda.synchronize()
        kc, vc = oc.raw.logical([(0, 1), (cap - 3, 3)])
        want, _ = oracle.attention_rows(synth.to_f64_numpy(q), oracle.bf16_bits_to_f64(kc), oracle.bf16_bits_to_f64(vc),
                                        synth.to_f64_numpy(k), synth.to_f64_numpy(v), rows, heads)
        assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, ifx.IFX_BF16, "fp8 sink + window", input_scale=gain)


def test_fp8_full_size_layer(gpu_device):
    """The Wan-1.3B-class layer with an fp8 cache: 12 heads x 128, block 4680, 6 cached blocks."""
    dev = gpu_device
    n, H, D, cap = 4680, 12, 128, 6
    with ifx.KVCache(1, H, D, cap * n, n, FP8) as cache:
        oc = OracleCacheFP8(cap)
        for b in range(cap):
            _, k, v = synth.draw_qkv(2, b, 0, 0, n, H, D, BF, dev, True)
            cache.commit(0, k, v)
            oc.commit(k, v)
        q, k, v = synth.draw_qkv(2, cap, 0, 0, n, H, D, BF, dev, True)
        out = torch.full((n, H, D), float("nan"), dtype=BF, device=dev)
        cache.attention(0, q, k, v, out)
        torch.cuda.synchronize()
        rows, heads = sample_rows(n, H, per_head=32, full_heads=(), seed=4)
        kc, vc = oc.logical()
        want, _ = oracle.attention_rows(synth.to_f64_numpy(q), kc, vc, synth.to_f64_numpy(k), synth.to_f64_numpy(v), rows, heads)
        mx, mean, rms = assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, ifx.IFX_BF16, "fp8 full size")
        print(f"fp8 full size: rows={len(rows)} max|err|={mx:.3e} mean|err|={mean:.3e} rms(out)={rms:.3e}")
        assert not torch.isnan(out.float()).any()
        assert_cache_bits(cache, 0, oc.raw, H, D, BF, dev)


def test_fp8_reserved_cache_grows_in_place(gpu_device):
    dev = gpu_device
    H, D, n = 2, 128, 2056
    rows = np.repeat(np.arange(0, n, 61), H)
    heads = np.tile(np.arange(H), len(rows) // H)
    with ifx.KVCache(1, H, D, 2 * n, n, FP8, reserve_tokens=5 * n) as cache:
        oc = OracleCacheFP8(2)
        for b in range(3):
            _, k, v = synth.draw_qkv(139, b, 0, 0, n, H, D, BF, dev, True)
            cache.commit(0, k, v)
            oc.commit(k, v)
        cache.grow(5 * n)
        oc.raw.grow(5)
        for b in range(3, 7):
            _, k, v = synth.draw_qkv(139, b, 0, 0, n, H, D, BF, dev, True)
            cache.commit(0, k, v)
            oc.commit(k, v)
        assert_cache_bits(cache, 0, oc.raw, H, D, BF, dev)
        q, k, v = synth.draw_qkv(139, 99, 0, 0, n, H, D, BF, dev, True)
        out = torch.full((n, H, D), float("nan"), dtype=BF, device=dev)
        cache.attention(0, q, k, v, out)
        torch.cuda.synchronize()
        kc, vc = oc.logical()
        want, _ = oracle.attention_rows(synth.to_f64_numpy(q), kc, vc, synth.to_f64_numpy(k), synth.to_f64_numpy(v), rows, heads)
        assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, ifx.IFX_BF16, "fp8 reserved")
