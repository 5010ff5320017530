"""GPU parity of the split-attention entry points: attention over caller-chosen
resident blocks with log-sum-exp output (ifx_block_attention_ranges) and the
merge of two partial results (ifx_attention_merge), against the fp64 oracle on
the same input bits."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_20714_amd import binding as ifx
from paper_2511_20714_amd import synth

from gpu_util import (TORCH_DTYPE, OracleCacheF, OracleCacheFP8, assert_attention_close, assert_cache_bits, expected_ids, sample_rows,
                      to_np_exact)

pytestmark = pytest.mark.gpu

LSE_TOL = {ifx.IFX_F32: 2e-5, ifx.IFX_BF16: 2e-3}  # absolute, on log-sum-exp values of about 5..12


def all_pairs(n, H):
    return np.repeat(np.arange(n), H), np.tile(np.arange(H), n)


def fill_cache(dev, dtype, H, D, n, cap, commits, seed):
    tdtype = TORCH_DTYPE[dtype]
    cache = ifx.KVCache(1, H, D, cap * n, n, dtype)
    oc = OracleCacheF(cap, tdtype)
    for b in range(commits):
        _, k, v = synth.draw_qkv(seed, b, 0, 0, n, H, D, tdtype, dev, True)
        cache.commit(0, k, v)
        oc.commit(k, v)
    return cache, oc


def oracle_ranges(oc, ranges, q, k, v, rows, heads):
    """Oracle attention over the named resident blocks (+ the block if k is given)."""
    kc, vc = oc.raw.logical(ranges)
    if kc is not None:
        if oc.tdtype == torch.bfloat16:
            kc, vc = oracle.bf16_bits_to_f64(kc), oracle.bf16_bits_to_f64(vc)
        else:
            kc, vc = kc.astype(np.float64), vc.astype(np.float64)
    kb = None if k is None else synth.to_f64_numpy(k)
    vb = None if v is None else synth.to_f64_numpy(v)
    return oracle.attention_rows(synth.to_f64_numpy(q), kc, vc, kb, vb, rows, heads)


def run_ranges(cache, q, k, v, ranges, dev, want_lse=True):
    n, H, D = q.shape
    out = torch.full((n, H, D), float("nan"), dtype=q.dtype, device=dev)
    lse = torch.full((n, H), float("nan"), dtype=torch.float32, device=dev) if want_lse else None
    cache.attention_ranges(0, q, k, v, ranges, out, lse)
    torch.cuda.synchronize()
    return out, lse


@pytest.mark.parametrize("dtype", [ifx.IFX_BF16, ifx.IFX_F32])
def test_ranges_on_a_wrapped_ring(gpu_device, dtype):
    """Ring of 5 slots after 7 commits (logical blocks 0..4 sit in slots 2,3,4,0,1).  Every
    selection below is compared with the oracle over exactly those blocks: the whole cache, a
    range that wraps, a sink block plus a window, cache only, block only."""
    dev = gpu_device
    H, D, n = 2, (128 if dtype == ifx.IFX_BF16 else 64), 72
    cache, oc = fill_cache(dev, dtype, H, D, n, cap=5, commits=7, seed=41)
    with cache:
        q, k, v = synth.draw_qkv(41, 99, 0, 0, n, H, D, TORCH_DTYPE[dtype], dev, True)
        rows, heads = all_pairs(n, H)
        cases = [
            ([(0, 5)], True), ([(1, 3)], True), ([(0, 1), (2, 3)], True), ([(0, 1), (3, 2)], True), ([(4, 1)], True),
            ([(0, 5)], False), ([(1, 3)], False), ([(0, 1), (2, 3)], False), ([(2, 1)], False),
            ([], True), ([(0, 1), (2, 1), (4, 1)], True), ([(0, 2), (2, 1), (3, 2)], True),  # adjacent ranges join
        ]
        for ranges, with_block in cases:
            kk, vv = (k, v) if with_block else (None, None)
            out, lse = run_ranges(cache, q, kk, vv, ranges, dev)
            want, want_lse = oracle_ranges(oc, ranges, q, kk, vv, rows, heads)
            label = f"ranges {ranges} block={with_block} dtype={dtype}"
            assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, dtype, label)
            got_lse = lse.cpu().numpy().astype(np.float64)[rows, heads]
            assert np.abs(got_lse - want_lse).max() <= LSE_TOL[dtype], (label, np.abs(got_lse - want_lse).max())
        # resident blocks untouched
        assert_cache_bits(cache, 0, oc.raw, H, D, TORCH_DTYPE[dtype], dev)


@pytest.mark.parametrize("dtype", [ifx.IFX_BF16, ifx.IFX_F32])
def test_split_then_merge_equals_whole(gpu_device, dtype):
    """Attention over the cache alone and over the block alone, merged on the device, equals the
    oracle's attention over both (the use in pass-Q ring attention); and a three-way split of the
    cache merged pairwise does too."""
    dev = gpu_device
    H, D, n = 3, (128 if dtype == ifx.IFX_BF16 else 64), 136
    cache, oc = fill_cache(dev, dtype, H, D, n, cap=4, commits=6, seed=43)
    with cache:
        q, k, v = synth.draw_qkv(43, 77, 0, 0, n, H, D, TORCH_DTYPE[dtype], dev, True)
        rows, heads = all_pairs(n, H)
        want, want_lse = oracle_ranges(oc, [(0, 4)], q, k, v, rows, heads)
        o_c, l_c = run_ranges(cache, q, None, None, [(0, 4)], dev)
        o_b, l_b = run_ranges(cache, q, k, v, [], dev)
        out = torch.empty_like(q)
        lse = torch.empty_like(l_c)
        ifx.ifx_attention_merge(o_c, l_c, o_b, l_b, out, lse, n * H, D, dtype)
        torch.cuda.synchronize()
        # two roundings to the storage type instead of one: the mean gate of the bf16 bar is for one
        got = to_np_exact(out)[rows, heads].astype(np.float64)
        err = np.abs(got - want)
        rms = np.sqrt(np.mean(want ** 2))
        if dtype == ifx.IFX_F32:
            assert err.max() <= 1e-5
        else:
            assert err.max() <= 2e-2 and err.mean() <= 2e-3 and err.max() <= 5e-2 * rms and err.mean() <= 3e-3 * rms
        assert np.abs(lse.cpu().numpy().astype(np.float64)[rows, heads] - want_lse).max() <= LSE_TOL[dtype]

        # ((blocks 0-1) + (block 2)) + (block 3 and the current block), in place
        o1, l1 = run_ranges(cache, q, None, None, [(0, 2)], dev)
        o2, l2 = run_ranges(cache, q, None, None, [(2, 1)], dev)
        o3, l3 = run_ranges(cache, q, k, v, [(3, 1)], dev)
        ifx.ifx_attention_merge(o1, l1, o2, l2, o1, l1, n * H, D, dtype)
        ifx.ifx_attention_merge(o1, l1, o3, l3, o1, l1, n * H, D, dtype)
        torch.cuda.synchronize()
        got = to_np_exact(o1)[rows, heads].astype(np.float64)
        err = np.abs(got - want)
        if dtype == ifx.IFX_F32:
            assert err.max() <= 1e-5
        else:
            assert err.max() <= 2e-2 and err.mean() <= 2e-3 and err.max() <= 5e-2 * rms and err.mean() <= 4e-3 * rms
        assert np.abs(l1.cpu().numpy().astype(np.float64)[rows, heads] - want_lse).max() <= LSE_TOL[dtype]


@pytest.mark.parametrize("dtype", [ifx.IFX_BF16, ifx.IFX_F32])
def test_merge_kernel_against_oracle_merge(gpu_device, dtype):
    """The merge alone, on arbitrary inputs: log-sum-exp values far apart, equal, and -inf on one side."""
    dev = gpu_device
    tdtype = TORCH_DTYPE[dtype]
    g = torch.Generator(device="cpu").manual_seed(5)
    rows, D = 1000, 128 if dtype == ifx.IFX_BF16 else 40
    oa = torch.randn(rows, D, generator=g).to(tdtype).to(dev)
    ob = torch.randn(rows, D, generator=g).to(tdtype).to(dev)
    la = (torch.randn(rows, generator=g) * 20.0).to(dev)
    lb = (torch.randn(rows, generator=g) * 20.0).to(dev)
    lb[:50] = la[:50]
    lb[50:100] = float("-inf")
    la[100:150] = float("-inf")
    out = torch.full_like(oa, float("nan"))
    lse = torch.full_like(la, float("nan"))
    ifx.ifx_attention_merge(oa, la, ob, lb, out, lse, rows, D, dtype)
    torch.cuda.synchronize()
    with np.errstate(invalid="ignore"):
        want, want_lse = oracle.merge(synth.to_f64_numpy(oa), la.cpu().numpy(), synth.to_f64_numpy(ob), lb.cpu().numpy())
    got = to_np_exact(out).astype(np.float64)
    tol = 2e-6 if dtype == ifx.IFX_F32 else 2.0 ** -8 * np.maximum(np.abs(want), 1e-3)  # one rounding to bf16
    assert (np.abs(got - want) <= tol).all()
    assert np.abs(lse.cpu().numpy().astype(np.float64) - want_lse).max() <= 1e-5 * 20
    # without an lse output, and writing over the first input
    ifx.ifx_attention_merge(oa, la, ob, lb, oa, None, rows, D, dtype)
    torch.cuda.synchronize()
    assert synth.raw_bytes(oa) == synth.raw_bytes(out)


def test_ranges_errors_leave_the_cache_usable(gpu_device):
    dev = gpu_device
    H, D, n = 2, 128, 64
    cache, oc = fill_cache(dev, ifx.IFX_BF16, H, D, n, cap=3, commits=2, seed=47)
    with cache:
        q, k, v = synth.draw_qkv(47, 9, 0, 0, n, H, D, torch.bfloat16, dev, True)
        out = torch.empty_like(q)
        for bad in ([(0, 3)], [(2, 1)], [(1, 1), (0, 1)], [(0, 2), (1, 1)], [(-1, 1)]):
            with pytest.raises(ifx.IfxError) as e:
                cache.attention_ranges(0, q, k, v, bad, out)
            assert e.value.code == ifx.IFX_ERR_INVALID_ARG, bad
        with pytest.raises(ifx.IfxError):
            cache.attention_ranges(0, q, None, None, [], out)  # no key at all
        with pytest.raises(ifx.IfxError):
            cache.attention_ranges(0, q, k, None, [(0, 1)], out)  # k without v
        with pytest.raises(ifx.IfxError):
            cache.attention_ranges(0, q, k, v, [(0, 1), (1, 1), (1, 0)], out)  # ranges not ascending
        with pytest.raises(ifx.IfxError):
            ifx.ifx_attention_merge(out, None, out, None, out, None, n * H, D, ifx.IFX_BF16)
        rows, heads = all_pairs(n, H)
        got, _ = run_ranges(cache, q, k, v, [(0, 2)], dev, want_lse=False)
        want, _ = oracle_ranges(oc, [(0, 2)], q, k, v, rows, heads)
        assert_attention_close(to_np_exact(got)[rows, heads].astype(np.float64), want, ifx.IFX_BF16, "after errors")


def test_sink_plus_window_at_full_size(gpu_device):
    """Wan-1.3B-class layer, ring of 7 blocks wrapped: first resident block + last three + the
    current block (key length 23400, five table entries), sampled rows with the full key set."""
    dev = gpu_device
    H, D, n = 12, 128, 4680
    cache, oc = fill_cache(dev, ifx.IFX_BF16, H, D, n, cap=7, commits=9, seed=53)
    with cache:
        q, k, v = synth.draw_qkv(53, 100, 0, 0, n, H, D, torch.bfloat16, dev, True)
        ranges = [(0, 1), (4, 3)]
        out, lse = run_ranges(cache, q, k, v, ranges, dev)
        rows, heads = sample_rows(n, H, q_tile=256, per_head=48, full_heads=(0,), seed=3)
        want, want_lse = oracle_ranges(oc, ranges, q, k, v, rows, heads)
        assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, ifx.IFX_BF16, "sink + window")
        assert np.abs(lse.cpu().numpy().astype(np.float64)[rows, heads] - want_lse).max() <= LSE_TOL[ifx.IFX_BF16]


def test_bf16_random_shapes_and_selections(gpu_device):
    """A seeded sweep over block sizes, head counts, ring sizes, fill levels, selections and logit
    gains (unit-scale rows take the bounded-maximum path, gain 8 the running-maximum path)."""
    dev = gpu_device
    rng = np.random.default_rng(2024)
    D = 128
    for case in range(40):
        n = int(rng.integers(1, 40)) * 8
        H = int(rng.integers(1, 5))
        cap = int(rng.integers(1, 6))
        commits = int(rng.integers(0, 2 * cap + 2))
        gain = 8.0 if case % 4 == 3 else 1.0
        cache, oc = fill_cache(dev, ifx.IFX_BF16, H, D, n, cap, commits, seed=1000 + case)
        with cache:
            resident = min(commits, cap)
            q, k, v = synth.draw_qkv(1000 + case, 99, 0, 0, n, H, D, torch.bfloat16, dev, True, gain)
            rows, heads = all_pairs(n, H)
            kind = case % 5
            if kind == 0 or resident == 0:
                ranges, with_block = None, True  # the plain call
            elif kind == 1:
                first = int(rng.integers(0, resident))
                ranges, with_block = [(first, int(rng.integers(1, resident - first + 1)))], True
            elif kind == 2 and resident >= 2:
                split = int(rng.integers(1, resident))
                a = int(rng.integers(1, split + 1))
                ranges, with_block = [(0, a), (split, resident - split)], True
            elif kind == 3:
                first = int(rng.integers(0, resident))
                ranges, with_block = [(first, resident - first)], False
            else:
                ranges, with_block = [], True
            label = f"case {case}: n={n} H={H} cap={cap} commits={commits} gain={gain} ranges={ranges} block={with_block}"
            kk, vv = (k, v) if with_block else (None, None)
            if ranges is None:
                out = torch.full((n, H, D), float("nan"), dtype=torch.bfloat16, device=dev)
                cache.attention(0, q, k, v, out)
                torch.cuda.synchronize()
                want, _ = oracle_ranges(oc, [(0, resident)] if resident else [], q, k, v, rows, heads)
            else:
                out, lse = run_ranges(cache, q, kk, vv, ranges, dev)
                want, want_lse = oracle_ranges(oc, ranges, q, kk, vv, rows, heads)
                assert np.abs(lse.cpu().numpy().astype(np.float64)[rows, heads] - want_lse).max() <= LSE_TOL[ifx.IFX_BF16] * gain, label
            assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, ifx.IFX_BF16, label, input_scale=gain)


@pytest.mark.parametrize("dtype", [ifx.IFX_BF16, ifx.IFX_FP8_E4M3])
def test_bf16_wide_random_sweep(gpu_device, dtype):
    """The sweep above over a wider box: up to 17 heads (every XCD share), up to six query tiles
    (blocks of 8 ... 1352 tokens: full, short and single-wavefront workgroups), rings of up to 4
    blocks in every fill state, plain calls, one range, sink + newest; every fourth case with
    logits x 8; both cache dtypes.  All rows of the first and the last head and the last 40 rows
    of every head are compared."""
    dev = gpu_device
    rng = np.random.default_rng(77 + dtype)
    D = 128
    for case in range(60):
        n = int(rng.integers(1, 170)) * 8
        H = int(rng.integers(1, 18))
        cap = int(rng.integers(1, 5))
        commits = int(rng.integers(0, 2 * cap + 2))
        gain = 8.0 if case % 4 == 3 else 1.0
        seed = 5000 + 100 * dtype + case
        if dtype == ifx.IFX_BF16:
            cache, oc = fill_cache(dev, dtype, H, D, n, cap, commits, seed=seed)
        else:
            cache, oc = ifx.KVCache(1, H, D, cap * n, n, dtype), OracleCacheFP8(cap)
            for b in range(commits):
                _, k0, v0 = synth.draw_qkv(seed, b, 0, 0, n, H, D, torch.bfloat16, dev, True)
                cache.commit(0, k0, v0)
                oc.commit(k0, v0)
        with cache:
            resident = min(commits, cap)
            q, k, v = synth.draw_qkv(seed, 99, 0, 0, n, H, D, torch.bfloat16, dev, True, gain)
            hs = sorted({0, H - 1})
            tail = np.arange(max(0, n - 40), n)
            rows = np.concatenate([np.repeat(np.arange(n), len(hs)), np.repeat(tail, H)])
            heads = np.concatenate([np.tile(np.array(hs), n), np.tile(np.arange(H), len(tail))])
            kind = case % 3
            if kind == 0 or resident == 0:
                ranges = None
            elif kind == 1:
                first = int(rng.integers(0, resident))
                ranges = [(first, int(rng.integers(1, resident - first + 1)))]
            else:
                ranges = ([(0, 1)] if resident > 1 else []) + [(resident - 1, 1)]
            label = f"case {case}: n={n} H={H} cap={cap} commits={commits} gain={gain} ranges={ranges}"
            if ranges is None:
                out = torch.full((n, H, D), float("nan"), dtype=torch.bfloat16, device=dev)
                cache.attention(0, q, k, v, out)
                torch.cuda.synchronize()
                want, _ = oracle_ranges(oc, [(0, resident)] if resident else [], q, k, v, rows, heads)
            else:
                out, _ = run_ranges(cache, q, k, v, ranges, dev)
                want, _ = oracle_ranges(oc, ranges, q, k, v, rows, heads)
            assert torch.isfinite(out.float()).all(), label
            assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, dtype, label, input_scale=gain)


@pytest.mark.parametrize("seed,n,H,cap,commits,ranges", [
    (11003, 744, 2, 3, 1, None),
    (11031, 1000, 17, 1, 3, [(0, 1)]),
    (11147, 720, 6, 4, 0, None),       # no cached keys at all: only the current block
    (11139, 1272, 17, 4, 8, [(1, 3)]),
    (7079, 560, 1, 4, 6, [(3, 1)]),
])
def test_bf16_peaked_rows_with_large_outputs(gpu_device, seed, n, H, cap, commits, ranges):
    """Logits x 8: most rows are dominated by one key, and with a thousand rows some outputs lie
    above 4, where bf16 values are 2^-5 apart and the absolute gate of 2e-2 leaves room for the
    output's own rounding and little else.  Every output element is compared.  (With the row sum
    taken from the unrounded exponentials these five cases came out at 2.1e-2 ... 2.7e-2: numerator
    and denominator of a dominated row then differ by the rounding of its one weight.)"""
    dev = gpu_device
    D, gain = 128, 8.0
    cache, oc = fill_cache(dev, ifx.IFX_BF16, H, D, n, cap, commits, seed=seed)
    with cache:
        resident = min(commits, cap)
        q, k, v = synth.draw_qkv(seed, 99, 0, 0, n, H, D, torch.bfloat16, dev, True, gain)
        rows, heads = all_pairs(n, H)
        if ranges is None:
            out = torch.full((n, H, D), float("nan"), dtype=torch.bfloat16, device=dev)
            cache.attention(0, q, k, v, out)
            torch.cuda.synchronize()
            want, _ = oracle_ranges(oc, [(0, resident)] if resident else [], q, k, v, rows, heads)
        else:
            out, _ = run_ranges(cache, q, k, v, ranges, dev)
            want, _ = oracle_ranges(oc, ranges, q, k, v, rows, heads)
        assert (np.abs(want) > 4.0).sum() > 0  # the case is what it claims to be
        assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, ifx.IFX_BF16,
                               f"peaked rows, seed {seed}", input_scale=gain)


@pytest.mark.parametrize("dtype", [ifx.IFX_BF16, ifx.IFX_F32])
def test_commit_layers_equals_commits(gpu_device, dtype):
    """One ifx_kv_cache_commit_layers call gives the same caches, bit for bit, as one
    ifx_kv_cache_commit per layer: layers at different fill levels, through fill, wrap and
    eviction, 70 layers (more than one launch holds), against the deque oracle."""
    dev = gpu_device
    tdtype = TORCH_DTYPE[dtype]
    L, H, D, n, cap = 70, 2, 128 if dtype == ifx.IFX_BF16 else 64, 40, 3
    with ifx.KVCache(L, H, D, cap * n, n, dtype) as a, ifx.KVCache(L, H, D, cap * n, n, dtype) as b:
        ocs = [OracleCacheF(cap, tdtype) for _ in range(L)]
        # layers start at different fill levels: layer l has l % 4 blocks
        for layer in range(L):
            for t in range(layer % 4):
                _, k0, v0 = synth.draw_qkv(67, 100 + t, 0, layer, n, H, D, tdtype, dev, True)
                a.commit(layer, k0, v0)
                b.commit(layer, k0, v0)
                ocs[layer].commit(k0, v0)
        for blk in range(cap + 2):
            kv = [synth.draw_qkv(67, blk, 0, layer, n, H, D, tdtype, dev, True)[1:] for layer in range(L)]
            for layer in range(L):
                a.commit(layer, *kv[layer])
                ocs[layer].commit(*kv[layer])
            b.commit_layers(0, [k for k, _ in kv], [v for _, v in kv])
            torch.cuda.synchronize()
            for layer in (0, 1, 2, 3, 63, 64, 69):
                assert b.block_ids(layer) == a.block_ids(layer) == expected_ids(ocs[layer].raw, cap), (blk, layer)
                assert_cache_bits(b, layer, ocs[layer].raw, H, D, tdtype, dev)
                assert_cache_bits(a, layer, ocs[layer].raw, H, D, tdtype, dev)
        # a sub-range of layers, and attention on both caches afterwards
        kv = [synth.draw_qkv(67, 50, 0, layer, n, H, D, tdtype, dev, True)[1:] for layer in range(5, 9)]
        for i, layer in enumerate(range(5, 9)):
            a.commit(layer, *kv[i])
        b.commit_layers(5, [k for k, _ in kv], [v for _, v in kv])
        q, k, v = synth.draw_qkv(67, 60, 0, 0, n, H, D, tdtype, dev, True)
        for layer in (4, 5, 8, 9):
            oa, ob = torch.empty_like(q), torch.empty_like(q)
            a.attention(layer, q, k, v, oa)
            b.attention(layer, q, k, v, ob)
            torch.cuda.synchronize()
            assert synth.raw_bytes(oa) == synth.raw_bytes(ob), layer
            assert a.block_ids(layer) == b.block_ids(layer)
        # error paths: layer range out of bounds, a NULL entry
        with pytest.raises(ifx.IfxError) as e:
            b.commit_layers(L - 1, [k, k], [v, v])
        assert e.value.code == ifx.IFX_ERR_INVALID_ARG
        with pytest.raises(ifx.IfxError) as e:
            b.commit_layers(0, [k, None], [v, v])
        assert e.value.code == ifx.IFX_ERR_INVALID_ARG
        with pytest.raises(ifx.IfxError):
            b.commit_layers(0, [], [])
        assert b.committed(0) == a.committed(0)  # a refused call commits nothing


def oracle_blocks(oc, blocks, q, k, v, rows, heads):
    kc, vc = oc.raw.logical(blocks=blocks)
    if kc is not None:
        if oc.tdtype == torch.bfloat16:
            kc, vc = oracle.bf16_bits_to_f64(kc), oracle.bf16_bits_to_f64(vc)
        else:
            kc, vc = kc.astype(np.float64), vc.astype(np.float64)
    kb = None if k is None else synth.to_f64_numpy(k)
    vb = None if v is None else synth.to_f64_numpy(v)
    return oracle.attention_rows(synth.to_f64_numpy(q), kc, vc, kb, vb, rows, heads)


def run_blocks(cache, q, k, v, blocks, dev):
    n, H, D = q.shape
    out = torch.full((n, H, D), float("nan"), dtype=q.dtype, device=dev)
    lse = torch.full((n, H), float("nan"), dtype=torch.float32, device=dev)
    cache.attention_blocks(0, q, k, v, blocks, out, lse)
    torch.cuda.synchronize()
    return out, lse


@pytest.mark.parametrize("dtype", [ifx.IFX_BF16, ifx.IFX_F32])
def test_block_lists_in_any_order(gpu_device, dtype):
    """Attention over a caller-given list of resident blocks (scattered, permuted, on a wrapped
    ring), with and without the current block, against the oracle over the same list."""
    dev = gpu_device
    H, D, n = 2, (128 if dtype == ifx.IFX_BF16 else 64), 72  # blocks are not multiples of the 64-key tile
    cache, oc = fill_cache(dev, dtype, H, D, n, cap=9, commits=13, seed=71)
    with cache:
        q, k, v = synth.draw_qkv(71, 99, 0, 0, n, H, D, TORCH_DTYPE[dtype], dev, True)
        rows, heads = all_pairs(n, H)
        for picks, with_block in [([0, 2, 4, 6, 8], True), ([8, 1, 5], True), ([7, 6, 5, 4, 3, 2, 1, 0], False),
                                  ([3], False), ([], True), (list(range(9)), True), ([2, 7, 0, 8, 3, 5], False)]:
            kk, vv = (k, v) if with_block else (None, None)
            out, lse = run_blocks(cache, q, kk, vv, picks, dev)
            want, want_lse = oracle_blocks(oc, picks, q, kk, vv, rows, heads)
            assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, dtype, f"blocks {picks}")
            assert np.abs(lse.cpu().numpy().astype(np.float64)[rows, heads] - want_lse).max() <= LSE_TOL[dtype], picks
        # None = every resident block where it lies: the plain call's bits, plus the log-sum-exp
        plain = torch.empty_like(q)
        cache.attention(0, q, k, v, plain)
        got, lse = run_blocks(cache, q, k, v, None, dev)
        view = torch.int16 if dtype == ifx.IFX_BF16 else torch.int32
        assert torch.equal(plain.view(view), got.view(view))
        _, want_lse = oracle_blocks(oc, list(range(9)), q, k, v, rows, heads)
        assert np.abs(lse.cpu().numpy().astype(np.float64)[rows, heads] - want_lse).max() <= LSE_TOL[dtype]
        # a range call is the same call with its blocks written out: identical bits
        a, la = run_ranges(cache, q, k, v, [(1, 2), (6, 3)], dev)
        b, lb = run_blocks(cache, q, k, v, [1, 2, 6, 7, 8], dev)
        assert torch.equal(a.view(torch.int16 if dtype == ifx.IFX_BF16 else torch.int32),
                           b.view(torch.int16 if dtype == ifx.IFX_BF16 else torch.int32)) and torch.equal(la, lb)
        out = torch.empty_like(q)
        for bad in ([9], [-1], [2, 2], [0, 1, 2, 3, 4, 5, 6, 7, 8, 0]):
            with pytest.raises(ifx.IfxError) as e:
                cache.attention_blocks(0, q, k, v, bad, out)
            assert e.value.code == ifx.IFX_ERR_INVALID_ARG, bad
        with pytest.raises(ifx.IfxError):
            cache.attention_blocks(0, q, None, None, [], out)  # no key at all


def test_long_block_lists(gpu_device):
    """A key set in the region's own order needs no table; a selection of up to
    IFX_MAX_LISTED_BLOCKS blocks travels with the launch; a longer one goes through the layer's
    device list, IFX_MAX_LISTED_BLOCKS entries per pass: 64, 126, 127 and all 130 resident blocks
    in scrambled order, with and without the current block, on a wrapped ring, both dtypes'
    kernels, against the oracle over exactly those blocks; and the same result as split calls
    merged."""
    dev = gpu_device
    H, D, n, cap = 1, 128, 8, 130
    cache, oc = fill_cache(dev, ifx.IFX_BF16, H, D, n, cap=cap, commits=cap, seed=5)
    with cache:
        q, k, v = synth.draw_qkv(5, 999, 0, 0, n, H, D, torch.bfloat16, dev, True)
        rows, heads = all_pairs(n, H)
        out = torch.empty_like(q)
        # 130 resident blocks, ring full but not wrapped: plain order, no table
        cache.attention(0, q, k, v, out)
        torch.cuda.synchronize()
        want, _ = oracle_blocks(oc, list(range(cap)), q, k, v, rows, heads)
        assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, ifx.IFX_BF16, "130 blocks in place")
        # 63 listed blocks (+ the current one): travels with the launch
        picks = list(range(129, 129 - 2 * 63, -2))
        assert len(picks) == ifx.IFX_MAX_LISTED_BLOCKS
        got, lse = run_blocks(cache, q, k, v, picks, dev)
        want, want_lse = oracle_blocks(oc, picks, q, k, v, rows, heads)
        assert_attention_close(to_np_exact(got)[rows, heads].astype(np.float64), want, ifx.IFX_BF16, "63 listed blocks")
        assert np.abs(lse.cpu().numpy().astype(np.float64)[rows, heads] - want_lse).max() <= LSE_TOL[ifx.IFX_BF16]
        # one more goes through the device list; the same keys as two calls and a merge
        picks = list(range(129, 129 - 64, -1))
        got, lse = run_blocks(cache, q, k, v, picks, dev)
        want, want_lse = oracle_blocks(oc, picks, q, k, v, rows, heads)
        assert_attention_close(to_np_exact(got)[rows, heads].astype(np.float64), want, ifx.IFX_BF16, "64 listed blocks")
        assert np.abs(lse.cpu().numpy().astype(np.float64)[rows, heads] - want_lse).max() <= LSE_TOL[ifx.IFX_BF16]
        o1, l1 = run_blocks(cache, q, None, None, list(range(129, 98, -1)), dev)
        o2, l2 = run_blocks(cache, q, k, v, list(range(98, 129 - 64, -1)), dev)
        ifx.ifx_attention_merge(o1, l1, o2, l2, o1, l1, n * H, D, ifx.IFX_BF16)
        torch.cuda.synchronize()
        err = np.abs(to_np_exact(o1)[rows, heads].astype(np.float64) - want)
        rms = np.sqrt(np.mean(want ** 2))
        assert err.max() <= 5e-2 * rms and err.mean() <= 3e-3 * rms
        assert np.abs(l1.cpu().numpy().astype(np.float64)[rows, heads] - want_lse).max() <= LSE_TOL[ifx.IFX_BF16]
        # after one more commit the ring has wrapped; "all resident blocks" is still read in slot order
        cache.commit(0, k, v)
        oc.commit(k, v)
        cache.attention(0, q, k, v, out)
        torch.cuda.synchronize()
        want, _ = oracle_blocks(oc, list(range(cap)), q, k, v, rows, heads)
        assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, ifx.IFX_BF16, "130 blocks, wrapped")
        # the same blocks oldest first (a range over the wrapped ring), and scrambled lists of 126, 127 (two full
        # passes and one entry) and 130 blocks, with and without the current block
        got, lse = run_ranges(cache, q, k, v, [(0, cap)], dev)
        assert_attention_close(to_np_exact(got)[rows, heads].astype(np.float64), want, ifx.IFX_BF16, "130 blocks oldest first")
        rng = np.random.default_rng(11)
        for count in (126, 127, 130):
            picks = rng.permutation(cap)[:count].tolist()
            for kk, vv in ((k, v), (None, None)):
                got, lse = run_blocks(cache, q, kk, vv, picks, dev)
                want, want_lse = oracle_blocks(oc, picks, q, kk, vv, rows, heads)
                label = f"{count} listed blocks, block={kk is not None}"
                assert_attention_close(to_np_exact(got)[rows, heads].astype(np.float64), want, ifx.IFX_BF16, label)
                assert np.abs(lse.cpu().numpy().astype(np.float64)[rows, heads] - want_lse).max() <= LSE_TOL[ifx.IFX_BF16], label
        # a list longer than what is resident is refused
        with pytest.raises(ifx.IfxError) as e:
            cache.attention_blocks(0, q, k, v, list(range(cap)) + [0], out)
        assert e.value.code == ifx.IFX_ERR_INVALID_ARG
    # fp32: blocks of 72 keys (entries straddle tiles), 70 of 80 blocks scrambled
    H, D, n, cap = 2, 64, 72, 80
    cache, oc = fill_cache(dev, ifx.IFX_F32, H, D, n, cap=cap, commits=cap + 3, seed=6)
    with cache:
        q, k, v = synth.draw_qkv(6, 999, 0, 0, n, H, D, torch.float32, dev, True)
        rows, heads = all_pairs(n, H)
        picks = np.random.default_rng(12).permutation(cap)[:70].tolist()
        got, lse = run_blocks(cache, q, k, v, picks, dev)
        want, want_lse = oracle_blocks(oc, picks, q, k, v, rows, heads)
        assert_attention_close(to_np_exact(got)[rows, heads].astype(np.float64), want, ifx.IFX_F32, "fp32 70 listed blocks")
        assert np.abs(lse.cpu().numpy().astype(np.float64)[rows, heads] - want_lse).max() <= LSE_TOL[ifx.IFX_F32]
