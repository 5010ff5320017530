"""Raising a cache's capacity on the device (ifx_kv_cache_grow): resident blocks, their order and
their numbers survive bit for bit, attention over them is unchanged, and the window evicts again
only when the larger capacity is full -- against the growing deque oracle."""
import numpy as np
import pytest
import torch

from paper_2511_20714_amd import binding as ifx
from paper_2511_20714_amd import synth

from gpu_util import TORCH_DTYPE, OracleCacheF, assert_attention_close, assert_cache_bits, oracle_rows, to_np_exact

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [ifx.IFX_BF16, ifx.IFX_F32])
def test_grow_keeps_the_blocks_and_widens_the_window(gpu_device, dtype):
    dev = gpu_device
    tdtype = TORCH_DTYPE[dtype]
    L, H, D, n = 2, 3, (128 if dtype == ifx.IFX_BF16 else 64), 72
    rows, heads = np.repeat(np.arange(n), H), np.tile(np.arange(H), n)
    with ifx.KVCache(L, H, D, 3 * n, n, dtype) as cache:
        ocs = [OracleCacheF(3, tdtype) for _ in range(L)]
        history = [[] for _ in range(L)]  # ordinals committed per layer

        def commit(layer, b):
            _, k, v = synth.draw_qkv(61, b, 0, layer, n, H, D, tdtype, dev, True)
            cache.commit(layer, k, v)
            ocs[layer].commit(k, v)
            history[layer].append(len(history[layer]))

        def check(layer, label, slots_expected=None):
            q, k, v = synth.draw_qkv(61, 1000 + len(history[layer]), 1, layer, n, H, D, tdtype, dev, True)
            out = torch.full((n, H, D), float("nan"), dtype=tdtype, device=dev)
            cache.attention(layer, q, k, v, out)
            torch.cuda.synchronize()
            want = oracle_rows(q, k, v, ocs[layer], rows, heads)
            assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, dtype, label)
            assert_cache_bits(cache, layer, ocs[layer].raw, H, D, tdtype, dev)
            assert cache.committed(layer) == ocs[layer].raw.committed
            assert cache.len(layer) == len(ocs[layer].raw.ordinals) * n
            if slots_expected is not None:
                assert cache.block_ids(layer) == slots_expected, label

        for b in range(5):
            commit(0, b)  # layer 0: wrapped, residents 2 3 4 in slots 2 0 1
        for b in range(2):
            commit(1, b)  # layer 1: not full yet
        check(0, "before, wrapped", [3, 4, 2])
        check(1, "before, not full", [0, 1, -1])

        for bad in (3 * n, 2 * n, 4 * n + 8, 0):
            with pytest.raises(ifx.IfxError) as e:
                cache.grow(bad)
            assert e.value.code == ifx.IFX_ERR_INVALID_ARG, bad
        cache.grow(6 * n)
        for oc in ocs:
            oc.raw.grow(6)
        check(0, "after grow, was wrapped", [2, 3, 4, -1, -1, -1])
        check(1, "after grow, was not full", [0, 1, -1, -1, -1, -1])
        # the new slots fill up without evicting, then the ring wraps again
        for b in range(5, 11):
            commit(0, b)
            check(0, f"layer 0 after commit {b}")
        assert ocs[0].raw.ordinals == [5, 6, 7, 8, 9, 10]
        assert cache.block_ids(0) == [8, 9, 10, 5, 6, 7]
        for b in range(2, 9):
            commit(1, b)
        check(1, "layer 1 wrapped after the grow", [6, 7, 8, 3, 4, 5])
        # chosen blocks and a second grow
        out = torch.full((n, H, D), float("nan"), dtype=tdtype, device=dev)
        q, k, v = synth.draw_qkv(61, 77, 2, 0, n, H, D, tdtype, dev, True)
        cache.attention_blocks(0, q, k, v, [5, 0, 3], out)
        cache.grow(8 * n)
        ocs[0].raw.grow(8), ocs[1].raw.grow(8)
        out2 = torch.full((n, H, D), float("nan"), dtype=tdtype, device=dev)
        cache.attention_blocks(0, q, k, v, [5, 0, 3], out2)
        torch.cuda.synchronize()
        view = torch.int16 if dtype == ifx.IFX_BF16 else torch.int32
        assert torch.equal(out.view(view), out2.view(view))  # same blocks, same order of the list: same bits
        check(0, "second grow", [5, 6, 7, 8, 9, 10, -1, -1])
        check(1, "second grow", [3, 4, 5, 6, 7, 8, -1, -1])


@pytest.mark.parametrize("dtype,L,H,n", [(ifx.IFX_BF16, 2, 3, 72), (ifx.IFX_F32, 2, 3, 72), (ifx.IFX_BF16, 2, 2, 2056)])
def test_reserved_cache_grows_in_place(gpu_device, dtype, L, H, n):
    """A cache with a reservation (ifx_kv_cache_reserve) grows by mapping memory behind every
    head's resident tokens: no block changes its slot (block_ids before == after), contents are
    bit-exact, a call enqueued just before the grow is not disturbed, the new slots fill up next
    and then the oldest block goes first, wherever it sits.  Grown while wrapped and while not
    full, twice, up to the reservation; one step beyond is refused.  With blocks of 72 tokens all
    of it happens inside each head's first piece of memory; with blocks of 2056 tokens (514 KiB per
    head) every grow maps new pieces behind the old ones."""
    dev = gpu_device
    tdtype = TORCH_DTYPE[dtype]
    D = 128 if dtype == ifx.IFX_BF16 else 64
    if n > 1000:  # a sample of rows is enough at this size
        rows = np.repeat(np.unique(np.concatenate([np.arange(0, n, 37), np.arange(n - 8, n), [255, 256, 2047, 2048]])), H)
        heads = np.tile(np.arange(H), len(rows) // H)
    else:
        rows, heads = np.repeat(np.arange(n), H), np.tile(np.arange(H), n)
    with ifx.KVCache(L, H, D, 3 * n, n, dtype, reserve_tokens=8 * n) as cache:
        ocs = [OracleCacheF(3, tdtype) for _ in range(L)]
        slot_of = [dict() for _ in range(L)]  # layer -> {ordinal: slot}, the documented slot rule replayed
        cap = [3]

        def commit(layer, b):
            _, k, v = synth.draw_qkv(71, b, 0, layer, n, H, D, tdtype, dev, True)
            resident = sorted(slot_of[layer])
            slot = slot_of[layer].pop(resident[0]) if len(resident) == cap[0] else len(resident)
            cache.commit(layer, k, v)
            ocs[layer].commit(k, v)
            slot_of[layer][ocs[layer].raw.committed - 1] = slot

        def ids(layer):
            want = [-1] * cap[0]
            for o, s in slot_of[layer].items():
                want[s] = o
            return want

        def check(layer, label):
            q, k, v = synth.draw_qkv(71, 1000 + ocs[layer].raw.committed, 1, layer, n, H, D, tdtype, dev, True)
            out = torch.full((n, H, D), float("nan"), dtype=tdtype, device=dev)
            cache.attention(layer, q, k, v, out)
            torch.cuda.synchronize()
            want = oracle_rows(q, k, v, ocs[layer], rows, heads)
            assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, dtype, label)
            assert_cache_bits(cache, layer, ocs[layer].raw, H, D, tdtype, dev)
            assert cache.committed(layer) == ocs[layer].raw.committed
            assert cache.len(layer) == len(ocs[layer].raw.ordinals) * n
            assert cache.block_ids(layer) == ids(layer), label
            assert sorted(ocs[layer].raw.ordinals) == sorted(slot_of[layer])

        for b in range(5):
            commit(0, b)  # layer 0: wrapped, residents 2 3 4 in slots 2 0 1
        for b in range(2):
            commit(1, b)  # layer 1: not full yet
        check(0, "before, wrapped")
        check(1, "before, not full")
        assert cache.block_ids(0) == [3, 4, 2]

        # a call enqueued right before the grow, checked after it
        q, k, v = synth.draw_qkv(71, 555, 1, 0, n, H, D, tdtype, dev, True)
        pending = torch.full((n, H, D), float("nan"), dtype=tdtype, device=dev)
        cache.attention(0, q, k, v, pending)
        cache.grow(6 * n)
        cap[0] = 6
        for oc in ocs:
            oc.raw.grow(6)
        torch.cuda.synchronize()
        want = oracle_rows(q, k, v, ocs[0], rows, heads)
        assert_attention_close(to_np_exact(pending)[rows, heads].astype(np.float64), want, dtype, "enqueued before the grow")
        assert cache.block_ids(0) == [3, 4, 2, -1, -1, -1]
        assert cache.block_ids(1) == [0, 1, -1, -1, -1, -1]
        check(0, "after grow, was wrapped")
        check(1, "after grow, was not full")
        # the new slots fill up without evicting; then the oldest block goes first: ordinal 2 in slot 2
        for b in range(5, 8):
            commit(0, b)
            check(0, f"layer 0 after commit {b}")
        assert cache.block_ids(0) == [3, 4, 2, 5, 6, 7]
        commit(0, 8)
        assert cache.block_ids(0) == [3, 4, 8, 5, 6, 7]
        commit(0, 9)
        assert cache.block_ids(0) == [9, 4, 8, 5, 6, 7]
        check(0, "layer 0 wrapped again")
        for b in range(2, 9):
            commit(1, b)
        check(1, "layer 1 wrapped after the grow")
        # chosen blocks and ranges on the scrambled slot order, across a second grow
        out = torch.full((n, H, D), float("nan"), dtype=tdtype, device=dev)
        q, k, v = synth.draw_qkv(71, 77, 2, 0, n, H, D, tdtype, dev, True)
        cache.attention_blocks(0, q, k, v, [5, 0, 3], out)
        cache.grow(8 * n)
        cap[0] = 8
        ocs[0].raw.grow(8), ocs[1].raw.grow(8)
        out2 = torch.full((n, H, D), float("nan"), dtype=tdtype, device=dev)
        cache.attention_blocks(0, q, k, v, [5, 0, 3], out2)
        torch.cuda.synchronize()
        view = torch.int16 if dtype == ifx.IFX_BF16 else torch.int32
        assert torch.equal(out.view(view), out2.view(view))
        kc, vc = ocs[0].raw.logical(blocks=[5, 0, 3])
        import oracle
        kc, vc = (oracle.bf16_bits_to_f64(kc), oracle.bf16_bits_to_f64(vc)) if dtype == ifx.IFX_BF16 else (kc.astype(np.float64), vc.astype(np.float64))
        want, _ = oracle.attention_rows(synth.to_f64_numpy(q), kc, vc, synth.to_f64_numpy(k), synth.to_f64_numpy(v), rows, heads)
        assert_attention_close(to_np_exact(out2)[rows, heads].astype(np.float64), want, dtype, "listed blocks after two grows")
        check(0, "second grow")
        check(1, "second grow")
        for b in range(10, 14):
            commit(0, b)
        check(0, "layer 0 after the second grow, wrapped")
        with pytest.raises(ifx.IfxError) as e:
            cache.grow(9 * n)  # beyond the reservation
        assert e.value.code == ifx.IFX_ERR_UNSUPPORTED
        check(1, "after the refused grow")
