"""ifx_block_attention_blocks_noalloc (the block list lives in the library's static device
memory) against ifx_block_attention_blocks: the same bits, on two calls in a row of which the
second lists fewer blocks, and on every kind of selection; plus its limit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_20714_amd import binding as ifx
from paper_2511_20714_amd import synth

from gpu_util import TORCH_DTYPE, OracleCacheF, assert_attention_close, to_np_exact

pytestmark = pytest.mark.gpu


def both(cache, q, k, v, blocks, dev):
    """(out, lse) of the existing entry point and of the no-allocation one."""
    n, H, D = q.shape
    res = []
    for call in (cache.attention_blocks, cache.attention_blocks_noalloc):
        out = torch.full((n, H, D), float("nan"), dtype=q.dtype, device=dev)
        lse = torch.full((n, H), float("nan"), dtype=torch.float32, device=dev)
        call(0, q, k, v, blocks, out, lse)
        res.append((out, lse))
    torch.cuda.synchronize()
    return res


@pytest.mark.parametrize("dtype,D", [(ifx.IFX_BF16, 128), (ifx.IFX_F32, 64)])
def test_noalloc_equals_blocks(gpu_device, dtype, D):
    dev = gpu_device
    tdtype = TORCH_DTYPE[dtype]
    H, n, cap = 2, 40, 100
    with ifx.KVCache(1, H, D, cap * n, n, dtype) as cache:
        oc = OracleCacheF(cap, tdtype)
        for b in range(cap + 7):  # wrapped
            _, k, v = synth.draw_qkv(107, b, 0, 0, n, H, D, tdtype, dev, True)
            cache.commit(0, k, v)
            oc.commit(k, v)
        q, k, v = synth.draw_qkv(107, 999, 0, 0, n, H, D, tdtype, dev, True)
        rng = np.random.default_rng(3)
        view = torch.int16 if dtype == ifx.IFX_BF16 else torch.int32
        # two calls in a row, the second with a smaller input: 90 listed blocks, then 5; then the other kinds
        selections = [rng.permutation(cap)[:90].tolist(), [7, 3, 99, 0, 50], rng.permutation(cap)[:64].tolist(), [42], [], None,
                      list(range(cap))]
        for i, picks in enumerate(selections):
            for kk, vv in ((k, v), (None, None)):
                if not picks and picks is not None and kk is None:
                    continue  # no key at all
                (o_ref, l_ref), (o_new, l_new) = both(cache, q, kk, vv, picks, dev)
                label = f"selection {i}, block={kk is not None}"
                assert torch.equal(o_ref.view(view), o_new.view(view)), label
                assert torch.equal(l_ref.view(torch.int32), l_new.view(torch.int32)), label
                assert torch.isfinite(o_new.float()).all(), label
        # ... and right: the first selection against the oracle
        picks = selections[0]
        rows, heads = np.repeat(np.arange(n), H), np.tile(np.arange(H), n)
        kc, vc = oc.raw.logical(blocks=picks)
        kc, vc = (oracle.bf16_bits_to_f64(kc), oracle.bf16_bits_to_f64(vc)) if dtype == ifx.IFX_BF16 else (kc.astype(np.float64), vc.astype(np.float64))
        want, _ = oracle.attention_rows(synth.to_f64_numpy(q), kc, vc, synth.to_f64_numpy(k), synth.to_f64_numpy(v), rows, heads)
        out = torch.empty_like(q)
        cache.attention_blocks_noalloc(0, q, k, v, picks, out)
        torch.cuda.synchronize()
        assert_attention_close(to_np_exact(out)[rows, heads].astype(np.float64), want, dtype, "noalloc vs oracle")
        # errors: what the existing entry point refuses, and a list beyond the static array
        with pytest.raises(ifx.IfxError) as e:
            cache.attention_blocks_noalloc(0, q, k, v, [1, 1], out)
        assert e.value.code == ifx.IFX_ERR_INVALID_ARG
        with pytest.raises(ifx.IfxError) as e:
            cache.attention_blocks_noalloc(0, q, k, v, list(range(ifx.IFX_NOALLOC_MAX_LISTED_BLOCKS + 1)), out)
        assert e.value.code == ifx.IFX_ERR_UNSUPPORTED
