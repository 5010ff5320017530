"""GPU parity at the full sizes of the benchmark configurations: the 7-block
generate-and-cache loop (30 layers, 4 denoising steps per block), the 40-block
ring-buffer stress, and the 720p 14B-class layer.  Attention is compared with
the fp64 oracle on sampled rows (every row of the first and last head, >= 64
rows of every other head, full key length); commit / ring indexing is compared
bit for bit."""
import time

import numpy as np
import pytest
import torch

import oracle
from paper_2511_20714_amd import binding as ifx
from paper_2511_20714_amd import synth

from gpu_util import (OracleCacheF, as_oracle_block, assert_attention_close, assert_cache_bits, expected_ids, sample_rows,
                      to_np_exact)

pytestmark = pytest.mark.gpu

H, D, N_BLK = 12, 128, 4680


def check_attention(out, q, k, v, ocache, label, seed):
    rows, heads = sample_rows(q.shape[0], q.shape[1], seed=seed)
    kc, vc = ocache.logical()
    want, _ = oracle.attention_rows(synth.to_f64_numpy(q), kc, vc, synth.to_f64_numpy(k), synth.to_f64_numpy(v),
                                    rows, heads)
    got = to_np_exact(out)[rows, heads].astype(np.float64)
    mx, mean, rms = assert_attention_close(got, want, ifx.IFX_BF16, label)
    print(f"{label}: rows={len(rows)} keys={q.shape[0] + (0 if kc is None else kc.shape[0])} "
          f"max|err|={mx:.2e} mean|err|={mean:.2e} rms(out)={rms:.2e}", flush=True)


def test_config2_every_output_element(gpu_device):
    """The headline shape (12 heads x 128, block of 4680, 28080 cached tokens, key length 32760),
    in the launch configuration the benchmark times: every one of the 4680 x 12 x 128 outputs
    against the fp64 oracle (about 45 s of oracle time on 16 host threads)."""
    dev = gpu_device
    cap = 6
    with ifx.KVCache(1, H, D, cap * N_BLK, N_BLK, ifx.IFX_BF16) as cache:
        oc = OracleCacheF(cap, torch.bfloat16)
        for b in range(cap):
            _, k, v = synth.draw_qkv(2, b, 0, 0, N_BLK, H, D, torch.bfloat16, dev, rms_norm=True)
            cache.commit(0, k, v)
            oc.commit(k, v)
        q, k, v = synth.draw_qkv(2, cap, 0, 0, N_BLK, H, D, torch.bfloat16, dev, rms_norm=True)
        out = torch.full((N_BLK, H, D), float("nan"), dtype=torch.bfloat16, device=dev)
        cache.attention(0, q, k, v, out)
        torch.cuda.synchronize()
        kc, vc = oc.logical()
        t0 = time.time()
        want, _ = oracle.attention(synth.to_f64_numpy(q), kc, vc, synth.to_f64_numpy(k), synth.to_f64_numpy(v))
        got = to_np_exact(out).astype(np.float64)
        mx, mean, rms = assert_attention_close(got.reshape(-1, D), want.reshape(-1, D), ifx.IFX_BF16, "config2, all rows")
        print(f"config2 all rows: oracle {time.time() - t0:.1f} s  max|err|={mx:.2e} mean|err|={mean:.2e} rms(out)={rms:.2e}",
              flush=True)


def test_config3_generate_and_cache_loop(gpu_device):
    """30 layers x 12 heads x 128; 7 blocks of 4680 tokens, 4 denoising steps each, fresh q/k/v per
    (block, step, layer); after a block's last step its K/V are committed.  Attention checked at
    (block 1, step 1), (block 4, step 2), (block 7, step 4) on two layers; the cache of three layers
    is read back and compared byte for byte after every block; slot ids on all layers."""
    dev = gpu_device
    L, blocks, steps, cap = 30, 7, 4, 7
    check_layers = (0, 17)
    byte_layers = (0, 17, 29)
    checks = {(0, 0), (3, 1), (6, 3)}
    with ifx.KVCache(L, H, D, cap * N_BLK, N_BLK, ifx.IFX_BF16) as cache:
        ocs = {l: OracleCacheF(cap, torch.bfloat16) for l in byte_layers}
        out = torch.empty((N_BLK, H, D), dtype=torch.bfloat16, device=dev)
        t_start = time.time()
        for b in range(blocks):
            for s in range(steps):
                for l in range(L):
                    q, k, v = synth.draw_qkv(3, b, s, l, N_BLK, H, D, torch.bfloat16, dev, rms_norm=True)
                    cache.attention(l, q, k, v, out)
                    if (b, s) in checks and l in check_layers:
                        torch.cuda.synchronize()
                        check_attention(out, q, k, v, ocs[l], f"config3 block {b + 1} step {s + 1} layer {l}", seed=b)
                    if s == steps - 1:
                        cache.commit(l, k, v)
                        if l in ocs:
                            ocs[l].commit(k, v)
            torch.cuda.synchronize()
            for l in range(L):
                assert cache.committed(l) == b + 1
                assert cache.len(l) == (b + 1) * N_BLK
                assert cache.block_ids(l) == list(range(b + 1)) + [-1] * (cap - b - 1)
            for l in byte_layers:
                assert_cache_bits(cache, l, ocs[l].raw, H, D, torch.bfloat16, dev)
        print(f"config3 loop wall time incl. checks: {time.time() - t_start:.1f} s", flush=True)


def test_config4_ring_buffer_40_blocks(gpu_device):
    """30 layers, 40 blocks through a ring of 7 block slots (32760 tokens), one attention + commit per
    block and layer.  Slot ids of all 30 layers after every commit; cache bytes and attention on two
    layers at blocks 1, 7, 8 and 40 (block 8 is the first to see a full ring, its commit the first
    eviction; block 40 sees ordinals 33..39 in slot order 36,37,38,39,33,34,35, 1-based)."""
    dev = gpu_device
    L, blocks, cap = 30, 40, 7
    check_layers = (3, 29)
    check_blocks = {0, 6, 7, 39}
    with ifx.KVCache(L, H, D, cap * N_BLK, N_BLK, ifx.IFX_BF16) as cache:
        ocs = {l: OracleCacheF(cap, torch.bfloat16) for l in check_layers}
        out = torch.empty((N_BLK, H, D), dtype=torch.bfloat16, device=dev)
        for b in range(blocks):
            for l in range(L):
                q, k, v = synth.draw_qkv(4, b, 0, l, N_BLK, H, D, torch.bfloat16, dev, rms_norm=True)
                cache.attention(l, q, k, v, out)
                if b in check_blocks and l in check_layers:
                    torch.cuda.synchronize()
                    assert cache.len(l) == min(b, cap) * N_BLK
                    assert_cache_bits(cache, l, ocs[l].raw, H, D, torch.bfloat16, dev)
                    check_attention(out, q, k, v, ocs[l], f"config4 block {b + 1} layer {l}", seed=b)
                cache.commit(l, k, v)
                if l in ocs:
                    ocs[l].commit(k, v)
            want_ids = [-1] * cap
            for o in range(max(0, b + 1 - cap), b + 1):
                want_ids[o % cap] = o
            for l in range(L):
                assert cache.block_ids(l) == want_ids
            for l in check_layers:
                assert cache.block_ids(l) == expected_ids(ocs[l].raw, cap)
        torch.cuda.synchronize()
        # after 40 commits: slots hold 1-based blocks 36,37,38,39,40,34,35; block 40 itself saw 33..39
        assert cache.block_ids(0) == [35, 36, 37, 38, 39, 33, 34]
        for l in check_layers:
            assert_cache_bits(cache, l, ocs[l].raw, H, D, torch.bfloat16, dev)


def test_config5_wan14b_720p_layer(gpu_device):
    """40 heads x 128, block of 10800 tokens, 43200 cached tokens: key length 54000."""
    dev = gpu_device
    n, H5, cap = 10800, 40, 4
    with ifx.KVCache(1, H5, D, cap * n, n, ifx.IFX_BF16) as cache:
        oc = OracleCacheF(cap, torch.bfloat16)
        for b in range(cap):
            _, k, v = synth.draw_qkv(5, b, 0, 0, n, H5, D, torch.bfloat16, dev, rms_norm=True)
            cache.commit(0, k, v)
            oc.commit(k, v)
        q, k, v = synth.draw_qkv(5, cap, 0, 0, n, H5, D, torch.bfloat16, dev, rms_norm=True)
        out = torch.full((n, H5, D), float("nan"), dtype=torch.bfloat16, device=dev)
        cache.attention(0, q, k, v, out)
        torch.cuda.synchronize()
        assert not torch.isnan(out.float()).any()
        rows, heads = sample_rows(n, H5, full_heads=(0,), seed=5)
        kc, vc = oc.logical()
        want, _ = oracle.attention_rows(synth.to_f64_numpy(q), kc, vc, synth.to_f64_numpy(k), synth.to_f64_numpy(v),
                                        rows, heads)
        got = to_np_exact(out)[rows, heads].astype(np.float64)
        mx, mean, rms = assert_attention_close(got, want, ifx.IFX_BF16, "config5")
        print(f"config5: rows={len(rows)} keys=54000 max|err|={mx:.2e} mean|err|={mean:.2e} rms(out)={rms:.2e}")
        assert_cache_bits(cache, 0, oc.raw, H5, D, torch.bfloat16, dev)
